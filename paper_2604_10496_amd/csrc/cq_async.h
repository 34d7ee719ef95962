// Vector-memory operations issued from inline assembly and waited for by explicit counts, shared by the
// kernels that keep loads in flight across pipeline steps (gfx950 only).
#ifndef CQ_ASYNC_H_
#define CQ_ASYNC_H_

#include "cq_internal.h"

namespace cq_async {

// ---- memory operations the compiler must not track -------------------------------------------------
// The pipeline keeps loads in flight across several K steps.  The compiler's own wait insertion would
// drain them (it treats an LDS read after a direct-to-LDS load as dependent on it), so the loop's
// global loads are issued from inline assembly and waited for by explicit vmcnt counts.  The kernel has
// no static LDS (verified by the launcher): dynamic LDS starts at address 0 and byte offsets are LDS
// addresses.

// 16 bytes per lane from global memory into the registers `dst`; valid only after a vm_wait that
// names `dst`
static __device__ __forceinline__ void load_global_async(cq_v4u& dst, const uint8_t* src) {
  asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(dst) : "v"(src) : "memory");
}
// (m0 is a reserved register: the compiler loads it right before each use of its own and does not
// keep values in it, which is what clobbering it here relies on)
#pragma clang diagnostic ignored "-Winline-asm"
// 16 bytes per lane from global memory straight into LDS at lds_base + 16 * lane (lds_base uniform)
static __device__ __forceinline__ void load_global_to_lds(uint32_t lds_base, const uint8_t* src) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_base), "v"(src) : "memory", "m0");
}
// The same two loads with the address given as a uniform base (a scalar register pair) plus a 32-bit
// per-lane byte offset plus an immediate (0 .. 4095): the per-step address arithmetic is then scalar.
template <int IMM>
static __device__ __forceinline__ void load_global_async_s(cq_v4u& dst, const void* base, uint32_t lane_off) {
  asm volatile("global_load_dwordx4 %0, %1, %2 offset:%3" : "=v"(dst) : "v"(lane_off), "s"(base), "n"(IMM) : "memory");
}
template <int IMM>
static __device__ __forceinline__ void load_global_to_lds_s(uint32_t lds_base, const void* base, uint32_t lane_off) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2 offset:%3" ::"s"(lds_base), "v"(lane_off),
               "s"(base), "n"(IMM)
               : "memory", "m0");
}
// wait until at most N of this wavefront's vector-memory loads are outstanding; the registers passed
// through become usable only after it
template <int N>
static __device__ __forceinline__ void vm_wait(cq_v4u& a, cq_v4u& b) {
  asm volatile("s_waitcnt vmcnt(%2)" : "+v"(a), "+v"(b) : "n"(N) : "memory");
}
template <int N>
static __device__ __forceinline__ void vm_wait(cq_v4u& a, cq_v4u& b, cq_v4u& c, cq_v4u& d) {
  asm volatile("s_waitcnt vmcnt(%4)" : "+v"(a), "+v"(b), "+v"(c), "+v"(d) : "n"(N) : "memory");
}
static __device__ __forceinline__ cq_v4u lds_read_u128(uint32_t byte_offset) {
  return *reinterpret_cast<const __attribute__((address_space(3))) cq_v4u*>((uintptr_t)byte_offset);
}

}  // namespace cq_async

#endif  // CQ_ASYNC_H_
