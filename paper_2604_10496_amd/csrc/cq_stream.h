// Device helpers shared by the streaming kernels of the codebook product (gfx950 only): conversion of the
// activation rows into matrix-core operands, the index-stream load, LDS access by byte offset.
#ifndef CQ_STREAM_H_
#define CQ_STREAM_H_

#include "cq_internal.h"

#ifndef CQ_STREAM_NT
#define CQ_STREAM_NT 1
#endif

namespace {

__device__ __forceinline__ uint32_t f32_to_f16_bits_sat(float x) {
  x = fminf(fmaxf(x, -65504.f), 65504.f);
  const _Float16 h = (_Float16)x;
  return (uint32_t) __builtin_bit_cast(uint16_t, h);
}

__device__ __forceinline__ uint32_t bf16_bits_to_f16_bits(uint32_t b) {
  const _Float16 h = (_Float16)__uint_as_float(b << 16);
  return (uint32_t) __builtin_bit_cast(uint16_t, h);
}

// integer code -> bf16 bits: a float holding a small integer has zero low mantissa bits.
__device__ __forceinline__ uint32_t code_to_bf16_bits(int c) { return __float_as_uint((float)c) >> 16; }

// Eight consecutive activations of one row, as loaded (raw) and as four dwords of 16-bit MFMA operand pairs:
// bf16 for integer codes and bf16 rows, f16 for f16 / f32 rows.  grouped: paired like the prepacked index
// bytes pair the weights, (k0 k4 | k1 k5 | k2 k6 | k3 k7), instead of (k0 k1 | k2 k3 | k4 k5 | k6 k7).
struct ActRaw { uint4 a, b; };

template <int AK>
__device__ __forceinline__ ActRaw act_load8(const void* A, size_t e0) {
  ActRaw r;
  r.b = make_uint4(0u, 0u, 0u, 0u);
  if constexpr (AK == CQ_A_INT8_CODES) {
    const uint2 v = *reinterpret_cast<const uint2*>(reinterpret_cast<const int8_t*>(A) + e0);
    r.a = make_uint4(v.x, v.y, 0u, 0u);
  } else if constexpr (AK == CQ_A_F16 || AK == CQ_A_BF16) {
    r.a = *reinterpret_cast<const uint4*>(reinterpret_cast<const uint16_t*>(A) + e0);
  } else {
    r.a = *reinterpret_cast<const uint4*>(reinterpret_cast<const float*>(A) + e0);
    r.b = *reinterpret_cast<const uint4*>(reinterpret_cast<const float*>(A) + e0 + 4);
  }
  return r;
}

template <int AK>
__device__ __forceinline__ uint4 act_pack8(const ActRaw& r, bool grouped) {
  if constexpr (AK == CQ_A_F16 || AK == CQ_A_BF16) {
    const uint4 v = r.a;
    if (!grouped) return v;
    return make_uint4(__builtin_amdgcn_perm(v.z, v.x, 0x05040100u), __builtin_amdgcn_perm(v.z, v.x, 0x07060302u),
                      __builtin_amdgcn_perm(v.w, v.y, 0x05040100u), __builtin_amdgcn_perm(v.w, v.y, 0x07060302u));
  } else {
    uint32_t c8[8];
    if constexpr (AK == CQ_A_INT8_CODES) {
      const uint32_t rw[2] = {r.a.x, r.a.y};
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        c8[4 * h] = code_to_bf16_bits((int)(int8_t)(rw[h] & 0xff));
        c8[4 * h + 1] = code_to_bf16_bits((int)(int8_t)((rw[h] >> 8) & 0xff));
        c8[4 * h + 2] = code_to_bf16_bits((int)(int8_t)((rw[h] >> 16) & 0xff));
        c8[4 * h + 3] = code_to_bf16_bits((int)(int8_t)(rw[h] >> 24));
      }
    } else {
      const uint32_t f[8] = {r.a.x, r.a.y, r.a.z, r.a.w, r.b.x, r.b.y, r.b.z, r.b.w};
#pragma unroll
      for (int i = 0; i < 8; ++i) c8[i] = f32_to_f16_bits_sat(__uint_as_float(f[i]));
    }
    return grouped ? make_uint4(c8[0] | (c8[4] << 16), c8[1] | (c8[5] << 16), c8[2] | (c8[6] << 16),
                                c8[3] | (c8[7] << 16))
                   : make_uint4(c8[0] | (c8[1] << 16), c8[2] | (c8[3] << 16), c8[4] | (c8[5] << 16),
                                c8[6] | (c8[7] << 16));
  }
}

// The pair table sits at LDS address 0 (the kernel has no static LDS, which the launcher verifies), so
// a table lookup can use the byte offset built by v_perm_b32 as the LDS address itself.
__device__ __forceinline__ uint32_t lds_read_u32(uint32_t byte_offset) {
  return *reinterpret_cast<const __attribute__((address_space(3))) uint32_t*>((uintptr_t)byte_offset);
}

// 16 bytes of the packed-index stream: read once, never reused, so the load carries the non-temporal hint
// (the bytes do not displace the activations, tables and partial sums that do get reused from the caches)
__device__ __forceinline__ uint4 load_stream(const uint8_t* p) {
#if CQ_STREAM_NT
  const cq_v4u v = __builtin_nontemporal_load(reinterpret_cast<const cq_v4u*>(p));
  return make_uint4(v[0], v[1], v[2], v[3]);
#else
  return *reinterpret_cast<const uint4*>(p);
#endif
}

}  // namespace

#endif  // CQ_STREAM_H_
