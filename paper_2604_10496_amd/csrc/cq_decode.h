// Register-resident decoding of packed 4-bit indices (Eq. W_c): shared by the HIP kernels of libcq.
#ifndef CQ_DECODE_H_
#define CQ_DECODE_H_

#include "cq_internal.h"

__device__ __forceinline__ uint32_t cq_bf16_to_f16_bits(uint32_t b) {
  const _Float16 h = (_Float16)__uint_as_float(b << 16);
  return (uint32_t) __builtin_bit_cast(uint16_t, h);
}

// Byte tables of one row's 16 centroids: lo[q] byte j = low byte of entry 4q+j, hi likewise.
struct RowTable {
  uint32_t lo[4], hi[4];
};

// p[i] = centroid entries 2i (low half) and 2i+1 as bf16 bits
template <bool F16>
__device__ __forceinline__ RowTable make_row_table(uint32_t (&p)[8]) {
  if constexpr (F16) {
#pragma unroll
    for (int i = 0; i < 8; ++i) p[i] = cq_bf16_to_f16_bits(p[i] & 0xffffu) | (cq_bf16_to_f16_bits(p[i] >> 16) << 16);
  }
  RowTable t;
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    // entries 4q..4q+3 live in p[2q] (4q, 4q+1) and p[2q+1] (4q+2, 4q+3)
    t.lo[q] = __builtin_amdgcn_perm(p[2 * q + 1], p[2 * q], 0x06040200u);
    t.hi[q] = __builtin_amdgcn_perm(p[2 * q + 1], p[2 * q], 0x07050301u);
  }
  return t;
}

template <bool F16>
__device__ __forceinline__ RowTable make_row_table(const uint16_t* crow) {
  const uint4 c0 = reinterpret_cast<const uint4*>(crow)[0];
  const uint4 c1 = reinterpret_cast<const uint4*>(crow)[1];
  uint32_t p[8] = {c0.x, c0.y, c0.z, c0.w, c1.x, c1.y, c1.z, c1.w};
  return make_row_table<F16>(p);
}

// 8 packed indices (one dword) -> 4 dwords of 16-bit pairs.  GROUPED = false: canonical bytes (weight 2i in
// the low nibble of byte i, 2i+1 in the high one).  GROUPED = true: the prepacked arrangement (weight i in the
// low nibble of byte i, weight i+4 in the high one): the two nibble planes are then the first and the second
// four weights, and the final re-pairing of even and odd weights falls away.
// ident: the byte selector 0x03020100 held in a vector register (the merge selector is then one
// v_and_or_b32; two constants in scalar registers would not fit one instruction).
template <bool GROUPED>
__device__ __forceinline__ cq_v4u decode8(uint32_t d, const RowTable& t, uint32_t ident) {
  // selectors within a half table: low nibbles (even weights, or weights 0..3), high nibbles (odd, or 4..7)
  const uint32_t sA = d & 0x07070707u;
  const uint32_t sB = (d >> 4) & 0x07070707u;
  // bit 3 of an index picks the upper half table: as a byte selector, byte i of the result comes from
  // the lower-half candidate (source bytes 0-3) or the upper-half one (bytes 4-7)
  const uint32_t mA = ((d >> 1) & 0x04040404u) | ident;
  const uint32_t mB = ((d >> 5) & 0x04040404u) | ident;
  const uint32_t loA0 = __builtin_amdgcn_perm(t.lo[1], t.lo[0], sA), loA1 = __builtin_amdgcn_perm(t.lo[3], t.lo[2], sA);
  const uint32_t hiA0 = __builtin_amdgcn_perm(t.hi[1], t.hi[0], sA), hiA1 = __builtin_amdgcn_perm(t.hi[3], t.hi[2], sA);
  const uint32_t loB0 = __builtin_amdgcn_perm(t.lo[1], t.lo[0], sB), loB1 = __builtin_amdgcn_perm(t.lo[3], t.lo[2], sB);
  const uint32_t hiB0 = __builtin_amdgcn_perm(t.hi[1], t.hi[0], sB), hiB1 = __builtin_amdgcn_perm(t.hi[3], t.hi[2], sB);
  const uint32_t loA = __builtin_amdgcn_perm(loA1, loA0, mA), hiA = __builtin_amdgcn_perm(hiA1, hiA0, mA);
  const uint32_t loB = __builtin_amdgcn_perm(loB1, loB0, mB), hiB = __builtin_amdgcn_perm(hiB1, hiB0, mB);
  // 16-bit values: xa01 = {low-nibble weights 0, 1}, xa23 = {2, 3}; same for the high-nibble weights
  const uint32_t xa01 = __builtin_amdgcn_perm(hiA, loA, 0x05010400u), xa23 = __builtin_amdgcn_perm(hiA, loA, 0x07030602u);
  const uint32_t xb01 = __builtin_amdgcn_perm(hiB, loB, 0x05010400u), xb23 = __builtin_amdgcn_perm(hiB, loB, 0x07030602u);
  if constexpr (GROUPED) return cq_v4u{xa01, xa23, xb01, xb23};
  cq_v4u o;
  o[0] = __builtin_amdgcn_perm(xb01, xa01, 0x05040100u);  // weights 0,1
  o[1] = __builtin_amdgcn_perm(xb01, xa01, 0x07060302u);  // weights 2,3
  o[2] = __builtin_amdgcn_perm(xb23, xa23, 0x05040100u);  // weights 4,5
  o[3] = __builtin_amdgcn_perm(xb23, xa23, 0x07060302u);  // weights 6,7
  return o;
}

#endif  // CQ_DECODE_H_
