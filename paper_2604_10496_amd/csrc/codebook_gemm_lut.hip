// a6 / a7 in the lookup formulation of the kernel section, in software: for every group of weights that
// shares a centroid table (a row, or g consecutive weights of a row) the 16 x 16 table of products
// centroid x 4-bit activation value is precomputed, and a (weight index, activation code) pair then selects
// one product, which is accumulated -- no multiplication in the inner loop.
//
// This is the comparison path for the matrix-core kernels (codebook_gemm_small.h, codebook_gemm_large.hip), built
// to measure what the paper's scheme costs on gfx950 without its hardware changes: every multiply-accumulate
// becomes one LDS read plus one addition, so the kernel is bound by the LDS read rate (64 lanes every two
// clocks per compute unit), far below the matrix cores.
//
// One workgroup of four wavefronts per (group of tokens, 64 weight rows).  lane = row slot.  The product
// tables of the 64 rows sit in LDS entry-major: product (centroid c, value v) of row slot r is the float at
// ((c*16 + v)*64 + r): whatever the indices and codes are, the 64 lanes of a read hit the 32 banks evenly
// (bank = row slot mod 32), which removes the conflicts the paper adds banks for.  The wavefronts split K
// (32 weights per step, step s to wavefront s mod 4); tokens are taken 8 at a time (4 when no more are left),
// their codes are the same for all lanes and live in scalar registers.  Partial sums of the four wavefronts
// are added in a fixed order.
#include <type_traits>

#include "cq_internal.h"

namespace {

constexpr int kLutTok = 8;                         // tokens per pass over the weights
constexpr int kLutTableFloats = 256 * 64;          // 64 KiB
constexpr int kLutRedFloats = 4 * kLutTok * 64;    // 8 KiB
constexpr int kLutLdsBytes = (kLutTableFloats + kLutRedFloats) * 4;

struct LutArgs {
  const uint8_t* idx;   // canonical [G, N, K/2]
  const uint16_t* cent; // [G, N, nblk, 16] bf16
  int nblk, group_k;    // tables per row and weights per table (group_k = K when nblk == 1)
  int N, K;
  const int8_t* A;      // [rows, K] codes in [-8, 7]
  const float* row_scale;
  const int32_t* row_gather;
  const int32_t* group_offsets;
  void* out;
  int out_ld;
};

__device__ __forceinline__ uint32_t lut_f16_bits_sat(float x) {
  x = fminf(fmaxf(x, -65504.f), 65504.f);
  const _Float16 h = (_Float16)x;
  return (uint32_t) __builtin_bit_cast(uint16_t, h);
}

template <int EPI, int OUTK>
__global__ __launch_bounds__(256, 2) void gemm_lut_kernel(const LutArgs p) {
  extern __shared__ float lut_lds[];
  float* lut = lut_lds;
  float* red = lut_lds + kLutTableFloats;   // [wavefront][token][row slot]
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int grp = blockIdx.y;
  const int m0 = p.group_offsets[grp], Me = p.group_offsets[grp + 1] - m0;
  if (Me <= 0) return;
  const int N = p.N, K = p.K;
  const int row = blockIdx.x * 64 + lane;
  const uint8_t* wrow = p.idx + ((size_t)grp * N + row) * ((size_t)K >> 1);
  const uint16_t* crow = p.cent + ((size_t)grp * N + row) * p.nblk * CQ_N_CENTROIDS;
  const char* lut_bytes = reinterpret_cast<const char*>(lut);
  const uint32_t slot = (uint32_t)lane * 4;

  // one pass over the weights for the tokens tb .. tb + TOK - 1 of the group (TOK = 8, or 4 when no more are left)
  auto pass = [&](auto tok_tag, const int tb) {
    constexpr int TOK = decltype(tok_tag)::value;
    const int Mb = min(TOK, Me - tb);
    // tokens past the end of the group repeat its last token (their sums are not stored): no branches below
    const int8_t* arow[TOK];
#pragma unroll
    for (int t = 0; t < TOK; ++t) {
      const int m = m0 + tb + min(t, Mb - 1);
      arow[t] = p.A + (size_t)(p.row_gather ? p.row_gather[m] : m) * K;
    }
    float acc[TOK];
#pragma unroll
    for (int t = 0; t < TOK; ++t) acc[t] = 0.f;

    for (int b = 0; b < p.nblk; ++b) {
      const int j0 = b * p.group_k, j1 = min(K, j0 + p.group_k);
      __syncthreads();  // the previous table is no longer read (nor the previous pass's partial sums)
      // product tables of this group of weights: wavefront w fills the sub-tables of centroids 4w .. 4w+3
#pragma unroll
      for (int ci = 0; ci < 4; ++ci) {
        const int c = wave * 4 + ci;
        const float cv = __uint_as_float((uint32_t)crow[b * CQ_N_CENTROIDS + c] << 16);
#pragma unroll
        for (int v = 0; v < 16; ++v) lut[(c * 16 + v) * 64 + lane] = cv * (float)(v - 8);  // exact in fp32
      }
      __syncthreads();
      const int nsteps = (j1 - j0) >> 5;
      for (int s = wave; s < nsteps; s += 4) {
        const int k0 = j0 + (s << 5);
        const uint4 w = *reinterpret_cast<const uint4*>(wrow + (k0 >> 1));
        const uint32_t wd[4] = {w.x, w.y, w.z, w.w};
        // The 32 codes of every token are the same in all lanes: they go to scalar registers, so that the
        // table offset of a code is scalar arithmetic.  Value v = q + 8 selects within a sub-table, and
        // (q ^ 8) & 15 = (q + 8) mod 16.
        uint32_t cd[TOK][8];
#pragma unroll
        for (int t = 0; t < TOK; ++t) {
          const uint4 c0 = *reinterpret_cast<const uint4*>(arow[t] + k0);
          const uint4 c1 = *reinterpret_cast<const uint4*>(arow[t] + k0 + 16);
          const uint32_t raw[8] = {c0.x, c0.y, c0.z, c0.w, c1.x, c1.y, c1.z, c1.w};
#pragma unroll
          for (int i = 0; i < 8; ++i)
            cd[t][i] = (__builtin_amdgcn_readfirstlane(raw[i]) ^ 0x08080808u) & 0x0f0f0f0fu;
        }
#pragma unroll
        for (int d = 0; d < 4; ++d) {
#pragma unroll
          for (int i = 0; i < 8; ++i) {  // weight 8d + i of the step: bits 4i .. 4i+3 of dword d
            const uint32_t at = (((wd[d] >> (4 * i)) & 15u) << 12) | slot;
            const int kk = 8 * d + i;
#pragma unroll
            for (int t = 0; t < TOK; ++t) {
              const uint32_t v = (cd[t][kk >> 2] >> (8 * (kk & 3))) & 15u;
              acc[t] += *reinterpret_cast<const float*>(lut_bytes + (at | (v << 8)));
            }
          }
        }
      }
    }
    // ---- the four partial sums of every (token, row), added in wavefront order ----
#pragma unroll
    for (int t = 0; t < TOK; ++t) red[(wave * kLutTok + t) * 64 + lane] = acc[t];
    __syncthreads();
    for (int t = wave; t < Mb; t += 4) {  // (uniform per wavefront)
      float sum = red[t * 64 + lane];
#pragma unroll
      for (int wv = 1; wv < 4; ++wv) sum += red[(wv * kLutTok + t) * 64 + lane];
      const int m = m0 + tb + t;
      const float sc = p.row_scale ? p.row_scale[p.row_gather ? p.row_gather[m] : m] : 1.f;
      const float x = sc * sum;
      if constexpr (EPI == CQ_EPI_SWIGLU) {
        // rows 2i (gate) and 2i+1 (up) sit in neighbouring lanes
        const float other = __shfl_xor(x, 1);
        if ((lane & 1) == 0) {
          const float h = x / (1.f + __expf(-x)) * other;
          const size_t o = (size_t)m * p.out_ld + (row >> 1);
          if constexpr (OUTK == CQ_OUT_F16) reinterpret_cast<uint16_t*>(p.out)[o] = (uint16_t)lut_f16_bits_sat(h);
          else reinterpret_cast<float*>(p.out)[o] = h;
        }
      } else {
        const size_t o = (size_t)m * p.out_ld + row;
        if constexpr (OUTK == CQ_OUT_F16) reinterpret_cast<uint16_t*>(p.out)[o] = (uint16_t)lut_f16_bits_sat(x);
        else reinterpret_cast<float*>(p.out)[o] = x;
      }
    }
  };
  for (int tb = 0; tb < Me; tb += kLutTok) {
    if (Me - tb <= kLutTok / 2) pass(std::integral_constant<int, kLutTok / 2>{}, tb);
    else pass(std::integral_constant<int, kLutTok>{}, tb);
  }
}

template <int EPI, int OUTK>
cq_status launch_lut(const LutArgs& a, int G, hipStream_t s) {
  auto kern = gemm_lut_kernel<EPI, OUTK>;
  static std::atomic<bool> configured{false};
  const cq_status cst = cq_configure_lds(kern, kLutLdsBytes, configured, false);
  if (cst != CQ_OK) return cst;
  hipLaunchKernelGGL(kern, dim3(a.N / 64, G), dim3(256), kLutLdsBytes, s, a);
  return cq_check_launch();
}

}  // namespace

extern "C" cq_status cq_codebook_grouped_gemm_lut(const cq_codebook_weights* W, const int8_t* codes,
                                                  const float* row_scale, const int32_t* row_gather,
                                                  const int32_t* group_offsets, int M_total, int epilogue, void* out,
                                                  int out_kind, cq_stream stream) {
  if (!W || !codes || !group_offsets || (!out && M_total > 0)) return CQ_ERR_NULL;
  if (!W->idx || !W->cent) return CQ_ERR_NULL;  // canonical index bytes are read (not the prepacked copy)
  if (W->G <= 0 || W->N <= 0 || W->K <= 0 || M_total < 0 || W->group_k < 0) return CQ_ERR_SHAPE;
  if (W->N % 64 != 0 || W->K % 64 != 0 || W->G > 65535) return CQ_ERR_SHAPE;
  if (cq_tables_per_row(W) > 1 && W->group_k % 32 != 0) return CQ_ERR_SHAPE;
  if (epilogue != CQ_EPI_NONE && epilogue != CQ_EPI_SWIGLU) return CQ_ERR_UNSUPPORTED;
  if (out_kind != CQ_OUT_F32 && out_kind != CQ_OUT_F16) return CQ_ERR_UNSUPPORTED;
  if (M_total == 0) return CQ_OK;
  LutArgs a;
  a.idx = W->idx;
  a.cent = W->cent;
  a.nblk = cq_tables_per_row(W);
  a.group_k = a.nblk > 1 ? W->group_k : W->K;
  a.N = W->N;
  a.K = W->K;
  a.A = codes;
  a.row_scale = row_scale;
  a.row_gather = row_gather;
  a.group_offsets = group_offsets;
  a.out = out;
  a.out_ld = epilogue == CQ_EPI_SWIGLU ? W->N / 2 : W->N;
  hipStream_t s = (hipStream_t)stream;
  if (epilogue == CQ_EPI_SWIGLU)
    return out_kind == CQ_OUT_F16 ? launch_lut<CQ_EPI_SWIGLU, CQ_OUT_F16>(a, W->G, s)
                                  : launch_lut<CQ_EPI_SWIGLU, CQ_OUT_F32>(a, W->G, s);
  return out_kind == CQ_OUT_F16 ? launch_lut<CQ_EPI_NONE, CQ_OUT_F16>(a, W->G, s)
                                : launch_lut<CQ_EPI_NONE, CQ_OUT_F32>(a, W->G, s);
}
