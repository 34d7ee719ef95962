// a6 / a7 for groups with many tokens (prefill regime, bound by the matrix cores).
//
// Workgroup tile: 256 weight rows x CT tokens (CT = 256 or 128), four wavefronts, each owning 64 rows
// and ALL the tile's tokens (accumulators 2 x CT/32 MFMA blocks of 32x32).  Consequences:
//   * every wavefront decodes only its own rows, straight into MFMA A-operand registers: the decoded
//     weights never touch LDS, and no weight is decoded twice;
//   * a lane owns one row of each of its two 32-row blocks for the whole K loop, so the two 16-entry
//     centroid tables it needs are loop invariant and live in registers.  Decoding is pure vector ALU:
//     nibbles become byte selectors, v_perm_b32 picks the low and the high bytes of the centroids out
//     of register-resident byte tables (two 8-entry halves merged by bit 3 of the index), two more
//     perm levels interleave them into bf16/f16 pairs.  About 4 ALU operations per weight, against
//     CT multiply-adds per weight on the matrix cores;
//   * LDS holds only the activation tile (double buffered, fragment order, conflict-free 16-byte reads)
//     and is read once per wavefront per K step: about 60 % of its bandwidth at full MFMA rate.
// Token tiles come from a device-built work list (groups are ragged and their sizes are only known on
// the device); the list index is remapped so that tiles sharing weights run on the same XCD (L2).
#include <type_traits>

#include "cq_internal.h"

namespace {

constexpr int kLargeRows = 256;  // weight rows per workgroup
constexpr int kStepK = 64;       // K per pipeline step

struct LargeArgs {
  const uint8_t* idx;
  const uint16_t* cent;
  int prepacked;
  int N, K;
  const void* A;
  const float* row_scale;
  const int32_t* row_gather;
  void* out;
  int out_ld;
  const int32_t* tiles;   // [cap][4]: group, first row (absolute sorted row), row count, unused
  const int32_t* n_tiles; // number of entries in tiles
  int row_tiles;          // N / 256
};

__device__ __forceinline__ uint32_t f32_to_f16_sat(float x) {
  x = fminf(fmaxf(x, -65504.f), 65504.f);
  const _Float16 h = (_Float16)x;
  return (uint32_t) __builtin_bit_cast(uint16_t, h);
}
__device__ __forceinline__ uint32_t bf16_to_f16_bits(uint32_t b) {
  const _Float16 h = (_Float16)__uint_as_float(b << 16);
  return (uint32_t) __builtin_bit_cast(uint16_t, h);
}
__device__ __forceinline__ uint32_t code_bf16(int c) { return __float_as_uint((float)c) >> 16; }

// Byte tables of one row's 16 centroids: lo[q] byte j = low byte of entry 4q+j, hi likewise.
struct RowTable {
  uint32_t lo[4], hi[4];
};

template <bool F16>
__device__ __forceinline__ RowTable make_row_table(const uint16_t* crow) {
  const uint4 c0 = reinterpret_cast<const uint4*>(crow)[0];
  const uint4 c1 = reinterpret_cast<const uint4*>(crow)[1];
  uint32_t p[8] = {c0.x, c0.y, c0.z, c0.w, c1.x, c1.y, c1.z, c1.w};  // p[i] = entries 2i (low half), 2i+1
  if constexpr (F16) {
#pragma unroll
    for (int i = 0; i < 8; ++i) p[i] = bf16_to_f16_bits(p[i] & 0xffffu) | (bf16_to_f16_bits(p[i] >> 16) << 16);
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

// 8 packed indices (one dword, weight 2i in the low nibble of byte i) -> 4 dwords of 16-bit pairs
__device__ __forceinline__ cq_v4u decode8(uint32_t d, const RowTable& t) {
  const uint32_t sA = d & 0x07070707u;                 // even weights: selector within a half table
  const uint32_t sB = (d >> 4) & 0x07070707u;          // odd weights
  const uint32_t mA = ((d >> 3) & 0x01010101u) * 0xffu;  // 0xff where bit 3 of the index is set
  const uint32_t mB = ((d >> 7) & 0x01010101u) * 0xffu;
  const uint32_t loA0 = __builtin_amdgcn_perm(t.lo[1], t.lo[0], sA), loA1 = __builtin_amdgcn_perm(t.lo[3], t.lo[2], sA);
  const uint32_t hiA0 = __builtin_amdgcn_perm(t.hi[1], t.hi[0], sA), hiA1 = __builtin_amdgcn_perm(t.hi[3], t.hi[2], sA);
  const uint32_t loB0 = __builtin_amdgcn_perm(t.lo[1], t.lo[0], sB), loB1 = __builtin_amdgcn_perm(t.lo[3], t.lo[2], sB);
  const uint32_t hiB0 = __builtin_amdgcn_perm(t.hi[1], t.hi[0], sB), hiB1 = __builtin_amdgcn_perm(t.hi[3], t.hi[2], sB);
  const uint32_t loA = (mA & loA1) | (~mA & loA0), hiA = (mA & hiA1) | (~mA & hiA0);
  const uint32_t loB = (mB & loB1) | (~mB & loB0), hiB = (mB & hiB1) | (~mB & hiB0);
  // 16-bit values: xa01 = {even0, even1}, xa23 = {even2, even3}; same for the odd weights
  const uint32_t xa01 = __builtin_amdgcn_perm(hiA, loA, 0x05010400u), xa23 = __builtin_amdgcn_perm(hiA, loA, 0x07030602u);
  const uint32_t xb01 = __builtin_amdgcn_perm(hiB, loB, 0x05010400u), xb23 = __builtin_amdgcn_perm(hiB, loB, 0x07030602u);
  cq_v4u o;
  o[0] = __builtin_amdgcn_perm(xb01, xa01, 0x05040100u);  // weights 0,1
  o[1] = __builtin_amdgcn_perm(xb01, xa01, 0x07060302u);  // weights 2,3
  o[2] = __builtin_amdgcn_perm(xb23, xa23, 0x05040100u);  // weights 4,5
  o[3] = __builtin_amdgcn_perm(xb23, xa23, 0x07060302u);  // weights 6,7
  return o;
}

template <bool F16>
__device__ __forceinline__ cq_v16f mfma_large(const cq_v4u a, const cq_v4u b, cq_v16f c) {
  if constexpr (F16)
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(cq_v8f16, a), __builtin_bit_cast(cq_v8f16, b), c,
                                                  0, 0, 0);
  else
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(cq_v8bf16, a),
                                                   __builtin_bit_cast(cq_v8bf16, b), c, 0, 0, 0);
}

// AK: activation kind; C = CT/32 token blocks per workgroup (8 or 4)
template <int AK, int EPI, int OUTK, int C>
__global__ __launch_bounds__(256, 1) void gemm_large_kernel(const LargeArgs p) {
  constexpr bool F16 = (AK == CQ_A_F16 || AK == CQ_A_F32);
  constexpr int CT = 32 * C;
  constexpr int TPT = 256 / CT;          // threads per token when staging
  constexpr int CPT = 8 / TPT;           // 16-byte chunks (8 k) per thread per step
  extern __shared__ uint4 smem[];        // two activation tiles of [8 chunks][CT tokens] x 16 bytes

  // ---- which tile: XCD-aware remap of the linear workgroup id (ids go round-robin over 8 XCDs) ----
  // XCD x takes the contiguous share [x*per_xcd, (x+1)*per_xcd) of the real work items (the grid is
  // sized for the worst case, the list is usually much shorter)
  const int n_work = p.n_tiles[0] * p.row_tiles;
  const int per_xcd = (n_work + 7) >> 3;
  const int slot = blockIdx.x >> 3;
  const int work = (blockIdx.x & 7) * per_xcd + slot;
  if (slot >= per_xcd || work >= n_work) return;
  const int tile = work / p.row_tiles, rt = work - tile * p.row_tiles;
  const int grp = p.tiles[tile * 4 + 0];
  const int mrow0 = p.tiles[tile * 4 + 1];
  const int mcnt = p.tiles[tile * 4 + 2];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int r32 = lane & 31, g2 = lane >> 5;
  const int N = p.N, K = p.K;
  const size_t rowbytes = (size_t)K >> 1;
  const int n0 = rt * kLargeRows + wave * 64;  // this wavefront's 64 rows
  const uint8_t* wbase = p.idx + ((size_t)grp * N + n0) * rowbytes;
  size_t lane_off0, lane_off1;
  int sstride;
  if (p.prepacked) {
    lane_off0 = (size_t)lane * 16;
    lane_off1 = 32 * rowbytes + (size_t)lane * 16;
    sstride = 1024;
  } else {
    lane_off0 = (size_t)r32 * rowbytes + g2 * 16;
    lane_off1 = (size_t)(32 + r32) * rowbytes + g2 * 16;
    sstride = 32;
  }
  const int nS = K / kStepK;

  const uint16_t* cbase = p.cent + ((size_t)grp * N + n0) * CQ_N_CENTROIDS;
  const RowTable t0 = make_row_table<F16>(cbase + (size_t)r32 * CQ_N_CENTROIDS);
  const RowTable t1 = make_row_table<F16>(cbase + (size_t)(32 + r32) * CQ_N_CENTROIDS);

  // ---- activation staging: thread -> (token, part of the 64-wide K step) ----
  const int stok = tid % CT, spart = tid / CT;
  const bool svalid = stok < mcnt;
  size_t srow = 0;
  if (svalid) {
    const int m = mrow0 + stok;
    srow = (p.row_gather ? (size_t)p.row_gather[m] : (size_t)m) * K;
  }
  uint4 sreg[CPT];
  auto stage_load = [&](int s) {
    const size_t e0 = srow + (size_t)s * kStepK + spart * (CPT * 8);
#pragma unroll
    for (int c = 0; c < CPT; ++c) {
      uint4 v = make_uint4(0u, 0u, 0u, 0u);
      if (svalid) {
        if constexpr (AK == CQ_A_F16 || AK == CQ_A_BF16) {
          v = *reinterpret_cast<const uint4*>(reinterpret_cast<const uint16_t*>(p.A) + e0 + c * 8);
        } else if constexpr (AK == CQ_A_INT8_CODES) {
          const uint2 raw = *reinterpret_cast<const uint2*>(reinterpret_cast<const int8_t*>(p.A) + e0 + c * 8);
          v.x = raw.x;
          v.y = raw.y;
        } else {
          const float4 f0 = *reinterpret_cast<const float4*>(reinterpret_cast<const float*>(p.A) + e0 + c * 8);
          const float4 f1 = *reinterpret_cast<const float4*>(reinterpret_cast<const float*>(p.A) + e0 + c * 8 + 4);
          v.x = f32_to_f16_sat(f0.x) | (f32_to_f16_sat(f0.y) << 16);
          v.y = f32_to_f16_sat(f0.z) | (f32_to_f16_sat(f0.w) << 16);
          v.z = f32_to_f16_sat(f1.x) | (f32_to_f16_sat(f1.y) << 16);
          v.w = f32_to_f16_sat(f1.z) | (f32_to_f16_sat(f1.w) << 16);
        }
      }
      sreg[c] = v;
    }
  };
  auto stage_store = [&](int buf) {
    uint4* dst = smem + buf * (8 * CT);
#pragma unroll
    for (int c = 0; c < CPT; ++c) {
      uint4 v = sreg[c];
      if constexpr (AK == CQ_A_INT8_CODES) {
        const uint32_t rw[2] = {v.x, v.y};
        uint32_t o[4];
#pragma unroll
        for (int h = 0; h < 2; ++h) {
          const int b0 = (int)(int8_t)(rw[h] & 0xff), b1 = (int)(int8_t)((rw[h] >> 8) & 0xff);
          const int b2 = (int)(int8_t)((rw[h] >> 16) & 0xff), b3 = (int)(int8_t)(rw[h] >> 24);
          o[2 * h] = code_bf16(b0) | (code_bf16(b1) << 16);
          o[2 * h + 1] = code_bf16(b2) | (code_bf16(b3) << 16);
        }
        v = make_uint4(o[0], o[1], o[2], o[3]);
      }
      dst[(spart * CPT + c) * CT + stok] = v;
    }
  };

  cq_v16f acc[2][C];
#pragma unroll
  for (int rb = 0; rb < 2; ++rb)
#pragma unroll
    for (int cb = 0; cb < C; ++cb)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[rb][cb][i] = 0.f;

  // prologue: activations of step 0 into buffer 0, weights of steps 0 and 1 into registers
  stage_load(0);
  uint4 wq[2][2];
  wq[0][0] = *reinterpret_cast<const uint4*>(wbase + lane_off0);
  wq[0][1] = *reinterpret_cast<const uint4*>(wbase + lane_off1);
  {
    const size_t o1 = (size_t)min(1, nS - 1) * sstride;
    wq[1][0] = *reinterpret_cast<const uint4*>(wbase + lane_off0 + o1);
    wq[1][1] = *reinterpret_cast<const uint4*>(wbase + lane_off1 + o1);
  }
  stage_store(0);
  __syncthreads();

  for (int s0 = 0; s0 < nS; s0 += 2) {
#pragma unroll
    for (int par = 0; par < 2; ++par) {
      const int s = s0 + par;  // K is a multiple of 128 on this path: both halves always exist
      {
        // next step's activations and the weights two steps ahead start their trip now
        stage_load(min(s + 1, nS - 1));
        const uint4 w0 = wq[par][0], w1 = wq[par][1];
        {
          const size_t o2 = (size_t)min(s + 2, nS - 1) * sstride;
          wq[par][0] = *reinterpret_cast<const uint4*>(wbase + lane_off0 + o2);
          wq[par][1] = *reinterpret_cast<const uint4*>(wbase + lane_off1 + o2);
        }
        const uint4* bt = smem + par * (8 * CT);
        const uint32_t wd0[4] = {w0.x, w0.y, w0.z, w0.w};
        const uint32_t wd1[4] = {w1.x, w1.y, w1.z, w1.w};
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
          const cq_v4u a0 = decode8(wd0[jj], t0);
          const cq_v4u a1 = decode8(wd1[jj], t1);
          const uint4* brow = bt + (g2 * 4 + jj) * CT + r32;
#pragma unroll
          for (int cb = 0; cb < C; ++cb) {
            const uint4 bq = brow[cb * 32];
            const cq_v4u b = {bq.x, bq.y, bq.z, bq.w};
            acc[0][cb] = mfma_large<F16>(a0, b, acc[0][cb]);
            acc[1][cb] = mfma_large<F16>(a1, b, acc[1][cb]);
          }
          // keep the four sub-steps apart: hoisting all decodes and fragment reads to the top would
          // cost more registers than the accumulators leave
          __builtin_amdgcn_sched_barrier(0);
        }
        stage_store(par ^ 1);
        __syncthreads();
      }
    }
  }

  // ---- epilogue: per-token scale, optional SiLU(gate)*up, store ----
#pragma unroll
  for (int cb = 0; cb < C; ++cb) {
    const int tok = cb * 32 + r32;
    if (tok < mcnt) {
      const int m = mrow0 + tok;
      float sc = 1.f;
      if (p.row_scale) sc = p.row_scale[p.row_gather ? p.row_gather[m] : m];
#pragma unroll
      for (int rb = 0; rb < 2; ++rb) {
#pragma unroll
        for (int vb = 0; vb < 4; ++vb) {
          // MFMA 32x32 output: register v holds row 8*(v/4) + 4*(lane/32) + v%4, column lane%32
          const int row = n0 + rb * 32 + vb * 8 + g2 * 4;
          const float x0 = sc * acc[rb][cb][4 * vb], x1 = sc * acc[rb][cb][4 * vb + 1];
          const float x2 = sc * acc[rb][cb][4 * vb + 2], x3 = sc * acc[rb][cb][4 * vb + 3];
          if constexpr (EPI == CQ_EPI_SWIGLU) {
            const float h0 = x0 / (1.f + __expf(-x0)) * x1;
            const float h1 = x2 / (1.f + __expf(-x2)) * x3;
            const size_t o = (size_t)m * p.out_ld + (row >> 1);
            if constexpr (OUTK == CQ_OUT_F16)
              *reinterpret_cast<uint32_t*>(reinterpret_cast<uint16_t*>(p.out) + o) =
                  f32_to_f16_sat(h0) | (f32_to_f16_sat(h1) << 16);
            else
              *reinterpret_cast<float2*>(reinterpret_cast<float*>(p.out) + o) = make_float2(h0, h1);
          } else {
            const size_t o = (size_t)m * p.out_ld + row;
            if constexpr (OUTK == CQ_OUT_F16)
              *reinterpret_cast<uint2*>(reinterpret_cast<uint16_t*>(p.out) + o) =
                  make_uint2(f32_to_f16_sat(x0) | (f32_to_f16_sat(x1) << 16),
                             f32_to_f16_sat(x2) | (f32_to_f16_sat(x3) << 16));
            else
              *reinterpret_cast<float4*>(reinterpret_cast<float*>(p.out) + o) = make_float4(x0, x1, x2, x3);
          }
        }
      }
    }
  }
}

// One workgroup: cut every group with more than `small_max` rows into token tiles of 256 (while more
// than 128 rows remain) and 128, in group order (deterministic).  lists: [0] = 256-wide, [1] = 128-wide.
__global__ __launch_bounds__(1024) void build_tiles_kernel(const int32_t* __restrict__ offsets, int G, int small_max,
                                                           int32_t* __restrict__ tiles256, int32_t* __restrict__ tiles128,
                                                           int32_t* __restrict__ counts) {
  __shared__ int n256[1024], n128[1024];
  __shared__ int base256, base128;
  const int tid = threadIdx.x;
  if (tid == 0) { base256 = 0; base128 = 0; }
  __syncthreads();
  for (int g0 = 0; g0 < G; g0 += 1024) {
    const int g = g0 + tid;
    int a = 0, b = 0, m0 = 0, me = 0;
    if (g < G) {
      m0 = offsets[g];
      me = offsets[g + 1] - m0;
      if (me > small_max) {
        a = me / 256;
        const int rem = me - a * 256;
        if (rem > 128) ++a; else if (rem > 0) b = 1;
      }
    }
    n256[tid] = a;
    n128[tid] = b;
    __syncthreads();
    if (tid == 0) {  // exclusive prefix in group order
      int s256 = base256, s128 = base128;
      for (int i = 0; i < 1024; ++i) {
        const int x = n256[i], y = n128[i];
        n256[i] = s256; n128[i] = s128;
        s256 += x; s128 += y;
      }
      base256 = s256; base128 = s128;
    }
    __syncthreads();
    if (g < G && me > small_max) {
      int at = n256[tid];
      for (int i = 0; i < a; ++i) {
        tiles256[(at + i) * 4 + 0] = g;
        tiles256[(at + i) * 4 + 1] = m0 + i * 256;
        tiles256[(at + i) * 4 + 2] = min(256, me - i * 256);
        tiles256[(at + i) * 4 + 3] = 0;
      }
      if (b) {
        const int at2 = n128[tid];
        tiles128[at2 * 4 + 0] = g;
        tiles128[at2 * 4 + 1] = m0 + a * 256;
        tiles128[at2 * 4 + 2] = me - a * 256;
        tiles128[at2 * 4 + 3] = 0;
      }
    }
    __syncthreads();
  }
  if (tid == 0) { counts[0] = base256; counts[1] = base128; }
}

template <int AK, int EPI, int OUTK, int C>
cq_status launch_large(const LargeArgs& a, int max_tiles, hipStream_t s) {
  auto kern = gemm_large_kernel<AK, EPI, OUTK, C>;
  constexpr int lds = 2 * 8 * (32 * C) * 16;
  static bool configured = false;
  if (!configured) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, lds) !=
        hipSuccess)
      return CQ_ERR_HIP;
    configured = true;
  }
  if (max_tiles <= 0) return CQ_OK;
  const int grid = ((max_tiles * a.row_tiles + 7) / 8) * 8;
  hipLaunchKernelGGL(kern, dim3(grid), dim3(256), lds, s, a);
  return cq_check_launch();
}

template <int AK, int EPI, int OUTK>
cq_status launch_both(LargeArgs a, const int32_t* t256, const int32_t* t128, const int32_t* counts, int max256,
                      int max128, hipStream_t s) {
  a.tiles = t256;
  a.n_tiles = counts;
  cq_status st = launch_large<AK, EPI, OUTK, 8>(a, max256, s);
  if (st != CQ_OK) return st;
  a.tiles = t128;
  a.n_tiles = counts + 1;
  return launch_large<AK, EPI, OUTK, 4>(a, max128, s);
}

template <int AK>
cq_status dispatch_large(const LargeArgs& a, int epilogue, int out_kind, const int32_t* t256, const int32_t* t128,
                         const int32_t* counts, int max256, int max128, hipStream_t s) {
  if (epilogue == CQ_EPI_SWIGLU)
    return out_kind == CQ_OUT_F16 ? launch_both<AK, CQ_EPI_SWIGLU, CQ_OUT_F16>(a, t256, t128, counts, max256, max128, s)
                                  : launch_both<AK, CQ_EPI_SWIGLU, CQ_OUT_F32>(a, t256, t128, counts, max256, max128, s);
  return out_kind == CQ_OUT_F16 ? launch_both<AK, CQ_EPI_NONE, CQ_OUT_F16>(a, t256, t128, counts, max256, max128, s)
                                : launch_both<AK, CQ_EPI_NONE, CQ_OUT_F32>(a, t256, t128, counts, max256, max128, s);
}

}  // namespace

// Upper bounds on the tile counts for M_total rows in G groups (host side; sizes on the device vary).
void cq_large_tile_caps(int G, int M_total, int* cap256, int* cap128) {
  *cap256 = M_total / 129 + 1;   // every 256-wide tile covers more than 128 rows
  *cap128 = G < M_total ? G : M_total;  // at most one per group
  if (*cap128 < 1) *cap128 = 1;
}

size_t cq_gemm_large_workspace_bytes(int G, int M_total) {
  int c256, c128;
  cq_large_tile_caps(G, M_total, &c256, &c128);
  return cq_align_up(256 + (size_t)(c256 + c128) * 4 * sizeof(int32_t), 256);
}

bool cq_gemm_large_supported(const cq_codebook_weights* W) {
  return W->N % kLargeRows == 0 && W->K % (2 * kStepK) == 0;
}

cq_status cq_gemm_large_launch(const cq_codebook_weights* W, const void* A, int a_kind, const float* row_scale,
                               const int32_t* row_gather, const int32_t* group_offsets, int M_total, int small_max,
                               int epilogue, void* out, int out_kind, void* workspace, hipStream_t s) {
  int cap256, cap128;
  cq_large_tile_caps(W->G, M_total, &cap256, &cap128);
  int32_t* counts = (int32_t*)workspace;
  int32_t* t256 = counts + 64;
  int32_t* t128 = t256 + (size_t)cap256 * 4;
  hipLaunchKernelGGL(build_tiles_kernel, dim3(1), dim3(1024), 0, s, group_offsets, W->G, small_max, t256, t128, counts);
  LargeArgs a;
  a.idx = W->prepacked ? (const uint8_t*)W->prepacked : W->idx;
  a.cent = W->cent;
  a.prepacked = W->prepacked ? 1 : 0;
  a.N = W->N;
  a.K = W->K;
  a.A = A;
  a.row_scale = row_scale;
  a.row_gather = row_gather;
  a.out = out;
  a.out_ld = epilogue == CQ_EPI_SWIGLU ? W->N / 2 : W->N;
  a.tiles = nullptr;
  a.n_tiles = nullptr;
  a.row_tiles = W->N / kLargeRows;
  switch (a_kind) {
    case CQ_A_INT8_CODES:
      return dispatch_large<CQ_A_INT8_CODES>(a, epilogue, out_kind, t256, t128, counts, cap256, cap128, s);
    case CQ_A_F16: return dispatch_large<CQ_A_F16>(a, epilogue, out_kind, t256, t128, counts, cap256, cap128, s);
    case CQ_A_BF16: return dispatch_large<CQ_A_BF16>(a, epilogue, out_kind, t256, t128, counts, cap256, cap128, s);
    default: return dispatch_large<CQ_A_F32>(a, epilogue, out_kind, t256, t128, counts, cap256, cap128, s);
  }
}
