// a6 / a7 for the smallest centroid budget of the ablation on centroid budgets (W2: four centroids per weight
// row, Eq. W_c with four columns in C), streaming the 2-bit indices as they are stored -- half the bytes of the
// 4-bit format -- for decode-sized groups.
//
// A byte of the index stream holds FOUR weights, so a byte has 256 possible decoded quadruples per row.  The
// workgroup keeps, for each of the 32 rows of a unit, the table of those quadruples (8 bytes: four 16-bit
// operands) in LDS, entry-major: entry b of row slot r at b*256 + r*8.  One v_perm_b32 forms the address, one
// ds_read_b64 returns four MFMA operands: half the instructions per weight of the pair table of the 4-bit
// kernel, which is what lets the kernel follow the halved byte stream.  A wavefront's lookups hit different
// banks whatever the indices are (the bank depends on the row slot only).
// Structure as in the pipelined loop of the 4-bit kernel (codebook_gemm_small.h): 8 wavefronts split K (one step =
// 128 weights of 32 rows = one 16-byte load per lane; lane (r, g) holds row r, weights [128 s + 64 g, +64));
// the activations of a wavefront's own K steps stay in registers; LDS holds two tables (2 x 64 KiB) and two
// buffers of K partials; while unit u is looked up, the table of unit u+1 is written and unit u-1 is finished;
// one barrier per unit.  A unit has 32 rows (its table fills 64 KiB), so the unit loop is unrolled twice and
// the ring holds the steps of two units.
// MFMA: v_mfma_f32_16x16x32.  Two looked-up bytes are one A fragment (8 consecutive weights); of the four
// bytes of a dword, bytes 0-1 and bytes 2-3 form the fragments x and y whose dwords v_permlane16_swap sorts into
// the row halves (rows 0-15, rows 16-31): lane rows then carry the k groups (g, fragment) in the order
// x(g=0), y(g=0), x(g=1), y(g=1), and the B operand is held in that order.
#include <type_traits>

#include "cq_internal.h"
#include "cq_route.h"
#include "cq_stream.h"

namespace {

constexpr int kW2Table = 65536;     // 256 entries x 32 row slots x 8 bytes
constexpr int kW2Red = 8192;        // K partials of a unit: 8 wavefronts x 8 registers x 32 columns x 4 bytes
constexpr int kW2Lds = 2 * kW2Table + 2 * kW2Red;
constexpr int kW2Waves = 8;

struct W2Args {
  const uint8_t* idx;       // canonical or prepacked 2-bit stream, group-major
  const uint16_t* cent;     // [G, N, 4]
  int prepacked;
  int N, K;
  const void* A;
  const float* row_scale;
  const int32_t* row_gather;
  const int32_t* group_offsets;
  void* out;
  int out_ld;
  cq_route_fuse route;      // grouping by expert folded into the launch (cq_route::group_rows_from_ids), else ids == NULL
  int upw;                  // 32-row units per workgroup
  int ksplit;               // K ranges (blockIdx.z); > 1: scaled fp32 partial sums go to `partials`
  float* partials;          // [ksplit][M_total][N]
  size_t part_stride;
};

typedef __attribute__((__vector_size__(2 * sizeof(uint32_t)))) uint32_t w2_v2u;
typedef __attribute__((address_space(3))) w2_v2u w2_lds_v2u;

__device__ __forceinline__ uint2 lds_read_u64(uint32_t byte_offset) {
  const w2_v2u v = *reinterpret_cast<const w2_lds_v2u*>((uintptr_t)byte_offset);
  return make_uint2(v[0], v[1]);
}

// Q = K steps (of 128) per wavefront and unit: 4 (a K range of 4096) or 7 (7168).
template <int AK, int EPI, int OUTK, int Q>
__global__ __launch_bounds__(64 * kW2Waves, 1) void gemm_w2_kernel(const W2Args p) {
  constexpr bool F16 = (AK == CQ_A_F16);
  constexpr int NW = kW2Waves;
  constexpr uint32_t kRed = 2 * kW2Table;
  // the ring holds the K steps of RU units: two for short K ranges (64 KiB in flight per compute unit at Q = 4),
  // one for long ones (56 KiB at Q = 7; a second unit's worth of slots would not fit the register file)
  constexpr int RU = Q >= 6 ? 1 : 2;
  typedef __attribute__((ext_vector_type(2))) unsigned pair_u32;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int r32 = lane & 31, g2 = lane >> 5, i16 = lane & 15, g4 = lane >> 4;
  const int N = p.N, K = p.K;
  const int grp = blockIdx.y;
  int m0, Me, row_token = 0;
  const bool fused = p.route.ids != nullptr;
  if (fused) {
    cq_route::group_rows_from_ids(p.route, grp, lane,
                                  blockIdx.x == 0 && blockIdx.y == 0 && blockIdx.z == 0 && wave == 0, m0, Me, row_token);
  } else {
    m0 = p.group_offsets[grp];
    Me = p.group_offsets[grp + 1] - m0;
  }
  if (Me <= 0) return;
  const int nUnits = N >> 5;
  const int ustep = gridDim.x, ufirst = blockIdx.x;   // a group's workgroups interleave its units
  if (ufirst >= nUnits) return;
  const int ucnt = (nUnits - ufirst + ustep - 1) / ustep;
  const size_t rowbytes = (size_t)K >> 2;
  const size_t ubytes = 32 * rowbytes;                // index bytes of one unit
  const int sb = blockIdx.z * (Q * NW);               // first K step of this workgroup's range
  const int sstride = p.prepacked ? 1024 : 32;        // bytes from one K step to the next
  const uint32_t loff = p.prepacked ? (uint32_t)lane * 16u : (uint32_t)r32 * (uint32_t)rowbytes + (uint32_t)g2 * 16u;
  const uint8_t* const kbase = p.idx + (size_t)grp * N * rowbytes + (size_t)sb * sstride;
  const uint32_t slot = (uint32_t)(g4 * 8 + (i16 & 7));

  // selector of this lane's constant high half of a table entry: wavefront w, lane half hh writes the entries
  // e = 32 w + 16 hh + i, whose weights 2, 3 are the centroids x & 3 and x >> 2 of x = 2 w + hh
  const uint32_t xh = (uint32_t)(2 * wave + g2);
  const uint32_t selhi = (2u * (xh & 3u)) | ((2u * (xh & 3u) + 1u) << 8) | ((2u * (xh >> 2)) << 16) |
                         ((2u * (xh >> 2) + 1u) << 24);
  const uint32_t twbase = (uint32_t)(wave * 8192 + g2 * 4096 + r32 * 8);   // this lane's first entry, row slot r32

  // the four centroids of row r32 of a unit, as two dwords (bf16 pairs)
  auto cent_req = [&](int u, uint32_t& c01, uint32_t& c23) {
    const uint2 v = *reinterpret_cast<const uint2*>(p.cent + ((size_t)grp * N + (size_t)u * 32 + r32) * 4);
    c01 = v.x;
    c23 = v.y;
  };
  // this lane's 16 entries of a unit's table (table at LDS offset tb)
  auto table_part = [&](uint32_t c01, uint32_t c23, const uint32_t tb, const int i0, const int i1) {
    if constexpr (F16) {
      c01 = bf16_bits_to_f16_bits(c01 & 0xffffu) | (bf16_bits_to_f16_bits(c01 >> 16) << 16);
      c23 = bf16_bits_to_f16_bits(c23 & 0xffffu) | (bf16_bits_to_f16_bits(c23 >> 16) << 16);
    }
    const uint32_t hi = __builtin_amdgcn_perm(c23, c01, selhi);
#pragma unroll
    for (int i = i0; i < i1; ++i) {
      const uint32_t a = i & 3, b = i >> 2;   // weights 0, 1 of the entry
      const uint32_t sel = (2u * a) | ((2u * a + 1u) << 8) | ((2u * b) << 16) | ((2u * b + 1u) << 24);
      const uint32_t lo = __builtin_amdgcn_perm(c23, c01, sel);
      *reinterpret_cast<w2_lds_v2u*>((uintptr_t)(tb + twbase + (uint32_t)(i * 256))) = w2_v2u{lo, hi};
    }
  };

  const int n_tb = (Me + 7) >> 3;
  for (int tb = 0; tb < n_tb; ++tb) {   // blocks of 8 tokens (a decode-sized group is one block)
    const int Mb = min(8, Me - 8 * tb);
    const int tcol = i16 & 7;
    const bool tok = tcol < Mb;
    // -- prologue: ring (the steps of the first two units), centroids, activations, first table
    uint4 ring[RU * Q];
#pragma unroll
    for (int h = 0; h < RU; ++h) {
      const uint8_t* wb = kbase + (size_t)(ufirst + (h < ucnt ? h : 0) * ustep) * ubytes;
#pragma unroll
      for (int q = 0; q < Q; ++q) ring[h * Q + q] = load_stream(wb + (size_t)(wave + NW * q) * sstride + loff);
    }
    // centroid rows: set P holds those of a unit of parity P; a unit requests the rows of the unit two ahead into
    // its own set at its top (its own table is built by then) and builds the next unit's table from the other set,
    // which was requested one whole unit earlier -- waiting for it never waits for the younger half of the ring
    uint32_t c01[2], c23[2];
    cent_req(ufirst, c01[0], c23[0]);
    cent_req(ufirst + (1 < ucnt ? ustep : 0), c01[1], c23[1]);
    __builtin_amdgcn_sched_barrier(0);
    float sc16 = 1.f;
    size_t arow = 0;
    const int col_token = __shfl(row_token, 8 * tb + tcol);   // (folded grouping: the token of this lane's column)
    if (tok) {
      const int m = m0 + 8 * tb + tcol;
      const size_t src = fused ? (size_t)col_token : p.row_gather ? (size_t)p.row_gather[m] : (size_t)m;
      arow = src * K;
      if (p.row_scale) sc16 = p.row_scale[src];
    }
    // B fragments of step q: register set j holds fragment pair 2j in the lanes of token columns 0..7 and pair
    // 2j+1 (of token column - 8) in the lanes of columns 8..15; a rotation by 8 inside each row of 16 lanes brings
    // the odd pair into place.  Pair pr of step s, lane group g: the 8 activations from k = 8 * (16 s + 2 pr +
    // g % 2 + 8 * (g / 2)).
    cq_v4u breg[Q][2];
    {
      ActRaw raw[Q][2];
#pragma unroll
      for (int q = 0; q < Q; ++q)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          const int chunk = (sb + wave + NW * q) * 16 + 2 * (2 * j + (i16 >> 3)) + (g4 & 1) + 8 * (g4 >> 1);
          raw[q][j] = act_load8<AK>(p.A, arow + (size_t)chunk * 8);
        }
#pragma unroll
      for (int q = 0; q < Q; ++q)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          const uint4 v = tok ? act_pack8<AK>(raw[q][j], false) : make_uint4(0u, 0u, 0u, 0u);
          breg[q][j] = cq_v4u{v.x, v.y, v.z, v.w};
        }
    }
    table_part(c01[0], c23[0], 0u, 0, 16);
    __syncthreads();

    // finish of a unit: wavefronts 0..3 add up accumulator registers 2w, 2w+1 (a gate/up pair of rows) of all
    // wavefronts' partials in buffer pb, in wavefront order (spreading this over all eight wavefronts, half the
    // token columns each, measured 5 % slower)
    auto finish = [&](const int uu, const uint32_t pb) {
      if (wave < 4 && i16 < 8) {
        const uint32_t rb0 = kRed + pb * kW2Red + (uint32_t)(2 * wave) * 128u + slot * 4u;
        float val[2];
#pragma unroll
        for (int i = 0; i < 2; ++i) {
          float sum = __uint_as_float(lds_read_u32(rb0 + (uint32_t)(i * 128)));
#pragma unroll
          for (int w = 1; w < NW; ++w) sum += __uint_as_float(lds_read_u32(rb0 + (uint32_t)(w * 1024 + i * 128)));
          val[i] = sum;
        }
        if (tok) {
          const int m = m0 + 8 * tb + i16;
          // register r = 4 * (row half) + v holds row 16 * (row half) + 4 * (lane / 16) + v of the unit
          const int r = 2 * wave;
          const int row = uu * 32 + (r >> 2) * 16 + g4 * 4 + (r & 3);
          const float x0 = sc16 * val[0], x1 = sc16 * val[1];
          if (p.ksplit > 1) {  // partial sum of this K range (CQ_EPI_NONE only)
            float* dst = p.partials + (size_t)blockIdx.z * p.part_stride + (size_t)m * N + row;
            *reinterpret_cast<float2*>(dst) = make_float2(x0, x1);
          } else if constexpr (EPI == CQ_EPI_SWIGLU) {
            const float h0 = x0 / (1.f + __expf(-x0)) * x1;
            const size_t o = (size_t)m * p.out_ld + (row >> 1);
            if constexpr (OUTK == CQ_OUT_F16)
              reinterpret_cast<uint16_t*>(p.out)[o] = (uint16_t)f32_to_f16_bits_sat(h0);
            else
              reinterpret_cast<float*>(p.out)[o] = h0;
          } else {
            const size_t o = (size_t)m * p.out_ld + row;
            if constexpr (OUTK == CQ_OUT_F16)
              *reinterpret_cast<uint32_t*>(reinterpret_cast<uint16_t*>(p.out) + o) =
                  f32_to_f16_bits_sat(x0) | (f32_to_f16_bits_sat(x1) << 16);
            else
              *reinterpret_cast<float2*>(reinterpret_cast<float*>(p.out) + o) = make_float2(x0, x1);
          }
        }
      }
    };

    // one unit: `half` (a constant once unrolled) is the unit's parity = its table, its partial buffer and its half
    // of the ring
    auto unit = [&](auto half_tag, const int ui) {
      constexpr int HALF = decltype(half_tag)::value;
      const int u = ufirst + ui * ustep;
      // the ring slots of this unit are refilled with the unit RU ahead (clamped to this unit at the end: cache hits)
      const uint8_t* wb2 = kbase + (size_t)(ui + RU < ucnt ? u + RU * ustep : u) * ubytes;
      constexpr int R0 = RU == 2 ? HALF * Q : 0;
      cent_req(ui + 2 < ucnt ? u + 2 * ustep : u, c01[HALF], c23[HALF]);
      __builtin_amdgcn_sched_barrier(0);
      const uint32_t lbase = (uint32_t)(r32 * 8) | ((uint32_t)HALF << 16);
      cq_v4f acc[2] = {cq_v4f{0.f, 0.f, 0.f, 0.f}, cq_v4f{0.f, 0.f, 0.f, 0.f}};
#pragma unroll
      for (int q = 0; q < Q; ++q) {
        if ((q ^ (wave >> 2)) & 1) __builtin_amdgcn_s_setprio(1);   // the two wavefronts of a SIMD take turns
        else __builtin_amdgcn_s_setprio(0);
        const uint4 w = ring[R0 + q];
        const uint32_t wd[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
        for (int pr = 0; pr < 4; ++pr) {
          cq_v4u bv = breg[q][pr >> 1];
          if (pr & 1) {
#pragma unroll
            for (int i = 0; i < 4; ++i)   // row_ror:8
              bv[i] = (uint32_t)__builtin_amdgcn_update_dpp((int)bv[i], (int)bv[i], 0x128, 0xf, 0xf, false);
          }
          // index byte -> table entry, row slot -> bank, byte 2 of the lane base -> table
          const uint2 x0 = lds_read_u64(__builtin_amdgcn_perm(wd[pr], lbase, 0x0c020400u));
          const uint2 x1 = lds_read_u64(__builtin_amdgcn_perm(wd[pr], lbase, 0x0c020500u));
          const uint2 y0 = lds_read_u64(__builtin_amdgcn_perm(wd[pr], lbase, 0x0c020600u));
          const uint2 y1 = lds_read_u64(__builtin_amdgcn_perm(wd[pr], lbase, 0x0c020700u));
          const uint32_t xs[4] = {x0.x, x0.y, x1.x, x1.y}, ys[4] = {y0.x, y0.y, y1.x, y1.y};
          cq_v4u a0, a1;
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const pair_u32 sw = __builtin_amdgcn_permlane16_swap(xs[i], ys[i], false, false);
            a0[i] = sw[0];
            a1[i] = sw[1];
          }
          if constexpr (F16) {
            acc[0] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(cq_v8f16, a0),
                                                            __builtin_bit_cast(cq_v8f16, bv), acc[0], 0, 0, 0);
            acc[1] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(cq_v8f16, a1),
                                                            __builtin_bit_cast(cq_v8f16, bv), acc[1], 0, 0, 0);
          } else {
            acc[0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(cq_v8bf16, a0),
                                                             __builtin_bit_cast(cq_v8bf16, bv), acc[0], 0, 0, 0);
            acc[1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(cq_v8bf16, a1),
                                                             __builtin_bit_cast(cq_v8bf16, bv), acc[1], 0, 0, 0);
          }
        }
        __builtin_amdgcn_sched_barrier(0);  // the refill must stay behind the last use of the slot
        ring[R0 + q] = load_stream(wb2 + (size_t)(wave + NW * q) * sstride + loff);
        // the previous unit's results (once), and this step's share of the next unit's table
        if (q == 0 && ui > 0) finish(u - ustep, (uint32_t)(HALF ^ 1));
        if (q >= 1)
          table_part(c01[HALF ^ 1], c23[HALF ^ 1], (uint32_t)((HALF ^ 1) << 16), ((q - 1) * 16) / (Q - 1),
                     (q * 16) / (Q - 1));
      }
      // this unit's K partials: register r = 4 * (row half) + v of wavefront w at [HALF][w][r][column]
      if (i16 < 8) {
        const uint32_t wbase = kRed + (uint32_t)HALF * kW2Red + (uint32_t)wave * 1024u + slot * 4u;
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
          for (int v = 0; v < 4; ++v)
            *reinterpret_cast<__attribute__((address_space(3))) float*>(
                (uintptr_t)(wbase + (uint32_t)((h * 4 + v) * 128))) = acc[h][v];
      }
      __syncthreads();
    };

    for (int ui = 0; ui < ucnt; ui += 2) {
      unit(std::integral_constant<int, 0>{}, ui);
      if (ui + 1 < ucnt) unit(std::integral_constant<int, 1>{}, ui + 1);
    }
    __builtin_amdgcn_s_setprio(0);
    finish(ufirst + (ucnt - 1) * ustep, (uint32_t)((ucnt - 1) & 1));
    __syncthreads();   // the next token block rewrites table 0 and the partial buffers
  }
}

template <int AK, int EPI, int OUTK, int Q>
cq_status launch_w2(const W2Args& a, int G, hipStream_t s) {
  auto kern = gemm_w2_kernel<AK, EPI, OUTK, Q>;
  static std::atomic<bool> configured{false};
  const cq_status cst = cq_configure_lds(kern, kW2Lds, configured, true);
  if (cst != CQ_OK) return cst;
  const int n_units = a.N / 32;
  const dim3 grid((n_units + a.upw - 1) / a.upw, G, a.ksplit);
  hipLaunchKernelGGL(kern, grid, dim3(64 * kW2Waves), kW2Lds, s, a);
  return cq_check_launch();
}

template <int AK, int Q>
cq_status dispatch_w2(const W2Args& a, int G, int epilogue, int out_kind, hipStream_t s) {
  if (epilogue == CQ_EPI_SWIGLU)
    return out_kind == CQ_OUT_F16 ? launch_w2<AK, CQ_EPI_SWIGLU, CQ_OUT_F16, Q>(a, G, s)
                                  : launch_w2<AK, CQ_EPI_SWIGLU, CQ_OUT_F32, Q>(a, G, s);
  return out_kind == CQ_OUT_F16 ? launch_w2<AK, CQ_EPI_NONE, CQ_OUT_F16, Q>(a, G, s)
                                : launch_w2<AK, CQ_EPI_NONE, CQ_OUT_F32, Q>(a, G, s);
}

template <int OUTK>
__global__ __launch_bounds__(256) void w2_sum_partials_kernel(const float* __restrict__ partials, size_t part_stride,
                                                              int ksplit, size_t n4, void* __restrict__ out) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= n4) return;
  float4 acc = reinterpret_cast<const float4*>(partials)[i];
  for (int q = 1; q < ksplit; ++q) {
    const float4 v = reinterpret_cast<const float4*>(partials + (size_t)q * part_stride)[i];
    acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
  }
  if constexpr (OUTK == CQ_OUT_F16)
    reinterpret_cast<uint2*>(out)[i] = make_uint2(f32_to_f16_bits_sat(acc.x) | (f32_to_f16_bits_sat(acc.y) << 16),
                                                  f32_to_f16_bits_sat(acc.z) | (f32_to_f16_bits_sat(acc.w) << 16));
  else
    reinterpret_cast<float4*>(out)[i] = acc;
}

}  // namespace

// K steps of 128 per K range: the kernel exists for ranges of 32 steps (4 per wavefront) and of 56 (7 per
// wavefront); 0 = no such split of K.
int cq_gemm_w2_range_steps(int K) {
  if (K <= 0 || K % 128 != 0) return 0;
  const int n = K / 128;
  if (n % 32 == 0) return 32;
  if (n % 56 == 0) return 56;
  return 0;
}

bool cq_gemm_w2_supported(const cq_codebook_weights* W, int a_kind, int epilogue) {
  const int steps = cq_gemm_w2_range_steps(W->K);
  if (steps == 0 || W->N % 64 != 0 || cq_tables_per_row(W) > 1) return false;
  if (a_kind != CQ_A_INT8_CODES && a_kind != CQ_A_F16 && a_kind != CQ_A_BF16) return false;
  if (epilogue != CQ_EPI_NONE && W->K / 128 != steps) return false;   // a nonlinear epilogue needs the whole sum
  return true;
}

cq_status cq_gemm_w2_launch(const cq_codebook_weights* W, const void* A, int a_kind, const float* row_scale,
                            const int32_t* row_gather, const int32_t* group_offsets, int M_total, int epilogue,
                            void* out, int out_kind, void* workspace, hipStream_t s, int* ksplit_left,
                            const cq_route_fuse* route) {
  if (ksplit_left) *ksplit_left = 1;
  if (!cq_gemm_w2_supported(W, a_kind, epilogue)) return CQ_ERR_UNSUPPORTED;
  const int steps = cq_gemm_w2_range_steps(W->K);
  W2Args a;
  a.idx = W->prepacked ? (const uint8_t*)W->prepacked : W->idx;
  a.cent = W->cent;
  a.prepacked = W->prepacked ? 1 : 0;
  a.N = W->N;
  a.K = W->K;
  a.A = A;
  a.row_scale = row_scale;
  a.row_gather = row_gather;
  a.group_offsets = group_offsets;
  a.route = route ? *route : cq_route_fuse{nullptr, 0, 0, 0, 0, nullptr, nullptr, nullptr, nullptr};
  a.out = out;
  a.out_ld = epilogue == CQ_EPI_SWIGLU ? W->N / 2 : W->N;
  a.ksplit = W->K / 128 / steps;
  a.partials = (float*)workspace;
  a.part_stride = (size_t)M_total * W->N;
  {
    const long units = (long)(W->N / 32) * W->G * a.ksplit;   // about one workgroup per compute unit
    long upw = (units + 255) / 256;
    if (upw < 1) upw = 1;
    if (upw > W->N / 32) upw = W->N / 32;
    a.upw = (int)upw;
  }
  cq_status st;
  if (steps == 32) {
    st = a_kind == CQ_A_INT8_CODES ? dispatch_w2<CQ_A_INT8_CODES, 4>(a, W->G, epilogue, out_kind, s)
         : a_kind == CQ_A_F16      ? dispatch_w2<CQ_A_F16, 4>(a, W->G, epilogue, out_kind, s)
                                   : dispatch_w2<CQ_A_BF16, 4>(a, W->G, epilogue, out_kind, s);
  } else {
    st = a_kind == CQ_A_INT8_CODES ? dispatch_w2<CQ_A_INT8_CODES, 7>(a, W->G, epilogue, out_kind, s)
         : a_kind == CQ_A_F16      ? dispatch_w2<CQ_A_F16, 7>(a, W->G, epilogue, out_kind, s)
                                   : dispatch_w2<CQ_A_BF16, 7>(a, W->G, epilogue, out_kind, s);
  }
  if (st != CQ_OK || a.ksplit == 1) return st;
  if (ksplit_left) {
    *ksplit_left = a.ksplit;   // the caller adds the partial sums itself
    return st;
  }
  // rows of empty tails of `out` are never written by the kernel; the sum covers the rows below group_offsets[G]
  // only when M_total equals it, so it adds all M_total rows of partials the kernel wrote (unwritten rows of
  // the partial buffers are rows past the last group: the caller's out rows there are unspecified anyway)
  const size_t n4 = (size_t)M_total * W->N / 4;
  const unsigned blocks = (unsigned)((n4 + 255) / 256);
  if (out_kind == CQ_OUT_F16)
    hipLaunchKernelGGL(w2_sum_partials_kernel<CQ_OUT_F16>, dim3(blocks), dim3(256), 0, s, a.partials, a.part_stride,
                       a.ksplit, n4, out);
  else
    hipLaunchKernelGGL(w2_sum_partials_kernel<CQ_OUT_F32>, dim3(blocks), dim3(256), 0, s, a.partials, a.part_stride,
                       a.ksplit, n4, out);
  return cq_check_launch();
}

size_t cq_gemm_w2_partials_bytes(const cq_codebook_weights* W, int M_total) {
  const int steps = cq_gemm_w2_range_steps(W->K);
  if (steps == 0) return 0;
  const int ksplit = W->K / 128 / steps;
  return ksplit > 1 ? cq_align_up((size_t)ksplit * M_total * W->N * sizeof(float), 256) : 0;
}
