// a6 / a7: grouped product with clustered weights (W_c[n,k] = C[n, idx[n,k]], Eq. W_c) for
// token blocks of up to 32 rows per pass -- the decode (GEMV-like) regime, where the kernel is
// bound by streaming the packed 4-bit indices from HBM.
//
// Design (gfx950), one workgroup of 8 wavefronts per run of 64-row units of one expert:
//   * Table.  A weight row has 16 centroids, so a BYTE of packed indices (two weights) has only 256
//     possible decoded values.  The workgroup builds, for each of the 64 rows of a unit, the 256-entry
//     table of decoded PAIRS (two 16-bit operands in one dword) in LDS, entry-major: entry b of row slot r
//     is the dword at b*256 + r*4.  A wavefront's 32-lane LDS pass then touches 32 different banks
//     whatever the indices are (bank = row slot), which removes the bank conflicts that random table
//     indexing causes -- the paper's stated obstacle for LUT kernels -- without replicating tables.
//     One v_perm_b32 builds the LDS address of a pair, one ds_read_b32 returns two MFMA operands.
//   * Stream.  Indices are read with 16-byte loads per lane through a register ring; lane
//     (r = lane%32, g = lane/32) reads the 32 weights [64 s + 32 g, +32) of row r in K step s, which are
//     four 8-wide MFMA A fragments.  With prepacked storage a wavefront load covers 1 KiB of contiguous
//     memory.  The wavefronts split K (step s goes to wavefront s % 8); K longer than 4096 is cut into
//     ranges handled by different workgroups (blockIdx.z) whose scaled fp32 partial sums are added later
//     in a fixed order.
//   * Math.  Token blocks of up to 16 columns: v_mfma_f32_16x16x32 (the 32x32x16 shape would spend half
//     its time on padding columns).  Every lane looks up the row it loaded and v_permlane16_swap sorts
//     each pair of looked-up dwords into the two 16-row halves; the lane rows then carry the k groups in
//     the order 2c + g%2 + 4(g/2), and the B operand is held in that order.  17..32 columns:
//     v_mfma_f32_32x32x16 with the decoded weights as A.  Integer codes and bf16 centroids are exact bf16
//     operands; f16 activations (the down projection) use f16 MFMA with centroids converted to f16.  Both
//     operands number K identically, so the sum over K is the plain dot product.
//   * Two unit loops.  Pipelined (groups of up to 16 tokens whose wavefronts have exactly 8 or 7 K steps
//     per unit -- run_units_pipe): activations of a wavefront's own K steps in registers, two tables and
//     the K partials in LDS, the next unit's table written and the previous unit finished inside the K
//     loop, one barrier per unit.  Plain (everything else): activations staged in a 64 KiB LDS slab one K
//     slab at a time, already in fragment order, one table rebuilt between units.
//   * Epilogue.  The wavefronts' partial accumulators are summed through LDS in a fixed order
//     (deterministic), scaled per token, optionally passed through SiLU(gate)*up (gate/up rows interleaved
//     so both sit in one lane), and stored.
//
// This header holds the kernel and its launchers; it is compiled once per operand kind (codebook_gemm_int8.hip,
// _f16.hip, _bf16.hip, _f32.hip: the instantiations of one kind each, so that they build in parallel), and
// codebook_gemm.hip holds the planning and the entry points.
#pragma once
#include <type_traits>

#include "cq_internal.h"
#include "cq_route.h"
#include "cq_stream.h"

struct cq_small_gemm_args {
  const uint8_t* idx;       // canonical or prepacked index bytes, group-major
  const uint16_t* cent;
  int prepacked;
  int N, K;
  const void* A;
  const float* row_scale;
  const int32_t* row_gather;
  const int32_t* group_offsets;
  void* out;
  int out_ld;
  int upw;                  // 64-row units per workgroup (consecutive, same expert)
  int max_rows;             // groups with more rows are left to the large-tile kernel
  int ksteps;               // K steps (of 64) per K split; blockIdx.z selects the split
  int ksplit;               // number of K splits; > 1: scaled fp32 partial sums go to `partials`
  int halves;               // 1, or 2: gridDim.z = ksplit * 2 (see the kernel)
  float* partials;          // [ksplit][M_total][N]
  size_t part_stride;       // M_total * N
  // device-built work list (launches that also use the large-tile kernel), else NULL: blockIdx.y is
  // the group and blockIdx.x * upw the first unit
  const int32_t* small_hdr; // {number of listed groups, units per workgroup, workgroups per group}
  const int32_t* small_ids; // the listed groups
  // grouping by expert folded into the launch (pipelined unit loop only), else route.ids == NULL
  cq_route_fuse route;
};
using GemmArgs = cq_small_gemm_args;

// one per operand kind, each in its own translation unit; qt: 0, or block-wise tables of 512 * qt weights
cq_status cq_gemm_small_dispatch_int8(const GemmArgs& a, int G, int qt, int epilogue, int out_kind, hipStream_t s);
cq_status cq_gemm_small_dispatch_f16(const GemmArgs& a, int G, int qt, int epilogue, int out_kind, hipStream_t s);
cq_status cq_gemm_small_dispatch_bf16(const GemmArgs& a, int G, int qt, int epilogue, int out_kind, hipStream_t s);
cq_status cq_gemm_small_dispatch_f32(const GemmArgs& a, int G, int qt, int epilogue, int out_kind, hipStream_t s);

namespace {

#ifndef CQ_SMALL_MAX_ROWS
#define CQ_SMALL_MAX_ROWS 32
#endif
constexpr int kSmallMaxRows = CQ_SMALL_MAX_ROWS;  // groups with more rows go to the large-tile kernel
constexpr int kTableBytes = 65536;   // 256 entries x 64 row slots x 4 bytes
constexpr int kSlabBytes = 65536;    // activation slab
#ifndef CQ_LISTED_WGS
#define CQ_LISTED_WGS 512
#endif
constexpr int kListedWorkgroups = CQ_LISTED_WGS;  // grid of a launch that runs off the device-built group list
constexpr int kRedBytes = 32768;     // K partials of up to 16 token columns: 8 wavefronts x 16 registers x 64 lanes
#ifndef CQ_GEMM_WAVES
#define CQ_GEMM_WAVES 8
#endif
constexpr int kWaves = CQ_GEMM_WAVES;  // wavefronts per workgroup: they split K (step s -> wavefront s % kWaves)
// K steps a wavefront keeps in flight: 4 (64 KiB per CU) or, when its step count is a multiple of 8,
// 8 (the per-unit phases in which nothing is consumed then find more data already on its way)
// Ring depth of the pipelined unit loop in HALF steps (one 16-byte load per lane: 32 rows x 64 k) for a
// wavefront with Q steps per unit.  It must divide 2Q so that a slot always meets the same half step of
// every unit: 8 for even Q (4 steps = 64 KiB in flight per compute unit; 16 was measured 5 % slower), Q for
// odd Q.
#ifndef CQ_PIPE_HD_EVEN
#define CQ_PIPE_HD_EVEN 8
#endif
#ifndef CQ_PIPE_HD_ODD
#define CQ_PIPE_HD_ODD 1
#endif
constexpr int pipe_ring_depth(int Q) {
  return (2 * Q) % CQ_PIPE_HD_EVEN == 0 ? CQ_PIPE_HD_EVEN : (Q % 2 ? CQ_PIPE_HD_ODD * Q : 2);
}
constexpr int kSlabCheck = 16 / kWaves;  // smallest number of wavefront steps in a slab (Mpad = 32)


template <bool F16>
__device__ __forceinline__ cq_v16f mfma32(const cq_v4u a, const uint4 b, cq_v16f c) {
  cq_v4u bv = {b.x, b.y, b.z, b.w};
  if constexpr (F16) {
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(cq_v8f16, a), __builtin_bit_cast(cq_v8f16, bv),
                                                  c, 0, 0, 0);
  } else {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(cq_v8bf16, a),
                                                   __builtin_bit_cast(cq_v8bf16, bv), c, 0, 0, 0);
  }
}


// QS > 0: a workgroup whose group has at most 32 rows and whose wavefronts have exactly QS K steps per unit
// runs the pipelined unit loop (run_units_pipe below); 0: that path is left out of the instantiation.
// QT > 0: block-wise centroid tables, one per 512 * QT weights of a row (QT K steps per wavefront and table; QT
// divides QS); the instantiation then holds nothing but the pipelined loop.  0: one table per row.
template <int AK, int EPI, int OUTK, int kRing, int QS, int QT = 0>
__global__ __launch_bounds__(64 * kWaves, 1) void gemm_small_kernel(const GemmArgs p) {
  constexpr bool F16 = (AK == CQ_A_F16 || AK == CQ_A_F32);
  constexpr int NW = kWaves;
  constexpr int NT = 64 * NW;
  extern __shared__ uint4 smem[];
  char* lds = reinterpret_cast<char*>(smem);
  uint32_t* tbl = reinterpret_cast<uint32_t*>(lds);
  float* red = reinterpret_cast<float*>(lds);  // aliases the table between units
  uint4* slab = reinterpret_cast<uint4*>(lds + kTableBytes);
  float* redc = reinterpret_cast<float*>(lds + kTableBytes + kSlabBytes);  // kRedBytes: partials of <= 16 tokens

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // uniform: what depends on it stays scalar
  const int N = p.N, K = p.K;
  const int nUnits = N >> 6;
  int grp, u0, upw;
  if (p.small_hdr) {
    const int chunks = p.small_hdr[2];
    if ((int)blockIdx.x >= p.small_hdr[0] * chunks) return;
    const int gi = blockIdx.x / chunks;
    grp = p.small_ids[gi];
    upw = p.small_hdr[1];
    u0 = (blockIdx.x - gi * chunks) * upw;
  } else {
    grp = blockIdx.y;
    upw = p.upw;
    u0 = blockIdx.x * upw;
  }
  // Rows of this group: from the grouped layout, or -- a5 folded into this launch -- from the selected expert
  // ids themselves (cq_route::group_rows_from_ids).
  // blockIdx.z = K range + ksplit * half: half 1 exists in launches in which groups of 17..32 rows are possible and
  // takes rows 16.. of such a group in the pipelined unit loop
  const int kz = p.halves > 1 ? (int)blockIdx.z % p.ksplit : (int)blockIdx.z;
  const int half = p.halves > 1 ? (int)blockIdx.z / p.ksplit : 0;
  int m0, Me, row_token = 0;
  bool fused = false;
  if constexpr (QS > 0) fused = p.route.ids != nullptr;
  if (fused) {
    cq_route::group_rows_from_ids(p.route, grp, lane,
                                  blockIdx.x == 0 && blockIdx.y == 0 && blockIdx.z == 0 && wave == 0, m0, Me, row_token);
  } else {
    m0 = p.group_offsets[grp];
    Me = p.group_offsets[grp + 1] - m0;
  }
  if (Me <= 0 || Me > p.max_rows) return;
  if (half > 0 && (Me <= 16 || Me > 32)) return;   // (second halves exist for groups of 17..32 rows only)
  const int u1 = min(nUnits, u0 + upw);
  if (u0 >= u1) return;
  const size_t rowbytes = (size_t)K >> 1;
  const uint8_t* gbase = p.idx + (size_t)grp * N * rowbytes;
  const int r32 = lane & 31, g2 = lane >> 5;
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
  const int sb = kz * p.ksteps;                     // first K step (of 64) of this workgroup's K range
  const int nS = min(p.ksteps, (K >> 6) - sb);      // its number of steps
  if (nS <= 0) return;
  const int Kl = nS << 6;
  lane_off0 += (size_t)sb * sstride;
  lane_off1 += (size_t)sb * sstride;
  const int Qmax = (nS + NW - 1) / NW;              // steps per wavefront (upper bound)
  const int Qpad = (Qmax + kRing - 1) / kRing * kRing;
  const uint32_t lanebase0 = (uint32_t)(r32 * 4);
  const uint32_t lanebase1 = (uint32_t)((32 + r32) * 4);
  const int n_tb = (Me + 31) >> 5;
  if (half > 0 && !(QS > 0 && nS == QS * NW)) return;   // (no pipelined loop here: the first half's workgroup takes all rows)

  // ---- up to 16 tokens, K range of exactly QS steps per wavefront: the unit loop as a pipeline ----
  // (described for up to 8 tokens; the form for 9..16 differs where WIDE says so)
  // With few tokens the activations of a wavefront's own K steps fit in registers (its K steps are the same
  // in every unit), so no slab is needed and LDS holds TWO pair tables and two buffers of K partials.  While
  // unit u is looked up in one table, the table of unit u+1 is written into the other, a few entries per K
  // step, and the partial sums of unit u-1 are added up, scaled, passed through the epilogue and stored: one
  // workgroup barrier per unit, and nothing but that barrier between two units' K loops.  Hazards: table
  // (u+1)%2 was last read in unit u-1, partial buffer u%2 last read (for unit u-2) in unit u-1 -- both
  // before the barrier that ends unit u-1.
  // Ring slot hs % HD serves half step hs = 2q + row block (one 16-byte load per lane) and is refilled with
  // half step hs + HD, of this unit or of the next one, as soon as step q's lookups are issued.
  // (a group of 17..32 rows is shared by two workgroups per run of units, 16 rows and the rest -- `half` above: it
  // streams its indices twice, which is still faster than the plain loop below, whose 32-token slab holds a quarter
  // of K and is restaged four times per unit)
  const int pass_row0 = 16 * half;
  const int pass_rows = min(16, Me - pass_row0);   // this workgroup's rows: m0 + pass_row0 .. + pass_rows - 1
  auto run_units_pipe = [&](auto wide_tag) {
    constexpr bool WIDE = decltype(wide_tag)::value;   // 9..16 tokens: see below
    constexpr int Q = QS > 0 ? QS : 1;
    constexpr int HD = pipe_ring_depth(Q);
    // A unit's K loop is a run of NSUB sub-units of QL steps, one per centroid table of the K range (one
    // sub-unit = the whole unit when a row has one table).  The next sub-unit's table is written during steps
    // TB0 .. QL-1 of the current one, and a workgroup barrier separates two sub-units like it separates two units.
    constexpr int QL = QT > 0 ? QT : Q;
    constexpr int NSUB = Q / QL;
    static_assert(Q % QL == 0, "whole tables per K range");
    constexpr int TB0 = QL / 2;
    const int i16 = lane & 15, g4 = lane >> 4;
    const int tcol = WIDE ? i16 : (i16 & 7);   // token column whose activations this lane holds
    const bool tok = tcol < pass_rows;      // ... a real token (of this pass's block of up to 16 rows)
    const bool grouped = p.prepacked != 0;
    constexpr uint32_t kRed = 2 * kTableBytes;   // partial buffers: [2][wave][16 registers][32 columns] floats
    const uint32_t slot = WIDE ? (uint32_t)lane : (uint32_t)(g4 * 8 + (i16 & 7));
    constexpr uint32_t kRegStride = WIDE ? 256u : 128u;    // bytes between two accumulator registers' partials
    constexpr uint32_t kWaveStride = 16u * kRegStride;     // ... between two wavefronts'
    const bool pcol = WIDE || i16 < 8;                     // this lane's output column carries partial sums
    // ring loads: uniform base (unit, K step, row block) + 32-bit lane offset
    const uint32_t loff = p.prepacked ? (uint32_t)lane * 16u : (uint32_t)r32 * (uint32_t)rowbytes + (uint32_t)g2 * 16u;
    const size_t rb1 = 32 * rowbytes;            // the unit's second block of 32 rows
    const uint8_t* const kbase = gbase + (size_t)sb * sstride;
    const size_t ubytes = 64 * rowbytes;         // index bytes of one unit
    // units of this workgroup: its index among the group's workgroups + i * (workgroups of the group), so
    // that the workgroups of a group read one contiguous window of the index stream at any time (measured
    // 1-2 % faster than a contiguous run of units per workgroup)
    const int ustep = (nUnits + upw - 1) / upw;
    const int ufirst = u0 / upw;
    const int ucnt = (nUnits - ufirst + ustep - 1) / ustep;

    // centroid rows of a unit (raw bf16 pairs; chp: the two entries this wavefront uses as high halves)
    uint32_t cp[8], chp;
    const int nblk = QT > 0 ? K / (512 * QL) : 1;      // tables per row
    const int blk0 = QT > 0 ? sb / (NW * QL) : 0;      // first table of this workgroup's K range
    auto cent_req = [&](int u, int sub) {
      const uint16_t* crow = p.cent + (((size_t)grp * N + (size_t)u * 64 + lane) * nblk + blk0 + sub) * CQ_N_CENTROIDS;
      const uint4 a = reinterpret_cast<const uint4*>(crow)[0];
      const uint4 b = reinterpret_cast<const uint4*>(crow)[1];
      cp[0] = a.x; cp[1] = a.y; cp[2] = a.z; cp[3] = a.w; cp[4] = b.x; cp[5] = b.y; cp[6] = b.z; cp[7] = b.w;
      chp = *reinterpret_cast<const uint32_t*>(crow + 2 * wave);
    };
    auto cent_f16 = [&]() {
      if constexpr (F16) {
#pragma unroll
        for (int i = 0; i < 8; ++i)
          cp[i] = bf16_bits_to_f16_bits(cp[i] & 0xffffu) | (bf16_bits_to_f16_bits(cp[i] >> 16) << 16);
        chp = bf16_bits_to_f16_bits(chp & 0xffffu) | (bf16_bits_to_f16_bits(chp >> 16) << 16);
      }
    };
    // entries [e0, e1) of this wavefront's 32 (entry e: high half = its centroid 2*wave + e/16, low half = e%16)
    auto table_part = [&](const uint32_t tbase, const int e0, const int e1) {
#pragma unroll
      for (int e = e0; e < e1; ++e) {
        const int i = e >> 4, l = e & 15;
        const uint32_t sel = ((l & 1) ? 0x0302u : 0x0100u) | ((i ? 0x0706u : 0x0504u) << 16);
        const uint32_t v = __builtin_amdgcn_perm(chp, cp[l >> 1], sel);
        *reinterpret_cast<__attribute__((address_space(3))) uint32_t*>((uintptr_t)(tbase + (uint32_t)(e * 256))) = v;
      }
    };
    typedef __attribute__((ext_vector_type(2))) unsigned pair_u32;

    // -- prologue: what depends only on the group goes first (centroid rows, the ring), then the token rows
    cent_req(ufirst, 0);
    uint4 ring[HD];
    {
      const uint8_t* wb = kbase + (size_t)ufirst * ubytes;
#pragma unroll
      for (int j = 0; j < HD; ++j)
        ring[j] = load_stream(wb + (size_t)(wave + NW * (j >> 1)) * sstride + ((j & 1) ? rb1 : 0) + loff);
    }
    __builtin_amdgcn_sched_barrier(0);
    float sc16 = 1.f;
    size_t arow = 0;
    const int col_token = __shfl(row_token, pass_row0 + tcol);   // (folded grouping: the token of this lane's column)
    if (tok) {
      const int m = m0 + pass_row0 + tcol;
      const size_t src = fused ? (size_t)col_token : p.row_gather ? (size_t)p.row_gather[m] : (size_t)m;
      arow = src * K;
      if (p.row_scale) sc16 = p.row_scale[src];
    }
    // B fragments of step q (up to 8 tokens): both K halves in ONE register set -- lanes of columns 0..7 hold the first half's
    // fragment of their token, lanes of columns 8..15 the second half's fragment of token column - 8 (the
    // matrix cores' output columns 8..15 are never stored, so what their B columns hold does not matter);
    // a rotation by 8 inside each row of 16 lanes brings the second half into place.
    // With 9..16 tokens every column is real: one register set per K half, no rotation.
    constexpr int NB = WIDE ? 2 : 1;
    cq_v4u breg[Q][NB];
    {
      ActRaw raw[Q][NB];
#pragma unroll
      for (int q = 0; q < Q; ++q)
#pragma unroll
        for (int c = 0; c < NB; ++c) {
          const int chunk = (wave + NW * q) * 8 + (g4 & 1) + 4 * (g4 >> 1) + 2 * (WIDE ? c : (i16 >> 3));
          raw[q][c] = act_load8<AK>(p.A, arow + (size_t)sb * 64 + (size_t)chunk * 8);
        }
#pragma unroll
      for (int q = 0; q < Q; ++q)
#pragma unroll
        for (int c = 0; c < NB; ++c) {
          const uint4 v = tok ? act_pack8<AK>(raw[q][c], grouped) : make_uint4(0u, 0u, 0u, 0u);
          breg[q][c] = cq_v4u{v.x, v.y, v.z, v.w};
        }
    }
    cent_f16();
    table_part((uint32_t)(wave * 8192 + lane * 4), 0, 32);
    __syncthreads();

    // finish of a unit: this wavefront adds up accumulator registers 2*wave and 2*wave+1 (a gate/up pair of
    // rows) of all wavefronts' partials in buffer pb, in wavefront order
    auto finish = [&](const int uu, const uint32_t pb) {
      if (pcol) {
        const uint32_t rb0 = kRed + pb * 16384u + (uint32_t)(2 * wave) * kRegStride + slot * 4u;
        float val[2];
#pragma unroll
        for (int i = 0; i < 2; ++i) {
          float sum = __uint_as_float(lds_read_u32(rb0 + (uint32_t)i * kRegStride));
#pragma unroll
          for (int w = 1; w < NW; ++w)
            sum += __uint_as_float(lds_read_u32(rb0 + (uint32_t)w * kWaveStride + (uint32_t)i * kRegStride));
          val[i] = sum;
        }
        if (i16 < pass_rows) {
          const int m = m0 + pass_row0 + i16;
          const int r = 2 * wave;
          const int row = uu * 64 + (r >> 3) * 32 + ((r >> 2) & 1) * 16 + g4 * 4 + (r & 3);
          const float x0 = sc16 * val[0], x1 = sc16 * val[1];
          if (p.ksplit > 1) {  // partial sum of this K range (CQ_EPI_NONE only)
            float* dst = p.partials + (size_t)kz * p.part_stride + (size_t)m * N + row;
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

    uint32_t par = 0;    // table of the current sub-unit
    uint32_t upar = 0;   // partial buffer of the current unit
    for (int ui = 0; ui < ucnt; ++ui) {
      const int u = ufirst + ui * ustep;
      const uint8_t* wb = kbase + (size_t)u * ubytes;
      const bool has_next = ui + 1 < ucnt;
      const uint8_t* wb_next = has_next ? wb + (size_t)ustep * ubytes : wb;
      // the centroid rows of the next table (this unit's second one, else the next unit's first), requested
      // ahead of the ring refills and used from step TB0 on
      if constexpr (NSUB > 1) cent_req(u, 1);
      else cent_req(has_next ? u + ustep : u, 0);
      __builtin_amdgcn_sched_barrier(0);
      uint32_t lbase[2] = {lanebase0 | (par << 16), lanebase1 | (par << 16)};
      uint32_t tnext = ((par ^ 1u) << 16) + (uint32_t)(wave * 8192 + lane * 4);

      cq_v4f acc[2][2];
#pragma unroll
      for (int rb = 0; rb < 2; ++rb)
#pragma unroll
        for (int h = 0; h < 2; ++h) acc[rb][h] = cq_v4f{0.f, 0.f, 0.f, 0.f};

#pragma unroll
      for (int q = 0; q < Q; ++q) {
        const int ql = q % QL;   // step within the sub-unit (a constant once the loop is unrolled)
        if (NSUB > 1 && ql == 0 && q > 0) {
          // the next table of this row block: every wavefront is done with the previous sub-unit's lookups,
          // whose table the coming steps overwrite, and has written its share of the table that is read now
          __syncthreads();
          par ^= 1u;
          lbase[0] = lanebase0 | (par << 16);
          lbase[1] = lanebase1 | (par << 16);
          tnext = ((par ^ 1u) << 16) + (uint32_t)(wave * 8192 + lane * 4);
          const int sub_next = q / QL + 1;
          if (sub_next < NSUB) cent_req(u, sub_next);
          else cent_req(has_next ? u + ustep : u, 0);
          __builtin_amdgcn_sched_barrier(0);
        }
        // The two wavefronts that share a SIMD (w and w + 4) take turns at the higher issue priority, step by
        // step: left alone, the older one always wins and the younger one finishes each unit late.
        if ((q ^ (wave >> 2)) & 1) __builtin_amdgcn_s_setprio(1);
        else __builtin_amdgcn_s_setprio(0);
#pragma unroll
        for (int c = 0; c < 2; ++c) {
          cq_v4u bv = breg[q][WIDE ? c : 0];
          if (!WIDE && c == 1) {
#pragma unroll
            for (int i = 0; i < 4; ++i)   // row_ror:8 -- lane l of a row of 16 takes lane (l + 8) % 16
              bv[i] = (uint32_t)__builtin_amdgcn_update_dpp((int)bv[i], (int)bv[i], 0x128, 0xf, 0xf, false);
          }
#pragma unroll
          for (int rb = 0; rb < 2; ++rb) {
            const uint4 w = ring[(2 * q + rb) % HD];
            const uint32_t wd[4] = {w.x, w.y, w.z, w.w};
            cq_v4u a0, a1;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
              // pair index byte -> table entry, row slot -> bank, byte 2 of the lane base -> table
              const uint32_t ox = __builtin_amdgcn_perm(wd[2 * c], lbase[rb], 0x0c020400u + (i << 8));
              const uint32_t oy = __builtin_amdgcn_perm(wd[2 * c + 1], lbase[rb], 0x0c020400u + (i << 8));
              const uint32_t x = lds_read_u32(ox);
              const uint32_t y = lds_read_u32(oy);
              const pair_u32 sw = __builtin_amdgcn_permlane16_swap(x, y, false, false);
              a0[i] = sw[0];
              a1[i] = sw[1];
            }
            if constexpr (F16) {
              acc[rb][0] = __builtin_amdgcn_mfma_f32_16x16x32_f16(
                  __builtin_bit_cast(cq_v8f16, a0), __builtin_bit_cast(cq_v8f16, bv), acc[rb][0], 0, 0, 0);
              acc[rb][1] = __builtin_amdgcn_mfma_f32_16x16x32_f16(
                  __builtin_bit_cast(cq_v8f16, a1), __builtin_bit_cast(cq_v8f16, bv), acc[rb][1], 0, 0, 0);
            } else {
              acc[rb][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                  __builtin_bit_cast(cq_v8bf16, a0), __builtin_bit_cast(cq_v8bf16, bv), acc[rb][0], 0, 0, 0);
              acc[rb][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                  __builtin_bit_cast(cq_v8bf16, a1), __builtin_bit_cast(cq_v8bf16, bv), acc[rb][1], 0, 0, 0);
            }
          }
        }
        __builtin_amdgcn_sched_barrier(0);  // the refills must stay behind the last use of their slots
#pragma unroll
        for (int rb = 0; rb < 2; ++rb) {
          const int hn = 2 * q + rb + HD;    // the half step that reuses this slot
          const bool same = hn < 2 * Q;
          const int h2 = same ? hn : hn - 2 * Q;
          const uint8_t* sp = (same ? wb : wb_next) + ((same || has_next) ? (size_t)(wave + NW * (h2 >> 1)) * sstride : 0) +
                              ((h2 & 1) ? rb1 : 0);
          ring[(2 * q + rb) % HD] = load_stream(sp + loff);
        }
        // the previous unit's results (once), and this step's share of the next unit's table
        if (q == 0 && ui > 0) finish(u - ustep, WIDE ? 0u : upar ^ 1u);
        if (ql == TB0) cent_f16();
        if (ql >= TB0) table_part(tnext, ((ql - TB0) * 32) / (QL - TB0), ((ql - TB0 + 1) * 32) / (QL - TB0));
      }
      // this unit's K partials: register r = rb*8 + h*4 + v of wavefront w at [par][w][r][column]
      // (9..16 tokens: the 32 KiB hold ONE buffer, so a barrier separates these writes from the reads of the
      // previous unit's partials at the top of this loop; it comes right before the unit's own barrier and
      // costs little)
      if constexpr (WIDE) __syncthreads();
      if (pcol) {
        const uint32_t wbase = kRed + (WIDE ? 0u : upar * 16384u) + (uint32_t)wave * kWaveStride + slot * 4u;
#pragma unroll
        for (int rb = 0; rb < 2; ++rb)
#pragma unroll
          for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int v = 0; v < 4; ++v)
              *reinterpret_cast<__attribute__((address_space(3))) float*>(
                  (uintptr_t)(wbase + (uint32_t)(rb * 8 + h * 4 + v) * kRegStride)) = acc[rb][h][v];
      }
      __syncthreads();
      par ^= 1u;
      upar ^= 1u;
    }
    __builtin_amdgcn_s_setprio(0);
    finish(ufirst + (ucnt - 1) * ustep, WIDE ? 0u : upar ^ 1u);
  };
#ifndef CQ_NO_PIPE
  if constexpr (QS > 0) {
    if (Me <= 16 * p.halves && nS == QS * NW) {   // every wavefront has exactly QS real steps
      if (pass_rows <= 8) run_units_pipe(std::false_type{});
      else run_units_pipe(std::true_type{});
      return;
    }
  }
#endif
  if constexpr (QT > 0) return;   // (block-wise tables exist in the pipelined loop only; the launcher sees to that)

  for (int tb = 0; tb < n_tb; ++tb) {
    const int Mb = min(32, Me - 32 * tb);
    const int Mpad = Mb <= 8 ? 8 : Mb <= 16 ? 16 : 32;     // divides the workgroup: a thread stages one token
    const int KSfull = 32768 / Mpad;                       // k values per slab (slab bytes / 2 / Mpad)
    const int qPerSlab = (KSfull >> 6) / NW;               // wavefront steps per slab
    const bool multi = KSfull < Kl;                        // activations do not fit: restage per slab
    const int tj = r32 < Mpad ? r32 : 0;                   // token column this lane feeds to the B operand
    const bool sep = Mpad <= 16;                           // 16x16x32 MFMA path, partial sums in their own region

    // ---- this thread's staging duty: token st, 8-wide k chunks sc0, sc0 + cstep, ... ----
    const int st = tid & (Mpad - 1);
    const int sc0 = tid / Mpad, cstep = NT / Mpad;
    const bool svalid = st < Mb;
    size_t srow = 0;
    if (svalid) {
      const int m = m0 + 32 * tb + st;
      srow = (p.row_gather ? (size_t)p.row_gather[m] : (size_t)m) * K;
    }
    // Four chunks per pass, all loads issued before the first conversion (unconditional, clamped to the
    // last chunk; rows of padding tokens read row 0 and store zeros): one memory latency per pass
    // instead of one per chunk.
    auto stage = [&](int sl) {
      const bool grouped = p.prepacked != 0;
      const int k0 = sl * KSfull;
      const int nC = min(KSfull, Kl - k0) >> 3;
      const size_t ebase = srow + (size_t)sb * 64 + k0;
      constexpr int kBatch = 4;
      for (int c = sc0; c < nC; c += kBatch * cstep) {
        ActRaw raw[kBatch];
#pragma unroll
        for (int i = 0; i < kBatch; ++i) raw[i] = act_load8<AK>(p.A, ebase + (size_t)min(c + i * cstep, nC - 1) * 8);
#pragma unroll
        for (int i = 0; i < kBatch; ++i) {
          const int ci = c + i * cstep;
          if (ci >= nC) break;
          slab[ci * Mpad + st] = svalid ? act_pack8<AK>(raw[i], grouped) : make_uint4(0u, 0u, 0u, 0u);
        }
      }
    };

    // ---- centroid rows of a unit, held raw in registers one unit ahead ----
    uint4 craw0, craw1;
    uint32_t chraw[(16 / NW + 1) / 2];
    auto cent_load = [&](int u) {
      const uint16_t* crow = p.cent + ((size_t)grp * N + (size_t)u * 64 + lane) * CQ_N_CENTROIDS;
      craw0 = reinterpret_cast<const uint4*>(crow)[0];
      craw1 = reinterpret_cast<const uint4*>(crow)[1];
#pragma unroll
      for (int i = 0; i < (16 / NW + 1) / 2; ++i)
        chraw[i] = *reinterpret_cast<const uint32_t*>(crow + (16 / NW) * wave + 2 * i);
    };
    // pair table: wavefront w writes the entries whose high nibble is in its share; lane = row slot
    auto build_table = [&]() {
      const uint32_t cp[8] = {craw0.x, craw0.y, craw0.z, craw0.w, craw1.x, craw1.y, craw1.z, craw1.w};
      uint32_t lo[16];
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        lo[2 * i] = cp[i] & 0xffffu;
        lo[2 * i + 1] = cp[i] >> 16;
      }
      if constexpr (F16) {
#pragma unroll
        for (int i = 0; i < 16; ++i) lo[i] = bf16_bits_to_f16_bits(lo[i]);
      }
#pragma unroll
      for (int i = 0; i < 16 / NW; ++i) {
        uint32_t hv = (i & 1) ? (chraw[i >> 1] >> 16) : (chraw[i >> 1] & 0xffffu);
        if constexpr (F16) hv = bf16_bits_to_f16_bits(hv);
        const int hi = (16 / NW) * wave + i;
        const uint32_t hs = hv << 16;
#pragma unroll
        for (int l = 0; l < 16; ++l) tbl[(hi * 16 + l) * 64 + lane] = lo[l] | hs;
      }
    };

    // per-token scale of this lane's output column (loop invariant: loaded once per token block)
    float sc = 1.f;
    if (p.row_scale && r32 < Mb) {
      const int m = m0 + 32 * tb + r32;
      sc = p.row_scale[p.row_gather ? p.row_gather[m] : m];
    }
    cent_load(u0);
    __builtin_amdgcn_sched_barrier(0);  // keep the centroid loads older than the ring loads

    // The unit loop exists in two instantiations.  When the block's activations fit in LDS for the whole
    // of K (the decode case) they are staged once, up front, and the loop body contains no conditional
    // loads at all: the number of loads in flight is then the same on every path, which lets each wait
    // cover exactly one ring slot.  Otherwise the slab is restaged inside the loop.
    auto run_units = [&](auto multi_tag) {
      constexpr bool MULTI = decltype(multi_tag)::value;
      float* rbase = red;  // the K partials alias the table (17..32 token columns: no room elsewhere)
      constexpr int rw = 64;
      const int rl = lane;
      uint4 ring[kRing][2];
      {
        const uint8_t* wb = gbase + (size_t)u0 * 64 * rowbytes;
#pragma unroll
        for (int j = 0; j < kRing; ++j) {
          const int gs = wave + NW * j;
          const size_t off = (size_t)(gs < nS ? gs : 0) * sstride;
          ring[j][0] = load_stream(wb + lane_off0 + off);
          ring[j][1] = load_stream(wb + lane_off1 + off);
        }
      }
      // single slab: the activations are staged here, behind the first ring requests, so that their
      // memory latency and the ring's overlap (the barrier after the first table build publishes them)
      if constexpr (!MULTI) stage(0);
      for (int u = u0; u < u1; ++u) {
        const uint8_t* wb = gbase + (size_t)u * 64 * rowbytes;
        const bool has_next = u + 1 < u1;
        const uint8_t* wb_next = has_next ? wb + 64 * rowbytes : wb;
        build_table();
        __syncthreads();

        cq_v16f acc0, acc1;
#pragma unroll
        for (int i = 0; i < 16; ++i) { acc0[i] = 0.f; acc1[i] = 0.f; }
        uint4 bf = make_uint4(0u, 0u, 0u, 0u);  // B operand; lanes of padding columns stay zero

        // Ring loads are issued unconditionally (address clamped to step 0 when the step does not exist)
        // so that the number of loads in flight is the same on every path and the wait before a slot
        // is consumed covers that slot only; the math of steps past the end of K is skipped.
        auto ring_round = [&](const int q0) {
#pragma unroll
          for (int j = 0; j < kRing; ++j) {
            const int q = q0 + j;
            if constexpr (MULTI) {
              if (j % kSlabCheck == 0) {
                // slab boundary: restage the activations for the next K range
                if (q < Qmax && q % qPerSlab == 0) {
                  __syncthreads();
                  stage(q / qPerSlab);
                  __syncthreads();
                }
              }
            }
            const int gs = wave + NW * q;
            // LDS addresses of this step's 32 table lookups (pair index byte -> entry, row slot -> bank);
            // computed first so that the ring slot is dead before it is refilled (the refill can then
            // land in the very same registers)
            uint32_t o0[16], o1[16];
            {
              const uint4 w0 = ring[j][0], w1 = ring[j][1];
              const uint32_t wd0[4] = {w0.x, w0.y, w0.z, w0.w};
              const uint32_t wd1[4] = {w1.x, w1.y, w1.z, w1.w};
#pragma unroll
              for (int jj = 0; jj < 4; ++jj)
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                  o0[jj * 4 + i] = __builtin_amdgcn_perm(wd0[jj], lanebase0, 0x0c0c0400u + (i << 8));
                  o1[jj * 4 + i] = __builtin_amdgcn_perm(wd1[jj], lanebase1, 0x0c0c0400u + (i << 8));
                  // pin the address here: it must not be recomputed from the ring slot after the refill
                  asm volatile("" : "+v"(o0[jj * 4 + i]), "+v"(o1[jj * 4 + i]));
                }
            }
            __builtin_amdgcn_sched_barrier(0);  // the refill below must not move above the last use of the slot
            {
              const int qq = q + kRing;  // the step that reuses this ring slot
              const bool same = qq < Qpad;
              const int gn = wave + NW * (same ? qq : qq - Qpad);
              const uint8_t* base = same ? wb : wb_next;
              const size_t off = (gn < nS && (same || has_next)) ? (size_t)gn * sstride : 0;
              ring[j][0] = load_stream(base + lane_off0 + off);
              ring[j][1] = load_stream(base + lane_off1 + off);
            }
            if (gs < nS) {
              // chunk (8 k) index inside the slab of this lane's first fragment
              const int ls = gs - (q / qPerSlab) * (qPerSlab * NW);
              const uint4* bsrc = slab + (size_t)(ls * 8 + g2 * 4) * Mpad + tj;
#pragma unroll
              for (int jj = 0; jj < 4; ++jj) {
                // only the lanes of real token columns fetch their fragment (the others keep zeros)
                if (r32 < Mpad) bf = bsrc[(size_t)jj * Mpad];
                cq_v4u a0, a1;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                  a0[i] = lds_read_u32(o0[jj * 4 + i]);
                  a1[i] = lds_read_u32(o1[jj * 4 + i]);
                }
                acc0 = mfma32<F16>(a0, bf, acc0);
                acc1 = mfma32<F16>(a1, bf, acc1);
              }
            }
          }
        };
        for (int q0 = 0; q0 < Qpad; q0 += kRing) {
          // The next unit's centroid rows are requested ahead of a round's weight loads (every round
          // in the single-slab loop, so that no load is conditional; only the last request matters):
          // a fixed number of younger loads then sits behind them, and the wait at the top of the
          // next unit does not drain the weight ring.
          if (MULTI ? (q0 + kRing >= Qpad) : true) {
            cent_load(has_next ? u + 1 : u);
            __builtin_amdgcn_sched_barrier(0);
          }
          ring_round(q0);
        }

        // ---- reduce the K partials (fixed order) through the table's LDS and finish ----
        // Only the lanes of real token columns carry results.  The partials alias the table, so
        // barriers fence them from the lookups on both sides.
        __syncthreads();
        if (r32 < Mpad) {
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            rbase[(wave * 32 + i) * rw + rl] = acc0[i];
            rbase[(wave * 32 + 16 + i) * rw + rl] = acc1[i];
          }
        }
        __syncthreads();
        // wavefront w finishes accumulator registers RPW*w .. RPW*w + RPW-1 of the 32
        constexpr int RPW = 32 / NW;
        float val[RPW];
        if (r32 < Mpad) {
#pragma unroll
          for (int i = 0; i < RPW; ++i) {
            const int r = wave * RPW + i;
            float s = rbase[r * rw + rl];
#pragma unroll
            for (int w = 1; w < NW; ++w) s += rbase[(w * 32 + r) * rw + rl];
            val[i] = s;
          }
        } else {
#pragma unroll
          for (int i = 0; i < RPW; ++i) val[i] = 0.f;
        }
        __syncthreads();  // the next unit's table overwrites this region
        if (r32 < Mb) {
          const int m = m0 + 32 * tb + r32;
#pragma unroll
          for (int h = 0; h < RPW / 4; ++h) {
            // MFMA 32x32 output: register v of a lane holds row 8*(v/4) + 4*(lane/32) + v%4, column lane%32
            const int r = wave * RPW + 4 * h;          // first of four registers: r = 16*rb + 4*vb
            const int row = u * 64 + (r >> 4) * 32 + ((r >> 2) & 3) * 8 + g2 * 4;
            const float x0 = sc * val[4 * h], x1 = sc * val[4 * h + 1], x2 = sc * val[4 * h + 2],
                        x3 = sc * val[4 * h + 3];
            if (p.ksplit > 1) {  // partial sum of this K range (the launcher allows this for CQ_EPI_NONE only)
              float* dst = p.partials + (size_t)kz * p.part_stride + (size_t)m * N + row;
              *reinterpret_cast<float4*>(dst) = make_float4(x0, x1, x2, x3);
              continue;
            }
            if constexpr (EPI == CQ_EPI_SWIGLU) {
              const float h0 = x0 / (1.f + __expf(-x0)) * x1;
              const float h1 = x2 / (1.f + __expf(-x2)) * x3;
              const size_t o = (size_t)m * p.out_ld + (row >> 1);
              if constexpr (OUTK == CQ_OUT_F16) {
                *reinterpret_cast<uint32_t*>(reinterpret_cast<uint16_t*>(p.out) + o) =
                    f32_to_f16_bits_sat(h0) | (f32_to_f16_bits_sat(h1) << 16);
              } else {
                *reinterpret_cast<float2*>(reinterpret_cast<float*>(p.out) + o) = make_float2(h0, h1);
              }
            } else {
              const size_t o = (size_t)m * p.out_ld + row;
              if constexpr (OUTK == CQ_OUT_F16) {
                *reinterpret_cast<uint2*>(reinterpret_cast<uint16_t*>(p.out) + o) =
                    make_uint2(f32_to_f16_bits_sat(x0) | (f32_to_f16_bits_sat(x1) << 16),
                               f32_to_f16_bits_sat(x2) | (f32_to_f16_bits_sat(x3) << 16));
              } else {
                *reinterpret_cast<float4*>(reinterpret_cast<float*>(p.out) + o) = make_float4(x0, x1, x2, x3);
              }
            }
          }
        }
      }
    };

    // ---- up to 16 tokens: the same loop on v_mfma_f32_16x16x32 ----
    // With at most 16 real token columns the 32x32x16 shape spends half its matrix-pipe time on padding.
    // MFMA lane (i = lane%16, g = lane/16) supplies row i, k group g (8 k) of a 16-row x 32-k block, so a
    // 32-row x 64-k step of a row block is four MFMAs (row half h, k half c).  Were the lookups issued in
    // that arrangement, the four lanes of a row would hit the same LDS bank with different entries (a
    // two-way conflict in each half wavefront, measured at 1.5x the time of a conflict-free read).  So
    // every lane looks up the row it loaded (row lane%32 of the block: 32 different banks per half
    // wavefront) and one v_permlane16_swap per pair of looked-up dwords then sorts the results: of the
    // swap of (dword 2c, dword 2c+1), the first result holds rows 0..15 and the second rows 16..31, lane
    // row g carrying k group 2c + g%2 + 4*(g/2) of the step -- the B operand is read in that same order.
    // Output register v of lane (n, q): row 4q + v, token n.
    auto run_units16 = [&](auto multi_tag) {
      constexpr bool MULTI = decltype(multi_tag)::value;
      const int i16 = lane & 15, g4 = lane >> 4;
      const int tj16 = i16 < Mpad ? i16 : 0;
      const uint32_t lbase[2] = {lanebase0, lanebase1};  // byte offset of this lane's row slot in a table entry
      float sc16 = 1.f;
      if (p.row_scale && i16 < Mb) {
        const int m = m0 + 32 * tb + i16;
        sc16 = p.row_scale[p.row_gather ? p.row_gather[m] : m];
      }
      uint4 ring[kRing][2];
      {
        const uint8_t* wb = gbase + (size_t)u0 * 64 * rowbytes;
#pragma unroll
        for (int j = 0; j < kRing; ++j) {
          const int gs = wave + NW * j;
          const size_t off = (size_t)(gs < nS ? gs : 0) * sstride;
          ring[j][0] = load_stream(wb + lane_off0 + off);
          ring[j][1] = load_stream(wb + lane_off1 + off);
        }
      }
      // single slab: the activations are staged here, behind the first ring requests, so that their
      // memory latency and the ring's overlap (the barrier after the first table build publishes them)
      if constexpr (!MULTI) stage(0);
      typedef __attribute__((ext_vector_type(2))) unsigned pair_u32;
      for (int u = u0; u < u1; ++u) {
        const uint8_t* wb = gbase + (size_t)u * 64 * rowbytes;
        const bool has_next = u + 1 < u1;
        const uint8_t* wb_next = has_next ? wb + 64 * rowbytes : wb;
        build_table();
        __syncthreads();

        cq_v4f acc[2][2];
#pragma unroll
        for (int rb = 0; rb < 2; ++rb)
#pragma unroll
          for (int h = 0; h < 2; ++h) acc[rb][h] = cq_v4f{0.f, 0.f, 0.f, 0.f};
        uint4 bf = make_uint4(0u, 0u, 0u, 0u);  // B operand; lanes of padding columns stay zero

        auto ring_round = [&](const int q0) {
#pragma unroll
          for (int j = 0; j < kRing; ++j) {
            const int q = q0 + j;
            if constexpr (MULTI) {
              if (j % kSlabCheck == 0) {
                if (q < Qmax && q % qPerSlab == 0) {  // slab boundary: restage the activations
                  __syncthreads();
                  stage(q / qPerSlab);
                  __syncthreads();
                }
              }
            }
            const int gs = wave + NW * q;
            // table addresses first, so that the slot is dead before its refill
            uint32_t o[2][16];
#pragma unroll
            for (int rb = 0; rb < 2; ++rb) {
              const uint4 w = ring[j][rb];
              const uint32_t wd[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
              for (int d = 0; d < 4; ++d)
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                  o[rb][d * 4 + i] = __builtin_amdgcn_perm(wd[d], lbase[rb], 0x0c0c0400u + (i << 8));
                  asm volatile("" : "+v"(o[rb][d * 4 + i]));
                }
            }
            __builtin_amdgcn_sched_barrier(0);
            {
              const int qq = q + kRing;  // the step that reuses this ring slot
              const bool same = qq < Qpad;
              const int gn = wave + NW * (same ? qq : qq - Qpad);
              const uint8_t* base = same ? wb : wb_next;
              const size_t off = (gn < nS && (same || has_next)) ? (size_t)gn * sstride : 0;
              ring[j][0] = load_stream(base + lane_off0 + off);
              ring[j][1] = load_stream(base + lane_off1 + off);
            }
            if (gs < nS) {
              const int ls = gs - (q / qPerSlab) * (qPerSlab * NW);
              // chunk ls*8 + 2c + g%2 + 4*(g/2)
              const uint4* bsrc = slab + (size_t)(ls * 8 + (g4 & 1) + 4 * (g4 >> 1)) * Mpad + tj16;
#pragma unroll
              for (int c = 0; c < 2; ++c) {
                if (i16 < Mpad) bf = bsrc[(size_t)(2 * c) * Mpad];
                const cq_v4u bv = {bf.x, bf.y, bf.z, bf.w};
#pragma unroll
                for (int rb = 0; rb < 2; ++rb) {
                  cq_v4u a0, a1;
#pragma unroll
                  for (int i = 0; i < 4; ++i) {
                    const uint32_t x = lds_read_u32(o[rb][(2 * c) * 4 + i]);
                    const uint32_t y = lds_read_u32(o[rb][(2 * c + 1) * 4 + i]);
                    const pair_u32 sw = __builtin_amdgcn_permlane16_swap(x, y, false, false);
                    a0[i] = sw[0];
                    a1[i] = sw[1];
                  }
                  if constexpr (F16) {
                    acc[rb][0] = __builtin_amdgcn_mfma_f32_16x16x32_f16(
                        __builtin_bit_cast(cq_v8f16, a0), __builtin_bit_cast(cq_v8f16, bv), acc[rb][0], 0, 0, 0);
                    acc[rb][1] = __builtin_amdgcn_mfma_f32_16x16x32_f16(
                        __builtin_bit_cast(cq_v8f16, a1), __builtin_bit_cast(cq_v8f16, bv), acc[rb][1], 0, 0, 0);
                  } else {
                    acc[rb][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                        __builtin_bit_cast(cq_v8bf16, a0), __builtin_bit_cast(cq_v8bf16, bv), acc[rb][0], 0, 0, 0);
                    acc[rb][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                        __builtin_bit_cast(cq_v8bf16, a1), __builtin_bit_cast(cq_v8bf16, bv), acc[rb][1], 0, 0, 0);
                  }
                }
              }
            }
          }
        };
        for (int q0 = 0; q0 < Qpad; q0 += kRing) {
          if (MULTI ? (q0 + kRing >= Qpad) : true) {  // next unit's centroid rows, ahead of the ring loads
            cent_load(has_next ? u + 1 : u);
            __builtin_amdgcn_sched_barrier(0);
          }
          ring_round(q0);
        }

        // ---- K partials through their own LDS region: register r = rb*8 + h*4 + v of wavefront w at
        // (w*16 + r)*64 + lane; wavefront w then finishes registers 2w and 2w+1 (rows 4q+v, 4q+v+1 of one
        // 16-row block: a gate/up pair).  One barrier per unit is enough: a wavefront can only reach the
        // next unit's partial writes after that unit's table barrier, which every wavefront passes after
        // its reads here. ----
        if (i16 < Mpad) {
#pragma unroll
          for (int rb = 0; rb < 2; ++rb)
#pragma unroll
            for (int h = 0; h < 2; ++h)
#pragma unroll
              for (int v = 0; v < 4; ++v) redc[(wave * 16 + rb * 8 + h * 4 + v) * 64 + lane] = acc[rb][h][v];
        }
        __syncthreads();
        float val[2] = {0.f, 0.f};
        if (i16 < Mpad) {
#pragma unroll
          for (int i = 0; i < 2; ++i) {
            const int r = 2 * wave + i;
            float sum = redc[r * 64 + lane];
#pragma unroll
            for (int w = 1; w < NW; ++w) sum += redc[(w * 16 + r) * 64 + lane];
            val[i] = sum;
          }
        }
        if (i16 < Mb) {
          const int m = m0 + 32 * tb + i16;
          const int r = 2 * wave;
          const int row = u * 64 + (r >> 3) * 32 + ((r >> 2) & 1) * 16 + g4 * 4 + (r & 3);
          const float x0 = sc16 * val[0], x1 = sc16 * val[1];
          if (p.ksplit > 1) {  // partial sum of this K range (CQ_EPI_NONE only)
            float* dst = p.partials + (size_t)kz * p.part_stride + (size_t)m * N + row;
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

    if (multi) {
      if (sep) run_units16(std::true_type{});
      else run_units(std::true_type{});
    } else {
      if (sep) run_units16(std::false_type{});
      else run_units(std::false_type{});
    }
    __syncthreads();  // the slab is restaged for the next token block
  }
}

template <int AK, int EPI, int OUTK, int RING, int QS, int QT = 0>
cq_status launch_small_ring(const GemmArgs& a, int G, hipStream_t s) {
  auto kern = gemm_small_kernel<AK, EPI, OUTK, RING, QS, QT>;
  static std::atomic<bool> configured{false};
  const cq_status cst = cq_configure_lds(kern, kTableBytes + kSlabBytes + kRedBytes, configured, true);
  if (cst != CQ_OK) return cst;
  const int n_units = a.N / 64;
  const dim3 grid = a.small_hdr ? dim3(G > kListedWorkgroups ? G : kListedWorkgroups, 1, a.ksplit * a.halves)
                                : dim3((n_units + a.upw - 1) / a.upw, G, a.ksplit * a.halves);
  hipLaunchKernelGGL(kern, grid, dim3(64 * kWaves), kTableBytes + kSlabBytes + kRedBytes, s, a);
  return cq_check_launch();
}

// qt: 0, or block-wise tables of 512 * qt weights (every K range then gives each wavefront exactly 8 or 4 steps)
template <int AK, int EPI, int OUTK>
cq_status launch_small(const GemmArgs& a, int G, int qt, hipStream_t s) {
  const int per_wave = (a.ksteps + kWaves - 1) / kWaves;  // steps of a wavefront in the (first) K range
  if (qt != 0) {
    if (kWaves == 8 && qt == 2 && a.ksteps == 8 * kWaves) return launch_small_ring<AK, EPI, OUTK, 8, 8, 2>(a, G, s);
    if (kWaves == 8 && qt == 2 && a.ksteps == 4 * kWaves) return launch_small_ring<AK, EPI, OUTK, 8, 4, 2>(a, G, s);
    return CQ_ERR_UNSUPPORTED;
  }
  if (kWaves == 8 && per_wave == 8) return launch_small_ring<AK, EPI, OUTK, 8, 8>(a, G, s);
  if (kWaves == 8 && per_wave == 7) return launch_small_ring<AK, EPI, OUTK, 4, 7>(a, G, s);
  return per_wave % 8 == 0 ? launch_small_ring<AK, EPI, OUTK, 8, 0>(a, G, s)
                           : launch_small_ring<AK, EPI, OUTK, 4, 0>(a, G, s);
}

template <int AK>
cq_status dispatch_epi(const GemmArgs& a, int G, int qt, int epilogue, int out_kind, hipStream_t s) {
  if (epilogue == CQ_EPI_SWIGLU) {
    return out_kind == CQ_OUT_F16 ? launch_small<AK, CQ_EPI_SWIGLU, CQ_OUT_F16>(a, G, qt, s)
                                  : launch_small<AK, CQ_EPI_SWIGLU, CQ_OUT_F32>(a, G, qt, s);
  }
  return out_kind == CQ_OUT_F16 ? launch_small<AK, CQ_EPI_NONE, CQ_OUT_F16>(a, G, qt, s)
                                : launch_small<AK, CQ_EPI_NONE, CQ_OUT_F32>(a, G, qt, s);
}

}  // namespace
