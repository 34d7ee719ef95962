// a6 / a7 for groups with many tokens (prefill regime, bound by the matrix cores).
//
// Workgroup tile: 256 weight rows x CT tokens (CT = 256, 128, 64 or 32), four wavefronts, each owning 64 rows
// and ALL the tile's tokens (accumulators 2 x CT/32 MFMA blocks of 32x32).  Consequences:
//   * every wavefront decodes only its own rows, straight into MFMA A-operand registers: the decoded
//     weights never touch LDS, and no weight is decoded twice;
//   * a lane owns one row of each of its two 32-row blocks for the whole K loop, so the two 16-entry
//     centroid tables it needs are loop invariant and live in registers.  Decoding is pure vector ALU:
//     nibbles become byte selectors, v_perm_b32 picks the low and the high bytes of the centroids out
//     of register-resident byte tables (two 8-entry halves; a third perm, steered by bit 3 of the
//     index, picks between them), one or two more perm levels interleave the bytes into bf16/f16 pairs.
//     About 1.4 ALU operations per MFMA, all full rate, mostly hidden behind the matrix pipe.
//     With block-wise tables (one per group of g weights along K, g a multiple of 512) the two tables are
//     replaced every g/64 steps; the raw tables of the next group are requested one group ahead;
//   * LDS holds only the activation tiles.  They arrive by direct global->LDS loads (no staging
//     registers, no ds_write), four tiles deep, and each wavefront reads a tile once per K step.
// The activation operand is 16-bit (bf16 integer codes or f16 rows); other kinds are converted by a
// small pre-pass.  Token tiles come from a device-built work list (groups are ragged and their sizes
// are only known on the device); the list index is remapped so that tiles sharing activations run on
// the same XCD (L2).
#include <type_traits>

#include "cq_internal.h"
#include "cq_async.h"
#include "cq_decode.h"

void cq_large_tile_caps(int G, int M_total, int* cap256, int* cap128);

namespace {

constexpr int kLargeRows = 256;  // weight rows per workgroup
constexpr int kStepK = 64;       // K per pipeline step
constexpr int kStepBytes = kStepK * 2;  // one token's share of a step in LDS and in global memory
constexpr int kLdsTileBytes = 4 * 256 * kStepBytes;  // activation tile rings: 4 x 256, 8 x 128 or 8 x 64 tokens
constexpr int kNextTableBytes = 2048;  // block-wise tables: raw next tables of a wavefront's 64 rows (x 4 wavefronts x 2)

struct LargeArgs {
  const uint8_t* idx;
  const uint16_t* cent;
  int prepacked;
  int N, K;
  const uint16_t* A;           // [rows, K] bf16 or f16
  const int32_t* a_gather;     // sorted row -> row of A, or NULL
  const float* row_scale;
  const int32_t* scale_gather; // sorted row -> entry of row_scale, or NULL
  void* out;
  int out_ld;
  const int32_t* tiles;    // 256-token tiles [cap][4]: group, first row (absolute sorted row), row count, unused
  const int32_t* tiles128; // 128-token tiles, same layout
  const int32_t* tiles64;  // 64-token tiles, same layout
  const int32_t* n_tiles;  // the builder's counts: [0] entries in tiles, [1] in tiles128, [5] in tiles64
  int row_tiles;          // N / 256
  int nblk;               // centroid tables per weight row (1: one table over all of K)
  int gsteps;             // K steps per table (block-wise tables: group size / 64, a multiple of 8)
  // K split (block-wise tables, plain products of few rows): workgroups with blockIdx.y = z take the K steps
  // [z * ksteps, (z+1) * ksteps), a whole number of table groups, and store fp32 partial sums at
  // out + z * part_stride elements; ksteps covers all of K when there is no split
  int ksteps;
  size_t part_stride;
  // K split of the narrow tiles of a plain fp32 product with a long K (tail_part != NULL): the builder chooses
  // S = n_tiles[6] in {1, 2, 4}; split z > 0 of the j-th 128-token (64-token) tile stores its partial sums at
  // rows j*128 (tail_rows128 + j*64) of slice z-1 of tail_part, [S-1][tail_rows][N] fp32 -- or, when the launch
  // has fewer rows than such slots (tail_abs), at the tile's own sorted rows -- and tail_sum_kernel adds them to
  // `out` in the order z = 1, 2, ...
  float* tail_part;
  int tail_rows128;   // rows reserved for the 128-token tiles (capacity of that list * 128)
  int tail_rows;      // rows per slice
  int tail_abs;       // 1: a slice has M_total rows and a tile stores at its own sorted rows (fewer rows than slots)
};

#ifndef CQ_TAIL_SPLIT_MAX
#define CQ_TAIL_SPLIT_MAX 4
#endif
constexpr int kTailSplitMax = CQ_TAIL_SPLIT_MAX;   // most K parts a narrow tile is cut into (1: never)
constexpr int kTailMinSteps = 128;   // K steps (of 64) from which the narrow tiles of a plain product may be split

__device__ __forceinline__ uint32_t f32_to_f16_sat(float x) {
  x = fminf(fmaxf(x, -65504.f), 65504.f);
  const _Float16 h = (_Float16)x;
  return (uint32_t) __builtin_bit_cast(uint16_t, h);
}
__device__ __forceinline__ uint32_t code_bf16(int c) { return __float_as_uint((float)c) >> 16; }

template <bool F16>
__device__ __forceinline__ cq_v16f mfma_large(const cq_v4u a, const cq_v4u b, cq_v16f c) {
  if constexpr (F16)
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(cq_v8f16, a), __builtin_bit_cast(cq_v8f16, b), c,
                                                  0, 0, 0);
  else
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(cq_v8bf16, a),
                                                   __builtin_bit_cast(cq_v8bf16, b), c, 0, 0, 0);
}

using namespace cq_async;

// LDS row stride (bytes) of the epilogue's staging tile of 64 tokens x the workgroup's output columns
constexpr int epilogue_row_stride(int epi, int outk) {
  const int esize = outk == CQ_OUT_F16 ? 2 : 4;
  const int row = (epi == CQ_EPI_SWIGLU ? kLargeRows / 2 : kLargeRows) * esize;
  const int quad = (epi == CQ_EPI_SWIGLU ? 2 : 4) * esize;
  return row + (quad == 16 ? 16 : 8);
}

// One tile: 256 weight rows (row tile rt) x up to 32*C tokens (rows mrow0 .. mrow0+mcnt-1 of group grp).
// F16: the activations are f16 (else bf16); C = CT/32 token blocks (8, 4 or 2); D = depth of the load
// pipeline in K steps (a power of two; narrow tiles spend less matrix time per step and need more).
// BLK: block-wise centroid tables (p.nblk per row, each serving p.gsteps K steps).  PRE: the indices are the
// prepacked copy (whose nibble arrangement decodes with four operations fewer per 8 weights).
// kz / kS: this workgroup takes part kz of kS equal parts of K (narrow tiles of a plain fp32 product; 0 / 1
// otherwise) and, for kz > 0, stores at row tail_row0 of slice kz-1 of p.tail_part instead of p.out.
template <bool F16, int EPI, int OUTK, int C, int D, bool BLK, bool PRE>
__device__ __forceinline__ void large_tile(const LargeArgs& p, const int grp, const int mrow0, const int mcnt,
                                           const int rt, const int kz = 0, const int kS = 1, const int tail_row0 = 0) {
  constexpr bool kTail = !BLK && EPI == CQ_EPI_NONE && OUTK == CQ_OUT_F32;
  constexpr int CT = 32 * C;
  constexpr uint32_t kBufBytes = CT * kStepBytes;  // one activation tile: CT tokens x 128 bytes

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int r32 = lane & 31, g2 = lane >> 5;
  const int N = p.N, K = p.K;
  const size_t rowbytes = (size_t)K >> 1;
  const int n0 = rt * kLargeRows + wave * 64;  // this wavefront's 64 rows
  const uint8_t* wbase = p.idx + ((size_t)grp * N + n0) * rowbytes;
  const uint8_t *wp0, *wp1;  // this lane's 16 bytes of step 0, for each of its two rows
  int sstride;
  if constexpr (PRE) {
    wp0 = wbase + (size_t)lane * 16;
    wp1 = wbase + 32 * rowbytes + (size_t)lane * 16;
    sstride = 1024;
  } else {
    wp0 = wbase + (size_t)r32 * rowbytes + g2 * 16;
    wp1 = wbase + (size_t)(32 + r32) * rowbytes + g2 * 16;
    sstride = 32;
  }
  // this workgroup's K range: steps [sb, sb + nS) (all of K unless the launch splits K)
  int sb = BLK ? (int)blockIdx.y * p.ksteps : 0;
  int nS = BLK ? min(p.ksteps, K / kStepK - sb) : K / kStepK;
  if constexpr (kTail) {
    if (kS > 1) {   // equal parts of an even number of steps (the last one takes what is left: at least two)
      const int per = ((nS + kS - 1) / kS + 1) & ~1;
      sb = kz * per;
      nS = min(per, nS - sb);
    }
  }
  if constexpr (BLK || kTail) {
    wp0 += (size_t)sb * sstride;
    wp1 += (size_t)sb * sstride;
  }

  const int nblk = BLK ? p.nblk : 1;
  const uint16_t* cgrp = p.cent + (size_t)grp * N * nblk * CQ_N_CENTROIDS;   // this group's tables (uniform)
  const int blk0 = BLK ? sb / p.gsteps : 0;                                     // first table group of the K range
  const uint32_t crow_off = ((uint32_t)(n0 + r32) * nblk + blk0) * (CQ_N_CENTROIDS * 2);  // row r32's first table, bytes
  const uint32_t crow_skip = 32u * nblk * (CQ_N_CENTROIDS * 2);                // from row r32 to row 32 + r32
  RowTable t0 = make_row_table<F16>(reinterpret_cast<const uint16_t*>(reinterpret_cast<const uint8_t*>(cgrp) + crow_off));
  RowTable t1 = make_row_table<F16>(
      reinterpret_cast<const uint16_t*>(reinterpret_cast<const uint8_t*>(cgrp) + crow_off + crow_skip));
  // Block-wise tables: the raw centroids of the next group of weights wait in LDS above the activation
  // tiles, 2 KiB per wavefront and parity of the group (two direct-to-LDS loads: lane (r32, g2) moves half
  // g2 of the 32-byte table of row r32, then of row 32 + r32), and become register tables when that group
  // starts.  Nothing but one byte offset per lane stays in registers meanwhile.
  int blk_next = 1;            // group (counted from the range's first) whose tables were requested last
  int switch_at = p.gsteps;    // first K step of that group
  const uint32_t tbl_lds = __builtin_amdgcn_readfirstlane(D * kBufBytes + wave * kNextTableBytes);  // above the ring
  auto fetch_tables = [&](int b) {
    // (clamped to the row's last table)
    const uint8_t* src = reinterpret_cast<const uint8_t*>(cgrp) + (size_t)min(b, nblk - 1 - blk0) * (CQ_N_CENTROIDS * 2);
    const uint32_t at = tbl_lds + (b & 1) * (4 * kNextTableBytes);
    const uint32_t lane_off = crow_off + g2 * 16;
    load_global_to_lds_s<0>(at, src, lane_off);
    load_global_to_lds_s<0>(at + 1024, src, lane_off + crow_skip);
  };

  // ---- activation tiles ----
  // LDS tile: token-major, 128 bytes (8 chunks of 8 k) per token; chunk c of token t sits at position
  // c ^ ((t >> 1) & 7) of the token's row.  With that swizzle the 16 lanes of one phase of a fragment
  // read (16 consecutive tokens, same chunk) hit 16 different 16-byte bank groups.
  // Transfer: one direct-to-LDS load moves 8 tokens x 128 bytes (8 lanes per token: whole contiguous
  // row segments on the global side, 1 KiB contiguous in LDS).  The swizzle is applied on the global
  // side: lane (token, position) fetches chunk position ^ ((token >> 1) & 7).  Wavefront w moves
  // tokens [w*CT/4, (w+1)*CT/4) of every step: C loads.
  // Tokens past the end of the tile load the tile's last row instead (no branches in the pipeline);
  // a token is one output column, and those columns are never stored.
  const uint8_t* ap[C];
#pragma unroll
  for (int i = 0; i < C; ++i) {
    const int tok = wave * (CT / 4) + i * 8 + (lane >> 3);
    const int m = mrow0 + min(tok, mcnt - 1);
    const size_t row = (size_t)(p.a_gather ? p.a_gather[m] : m);
    const int chunk = (lane & 7) ^ ((tok >> 1) & 7);
    ap[i] = reinterpret_cast<const uint8_t*>(p.A) + (row * (size_t)K + (size_t)sb * kStepK + chunk * 8) * 2;
  }
  const uint32_t lds_wave = __builtin_amdgcn_readfirstlane(wave * (CT / 4) * kStepBytes);
  // this wavefront's loads i0 .. i0+n-1 of the activations of step s into tile `buf`
  auto fetch_tile = [&](int s, int buf, int i0, int n) {
    const size_t o = (size_t)s * kStepBytes;
#pragma unroll
    for (int i = 0; i < C; ++i)
      if (i >= i0 && i < i0 + n) load_global_to_lds(buf * kBufBytes + lds_wave + i * 1024, ap[i] + o);
  };
  auto fetch_weights = [&](cq_v4u (&w)[2], int s) {
    const size_t o = (size_t)s * sstride;
    load_global_async(w[0], wp0 + o);
    load_global_async(w[1], wp1 + o);
  };
  // fragment read: lane (token r32 of block cb, k group g2) wants chunk g2*4 + jj of sub-step jj
  const uint32_t boff = (uint32_t)r32 * kStepBytes + ((uint32_t)((g2 * 4) ^ ((r32 >> 1) & 7)) << 4);
  auto read_b = [&](int buf, int jj, int cb) {
    return lds_read_u128((boff ^ ((uint32_t)jj << 4)) + buf * kBufBytes + cb * 32 * kStepBytes);
  };

  cq_v16f acc[2][C];
#pragma unroll
  for (int rb = 0; rb < 2; ++rb)
#pragma unroll
    for (int cb = 0; cb < C; ++cb)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[rb][cb][i] = 0.f;

  // Pipeline: at the start of step s the weights and the activation tile of step s+D-1 are requested
  // (weights: ring of D register pairs; tiles: ring of D LDS buffers, tile s in buffer s%D).  At the
  // end of step s every wavefront waits for its own share of tile s+2 (the loads of the D-3 steps
  // requested after it may stay in flight), then the workgroup barrier publishes it; the last sub-step
  // of step s+1 already reads from it.  The barrier also retires tile s, which the requests of step
  // s+1 overwrite.  Loads thus have D-2 full steps to arrive (two steps = about 2 us for 256 tokens).
  // vector-memory loads a wavefront issues per step: the wait counts below depend on it
  constexpr int kPerStep = C + 2;  // C tile loads + 2 weight loads
  constexpr int kInFlight = (D - 3) * kPerStep;
  static_assert(D >= 4 && (D & (D - 1)) == 0 && kInFlight < 64, "ring depth / vmcnt range");
  static_assert(2 * kPerStep > 2 && kInFlight + kPerStep + 2 < 64,
                "the waits of D - 1 steps retire the table loads before they are used");
  cq_v4u wq[D][2];
#pragma unroll
  for (int i = 0; i < D - 1; ++i) {
    // (block-wise tables: the first request for tables sits where the loop's requests will sit, in front
    // of the last step requested ahead -- the wait counts below are the same in every pass)
    if constexpr (BLK) {
      if (i == D - 2) fetch_tables(1);
    }
    fetch_weights(wq[i], min(i, nS - 1));
    fetch_tile(min(i, nS - 1), i, 0, C);
  }
  vm_wait<kInFlight>(wq[0][0], wq[0][1], wq[1][0], wq[1][1]);
  __syncthreads();

  // Software pipeline over the 16-wide K sub-steps.  While the matrix cores work through the 2*C MFMAs
  // of one sub-step, the vector ALU decodes the A fragments of the next one and LDS delivers its B
  // fragments (a wavefront issues in order, so the pipes only overlap if their instructions alternate;
  // the group barriers below ask the scheduler for exactly that).
  // The B fragments live in one register set: as soon as the two MFMAs of a token block are issued,
  // its registers take the block's fragment of the next sub-step (a full sub-step of slack).
  cq_v4u af[2][2];
  cq_v4u bfr[C];
  uint32_t ident = 0x03020100u;   // kept in a vector register (see decode8)
  asm volatile("" : "+v"(ident));
  af[0][0] = decode8<PRE>(wq[0][0][0], t0, ident);
  af[0][1] = decode8<PRE>(wq[0][1][0], t1, ident);
#pragma unroll
  for (int cb = 0; cb < C; ++cb) bfr[cb] = read_b(0, 0, cb);

  int s0 = 0;
  do {  // at least two steps exist (no zero-trip path: the accumulators stay in their AGPRs throughout)
#pragma unroll
    for (int par = 0; par < D; ++par) {  // step s0 + par uses weights wq[par] and tile buffer par
      if (par > 0 && (par & 1) == 0 && s0 + par >= nS) break;  // K is a multiple of 128: steps come in pairs
      const int s3 = min(s0 + par + D - 1, nS - 1);
      fetch_weights(wq[(par + D - 1) & (D - 1)], s3);
#pragma unroll
      for (int jj = 0; jj < 4; ++jj) {
        const int cur = jj & 1, nxt = cur ^ 1;
        if constexpr (BLK) {
          if (par == D - 1 && jj == 3) {
            // A group of weights ends with this step (groups are whole multiples of D steps, so only here;
            // the branch sits at a sub-step boundary, where the instruction scheduler is fenced anyway).
            // Its successor's tables were requested at least D steps ago and have arrived: the waits since
            // left fewer loads outstanding than were issued after that request.  The wait below never
            // stalls (no more than that many loads are ever outstanding); it orders the LDS reads behind
            // the arrival.
            if (s0 + D == switch_at) {
              asm volatile("s_waitcnt vmcnt(%0)" ::"n"(kInFlight + kPerStep + 2) : "memory");
              const uint32_t at = tbl_lds + (blk_next & 1) * (4 * kNextTableBytes) + r32 * 16;
              const cq_v4u a0 = lds_read_u128(at), a1 = lds_read_u128(at + 512);
              const cq_v4u b0 = lds_read_u128(at + 1024), b1 = lds_read_u128(at + 1536);
              uint32_t r0[8] = {a0[0], a0[1], a0[2], a0[3], a1[0], a1[1], a1[2], a1[3]};
              uint32_t r1[8] = {b0[0], b0[1], b0[2], b0[3], b1[0], b1[1], b1[2], b1[3]};
              t0 = make_row_table<F16>(r0);
              t1 = make_row_table<F16>(r1);
              ++blk_next;
              switch_at += p.gsteps;
            }
            // The tables of the group after the current one are requested in EVERY pass (again, if they
            // were requested before: 2 KiB per wavefront from L2, the same bytes to the same place), so
            // that the number of loads in flight, and with it every wait count, is a compile-time constant.
            fetch_tables(blk_next);
          }
        }
        // the C tile loads are spread over the step: no LDS write bursts
        if constexpr (C >= 4) fetch_tile(s3, (par + D - 1) & (D - 1), jj * (C / 4), C / 4);
        else if (jj < C) fetch_tile(s3, (par + D - 1) & (D - 1), jj, 1);
        // next sub-step: jj + 1 of this step, or the first one of the next step
        const int nbuf = jj < 3 ? par : (par + 1) & (D - 1), njj = (jj + 1) & 3;
        af[nxt][0] = decode8<PRE>(wq[nbuf][0][njj], t0, ident);
        af[nxt][1] = decode8<PRE>(wq[nbuf][1][njj], t1, ident);
#pragma unroll
        for (int cb = 0; cb < C; ++cb) {
          const cq_v4u b = bfr[cb];
          acc[0][cb] = mfma_large<F16>(af[cur][0], b, acc[0][cb]);
          acc[1][cb] = mfma_large<F16>(af[cur][1], b, acc[1][cb]);
          bfr[cb] = read_b(nbuf, njj, cb);
        }
#pragma unroll
        for (int i = 0; i < 2 * C; ++i) {
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                   // one MFMA
          __builtin_amdgcn_sched_group_barrier(0x002, 4, 0);                   // four vector ALU operations
          if (i % 2 == 1) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);   // one LDS read
        }
        __builtin_amdgcn_sched_barrier(0);
      }
      // (block-wise tables: the two table requests of a pass's last step are younger than what the waits
      // of that step and of the next D - 4 steps are for, and may stay in flight as well)
      // (par is a constant once the loop is unrolled: no branch is left here)
      if (BLK && (par == D - 1 || par <= D - 5))
        vm_wait<kInFlight + 2>(wq[(par + 2) & (D - 1)][0], wq[(par + 2) & (D - 1)][1]);
      else
        vm_wait<kInFlight>(wq[(par + 2) & (D - 1)][0], wq[(par + 2) & (D - 1)][1]);
      __syncthreads();
    }
    s0 += D;
  } while (s0 < nS);
  // nothing of this workgroup may still be on its way into LDS when the loop is left
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");

  // ---- epilogue: per-token scale, optional SiLU(gate)*up, store ----
  // A lane holds 4 consecutive outputs of ONE token per accumulator quad, so storing from registers
  // would touch 64 different cache lines per instruction.  Instead the tile goes through LDS (free
  // now) 64 tokens at a time: row-major [token][this workgroup's columns] with a padded row stride
  // (conflict-free writes), then the workgroup streams whole rows out, neighbouring lanes writing
  // neighbouring bytes.
  constexpr int kOutCols = EPI == CQ_EPI_SWIGLU ? kLargeRows / 2 : kLargeRows;
  constexpr int kEsize = OUTK == CQ_OUT_F16 ? 2 : 4;
  constexpr int kRowBytes = kOutCols * kEsize;                    // 256 .. 1024
  constexpr int kQuadBytes = (EPI == CQ_EPI_SWIGLU ? 2 : 4) * kEsize;  // what one accumulator quad becomes
  constexpr int kRowStride = kRowBytes + (kQuadBytes == 16 ? 16 : 8);
  constexpr int kPiece = kRowStride % 16 == 0 ? 16 : 8;           // bytes per lane when streaming out
  constexpr int kPiecesPerRow = kRowBytes / kPiece;
  static_assert(kRowStride == epilogue_row_stride(EPI, OUTK), "the launcher sizes LDS with the same formula");
  const size_t out_col0 = (size_t)rt * kOutCols;
  typedef __attribute__((address_space(3))) uint32_t lds_u32;
  typedef __attribute__((address_space(3))) cq_v4u lds_v4u;
  typedef __attribute__((__vector_size__(2 * sizeof(uint32_t)))) uint32_t v2u;
  typedef __attribute__((address_space(3))) v2u lds_v2u;
#pragma unroll
  for (int pass = 0; pass < (C + 1) / 2; ++pass) {
    __syncthreads();  // the tile buffers (first pass) or the previous pass's rows are no longer read
#pragma unroll
    for (int half = 0; half < (C >= 2 ? 2 : 1); ++half) {
      const int cb = pass * 2 + half;
      const int tl = half * 32 + r32;  // token within the pass
      float sc = 1.f;
      if (p.row_scale) {
        const int m = mrow0 + min(cb * 32 + r32, mcnt - 1);
        sc = p.row_scale[p.scale_gather ? p.scale_gather[m] : m];
      }
#pragma unroll
      for (int rb = 0; rb < 2; ++rb) {
#pragma unroll
        for (int vb = 0; vb < 4; ++vb) {
          // MFMA 32x32 output: register v holds row 8*(v/4) + 4*(lane/32) + v%4, column lane%32
          const int quad = (wave * 64 + rb * 32 + vb * 8 + g2 * 4) >> 2;  // which 4 weight rows of the tile
          const uint32_t at = (uint32_t)tl * kRowStride + (uint32_t)quad * kQuadBytes;
          const float x0 = sc * acc[rb][cb][4 * vb], x1 = sc * acc[rb][cb][4 * vb + 1];
          const float x2 = sc * acc[rb][cb][4 * vb + 2], x3 = sc * acc[rb][cb][4 * vb + 3];
          if constexpr (EPI == CQ_EPI_SWIGLU) {
            const float h0 = x0 * __builtin_amdgcn_rcpf(1.f + __expf(-x0)) * x1;
            const float h1 = x2 * __builtin_amdgcn_rcpf(1.f + __expf(-x2)) * x3;
            if constexpr (OUTK == CQ_OUT_F16)
              *reinterpret_cast<lds_u32*>((uintptr_t)at) = f32_to_f16_sat(h0) | (f32_to_f16_sat(h1) << 16);
            else
              *reinterpret_cast<lds_v2u*>((uintptr_t)at) = v2u{__float_as_uint(h0), __float_as_uint(h1)};
          } else {
            if constexpr (OUTK == CQ_OUT_F16)
              *reinterpret_cast<lds_v2u*>((uintptr_t)at) = v2u{f32_to_f16_sat(x0) | (f32_to_f16_sat(x1) << 16),
                                                                f32_to_f16_sat(x2) | (f32_to_f16_sat(x3) << 16)};
            else
              *reinterpret_cast<lds_v4u*>((uintptr_t)at) =
                  cq_v4u{__float_as_uint(x0), __float_as_uint(x1), __float_as_uint(x2), __float_as_uint(x3)};
          }
        }
      }
    }
    __syncthreads();
    // stream the 64 rows out: piece i of the pass = (token i / kPiecesPerRow, piece i % kPiecesPerRow)
#pragma unroll
    for (int it = 0; it < 64 * kPiecesPerRow / 256; ++it) {
      const int i = it * 256 + tid;
      const int tl = i / kPiecesPerRow, pc = i - tl * kPiecesPerRow;
      const int tok = pass * 64 + tl;
      if (tok < mcnt) {
        const uint32_t at = (uint32_t)tl * kRowStride + (uint32_t)pc * kPiece;
        char* dst = reinterpret_cast<char*>(p.out) + ((size_t)(mrow0 + tok) * p.out_ld + out_col0) * kEsize + (size_t)pc * kPiece;
        if constexpr (BLK) dst += (size_t)blockIdx.y * p.part_stride * kEsize;
        if constexpr (kTail) {
          if (kz > 0)
            dst = reinterpret_cast<char*>(p.tail_part) +
                  (((size_t)(kz - 1) * p.tail_rows + tail_row0 + tok) * p.out_ld + out_col0) * kEsize + (size_t)pc * kPiece;
        }
        if constexpr (kPiece == 16)
          *reinterpret_cast<cq_v4u*>(dst) = *reinterpret_cast<const lds_v4u*>((uintptr_t)at);
        else
          *reinterpret_cast<v2u*>(dst) = *reinterpret_cast<const lds_v2u*>((uintptr_t)at);
      }
    }
  }
}

// Work items = (token tile, row tile); tiles of 256, 128 and 64 tokens in ONE launch so that the
// short lists do not leave most of the chip idle.  XCD-aware remap of the linear workgroup id (ids go
// round-robin over the 8 XCDs): XCD x takes a contiguous share of the 256-token work and then a
// contiguous share of the 128-token and of the 64-token work (neighbours share activations in its L2;
// equal mix on every XCD).  The grid is sized for the worst case; the lists are usually much shorter.
template <bool F16, int EPI, int OUTK, bool BLK, bool PRE>
__global__ __launch_bounds__(256, 1) void gemm_large_kernel(const LargeArgs p) {
  const int kS = p.tail_part ? p.n_tiles[6] : 1;   // K parts of a narrow tile
  const int kS256 = p.tail_part && p.tail_abs ? p.n_tiles[7] : 1;   // ... of a 256-token tile (launches of few tiles)
  const int n256 = p.n_tiles[0] * p.row_tiles * kS256, n128 = p.n_tiles[1] * p.row_tiles * kS,
            n64 = p.n_tiles[5] * p.row_tiles * kS;
  const int per256 = (n256 + 7) >> 3, per128 = (n128 + 7) >> 3, per64 = (n64 + 7) >> 3;
  const int xcd = blockIdx.x & 7;
  int slot = blockIdx.x >> 3;
  if (slot < per256) {
    const int work = xcd * per256 + slot;
    if (work >= n256) return;
    const int item = work / kS256, kz = work - item * kS256;
    const int tile = item / p.row_tiles, rt = item - tile * p.row_tiles;
    const int32_t* t = p.tiles + tile * 4;
    large_tile<F16, EPI, OUTK, 8, 4, BLK, PRE>(p, t[0], t[1], t[2], rt, kz, kS256, t[1]);
    return;
  }
  slot -= per256;
  if (slot < per128) {
    const int work = xcd * per128 + slot;
    if (work >= n128) return;
    const int item = work / kS, kz = work - item * kS;
    const int tile = item / p.row_tiles, rt = item - tile * p.row_tiles;
    const int32_t* t = p.tiles128 + tile * 4;
    large_tile<F16, EPI, OUTK, 4, 8, BLK, PRE>(p, t[0], t[1], t[2], rt, kz, kS, p.tail_abs ? t[1] : tile * 128);
    return;
  }
  slot -= per128;
  if (slot < per64) {
    const int work = xcd * per64 + slot;
    if (work >= n64) return;
    const int item = work / kS, kz = work - item * kS;
    const int tile = item / p.row_tiles, rt = item - tile * p.row_tiles;
    const int32_t* t = p.tiles64 + tile * 4;
    large_tile<F16, EPI, OUTK, 2, 8, BLK, PRE>(p, t[0], t[1], t[2], rt, kz, kS,
                                               p.tail_abs ? t[1] : p.tail_rows128 + tile * 64);
  }
}

// out[row] += slice 0 + slice 1 + ... of the narrow tiles' K parts, in that order (see LargeArgs::tail_part).
// blockIdx.y: entry of the 128-token list, then of the 64-token list; blockIdx.x: 1024 columns; blockIdx.z: 8 rows.
constexpr int kTailSumRows = 8;
__global__ __launch_bounds__(256) void tail_sum_kernel(const LargeArgs p, int cap128) {
  // blockIdx.y: entries of the 128-token list, of the 64-token list, then (launches of few tiles) of the 256-token list
  const int list = (int)blockIdx.y < cap128 ? 0 : (int)blockIdx.y < 2 * cap128 ? 1 : 2;
  const int j = (int)blockIdx.y - list * cap128;
  const int kS = list == 2 ? p.n_tiles[7] : p.n_tiles[6];
  if (kS <= 1) return;
  if (j >= (list == 0 ? p.n_tiles[1] : list == 1 ? p.n_tiles[5] : p.n_tiles[0])) return;
  const int32_t* t = (list == 0 ? p.tiles128 : list == 1 ? p.tiles64 : p.tiles) + j * 4;
  const int mrow0 = t[1], mcnt = t[2];
  const int row0 = p.tail_abs ? mrow0 : list == 1 ? p.tail_rows128 + j * 64 : j * 128;
  const int c = (blockIdx.x * 256 + threadIdx.x) * 4;
  const int r0 = blockIdx.z * kTailSumRows;
  if (c >= p.N || r0 >= mcnt) return;
  float* out = reinterpret_cast<float*>(p.out);
  float4 acc[kTailSumRows], part[kTailSumRows][kTailSplitMax > 1 ? kTailSplitMax - 1 : 1];
#pragma unroll
  for (int i = 0; i < kTailSumRows; ++i) {   // all loads first (rows past the tile's end read its last row)
    const int r = min(r0 + i, mcnt - 1);
    acc[i] = *reinterpret_cast<const float4*>(out + (size_t)(mrow0 + r) * p.N + c);
#pragma unroll
    for (int z = 1; z < kTailSplitMax; ++z)
      if (z < kS)
        part[i][z - 1] = *reinterpret_cast<const float4*>(p.tail_part + ((size_t)(z - 1) * p.tail_rows + row0 + r) * p.N + c);
  }
#pragma unroll
  for (int i = 0; i < kTailSumRows; ++i) {
    if (r0 + i >= mcnt) break;
#pragma unroll
    for (int z = 1; z < kTailSplitMax; ++z)
      if (z < kS) {
        acc[i].x += part[i][z - 1].x; acc[i].y += part[i][z - 1].y;
        acc[i].z += part[i][z - 1].z; acc[i].w += part[i][z - 1].w;
      }
    *reinterpret_cast<float4*>(out + (size_t)(mrow0 + r0 + i) * p.N + c) = acc[i];
  }
}

// Narrow tiles alone, for launches in which no group has more than 64 (C = 2) or 32 (C = 1) rows (block-wise
// tables at decode sizes): few accumulators and at most half the LDS, so two workgroups share a compute
// unit.  The list of 64-token tiles holds one entry per non-empty group in such a launch.
// (pipeline depth: 8 steps for 32-token tiles; 4 for 64-token tiles, whose accumulators leave no room for the
// register ring of 8 -- with 8 the bf16 instantiations spilled one or two registers, which kernels with
// asynchronous register loads must not do)
constexpr int narrow_depth(int C) { return C >= 2 ? 4 : 8; }
template <bool F16, int EPI, int OUTK, bool BLK, bool PRE, int C>
__global__ __launch_bounds__(256, 2) void gemm_narrow_kernel(const LargeArgs p) {
  const int n64 = p.n_tiles[5] * p.row_tiles;
  const int per64 = (n64 + 7) >> 3;
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  if (slot >= per64) return;
  const int work = xcd * per64 + slot;
  if (work >= n64) return;
  const int tile = work / p.row_tiles, rt = work - tile * p.row_tiles;
  const int32_t* t = p.tiles64 + tile * 4;
  large_tile<F16, EPI, OUTK, C, narrow_depth(C), BLK, PRE>(p, t[0], t[1], t[2], rt);
}

// Pre-pass for activation kinds the main kernel does not read: sorted row m of the result is row
// src(m) of A as bf16 (exact for integer codes) or f16 (saturating, from fp32).  8 values per thread.
template <int AK>
__global__ __launch_bounds__(256) void convert_rows_kernel(const void* __restrict__ A, const int32_t* __restrict__ gather,
                                                           int M, int K, uint16_t* __restrict__ out) {
  const int cpr = K >> 3;  // 8-value chunks per row
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= (size_t)M * cpr) return;
  const int m = (int)(i / cpr), c = (int)(i - (size_t)m * cpr);
  const size_t src = (size_t)(gather ? gather[m] : m) * K + (size_t)c * 8;
  uint32_t o[4];
  if constexpr (AK == CQ_A_INT8_CODES) {
    const uint2 raw = *reinterpret_cast<const uint2*>(reinterpret_cast<const int8_t*>(A) + src);
    const uint32_t rw[2] = {raw.x, raw.y};
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int b0 = (int)(int8_t)(rw[h] & 0xff), b1 = (int)(int8_t)((rw[h] >> 8) & 0xff);
      const int b2 = (int)(int8_t)((rw[h] >> 16) & 0xff), b3 = (int)(int8_t)(rw[h] >> 24);
      o[2 * h] = code_bf16(b0) | (code_bf16(b1) << 16);
      o[2 * h + 1] = code_bf16(b2) | (code_bf16(b3) << 16);
    }
  } else {
    const float4 f0 = *reinterpret_cast<const float4*>(reinterpret_cast<const float*>(A) + src);
    const float4 f1 = *reinterpret_cast<const float4*>(reinterpret_cast<const float*>(A) + src + 4);
    o[0] = f32_to_f16_sat(f0.x) | (f32_to_f16_sat(f0.y) << 16);
    o[1] = f32_to_f16_sat(f0.z) | (f32_to_f16_sat(f0.w) << 16);
    o[2] = f32_to_f16_sat(f1.x) | (f32_to_f16_sat(f1.y) << 16);
    o[3] = f32_to_f16_sat(f1.z) | (f32_to_f16_sat(f1.w) << 16);
  }
  *reinterpret_cast<uint4*>(out + (size_t)m * K + (size_t)c * 8) = make_uint4(o[0], o[1], o[2], o[3]);
}

// One workgroup: cut every group with more than `small_max` rows into token tiles of 256 (while more
// than 128 rows remain), then one of 128 or (up to 64 rows left) 64, in group order (deterministic), and list the non-empty groups with up
// to `small_max` rows for the streaming kernel, together with a split of their 64-row units over
// `small_wgs` workgroups.  counts: [0] 256-wide tiles, [1] 128-wide tiles, [2] small groups,
// [3] units per workgroup, [4] workgroups per small group, [5] 64-wide tiles, [6] K parts of the narrow tiles,
// [7] K parts of the 256-wide tiles.
__global__ __launch_bounds__(1024) void build_tiles_kernel(const int32_t* __restrict__ offsets, int G, int small_max,
                                                           int n_units, int small_wgs,
                                                           int32_t* __restrict__ tiles256, int32_t* __restrict__ tiles128,
                                                           int32_t* __restrict__ tiles64,
                                                           int32_t* __restrict__ small_groups,
                                                           int32_t* __restrict__ counts, int split_max, int split_all) {
  __shared__ int n256[1024], n128[1024], n64[1024], nsm[1024];
  __shared__ int base256, base128, base64, basesm;
  const int tid = threadIdx.x;
  if (tid == 0) { base256 = 0; base128 = 0; base64 = 0; basesm = 0; }
  __syncthreads();
  for (int g0 = 0; g0 < G; g0 += 1024) {
    const int g = g0 + tid;
    int a = 0, b = 0, b64 = 0, c = 0, m0 = 0, me = 0;
    if (g < G) {
      m0 = offsets[g];
      me = offsets[g + 1] - m0;
      if (me > small_max) {
        a = me / 256;
        const int rem = me - a * 256;
        if (rem > 128) ++a; else if (rem > 64) b = 1; else if (rem > 0) b64 = 1;
      } else if (me > 0) {
        c = 1;
      }
    }
    n256[tid] = a;
    n128[tid] = b;
    n64[tid] = b64;
    nsm[tid] = c;
    __syncthreads();
    if (tid == 0) {  // exclusive prefix in group order
      int s256 = base256, s128 = base128, s64 = base64, ssm = basesm;
      const int n = min(1024, G - g0);
      for (int i = 0; i < n; ++i) {
        const int x = n256[i], y = n128[i], y2 = n64[i], z = nsm[i];
        n256[i] = s256; n128[i] = s128; n64[i] = s64; nsm[i] = ssm;
        s256 += x; s128 += y; s64 += y2; ssm += z;
      }
      base256 = s256; base128 = s128; base64 = s64; basesm = ssm;
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
      if (b || b64) {
        int32_t* t = b ? tiles128 + n128[tid] * 4 : tiles64 + n64[tid] * 4;
        t[0] = g;
        t[1] = m0 + a * 256;
        t[2] = me - a * 256;
        t[3] = 0;
      }
    }
    if (c) small_groups[nsm[tid]] = g;
    __syncthreads();
  }
  if (tid == 0) {
    counts[0] = base256;
    counts[1] = base128;
    counts[2] = basesm;
    counts[5] = base64;
    // [6] K parts of the narrow tiles (split_max > 1: a plain fp32 product with a long K).  The narrow tiles
    // come last; when there are fewer of them than compute units, the tail of the launch runs on a part of the
    // chip for the length of a whole K loop -- parts of K on more workgroups shorten it.
    {
      const int narrow = (base128 + base64) * (n_units / 4);
      int parts = 1;
      while (parts < split_max && narrow > 0 && narrow * parts * 2 <= 256) parts *= 2;
      counts[6] = parts;
      // [7] K parts of the 256-token tiles: a launch of few tiles in all (split_all: its partial sums are kept by
      // sorted row, so any tile can have them) leaves most of the chip idle for a whole K loop otherwise
      const int all = narrow + base256 * (n_units / 4);
      parts = 1;
      while (split_all && parts < split_max && base256 > 0 && all * parts * 2 <= 256) parts *= 2;
      counts[7] = parts;
    }
    // fewest units per workgroup such that all small groups fit into small_wgs workgroups
    int upw = 1, chunks = n_units;
    if (basesm > 0) {
      const int per_group = max(1, small_wgs / basesm);       // workgroups a group may take
      upw = (n_units + per_group - 1) / per_group;
      chunks = (n_units + upw - 1) / upw;
    }
    counts[3] = upw;
    counts[4] = chunks;
  }
}

template <bool F16, int EPI, int OUTK, bool BLK, bool PRE, int C>
cq_status launch_narrow(const LargeArgs& a, int max128, hipStream_t s) {
  auto kern = gemm_narrow_kernel<F16, EPI, OUTK, BLK, PRE, C>;
  constexpr int lds_epi = 64 * epilogue_row_stride(EPI, OUTK);
  constexpr int lds_loop = narrow_depth(C) * 32 * C * kStepBytes + (BLK ? 8 * kNextTableBytes : 0);
  constexpr int lds = lds_loop > lds_epi ? lds_loop : lds_epi;
  static_assert(2 * lds <= 160 * 1024, "two workgroups per compute unit");
  static std::atomic<bool> configured{false};
  const cq_status st = cq_configure_lds(kern, lds, configured, true);
  if (st != CQ_OK) return st;
  const long grid = (((long)max128 * a.row_tiles + 7) / 8) * 8;
  if (grid <= 0) return CQ_OK;
  const int total = a.K / kStepK;
  hipLaunchKernelGGL(kern, dim3((unsigned)grid, (unsigned)((total + a.ksteps - 1) / a.ksteps)), dim3(256), lds, s, a);
  return cq_check_launch();
}

// narrow: 64 or 32 when the caller knows that no group has more rows than that, else 0
template <bool F16, int EPI, int OUTK, bool BLK, bool PRE>
cq_status launch_both(LargeArgs a, const int32_t* t256, const int32_t* t128, const int32_t* counts, int max256,
                      int max128, int narrow, hipStream_t s) {
  a.tiles = t256;
  a.tiles128 = t128;
  a.tiles64 = t128 + (size_t)max128 * 4;
  a.n_tiles = counts;
  constexpr int lds_epi = 64 * epilogue_row_stride(EPI, OUTK);
  if constexpr (BLK) {
    if (narrow == 32) return launch_narrow<F16, EPI, OUTK, BLK, PRE, 1>(a, max128, s);
    if (narrow == 64) return launch_narrow<F16, EPI, OUTK, BLK, PRE, 2>(a, max128, s);
  }
  auto kern = gemm_large_kernel<F16, EPI, OUTK, BLK, PRE>;
  constexpr int lds_loop = kLdsTileBytes + (BLK ? 8 * kNextTableBytes : 0);
  constexpr int lds = lds_loop > lds_epi ? lds_loop : lds_epi;
  static std::atomic<bool> configured{false};
  const cq_status st = cq_configure_lds(kern, lds, configured, true);
  if (st != CQ_OK) return st;
  // worst case of the kernel's per-XCD shares (a group ends in at most one 128- or 64-token tile, but the
  // two lists round up separately): ceil(n256/8) + ceil(n128/8) + ceil(n64/8) slots on each of 8 XCDs
  const long w256 = (long)max256 * a.row_tiles * (a.tail_part && a.tail_abs ? kTailSplitMax : 1),
             w128 = (long)max128 * a.row_tiles * (a.tail_part ? kTailSplitMax : 1);   // (narrow tiles may come in K parts)
  const long grid = ((w256 + 7) / 8 + (w128 + 7) / 8 + 1) * 8;
  if (grid <= 0) return CQ_OK;
  hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(256), lds, s, a);
  return cq_check_launch();
}

template <bool F16, bool BLK, bool PRE>
cq_status dispatch_large_pre(const LargeArgs& a, int epilogue, int out_kind, const int32_t* t256, const int32_t* t128,
                             const int32_t* counts, int max256, int max128, int narrow, hipStream_t s) {
  if (epilogue == CQ_EPI_SWIGLU)
    return out_kind == CQ_OUT_F16
               ? launch_both<F16, CQ_EPI_SWIGLU, CQ_OUT_F16, BLK, PRE>(a, t256, t128, counts, max256, max128, narrow, s)
               : launch_both<F16, CQ_EPI_SWIGLU, CQ_OUT_F32, BLK, PRE>(a, t256, t128, counts, max256, max128, narrow, s);
  return out_kind == CQ_OUT_F16
             ? launch_both<F16, CQ_EPI_NONE, CQ_OUT_F16, BLK, PRE>(a, t256, t128, counts, max256, max128, narrow, s)
             : launch_both<F16, CQ_EPI_NONE, CQ_OUT_F32, BLK, PRE>(a, t256, t128, counts, max256, max128, narrow, s);
}

template <bool F16, bool BLK>
cq_status dispatch_large_blk(const LargeArgs& a, int epilogue, int out_kind, const int32_t* t256, const int32_t* t128,
                             const int32_t* counts, int max256, int max128, int narrow, hipStream_t s) {
  return a.prepacked
             ? dispatch_large_pre<F16, BLK, true>(a, epilogue, out_kind, t256, t128, counts, max256, max128, narrow, s)
             : dispatch_large_pre<F16, BLK, false>(a, epilogue, out_kind, t256, t128, counts, max256, max128, narrow, s);
}

// The two-workgroup kernel for 64-token tiles exists for block-wise tables only (the streaming kernel takes
// the small groups otherwise).
template <bool F16>
cq_status dispatch_large(const LargeArgs& a, int epilogue, int out_kind, const int32_t* t256, const int32_t* t128,
                         const int32_t* counts, int max256, int max128, int narrow, hipStream_t s) {
  return a.nblk > 1
             ? dispatch_large_blk<F16, true>(a, epilogue, out_kind, t256, t128, counts, max256, max128, narrow, s)
             : dispatch_large_blk<F16, false>(a, epilogue, out_kind, t256, t128, counts, max256, max128, 0, s);
}

size_t tile_list_bytes(int G, int M_total) {
  int c256, c128;
  cq_large_tile_caps(G, M_total, &c256, &c128);
  return cq_align_up(256 + ((size_t)(c256 + 2 * c128) * 4 + (size_t)G) * sizeof(int32_t), 256);
}

}  // namespace

// Upper bounds on the tile counts for M_total rows in G groups (host side; sizes on the device vary).
void cq_large_tile_caps(int G, int M_total, int* cap256, int* cap128) {
  *cap256 = M_total / 129 + 1;   // every 256-wide tile covers more than 128 rows
  *cap128 = G < M_total ? G : M_total;  // at most one per group
  if (*cap128 < 1) *cap128 = 1;
}

// Narrow tiles of a plain fp32 product with a long K may be cut into K parts (LargeArgs::tail_part).
bool cq_gemm_large_tail_split(const cq_codebook_weights* W, int epilogue, int out_kind) {
  return epilogue == CQ_EPI_NONE && out_kind == CQ_OUT_F32 && cq_tables_per_row(W) == 1 &&
         W->K / kStepK >= kTailMinSteps;
}

namespace {
// rows of a slice of partial sums: a slot per possible narrow tile (128 + 64 rows per group), or the launch's own
// rows when those are fewer
int tail_slice_rows(int G, int M_total, bool* absolute) {
  int c256, c128;
  cq_large_tile_caps(G, M_total, &c256, &c128);
  *absolute = M_total < c128 * 192;
  return *absolute ? M_total : c128 * 192;
}
// partial sums of those K parts: [kTailSplitMax - 1][rows of a slice][N] fp32
size_t tail_part_bytes(int G, int M_total, int N) {
  bool absolute;
  const int rows = tail_slice_rows(G, M_total, &absolute);
  return cq_align_up((size_t)(kTailSplitMax - 1) * rows * N * sizeof(float), 256);
}
}  // namespace

// tile lists, plus (tail_N > 0: a plain fp32 product of N columns whose K is long enough) the partial sums of
// the narrow tiles' K parts, plus (with_conversion) room for the activations as 16-bit rows [M_total, K]
size_t cq_gemm_large_workspace_bytes(int G, int M_total, int K, bool with_conversion, int tail_N) {
  size_t n = tile_list_bytes(G, M_total);
  if (tail_N > 0 && K / kStepK >= kTailMinSteps) n += tail_part_bytes(G, M_total, tail_N);
  if (with_conversion) n += cq_align_up((size_t)M_total * K * sizeof(uint16_t), 256);
  return n;
}

bool cq_gemm_large_supported(const cq_codebook_weights* W) {
  if (W->N % kLargeRows != 0 || W->K % (2 * kStepK) != 0) return false;
  // block-wise tables change between two passes of the unrolled pipeline (8 steps of 64)
  // (and the kernel addresses a group's tables with 32-bit byte offsets)
  const int nblk = cq_tables_per_row(W);
  return nblk == 1 || (W->group_k % (8 * kStepK) == 0 && (long)W->N * nblk * (CQ_N_CENTROIDS * 2) < (1L << 31));
}

// Builds the work lists of both kernels in `workspace` (first step of a mixed launch).  Returns the list
// of small groups for the streaming kernel: header {count, units per workgroup, workgroups per group,
// unused} followed by the group ids... as two pointers: *small_hdr -> counts + 2, *small_ids -> ids.
cq_status cq_gemm_build_lists(const cq_codebook_weights* W, const int32_t* group_offsets, int M_total, int small_max,
                              int small_wgs, void* workspace, const int32_t** small_hdr, const int32_t** small_ids,
                              hipStream_t s, bool tail_split) {
  int cap256, cap128;
  cq_large_tile_caps(W->G, M_total, &cap256, &cap128);
  bool split_all = false;
  if (tail_split) (void)tail_slice_rows(W->G, M_total, &split_all);   // partial sums by sorted row: any tile may split
  int32_t* counts = (int32_t*)workspace;
  int32_t* t256 = counts + 64;
  int32_t* t128 = t256 + (size_t)cap256 * 4;
  int32_t* t64 = t128 + (size_t)cap128 * 4;
  int32_t* small = t64 + (size_t)cap128 * 4;
  hipLaunchKernelGGL(build_tiles_kernel, dim3(1), dim3(1024), 0, s, group_offsets, W->G, small_max, W->N / 64, small_wgs,
                     t256, t128, t64, small, counts, tail_split ? kTailSplitMax : 1, split_all ? 1 : 0);
  *small_hdr = counts + 2;
  *small_ids = small;
  return cq_check_launch();
}

// the lists must have been built by cq_gemm_build_lists in the same workspace
cq_status cq_gemm_large_launch(const cq_codebook_weights* W, const void* A, int a_kind, const float* row_scale,
                               const int32_t* row_gather, const int32_t* group_offsets, int M_total, int small_max,
                               int epilogue, void* out, int out_kind, void* workspace, hipStream_t s) {
  int cap256, cap128;
  cq_large_tile_caps(W->G, M_total, &cap256, &cap128);
  int32_t* counts = (int32_t*)workspace;
  int32_t* t256 = counts + 64;
  int32_t* t128 = t256 + (size_t)cap256 * 4;
  LargeArgs a;
  a.idx = W->prepacked ? (const uint8_t*)W->prepacked : W->idx;
  a.cent = W->cent;
  a.prepacked = W->prepacked ? 1 : 0;
  a.N = W->N;
  a.K = W->K;
  a.A = (const uint16_t*)A;
  a.a_gather = row_gather;
  a.row_scale = row_scale;
  a.scale_gather = row_gather;
  a.out = out;
  a.out_ld = epilogue == CQ_EPI_SWIGLU ? W->N / 2 : W->N;
  a.tiles = nullptr;
  a.tiles128 = nullptr;
  a.tiles64 = nullptr;
  a.n_tiles = nullptr;
  a.row_tiles = W->N / kLargeRows;
  a.nblk = cq_tables_per_row(W);
  a.gsteps = a.nblk > 1 ? W->group_k / kStepK : W->K / kStepK;
  {
    int ksplit;
    cq_gemm_split_plan(W, M_total, epilogue, &ksplit, &a.ksteps);  // a split is planned for 64-token launches only
    a.part_stride = ksplit > 1 ? (size_t)M_total * W->N : 0;
  }
  // workspace: tile lists, then the partial sums of the narrow tiles' K parts (if the launch may split them:
  // the builder was told so with the same rule), then the 16-bit copy of the rows
  size_t ws_off = tile_list_bytes(W->G, M_total);
  const bool tail = cq_gemm_large_tail_split(W, epilogue, out_kind);
  a.tail_part = nullptr;
  a.tail_rows128 = cap128 * 128;
  {
    bool absolute;
    a.tail_rows = tail_slice_rows(W->G, M_total, &absolute);
    a.tail_abs = absolute ? 1 : 0;
  }
  if (tail) {
    a.tail_part = (float*)((char*)workspace + ws_off);
    ws_off += tail_part_bytes(W->G, M_total, W->N);
  }
  if (a_kind == CQ_A_INT8_CODES || a_kind == CQ_A_F32) {
    // 16-bit copy of the rows in sorted order (the gather is applied here)
    uint16_t* A16 = (uint16_t*)((char*)workspace + ws_off);
    const size_t chunks = (size_t)M_total * (W->K / 8);
    const unsigned blocks = (unsigned)((chunks + 255) / 256);
    if (a_kind == CQ_A_INT8_CODES)
      hipLaunchKernelGGL(convert_rows_kernel<CQ_A_INT8_CODES>, dim3(blocks), dim3(256), 0, s, A, row_gather, M_total,
                         W->K, A16);
    else
      hipLaunchKernelGGL(convert_rows_kernel<CQ_A_F32>, dim3(blocks), dim3(256), 0, s, A, row_gather, M_total, W->K,
                         A16);
    a.A = A16;
    a.a_gather = nullptr;
  }
  const bool f16 = a_kind == CQ_A_F16 || a_kind == CQ_A_F32;
  // with so few rows in all, every group has at most that many: one narrow tile each
  const int narrow = M_total <= 32 ? 32 : M_total <= 64 ? 64 : 0;
  const cq_status st = f16 ? dispatch_large<true>(a, epilogue, out_kind, t256, t128, counts, cap256, cap128, narrow, s)
                           : dispatch_large<false>(a, epilogue, out_kind, t256, t128, counts, cap256, cap128, narrow, s);
  if (st != CQ_OK || !tail) return st;
  // (a launch of a few dozen workgroups that return at once when the builder chose not to split)
  a.tiles = t256;
  a.tiles128 = t128;
  a.tiles64 = t128 + (size_t)cap128 * 4;
  a.n_tiles = counts;
  hipLaunchKernelGGL(tail_sum_kernel, dim3((W->N / 4 + 255) / 256, 2 * cap128 + (a.tail_abs ? cap256 : 0), (a.tail_abs ? 256 : 128) / kTailSumRows),
                     dim3(256), 0, s, a, cap128);
  return cq_check_launch();
}
