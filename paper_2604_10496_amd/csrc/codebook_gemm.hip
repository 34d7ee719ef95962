// a6 / a7, streaming kernel: planning (K ranges, workgroups per group, which kernel takes which groups), the
// internal launcher and the entry point cq_codebook_grouped_gemm.  The kernel itself is in codebook_gemm_small.h.
#include "codebook_gemm_small.h"

namespace {

// out[m, :] = sum over the K splits of partials[s][m, :] in the order s = 0, 1, ... for the rows of the
// groups the streaming kernel handled (at most max_rows rows); other rows are left alone.
template <int OUTK>
__global__ __launch_bounds__(256) void sum_partials_kernel(const float* __restrict__ partials, size_t part_stride,
                                                           int ksplit, const int32_t* __restrict__ group_offsets,
                                                           int max_rows, int N, void* __restrict__ out) {
  const int grp = blockIdx.y;
  const int m0 = group_offsets[grp], Me = group_offsets[grp + 1] - m0;
  if (Me <= 0 || Me > max_rows) return;
  const int c = (blockIdx.x * 256 + threadIdx.x) * 4;
  if (c >= N) return;
  for (int m = m0 + blockIdx.z; m < m0 + Me; m += gridDim.z) {   // (blockIdx.z: rows of the group in parallel)
    const size_t at = (size_t)m * N + c;
    float4 acc = *reinterpret_cast<const float4*>(partials + at);
    for (int q = 1; q < ksplit; ++q) {
      const float4 v = *reinterpret_cast<const float4*>(partials + (size_t)q * part_stride + at);
      acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
    }
    if constexpr (OUTK == CQ_OUT_F16)
      *reinterpret_cast<uint2*>(reinterpret_cast<uint16_t*>(out) + at) =
          make_uint2(f32_to_f16_bits_sat(acc.x) | (f32_to_f16_bits_sat(acc.y) << 16),
                     f32_to_f16_bits_sat(acc.z) | (f32_to_f16_bits_sat(acc.w) << 16));
    else
      *reinterpret_cast<float4*>(reinterpret_cast<float*>(out) + at) = acc;
  }
}

}  // namespace


// K split of the streaming kernel.  One workgroup keeps the activations of its K range in LDS for all
// its 64-row units; with few tokens (the decode regime) a long K (the down projection) is therefore cut
// into ranges of at most 4096 that different workgroups stream, and their partial sums are added in a
// fixed order afterwards.  Plain products only (a nonlinear epilogue needs the whole sum).
// Block-wise tables on the streaming kernel's pipelined loop: tables of 1024 weights (two K steps per wavefront
// and table), groups of at most 32 rows (the loop's limit: two passes of 16), and K ranges of whole tables that give every wavefront
// exactly 8 steps (4096 weights) or 4 (2048); a nonlinear epilogue needs all of K in one range.
bool cq_gemm_blockwise_streams(const cq_codebook_weights* W, int M_total, int epilogue, int max_group_rows) {
  if (kWaves != 8 || cq_is_w2(W) || W->group_k != 1024 || W->K % 2048 != 0) return false;
  const int bound = max_group_rows > 0 && max_group_rows < M_total ? max_group_rows : M_total;
  if (bound > 32) return false;
  return epilogue == CQ_EPI_NONE || W->K == 4096;
}

void cq_gemm_split_plan(const cq_codebook_weights* W, int M_total, int epilogue, int* ksplit, int* ksteps,
                        int max_group_rows) {
  const int nS = W->K / 64;
  *ksplit = 1;
  *ksteps = nS;
  const int nblk = cq_tables_per_row(W);
  if (nblk > 1 && cq_gemm_blockwise_streams(W, M_total, epilogue, max_group_rows)) {
    *ksteps = W->K % 4096 == 0 ? 64 : 32;
    *ksplit = nS / *ksteps;
    return;
  }
  if (nblk > 1) {
    // Block-wise tables run on the large-tile kernel, one workgroup per 256 rows and group of tokens.  With
    // at most 64 rows in all (one 64-token tile per group) and a short N there are too few of those to fill
    // the chip, so K is cut into ranges of whole table groups, up to about two workgroups per compute unit.
    if (epilogue != CQ_EPI_NONE || M_total > 64 || !cq_gemm_large_supported(W)) return;
    const long wgs = (long)(W->G < M_total ? W->G : M_total) * (W->N / 256);
    long want = wgs > 0 ? 512 / wgs : 1;
    if (want > nblk) want = nblk;
    if (want <= 1) return;
    const int per = (nblk + (int)want - 1) / (int)want;   // table groups per range
    *ksteps = per * (W->group_k / 64);
    *ksplit = (nblk + per - 1) / per;
    return;
  }
  if (epilogue != CQ_EPI_NONE || M_total > 256 || nS <= 64) return;
  const int want = (nS + 63) / 64;
  const int per = ((nS + want - 1) / want + kWaves - 1) / kWaves * kWaves;  // whole rounds of the wavefronts
  *ksteps = per;
  *ksplit = (nS + per - 1) / per;
}

size_t cq_gemm_partials_bytes(const cq_codebook_weights* W, int M_total, int epilogue, int max_group_rows) {
  if (cq_is_w2(W)) return epilogue == CQ_EPI_NONE ? cq_gemm_w2_partials_bytes(W, M_total) : 0;
  int ksplit, ksteps;
  cq_gemm_split_plan(W, M_total, epilogue, &ksplit, &ksteps, max_group_rows);
  return ksplit > 1 ? cq_align_up((size_t)ksplit * M_total * W->N * sizeof(float), 256) : 0;
}

// The grouping by expert can be folded into a launch when every workgroup of it runs the pipelined unit loop
// (at most 32 rows per group, a K range of exactly 8 or 7 steps per wavefront) and one lane per assignment
// suffices: at most 32 tokens (a group has at most one row per token), at most 64 assignments and experts.
bool cq_gemm_can_fuse_route(const cq_codebook_weights* W, int T, int E, int S, int top_k, int epilogue) {
  if (kWaves != 8) return false;
  if (T < 1 || T > 32 || top_k < 1 || T * top_k > 64 || E < 1 || E > 64 || S < 0 || W->G != E + S) return false;
  // (the 2-bit kernel takes every group of a launch it supports: its workgroups all derive their rows alike)
  if (cq_is_w2(W)) return cq_gemm_w2_supported(W, CQ_A_INT8_CODES, epilogue);
  const int M_total = T * (top_k + S);
  if (cq_tables_per_row(W) > 1 && !cq_gemm_blockwise_streams(W, M_total, epilogue, T)) return false;
  if (cq_gemm_uses_large_tiles(W, M_total, epilogue, T)) return false;
  int ksplit, ksteps;
  cq_gemm_split_plan(W, M_total, epilogue, &ksplit, &ksteps, T);
  return ksplit == 1 && (ksteps == 8 * kWaves || (ksteps == 7 * kWaves && cq_tables_per_row(W) == 1));
}

cq_status cq_gemm_codebook_launch(const cq_codebook_weights* W, const void* A, int a_kind, const float* row_scale,
                                  const int32_t* row_gather, const int32_t* group_offsets, int M_total,
                                  int epilogue, void* out, int out_kind, void* workspace, hipStream_t s,
                                  int* ksplit_left, const cq_route_fuse* route, int max_group_rows) {
  if (route && !cq_gemm_can_fuse_route(W, route->T, route->E, route->S, route->top_k, epilogue))
    return CQ_ERR_UNSUPPORTED;
  if (cq_is_w2(W))
    return cq_gemm_w2_launch(W, A, a_kind, row_scale, row_gather, group_offsets, M_total, epilogue, out, out_kind,
                             workspace, s, ksplit_left, route);
  if (ksplit_left) *ksplit_left = 1;
  GemmArgs a;
  a.route = route ? *route : cq_route_fuse{nullptr, 0, 0, 0, 0, nullptr, nullptr, nullptr, nullptr};
  a.idx = W->prepacked ? (const uint8_t*)W->prepacked : W->idx;
  a.cent = W->cent;
  a.prepacked = W->prepacked ? 1 : 0;
  a.N = W->N;
  a.K = W->K;
  a.A = A;
  a.row_scale = row_scale;
  a.row_gather = row_gather;
  a.group_offsets = group_offsets;
  a.out = out;
  a.out_ld = epilogue == CQ_EPI_SWIGLU ? W->N / 2 : W->N;
  {
    // about one workgroup per compute unit: the per-workgroup prologue (activation staging, first
    // table, ring fill) is paid once and there is no partially filled last round of workgroups
    cq_gemm_split_plan(W, M_total, epilogue, &a.ksplit, &a.ksteps, max_group_rows);
    a.partials = (float*)workspace;  // partial sums first, then the large-tile kernel's lists
    a.part_stride = (size_t)M_total * W->N;
    // (a whole number of workgroups per (group, K range), at most 256 in all: 56 pairs take 4 each, not 5 --
    // 280 workgroups would run as a full round and a nearly empty one)
    // The pipelined unit loop takes 16 rows at a time: when groups of 17..32 rows are possible the launch gets a
    // second set of workgroups for rows 16.. of such groups (they return at once for the other groups).
    const int row_bound = max_group_rows > 0 && max_group_rows < M_total ? max_group_rows : M_total;
    a.halves = row_bound > 16 ? 2 : 1;
    // (when groups above 16 rows are likely -- 8 rows per group on average -- the workgroups are half as long, so
    // that the second halves, which start when a compute unit comes free, do not add a whole round)
    // Where the pipelined loop is not available (other K), a group of 17..32 rows runs the plain loop on one
    // set of workgroups, several times slower per unit than the small groups around it: many short workgroups
    // then, so that the compute units the small groups leave early take the rest of the big ones.
    const bool piped = a.ksteps == 8 * kWaves || (a.ksteps == 7 * kWaves && cq_tables_per_row(W) == 1);
    const long target = a.halves == 1 ? 256 : !piped ? 1024 : (long)M_total >= 8L * W->G ? 512 : 256;
    const long pairs = (long)W->G * a.ksplit;
    const long per_pair = pairs < target ? target / pairs : 1;
    long upw = (W->N / 64 + per_pair - 1) / per_pair;
    if (upw < 1) upw = 1;
    a.upw = (int)upw;
  }
  // Groups of up to 32 rows go to the streaming kernel above; larger ones to the large-tile kernel (when
  // the row count allows its 256-row tiles), which runs off a device-built tile list.  Block-wise tables
  // go to the large-tile kernel with every group, except tables of 1024 weights at decode sizes, which the
  // streaming kernel's pipelined loop takes (cq_gemm_blockwise_streams).
  const bool bw_streams = cq_gemm_blockwise_streams(W, M_total, epilogue, max_group_rows) && cq_tables_per_row(W) > 1;
  const bool blockwise = cq_tables_per_row(W) > 1 && !bw_streams;
  const bool large = cq_gemm_uses_large_tiles(W, M_total, epilogue, max_group_rows);
  if (blockwise && !large) return CQ_ERR_UNSUPPORTED;
  const int small_max = blockwise ? 0 : kSmallMaxRows;
  const int qt = bw_streams ? W->group_k / 512 : 0;
  a.max_rows = large ? small_max : 0x7fffffff;
  a.small_hdr = nullptr;
  a.small_ids = nullptr;
  void* large_ws = (char*)workspace + cq_gemm_partials_bytes(W, M_total, epilogue, max_group_rows);
  cq_status st;
  if (large) {
    // the host does not know which groups are small: a device-built list spreads exactly those over
    // the grid (a grid over all groups would leave most workgroups without work)
    // (the listed workgroups exist once per K range: a K-split launch lists fewer per range)
    const int listed = kListedWorkgroups / a.ksplit;
    st = cq_gemm_build_lists(W, group_offsets, M_total, small_max, W->G > listed ? W->G : listed, large_ws, &a.small_hdr,
                             &a.small_ids, s, cq_gemm_large_tail_split(W, epilogue, out_kind));
    if (st != CQ_OK) return st;
  }
  if (blockwise) {
    // (with a K split the kernel stores fp32 partial sums, per split, where the streaming kernel would)
    st = cq_gemm_large_launch(W, A, a_kind, row_scale, row_gather, group_offsets, M_total, small_max, epilogue,
                              a.ksplit > 1 ? (void*)a.partials : out, a.ksplit > 1 ? CQ_OUT_F32 : out_kind, large_ws, s);
    if (st != CQ_OK || a.ksplit == 1) return st;
    if (ksplit_left) {
      *ksplit_left = a.ksplit;  // the caller adds the partial sums itself
      return st;
    }
    const dim3 grid((W->N / 4 + 255) / 256, W->G, 16);   // (z: up to 16 rows of a group at a time)
    if (out_kind == CQ_OUT_F16)
      hipLaunchKernelGGL(sum_partials_kernel<CQ_OUT_F16>, grid, dim3(256), 0, s, a.partials, a.part_stride, a.ksplit,
                         group_offsets, 0x7fffffff, W->N, out);
    else
      hipLaunchKernelGGL(sum_partials_kernel<CQ_OUT_F32>, grid, dim3(256), 0, s, a.partials, a.part_stride, a.ksplit,
                         group_offsets, 0x7fffffff, W->N, out);
    return cq_check_launch();
  }
  switch (a_kind) {
    case CQ_A_INT8_CODES: st = cq_gemm_small_dispatch_int8(a, W->G, qt, epilogue, out_kind, s); break;
    case CQ_A_F16: st = cq_gemm_small_dispatch_f16(a, W->G, qt, epilogue, out_kind, s); break;
    case CQ_A_BF16: st = cq_gemm_small_dispatch_bf16(a, W->G, qt, epilogue, out_kind, s); break;
    default: st = cq_gemm_small_dispatch_f32(a, W->G, qt, epilogue, out_kind, s); break;
  }
  if (st != CQ_OK) return st;
  if (a.ksplit > 1) {
    if (ksplit_left && !large) {
      *ksplit_left = a.ksplit;  // the caller adds the partial sums itself (they are all there is)
    } else {
      const dim3 grid((W->N / 4 + 255) / 256, W->G, 16);   // (z: up to 16 rows of a group at a time)
      if (out_kind == CQ_OUT_F16)
        hipLaunchKernelGGL(sum_partials_kernel<CQ_OUT_F16>, grid, dim3(256), 0, s, a.partials, a.part_stride, a.ksplit,
                           group_offsets, a.max_rows, W->N, out);
      else
        hipLaunchKernelGGL(sum_partials_kernel<CQ_OUT_F32>, grid, dim3(256), 0, s, a.partials, a.part_stride, a.ksplit,
                           group_offsets, a.max_rows, W->N, out);
      st = cq_check_launch();
      if (st != CQ_OK) return st;
    }
  }
  if (!large) return st;
  return cq_gemm_large_launch(W, A, a_kind, row_scale, row_gather, group_offsets, M_total, kSmallMaxRows, epilogue,
                              out, out_kind, large_ws, s);
}


bool cq_gemm_uses_large_tiles(const cq_codebook_weights* W, int M_total, int epilogue, int max_group_rows) {
  if (cq_tables_per_row(W) > 1 && cq_gemm_blockwise_streams(W, M_total, epilogue, max_group_rows)) return false;
  // no group can have more rows than the streaming kernel takes: nothing for the large tiles to do
  if (cq_tables_per_row(W) == 1 && max_group_rows > 0 && max_group_rows <= kSmallMaxRows) return false;
  return !cq_is_w2(W) && cq_gemm_large_supported(W) && (M_total > kSmallMaxRows || cq_tables_per_row(W) > 1);
}

extern "C" size_t cq_grouped_gemm_workspace_bytes(const cq_codebook_weights* W, int M_total) {
  if (!W || W->G <= 0 || W->N <= 0 || W->K <= 0 || M_total <= 0) return 0;
  size_t need = 0;
  for (const int epi : {CQ_EPI_NONE, CQ_EPI_SWIGLU}) {   // the kernel, and with it the need, can depend on the epilogue
    size_t n = cq_gemm_partials_bytes(W, M_total, epi);
    if (cq_gemm_uses_large_tiles(W, M_total, epi))
      n += cq_gemm_large_workspace_bytes(W->G, M_total, W->K, true, W->N);  // worst case over the operand kinds
    if (n > need) need = n;
  }
  return need;
}

extern "C" cq_status cq_codebook_grouped_gemm(const cq_codebook_weights* W, const void* A, int a_kind,
                                              const float* row_scale, const int32_t* row_gather,
                                              const int32_t* group_offsets, int M_total, int epilogue, void* out,
                                              int out_kind, void* workspace, size_t workspace_bytes,
                                              cq_stream stream) {
  if (!W || !A || !group_offsets || (!out && M_total > 0)) return CQ_ERR_NULL;
  if ((!W->idx && !W->prepacked) || !W->cent) return CQ_ERR_NULL;
  if (W->G <= 0 || W->N <= 0 || W->K <= 0 || M_total < 0) return CQ_ERR_SHAPE;
  if (W->N % 64 != 0 || W->K % 64 != 0 || W->group_k < 0) return CQ_ERR_SHAPE;
  if (W->index_bits != 0 && W->index_bits != 4 && W->index_bits != 2) return CQ_ERR_UNSUPPORTED;
  if (cq_is_w2(W) && !cq_gemm_w2_supported(W, a_kind, epilogue)) return CQ_ERR_UNSUPPORTED;
  if (cq_tables_per_row(W) > 1 && !cq_gemm_large_supported(W)) return CQ_ERR_UNSUPPORTED;
  if (a_kind != CQ_A_INT8_CODES && a_kind != CQ_A_F16 && a_kind != CQ_A_F32 && a_kind != CQ_A_BF16)
    return CQ_ERR_UNSUPPORTED;
  if (epilogue != CQ_EPI_NONE && epilogue != CQ_EPI_SWIGLU) return CQ_ERR_UNSUPPORTED;
  if (out_kind != CQ_OUT_F32 && out_kind != CQ_OUT_F16) return CQ_ERR_UNSUPPORTED;
  if (M_total == 0) return CQ_OK;
  {
    const size_t need = cq_grouped_gemm_workspace_bytes(W, M_total);
    if (need > 0 && (!workspace || workspace_bytes < need)) return CQ_ERR_WORKSPACE;
  }
  return cq_gemm_codebook_launch(W, A, a_kind, row_scale, row_gather, group_offsets, M_total, epilogue, out,
                                 out_kind, workspace, (hipStream_t)stream, nullptr);
}
