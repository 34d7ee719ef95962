// a3 + a4 + a5: router logits, wavefront top-k, softmax over the selected logits, and the stable
// grouping of assignments by expert.
//
// Top-k: one wavefront per token.  Logits become order-preserving 32-bit keys; the k-th largest key
// is found by a bitwise descent that counts candidates with wave ballots (32 rounds, no sorting);
// equal keys are admitted in ascending expert id with a ballot prefix count; the <= 64 survivors are
// ranked by (logit descending, id ascending).  Permutation: a three-pass counting sort over blocks
// of 256 assignments whose in-block ranks come from ballot match masks, so the order inside every
// expert is ascending assignment number (a stable sort) and the result is unique.
#include "cq_internal.h"
#include "cq_route.h"

namespace {

using namespace cq_route;

constexpr int kMaxSlots = 16;       // experts per lane: E <= 1024
constexpr int kPermBlock = 256;     // assignments per counting-sort block (one wavefront, 4 rounds)

__global__ __launch_bounds__(256) void topk_kernel(const float* __restrict__ part, int ksplit,
                                                   const float* __restrict__ bias, int T, int E, int k,
                                                   float* __restrict__ logits_out, int32_t* __restrict__ ids,
                                                   float* __restrict__ w) {
  __shared__ uint32_t s_key[4][64];
  __shared__ int s_id[4][64];
  __shared__ float s_val[4][64];
  __shared__ float s_sorted[4][64];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int t = blockIdx.x * 4 + wave;
  const bool active = t < T;
  const int nslot = (E + 63) / 64;
  float val[kMaxSlots];
#pragma unroll
  for (int s = 0; s < kMaxSlots; ++s) {
    const int e = s * 64 + lane;
    val[s] = 0.f;
    if (s < nslot && e < E && active) {
      float x = part[(size_t)t * E + e];
      for (int z = 1; z < ksplit; ++z) x += part[((size_t)z * T + t) * E + e];
      if (bias) x += bias[e];
      if (logits_out) logits_out[(size_t)t * E + e] = x;
      val[s] = x;
    }
  }
  const size_t o = active ? (size_t)t * k : 0;
  wave_topk<kMaxSlots>(val, nslot, E, k, active, lane, s_key[wave], s_id[wave], s_val[wave], s_sorted[wave], ids + o,
                       w + o, nullptr);
}

// Router logits for decode-sized batches: one workgroup per (token, four experts); its four wavefronts
// split K, issue all their loads at once (one memory latency in total) and combine through LDS in a
// fixed order.  Plain fp32 FMAs: T*E*H is tiny here.
__global__ __launch_bounds__(256) void logits_small_kernel(const float* __restrict__ XR, const float* __restrict__ Wr,
                                                           const float* __restrict__ bias, int H, int E,
                                                           float* __restrict__ logits) {
  __shared__ float part[4][4];
  const int t = blockIdx.y, e0 = blockIdx.x * 4;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const float* xr = XR + (size_t)t * H;
  const float* wr[4];
#pragma unroll
  for (int u = 0; u < 4; ++u) wr[u] = Wr + (size_t)min(e0 + u, E - 1) * H;
  float sum[4] = {0.f, 0.f, 0.f, 0.f};
  for (int c0 = wave * 1024 + lane * 4; c0 < H; c0 += 4096) {
    float4 a[4], b[4][4];
    float keep[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int c = c0 + 256 * i;
      keep[i] = c < H ? 1.f : 0.f;
      const int cc = c < H ? c : 0;
      a[i] = *reinterpret_cast<const float4*>(xr + cc);
#pragma unroll
      for (int u = 0; u < 4; ++u) b[u][i] = *reinterpret_cast<const float4*>(wr[u] + cc);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int u = 0; u < 4; ++u)
        sum[u] += keep[i] * (a[i].x * b[u][i].x + a[i].y * b[u][i].y + a[i].z * b[u][i].z + a[i].w * b[u][i].w);
  }
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    float v = sum[u];
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
    if (lane == 0) part[wave][u] = v;
  }
  __syncthreads();
  if (threadIdx.x < 4 && e0 + threadIdx.x < E) {
    const int u = threadIdx.x;
    float v = ((part[0][u] + part[1][u]) + part[2][u]) + part[3][u];
    if (bias) v += bias[e0 + u];
    logits[(size_t)t * E + e0 + u] = v;
  }
}

// Decode-sized batches: top-k and the whole stable grouping in ONE workgroup of 16 wavefronts (a
// launch costs more than this work does).  Requires T*k <= 1024 and E <= 128.
constexpr int kFusedMaxAssign = 1024;
constexpr int kFusedMaxE = 128;
__global__ __launch_bounds__(1024) void route_fused_kernel(const float* logits_in, int T, int E, int k, int S,
                                                           float* logits_out,
                                                           int32_t* __restrict__ ids, float* __restrict__ w,
                                                           int32_t* __restrict__ offsets, int32_t* __restrict__ perm,
                                                           int32_t* __restrict__ inv_perm,
                                                           int32_t* __restrict__ src_token, int ids_given) {
  __shared__ uint32_t s_key[16][64];
  __shared__ int s_id[16][64];
  __shared__ float s_val[16][64];
  __shared__ float s_sorted[16][64];
  __shared__ int s_ids[kFusedMaxAssign];
  __shared__ int s_chunk[16][kFusedMaxE];
  __shared__ int s_off[kFusedMaxE + 1];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int nslot = (E + 63) / 64;
  // ids_given: the experts were selected already (ids and w hold them): only the grouping is left
  if (ids_given)
    for (int a = tid; a < T * k; a += 1024) s_ids[a] = ids[a];
  // at most 64 experts: every wavefront takes its tokens through the register top-k on its own, no barriers
  if (!ids_given && nslot == 1)
    for (int t = wave; t < T; t += 16) {
      const float v = lane < E ? logits_in[(size_t)t * E + lane] : 0.f;
      if (logits_out && logits_out != logits_in && lane < E) logits_out[(size_t)t * E + lane] = v;
      wave_topk_regs(v, E, k, lane, ids + (size_t)t * k, w + (size_t)t * k, s_ids + t * k);
    }
  for (int t0 = 0; t0 < (ids_given || nslot == 1 ? 0 : T); t0 += 16) {
    const int t = t0 + wave;
    const bool active = t < T;
    float val[2] = {0.f, 0.f};
    if (active) {
#pragma unroll
      for (int s = 0; s < 2; ++s)
        if (s < nslot && s * 64 + lane < E) val[s] = logits_in[(size_t)t * E + s * 64 + lane];
      if (logits_out && logits_out != logits_in) {
#pragma unroll
        for (int s = 0; s < 2; ++s)
          if (s < nslot && s * 64 + lane < E) logits_out[(size_t)t * E + s * 64 + lane] = val[s];
      }
    }
    const size_t o = active ? (size_t)t * k : 0;
    wave_topk<2>(val, nslot, E, k, active, lane, s_key[wave], s_id[wave], s_val[wave], s_sorted[wave], ids + o, w + o,
                 active ? s_ids + o : nullptr);
  }
  // ---- stable grouping by expert: wavefront c ranks assignments 64c .. 64c+63 ----
  const int A = T * k;
  for (int i = tid; i < 16 * kFusedMaxE; i += 1024) (&s_chunk[0][0])[i] = 0;
  __syncthreads();
  const int a = tid;
  const bool valid = a < A;
  const int id = valid ? s_ids[a] : 0;
  uint64_t mask = __ballot(valid);
  for (int bit = 0; bit < 7; ++bit) {
    const bool set = (id >> bit) & 1;
    const uint64_t bal = __ballot(valid && set);
    mask &= set ? bal : ~bal;
  }
  const int rank = __popcll(mask & lanemask_lt(lane));
  if (valid && rank == 0) s_chunk[wave][id] = __popcll(mask);
  __syncthreads();
  if (tid < E) {
    int tot = 0;
    for (int c = 0; c < 16; ++c) {  // exclusive prefix over chunks, in place
      const int v = s_chunk[c][tid];
      s_chunk[c][tid] = tot;
      tot += v;
    }
    s_off[tid + 1] = tot;
  }
  if (tid == 0) s_off[0] = 0;
  __syncthreads();
  if (tid == 0)
    for (int e = 0; e < E; ++e) s_off[e + 1] += s_off[e];
  __syncthreads();
  if (tid <= E) offsets[tid] = s_off[tid];
  for (int s = tid; s < S; s += 1024) offsets[E + s + 1] = A + (s + 1) * T;
  if (valid) {
    const int pos = s_off[id] + s_chunk[wave][id] + rank;
    perm[pos] = a;
    inv_perm[a] = pos;
    if (src_token) src_token[pos] = a / k;
  }
  if (src_token)
    for (int i = tid; i < S * T; i += 1024) src_token[A + i] = i % T;
}

// pass 1: per-block histogram of expert ids
__global__ __launch_bounds__(64) void perm_hist_kernel(const int32_t* __restrict__ ids, int n_assign, int E,
                                                       int32_t* __restrict__ blockhist) {
  __shared__ int hist[1024];
  const int lane = threadIdx.x, b = blockIdx.x;
  for (int e = lane; e < E; e += 64) hist[e] = 0;
  __syncthreads();
  for (int it = 0; it < kPermBlock / 64; ++it) {
    const int a = b * kPermBlock + it * 64 + lane;
    if (a < n_assign) atomicAdd(&hist[ids[a]], 1);
  }
  __syncthreads();
  for (int e = lane; e < E; e += 64) blockhist[(size_t)b * E + e] = hist[e];
}

// pass 2 (one workgroup): exclusive prefix over blocks per expert, exclusive prefix over experts,
// offsets of the always-on groups, and the source tokens of their rows.
__global__ __launch_bounds__(1024) void perm_scan_kernel(int32_t* __restrict__ blockhist, int nb, int E, int T,
                                                         int top_k, int n_shared, int32_t* __restrict__ offsets,
                                                         int32_t* __restrict__ src_token) {
  __shared__ int tot[1024];
  const int tid = threadIdx.x;
  int total = 0;
  if (tid < E) {
    for (int b = 0; b < nb; ++b) {
      const int c = blockhist[(size_t)b * E + tid];
      blockhist[(size_t)b * E + tid] = total;
      total += c;
    }
  }
  tot[tid] = tid < E ? total : 0;
  __syncthreads();
  for (int off = 1; off < 1024; off <<= 1) {  // inclusive scan, then shift
    const int v = tid >= off ? tot[tid - off] : 0;
    __syncthreads();
    tot[tid] += v;
    __syncthreads();
  }
  if (tid < E) offsets[tid + 1] = tot[tid];
  if (tid == 0) offsets[0] = 0;
  const int n_assign = T * top_k;
  for (int s = tid; s < n_shared; s += 1024) offsets[E + s + 1] = n_assign + (s + 1) * T;
  if (src_token)
    for (int i = tid; i < n_shared * T; i += 1024) src_token[n_assign + i] = i % T;
}

// pass 3: scatter with stable in-block ranks
__global__ __launch_bounds__(64) void perm_scatter_kernel(const int32_t* __restrict__ ids, int n_assign, int E,
                                                          int idbits, int top_k,
                                                          const int32_t* __restrict__ blockprefix,
                                                          const int32_t* __restrict__ offsets,
                                                          int32_t* __restrict__ perm, int32_t* __restrict__ inv_perm,
                                                          int32_t* __restrict__ src_token) {
  __shared__ int cnt[1024];
  const int lane = threadIdx.x, b = blockIdx.x;
  const uint64_t lt = lanemask_lt(lane);
  for (int e = lane; e < E; e += 64) cnt[e] = 0;
  __syncthreads();
  for (int it = 0; it < kPermBlock / 64; ++it) {
    const int a = b * kPermBlock + it * 64 + lane;
    const bool valid = a < n_assign;
    const int id = valid ? ids[a] : 0;
    uint64_t mask = __ballot(valid);
    for (int bit = 0; bit < idbits; ++bit) {
      const bool set = (id >> bit) & 1;
      const uint64_t bal = __ballot(valid && set);
      mask &= set ? bal : ~bal;
    }
    const int rank = __popcll(mask & lt);
    const int before = valid ? cnt[id] : 0;
    __syncthreads();
    if (valid && rank == 0) cnt[id] = before + __popcll(mask);
    __syncthreads();
    if (valid) {
      const int pos = offsets[id] + blockprefix[(size_t)b * E + id] + before + rank;
      perm[pos] = a;
      inv_perm[a] = pos;
      if (src_token) src_token[pos] = a / top_k;
    }
  }
}

}  // namespace

cq_status cq_topk_launch(const float* logit_partials, int ksplit, const float* bias, int T, int E, int top_k,
                         float* logits_out, int32_t* topk_ids, float* topk_w, hipStream_t s) {
  hipLaunchKernelGGL(topk_kernel, dim3((T + 3) / 4), dim3(256), 0, s, logit_partials, ksplit, bias, T, E, top_k,
                     logits_out, topk_ids, topk_w);
  return cq_check_launch();
}

size_t cq_permute_workspace_bytes(int T, int E, int top_k) {
  const size_t nb = ((size_t)T * top_k + kPermBlock - 1) / kPermBlock;
  return cq_align_up(nb * E * sizeof(int32_t), 256);
}

cq_status cq_permute_launch(const int32_t* topk_ids, int T, int E, int top_k, int n_shared, int32_t* expert_offsets,
                            int32_t* perm, int32_t* inv_perm, int32_t* src_token, void* workspace, hipStream_t s) {
  const int n_assign = T * top_k;
  const int nb = (n_assign + kPermBlock - 1) / kPermBlock;
  int idbits = 0;
  while ((1 << idbits) < E) ++idbits;
  int32_t* blockhist = (int32_t*)workspace;
  hipLaunchKernelGGL(perm_hist_kernel, dim3(nb), dim3(64), 0, s, topk_ids, n_assign, E, blockhist);
  hipLaunchKernelGGL(perm_scan_kernel, dim3(1), dim3(1024), 0, s, blockhist, nb, E, T, top_k, n_shared,
                     expert_offsets, src_token);
  hipLaunchKernelGGL(perm_scatter_kernel, dim3(nb), dim3(64), 0, s, topk_ids, n_assign, E, idbits, top_k,
                     (const int32_t*)blockhist, (const int32_t*)expert_offsets, perm, inv_perm, src_token);
  return cq_check_launch();
}

extern "C" size_t cq_route_permute_workspace_bytes(int T, int H, int E, int top_k) {
  if (T <= 0 || H <= 0 || E <= 0 || top_k <= 0) return 0;
  const cq_gemm_f32_plan p = cq_gemm_f32_make_plan(T, E, H);
  return cq_align_up((size_t)p.ksplit * T * E * sizeof(float), 256) + cq_permute_workspace_bytes(T, E, top_k);
}

extern "C" cq_status cq_route_permute(const float* XR, const float* Wr, const float* bias, const float* logits_in,
                                      int T, int H, int E, int top_k, int n_shared, float* logits_out,
                                      int32_t* topk_ids, float* topk_w, int32_t* expert_offsets, int32_t* perm,
                                      int32_t* inv_perm, int32_t* src_token, void* workspace,
                                      size_t workspace_bytes, cq_stream stream) {
  if (!topk_ids || !topk_w || !expert_offsets || !perm || !inv_perm) return CQ_ERR_NULL;
  if (!XR && !logits_in) return CQ_ERR_NULL;
  if (XR && !Wr) return CQ_ERR_NULL;
  if (T <= 0 || H <= 0 || E <= 0 || top_k <= 0 || n_shared < 0) return CQ_ERR_SHAPE;
  if (top_k > E || top_k > 64 || E > 1024 || H % 64 != 0) return CQ_ERR_SHAPE;
  if ((long)T * (top_k + n_shared) > 0x7fffffffL) return CQ_ERR_SHAPE;
  const size_t need = cq_route_permute_workspace_bytes(T, H, E, top_k);
  if (!workspace || workspace_bytes < need) return CQ_ERR_WORKSPACE;
  hipStream_t s = (hipStream_t)stream;
  const cq_gemm_f32_plan p = cq_gemm_f32_make_plan(T, E, H);
  const size_t part_bytes = cq_align_up((size_t)p.ksplit * T * E * sizeof(float), 256);
  cq_status st;
  // decode-sized problems: a small logits kernel, then top-k + grouping fused in one workgroup
  if ((long)T * top_k <= kFusedMaxAssign && E <= kFusedMaxE && (!XR || (long)T * E * H <= (1L << 22))) {
    const float* lg = logits_in;
    if (XR) {
      float* dst = logits_out ? logits_out : (float*)workspace;
      hipLaunchKernelGGL(logits_small_kernel, dim3((E + 3) / 4, T), dim3(256), 0, s, XR, Wr, bias, H, E, dst);
      lg = dst;
    }
    hipLaunchKernelGGL(route_fused_kernel, dim3(1), dim3(1024), 0, s, lg, T, E, top_k, n_shared,
                       XR ? (float*)nullptr : logits_out, topk_ids, topk_w, expert_offsets, perm, inv_perm,
                       src_token, 0);
    return cq_check_launch();
  }
  if (XR) {
    st = cq_gemm_f32_launch(XR, Wr, 1, T, E, H, p, (float*)workspace, nullptr, 0, s);
    if (st != CQ_OK) return st;
    st = cq_topk_launch((const float*)workspace, p.ksplit, bias, T, E, top_k, logits_out, topk_ids, topk_w, s);
  } else {
    st = cq_topk_launch(logits_in, 1, nullptr, T, E, top_k, logits_out, topk_ids, topk_w, s);
  }
  if (st != CQ_OK) return st;
  // (up to 1024 assignments: one workgroup groups them in one launch instead of the three counting-sort passes)
  if ((long)T * top_k <= kFusedMaxAssign && E <= kFusedMaxE) {
    hipLaunchKernelGGL(route_fused_kernel, dim3(1), dim3(1024), 0, s, (const float*)nullptr, T, E, top_k, n_shared,
                       (float*)nullptr, topk_ids, topk_w, expert_offsets, perm, inv_perm, src_token, 1);
    return cq_check_launch();
  }
  return cq_permute_launch(topk_ids, T, E, top_k, n_shared, expert_offsets, perm, inv_perm, src_token,
                           (char*)workspace + part_bytes, s);
}

// a5 alone for decode-sized batches whose experts were selected by the front launch: the one-workgroup kernel
// without its top-k loop.  Requires T * top_k <= 1024 and E <= 128 (cq_group_small_supported).
bool cq_group_small_supported(int T, int E, int top_k) {
  return (long)T * top_k <= kFusedMaxAssign && E <= kFusedMaxE;
}
cq_status cq_group_small_launch(int32_t* topk_ids, float* topk_w, int T, int E, int top_k, int n_shared,
                                int32_t* expert_offsets, int32_t* perm, int32_t* inv_perm, int32_t* src_token,
                                hipStream_t s) {
  hipLaunchKernelGGL(route_fused_kernel, dim3(1), dim3(1024), 0, s, (const float*)nullptr, T, E, top_k, n_shared,
                     (float*)nullptr, topk_ids, topk_w, expert_offsets, perm, inv_perm, src_token, 1);
  return cq_check_launch();
}
