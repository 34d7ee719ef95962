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

namespace {

constexpr int kMaxSlots = 16;       // experts per lane: E <= 1024
constexpr int kPermBlock = 256;     // assignments per counting-sort block (one wavefront, 4 rounds)

__device__ __forceinline__ uint32_t order_key(float x) {
  const uint32_t u = __float_as_uint(x);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__device__ __forceinline__ uint64_t lanemask_lt(int lane) { return (1ull << lane) - 1ull; }

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
  const uint64_t lt = lanemask_lt(lane);

  float val[kMaxSlots];
  uint32_t key[kMaxSlots];
#pragma unroll
  for (int s = 0; s < kMaxSlots; ++s) {
    const int e = s * 64 + lane;
    val[s] = 0.f;
    key[s] = 0u;
    if (s < nslot && e < E && active) {
      float x = part[(size_t)t * E + e];
      for (int z = 1; z < ksplit; ++z) x += part[((size_t)z * T + t) * E + e];
      if (bias) x += bias[e];
      if (logits_out) logits_out[(size_t)t * E + e] = x;
      val[s] = x;
      key[s] = order_key(x);
    }
  }
  // k-th largest key: keep the largest prefix such that at least k keys are >= it.
  uint32_t kth = 0u;
  for (int bit = 31; bit >= 0; --bit) {
    const uint32_t cand = kth | (1u << bit);
    int cnt = 0;
#pragma unroll
    for (int s = 0; s < kMaxSlots; ++s)
      if (s < nslot) cnt += __popcll(__ballot((s * 64 + lane) < E && key[s] >= cand));
    if (cnt >= k) kth = cand;
  }
  int n_gt = 0;
#pragma unroll
  for (int s = 0; s < kMaxSlots; ++s)
    if (s < nslot) n_gt += __popcll(__ballot((s * 64 + lane) < E && key[s] > kth));
  const int need = k - n_gt;  // how many of the keys equal to kth are admitted (lowest ids first)
  int base = 0, ties_seen = 0;
#pragma unroll
  for (int s = 0; s < kMaxSlots; ++s) {
    if (s < nslot) {
      const bool valid = (s * 64 + lane) < E;
      const bool eq = valid && key[s] == kth;
      const uint64_t m_eq = __ballot(eq);
      const int tie_rank = ties_seen + __popcll(m_eq & lt);
      const bool sel = valid && (key[s] > kth || (eq && tie_rank < need));
      const uint64_t m_sel = __ballot(sel);
      const int pos = base + __popcll(m_sel & lt);
      if (sel && active) {
        s_key[wave][pos] = key[s];
        s_id[wave][pos] = s * 64 + lane;
        s_val[wave][pos] = val[s];
      }
      base += __popcll(m_sel);
      ties_seen += __popcll(m_eq);
    }
  }
  __syncthreads();
  if (active && lane < k) {
    const uint32_t mk = s_key[wave][lane];
    const int mi = s_id[wave][lane];
    int rank = 0;
    for (int p = 0; p < k; ++p) {
      const uint32_t ok = s_key[wave][p];
      const int oi = s_id[wave][p];
      rank += (ok > mk || (ok == mk && oi < mi)) ? 1 : 0;
    }
    ids[(size_t)t * k + rank] = mi;
    s_sorted[wave][rank] = s_val[wave][lane];
  }
  __syncthreads();
  float ex = 0.f;
  if (active && lane < k) ex = expf(s_sorted[wave][lane] - s_sorted[wave][0]);
  float sum = ex;
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) sum += __shfl_xor(sum, off);
  if (active && lane < k) w[(size_t)t * k + lane] = ex / sum;
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
  if (XR) {
    st = cq_gemm_f32_launch(XR, Wr, 1, T, E, H, p, (float*)workspace, s);
    if (st != CQ_OK) return st;
    st = cq_topk_launch((const float*)workspace, p.ksplit, bias, T, E, top_k, logits_out, topk_ids, topk_w, s);
  } else {
    st = cq_topk_launch(logits_in, 1, nullptr, T, E, top_k, logits_out, topk_ids, topk_w, s);
  }
  if (st != CQ_OK) return st;
  return cq_permute_launch(topk_ids, T, E, top_k, n_shared, expert_offsets, perm, inv_perm, src_token,
                           (char*)workspace + part_bytes, s);
}
