// Device helpers of the routing step (a4) shared by the routing kernels and the decode front end:
// order-preserving logit keys and the wavefront top-k with softmax over the selected logits.
#pragma once
#include "cq_internal.h"

namespace cq_route {

// Order-preserving key of a logit.  -0 is folded into +0 first (they are equal logits: the lower expert id
// wins), and a NaN, whatever its sign, gets the smallest key (it is never preferred to a number).
__device__ __forceinline__ uint32_t order_key(float x) {
  if (x != x) return 0u;
  const uint32_t u = __float_as_uint(x + 0.0f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__device__ __forceinline__ uint64_t lanemask_lt(int lane) { return (1ull << lane) - 1ull; }

// Top-k of one token by one wavefront.  val[s] is the logit of expert s*64 + lane.  Called by all
// wavefronts of the workgroup together (it contains workgroup barriers); sk/si/sv/ss are this
// wavefront's 64-entry LDS scratch arrays.  Writes ids (descending logit, ties -> lower id) and the
// softmax over the selected logits; lds_ids, if given, also receives the ids.
template <int NSLOT>
__device__ __forceinline__ void wave_topk(const float (&val)[NSLOT], int nslot, int E, int k, bool active, int lane,
                                          uint32_t* sk, int* si, float* sv, float* ss, int32_t* ids_out,
                                          float* w_out, int* lds_ids) {
  const uint64_t lt = lanemask_lt(lane);
  uint32_t key[NSLOT];
#pragma unroll
  for (int s = 0; s < NSLOT; ++s) key[s] = (s < nslot && (s * 64 + lane) < E) ? order_key(val[s]) : 0u;
  // k-th largest key: keep the largest prefix such that at least k keys are >= it.
  uint32_t kth = 0u;
  for (int bit = 31; bit >= 0; --bit) {
    const uint32_t cand = kth | (1u << bit);
    int cnt = 0;
#pragma unroll
    for (int s = 0; s < NSLOT; ++s)
      if (s < nslot) cnt += __popcll(__ballot((s * 64 + lane) < E && key[s] >= cand));
    if (cnt >= k) kth = cand;
  }
  int n_gt = 0;
#pragma unroll
  for (int s = 0; s < NSLOT; ++s)
    if (s < nslot) n_gt += __popcll(__ballot((s * 64 + lane) < E && key[s] > kth));
  const int need = k - n_gt;  // how many of the keys equal to kth are admitted (lowest ids first)
  int base = 0, ties_seen = 0;
#pragma unroll
  for (int s = 0; s < NSLOT; ++s) {
    if (s < nslot) {
      const bool valid = (s * 64 + lane) < E;
      const bool eq = valid && key[s] == kth;
      const uint64_t m_eq = __ballot(eq);
      const int tie_rank = ties_seen + __popcll(m_eq & lt);
      const bool sel = valid && (key[s] > kth || (eq && tie_rank < need));
      const uint64_t m_sel = __ballot(sel);
      const int pos = base + __popcll(m_sel & lt);
      if (sel && active) {
        sk[pos] = key[s];
        si[pos] = s * 64 + lane;
        sv[pos] = val[s];
      }
      base += __popcll(m_sel);
      ties_seen += __popcll(m_eq);
    }
  }
  __syncthreads();
  if (active && lane < k) {
    const uint32_t mk = sk[lane];
    const int mi = si[lane];
    int rank = 0;
    for (int p = 0; p < k; ++p) {
      const uint32_t ok = sk[p];
      const int oi = si[p];
      rank += (ok > mk || (ok == mk && oi < mi)) ? 1 : 0;
    }
    ids_out[rank] = mi;
    if (lds_ids) lds_ids[rank] = mi;
    ss[rank] = sv[lane];
  }
  __syncthreads();
  float ex = 0.f;
  if (active && lane < k) ex = expf(ss[lane] - ss[0]);
  float sum = ex;
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) sum += __shfl_xor(sum, off);
  if (active && lane < k) w_out[lane] = ex / sum;
  __syncthreads();  // the scratch arrays may be reused by the caller's next token
}

// Top-k of one token by one wavefront on its own, for at most 64 experts: lane e holds the logit of expert e.  No
// LDS and no barrier (only this wavefront's lanes take part): the k-th largest key by the same bitwise descent,
// ties admitted in ascending expert id, the selected lanes ranked by (logit descending, id ascending) against each
// other through lane reads, and one lane permutation that brings the pair of rank r to lane r.  Results as
// wave_topk writes them: ids in rank order (also to lds_ids, if given) and the softmax over the selected logits.
// Called by all 64 lanes.
__device__ __forceinline__ void wave_topk_regs(float val, int E, int k, int lane, int32_t* ids_out, float* w_out,
                                               int* lds_ids = nullptr) {
  const uint64_t lt = lanemask_lt(lane);
  const bool valid = lane < E;
  const uint32_t key = valid ? order_key(val) : 0u;
  uint32_t kth = 0u;
  for (int bit = 31; bit >= 0; --bit) {
    const uint32_t cand = kth | (1u << bit);
    if (__popcll(__ballot(valid && key >= cand)) >= k) kth = cand;
  }
  const int need = k - __popcll(__ballot(valid && key > kth));   // how many of the keys equal to kth are admitted
  const uint64_t m_eq = __ballot(valid && key == kth);
  const bool sel = valid && (key > kth || (key == kth && __popcll(m_eq & lt) < need));
  const uint64_t m_sel = __ballot(sel);
  int rank = 0;
  for (uint64_t m = m_sel; m; m &= m - 1) {
    const int j = __ffsll((long long)m) - 1;
    const uint32_t kj = (uint32_t)__builtin_amdgcn_readlane((int)key, j);
    rank += (kj > key || (kj == key && j < lane)) ? 1 : 0;
  }
  // selected lanes go to lane `rank`, the others fill the lanes from k on in order: a permutation
  const int dest = sel ? rank : k + __popcll(~m_sel & lt);
  const int id_sorted = __builtin_amdgcn_ds_permute(dest << 2, lane);
  const float v_sorted = __int_as_float(__builtin_amdgcn_ds_permute(dest << 2, __float_as_int(val)));
  const float top = __shfl(v_sorted, 0);
  const float ex = lane < k ? expf(v_sorted - top) : 0.f;
  float sum = ex;
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) sum += __shfl_xor(sum, off);
  if (lane < k) {
    ids_out[lane] = id_sorted;
    if (lds_ids) lds_ids[lane] = id_sorted;
    w_out[lane] = ex / sum;
  }
}

// a5 folded into a product launch for decode-sized batches (cq_route_fuse): the rows of group `grp`, derived by
// one wavefront from the selected expert ids.  There are at most 64 assignments (token, choice), one per lane,
// numbered a = token * top_k + choice; the rows of expert e are the assignments that chose e, in ascending a, and
// the experts' row ranges follow each other in ascending e (the stable grouping of the routing step), so two
// ballots give the first row m0 and the row count Me, and one lane permutation hands row i's token to lane i
// (row_token).  Shared experts (grp >= E) take every token, in token order, behind the routed rows.
// writer: this wavefront also leaves offsets / perm / inv_perm / src_token behind for the launches that follow
// (exactly one wavefront of the launch must do so).  Called by all 64 lanes.
__device__ __forceinline__ void group_rows_from_ids(const cq_route_fuse& rt, int grp, int lane, bool writer, int& m0,
                                                    int& Me, int& row_token) {
  const int n_assign = rt.T * rt.top_k;
  const bool va = lane < n_assign;
  const int id = va ? rt.ids[lane] : 0x7fffffff;
  const uint64_t lt = lanemask_lt(lane);
  if (grp < rt.E) {
    const uint64_t mine = __ballot(va && id == grp);
    m0 = __popcll(__ballot(va && id < grp));
    Me = __popcll(mine);
    const int before = __popcll(mine & lt);
    // members go to lanes 0 .. Me-1 in order, the others fill the lanes behind them: a permutation
    const int dest = ((mine >> lane) & 1ull) ? before : Me + lane - before;
    row_token = __builtin_amdgcn_ds_permute(dest << 2, lane / rt.top_k);
  } else {
    m0 = n_assign + (grp - rt.E) * rt.T;
    Me = rt.T;
    row_token = lane;
  }
  if (writer) {
    int pos = 0, base = 0, my_off = 0;
    for (int e = 0; e < rt.E; ++e) {
      const uint64_t m = __ballot(va && id == e);
      if (va && id == e) pos = base + __popcll(m & lt);
      if (lane == e) my_off = base;
      base += __popcll(m);
    }
    if (lane < rt.E) rt.offsets[lane] = my_off;
    if (lane == 0) rt.offsets[rt.E] = n_assign;
    for (int sh = lane; sh < rt.S; sh += 64) rt.offsets[rt.E + sh + 1] = n_assign + (sh + 1) * rt.T;
    if (va) {
      rt.perm[pos] = lane;
      rt.inv_perm[lane] = pos;
      rt.src_token[pos] = lane / rt.top_k;
    }
    for (int i = lane; i < rt.S * rt.T; i += 64) rt.src_token[n_assign + i] = i % rt.T;
  }
}

}  // namespace cq_route
