// a2 + a3 for decode-sized batches in one launch: the K-split partial sums of the rotation are added up,
// the row is quantized, and the router logits are formed from the row while it is still in registers.
//
// One workgroup of 1024 threads per token; a thread owns up to NC groups of four neighbouring columns.
// Every sum has a fixed order (partials in ascending split; logits: four columns, xor-shuffle tree over
// the wavefront, wavefronts in ascending order), so the result does not depend on scheduling.  All loads
// (up to 16 partial sums and the router rows of up to 8 experts) are issued before the first use: the
// kernel costs about one memory latency.
//
// A token's top-k (a4) needs nothing but the token's own logits, so the same workgroup can select the
// experts and form their weights (topk_ids given); the grouping by expert (a5), which needs every token's
// choice, is then left to the launch that follows.
//
// (Letting the workgroup that finishes last also do the grouping, behind a device-scope fence and a ticket
// counter, was measured and is slower than a second launch: the fence writes back the L2, which still
// holds the rotation's partial sums.)
#include "cq_internal.h"
#include "cq_route.h"

namespace {

constexpr int kFrontMaxE = 16;    // experts whose logits a token's workgroup forms
constexpr int kFrontThreads = 1024;
constexpr int kBatch = 15;        // partial sums 1..15 are requested together with sum 0
constexpr int kEarlyE = 8;        // experts whose router rows are requested up front

template <int NC>
__global__ __launch_bounds__(kFrontThreads) void front_small_kernel(
    const float* part, int ksplit, int in_place, int T, int H, float qmax, const float* __restrict__ Wr,
    const float* __restrict__ bias, int E, float* XR, int8_t* __restrict__ Q, uint16_t* __restrict__ Q16,
    float* __restrict__ scale, float* __restrict__ logits, int top_k, int32_t* __restrict__ topk_ids,
    float* __restrict__ topk_w) {
  __shared__ float red[16];
  __shared__ float lred[16][kFrontMaxE];
  const int t = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

  float4 v[NC];
  float lsum[kFrontMaxE];
#pragma unroll
  for (int e = 0; e < kFrontMaxE; ++e) lsum[e] = 0.f;
  float amax = 0.f;
#pragma unroll
  for (int i = 0; i < NC; ++i) {
    const int c = (i * kFrontThreads + tid) * 4;
    v[i] = make_float4(0.f, 0.f, 0.f, 0.f);
    if (c < H) {
      // ---- rotated row: partial sums in ascending split order ----
      float4 acc = *reinterpret_cast<const float4*>(part + (size_t)t * H + c);
      float4 p[kBatch];
#pragma unroll
      for (int u = 0; u < kBatch; ++u)  // clamped: a split past the end is loaded (again) but not added
        p[u] = *reinterpret_cast<const float4*>(part + ((size_t)min(1 + u, ksplit - 1) * T + t) * H + c);
      float4 b[kEarlyE];
#pragma unroll
      for (int e = 0; e < kEarlyE; ++e) b[e] = *reinterpret_cast<const float4*>(Wr + (size_t)min(e, E - 1) * H + c);
#pragma unroll
      for (int u = 0; u < kBatch; ++u)
        if (1 + u < ksplit) { acc.x += p[u].x; acc.y += p[u].y; acc.z += p[u].z; acc.w += p[u].w; }
      for (int z = 1 + kBatch; z < ksplit; ++z) {
        const float4 q = *reinterpret_cast<const float4*>(part + ((size_t)z * T + t) * H + c);
        acc.x += q.x; acc.y += q.y; acc.z += q.z; acc.w += q.w;
      }
      if (!in_place) *reinterpret_cast<float4*>(XR + (size_t)t * H + c) = acc;
      v[i] = acc;
      amax = fmaxf(amax, fmaxf(fmaxf(fabsf(acc.x), fabsf(acc.y)), fmaxf(fabsf(acc.z), fabsf(acc.w))));
      // ---- this thread's share of the router logits ----
#pragma unroll
      for (int e = 0; e < kEarlyE; ++e) lsum[e] += acc.x * b[e].x + acc.y * b[e].y + acc.z * b[e].z + acc.w * b[e].w;
#pragma unroll
      for (int e = kEarlyE; e < kFrontMaxE; ++e)
        if (e < E) {
          const float4 w = *reinterpret_cast<const float4*>(Wr + (size_t)e * H + c);
          lsum[e] += acc.x * w.x + acc.y * w.y + acc.z * w.z + acc.w * w.w;
        }
    }
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) amax = fmaxf(amax, __shfl_xor(amax, off));
#pragma unroll
  for (int e = 0; e < kFrontMaxE; ++e)
    if (e < E) {
      float x = lsum[e];
#pragma unroll
      for (int off = 32; off > 0; off >>= 1) x += __shfl_xor(x, off);
      if (lane == 0) lred[wave][e] = x;
    }
  if (lane == 0) red[wave] = amax;
  __syncthreads();
  amax = red[0];
#pragma unroll
  for (int i = 1; i < 16; ++i) amax = fmaxf(amax, red[i]);
  const float s = amax == 0.f ? 1.f : amax / qmax;
  if (tid == 0) scale[t] = s;
  {
    float x = 0.f;
    if (tid < E) {
      x = lred[0][tid];
#pragma unroll
      for (int i = 1; i < 16; ++i) x += lred[i][tid];
      if (bias) x += bias[tid];
      logits[(size_t)t * E + tid] = x;
    }
    // a4 for this token: the logits are in the lanes of wavefront 0, which selects on its own (no LDS, no
    // barrier) while the other wavefronts go on to the codes
    if (topk_ids && wave == 0)   // (uniform per wavefront)
      cq_route::wave_topk_regs(x, E, top_k, lane, topk_ids + (size_t)t * top_k, topk_w + (size_t)t * top_k);
  }

  // ---- integer codes: round to nearest, ties to even (v_rndne_f32) ----
#pragma unroll
  for (int i = 0; i < NC; ++i) {
    const int c = (i * kFrontThreads + tid) * 4;
    if (c < H) {
      const float r0 = fminf(fmaxf(rintf(v[i].x / s), -qmax), qmax);
      const float r1 = fminf(fmaxf(rintf(v[i].y / s), -qmax), qmax);
      const float r2 = fminf(fmaxf(rintf(v[i].z / s), -qmax), qmax);
      const float r3 = fminf(fmaxf(rintf(v[i].w / s), -qmax), qmax);
      const uint32_t packed = ((uint32_t)(int)r0 & 0xffu) | (((uint32_t)(int)r1 & 0xffu) << 8) |
                              (((uint32_t)(int)r2 & 0xffu) << 16) | (((uint32_t)(int)r3 & 0xffu) << 24);
      *reinterpret_cast<uint32_t*>(Q + (size_t)t * H + c) = packed;
      if (Q16)  // the same codes as bf16 bit patterns (exact: small integers)
        *reinterpret_cast<uint2*>(Q16 + (size_t)t * H + c) =
            make_uint2((__float_as_uint(r0) >> 16) | (__float_as_uint(r1) & 0xffff0000u),
                       (__float_as_uint(r2) >> 16) | (__float_as_uint(r3) & 0xffff0000u));
    }
  }
}

}  // namespace

bool cq_front_small_supported(int T, int H, int E, int top_k) {
  // the limits of the one-workgroup routing kernel that follows, and of this kernel's registers
  return (long)T * top_k <= 1024 && E <= kFrontMaxE && H <= 2 * 4 * kFrontThreads && H % 4 == 0 &&
         (long)T * E * H <= (1L << 23);
}

cq_status cq_front_small_launch(const float* partials, int ksplit, int T, int H, int act_bits, const float* Wr,
                                const float* bias, int E, float* XR, int8_t* Q, uint16_t* Q16, float* scale,
                                float* logits, int top_k, int32_t* topk_ids, float* topk_w, hipStream_t s) {
  const float qmax = (float)((1 << (act_bits - 1)) - 1);
  const int in_place = (partials == XR && ksplit == 1) ? 1 : 0;
  if (H <= 4 * kFrontThreads)
    hipLaunchKernelGGL(front_small_kernel<1>, dim3(T), dim3(kFrontThreads), 0, s, partials, ksplit, in_place, T, H, qmax,
                       Wr, bias, E, XR, Q, Q16, scale, logits, top_k, topk_ids, topk_w);
  else
    hipLaunchKernelGGL(front_small_kernel<2>, dim3(T), dim3(kFrontThreads), 0, s, partials, ksplit, in_place, T, H, qmax,
                       Wr, bias, E, XR, Q, Q16, scale, logits, top_k, topk_ids, topk_w);
  return cq_check_launch();
}
