// a1 + a2: X_R = X R on fp32 matrix cores, then per-token symmetric integer quantization.
//
// The rotation must be accurate to about fp32 so that the integer codes agree with an exact
// evaluation everywhere except at rounding ties, so it runs on v_mfma_f32_16x16x4_f32 (fp32 in,
// fp32 accumulate) rather than on bf16 MFMA.  The same kernel, with B given transposed, computes
// the router logits X_R Wr^T.
//
// Wave tile: (16*MB tokens) x 64 columns.  A lane with (j = lane%16, g = lane/16) loads four
// consecutive K values per operand (16-byte loads) and feeds element m of them to the m-th of
// four MFMAs; both operands use the same K numbering, so the sum over K is unchanged.  For the
// row-major B the four elements of a 16-byte load are four neighbouring columns, which become
// four column sets {c0 + 4j + n}; for the transposed B they are four K values of column
// c0 + 16n + j.  No LDS: operands are small enough to be served by L1/L2.
#include "cq_internal.h"

namespace {

template <int MB, int WM, bool BT, int D>
__global__ __launch_bounds__(256) void gemm_f32_kernel(const float* __restrict__ A, const float* __restrict__ B,
                                                       float* __restrict__ C, int T, int N, int K, int kchunk,
                                                       uint32_t* __restrict__ zero_me, int zero_n) {
  constexpr int WN = 4 / WM;
  // side job of the first workgroup: clear a small buffer the next kernel accumulates into
  if (zero_me && blockIdx.x == 0 && blockIdx.y == 0 && blockIdx.z == 0)
    for (int i = threadIdx.x; i < zero_n; i += 256) zero_me[i] = 0u;
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int wm = wave % WM, wn = wave / WM;
  const int t0 = (blockIdx.y * WM + wm) * 16 * MB;
  const int c0 = (blockIdx.x * WN + wn) * 64;
  if (t0 >= T || c0 >= N) return;
  const int j = lane & 15, g = lane >> 4;
  const int kbeg = blockIdx.z * kchunk;
  const int kend = min(K, kbeg + kchunk);
  const int steps = (kend - kbeg) >> 4;

  const float* pa[MB];
#pragma unroll
  for (int mb = 0; mb < MB; ++mb) {
    const int row = min(t0 + 16 * mb + j, T - 1);  // rows past T only feed outputs that are never stored
    pa[mb] = A + (size_t)row * K + 4 * g;
  }
  const float* pb[4];
#pragma unroll
  for (int x = 0; x < 4; ++x) {
    if (BT) {
      const int col = min(c0 + 16 * x + j, N - 1);
      pb[x] = B + (size_t)col * K + 4 * g;
    } else {
      pb[x] = B + (size_t)(4 * g + x) * N + c0 + 4 * j;
    }
  }

  cq_v4f acc[MB][4];
#pragma unroll
  for (int mb = 0; mb < MB; ++mb)
#pragma unroll
    for (int n = 0; n < 4; ++n) acc[mb][n] = cq_v4f{0.f, 0.f, 0.f, 0.f};

  // register ring of D K-steps; loads are unconditional (step index clamped) so that every wait
  // covers exactly one slot
  float4 ra[D][MB], rb[D][4];
  auto load = [&](float4* a, float4* b, int step) {
    const int ks = kbeg + 16 * min(step, steps - 1);
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) a[mb] = *reinterpret_cast<const float4*>(pa[mb] + ks);
#pragma unroll
    for (int x = 0; x < 4; ++x)
      b[x] = BT ? *reinterpret_cast<const float4*>(pb[x] + ks)
                : *reinterpret_cast<const float4*>(pb[x] + (size_t)ks * N);
  };
#pragma unroll
  for (int d = 0; d < D; ++d) load(ra[d], rb[d], d);
  for (int s0 = 0; s0 < steps; s0 += D) {
#pragma unroll
    for (int d = 0; d < D; ++d) {
      const int st = s0 + d;
      float4 a_cur[MB], b_cur[4];
#pragma unroll
      for (int mb = 0; mb < MB; ++mb) a_cur[mb] = ra[d][mb];
#pragma unroll
      for (int x = 0; x < 4; ++x) b_cur[x] = rb[d][x];
      load(ra[d], rb[d], st + D);
      if (st < steps) {
#pragma unroll
        for (int m = 0; m < 4; ++m) {
#pragma unroll
          for (int n = 0; n < 4; ++n) {
            const float4 bq = BT ? b_cur[n] : b_cur[m];
            const int be = BT ? m : n;
            const float bval = be == 0 ? bq.x : be == 1 ? bq.y : be == 2 ? bq.z : bq.w;
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) {
              const float4 aq = a_cur[mb];
              const float aval = m == 0 ? aq.x : m == 1 ? aq.y : m == 2 ? aq.z : aq.w;
              acc[mb][n] = __builtin_amdgcn_mfma_f32_16x16x4f32(aval, bval, acc[mb][n], 0, 0, 0);
            }
          }
        }
      }
    }
  }

  // D of the 16x16 MFMA: lane holds column j and rows 4*g + v, v = 0..3.
  float* Cz = C + (size_t)blockIdx.z * T * N;
#pragma unroll
  for (int mb = 0; mb < MB; ++mb) {
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const int tok = t0 + 16 * mb + 4 * g + v;
      if (tok >= T) continue;
      if (BT) {
#pragma unroll
        for (int n = 0; n < 4; ++n) {
          const int col = c0 + 16 * n + j;
          if (col < N) Cz[(size_t)tok * N + col] = acc[mb][n][v];
        }
      } else {
        float4 o = make_float4(acc[mb][0][v], acc[mb][1][v], acc[mb][2][v], acc[mb][3][v]);
        *reinterpret_cast<float4*>(Cz + (size_t)tok * N + c0 + 4 * j) = o;
      }
    }
  }
}

// Few tokens: a row is spread over several workgroups.  Pass 1 reduces the K-split partials in a fixed
// order, keeps X_R and folds the chunk maximum into amax_bits[t] with an integer atomic max (the bit
// pattern of a non-negative float orders like the float, and a maximum does not depend on the order of
// its operands, so the result is deterministic).  Pass 2 rounds x / s to the nearest integer.
__global__ __launch_bounds__(256) void reduce_amax_kernel(const float* part, int ksplit, int in_place, int T, int H,
                                                          float* XR, uint32_t* __restrict__ amax_bits) {
  __shared__ float red[4];
  const int t = blockIdx.y, tid = threadIdx.x;
  const int c = (blockIdx.x * 256 + tid) * 4;
  float amax = 0.f;
  if (c < H) {
    float4 v = *reinterpret_cast<const float4*>(part + (size_t)t * H + c);
    for (int z = 1; z < ksplit; ++z) {
      const float4 p = *reinterpret_cast<const float4*>(part + ((size_t)z * T + t) * H + c);
      v.x += p.x; v.y += p.y; v.z += p.z; v.w += p.w;
    }
    if (!in_place) *reinterpret_cast<float4*>(XR + (size_t)t * H + c) = v;
    amax = fmaxf(fmaxf(fabsf(v.x), fabsf(v.y)), fmaxf(fabsf(v.z), fabsf(v.w)));
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) amax = fmaxf(amax, __shfl_xor(amax, off));
  if ((tid & 63) == 0) red[tid >> 6] = amax;
  __syncthreads();
  if (tid == 0) {
    amax = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    atomicMax(amax_bits + t, __float_as_uint(amax));
  }
}

__global__ __launch_bounds__(256) void codes_kernel(const float* __restrict__ XR, const uint32_t* __restrict__ amax_bits,
                                                    int H, float qmax, int8_t* __restrict__ Q,
                                                    uint16_t* __restrict__ Q16, float* __restrict__ scale) {
  const int t = blockIdx.y, tid = threadIdx.x;
  const int c = (blockIdx.x * 256 + tid) * 4;
  const float amax = __uint_as_float(amax_bits[t]);
  const float s = amax == 0.f ? 1.f : amax / qmax;
  if (blockIdx.x == 0 && tid == 0) scale[t] = s;
  if (c < H) {
    const float4 v = *reinterpret_cast<const float4*>(XR + (size_t)t * H + c);
    const float r0 = fminf(fmaxf(rintf(v.x / s), -qmax), qmax);
    const float r1 = fminf(fmaxf(rintf(v.y / s), -qmax), qmax);
    const float r2 = fminf(fmaxf(rintf(v.z / s), -qmax), qmax);
    const float r3 = fminf(fmaxf(rintf(v.w / s), -qmax), qmax);
    const uint32_t packed = ((uint32_t)(int)r0 & 0xffu) | (((uint32_t)(int)r1 & 0xffu) << 8) |
                            (((uint32_t)(int)r2 & 0xffu) << 16) | (((uint32_t)(int)r3 & 0xffu) << 24);
    *reinterpret_cast<uint32_t*>(Q + (size_t)t * H + c) = packed;
    if (Q16)  // the same codes as bf16 bit patterns (exact: small integers), ready to be an MFMA operand
      *reinterpret_cast<uint2*>(Q16 + (size_t)t * H + c) =
          make_uint2((__float_as_uint(r0) >> 16) | (__float_as_uint(r1) & 0xffff0000u),
                     (__float_as_uint(r2) >> 16) | (__float_as_uint(r3) & 0xffff0000u));
  }
}

// One workgroup per token: reduce the K-split partials in a fixed order, keep X_R, find the row
// maximum, then round x / s to the nearest integer (ties to even, v_rndne_f32).
__global__ __launch_bounds__(256) void quantize_kernel(const float* part, int ksplit, int in_place, int T, int H,
                                                       float qmax, float* XR, int8_t* __restrict__ Q,
                                                       uint16_t* __restrict__ Q16, float* __restrict__ scale) {
  __shared__ float red[4];
  const int t = blockIdx.x;
  const int tid = threadIdx.x;
  float amax = 0.f;
  float* xr = XR + (size_t)t * H;
  for (int c = tid * 4; c < H; c += 256 * 4) {
    float4 v = *reinterpret_cast<const float4*>(part + (size_t)t * H + c);
    for (int z = 1; z < ksplit; ++z) {
      const float4 p = *reinterpret_cast<const float4*>(part + ((size_t)z * T + t) * H + c);
      v.x += p.x; v.y += p.y; v.z += p.z; v.w += p.w;
    }
    if (!in_place) *reinterpret_cast<float4*>(xr + c) = v;
    amax = fmaxf(amax, fmaxf(fmaxf(fabsf(v.x), fabsf(v.y)), fmaxf(fabsf(v.z), fabsf(v.w))));
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) amax = fmaxf(amax, __shfl_xor(amax, off));
  if ((tid & 63) == 0) red[tid >> 6] = amax;
  __syncthreads();
  amax = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
  const float s = amax == 0.f ? 1.f : amax / qmax;
  if (tid == 0) scale[t] = s;
  int8_t* q = Q + (size_t)t * H;
  for (int c = tid * 4; c < H; c += 256 * 4) {
    const float4 v = *reinterpret_cast<const float4*>(xr + c);  // this thread's own stores above
    const float r0 = fminf(fmaxf(rintf(v.x / s), -qmax), qmax);
    float r1 = fminf(fmaxf(rintf(v.y / s), -qmax), qmax);
    float r2 = fminf(fmaxf(rintf(v.z / s), -qmax), qmax);
    float r3 = fminf(fmaxf(rintf(v.w / s), -qmax), qmax);
    const uint32_t packed = ((uint32_t)(int)r0 & 0xffu) | (((uint32_t)(int)r1 & 0xffu) << 8) |
                            (((uint32_t)(int)r2 & 0xffu) << 16) | (((uint32_t)(int)r3 & 0xffu) << 24);
    *reinterpret_cast<uint32_t*>(q + c) = packed;
    if (Q16)
      *reinterpret_cast<uint2*>(Q16 + (size_t)t * H + c) =
          make_uint2((__float_as_uint(r0) >> 16) | (__float_as_uint(r1) & 0xffff0000u),
                     (__float_as_uint(r2) >> 16) | (__float_as_uint(r3) & 0xffff0000u));
  }
}

}  // namespace

cq_gemm_f32_plan cq_gemm_f32_make_plan(int T, int N, int K) {
  cq_gemm_f32_plan p;
  p.mb = T >= 64 ? 4 : 1;
  const int tm = p.mb == 4 ? 128 : 16;
  const int tn = p.mb == 4 ? 128 : 256;
  const long wgs = (long)((N + tn - 1) / tn) * ((T + tm - 1) / tm);
  int ks = (int)(256 / wgs);   // K chunks such that one round of workgroups covers the launch (96 tiles: 2, not 3)
  if (ks > 16) ks = 16;
  if (ks > K / 64) ks = K / 64;
  if (ks < 1) ks = 1;
  int kchunk = (K + ks - 1) / ks;
  kchunk = (kchunk + 15) / 16 * 16;
  p.kchunk = kchunk;
  p.ksplit = (K + kchunk - 1) / kchunk;
  return p;
}

cq_status cq_gemm_f32_launch(const float* A, const float* B, int b_transposed, int T, int N, int K,
                             const cq_gemm_f32_plan& plan, float* C, uint32_t* zero_me, int zero_n, hipStream_t s) {
  const int kchunk = plan.kchunk;
  dim3 block(256);
  if (plan.mb == 4) {
    dim3 grid((N + 127) / 128, (T + 127) / 128, plan.ksplit);
    if (b_transposed)
      hipLaunchKernelGGL((gemm_f32_kernel<4, 2, true, 2>), grid, block, 0, s, A, B, C, T, N, K, kchunk, zero_me,
                         zero_n);
    else
      hipLaunchKernelGGL((gemm_f32_kernel<4, 2, false, 2>), grid, block, 0, s, A, B, C, T, N, K, kchunk, zero_me,
                         zero_n);
  } else {
    dim3 grid((N + 255) / 256, (T + 15) / 16, plan.ksplit);
    if (b_transposed)
      hipLaunchKernelGGL((gemm_f32_kernel<1, 1, true, 4>), grid, block, 0, s, A, B, C, T, N, K, kchunk, zero_me,
                         zero_n);
    else
      hipLaunchKernelGGL((gemm_f32_kernel<1, 1, false, 4>), grid, block, 0, s, A, B, C, T, N, K, kchunk, zero_me,
                         zero_n);
  }
  return cq_check_launch();
}

cq_status cq_quantize_launch(const float* partials, int ksplit, int T, int H, int act_bits, float* XR_out,
                             int8_t* Q_out, uint16_t* Q16_out, float* scale_out, uint32_t* amax_bits,
                             hipStream_t s) {
  const float qmax = (float)((1 << (act_bits - 1)) - 1);
  const int in_place = (partials == XR_out && ksplit == 1) ? 1 : 0;
  if (amax_bits) {  // few tokens: spread every row over several workgroups (amax_bits was zeroed upstream)
    dim3 grid((H + 1023) / 1024, T);
    hipLaunchKernelGGL(reduce_amax_kernel, grid, dim3(256), 0, s, partials, ksplit, in_place, T, H, XR_out,
                       amax_bits);
    hipLaunchKernelGGL(codes_kernel, grid, dim3(256), 0, s, (const float*)XR_out, (const uint32_t*)amax_bits, H, qmax,
                       Q_out, Q16_out, scale_out);
  } else {
    hipLaunchKernelGGL(quantize_kernel, dim3(T), dim3(256), 0, s, partials, ksplit, in_place, T, H, qmax, XR_out,
                       Q_out, Q16_out, scale_out);
  }
  return cq_check_launch();
}

namespace {
constexpr int kFewTokens = 256;  // below this a token row is quantized by several workgroups
size_t amax_bytes(int T) { return T < kFewTokens ? cq_align_up((size_t)T * sizeof(uint32_t), 256) : 0; }
}  // namespace

extern "C" size_t cq_rotate_quant_workspace_bytes(int T, int H) {
  if (T <= 0 || H <= 0) return 0;
  const cq_gemm_f32_plan p = cq_gemm_f32_make_plan(T, H, H);
  return amax_bytes(T) + (p.ksplit > 1 ? cq_align_up((size_t)p.ksplit * T * H * sizeof(float), 256) : 0);
}

cq_status cq_rotate_quant_ex(const float* X, const float* R, int T, int H, int act_bits, float* XR_out,
                             int8_t* Q_out, uint16_t* Q16_out, float* scale_out, void* workspace,
                             size_t workspace_bytes, cq_stream stream) {
  if (!X || !R || !XR_out || !Q_out || !scale_out) return CQ_ERR_NULL;
  if (T <= 0 || H <= 0 || H % 64 != 0) return CQ_ERR_SHAPE;
  if (act_bits != 4 && act_bits != 8) return CQ_ERR_UNSUPPORTED;
  const size_t need = cq_rotate_quant_workspace_bytes(T, H);
  if (need > 0 && (!workspace || workspace_bytes < need)) return CQ_ERR_WORKSPACE;
  hipStream_t s = (hipStream_t)stream;
  const cq_gemm_f32_plan p = cq_gemm_f32_make_plan(T, H, H);
  uint32_t* amax = amax_bytes(T) ? (uint32_t*)workspace : nullptr;
  float* part = (float*)((char*)workspace + amax_bytes(T));
  float* dst = p.ksplit > 1 ? part : XR_out;
  cq_status st = cq_gemm_f32_launch(X, R, 0, T, H, H, p, dst, amax, T, s);
  if (st != CQ_OK) return st;
  return cq_quantize_launch(dst, p.ksplit, T, H, act_bits, XR_out, Q_out, Q16_out, scale_out, amax, s);
}

extern "C" cq_status cq_rotate_quant(const float* X, const float* R, int T, int H, int act_bits, float* XR_out,
                                     int8_t* Q_out, float* scale_out, void* workspace, size_t workspace_bytes,
                                     cq_stream stream) {
  return cq_rotate_quant_ex(X, R, T, H, act_bits, XR_out, Q_out, nullptr, scale_out, workspace, workspace_bytes,
                            stream);
}
