// Online-Hadamard variant (evaluation section, the "had" setting): the intermediate of the expert FFN is
// rotated by a Hadamard matrix in front of the down projection, h' = h H_I / sqrt(I), and quantized per row
// like the layer's input.
//
// H_I = H_m (x) H_p with p = 2^k and m = 1 (I a power of two) or m = 4 * (odd part of I) in {12, 28, 44}, H_m
// from Paley's constructions (index i = a*p + b).  One workgroup per row keeps the row in LDS: k butterfly
// stages over the blocks of p (a fast Walsh-Hadamard transform, two stages per barrier), then every thread
// combines the m values at its positions b with the signs of H_m (a compile-time table), scales, and the row
// maximum gives the integer codes.  Cost O(I (log p + m)) per row instead of O(I^2).
#include "cq_internal.h"

namespace {

constexpr int kHadThreads = 512;
constexpr int kHadMaxI = 16384;   // the row as fp32 in 64 KiB of LDS

// Legendre symbol of x modulo the odd prime q
constexpr int legendre(int x, int q) {
  x = ((x % q) + q) % q;
  if (x == 0) return 0;
  for (int y = 1; y < q; ++y)
    if ((y * y) % q == x) return 1;
  return -1;
}

// H_m[a][a2], m in {12, 44}: I + S, S = [[0, 1^T], [-1, Q]], Q[i][j] = chi(j - i) (Paley, q = m - 1 = 3 mod 4);
// m = 28: S (x) [[1,1],[1,-1]] + I (x) [[1,-1],[-1,-1]], S = [[0, 1^T], [1, Q]], Q[i][j] = chi(i - j) (q = 13)
constexpr int paley_entry(int m, int a, int a2) {
  if (m == 12 || m == 44) {
    const int q = m - 1;
    if (a == a2) return 1;
    if (a == 0) return 1;
    if (a2 == 0) return -1;
    return legendre((a2 - 1) - (a - 1), q);
  }
  const int q = 13;
  const int i = a >> 1, u = a & 1, j = a2 >> 1, v = a2 & 1;
  int s = 0;
  if (i == 0 && j == 0) s = 0;
  else if (i == 0 || j == 0) s = 1;
  else s = legendre((i - 1) - (j - 1), q);
  const int A = (u == 1 && v == 1) ? -1 : 1;
  const int B = (u == 0 && v == 0) ? 1 : -1;
  return s * A + (i == j ? B : 0);
}

// the signs as a compile-time table: the unrolled combination below becomes plain additions and subtractions
template <int M_>
struct PaleySigns {
  bool neg[M_][M_];
  constexpr PaleySigns() : neg{} {
    for (int a = 0; a < M_; ++a)
      for (int a2 = 0; a2 < M_; ++a2) neg[a][a2] = M_ > 1 && paley_entry(M_, a, a2) < 0;
  }
};

template <int M_>
__global__ __launch_bounds__(kHadThreads) void hadamard_quant_kernel(const float* __restrict__ Hin, int I, int p, int k,
                                                                     float qmax,
                                                                     int8_t* __restrict__ Q, uint16_t* __restrict__ Q16,
                                                                     float* __restrict__ scale,
                                                                     float* __restrict__ HR) {
  extern __shared__ float row[];
  __shared__ float red[kHadThreads / 64];
  const int tid = threadIdx.x;
  const size_t r = blockIdx.x;
  const float* src = Hin + r * (size_t)I;
  for (int c = tid * 4; c < I; c += kHadThreads * 4)
    *reinterpret_cast<float4*>(row + c) = *reinterpret_cast<const float4*>(src + c);
  __syncthreads();

  // ---- Walsh-Hadamard butterflies inside every block of p = 2^k values, two stages per barrier ----
  int s = 0;
  for (; s + 1 < k; s += 2) {
    // quadruple (i, i+d, i+2d, i+3d), d = 2^s: index bits s and s+1 are the local ones
    const int d = 1 << s;
    for (int idx = tid; idx < (I >> 2); idx += kHadThreads) {
      const int i = ((idx >> s) << (s + 2)) | (idx & (d - 1));
      const float a = row[i], b = row[i + d], c = row[i + 2 * d], e = row[i + 3 * d];
      const float ab = a + b, amb = a - b, ce = c + e, cme = c - e;
      row[i] = ab + ce;
      row[i + d] = amb + cme;
      row[i + 2 * d] = ab - ce;
      row[i + 3 * d] = amb - cme;
    }
    __syncthreads();
  }
  if (s < k) {
    const int d = 1 << s;
    for (int idx = tid; idx < (I >> 1); idx += kHadThreads) {
      const int i = ((idx >> s) << (s + 1)) | (idx & (d - 1));
      const float a = row[i], b = row[i + d];
      row[i] = a + b;
      row[i + d] = a - b;
    }
    __syncthreads();
  }

  // ---- the m blocks are combined with the signs of H_m: out[a2] = sum_a v[a] H_m[a][a2]; scaling ----
  const float norm = 1.f / sqrtf((float)I);
  float amax = 0.f;
  for (int b = tid; b < p; b += kHadThreads) {
    float v[M_];
#pragma unroll
    for (int a = 0; a < M_; ++a) v[a] = row[a * p + b];
    if constexpr (M_ == 1) {
      const float o = v[0] * norm;
      row[b] = o;
      amax = fmaxf(amax, fabsf(o));
    } else {
      constexpr PaleySigns<M_> sg{};
#pragma unroll
      for (int a2 = 0; a2 < M_; ++a2) {
        float acc = 0.f;
#pragma unroll
        for (int a = 0; a < M_; ++a) acc += sg.neg[a][a2] ? -v[a] : v[a];
        const float o = acc * norm;
        row[a2 * p + b] = o;   // only this thread touches position b of any block
        amax = fmaxf(amax, fabsf(o));
      }
    }
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) amax = fmaxf(amax, __shfl_xor(amax, off));
  if ((tid & 63) == 0) red[tid >> 6] = amax;
  __syncthreads();
  amax = red[0];
#pragma unroll
  for (int i = 1; i < kHadThreads / 64; ++i) amax = fmaxf(amax, red[i]);
  const float sc = amax == 0.f ? 1.f : amax / qmax;
  if (tid == 0) scale[r] = sc;

  // ---- integer codes: round to nearest, ties to even ----
  for (int c = tid * 4; c < I; c += kHadThreads * 4) {
    const float4 v = *reinterpret_cast<const float4*>(row + c);
    if (HR) *reinterpret_cast<float4*>(HR + r * (size_t)I + c) = v;
    const float r0 = fminf(fmaxf(rintf(v.x / sc), -qmax), qmax);
    const float r1 = fminf(fmaxf(rintf(v.y / sc), -qmax), qmax);
    const float r2 = fminf(fmaxf(rintf(v.z / sc), -qmax), qmax);
    const float r3 = fminf(fmaxf(rintf(v.w / sc), -qmax), qmax);
    const uint32_t packed = ((uint32_t)(int)r0 & 0xffu) | (((uint32_t)(int)r1 & 0xffu) << 8) |
                            (((uint32_t)(int)r2 & 0xffu) << 16) | (((uint32_t)(int)r3 & 0xffu) << 24);
    if (Q) *reinterpret_cast<uint32_t*>(Q + r * (size_t)I + c) = packed;
    if (Q16)  // the same codes as bf16 bit patterns (exact: small integers)
      *reinterpret_cast<uint2*>(Q16 + r * (size_t)I + c) =
          make_uint2((__float_as_uint(r0) >> 16) | (__float_as_uint(r1) & 0xffff0000u),
                     (__float_as_uint(r2) >> 16) | (__float_as_uint(r3) & 0xffff0000u));
  }
}

// I = m * 2^k with m in {1, 12, 28, 44}; false if I has no such form
bool had_split(int I, int* m, int* p, int* k) {
  if (I <= 0) return false;
  int odd = I, twos = 0;
  while ((odd & 1) == 0) { odd >>= 1; ++twos; }
  if (odd == 1) { *m = 1; *p = I; *k = twos; return true; }
  if (odd != 3 && odd != 7 && odd != 11) return false;
  if (twos < 2) return false;
  *m = 4 * odd;
  *k = twos - 2;
  *p = 1 << *k;
  return true;
}

}  // namespace

bool cq_hadamard_supported(int I) {
  int m, p, k;
  return had_split(I, &m, &p, &k) && I % 4 == 0 && I <= kHadMaxI;
}

cq_status cq_hadamard_quant_launch(const float* Hin, int M, int I, int bits, int8_t* Q, uint16_t* Q16, float* scale,
                                   float* HR, hipStream_t s) {
  int m, p, k;
  if (!had_split(I, &m, &p, &k)) return CQ_ERR_SHAPE;
  if (M == 0) return CQ_OK;
  {
    static std::atomic<bool> c1{false}, c12{false}, c28{false}, c44{false};
    constexpr int kMaxLds = kHadMaxI * 4;
    if (cq_configure_lds(hadamard_quant_kernel<1>, kMaxLds, c1, false) != CQ_OK ||
        cq_configure_lds(hadamard_quant_kernel<12>, kMaxLds, c12, false) != CQ_OK ||
        cq_configure_lds(hadamard_quant_kernel<28>, kMaxLds, c28, false) != CQ_OK ||
        cq_configure_lds(hadamard_quant_kernel<44>, kMaxLds, c44, false) != CQ_OK)
      return CQ_ERR_HIP;
  }
  const float qmax = (float)((1 << (bits - 1)) - 1);
  const size_t lds = (size_t)I * 4;
  switch (m) {
    case 1:
      hipLaunchKernelGGL(hadamard_quant_kernel<1>, dim3(M), dim3(kHadThreads), lds, s, Hin, I, p, k, qmax, Q, Q16,
                         scale, HR);
      break;
    case 12:
      hipLaunchKernelGGL(hadamard_quant_kernel<12>, dim3(M), dim3(kHadThreads), lds, s, Hin, I, p, k, qmax, Q, Q16,
                         scale, HR);
      break;
    case 28:
      hipLaunchKernelGGL(hadamard_quant_kernel<28>, dim3(M), dim3(kHadThreads), lds, s, Hin, I, p, k, qmax, Q, Q16,
                         scale, HR);
      break;
    default:
      hipLaunchKernelGGL(hadamard_quant_kernel<44>, dim3(M), dim3(kHadThreads), lds, s, Hin, I, p, k, qmax, Q, Q16,
                         scale, HR);
      break;
  }
  return cq_check_launch();
}

extern "C" cq_status cq_hadamard_quant(const float* Hrows, int M, int I, int bits, float* HR_out, int8_t* Q_out,
                                       float* scale_out, cq_stream stream) {
  if (M < 0 || I <= 0) return CQ_ERR_SHAPE;
  if (!cq_hadamard_supported(I)) return CQ_ERR_SHAPE;
  if (bits != 4 && bits != 8) return CQ_ERR_UNSUPPORTED;
  if (M == 0) return CQ_OK;  // nothing to do (the pointers may be NULL)
  if (!Hrows || !Q_out || !scale_out) return CQ_ERR_NULL;
  return cq_hadamard_quant_launch(Hrows, M, I, bits, Q_out, nullptr, scale_out, HR_out, (hipStream_t)stream);
}
