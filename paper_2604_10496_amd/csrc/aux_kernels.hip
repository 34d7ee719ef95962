// a8 (weighted combine) and the small helpers: offline prepack of the index bytes, the dense-decode
// test hook, the streaming-read probe and device facts.
#include "cq_internal.h"

namespace {

// Y[t,:] = sum_j w[t,j] * O[inv_perm[t*k+j], :] + sum_s O[T*k + s*T + t, :], fixed order.  O may come
// as `slices` partial copies (K splits of the down projection), added in slice order first.
__global__ __launch_bounds__(256) void combine_kernel(const float* __restrict__ O, int slices, size_t slice_stride,
                                                      const float* __restrict__ w,
                                                      const int32_t* __restrict__ inv_perm, int T, int H, int k,
                                                      int S, float* __restrict__ Y) {
  // one thread per (token, 4 columns): blockIdx.x = token, blockIdx.y = block of 1024 columns
  const int t = blockIdx.x;
  const int c = (blockIdx.y * 256 + threadIdx.x) * 4;
  if (c >= H) return;
  auto row_of = [&](size_t row) {
    const float* src = O + row * H + c;
    float4 o = *reinterpret_cast<const float4*>(src);
#pragma unroll 4
    for (int q = 1; q < slices; ++q) {
      const float4 v = *reinterpret_cast<const float4*>(src + (size_t)q * slice_stride);
      o.x += v.x; o.y += v.y; o.z += v.z; o.w += v.w;
    }
    return o;
  };
  float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
  for (int j = 0; j < k; ++j) {
    const float wt = w[(size_t)t * k + j];
    const float4 o = row_of((size_t)inv_perm[(size_t)t * k + j]);
    acc.x += wt * o.x; acc.y += wt * o.y; acc.z += wt * o.z; acc.w += wt * o.w;
  }
  for (int s = 0; s < S; ++s) {
    const float4 o = row_of((size_t)T * k + (size_t)s * T + t);
    acc.x += o.x; acc.y += o.y; acc.z += o.z; acc.w += o.w;
  }
  *reinterpret_cast<float4*>(Y + (size_t)t * H + c) = acc;
}

// canonical [rows, K/2] -> tiles of 32 rows x 64 weights (1 KiB): lane l of a tile owns the 16 bytes
// of row l%32, byte columns s*32 + (l/32)*16.  Inside every dword (8 weights w0..w7) the nibbles are
// regrouped: byte i holds w_i (low nibble) and w_{i+4} (high nibble), so that the register decoder's two
// nibble planes are the first and the second four weights (no reordering after the lookup).
__device__ __forceinline__ uint32_t regroup_nibbles(uint32_t d) {
  const uint32_t lo = d & 0x0f0f0f0fu;         // w0 w2 w4 w6
  const uint32_t hi = (d >> 4) & 0x0f0f0f0fu;  // w1 w3 w5 w7
  const uint32_t x = __builtin_amdgcn_perm(hi, lo, 0x05010400u);  // w0 w1 w2 w3
  const uint32_t y = __builtin_amdgcn_perm(hi, lo, 0x07030602u);  // w4 w5 w6 w7
  return x | (y << 4);
}

// (regroup = 0: the bytes are moved unchanged -- the 2-bit stream, whose rows of K/4 bytes are passed as K/2 "weights")
__global__ __launch_bounds__(256) void prepack_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst,
                                                      size_t n_rows, int K, int regroup) {
  const size_t n16 = n_rows * (size_t)(K / 32);  // 16-byte pieces in total
  const int steps = K / 64;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += (size_t)gridDim.x * 256) {
    const size_t tile = i >> 6;
    const int l = (int)(i & 63);
    const size_t rb = tile / steps;
    const int s = (int)(tile - rb * steps);
    const size_t row = rb * 32 + (l & 31);
    const size_t piece = (size_t)s * 2 + (l >> 5);  // 16-byte piece inside the row
    const uint4 v = src[row * (size_t)(K / 32) + piece];
    dst[i] = regroup ? make_uint4(regroup_nibbles(v.x), regroup_nibbles(v.y), regroup_nibbles(v.z), regroup_nibbles(v.w))
                     : v;
  }
}

__global__ __launch_bounds__(256) void decode_dense_kernel(const uint8_t* __restrict__ idx, int prepacked,
                                                           const uint16_t* __restrict__ cent, int nblk, int group_k,
                                                           int N, int K, uint16_t* __restrict__ out) {
  const size_t total = (size_t)N * (K / 2);
  const int steps = K / 64;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (size_t)gridDim.x * 256) {
    const size_t n = i / (K / 2);
    const int bc = (int)(i - n * (K / 2));  // canonical byte column: weights 2 bc and 2 bc + 1
    const uint16_t* c = cent + (n * nblk + (size_t)((2 * bc) / group_k)) * CQ_N_CENTROIDS;  // group_k is even
    uint32_t i0, i1;
    if (prepacked) {
      // 16-byte piece of (row block, step, lane); inside a dword weight w of 8 sits in byte w % 4, nibble w / 4
      const int s = bc >> 5, g = (bc >> 4) & 1, within = bc & 15;
      const size_t piece = (((n >> 5) * steps + s) * 64 + g * 32 + (n & 31)) * 16 + (within & ~3);
      const int w0 = 2 * (within & 3), w1 = w0 + 1;
      i0 = (idx[piece + (w0 & 3)] >> (4 * (w0 >> 2))) & 15u;
      i1 = (idx[piece + (w1 & 3)] >> (4 * (w1 >> 2))) & 15u;
    } else {
      const uint32_t b = idx[i];
      i0 = b & 15u;
      i1 = b >> 4;
    }
    out[n * K + 2 * bc] = c[i0];
    out[n * K + 2 * bc + 1] = c[i1];
  }
}

// index_bits = 2: W_c[n, k] = C[n, (byte k/4 of row n >> 2(k%4)) & 3], from canonical bytes or from the prepacked
// tiles (32 rows x 128 weights: lane l = row%32 + 32 * ((k%128)/64) holds 16 bytes at l*16); one thread per byte
__global__ __launch_bounds__(256) void decode_dense_w2_kernel(const uint8_t* __restrict__ idx, int prepacked,
                                                              const uint16_t* __restrict__ cent, int N, int K,
                                                              uint16_t* __restrict__ out) {
  const size_t rowbytes = (size_t)K / 4, total = (size_t)N * rowbytes;
  const int steps = K / 128;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (size_t)gridDim.x * 256) {
    const size_t n = i / rowbytes;
    const int bc = (int)(i - n * rowbytes);   // canonical byte column: weights 4 bc .. 4 bc + 3
    uint32_t b;
    if (prepacked) {
      const int s = bc >> 5, g = (bc >> 4) & 1, within = bc & 15;
      b = idx[(((n >> 5) * steps + s) * 64 + g * 32 + (n & 31)) * 16 + within];
    } else {
      b = idx[i];
    }
    const uint16_t* c = cent + n * 4;
#pragma unroll
    for (int w = 0; w < 4; ++w) out[n * K + 4 * (size_t)bc + w] = c[(b >> (2 * w)) & 3u];
  }
}

// Budgets of 4 or 8 centroids: indices packed as a little-endian bit stream per row (weight j at bits
// [j*bits, (j+1)*bits)) -> the canonical 4-bit bytes; one thread per output byte (two weights).
__global__ __launch_bounds__(256) void expand_indices_kernel(const uint8_t* __restrict__ src, int bits, size_t n_rows,
                                                             int K, uint8_t* __restrict__ dst) {
  const size_t half = (size_t)K / 2, total = n_rows * half;
  const size_t src_row = (size_t)K * bits / 8;
  const uint32_t mask = (1u << bits) - 1u;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (size_t)gridDim.x * 256) {
    const size_t n = i / half;
    const uint32_t j = (uint32_t)(i - n * half);
    const uint8_t* row = src + n * src_row;
    uint32_t v[2];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const uint32_t bit = (2 * j + h) * bits, byte = bit >> 3;
      uint32_t w = row[byte];
      if (byte + 1 < src_row) w |= (uint32_t)row[byte + 1] << 8;  // a field may straddle two bytes
      v[h] = (w >> (bit & 7)) & mask;
    }
    dst[i] = (uint8_t)(v[0] | (v[1] << 4));
  }
}

// tables of 2^bits entries -> 16 entries (the entries that no index can address repeat the last real one)
__global__ __launch_bounds__(256) void expand_tables_kernel(const uint16_t* __restrict__ src, int bits, size_t n_tables,
                                                            uint16_t* __restrict__ dst) {
  const int n = 1 << bits;
  const size_t total = n_tables * CQ_N_CENTROIDS;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (size_t)gridDim.x * 256) {
    const size_t t = i / CQ_N_CENTROIDS;
    const int c = (int)(i - t * CQ_N_CENTROIDS);
    dst[i] = src[t * n + (c < n ? c : n - 1)];
  }
}

// 16 independent accumulators per wavefront: the matrix pipe never waits for a result
__global__ __launch_bounds__(256) void mfma_loop_kernel(int iters, float* __restrict__ sink) {
  cq_v16f acc[16];
#pragma unroll
  for (int i = 0; i < 16; ++i)
#pragma unroll
    for (int j = 0; j < 16; ++j) acc[i][j] = 0.f;
  const cq_v4u av = {0x3f803f80u + threadIdx.x, 0x3f803f80u, 0x3f803f80u, 0x3f803f80u};  // ~1.0 in bf16 pairs
  const cq_v8bf16 a = __builtin_bit_cast(cq_v8bf16, av);
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, a, acc[i], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 16; ++i) s += acc[i][i];
  sink[(size_t)blockIdx.x * 256 + threadIdx.x] = s;
}

// Streaming-read yardstick, shaped like the product kernel's index stream: one workgroup of 8 wavefronts per
// contiguous chunk of 512 KiB; a wavefront load is one contiguous KiB (16 bytes per lane, non-temporal); the
// wavefronts take the chunk's KiB steps in turn and keep 8 of them in flight each (64 KiB per workgroup).
constexpr int kReadChunk = 512 << 10;
__global__ __launch_bounds__(512, 1) void stream_read_kernel(const uint4* __restrict__ src, uint32_t* __restrict__ sink) {
  constexpr int NW = 8, D = 8, kSteps = kReadChunk / 1024, Q = kSteps / NW;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const cq_v4u* base = reinterpret_cast<const cq_v4u*>(src) + (size_t)blockIdx.x * (kReadChunk / 16) + lane;
  cq_v4u ring[D];
#pragma unroll
  for (int j = 0; j < D; ++j) ring[j] = __builtin_nontemporal_load(base + (size_t)(wave + NW * j) * 64);
  cq_v4u acc = {0u, 0u, 0u, 0u};
  for (int q0 = 0; q0 < Q; q0 += D) {
#pragma unroll
    for (int j = 0; j < D; ++j) {
      const cq_v4u w = ring[j];
      const int qn = q0 + j + D;   // (clamped re-reads of step 0 at the end: cache hits, a few per cent of the loads)
      ring[j] = __builtin_nontemporal_load(base + (size_t)(qn < Q ? wave + NW * qn : 0) * 64);
      acc ^= w;
    }
  }
  // keeps the loads alive; the branch is practically never taken
  if ((acc[0] ^ acc[1] ^ acc[2] ^ acc[3]) == 0x9e3779b9u) {
    sink[0] = acc[0]; sink[1] = acc[1]; sink[2] = acc[2]; sink[3] = acc[3];
  }
}

// the bytes past the last whole chunk
__global__ __launch_bounds__(256) void stream_read_tail_kernel(const uint4* __restrict__ src, size_t n16,
                                                               uint32_t* __restrict__ sink) {
  uint4 acc = make_uint4(0u, 0u, 0u, 0u);
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += (size_t)gridDim.x * 256) {
    const uint4 a = src[i];
    acc.x ^= a.x; acc.y ^= a.y; acc.z ^= a.z; acc.w ^= a.w;
  }
  if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x9e3779b9u) {
    sink[0] = acc.x; sink[1] = acc.y; sink[2] = acc.z; sink[3] = acc.w;
  }
}

}  // namespace

extern "C" const char* cq_status_string(cq_status st) {
  switch (st) {
    case CQ_OK: return "CQ_OK";
    case CQ_ERR_NULL: return "CQ_ERR_NULL: a required pointer is NULL";
    case CQ_ERR_SHAPE: return "CQ_ERR_SHAPE: size out of range or not a multiple of the tile";
    case CQ_ERR_UNSUPPORTED: return "CQ_ERR_UNSUPPORTED: unsupported bit width or enum value";
    case CQ_ERR_WORKSPACE: return "CQ_ERR_WORKSPACE: workspace missing or too small";
    case CQ_ERR_HIP: return "CQ_ERR_HIP: HIP runtime error";
    default: return "unknown cq_status";
  }
}

cq_status cq_combine_launch(const float* O, int slices, size_t slice_stride, const float* topk_w,
                            const int32_t* inv_perm, int T, int H, int top_k, int n_shared, float* Y, hipStream_t s) {
  hipLaunchKernelGGL(combine_kernel, dim3(T, (H + 1023) / 1024), dim3(256), 0, s, O, slices, slice_stride, topk_w,
                     inv_perm, T, H, top_k, n_shared, Y);
  return cq_check_launch();
}

extern "C" cq_status cq_combine(const float* O, const float* topk_w, const int32_t* inv_perm, int T, int H,
                                int top_k, int n_shared, float* Y, cq_stream stream) {
  if (!O || !topk_w || !inv_perm || !Y) return CQ_ERR_NULL;
  if (T <= 0 || H <= 0 || H % 4 != 0 || top_k <= 0 || n_shared < 0) return CQ_ERR_SHAPE;
  return cq_combine_launch(O, 1, 0, topk_w, inv_perm, T, H, top_k, n_shared, Y, (hipStream_t)stream);
}

extern "C" size_t cq_prepack_bytes(const cq_codebook_weights* W) {
  if (!W || W->G <= 0 || W->N <= 0 || W->K <= 0) return 0;
  return (size_t)W->G * W->N * (W->K / (cq_is_w2(W) ? 4 : 2));
}

extern "C" cq_status cq_prepack(const cq_codebook_weights* W, void* dst, size_t dst_bytes, cq_stream stream) {
  if (!W || !W->idx || !dst) return CQ_ERR_NULL;
  if (W->G <= 0 || W->N <= 0 || W->K <= 0 || W->N % 64 != 0 || W->K % 64 != 0) return CQ_ERR_SHAPE;
  if (W->index_bits != 0 && W->index_bits != 4 && W->index_bits != 2) return CQ_ERR_UNSUPPORTED;
  if (cq_is_w2(W) && W->K % 128 != 0) return CQ_ERR_SHAPE;
  if (dst_bytes < cq_prepack_bytes(W)) return CQ_ERR_WORKSPACE;
  const size_t rows = (size_t)W->G * W->N;
  const int k_eff = cq_is_w2(W) ? W->K / 2 : W->K;   // a row of K/4 bytes tiles like a 4-bit row of K/2 weights
  const size_t n16 = rows * (k_eff / 32);
  const unsigned grid = (unsigned)((n16 + 255) / 256 < 65536 ? (n16 + 255) / 256 : 65536);
  hipLaunchKernelGGL(prepack_kernel, dim3(grid), dim3(256), 0, (hipStream_t)stream, (const uint4*)W->idx,
                     (uint4*)dst, rows, k_eff, cq_is_w2(W) ? 0 : 1);
  return cq_check_launch();
}

extern "C" cq_status cq_expand_centroid_budget(const uint8_t* idx_bits, const uint16_t* cent_bits, int bits, int G,
                                               int N, int K, int tables_per_row, uint8_t* idx4_out,
                                               uint16_t* cent16_out, cq_stream stream) {
  if (!idx_bits || !cent_bits || !idx4_out || !cent16_out) return CQ_ERR_NULL;
  if (G <= 0 || N <= 0 || K <= 0 || tables_per_row <= 0 || K % 64 != 0) return CQ_ERR_SHAPE;
  if (bits != 2 && bits != 3) return CQ_ERR_UNSUPPORTED;
  const size_t rows = (size_t)G * N, bytes = rows * (K / 2), entries = rows * tables_per_row * CQ_N_CENTROIDS;
  const unsigned g1 = (unsigned)((bytes + 255) / 256 < 65536 ? (bytes + 255) / 256 : 65536);
  const unsigned g2 = (unsigned)((entries + 255) / 256 < 65536 ? (entries + 255) / 256 : 65536);
  hipLaunchKernelGGL(expand_indices_kernel, dim3(g1), dim3(256), 0, (hipStream_t)stream, idx_bits, bits, rows, K,
                     idx4_out);
  hipLaunchKernelGGL(expand_tables_kernel, dim3(g2), dim3(256), 0, (hipStream_t)stream, cent_bits, bits,
                     rows * tables_per_row, cent16_out);
  return cq_check_launch();
}

extern "C" cq_status cq_decode_dense(const cq_codebook_weights* W, int g, uint16_t* Wc_bf16, cq_stream stream) {
  if (!W || (!W->idx && !W->prepacked) || !W->cent || !Wc_bf16) return CQ_ERR_NULL;
  if (W->G <= 0 || W->N <= 0 || W->K <= 0 || W->N % 64 != 0 || W->K % 64 != 0) return CQ_ERR_SHAPE;
  if (g < 0 || g >= W->G || W->group_k < 0 || W->group_k % 2 != 0) return CQ_ERR_SHAPE;
  if (cq_is_w2(W)) {
    if (W->K % 128 != 0 || cq_tables_per_row(W) > 1) return CQ_ERR_UNSUPPORTED;
    const size_t gb = (size_t)W->N * (W->K / 4);
    const uint8_t* src2 = (W->prepacked ? (const uint8_t*)W->prepacked : W->idx) + (size_t)g * gb;
    const unsigned grid2 = (unsigned)((gb + 255) / 256 < 65536 ? (gb + 255) / 256 : 65536);
    hipLaunchKernelGGL(decode_dense_w2_kernel, dim3(grid2), dim3(256), 0, (hipStream_t)stream, src2,
                       W->prepacked ? 1 : 0, W->cent + (size_t)g * W->N * 4, W->N, W->K, Wc_bf16);
    return cq_check_launch();
  }
  const int nblk = cq_tables_per_row(W);
  const size_t gbytes = (size_t)W->N * (W->K / 2);
  const uint8_t* src = (W->prepacked ? (const uint8_t*)W->prepacked : W->idx) + (size_t)g * gbytes;
  const unsigned grid = (unsigned)((gbytes + 255) / 256 < 65536 ? (gbytes + 255) / 256 : 65536);
  hipLaunchKernelGGL(decode_dense_kernel, dim3(grid), dim3(256), 0, (hipStream_t)stream, src,
                     W->prepacked ? 1 : 0, W->cent + (size_t)g * W->N * nblk * CQ_N_CENTROIDS, nblk,
                     nblk > 1 ? W->group_k : W->K, W->N, W->K, Wc_bf16);
  return cq_check_launch();
}

extern "C" cq_status cq_device_info(int* cu_count, int* clock_khz, int* mem_clock_khz, int* bus_bits,
                                    int* lds_bytes) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return CQ_ERR_HIP;
  struct { int* dst; hipDeviceAttribute_t attr; } q[] = {
      {cu_count, hipDeviceAttributeMultiprocessorCount}, {clock_khz, hipDeviceAttributeClockRate},
      {mem_clock_khz, hipDeviceAttributeMemoryClockRate}, {bus_bits, hipDeviceAttributeMemoryBusWidth},
      {lds_bytes, hipDeviceAttributeMaxSharedMemoryPerBlock}};
  for (auto& e : q) {
    int v = 0;
    if (hipDeviceGetAttribute(&v, e.attr, dev) != hipSuccess) return CQ_ERR_HIP;
    if (e.dst) *e.dst = v;
  }
  return CQ_OK;
}

extern "C" cq_status cq_mfma_loop(int workgroups, int iters, float* sink, cq_stream stream) {
  if (!sink) return CQ_ERR_NULL;
  if (workgroups <= 0 || iters <= 0) return CQ_ERR_SHAPE;
  hipLaunchKernelGGL(mfma_loop_kernel, dim3(workgroups), dim3(256), 0, (hipStream_t)stream, iters, sink);
  return cq_check_launch();
}

extern "C" cq_status cq_stream_read(const void* src, size_t bytes, uint32_t* sink, cq_stream stream) {
  if (!src || !sink) return CQ_ERR_NULL;
  if (bytes == 0 || bytes % 16 != 0) return CQ_ERR_SHAPE;
  const size_t chunks = bytes / kReadChunk;
  if (chunks > 0x7fffffffu) return CQ_ERR_SHAPE;
  if (chunks > 0)
    hipLaunchKernelGGL(stream_read_kernel, dim3((unsigned)chunks), dim3(512), 0, (hipStream_t)stream, (const uint4*)src,
                       sink);
  const size_t rest16 = (bytes - chunks * kReadChunk) / 16;
  if (rest16 > 0)
    hipLaunchKernelGGL(stream_read_tail_kernel, dim3((unsigned)((rest16 + 255) / 256)), dim3(256), 0,
                       (hipStream_t)stream, (const uint4*)src + chunks * (kReadChunk / 16), rest16, sink);
  return cq_check_launch();
}
