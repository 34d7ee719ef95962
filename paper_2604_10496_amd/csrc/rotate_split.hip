// a1 for prefill-sized batches: X_R = X R on the f16 matrix cores at (about) fp32 accuracy.
//
// Every fp32 operand is written as hi + 2^-11 lo with hi = f16(v) and lo = f16((v - hi) 2^11): v - hi is
// exact in fp32 and has at most 13 significant bits, so hi + 2^-11 lo differs from v by at most 2^-23 |v|.
// Products of two f16 numbers are exact in fp32, and the matrix cores accumulate in fp32, so
//     2^11 X R  =  Xh (2^11 Rh)  +  Xh Rl  +  Xl Rh  +  2^-11 Xl Rl
// evaluated without its last term (relative size 2^-22) is as accurate as an fp32 product, at three f16
// MFMAs per tile step instead of one fp32 MFMA step that is sixteen times slower.  All three products
// carry the same factor 2^11 and go into ONE accumulator (2^11 Rh is formed in registers from Rh: an
// exact exponent shift, |R| < 32 assumed -- R is orthogonal).  Rows of X are divided by a power of two
// first (exact) so that their largest entry lies in [1, 2): no f16 overflow or underflow whatever the
// scale of the activations.  R is split once, when the layer is set up, into the order the MFMA
// fragments are loaded in.
//
// Kernel: workgroup tile 256 output columns x 128 tokens, four wavefronts, each owning 64 columns (as
// MFMA "A" rows, two blocks of 32) and all 128 tokens (2 x 4 accumulator blocks of 32x32).  R fragments
// go from global memory (L2) straight into registers, one step (64 k) ahead; token tiles (both halves)
// arrive by direct global->LDS loads, four steps deep.
#include "cq_internal.h"
#include "cq_async.h"

namespace {

using namespace cq_async;

constexpr int kCols = 256;             // output columns per workgroup
constexpr int kTok = 128;              // tokens per workgroup
constexpr int kC = kTok / 32;          // token blocks
constexpr int kStepK = 64;             // K per pipeline step (four MFMA sub-steps of 16)
constexpr int kStepBytes = kStepK * 2; // one token's share of a step and plane, in LDS and in memory
constexpr int kPlaneBytes = kTok * kStepBytes;   // 16 KiB
constexpr int kStageBytes = 2 * kPlaneBytes;     // hi and lo tile of one step
constexpr int kDepth = 4;                        // token tiles in LDS
constexpr int kRotLdsBytes = kDepth * kStageBytes;  // 128 KiB
constexpr int kOutStride = kCols * 4 + 16;       // epilogue staging row (64 tokens at a time)
constexpr float kLoScale = 2048.f, kLoUnscale = 1.f / 2048.f;

__device__ __forceinline__ uint32_t f16_bits(float x) {
  const _Float16 h = (_Float16)x;
  return (uint32_t) __builtin_bit_cast(uint16_t, h);
}
__device__ __forceinline__ float f16_value(float x) { return (float)(_Float16)x; }

// R [K, N] fp32 -> fragments: block nb = n/32, sub-step j = k/16, plane p (0 hi, 1 lo): 1 KiB at
// ((nb*(K/16) + j)*2 + p)*1024 holding, for lane l, R[j*16 + (l/32)*8 + i][nb*32 + l%32], i = 0..7.
__global__ __launch_bounds__(256) void split_R_kernel(const float* __restrict__ R, int H, uint4* __restrict__ out) {
  const int nJ = H / 16;
  const size_t frag = (size_t)blockIdx.x * 4 + (threadIdx.x >> 6);  // (nb, j)
  const int lane = threadIdx.x & 63;
  if (frag >= (size_t)(H / 32) * nJ) return;
  const int nb = (int)(frag / nJ), j = (int)(frag - (size_t)nb * nJ);
  const int n = nb * 32 + (lane & 31), k0 = j * 16 + (lane >> 5) * 8;
  uint32_t hi[4], lo[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const float a = R[(size_t)(k0 + 2 * i) * H + n], b = R[(size_t)(k0 + 2 * i + 1) * H + n];
    const float ah = f16_value(a), bh = f16_value(b);
    hi[i] = f16_bits(ah) | (f16_bits(bh) << 16);
    lo[i] = f16_bits((a - ah) * kLoScale) | (f16_bits((b - bh) * kLoScale) << 16);
  }
  out[(frag * 2 + 0) * 64 + lane] = make_uint4(hi[0], hi[1], hi[2], hi[3]);
  out[(frag * 2 + 1) * 64 + lane] = make_uint4(lo[0], lo[1], lo[2], lo[3]);
}

// One workgroup per token: row maximum, power-of-two scale s (largest entry of x/s in [1, 2)), then the
// two f16 planes of x/s.  planes: hi [T, H], lo [T, H] (the latter times 2^11); row_pow2 [T] = s.
__global__ __launch_bounds__(256) void split_X_kernel(const float* __restrict__ X, int T, int H,
                                                      uint16_t* __restrict__ hi, uint16_t* __restrict__ lo,
                                                      float* __restrict__ row_pow2) {
  __shared__ float red[4];
  const int t = blockIdx.x, tid = threadIdx.x;
  const float* x = X + (size_t)t * H;
  float amax = 0.f;
  for (int c = tid * 4; c < H; c += 1024) {
    const float4 v = *reinterpret_cast<const float4*>(x + c);
    amax = fmaxf(amax, fmaxf(fmaxf(fabsf(v.x), fabsf(v.y)), fmaxf(fabsf(v.z), fabsf(v.w))));
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) amax = fmaxf(amax, __shfl_xor(amax, off));
  if ((tid & 63) == 0) red[tid >> 6] = amax;
  __syncthreads();
  amax = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
  // s = 2^floor(log2(amax)): the exponent field alone (1 for a zero or denormal maximum)
  const uint32_t ebits = __float_as_uint(amax) & 0x7f800000u;
  const float s = ebits == 0u ? 1.f : __uint_as_float(ebits);
  const float inv = 1.f / s;  // exact: a power of two
  if (tid == 0) row_pow2[t] = s;
  for (int c = tid * 4; c < H; c += 1024) {
    const float4 v = *reinterpret_cast<const float4*>(x + c);
    const float a[4] = {v.x * inv, v.y * inv, v.z * inv, v.w * inv};
    float h[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) h[i] = f16_value(a[i]);
    *reinterpret_cast<uint2*>(hi + (size_t)t * H + c) =
        make_uint2(f16_bits(h[0]) | (f16_bits(h[1]) << 16), f16_bits(h[2]) | (f16_bits(h[3]) << 16));
    *reinterpret_cast<uint2*>(lo + (size_t)t * H + c) =
        make_uint2(f16_bits((a[0] - h[0]) * kLoScale) | (f16_bits((a[1] - h[1]) * kLoScale) << 16),
                   f16_bits((a[2] - h[2]) * kLoScale) | (f16_bits((a[3] - h[3]) * kLoScale) << 16));
  }
}

struct RotArgs {
  const uint8_t* Rs;       // split R fragments
  const uint16_t* Xh;      // [T, K] f16
  const uint16_t* Xl;      // [T, K] f16 (times 2^11)
  const float* row_pow2;   // [T]
  float* XR;               // [T, N] fp32
  int T, N, K;
  int row_tiles;           // N / 256
  int n_work;              // token tiles x row tiles
};

// pairs of f16 times 2^11 (exact: an exponent shift)
typedef _Float16 cq_h2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pair_times_2048(uint32_t a) {
  const cq_h2 k = {(_Float16)2048.f, (_Float16)2048.f};
  const cq_h2 v = __builtin_bit_cast(cq_h2, a) * k;
  return __builtin_bit_cast(uint32_t, v);
}
__device__ __forceinline__ cq_v4u times_2048(const cq_v4u a) {
  // (built in one piece: element-wise stores into an uninitialised vector were seen to compile into a
  // broadcast of element 0 here)
  const cq_v4u r = {pair_times_2048(a[0]), pair_times_2048(a[1]), pair_times_2048(a[2]), pair_times_2048(a[3])};
  return r;
}

__device__ __forceinline__ cq_v16f mfma_f16(const cq_v4u a, const cq_v4u b, cq_v16f c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(cq_v8f16, a), __builtin_bit_cast(cq_v8f16, b), c, 0,
                                                0, 0);
}

__global__ __launch_bounds__(256, 1) void rot_split_kernel(const RotArgs p) {
  // XCD-aware remap of the linear workgroup id (ids go round-robin over the 8 XCDs): XCD x takes a
  // contiguous share of the work, so that neighbours in its L2 share token tiles and columns of R
  const int per = (p.n_work + 7) >> 3;
  const int work = (blockIdx.x & 7) * per + (blockIdx.x >> 3);
  if ((int)(blockIdx.x >> 3) >= per || work >= p.n_work) return;
  const int tile = work / p.row_tiles, rt = work - tile * p.row_tiles;
  const int mrow0 = tile * kTok, mcnt = min(kTok, p.T - mrow0);

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int r32 = lane & 31, g2 = lane >> 5;
  const int N = p.N, K = p.K;
  const int nS = K / kStepK, nJ = K / 16;
  // this wavefront's two column blocks: nb0, nb0 + 1.  Fragment (rb, sub-step j, plane pl) of lane l is at
  // Rs + (((nb0 + rb)*nJ + j)*2 + pl)*1024 + 16 l: a uniform base, the lane offset, an immediate.
  const int nb0 = __builtin_amdgcn_readfirstlane((rt * kCols + wave * 64) / 32);
  const uint8_t* wbase = p.Rs + (size_t)nb0 * nJ * 2048;
  const size_t rbstride = (size_t)nJ * 2048;
  const uint32_t lane16 = (uint32_t)lane * 16;

  // ---- token tiles: as in the codebook product's large-tile kernel (token-major rows of 128 bytes,
  // chunk c of token t at position c ^ ((t >> 1) & 7); one direct-to-LDS load moves 8 tokens x 128 bytes;
  // the swizzle is applied on the global side).  Wavefront w moves tokens [32w, 32w + 32) of both planes:
  // 2 x 4 loads per step, one of each plane per sub-step. ----
  uint32_t aoff[4];  // byte offset of this lane's 16 bytes of step 0 within a plane (T*K*2 < 2^32)
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int tok = wave * 32 + i * 8 + (lane >> 3);
    const uint32_t row = (uint32_t)(mrow0 + min(tok, mcnt - 1));  // tokens past the end repeat the last row
    const int chunk = (lane & 7) ^ ((tok >> 1) & 7);
    aoff[i] = (row * (uint32_t)K + (uint32_t)chunk * 8) * 2;
  }
  const uint8_t* xh = reinterpret_cast<const uint8_t*>(p.Xh);
  const uint8_t* xl = reinterpret_cast<const uint8_t*>(p.Xl);
  const uint32_t lds_wave = __builtin_amdgcn_readfirstlane(wave * 32 * kStepBytes);
  auto fetch_tile_part = [&](int s, int buf, int i) {  // tokens 32w + 8i .. +7 of step s, both planes
    const size_t o = (size_t)s * kStepBytes;
    load_global_to_lds_s<0>(buf * kStageBytes + lds_wave + i * 1024, xh + o, aoff[i]);
    load_global_to_lds_s<0>(buf * kStageBytes + kPlaneBytes + lds_wave + i * 1024, xl + o, aoff[i]);
  };
  // R fragments of sub-step jj of step s: [rb][plane]
  auto fetch_R = [&](cq_v4u (&w)[2][2], int s, int jj) {
    const uint8_t* src = wbase + (size_t)(s * 4 + jj) * 2048;
    load_global_async_s<0>(w[0][0], src, lane16);
    load_global_async_s<1024>(w[0][1], src, lane16);
    load_global_async_s<0>(w[1][0], src + rbstride, lane16);
    load_global_async_s<1024>(w[1][1], src + rbstride, lane16);
  };
  // token fragment: lane (token r32 of block cb, k group g2) wants chunk 2*jj + g2 of the step (the k
  // order of the R fragments), stored at position (2*jj + g2) ^ ((r32 >> 1) & 7) = (g2 ^ ..) ^ (2*jj)
  const uint32_t boff = (uint32_t)r32 * kStepBytes + ((uint32_t)(g2 ^ ((r32 >> 1) & 7)) << 4);
  // Eight address registers (sub-step x lower / upper pair of tile buffers), made opaque to the compiler;
  // buffer, plane and token block go into the instruction's offset field.  (Left to itself the compiler
  // keeps all 128 loop-invariant addresses in registers it does not have.)
  uint32_t bx[2][4];
#pragma unroll
  for (int jj = 0; jj < 4; ++jj) {
    bx[0][jj] = boff ^ ((uint32_t)jj << 5);
    bx[1][jj] = bx[0][jj] + 2 * kStageBytes;
    asm volatile("" : "+v"(bx[0][jj]), "+v"(bx[1][jj]));
  }
  auto read_b = [&](int buf, int plane, int jj, int cb) {
    return lds_read_u128(bx[buf >> 1][jj] + (uint32_t)((buf & 1) * kStageBytes + plane * kPlaneBytes + cb * 32 * kStepBytes));
  };

  cq_v16f acc[2][kC];  // 2^11 X R
#pragma unroll
  for (int rb = 0; rb < 2; ++rb)
#pragma unroll
    for (int cb = 0; cb < kC; ++cb)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[rb][cb][i] = 0.f;

  // Vector-memory operations per sub-step, in this order: 4 R fragment loads (sub-step jj of the NEXT
  // step, into the registers just consumed), then 2 tile loads (part jj of the tile three steps ahead).
  // A fragment is therefore followed by 2 + 3*6 = 20 younger operations when its sub-step comes round,
  // and the last part of the tile two steps ahead by the 24 operations of the current step: those are
  // the two wait counts.  (A count is safe as long as at least that many younger operations exist.)
  constexpr int kPerSub = 6, kWaitR = 2 + 3 * kPerSub, kWaitTile = 4 * kPerSub;
  cq_v4u wq[4][2][2];
  // prologue, oldest first: tiles 0 and 1, the R fragments of step 0, tile 2
#pragma unroll
  for (int i = 0; i < 4; ++i) fetch_tile_part(0, 0, i);
#pragma unroll
  for (int i = 0; i < 4; ++i) fetch_tile_part(min(1, nS - 1), 1, i);
#pragma unroll
  for (int jj = 0; jj < 4; ++jj) fetch_R(wq[jj], 0, jj);
#pragma unroll
  for (int i = 0; i < 4; ++i) fetch_tile_part(min(2, nS - 1), 2, i);
  vm_wait<kWaitTile>(wq[0][0][0], wq[0][0][1], wq[0][1][0], wq[0][1][1]);  // tiles 0 and 1 have landed
  __syncthreads();

  cq_v4u bh[kC], bl[kC];
#pragma unroll
  for (int cb = 0; cb < kC; ++cb) {
    bh[cb] = read_b(0, 0, 0, cb);
    bl[cb] = read_b(0, 1, 0, cb);
  }

  int s0 = 0;
  do {  // K is a multiple of 256: steps come in fours (no zero-trip path, accumulators stay in place)
#pragma unroll
    for (int par = 0; par < kDepth; ++par) {  // step s0 + par reads tile buffer par
      const int s = s0 + par;
      const int s_next = min(s + 1, nS - 1), s_tile = min(s + 3, nS - 1);
#pragma unroll
      for (int jj = 0; jj < 4; ++jj) {
        vm_wait<kWaitR>(wq[jj][0][0], wq[jj][0][1], wq[jj][1][0], wq[jj][1][1]);
        const cq_v4u ah0 = wq[jj][0][0], al0 = wq[jj][0][1], ah1 = wq[jj][1][0], al1 = wq[jj][1][1];
        const cq_v4u aH0 = times_2048(ah0), aH1 = times_2048(ah1);
        // next sub-step's token fragments: jj + 1 of this step, or the first of the next step
        const int nbuf = jj < 3 ? par : (par + 1) & (kDepth - 1), njj = (jj + 1) & 3;
        // three products per accumulator block, a whole round of blocks apart (no back-to-back dependence)
#pragma unroll
        for (int cb = 0; cb < kC; ++cb) {
          acc[0][cb] = mfma_f16(aH0, bh[cb], acc[0][cb]);
          acc[1][cb] = mfma_f16(aH1, bh[cb], acc[1][cb]);
        }
#pragma unroll
        for (int cb = 0; cb < kC; ++cb) {
          acc[0][cb] = mfma_f16(ah0, bl[cb], acc[0][cb]);
          acc[1][cb] = mfma_f16(ah1, bl[cb], acc[1][cb]);
          bl[cb] = read_b(nbuf, 1, njj, cb);
        }
#pragma unroll
        for (int cb = 0; cb < kC; ++cb) {
          acc[0][cb] = mfma_f16(al0, bh[cb], acc[0][cb]);
          acc[1][cb] = mfma_f16(al1, bh[cb], acc[1][cb]);
          bh[cb] = read_b(nbuf, 0, njj, cb);
        }
        __builtin_amdgcn_sched_barrier(0);
        // the consumed registers take the same sub-step of the next step; then this sub-step's tile part
        fetch_R(wq[jj], s_next, jj);
        fetch_tile_part(s_tile, (par + 3) & (kDepth - 1), jj);
        __builtin_amdgcn_sched_barrier(0);
      }
      vm_wait<kWaitTile>(wq[0][0][0], wq[0][0][1], wq[0][1][0], wq[0][1][1]);  // own share of the tile two steps ahead
      __syncthreads();
    }
    s0 += kDepth;
  } while (s0 < nS);
  // Nothing of this workgroup may still be on its way into LDS when the tile buffers are reused, nor into
  // registers: the last (clamped, unused) fragment loads still target the ring, which therefore has to
  // stay allocated up to this wait -- it is named here so that the compiler cannot reuse it earlier.
  asm volatile("s_waitcnt vmcnt(0)"
               : "+v"(wq[0][0][0]), "+v"(wq[0][0][1]), "+v"(wq[0][1][0]), "+v"(wq[0][1][1]), "+v"(wq[1][0][0]),
                 "+v"(wq[1][0][1]), "+v"(wq[1][1][0]), "+v"(wq[1][1][1]), "+v"(wq[2][0][0]), "+v"(wq[2][0][1]),
                 "+v"(wq[2][1][0]), "+v"(wq[2][1][1]), "+v"(wq[3][0][0]), "+v"(wq[3][0][1]), "+v"(wq[3][1][0]),
                 "+v"(wq[3][1][1])
               :
               : "memory");

  // ---- epilogue: x = s_t 2^-11 acc; through LDS, 64 tokens at a time, so that stores are
  // row-contiguous (a lane holds 4 consecutive columns of ONE token per accumulator quad) ----
  typedef __attribute__((address_space(3))) cq_v4u lds_v4u;
#pragma unroll
  for (int pass = 0; pass < kC / 2; ++pass) {
    __syncthreads();  // the tile buffers (first pass) or the previous pass's rows are no longer read
#pragma unroll
    for (int half = 0; half < 2; ++half) {
      const int cb = pass * 2 + half;
      const int tl = half * 32 + r32;
      const float sc = p.row_pow2[mrow0 + min(cb * 32 + r32, mcnt - 1)] * kLoUnscale;
#pragma unroll
      for (int rb = 0; rb < 2; ++rb)
#pragma unroll
        for (int vb = 0; vb < 4; ++vb) {
          // MFMA 32x32 output: register v holds row 8*(v/4) + 4*(lane/32) + v%4, column lane%32
          const int col = wave * 64 + rb * 32 + vb * 8 + g2 * 4;
          const uint32_t at = (uint32_t)tl * kOutStride + (uint32_t)col * 4;
          const cq_v4u o = {__float_as_uint(sc * acc[rb][cb][4 * vb]), __float_as_uint(sc * acc[rb][cb][4 * vb + 1]),
                            __float_as_uint(sc * acc[rb][cb][4 * vb + 2]), __float_as_uint(sc * acc[rb][cb][4 * vb + 3])};
          *reinterpret_cast<lds_v4u*>((uintptr_t)at) = o;
        }
    }
    __syncthreads();
#pragma unroll
    for (int it = 0; it < 64 * (kCols / 4) / 256; ++it) {
      const int i = it * 256 + tid;
      const int tl = i / (kCols / 4), pc = i - tl * (kCols / 4);
      const int tok = pass * 64 + tl;
      if (tok < mcnt) {
        const uint32_t at = (uint32_t)tl * kOutStride + (uint32_t)pc * 16;
        float* dst = p.XR + (size_t)(mrow0 + tok) * N + (size_t)rt * kCols + pc * 4;
        *reinterpret_cast<cq_v4u*>(dst) = *reinterpret_cast<const lds_v4u*>((uintptr_t)at);
      }
    }
  }
}

}  // namespace

bool cq_rotate_split_supported(int T, int H) {
  // whole column tiles and K steps in fours; enough tokens to fill tiles; 32-bit byte offsets into a plane
  return H % 256 == 0 && H >= 256 && T >= 256 && (long)T * H * 2 < (1L << 32);
}

// The tile grid must be able to fill a good part of the chip: below that the fp32 kernel, which splits K
// over workgroups, is faster (measured: T = 512, H = 2048 -> 32 tiles: 72 us against 53 us).
bool cq_rotate_split_preferred(int T, int H) {
  return cq_rotate_split_supported(T, H) && (long)((T + kTok - 1) / kTok) * (H / kCols) >= 48;
}

extern "C" size_t cq_rotate_quant_split_workspace_bytes(int T, int H) {
  return T > 0 && H > 0 ? cq_rotate_split_workspace_bytes(T, H) : 0;
}

extern "C" cq_status cq_rotate_quant_split(const float* X, const void* R_split, int T, int H, int act_bits,
                                           float* XR_out, int8_t* Q_out, float* scale_out, void* workspace,
                                           size_t workspace_bytes, cq_stream stream) {
  if (!X || !R_split || !XR_out || !Q_out || !scale_out) return CQ_ERR_NULL;
  if (T <= 0 || H <= 0) return CQ_ERR_SHAPE;
  if (!cq_rotate_split_supported(T, H)) return CQ_ERR_SHAPE;
  if (act_bits != 4 && act_bits != 8) return CQ_ERR_UNSUPPORTED;
  if (!workspace || workspace_bytes < cq_rotate_split_workspace_bytes(T, H)) return CQ_ERR_WORKSPACE;
  const cq_status st = cq_rotate_split_launch(X, R_split, T, H, XR_out, workspace, (hipStream_t)stream);
  if (st != CQ_OK) return st;
  return cq_quantize_launch(XR_out, 1, T, H, act_bits, XR_out, Q_out, nullptr, scale_out, nullptr, (hipStream_t)stream);
}

extern "C" size_t cq_rotation_split_bytes(int H) {
  return H > 0 && H % 32 == 0 ? (size_t)H * H * 4 : 0;  // two f16 planes
}

extern "C" cq_status cq_rotation_split(const float* R, int H, void* out, size_t out_bytes, cq_stream stream) {
  if (!R || !out) return CQ_ERR_NULL;
  if (H <= 0 || H % 32 != 0) return CQ_ERR_SHAPE;
  if (out_bytes < cq_rotation_split_bytes(H)) return CQ_ERR_WORKSPACE;
  const size_t frags = (size_t)(H / 32) * (H / 16);
  hipLaunchKernelGGL(split_R_kernel, dim3((unsigned)((frags + 3) / 4)), dim3(256), 0, (hipStream_t)stream, R, H,
                     (uint4*)out);
  return cq_check_launch();
}

size_t cq_rotate_split_workspace_bytes(int T, int H) {
  return cq_align_up((size_t)T * sizeof(float), 256) + 2 * cq_align_up((size_t)T * H * 2, 256);
}

// X_R = X R from the split R; XR_out [T, H] fp32.  workspace: cq_rotate_split_workspace_bytes(T, H).
cq_status cq_rotate_split_launch(const float* X, const void* R_split, int T, int H, float* XR_out, void* workspace,
                                 hipStream_t s) {
  static std::atomic<bool> configured{false};
  const cq_status cst = cq_configure_lds(rot_split_kernel, kRotLdsBytes, configured, true);
  if (cst != CQ_OK) return cst;
  char* ws = (char*)workspace;
  float* row_pow2 = (float*)ws;
  uint16_t* Xh = (uint16_t*)(ws + cq_align_up((size_t)T * sizeof(float), 256));
  uint16_t* Xl = (uint16_t*)((char*)Xh + cq_align_up((size_t)T * H * 2, 256));
  hipLaunchKernelGGL(split_X_kernel, dim3(T), dim3(256), 0, s, X, T, H, Xh, Xl, row_pow2);
  RotArgs a;
  a.Rs = (const uint8_t*)R_split;
  a.Xh = Xh;
  a.Xl = Xl;
  a.row_pow2 = row_pow2;
  a.XR = XR_out;
  a.T = T;
  a.N = H;
  a.K = H;
  a.row_tiles = H / kCols;
  a.n_work = ((T + kTok - 1) / kTok) * a.row_tiles;
  const int per = (a.n_work + 7) / 8;
  hipLaunchKernelGGL(rot_split_kernel, dim3(per * 8), dim3(256), kRotLdsBytes, s, a);
  return cq_check_launch();
}
