// The whole layer a1..a8 on one stream: rotate + quantize, route + permute, gate/up codebook product
// with the SiLU-gated epilogue, down codebook product, weighted combine.  Host code only enqueues.
#include <atomic>

#include "cq_internal.h"

namespace {

// Workspace of cq_moe_forward_static: one array per GPU in the library's own device memory, so that the
// call needs no allocation by anybody.  In host code the array's name is only a handle for
// hipGetSymbolAddress; kernels and launchers get the address that call returns for the current device.
static __device__ __align__(256) unsigned char scratch[CQ_STATIC_SCRATCH_BYTES];
constexpr int kMaxDevices = 64;
std::atomic<void*> g_scratch_ptr[kMaxDevices];

// device address of `scratch` on the current device (looked up once per device, then cached)
cq_status static_scratch(void** out) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return CQ_ERR_HIP;
  void* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (!p) {
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return CQ_ERR_HIP;
    g_scratch_ptr[dev].store(p, std::memory_order_release);  // racing threads store the same address
  }
  *out = p;
  return CQ_OK;
}

cq_status validate_layer(const cq_layer* L, int T) {
  if (!L) return CQ_ERR_NULL;
  if ((!L->R && !L->r_hadamard) || !L->Wr || !L->gate_up.cent || !L->down.cent) return CQ_ERR_NULL;
  if ((!L->gate_up.idx && !L->gate_up.prepacked) || (!L->down.idx && !L->down.prepacked)) return CQ_ERR_NULL;
  if (T <= 0 || L->H <= 0 || L->I <= 0 || L->E <= 0 || L->top_k <= 0 || L->S < 0) return CQ_ERR_SHAPE;
  if (L->H % 64 != 0 || L->I % 64 != 0 || L->top_k > L->E || L->top_k > 64 || L->E > 1024) return CQ_ERR_SHAPE;
  if ((long)T * (L->top_k + L->S) > 0x7fffffffL) return CQ_ERR_SHAPE;
  if (L->act_bits != 4 && L->act_bits != 8) return CQ_ERR_UNSUPPORTED;
  if (L->h_bits != 0 && L->h_bits != 4 && L->h_bits != 8) return CQ_ERR_UNSUPPORTED;
  if (L->h_bits != 0 && !cq_hadamard_supported(L->I)) return CQ_ERR_SHAPE;
  if (L->r_hadamard && !cq_hadamard_supported(L->H)) return CQ_ERR_SHAPE;
  const int G = L->E + L->S;
  if (L->gate_up.G != G || L->gate_up.N != 2 * L->I || L->gate_up.K != L->H) return CQ_ERR_SHAPE;
  if (L->down.G != G || L->down.N != L->H || L->down.K != L->I) return CQ_ERR_SHAPE;
  if (L->gate_up.group_k < 0 || L->down.group_k < 0) return CQ_ERR_SHAPE;
  for (const cq_codebook_weights* W : {&L->gate_up, &L->down})
    if (W->index_bits != 0 && W->index_bits != 4 && W->index_bits != 2) return CQ_ERR_UNSUPPORTED;
  // W2 weights streamed as stored: int8 codes into the SiLU-gated gate/up product, f16 (or, in the online-Hadamard
  // variant, int8 codes) into the plain down product
  if (cq_is_w2(&L->gate_up) && !cq_gemm_w2_supported(&L->gate_up, CQ_A_INT8_CODES, CQ_EPI_SWIGLU)) return CQ_ERR_UNSUPPORTED;
  if (cq_is_w2(&L->down) && !cq_gemm_w2_supported(&L->down, L->h_bits ? CQ_A_INT8_CODES : CQ_A_F16, CQ_EPI_NONE))
    return CQ_ERR_UNSUPPORTED;
  if ((cq_tables_per_row(&L->gate_up) > 1 && !cq_gemm_large_supported(&L->gate_up)) ||
      (cq_tables_per_row(&L->down) > 1 && !cq_gemm_large_supported(&L->down)))
    return CQ_ERR_UNSUPPORTED;
  return CQ_OK;
}

// Many tokens and a split copy of R at hand: the rotation runs on the f16 matrix cores.
bool use_split_rotation(const cq_layer* L, int T) { return L->R_split && cq_rotate_split_preferred(T, L->H); }

// Batches large enough for the large-tile product get the codes a second time as bf16, so that staging
// them into LDS is a plain copy.
bool use_bf16_codes(const cq_layer* L, int T) {
  return cq_gemm_uses_large_tiles(&L->gate_up, (int)((long)T * (L->top_k + L->S)), CQ_EPI_SWIGLU, T);
}

void make_layout(const cq_layer* L, int T, cq_moe_layout* o) {
  const size_t M = (size_t)T * (L->top_k + L->S), A = (size_t)T * L->top_k;
  size_t off = 0;
  auto take = [&](size_t bytes) {
    const size_t at = off;
    off += cq_align_up(bytes, 256);
    return at;
  };
  o->XR = take((size_t)T * L->H * 4);
  o->Q = take((size_t)T * L->H);
  o->Q16 = take(use_bf16_codes(L, T) ? (size_t)T * L->H * 2 : 0);
  o->scale = take((size_t)T * 4);
  o->logits = take((size_t)T * L->E * 4);
  o->topk_ids = take(A * 4);
  o->topk_w = take(A * 4);
  o->offsets = take((size_t)(L->E + L->S + 1) * 4);
  o->perm = take(A * 4);
  o->inv_perm = take(A * 4);
  o->src_token = take(M * 4);
  o->Hbuf = take(M * L->I * (L->h_bits ? 4 : 2));  // f16, or fp32 when it is rotated and quantized next
  o->Obuf = take(M * L->H * 4);
  const bool hq16 = L->h_bits && cq_gemm_uses_large_tiles(&L->down, (int)M, CQ_EPI_NONE, T);
  o->HQ = take(L->h_bits ? M * L->I : 0);
  o->HQ16 = take(hq16 ? M * L->I * 2 : 0);
  o->hscale = take(L->h_bits ? M * 4 : 0);
  size_t scratch = cq_rotate_quant_workspace_bytes(T, L->H);
  const size_t r = cq_route_permute_workspace_bytes(T, L->H, L->E, L->top_k);
  if (r > scratch) scratch = r;
  if (use_split_rotation(L, T)) {
    const size_t x = cq_rotate_split_workspace_bytes(T, L->H);
    if (x > scratch) scratch = x;
  }
  // the layer feeds both products 16-bit operands (bf16 codes, f16 h): tile lists only
  if (use_bf16_codes(L, T)) {
    const size_t g1 = cq_gemm_large_workspace_bytes(L->gate_up.G, (int)M, L->gate_up.K, false);
    if (g1 > scratch) scratch = g1;
  }
  {
    size_t g2 = cq_gemm_partials_bytes(&L->down, (int)M, CQ_EPI_NONE, T);   // (a group has at most T rows)
    if (cq_gemm_uses_large_tiles(&L->down, (int)M, CQ_EPI_NONE, T))  // (16-bit operands in either variant: f16 h or bf16 codes)
      g2 += cq_gemm_large_workspace_bytes(L->down.G, (int)M, L->down.K, false, L->down.N);
    if (g2 > scratch) scratch = g2;
  }
  o->scratch = take(scratch);
  o->total = off;
}

}  // namespace

extern "C" size_t cq_moe_workspace_bytes(const cq_layer* L, int T) {
  if (validate_layer(L, T) != CQ_OK) return 0;
  cq_moe_layout lay;
  make_layout(L, T, &lay);
  return lay.total;
}

extern "C" cq_status cq_moe_workspace_layout(const cq_layer* L, int T, cq_moe_layout* out) {
  if (!out) return CQ_ERR_NULL;
  const cq_status st = validate_layer(L, T);
  if (st != CQ_OK) return st;
  make_layout(L, T, out);
  return CQ_OK;
}

namespace {

// ev: NULL, or CQ_N_STAGES + 1 events recorded at the stage boundaries.
cq_status run_layer(const cq_layer* L, const float* X, int T, float* Y, void* workspace, size_t workspace_bytes,
                    cq_stream stream, hipEvent_t* ev) {
  cq_status st = validate_layer(L, T);
  if (st != CQ_OK) return st;
  if (!X || !Y) return CQ_ERR_NULL;
  cq_moe_layout lay;
  make_layout(L, T, &lay);
  if (!workspace || workspace_bytes < lay.total) return CQ_ERR_WORKSPACE;
  char* ws = (char*)workspace;
  float* XR = (float*)(ws + lay.XR);
  int8_t* Q = (int8_t*)(ws + lay.Q);
  float* scale = (float*)(ws + lay.scale);
  float* logits = (float*)(ws + lay.logits);
  int32_t* ids = (int32_t*)(ws + lay.topk_ids);
  float* tw = (float*)(ws + lay.topk_w);
  int32_t* offsets = (int32_t*)(ws + lay.offsets);
  int32_t* perm = (int32_t*)(ws + lay.perm);
  int32_t* inv_perm = (int32_t*)(ws + lay.inv_perm);
  int32_t* src_token = (int32_t*)(ws + lay.src_token);
  void* Hbuf = ws + lay.Hbuf;
  float* Obuf = (float*)(ws + lay.Obuf);
  void* scratch = ws + lay.scratch;
  const size_t scratch_bytes = lay.total - lay.scratch;
  const int M = T * (L->top_k + L->S);
  hipStream_t hs = (hipStream_t)stream;
  auto mark = [&](int i) -> bool { return !ev || hipEventRecord(ev[i], hs) == hipSuccess; };

  if (!mark(0)) return CQ_ERR_HIP;
  const bool bf16_codes = use_bf16_codes(L, T);
  bool fuse_route = false;   // a5 folded into the gate/up launch (decode-sized batches)
  uint16_t* Q16 = bf16_codes ? (uint16_t*)(ws + lay.Q16) : nullptr;
  if (L->r_hadamard) {
    // the rotation is a Hadamard matrix: transform and quantization in one launch, no matrix is read
    st = cq_hadamard_quant_launch(X, T, L->H, L->act_bits, Q, Q16, scale, XR, hs);
    if (st != CQ_OK) return st;
    if (!mark(1)) return CQ_ERR_HIP;
    st = cq_route_permute(XR, L->Wr, L->bias, nullptr, T, L->H, L->E, L->top_k, L->S, logits, ids, tw, offsets, perm,
                          inv_perm, src_token, scratch, scratch_bytes, stream);
    if (st != CQ_OK) return st;
    if (!mark(2)) return CQ_ERR_HIP;
  } else if (cq_front_small_supported(T, L->H, L->E, L->top_k)) {
    // decode-sized batch: the rotation; one launch for quantization and logits; one for top-k and grouping
    // (the second stage boundary therefore falls between the rotation and everything else)
    const cq_gemm_f32_plan p = cq_gemm_f32_make_plan(T, L->H, L->H);
    float* part = p.ksplit > 1 ? (float*)scratch : XR;
    st = cq_gemm_f32_launch(X, L->R, 0, T, L->H, L->H, p, part, nullptr, 0, hs);
    if (st != CQ_OK) return st;
    if (!mark(1)) return CQ_ERR_HIP;
    // when the gate/up launch can do the grouping itself, the front launch also selects the experts and
    // the routing launch falls away
    fuse_route = cq_gemm_can_fuse_route(&L->gate_up, T, L->E, L->S, L->top_k, CQ_EPI_SWIGLU);
    // (the front launch selects the experts whenever a launch that only groups can follow it)
    const bool front_topk = fuse_route || cq_group_small_supported(T, L->E, L->top_k);
    st = cq_front_small_launch(part, p.ksplit, T, L->H, L->act_bits, L->Wr, L->bias, L->E, XR, Q, Q16, scale, logits,
                               L->top_k, front_topk ? ids : nullptr, front_topk ? tw : nullptr, hs);
    if (st != CQ_OK) return st;
    if (!fuse_route) {
      st = front_topk ? cq_group_small_launch(ids, tw, T, L->E, L->top_k, L->S, offsets, perm, inv_perm, src_token, hs)
                      : cq_route_permute(nullptr, nullptr, nullptr, logits, T, L->H, L->E, L->top_k, L->S, logits, ids,
                                         tw, offsets, perm, inv_perm, src_token, scratch, scratch_bytes, stream);
      if (st != CQ_OK) return st;
    }
    if (!mark(2)) return CQ_ERR_HIP;
  } else {
    if (use_split_rotation(L, T)) {
      st = cq_rotate_split_launch(X, L->R_split, T, L->H, XR, scratch, hs);
      if (st != CQ_OK) return st;
      st = cq_quantize_launch(XR, 1, T, L->H, L->act_bits, XR, Q, Q16, scale, nullptr, hs);
    } else {
      st = cq_rotate_quant_ex(X, L->R, T, L->H, L->act_bits, XR, Q, Q16, scale, scratch, scratch_bytes, stream);
    }
    if (st != CQ_OK) return st;
    if (!mark(1)) return CQ_ERR_HIP;
    st = cq_route_permute(XR, L->Wr, L->bias, nullptr, T, L->H, L->E, L->top_k, L->S, logits, ids, tw, offsets, perm,
                          inv_perm, src_token, scratch, scratch_bytes, stream);
    if (st != CQ_OK) return st;
    if (!mark(2)) return CQ_ERR_HIP;
  }
  // (internal launcher: the layer was validated above and the scratch area is sized for 16-bit operands)
  const cq_route_fuse route = {ids, T, L->E, L->S, L->top_k, offsets, perm, inv_perm, src_token};
  st = cq_gemm_codebook_launch(&L->gate_up, bf16_codes ? (const void*)Q16 : (const void*)Q,
                               bf16_codes ? CQ_A_BF16 : CQ_A_INT8_CODES, scale, src_token, offsets, M, CQ_EPI_SWIGLU,
                               Hbuf, L->h_bits ? CQ_OUT_F32 : CQ_OUT_F16, scratch, hs, nullptr,
                               fuse_route ? &route : nullptr, T);
  if (st != CQ_OK) return st;
  if (!mark(3)) return CQ_ERR_HIP;
  int down_splits = 1;  // > 1: the down projection left K-split partial sums in the scratch area
  if (L->h_bits) {
    // online-Hadamard variant: rotate and quantize the intermediate (counted in the down stage), then the
    // down projection reads integer codes and per-row scales like the gate/up projection does
    int8_t* HQ = (int8_t*)(ws + lay.HQ);
    float* hscale = (float*)(ws + lay.hscale);
    const bool hq16 = cq_gemm_uses_large_tiles(&L->down, (int)M, CQ_EPI_NONE, T);
    uint16_t* HQ16 = hq16 ? (uint16_t*)(ws + lay.HQ16) : nullptr;
    st = cq_hadamard_quant_launch((const float*)Hbuf, M, L->I, L->h_bits, HQ, HQ16, hscale, nullptr, hs);
    if (st != CQ_OK) return st;
    st = cq_gemm_codebook_launch(&L->down, hq16 ? (const void*)HQ16 : (const void*)HQ,
                                 hq16 ? CQ_A_BF16 : CQ_A_INT8_CODES, hscale, nullptr, offsets, M, CQ_EPI_NONE, Obuf,
                                 CQ_OUT_F32, scratch, hs, &down_splits, nullptr, T);
  } else {
    st = cq_gemm_codebook_launch(&L->down, Hbuf, CQ_A_F16, nullptr, nullptr, offsets, M, CQ_EPI_NONE, Obuf, CQ_OUT_F32,
                                 scratch, hs, &down_splits, nullptr, T);
  }
  if (st != CQ_OK) return st;
  if (!mark(4)) return CQ_ERR_HIP;
  st = down_splits > 1 ? cq_combine_launch((const float*)scratch, down_splits, (size_t)M * L->H, tw, inv_perm, T,
                                           L->H, L->top_k, L->S, Y, hs)
                       : cq_combine_launch(Obuf, 1, 0, tw, inv_perm, T, L->H, L->top_k, L->S, Y, hs);
  if (st != CQ_OK) return st;
  if (!mark(5)) return CQ_ERR_HIP;
  return CQ_OK;
}

}  // namespace

extern "C" cq_status cq_moe_forward(const cq_layer* L, const float* X, int T, float* Y, void* workspace,
                                    size_t workspace_bytes, cq_stream stream) {
  return run_layer(L, X, T, Y, workspace, workspace_bytes, stream, nullptr);
}

extern "C" cq_status cq_moe_forward_static(const cq_layer* L, const float* X, int T, float* Y, cq_stream stream) {
  cq_status st = validate_layer(L, T);
  if (st != CQ_OK) return st;
  if (!X || !Y) return CQ_ERR_NULL;
  cq_moe_layout lay;
  make_layout(L, T, &lay);
  if (lay.total > (size_t)CQ_STATIC_SCRATCH_BYTES) return CQ_ERR_WORKSPACE;  // batch too large for the array
  void* ws = nullptr;
  st = static_scratch(&ws);
  if (st != CQ_OK) return st;
  return run_layer(L, X, T, Y, ws, (size_t)CQ_STATIC_SCRATCH_BYTES, stream, nullptr);
}

extern "C" cq_status cq_moe_forward_timed(const cq_layer* L, const float* X, int T, float* Y, void* workspace,
                                          size_t workspace_bytes, cq_stream stream, float* stage_ms) {
  if (!stage_ms) return CQ_ERR_NULL;
  hipEvent_t ev[CQ_N_STAGES + 1];
  int made = 0;
  cq_status st = CQ_OK;
  for (; made <= CQ_N_STAGES; ++made)
    if (hipEventCreate(&ev[made]) != hipSuccess) { st = CQ_ERR_HIP; break; }
  if (st == CQ_OK) st = run_layer(L, X, T, Y, workspace, workspace_bytes, stream, ev);
  if (st == CQ_OK && hipEventSynchronize(ev[CQ_N_STAGES]) != hipSuccess) st = CQ_ERR_HIP;
  if (st == CQ_OK)
    for (int i = 0; i < CQ_N_STAGES; ++i)
      if (hipEventElapsedTime(&stage_ms[i], ev[i], ev[i + 1]) != hipSuccess) st = CQ_ERR_HIP;
  for (int i = 0; i < made; ++i) (void)hipEventDestroy(ev[i]);
  return st;
}
