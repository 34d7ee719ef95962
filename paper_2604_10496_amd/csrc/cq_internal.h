// Internal declarations shared by the HIP translation units of libcq (gfx950 only).
#ifndef CQ_INTERNAL_H_
#define CQ_INTERNAL_H_

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

#include "cq.h"
#include "cq_measure.h"

#define CQ_WAVE 64

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 cq_v8bf16;
typedef __attribute__((__vector_size__(8 * sizeof(_Float16)))) _Float16 cq_v8f16;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float cq_v16f;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float cq_v4f;
typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t cq_v4u;

static inline cq_status cq_check_launch() {
  return hipGetLastError() == hipSuccess ? CQ_OK : CQ_ERR_HIP;
}

static inline size_t cq_align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Raises a kernel's dynamic-LDS limit before its first launch.  `done` is the launcher's own flag; threads that
// meet in a first call may each set the attribute (the same value: harmless), and none launches before it is set.
// at_zero: the kernel addresses LDS from 0, so it must have no static LDS in front of the dynamic part.
template <typename Kernel>
static inline cq_status cq_configure_lds(Kernel kern, int lds_bytes, std::atomic<bool>& done, bool at_zero) {
  if (done.load(std::memory_order_acquire)) return CQ_OK;
  if (at_zero) {
    hipFuncAttributes fa;
    if (hipFuncGetAttributes(&fa, reinterpret_cast<const void*>(kern)) != hipSuccess) return CQ_ERR_HIP;
    if (fa.sharedSizeBytes != 0) return CQ_ERR_HIP;
  }
  if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                          lds_bytes) != hipSuccess)
    return CQ_ERR_HIP;
  done.store(true, std::memory_order_release);
  return CQ_OK;
}

// centroid tables per weight row: one, or with block-wise tables one per group of group_k weights along K
static inline int cq_tables_per_row(const cq_codebook_weights* W) {
  return (W->group_k > 0 && W->group_k < W->K) ? (W->K + W->group_k - 1) / W->group_k : 1;
}

// ---- internal launchers (arguments already validated) -------------------------------------
// C[T,N] (or partials [ksplit][T][N]) = A[T,K] * B, with B given row-major [K,N] (b_transposed = 0)
// or as its transpose [N,K] (b_transposed = 1); fp32 MFMA, fp32 accumulation.
struct cq_gemm_f32_plan {
  int mb;      // 16-token blocks per wave (1 or 4)
  int ksplit;  // number of K chunks
  int kchunk;  // K values per chunk (a multiple of 16)
};
cq_gemm_f32_plan cq_gemm_f32_make_plan(int T, int N, int K);
cq_status cq_gemm_f32_launch(const float* A, const float* B, int b_transposed, int T, int N, int K,
                             const cq_gemm_f32_plan& plan, float* C_or_partials, uint32_t* zero_me, int zero_n,
                             hipStream_t s);

cq_status cq_quantize_launch(const float* partials, int ksplit, int T, int H, int act_bits,
                             float* XR_out, int8_t* Q_out, uint16_t* Q16_out, float* scale_out,
                             uint32_t* amax_bits, hipStream_t s);
// cq_rotate_quant with an optional second copy of the codes as bf16 bit patterns [T,H]
cq_status cq_rotate_quant_ex(const float* X, const float* R, int T, int H, int act_bits, float* XR_out,
                             int8_t* Q_out, uint16_t* Q16_out, float* scale_out, void* workspace,
                             size_t workspace_bytes, cq_stream stream);

// Decode-sized batches: quantization of the rotated rows (given as K-split partial sums) and the router
// logits in one launch.  Supported sizes also fit the one-workgroup routing kernel that follows.
// topk_ids / topk_w [T, top_k]: NULL, or the launch also selects every token's experts (a4).
bool cq_front_small_supported(int T, int H, int E, int top_k);
cq_status cq_front_small_launch(const float* partials, int ksplit, int T, int H, int act_bits, const float* Wr,
                                const float* bias, int E, float* XR, int8_t* Q, uint16_t* Q16, float* scale,
                                float* logits, int top_k, int32_t* topk_ids, float* topk_w, hipStream_t s);

// X_R = X R on f16 matrix cores from a split copy of R (cq_rotation_split), accurate to about fp32
bool cq_rotate_split_supported(int T, int H);
bool cq_rotate_split_preferred(int T, int H);  // supported, and enough tiles to beat the fp32 kernel
size_t cq_rotate_split_workspace_bytes(int T, int H);
cq_status cq_rotate_split_launch(const float* X, const void* R_split, int T, int H, float* XR_out, void* workspace,
                                 hipStream_t s);

// online-Hadamard variant: h' = h H / sqrt(I) per row, then integer codes (int8 and/or bf16 copies) and scales
bool cq_hadamard_supported(int I);
cq_status cq_hadamard_quant_launch(const float* Hin, int M, int I, int bits, int8_t* Q, uint16_t* Q16, float* scale,
                                   float* HR, hipStream_t s);

// a5 alone (one workgroup) for decode-sized batches whose experts the front launch has selected
bool cq_group_small_supported(int T, int E, int top_k);
cq_status cq_group_small_launch(int32_t* topk_ids, float* topk_w, int T, int E, int top_k, int n_shared,
                                int32_t* expert_offsets, int32_t* perm, int32_t* inv_perm, int32_t* src_token,
                                hipStream_t s);
cq_status cq_topk_launch(const float* logit_partials, int ksplit, const float* bias, int T, int E, int top_k,
                         float* logits_out, int32_t* topk_ids, float* topk_w, hipStream_t s);
size_t cq_permute_workspace_bytes(int T, int E, int top_k);
cq_status cq_permute_launch(const int32_t* topk_ids, int T, int E, int top_k, int n_shared,
                            int32_t* expert_offsets, int32_t* perm, int32_t* inv_perm, int32_t* src_token,
                            void* workspace, hipStream_t s);

// ksplit_left: NULL, or receives the number of K splits whose partial sums [ksplit][M_total][N] (fp32,
// at the start of `workspace`) the caller must add itself; 1 means `out` is final.  With NULL the
// launcher always finishes `out`.
// route: NULL, or the grouping by expert (a5) is folded into this launch (cq_gemm_can_fuse_route): every
// workgroup derives its group's rows from the selected expert ids, row_gather and group_offsets are not
// read, rows gather by token, and the launch leaves offsets / perm / inv_perm / src_token behind for the
// launches that follow.
struct cq_route_fuse {
  const int32_t* ids;                               // [T, top_k] selected experts (a4)
  int T, E, S, top_k;
  int32_t *offsets, *perm, *inv_perm, *src_token;   // written as cq_route_permute writes them
};
bool cq_gemm_can_fuse_route(const cq_codebook_weights* W, int T, int E, int S, int top_k, int epilogue);
cq_status cq_gemm_codebook_launch(const cq_codebook_weights* W, const void* A, int a_kind,
                                  const float* row_scale, const int32_t* row_gather,
                                  const int32_t* group_offsets, int M_total, int epilogue,
                                  void* out, int out_kind, void* workspace, hipStream_t s, int* ksplit_left,
                                  const cq_route_fuse* route = nullptr, int max_group_rows = 0);
// max_group_rows (here and below): an upper bound on the rows of any one group if the caller has one (the
// layer: a group has at most one row per token), else 0 = M_total.
size_t cq_gemm_partials_bytes(const cq_codebook_weights* W, int M_total, int epilogue, int max_group_rows = 0);
// K split of a product: ksplit ranges of ksteps K steps (of 64) each; 1 and K/64 when K is not split
void cq_gemm_split_plan(const cq_codebook_weights* W, int M_total, int epilogue, int* ksplit, int* ksteps,
                        int max_group_rows = 0);
// block-wise tables of 1024 weights on the streaming kernel (groups of at most 16 rows, K ranges of whole tables)
bool cq_gemm_blockwise_streams(const cq_codebook_weights* W, int M_total, int epilogue, int max_group_rows = 0);
// W2 weights streamed as stored (index_bits = 2): quadruple tables in LDS, decode-sized groups
static inline bool cq_is_w2(const cq_codebook_weights* W) { return W->index_bits == 2; }
int cq_gemm_w2_range_steps(int K);   // K steps (of 128) per K range, 0 if K cannot be split that way
bool cq_gemm_w2_supported(const cq_codebook_weights* W, int a_kind, int epilogue);
size_t cq_gemm_w2_partials_bytes(const cq_codebook_weights* W, int M_total);
cq_status cq_gemm_w2_launch(const cq_codebook_weights* W, const void* A, int a_kind, const float* row_scale,
                            const int32_t* row_gather, const int32_t* group_offsets, int M_total, int epilogue,
                            void* out, int out_kind, void* workspace, hipStream_t s, int* ksplit_left,
                            const cq_route_fuse* route = nullptr);
// weighted combine over `slices` partial copies of O that are `slice_stride` floats apart
cq_status cq_combine_launch(const float* O, int slices, size_t slice_stride, const float* topk_w,
                            const int32_t* inv_perm, int T, int H, int top_k, int n_shared, float* Y, hipStream_t s);

// large-tile (prefill) path of the codebook product
bool cq_gemm_large_supported(const cq_codebook_weights* W);
// whether a product over M_total rows launches it (more rows than the streaming kernel takes per group, or
// block-wise tables, which only the large-tile kernel decodes)
bool cq_gemm_uses_large_tiles(const cq_codebook_weights* W, int M_total, int epilogue = CQ_EPI_NONE,
                              int max_group_rows = 0);
// with_conversion: include room for a 16-bit copy of the activation rows (needed for CQ_A_INT8_CODES
// and CQ_A_F32 operands; bf16 / f16 operands are read in place)
size_t cq_gemm_large_workspace_bytes(int G, int M_total, int K, bool with_conversion, int tail_N = 0);
// narrow tiles of a plain fp32 product with a long K are cut into K parts (their partial sums live in the workspace)
bool cq_gemm_large_tail_split(const cq_codebook_weights* W, int epilogue, int out_kind);
// work lists of a launch that uses both kernels (device-built: group sizes are device data); small_hdr:
// {number of small groups, 64-row units per workgroup, workgroups per small group}, small_ids: their ids
cq_status cq_gemm_build_lists(const cq_codebook_weights* W, const int32_t* group_offsets, int M_total, int small_max,
                              int small_wgs, void* workspace, const int32_t** small_hdr, const int32_t** small_ids,
                              hipStream_t s, bool tail_split = false);
cq_status cq_gemm_large_launch(const cq_codebook_weights* W, const void* A, int a_kind, const float* row_scale,
                               const int32_t* row_gather, const int32_t* group_offsets, int M_total, int small_max,
                               int epilogue, void* out, int out_kind, void* workspace, hipStream_t s);

#endif  // CQ_INTERNAL_H_
