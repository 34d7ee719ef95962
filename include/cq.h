/*
 * cq.h -- C ABI of the MI355X (gfx950) library for the forward pass of a low-precision
 * Mixture-of-Experts expert layer in the CodeQuant deployment format.
 *
 * The layer (paper: Methodology, "Activation-Oriented Outlier Smoothing", "Adaptive Weight
 * Clustering and Centroid Finetuning", "CodeQuant Kernel and System Implementation"):
 *   X_R = X R                      rotation by the orthogonal matrix R         (AOS section)
 *   q, s = Q(X_R)                  integer quantization, symmetric per token    (AOS objective)
 *   Pi   = top-k of X_R Wr^T       the router is a linear layer                 (AOS section)
 *   X_t  = tokens of each expert   grouping by expert                           (AOS section)
 *   W_c[i,j] = sum_k C[i,k] A[i,j,k]   weights exist only as a 4-bit index per weight into a
 *                                  16-entry centroid table per output row       (Eq. W_c)
 *   o    = (SiLU(a Wg_c^T) . a Wu_c^T) Wd_c^T,  a = s q                          (invariance eq.)
 *   Y    = sum_j Pi_j o_j + shared experts                                      (MoE case of Eq. L)
 *
 * Conventions for every entry point
 *   - All data pointers are DEVICE pointers owned by the caller; the library neither allocates
 *     nor frees device memory inside these calls and never synchronises the host.
 *   - Work is enqueued on `stream` (a hipStream_t passed as void*; NULL = the null stream).
 *   - Buffers must be 16-byte aligned.  Matrices are row-major.
 *   - Arguments are validated BEFORE any HIP call; on a bad argument nothing is launched.
 *   - Return value: CQ_OK or one of the error codes below; cq_status_string() names them.
 *   - Weight matrices are in [out, in] layout: row n holds the K input weights of output n.
 */
#ifndef CQ_H_
#define CQ_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int cq_status;
enum {
  CQ_OK = 0,
  CQ_ERR_NULL = 1,        /* a required pointer is NULL                                   */
  CQ_ERR_SHAPE = 2,       /* non-positive size, top_k > E, H or I not a multiple of 64 ... */
  CQ_ERR_UNSUPPORTED = 3, /* act_bits not in {4,8}, unknown enum value                     */
  CQ_ERR_WORKSPACE = 4,   /* workspace NULL or smaller than the *_workspace_bytes() figure */
  CQ_ERR_HIP = 5          /* a HIP runtime call failed (launch error, no device)           */
};

typedef void* cq_stream; /* hipStream_t */

#define CQ_N_CENTROIDS 16

/* kinds of the activation operand of cq_codebook_grouped_gemm */
enum { CQ_A_INT8_CODES = 0, /* int8 container holding integer codes (|q| <= 127)          */
       CQ_A_F16 = 1,        /* IEEE half                                                    */
       CQ_A_F32 = 2,        /* float; rounded to half (RNE, saturating) when staged         */
       CQ_A_BF16 = 3 };     /* bfloat16 bit patterns (e.g. integer codes stored as bf16)    */
/* epilogues */
enum { CQ_EPI_NONE = 0,     /* out[m, n] = scale[m] * sum_k W_c[n,k] a[m,k]                 */
       CQ_EPI_SWIGLU = 1 }; /* N = 2I rows interleaved (2i = gate i, 2i+1 = up i):
                               out[m, i] = SiLU(g) * u                                      */
/* kinds of the output */
enum { CQ_OUT_F32 = 0, CQ_OUT_F16 = 1 };

/*
 * A group (expert) array of clustered weight matrices (Eq. W_c; 16 centroids, paper's W4 budget).
 *   idx       [G, N, K/2] bytes, canonical: byte j of a row = index of weight 2j in bits 0-3 and
 *             of weight 2j+1 in bits 4-7.  May be NULL if `prepacked` is given.
 *   cent      [G, N, 16] bf16 bit patterns: row n's centroid table.
 *   prepacked optional kernel-native copy of idx written by cq_prepack() (same byte count):
 *             rows are taken 32 at a time and K 64 weights at a time; the 1 KiB tile of row block
 *             rb and K step s is at ((rb*(K/64) + s) * 1024) and holds, for l = 0..63, the 16
 *             canonical bytes of row rb*32 + l%32, byte columns s*32 + (l/32)*16 .. +15, at l*16, with
 *             the nibbles of every 4 bytes (8 weights w0..w7) regrouped: byte i of the four holds w_i in
 *             bits 0-3 and w_{i+4} in bits 4-7.
 *   K must be a multiple of 64 and N a multiple of 64.
 *   group_k   0 (or >= K): one table per row over all of K ("Embedding-wise", experimental setup).
 *             g > 0: "Block-wise" tables, one per group of g consecutive weights of a row; cent is then
 *             [G, N, ceil(K/g), 16] and weight k of a row is decoded through table k / g (the last group
 *             is shorter when g does not divide K).  g must be a multiple of 512 and N of 256
 *             (other values: CQ_ERR_UNSUPPORTED).  Which kernel runs is the library's choice (prefill-sized
 *             groups: large token tiles; g = 1024 with at most 16 rows per group and K a multiple of 2048:
 *             the streaming kernel); the results do not depend on it beyond fp32 summation order.
 *   index_bits 0 or 4: the format above.  2: the smallest budget of the ablation on centroid budgets (W2, four
 *             centroids per row) streamed as stored, at half the bytes: idx is [G, N, K/4] bytes, the indices
 *             of a row as one little-endian bit stream (weight j in bits 2(j%4), 2(j%4)+1 of byte j/4), cent is
 *             [G, N, 4] bf16.  Prepacked copy (cq_prepack; same byte count): rows 32 at a time, K 128 weights
 *             at a time; the 1 KiB tile of row block rb and K step s is at ((rb*(K/128) + s) * 1024) and holds,
 *             for l = 0..63, the 16 canonical bytes of row rb*32 + l%32, byte columns s*32 + (l/32)*16 .. +15,
 *             at l*16, unchanged.  Taken by cq_codebook_grouped_gemm and cq_moe_forward for group_k = 0, K a
 *             multiple of 4096 or of 7168 (with the SiLU-gated epilogue: K = 4096 or 7168) and int8-code, f16
 *             or bf16 operands; anything else returns CQ_ERR_UNSUPPORTED (expand such weights once with
 *             cq_expand_centroid_budget).  Meant for decode-sized groups: groups of more than 8 rows are
 *             processed 8 rows at a time, re-reading the indices.
 */
typedef struct {
  const uint8_t* idx;
  const uint16_t* cent;
  const void* prepacked;
  int G, N, K;
  int group_k;
  int index_bits;
} cq_codebook_weights;

/* One MoE expert layer.  Groups 0..E-1 are routed experts, E..E+S-1 always-on shared experts. */
typedef struct {
  int H, I, E, top_k, S, act_bits;
  const float* R;     /* [H, H] orthogonal, X_R = X R                                   */
  const float* Wr;    /* [E, H] router weight in the rotated basis                      */
  const float* bias;  /* [E] or NULL                                                    */
  cq_codebook_weights gate_up; /* G = E+S, N = 2I (gate/up interleaved), K = H          */
  cq_codebook_weights down;    /* G = E+S, N = H, K = I                                 */
  const void* R_split; /* optional: copy of R written by cq_rotation_split(); NULL if absent */
  int h_bits;          /* 0, or 4 / 8: online-Hadamard variant -- the intermediate h is multiplied by
                          H_I / sqrt(I) and quantized per row to h_bits before the down projection,
                          whose weights are then clustered in that rotated basis (cq_hadamard_quant) */
  int r_hadamard;      /* non-zero: the rotation is R = H_H / sqrt(H) (same matrices as cq_hadamard_quant) and a1
                          runs as a fast transform; R is then not read and may be NULL                       */
} cq_layer;

const char* cq_status_string(cq_status st);

/*
 * a1 + a2: X_R = X R (AOS section) and per-token symmetric integer quantization Q(X_R).
 *   X [T,H] f32, R [H,H] f32  ->  XR_out [T,H] f32 (the router reads it), Q_out [T,H] int8
 *   codes in [-qmax, qmax] with qmax = 2^(act_bits-1)-1, scale_out [T] f32 = max|X_R[t,:]|/qmax
 *   (1 for an all-zero row).  Rounding is to nearest, ties to even.  The product is accumulated
 *   in fp32 on fp32 matrix cores so that codes differ from an exact evaluation only at ties.
 *   H % 64 == 0.  workspace: cq_rotate_quant_workspace_bytes(T, H) bytes.
 */
size_t cq_rotate_quant_workspace_bytes(int T, int H);
cq_status cq_rotate_quant(const float* X, const float* R, int T, int H, int act_bits,
                          float* XR_out, int8_t* Q_out, float* scale_out,
                          void* workspace, size_t workspace_bytes, cq_stream stream);

/*
 * a1 for many tokens: a copy of R (AOS section) as two f16 planes, R = Rh + 2^-11 Rl, in the order the
 * matrix-core fragments are loaded in.  With it cq_moe_forward computes X R (for T >= 256, H % 256 == 0)
 * as Xh Rh + 2^-11 (Xh Rl + Xl Rh) on the f16 matrix cores with fp32 accumulation: every operand is
 * represented to 2^-23 of its size and only the 2^-22 Xl Rl term is dropped, so the result is as accurate
 * as the fp32 product and the codes still differ from an exact evaluation only at rounding ties.
 *   R [H,H] f32 device, H % 32 == 0; out: cq_rotation_split_bytes(H) bytes of device memory, owned by
 *   the caller, read by every later cq_moe_forward on a layer whose R_split points to it.
 */
size_t cq_rotation_split_bytes(int H);
cq_status cq_rotation_split(const float* R, int H, void* out, size_t out_bytes, cq_stream stream);
/*
 * cq_rotate_quant on that copy (the path cq_moe_forward takes when the batch fills enough 128-token x
 * 256-column tiles): same outputs, same accuracy statement.  T >= 256, H % 256 == 0, T*H < 2^31;
 * other sizes return CQ_ERR_SHAPE.  workspace: cq_rotate_quant_split_workspace_bytes(T, H) bytes.
 */
size_t cq_rotate_quant_split_workspace_bytes(int T, int H);
cq_status cq_rotate_quant_split(const float* X, const void* R_split, int T, int H, int act_bits,
                                float* XR_out, int8_t* Q_out, float* scale_out,
                                void* workspace, size_t workspace_bytes, cq_stream stream);

/*
 * a3 + a4 + a5: router logits L = X_R Wr^T (+bias) in fp32, top-k by descending logit (equal
 * logits -> lower expert id), weights = softmax over the k selected logits, and the stable
 * grouping of assignments a = t*k + j by expert ("tokens assigned to that expert", AOS section).
 *   XR [T,H] or NULL; if NULL, logits_in [T,E] is used as the logits (bias is then ignored).
 *   Outputs: logits_out [T,E] or NULL; topk_ids [T,k] i32; topk_w [T,k] f32;
 *   expert_offsets [E+S+1] i32; perm [T*k] (sorted position -> a); inv_perm [T*k] (a -> position);
 *   src_token [T*(k+S)] or NULL: token whose activations feed each sorted row.
 *   n_shared = S appends S always-on groups E..E+S-1, each holding all T tokens in order
 *   (rows T*k + s*T + t); they are not part of the softmax.
 *   1 <= top_k <= min(E, 64), E <= 1024, H % 64 == 0.
 *   workspace: cq_route_permute_workspace_bytes(T, H, E, top_k) bytes.
 */
size_t cq_route_permute_workspace_bytes(int T, int H, int E, int top_k);
cq_status cq_route_permute(const float* XR, const float* Wr, const float* bias, const float* logits_in,
                           int T, int H, int E, int top_k, int n_shared,
                           float* logits_out, int32_t* topk_ids, float* topk_w,
                           int32_t* expert_offsets, int32_t* perm, int32_t* inv_perm, int32_t* src_token,
                           void* workspace, size_t workspace_bytes, cq_stream stream);

/*
 * a6 / a7: grouped product with clustered weights (Eq. W_c): for every group g and every sorted
 * row m in [group_offsets[g], group_offsets[g+1]):
 *     acc[m, n] = sum_k W_c^{(g)}[n, k] * A[src(m), k],  src(m) = row_gather ? row_gather[m] : m
 *     out[m, n] = (row_scale ? row_scale[src(m)] : 1) * acc[m, n]          (CQ_EPI_NONE, N outputs)
 *     out[m, i] = SiLU(sc*acc[m,2i]) * (sc*acc[m,2i+1])                    (CQ_EPI_SWIGLU, N/2 outputs)
 *   Weights are never materialised: packed indices stream from HBM, are turned into centroid
 *   values through a table staged in LDS (groups of up to 32 rows) or held in registers (larger
 *   groups, and all groups when the tables are block-wise), and feed the matrix cores directly.  Integer codes and
 *   bf16 centroids are exact operands (bf16 MFMA, fp32 accumulation); CQ_A_F16 / CQ_A_F32 rows
 *   use f16 MFMA with centroids converted bf16 -> f16.
 *   A: [rows, K] of a_kind.  out: [M_total, N or N/2] of out_kind (CQ_OUT_F16 saturates).
 *   group_offsets [G+1] device i32, non-decreasing, group_offsets[G] <= M_total.  Empty groups ok.
 *   workspace: cq_grouped_gemm_workspace_bytes(W, M_total) bytes (may be 0 -> NULL allowed).
 */
size_t cq_grouped_gemm_workspace_bytes(const cq_codebook_weights* W, int M_total);
cq_status cq_codebook_grouped_gemm(const cq_codebook_weights* W,
                                   const void* A, int a_kind,
                                   const float* row_scale, const int32_t* row_gather,
                                   const int32_t* group_offsets, int M_total,
                                   int epilogue, void* out, int out_kind,
                                   void* workspace, size_t workspace_bytes, cq_stream stream);

/*
 * Smaller centroid budgets (ablation on centroid budgets: W2 = 4 centroids, W3 = 8): conversion of such
 * weights into the 16-entry format above, once, at load time.
 *   idx_bits  [G, N, K*bits/8] bytes: the indices of a row as one little-endian bit stream, weight j at bits
 *             [j*bits, (j+1)*bits) (bit i of the stream = bit i%8 of byte i/8);  bits in {2, 3}
 *   cent_bits [G, N, tables_per_row, 2^bits] bf16 (tables_per_row = 1, or ceil(K/group_k) for block-wise tables)
 *   idx4_out  [G, N, K/2] canonical 4-bit bytes;  cent16_out [G, N, tables_per_row, 16]: entries >= 2^bits,
 *             which no index addresses, repeat the table's last entry.
 * The products then run on the 4-bit kernels: the results are those of the smaller budget exactly, the bytes
 * streamed per weight are those of W4.  (W2 weights can also be streamed as stored: cq_codebook_weights.index_bits.)
 */
cq_status cq_expand_centroid_budget(const uint8_t* idx_bits, const uint16_t* cent_bits, int bits, int G, int N, int K,
                                    int tables_per_row, uint8_t* idx4_out, uint16_t* cent16_out, cq_stream stream);

/*
 * The same product in the lookup formulation of the kernel section (Fig. 4b and the text beside it): per
 * group of weights that shares a table, the 16 sub-tables (one per centroid) of 16 products centroid x 4-bit
 * activation value are precomputed in LDS; every (weight index, activation code) pair then selects a
 * product, which is accumulated in fp32 -- no multiplication in the inner loop.  A software rendering for
 * comparison with the matrix-core kernels above (the paper's version needs modified tensor cores); same
 * results up to fp32 summation order.
 *   codes [rows, K] int8 holding 4-bit codes in [-8, 7] (values outside wrap modulo 16: the caller's duty);
 *   W->idx (canonical bytes) is read, W->prepacked is ignored; group_k: 0 or a multiple of 32.
 *   Other arguments as for cq_codebook_grouped_gemm; no workspace.
 */
cq_status cq_codebook_grouped_gemm_lut(const cq_codebook_weights* W, const int8_t* codes,
                                       const float* row_scale, const int32_t* row_gather,
                                       const int32_t* group_offsets, int M_total,
                                       int epilogue, void* out, int out_kind, cq_stream stream);

/*
 * Online-Hadamard variant (evaluation section, the "had" setting): rows h [M, I] f32 -> h' = h H_I / sqrt(I)
 * and its per-row symmetric integer quantization (same rule as cq_rotate_quant).  H_I = H_m (x) H_{2^k}
 * (Kronecker product, index i = a*2^k + b) with the Sylvester matrix H_{2^k}[b,b'] = (-1)^popcount(b & b')
 * and m = 1 when I is a power of two, else m = 4 * (odd part of I) in {12, 28, 44} with Paley's matrices:
 * m = 12, 44: H_m = I + S, S = [[0, 1^T], [-1, Q]], Q[i,j] = chi(j - i) mod m-1; m = 28:
 * H_m = S (x) [[1,1],[1,-1]] + I (x) [[1,-1],[-1,-1]], S = [[0, 1^T], [1, Q]], Q[i,j] = chi(i - j) mod 13.
 *   HR_out [M, I] f32 or NULL (the rotated rows), Q_out [M, I] int8, scale_out [M] f32.
 *   I % 4 == 0, I <= 16384, I of the form above (else CQ_ERR_SHAPE); bits in {4, 8}; M = 0 is allowed.
 */
cq_status cq_hadamard_quant(const float* Hrows, int M, int I, int bits, float* HR_out, int8_t* Q_out,
                            float* scale_out, cq_stream stream);

/*
 * a8: weighted combine (MoE weighted sum; shared expert per the appendix on DeepSeek-V2-Lite):
 *   Y[t,:] = sum_{j<k} topk_w[t,j] * O[inv_perm[t*k+j], :] + sum_{s<S} O[T*k + s*T + t, :]
 * summed in the fixed order j = 0..k-1, then s = 0..S-1 (deterministic).  O [T*(k+S), H] f32.
 */
cq_status cq_combine(const float* O, const float* topk_w, const int32_t* inv_perm,
                     int T, int H, int top_k, int n_shared, float* Y, cq_stream stream);

/*
 * The whole layer, a1..a8, on one stream with no host synchronisation:
 *   X [T,H] f32 -> Y [T,H] f32 (in the rotated basis; no R^T is applied).
 * workspace: cq_moe_workspace_bytes(L, T) bytes.  Intermediates live in the workspace; their
 * locations are reported by cq_moe_workspace_layout() for inspection by tests.
 */
typedef struct {
  size_t total;
  size_t XR, Q, Q16, scale, logits, topk_ids, topk_w, offsets, perm, inv_perm, src_token, Hbuf, Obuf, scratch;
  size_t HQ, HQ16, hscale; /* online-Hadamard variant: codes of the rotated intermediate [T*(k+S), I] i8,
                              the same as bf16 (large batches), their scales [T*(k+S)] f32; Hbuf is f32 then */
} cq_moe_layout;
size_t cq_moe_workspace_bytes(const cq_layer* L, int T);
cq_status cq_moe_workspace_layout(const cq_layer* L, int T, cq_moe_layout* out);
cq_status cq_moe_forward(const cq_layer* L, const float* X, int T, float* Y,
                         void* workspace, size_t workspace_bytes, cq_stream stream);

/*
 * cq_moe_forward for callers that cannot allocate device memory or hand over a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same launches and same results as
 * cq_moe_forward, bit for bit; the intermediates live in an array of CQ_STATIC_SCRATCH_BYTES bytes that
 * the library itself holds in the device memory of every GPU it has run on (until the process ends).  The
 * call allocates and frees nothing and does not synchronise the host.
 *   A batch whose cq_moe_workspace_bytes(L, T) exceeds CQ_STATIC_SCRATCH_BYTES returns CQ_ERR_WORKSPACE
 *   and launches nothing (the Mixtral-8x7B shape fits up to T = 96 tokens).
 *   All calls on one GPU share the array, which keeps the previous call's contents (no kernel of the layer
 *   needs it cleared): calls that overlap on one GPU -- two streams, two threads -- race; serialise them.
 */
#define CQ_STATIC_SCRATCH_BYTES (32u << 20)
cq_status cq_moe_forward_static(const cq_layer* L, const float* X, int T, float* Y, cq_stream stream);

/*
 * Offline, one-time re-layout of canonical indices into the kernel-native tile order described at
 * cq_codebook_weights (the paper's pipeline is fully offline, so the stored order is free; the
 * byte count streamed is unchanged).  dst must hold cq_prepack_bytes(W) bytes.
 */
size_t cq_prepack_bytes(const cq_codebook_weights* W);
cq_status cq_prepack(const cq_codebook_weights* W, void* dst, size_t dst_bytes, cq_stream stream);

/*
 * Test hook for the bit-exact decode check: writes W_c of group g as bf16 bit patterns [N, K],
 * reading `prepacked` if present, else `idx` (Eq. W_c); index_bits = 2 weights are decoded through their
 * 4-entry tables.
 */
cq_status cq_decode_dense(const cq_codebook_weights* W, int g, uint16_t* Wc_bf16, cq_stream stream);

#ifdef __cplusplus
}
#endif
#endif /* CQ_H_ */
