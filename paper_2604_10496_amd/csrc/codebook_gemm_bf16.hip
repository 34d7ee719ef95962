// The streaming kernel's instantiations for one operand kind (CQ_A_BF16); see codebook_gemm_small.h.
#include "codebook_gemm_small.h"

cq_status cq_gemm_small_dispatch_bf16(const GemmArgs& a, int G, int qt, int epilogue, int out_kind, hipStream_t s) {
  return dispatch_epi<CQ_A_BF16>(a, G, qt, epilogue, out_kind, s);
}
