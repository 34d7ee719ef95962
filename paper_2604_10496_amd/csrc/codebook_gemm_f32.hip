// The streaming kernel's instantiations for one operand kind (CQ_A_F32); see codebook_gemm_small.h.
#include "codebook_gemm_small.h"

cq_status cq_gemm_small_dispatch_f32(const GemmArgs& a, int G, int qt, int epilogue, int out_kind, hipStream_t s) {
  return dispatch_epi<CQ_A_F32>(a, G, qt, epilogue, out_kind, s);
}
