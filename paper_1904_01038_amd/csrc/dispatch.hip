// Chooses, per call, between the MFMA kernels and the shape-agnostic vector-ALU kernels.
#include "kernels.h"
#include "common.h"

namespace tfm {

void launch_gemm(hipStream_t s, const GemmArgs& a) {
  if (a.deferred_splits) *a.deferred_splits = 0;       // (only a split-K launch of the matrix-core kernels sets it)
  if (gemm_mfma_supported(a)) launch_gemm_mfma(s, a);
  else launch_gemm_naive(s, a);
}

void launch_attention_fwd(hipStream_t s, const AttnArgs& a) {
  if (a.B <= 0 || a.max_lq <= 0 || a.max_lk <= 0) return;
  if (attention_mfma_supported(a, false)) launch_attention_fwd_mfma(s, a);
  else launch_attention_fwd_naive(s, a);
}
void launch_attention_bwd(hipStream_t s, const AttnArgs& a) {
  if (a.B <= 0 || a.max_lq <= 0 || a.max_lk <= 0) return;
  if (attention_mfma_supported(a, true)) launch_attention_bwd_mfma(s, a);
  else launch_attention_bwd_naive(s, a);
}

}  // namespace tfm
