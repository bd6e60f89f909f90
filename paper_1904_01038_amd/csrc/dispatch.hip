// Chooses, per call, between the MFMA kernels and the shape-agnostic vector-ALU kernels.
#include "kernels.h"
#include "common.h"

namespace tfm {

void launch_gemm(hipStream_t s, const GemmArgs& a) {
  if (gemm_mfma_supported(a)) launch_gemm_mfma(s, a);
  else launch_gemm_naive(s, a);
}

void launch_attention_fwd(hipStream_t s, const AttnArgs& a) { launch_attention_fwd_naive(s, a); }
void launch_attention_bwd(hipStream_t s, const AttnArgs& a) { launch_attention_bwd_naive(s, a); }

}  // namespace tfm
