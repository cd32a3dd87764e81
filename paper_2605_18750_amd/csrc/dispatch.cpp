// Chooses the kernel family for each GEMM and attention call.  The choice is a pure function
// of dtype and shape, never of machine state, so a task always runs the same kernels.
#include "kernels.h"

namespace rrfp {

hipError_t launch_gemm(const GemmArgs& g, hipStream_t s) {
  if (g.act != ACT_NONE) return gemm_act_supported(g) ? launch_gemm_mfma(g, s) : hipErrorInvalidValue;
  return gemm_mfma_supports(g) ? launch_gemm_mfma(g, s) : launch_gemm_simt(g, s);
}
hipError_t launch_attn_fwd(const AttnArgs& a, hipStream_t s) {
  return attn_mfma_supports(a) ? launch_attn_fwd_mfma(a, s) : launch_attn_fwd_simt(a, s);
}
hipError_t launch_attn_bwd(const AttnArgs& a, hipStream_t s) {
  return attn_mfma_supports(a) ? launch_attn_bwd_mfma(a, s) : launch_attn_bwd_simt(a, s);
}

}  // namespace rrfp
