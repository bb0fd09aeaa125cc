// Attention-mass scores (Eq. 1) on the matrix cores: bf16 operands, fp32 accumulation.
#include "common.hpp"

namespace obf {

bool mfma_score_supported(const Dims& m) {
  (void)m;
  return false;
}

obf_status_t launch_score_mfma(const Dims& m, const Workspace& w, char* ws, const void* K, const void* Q,
                               float* scores, double* row_lse, hipStream_t st) {
  (void)m; (void)w; (void)ws; (void)K; (void)Q; (void)scores; (void)row_lse; (void)st;
  set_error("MFMA score path not available for this shape");
  return OBF_ERR_UNSUPPORTED;
}

}  // namespace obf
