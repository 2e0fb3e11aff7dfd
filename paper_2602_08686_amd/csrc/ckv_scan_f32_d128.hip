// Scan kernels for f32, d128: see ckv_scan.h.
#include "ckv_scan.h"

namespace ckv {
hipError_t launch_scores_f32_d128(const Shape &s, ScoreArgs &a, bool need_lse, bool need_scores,
                                  hipStream_t stream) {
  return launch_scores_t<CKV_F32, 128>(s, a, need_lse, need_scores, stream);
}
}  // namespace ckv
