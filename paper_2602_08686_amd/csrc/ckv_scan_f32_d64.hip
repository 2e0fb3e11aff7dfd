// Scan kernels for f32, d = 64: see ckv_scan.h.
#include "ckv_scan.h"

namespace ckv {
CKV_DECLARE_SCAN(launch_scores_f32_d64) {
  return launch_scores_t<CKV_F32, 64, 1, 4>(s, a, need_lse, need_scores, stream);
}
}  // namespace ckv
