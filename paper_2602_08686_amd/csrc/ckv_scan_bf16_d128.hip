// Scan kernels for bf16, d = 128, 1-4 query tiles per wave: see ckv_scan.h.
#include "ckv_scan.h"

namespace ckv {
CKV_DECLARE_SCAN(launch_scores_bf16_d128) {
  return launch_scores_t<CKV_BF16, 128, 1, 4>(s, a, need_lse, need_scores, stream);
}
}  // namespace ckv
