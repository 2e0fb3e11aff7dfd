// Scan kernels for bf16, d = 64, 5-6 query tiles per wave: see ckv_scan.h.
#include "ckv_scan.h"

namespace ckv {
CKV_DECLARE_SCAN(launch_scores_bf16_d64_nq56) {
  return launch_scores_t<CKV_BF16, 64, 5, 6>(s, a, need_lse, need_scores, stream);
}
}  // namespace ckv
