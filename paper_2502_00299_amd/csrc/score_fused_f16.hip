// fp16 instantiations of the single-pass scoring kernel.
#include "score_fused.h"

namespace ckv {
int launch_score_fused_f16(int head_dim, const ScoreGeom &g, const ScoreArgs &a, dim3 grid, hipStream_t s) {
  return launch_fused_dt<CHUNKKV_F16>(head_dim, g, a, grid, s);
}
}  // namespace ckv
