// fp16 instantiations of the scoring kernels (v_mfma_f32_32x32x16_f16).
#include "score_impl.h"

namespace ckv {
int launch_score_f16(int pass, int head_dim, const ScoreGeom &g, const ScoreArgs &a, dim3 grid, hipStream_t s) {
  if (head_dim == 128) return launch_score_hd<CHUNKKV_F16, 128>(pass, g, a, grid, s);
  if (head_dim == 64) return launch_score_hd<CHUNKKV_F16, 64>(pass, g, a, grid, s);
  return CHUNKKV_ERR_UNSUPPORTED;
}
}  // namespace ckv
