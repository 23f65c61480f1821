// Instantiations of the single-pass bf16 scoring kernel.
#include "score_fused.h"

namespace ckv {
int launch_score_fused(int head_dim, const ScoreGeom &g, const ScoreArgs &a, dim3 grid, hipStream_t s) {
  if (grid.x == 0 || grid.y == 0 || grid.z == 0) return CHUNKKV_OK;
  if (g.wq != 4) return CHUNKKV_ERR_UNSUPPORTED;
  if (head_dim == 128) {
    if (g.nqw == 1) return launch_fused_cfg<128, 1>(a, grid, s);
    if (g.nqw == 2) return launch_fused_cfg<128, 2>(a, grid, s);
    if (g.nqw == 4) return launch_fused_cfg<128, 4>(a, grid, s);
  } else if (head_dim == 64) {
    if (g.nqw == 1) return launch_fused_cfg<64, 1>(a, grid, s);
    if (g.nqw == 2) return launch_fused_cfg<64, 2>(a, grid, s);
    if (g.nqw == 4) return launch_fused_cfg<64, 4>(a, grid, s);
  }
  return CHUNKKV_ERR_UNSUPPORTED;
}
}  // namespace ckv
