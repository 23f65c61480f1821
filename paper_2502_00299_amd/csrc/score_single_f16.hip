// fp16 instantiations of the single-pass scoring kernel.
#include "score_single.h"

namespace ckv {
int launch_score_single_f16(const ScoreArgs &a, dim3 grid, hipStream_t s) { return launch_single_dt<CHUNKKV_F16>(a, grid, s); }
}  // namespace ckv
