// The score passes for head_dim 128, FP8 E4M3 keys (one translation unit per pair: they compile side by side).
#include "score_pass.h"

namespace codecomp {
template int dispatch_waves<128, true>(const Plan&, const ScoreArgs&, hipStream_t, unsigned);
}  // namespace codecomp
