// Matrix-core predictor scoring (bf16).  Placeholder until the MFMA kernels land: declines every shape.
#include "common.h"

namespace dllava {
struct ScoreArgs;
int score_mfma_launch(const ScoreArgs&, hipStream_t) { return 1; }
size_t score_mfma_workspace(int64_t, int64_t, int64_t) { return 0; }
}  // namespace dllava
