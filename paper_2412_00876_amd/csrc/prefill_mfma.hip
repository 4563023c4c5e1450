// Matrix-core prefill attention (bf16).  Placeholder until the MFMA kernel lands: declines every shape.
#include "attend.h"

namespace dllava {
struct PrefillArgs;
int prefill_mfma_launch(const PrefillArgs&, int64_t, int, hipStream_t) { return 1; }
}  // namespace dllava
