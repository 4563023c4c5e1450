// Arguments of the predictor-scoring kernels and the row mapping shared by them.
#pragma once

#include "common.h"

namespace dllava {

struct ScoreArgs {
  const void* x;
  int64_t ldx, M, d, dh;
  int32_t B;
  const int32_t* seq_off;
  const int32_t* vis_start;
  const int32_t* vis_len;
  const void* W1;
  const float* b1;
  const void* W2;
  const float* b2;
  float* logits;
  void* workspace;
};

// Sixteen zero bytes in device memory.  Epilogue operands that must read as zero (no bias given, hidden unit
// past dh) are loaded from here through a selected ADDRESS, so the load itself stays unconditional: a load whose
// result is selected against a constant gets sunk under a branch by the compiler, with a full memory wait at
// the end of every such branch (measured: a dozen serial round trips per block).
static __device__ __attribute__((aligned(16))) float kZeroWords[4] = {0.f, 0.f, 0.f, 0.f};

// Source row of x for logits row m (vision spans back to back), or -1 if m is beyond the spans.
__device__ __forceinline__ int64_t score_src_row(const int32_t* seq_off, const int32_t* vis_start,
                                                 const int32_t* vis_len, int B, int64_t m) {
  if (!seq_off) return m;
  int64_t acc = 0;
  for (int b = 0; b < B; ++b) {
    const int n = vis_len[b] > 0 ? vis_len[b] : 0;
    if (m < acc + n) return static_cast<int64_t>(seq_off[b]) + vis_start[b] + (m - acc);
    acc += n;
  }
  return -1;
}

// matrix-core paths (score_mfma.hip); score_mfma_launch returns 1 if it does not handle the shape
int score_mfma_launch(const ScoreArgs& a, hipStream_t st);
size_t score_mfma_workspace(int64_t M, int64_t d, int64_t dh);

}  // namespace dllava
