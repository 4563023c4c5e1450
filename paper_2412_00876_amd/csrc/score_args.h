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

// The same mapping for a whole block: the spans of up to kSpanLdsMax sequences as a table in LDS (exclusive prefix
// sums of the clamped span lengths and each span's first row), built with one round of loads, then searched per row
// with LDS reads only.  The per-row loop above is a chain of dependent loads, B long, for every row a lane maps: at
// 32 sequences and eight rows per lane that was a fifth of a whole scoring launch.
constexpr int kSpanLdsMax = 1024;

struct SpanTable {
  int32_t prefix[kSpanLdsMax + 1];  // prefix[b] = logits row of span b's first token; prefix[B] = all vision rows
  int32_t base[kSpanLdsMax];        // seq_off[b] + vis_start[b]
  int32_t wave_sum[16];
};

// All THREADS threads of the block call this with 0 < B <= kSpanLdsMax; it ends with a barrier.
template <int THREADS>
__device__ __forceinline__ void span_table_build(SpanTable* t, const int32_t* seq_off,
                                                 const int32_t* vis_start, const int32_t* vis_len, int B) {
  static_assert(kSpanLdsMax % THREADS == 0 && THREADS % kWave == 0 && THREADS / kWave <= 16, "block shape");
  constexpr int C = kSpanLdsMax / THREADS;  // consecutive sequences per thread
  const int tid = threadIdx.x, lane = tid & (kWave - 1), w = tid / kWave;
  int n[C], base[C], s = 0;
#pragma unroll
  for (int i = 0; i < C; ++i) {
    const int b = tid * C + i;
    const bool ok = b < B;
    const int bb = ok ? b : 0;
    const int v = vis_len[bb];
    n[i] = (ok && v > 0) ? v : 0;
    base[i] = seq_off[bb] + vis_start[bb];
    s += n[i];
  }
  int inc = s;  // inclusive scan over the wave, then over the waves through LDS
#pragma unroll
  for (int o = 1; o < kWave; o <<= 1) {
    const int v = __shfl_up(inc, o, kWave);
    if (lane >= o) inc += v;
  }
  if (lane == kWave - 1) t->wave_sum[w] = inc;
  __syncthreads();
  int run = inc - s;
#pragma unroll
  for (int i = 0; i < THREADS / kWave; ++i) run += (i < w) ? t->wave_sum[i] : 0;
#pragma unroll
  for (int i = 0; i < C; ++i) {
    const int b = tid * C + i;
    if (b < B) {
      t->prefix[b] = run;
      t->base[b] = base[i];
    }
    run += n[i];
  }
  if (tid == THREADS - 1) t->prefix[B] = run;
  __syncthreads();
}

// Source row of logits row m from the table, or -1 beyond the spans (empty spans are skipped, as above).
__device__ __forceinline__ int64_t span_table_row(const SpanTable* t, int B, int64_t m) {
  if (m >= t->prefix[B]) return -1;
  int lo = 0, hi = B - 1;
  while (lo < hi) {
    const int mid = (lo + hi) >> 1;
    if (t->prefix[mid + 1] <= m) lo = mid + 1; else hi = mid;
  }
  return static_cast<int64_t>(t->base[lo]) + (m - t->prefix[lo]);
}

// matrix-core paths (score_mfma.hip); score_mfma_launch returns 1 if it does not handle the shape
int score_mfma_launch(const ScoreArgs& a, hipStream_t st);
size_t score_mfma_workspace(int64_t M, int64_t d, int64_t dh);

}  // namespace dllava
