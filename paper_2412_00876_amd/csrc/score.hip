// dllava_score: predictor logits D = GELU(x W1^T + b1) W2^T + b2 (Eq. 5 line 1 / Eq. 11 line 1 of the
// paper, with the two-layer predictor d -> dh -> 2).
//
// Precision-generic path: one block per scored row.  The row is staged in LDS as float32; each wave
// takes hidden units round-robin, lanes stride over d with 16-byte loads of the W1 row, a butterfly
// sums the wave, and lane 0 applies bias + GELU and accumulates the two logit terms.  The four wave
// partials are added in wave order, so the result is bit-reproducible.  It serves float32 inputs and
// shapes the matrix-core kernels do not cover.
#include "score_args.h"

namespace dllava {

namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / kWave;

template <typename T>
__global__ __launch_bounds__(kThreads) void score_generic_kernel(ScoreArgs a) {
  extern __shared__ float xs[];  // [d]
  __shared__ float sm_l[kWaves][2];
  constexpr int E = Elem<T>::kPer16B;
  const int64_t m = blockIdx.x;
  const int tid = threadIdx.x, lane = tid & (kWave - 1), w = tid / kWave;
  const int64_t src = score_src_row(a.seq_off, a.vis_start, a.vis_len, a.B, m);
  if (src < 0) return;
  const T* xrow = static_cast<const T*>(a.x) + src * a.ldx;
  const int chunks = static_cast<int>(a.d / E);
  for (int c = tid; c < chunks; c += kThreads) {
    float f[E];
    Elem<T>::unpack(*reinterpret_cast<const uint4*>(xrow + c * E), f);
#pragma unroll
    for (int e = 0; e < E; ++e) xs[c * E + e] = f[e];
  }
  __syncthreads();
  const T* W1 = static_cast<const T*>(a.W1);
  const T* W2 = static_cast<const T*>(a.W2);
  float l0 = 0.f, l1 = 0.f;
  for (int64_t j = w; j < a.dh; j += kWaves) {
    const T* wrow = W1 + j * a.d;
    float acc = 0.f;
    for (int c = lane; c < chunks; c += kWave) {
      float f[E];
      Elem<T>::unpack(*reinterpret_cast<const uint4*>(wrow + c * E), f);
#pragma unroll
      for (int e = 0; e < E; ++e) acc = fmaf(xs[c * E + e], f[e], acc);
    }
    acc = wave_sum(acc);
    const float g = gelu_erf(acc + (a.b1 ? a.b1[j] : 0.f));
    l0 = fmaf(g, Elem<T>::load(W2 + j), l0);
    l1 = fmaf(g, Elem<T>::load(W2 + a.dh + j), l1);
  }
  if (lane == 0) {
    sm_l[w][0] = l0;
    sm_l[w][1] = l1;
  }
  __syncthreads();
  if (tid == 0) {
    float s0 = a.b2 ? a.b2[0] : 0.f, s1 = a.b2 ? a.b2[1] : 0.f;
#pragma unroll
    for (int i = 0; i < kWaves; ++i) {
      s0 += sm_l[i][0];
      s1 += sm_l[i][1];
    }
    a.logits[2 * m] = s0;
    a.logits[2 * m + 1] = s1;
  }
}

template <typename T>
int launch_generic(const ScoreArgs& a, hipStream_t st) {
  hipLaunchKernelGGL((score_generic_kernel<T>), dim3(static_cast<unsigned>(a.M)), dim3(kThreads),
                     static_cast<size_t>(a.d) * sizeof(float), st, a);
  DLLAVA_CHECK_LAUNCH("score_generic_kernel");
  return DLLAVA_OK;
}

}  // namespace

}  // namespace dllava

using namespace dllava;

extern "C" size_t dllava_score_workspace(int64_t M, int64_t d, int64_t dh, int dtype) {
  if (dtype != DLLAVA_BF16 || M <= 0) return 256;
  return score_mfma_workspace(M, d, dh) + 256;
}

extern "C" int dllava_score(const void* x, int64_t ldx, int64_t M, int32_t B, const int32_t* seq_off,
                            const int32_t* vis_start, const int32_t* vis_len, int64_t d, int64_t dh,
                            const void* W1, const float* b1, const void* W2, const float* b2, int dtype,
                            float* logits, void* workspace, size_t workspace_bytes, void* stream) {
  DLLAVA_REQUIRE(dtype == DLLAVA_F32 || dtype == DLLAVA_BF16, DLLAVA_EDTYPE, "score: unknown dtype %d", dtype);
  DLLAVA_REQUIRE(M >= 0 && M <= 0x7fffffffLL, DLLAVA_ESHAPE, "score: bad M = %lld", (long long)M);
  DLLAVA_REQUIRE(d > 0 && d % 8 == 0 && d <= 16384, DLLAVA_ESHAPE, "score: d must be a multiple of 8, at most 16384 (got %lld)",
                 (long long)d);
  DLLAVA_REQUIRE(dh >= 1 && dh <= (1 << 20), DLLAVA_ESHAPE, "score: bad dh = %lld", (long long)dh);
  DLLAVA_REQUIRE(ldx >= d && (ldx * dtype_size(dtype)) % 16 == 0, DLLAVA_ESHAPE,
                 "score: ldx must be >= d and keep rows 16-byte aligned (got %lld)", (long long)ldx);
  if (M == 0) return DLLAVA_OK;
  DLLAVA_REQUIRE(x && W1 && W2 && logits, DLLAVA_ENULL, "score: x, W1, W2, logits are required");
  DLLAVA_REQUIRE(aligned(x, 16) && aligned(W1, 16), DLLAVA_EINVAL, "score: x and W1 must be 16-byte aligned");
  if (seq_off) {
    DLLAVA_REQUIRE(vis_start && vis_len, DLLAVA_ENULL, "score: vis_start and vis_len go with seq_off");
    DLLAVA_REQUIRE(B > 0, DLLAVA_EINVAL, "score: B must be positive when seq_off is given");
  }
  const size_t need = dllava_score_workspace(M, d, dh, dtype);
  DLLAVA_REQUIRE(workspace && aligned(workspace, 256) && workspace_bytes >= need, DLLAVA_EWORKSPACE,
                 "score: workspace needs %zu bytes, 256-byte aligned (got %zu)", need, workspace_bytes);

  ScoreArgs a{x, ldx, M, d, dh, B, seq_off, vis_start, vis_len, W1, b1, W2, b2, logits, workspace};
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (dtype == DLLAVA_BF16) {
    const int rc = score_mfma_launch(a, st);
    if (rc <= 0) return rc;
    return launch_generic<bf16_t>(a, st);
  }
  return launch_generic<float>(a, st);
}
