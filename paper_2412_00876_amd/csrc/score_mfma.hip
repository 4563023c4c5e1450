// Matrix-core predictor scoring for bfloat16 inputs (Eq. 5 line 1 / Eq. 11 line 1 of the paper):
//   D = GELU(x W1^T + b1) W2^T + b2,   x [M,d], W1 [dh,d], W2 [2,dh].
//
// Both kernels compute the TRANSPOSED product  A^T = W1 . x^T  (hidden units down the rows, tokens
// across the columns).  x and W1 are both contiguous along d, so either operand fragment is one 16-byte
// load per lane, and in the MFMA result layout a lane then holds many hidden units of ONE token: bias,
// GELU and the 2-way logit contraction over hidden units happen in registers, the pre-activations never
// leave the chip, and only one cross-lane step (lanes l and l+32, or l+16/l+32/l+48) is left.
//
//  * score_gemm_kernel   (M > 64, prefill): 128 units x 128 tokens per block, 4 waves of 64x64 built from
//    v_mfma_f32_32x32x16_bf16, K staged through double-buffered padded LDS tiles.  Each block leaves a
//    partial logit pair per token; the last block of a token tile (device-scope counter) adds the dh/128
//    partials in tile order and the bias.
//  * score_skinny_kernel (M <= 64, decode: one row per sequence): bandwidth-bound on W1; see score_skinny.h.
// All reductions run in a fixed order: results are bit-reproducible.  Counters live at the start of the
// workspace, start at zero and are returned to zero by the block that consumes them.
#include "score_skinny.h"

namespace dllava {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ bf16x8 as_frag(const uint4& v) {
  union { uint4 u; bf16x8 f; } c;
  c.u = v;
  return c.f;
}

constexpr size_t kCounterBytes = 4096;  // up to 1024 int32 counters at the start of the workspace
constexpr int kMaxCounters = 1024;

// ------------------------------------------------------------------------------------------------
// skinny: M <= 16*NT tokens (score_skinny.h)
// ------------------------------------------------------------------------------------------------
constexpr int kSkWaves = 8;
constexpr int kSkThreads = kSkWaves * kWave;

template <int NT>
__global__ __launch_bounds__(kSkThreads) void score_skinny_kernel(ScoreArgs a, int32_t* counter, float* partial) {
  score_skinny_block<NT, kSkWaves, 16>(a, blockIdx.x, gridDim.x, counter, partial);
}

// ------------------------------------------------------------------------------------------------
// GEMM: 128 units x 128 tokens per block
// ------------------------------------------------------------------------------------------------
constexpr int kGThreads = 256;
constexpr int kTU = 128, kTM = 128, kBK = 64;
constexpr int kLd = kBK + 8;  // padded LDS row (elements): 144 bytes, conflict-free 16-byte fragment reads
constexpr int kTileElems = 128 * kLd;

__global__ __launch_bounds__(kGThreads) __attribute__((amdgpu_waves_per_eu(2, 2))) void score_gemm_kernel(ScoreArgs a, int32_t* counters, float* partial) {
  extern __shared__ __align__(16) unsigned char smem_raw[];
  bf16_t* sA = reinterpret_cast<bf16_t*>(smem_raw);  // [2][128][kLd]  W1 tile (units)
  bf16_t* sB = sA + 2 * kTileElems;                  // [2][128][kLd]  x tile (tokens)
  __shared__ float sm_p[2][kTM][2];
  __shared__ int sm_last;

  const int tid = threadIdx.x, lane = tid & (kWave - 1), w = tid / kWave;
  const int ut = blockIdx.x, mt = blockIdx.y, n_ut = gridDim.x;
  const int64_t M = a.M, d = a.d, dh = a.dh;
  const bf16_t* W1 = static_cast<const bf16_t*>(a.W1);
  const bf16_t* X = static_cast<const bf16_t*>(a.x);

  // global -> LDS staging: thread handles chunk c = tid%8 (16 bytes) of rows tid/8 + 32*i, i < 4
  const int lc = tid & 7, lr = tid >> 3;
  const bf16_t* gA[4];
  const bf16_t* gB[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    int64_t u = static_cast<int64_t>(ut) * kTU + lr + 32 * i;
    if (u >= dh) u = dh - 1;
    gA[i] = W1 + u * d + lc * 8;
    int64_t m = static_cast<int64_t>(mt) * kTM + lr + 32 * i;
    if (m >= M) m = M - 1;
    int64_t src = score_src_row(a.seq_off, a.vis_start, a.vis_len, a.B, m);
    if (src < 0) src = 0;
    gB[i] = X + src * a.ldx + lc * 8;
  }
  uint4 ra0, ra1, ra2, ra3, rb0, rb1, rb2, rb3;  // staging registers (scalars, so they stay in VGPRs)
#define DLLAVA_GLOAD(kt)                                                              \
  {                                                                                    \
    const int64_t ko = static_cast<int64_t>(kt) * kBK;                                 \
    ra0 = *reinterpret_cast<const uint4*>(gA[0] + ko);                                 \
    ra1 = *reinterpret_cast<const uint4*>(gA[1] + ko);                                 \
    ra2 = *reinterpret_cast<const uint4*>(gA[2] + ko);                                 \
    ra3 = *reinterpret_cast<const uint4*>(gA[3] + ko);                                 \
    rb0 = *reinterpret_cast<const uint4*>(gB[0] + ko);                                 \
    rb1 = *reinterpret_cast<const uint4*>(gB[1] + ko);                                 \
    rb2 = *reinterpret_cast<const uint4*>(gB[2] + ko);                                 \
    rb3 = *reinterpret_cast<const uint4*>(gB[3] + ko);                                 \
  }
#define DLLAVA_SSTORE(buf)                                                            \
  {                                                                                    \
    const int o = (buf) * kTileElems + lr * kLd + lc * 8;                              \
    *reinterpret_cast<uint4*>(sA + o) = ra0;                                           \
    *reinterpret_cast<uint4*>(sA + o + 32 * kLd) = ra1;                                \
    *reinterpret_cast<uint4*>(sA + o + 64 * kLd) = ra2;                                \
    *reinterpret_cast<uint4*>(sA + o + 96 * kLd) = ra3;                                \
    *reinterpret_cast<uint4*>(sB + o) = rb0;                                           \
    *reinterpret_cast<uint4*>(sB + o + 32 * kLd) = rb1;                                \
    *reinterpret_cast<uint4*>(sB + o + 64 * kLd) = rb2;                                \
    *reinterpret_cast<uint4*>(sB + o + 96 * kLd) = rb3;                                \
  }

  const int wu = (w >> 1) * 64, wm = (w & 1) * 64;  // this wave's 64 units x 64 tokens
  f32x16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  const int nk = static_cast<int>(d / kBK);
  DLLAVA_GLOAD(0)
  DLLAVA_SSTORE(0)
  __syncthreads();
  for (int kt = 0; kt < nk; ++kt) {
    const int buf = kt & 1;
    if (kt + 1 < nk) { DLLAVA_GLOAD(kt + 1) }
    const bf16_t* tA = sA + buf * kTileElems + (wu + (lane & 31)) * kLd + 8 * (lane >> 5);
    const bf16_t* tB = sB + buf * kTileElems + (wm + (lane & 31)) * kLd + 8 * (lane >> 5);
#pragma unroll
    for (int ks = 0; ks < kBK / 16; ++ks) {
      bf16x8 fa[2], fb[2];
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        fa[i] = as_frag(*reinterpret_cast<const uint4*>(tA + i * 32 * kLd + ks * 16));
        fb[i] = as_frag(*reinterpret_cast<const uint4*>(tB + i * 32 * kLd + ks * 16));
      }
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
    }
    if (kt + 1 < nk) { DLLAVA_SSTORE(buf ^ 1) }
    __syncthreads();
  }

#undef DLLAVA_GLOAD
#undef DLLAVA_SSTORE

  // epilogue: lane holds, for token column (lane%32) of token tile j, units 8*(r/4) + 4*(lane/32) + r%4 of unit tile i
  const bf16_t* W2 = static_cast<const bf16_t*>(a.W2);
  float p[2][2] = {{0.f, 0.f}, {0.f, 0.f}};
#pragma unroll
  for (int i = 0; i < 2; ++i) {
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int64_t u = static_cast<int64_t>(ut) * kTU + wu + i * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
      const bool ok = u < dh;
      const float bias = (ok && a.b1) ? a.b1[u] : 0.f;
      const float w20 = ok ? bf16_to_f32(W2[u]) : 0.f;
      const float w21 = ok ? bf16_to_f32(W2[dh + u]) : 0.f;
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const float g = gelu_erf_fast(acc[i][j][r] + bias);
        p[j][0] = fmaf(g, w20, p[j][0]);
        p[j][1] = fmaf(g, w21, p[j][1]);
      }
    }
  }
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    p[j][0] += __shfl_xor(p[j][0], 32, kWave);
    p[j][1] += __shfl_xor(p[j][1], 32, kWave);
    if (lane < 32) {
      sm_p[w >> 1][wm + j * 32 + lane][0] = p[j][0];
      sm_p[w >> 1][wm + j * 32 + lane][1] = p[j][1];
    }
  }
  __syncthreads();
  {
    const int tok = tid >> 1, c = tid & 1;  // 256 threads = 128 tokens x 2 logits
    const int64_t m = static_cast<int64_t>(mt) * kTM + tok;
    if (m < M) st_agent(partial + (static_cast<size_t>(ut) * M + m) * 2 + c, sm_p[0][tok][c] + sm_p[1][tok][c]);
  }
  block_publish();
  if (tid == 0) sm_last = (add_agent(&counters[mt % kMaxCounters], 1) == n_ut - 1);
  __syncthreads();
  if (!sm_last) return;
  {
    const int tok = tid >> 1, c = tid & 1;
    const int64_t m = static_cast<int64_t>(mt) * kTM + tok;
    if (m < M && score_src_row(a.seq_off, a.vis_start, a.vis_len, a.B, m) >= 0) {
      float s = a.b2 ? a.b2[c] : 0.f;
      for (int t0 = 0; t0 < n_ut; t0 += 16) {  // 16 independent loads in flight, then a fixed-order sum
        float v[16];
#pragma unroll
        for (int t = 0; t < 16; ++t)
          v[t] = (t0 + t < n_ut) ? ld_agent(partial + (static_cast<size_t>(t0 + t) * M + m) * 2 + c) : 0.f;
#pragma unroll
        for (int t = 0; t < 16; ++t) s += v[t];
      }
      a.logits[2 * m + c] = s;
    }
  }
  if (tid == 0) zero_agent(&counters[mt % kMaxCounters]);
}

}  // namespace

size_t score_mfma_workspace(int64_t M, int64_t d, int64_t dh) {
  (void)d;
  size_t part;
  if (M <= 64)
    part = static_cast<size_t>(ceil_div(dh, kSkUnits)) * 64 * 2 * sizeof(float);
  else
    part = static_cast<size_t>(ceil_div(dh, kTU)) * M * 2 * sizeof(float);
  return kCounterBytes + round_up(part, 256);
}

// returns 1 if the shape is not handled here
int score_mfma_launch(const ScoreArgs& a, hipStream_t st) {
  if (a.d % kBK != 0 || a.ldx % 8 != 0) return 1;
  int32_t* counters = static_cast<int32_t*>(a.workspace);
  float* partial = reinterpret_cast<float*>(static_cast<char*>(a.workspace) + kCounterBytes);
  if (a.M <= 64) {
    if (a.seq_off) return 1;  // span gathering is only wired into the GEMM path
    const unsigned grid = static_cast<unsigned>(ceil_div(a.dh, kSkUnits));
    if (a.M <= 16)
      hipLaunchKernelGGL(score_skinny_kernel<1>, dim3(grid), dim3(kSkThreads), 0, st, a, counters, partial);
    else if (a.M <= 32)
      hipLaunchKernelGGL(score_skinny_kernel<2>, dim3(grid), dim3(kSkThreads), 0, st, a, counters, partial);
    else
      hipLaunchKernelGGL(score_skinny_kernel<4>, dim3(grid), dim3(kSkThreads), 0, st, a, counters, partial);
    DLLAVA_CHECK_LAUNCH("score_skinny_kernel");
    return DLLAVA_OK;
  }
  const int64_t n_mt = ceil_div(a.M, kTM);
  if (n_mt > 65535) return 1;
  // a token tile's counter may be shared with tile mt + 1024*k: those tiles are far apart in launch order,
  // but to stay exact we only take the path when every tile has its own counter
  if (n_mt > kMaxCounters) return 1;
  static bool attr_set = false;
  const size_t smem = static_cast<size_t>(4) * kTileElems * sizeof(bf16_t);
  if (!attr_set) {
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(score_gemm_kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                        static_cast<int>(smem));
    attr_set = true;
  }
  dim3 grid(static_cast<unsigned>(ceil_div(a.dh, kTU)), static_cast<unsigned>(n_mt));
  hipLaunchKernelGGL(score_gemm_kernel, grid, dim3(kGThreads), smem, st, a, counters, partial);
  DLLAVA_CHECK_LAUNCH("score_gemm_kernel");
  return DLLAVA_OK;
}

}  // namespace dllava
