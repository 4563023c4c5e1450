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
//    v_mfma_f32_32x32x16_bf16, the hidden dimension streamed in 64-element stages (whole 128-byte memory lines
//    per row) through one swizzled LDS tile pair, the global loads two stages ahead in registers, LDS-only
//    barriers, three blocks per compute unit, XCD-aware tile order.  Each block leaves a
//    partial logit pair per token; the last block of a token tile (device-scope counter) adds the dh/128
//    partials in tile order and the bias.
//  * score_splitk_kernel (M <= 64, decode: one row per sequence): W1 read once, cut over units and d; see
//    score_splitk.h.
// All reductions run in a fixed order: results are bit-reproducible.  The counters of the two forms live in
// disjoint regions at the start of the workspace (layout in score_splitk.h), start at zero and are returned to
// zero by the block that consumes them, so one workspace serves calls of either form in any order.
#include "gemm_ring.h"
#include "gemm_tile.h"
#include "score_splitk.h"

namespace dllava {

namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kMaxCounters = static_cast<int>(kGemmCntBytes / sizeof(int32_t));  // one per token tile

// ------------------------------------------------------------------------------------------------
// GEMM: 128 units x 128 tokens per block
// ------------------------------------------------------------------------------------------------
constexpr int kTU = 128, kTM = 128;
constexpr int kXcds = 8;            // accelerator complex dies of the chip

__global__ __launch_bounds__(kGThreads) __attribute__((amdgpu_waves_per_eu(3, 4))) void score_gemm_kernel(
    ScoreArgs a, int32_t* counters, float* partial, int n_unit_tiles) {
  __shared__ __align__(16) bf16_t sA[kTileElems];  // [128][64]  W1 tile (units), chunks swizzled
  __shared__ __align__(16) bf16_t sB[kTileElems];  // [128][64]  x tile (tokens)
  __shared__ float sm_p[2][kTM][2];
  __shared__ int sm_last;

  const int tid = threadIdx.x, lane = tid & (kWave - 1), w = tid / kWave;
  // XCD-aware tile order.  Consecutive block ids go round-robin to the 8 XCDs, each with its own 4 MiB L2.
  // XCD x takes the token tiles x, x+8, ... and, for each, all unit tiles: its blocks are resident together and
  // walk the hidden dimension roughly in step, so each XCD pulls W1 and its share of x through its L2 about once
  // (the plain (unit tile, token tile) order made every XCD stream all of x: 4x the traffic beyond L2).
  const int n_ut = n_unit_tiles;
  const int xcd = blockIdx.x % kXcds, jb = blockIdx.x / kXcds;
  const int ut = jb % n_ut, mt = (jb / n_ut) * kXcds + xcd;
  const int64_t M = a.M, d = a.d, dh = a.dh;
  if (static_cast<int64_t>(mt) * kTM >= M) return;  // padding of the last round of token tiles
  const bf16_t* W1 = static_cast<const bf16_t*>(a.W1);
  const bf16_t* X = static_cast<const bf16_t*>(a.x);

  // staging thread: 16-byte chunk lc of rows lr + 32*j of both tiles (see gemm_tile.h)
  const int lc = tid & 7, lr = tid >> 3;
  static_assert(sizeof(SpanTable) <= sizeof(sA), "the span table borrows the W1 tile's memory");
  SpanTable* spans = reinterpret_cast<SpanTable*>(sA);
  const bool use_table = a.seq_off != nullptr && a.B > 0 && a.B <= kSpanLdsMax;
  if (use_table) span_table_build<kGThreads>(spans, a.seq_off, a.vis_start, a.vis_len, a.B);
  const int64_t rows_in_spans = use_table ? spans->prefix[a.B] : -1;
  const bf16_t *gA0, *gA1, *gA2, *gA3, *gB0, *gB1, *gB2, *gB3;
  {
    const bf16_t* ga[4];
    const bf16_t* gb[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      int64_t u = static_cast<int64_t>(ut) * kTU + lr + 32 * j;
      if (u >= dh) u = dh - 1;  // clamped rows carry zero W2 weights in the epilogue
      ga[j] = W1 + u * d + lc * 8;
      int64_t m = static_cast<int64_t>(mt) * kTM + lr + 32 * j;
      if (m >= M) m = M - 1;
      int64_t sr = use_table ? span_table_row(spans, a.B, m) : score_src_row(a.seq_off, a.vis_start, a.vis_len, a.B, m);
      if (sr < 0) sr = 0;
      gb[j] = X + sr * a.ldx + lc * 8;
    }
    gA0 = ga[0]; gA1 = ga[1]; gA2 = ga[2]; gA3 = ga[3];
    gB0 = gb[0]; gB1 = gb[1]; gB2 = gb[2]; gB3 = gb[3];
  }
  if (use_table) __syncthreads();  // the tile loads overwrite the table
  const int nk = static_cast<int>(d / kBK);
  const int wu = (w >> 1) * 64, wm = (w & 1) * 64;  // this wave's 64 units x 64 tokens
  f32x16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
  gemm_tile_128x128<32>(gA0, gA1, gA2, gA3, gB0, gB1, gB2, gB3, nk, sA, sB, wu, wm, acc);

  // epilogue: lane holds, for token column (lane%32) of token tile j, units 8*(r/4) + 4*(lane/32) + r%4 of unit tile i
  const bf16_t* W2 = static_cast<const bf16_t*>(a.W2);
  const bool has_b1 = a.b1 != nullptr;
  const bf16_t* zero16 = reinterpret_cast<const bf16_t*>(kZeroWords);
  float p[2][2] = {{0.f, 0.f}, {0.f, 0.f}};
#pragma unroll
  for (int i = 0; i < 2; ++i) {
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int64_t u = static_cast<int64_t>(ut) * kTU + wu + i * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
      const bool ok = u < dh;  // operands that must be zero come from kZeroWords: no load under a condition
      const float bias = *((ok & has_b1) ? a.b1 + u : kZeroWords);
      const float w20 = bf16_to_f32(*(ok ? W2 + u : zero16));
      const float w21 = bf16_to_f32(*(ok ? W2 + dh + u : zero16));
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
    const bool in_spans = use_table ? m < rows_in_spans : score_src_row(a.seq_off, a.vis_start, a.vis_len, a.B, m) >= 0;
    if (m < M && in_spans) {
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

// ------------------------------------------------------------------------------------------------
// GEMM for many rows: 256 units x 32*JB tokens per block, one block per compute unit (gemm_ring.h)
// ------------------------------------------------------------------------------------------------
// Same decomposition and the same cross-block reduction as score_gemm_kernel (partial logit pairs per unit tile,
// the last block of a token tile adds them in tile order), on the large-tile product: wave w holds units 64w + [0,64)
// of the unit tile for all 32*JB tokens of the token tile.  The token-tile width is chosen on the host so that the
// launch fills the 256 compute units evenly (score_ring_pick).
template <int JB>
__global__ __launch_bounds__(kRingThreads, 1) void score_ring_kernel(ScoreArgs a, int32_t* counters, float* partial,
                                                                     int n_unit_tiles) {
  constexpr int kTok = 32 * JB;
  __shared__ __align__(1024) char smem_raw[kRingLdsBytes];
  DLLAVA_LDS char* smem = (DLLAVA_LDS char*)smem_raw;
  const int tid = threadIdx.x, lane = tid & (kWave - 1);
  const int w = __builtin_amdgcn_readfirstlane(tid / kWave);
  // XCD x takes the token tiles x, x+8, ... and, for each, all unit tiles (see score_gemm_kernel)
  const int n_ut = n_unit_tiles;
  const int xcd = blockIdx.x % kXcds, jb = blockIdx.x / kXcds;
  const int ut = jb % n_ut, mt = (jb / n_ut) * kXcds + xcd;
  const int64_t M = a.M, d = a.d, dh = a.dh;
  if (static_cast<int64_t>(mt) * kTok >= M) return;  // padding of the last round of token tiles

  // this lane's tile loads: byte offsets from W1 / x (rows past the end repeat the last row: their units carry
  // zero W2 weights, their tokens are not written)
  uint32_t ga[kRingALoads];
  int64_t gb[JB];  // gathered rows of x may lie far apart
#pragma unroll
  for (int j = 0; j < kRingALoads; ++j) {
    const int row = ring_load_row(w, j, lane);
    int64_t u = static_cast<int64_t>(ut) * 256 + row;
    if (u >= dh) u = dh - 1;
    ga[j] = static_cast<uint32_t>(u * d * 2) + ring_load_chunk_bytes(row, lane);
  }
  // gathered spans: the row mapping from a table in the (not yet used) ring memory
  SpanTable* spans = reinterpret_cast<SpanTable*>(smem_raw);
  const bool use_table = a.seq_off != nullptr && a.B > 0 && a.B <= kSpanLdsMax;
  if (use_table) span_table_build<kRingThreads>(spans, a.seq_off, a.vis_start, a.vis_len, a.B);
  const int64_t rows_in_spans = use_table ? spans->prefix[a.B] : -1;
#pragma unroll
  for (int j = 0; j < JB; ++j) {
    const int row = ring_load_row(w, j, lane);
    int64_t m = static_cast<int64_t>(mt) * kTok + row;
    if (m >= M) m = M - 1;
    int64_t sr = use_table ? span_table_row(spans, a.B, m) : score_src_row(a.seq_off, a.vis_start, a.vis_len, a.B, m);
    if (sr < 0) sr = 0;
    gb[j] = sr * a.ldx * 2 + ring_load_chunk_bytes(row, lane);
  }
  if (use_table) __syncthreads();  // the tile loads overwrite the table
  ring_f32x16 acc[2][JB];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < JB; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
  gemm_ring_256<JB, 32, int64_t>(static_cast<const char*>(a.W1), ga, static_cast<const char*>(a.x), gb, static_cast<int>(d / kRingBK),
                        smem, w, 64 * w, acc);

  // epilogue: lane holds, for token column (lane%32) of token tile j, units 8*(r/4) + 4*(lane/32) + r%4 of unit
  // tile i of this wave
  const bf16_t* W2 = static_cast<const bf16_t*>(a.W2);
  const bool has_b1 = a.b1 != nullptr;
  const bf16_t* zero16 = reinterpret_cast<const bf16_t*>(kZeroWords);
  float p[JB][2];
#pragma unroll
  for (int j = 0; j < JB; ++j) p[j][0] = p[j][1] = 0.f;
#pragma unroll
  for (int i = 0; i < 2; ++i) {
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int64_t u = static_cast<int64_t>(ut) * 256 + 64 * w + i * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
      const bool ok = u < dh;  // operands that must be zero come from kZeroWords: no load under a condition
      const float bias = *((ok & has_b1) ? a.b1 + u : kZeroWords);
      const float w20 = bf16_to_f32(*(ok ? W2 + u : zero16));
      const float w21 = bf16_to_f32(*(ok ? W2 + dh + u : zero16));
#pragma unroll
      for (int j = 0; j < JB; ++j) {
        const float g = gelu_erf_fast(acc[i][j][r] + bias);
        p[j][0] = fmaf(g, w20, p[j][0]);
        p[j][1] = fmaf(g, w21, p[j][1]);
      }
    }
  }
  // the ring memory becomes the waves' partial sums: every wave has drained its own tile loads, the barrier covers
  // the others'
  __syncthreads();
  float* sm_p = reinterpret_cast<float*>(smem_raw);  // [4 waves][kTok][2]
  int* sm_last = reinterpret_cast<int*>(smem_raw + 4 * kTok * 2 * sizeof(float));
#pragma unroll
  for (int j = 0; j < JB; ++j) {
    p[j][0] += __shfl_xor(p[j][0], 32, kWave);
    p[j][1] += __shfl_xor(p[j][1], 32, kWave);
    if (lane < 32) {
      sm_p[(w * kTok + j * 32 + lane) * 2 + 0] = p[j][0];
      sm_p[(w * kTok + j * 32 + lane) * 2 + 1] = p[j][1];
    }
  }
  __syncthreads();
  for (int t = tid; t < 2 * kTok; t += kRingThreads) {
    const int tok = t >> 1, c = t & 1;
    const int64_t m = static_cast<int64_t>(mt) * kTok + tok;
    const float v = (sm_p[(0 * kTok + tok) * 2 + c] + sm_p[(1 * kTok + tok) * 2 + c]) +
                    (sm_p[(2 * kTok + tok) * 2 + c] + sm_p[(3 * kTok + tok) * 2 + c]);
    if (m < M) st_agent(partial + (static_cast<size_t>(ut) * M + m) * 2 + c, v);
  }
  block_publish();
  if (tid == 0) *sm_last = (add_agent(&counters[mt % kMaxCounters], 1) == n_ut - 1);
  __syncthreads();
  if (!*sm_last) return;
  for (int t = tid; t < 2 * kTok; t += kRingThreads) {
    const int tok = t >> 1, c = t & 1;
    const int64_t m = static_cast<int64_t>(mt) * kTok + tok;
    const bool in_spans = use_table ? m < rows_in_spans : score_src_row(a.seq_off, a.vis_start, a.vis_len, a.B, m) >= 0;
    if (m < M && in_spans) {
      float s = a.b2 ? a.b2[c] : 0.f;
      for (int t0 = 0; t0 < n_ut; t0 += 8) {  // independent loads in flight, then a fixed-order sum
        float v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u)
          v[u] = (t0 + u < n_ut) ? ld_agent(partial + (static_cast<size_t>(t0 + u) * M + m) * 2 + c) : 0.f;
#pragma unroll
        for (int u = 0; u < 8; ++u) s += v[u];
      }
      a.logits[2 * m + c] = s;
    }
  }
  if (tid == 0) zero_agent(&counters[mt % kMaxCounters]);
}

// Token-tile width (in 32-token units, 4..8) that fills the chip's compute units most evenly, or 0 when the launch
// would leave most of them idle (the 128 x 128 kernel with three blocks per compute unit serves those).
// Cost model: a block's time is proportional to its stages' products plus a fixed part per stage (measured: 2540
// clocks per stage at 256 tokens, of which 2048 are the products); a launch takes as many rounds as its blocks
// need on 256 compute units.
int score_ring_pick(int64_t M, int64_t dh) {
  const int64_t n_ut = ceil_div(dh, 256);
  int best = 0;
  int64_t best_cost = 0;
  for (int jb = 8; jb >= 4; --jb) {
    const int64_t blocks = ceil_div(M, 32 * jb) * n_ut;
    if (blocks < 128) continue;
    const int64_t cost = ceil_div(blocks, 256) * (256 * jb + 500);
    if (!best || cost < best_cost) best = jb, best_cost = cost;
  }
  return best;
}

template <int JB>
int score_ring_launch(const ScoreArgs& a, int32_t* counters, float* partial, hipStream_t st) {
  const int64_t n_mt = ceil_div(a.M, 32 * JB);
  const int n_ut = static_cast<int>(ceil_div(a.dh, 256));
  const int64_t blocks = ceil_div(n_mt, kXcds) * kXcds * n_ut;
  hipLaunchKernelGGL(score_ring_kernel<JB>, dim3(static_cast<unsigned>(blocks)), dim3(kRingThreads), 0, st, a, counters,
                     partial, n_ut);
  DLLAVA_CHECK_LAUNCH("score_ring_kernel");
  return DLLAVA_OK;
}

}  // namespace

size_t score_mfma_workspace(int64_t M, int64_t d, int64_t dh) {
  // Non-decreasing in M, so a workspace sized for the largest row count serves every smaller one: the split-K form
  // of at most 64 rows needs more than the GEMM form of a few hundred.
  const size_t small = round_up(split_workspace(M < 64 ? M : 64, d, dh), 256);
  if (M <= 64) return small;
  const size_t part = static_cast<size_t>(ceil_div(dh, kTU)) * M * 2 * sizeof(float);
  const size_t gemm = kScoreScratchOffset + round_up(part, 256);
  return gemm > small ? gemm : small;
}

// returns 1 if the shape is not handled here
int score_mfma_launch(const ScoreArgs& a, hipStream_t st) {
  if (a.d % 64 != 0 || a.ldx % 8 != 0) return 1;
  int32_t* counters = reinterpret_cast<int32_t*>(static_cast<char*>(a.workspace) + kSpAccBytes + kSpCntBytes);
  float* partial = reinterpret_cast<float*>(static_cast<char*>(a.workspace) + kScoreScratchOffset);
  if (a.M <= 64) {
    if (a.seq_off) return 1;  // span gathering is only wired into the GEMM path
    const SplitPlan p = split_plan(a.d, a.dh);
    if (p.G > kSpMaxGroups) return 1;
    const dim3 grid(static_cast<unsigned>(p.G * p.KS)), block(kSpThreads);
    if (a.M <= 16)
      hipLaunchKernelGGL(score_splitk_kernel<1>, grid, block, 0, st, a, p.G, p.KS, p.ppb);
    else if (a.M <= 32)
      hipLaunchKernelGGL(score_splitk_kernel<2>, grid, block, 0, st, a, p.G, p.KS, p.ppb);
    else
      hipLaunchKernelGGL(score_splitk_kernel<4>, grid, block, 0, st, a, p.G, p.KS, p.ppb);
    DLLAVA_CHECK_LAUNCH("score_splitk_kernel");
    return DLLAVA_OK;
  }
  // Many rows: the large-tile kernel, unless forced off (DLLAVA_LAUNCH_SCORE_TILE = 1) or the shape does not fit it:
  // lane offsets into W1 are 32-bit, and every token tile needs its own counter.
  {
    int jb = score_ring_pick(a.M, a.dh);
    const int forced = launch_override(DLLAVA_LAUNCH_SCORE_TILE);
    if (forced == 1) jb = 0;
    if (forced >= 4 && forced <= 8) jb = forced;
    const bool fits = a.dh * a.d * 2 < (int64_t{1} << 32) && (jb == 0 || ceil_div(a.M, 32 * jb) <= kMaxCounters);
    if (jb && fits) {
      switch (jb) {
        case 4: return score_ring_launch<4>(a, counters, partial, st);
        case 5: return score_ring_launch<5>(a, counters, partial, st);
        case 6: return score_ring_launch<6>(a, counters, partial, st);
        case 7: return score_ring_launch<7>(a, counters, partial, st);
        default: return score_ring_launch<8>(a, counters, partial, st);
      }
    }
  }
  const int64_t n_mt = ceil_div(a.M, kTM);
  if (n_mt > 65535) return 1;
  // a token tile's counter may be shared with tile mt + 1024*k: those tiles are far apart in launch order,
  // but to stay exact we only take the path when every tile has its own counter
  if (n_mt > kMaxCounters) return 1;
  const int n_ut = static_cast<int>(ceil_div(a.dh, kTU));
  const int64_t blocks = ceil_div(n_mt, kXcds) * kXcds * n_ut;
  if (blocks > 0x7fffffffLL) return 1;
  hipLaunchKernelGGL(score_gemm_kernel, dim3(static_cast<unsigned>(blocks)), dim3(kGThreads), 0, st, a, counters,
                     partial, n_ut);
  DLLAVA_CHECK_LAUNCH("score_gemm_kernel");
  return DLLAVA_OK;
}

}  // namespace dllava
