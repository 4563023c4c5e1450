// Predictors in the form of the paper's appendix (Appendix A.4.1): a linear layer that reduces the decoder width to
// 512, for the image predictor two pre-norm transformer blocks over the image tokens of each sequence, and the MLP
// head 512 -> 256 -> 128 -> 2.  bfloat16 storage, float32 sums.
//
//  * lin_gemm_kernel   Y = act(X W^T + b) (+ R): the 128 x 128 matrix-core tile product of gemm_tile.h (transposed
//                      product W . X^T, so a lane holds many output features of ONE token), bias / GELU / residual in
//                      registers, then a transposition through LDS so that every token leaves as whole 16-byte
//                      pieces of a 256-byte run.  The first layer gathers its rows from the vision spans.
//  * ln_kernel         LayerNorm of 512-wide rows, one wave per row, the row held in registers.
//  * attention         prefill_mfma_kernel without the causal mask, 8 heads of 64, one "sequence" per span.
//  * head_out_kernel   the last layer 128 -> 2, one wave per row.
//  * small_in_kernel, small_head_kernel   the whole text form on at most 64 rows (a decode step), see below.
// The same file holds the remaining layers of a LLaMA-family decoder layer (Eq. 2-3 of the paper name only W^Q, W^K,
// W^V, W^O and an FFN; RMSNorm, rotary positions and the gated FFN are the family's):
//  * rms_norm_kernel, rms_norm_row_kernel   RMSNorm, one wave or (few rows) one block per row.
//  * rope_kernel       rotary rotation in place.
//  * few_fused_kernel  a linear layer on at most 64 rows in one launch (the weights are the traffic), with the
//                      epilogues of a decode step: bias / GELU / residual / gate, q|k|v with rotary rotation,
//                      gate|up with the gating.
// Every output element is produced by one thread summing in a fixed order (sums that cross waves or blocks are
// added in wave / part order), so the results are bit-reproducible.
#include <cmath>

#include "gemm_tile.h"
#include "prefill_args.h"
#include "score_args.h"

namespace dllava {

namespace {

constexpr int kPW = 512;       // predictor width (Appendix A.4.1)
constexpr int kPHeads = 8;     // heads of 64
constexpr int kPMlp = 2048;    // hidden width of a block's MLP
constexpr int kPH1 = 256, kPH2 = 128;  // head: 512 -> 256 -> 128 -> 2
constexpr float kLnEps = 1e-6f;
constexpr int kXcds = 8;

// SiLU g / (1 + e^-g) with the hardware exponential and reciprocal (relative error ~1e-6)
__device__ __forceinline__ float silu_fast(float g) {
  return g * __builtin_amdgcn_rcpf(1.f + __builtin_amdgcn_exp2f(-1.44269504088896340736f * g));
}

struct LinArgs {
  const bf16_t* X;   // [*, K], row stride ldx
  int64_t ldx, M;
  int K, N;
  const bf16_t* W;   // [N, K]
  const float* bias; // [N] or null
  // feature f of row m goes to Y[(f / group) * group_stride + m * ldy + f % group]  (group = N: one plain matrix)
  bf16_t* Y;
  int64_t ldy, group_stride;
  int group;
  const bf16_t* R;   // residual, indexed like Y (may be Y itself), or null
  int act;           // 1: GELU; 2: multiply by SiLU(R) instead of adding R
  // rows of X: the vision spans back to back when seq_off is given, else rows 0..M-1
  int32_t B;
  const int32_t* seq_off;
  const int32_t* vis_start;
  const int32_t* vis_len;
};

__global__ __launch_bounds__(kGThreads) __attribute__((amdgpu_waves_per_eu(3, 4))) void lin_gemm_kernel(LinArgs a,
                                                                                                         int n_ut) {
  __shared__ __align__(16) bf16_t sAB[2 * kTileElems];  // W tile | X tile during the product, output tile afterwards
  bf16_t* sA = sAB;
  bf16_t* sB = sAB + kTileElems;
  const int tid = threadIdx.x, lane = tid & (kWave - 1), w = tid / kWave;
  // XCD x takes the token tiles x, x+8, ... and, for each, all feature tiles (see score_gemm_kernel)
  const int xcd = blockIdx.x % kXcds, jb = blockIdx.x / kXcds;
  const int ut = jb % n_ut, mt = (jb / n_ut) * kXcds + xcd;
  const int64_t M = a.M;
  const int N = a.N, K = a.K;
  if (static_cast<int64_t>(mt) * 128 >= M) return;

  const int lc = tid & 7, lr = tid >> 3;
  static_assert(sizeof(SpanTable) <= sizeof(sAB), "the span table borrows the tiles' memory");
  SpanTable* spans = reinterpret_cast<SpanTable*>(sAB);
  const bool use_table = a.seq_off != nullptr && a.B > 0 && a.B <= kSpanLdsMax;
  if (use_table) span_table_build<kGThreads>(spans, a.seq_off, a.vis_start, a.vis_len, a.B);
  const bf16_t *ga[4], *gb[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    int u = ut * 128 + lr + 32 * j;
    if (u >= N) u = N - 1;  // such features are computed and dropped
    ga[j] = a.W + static_cast<int64_t>(u) * K + lc * 8;
    int64_t m = static_cast<int64_t>(mt) * 128 + lr + 32 * j;
    if (m >= M) m = M - 1;
    int64_t sr = use_table ? span_table_row(spans, a.B, m) : score_src_row(a.seq_off, a.vis_start, a.vis_len, a.B, m);
    if (sr < 0) sr = 0;
    gb[j] = a.X + sr * a.ldx + lc * 8;
  }
  if (use_table) __syncthreads();  // the tile loads overwrite the table
  const int wu = (w >> 1) * 64, wm = (w & 1) * 64;  // this wave's 64 features x 64 tokens
  f32x16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
  gemm_tile_128x128<32>(ga[0], ga[1], ga[2], ga[3], gb[0], gb[1], gb[2], gb[3], K / kBK, sA, sB, wu, wm, acc);

  // lane: token column wm + 32*j + lane%32; register r of fragment i: feature wu + 32*i + 8*(r/4) + 4*(lane/32) + r%4
  const int g = lane >> 5;
  bf16_t* sO = sAB;  // [128 tokens][16 chunks of 8 features], chunk c of token t at chunk position c ^ (t % 16)
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int q4 = 0; q4 < 4; ++q4) {
      const int fl = wu + 32 * i + 8 * q4 + 4 * g;  // this lane's four features of the tile
      const int f0 = ut * 128 + fl;
      const bool ok = f0 < N;
      const float4 bs = *reinterpret_cast<const float4*>((ok && a.bias) ? a.bias + f0 : kZeroWords);
      const int fs = ok ? f0 : 0;  // features past N: any valid address, the result is dropped
      const int64_t col = static_cast<int64_t>(fs / a.group) * a.group_stride + fs % a.group;
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const int t = wm + 32 * j + (lane & 31);
        int64_t m = static_cast<int64_t>(mt) * 128 + t;
        if (m >= M) m = M - 1;
        float v0 = acc[i][j][4 * q4] + bs.x, v1 = acc[i][j][4 * q4 + 1] + bs.y;
        float v2 = acc[i][j][4 * q4 + 2] + bs.z, v3 = acc[i][j][4 * q4 + 3] + bs.w;
        if (a.act == 1) {
          v0 = gelu_erf_fast(v0); v1 = gelu_erf_fast(v1); v2 = gelu_erf_fast(v2); v3 = gelu_erf_fast(v3);
        }
        if (a.R) {  // block-uniform; the result is rounded once, after the addition / the product
          const uint2 rr = *reinterpret_cast<const uint2*>(a.R + col + m * a.ldy);
          const float r0 = bf16lo_to_f32(rr.x), r1 = bf16hi_to_f32(rr.x), r2 = bf16lo_to_f32(rr.y), r3 = bf16hi_to_f32(rr.y);
          if (a.act == 2) {  // gated unit: R holds the gate, the output is this product times SiLU(gate)
            v0 *= silu_fast(r0); v1 *= silu_fast(r1); v2 *= silu_fast(r2); v3 *= silu_fast(r3);
          } else {
            v0 += r0; v1 += r1; v2 += r2; v3 += r3;
          }
        }
        uint2 v;
        v.x = pack_bf16x2(v0, v1);
        v.y = pack_bf16x2(v2, v3);
        *reinterpret_cast<uint2*>(sO + t * 128 + (((fl >> 3) ^ (t & 15)) * 8) + g * 4) = v;
      }
    }
  __syncthreads();
#pragma unroll
  for (int k = 0; k < 8; ++k) {
    const int idx = tid + kGThreads * k, t = idx >> 4, c = idx & 15;
    const int64_t m = static_cast<int64_t>(mt) * 128 + t;
    const int f = ut * 128 + c * 8;
    if (m < M && f < N)
      *reinterpret_cast<uint4*>(a.Y + static_cast<int64_t>(f / a.group) * a.group_stride + m * a.ldy + f % a.group) =
          *reinterpret_cast<const uint4*>(sO + t * 128 + ((c ^ (t & 15)) * 8));
  }
}

int launch_lin(const LinArgs& a, hipStream_t st) {
  const int n_ut = static_cast<int>(ceil_div(a.N, 128));
  const int64_t n_mt = ceil_div(a.M, 128);
  const int64_t blocks = ceil_div(n_mt, kXcds) * kXcds * n_ut;
  if (blocks > 0x7fffffffLL) DLLAVA_FAIL(DLLAVA_ESHAPE, "predict: too many rows");
  hipLaunchKernelGGL(lin_gemm_kernel, dim3(static_cast<unsigned>(blocks)), dim3(kGThreads), 0, st, a, n_ut);
  DLLAVA_CHECK_LAUNCH("lin_gemm_kernel");
  return DLLAVA_OK;
}

// LayerNorm over rows of 512: lane holds 8 consecutive elements; mean and biased variance in two passes over the
// registers.
__global__ __launch_bounds__(256) void ln_kernel(const bf16_t* __restrict__ Z, bf16_t* __restrict__ Y,
                                                 const float* __restrict__ gam, const float* __restrict__ bet,
                                                 int64_t M) {
  const int lane = threadIdx.x & (kWave - 1), w = threadIdx.x / kWave;
  const int64_t row = static_cast<int64_t>(blockIdx.x) * 4 + w;
  if (row >= M) return;
  const uint4 raw = *reinterpret_cast<const uint4*>(Z + row * kPW + lane * 8);
  float v[8];
  Elem<bf16_t>::unpack(raw, v);
  float s = 0.f;
#pragma unroll
  for (int e = 0; e < 8; ++e) s += v[e];
  const float mean = wave_sum(s) * (1.f / kPW);
  float ss = 0.f;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    v[e] -= mean;
    ss = fmaf(v[e], v[e], ss);
  }
  const float rstd = 1.f / sqrtf(wave_sum(ss) * (1.f / kPW) + kLnEps);
  // scale and shift: two 16-byte loads each (eight scalar loads per vector would touch every cache line of the
  // vector eight times per wave); a missing vector reads as ones / zeros
  float gm[8], bt[8];
  if (gam) {
    *reinterpret_cast<float4*>(gm) = *reinterpret_cast<const float4*>(gam + lane * 8);
    *reinterpret_cast<float4*>(gm + 4) = *reinterpret_cast<const float4*>(gam + lane * 8 + 4);
  } else {
#pragma unroll
    for (int e = 0; e < 8; ++e) gm[e] = 1.f;
  }
  if (bet) {
    *reinterpret_cast<float4*>(bt) = *reinterpret_cast<const float4*>(bet + lane * 8);
    *reinterpret_cast<float4*>(bt + 4) = *reinterpret_cast<const float4*>(bet + lane * 8 + 4);
  } else {
#pragma unroll
    for (int e = 0; e < 8; ++e) bt[e] = 0.f;
  }
  float y[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) y[e] = fmaf(v[e] * rstd, gm[e], bt[e]);
  uint4 o;
  o.x = pack_bf16x2(y[0], y[1]);
  o.y = pack_bf16x2(y[2], y[3]);
  o.z = pack_bf16x2(y[4], y[5]);
  o.w = pack_bf16x2(y[6], y[7]);
  *reinterpret_cast<uint4*>(Y + row * kPW + lane * 8) = o;
}

// last layer of the head: D[m] = h[m] W^T + b, h [M, 128], W [2, 128]; one wave per row, lane holds two inputs
__global__ __launch_bounds__(256) void head_out_kernel(const bf16_t* __restrict__ Hd, const bf16_t* __restrict__ W,
                                                       const float* __restrict__ b, float* __restrict__ logits,
                                                       int64_t M, const int32_t* __restrict__ span_off, int32_t B) {
  const int lane = threadIdx.x & (kWave - 1), w = threadIdx.x / kWave;
  const int64_t row = static_cast<int64_t>(blockIdx.x) * 4 + w;
  const int64_t total = span_off ? span_off[B] : M;  // rows beyond the spans are left untouched
  if (row >= M || row >= total) return;
  const uint32_t x = *reinterpret_cast<const uint32_t*>(Hd + row * kPH2 + lane * 2);
  const uint32_t w0 = *reinterpret_cast<const uint32_t*>(W + lane * 2);
  const uint32_t w1 = *reinterpret_cast<const uint32_t*>(W + kPH2 + lane * 2);
  const float x0 = bf16lo_to_f32(x), x1 = bf16hi_to_f32(x);
  float p0 = fmaf(x1, bf16hi_to_f32(w0), x0 * bf16lo_to_f32(w0));
  float p1 = fmaf(x1, bf16hi_to_f32(w1), x0 * bf16lo_to_f32(w1));
  p0 = wave_sum(p0);
  p1 = wave_sum(p1);
  if (lane == 0) {
    logits[2 * row] = p0 + (b ? b[0] : 0.f);
    logits[2 * row + 1] = p1 + (b ? b[1] : 0.f);
  }
}

// span_off[b] = sum of the span lengths before b (one wave; B+1 entries); without spans: {0, M}
__global__ __launch_bounds__(kWave) void span_offsets_kernel(const int32_t* __restrict__ vis_len, int32_t B, int64_t M,
                                                             int32_t* __restrict__ span_off) {
  const int lane = threadIdx.x;
  if (!vis_len) {
    if (lane == 0) {
      span_off[0] = 0;
      span_off[1] = static_cast<int32_t>(M);
    }
    return;
  }
  int carry = 0;
  if (lane == 0) span_off[0] = 0;
  for (int base = 0; base < B; base += kWave) {
    const int i = base + lane;
    int n = i < B ? vis_len[i] : 0;
    if (n < 0) n = 0;
    const int incl = wave_incl_scan(n);
    if (i < B) span_off[i + 1] = carry + incl;
    carry += __shfl(incl, kWave - 1, kWave);
  }
}


// ---- the output-text predictor on a handful of rows (one per sequence and decode step) ---------------------------
// With at most 64 rows the tile kernel above would pull the 2*512*d bytes of W_in through four compute units.
// small_in_kernel spreads W_in over 64 blocks of 4 waves: block = 32 output features x a quarter of d, wave = a
// sixteenth of d (every byte of W_in is read once, all loads of a wave in flight together), the four waves summed
// through LDS in wave order, one partial per block.  small_head_kernel (one block per 32 rows) adds the four
// partials and the bias in a fixed order, rounds the 512 features to the storage type into LDS, and runs the head
// 512 -> 256 -> 128 -> 2 from there on the matrix cores, the weights of both layers requested at its very start.
constexpr int kSmallRows = 64;
constexpr int kSmallSplit = 4;    // blocks along d
constexpr int kZs = 520, kH1s = 264, kH2s = 136;  // LDS row strides (elements): 16-byte pieces of 16 rows fall in 16 bank groups

// Register-to-LDS order inside ONE wave: the area written and read is private to the wave and the wave's LDS
// instructions execute in order; the fences only keep the compiler from moving them across one another.
__device__ __forceinline__ void wave_lds_order() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}
__device__ __forceinline__ void want_now(const uint4& v) { asm volatile("" ::"v"(v.x), "v"(v.y), "v"(v.z), "v"(v.w)); }

// Operands are loaded 8 lanes per 128-byte line (a load instruction then touches 8 whole lines; a fragment-shaped
// load, one row per lane, touches 32 lines for the same bytes and was measured 4x slower here) and turned into
// matrix-core fragments through a wave-private LDS area in the swizzled row-major form of gemm_tile.h: chunk c of
// row rr at chunk position c ^ ((rr / 2) % 8).
//
// few_accumulate: one wave's share of a product on few rows.  wrow[j] / xrow[tt][j]: this lane's 16-byte column
// (8 * (lane % 8) elements into a 128-byte line) of weight row 8j + lane/8 of the block's 32 features and of input
// row 8j + lane/8 of row tile tt; lines lbeg .. lend-1 of the input width, LB lines of every row requested together.
// Result: acc[tt] register i of lane = feature 8*(i/4) + 4*(lane/32) + i%4 of input row 32*tt + lane%32.
template <int NT, int LB, bool HALF = false>  // HALF: only weight rows 0..15 exist (features 16..31 of the result are zero)
__device__ __forceinline__ void few_accumulate(const bf16_t* const (&wrow)[4], const bf16_t* const (&xrow)[NT][4], int lbeg,
                                               int lend, bf16_t* sw, int lane, f32x16 (&acc)[NT], int jx = 4) {
  // jx (uniform): row groups of 8 of the LAST row tile that hold input rows; the others are neither loaded nor
  // staged: they are zeroed once, like the absent weight rows of HALF, and feed result entries nobody reads
  const int r = lane & 31, g = lane >> 5;
  const int lr8 = lane >> 3, lc = lane & 7;
  bf16_t* sx = sw + 32 * 64;
  const int st_off = lr8 * 64 + ((lc ^ ((lr8 >> 1) & 3)) * 8);  // row 8j + lane/8: ((8j + lr8) / 2) % 8 = 4*(j%2) + lr8/2
  const int fr_off = r * 64 + ((g ^ ((r >> 1) & 7)) * 8);       // row r, chunk 2*step + g
  if (HALF || jx < 4) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int o = 8 * j * 64 + (st_off ^ ((j & 1) * 32));
      if (HALF && j >= 2) *reinterpret_cast<uint4*>(sw + o) = uint4{0u, 0u, 0u, 0u};
      if (j >= jx) *reinterpret_cast<uint4*>(sx + (NT - 1) * 32 * 64 + o) = uint4{0u, 0u, 0u, 0u};
    }
  }
  for (int l0 = lbeg; l0 < lend; l0 += LB) {
    constexpr int JW = HALF ? 2 : 4;
    uint4 wf[LB][JW], xf[NT][LB][4];  // [line of the batch][row group j]
#pragma unroll
    for (int c = 0; c < LB; ++c) {  // all loads of the batch first (past the end: the last line again, unused)
      const int line = l0 + c < lend ? l0 + c : lend - 1;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        if (j < JW) wf[c][j] = *reinterpret_cast<const uint4*>(wrow[j] + 64 * line);
#pragma unroll
        for (int tt = 0; tt < NT; ++tt)
          xf[tt][c][j] = (tt < NT - 1 || j < jx) ? *reinterpret_cast<const uint4*>(xrow[tt][j] + 64 * line) : uint4{0u, 0u, 0u, 0u};
      }
    }
#pragma unroll
    for (int c = 0; c < LB; ++c)
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        if (j < JW) want_now(wf[c][j]);
#pragma unroll
        for (int tt = 0; tt < NT; ++tt) want_now(xf[tt][c][j]);
      }
#pragma unroll
    for (int c = 0; c < LB; ++c)
      if (l0 + c < lend) {  // wave-uniform
        wave_lds_order();
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const int o = 8 * j * 64 + (st_off ^ ((j & 1) * 32));
          if (j < JW) *reinterpret_cast<uint4*>(sw + o) = wf[c][j];
#pragma unroll
          for (int tt = 0; tt < NT; ++tt)
            if (tt < NT - 1 || j < jx) *reinterpret_cast<uint4*>(sx + tt * 32 * 64 + o) = xf[tt][c][j];
        }
        wave_lds_order();
#pragma unroll
        for (int sk = 0; sk < 4; ++sk) {
          const bf16x8 fa = as_frag(*reinterpret_cast<const uint4*>(sw + (fr_off ^ (sk * 16))));
#pragma unroll
          for (int tt = 0; tt < NT; ++tt)
            acc[tt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                fa, as_frag(*reinterpret_cast<const uint4*>(sx + tt * 32 * 64 + (fr_off ^ (sk * 16)))), acc[tt], 0, 0, 0);
        }
      }
  }
}

// Leaves the wave's sums in its own staging area as float32 [(16*tt + i) * 64 + lane].
template <int NT>
__device__ __forceinline__ void few_leave_sums(const f32x16 (&acc)[NT], bf16_t* sw, int lane) {
  static_assert(NT * 16 * kWave * sizeof(float) <= (1 + NT) * 32 * 64 * sizeof(bf16_t), "a wave's sums fit its own area");
  wave_lds_order();  // the wave's last fragment reads come before its sums go to the same area
  float* mine = reinterpret_cast<float*>(sw);
#pragma unroll
  for (int tt = 0; tt < NT; ++tt)
#pragma unroll
    for (int i = 0; i < 16; ++i) mine[(tt * 16 + i) * kWave + lane] = acc[tt][i];
}

// First layer of the output-text predictor: block = feature group fg (32 of the 512 features) x part kq of the input
// width (each cut again over the block's 4 waves); partial sums [KQ][32*NT rows][N] float32 for small_head_kernel.
template <int NT>  // tiles of 32 rows
__global__ __launch_bounds__(256) void small_in_kernel(const bf16_t* __restrict__ X, int64_t ldx, int M, int K,
                                                       const bf16_t* __restrict__ W, float* __restrict__ partial,
                                                       int32_t B, const int32_t* __restrict__ seq_off,
                                                       const int32_t* __restrict__ vis_start,
                                                       const int32_t* __restrict__ vis_len, int n_fg, int KQ, int N) {
  // per wave: 32 weight rows and 32*NT input rows x 64 elements; after its last line a wave's area carries its sums
  __shared__ __align__(16) bf16_t stage[4][(1 + NT) * 32 * 64];
  const int tid = threadIdx.x, lane = tid & (kWave - 1), w = tid / kWave;
  const int fg = blockIdx.x % n_fg, kq = blockIdx.x / n_fg;
  const int r = lane & 31, g = lane >> 5;
  const int lr8 = lane >> 3, lc = lane & 7;
  const int total = K / 64;                        // 128-byte lines per row
  const int per = (total + 4 * KQ - 1) / (4 * KQ); // lines of one wave (4*KQ slices of the input width)
  const int lbeg = (kq * 4 + w) * per;
  const int lend = lbeg + per < total ? lbeg + per : total;
  const bf16_t* wrow[4];
  const bf16_t* xrow[NT][4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    wrow[j] = W + static_cast<int64_t>(32 * fg + 8 * j + lr8) * K + 8 * lc;
#pragma unroll
    for (int tt = 0; tt < NT; ++tt) {
      int64_t m = 32 * tt + 8 * j + lr8;
      if (m >= M) m = M - 1;  // rows past M repeat the last one and are dropped later
      int64_t sr = score_src_row(seq_off, vis_start, vis_len, B, m);
      if (sr < 0) sr = 0;
      xrow[tt][j] = X + sr * ldx + 8 * lc;
    }
  }
  f32x16 acc[NT];
#pragma unroll
  for (int tt = 0; tt < NT; ++tt)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[tt][i] = 0.f;
  few_accumulate<NT, 4>(wrow, xrow, lbeg, lend, stage[w], lane, acc);
  if (w > 0) few_leave_sums<NT>(acc, stage[w], lane);
  __syncthreads();
  if (w != 0) return;
  const float* red1 = reinterpret_cast<const float*>(stage[1]);
  const float* red2 = reinterpret_cast<const float*>(stage[2]);
  const float* red3 = reinterpret_cast<const float*>(stage[3]);
  // lane: row 32*tt + r; register i: feature 32*fg + 8*(i/4) + 4*g + i%4
#pragma unroll
  for (int tt = 0; tt < NT; ++tt)
#pragma unroll
    for (int q4 = 0; q4 < 4; ++q4) {
      float4 v;
      float* pv = &v.x;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int i = 4 * q4 + e, o = (tt * 16 + i) * kWave + lane;
        pv[e] = ((acc[tt][i] + red1[o]) + red2[o]) + red3[o];
      }
      if (32 * tt + r < M)  // rows past M were copies of the last one
        *reinterpret_cast<float4*>(partial + (static_cast<int64_t>(kq * (32 * NT) + 32 * tt + r)) * N + 32 * fg +
                                   8 * q4 + 4 * g) = v;
    }
}

// ---- a linear layer of the decoder on few rows (one row per sequence of a decode step), whole in one launch --------
// The weights are the traffic (the rows are few): block = 32 output features x part kq of the input width, cut again
// over the block's 4 or 8 waves, every weight byte read once.  The waves' sums meet in LDS; with KQ > 1 the blocks
// of one feature group hand their sums over through the workspace and a device-scope counter, and the last one to
// arrive adds them in part order (fixed order: bit-reproducible), so the epilogue runs in the same launch:
//   kFewPlain  y = act(x W^T + bias) (+ residual | * SiLU(gate rows));
//   kFewQkv    [q | k | v] = x [Wq | Wk | Wv]^T with the rotary rotation of q and k: a q/k block takes 16 features of
//              the lower half of a head and their 16 partners of the upper half, so a pair sits in one thread;
//   kFewGated  y = (x Wu^T) * SiLU(x Wg^T): a block takes 16 gate features and the same 16 up features.
//   kFewPlainHalf  kFewPlain with 16 features per block and 8 waves along the input width: for a narrow output
//              (N up to 4096: at most one such block per compute unit) there are then enough blocks without cutting
//              the input width across blocks, whose hand-over costs about 5 us; the upper half of the matrix-core
//              tile idles, which costs nothing here, but every block reads all input rows: twice the input traffic.
//   kFewPlain8 kFewPlain with 8 waves along the input width: the outputs between those and the wide ones.
// In all of them a thread of the epilogue owns block-local features 8*q4 + 4*g + e ("lo") and 16 + the same ("hi",
// absent in kFewPlainHalf), e = 0..3, of one row.
enum { kFewPlain = 0, kFewQkv = 1, kFewGated = 2, kFewPlainHalf = 3, kFewPlain8 = 4 };
constexpr int kFewBatch = 2;     // 128-byte lines per row in flight per wave (2: about 110 registers; 4 measured 7 % slower)
constexpr int kFewBlocks = 384;  // blocks aimed at (more measured slower: the launch is bound by its ramp and memory)
constexpr size_t kFewCounterBytes = 4096;

struct FewEpi {
  float* partial;     // [KQ][32*NT][32 * n_fg] block-local feature order
  int32_t* counters;  // one per feature group, zero between launches
  const float* bias;  // plain
  int act;
  const bf16_t* R;
  bf16_t* Y;          // plain, gated
  int64_t ldy;
  int H, Dh;          // qkv
  const int32_t* pos;
  double rope_ratio;  // base^(-2/Dh)
  bf16_t *q, *k, *v;
};

// waves of a block, each with its own part of the input width (8 for q|k|v or gate|up measured 3-10 % slower than 4)
template <int EPI>
constexpr int few_waves() { return (EPI == kFewPlainHalf || EPI == kFewPlain8) ? 8 : 4; }
template <int NT, int EPI>
__global__ __launch_bounds__(64 * few_waves<EPI>()) void few_fused_kernel(const bf16_t* __restrict__ X, int64_t ldx, int M, int K,
                                                        const bf16_t* __restrict__ W0, const bf16_t* __restrict__ W1,
                                                        const bf16_t* __restrict__ W2, int n_fg, int KQ, int fg_each,
                                                        FewEpi ep) {
  constexpr bool HALF = EPI == kFewPlainHalf;
  constexpr int NW = few_waves<EPI>();
  constexpr int FB = HALF ? 16 : 32; // features of a block
  __shared__ __align__(16) bf16_t stage[NW][(1 + NT) * 32 * 64];
  __shared__ int sm_last;
  const int tid = threadIdx.x, lane = tid & (kWave - 1), w = tid / kWave;
  const int fg = blockIdx.x % n_fg, kq = blockIdx.x / n_fg;
  const int lr8 = lane >> 3, lc = lane & 7;
  const int total = K / 64;
  const int per = (total + NW * KQ - 1) / (NW * KQ);
  const int lbeg = (kq * NW + w) * per;
  const int lend = lbeg + per < total ? lbeg + per : total;
  // which matrix and which of its rows the block's 32 features are
  const int which = EPI == kFewQkv ? fg / fg_each : 0, lf = EPI == kFewQkv ? fg % fg_each : fg;
  const int half = ep.Dh / 2, per_head = EPI == kFewQkv ? ep.Dh / 32 : 1;
  const int head = lf / per_head, t16 = lf % per_head;
  const bf16_t* wrow[4];
  const bf16_t* xrow[NT][4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int f = 8 * j + lr8;
    const bf16_t* Wm = W0;
    int64_t row = 32 * static_cast<int64_t>(fg) + f;
    if (HALF) {
      row = 16 * static_cast<int64_t>(fg) + (f & 15);
    } else if (EPI == kFewQkv) {
      Wm = which == 0 ? W0 : (which == 1 ? W1 : W2);
      row = which < 2 ? static_cast<int64_t>(head) * ep.Dh + 16 * t16 + (f & 15) + (f >> 4) * half
                      : 32 * static_cast<int64_t>(lf) + f;
    } else if (EPI == kFewGated) {
      Wm = f < 16 ? W0 : W1;
      row = 16 * static_cast<int64_t>(fg) + (f & 15);
    }
    wrow[j] = Wm + row * K + 8 * lc;
#pragma unroll
    for (int tt = 0; tt < NT; ++tt) {
      int m = 32 * tt + f;
      if (m >= M) m = M - 1;  // rows past M repeat the last one and are dropped later
      xrow[tt][j] = X + static_cast<int64_t>(m) * ldx + 8 * lc;
    }
  }
  f32x16 acc[NT];
#pragma unroll
  for (int tt = 0; tt < NT; ++tt)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[tt][i] = 0.f;
  few_accumulate<NT, kFewBatch, HALF>(wrow, xrow, lbeg, lend, stage[w], lane, acc, (M - 32 * (NT - 1) + 7) / 8);
  few_leave_sums<NT>(acc, stage[w], lane);
  __syncthreads();

  // epilogue thread: row m, block-local features lo = 8*q4 + 4*g + e and hi = 16 + lo
  const bool has = tid < 128 * NT;
  const int r = tid & 31, g = (tid >> 5) & 1, q4 = (tid >> 6) & 1, tt = (tid >> 7) & (NT - 1);
  const int m = 32 * tt + r, f0 = 8 * q4 + 4 * g;
  const bool live = has && m < M;
  float lo[4], hi[4];
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const int o = (tt * 16 + 4 * q4 + e) * kWave + g * 32 + r;
    lo[e] = hi[e] = 0.f;
#pragma unroll
    for (int ww = 0; ww < NW; ++ww) {  // wave order
      const float* sums = reinterpret_cast<const float*>(stage[ww]);
      lo[e] += sums[o];
      if (!HALF) hi[e] += sums[o + 8 * kWave];
    }
  }
  if (KQ > 1) {  // uniform over the launch
    const int64_t cols = FB * static_cast<int64_t>(n_fg);
    float* mine = ep.partial + (static_cast<int64_t>(kq) * (32 * NT) + m) * cols + FB * fg + f0;
    if (live) {
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        st_agent(mine + e, lo[e]);
        if (!HALF) st_agent(mine + 16 + e, hi[e]);
      }
    }
    block_publish();
    if (tid == 0) sm_last = (add_agent(&ep.counters[fg], 1) == KQ - 1);
    __syncthreads();
    if (!sm_last) return;
    if (live) {
#pragma unroll
      for (int e = 0; e < 4; ++e) lo[e] = hi[e] = 0.f;
      for (int p = 0; p < KQ; ++p) {
        const float* src = ep.partial + (static_cast<int64_t>(p) * (32 * NT) + m) * cols + FB * fg + f0;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          lo[e] += ld_agent(src + e);
          if (!HALF) hi[e] += ld_agent(src + 16 + e);
        }
      }
    }
    if (tid == 0) zero_agent(&ep.counters[fg]);
  }
  if (!live) return;

  if (EPI == kFewPlain || EPI == kFewPlain8 || HALF) {
#pragma unroll
    for (int hf = 0; hf < (HALF ? 1 : 2); ++hf) {
      float* v = hf ? hi : lo;
      const int64_t f = FB * static_cast<int64_t>(fg) + 16 * hf + f0;
      if (ep.bias) {
        const float4 bb = *reinterpret_cast<const float4*>(ep.bias + f);
        v[0] += bb.x; v[1] += bb.y; v[2] += bb.z; v[3] += bb.w;
      }
      if (ep.act == 1) {
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = gelu_erf_fast(v[e]);
      }
      if (ep.R) {
        const uint2 rr = *reinterpret_cast<const uint2*>(ep.R + m * ep.ldy + f);
        const float r0 = bf16lo_to_f32(rr.x), r1 = bf16hi_to_f32(rr.x), r2 = bf16lo_to_f32(rr.y), r3 = bf16hi_to_f32(rr.y);
        if (ep.act == 2) {
          v[0] *= silu_fast(r0); v[1] *= silu_fast(r1); v[2] *= silu_fast(r2); v[3] *= silu_fast(r3);
        } else {
          v[0] += r0; v[1] += r1; v[2] += r2; v[3] += r3;
        }
      }
      uint2 o;
      o.x = pack_bf16x2(v[0], v[1]);
      o.y = pack_bf16x2(v[2], v[3]);
      *reinterpret_cast<uint2*>(ep.Y + m * ep.ldy + f) = o;
    }
  } else if (EPI == kFewQkv) {
    const int64_t HD = static_cast<int64_t>(ep.H) * ep.Dh;
    bf16_t* out = (which == 0 ? ep.q : (which == 1 ? ep.k : ep.v)) + m * HD;
    int64_t at_lo, at_hi;
    if (which < 2) {  // uniform over the block
      const int i4 = 16 * t16 + f0;  // index into the lower half of the head
      // angle of pair i: pos * ratio^i with ratio = base^(-2/Dh), in float64 and in turns; only its fraction
      // goes to the float32 sine and cosine (absolute error about 1e-6, far below the step of the storage type)
      double freq = 1.0, sq = ep.rope_ratio;
      for (int n = i4; n > 0; n >>= 1, sq *= sq)
        if (n & 1) freq *= sq;
      const double turns0 = static_cast<double>(ep.pos[m]) * 0.15915494309189535;  // pos / (2 pi)
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        double tn = turns0 * freq;
        tn -= rint(tn);
        const float cs = __builtin_amdgcn_cosf(static_cast<float>(tn)), sn = __builtin_amdgcn_sinf(static_cast<float>(tn));
        const float a = lo[e], b = hi[e];
        lo[e] = a * cs - b * sn;
        hi[e] = b * cs + a * sn;
        freq *= ep.rope_ratio;
      }
      at_lo = static_cast<int64_t>(head) * ep.Dh + i4;
      at_hi = at_lo + half;
    } else {
      at_lo = 32 * static_cast<int64_t>(lf) + f0;
      at_hi = at_lo + 16;
    }
    uint2 w0, w1;
    w0.x = pack_bf16x2(lo[0], lo[1]); w0.y = pack_bf16x2(lo[2], lo[3]);
    w1.x = pack_bf16x2(hi[0], hi[1]); w1.y = pack_bf16x2(hi[2], hi[3]);
    *reinterpret_cast<uint2*>(out + at_lo) = w0;
    *reinterpret_cast<uint2*>(out + at_hi) = w1;
  } else {  // gated: lo = gate (rounded to the storage type first, as if stored), hi = up
    float gte[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) gte[e] = bf16_to_f32(f32_to_bf16(lo[e]));
    uint2 o;
    o.x = pack_bf16x2(hi[0] * silu_fast(gte[0]), hi[1] * silu_fast(gte[1]));
    o.y = pack_bf16x2(hi[2] * silu_fast(gte[2]), hi[3] * silu_fast(gte[3]));
    *reinterpret_cast<uint2*>(ep.Y + m * ep.ldy + 16 * static_cast<int64_t>(fg) + f0) = o;
  }
}

template <int EPI>
void launch_few_fused(int nt, hipStream_t st, const bf16_t* X, int64_t ldx, int M, int K, const bf16_t* W0, const bf16_t* W1,
                      const bf16_t* W2, int n_fg, int KQ, int fg_each, const FewEpi& ep) {
  const dim3 grid(static_cast<unsigned>(n_fg) * static_cast<unsigned>(KQ)), block(64 * few_waves<EPI>());
  if (nt == 1)
    hipLaunchKernelGGL((few_fused_kernel<1, EPI>), grid, block, 0, st, X, ldx, M, K, W0, W1, W2, n_fg, KQ, fg_each, ep);
  else
    hipLaunchKernelGGL((few_fused_kernel<2, EPI>), grid, block, 0, st, X, ldx, M, K, W0, W1, W2, n_fg, KQ, fg_each, ep);
}

__global__ __launch_bounds__(256) void small_head_kernel(const float* __restrict__ partial, int rows_pad, int M,
                                                         const float* __restrict__ b_in,
                                                         const bf16_t* __restrict__ W1, const float* __restrict__ b1,
                                                         const bf16_t* __restrict__ W2, const float* __restrict__ b2,
                                                         const bf16_t* __restrict__ W3, const float* __restrict__ b3,
                                                         float* __restrict__ logits,
                                                         const int32_t* __restrict__ span_off, int32_t B) {
  __shared__ __align__(16) bf16_t zT[32 * kZs];
  __shared__ __align__(16) bf16_t h1T[32 * kH1s];
  __shared__ __align__(16) bf16_t h2T[32 * kH2s];
  __shared__ __align__(16) bf16_t stage[4][64 * 64];  // per wave: 64 weight rows x 64 elements
  __shared__ float w3s[2 * kPH2];
  const int tid = threadIdx.x, lane = tid & (kWave - 1), w = tid / kWave;
  const int r = lane & 31, g = lane >> 5;
  const int lr8 = lane >> 3, lc = lane & 7;
  const int t0 = blockIdx.x * 32;
  const bf16_t w3v = W3[tid];  // last layer's 2 x 128 weights: one per thread, into LDS before the first barrier
  // The weights of both layers, requested before anything else: wave w owns features 64w..64w+63 of the first layer
  // and 32w..32w+31 of the second.  Register [j][c] of a lane: row 8j + lane/8 of the wave's rows, elements
  // 64c + 8*(lane%8) .. +7.
  uint4 w1r[8][8], w2r[4][4];
#pragma unroll
  for (int j = 0; j < 8; ++j)
#pragma unroll
    for (int c = 0; c < 8; ++c)
      w1r[j][c] = *reinterpret_cast<const uint4*>(W1 + static_cast<int64_t>(64 * w + 8 * j + lr8) * kPW + 64 * c + 8 * lc);
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int c = 0; c < 4; ++c)
      w2r[j][c] = *reinterpret_cast<const uint4*>(W2 + static_cast<int64_t>(32 * w + 8 * j + lr8) * kPH1 + 64 * c + 8 * lc);
  // z = bias + the partial sums, in a fixed order, rounded to the storage type: rows of this tile that exist only
  // (the others stay undefined in LDS: a row only ever influences its own outputs, which are dropped), four
  // items per thread at a time; the loads of the first four are issued together with the weights.
  const int n_valid = M - t0 < 32 ? M - t0 : 32;
  const int items = n_valid * (kPW / 4);
  float4 sum[4], pq[4][kSmallSplit];
  auto z_load = [&](int base) {
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      int it = base + 256 * u + tid;
      if (it >= items) it = items - 1;
      const int tok = it / (kPW / 4), f = (it % (kPW / 4)) * 4;
      sum[u] = *reinterpret_cast<const float4*>(b_in ? b_in + f : kZeroWords);
#pragma unroll
      for (int q = 0; q < kSmallSplit; ++q)
        pq[u][q] = *reinterpret_cast<const float4*>(partial + static_cast<int64_t>(q * rows_pad + t0 + tok) * kPW + f);
    }
  };
  auto z_finish = [&](int base) {
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int it = base + 256 * u + tid;
      if (it < items) {
        const int tok = it / (kPW / 4), f = (it % (kPW / 4)) * 4;
#pragma unroll
        for (int q = 0; q < kSmallSplit; ++q) {
          sum[u].x += pq[u][q].x; sum[u].y += pq[u][q].y; sum[u].z += pq[u][q].z; sum[u].w += pq[u][q].w;
        }
        uint2 v;
        v.x = pack_bf16x2(sum[u].x, sum[u].y);
        v.y = pack_bf16x2(sum[u].z, sum[u].w);
        *reinterpret_cast<uint2*>(zT + tok * kZs + f) = v;
      }
    }
  };
  z_load(0);
  // The weights are wanted in registers HERE, all loads of a lane in flight together: without a use at this point
  // the compiler moves each load down to its slice of the product, one memory round trip per slice.
#pragma unroll
  for (int j = 0; j < 8; ++j)
#pragma unroll
    for (int c = 0; c < 8; ++c) want_now(w1r[j][c]);
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int c = 0; c < 4; ++c) want_now(w2r[j][c]);
  w3s[tid] = bf16_to_f32(w3v);
  z_finish(0);
  for (int base = 4 * 256; base < items; base += 4 * 256) {
    z_load(base);
    z_finish(base);
  }
  __syncthreads();
  bf16_t* st = stage[w];
  const int st_off = lr8 * 64 + ((lc ^ ((lr8 >> 1) & 3)) * 8);  // row 8j + lane/8: ((8j + lr8) / 2) % 8 = 4*(j%2) + lr8/2
  const int fr_off = r * 64 + ((g ^ ((r >> 1) & 7)) * 8);       // row r (+32), chunk 2s + g
  {  // h1 = GELU(W1 z + b1): two 32-feature tiles per wave
    f32x16 a0, a1;
#pragma unroll
    for (int i = 0; i < 16; ++i) a0[i] = a1[i] = 0.f;
    const bf16_t* zb = zT + r * kZs + 8 * g;
#pragma unroll
    for (int c = 0; c < 8; ++c) {
      wave_lds_order();
#pragma unroll
      for (int j = 0; j < 8; ++j)
        *reinterpret_cast<uint4*>(st + 8 * j * 64 + (st_off ^ ((j & 1) * 32))) = w1r[j][c];
      wave_lds_order();
#pragma unroll
      for (int sk = 0; sk < 4; ++sk) {
        const bf16x8 bz = as_frag(*reinterpret_cast<const uint4*>(zb + 64 * c + 16 * sk));
        const bf16x8 fa = as_frag(*reinterpret_cast<const uint4*>(st + (fr_off ^ (sk * 16))));
        const bf16x8 fb = as_frag(*reinterpret_cast<const uint4*>(st + 32 * 64 + (fr_off ^ (sk * 16))));
        a0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, bz, a0, 0, 0, 0);
        a1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb, bz, a1, 0, 0, 0);
      }
    }
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        const int f = 64 * w + 32 * i + 8 * q4 + 4 * g;
        const float4 bs = *reinterpret_cast<const float4*>(b1 ? b1 + f : kZeroWords);
        const f32x16& a = i ? a1 : a0;
        uint2 v;
        v.x = pack_bf16x2(gelu_erf_fast(a[4 * q4] + bs.x), gelu_erf_fast(a[4 * q4 + 1] + bs.y));
        v.y = pack_bf16x2(gelu_erf_fast(a[4 * q4 + 2] + bs.z), gelu_erf_fast(a[4 * q4 + 3] + bs.w));
        *reinterpret_cast<uint2*>(h1T + r * kH1s + f) = v;
      }
  }
  __syncthreads();
  {  // h2 = GELU(W2 h1 + b2): one 32-feature tile per wave
    f32x16 a;
#pragma unroll
    for (int i = 0; i < 16; ++i) a[i] = 0.f;
    const bf16_t* hb = h1T + r * kH1s + 8 * g;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      wave_lds_order();
#pragma unroll
      for (int j = 0; j < 4; ++j)
        *reinterpret_cast<uint4*>(st + 8 * j * 64 + (st_off ^ ((j & 1) * 32))) = w2r[j][c];
      wave_lds_order();
#pragma unroll
      for (int sk = 0; sk < 4; ++sk) {
        const bf16x8 bh = as_frag(*reinterpret_cast<const uint4*>(hb + 64 * c + 16 * sk));
        const bf16x8 fa = as_frag(*reinterpret_cast<const uint4*>(st + (fr_off ^ (sk * 16))));
        a = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, bh, a, 0, 0, 0);
      }
    }
#pragma unroll
    for (int q4 = 0; q4 < 4; ++q4) {
      const int f = 32 * w + 8 * q4 + 4 * g;
      const float4 bs = *reinterpret_cast<const float4*>(b2 ? b2 + f : kZeroWords);
      uint2 v;
      v.x = pack_bf16x2(gelu_erf_fast(a[4 * q4] + bs.x), gelu_erf_fast(a[4 * q4 + 1] + bs.y));
      v.y = pack_bf16x2(gelu_erf_fast(a[4 * q4 + 2] + bs.z), gelu_erf_fast(a[4 * q4 + 3] + bs.w));
      *reinterpret_cast<uint2*>(h2T + r * kH2s + f) = v;
    }
  }
  __syncthreads();
  {  // the two logits of a row: four threads sum a quarter of the 128 inputs each, combined in a fixed order
    const int out = tid >> 2, part = tid & 3, tok = out >> 1, c = out & 1;
    const int64_t m = t0 + tok;
    const int64_t lim = span_off ? span_off[B] : M;
    float ps = 0.f;
#pragma unroll
    for (int k = 32 * part; k < 32 * part + 32; ++k) ps = fmaf(bf16_to_f32(h2T[tok * kH2s + k]), w3s[c * kPH2 + k], ps);
    const int l0 = lane & ~3;
    const float p0 = __shfl(ps, l0, kWave), p1 = __shfl(ps, l0 + 1, kWave), p2 = __shfl(ps, l0 + 2, kWave),
                p3 = __shfl(ps, l0 + 3, kWave);
    if (part == 0 && m < M && m < lim) logits[2 * m + c] = ((((b3 ? b3[c] : 0.f) + p0) + p1) + p2) + p3;
  }
}

// RMSNorm of d-wide rows: y = x / sqrt(mean(x^2) + eps) * w.  One wave per row, the row held in registers
// (16-byte pieces, lane-strided: up to 16 pieces = 8192 elements), sum of squares in float32.
constexpr int kRmsMaxPieces = 16;
__global__ __launch_bounds__(256) void rms_norm_kernel(const bf16_t* __restrict__ X, int64_t ldx, bf16_t* __restrict__ Y,
                                                       int64_t ldy, const float* __restrict__ wgt, int64_t M, int d,
                                                       float eps) {
  const int lane = threadIdx.x & (kWave - 1), w = threadIdx.x / kWave;
  const int64_t row = static_cast<int64_t>(blockIdx.x) * 4 + w;
  if (row >= M) return;
  const int pieces = (d / 8 + kWave - 1) / kWave;  // per lane
  uint4 raw[kRmsMaxPieces];
  const bf16_t* x = X + row * ldx;
#pragma unroll
  for (int c = 0; c < kRmsMaxPieces; ++c) {
    const int col = (c * kWave + lane) * 8;
    raw[c] = (c < pieces && col < d) ? *reinterpret_cast<const uint4*>(x + col) : uint4{0u, 0u, 0u, 0u};
  }
  float ss = 0.f;
#pragma unroll
  for (int c = 0; c < kRmsMaxPieces; ++c) {
    float v[8];
    Elem<bf16_t>::unpack(raw[c], v);
#pragma unroll
    for (int e = 0; e < 8; ++e) ss = fmaf(v[e], v[e], ss);
  }
  const float rs = 1.f / sqrtf(wave_sum(ss) / static_cast<float>(d) + eps);
  bf16_t* y = Y + row * ldy;
#pragma unroll
  for (int c = 0; c < kRmsMaxPieces; ++c) {
    const int col = (c * kWave + lane) * 8;
    if (c < pieces && col < d) {
      float v[8], g[8];
      Elem<bf16_t>::unpack(raw[c], v);
      if (wgt) {
        *reinterpret_cast<float4*>(g) = *reinterpret_cast<const float4*>(wgt + col);
        *reinterpret_cast<float4*>(g + 4) = *reinterpret_cast<const float4*>(wgt + col + 4);
      } else {
#pragma unroll
        for (int e = 0; e < 8; ++e) g[e] = 1.f;
      }
      uint4 o;
      o.x = pack_bf16x2(v[0] * rs * g[0], v[1] * rs * g[1]);
      o.y = pack_bf16x2(v[2] * rs * g[2], v[3] * rs * g[3]);
      o.z = pack_bf16x2(v[4] * rs * g[4], v[5] * rs * g[5]);
      o.w = pack_bf16x2(v[6] * rs * g[6], v[7] * rs * g[7]);
      *reinterpret_cast<uint4*>(y + col) = o;
    }
  }
}

// The same on few rows (a decode step): one block per row, every load of the row and of the weights requested at
// once, the four waves' sums of squares added in wave order.
__global__ __launch_bounds__(256) void rms_norm_row_kernel(const bf16_t* __restrict__ X, int64_t ldx, bf16_t* __restrict__ Y,
                                                           int64_t ldy, const float* __restrict__ wgt, int d, float eps) {
  __shared__ float part[4];
  const int tid = threadIdx.x, lane = tid & (kWave - 1), w = tid / kWave;
  const bf16_t* x = X + static_cast<int64_t>(blockIdx.x) * ldx;
  constexpr int kP = kRmsMaxPieces * kWave / 256;  // 16-byte pieces per thread
  uint4 raw[kP];
  float4 g[kP][2];
#pragma unroll
  for (int c = 0; c < kP; ++c) {
    const int col = (c * 256 + tid) * 8;
    const bool in = col < d;
    raw[c] = in ? *reinterpret_cast<const uint4*>(x + col) : uint4{0u, 0u, 0u, 0u};
    g[c][0] = (in && wgt) ? *reinterpret_cast<const float4*>(wgt + col) : float4{1.f, 1.f, 1.f, 1.f};
    g[c][1] = (in && wgt) ? *reinterpret_cast<const float4*>(wgt + col + 4) : float4{1.f, 1.f, 1.f, 1.f};
  }
  float ss = 0.f;
#pragma unroll
  for (int c = 0; c < kP; ++c) {
    float v[8];
    Elem<bf16_t>::unpack(raw[c], v);
#pragma unroll
    for (int e = 0; e < 8; ++e) ss = fmaf(v[e], v[e], ss);
  }
  ss = wave_sum(ss);
  if (lane == 0) part[w] = ss;
  __syncthreads();
  const float rs = 1.f / sqrtf((((part[0] + part[1]) + part[2]) + part[3]) / static_cast<float>(d) + eps);
  bf16_t* y = Y + static_cast<int64_t>(blockIdx.x) * ldy;
#pragma unroll
  for (int c = 0; c < kP; ++c) {
    const int col = (c * 256 + tid) * 8;
    if (col < d) {
      float v[8];
      Elem<bf16_t>::unpack(raw[c], v);
      uint4 o;
      o.x = pack_bf16x2(v[0] * rs * g[c][0].x, v[1] * rs * g[c][0].y);
      o.y = pack_bf16x2(v[2] * rs * g[c][0].z, v[3] * rs * g[c][0].w);
      o.z = pack_bf16x2(v[4] * rs * g[c][1].x, v[5] * rs * g[c][1].y);
      o.w = pack_bf16x2(v[6] * rs * g[c][1].z, v[7] * rs * g[c][1].w);
      *reinterpret_cast<uint4*>(y + col) = o;
    }
  }
}

// Rotary rotation in place of rows x [rows, H, Dh] at positions pos[row] (half-split pairing: feature i with i + Dh/2,
// angle pos * base^(-2i/Dh), taken in float64).  Thread = one pair of one (row, head).
__global__ __launch_bounds__(256) void rope_kernel(bf16_t* __restrict__ x, const int32_t* __restrict__ pos, int64_t rows, int H,
                                                   int Dh, double log2_base) {
  const int half = Dh / 2;
  const int64_t it = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
  if (it >= rows * H * half) return;
  const int i = static_cast<int>(it % half);
  const int64_t rh = it / half;  // row * H + head
  const int64_t row = rh / H;
  const double ang = static_cast<double>(pos[row]) * exp2(-2.0 * i / Dh * log2_base);
  const float cs = static_cast<float>(cos(ang)), sn = static_cast<float>(sin(ang));
  bf16_t* p = x + rh * Dh;
  const float lo = bf16_to_f32(p[i]), hi = bf16_to_f32(p[i + half]);
  p[i] = f32_to_bf16(lo * cs - hi * sn);
  p[i + half] = f32_to_bf16(hi * cs + lo * sn);
}

struct Regions {
  int32_t* span_off;
  bf16_t *Z, *Y, *QKV, *Hb;
  float* small;  // partial sums of the small-batch path
  size_t bytes;
};

Regions carve(void* ws, int64_t M, int32_t B, int32_t n_blocks) {
  Regions r{};
  size_t o = 0;
  auto take = [&](size_t n) {
    char* p = ws ? static_cast<char*>(ws) + o : nullptr;
    o += round_up(n, 256);
    return p;
  };
  const size_t rows = static_cast<size_t>(M > 0 ? M : 0);
  r.span_off = reinterpret_cast<int32_t*>(take((static_cast<size_t>(B > 0 ? B : 0) + 2) * sizeof(int32_t)));
  r.Z = reinterpret_cast<bf16_t*>(take(rows * kPW * 2));
  r.Y = reinterpret_cast<bf16_t*>(take(rows * kPW * 2));
  r.QKV = reinterpret_cast<bf16_t*>(take(n_blocks > 0 ? rows * 3 * kPW * 2 : 0));
  r.Hb = reinterpret_cast<bf16_t*>(take(rows * (n_blocks > 0 ? kPMlp : kPH1) * 2));
  r.small = reinterpret_cast<float*>(take(n_blocks == 0 && M <= kSmallRows ? size_t(kSmallSplit) * kSmallRows * kPW * 4 : 0));
  r.bytes = o;
  return r;
}

}  // namespace

}  // namespace dllava

using namespace dllava;

extern "C" size_t dllava_predict_workspace(int64_t M, int32_t B, int32_t n_blocks) {
  return carve(nullptr, M, B, n_blocks).bytes;
}

extern "C" int dllava_predict(const void* x, int64_t ldx, int64_t M, int32_t B, const int32_t* seq_off,
                              const int32_t* vis_start, const int32_t* vis_len, const dllava_predictor* p, int dtype,
                              float* logits, void* workspace, size_t workspace_bytes, void* stream) {
  DLLAVA_REQUIRE(p, DLLAVA_ENULL, "predict: the predictor struct is required");
  DLLAVA_REQUIRE(dtype == DLLAVA_BF16, DLLAVA_EDTYPE, "predict: only DLLAVA_BF16 is supported (got dtype %d)", dtype);
  DLLAVA_REQUIRE(M >= 0 && M <= 0x7fffffffLL, DLLAVA_ESHAPE, "predict: bad M = %lld", (long long)M);
  DLLAVA_REQUIRE(B >= 0, DLLAVA_EINVAL, "predict: B = %d < 0", B);
  DLLAVA_REQUIRE(p->n_blocks >= 0 && p->n_blocks <= DLLAVA_PREDICTOR_MAX_BLOCKS, DLLAVA_EINVAL,
                 "predict: n_blocks = %d outside 0..%d", p->n_blocks, DLLAVA_PREDICTOR_MAX_BLOCKS);
  DLLAVA_REQUIRE(p->d > 0 && p->d % 64 == 0 && p->d <= 0x7fffffffLL, DLLAVA_ESHAPE,
                 "predict: d must be a positive multiple of 64 (got %lld)", (long long)p->d);
  DLLAVA_REQUIRE(ldx >= p->d && ldx % 8 == 0, DLLAVA_ESHAPE,
                 "predict: ldx must be >= d and a multiple of 8 (got %lld)", (long long)ldx);
  if (M == 0) return DLLAVA_OK;
  DLLAVA_REQUIRE(x && logits, DLLAVA_ENULL, "predict: x and logits are required");
  DLLAVA_REQUIRE(!seq_off || (vis_start && vis_len), DLLAVA_ENULL, "predict: vis_start and vis_len go with seq_off");
  DLLAVA_REQUIRE(p->W_in && p->W_h1 && p->W_h2 && p->W_h3, DLLAVA_ENULL, "predict: W_in, W_h1, W_h2, W_h3 are required");
  DLLAVA_REQUIRE(aligned(x, 16) && aligned(p->W_in, 16) && aligned(p->W_h1, 16) && aligned(p->W_h2, 16) &&
                     aligned(p->W_h3, 4),
                 DLLAVA_EINVAL, "predict: x and the matrices must be 16-byte aligned");
  DLLAVA_REQUIRE(aligned(p->b_in, 16) && aligned(p->b_h1, 16) && aligned(p->b_h2, 16), DLLAVA_EINVAL,
                 "predict: bias vectors must be 16-byte aligned");
  for (int i = 0; i < p->n_blocks; ++i) {
    const dllava_vit_block& k = p->blocks[i];
    DLLAVA_REQUIRE(k.Wqkv && k.Wo && k.Wfc1 && k.Wfc2, DLLAVA_ENULL, "predict: block %d lacks a matrix", i);
    DLLAVA_REQUIRE(aligned(k.Wqkv, 16) && aligned(k.Wo, 16) && aligned(k.Wfc1, 16) && aligned(k.Wfc2, 16) &&
                       aligned(k.bqkv, 16) && aligned(k.bo, 16) && aligned(k.bfc1, 16) && aligned(k.bfc2, 16) &&
                       aligned(k.ln1_g, 16) && aligned(k.ln1_b, 16) && aligned(k.ln2_g, 16) && aligned(k.ln2_b, 16),
                   DLLAVA_EINVAL, "predict: block %d: matrices and vectors must be 16-byte aligned", i);
  }
  const int nb = p->n_blocks;
  const Regions r = carve(workspace, M, B, nb);
  DLLAVA_REQUIRE(workspace && aligned(workspace, 256) && workspace_bytes >= r.bytes, DLLAVA_EWORKSPACE,
                 "predict: workspace needs %zu bytes, 256-byte aligned (got %zu)", r.bytes, workspace_bytes);
  hipStream_t st = static_cast<hipStream_t>(stream);
  const bf16_t* X = static_cast<const bf16_t*>(x);
  const int32_t n_spans = seq_off ? B : 1;

  auto lin = [&](const bf16_t* in, int64_t ldin, int K, const void* W, const float* bias, int N, bf16_t* out,
                 int64_t ldout, int act, const bf16_t* res) {
    LinArgs a{};
    a.X = in; a.ldx = ldin; a.M = M; a.K = K; a.N = N;
    a.W = static_cast<const bf16_t*>(W); a.bias = bias;
    a.Y = out; a.ldy = ldout; a.group = N; a.group_stride = 0;
    a.R = res; a.act = act;
    return a;
  };

  if (nb > 0 || seq_off) {
    hipLaunchKernelGGL(span_offsets_kernel, dim3(1), dim3(kWave), 0, st, seq_off ? vis_len : nullptr, B, M, r.span_off);
    DLLAVA_CHECK_LAUNCH("span_offsets_kernel");
  }
  if (nb == 0 && M <= kSmallRows) {  // a handful of rows: the output-text predictor of a decode step
    const int nt = M <= 32 ? 1 : 2;
    const int Mi = static_cast<int>(M), Ki = static_cast<int>(p->d);
    const bf16_t* Wi = static_cast<const bf16_t*>(p->W_in);
    if (nt == 1)
      hipLaunchKernelGGL(small_in_kernel<1>, dim3(16 * kSmallSplit), dim3(256), 0, st, X, ldx, Mi, Ki, Wi, r.small, B,
                         seq_off, vis_start, vis_len, 16, kSmallSplit, kPW);
    else
      hipLaunchKernelGGL(small_in_kernel<2>, dim3(16 * kSmallSplit), dim3(256), 0, st, X, ldx, Mi, Ki, Wi, r.small, B,
                         seq_off, vis_start, vis_len, 16, kSmallSplit, kPW);
    DLLAVA_CHECK_LAUNCH("small_in_kernel");
    hipLaunchKernelGGL(small_head_kernel, dim3(nt), dim3(256), 0, st, r.small, 32 * nt, Mi, p->b_in,
                       static_cast<const bf16_t*>(p->W_h1), p->b_h1, static_cast<const bf16_t*>(p->W_h2), p->b_h2,
                       static_cast<const bf16_t*>(p->W_h3), p->b_h3, logits, seq_off ? r.span_off : nullptr, B);
    DLLAVA_CHECK_LAUNCH("small_head_kernel");
    return DLLAVA_OK;
  }
  {  // z = x W_in^T + b_in over the rows of the spans
    LinArgs a = lin(X, ldx, static_cast<int>(p->d), p->W_in, p->b_in, kPW, r.Z, kPW, 0, nullptr);
    a.B = B; a.seq_off = seq_off; a.vis_start = vis_start; a.vis_len = vis_len;
    if (int rc = launch_lin(a, st)) return rc;
  }
  const unsigned row_blocks = static_cast<unsigned>(ceil_div(M, 4));
  for (int i = 0; i < nb; ++i) {
    const dllava_vit_block& k = p->blocks[i];
    hipLaunchKernelGGL(ln_kernel, dim3(row_blocks), dim3(256), 0, st, r.Z, r.Y, k.ln1_g, k.ln1_b, M);
    DLLAVA_CHECK_LAUNCH("ln_kernel");
    {  // q | k | v into three [M, 512] matrices
      LinArgs a = lin(r.Y, kPW, kPW, k.Wqkv, k.bqkv, 3 * kPW, r.QKV, kPW, 0, nullptr);
      a.group = kPW;
      a.group_stride = M * kPW;
      if (int rc = launch_lin(a, st)) return rc;
    }
    {  // attention of every image token over all image tokens of its sequence, into Y
      PrefillArgs pa{};
      pa.Q = r.QKV; pa.K = r.QKV + M * kPW; pa.V = r.QKV + 2 * M * kPW; pa.O = r.Y;
      pa.off = r.span_off; pa.B = n_spans; pa.H = kPHeads;
      pa.scale_log2 = 0.125f * 1.44269504088896340736f;  // 1 / sqrt(64), in the base-2 exponent
      pa.full = 1;
      const int rc = prefill_mfma_launch(pa, M, kPW / kPHeads, st);
      if (rc < 0) return rc;
      if (rc > 0) DLLAVA_FAIL(DLLAVA_ESHAPE, "predict: too many rows or spans for the attention step");
    }
    if (int rc = launch_lin(lin(r.Y, kPW, kPW, k.Wo, k.bo, kPW, r.Z, kPW, 0, r.Z), st)) return rc;
    hipLaunchKernelGGL(ln_kernel, dim3(row_blocks), dim3(256), 0, st, r.Z, r.Y, k.ln2_g, k.ln2_b, M);
    DLLAVA_CHECK_LAUNCH("ln_kernel");
    if (int rc = launch_lin(lin(r.Y, kPW, kPW, k.Wfc1, k.bfc1, kPMlp, r.Hb, kPMlp, 1, nullptr), st)) return rc;
    if (int rc = launch_lin(lin(r.Hb, kPMlp, kPMlp, k.Wfc2, k.bfc2, kPW, r.Z, kPW, 0, r.Z), st)) return rc;
  }
  if (int rc = launch_lin(lin(r.Z, kPW, kPW, p->W_h1, p->b_h1, kPH1, r.Hb, kPH1, 1, nullptr), st)) return rc;
  if (int rc = launch_lin(lin(r.Hb, kPH1, kPH1, p->W_h2, p->b_h2, kPH2, r.Y, kPH2, 1, nullptr), st)) return rc;
  hipLaunchKernelGGL(head_out_kernel, dim3(row_blocks), dim3(256), 0, st, r.Y, static_cast<const bf16_t*>(p->W_h3),
                     p->b_h3, logits, M, seq_off ? r.span_off : nullptr, B);
  DLLAVA_CHECK_LAUNCH("head_out_kernel");
  return DLLAVA_OK;
}

// ---- the layers of the predictor as calls of their own ---------------------------------------------------------

extern "C" int dllava_linear(const void* x, int64_t ldx, int64_t M, int64_t K, const void* W, const float* bias,
                             int64_t N, int act, const void* residual, void* y, int64_t ldy, int dtype, void* stream) {
  DLLAVA_REQUIRE(dtype == DLLAVA_BF16, DLLAVA_EDTYPE, "linear: only DLLAVA_BF16 is supported (got dtype %d)", dtype);
  DLLAVA_REQUIRE(M >= 0 && M <= 0x7fffffffLL, DLLAVA_ESHAPE, "linear: bad M = %lld", (long long)M);
  DLLAVA_REQUIRE(K > 0 && K % 64 == 0 && K <= 0x7fffffffLL, DLLAVA_ESHAPE,
                 "linear: K must be a positive multiple of 64 (got %lld)", (long long)K);
  DLLAVA_REQUIRE(N > 0 && N % 8 == 0 && N <= 0x7fffffffLL, DLLAVA_ESHAPE,
                 "linear: N must be a positive multiple of 8 (got %lld)", (long long)N);
  DLLAVA_REQUIRE(ldx >= K && ldx % 8 == 0 && ldy >= N && ldy % 8 == 0, DLLAVA_ESHAPE,
                 "linear: ldx >= K, ldy >= N, both multiples of 8 (got %lld, %lld)", (long long)ldx, (long long)ldy);
  DLLAVA_REQUIRE(act >= 0 && act <= 2, DLLAVA_EINVAL, "linear: act = %d (0: none, 1: GELU, 2: gated)", act);
  DLLAVA_REQUIRE(act != 2 || residual, DLLAVA_ENULL, "linear: act = 2 takes the gate in `residual`");
  if (M == 0) return DLLAVA_OK;
  DLLAVA_REQUIRE(x && W && y, DLLAVA_ENULL, "linear: x, W and y are required");
  DLLAVA_REQUIRE(aligned(x, 16) && aligned(W, 16) && aligned(y, 16) && aligned(residual, 16) && aligned(bias, 16),
                 DLLAVA_EINVAL, "linear: x, W, bias, residual, y must be 16-byte aligned");
  LinArgs a{};
  a.X = static_cast<const bf16_t*>(x); a.ldx = ldx; a.M = M; a.K = static_cast<int>(K); a.N = static_cast<int>(N);
  a.W = static_cast<const bf16_t*>(W); a.bias = bias;
  a.Y = static_cast<bf16_t*>(y); a.ldy = ldy; a.group = static_cast<int>(N); a.group_stride = 0;
  a.R = static_cast<const bf16_t*>(residual); a.act = act;
  return launch_lin(a, static_cast<hipStream_t>(stream));
}

extern "C" int dllava_layer_norm(const void* z, int64_t M, const float* gamma, const float* beta, void* y, int dtype,
                                    void* stream) {
  DLLAVA_REQUIRE(dtype == DLLAVA_BF16, DLLAVA_EDTYPE, "layer_norm: only DLLAVA_BF16 is supported (got dtype %d)", dtype);
  DLLAVA_REQUIRE(M >= 0 && M <= 0x7fffffffLL, DLLAVA_ESHAPE, "layer_norm: bad M = %lld", (long long)M);
  if (M == 0) return DLLAVA_OK;
  DLLAVA_REQUIRE(z && y, DLLAVA_ENULL, "layer_norm: z and y are required");
  DLLAVA_REQUIRE(aligned(z, 16) && aligned(y, 16) && aligned(gamma, 16) && aligned(beta, 16), DLLAVA_EINVAL,
                 "layer_norm: z, y, gamma, beta must be 16-byte aligned");
  hipLaunchKernelGGL(ln_kernel, dim3(static_cast<unsigned>(ceil_div(M, 4))), dim3(256), 0,
                     static_cast<hipStream_t>(stream), static_cast<const bf16_t*>(z), static_cast<bf16_t*>(y), gamma,
                     beta, M);
  DLLAVA_CHECK_LAUNCH("ln_kernel");
  return DLLAVA_OK;
}

extern "C" int dllava_span_attn(const void* Q, const void* K, const void* V, int32_t B, const int32_t* off, int64_t rows,
                                int32_t H, int32_t Dh, float scale, void* O, int dtype, void* stream) {
  DLLAVA_REQUIRE(dtype == DLLAVA_BF16, DLLAVA_EDTYPE, "span_attn: only DLLAVA_BF16 is supported (got dtype %d)", dtype);
  DLLAVA_REQUIRE(B >= 0 && rows >= 0 && rows <= 0x7fffffffLL, DLLAVA_EINVAL, "span_attn: B = %d, rows = %lld", B,
                 (long long)rows);
  DLLAVA_REQUIRE(H > 0 && (Dh == 64 || Dh == 128), DLLAVA_ESHAPE, "span_attn: H = %d, Dh = %d (Dh must be 64 or 128)", H, Dh);
  DLLAVA_REQUIRE(scale == scale && scale > 0.f && scale < INFINITY, DLLAVA_EINVAL, "span_attn: bad scale");
  if (B == 0 || rows == 0) return DLLAVA_OK;
  DLLAVA_REQUIRE(Q && K && V && O && off, DLLAVA_ENULL, "span_attn: Q, K, V, O and off are required");
  DLLAVA_REQUIRE(aligned(Q, 16) && aligned(K, 16) && aligned(V, 16) && aligned(O, 16), DLLAVA_EINVAL,
                 "span_attn: Q, K, V, O must be 16-byte aligned");
  PrefillArgs pa{};
  pa.Q = Q; pa.K = K; pa.V = V; pa.O = O; pa.off = off; pa.B = B; pa.H = H;
  pa.scale_log2 = scale * 1.44269504088896340736f;
  pa.full = 1;
  const int rc = prefill_mfma_launch(pa, rows, Dh, static_cast<hipStream_t>(stream));
  if (rc > 0) DLLAVA_FAIL(DLLAVA_ESHAPE, "span_attn: too many rows, spans or heads");
  return rc;
}

extern "C" int dllava_rms_norm(const void* x, int64_t ldx, int64_t M, int64_t d, const float* weight, float eps, void* y,
                               int64_t ldy, int dtype, void* stream) {
  DLLAVA_REQUIRE(dtype == DLLAVA_BF16, DLLAVA_EDTYPE, "rms_norm: only DLLAVA_BF16 is supported (got dtype %d)", dtype);
  DLLAVA_REQUIRE(M >= 0 && M <= 0x7fffffffLL, DLLAVA_ESHAPE, "rms_norm: bad M = %lld", (long long)M);
  DLLAVA_REQUIRE(d > 0 && d % 8 == 0 && d <= 8 * kWave * kRmsMaxPieces, DLLAVA_ESHAPE,
                 "rms_norm: d must be a multiple of 8, at most %d (got %lld)", 8 * kWave * kRmsMaxPieces, (long long)d);
  DLLAVA_REQUIRE(ldx >= d && ldx % 8 == 0 && ldy >= d && ldy % 8 == 0, DLLAVA_ESHAPE,
                 "rms_norm: ldx, ldy >= d, multiples of 8 (got %lld, %lld)", (long long)ldx, (long long)ldy);
  DLLAVA_REQUIRE(eps == eps && eps >= 0.f && eps < INFINITY, DLLAVA_EINVAL, "rms_norm: bad eps");
  if (M == 0) return DLLAVA_OK;
  DLLAVA_REQUIRE(x && y, DLLAVA_ENULL, "rms_norm: x and y are required");
  DLLAVA_REQUIRE(aligned(x, 16) && aligned(y, 16) && aligned(weight, 16), DLLAVA_EINVAL,
                 "rms_norm: x, y, weight must be 16-byte aligned");
  if (M <= 1024)  // too few rows to fill the chip one wave per row: one block per row
    hipLaunchKernelGGL(rms_norm_row_kernel, dim3(static_cast<unsigned>(M)), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<const bf16_t*>(x), ldx, static_cast<bf16_t*>(y), ldy, weight, static_cast<int>(d), eps);
  else
    hipLaunchKernelGGL(rms_norm_kernel, dim3(static_cast<unsigned>(ceil_div(M, 4))), dim3(256), 0,
                       static_cast<hipStream_t>(stream), static_cast<const bf16_t*>(x), ldx, static_cast<bf16_t*>(y), ldy,
                       weight, M, static_cast<int>(d), eps);
  DLLAVA_CHECK_LAUNCH("rms_norm_kernel");
  return DLLAVA_OK;
}

// ---- linear layer on few rows (one row per sequence of a decode step) ----------------------------------------------

namespace {
// parts of the input width across blocks for n_groups feature groups, nw waves per block, about `aim` blocks in all
int few_parts_of(int64_t n_groups, int64_t K, int nw, int aim) {
  const int64_t lines = K / 64;
  int64_t kq = (aim + n_groups - 1) / n_groups;
  if (kq > 8) kq = 8;
  if (kq * nw > lines) kq = (lines + nw - 1) / nw;
  return static_cast<int>(kq < 1 ? 1 : kq);
}
int few_parts(int64_t N, int64_t K) { return few_parts_of(N / 32, K, 4, kFewBlocks); }
// A plain layer whose 32-feature groups are too few for blocks of 4 waves takes 8 waves per block instead, and
// 16-feature groups when those still fit one block per compute unit (measured at d = 4096 / 5120, 16 and 32 rows:
// W_O 10 / 17 us against 13 / 20 the other way round, down-projection 22.5 / 34 against 28.5 / 44).
struct FewPlan {
  int kind;  // kFewPlain, kFewPlainHalf or kFewPlain8
  int n_fg, kq;
  int64_t cols;  // width of one row of handed-over sums
};
FewPlan few_plan_plain(int64_t N, int64_t K) {
  FewPlan p;
  p.cols = N;
  if (few_parts(N, K) == 1) {
    p.kind = kFewPlain, p.n_fg = static_cast<int>(N / 32), p.kq = 1;
  } else if (N / 16 <= 256) {
    p.kind = kFewPlainHalf, p.n_fg = static_cast<int>(N / 16), p.kq = few_parts_of(p.n_fg, K, 8, 256);
  } else {
    p.kind = kFewPlain8, p.n_fg = static_cast<int>(N / 32), p.kq = 1;
  }
  return p;
}
// counters, then the sums that the blocks of one feature group hand over (none when the input width is not cut)
FewEpi few_epilogue(void* workspace) {
  FewEpi ep = {};
  ep.counters = static_cast<int32_t*>(workspace);
  ep.partial = reinterpret_cast<float*>(static_cast<char*>(workspace) + kFewCounterBytes);
  return ep;
}
}  // namespace

extern "C" size_t dllava_linear_few_workspace(int64_t N, int64_t K) {
  if (N <= 0 || K <= 0) return kFewCounterBytes;
  const FewPlan p = few_plan_plain(N, K);
  const size_t sums = p.kq > 1 ? static_cast<size_t>(p.kq) * kSmallRows * static_cast<size_t>(p.cols) * sizeof(float) : 0;
  return kFewCounterBytes + round_up(sums, 256);
}

extern "C" int dllava_linear_few(const void* x, int64_t ldx, int64_t M, int64_t K, const void* W, const float* bias,
                                 int64_t N, int act, const void* residual, void* y, int64_t ldy, int dtype,
                                 void* workspace, size_t workspace_bytes, void* stream) {
  DLLAVA_REQUIRE(dtype == DLLAVA_BF16, DLLAVA_EDTYPE, "linear_few: only DLLAVA_BF16 is supported (got dtype %d)", dtype);
  DLLAVA_REQUIRE(M >= 0 && M <= kSmallRows, DLLAVA_ESHAPE, "linear_few: at most %d rows (got %lld)", kSmallRows, (long long)M);
  DLLAVA_REQUIRE(K > 0 && K % 64 == 0 && K <= 0x7fffffffLL, DLLAVA_ESHAPE,
                 "linear_few: K must be a positive multiple of 64 (got %lld)", (long long)K);
  DLLAVA_REQUIRE(N > 0 && N % 32 == 0 && N <= 0x7fffffffLL, DLLAVA_ESHAPE,
                 "linear_few: N must be a positive multiple of 32 (got %lld)", (long long)N);
  DLLAVA_REQUIRE(ldx >= K && ldx % 8 == 0 && ldy >= N && ldy % 8 == 0, DLLAVA_ESHAPE,
                 "linear_few: ldx >= K, ldy >= N, both multiples of 8 (got %lld, %lld)", (long long)ldx, (long long)ldy);
  DLLAVA_REQUIRE(act >= 0 && act <= 2, DLLAVA_EINVAL, "linear_few: act = %d (0: none, 1: GELU, 2: gated)", act);
  DLLAVA_REQUIRE(act != 2 || residual, DLLAVA_ENULL, "linear_few: act = 2 takes the gate in `residual`");
  if (M == 0) return DLLAVA_OK;
  DLLAVA_REQUIRE(x && W && y, DLLAVA_ENULL, "linear_few: x, W and y are required");
  DLLAVA_REQUIRE(aligned(x, 16) && aligned(W, 16) && aligned(y, 16) && aligned(residual, 16) && aligned(bias, 16),
                 DLLAVA_EINVAL, "linear_few: x, W, bias, residual, y must be 16-byte aligned");
  const size_t need = dllava_linear_few_workspace(N, K);
  DLLAVA_REQUIRE(workspace && aligned(workspace, 256) && workspace_bytes >= need, DLLAVA_EWORKSPACE,
                 "linear_few: workspace needs %zu bytes, 256-byte aligned (got %zu)", need, workspace_bytes);
  hipStream_t st = static_cast<hipStream_t>(stream);
  const FewPlan plan = few_plan_plain(N, K);
  const int nt = M <= 32 ? 1 : 2;
  const bf16_t* X = static_cast<const bf16_t*>(x);
  const bf16_t* Wb = static_cast<const bf16_t*>(W);
  FewEpi ep = few_epilogue(workspace);
  ep.bias = bias;
  ep.act = act;
  ep.R = static_cast<const bf16_t*>(residual);
  ep.Y = static_cast<bf16_t*>(y);
  ep.ldy = ldy;
  if (plan.kind == kFewPlain8)
    launch_few_fused<kFewPlain8>(nt, st, X, ldx, static_cast<int>(M), static_cast<int>(K), Wb, nullptr, nullptr, plan.n_fg,
                                 plan.kq, plan.n_fg, ep);
  else if (plan.kind == kFewPlainHalf)
    launch_few_fused<kFewPlainHalf>(nt, st, X, ldx, static_cast<int>(M), static_cast<int>(K), Wb, nullptr, nullptr, plan.n_fg,
                                    plan.kq, plan.n_fg, ep);
  else
    launch_few_fused<kFewPlain>(nt, st, X, ldx, static_cast<int>(M), static_cast<int>(K), Wb, nullptr, nullptr, plan.n_fg,
                                plan.kq, plan.n_fg, ep);
  DLLAVA_CHECK_LAUNCH("few_fused_kernel");
  return DLLAVA_OK;
}

extern "C" int dllava_rope(void* x, const int32_t* pos, int64_t rows, int32_t H, int32_t Dh, float rope_base, int dtype,
                           void* stream) {
  DLLAVA_REQUIRE(dtype == DLLAVA_BF16, DLLAVA_EDTYPE, "rope: only DLLAVA_BF16 is supported (got dtype %d)", dtype);
  DLLAVA_REQUIRE(rows >= 0 && rows <= 0x7fffffffLL && H > 0 && Dh > 0 && Dh % 2 == 0, DLLAVA_ESHAPE,
                 "rope: rows = %lld, H = %d, Dh = %d", (long long)rows, H, Dh);
  DLLAVA_REQUIRE(rope_base > 0.f && rope_base < INFINITY, DLLAVA_EINVAL, "rope: bad rope_base");
  if (rows == 0) return DLLAVA_OK;
  DLLAVA_REQUIRE(x && pos, DLLAVA_ENULL, "rope: x and pos are required");
  const int64_t items = rows * H * (Dh / 2);
  hipLaunchKernelGGL(rope_kernel, dim3(static_cast<unsigned>(ceil_div(items, 256))), dim3(256), 0,
                     static_cast<hipStream_t>(stream), static_cast<bf16_t*>(x), pos, rows, H, Dh,
                     log2(static_cast<double>(rope_base)));
  DLLAVA_CHECK_LAUNCH("rope_kernel");
  return DLLAVA_OK;
}

// ---- fused forms for a decode step: q|k|v with rotary rotation, gate|up with the gating ---------------------------

extern "C" size_t dllava_decode_proj_workspace(int64_t N_total, int64_t K) {
  if (N_total <= 0 || K <= 0) return kFewCounterBytes;
  const int kq = few_parts(N_total, K);
  const size_t sums = kq > 1 ? static_cast<size_t>(kq) * kSmallRows * static_cast<size_t>(N_total) * sizeof(float) : 0;
  return kFewCounterBytes + round_up(sums, 256);
}

extern "C" int dllava_qkv_few(const void* x, int64_t ldx, int64_t M, int64_t d, const void* Wq, const void* Wk,
                              const void* Wv, int32_t H, int32_t Dh, const int32_t* pos, float rope_base, void* q, void* k,
                              void* v, int dtype, void* workspace, size_t workspace_bytes, void* stream) {
  DLLAVA_REQUIRE(dtype == DLLAVA_BF16, DLLAVA_EDTYPE, "qkv_few: only DLLAVA_BF16 is supported (got dtype %d)", dtype);
  DLLAVA_REQUIRE(M >= 0 && M <= kSmallRows, DLLAVA_ESHAPE, "qkv_few: at most %d rows (got %lld)", kSmallRows, (long long)M);
  DLLAVA_REQUIRE(d > 0 && d % 64 == 0 && d <= 0x7fffffffLL && ldx >= d && ldx % 8 == 0, DLLAVA_ESHAPE,
                 "qkv_few: d must be a positive multiple of 64, ldx >= d a multiple of 8 (got %lld, %lld)", (long long)d,
                 (long long)ldx);
  DLLAVA_REQUIRE(H > 0 && Dh > 0 && Dh % 32 == 0, DLLAVA_ESHAPE, "qkv_few: H = %d, Dh = %d (Dh %% 32 == 0)", H, Dh);
  DLLAVA_REQUIRE(rope_base > 0.f && rope_base < INFINITY, DLLAVA_EINVAL, "qkv_few: bad rope_base");
  if (M == 0) return DLLAVA_OK;
  DLLAVA_REQUIRE(x && Wq && Wk && Wv && pos && q && k && v, DLLAVA_ENULL, "qkv_few: x, Wq, Wk, Wv, pos, q, k, v are required");
  DLLAVA_REQUIRE(aligned(x, 16) && aligned(Wq, 16) && aligned(Wk, 16) && aligned(Wv, 16) && aligned(q, 16) && aligned(k, 16) &&
                     aligned(v, 16),
                 DLLAVA_EINVAL, "qkv_few: tensors must be 16-byte aligned");
  const int64_t HD = static_cast<int64_t>(H) * Dh, N = 3 * HD;
  const size_t need = dllava_decode_proj_workspace(N, d);
  DLLAVA_REQUIRE(workspace && aligned(workspace, 256) && workspace_bytes >= need, DLLAVA_EWORKSPACE,
                 "qkv_few: workspace needs %zu bytes, 256-byte aligned (got %zu)", need, workspace_bytes);
  hipStream_t st = static_cast<hipStream_t>(stream);
  const int kq = few_parts(N, d), n_fg = static_cast<int>(N / 32), nt = M <= 32 ? 1 : 2;
  const bf16_t* X = static_cast<const bf16_t*>(x);
  FewEpi ep = few_epilogue(workspace);
  ep.H = H;
  ep.Dh = Dh;
  ep.pos = pos;
  ep.rope_ratio = pow(static_cast<double>(rope_base), -2.0 / Dh);
  ep.q = static_cast<bf16_t*>(q);
  ep.k = static_cast<bf16_t*>(k);
  ep.v = static_cast<bf16_t*>(v);
  launch_few_fused<kFewQkv>(nt, st, X, ldx, static_cast<int>(M), static_cast<int>(d), static_cast<const bf16_t*>(Wq),
                            static_cast<const bf16_t*>(Wk), static_cast<const bf16_t*>(Wv), n_fg, kq,
                            static_cast<int>(HD / 32), ep);
  DLLAVA_CHECK_LAUNCH("few_fused_kernel");
  return DLLAVA_OK;
}

extern "C" int dllava_gated_few(const void* x, int64_t ldx, int64_t M, int64_t d, const void* Wg, const void* Wu, int64_t F,
                                void* y, int64_t ldy, int dtype, void* workspace, size_t workspace_bytes, void* stream) {
  DLLAVA_REQUIRE(dtype == DLLAVA_BF16, DLLAVA_EDTYPE, "gated_few: only DLLAVA_BF16 is supported (got dtype %d)", dtype);
  DLLAVA_REQUIRE(M >= 0 && M <= kSmallRows, DLLAVA_ESHAPE, "gated_few: at most %d rows (got %lld)", kSmallRows, (long long)M);
  DLLAVA_REQUIRE(d > 0 && d % 64 == 0 && d <= 0x7fffffffLL && ldx >= d && ldx % 8 == 0, DLLAVA_ESHAPE,
                 "gated_few: d must be a positive multiple of 64, ldx >= d a multiple of 8 (got %lld, %lld)", (long long)d,
                 (long long)ldx);
  DLLAVA_REQUIRE(F > 0 && F % 32 == 0 && F <= 0x3fffffffLL && ldy >= F && ldy % 8 == 0, DLLAVA_ESHAPE,
                 "gated_few: F must be a positive multiple of 32, ldy >= F a multiple of 8 (got %lld, %lld)", (long long)F,
                 (long long)ldy);
  if (M == 0) return DLLAVA_OK;
  DLLAVA_REQUIRE(x && Wg && Wu && y, DLLAVA_ENULL, "gated_few: x, Wg, Wu and y are required");
  DLLAVA_REQUIRE(aligned(x, 16) && aligned(Wg, 16) && aligned(Wu, 16) && aligned(y, 16), DLLAVA_EINVAL,
                 "gated_few: tensors must be 16-byte aligned");
  const int64_t N = 2 * F;
  const size_t need = dllava_decode_proj_workspace(N, d);
  DLLAVA_REQUIRE(workspace && aligned(workspace, 256) && workspace_bytes >= need, DLLAVA_EWORKSPACE,
                 "gated_few: workspace needs %zu bytes, 256-byte aligned (got %zu)", need, workspace_bytes);
  hipStream_t st = static_cast<hipStream_t>(stream);
  const int kq = few_parts(N, d), n_fg = static_cast<int>(N / 32), nt = M <= 32 ? 1 : 2;
  const bf16_t* X = static_cast<const bf16_t*>(x);
  FewEpi ep = few_epilogue(workspace);
  ep.Y = static_cast<bf16_t*>(y);
  ep.ldy = ldy;
  launch_few_fused<kFewGated>(nt, st, X, ldx, static_cast<int>(M), static_cast<int>(d), static_cast<const bf16_t*>(Wg),
                              static_cast<const bf16_t*>(Wu), nullptr, n_fg, kq, n_fg, ep);
  DLLAVA_CHECK_LAUNCH("few_fused_kernel");
  return DLLAVA_OK;
}
