// Predictor scoring for a handful of rows (decode: one row per sequence), bfloat16.
//
// The call reads W1 exactly once; what costs time is latency and the number of memory lines a compute unit has to
// pull, not flops.  The work is therefore cut in BOTH directions so that every compute unit gets a small piece:
// block (g, ks) owns 64 hidden units (g) and one slice of d (ks); each of its 4 waves takes 16 of the units over
// the whole slice with v_mfma_f32_16x16x32_bf16 in the transposed orientation (hidden units down the rows, tokens
// across the columns) on fragments loaded straight from global memory, all loads of the slice in flight together.
// A block reads 1/KS of x instead of all of it.
//
// Cross-block reduction (the activation is not linear, so the slices of d must be summed before it):
//   1. every block stores its 64 x Mpad tile of partial pre-activations (plain device-scope stores),
//   2. draws a ticket on its unit group's counter,
//   3. the block with the group's last ticket reloads the KS tiles, adds them in slice order (fixed order:
//      bit-reproducible), applies bias + GELU, contracts with W2 over its 64 units,
//   4. and adds the resulting partial logits to the logit accumulators as 64-bit fixed-point integers with one
//      returning device-scope atomic each (integer addition is associative: order-independent); the low 8 bits of
//      the same word count the arrivals, and the last arrival converts, adds b2, writes the logit and clears the
//      accumulator.
// Counters and accumulators start at zero and are left at zero; the partial tiles need no initialisation.
#pragma once

#include "score_args.h"

namespace dllava {

typedef __bf16 sp_bf16x8 __attribute__((ext_vector_type(8)));
typedef float sp_f32x4 __attribute__((ext_vector_type(4)));

constexpr int kSpUnits = 64;       // hidden units per block
constexpr int kSpWaves = 4;        // 16 units each
constexpr int kSpThreads = kSpWaves * kWave;
constexpr int kSpMaxSplit = 16;    // slices of d
constexpr int kSpBatch = 4;        // 64-element pairs of k-steps whose loads are issued together
constexpr int kSpMaxGroups = 255;  // the arrival count shares a word with the sum (8 bits)
// One accumulator / counter per 256 bytes (atomics that share a memory line serialise at the memory side).
constexpr int kSpAccStride = 32;   // in 8-byte words
constexpr int kSpCntStride = 64;   // in 4-byte words
constexpr size_t kSpAccBytes = static_cast<size_t>(2 * 64) * kSpAccStride * 8;      // 2 logits x up to 64 tokens
constexpr size_t kSpCntBytes = static_cast<size_t>(kSpMaxGroups + 1) * kSpCntStride * 4;
// Workspace layout of dllava_score, shared by its two bfloat16 forms so that one buffer serves both in any order:
//   [0, kSpAccBytes)                 logit accumulators of the few-rows form      (zero between calls)
//   [.., + kSpCntBytes)              unit-group tickets of the few-rows form      (zero between calls)
//   [.., + kGemmCntBytes)            token-tile counters of the GEMM form         (zero between calls)
//   [kScoreScratchOffset, ...)       partial pre-activation tiles (few rows) or partial logits (GEMM): written
//                                    before they are read within a call, so either form may leave anything there
constexpr size_t kGemmCntBytes = 4096;
constexpr size_t kScoreScratchOffset = kSpAccBytes + kSpCntBytes + kGemmCntBytes;

struct SplitPlan {
  int G;    // unit groups
  int KS;   // slices of d
  int ppb;  // 64-element pairs per slice
};

// Host and device agree on the plan through the launch arguments; about 256 blocks, one per compute unit.
inline SplitPlan split_plan(int64_t d, int64_t dh) {
  SplitPlan p;
  p.G = static_cast<int>((dh + kSpUnits - 1) / kSpUnits);
  const int npairs = static_cast<int>(d / 64);
  int ks = 256 / p.G;
  if (ks > kSpMaxSplit) ks = kSpMaxSplit;
  if (ks > npairs) ks = npairs;
  if (ks < 1) ks = 1;
  p.ppb = (npairs + ks - 1) / ks;
  p.KS = (npairs + p.ppb - 1) / p.ppb;  // no empty slice
  return p;
}

inline size_t split_workspace(int64_t M, int64_t d, int64_t dh) {
  const SplitPlan p = split_plan(d, dh);
  const size_t mpad = static_cast<size_t>((M + 15) / 16) * 16;
  return kScoreScratchOffset + static_cast<size_t>(p.KS) * p.G * kSpUnits * mpad * sizeof(float);
}

__device__ __forceinline__ sp_bf16x8 sp_frag(const uint4& v) {
  union { uint4 u; sp_bf16x8 f; } c;
  c.u = v;
  return c.f;
}

// The work of block `bid` of the G*KS blocks (threads 0..kSpThreads-1 of the calling block; the function contains
// block barriers, so the block's other waves, if any, must have ended).
// NT = 16-token column tiles (M <= 16*NT).  workspace = [accumulators | tickets | (GEMM counters) | partial tiles].
template <int NT>
__device__ __forceinline__ void score_splitk_block(const ScoreArgs& a, int G, int KS, int ppb, int bid) {
  constexpr int MP = 16 * NT;  // padded token count
  __shared__ float sm_p[kSpWaves][MP][2];
  __shared__ int sm_last;
  const int tid = threadIdx.x, lane = tid & (kWave - 1), w = tid / kWave;
  const int g = bid / KS, ks = bid % KS;
  const int M = static_cast<int>(a.M);
  const int64_t d = a.d, dh = a.dh;
  const bf16_t* W1 = static_cast<const bf16_t*>(a.W1);
  const bf16_t* W2 = static_cast<const bf16_t*>(a.W2);
  const bf16_t* X = static_cast<const bf16_t*>(a.x);
  unsigned long long* acc_logit = static_cast<unsigned long long*>(a.workspace);
  int32_t* counters = reinterpret_cast<int32_t*>(static_cast<char*>(a.workspace) + kSpAccBytes);
  float* partial = reinterpret_cast<float*>(static_cast<char*>(a.workspace) + kScoreScratchOffset);
  const bf16_t* zero16 = reinterpret_cast<const bf16_t*>(kZeroWords);

  // Epilogue operands of the thread's four units (used only by the group's last block), requested first so that
  // they never add a round trip; operands that must be zero come from kZeroWords through the address.
  // epilogue mapping: thread -> token column tid%16 (+16t), units 4*(tid/16) .. +3 of the group
  float eb[4], ew0[4], ew1[4], eb2[2];
  {
    const bool has_b1 = a.b1 != nullptr;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int64_t u = static_cast<int64_t>(g) * kSpUnits + 4 * (tid >> 4) + r;
      const bool ok = u < dh;
      eb[r] = *((ok & has_b1) ? a.b1 + u : kZeroWords);
      ew0[r] = bf16_to_f32(*(ok ? W2 + u : zero16));
      ew1[r] = bf16_to_f32(*(ok ? W2 + dh + u : zero16));
    }
    eb2[0] = *(a.b2 ? a.b2 : kZeroWords);
    eb2[1] = *(a.b2 ? a.b2 + 1 : kZeroWords);
  }

  // fragment addressing: lane -> (row = lane%16, 8 consecutive k at 8*(lane/16))
  int64_t unit = static_cast<int64_t>(g) * kSpUnits + w * 16 + (lane & 15);
  if (unit >= dh) unit = dh - 1;  // rows past dh duplicate the last unit; their W2 weights are zero
  const bf16_t* wrow = W1 + unit * d + 8 * (lane >> 4);
  const bf16_t* xrow[NT];
#pragma unroll
  for (int t = 0; t < NT; ++t) {
    int tok = t * 16 + (lane & 15);
    if (tok >= M) tok = M - 1;  // columns past M duplicate the last token; they are never written out
    xrow[t] = X + static_cast<int64_t>(tok) * a.ldx + 8 * (lane >> 4);
  }
  const int npairs = static_cast<int>(d / 64);
  const int pbeg = ks * ppb, pend = (pbeg + ppb < npairs) ? pbeg + ppb : npairs;
  sp_f32x4 acc[NT];
#pragma unroll
  for (int t = 0; t < NT; ++t) acc[t] = sp_f32x4{0.f, 0.f, 0.f, 0.f};
  for (int p0 = pbeg; p0 < pend; p0 += kSpBatch) {
    uint4 ra[2 * kSpBatch], rb[NT][2 * kSpBatch];
#pragma unroll
    for (int u = 0; u < 2 * kSpBatch; ++u) {
      const int p = p0 + (u >> 1);
      const bool ok = p < pend;
      // a pair = 64 elements = one 128-byte memory line per row, fetched by two back-to-back 64-byte fragment loads;
      // past the end of the slice: a zero W1 fragment (through the address: the load stays unconditional)
      const int64_t ko = static_cast<int64_t>(ok ? p : pend - 1) * 64 + (u & 1) * 32;
      ra[u] = *reinterpret_cast<const uint4*>(ok ? wrow + ko : zero16);
#pragma unroll
      for (int t = 0; t < NT; ++t) rb[t][u] = *reinterpret_cast<const uint4*>(xrow[t] + ko);
    }
    // every load of the batch is issued before the first product (the scheduler would otherwise hold some back
    // to save registers, and the kernel is nothing but this latency)
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int u = 0; u < 2 * kSpBatch; ++u)
#pragma unroll
      for (int t = 0; t < NT; ++t)
        acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(sp_frag(ra[u]), sp_frag(rb[t][u]), acc[t], 0, 0, 0);
  }

  // 1. partial tile [64 units][MP tokens] of (ks, g); accumulator layout: unit 4*(lane/16)+r, token lane%16
  {
    float* tile = partial + ((static_cast<size_t>(ks) * G + g) * kSpUnits + w * 16) * MP;
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
      for (int r = 0; r < 4; ++r) st_agent(tile + (4 * (lane >> 4) + r) * MP + t * 16 + (lane & 15), acc[t][r]);
  }
  // 2. ticket
  block_publish();
  if (tid == 0) sm_last = (add_agent(&counters[g * kSpCntStride], 1) == KS - 1);
  __syncthreads();
  if (!sm_last) return;

  // 3. the group's last block: sum the KS tiles in slice order, bias, GELU, contraction with W2 over 64 units
  {
    const float* col = partial + (static_cast<size_t>(g) * kSpUnits + 4 * (tid >> 4)) * MP + (tid & 15);
    const size_t kstride = static_cast<size_t>(G) * kSpUnits * MP;
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      float s[4] = {0.f, 0.f, 0.f, 0.f};
      for (int k0 = 0; k0 < KS; k0 += 4) {  // 16 independent loads in flight, then a fixed-order sum
        float v[4][4];
#pragma unroll
        for (int kk = 0; kk < 4; ++kk)
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            const int k = (k0 + kk < KS) ? k0 + kk : KS - 1;
            v[kk][r] = ld_agent(col + k * kstride + r * MP + t * 16);
          }
#pragma unroll
        for (int kk = 0; kk < 4; ++kk)
#pragma unroll
          for (int r = 0; r < 4; ++r) s[r] += (k0 + kk < KS) ? v[kk][r] : 0.f;
      }
      float p0 = 0.f, p1 = 0.f;
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const float gl = gelu_erf_fast(s[r] + eb[r]);
        p0 = fmaf(gl, ew0[r], p0);
        p1 = fmaf(gl, ew1[r], p1);
      }
      // lanes l, l+16, l+32, l+48 hold the same token: wave sum, then the four waves through LDS in wave order
      p0 += __shfl_xor(p0, 16, kWave);
      p1 += __shfl_xor(p1, 16, kWave);
      p0 += __shfl_xor(p0, 32, kWave);
      p1 += __shfl_xor(p1, 32, kWave);
      if (lane < 16) {
        sm_p[w][t * 16 + lane][0] = p0;
        sm_p[w][t * 16 + lane][1] = p1;
      }
    }
  }
  if (tid == 0) zero_agent(&counters[g * kSpCntStride]);
  __syncthreads();
  // 4. one fixed-point atomic per logit of this group
  if (tid < 2 * MP) {
    const int tok = tid >> 1, c = tid & 1;
    if (tok < M) {
      const float pc = (sm_p[0][tok][c] + sm_p[1][tok][c]) + (sm_p[2][tok][c] + sm_p[3][tok][c]);
      // resolution 2^-32, magnitudes below 2^23
      unsigned long long* slot = acc_logit + static_cast<size_t>(2 * tok + c) * kSpAccStride;
      const long long fx = __float2ll_rn(pc * 4294967296.0f);
      const unsigned long long mine = (static_cast<unsigned long long>(fx) << 8) + 1ull;
      const unsigned long long old = __hip_atomic_fetch_add(slot, mine, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (static_cast<int>(old & 0xffull) == G - 1) {
        const long long total = static_cast<long long>(old + mine) >> 8;  // arithmetic shift drops the count
        a.logits[2 * tok + c] = static_cast<float>(static_cast<double>(total) * (1.0 / 4294967296.0)) + eb2[c];
        __hip_atomic_store(slot, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
    }
  }
}

template <int NT>
__global__ __launch_bounds__(kSpThreads) __attribute__((amdgpu_waves_per_eu(1, 2))) void score_splitk_kernel(ScoreArgs a, int G, int KS,
                                                                                                      int ppb) {
  score_splitk_block<NT>(a, G, KS, ppb, blockIdx.x);
}

}  // namespace dllava
