// Predictor scoring for a handful of rows (decode: one row per sequence), bfloat16, as block-level routines.
//
// Bandwidth-bound on W1 (it is read exactly once per call).  Block `blk` of `nblk` owns 16 hidden units; its
// WAVES waves each take a slice of d with v_mfma_f32_16x16x32_bf16 in the transposed orientation (hidden units
// down the rows, tokens across the columns) on fragments loaded straight from global memory, many loads in
// flight together; LDS reduction over the slices in slice order, bias + GELU + contraction with W2 in
// registers, one partial logit pair per token and block, summed across blocks in integer arithmetic by
// device-scope atomics (order-independent, hence bit-reproducible; see the end of the routine).
#pragma once

#include "score_args.h"

namespace dllava {

typedef __bf16 sk_bf16x8 __attribute__((ext_vector_type(8)));
typedef float sk_f32x4 __attribute__((ext_vector_type(4)));

constexpr int kSkUnits = 16;
constexpr int kSkSlices = 8;  // independent slices of d, summed in slice order

__device__ __forceinline__ sk_bf16x8 sk_frag(const uint4& v) {
  union { uint4 u; sk_bf16x8 f; } c;
  c.u = v;
  return c.f;
}

// One accumulator per logit, 256 bytes apart (atomics that share a memory line serialise at the memory side).
constexpr int kSkAccStride = 32;  // in 8-byte words

// BATCH = k-steps whose loads are issued together (more in flight = shorter, but more registers).
// acc = zero-filled accumulators [2*M][kSkAccStride] (left zero-filled again); nblk <= 255.
template <int NT, int WAVES, int BATCH>
__device__ __forceinline__ void score_skinny_block(const ScoreArgs& a, int blk, int nblk, unsigned long long* acc) {
  static_assert(kSkSlices % WAVES == 0, "waves must divide the slices");
  static_assert(BATCH % 2 == 0, "k-steps are issued in pairs");
  __shared__ float red[kSkSlices][NT][kWave][4];
  const int tid = threadIdx.x, lane = tid & (kWave - 1), w = tid / kWave;
  const int M = static_cast<int>(a.M);
  const int64_t d = a.d;
  const bf16_t* W1 = static_cast<const bf16_t*>(a.W1);
  const bf16_t* W2 = static_cast<const bf16_t*>(a.W2);
  const bf16_t* X = static_cast<const bf16_t*>(a.x);

  // fragment addressing: lane -> (row = lane%16, 8 consecutive k at 8*(lane/16))
  int64_t unit = static_cast<int64_t>(blk) * kSkUnits + (lane & 15);
  if (unit >= a.dh) unit = a.dh - 1;  // clamped rows are masked out below
  const bf16_t* wrow = W1 + unit * d + 8 * (lane >> 4);
  const bf16_t* xrow[NT];
#pragma unroll
  for (int t = 0; t < NT; ++t) {
    int tok = t * 16 + (lane & 15);
    if (tok >= M) tok = M - 1;
    xrow[t] = X + static_cast<int64_t>(tok) * a.ldx + 8 * (lane >> 4);
  }
  // Epilogue operands, requested now so that they are there when the products are; operands that must be zero
  // (no bias, unit past dh) come from kZeroWords through the address, so that no load sits under a condition.
  float eb[4], ew0[4], ew1[4], eb2[2];
  {
    const bool has_b1 = a.b1 != nullptr;
    const bf16_t* zero16 = reinterpret_cast<const bf16_t*>(kZeroWords);
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int64_t u = static_cast<int64_t>(blk) * kSkUnits + 4 * (lane >> 4) + r;
      const bool ok = u < a.dh;
      eb[r] = *((ok & has_b1) ? a.b1 + u : kZeroWords);
      ew0[r] = bf16_to_f32(*(ok ? W2 + u : zero16));
      ew1[r] = bf16_to_f32(*(ok ? W2 + a.dh + u : zero16));
    }
    eb2[0] = *(a.b2 ? a.b2 : kZeroWords);
    eb2[1] = *(a.b2 ? a.b2 + 1 : kZeroWords);
  }
  // d is split among kSkSlices slices, each accumulated on its own, so the arithmetic does not depend on how many
  // waves the block has (wave w takes slices w, w+WAVES, ..).  The unit of the split is a PAIR of k-steps = 64
  // elements = one 128-byte memory line per row: slice v takes the pairs v, v+8, ...; its two 64-byte fragment
  // loads of a row are issued back to back and the line crosses the memory system once.
  // BATCH k-steps are in flight at a time: the routine is a stream over W1, so what matters is the number of
  // outstanding 16-byte loads, not the MFMA rate.
  const int npairs = static_cast<int>(d / 64);
  // blocks start at different columns, so that they do not sweep W1 in lockstep through the same few memory
  // channels (rows are 2*d bytes apart); the order of a block's sum is fixed by its index
  const int rot = npairs / nblk > 0 ? npairs / nblk : 1;
  const int shift = (blk * rot) % npairs;  // this block's first column, in pairs
  for (int v = w; v < kSkSlices; v += WAVES) {
    sk_f32x4 acc[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) acc[t] = sk_f32x4{0.f, 0.f, 0.f, 0.f};
    const int n_it = 2 * ((npairs - v + kSkSlices - 1) / kSkSlices);
    for (int it0 = 0; it0 < n_it; it0 += BATCH) {
      uint4 ra[BATCH], rb[NT][BATCH];
#pragma unroll
      for (int u = 0; u < BATCH; ++u) {
        const bool ok = it0 + u < n_it;
        // in range: v + 8*i < npairs and shift < npairs, so one wrap at most; past the end: pair 0, result unused
        int pair = ok ? v + ((it0 + u) >> 1) * kSkSlices + shift : 0;
        if (pair >= npairs) pair -= npairs;
        const int ks = 2 * pair + (u & 1);  // it0 and BATCH are even
        const int64_t ko = static_cast<int64_t>(ks) * 32;
        ra[u] = *reinterpret_cast<const uint4*>(wrow + ko);
        if (!ok) ra[u] = make_uint4(0, 0, 0, 0);  // a zero W1 fragment contributes nothing
#pragma unroll
        for (int t = 0; t < NT; ++t) rb[t][u] = *reinterpret_cast<const uint4*>(xrow[t] + ko);
      }
#pragma unroll
      for (int u = 0; u < BATCH; ++u)
#pragma unroll
        for (int t = 0; t < NT; ++t)
          acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(sk_frag(ra[u]), sk_frag(rb[t][u]), acc[t], 0, 0, 0);
    }
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
      for (int r = 0; r < 4; ++r) red[v][t][lane][r] = acc[t][r];
  }
  __syncthreads();

  // wave 0 finishes: sum over waves (fixed order), bias, GELU, contraction with W2 over this block's units
  if (w == 0) {
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      float p0 = 0.f, p1 = 0.f;
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        float s = 0.f;
#pragma unroll
        for (int i = 0; i < kSkSlices; ++i) s += red[i][t][lane][r];
        const float g = gelu_erf_fast(s + eb[r]);  // units past dh carry zero weights
        p0 = fmaf(g, ew0[r], p0);
        p1 = fmaf(g, ew1[r], p1);
      }
      p0 += __shfl_xor(p0, 16, kWave);
      p1 += __shfl_xor(p1, 16, kWave);
      p0 += __shfl_xor(p0, 32, kWave);
      p1 += __shfl_xor(p1, 32, kWave);
      // Cross-block sum without a second pass.  Each partial is added, as a 64-bit fixed-point number (resolution
      // 2^-32, magnitudes below 2^23), to the logit's accumulator with one
      // returning device-scope atomic; the low 8 bits of the same word count the arrivals.  Integer addition is
      // associative, so the sum does not depend on the order of arrival, and
      // the block whose atomic returns the last count holds the total: it converts, adds the bias, writes the
      // logit and clears the accumulator.  One memory round trip instead of store + counter + reload.
      const int tok = t * 16 + lane;
      if (lane < 16 && tok < M) {
        const float pc[2] = {p0, p1};
#pragma unroll
        for (int c = 0; c < 2; ++c) {
          unsigned long long* slot = acc + static_cast<size_t>(2 * tok + c) * kSkAccStride;
          const long long fx = __float2ll_rn(pc[c] * 4294967296.0f);
          const unsigned long long mine = (static_cast<unsigned long long>(fx) << 8) + 1ull;
          const unsigned long long old =
              __hip_atomic_fetch_add(slot, mine, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          if (static_cast<int>(old & 0xffull) == nblk - 1) {
            const long long total = static_cast<long long>(old + mine) >> 8;  // arithmetic shift drops the count
            a.logits[2 * tok + c] = static_cast<float>(static_cast<double>(total) * (1.0 / 4294967296.0)) +
                                    eb2[c];
            __hip_atomic_store(slot, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          }
        }
      }
    }
  }
}

}  // namespace dllava
