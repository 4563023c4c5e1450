// Wave-level streaming attention for ONE query vector: online softmax over 16-token chunks of
// K/V rows, plain VALU arithmetic.  Used where attention is bandwidth-bound (decode: one flop per
// byte, every K/V byte is used by exactly one query) and by the precision-generic prefill path.
//
// Lane mapping.  A token row of DH elements is covered by G = DH*sizeof(T)/16 lanes holding 16 bytes
// each; the wave's 64 lanes therefore cover R = 64/G consecutive token rows per load instruction, and
// a 16-token chunk takes NL = 16/R fully coalesced loads for K and NL for V.  Lane (r = lane/G,
// c = lane%G) owns elements [c*E, c*E+E) of the rows r, r+R, r+2R, ...  Each group of G lanes keeps
// its own running (max, sum, accumulator) and the R groups are merged once at the end, so the loop
// over chunks has no cross-group traffic: per row one E-term dot product, a log2(G)-step butterfly
// inside the group, and E fused multiply-adds for the value row.
#pragma once

#include "common.h"

namespace dllava {

template <typename T, int DH>
struct AttendCfg {
  static constexpr int E = 16 / sizeof(T);  // elements per lane per row
  static constexpr int G = DH / E;          // lanes per row
  static constexpr int R = kWave / G;       // rows per wave-wide load
  static constexpr int NL = kPage / R;      // loads per 16-token chunk
  static_assert(G * E == DH && R * G == kWave && NL * R == kPage, "unsupported head size");
};

template <int E>
struct AttnState {
  float m;  // running maximum of the scaled logits (log2 domain), -inf when empty
  float l;  // running sum of exp2(logit - m)
  float acc[E];
  __device__ __forceinline__ void clear() {
    m = -INFINITY;
    l = 0.f;
#pragma unroll
    for (int e = 0; e < E; ++e) acc[e] = 0.f;
  }
};

// Sum over the G lanes that share a token row.
template <int G>
__device__ __forceinline__ float group_sum(float v) {
#pragma unroll
  for (int o = G / 2; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
  return v;
}

// One 16-token chunk.  kbase/vbase point at element 0 of the chunk's first row for this head;
// consecutive rows are `stride` elements apart.  Rows >= nvalid are ignored (MASKED only).
// qs holds this lane's E query elements already multiplied by scale*log2(e).
template <typename T, int DH, bool MASKED>
__device__ __forceinline__ void attend_chunk(const T* __restrict__ kbase, const T* __restrict__ vbase,
                                             size_t stride, int nvalid, const float* qs,
                                             AttnState<AttendCfg<T, DH>::E>& st) {
  using C = AttendCfg<T, DH>;
  const int lane = threadIdx.x & (kWave - 1);
  const int r = lane / C::G, c = lane % C::G;
  uint4 kr[C::NL], vr[C::NL];
#pragma unroll
  for (int i = 0; i < C::NL; ++i) {
    const int tok = i * C::R + r;
    const bool ok = !MASKED || tok < nvalid;
    const size_t o = static_cast<size_t>(tok) * stride + c * C::E;
    kr[i] = ok ? *reinterpret_cast<const uint4*>(kbase + o) : make_uint4(0, 0, 0, 0);
    vr[i] = ok ? *reinterpret_cast<const uint4*>(vbase + o) : make_uint4(0, 0, 0, 0);
  }
  float s[C::NL];
  float mx = st.m;
#pragma unroll
  for (int i = 0; i < C::NL; ++i) {
    float kf[C::E];
    Elem<T>::unpack(kr[i], kf);
    float d = 0.f;
#pragma unroll
    for (int e = 0; e < C::E; ++e) d = fmaf(qs[e], kf[e], d);
    d = group_sum<C::G>(d);
    if (MASKED && (i * C::R + r) >= nvalid) d = -INFINITY;
    s[i] = d;
    mx = fmaxf(mx, d);
  }
  const float ms = (mx == -INFINITY) ? 0.f : mx;  // keeps exp2 arguments finite when nothing is valid yet
  const float alpha = exp2f(st.m - ms);           // st.m == -inf -> 0
  st.l *= alpha;
#pragma unroll
  for (int e = 0; e < C::E; ++e) st.acc[e] *= alpha;
#pragma unroll
  for (int i = 0; i < C::NL; ++i) {
    const float p = exp2f(s[i] - ms);  // masked rows: exp2(-inf) = 0 and their values were loaded as 0
    st.l += p;
    float vf[C::E];
    Elem<T>::unpack(vr[i], vf);
#pragma unroll
    for (int e = 0; e < C::E; ++e) st.acc[e] = fmaf(p, vf[e], st.acc[e]);
  }
  st.m = mx;
}

// A single extra row (the current token of a decode step) folded into group r == 0 only.
template <typename T, int DH>
__device__ __forceinline__ void attend_single(const T* __restrict__ krow, const T* __restrict__ vrow,
                                              const float* qs, AttnState<AttendCfg<T, DH>::E>& st) {
  using C = AttendCfg<T, DH>;
  const int lane = threadIdx.x & (kWave - 1);
  const int r = lane / C::G, c = lane % C::G;
  const uint4 kr = *reinterpret_cast<const uint4*>(krow + c * C::E);
  const uint4 vr = *reinterpret_cast<const uint4*>(vrow + c * C::E);
  float kf[C::E], vf[C::E];
  Elem<T>::unpack(kr, kf);
  Elem<T>::unpack(vr, vf);
  float d = 0.f;
#pragma unroll
  for (int e = 0; e < C::E; ++e) d = fmaf(qs[e], kf[e], d);
  d = group_sum<C::G>(d);
  if (r != 0) return;
  const float mx = fmaxf(st.m, d);
  const float alpha = exp2f(st.m - mx);
  const float p = exp2f(d - mx);
  st.l = st.l * alpha + p;
#pragma unroll
  for (int e = 0; e < C::E; ++e) st.acc[e] = fmaf(p, vf[e], st.acc[e] * alpha);
  st.m = mx;
}

// Merge the R row groups of a wave; afterwards every lane with the same c holds the same state.
template <typename T, int DH>
__device__ __forceinline__ void merge_groups(AttnState<AttendCfg<T, DH>::E>& st) {
  using C = AttendCfg<T, DH>;
#pragma unroll
  for (int o = C::G; o < kWave; o <<= 1) {
    const float m2 = __shfl_xor(st.m, o, kWave);
    const float l2 = __shfl_xor(st.l, o, kWave);
    const float M = fmaxf(st.m, m2);
    const float a = (st.m == -INFINITY) ? 0.f : exp2f(st.m - M);
    const float b = (m2 == -INFINITY) ? 0.f : exp2f(m2 - M);
    st.l = st.l * a + l2 * b;
#pragma unroll
    for (int e = 0; e < C::E; ++e) {
      const float a2 = __shfl_xor(st.acc[e], o, kWave);
      st.acc[e] = st.acc[e] * a + a2 * b;
    }
    st.m = M;
  }
}

// Load this lane's E query elements, scaled by scale*log2(e) so that softmax can use exp2.
template <typename T, int DH>
__device__ __forceinline__ void load_query(const T* __restrict__ qrow, float scale_log2, float* qs) {
  using C = AttendCfg<T, DH>;
  const int c = (threadIdx.x & (kWave - 1)) % C::G;
  const uint4 qr = *reinterpret_cast<const uint4*>(qrow + c * C::E);
  Elem<T>::unpack(qr, qs);
#pragma unroll
  for (int e = 0; e < C::E; ++e) qs[e] *= scale_log2;
}

}  // namespace dllava
