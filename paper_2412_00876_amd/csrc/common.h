// Internal helpers shared by the dllava HIP sources (gfx950, 64-wide wavefronts).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>

#include "dllava.h"

namespace dllava {

constexpr int kWave = 64;
constexpr int kPage = 16;  // tokens per KV page

// ---- host-side error reporting -------------------------------------------------------------
void set_error(const char* fmt, ...) __attribute__((format(printf, 1, 2)));

#define DLLAVA_FAIL(code, ...)      \
  do {                              \
    ::dllava::set_error(__VA_ARGS__); \
    return (code);                  \
  } while (0)

#define DLLAVA_REQUIRE(cond, code, ...) \
  do {                                  \
    if (!(cond)) DLLAVA_FAIL(code, __VA_ARGS__); \
  } while (0)

// Checks the launch that was just issued.
#define DLLAVA_CHECK_LAUNCH(what)                                                        \
  do {                                                                                   \
    hipError_t e__ = hipGetLastError();                                                  \
    if (e__ != hipSuccess) DLLAVA_FAIL(DLLAVA_ELAUNCH, "%s: %s", what, hipGetErrorString(e__)); \
  } while (0)

inline bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }
inline size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }
inline size_t dtype_size(int dtype) { return dtype == DLLAVA_F32 ? 4 : 2; }
int check_cache(const dllava_kv_cache* c, const char* who);  // host validation of the struct
int launch_override(int knob);  // value set through dllava_set_launch_override, 0 = automatic

// ---- bfloat16 <-> float32 on the device ------------------------------------------------------
typedef uint16_t bf16_t;  // raw bit pattern

__device__ __forceinline__ float bf16_to_f32(bf16_t v) { return __uint_as_float(static_cast<uint32_t>(v) << 16); }
__device__ __forceinline__ float bf16lo_to_f32(uint32_t pair) { return __uint_as_float(pair << 16); }
__device__ __forceinline__ float bf16hi_to_f32(uint32_t pair) { return __uint_as_float(pair & 0xffff0000u); }

// round to nearest even; NaN stays NaN (quiet)
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return static_cast<bf16_t>((u >> 16) | 0x0040u);
  u += 0x7fffu + ((u >> 16) & 1u);
  return static_cast<bf16_t>(u >> 16);
}
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  return static_cast<uint32_t>(f32_to_bf16(lo)) | (static_cast<uint32_t>(f32_to_bf16(hi)) << 16);
}

template <typename T>
struct Elem;
template <>
struct Elem<float> {
  static constexpr int kPer16B = 4;
  __device__ static __forceinline__ void unpack(const uint4& r, float* f) {
    f[0] = __uint_as_float(r.x); f[1] = __uint_as_float(r.y);
    f[2] = __uint_as_float(r.z); f[3] = __uint_as_float(r.w);
  }
  __device__ static __forceinline__ float load(const float* p) { return *p; }
  __device__ static __forceinline__ void store(float* p, float v) { *p = v; }
};
template <>
struct Elem<bf16_t> {
  static constexpr int kPer16B = 8;
  __device__ static __forceinline__ void unpack(const uint4& r, float* f) {
    f[0] = bf16lo_to_f32(r.x); f[1] = bf16hi_to_f32(r.x);
    f[2] = bf16lo_to_f32(r.y); f[3] = bf16hi_to_f32(r.y);
    f[4] = bf16lo_to_f32(r.z); f[5] = bf16hi_to_f32(r.z);
    f[6] = bf16lo_to_f32(r.w); f[7] = bf16hi_to_f32(r.w);
  }
  __device__ static __forceinline__ float load(const bf16_t* p) { return bf16_to_f32(*p); }
  __device__ static __forceinline__ void store(bf16_t* p, float v) { *p = f32_to_bf16(v); }
};

// ---- wavefront helpers -----------------------------------------------------------------------
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
  return v;
}
__device__ __forceinline__ int wave_sum_i(int v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
  return v;
}
// inclusive prefix sum across the 64 lanes of a wave
__device__ __forceinline__ int wave_incl_scan(int v) {
  const int lane = threadIdx.x & (kWave - 1);
#pragma unroll
  for (int o = 1; o < kWave; o <<= 1) {
    int t = __shfl_up(v, o, kWave);
    if (lane >= o) v += t;
  }
  return v;
}

// ---- cross-block hand-off without cache flushes ----------------------------------------------------
// Data that one block leaves for another goes through device-scope relaxed atomics: the stores write
// through to the memory side and the loads miss the per-XCD caches, so no L2 write-back / invalidate
// (which a device-scope fence would cost on every block) is needed.  Protocol: every thread st_agent()s
// its values, block_publish() waits until those stores have been acknowledged and joins the block, one thread
// bumps the counter with add_agent(); the block that sees the final count ld_agent()s the data.
__device__ __forceinline__ void st_agent(float* p, float v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float ld_agent(const float* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ int add_agent(int* p, int v) {
  return __hip_atomic_fetch_add(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void zero_agent(int* p) { __hip_atomic_store(p, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
// All vector-memory operations this wave has issued, write-through stores included, have been acknowledged.
// (A workgroup-scope release fence is not enough: on this target it emits no wait at all, and the counter
// bump of another wave could then overtake the data.)
__device__ __forceinline__ void wave_stores_done() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }
__device__ __forceinline__ void block_publish() {
  wave_stores_done();
  __syncthreads();
}

// LDS-only block barrier: waits for this wave's LDS traffic, not for its outstanding global loads.  The generic
// __syncthreads() drains the vector-memory counter as well, which would stall every stage of the pipeline on
// the prefetches that were just issued.
__device__ __forceinline__ void lds_barrier() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
}

// The keep decision of Eq. 5 for one text token: margin of the float32 logits against a threshold.
__device__ __forceinline__ bool keep_from_logits(const float* logits, int row, float threshold) {
  const float margin = logits[2 * row + 1] - logits[2 * row];
  return margin > threshold;
}

// erf-form GELU, 0.5 a (1 + erf(a / sqrt 2)), with the library erff
__device__ __forceinline__ float gelu_erf(float a) { return 0.5f * a * (1.0f + erff(a * 0.70710678118654752440f)); }

// The same GELU with a branch-free erf: Abramowitz & Stegun 7.1.26,
//   erf(x) = 1 - (a1 t + ... + a5 t^5) exp(-x^2),  t = 1 / (1 + p x),  x >= 0,  |error| <= 1.5e-7,
// which is at the level of float32 rounding and keeps fused epilogues short (about a dozen instructions).
__device__ __forceinline__ float gelu_erf_fast(float a) {
  const float x = fabsf(a) * 0.70710678118654752440f;
  const float t = __builtin_amdgcn_rcpf(fmaf(0.3275911f, x, 1.0f));
  float poly = fmaf(1.061405429f, t, -1.453152027f);
  poly = fmaf(poly, t, 1.421413741f);
  poly = fmaf(poly, t, -0.284496736f);
  poly = fmaf(poly, t, 0.254829592f);
  poly *= t;
  const float e = __builtin_amdgcn_exp2f(-1.44269504088896340736f * x * x);
  const float erf_abs = fmaf(-poly, e, 1.0f);
  const float erf_signed = copysignf(erf_abs, a);
  return 0.5f * a * (1.0f + erf_signed);
}

}  // namespace dllava
