// 128 x 128 x d tile product on the matrix cores, shared by the kernels that multiply a [128, d] tile of one
// bfloat16 matrix with a [128, d] tile of another (both contiguous along d):
//   acc[i][j] (32 x 32) += A[a_row0 + A_FRAG_STRIDE*i + 0..31, :] . B[b_row0 + 32*j + 0..31, :]^T
// for the calling wave, with v_mfma_f32_32x32x16_bf16.  256 threads; the hidden dimension is streamed in
// 64-element stages (whole 128-byte memory lines per row) through one swizzled LDS tile pair, the global loads
// two stages ahead in registers, LDS-only barriers.
#pragma once

#include "common.h"

namespace dllava {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ bf16x8 as_frag(const uint4& v) {
  union { uint4 u; bf16x8 f; } c;
  c.u = v;
  return c.f;
}

constexpr int kGThreads = 256;
constexpr int kBK = 64;             // hidden-dimension elements per pipeline stage: 128 bytes per row, one memory line
constexpr int kTileElems = 128 * kBK;

// Global -> registers -> LDS staging.  A stage is 128 bytes of each row, and 8 consecutive lanes fetch one
// row's piece as one whole memory line: a half-line piece (32 elements) moves the full line through the
// caches anyway and was measured at half the load throughput.  Thread: 16-byte chunk lc = tid%8 of rows
// lr + 32*j, lr = tid/8; gA[j] / gB[j] point at that chunk of stage 0 of those rows.
// LDS swizzle: chunk c of row r sits at chunk position c ^ ((r / 2) % 8).  The LDS serves a 16-byte access 16
// lanes at a time over 64 banks (16 bank groups of 16 bytes); with this placement the staging stores (2 rows
// x 8 chunks per 16 lanes) and the fragment loads (16 rows x 1 chunk) each touch 16 different bank groups.
template <int A_FRAG_STRIDE>
__device__ __forceinline__ void gemm_tile_128x128(const bf16_t* gA0, const bf16_t* gA1, const bf16_t* gA2,
                                                  const bf16_t* gA3, const bf16_t* gB0, const bf16_t* gB1,
                                                  const bf16_t* gB2, const bf16_t* gB3, int nk, bf16_t* sA,
                                                  bf16_t* sB, int a_row0, int b_row0, f32x16 (&acc)[2][2]) {
  const int tid = threadIdx.x, lane = tid & (kWave - 1);
  const int lc = tid & 7, lr = tid >> 3;
  const int st_off = lr * kBK + (lc ^ ((lr >> 1) & 7)) * 8;
  // two register sets: the loads of stages kt+1 and kt+2 are in flight while stage kt is multiplied
  u32x4 pa0, pa1, pa2, pa3, pb0, pb1, pb2, pb3, qa0, qa1, qa2, qa3, qb0, qb1, qb2, qb3;
  // Loads are issued unconditionally (past the end they re-read the last stage): a conditional load would make
  // the number of outstanding loads path-dependent, and the compiler would then wait for all of them before
  // every LDS store instead of only for the older register set.
#define DLLAVA_GLOAD(S, kt)                                                      \
  {                                                                              \
    const int64_t ko = static_cast<int64_t>((kt) < nk ? (kt) : nk - 1) * kBK;    \
    S##a0 = *reinterpret_cast<const u32x4*>(gA0 + ko);                           \
    S##a1 = *reinterpret_cast<const u32x4*>(gA1 + ko);                           \
    S##a2 = *reinterpret_cast<const u32x4*>(gA2 + ko);                           \
    S##a3 = *reinterpret_cast<const u32x4*>(gA3 + ko);                           \
    S##b0 = *reinterpret_cast<const u32x4*>(gB0 + ko);                           \
    S##b1 = *reinterpret_cast<const u32x4*>(gB1 + ko);                           \
    S##b2 = *reinterpret_cast<const u32x4*>(gB2 + ko);                           \
    S##b3 = *reinterpret_cast<const u32x4*>(gB3 + ko);                           \
  }
  // a stage past the end (odd stage count) is stored with a zero A tile, so it adds nothing
#define DLLAVA_SSTORE(S, kt)                                                     \
  {                                                                              \
    if ((kt) >= nk) S##a0 = S##a1 = S##a2 = S##a3 = u32x4{0u, 0u, 0u, 0u};       \
    *reinterpret_cast<u32x4*>(sA + st_off) = S##a0;                              \
    *reinterpret_cast<u32x4*>(sA + st_off + 32 * kBK) = S##a1;                   \
    *reinterpret_cast<u32x4*>(sA + st_off + 64 * kBK) = S##a2;                   \
    *reinterpret_cast<u32x4*>(sA + st_off + 96 * kBK) = S##a3;                   \
    *reinterpret_cast<u32x4*>(sB + st_off) = S##b0;                              \
    *reinterpret_cast<u32x4*>(sB + st_off + 32 * kBK) = S##b1;                   \
    *reinterpret_cast<u32x4*>(sB + st_off + 64 * kBK) = S##b2;                   \
    *reinterpret_cast<u32x4*>(sB + st_off + 96 * kBK) = S##b3;                   \
  }

  // fragment of k-step ks: chunk 2*ks + lane/32 of row lane%32 (+ multiples of 32), at its swizzled position
  const int ld_off = (lane & 31) * kBK + ((lane >> 5) ^ ((lane >> 1) & 7)) * 8;
#define DLLAVA_FRAGS(F, ks)                                                                              \
  _Pragma("unroll") for (int i = 0; i < 2; ++i) {                                                        \
    F##a[i] = as_frag(*reinterpret_cast<const uint4*>(tA + i * A_FRAG_STRIDE * kBK + (ld_off ^ ((ks) * 16)))); \
    F##b[i] = as_frag(*reinterpret_cast<const uint4*>(tB + i * 32 * kBK + (ld_off ^ ((ks) * 16))));      \
  }
#define DLLAVA_MFMAS(F)                                                                                  \
  _Pragma("unroll") for (int i = 0; i < 2; ++i)                                                          \
    _Pragma("unroll") for (int j = 0; j < 2; ++j)                                                        \
      acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(F##a[i], F##b[j], acc[i][j], 0, 0, 0);
  // two fragment sets: the LDS reads of k-step ks+1 are in flight while the products of ks are issued
#define DLLAVA_COMPUTE()                                                                                 \
  {                                                                                                      \
    const bf16_t* tA = sA + a_row0 * kBK;                                                                \
    const bf16_t* tB = sB + b_row0 * kBK;                                                                \
    bf16x8 ua[2], ub[2], va[2], vb[2];                                                                   \
    DLLAVA_FRAGS(u, 0)                                                                                   \
    DLLAVA_FRAGS(v, 1)                                                                                   \
    DLLAVA_MFMAS(u)                                                                                      \
    DLLAVA_FRAGS(u, 2)                                                                                   \
    DLLAVA_MFMAS(v)                                                                                      \
    DLLAVA_FRAGS(v, 3)                                                                                   \
    DLLAVA_MFMAS(u)                                                                                      \
    DLLAVA_MFMAS(v)                                                                                      \
  }

  // One LDS buffer (32 KiB, so three blocks share a compute unit): multiply stage kt, barrier, overwrite it with
  // stage kt+1 from the older register set, barrier.  Other resident blocks fill the barrier gaps.
  DLLAVA_GLOAD(p, 0)
  DLLAVA_GLOAD(q, 1)
  DLLAVA_SSTORE(p, 0)
  lds_barrier();
  for (int kt = 0; kt < nk; kt += 2) {
    DLLAVA_GLOAD(p, kt + 2)
    DLLAVA_COMPUTE()
    lds_barrier();
    DLLAVA_SSTORE(q, kt + 1)
    lds_barrier();
    DLLAVA_GLOAD(q, kt + 3)
    DLLAVA_COMPUTE()
    lds_barrier();
    DLLAVA_SSTORE(p, kt + 2)
    lds_barrier();
  }
#undef DLLAVA_GLOAD
#undef DLLAVA_SSTORE
#undef DLLAVA_COMPUTE
#undef DLLAVA_FRAGS
#undef DLLAVA_MFMAS

}

}  // namespace dllava
