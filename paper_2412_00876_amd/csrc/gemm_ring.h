// 256 x (32*JB) x d tile product on the matrix cores for the large bfloat16 products of the path (predictor scoring
// over all vision tokens, Q/K/V projection of the kept rows): one block of 4 waves per compute unit,
//   acc[i][j] (32 x 32) += A[a_wave_row0 + A_STRIDE*i + 0..31, :] . B[32*j + 0..31, :]^T ,   i < 2, j < JB,
// for the calling wave (64 rows of the 256-row A tile against all 32*JB rows of the B tile), with
// v_mfma_f32_32x32x16_bf16.  Both operands are contiguous along d and are streamed in 64-element stages (one whole
// 128-byte memory line per row).
//
// What shapes the loop (each point is a measurement on MI355X, not a guess):
//  * A compute unit pulls its operands from L2 at 40-45 bytes per clock at best, so the tile must be large: 256 x 256
//    needs 32 bytes per clock at the full matrix rate, 128 x 128 twice that.  The accumulators of the wave tile
//    (up to 64 x 256) fill the 256 accumulation registers; one wave per SIMD.
//  * Tiles go from global memory straight into LDS (global_load_lds_dwordx4, no staging registers).  A stage is 64 KiB,
//    LDS holds 160 KiB, and a tile requested one stage ahead does not arrive in time (latency plus transfer exceed a
//    stage's arithmetic), so the LDS is a ring of FIVE 32 KiB half-stage slots (B, A, B, A, ...): while stage k is
//    multiplied, A of stage k+1 and B of stages k+1 and k+2 are in flight or landed -- every tile is requested
//    a whole stage before the barrier that needs it.
//  * A wave issues in order: a burst of tile loads stalls it (the memory pipeline accepts about one 1 KiB load
//    per 25 clocks per compute unit) and the matrix pipe idles meanwhile (measured: products + loads took the SUM
//    of their times).  So the loads are dealt out one behind every other product, the fragment reads one behind each
//    of the first products of a k-step, and scheduling barriers keep the compiler from regrouping them.
//  * The stage barrier sits before the LAST k-step of a stage: by then the fragments of that k-step are in
//    registers, so the stage's slots are free, and the first fragments of the next stage are read behind the
//    products of the last k-step instead of after a barrier with nothing to hide them.
// LDS layout of a slot: row r at r*128 bytes, 16-byte chunk c of the row at position c ^ ((r/2) % 8): the 16 lanes
// that the LDS serves together hit 16 different bank groups both when a tile load deposits 8 rows x 8 chunks and
// when a fragment read takes one chunk of 16 rows.
#pragma once

#include "common.h"

namespace dllava {

typedef __bf16 ring_bf16x8 __attribute__((ext_vector_type(8)));
typedef float ring_f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t ring_u32x4 __attribute__((ext_vector_type(4)));

#define DLLAVA_LDS __attribute__((address_space(3)))
#define DLLAVA_GLB __attribute__((address_space(1)))

constexpr int kRingThreads = 256;
constexpr int kRingBK = 64;                       // elements of d per stage
constexpr int kRingRowBytes = 128;                // bytes per row per stage
constexpr int kRingSlotBytes = 256 * kRingRowBytes;
constexpr int kRingSlots = 5;
constexpr int kRingLdsBytes = kRingSlots * kRingSlotBytes;  // 160 KiB: all of a compute unit's LDS
constexpr int kRingALoads = 8;                    // tile loads per wave per stage for A (256 rows)

template <int OFF>
__device__ __forceinline__ ring_u32x4 ring_lds_read16(uint32_t addr) {
  ring_u32x4 v;
  asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF));
  return v;
}
__device__ __forceinline__ ring_bf16x8 ring_frag(const ring_u32x4& v) { return __builtin_bit_cast(ring_bf16x8, v); }

// Byte offset, from the first row of a tile, of the 16 bytes that this lane fetches with tile load j of wave w:
// the load covers rows 8*(w + 4j) + lane/8, the lane's position lane%8 holds chunk (lane%8) ^ ((row/2)%8).
// `row_of(r)` maps tile row r to the row of the matrix (clamping and gathering are the caller's).
__device__ __forceinline__ int ring_load_row(int w, int j, int lane) { return 8 * (w + 4 * j) + (lane >> 3); }
__device__ __forceinline__ uint32_t ring_load_chunk_bytes(int row, int lane) {
  return 16u * static_cast<uint32_t>((lane & 7) ^ ((row >> 1) & 7));
}

// The fragment registers pass through the waiting statement, so nothing that uses them can be scheduled above it.
template <int N>
__device__ __forceinline__ void ring_tie(ring_u32x4 (&f)[N]) {
#pragma unroll
  for (int i = 0; i < N; ++i) asm volatile("" : "+v"(f[i]));
}

// Main loop.  Abase / Bbase: wave-uniform byte pointers to element 0 of the tiles' first rows; ga[j] / gb[j]: this
// lane's byte offsets (ring_load_row / ring_load_chunk_bytes) for its tile loads; nk = d / 64 >= 1;
// w = wave index 0..3 (wave-uniform); a_wave_row0: first A-tile row of this wave's fragments (multiple of 32).
// Every row touched must be readable for all d (clamp rows past the end of a matrix to its last row).
// On return all LDS traffic of the loop has completed; the caller must still place a block barrier before it
// reuses the ring memory for something else.
// BOff: uint32_t, or int64_t when the rows of B may lie more than 4 GiB apart (gathered rows).
template <int JB, int A_STRIDE, typename BOff>
__device__ __forceinline__ void gemm_ring_256(const char* Abase, const uint32_t (&ga)[kRingALoads], const char* Bbase,
                                              const BOff (&gb)[JB], int nk, DLLAVA_LDS char* smem, int w,
                                              int a_wave_row0, ring_f32x16 (&acc)[2][JB]) {
  static_assert(JB >= 4 && JB <= 8, "B tile of 128 .. 256 rows");
  static_assert(A_STRIDE % 32 == 0 && A_STRIDE * kRingRowBytes < 65536, "fragment offset must fit the instruction");
  constexpr int kMF = 2 * JB;       // products per k-step
  constexpr int kNR = 2 + JB;       // fragment reads per k-step
  const int lane = threadIdx.x & (kWave - 1);
  const uint32_t s0 = static_cast<uint32_t>(reinterpret_cast<uintptr_t>(smem));
  const uint32_t fo = (lane & 31) * kRingRowBytes + (((lane >> 5) ^ ((lane >> 1) & 7)) * 16);
  const uint32_t fa_off = a_wave_row0 * kRingRowBytes + fo, fb_off = fo;

  ring_u32x4 ua[2], ub[JB], va[2], vb[JB];

#define RING_KOFF(kt) (static_cast<int64_t>((kt) < nk ? (kt) : nk - 1) * (kRingBK * 2))
#define RING_DMA(base, off, ko, slot, j)                                                                       \
  __builtin_amdgcn_global_load_lds((const DLLAVA_GLB void*)((base) + (ko) + (off)),                            \
                                   (DLLAVA_LDS void*)(smem + (slot) * kRingSlotBytes + (w + 4 * (j)) * 1024), 16, 0, 0);
  // fragment read idx of a k-step: 0, 1 = A rows + A_STRIDE*idx; 2 .. = B rows + 32*(idx-2)
#define RING_READ1(F, ab, bb, ks, idx)                                                                         \
  if constexpr ((idx) < 2) F##a[(idx) & 1] = ring_lds_read16<((idx) & 1) * A_STRIDE * kRingRowBytes>((ab) ^ ((ks) * 32)); \
  else if constexpr ((idx) < kNR) F##b[((idx) - 2) & 7] = ring_lds_read16<(((idx) - 2) & 7) * 4096>((bb) ^ ((ks) * 32));
#define RING_WAIT(F)                                \
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); \
  ring_tie(F##a);                                    \
  ring_tie(F##b);
#define RING_MFMA1(F, m)                                                                                        \
  acc[(m) / JB][(m) % JB] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ring_frag(F##a[(m) / JB]), ring_frag(F##b[(m) % JB]), \
                                                                    acc[(m) / JB][(m) % JB], 0, 0, 0);
  // Step m of a k-step: product m of set F; behind it, fragment read m of the NEXT k-step into set G, and one of the
  // k-step's tile loads if m is among its last NL steps (load index L0 + m - (kMF - NL) of kind X into `slot`).
#define RING_STEP(F, G, ab, bb, rks, X, off, ko, slot, L0, NL, m)                                              \
  if constexpr ((m) < kMF) {                                                                                   \
    RING_MFMA1(F, m)                                                                                           \
    RING_READ1(G, ab, bb, rks, m)                                                                              \
    if constexpr ((m) >= kMF - (NL)) { RING_DMA(X##base, off[((L0) + (m) - (kMF - (NL))) & 7], ko, slot, (L0) + (m) - (kMF - (NL))) } \
    __builtin_amdgcn_sched_barrier(0);                                                                         \
  }
#define RING_KSTEP(F, G, ab, bb, rks, X, off, ko, slot, L0, NL)                                                \
  RING_WAIT(F)                                                                                                 \
  RING_STEP(F, G, ab, bb, rks, X, off, ko, slot, L0, NL, 0) RING_STEP(F, G, ab, bb, rks, X, off, ko, slot, L0, NL, 1)   \
  RING_STEP(F, G, ab, bb, rks, X, off, ko, slot, L0, NL, 2) RING_STEP(F, G, ab, bb, rks, X, off, ko, slot, L0, NL, 3)   \
  RING_STEP(F, G, ab, bb, rks, X, off, ko, slot, L0, NL, 4) RING_STEP(F, G, ab, bb, rks, X, off, ko, slot, L0, NL, 5)   \
  RING_STEP(F, G, ab, bb, rks, X, off, ko, slot, L0, NL, 6) RING_STEP(F, G, ab, bb, rks, X, off, ko, slot, L0, NL, 7)   \
  RING_STEP(F, G, ab, bb, rks, X, off, ko, slot, L0, NL, 8) RING_STEP(F, G, ab, bb, rks, X, off, ko, slot, L0, NL, 9)   \
  RING_STEP(F, G, ab, bb, rks, X, off, ko, slot, L0, NL, 10) RING_STEP(F, G, ab, bb, rks, X, off, ko, slot, L0, NL, 11) \
  RING_STEP(F, G, ab, bb, rks, X, off, ko, slot, L0, NL, 12) RING_STEP(F, G, ab, bb, rks, X, off, ko, slot, L0, NL, 13) \
  RING_STEP(F, G, ab, bb, rks, X, off, ko, slot, L0, NL, 14) RING_STEP(F, G, ab, bb, rks, X, off, ko, slot, L0, NL, 15)

  // Half-stages in ring order: h(2k) = B of stage k, h(2k+1) = A of stage k; h(n) lives in slot n % 5.
  // Iteration k multiplies stage k and issues, into the slots that stage k-1 used, the second half of A(k+1)
  // (k-step 0), B(k+2) (k-steps 1 and 2), and after its barrier, into stage k's own B slot, the first half of A(k+2)
  // (k-step 3).  The barrier of iteration k needs B(k+1) and A(k+1): everything but the JB loads of B(k+2).
  constexpr int kB1 = (JB + 1) / 2, kB2 = JB - kB1;  // loads of B dealt to k-steps 1 and 2
  // prologue: B0, A0, B1, first half of A1
#pragma unroll
  for (int j = 0; j < JB; ++j) RING_DMA(Bbase, gb[j], RING_KOFF(0), 0, j)
#pragma unroll
  for (int j = 0; j < kRingALoads; ++j) RING_DMA(Abase, ga[j], RING_KOFF(0), 1, j)
#pragma unroll
  for (int j = 0; j < JB; ++j) RING_DMA(Bbase, gb[j], RING_KOFF(1), 2, j)
#pragma unroll
  for (int j = 0; j < 4; ++j) RING_DMA(Abase, ga[j], RING_KOFF(1), 3, j)
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(JB + 4) : "memory");
  __builtin_amdgcn_s_barrier();

  int sb = 0, sa = 1;  // slots of B and A of the stage being multiplied
  {
    const uint32_t ab = s0 + sa * kRingSlotBytes + fa_off, bb = s0 + sb * kRingSlotBytes + fb_off;
    RING_READ1(u, ab, bb, 0, 0) RING_READ1(u, ab, bb, 0, 1) RING_READ1(u, ab, bb, 0, 2) RING_READ1(u, ab, bb, 0, 3)
    RING_READ1(u, ab, bb, 0, 4) RING_READ1(u, ab, bb, 0, 5) RING_READ1(u, ab, bb, 0, 6) RING_READ1(u, ab, bb, 0, 7)
    RING_READ1(u, ab, bb, 0, 8) RING_READ1(u, ab, bb, 0, 9)
  }
  for (int kt = 0; kt < nk; ++kt) {
    const uint32_t ab = s0 + sa * kRingSlotBytes + fa_off, bb = s0 + sb * kRingSlotBytes + fb_off;
    const int sa1 = sb + 3 >= kRingSlots ? sb + 3 - kRingSlots : sb + 3;  // slot of A(k+1) = h(2k+3)
    const int sb1 = sb + 2 >= kRingSlots ? sb + 2 - kRingSlots : sb + 2;  // slot of B(k+1) = h(2k+2)
    const int sb2 = sb + 4 >= kRingSlots ? sb + 4 - kRingSlots : sb + 4;  // slot of B(k+2) = h(2k+4)
    const int64_t ko1 = RING_KOFF(kt + 1), ko2 = RING_KOFF(kt + 2);
    RING_KSTEP(u, v, ab, bb, 1, A, ga, ko1, sa1, 4, 4)
    RING_KSTEP(v, u, ab, bb, 2, B, gb, ko2, sb2, 0, kB1)
    RING_KSTEP(u, v, ab, bb, 3, B, gb, ko2, sb2, kB1, kB2)
    // the fragments of the last k-step are in registers: this wave is done with the stage's slots
    RING_WAIT(v)
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(JB) : "memory");
    __builtin_amdgcn_s_barrier();
    {
      // last k-step; behind it the first fragments of stage k+1 and the first half of A(k+2) into this stage's B slot
      const uint32_t nab = s0 + sa1 * kRingSlotBytes + fa_off, nbb = s0 + sb1 * kRingSlotBytes + fb_off;
      RING_STEP(v, u, nab, nbb, 0, A, ga, ko2, sb, 0, 4, 0) RING_STEP(v, u, nab, nbb, 0, A, ga, ko2, sb, 0, 4, 1)
      RING_STEP(v, u, nab, nbb, 0, A, ga, ko2, sb, 0, 4, 2) RING_STEP(v, u, nab, nbb, 0, A, ga, ko2, sb, 0, 4, 3)
      RING_STEP(v, u, nab, nbb, 0, A, ga, ko2, sb, 0, 4, 4) RING_STEP(v, u, nab, nbb, 0, A, ga, ko2, sb, 0, 4, 5)
      RING_STEP(v, u, nab, nbb, 0, A, ga, ko2, sb, 0, 4, 6) RING_STEP(v, u, nab, nbb, 0, A, ga, ko2, sb, 0, 4, 7)
      RING_STEP(v, u, nab, nbb, 0, A, ga, ko2, sb, 0, 4, 8) RING_STEP(v, u, nab, nbb, 0, A, ga, ko2, sb, 0, 4, 9)
      RING_STEP(v, u, nab, nbb, 0, A, ga, ko2, sb, 0, 4, 10) RING_STEP(v, u, nab, nbb, 0, A, ga, ko2, sb, 0, 4, 11)
      RING_STEP(v, u, nab, nbb, 0, A, ga, ko2, sb, 0, 4, 12) RING_STEP(v, u, nab, nbb, 0, A, ga, ko2, sb, 0, 4, 13)
      RING_STEP(v, u, nab, nbb, 0, A, ga, ko2, sb, 0, 4, 14) RING_STEP(v, u, nab, nbb, 0, A, ga, ko2, sb, 0, 4, 15)
    }
    sb = sb1;
    sa = sa1;
  }
  // the reads and loads issued for stages past the end (clamped to the last stage: in bounds, unused) are drained
  RING_WAIT(u)
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#undef RING_KOFF
#undef RING_DMA
#undef RING_READ1
#undef RING_WAIT
#undef RING_MFMA1
#undef RING_STEP
#undef RING_KSTEP
}

}  // namespace dllava
