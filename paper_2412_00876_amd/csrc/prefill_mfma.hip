// Matrix-core causal attention over the reduced prefill set (Eq. 1 of the paper applied to S^{P*}), bfloat16.
//
// One block serves (sequence, head, tile of NWQ*32 compacted query rows); each of its NWQ waves owns 32
// queries and walks the key tiles (32 keys) up to its diagonal.  K and V tiles are staged through LDS once
// per block (next tile prefetched into registers while the current one is used).
//
// The score tile is computed TRANSPOSED, S^T = K Q^T (keys down the rows, queries across the columns) with
// v_mfma_f32_32x32x16_bf16.  In the result layout a lane then holds 16 keys of ONE query (its partner lane
// l^32 holds the other 16), so the online-softmax maximum and sum are register reductions plus a single
// cross-lane step, and the probabilities are already laid out as the B operand of the second product
// O^T = V^T P^T: they are split in place into two bfloat16 operands (16 significant bits) and never leave registers.  The contraction order of
// that second product is chosen to match the order in which S^T leaves the keys in a lane; V is stored
// transposed in LDS ([dim][key]) so that the matching A fragments are two 8-byte reads.
#include "attend.h"
#include "prefill_args.h"

namespace dllava {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));  // native vector: always promoted to registers

constexpr int kBN = 32;         // keys per tile
constexpr int kVPad = kBN + 4;  // V^T row (keys) padded: conflict-free 8-byte fragment reads

// Staging registers are named scalars (not arrays) so that they are certain to live in VGPRs.
template <int N>
struct Stage {
  u32x4 k0, k1, k2, k3, k4, k5, k6, k7;
  u32x4 v0, v1, v2, v3, v4, v5, v6, v7;
};
#define DLLAVA_FOR_STAGE(X) X(0) X(1) X(2) X(3) X(4) X(5) X(6) X(7)

// global -> registers: rows of K and V for key tile t (rows past last_key repeat it; the causal test masks them).
// PAGED: K/V come from the cache pages.  A tile of 32 keys lies in two pages whose ids are the same for the whole
// block, so they arrive as two scalar loads per tile (pg_lo for keys < 16 of the tile, pg_hi for the rest) and the
// 16-byte loads themselves are straight-line; a page-table lookup per load would put a dependent round trip, and a
// branch, in front of every one of them.
template <int DH, int N, int THREADS, bool PAGED>
__device__ __forceinline__ void stage_load(Stage<N>& st, const PrefillArgs& a, int t, int r0, int h, int last_key,
                                           int sr, int sc, int pg_lo, int pg_hi) {
  constexpr int kRowStep = THREADS / (DH / 8);
  const int H = a.H;
  const size_t tl = static_cast<size_t>(kPage) * DH;
#define DLLAVA_LD(i)                                                                              \
  if constexpr (i < N) {                                                                          \
    int key = t * kBN + sr + kRowStep * i;                                                        \
    if (key > last_key) key = last_key;                                                           \
    if constexpr (PAGED) {                                                                        \
      const int pg = (key - t * kBN) < kPage ? pg_lo : pg_hi;                                     \
      const size_t o = ((static_cast<size_t>(pg) * 2) * H + h) * tl +                             \
                       static_cast<size_t>(key % kPage) * DH + sc * 8;                            \
      const bf16_t* base = static_cast<const bf16_t*>(a.pages) + o;                               \
      st.k##i = *reinterpret_cast<const u32x4*>(base);                                            \
      st.v##i = *reinterpret_cast<const u32x4*>(base + static_cast<size_t>(H) * tl);              \
    } else {                                                                                      \
      const size_t o = (static_cast<size_t>(r0 + key) * H + h) * DH + sc * 8;                     \
      st.k##i = *reinterpret_cast<const u32x4*>(static_cast<const bf16_t*>(a.K) + o);             \
      st.v##i = *reinterpret_cast<const u32x4*>(static_cast<const bf16_t*>(a.V) + o);             \
    }                                                                                             \
  }
  DLLAVA_FOR_STAGE(DLLAVA_LD)
#undef DLLAVA_LD
}

// registers -> LDS: K rows as they are, V transposed to [dim][key]
template <int DH, int N, int THREADS>
__device__ __forceinline__ void stage_store(const Stage<N>& st, bf16_t* sK, bf16_t* sVt, int sr, int sc) {
  constexpr int kRowStep = THREADS / (DH / 8);
  constexpr int kKLd = DH + 8;
#define DLLAVA_ST(i)                                                                              \
  if constexpr (i < N) {                                                                          \
    const int row = sr + kRowStep * i;                                                            \
    *reinterpret_cast<u32x4*>(sK + row * kKLd + sc * 8) = st.k##i;                                \
    /* dims 8*sc + 0..7 of key `row`; the key position is XORed with 8*(dim/32) so that the 16 chunks */ \
    /* of a key row, whose V^T rows are 8*kVPad elements apart, do not fall on four banks only       */ \
    bf16_t* vt = sVt + (sc * 8) * kVPad + (row ^ (8 * (sc >> 2)));                                \
    const u32x4 v = st.v##i;                                                                      \
    vt[0 * kVPad] = static_cast<bf16_t>(v.x & 0xffffu);                                           \
    vt[1 * kVPad] = static_cast<bf16_t>(v.x >> 16);                                               \
    vt[2 * kVPad] = static_cast<bf16_t>(v.y & 0xffffu);                                           \
    vt[3 * kVPad] = static_cast<bf16_t>(v.y >> 16);                                               \
    vt[4 * kVPad] = static_cast<bf16_t>(v.z & 0xffffu);                                           \
    vt[5 * kVPad] = static_cast<bf16_t>(v.z >> 16);                                               \
    vt[6 * kVPad] = static_cast<bf16_t>(v.w & 0xffffu);                                           \
    vt[7 * kVPad] = static_cast<bf16_t>(v.w >> 16);                                               \
  }
  DLLAVA_FOR_STAGE(DLLAVA_ST)
#undef DLLAVA_ST
}

template <int DH, int NWQ>
__global__ __launch_bounds__(NWQ * kWave, NWQ >= 2 ? 2 : 1) void prefill_mfma_kernel(PrefillArgs a, int tiles_cap) {
  constexpr int kThreads = NWQ * kWave;
  constexpr int kBM = NWQ * 32;
  constexpr int kKLd = DH + 8;           // K tile row (elements), padded: conflict-free 16-byte fragment reads
  constexpr int kChunks = DH / 8;        // 16-byte chunks per row
  constexpr int kLoads = kBN * kChunks / kThreads;  // staging loads per thread per tile (K, and again V)
  constexpr int kDB = DH / 32;           // 32-dim blocks of the output
  static_assert(kLoads >= 1 && kLoads <= 8 && kLoads * kThreads == kBN * kChunks, "tile does not divide among the threads");

  __shared__ __align__(16) bf16_t sK[kBN * kKLd];
  __shared__ __align__(16) bf16_t sVt[DH * kVPad];

  const int tid = threadIdx.x, lane = tid & (kWave - 1), wq = tid / kWave;
  const int h = blockIdx.y, H = a.H;
  // which (sequence, query tile) is this block?  tiles are numbered sequence by sequence
  int b = 0, tile = blockIdx.x, n = 0, r0 = 0;
  for (;; ++b) {
    if (b >= a.B) return;
    r0 = a.off[b];
    n = a.off[b + 1] - r0;
    const int nt = (n + kBM - 1) / kBM;
    if (tile < nt) {
      // Causal attention: a sequence's late query tiles walk the most key tiles.  They are given the low block
      // ids of the sequence, so that the blocks dispatched last -- the tail of the launch -- are short ones.
      tile = nt - 1 - tile;
      break;
    }
    tile -= nt;
  }
  (void)tiles_cap;
  const int i0 = tile * kBM;            // first query row of the block (sequence-relative)
  const int iw = i0 + wq * 32;          // first query row of this wave
  const int g = lane >> 5, lq = lane & 31;
  const bf16_t* Qp = static_cast<const bf16_t*>(a.Q);

  // Q^T fragments of this wave: lane -> query iw + lq (clamped), 8 consecutive d at 16*ks + 8*g
  int qi = iw + lq;
  const bool q_ok = qi < n;
  if (!q_ok) qi = n - 1;
  uint4 qf[DH / 16];
  {
    const bf16_t* qrow = Qp + (static_cast<size_t>(r0 + qi) * H + h) * DH + 8 * g;
#pragma unroll
    for (int ks = 0; ks < DH / 16; ++ks) qf[ks] = *reinterpret_cast<const uint4*>(qrow + 16 * ks);
  }

  f32x16 o_acc[kDB];
#pragma unroll
  for (int nb = 0; nb < kDB; ++nb)
#pragma unroll
    for (int r = 0; r < 16; ++r) o_acc[nb][r] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;

  const int last_key = (i0 + kBM < n ? i0 + kBM : n) - 1;  // keys 0..last_key are needed by this block
  const int n_tiles = last_key / kBN + 1;

  // staging: thread -> (key row sr + (kThreads/kChunks)*i, chunk sc)
  const int sc = tid % kChunks, sr = tid / kChunks;
  Stage<kLoads> stg;
  const bool paged = a.K == nullptr;  // block-uniform
  const int32_t* bt = a.block_table + static_cast<size_t>(b) * a.max_pages;
  const int last_page = last_key / kPage;
  // page ids of tile t: block-uniform indices, so these are scalar loads
#define STAGE_LOAD(t)                                                                                      \
  {                                                                                                        \
    if (paged) {                                                                                           \
      const int p_lo = 2 * (t), p_hi = 2 * (t) + 1 < last_page ? 2 * (t) + 1 : last_page;                  \
      stage_load<DH, kLoads, kThreads, true>(stg, a, (t), r0, h, last_key, sr, sc, bt[p_lo], bt[p_hi]);    \
    } else {                                                                                               \
      stage_load<DH, kLoads, kThreads, false>(stg, a, (t), r0, h, last_key, sr, sc, 0, 0);                 \
    }                                                                                                      \
  }
#define STAGE_STORE() stage_store<DH, kLoads, kThreads>(stg, sK, sVt, sr, sc)

  STAGE_LOAD(0);
  for (int t = 0; t < n_tiles; ++t) {
    __syncthreads();  // the previous tile has been consumed
    STAGE_STORE();
    __syncthreads();
    if (t + 1 < n_tiles) STAGE_LOAD(t + 1);

    const int j0 = t * kBN;
    if (j0 > iw + 31) continue;  // tile lies entirely above this wave's diagonal (wave-uniform)

    // S^T = K Q^T : rows = keys j0..j0+31, columns = queries
    f32x16 s;
#pragma unroll
    for (int r = 0; r < 16; ++r) s[r] = 0.f;
#pragma unroll
    for (int ks = 0; ks < DH / 16; ++ks) {
      const uint4 kf = *reinterpret_cast<const uint4*>(sK + lq * kKLd + 16 * ks + 8 * g);
      union { uint4 u; bf16x8 f; } ka, qb;
      ka.u = kf;
      qb.u = qf[ks];
      s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka.f, qb.f, s, 0, 0, 0);
    }
    // lane holds keys j0 + 8*(r/4) + 4*g + r%4 of query qi
    const bool diag = j0 + kBN - 1 > iw;  // some key of the tile may exceed some query of the wave
    float tmax = -INFINITY;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      float v = s[r] * a.scale_log2;
      if (diag) {
        const int key = j0 + 8 * (r >> 2) + 4 * g + (r & 3);
        if (key > qi) v = -INFINITY;
      }
      s[r] = v;
      tmax = fmaxf(tmax, v);
    }
    tmax = fmaxf(tmax, __shfl_xor(tmax, 32, kWave));
    const float m_new = fmaxf(m_run, tmax);  // finite: key j0 <= iw <= qi is never masked in a visited tile
    const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
    // probabilities as TWO bfloat16 operands, p = p_hi + p_lo with p_hi the top 16 bits of p and p_lo the
    // top 16 bits of the (exact) remainder: 16 significant bits in all, so the second product is as accurate
    // as the float32 accumulation around it instead of carrying 2^-9 relative rounding on every weight
    float psum = 0.f;
    uint32_t pk_hi[8], pk_lo[8];
#pragma unroll
    for (int r = 0; r < 16; r += 2) {
      const float p0 = __builtin_amdgcn_exp2f(s[r] - m_new);
      const float p1 = __builtin_amdgcn_exp2f(s[r + 1] - m_new);
      psum += p0 + p1;
      const uint32_t b0 = __float_as_uint(p0), b1 = __float_as_uint(p1);
      pk_hi[r >> 1] = __builtin_amdgcn_perm(b1, b0, 0x07060302u);  // {hi16(p0), hi16(p1)}
      const float r0 = p0 - __uint_as_float(b0 & 0xffff0000u);
      const float r1 = p1 - __uint_as_float(b1 & 0xffff0000u);
      pk_lo[r >> 1] = __builtin_amdgcn_perm(__float_as_uint(r1), __float_as_uint(r0), 0x07060302u);
    }
    l_run = l_run * alpha + psum;
    m_run = m_new;
#pragma unroll
    for (int nb = 0; nb < kDB; ++nb)
#pragma unroll
      for (int r = 0; r < 16; ++r) o_acc[nb][r] *= alpha;

    // O^T += V^T P^T, two contraction steps of 16 keys; slot e of lane group g <-> the key held in s[8*half + e]
#pragma unroll
    for (int half = 0; half < 2; ++half) {
      union { uint32_t u[4]; bf16x8 f; } pb_hi, pb_lo;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        pb_hi.u[e] = pk_hi[4 * half + e];
        pb_lo.u[e] = pk_lo[4 * half + e];
      }
#pragma unroll
      for (int nb = 0; nb < kDB; ++nb) {
        // key positions are XORed with 8*nb in this block of 32 dims (see stage_store)
        const bf16_t* vrow = sVt + (nb * 32 + lq) * kVPad + 4 * g;
        union { uint2 u[2]; bf16x8 f; } va;
        va.u[0] = *reinterpret_cast<const uint2*>(vrow + ((16 * half) ^ (8 * nb)));      // keys 16*half + 4g + 0..3
        va.u[1] = *reinterpret_cast<const uint2*>(vrow + ((16 * half + 8) ^ (8 * nb)));  // keys 16*half + 8 + 4g + 0..3
        o_acc[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va.f, pb_hi.f, o_acc[nb], 0, 0, 0);
        o_acc[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va.f, pb_lo.f, o_acc[nb], 0, 0, 0);
      }
    }
  }

#undef STAGE_LOAD
#undef STAGE_STORE

  // l is split between the two lanes of a query
  l_run += __shfl_xor(l_run, 32, kWave);
  if (!q_ok) return;
  const float inv = 1.f / l_run;
  bf16_t* orow = static_cast<bf16_t*>(a.O) + (static_cast<size_t>(r0 + qi) * H + h) * DH;
#pragma unroll
  for (int nb = 0; nb < kDB; ++nb)
#pragma unroll
    for (int q4 = 0; q4 < 4; ++q4) {  // dims nb*32 + 8*q4 + 4*g + 0..3
      uint2 w2;
      w2.x = pack_bf16x2(o_acc[nb][4 * q4] * inv, o_acc[nb][4 * q4 + 1] * inv);
      w2.y = pack_bf16x2(o_acc[nb][4 * q4 + 2] * inv, o_acc[nb][4 * q4 + 3] * inv);
      *reinterpret_cast<uint2*>(orow + nb * 32 + 8 * q4 + 4 * g) = w2;
    }
}

template <int DH, int NWQ>
int launch(const PrefillArgs& a, int64_t rows, hipStream_t st) {
  constexpr int kBM = NWQ * 32;
  const int64_t tiles = ceil_div(rows, kBM) + a.B;  // upper bound on sum_b ceil(n_b / kBM)
  if (tiles > 0x7fffffffLL) return 1;
  dim3 grid(static_cast<unsigned>(tiles), static_cast<unsigned>(a.H));
  hipLaunchKernelGGL((prefill_mfma_kernel<DH, NWQ>), grid, dim3(NWQ * kWave), 0, st, a, static_cast<int>(tiles));
  DLLAVA_CHECK_LAUNCH("prefill_mfma_kernel");
  return DLLAVA_OK;
}

}  // namespace

// returns 1 if the shape is not handled here
int prefill_mfma_launch(const PrefillArgs& a, int64_t rows, int Dh, hipStream_t st) {
  if (a.H > 65535) return 1;
  // wide tiles (K/V tiles staged once for 128 queries) unless there is too little work to spread over the chip;
  // measured: 4 waves win from the 7B batch-1 prefill (214 rows x 32 heads) upwards
  const int64_t work = rows * a.H;  // query rows x heads
  int nwq = work >= 4 * 1024 ? 4 : (work >= 1024 ? 2 : 1);
  if (const char* e = getenv("DLLAVA_PREFILL_WAVES")) {  // tuning override
    const int v = atoi(e);
    if (v == 1 || v == 2 || v == 4) nwq = v;
  }
  if (Dh == 128) {
    if (nwq == 4) return launch<128, 4>(a, rows, st);
    if (nwq == 2) return launch<128, 2>(a, rows, st);
    return launch<128, 1>(a, rows, st);
  }
  if (Dh == 64) {
    if (nwq == 4) return launch<64, 4>(a, rows, st);
    if (nwq == 2) return launch<64, 2>(a, rows, st);
    return launch<64, 1>(a, rows, st);
  }
  return 1;
}

}  // namespace dllava
