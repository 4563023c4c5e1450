// Matrix-core causal attention over the reduced prefill set (Eq. 1 of the paper applied to S^{P*}), bfloat16.
//
// One block serves (sequence, head, tile of NWQ*32 compacted query rows); each of its NWQ waves owns 32
// queries and walks the key tiles (32 keys) up to its diagonal.  K and V tiles go from global memory straight
// into a ring of three LDS buffers (asynchronous loads, two tiles ahead of the one in use; one block barrier
// per tile).
//
// The score tile is computed TRANSPOSED, S^T = K Q^T (keys down the rows, queries across the columns) with
// v_mfma_f32_32x32x16_bf16.  In the result layout a lane then holds 16 keys of ONE query (its partner lane
// l^32 holds the other 16), so the online-softmax maximum and sum are register reductions plus a single
// cross-lane step, and the probabilities are already laid out as the B operand of the second product
// O^T = V^T P^T: they are split in place into two bfloat16 operands (16 significant bits) and never leave
// registers.  The contraction order of that second product is chosen to match the order in which S^T leaves
// the keys in a lane; V stays row-major ([key][dim]) in LDS and the matching A fragments (four consecutive keys
// of one dim per lane) come from the transposing LDS read of this target.
#include <type_traits>

#include "attend.h"
#include "prefill_args.h"

namespace dllava {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));  // native vector: always promoted to registers

constexpr int kBN = 32;  // keys per tile
#define DLLAVA_LDS __attribute__((address_space(3)))
#define DLLAVA_GLB __attribute__((address_space(1)))

// Tile staging.  K and V rows of a key tile go from global memory straight into LDS (no registers in between):
// a wave-wide 16-byte load deposits its 64 pieces at consecutive LDS addresses, i.e. 1 KiB = 64/(DH/8) whole rows,
// so a tile is row-major without padding and bank conflicts are avoided by permuting the 16-byte chunks of a row
// on the way in (the lane that fills physical chunk pc of tile row rr fetches logical chunk pc ^ f(rr)):
//   K: f(rr) = rr mod chunks-per-row.  The 16 lanes that read one logical chunk of 16 different rows hit 16 different bank groups.
//   V: f(rr) = 4*(rr mod chunks/4).   V is read with the transposing LDS load (4 keys x 16 dims per 16 lanes); the
//      4 keys of such a read then lie in 4 different 64-byte bank groups.
// Rows past the last needed key repeat it (lim = last_key - t*kBN): the causal test masks them, but they must
// hold finite data, which unwritten page slots need not.
template <int DH, int NWQ>
struct Dma {
  static constexpr int kChunks = DH / 8;            // 16-byte chunks per row
  static constexpr int kRowsPerLoad = kWave / kChunks;
  static constexpr int kLoads = kBN / (kRowsPerLoad * NWQ);  // wave-wide loads per wave per tile, for K and again for V
  static_assert(kLoads >= 1 && kLoads * kRowsPerLoad * NWQ == kBN, "tile does not divide among the waves");

  // paged: lo/hi = this head's K rows of the two pages of the tile, V rows v_off elements further
  static __device__ __forceinline__ void paged(bf16_t* sK, bf16_t* sV, const bf16_t* lo, const bf16_t* hi, uint32_t v_off,
                                               int lim, int wq, int lane) {
#pragma unroll
    for (int i = 0; i < kLoads; ++i) {
      const int slab = wq + NWQ * i;  // which 1 KiB of the tile
      const int rr = kRowsPerLoad * slab + lane / kChunks, pc = lane % kChunks;
      const int row = rr < lim ? rr : lim;
      const bf16_t* src = (row < kPage ? lo : hi) + (row % kPage) * DH;
      __builtin_amdgcn_global_load_lds((const DLLAVA_GLB void*)(src + 8 * (pc ^ (rr % kChunks))),
                                       (DLLAVA_LDS void*)(sK + slab * (kWave * 8)), 16, 0, 0);
      __builtin_amdgcn_global_load_lds((const DLLAVA_GLB void*)(src + v_off + 8 * (pc ^ (4 * (rr % (kChunks / 4))))),
                                       (DLLAVA_LDS void*)(sV + slab * (kWave * 8)), 16, 0, 0);
    }
  }
  // plain rows: gk / gv = row 0 of the tile for this head, consecutive rows row_stride elements apart
  static __device__ __forceinline__ void rows(bf16_t* sK, bf16_t* sV, const bf16_t* gk, const bf16_t* gv,
                                              uint32_t row_stride, int lim, int wq, int lane) {
#pragma unroll
    for (int i = 0; i < kLoads; ++i) {
      const int slab = wq + NWQ * i;
      const int rr = kRowsPerLoad * slab + lane / kChunks, pc = lane % kChunks;
      const int row = rr < lim ? rr : lim;
      const uint32_t o = static_cast<uint32_t>(row) * row_stride;
      __builtin_amdgcn_global_load_lds((const DLLAVA_GLB void*)(gk + o + 8 * (pc ^ (rr % kChunks))),
                                       (DLLAVA_LDS void*)(sK + slab * (kWave * 8)), 16, 0, 0);
      __builtin_amdgcn_global_load_lds((const DLLAVA_GLB void*)(gv + o + 8 * (pc ^ (4 * (rr % (kChunks / 4))))),
                                       (DLLAVA_LDS void*)(sV + slab * (kWave * 8)), 16, 0, 0);
    }
  }
};

// The running maximum is only a reference point of the exponentials: any value within a few powers of two of the
// true maximum serves.  The accumulators are rescaled only when some query's tile maximum exceeds its reference by
// more than this many powers of two (probabilities then stay below 2^kSlack; their bfloat16 split is relative, so
// nothing is lost), which after the first tile of a sequence is rare: the 64 multiplications of the output
// accumulator leave the common path.
constexpr float kSlack = 8.f;

// LDS reads of the tiles are written as instructions: the compiler would otherwise order every LDS read after ALL
// outstanding asynchronous fills (it cannot tell the buffers apart) and so wait for the tiles just requested.
// The reads return in order; lds_wait() is the point after which all of them have arrived.
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ u32x4 lds_read16(uint32_t addr) {
  u32x4 v;
  asm volatile("ds_read_b128 %0, %1" : "=v"(v) : "v"(addr) : "memory");
  return v;
}
template <int OFF>
__device__ __forceinline__ u32x2 lds_read8_tr16(uint32_t addr) {
  u32x2 v;
  asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF) : "memory");
  return v;
}

// One key tile for one wave.  diag: some score of the tile has to be masked: the tile reaches above the diagonal of
// some query of the wave (keys > qi), or kmask (bit i: key j0 + i may be seen by other queries than itself) has a
// zero bit.
// kb / vb: LDS byte addresses of this lane's first K and V fragment pieces in the tile (see the kernel).
template <int DH, bool MASKED>
__device__ __forceinline__ void tile_step(uint32_t kb, uint32_t vb_in, const uint4 (&qf)[DH / 16],
                                          f32x16 (&o_acc)[DH / 32], float& m_ref, float& l_run, float scale_log2,
                                          int j0, int qi, int g, bool diag, uint32_t kmask, int q_self) {
  constexpr int kDB = DH / 32;
  constexpr int kRowBytes = DH * 2;
  uint32_t vb = vb_in;
  // S^T = K Q^T : rows = keys j0..j0+31, columns = queries
  u32x4 kf[DH / 16];
#pragma unroll
  for (int ks = 0; ks < DH / 16; ++ks) kf[ks] = lds_read16(kb ^ (ks * 32));
  // The fragments pass through the waiting statement, so that nothing that uses them can be scheduled ahead of it.
  static_assert(DH == 128 || DH == 64, "fragment lists below are written out for these head sizes");
  if constexpr (DH == 128)
    asm volatile("s_waitcnt lgkmcnt(0)"
                 : "+v"(kf[0]), "+v"(kf[1]), "+v"(kf[2]), "+v"(kf[3]), "+v"(kf[4]), "+v"(kf[5]), "+v"(kf[6]), "+v"(kf[7])
                 :
                 : "memory");
  else
    asm volatile("s_waitcnt lgkmcnt(0)"
                 : "+v"(kf[0]), "+v"(kf[1]), "+v"(kf[2]), "+v"(kf[3])
                 :
                 : "memory");
  f32x16 s;
#pragma unroll
  for (int r = 0; r < 16; ++r) s[r] = 0.f;
#pragma unroll
  for (int ks = 0; ks < DH / 16; ++ks) {
    union { u32x4 u; bf16x8 f; } ka;
    union { uint4 u; bf16x8 f; } qb;
    ka.u = kf[ks];
    qb.u = qf[ks];
    s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka.f, qb.f, s, 0, 0, 0);
  }
  // V^T fragments: slot e of lane group g <-> the key held in s[8*half + e], i.e. keys 16*half + 8*u + 4*g + 0..3
  // for u = e/4: one transposing read each.  Requested once the
  // K fragments are used up (the address passes through a statement that reads the scores), they arrive while the
  // softmax runs.
  u32x2 vf[kDB][2][2];
  asm volatile("" : "+v"(vb) : "v"(s[0]));
#pragma unroll
  for (int nb = 0; nb < kDB; ++nb) {
    const uint32_t va = vb ^ (nb * 64);
    vf[nb][0][0] = lds_read8_tr16<0 * kRowBytes>(va);
    vf[nb][0][1] = lds_read8_tr16<8 * kRowBytes>(va);
    vf[nb][1][0] = lds_read8_tr16<16 * kRowBytes>(va);
    vf[nb][1][1] = lds_read8_tr16<24 * kRowBytes>(va);
  }
  // lane holds keys j0 + 8*(r/4) + 4*g + r%4 of query qi
  if (diag) {  // wave-uniform; kept a branch (not sixteen selects on every tile) by the empty statement
    asm volatile("" ::: "memory");
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int key = j0 + 8 * (r >> 2) + 4 * g + (r & 3);
      const bool open = !MASKED || ((kmask >> (8 * (r >> 2) + (r & 3) + 4 * g)) & 1u);
      if (key > qi || (!open && key != q_self)) s[r] = -INFINITY;
    }
  }
  float tmax = -INFINITY;
#pragma unroll
  for (int r = 0; r < 16; ++r) tmax = fmaxf(tmax, s[r]);
  tmax = fmaxf(tmax, __shfl_xor(tmax, 32, kWave));
  // scale > 0: the maximum of the scaled scores; -inf for a query that sees no key of this tile (possible with key
  // masks only).  m_ref starts at a finite floor, so such a tile leaves the query's state as it is (alpha = 1, p = 0).
  const float m_t = tmax * scale_log2;
  if (__any(m_t > m_ref + kSlack)) {
    const float m_new = fmaxf(m_ref, m_t);
    const float alpha = __builtin_amdgcn_exp2f(m_ref - m_new);
    m_ref = m_new;
    l_run *= alpha;
#pragma unroll
    for (int nb = 0; nb < kDB; ++nb)
#pragma unroll
      for (int r = 0; r < 16; ++r) o_acc[nb][r] *= alpha;
  }
  // probabilities as TWO bfloat16 operands, p = p_hi + p_lo with p_hi the top 16 bits of p and p_lo the
  // top 16 bits of the (exact) remainder: 16 significant bits in all, so the second product is as accurate
  // as the float32 accumulation around it instead of carrying 2^-9 relative rounding on every weight
  float psum = 0.f;
  uint32_t pk_hi[8], pk_lo[8];
#pragma unroll
  for (int r = 0; r < 16; r += 2) {
    const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[r], scale_log2, -m_ref));
    const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[r + 1], scale_log2, -m_ref));
    psum += p0 + p1;
    const uint32_t b0 = __float_as_uint(p0), b1 = __float_as_uint(p1);
    pk_hi[r >> 1] = __builtin_amdgcn_perm(b1, b0, 0x07060302u);  // {hi16(p0), hi16(p1)}
    const float r0 = p0 - __uint_as_float(b0 & 0xffff0000u);
    const float r1 = p1 - __uint_as_float(b1 & 0xffff0000u);
    pk_lo[r >> 1] = __builtin_amdgcn_perm(__float_as_uint(r1), __float_as_uint(r0), 0x07060302u);
  }
  l_run += psum;

  // O^T += V^T P^T, two contraction steps of 16 keys
#pragma unroll
  for (int nb = 0; nb < kDB; ++nb)  // as above: all reads have arrived, and the V fragments are used after this point only
    asm volatile("s_waitcnt lgkmcnt(0)"
                 : "+v"(vf[nb][0][0]), "+v"(vf[nb][0][1]), "+v"(vf[nb][1][0]), "+v"(vf[nb][1][1])
                 :
                 : "memory");
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
      union { u32x2 h[2]; bf16x8 f; } va;
      va.h[0] = vf[nb][half][0];
      va.h[1] = vf[nb][half][1];
      o_acc[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va.f, pb_hi.f, o_acc[nb], 0, 0, 0);
      o_acc[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va.f, pb_lo.f, o_acc[nb], 0, 0, 0);
    }
  }
}

// One work item = (sequence, head, tile of NWQ*32 compacted query rows).  Blocks are PERSISTENT: the launch holds as
// many blocks as fit the chip at once (slots), block p takes every slots-th item and walks their key
// tiles as ONE stream: the tile loads run two tiles ahead of the arithmetic across item boundaries, the page ids one
// step further, the queries of the next item are requested (into a second register set) when the current item begins,
// and an item's outputs are stored after the first tile of the next item has been requested.  A block that starts
// needs four or five dependent trips to memory before its first tile (offsets, page ids, queries, tile): with one
// item per block every item paid them (measured: 4-6 us per block against 4-14 us of arithmetic, the compute units
// idle two thirds of the time); a persistent block pays them once.
// Items are numbered by DESCENDING query-tile index over all sequences, heads adjacent: a causal item's work grows
// with its tile index, so every block takes its longest items first and the launch ends with the shortest ones.
// MASKED: the variant with key masks (a.key_words); the plain kernel carries none of its registers.
template <int DH, int NWQ, bool MASKED>
__global__ __launch_bounds__(NWQ * kWave, (NWQ >= 2 && !MASKED) ? 2 : 1) void prefill_mfma_kernel(PrefillArgs args, int items_cap) {
  // the arguments as locals (the closures below then capture plain values, which the compiler keeps in registers)
  const int aB = args.B, aMaxPages = args.max_pages;
  const float aScale = args.scale_log2;
  const void* const aK = args.K;
  const void* const aV = args.V;
  const void* const aPages = args.pages;
  void* const aO = args.O;
  constexpr int kBM = NWQ * 32;
  constexpr int kChunks = DH / 8;  // 16-byte chunks per row
  constexpr int kDB = DH / 32;     // 32-dim blocks of the output
  constexpr int kRowBytes = DH * 2;
  constexpr int kTileElems = kBN * DH;
  constexpr int kStages = 3;
  using D = Dma<DH, NWQ>;

  // a ring of three K tiles and three V tiles: tile t+2 is requested while tile t is used
  __shared__ __align__(1024) bf16_t sK[kStages * kTileElems];
  __shared__ __align__(1024) bf16_t sV[kStages * kTileElems];

  const int tid = threadIdx.x, lane = tid & (kWave - 1);
  const int wq = __builtin_amdgcn_readfirstlane(tid / kWave);
  const int H = args.H;
  const int g = lane >> 5, lq = lane & 31;
  // Offsets, page table and mask words were written by earlier launches and do not change while this kernel runs:
  // read through the constant address space, block-uniform indices become scalar loads.  (As plain pointers they
  // may alias the output, which this kernel now stores inside its loop, and every page id became a vector load
  // with a full vector-memory wait behind it -- a wait for the tile loads in flight.)
  typedef const int32_t __attribute__((address_space(4)))* ConstI32;
  typedef const uint32_t __attribute__((address_space(4)))* ConstU32;
  const ConstI32 off_c = (ConstI32)args.off;
  const ConstI32 bt_c = (ConstI32)args.block_table;
  const ConstU32 kw_c = (ConstU32)args.key_words;
  const bool full = args.full != 0;  // no causal mask: all keys of the sequence (block-uniform)
  const bool paged = aK == nullptr;  // block-uniform
  const int step = static_cast<int>(gridDim.x);

  // Which (sequence, query tile) is item k?  With at most 64 sequences every wave keeps the sequences' offsets in
  // its lanes (lane = sequence; one trip to memory per block) and counts with ballots; with more, the sequences are
  // walked with scalar loads (then there is one item per block).
  const bool by_lane = aB <= kWave;
  int off_l = 0, end_l = 0, nb_l = 0, total = 0;
  if (by_lane) {
    off_l = lane < aB ? off_c[lane] : 0;
    end_l = lane < aB ? off_c[lane + 1] : 0;
    // The offsets have arrived; the statement also tells the compiler so: it would otherwise order every later use
    // of them, in loops it cannot see through, behind ALL outstanding vector-memory operations -- the tile loads.
    asm volatile("s_waitcnt vmcnt(0)" : "+v"(off_l), "+v"(end_l));
    nb_l = (end_l - off_l + kBM - 1) / kBM;  // tiles of sequence `lane`
    int cnt = 0;
    for (int i = 0; (cnt = __builtin_popcountll(__ballot(nb_l > i))) != 0; ++i) total += cnt;
  }
  struct Item {
    int valid, b, h, tile, r0, n;
  };
  auto locate = [&](int k) __attribute__((always_inline)) {
    Item it{0, 0, 0, 0, 0, 0};
    if (k >= items_cap) return it;
    const int yd = k / H;  // position in DESCENDING tile-index order
    it.h = k - yd * H;
    if (by_lane) {
      const int y = total - 1 - yd;  // position in ascending order
      if (y < 0) return it;
      int below = 0, tile = 0;  // tiles with a smaller index
      for (;; ++tile) {
        const int cnt = __builtin_popcountll(__ballot(nb_l > tile));
        if (below + cnt > y) break;
        below += cnt;
      }
      // the (y - below)-th sequence, in ascending order, that has a tile of this index
      const unsigned long long has = __ballot(nb_l > tile);
      const int before = __builtin_amdgcn_mbcnt_hi(static_cast<uint32_t>(has >> 32),
                                                   __builtin_amdgcn_mbcnt_lo(static_cast<uint32_t>(has), 0));
      const unsigned long long me = __ballot(nb_l > tile && before == y - below);
      it.b = __builtin_ctzll(me);
      it.tile = tile;
      it.r0 = __builtin_amdgcn_readlane(off_l, it.b);
      it.n = __builtin_amdgcn_readlane(end_l, it.b) - it.r0;
      it.valid = 1;
    } else {
      // many sequences: numbered sequence by sequence, the late (long) tiles of each first
      int tile = yd;
      for (int b = 0; b < aB; ++b) {
        const int r0 = off_c[b], n = off_c[b + 1] - r0;
        const int nt = (n + kBM - 1) / kBM;
        if (tile < nt) {
          it.b = b; it.tile = nt - 1 - tile; it.r0 = r0; it.n = n; it.valid = 1;
          break;
        }
        tile -= nt;
      }
    }
    return it;
  };
  // keys 0..last_key of its sequence are needed by an item
  auto last_key_of = [&](const Item& it) __attribute__((always_inline)) { return (!full && it.tile * kBM + kBM < it.n ? it.tile * kBM + kBM : it.n) - 1; };

  // Round j of block p takes item p + j*step, in odd rounds (step-1-p) + j*step: the rounds run through the items
  // (sorted by descending work) in alternating directions, so a block that got a longer item in one round gets a
  // shorter one in the next and the blocks' totals stay close (C5 shape: 40..42 tiles per block instead of 36..46).
  const int pblk = static_cast<int>(blockIdx.x);
  auto item_of = [&](int j) __attribute__((always_inline)) { return ((j & 1) ? step - 1 - pblk : pblk) + j * step; };
  int jC = 0;
  Item C = locate(item_of(0));
  if (!C.valid) return;
  Item nextC = locate(item_of(1));

  // ---- per-wave state of the item being computed -------------------------------------------------------------------
  const bf16_t* Qp = static_cast<const bf16_t*>(args.Q);
  uint4 qf[DH / 16];       // Q^T fragments: lane -> query iw + lq (clamped), 8 consecutive d at 16*ks + 8*g
  uint4 qn[DH / 16];       // the same for the block's NEXT item, requested a whole item ahead
  auto load_queries = [&](const Item& it, uint4 (&dst)[DH / 16]) __attribute__((always_inline)) {
    int q = it.tile * kBM + wq * 32 + lq;
    if (q >= it.n) q = it.n - 1;
    const bf16_t* qrow = Qp + (static_cast<size_t>(it.r0 + q) * H + it.h) * DH + 8 * g;
#pragma unroll
    for (int ks = 0; ks < DH / 16; ++ks) dst[ks] = *reinterpret_cast<const uint4*>(qrow + 16 * ks);
  };
  load_queries(C, qn);
  // key-mask word of a tile: a block-uniform scalar load, fetched one tile before it is used
  uint32_t kmask_next = ~0u;
  auto mask_word = [&](const Item& it, int t) __attribute__((always_inline)) {
    return MASKED ? kw_c[(it.r0 >> 5) + it.b + t] : ~0u;
  };
  kmask_next = mask_word(C, 0);

  f32x16 o_acc[kDB];
  float m_ref = -1e30f, l_run = 0.f;  // finite floor, not -inf: see tile_step
  int iw = 0, qi = 0;                 // first query row of this wave; this lane's query (clamped)
  bf16_t* orow = nullptr;             // where this lane's query goes; null for a lane without a query
  auto begin_item = [&](const Item& it) __attribute__((always_inline)) {
#pragma unroll
    for (int nb = 0; nb < kDB; ++nb)
#pragma unroll
      for (int r = 0; r < 16; ++r) o_acc[nb][r] = 0.f;
    m_ref = -1e30f;
    l_run = 0.f;
    iw = it.tile * kBM + wq * 32;
    qi = iw + lq;
    const bool q_ok = qi < it.n;
    if (!q_ok) qi = it.n - 1;
    orow = q_ok ? static_cast<bf16_t*>(aO) + (static_cast<size_t>(it.r0 + qi) * H + it.h) * DH : nullptr;
  };
  auto store_item = [&]() __attribute__((always_inline)) {
    // l is split between the two lanes of a query
    l_run += __shfl_xor(l_run, 32, kWave);
    if (orow) {
      const float inv = 1.f / l_run;
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
  };

  // Fragment addresses (LDS bytes, stage 0).  K: row lq, logical chunk 2*ks + g, stored at chunk ^ (lq mod chunks):
  // the step ks enters as an exclusive-or with 32*ks.  V: the transposing read of 16 lanes (j = lane mod 16) returns
  // to lane j four keys of dim j; lane j points at key j/4, dims 4*(j mod 4)..+3 of the 16 dims of its group.
  const uint32_t kb0 = static_cast<uint32_t>(reinterpret_cast<uintptr_t>((DLLAVA_LDS bf16_t*)sK)) + lq * kRowBytes +
                       (((lq % kChunks) & ~1) * 16) + ((g ^ (lq & 1)) * 16);
  const int j = lane & 15, lqh = (lane >> 4) & 1;
  const uint32_t vb0 = static_cast<uint32_t>(reinterpret_cast<uintptr_t>((DLLAVA_LDS bf16_t*)sV)) +
                       (4 * g + (j >> 2)) * kRowBytes + ((j >> 2) % (kChunks / 4)) * 64 + lqh * 32 + (j & 3) * 8;

  const size_t tl = static_cast<size_t>(kPage) * DH;           // one head's K (or V) rows of a page
  const uint32_t v_off = static_cast<uint32_t>(H * tl);        // from a page's K block to its V block
  const uint32_t row_stride = static_cast<uint32_t>(H) * DH;   // between consecutive rows of K / V

  // ---- the stream of tile loads: item P, its tile tP is the next one to request ---------------------------------------
  int jP = 0, tP = 0;
  Item P = C;
  int lastP = last_key_of(P);
  // Page ids of a tile are block-uniform scalar loads, fetched one step before the tile is requested.  The index is
  // clamped to the block table: a sequence longer than the cache capacity (flagged by the call that filled the
  // cache) then reads allocated pages, not whatever follows its row of the table.
  int pg_lo = 0, pg_hi = 0;
  auto fetch_page_ids = [&]() __attribute__((always_inline)) {  // for tile tP of item P
    if (paged && P.valid) {
      const ConstI32 bt = bt_c + static_cast<size_t>(P.b) * aMaxPages;
      const int last_page = lastP / kPage < aMaxPages - 1 ? lastP / kPage : aMaxPages - 1;
      const int p_lo = 2 * tP < last_page ? 2 * tP : last_page;
      const int p_hi = 2 * tP + 1 < last_page ? 2 * tP + 1 : last_page;
      pg_lo = bt[p_lo];
      pg_hi = bt[p_hi];
    }
  };
  auto request_tile = [&](int stage) __attribute__((always_inline)) {  // tile tP of item P into `stage`, then on to the next tile of the stream
    const int lim = lastP - tP * kBN;
    bf16_t* dk = sK + stage * kTileElems;
    bf16_t* dv = sV + stage * kTileElems;
    if (paged) {
      const bf16_t* pages = static_cast<const bf16_t*>(aPages);
      D::paged(dk, dv, pages + (static_cast<size_t>(pg_lo) * 2 * H + P.h) * tl,
               pages + (static_cast<size_t>(pg_hi) * 2 * H + P.h) * tl, v_off, lim, wq, lane);
    } else {
      const size_t o = (static_cast<size_t>(P.r0 + tP * kBN) * H + P.h) * DH;
      D::rows(dk, dv, static_cast<const bf16_t*>(aK) + o, static_cast<const bf16_t*>(aV) + o, row_stride, lim, wq, lane);
    }
    if (++tP > lastP / kBN) {  // the item's last tile: the stream goes on with the block's next item
      ++jP;
      P = locate(item_of(jP));
      tP = 0;
      lastP = P.valid ? last_key_of(P) : 0;
    }
    fetch_page_ids();
  };

  fetch_page_ids();
  request_tile(0);
  int ahead = 0;  // tiles requested beyond the one the arithmetic is at
  if (P.valid) {
    request_tile(1);
    ahead = 1;
  }
  int cur = 0;       // stage of the tile the arithmetic is at
  int nC = last_key_of(C) / kBN + 1;
  bool have_prev = false;  // an item's outputs are still to be stored
  // One tile of the stream.  FIRST: it is the first tile of item C -- its queries (requested when the previous item
  // ended) must have arrived, and the previous item's outputs leave behind this tile's request.  (A separate
  // instantiation rather than a flag: the compiler places its own waits for the query loads by what MAY be
  // outstanding on any path, and would wait for the tile loads just requested in every iteration.)
  auto tile_iteration = [&](auto first_tag, const int tC) __attribute__((always_inline)) {
    constexpr bool FIRST = decltype(first_tag)::value;
    // This wave's own loads of the tile are waited for (those of the next tile, requested later, may stay in flight),
    // then the barrier makes every wave's part of the tile visible and says that all waves have left the tile before.
    // The count assumes that nothing but the tile loads of the NEXT tile was issued after this tile's loads; whatever
    // else is in flight (queries of a new item, an item's output stores, mask words) only makes the wait longer.
    // The kernel must not spill registers (scratch traffic would count too): the tests check the build's resource report.
    if (ahead > 0)
      asm volatile("s_waitcnt vmcnt(%0)" ::"n"(2 * D::kLoads) : "memory");
    else
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    if (FIRST) {
      // the item's queries were requested a whole item ago (the first item's: before the first tiles); they move into
      // the registers the products read, and the next item's are requested into the other set
#pragma unroll
      for (int ks = 0; ks < DH / 16; ++ks) qf[ks] = qn[ks];
#pragma unroll
      for (int ks = 0; ks < DH / 16; ++ks) asm volatile("" : "+v"(qf[ks].x), "+v"(qf[ks].y), "+v"(qf[ks].z), "+v"(qf[ks].w));
    }
    __builtin_amdgcn_s_barrier();
    const int prv = cur == 0 ? kStages - 1 : cur - 1;  // the stage of the tile before: free now
    if (P.valid) {
      request_tile(prv);
      ++ahead;
    }
    if (FIRST) {
      if (have_prev) store_item();  // the previous item's outputs, behind the tile request
      begin_item(C);
      if (nextC.valid) load_queries(nextC, qn);
    }
    const int j0 = tC * kBN;
    const uint32_t kmask = kmask_next;  // wave-uniform
    if (MASKED && tC + 1 < nC) kmask_next = mask_word(C, tC + 1);
    // skipped (wave-uniform): the tile lies entirely above this wave's diagonal, the wave has no query, or every key
    // of the tile is masked and none of them is a query of this wave
    if ((full || j0 <= iw + 31) && iw < C.n && !(kmask == 0u && j0 + kBN - 1 < iw)) {
      const uint32_t kb = kb0 + cur * (kTileElems * 2), vb = vb0 + cur * (kTileElems * 2);
      // masking needed: some key of the tile may exceed some query of the wave (causal) or the end of the sequence
      // (full), or is hidden by its mask bit
      tile_step<DH, MASKED>(kb, vb, qf, o_acc, m_ref, l_run, aScale, j0, full ? C.n - 1 : qi, g,
                            j0 + kBN - 1 > (full ? C.n - 1 : iw) || kmask != ~0u, kmask, qi);
    }
    cur = cur == kStages - 1 ? 0 : cur + 1;
    --ahead;
  };
  for (;;) {
    tile_iteration(std::true_type{}, 0);
    for (int t = 1; t < nC; ++t) tile_iteration(std::false_type{}, t);
    have_prev = true;
    if (!nextC.valid) break;
    // next item (its queries were requested when this one began)
    ++jC;
    C = nextC;
    nextC = locate(item_of(jC + 1));
    nC = last_key_of(C) / kBN + 1;
    kmask_next = mask_word(C, 0);
  }
  store_item();
}

// blocks that fit the chip at once (persistent launch): compute units x blocks per compute unit, found once per kernel
template <int DH, int NWQ, bool MASKED>
int64_t resident_blocks() {
  static int64_t cached = 0;  // the same value whichever thread gets here first
  if (cached) return cached;
  int dev = 0, cus = 0, per_cu = 0;
  if (hipGetDevice(&dev) != hipSuccess ||
      hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
    cus = 256;
  if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, prefill_mfma_kernel<DH, NWQ, MASKED>, NWQ * kWave, 0) != hipSuccess ||
      per_cu <= 0)
    per_cu = 2;
  cached = static_cast<int64_t>(cus) * per_cu;
  return cached;
}

template <int DH, int NWQ>
int launch(const PrefillArgs& a, int64_t rows, hipStream_t st) {
  constexpr int kBM = NWQ * 32;
  const int64_t tiles = ceil_div(rows, kBM) + a.B;  // upper bound on sum_b ceil(n_b / kBM)
  const int64_t items = tiles * a.H;
  if (items > 0x7fffffffLL) return 1;
  // one item per block when the sequences are too many to be numbered in a wave's lanes (see the kernel)
  const bool persistent = a.B <= kWave;
  const int forced = persistent ? launch_override(DLLAVA_LAUNCH_PREFILL_BLOCKS) : 0;  // tests: few blocks, many items each
  if (a.key_words) {
    const int64_t slots = forced ? forced : (persistent ? resident_blocks<DH, NWQ, true>() : items);
    const dim3 grid(static_cast<unsigned>(items < slots ? items : slots));
    hipLaunchKernelGGL((prefill_mfma_kernel<DH, NWQ, true>), grid, dim3(NWQ * kWave), 0, st, a, static_cast<int>(items));
  } else {
    const int64_t slots = forced ? forced : (persistent ? resident_blocks<DH, NWQ, false>() : items);
    const dim3 grid(static_cast<unsigned>(items < slots ? items : slots));
    hipLaunchKernelGGL((prefill_mfma_kernel<DH, NWQ, false>), grid, dim3(NWQ * kWave), 0, st, a, static_cast<int>(items));
  }
  DLLAVA_CHECK_LAUNCH("prefill_mfma_kernel");
  return DLLAVA_OK;
}

}  // namespace

// returns 1 if the shape is not handled here
int prefill_mfma_launch(const PrefillArgs& a, int64_t rows, int Dh, hipStream_t st) {
  if (a.H > 65535) return 1;
  // wide tiles (K/V tiles staged once for 128 queries) unless there is too little work to spread over the chip;
  // measured: 2 waves win for the 7B batch-1 prefill (214 rows x 32 heads), 4 waves from batch 2 upwards
  const int64_t work = rows * a.H;  // query rows x heads
  int nwq = work >= 8 * 1024 ? 4 : (work >= 1024 ? 2 : 1);
  if (const int v = launch_override(DLLAVA_LAUNCH_PREFILL_WAVES)) {  // forced through dllava_set_launch_override
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
