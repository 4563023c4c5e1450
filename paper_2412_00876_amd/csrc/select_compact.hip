// dllava_select_compact: keep decisions (Eq. 5 line 2 / Eq. 11 line 2 of the paper) and order-preserving
// stream compaction of hidden states, queries and K/V into the reduced token set / paged cache
// (Eq. 5 line 3 / Eq. 11 line 3).
//
// Selection, one block per sequence.  Top-k: the k-th largest score is found exactly by a 4-pass
// most-significant-byte radix select over an order-preserving 32-bit key, then one in-order pass keeps keys above
// it plus the first (k - #above) equal keys, which is the "ties go to the lower index" rule.  The same pass ranks
// the kept rows of the sequence (prefix sum), so kept positions come out ascending.  Selection is integer-exact:
// it only compares float32 keys.
//
// Compaction, one block per kept row: 16-byte coalesced copies of its hidden, Q, K and V rows; K/V rows are
// scattered head by head into their page slot.
//
// Two launches, in one of two arrangements:
//   top-k, up to 256 sequences   Top-k keeps exactly k = floor(ratio * n) rows of a span, whatever the scores, so
//                      every sequence's kept count, the offsets of the compacted batch and the destination of
//                      every row OUTSIDE the vision span are known before a score is read.  Launch 1 runs the
//                      selection blocks and, beside them, the copies of those rows (system and text tokens);
//                      launch 2 copies the kept vision rows.  The selection's latency hides behind the first
//                      copies, and a copying block finds its row with one round of loads (the per-sequence layout
//                      built in LDS) instead of a chain of dependent ones.
//   otherwise          select_kernel, whose last block (device-scope ticket) scans the per-sequence counts into
//                      out_off, sets cache_len and checks the capacity; then gather_kernel over all kept rows.
#include "common.h"

namespace dllava {
namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / kWave;

// Order-preserving key: larger score <-> larger key; -0 and +0 share a key; NaN gets the lowest key.
__device__ __forceinline__ uint32_t score_key(float s) {  // selects only: no branch for a load to be sunk under
  const uint32_t u = __float_as_uint(s);
  uint32_t key = (u & 0x80000000u) ? ~u : (u | 0x80000000u);
  key = s == 0.f ? 0x80000000u : key;
  return s != s ? 0u : key;
}

// Exclusive prefix sum of one int per thread over the block; `total` receives the block sum.
__device__ __forceinline__ int block_excl_scan(int v, int* sm_tot /*[kWaves]*/, int& total) {
  const int lane = threadIdx.x & (kWave - 1), w = threadIdx.x / kWave;
  const int incl = wave_incl_scan(v);
  __syncthreads();  // previous use of sm_tot is over
  if (lane == kWave - 1) sm_tot[w] = incl;
  __syncthreads();
  int off = 0, t = 0;
#pragma unroll
  for (int i = 0; i < kWaves; ++i) {
    const int x = sm_tot[i];
    if (i < w) off += x;
    t += x;
  }
  total = t;
  return off + incl - v;
}

struct SelectArgs {
  const float* logits;
  const int32_t* seq_off;
  const int32_t* vis_start;
  const int32_t* vis_len;
  int32_t B;
  int32_t mode;
  double keep_ratio;
  float threshold;
  uint8_t* keep_mask;
  int32_t* ws_kept;    // [sumN]: kept positions of sequence b at [seq_off[b] ...)
  int32_t* ws_counts;  // [B]
  int32_t* ws_ticket;  // one device-scope counter, zero between calls
  int32_t* out_off;    // [B+1]
  int32_t* cache_len;  // [B] or null
  int32_t cap;         // tokens a sequence's pages can hold
  int32_t* err_flag;
  int32_t* ws_sync;    // top-k arrangement: [3][kLayoutSeqs] claim / ready / done words, zero between calls
  int32_t stand_back;  // tests: the selection blocks of sequences with kept vision rows leave the selection to a copying block
};

constexpr int kKeyCache = 4096;  // scores of one vision span kept in LDS (16 KiB); longer spans re-read them

template <int KC>  // scores cached in LDS; 0: none (every pass reads them from memory)
struct SelectSharedT {
  int hist[256];
  int sm_tot[kWaves];
  int sm_sel[2];
  uint32_t skey[KC > 0 ? KC : 1];
  int sm_last;
};

// Rows a sequence of N tokens keeps under top-k, and its clamped vision span (Eq. 5: k = floor(ratio * n) of the n
// vision tokens, every other token).
struct SeqShape {
  int N, v0, n, k;
  __device__ __forceinline__ int kept() const { return N - n + k; }
};

__device__ __forceinline__ SeqShape seq_shape(int s0, int s1, int vis_start, int vis_len, double keep_ratio) {
  SeqShape q;
  q.N = s1 - s0 < 0 ? 0 : s1 - s0;
  q.v0 = vis_start < 0 ? 0 : (vis_start > q.N ? q.N : vis_start);
  q.n = vis_len < 0 ? 0 : (vis_len > q.N - q.v0 ? q.N - q.v0 : vis_len);
  const int64_t k = static_cast<int64_t>(floor(keep_ratio * static_cast<double>(q.n)));
  q.k = k <= 0 ? 0 : (k >= q.n ? q.n : static_cast<int>(k));
  return q;
}

// The selection of sequence b by one block.  analytic (top-k only): the offsets follow from the sequences' shapes,
// so this block writes its own out_off / cache_len entries and no block waits for another.
template <bool ANALYTIC, int KC>
__device__ __forceinline__ void select_block(const SelectArgs& a, SelectSharedT<KC>& S, const int b) {
  int (&hist)[256] = S.hist;
  int (&sm_tot)[kWaves] = S.sm_tot;
  int (&sm_sel)[2] = S.sm_sel;
  uint32_t* skey = S.skey;
  const int tid = threadIdx.x;
  const int s0 = a.seq_off[b];
  int N = a.seq_off[b + 1] - s0;
  if (N < 0) N = 0;
  int v0 = a.vis_start[b];
  v0 = v0 < 0 ? 0 : (v0 > N ? N : v0);
  int n = a.vis_len[b];
  n = n < 0 ? 0 : (n > N - v0 ? N - v0 : n);

  // row of this sequence's first vision token in `logits` (and, analytic, of its first kept row in the outputs)
  int part = 0, part_kept = 0;
  for (int i = tid; i < b; i += kThreads) {
    const int x = a.vis_len[i];
    part += x > 0 ? x : 0;
    if (ANALYTIC) part_kept += seq_shape(a.seq_off[i], a.seq_off[i + 1], a.vis_start[i], x, a.keep_ratio).kept();
  }
  int lo, first_kept = 0;
  block_excl_scan(part, sm_tot, lo);
  if (ANALYTIC) block_excl_scan(part_kept, sm_tot, first_kept);
  const float* D = a.logits + 2 * static_cast<size_t>(lo);

  const bool cached = KC > 0 && n <= KC;
  uint32_t kth = 0;     // key of the k-th largest score
  int need = 0;         // how many rows with key == kth are kept (taken in index order)
  bool all = false, none = false;
  if (a.mode == DLLAVA_MODE_TOPK) {
    int64_t k = static_cast<int64_t>(floor(a.keep_ratio * static_cast<double>(n)));
    if (k <= 0) none = true;
    else if (k >= n) all = true;
    else {
      uint32_t prefix = 0, mask = 0;
      int remaining = static_cast<int>(k);
      // the keys are read from memory once (all loads of a thread in flight together) and kept in LDS
      // (every load of a thread is issued before the first is used: a loop of load-convert-store rounds would pay
      // a memory round trip per 256 scores)
      if (cached) {
        constexpr int kPer = KC > 0 ? KC / kThreads : 1;
        const int live = (n + kThreads - 1) / kThreads;  // the same for the whole block
        float raw[kPer];
#pragma unroll
        for (int e = 0; e < kPer; ++e)
          if (e < live) {
            const int i = tid + e * kThreads;
            raw[e] = D[2 * (i < n ? i : n - 1) + 1];
          }
#pragma unroll
        for (int e = 0; e < kPer; ++e)
          if (e < live) {
            const int i = tid + e * kThreads;
            if (i < n) skey[i] = score_key(raw[e]);
          }
      }
      for (int shift = 24; shift >= 0; shift -= 8) {
        hist[tid] = 0;
        __syncthreads();
        for (int i = tid; i < n; i += kThreads) {
          const uint32_t key = cached ? skey[i] : score_key(D[2 * i + 1]);
          if ((key & mask) == prefix) atomicAdd(&hist[(key >> shift) & 255u], 1);
        }
        __syncthreads();
        // suffix sums over the bins: thread t looks at bin 255 - t
        const int bin = 255 - tid;
        const int c = hist[bin];
        int tot;
        const int above = block_excl_scan(c, sm_tot, tot);  // rows in higher bins
        if (above < remaining && above + c >= remaining) {
          sm_sel[0] = bin;
          sm_sel[1] = remaining - above;
        }
        __syncthreads();
        prefix |= static_cast<uint32_t>(sm_sel[0]) << shift;
        mask |= 0xffu << shift;
        remaining = sm_sel[1];
        __syncthreads();
      }
      kth = prefix;
      need = remaining;
    }
  }

  // In-order pass over all rows of the sequence.  Thread t owns E consecutive rows of a chunk of 256*E rows
  // (one chunk covers sequences of up to 8192 rows), so the whole pass costs two block scans -- the rank of
  // the rows that tie with the k-th score, then the rank of the kept rows -- instead of two per 256 rows.
  const bool partial = a.mode == DLLAVA_MODE_TOPK && !all && !none;
  int E = (N + kThreads - 1) / kThreads;
  E = E < 1 ? 1 : (E > 32 ? 32 : E);
  int carry_eq = 0, carry_keep = 0;
  for (int base = 0; base < N; base += kThreads * E) {
    const int p0 = base + tid * E;
    uint32_t keep_bits = 0, eq_bits = 0;
    for (int e = 0; e < E; ++e) {
      const int p = p0 + e;
      const bool in = p < N;
      const bool vis = in && p >= v0 && p < v0 + n;
      bool keep = in && !vis;
      bool eq = false;
      if (vis) {
        const int i = p - v0;
        if (a.mode == DLLAVA_MODE_TOPK) {
          if (all) keep = true;
          else if (!none) {
            const uint32_t key = cached ? skey[i] : score_key(D[2 * i + 1]);
            keep = key > kth;
            eq = key == kth;
          }
        } else {
          keep = keep_from_logits(D, i, a.threshold);
          // decoding without KV cache: the last output token produces the next one and is always kept
          if (a.mode == DLLAVA_MODE_THRESHOLD_KEEP_LAST && i == n - 1) keep = true;
        }
      }
      keep_bits |= (keep ? 1u : 0u) << e;
      eq_bits |= (eq ? 1u : 0u) << e;
    }
    if (partial) {  // block-uniform
      int tot_eq;
      int rank_eq = carry_eq + block_excl_scan(__popc(eq_bits), sm_tot, tot_eq);
      carry_eq += tot_eq;
      for (int e = 0; e < E; ++e)
        if ((eq_bits >> e) & 1u) {
          if (rank_eq < need) keep_bits |= 1u << e;
          ++rank_eq;
        }
    }
    int tot_keep;
    int pos = carry_keep + block_excl_scan(__popc(keep_bits), sm_tot, tot_keep);
    carry_keep += tot_keep;
    for (int e = 0; e < E; ++e) {
      const int p = p0 + e;
      if (p < N) {
        const bool keep = (keep_bits >> e) & 1u;
        a.keep_mask[static_cast<size_t>(s0) + p] = keep ? 1 : 0;
        if (keep) {
          int32_t* dst = &a.ws_kept[static_cast<size_t>(s0) + pos++];
          if (ANALYTIC) __hip_atomic_store(dst, p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);  // read in this launch
          else *dst = p;
        }
      }
    }
  }
  if (ANALYTIC) {
    if (tid == 0) {
      a.out_off[b] = first_kept;
      if (b == a.B - 1) a.out_off[a.B] = first_kept + carry_keep;
      if (a.cache_len) {
        a.cache_len[b] = carry_keep > a.cap ? a.cap : carry_keep;
        if (carry_keep > a.cap && a.err_flag) *a.err_flag = 1;
      }
    }
    return;
  }
  // The block that finishes last turns the per-sequence counts into offsets (exclusive scan), sets the cache
  // lengths and checks the capacity: no second launch.  Hand-off through device-scope stores and a ticket.
  int& sm_last = S.sm_last;
  if (tid == 0) {
    __hip_atomic_store(&a.ws_counts[b], carry_keep, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    wave_stores_done();
    sm_last = (add_agent(a.ws_ticket, 1) == a.B - 1);
  }
  __syncthreads();
  if (!sm_last) return;
  int carry = 0;
  for (int base = 0; base < a.B; base += kThreads) {
    const int bb = base + tid;
    const int c = bb < a.B ? __hip_atomic_load(&a.ws_counts[bb], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0;
    int tot;
    const int ex = carry + block_excl_scan(c, sm_tot, tot);
    carry += tot;
    if (bb < a.B) {
      a.out_off[bb] = ex;
      if (a.cache_len) {
        a.cache_len[bb] = c > a.cap ? a.cap : c;
        if (c > a.cap && a.err_flag) *a.err_flag = 1;
      }
    }
  }
  if (tid == 0) {
    a.out_off[a.B] = carry;
    zero_agent(a.ws_ticket);
  }
}

__global__ __launch_bounds__(kThreads) void select_kernel(SelectArgs a) {
  __shared__ SelectSharedT<kKeyCache> S;
  select_block<false, kKeyCache>(a, S, blockIdx.x);
}

struct GatherArgs {
  const int32_t* seq_off;
  const int32_t* out_off;
  const int32_t* ws_kept;
  int32_t* kept_idx;
  int32_t B;
  const uint4* hidden; uint4* hidden_out; int64_t hidden_chunks;  // 16-byte chunks per row
  const uint4* Q; uint4* Q_out; int64_t q_chunks;
  const uint4* K; const uint4* V; int64_t kv_chunks;              // per row, all heads
  uint4* pages; const int32_t* block_table;
  int32_t max_pages, H, head_chunks;                              // 16-byte chunks per (token, head)
  // decisions taken earlier (dllava_compact): kept_idx is an INPUT, indexed by compacted row, and block 0 sets the
  // cache lengths and the capacity flag
  int32_t given;
  int32_t* cache_len;
  int32_t cap;
  int32_t* err_flag;
  // top-k arrangement: the sequences' shapes, from which every block derives the layout of the outputs
  const int32_t* vis_start;
  const int32_t* vis_len;
  double keep_ratio;
};

// 16 readable bytes: the source of the (unused) clamped loads of a tensor that is not being moved
static __device__ __attribute__((aligned(16))) uint32_t kGatherPad[4] = {0u, 0u, 0u, 0u};

// One block per compacted row moves all of its tensors: hidden, Q, K, V.  The dependent chain in front of the
// copies (total, binary search for the sequence, kept position) is paid once per row, and every 16-byte load of
// a trip -- two per thread and tensor, index clamped so that none sits under a condition -- is in flight
// before the first store.
__device__ __forceinline__ void copy_row(const GatherArgs& a, int b, int pos, size_t src, int j);

__global__ __launch_bounds__(kThreads) void gather_kernel(GatherArgs a) {
  const int j = blockIdx.x, tid = threadIdx.x;
  const int total = a.out_off[a.B];
  if (a.given && j == 0 && a.cache_len) {  // decisions taken earlier: the lengths of THIS cache follow from them
    for (int bb = tid; bb < a.B; bb += kThreads) {
      const int c = a.out_off[bb + 1] - a.out_off[bb];
      a.cache_len[bb] = c > a.cap ? a.cap : c;
      if (c > a.cap && a.err_flag) *a.err_flag = 1;
    }
  }
  if (j >= total) return;
  int lo = 0, hi = a.B;  // largest b with out_off[b] <= j
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (a.out_off[mid] <= j) lo = mid; else hi = mid;
  }
  const int b = lo;
  const int pos = j - a.out_off[b];
  const int s0 = a.seq_off[b];
  const int rel = a.given ? a.kept_idx[j] : a.ws_kept[static_cast<size_t>(s0) + pos];
  const size_t src = static_cast<size_t>(s0) + rel;
  if (tid == 0 && !a.given) a.kept_idx[j] = rel;
  copy_row(a, b, pos, src, j);
}

// The block moves source row `src` (kept row `pos` of sequence b) to compacted row j and its page slot.
__device__ __forceinline__ void copy_row(const GatherArgs& a, int b, int pos, size_t src, int j) {
  const int tid = threadIdx.x;
  const bool do_h = a.hidden != nullptr, do_q = a.Q != nullptr;
  const bool do_kv = a.K != nullptr && pos < a.max_pages * kPage;
  const int64_t nh = do_h ? a.hidden_chunks : 0, nq = do_q ? a.q_chunks : 0, nkv = do_kv ? a.kv_chunks : 0;
  // sources (a valid address even when the tensor is absent: the clamped loads are then simply not stored)
  const uint4* in_h = do_h ? a.hidden + src * a.hidden_chunks : reinterpret_cast<const uint4*>(kGatherPad);
  const uint4* in_q = do_q ? a.Q + src * a.q_chunks : reinterpret_cast<const uint4*>(kGatherPad);
  const uint4* in_k = do_kv ? a.K + src * a.kv_chunks : reinterpret_cast<const uint4*>(kGatherPad);
  const uint4* in_v = do_kv ? a.V + src * a.kv_chunks : reinterpret_cast<const uint4*>(kGatherPad);
  uint4* out_h = do_h ? a.hidden_out + static_cast<size_t>(j) * a.hidden_chunks : nullptr;
  uint4* out_q = do_q ? a.Q_out + static_cast<size_t>(j) * a.q_chunks : nullptr;
  uint4* page_k = nullptr;
  size_t tile_chunks = 0;
  if (do_kv) {
    const int pg = a.block_table[static_cast<size_t>(b) * a.max_pages + pos / kPage];
    tile_chunks = static_cast<size_t>(kPage) * a.head_chunks;
    page_k = a.pages + static_cast<size_t>(pg) * 2 * a.H * tile_chunks + static_cast<size_t>(pos % kPage) * a.head_chunks;
  }
  const size_t v_off = static_cast<size_t>(a.H) * tile_chunks;  // from the K half of a page to its V half
  int64_t nmax = nh > nq ? nh : nq;
  nmax = nmax > nkv ? nmax : nkv;
  for (int64_t c0 = tid; c0 < nmax; c0 += 2 * kThreads) {
    const int64_t c1 = c0 + kThreads;
#define DLLAVA_CLAMP(c, n) ((n) > 0 ? ((c) < (n) ? (c) : (n)-1) : 0)
    const uint4 h0 = in_h[DLLAVA_CLAMP(c0, nh)], h1 = in_h[DLLAVA_CLAMP(c1, nh)];
    const uint4 q0 = in_q[DLLAVA_CLAMP(c0, nq)], q1 = in_q[DLLAVA_CLAMP(c1, nq)];
    const uint4 k0 = in_k[DLLAVA_CLAMP(c0, nkv)], k1 = in_k[DLLAVA_CLAMP(c1, nkv)];
    const uint4 v0 = in_v[DLLAVA_CLAMP(c0, nkv)], v1 = in_v[DLLAVA_CLAMP(c1, nkv)];
#undef DLLAVA_CLAMP
    if (c0 < nh) out_h[c0] = h0;
    if (c1 < nh) out_h[c1] = h1;
    if (c0 < nq) out_q[c0] = q0;
    if (c1 < nq) out_q[c1] = q1;
    if (c0 < nkv) {
      const size_t o = static_cast<size_t>(c0 / a.head_chunks) * tile_chunks + static_cast<size_t>(c0 % a.head_chunks);
      page_k[o] = k0;
      page_k[v_off + o] = v0;
    }
    if (c1 < nkv) {
      const size_t o = static_cast<size_t>(c1 / a.head_chunks) * tile_chunks + static_cast<size_t>(c1 % a.head_chunks);
      page_k[o] = k1;
      page_k[v_off + o] = v1;
    }
  }
}

// ------------------------------------------------------------------------------------------------
// top-k arrangement: the layout of the outputs from the sequences' shapes
// ------------------------------------------------------------------------------------------------
constexpr int kLayoutSeqs = kThreads;  // one sequence per thread
constexpr int kRestBlocks = 2048;      // blocks that loop over the rows outside the spans: eight per compute unit

// Rows are copied in two classes: 0 = rows outside the vision span (all kept; their destination does not depend on
// the scores), 1 = kept vision rows (k per sequence; which rows they are comes from the selection).
struct Layout {
  int s0[kLayoutSeqs], v0[kLayoutSeqs], n[kLayoutSeqs], k[kLayoutSeqs];
  int out_off[kLayoutSeqs + 1];  // first compacted row of each sequence
  int cls_off[kLayoutSeqs + 1];  // first row of each sequence among this class's rows; [B] = their number
  int sm_tot[kWaves];
};

template <int CLASS>
__device__ __forceinline__ void layout_build(Layout& L, const GatherArgs& a) {
  const int tid = threadIdx.x;
  const bool ok = tid < a.B;
  const int i = ok ? tid : 0;
  const int s0 = a.seq_off[i];
  SeqShape q = seq_shape(s0, a.seq_off[i + 1], a.vis_start[i], a.vis_len[i], a.keep_ratio);
  if (!ok) q.N = q.n = q.k = q.v0 = 0;
  int total_kept, total_cls;
  const int ex_kept = block_excl_scan(q.kept(), L.sm_tot, total_kept);
  const int ex_cls = block_excl_scan(CLASS == 0 ? q.N - q.n : q.k, L.sm_tot, total_cls);
  L.s0[tid] = s0;
  L.v0[tid] = q.v0;
  L.n[tid] = q.n;
  L.k[tid] = q.k;
  L.out_off[tid] = ex_kept;   // threads past the last sequence write the totals
  L.cls_off[tid] = ex_cls;
  if (tid == 0) {
    L.out_off[kLayoutSeqs] = total_kept;
    L.cls_off[kLayoutSeqs] = total_cls;
  }
  __syncthreads();
}

// The selection of the one-launch arrangement: spans of up to kRegKeys scores, the keys of a thread in registers
// (row i of the span belongs to thread i % 256), so the block needs about 2 KiB of LDS instead of the key cache's
// 16 KiB -- LDS is allocated alike for every block of the launch, and the copying blocks want eight per compute unit.
// Ranks in index order come from wave ballots and one table of per-(256 rows, wave) counts, one barrier each for
// the rows that tie with the k-th score and for the kept rows.  Returns false (nothing done) for a longer span.
constexpr int kRegKeys = 4096, kRegPer = kRegKeys / kThreads;

struct TopkShared {
  int hist[256];
  int sm_tot[kWaves];
  int sm_sel[2];
  int cnt_eq[kRegPer][kWaves];
  int cnt_keep[kRegPer][kWaves];
};

__device__ __forceinline__ bool select_topk_regs(const SelectArgs& a, TopkShared& S, const int b) {
  const int tid = threadIdx.x, lane = tid & (kWave - 1), w = tid / kWave;
  const int s0 = a.seq_off[b];
  const SeqShape q = seq_shape(s0, a.seq_off[b + 1], a.vis_start[b], a.vis_len[b], a.keep_ratio);
  const int N = q.N, v0 = q.v0, n = q.n, k = q.k;
  if (n > kRegKeys) return false;

  int part = 0, part_kept = 0;
  for (int i = tid; i < b; i += kThreads) {
    const int x = a.vis_len[i];
    part += x > 0 ? x : 0;
    part_kept += seq_shape(a.seq_off[i], a.seq_off[i + 1], a.vis_start[i], x, a.keep_ratio).kept();
  }
  int lo, first_kept;
  block_excl_scan(part, S.sm_tot, lo);
  block_excl_scan(part_kept, S.sm_tot, first_kept);
  const float* D = a.logits + 2 * static_cast<size_t>(lo);

  const int live = (n + kThreads - 1) / kThreads;  // registers in use, the same for the whole block
  const bool partial = k > 0 && k < n;
  uint32_t kr[kRegPer];
  uint32_t kth = 0;
  int need = 0;
  if (partial) {
    float raw[kRegPer];  // every load is issued before the first is used
#pragma unroll
    for (int e = 0; e < kRegPer; ++e)
      if (e < live) {
        const int i = tid + e * kThreads;
        raw[e] = D[2 * (i < n ? i : n - 1) + 1];
      }
#pragma unroll
    for (int e = 0; e < kRegPer; ++e) kr[e] = (e < live && tid + e * kThreads < n) ? score_key(raw[e]) : 0u;
    uint32_t prefix = 0, mask = 0;
    int remaining = k;
    for (int shift = 24; shift >= 0; shift -= 8) {
      S.hist[tid] = 0;
      __syncthreads();
#pragma unroll
      for (int e = 0; e < kRegPer; ++e)
        if (e < live && tid + e * kThreads < n && (kr[e] & mask) == prefix)
          atomicAdd(&S.hist[(kr[e] >> shift) & 255u], 1);
      __syncthreads();
      const int bin = 255 - tid;  // suffix sums over the bins
      const int c = S.hist[bin];
      int tot;
      const int above = block_excl_scan(c, S.sm_tot, tot);  // rows in higher bins
      if (above < remaining && above + c >= remaining) {
        S.sm_sel[0] = bin;
        S.sm_sel[1] = remaining - above;
      }
      __syncthreads();
      prefix |= static_cast<uint32_t>(S.sm_sel[0]) << shift;
      mask |= 0xffu << shift;
      remaining = S.sm_sel[1];
      __syncthreads();
    }
    kth = prefix;
    need = remaining;
  }

  const uint64_t below = (1ull << lane) - 1;  // the lanes before this one
  uint32_t keep_bits = 0;                     // bit e: row tid + 256 e of the span is kept
  if (partial) {
    uint32_t eq_bits = 0;
#pragma unroll
    for (int e = 0; e < kRegPer; ++e)
      if (e < live) {
        const bool in = tid + e * kThreads < n;
        const bool eq = in && kr[e] == kth;
        keep_bits |= ((in && kr[e] > kth) ? 1u : 0u) << e;
        eq_bits |= (eq ? 1u : 0u) << e;
        const uint64_t bal = __ballot(eq);
        if (lane == 0) S.cnt_eq[e][w] = __popcll(bal);
      }
    __syncthreads();
    int running = 0;  // ties in the 256-row groups before group e
#pragma unroll
    for (int e = 0; e < kRegPer; ++e)
      if (e < live) {
        int base = running;
#pragma unroll
        for (int ww = 0; ww < kWaves; ++ww) {
          const int c = S.cnt_eq[e][ww];
          base += ww < w ? c : 0;
          running += c;
        }
        const bool eq = (eq_bits >> e) & 1u;
        const uint64_t bal = __ballot(eq);
        if (eq && base + __popcll(bal & below) < need) keep_bits |= 1u << e;  // the first `need` ties, by index
      }
  } else if (k > 0) {  // k == n: every row
#pragma unroll
    for (int e = 0; e < kRegPer; ++e)
      if (e < live && tid + e * kThreads < n) keep_bits |= 1u << e;
  }
#pragma unroll
  for (int e = 0; e < kRegPer; ++e)
    if (e < live) {
      const uint64_t bal = __ballot((keep_bits >> e) & 1u);
      if (lane == 0) S.cnt_keep[e][w] = __popcll(bal);
    }
  __syncthreads();
  {
    int running = 0;
#pragma unroll
    for (int e = 0; e < kRegPer; ++e)
      if (e < live) {
        int base = running;
#pragma unroll
        for (int ww = 0; ww < kWaves; ++ww) {
          const int c = S.cnt_keep[e][ww];
          base += ww < w ? c : 0;
          running += c;
        }
        const bool keep = (keep_bits >> e) & 1u;
        const uint64_t bal = __ballot(keep);
        const int i = tid + e * kThreads;
        if (i < n) a.keep_mask[static_cast<size_t>(s0) + v0 + i] = keep ? 1 : 0;
        if (keep)  // read by the copying blocks of this launch: through to the memory side
          __hip_atomic_store(&a.ws_kept[static_cast<size_t>(s0) + v0 + base + __popcll(bal & below)], v0 + i,
                             __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
  }
  for (int p = tid; p < N - n; p += kThreads)  // the rows outside the span are all kept
    a.keep_mask[static_cast<size_t>(s0) + (p < v0 ? p : p + n)] = 1;
  if (tid == 0) {
    const int kept = q.kept();
    a.out_off[b] = first_kept;
    if (b == a.B - 1) a.out_off[a.B] = first_kept + kept;
    if (a.cache_len) {
      a.cache_len[b] = kept > a.cap ? a.cap : kept;
      if (kept > a.cap && a.err_flag) *a.err_flag = 1;
    }
  }
  return true;
}

// Destination and source of row r of class CLASS.
struct RowPlace {
  int b, pos, j, s0, q, first;  // q: index of the row among the sequence's rows of the class, first: cls_off[b]
};

template <int CLASS>
__device__ __forceinline__ RowPlace place_row(const Layout& L, int B, int r) {
  int lo = 0, hi = B - 1;  // the sequence that holds row r of the class (sequences without such rows are skipped)
  while (lo < hi) {
    const int mid = (lo + hi) >> 1;
    if (L.cls_off[mid + 1] <= r) lo = mid + 1; else hi = mid;
  }
  RowPlace p;
  p.b = lo;
  const int q = r - L.cls_off[lo];
  // class 0, q-th row outside the span: before it, or after it (k of the n vision rows stay in between);
  // class 1, q-th kept vision row
  p.pos = CLASS == 0 ? (q < L.v0[lo] ? q : q + L.k[lo]) : L.v0[lo] + q;
  p.j = L.out_off[lo] + p.pos;
  p.s0 = L.s0[lo];
  p.q = q;
  p.first = L.cls_off[lo];
  return p;
}

constexpr int kHeadStart = 48;       // s_sleep units (64 clocks) the first copying blocks pause before their loads
constexpr int kDoneStripes = 16;     // completion counters per sequence (the copy of kept row q bumps counter q % 16)
constexpr int kPatience = 1 << 12;   // polls of a ready word (a few milliseconds) before a block looks for itself
constexpr int kSpinLimit = 1 << 18;  // polls before it gives up (over a tenth of a second)

// One launch: blocks [0, B) select; the next rest_blocks copy the rows outside the vision spans (looping over
// them); the others copy one kept vision row each.
//
// A kept vision row needs its sequence's selection.  Hand-off per sequence b through three words, zero between
// calls: the block that first swaps a 1 into claim[b] runs the selection and then sets ready[b]; a copying block
// polls ready[b].  The selection blocks come first in the grid, so they are running by the time a copying block
// starts and the poll normally ends after the selection's own latency; a copying block that has polled for
// milliseconds tries the claim itself and, if it gets it, runs the selection.  So a block only ever waits for a
// block that is already running and that waits for nothing itself: the waits end under any dispatch order.
// The words are cleared for the next call by the last block that needs them, found by counting -- in two levels,
// because a hundred blocks bumping one word would queue up on it (measured: atomics on one address complete at
// about 20 per microsecond): the copy of a sequence's q-th kept row bumps the sequence's counter q % 16 (how many
// rows share it follows from k), the last block on each of those and the sequence's selection block bump done[b],
// and the last of those clears claim[b], ready[b] and done[b].  All of these words sit at fixed offsets at the
// start of the workspace, whatever the call's shape: a workspace serves calls of different shapes in turn, and a
// word that one shape expects to be zero must never lie where another shape keeps data.
__global__ __launch_bounds__(kThreads) void select_compact_topk_kernel(SelectArgs a, GatherArgs g, int rest_blocks) {
  union Shared {
    TopkShared sel;
    SelectSharedT<0> long_span;
    Layout lay;
  };
  __shared__ Shared S;
  __shared__ int sm_state;
  const int tid = threadIdx.x, blk = blockIdx.x;
  int32_t* claim = a.ws_sync;
  int32_t* ready = claim + kLayoutSeqs;
  int32_t* done = ready + kLayoutSeqs;
  int32_t* stripe_done = done + kLayoutSeqs;  // [kLayoutSeqs][kDoneStripes]

  int b, k;  // the sequence whose hand-off this block takes part in, and its number of kept vision rows
  RowPlace place{};
  const bool copies = blk >= a.B;
  if (!copies) {
    b = blk;
    k = seq_shape(a.seq_off[b], a.seq_off[b + 1], a.vis_start[b], a.vis_len[b], a.keep_ratio).k;
  } else if (blk < a.B + rest_blocks) {
    layout_build<0>(S.lay, g);
    // The selection blocks are about to read their scores.  Behind the first burst of copies (eight blocks per
    // compute unit, 64 KiB each) those few loads wait until the burst has drained, and every kept vision row waits
    // with them; a pause of a microsecond or two here lets them go first.
    __builtin_amdgcn_s_sleep(kHeadStart);
    const int rows = S.lay.cls_off[a.B];
    for (int r = blk - a.B; r < rows; r += rest_blocks) {
      const RowPlace p = place_row<0>(S.lay, a.B, r);
      const int rel = p.pos < S.lay.v0[p.b] ? p.pos : p.pos - S.lay.k[p.b] + S.lay.n[p.b];
      if (tid == 0) g.kept_idx[p.j] = rel;
      copy_row(g, p.b, p.pos, static_cast<size_t>(p.s0) + rel, p.j);
    }
    return;
  } else {
    layout_build<1>(S.lay, g);
    const int r = blk - a.B - rest_blocks;
    if (r >= S.lay.cls_off[a.B]) return;
    place = place_row<1>(S.lay, a.B, r);
    b = place.b;
    k = S.lay.k[b];
    __syncthreads();  // the layout is not read again: the selection may reuse its memory
  }

  // state: 0 = the selection is ready, 1 = this block runs it, 2 = gave up
  if (tid == 0) {
    int state = -1;
    if (!copies) {
      // (stand_back: as if this block had not been dispatched yet -- the path a copying block takes when its patience
      // runs out is then the one that selects; a sequence without kept vision rows has no copying block to do it)
      if (a.stand_back && k > 0) state = 0;
      else state = __hip_atomic_exchange(&claim[b], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == 0 ? 1 : 0;
    } else {
      for (int spins = 0; state < 0; ++spins) {
        if (__hip_atomic_load(&ready[b], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) state = 0;
        else if (spins == kPatience &&
                 __hip_atomic_exchange(&claim[b], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == 0) state = 1;
        else if (spins >= kSpinLimit) state = 2;
        else __builtin_amdgcn_s_sleep(32);
      }
    }
    sm_state = state;
  }
  __syncthreads();
  const int state = sm_state;
  if (state == 1) {
    if (!select_topk_regs(a, S.sel, b)) select_block<true, 0>(a, S.long_span, b);
    block_publish();  // the kept positions have reached the memory side
    if (tid == 0) __hip_atomic_store(&ready[b], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  if (state == 2) {
    if (tid == 0 && a.err_flag) *a.err_flag = 2;
  } else if (copies) {
    const int rel = __hip_atomic_load(&a.ws_kept[static_cast<size_t>(place.s0) + place.pos], __ATOMIC_RELAXED,
                                      __HIP_MEMORY_SCOPE_AGENT);
    if (tid == 0) g.kept_idx[place.j] = rel;
    copy_row(g, b, place.pos, static_cast<size_t>(place.s0) + rel, place.j);
  }
  // (only this thread read the hand-off words, before the barrier above; the kept positions themselves stay)
  if (tid == 0) {
    bool last_of_group = true;
    if (copies) {
      const int stripe = place.q % kDoneStripes;
      const int members = (k - 1 - stripe) / kDoneStripes + 1;  // rows q < k with q % 16 == stripe (q itself is one)
      int32_t* cnt = &stripe_done[b * kDoneStripes + stripe];
      last_of_group = add_agent(cnt, 1) == members - 1;
      if (last_of_group) zero_agent(cnt);
    }
    const int groups = k < kDoneStripes ? k : kDoneStripes;  // stripes that have rows
    if (last_of_group && add_agent(&done[b], 1) == groups) {
      zero_agent(&claim[b]);
      zero_agent(&ready[b]);
      zero_agent(&done[b]);
    }
  }
}

}  // namespace
}  // namespace dllava

using namespace dllava;

// Workspace layout: [words that are zero between calls, at fixed offsets | per-sequence counts | kept positions].
// The fixed part: the ticket of select_kernel (256 bytes of its own), then claim / ready / done per sequence and
// the stripe counters of the one-launch arrangement.
static constexpr size_t kTicketBytes = 256;
static constexpr size_t kSyncWords = 3 * kLayoutSeqs + kLayoutSeqs * kDoneStripes;
static constexpr size_t kFixedBytes = (kTicketBytes + kSyncWords * sizeof(int32_t) + 255) / 256 * 256;

extern "C" size_t dllava_select_compact_workspace(int32_t B, int64_t sumN) {
  const size_t b = B > 0 ? B : 0, n = sumN > 0 ? sumN : 0;
  return kFixedBytes + round_up(b * sizeof(int32_t), 256) + round_up(n * sizeof(int32_t), 256);
}

extern "C" int dllava_select_compact(const float* logits, int32_t B, const int32_t* seq_off,
                                     const int32_t* vis_start, const int32_t* vis_len, int64_t sumN, int mode,
                                     double keep_ratio, float threshold, const void* hidden, void* hidden_out,
                                     int64_t d, const void* Q, void* Q_out, const void* K, const void* V,
                                     const dllava_kv_cache* cache, uint8_t* keep_mask, int32_t* kept_idx,
                                     int32_t* out_off, int32_t* err_flag, int dtype, void* workspace,
                                     size_t workspace_bytes, void* stream) {
  DLLAVA_REQUIRE(B >= 0 && sumN >= 0, DLLAVA_EINVAL, "select_compact: B = %d, sumN = %lld", B, (long long)sumN);
  DLLAVA_REQUIRE(sumN <= 0x7fffffffLL, DLLAVA_ESHAPE, "select_compact: sumN must fit in int32");
  DLLAVA_REQUIRE(dtype == DLLAVA_F32 || dtype == DLLAVA_BF16, DLLAVA_EDTYPE, "select_compact: unknown dtype %d", dtype);
  DLLAVA_REQUIRE(mode == DLLAVA_MODE_TOPK || mode == DLLAVA_MODE_THRESHOLD || mode == DLLAVA_MODE_THRESHOLD_KEEP_LAST,
                 DLLAVA_EINVAL,
                 "select_compact: unknown mode %d", mode);
  if (mode == DLLAVA_MODE_TOPK)
    DLLAVA_REQUIRE(keep_ratio >= 0.0 && keep_ratio <= 1.0, DLLAVA_EINVAL,
                   "select_compact: keep_ratio must lie in [0,1] (got %g)", keep_ratio);
  else
    DLLAVA_REQUIRE(threshold == threshold, DLLAVA_EINVAL, "select_compact: threshold is NaN");
  DLLAVA_REQUIRE(out_off, DLLAVA_ENULL, "select_compact: out_off is required");
  DLLAVA_REQUIRE((hidden == nullptr) == (hidden_out == nullptr), DLLAVA_ENULL,
                 "select_compact: hidden and hidden_out go together");
  DLLAVA_REQUIRE((Q == nullptr) == (Q_out == nullptr), DLLAVA_ENULL, "select_compact: Q and Q_out go together");
  DLLAVA_REQUIRE((K == nullptr) == (V == nullptr), DLLAVA_ENULL, "select_compact: K and V go together");
  DLLAVA_REQUIRE(!K || cache, DLLAVA_ENULL, "select_compact: K/V need a cache to be written to");
  DLLAVA_REQUIRE(!Q || cache, DLLAVA_ENULL, "select_compact: Q needs cache->H and cache->Dh");
  const size_t es = dtype_size(dtype);
  if (cache) {
    if (int rc = check_cache(cache, "select_compact")) return rc;
    DLLAVA_REQUIRE(cache->dtype == dtype, DLLAVA_EDTYPE, "select_compact: cache dtype differs from dtype");
  }
  if (hidden) {
    DLLAVA_REQUIRE(d > 0 && (d * es) % 16 == 0, DLLAVA_ESHAPE,
                   "select_compact: hidden rows must be a multiple of 16 bytes (d = %lld)", (long long)d);
    DLLAVA_REQUIRE(aligned(hidden, 16) && aligned(hidden_out, 16), DLLAVA_EINVAL,
                   "select_compact: hidden buffers must be 16-byte aligned");
  }
  DLLAVA_REQUIRE((!Q || (aligned(Q, 16) && aligned(Q_out, 16))) && (!K || (aligned(K, 16) && aligned(V, 16))),
                 DLLAVA_EINVAL, "select_compact: Q/K/V buffers must be 16-byte aligned");
  if (B == 0) return DLLAVA_OK;  // nothing to read: out_off[0] is left to the caller
  DLLAVA_REQUIRE(logits && seq_off && vis_start && vis_len && keep_mask && kept_idx, DLLAVA_ENULL,
                 "select_compact: logits, seq_off, vis_start, vis_len, keep_mask, kept_idx are required");
  const size_t need = dllava_select_compact_workspace(B, sumN);
  DLLAVA_REQUIRE(workspace && aligned(workspace, 256) && workspace_bytes >= need, DLLAVA_EWORKSPACE,
                 "select_compact: workspace needs %zu bytes, 256-byte aligned (got %zu)", need, workspace_bytes);

  hipStream_t st = static_cast<hipStream_t>(stream);
  char* ws = static_cast<char*>(workspace);
  int32_t* ws_ticket = reinterpret_cast<int32_t*>(ws);
  int32_t* ws_sync = reinterpret_cast<int32_t*>(ws + kTicketBytes);
  int32_t* ws_counts = reinterpret_cast<int32_t*>(ws + kFixedBytes);
  int32_t* ws_kept = reinterpret_cast<int32_t*>(ws + kFixedBytes + round_up(static_cast<size_t>(B) * 4, 256));
  const bool write_cache = K != nullptr;
  const int32_t cap = cache ? cache->max_pages_per_seq * cache->page_size : 0;
  SelectArgs sa{logits, seq_off, vis_start, vis_len, B, mode, keep_ratio, threshold, keep_mask, ws_kept, ws_counts,
                ws_ticket, out_off, write_cache ? cache->cache_len : nullptr, cap, err_flag, ws_sync,
                launch_override(DLLAVA_LAUNCH_SELECT_LAUNCHES) == 3};
  const bool analytic =
      mode == DLLAVA_MODE_TOPK && B <= kLayoutSeqs && sumN > 0 && launch_override(DLLAVA_LAUNCH_SELECT_LAUNCHES) != 2;
  if (!analytic) {
    hipLaunchKernelGGL(select_kernel, dim3(B), dim3(kThreads), 0, st, sa);
    DLLAVA_CHECK_LAUNCH("select_kernel");
  }

  if (sumN == 0) return DLLAVA_OK;
  GatherArgs ga{};
  ga.vis_start = vis_start; ga.vis_len = vis_len; ga.keep_ratio = keep_ratio;
  ga.seq_off = seq_off; ga.out_off = out_off; ga.ws_kept = ws_kept; ga.kept_idx = kept_idx; ga.B = B;
  ga.hidden = static_cast<const uint4*>(hidden); ga.hidden_out = static_cast<uint4*>(hidden_out);
  ga.hidden_chunks = hidden ? static_cast<int64_t>(d * es / 16) : 0;
  if (cache) {
    ga.H = cache->H;
    ga.head_chunks = static_cast<int32_t>(cache->Dh * es / 16);
    ga.kv_chunks = static_cast<int64_t>(ga.H) * ga.head_chunks;
    ga.q_chunks = ga.kv_chunks;
    ga.max_pages = cache->max_pages_per_seq;
    ga.pages = static_cast<uint4*>(cache->pages);
    ga.block_table = cache->block_table;
  }
  ga.Q = static_cast<const uint4*>(Q); ga.Q_out = static_cast<uint4*>(Q_out);
  ga.K = static_cast<const uint4*>(K); ga.V = static_cast<const uint4*>(V);
  if (analytic) {
    // rows outside the spans number at most sumN (their blocks loop: the grid is not sized for the worst case); the
    // kept vision rows number sum of floor(ratio * n) <= ratio * sumN
    const int64_t rest_blocks = sumN < kRestBlocks ? sumN : kRestBlocks;
    int64_t vis_blocks = static_cast<int64_t>(ceil(keep_ratio * static_cast<double>(sumN))) + 1;
    if (vis_blocks > sumN) vis_blocks = sumN;
    hipLaunchKernelGGL(select_compact_topk_kernel, dim3(static_cast<unsigned>(B + rest_blocks + vis_blocks)),
                       dim3(kThreads), 0, st, sa, ga, static_cast<int>(rest_blocks));
    DLLAVA_CHECK_LAUNCH("select_compact_topk_kernel");
    return DLLAVA_OK;
  }
  hipLaunchKernelGGL(gather_kernel, dim3(static_cast<unsigned>(sumN)), dim3(kThreads), 0, st, ga);
  DLLAVA_CHECK_LAUNCH("gather_kernel");
  return DLLAVA_OK;
}

extern "C" int dllava_compact(int32_t B, const int32_t* seq_off, const int32_t* kept_idx, const int32_t* out_off,
                              int64_t sumN, const void* hidden, void* hidden_out, int64_t d, const void* Q, void* Q_out,
                              const void* K, const void* V, const dllava_kv_cache* cache, int32_t* err_flag, int dtype,
                              void* stream) {
  DLLAVA_REQUIRE(B >= 0 && sumN >= 0 && sumN <= 0x7fffffffLL, DLLAVA_EINVAL, "compact: B = %d, sumN = %lld", B,
                 (long long)sumN);
  DLLAVA_REQUIRE(dtype == DLLAVA_F32 || dtype == DLLAVA_BF16, DLLAVA_EDTYPE, "compact: unknown dtype %d", dtype);
  const int64_t es = dtype == DLLAVA_BF16 ? 2 : 4;
  DLLAVA_REQUIRE(!hidden || (d > 0 && (d * es) % 16 == 0), DLLAVA_ESHAPE,
                 "compact: rows of hidden must be a multiple of 16 bytes (d = %lld)", (long long)d);
  DLLAVA_REQUIRE((hidden == nullptr) == (hidden_out == nullptr) && (Q == nullptr) == (Q_out == nullptr) &&
                     (K == nullptr) == (V == nullptr),
                 DLLAVA_ENULL, "compact: hidden/hidden_out, Q/Q_out and K/V go together");
  if (Q || K) {
    if (int rc = check_cache(cache, "compact")) return rc;
    DLLAVA_REQUIRE(cache->dtype == dtype, DLLAVA_EDTYPE, "compact: cache dtype differs from the call's");
  }
  if (B == 0 || sumN == 0) return DLLAVA_OK;
  DLLAVA_REQUIRE(seq_off && kept_idx && out_off, DLLAVA_ENULL, "compact: seq_off, kept_idx and out_off are required");
  DLLAVA_REQUIRE(aligned(hidden, 16) && aligned(hidden_out, 16) && aligned(Q, 16) && aligned(Q_out, 16) &&
                     aligned(K, 16) && aligned(V, 16),
                 DLLAVA_EINVAL, "compact: tensors must be 16-byte aligned");
  GatherArgs ga{};
  ga.seq_off = seq_off; ga.out_off = out_off; ga.kept_idx = const_cast<int32_t*>(kept_idx); ga.B = B;
  ga.given = 1;
  ga.hidden = static_cast<const uint4*>(hidden); ga.hidden_out = static_cast<uint4*>(hidden_out);
  ga.hidden_chunks = hidden ? static_cast<int64_t>(d * es / 16) : 0;
  if (cache && (Q || K)) {
    ga.H = cache->H;
    ga.head_chunks = static_cast<int32_t>(cache->Dh * es / 16);
    ga.kv_chunks = static_cast<int64_t>(ga.H) * ga.head_chunks;
    ga.q_chunks = ga.kv_chunks;
    ga.max_pages = cache->max_pages_per_seq;
    ga.pages = static_cast<uint4*>(cache->pages);
    ga.block_table = cache->block_table;
    if (K) {
      ga.cache_len = cache->cache_len;
      ga.cap = cache->max_pages_per_seq * cache->page_size;
      ga.err_flag = err_flag;
    }
  }
  ga.Q = static_cast<const uint4*>(Q); ga.Q_out = static_cast<uint4*>(Q_out);
  ga.K = static_cast<const uint4*>(K); ga.V = static_cast<const uint4*>(V);
  hipLaunchKernelGGL(gather_kernel, dim3(static_cast<unsigned>(sumN)), dim3(kThreads), 0, static_cast<hipStream_t>(stream),
                     ga);
  DLLAVA_CHECK_LAUNCH("gather_kernel");
  return DLLAVA_OK;
}
