// dllava_select_compact: keep decisions (Eq. 5 line 2 / Eq. 11 line 2 of the paper) and order-preserving
// stream compaction of hidden states, queries and K/V into the reduced token set / paged cache
// (Eq. 5 line 3 / Eq. 11 line 3).
//
// Two launches:
//   1. select_kernel   one block per sequence.  Top-k: the k-th largest score is found exactly by a
//                      4-pass most-significant-byte radix select over an order-preserving 32-bit key,
//                      then one in-order pass keeps keys above it plus the first (k - #above) equal keys,
//                      which is the "ties go to the lower index" rule.  The same pass ranks the kept
//                      rows of the sequence (prefix sum), so kept positions come out ascending.
//                      The block that finishes last (device-scope ticket) scans the per-sequence counts
//                      into out_off, sets cache_len and checks the capacity.
//   2. gather_kernel   one block per compacted row: 16-byte coalesced copies of its hidden, Q, K and V rows;
//                      K/V rows are scattered head by head into their page slot.
// Selection is integer-exact: it only compares float32 keys.
#include "common.h"

namespace dllava {
namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / kWave;

// Order-preserving key: larger score <-> larger key; -0 and +0 share a key; NaN gets the lowest key.
__device__ __forceinline__ uint32_t score_key(float s) {
  if (s != s) return 0u;
  if (s == 0.f) return 0x80000000u;
  const uint32_t u = __float_as_uint(s);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
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
};

constexpr int kKeyCache = 4096;  // scores of one vision span kept in LDS (16 KiB); longer spans re-read them

__global__ __launch_bounds__(kThreads) void select_kernel(SelectArgs a) {
  __shared__ int hist[256];
  __shared__ int sm_tot[kWaves];
  __shared__ int sm_sel[2];
  __shared__ uint32_t skey[kKeyCache];
  __shared__ int sm_last;
  const int b = blockIdx.x, tid = threadIdx.x;
  const int s0 = a.seq_off[b];
  int N = a.seq_off[b + 1] - s0;
  if (N < 0) N = 0;
  int v0 = a.vis_start[b];
  v0 = v0 < 0 ? 0 : (v0 > N ? N : v0);
  int n = a.vis_len[b];
  n = n < 0 ? 0 : (n > N - v0 ? N - v0 : n);

  // row of this sequence's first vision token in `logits`
  int part = 0;
  for (int i = tid; i < b; i += kThreads) {
    const int x = a.vis_len[i];
    part += x > 0 ? x : 0;
  }
  int lo;
  block_excl_scan(part, sm_tot, lo);
  const float* D = a.logits + 2 * static_cast<size_t>(lo);

  const bool cached = n <= kKeyCache;
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
      if (cached)
        for (int i = tid; i < n; i += kThreads) skey[i] = score_key(D[2 * i + 1]);
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
        if (keep) a.ws_kept[static_cast<size_t>(s0) + pos++] = p;
      }
    }
  }
  // The block that finishes last turns the per-sequence counts into offsets (exclusive scan), sets the cache
  // lengths and checks the capacity: no second launch.  Hand-off through device-scope stores and a ticket.
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
};

// 16 readable bytes: the source of the (unused) clamped loads of a tensor that is not being moved
static __device__ __attribute__((aligned(16))) uint32_t kGatherPad[4] = {0u, 0u, 0u, 0u};

// One block per compacted row moves all of its tensors: hidden, Q, K, V.  The dependent chain in front of the
// copies (total, binary search for the sequence, kept position) is paid once per row, and every 16-byte load of
// a trip -- two per thread and tensor, index clamped so that none sits under a condition -- is in flight
// before the first store.
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

}  // namespace
}  // namespace dllava

using namespace dllava;

extern "C" size_t dllava_select_compact_workspace(int32_t B, int64_t sumN) {
  const size_t b = B > 0 ? B : 0, n = sumN > 0 ? sumN : 0;
  return round_up(n * sizeof(int32_t), 256) + round_up(b * sizeof(int32_t), 256) + 256;
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
  int32_t* ws_kept = static_cast<int32_t*>(workspace);
  int32_t* ws_counts =
      reinterpret_cast<int32_t*>(static_cast<char*>(workspace) + round_up(static_cast<size_t>(sumN) * 4, 256));

  int32_t* ws_ticket = ws_counts + round_up(static_cast<size_t>(B) * 4, 256) / 4;
  const bool write_cache = K != nullptr;
  const int32_t cap = cache ? cache->max_pages_per_seq * cache->page_size : 0;
  SelectArgs sa{logits, seq_off, vis_start, vis_len, B, mode, keep_ratio, threshold, keep_mask, ws_kept, ws_counts,
                ws_ticket, out_off, write_cache ? cache->cache_len : nullptr, cap, err_flag};
  hipLaunchKernelGGL(select_kernel, dim3(B), dim3(kThreads), 0, st, sa);
  DLLAVA_CHECK_LAUNCH("select_kernel");

  if (sumN == 0) return DLLAVA_OK;
  GatherArgs ga{};
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
