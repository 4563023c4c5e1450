// dllava_decode_attn_append: one decode step with online KV-cache reduction (Eq. 6 of the paper).
//
// The step is a pure stream over the reduced cache: LLaVA-1.5 is plain multi-head attention, so every
// cached K/V byte is read by exactly one (sequence, head) query and there is one flop per byte.  The
// kernel therefore uses fully coalesced 16-byte loads and VALU arithmetic, not matrix cores.
//
// ONE launch per step.  Grid (n_split, H, B), NW waves per block (4 or 8).  The S*NW waves that serve
// (b, h) take the P = ceil(cache_len[b]/16) pages of sequence b round-robin, 8 KiB of K and V per page,
// and the waves of a block are merged through LDS.  The kernel is latency-bound at short contexts, so the
// dependent-load chain is kept short: page ids and, with a single split, the first page itself are
// requested before cache_len has arrived.  Split 0 also folds in the current token (it always takes part
// in its own attention).

//
// Cross-block steps use device-scope counters kept at the start of the workspace (zero before the first
// call; each is reset by the block that consumes it):
//   * cache_len[b] may only advance once every block of sequence b has read it.  Each block draws a ticket
//     right after its read; the block holding the last ticket commits the keep decision: it stores the new
//     token's K/V for all heads at position cache_len[b] (a slot whose content no block uses in this launch)
//     and advances the length -- at once when there is one block per (b, h), at its end otherwise.  Same-address
//     atomics are slow (they serialise at the memory side), but drawn at the start their latency is hidden
//     behind the page stream.
//   * with S > 1, the last of the S blocks of (b, h) to finish merges the S partial (max, sum, accumulator)
//     triples in split order -- a fixed order, so the result is bit-reproducible -- and writes o[b, h].
#include <limits.h>

#include <mutex>

#include "attend.h"
#include "score_splitk.h"

// Scratch of dllava_decode_attn_append_static (see there): counters first, then the partial results of split launches.
constexpr size_t kStaticCounterBytes = size_t{3} << 20;  // counters: (2*B*H + B) * 256 bytes at most this
constexpr size_t kStaticPartialBytes = size_t{1} << 20;  // partial results of the split count actually launched
constexpr size_t kStaticScratchBytes = kStaticCounterBytes + kStaticPartialBytes;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace dllava {
namespace {

constexpr int kMaxSplit = 16;
constexpr int kCnt = 64;  // int32 slots per counter: each counter owns 256 bytes, because atomics that share a
                          // memory line serialise at the memory side even when their addresses differ

struct DecodeArgs {
  const void* q;
  const void* k_new;
  const void* v_new;
  const float* logits;
  const uint8_t* keep_override;
  float threshold;
  float scale_log2;
  void* pages;
  const int32_t* block_table;
  int32_t* cache_len;
  int32_t max_pages;
  int32_t H;
  int32_t B;
  int32_t n_split;
  int32_t* cnt_bh;    // [B*H] blocks of (b, h) that have read cache_len[b]   (used when S > 1)
  int32_t* cnt_done;  // [B*H] blocks of (b, h) whose partial result is published
  int32_t* cnt_b;     // [B]   heads of sequence b all of whose blocks have read cache_len[b]
  float* part_acc;  // [B*H*S][DH]
  float* part_ml;   // [B*H*S][2]
  void* o;
  uint8_t* keep_out;
  int32_t* err_flag;
  // deferred form (dllava_decode_step): the tokens of the PREVIOUS step, whose keep decision is applied now
  const void* k_prev;
  const void* v_prev;
  const float* logits_prev;
  const uint8_t* keep_prev_override;
};

// ---- one 16-token page held in registers -------------------------------------------------------
template <typename T, int DH>
struct PageRegs {
  uint4 k[AttendCfg<T, DH>::NL];
  uint4 v[AttendCfg<T, DH>::NL];
};

template <typename T, int DH>
__device__ __forceinline__ void load_page(PageRegs<T, DH>& r, const T* __restrict__ kt, const T* __restrict__ vt) {
  using C = AttendCfg<T, DH>;
  const int lane = threadIdx.x & (kWave - 1);
  // lane -> (row lane/G of each group of R rows, 16-byte chunk lane%G): consecutive lanes, consecutive bytes
#pragma unroll
  for (int i = 0; i < C::NL; ++i) {
    r.k[i] = reinterpret_cast<const uint4*>(kt)[i * kWave + lane];
    r.v[i] = reinterpret_cast<const uint4*>(vt)[i * kWave + lane];
  }
}

// sum over the G lanes that share a token row, on the DPP data path where the group fits a 16-lane row
template <int G>
__device__ __forceinline__ float row_group_sum(float v) {
  static_assert(G == 8 || G == 16 || G == 32, "group size");
#define DLLAVA_DPP_ADD(ctrl) \
  v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), ctrl, 0xf, 0xf, true))
  DLLAVA_DPP_ADD(0xB1);   // quad_perm [1,0,3,2]
  DLLAVA_DPP_ADD(0x4E);   // quad_perm [2,3,0,1]
  DLLAVA_DPP_ADD(0x141);  // row_half_mirror: joins the two quads of each 8 lanes
  if (G >= 16) DLLAVA_DPP_ADD(0x140);  // row_mirror: joins the two halves of each 16 lanes
#undef DLLAVA_DPP_ADD
  if (G == 32) v += __shfl_xor(v, 16, kWave);
  return v;
}

// q . k for this lane's 16 bytes of a key row; q is pre-scaled float32 (generic) ...
template <typename T>
struct LaneDot {
  static constexpr int E = 16 / sizeof(T);
  float qs[E];
  __device__ __forceinline__ void init(const T* qrow, int c, float scale_log2) {
    Elem<T>::unpack(*reinterpret_cast<const uint4*>(qrow + c * E), qs);
#pragma unroll
    for (int e = 0; e < E; ++e) qs[e] *= scale_log2;
  }
  __device__ __forceinline__ float dot(const uint4& kr) const {
    float kf[E];
    Elem<T>::unpack(kr, kf);
    float d = 0.f;
#pragma unroll
    for (int e = 0; e < E; ++e) d = fmaf(qs[e], kf[e], d);
    return d;
  }
};
// ... or, for bfloat16, the raw bf16 pairs fed to the packed dot-product instruction (float32 accumulate)
template <>
struct LaneDot<bf16_t> {
  typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
  uint4 qraw;
  float scale_log2;
  __device__ __forceinline__ void init(const bf16_t* qrow, int c, float s) {
    qraw = *reinterpret_cast<const uint4*>(qrow + c * 8);
    scale_log2 = s;
  }
  __device__ static __forceinline__ bf16x2 pair(uint32_t u) {
    union { uint32_t u; bf16x2 p; } c;
    c.u = u;
    return c.p;
  }
  __device__ __forceinline__ float dot(const uint4& kr) const {
    float d = __builtin_amdgcn_fdot2_f32_bf16(pair(qraw.x), pair(kr.x), 0.f, false);
    d = __builtin_amdgcn_fdot2_f32_bf16(pair(qraw.y), pair(kr.y), d, false);
    d = __builtin_amdgcn_fdot2_f32_bf16(pair(qraw.z), pair(kr.z), d, false);
    d = __builtin_amdgcn_fdot2_f32_bf16(pair(qraw.w), pair(kr.w), d, false);
    return d * scale_log2;
  }
};

// online-softmax update of one lane group with the 16/R rows it owns in this page
template <typename T, int DH, bool MASKED>
__device__ __forceinline__ void consume_page(const PageRegs<T, DH>& pr, int nvalid, const LaneDot<T>& qd,
                                             AttnState<AttendCfg<T, DH>::E>& st) {
  using C = AttendCfg<T, DH>;
  const int r = (threadIdx.x & (kWave - 1)) / C::G;
  float s[C::NL];
  float mx = st.m;
#pragma unroll
  for (int i = 0; i < C::NL; ++i) {
    float d = row_group_sum<C::G>(qd.dot(pr.k[i]));
    if (MASKED && (i * C::R + r) >= nvalid) d = -INFINITY;
    s[i] = d;
    mx = fmaxf(mx, d);
  }
  const float ms = (MASKED && mx == -INFINITY) ? 0.f : mx;
  const float alpha = __builtin_amdgcn_exp2f(st.m - ms);
  st.l *= alpha;
#pragma unroll
  for (int e = 0; e < C::E; ++e) st.acc[e] *= alpha;
#pragma unroll
  for (int i = 0; i < C::NL; ++i) {
    const float p = __builtin_amdgcn_exp2f(s[i] - ms);
    st.l += p;
    float vf[C::E];
    Elem<T>::unpack(pr.v[i], vf);
#pragma unroll
    for (int e = 0; e < C::E; ++e) {
      const float ve = (MASKED && (i * C::R + r) >= nvalid) ? 0.f : vf[e];  // slots past the end hold anything
      st.acc[e] = fmaf(p, ve, st.acc[e]);
    }
  }
  st.m = mx;
}

// Commits the decision of sequence b: keep flag, the new token's K/V for all heads at position cache_len[b],
// the length.  Called by all threads of exactly one block per sequence and launch, after every block of the
// sequence has read cache_len[b].
template <typename T, int DH>
__device__ __forceinline__ void commit_sequence(const DecodeArgs& a, int b) {
  const int tid = threadIdx.x, nthr = blockDim.x;
  const int H = a.H, cap = a.max_pages * kPage;
  const bool keep = a.keep_override ? a.keep_override[b] != 0 : keep_from_logits(a.logits, b, a.threshold);
  const int L = a.cache_len[b];
  if (tid == 0 && a.keep_out) a.keep_out[b] = keep ? 1 : 0;
  if (!keep) return;  // block-uniform
  if (L < 0 || L >= cap) {
    if (tid == 0 && a.err_flag) *a.err_flag = 1;
    return;
  }
  constexpr int kChunks = DH * sizeof(T) / 16;  // 16-byte chunks per (token, head)
  const size_t tile = static_cast<size_t>(kPage) * DH;
  const int pg = a.block_table[static_cast<size_t>(b) * a.max_pages + L / kPage];
  T* pages = static_cast<T*>(a.pages);
  for (int i = tid; i < 2 * H * kChunks; i += nthr) {
    const int kv = i / (H * kChunks), hh = (i / kChunks) % H, cc = i % kChunks;
    T* dst = pages + ((static_cast<size_t>(pg) * 2 + kv) * H + hh) * tile + static_cast<size_t>(L % kPage) * DH;
    const T* src = static_cast<const T*>(kv ? a.v_new : a.k_new) + (static_cast<size_t>(b) * H + hh) * DH;
    reinterpret_cast<uint4*>(dst)[cc] = reinterpret_cast<const uint4*>(src)[cc];
  }
  __syncthreads();  // every thread has read L before it moves
  if (tid == 0) a.cache_len[b] = L + 1;
}

// Keep decision of the previous step's token of sequence b (deferred form); false when there is none.
__device__ __forceinline__ bool keep_prev_token(const DecodeArgs& a, int b) {
  if (a.keep_prev_override) return a.keep_prev_override[b] != 0;
  if (a.logits_prev) return keep_from_logits(a.logits_prev, b, a.threshold);
  return false;
}

// Deferred form: every (b, h) block has appended its own head's slice of the previous token, so the block that
// knows that all blocks of b have read cache_len[b] only moves the length (and reports decision and overflow).
__device__ __forceinline__ void commit_length(const DecodeArgs& a, int b, bool keep_prev) {
  if (threadIdx.x != 0) return;
  if (a.keep_out && (a.logits_prev || a.keep_prev_override)) a.keep_out[b] = keep_prev ? 1 : 0;
  if (!keep_prev) return;
  const int L = a.cache_len[b];
  if (L < 0 || L >= a.max_pages * kPage) {
    if (a.err_flag) *a.err_flag = 1;
    return;
  }
  a.cache_len[b] = L + 1;
}

// The work of block (s, h, b).  DEFER: the current token is not appended; instead the previous step's token is
// (its decision is known by now), by every block for its own head, and attended as a second in-register key.
template <typename T, int DH, int NW, bool DEFER>
__device__ __forceinline__ void attn_block(const DecodeArgs& a, int s, int h, int b) {
  using C = AttendCfg<T, DH>;
  const int tid = threadIdx.x, lane = tid & (kWave - 1), w = tid / kWave;
  const int S = a.n_split, H = a.H;
  const int cap = a.max_pages * kPage;
  const size_t bh = static_cast<size_t>(b) * H + h;
  const T* qrow = static_cast<const T*>(a.q) + bh * DH;
  const T* knew = static_cast<const T*>(a.k_new) + bh * DH;
  const T* vnew = static_cast<const T*>(a.v_new) + bh * DH;
  const T* pages = static_cast<const T*>(a.pages);
  const int32_t* bt = a.block_table + static_cast<size_t>(b) * a.max_pages;
  const size_t tile = static_cast<size_t>(kPage) * DH;  // elements of one (page, K|V, head) tile
  const size_t vofs = static_cast<size_t>(H) * tile;    // from a K tile to the V tile of the same page/head

  // Pages are dealt round-robin to the S*NW waves that serve (b, h): wave g takes pages g, g+S*NW, ...
  // The indices of a wave's first two pages do not depend on cache_len, so their page-id loads and (with one
  // split) the first K/V loads are issued without waiting for the length: every block-table entry names an
  // allocated page, so the loads are in bounds even if the page turns out to lie beyond the end.
  const int stride = S * NW;
  int p = s * NW + w;
  const int last_entry = a.max_pages - 1;
  int pg = bt[p < last_entry ? p : last_entry];
  int pg_next = bt[p + stride < last_entry ? p + stride : last_entry];
  const bool keep_prev = DEFER ? keep_prev_token(a, b) : false;  // block-uniform
  PageRegs<T, DH> cur;
  const bool spec = (S == 1);
  if (spec) {
    const T* kt = pages + (static_cast<size_t>(pg) * 2 * H + h) * tile;
    load_page<T, DH>(cur, kt, kt + vofs);
  }
  // ONE thread of the block reads cache_len[b] and then announces the read with a ticket; the other waves take the
  // length from LDS after the barrier below.  The block that draws a sequence's last ticket may move cache_len[b]
  // at once, so no wave may read the length from memory after its block's ticket is out: a wave that did would
  // count slot L (the token being appended) as cached.  The increment depends on the loaded value, so it cannot
  // be issued before the load has returned; its own latency hides behind the page stream.
  __shared__ int sm_len, sm_flag, sm_commit;
  int ticket = 0;
  if (tid == 0) {
    // (an atomic load so that it is performed exactly once; the value was written by an earlier launch, so the
    // narrowest scope -- an ordinary cached load -- is enough)
    const int L0 = __hip_atomic_load(&a.cache_len[b], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    ticket = add_agent(S == 1 ? &a.cnt_b[b * kCnt] : &a.cnt_bh[bh * kCnt], 1 + (L0 == INT32_MIN));
    sm_len = L0;
    // With one block per (b, h) the block that drew the last ticket of sequence b already knows that every block
    // of b has read cache_len[b]: it appends and advances the length NOW, while its first page is still on its
    // way, instead of at its end, where the work would lengthen the tail of the launch.  Slot cache_len[b] lies
    // beyond what any block of this launch uses (rows past the length are masked by position, whatever they hold).
    if (S == 1) {
      const int commit = (ticket == H - 1);
      if (commit) zero_agent(&a.cnt_b[b * kCnt]);
      sm_commit = commit;
    }
  }
  __syncthreads();
  int L = sm_len;
  const bool append_prev = DEFER && keep_prev && L >= 0 && L < cap;  // the previous token goes to slot L
  L = L < 0 ? 0 : (L > cap ? cap : L);
  const int P = (L + kPage - 1) / kPage;
  if (!spec && p < P) {
    const T* kt = pages + (static_cast<size_t>(pg) * 2 * H + h) * tile;
    load_page<T, DH>(cur, kt, kt + vofs);
  }
  if (S == 1 && sm_commit) {
    if (DEFER) commit_length(a, b, keep_prev);
    else commit_sequence<T, DH>(a, b);
  }

  LaneDot<T> qd;
  qd.init(qrow, lane % C::G, a.scale_log2);
  AttnState<C::E> st;
  st.clear();

  if (s == 0 && w == 0) {  // the current token, folded into lane group 0
    const uint4 kr = *reinterpret_cast<const uint4*>(knew + (lane % C::G) * C::E);
    const uint4 vr = *reinterpret_cast<const uint4*>(vnew + (lane % C::G) * C::E);
    const float d = row_group_sum<C::G>(qd.dot(kr));
    if (lane < C::G) {
      st.m = d;
      st.l = 1.f;
      Elem<T>::unpack(vr, st.acc);
    }
    if (append_prev) {  // block-uniform
      const T* kp = static_cast<const T*>(a.k_prev) + bh * DH;
      const T* vp = static_cast<const T*>(a.v_prev) + bh * DH;
      const uint4 kr2 = *reinterpret_cast<const uint4*>(kp + (lane % C::G) * C::E);
      const uint4 vr2 = *reinterpret_cast<const uint4*>(vp + (lane % C::G) * C::E);
      const int pgL = bt[L / kPage];  // the clamp left L as it was (append_prev implies 0 <= L < cap)
      T* dstk = const_cast<T*>(pages) + (static_cast<size_t>(pgL) * 2 * H + h) * tile + static_cast<size_t>(L % kPage) * DH;
      if (lane < C::G) {
        *reinterpret_cast<uint4*>(dstk + lane * C::E) = kr2;
        *reinterpret_cast<uint4*>(dstk + vofs + lane * C::E) = vr2;
      }
      const float d2 = row_group_sum<C::G>(qd.dot(kr2));
      if (lane < C::G) {  // online-softmax fold of a second single key into lane group 0
        float v2[C::E];
        Elem<T>::unpack(vr2, v2);
        const float m_new = fmaxf(st.m, d2);
        const float a0 = __builtin_amdgcn_exp2f(st.m - m_new), p2 = __builtin_amdgcn_exp2f(d2 - m_new);
        st.l = st.l * a0 + p2;
#pragma unroll
        for (int e = 0; e < C::E; ++e) st.acc[e] = st.acc[e] * a0 + p2 * v2[e];
        st.m = m_new;
      }
    }
  }

  while (p < P) {
    const int pn = p + stride;
    const int nvalid = L - p * kPage;
    if (nvalid >= kPage)
      consume_page<T, DH, false>(cur, kPage, qd, st);
    else
      consume_page<T, DH, true>(cur, nvalid, qd, st);
    if (pn < P) {
      const T* kt = pages + (static_cast<size_t>(pg_next) * 2 * H + h) * tile;
      load_page<T, DH>(cur, kt, kt + vofs);
      if (pn + stride < P) pg_next = bt[pn + stride];
    }
    p = pn;
  }
  merge_groups<T, DH>(st);

  __shared__ float sm_acc[NW][DH];
  __shared__ float sm_m[NW], sm_l[NW];
  if (lane < C::G) {
#pragma unroll
    for (int e = 0; e < C::E; ++e) sm_acc[w][lane * C::E + e] = st.acc[e];
    if (lane == 0) {
      sm_m[w] = st.m;
      sm_l[w] = st.l;
    }
  }
  const int target = H;  // tickets on cnt_b[b] before the sequence may be committed
  if (S > 1 && tid == 0) {
    int commit = 0;
    if (ticket == S - 1) {
      // every block of (b, h) has read the length once the last reader's ticket is out; that block reports
      // the head to the sequence counter
      zero_agent(&a.cnt_bh[bh * kCnt]);
      commit = (add_agent(&a.cnt_b[b * kCnt], 1) == target - 1);
    }
    if (commit) zero_agent(&a.cnt_b[b * kCnt]);
    sm_commit = commit;
  }
  __syncthreads();

  float M = -INFINITY, l = 0.f, acc = 0.f;
  if (tid < DH) {
    M = sm_m[0];
#pragma unroll
    for (int i = 1; i < NW; ++i) M = fmaxf(M, sm_m[i]);
#pragma unroll
    for (int i = 0; i < NW; ++i) {
      const float wgt = (sm_m[i] == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(sm_m[i] - M);
      l += wgt * sm_l[i];
      acc += wgt * sm_acc[i][tid];
    }
  }
  bool finalize = true;  // this block writes o[b, h]
  if (S > 1) {
    if (tid < DH) {
      const size_t ps = bh * S + s;
      st_agent(a.part_acc + ps * DH + tid, acc);
      if (tid == 0) {
        st_agent(a.part_ml + 2 * ps, M);
        st_agent(a.part_ml + 2 * ps + 1, l);
      }
    }
    block_publish();  // partials have reached the memory side before the counter moves
    if (tid == 0) sm_flag = (add_agent(&a.cnt_done[bh * kCnt], 1) == S - 1);
    __syncthreads();
    finalize = sm_flag != 0;
    if (finalize) {
      if (tid < DH) {
        // all S partials are requested before any is used (S <= kMaxSplit): a dependent chain of
        // device-scope loads would cost one memory round trip per split
        const float* ml = a.part_ml + 2 * bh * S;
        float pm[kMaxSplit], pl[kMaxSplit], pa[kMaxSplit];
#pragma unroll
        for (int i = 0; i < kMaxSplit; ++i) {
          const bool ok = i < S;
          pm[i] = ok ? ld_agent(ml + 2 * i) : -INFINITY;
          pl[i] = ok ? ld_agent(ml + 2 * i + 1) : 0.f;
          pa[i] = ok ? ld_agent(a.part_acc + (bh * S + i) * DH + tid) : 0.f;
        }
        M = pm[0];
#pragma unroll
        for (int i = 1; i < kMaxSplit; ++i) M = fmaxf(M, pm[i]);
        l = 0.f;
        acc = 0.f;
#pragma unroll
        for (int i = 0; i < kMaxSplit; ++i) {
          const float wgt = (pm[i] == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(pm[i] - M);
          l += wgt * pl[i];
          acc += wgt * pa[i];
        }
      }
      if (tid == 0) zero_agent(&a.cnt_done[bh * kCnt]);
    }
  }
  // split 0 always holds the current token, so l > 0
  if (finalize && tid < DH) Elem<T>::store(static_cast<T*>(a.o) + bh * DH + tid, acc / l);

  // The block that drew the last ticket of sequence b knows every block of b has read cache_len[b]: it alone
  // appends and advances the length.
  if (S > 1 && sm_commit) {
    if (DEFER) commit_length(a, b, keep_prev);
    else commit_sequence<T, DH>(a, b);
  }
}

template <typename T, int DH, int NW>
__global__ __launch_bounds__(NW * kWave) void decode_attn_kernel(DecodeArgs a) {
  attn_block<T, DH, NW, false>(a, blockIdx.x, blockIdx.y, blockIdx.z);
}

// dllava_decode_step: one launch = the predictor scoring of the current tokens (first n_score blocks, split-K form of
// score_splitk.h; NT = 0: no scoring blocks in this launch) + the deferred-append attention.  The two halves do
// not depend on each other: the logits written here are read by the NEXT launch.
// (Register budget: with at most 96 registers five waves fit a SIMD -- one scoring wave beside the two 8-wave
// attention blocks of a compute unit -- so that the attention half starts at full occupancy; the scoring code for
// up to 32 rows needs 122 registers: four waves.  The code for 64 rows would leave two waves per SIMD, which costs the
// attention half more than reading W1 twice does: 33..64 rows are scored as two groups of blocks.)
template <typename T, int DH, int NW, int NT>
__global__ __launch_bounds__(NW * kWave, NT == 1 ? 5 : (NT == 2 ? 4 : 1)) void decode_step_kernel(DecodeArgs a, ScoreArgs sa, int G, int KS, int ppb,
                                                                   int n_score, size_t ws_group_stride) {
  if constexpr (NT > 0) {
    if (static_cast<int>(blockIdx.x) < n_score) {
      // the scoring code runs on four waves and contains block barriers; the other waves end here (a barrier waits
      // for the surviving waves of a block only)
      if (threadIdx.x >= kSpThreads) return;
      // Rows are scored in groups of 16*NT (more rows per block would cost registers, see above): group gi has its own
      // blocks, its own slice of x and of the logits, and its own workspace region.
      const int per_group = G * KS, gi = static_cast<int>(blockIdx.x) / per_group;
      const int64_t r0 = static_cast<int64_t>(gi) * 16 * NT;
      ScoreArgs sg = sa;
      sg.x = static_cast<const char*>(sa.x) + r0 * sa.ldx * static_cast<int64_t>(sizeof(bf16_t));
      sg.logits = sa.logits + 2 * r0;
      sg.M = sa.M - r0 < 16 * NT ? sa.M - r0 : 16 * NT;
      sg.workspace = static_cast<char*>(sa.workspace) + static_cast<size_t>(gi) * ws_group_stride;
      score_splitk_block<NT>(sg, G, KS, ppb, static_cast<int>(blockIdx.x) % per_group);
      return;
    }
  }
  const int id = static_cast<int>(blockIdx.x) - n_score, S = a.n_split;
  attn_block<T, DH, NW, true>(a, id % S, (id / S) % a.H, id / (S * a.H));
}

// appends the tokens of the last step whose decision is still outstanding (dllava_decode_commit)
template <typename T, int DH>
__global__ __launch_bounds__(256) void decode_commit_kernel(DecodeArgs a) {
  commit_sequence<T, DH>(a, blockIdx.x);
}

struct DecodeShape {
  int nw;       // waves per block: 4 or 8
  int n_split;  // blocks per (sequence, head)
};

// Launch shape from host-known sizes only (cache lengths live on the device).  Measured on MI355X: about
// 16 waves per CU (4096 in all) already saturate the memory pipeline, and a single split per (b, h) wins
// whenever that many waves are available, because every further split adds a round trip through memory
// for the partial results and speculative first-page loads are only used with one split.
DecodeShape pick_shape(int64_t n_bh, int max_pages) {
  DecodeShape sh;
  const int64_t target_waves = 4096;
  sh.nw = n_bh * 8 <= 2 * target_waves ? 8 : 4;
  int64_t S = target_waves / (n_bh * sh.nw);
  if (S > kMaxSplit) S = kMaxSplit;
  const int64_t max_useful = ceil_div(max_pages, sh.nw);
  if (S > max_useful) S = max_useful;
  if (S < 1) S = 1;
  sh.n_split = static_cast<int>(S);
  // shapes forced through dllava_set_launch_override (tests reach every kernel variant that way)
  if (int v = launch_override(DLLAVA_LAUNCH_DECODE_WAVES)) sh.nw = (v == 4 || v == 8) ? v : sh.nw;
  if (int v = launch_override(DLLAVA_LAUNCH_DECODE_SPLITS)) sh.n_split = v > kMaxSplit ? kMaxSplit : v;
  return sh;
}

template <typename T, int DH, int NW>
int launch2(const DecodeArgs& a, hipStream_t st) {
  dim3 grid(a.n_split, a.H, a.B);
  hipLaunchKernelGGL((decode_attn_kernel<T, DH, NW>), grid, dim3(NW * kWave), 0, st, a);
  DLLAVA_CHECK_LAUNCH("decode_attn_kernel");
  return DLLAVA_OK;
}
template <typename T, int DH>
int launch(const DecodeArgs& a, const DecodeShape& sh, hipStream_t st) {
  return sh.nw == 8 ? launch2<T, DH, 8>(a, st) : launch2<T, DH, 4>(a, st);
}

size_t counter_bytes(int64_t B, int64_t H) { return static_cast<size_t>(2 * B * H + B) * kCnt * sizeof(int32_t); }

size_t partial_bytes(int64_t B, int64_t H, int64_t Dh) {
  const size_t n = static_cast<size_t>(B) * H * kMaxSplit;
  return round_up(n * Dh * sizeof(float), 256) + round_up(n * 2 * sizeof(float), 256);
}

// host validation shared by the two entry points; fills `a` and the launch shape
// partial_offset: where the partial results of split launches start in the workspace (0 = right after the counters)
int prepare(const char* who, const void* q, const void* k_new, const void* v_new, int32_t B, const float* logits,
            float threshold, const uint8_t* keep_override, const dllava_kv_cache* cache, float scale, void* o,
            uint8_t* keep_out, int32_t* err_flag, void* workspace, size_t workspace_bytes, size_t need,
            DecodeArgs& a, DecodeShape& sh, size_t partial_offset = 0) {
  DLLAVA_REQUIRE(q && k_new && v_new && o, DLLAVA_ENULL, "%s: q, k_new, v_new and o are required", who);
  DLLAVA_REQUIRE(threshold == threshold, DLLAVA_EINVAL, "%s: threshold is NaN", who);
  DLLAVA_REQUIRE(scale == scale && scale > 0.f && scale < INFINITY, DLLAVA_EINVAL, "%s: bad scale", who);
  DLLAVA_REQUIRE(aligned(q, 16) && aligned(k_new, 16) && aligned(v_new, 16) && aligned(o, 16), DLLAVA_EINVAL,
                 "%s: q, k_new, v_new, o must be 16-byte aligned", who);
  DLLAVA_REQUIRE(B <= 65535 && cache->H <= 65535, DLLAVA_ESHAPE, "%s: B and H must be <= 65535", who);
  DLLAVA_REQUIRE(workspace && aligned(workspace, 256) && workspace_bytes >= need, DLLAVA_EWORKSPACE,
                 "%s: workspace needs %zu bytes, 256-byte aligned (got %zu)", who, need, workspace_bytes);
  a.q = q; a.k_new = k_new; a.v_new = v_new;
  a.logits = logits; a.keep_override = keep_override;
  a.threshold = threshold;
  a.scale_log2 = scale * 1.44269504088896340736f;
  a.pages = cache->pages; a.block_table = cache->block_table; a.cache_len = cache->cache_len;
  a.max_pages = cache->max_pages_per_seq; a.H = cache->H; a.B = B;
  sh = pick_shape(static_cast<int64_t>(B) * cache->H, cache->max_pages_per_seq);
  a.n_split = sh.n_split;
  // partial results are indexed (b*H + h) * n_split + s: a region laid out for kMaxSplit serves every split count
  const size_t n = static_cast<size_t>(B) * cache->H * (partial_offset ? sh.n_split : kMaxSplit);
  char* ws = static_cast<char*>(workspace);
  a.cnt_bh = reinterpret_cast<int32_t*>(ws);
  a.cnt_done = a.cnt_bh + static_cast<size_t>(B) * cache->H * kCnt;
  a.cnt_b = a.cnt_done + static_cast<size_t>(B) * cache->H * kCnt;
  ws += partial_offset ? partial_offset : counter_bytes(B, cache->H);
  a.part_acc = reinterpret_cast<float*>(ws);
  a.part_ml = reinterpret_cast<float*>(ws + round_up(n * cache->Dh * sizeof(float), 256));
  a.o = o; a.keep_out = keep_out; a.err_flag = err_flag;
  return DLLAVA_OK;
}

template <typename T, int DH, int NW, int NT>
int launch_step3(const DecodeArgs& a, const ScoreArgs& sa, const SplitPlan& p, hipStream_t st) {
  const int n_groups = NT > 0 ? static_cast<int>(ceil_div(a.B, 16 * NT)) : 0;  // row groups of the scoring half
  const int n_score = n_groups * p.G * p.KS;
  const int64_t blocks = static_cast<int64_t>(n_score) + static_cast<int64_t>(a.n_split) * a.H * a.B;
  if (blocks > 0x7fffffffLL) DLLAVA_FAIL(DLLAVA_ESHAPE, "decode_step: too many blocks");
  hipLaunchKernelGGL((decode_step_kernel<T, DH, NW, NT>), dim3(static_cast<unsigned>(blocks)), dim3(NW * kWave), 0, st, a,
                     sa, p.G, p.KS, p.ppb, n_score, NT > 0 ? round_up(split_workspace(16 * NT, sa.d, sa.dh), 256) : size_t{0});
  DLLAVA_CHECK_LAUNCH("decode_step_kernel");
  return DLLAVA_OK;
}
template <typename T, int DH, int NW>
int launch_step2(const DecodeArgs& a, const ScoreArgs& sa, const SplitPlan& p, int nt, hipStream_t st) {
  if constexpr (sizeof(T) == 2) {
    if (nt == 1) return launch_step3<T, DH, NW, 1>(a, sa, p, st);
    if (nt == 2) return launch_step3<T, DH, NW, 2>(a, sa, p, st);
  }
  return launch_step3<T, DH, NW, 0>(a, sa, p, st);
}
template <typename T, int DH>
int launch_step(const DecodeArgs& a, const DecodeShape& sh, const ScoreArgs& sa, const SplitPlan& p, int nt,
                hipStream_t st) {
  return sh.nw == 8 ? launch_step2<T, DH, 8>(a, sa, p, nt, st) : launch_step2<T, DH, 4>(a, sa, p, nt, st);
}

// ---- scratch of dllava_decode_attn_append_static ---------------------------------------------------------------
// For callers that cannot bring a workspace (no allocation possible where they run): the counters and the partial
// results of split launches live in this array instead.  Every GPU holds its own copy at its own address until the
// process ends.  In host code the array's NAME is only a stand-in for hipGetSymbolAddress: the kernels get the
// address that call returned for the current device, as they get the workspace pointer in the other entry point.

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices];  // device address of `scratch` per device, resolved at the first call on it

int static_scratch(void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) DLLAVA_FAIL(DLLAVA_ELAUNCH, "decode_static: hipGetDevice: %s", hipGetErrorString(e));
  DLLAVA_REQUIRE(dev >= 0 && dev < kMaxDevices, DLLAVA_ESHAPE, "decode_static: device %d not supported (at most %d)", dev,
                 kMaxDevices);
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !ptr)
      DLLAVA_FAIL(DLLAVA_ELAUNCH, "decode_static: hipGetSymbolAddress on device %d: %s", dev, hipGetErrorString(e));
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return DLLAVA_OK;
}

}  // namespace
}  // namespace dllava

using namespace dllava;

extern "C" size_t dllava_decode_workspace(int32_t B, int32_t H, int32_t Dh, int32_t max_pages_per_seq) {
  if (B <= 0 || H <= 0 || Dh <= 0) return 256;
  (void)max_pages_per_seq;
  return counter_bytes(B, H) + partial_bytes(B, H, Dh);
}

extern "C" int dllava_decode_attn_append(const void* q, const void* k_new, const void* v_new, int32_t B,
                                         const float* logits, float threshold, const uint8_t* keep_override,
                                         const dllava_kv_cache* cache, float scale, void* o, uint8_t* keep_out,
                                         int32_t* err_flag, void* workspace, size_t workspace_bytes,
                                         void* stream) {
  DLLAVA_REQUIRE(B >= 0, DLLAVA_EINVAL, "decode: B = %d < 0", B);
  if (int rc = check_cache(cache, "decode")) return rc;
  if (B == 0) return DLLAVA_OK;
  DLLAVA_REQUIRE(logits || keep_override, DLLAVA_ENULL, "decode: need logits or keep_override");
  DecodeArgs a{};
  DecodeShape sh;
  const size_t need = dllava_decode_workspace(B, cache->H, cache->Dh, cache->max_pages_per_seq);
  if (int rc = prepare("decode", q, k_new, v_new, B, logits, threshold, keep_override, cache, scale, o, keep_out,
                       err_flag, workspace, workspace_bytes, need, a, sh))
    return rc;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const bool bf = cache->dtype == DLLAVA_BF16;
  if (cache->Dh == 128) return bf ? launch<bf16_t, 128>(a, sh, st) : launch<float, 128>(a, sh, st);
  return bf ? launch<bf16_t, 64>(a, sh, st) : launch<float, 64>(a, sh, st);
}

extern "C" int dllava_decode_attn_append_static(const void* q, const void* k_new, const void* v_new, int32_t B,
                                                const float* logits, float threshold, const uint8_t* keep_override,
                                                const dllava_kv_cache* cache, float scale, void* o, uint8_t* keep_out,
                                                int32_t* err_flag, void* stream) {
  DLLAVA_REQUIRE(B >= 0, DLLAVA_EINVAL, "decode_static: B = %d < 0", B);
  if (int rc = check_cache(cache, "decode_static")) return rc;
  if (B == 0) return DLLAVA_OK;
  DLLAVA_REQUIRE(logits || keep_override, DLLAVA_ENULL, "decode_static: need logits or keep_override");
  // sizes first: the array is fixed, so shapes that need more are refused before anything is launched
  const size_t cnt = counter_bytes(B, cache->H);
  DLLAVA_REQUIRE(cnt <= kStaticCounterBytes, DLLAVA_ECAPACITY,
                 "decode_static: 2*B*H + B = %lld counters exceed the %zu the static scratch holds; use "
                 "dllava_decode_attn_append with a workspace",
                 2LL * B * cache->H + B, kStaticCounterBytes / (kCnt * sizeof(int32_t)));
  const DecodeShape want = pick_shape(static_cast<int64_t>(B) * cache->H, cache->max_pages_per_seq);
  const size_t n = static_cast<size_t>(B) * cache->H * want.n_split;
  const size_t part =
      want.n_split > 1 ? round_up(n * cache->Dh * sizeof(float), 256) + round_up(n * 2 * sizeof(float), 256) : 0;
  DLLAVA_REQUIRE(part <= kStaticPartialBytes, DLLAVA_ECAPACITY,
                 "decode_static: %zu bytes of partial results (B*H = %lld, %d splits) exceed the %zu the static scratch "
                 "holds; use dllava_decode_attn_append with a workspace",
                 part, static_cast<long long>(B) * cache->H, want.n_split, kStaticPartialBytes);
  void* ptr = nullptr;
  if (int rc = static_scratch(&ptr)) return rc;
  DecodeArgs a{};
  DecodeShape sh;
  if (int rc = prepare("decode_static", q, k_new, v_new, B, logits, threshold, keep_override, cache, scale, o, keep_out,
                       err_flag, ptr, kStaticScratchBytes, 0, a, sh, kStaticCounterBytes))
    return rc;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const bool bf = cache->dtype == DLLAVA_BF16;
  if (cache->Dh == 128) return bf ? launch<bf16_t, 128>(a, sh, st) : launch<float, 128>(a, sh, st);
  return bf ? launch<bf16_t, 64>(a, sh, st) : launch<float, 64>(a, sh, st);
}

extern "C" size_t dllava_decode_step_workspace(int32_t B, int32_t H, int32_t Dh, int32_t max_pages_per_seq, int64_t d,
                                               int64_t dh, int dtype) {
  // the scoring half may run as two row groups with a workspace region each
  const size_t two_groups = (dtype == DLLAVA_BF16 && d > 0 && dh > 0) ? 2 * round_up(split_workspace(32, d, dh), 256) : 0;
  const size_t score = round_up(dllava_score_workspace(B > 0 ? B : 1, d, dh, dtype), 256);
  return round_up(dllava_decode_workspace(B, H, Dh, max_pages_per_seq), 256) + (score > two_groups ? score : two_groups);
}

extern "C" int dllava_decode_step(const void* x, int64_t ldx, int64_t d, int64_t dh, const void* W1, const float* b1,
                                  const void* W2, const float* b2, const void* q, const void* k_new,
                                  const void* v_new, const void* k_prev, const void* v_prev,
                                  const float* logits_prev, const uint8_t* keep_prev_override, int32_t B,
                                  float threshold, const dllava_kv_cache* cache, float scale, void* o, float* logits,
                                  uint8_t* keep_prev_out, int32_t* err_flag, void* workspace, size_t workspace_bytes,
                                  void* stream) {
  DLLAVA_REQUIRE(B >= 0, DLLAVA_EINVAL, "decode_step: B = %d < 0", B);
  if (int rc = check_cache(cache, "decode_step")) return rc;
  if (B == 0) return DLLAVA_OK;
  // x == NULL: no scoring in this call (the logits of this step's tokens come from elsewhere, e.g. dllava_predict
  // running beside this launch); attention and the deferred append only
  const bool score_here = x != nullptr;
  DLLAVA_REQUIRE(!score_here || (W1 && W2 && logits), DLLAVA_ENULL, "decode_step: W1, W2 and logits go with x");
  const bool have_prev = logits_prev || keep_prev_override;
  DLLAVA_REQUIRE(!have_prev || (k_prev && v_prev), DLLAVA_ENULL,
                 "decode_step: k_prev and v_prev go with logits_prev / keep_prev_override");
  DLLAVA_REQUIRE(aligned(k_prev, 16) && aligned(v_prev, 16), DLLAVA_EINVAL, "decode_step: k_prev, v_prev must be 16-byte aligned");
  DLLAVA_REQUIRE(!score_here || logits_prev != logits, DLLAVA_EINVAL,
                 "decode_step: logits and logits_prev must be different buffers");
  if (!score_here) { d = 0; dh = 0; }
  const int dtype = cache->dtype;
  const size_t need_dec = round_up(dllava_decode_workspace(B, cache->H, cache->Dh, cache->max_pages_per_seq), 256);
  const size_t need_score =
      score_here ? dllava_decode_step_workspace(B, cache->H, cache->Dh, cache->max_pages_per_seq, d, dh, dtype) - need_dec : 0;
  DecodeArgs a{};
  DecodeShape sh;
  if (int rc = prepare("decode_step", q, k_new, v_new, B, nullptr, threshold, nullptr, cache, scale, o, keep_prev_out,
                       err_flag, workspace, workspace_bytes, need_dec + need_score, a, sh))
    return rc;
  a.k_prev = have_prev ? k_prev : nullptr;
  a.v_prev = have_prev ? v_prev : nullptr;
  a.logits_prev = logits_prev;
  a.keep_prev_override = keep_prev_override;
  void* ws_score = static_cast<char*>(workspace) + need_dec;
  hipStream_t st = static_cast<hipStream_t>(stream);

  // the scoring half rides in the same launch when the split-K form covers the shape; otherwise it is a launch of its own
  ScoreArgs sa{x, ldx, B, d, dh, B, nullptr, nullptr, nullptr, W1, b1, W2, b2, logits, ws_score};
  SplitPlan p = split_plan(d > 0 ? d : 64, dh > 0 ? dh : 1);
  int nt = 0;
  const bool bf = dtype == DLLAVA_BF16;
  if (score_here && bf && B <= 64 && d > 0 && d % 64 == 0 && ldx >= d && ldx % 8 == 0 && dh >= 1 && p.G <= kSpMaxGroups && d <= 16384 &&
      aligned(x, 16) && aligned(W1, 16))
    nt = B <= 16 ? 1 : 2;  // up to 64 rows: one or two groups of at most 32
  if (nt > 0) {
    // Inside the attention launch the scoring half is not latency-critical (it only has to finish before the
    // attention does) but every one of its dependent trips to memory queues behind the K/V stream: fewer, longer
    // slices of d (about 128 blocks instead of one per compute unit) were measured faster here.
    const int npairs = static_cast<int>(d / 64);
    int ks = 128 / p.G;
    ks = ks < 1 ? 1 : (ks > kSpMaxSplit ? kSpMaxSplit : ks);
    if (ks < p.KS) {
      p.ppb = (npairs + ks - 1) / ks;
      p.KS = (npairs + p.ppb - 1) / p.ppb;
    }
  }
  if (nt == 0 && score_here) {
    if (int rc = dllava_score(x, ldx, B, 0, nullptr, nullptr, nullptr, d, dh, W1, b1, W2, b2, dtype, logits, ws_score,
                              need_score, stream))
      return rc;
  }
  if (cache->Dh == 128) return bf ? launch_step<bf16_t, 128>(a, sh, sa, p, nt, st) : launch_step<float, 128>(a, sh, sa, p, nt, st);
  return bf ? launch_step<bf16_t, 64>(a, sh, sa, p, nt, st) : launch_step<float, 64>(a, sh, sa, p, nt, st);
}

extern "C" int dllava_decode_commit(const void* k_prev, const void* v_prev, const float* logits_prev,
                                    const uint8_t* keep_prev_override, int32_t B, float threshold,
                                    const dllava_kv_cache* cache, uint8_t* keep_out, int32_t* err_flag, void* stream) {
  DLLAVA_REQUIRE(B >= 0, DLLAVA_EINVAL, "decode_commit: B = %d < 0", B);
  if (int rc = check_cache(cache, "decode_commit")) return rc;
  if (B == 0) return DLLAVA_OK;
  DLLAVA_REQUIRE(k_prev && v_prev && (logits_prev || keep_prev_override), DLLAVA_ENULL,
                 "decode_commit: k_prev, v_prev and logits_prev or keep_prev_override are required");
  DLLAVA_REQUIRE(threshold == threshold, DLLAVA_EINVAL, "decode_commit: threshold is NaN");
  DLLAVA_REQUIRE(aligned(k_prev, 16) && aligned(v_prev, 16), DLLAVA_EINVAL, "decode_commit: k_prev, v_prev must be 16-byte aligned");
  DecodeArgs a{};
  a.k_new = k_prev; a.v_new = v_prev; a.logits = logits_prev; a.keep_override = keep_prev_override;
  a.threshold = threshold;
  a.pages = cache->pages; a.block_table = cache->block_table; a.cache_len = cache->cache_len;
  a.max_pages = cache->max_pages_per_seq; a.H = cache->H; a.B = B;
  a.keep_out = keep_out; a.err_flag = err_flag;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const bool bf = cache->dtype == DLLAVA_BF16;
  const dim3 grid(static_cast<unsigned>(B)), block(256);
  if (cache->Dh == 128) {
    if (bf) hipLaunchKernelGGL((decode_commit_kernel<bf16_t, 128>), grid, block, 0, st, a);
    else hipLaunchKernelGGL((decode_commit_kernel<float, 128>), grid, block, 0, st, a);
  } else {
    if (bf) hipLaunchKernelGGL((decode_commit_kernel<bf16_t, 64>), grid, block, 0, st, a);
    else hipLaunchKernelGGL((decode_commit_kernel<float, 64>), grid, block, 0, st, a);
  }
  DLLAVA_CHECK_LAUNCH("decode_commit_kernel");
  return DLLAVA_OK;
}
