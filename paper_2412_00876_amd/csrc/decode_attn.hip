// dllava_decode_attn_append: one decode step with online KV-cache reduction (Eq. 6 of the paper).
//
// The step is a pure stream over the reduced cache: LLaVA-1.5 is plain multi-head attention, so every
// cached K/V byte is read by exactly one (sequence, head) query and there is one flop per byte.  The
// kernel therefore uses fully coalesced 16-byte loads and VALU arithmetic, not matrix cores.
//
// ONE launch per step.  Grid (n_split, H, B), 256 threads = 4 waves per block.  Block (s, h, b) owns pages
// [s*P/S, (s+1)*P/S) of the P = ceil(cache_len[b]/16) pages of sequence b; its waves take those pages
// round-robin, each wave keeping the next page's 8 KiB of K and V in flight while it works on the current
// one, and are merged through LDS.  Split 0 also folds in the current token (it always takes part in its
// own attention) and, when the token is kept, stores its K/V at position cache_len[b], a slot no block
// reads in this launch.
//
// Cross-block steps use device-scope counters kept at the start of the workspace (zero before the first
// call; each is reset by the block that consumes it):
//   * the last of the S blocks of (b, h) to finish merges the S partial (max, sum, accumulator) triples in
//     split order -- a fixed order, so the result is bit-reproducible -- and writes o[b, h];
//   * the last of the H heads of sequence b to be finalised commits the keep decision: cache_len[b] += 1.
//     Every block of sequence b has read cache_len[b] long before, so the update cannot race with a read.
#include "attend.h"

namespace dllava {
namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / kWave;
constexpr int kMaxSplit = 16;

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
  int32_t* cnt_bh;  // [B*H] splits finished per (b, h)
  int32_t* cnt_b;   // [B]   heads finalised per sequence
  float* part_acc;  // [B*H*S][DH]
  float* part_ml;   // [B*H*S][2]
  void* o;
  uint8_t* keep_out;
  int32_t* err_flag;
};

__device__ __forceinline__ bool decode_keep(const float* logits, const uint8_t* keep_override, float threshold, int b) {
  if (keep_override) return keep_override[b] != 0;
  return keep_from_logits(logits, b, threshold);
}

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

template <typename T, int DH>
__global__ __launch_bounds__(kThreads) void decode_attn_kernel(DecodeArgs a) {
  using C = AttendCfg<T, DH>;
  const int s = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
  const int tid = threadIdx.x, lane = tid & (kWave - 1), w = tid / kWave;
  const int S = a.n_split, H = a.H;
  const int cap = a.max_pages * kPage;
  int L = a.cache_len[b];
  L = L < 0 ? 0 : (L > cap ? cap : L);
  const int P = (L + kPage - 1) / kPage;
  const int p0 = static_cast<int>(static_cast<int64_t>(s) * P / S);
  const int p1 = static_cast<int>(static_cast<int64_t>(s + 1) * P / S);

  const size_t bh = static_cast<size_t>(b) * H + h;
  const T* qrow = static_cast<const T*>(a.q) + bh * DH;
  const T* knew = static_cast<const T*>(a.k_new) + bh * DH;
  const T* vnew = static_cast<const T*>(a.v_new) + bh * DH;
  T* pages = static_cast<T*>(a.pages);
  const int32_t* bt = a.block_table + static_cast<size_t>(b) * a.max_pages;
  const size_t tile = static_cast<size_t>(kPage) * DH;  // elements of one (page, K|V, head) tile
  const size_t vofs = static_cast<size_t>(H) * tile;    // from a K tile to the V tile of the same page/head

  LaneDot<T> qd;
  qd.init(qrow, lane % C::G, a.scale_log2);
  AttnState<C::E> st;
  st.clear();

  // pipeline: the next page's loads are issued before the current page is consumed
  int p = p0 + w;
  PageRegs<T, DH> cur;
  if (p < p1) {
    const T* kt = pages + (static_cast<size_t>(bt[p]) * 2 * H + h) * tile;
    load_page<T, DH>(cur, kt, kt + vofs);
  }
  int pg_next = (p + kWaves < p1) ? bt[p + kWaves] : 0;

  if (s == 0 && w == 0) {  // the current token, folded into lane group 0
    const uint4 kr = *reinterpret_cast<const uint4*>(knew + (lane % C::G) * C::E);
    const uint4 vr = *reinterpret_cast<const uint4*>(vnew + (lane % C::G) * C::E);
    const float d = row_group_sum<C::G>(qd.dot(kr));
    if (lane < C::G) {
      st.m = d;
      st.l = 1.f;
      Elem<T>::unpack(vr, st.acc);
    }
  }

  while (p < p1) {
    const int pn = p + kWaves;
    PageRegs<T, DH> nxt;
    if (pn < p1) {
      const T* kt = pages + (static_cast<size_t>(pg_next) * 2 * H + h) * tile;
      load_page<T, DH>(nxt, kt, kt + vofs);
      if (pn + kWaves < p1) pg_next = bt[pn + kWaves];
    }
    const int nvalid = L - p * kPage;
    if (nvalid >= kPage)
      consume_page<T, DH, false>(cur, kPage, qd, st);
    else
      consume_page<T, DH, true>(cur, nvalid, qd, st);
    if (pn < p1) cur = nxt;
    p = pn;
  }
  merge_groups<T, DH>(st);

  __shared__ float sm_acc[kWaves][DH];
  __shared__ float sm_m[kWaves], sm_l[kWaves];
  __shared__ int sm_flag;
  if (lane < C::G) {
#pragma unroll
    for (int e = 0; e < C::E; ++e) sm_acc[w][lane * C::E + e] = st.acc[e];
    if (lane == 0) {
      sm_m[w] = st.m;
      sm_l[w] = st.l;
    }
  }

  // conditional append: position L is read by nobody in this launch
  if (s == 0 && L < cap && decode_keep(a.logits, a.keep_override, a.threshold, b)) {
    constexpr int kChunks = DH * sizeof(T) / 16;
    if (tid < 2 * kChunks) {
      const int kv = tid / kChunks, cc = tid % kChunks;
      const int pg = bt[L / kPage];
      T* dst = pages + ((static_cast<size_t>(pg) * 2 + kv) * H + h) * tile + static_cast<size_t>(L % kPage) * DH;
      const T* src = kv ? vnew : knew;
      reinterpret_cast<uint4*>(dst)[cc] = reinterpret_cast<const uint4*>(src)[cc];
    }
  }
  __syncthreads();

  float M = -INFINITY, l = 0.f, acc = 0.f;
  if (tid < DH) {
    M = sm_m[0];
#pragma unroll
    for (int i = 1; i < kWaves; ++i) M = fmaxf(M, sm_m[i]);
#pragma unroll
    for (int i = 0; i < kWaves; ++i) {
      const float wgt = (sm_m[i] == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(sm_m[i] - M);
      l += wgt * sm_l[i];
      acc += wgt * sm_acc[i][tid];
    }
  }
  if (S > 1) {
    if (tid < DH) {
      const size_t ps = bh * S + s;
      a.part_acc[ps * DH + tid] = acc;
      if (tid == 0) {
        a.part_ml[2 * ps] = M;
        a.part_ml[2 * ps + 1] = l;
      }
    }
    __threadfence();  // partials visible device-wide before the counter moves
    __syncthreads();
    if (tid == 0) sm_flag = (atomicAdd(&a.cnt_bh[bh], 1) == S - 1);
    __syncthreads();
    if (!sm_flag) return;
    __threadfence();
    if (tid < DH) {
      const float* ml = a.part_ml + 2 * bh * S;
      M = ml[0];
      for (int i = 1; i < S; ++i) M = fmaxf(M, ml[2 * i]);
      l = 0.f;
      acc = 0.f;
      for (int i = 0; i < S; ++i) {
        const float m = ml[2 * i];
        const float wgt = (m == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(m - M);
        l += wgt * ml[2 * i + 1];
        acc += wgt * a.part_acc[(bh * S + i) * DH + tid];
      }
    }
    if (tid == 0) a.cnt_bh[bh] = 0;
  }
  // split 0 always holds the current token, so l > 0
  if (tid < DH) Elem<T>::store(static_cast<T*>(a.o) + bh * DH + tid, acc / l);

  if (tid == 0 && atomicAdd(&a.cnt_b[b], 1) == H - 1) {  // last head of sequence b: commit the decision
    a.cnt_b[b] = 0;
    const bool keep = decode_keep(a.logits, a.keep_override, a.threshold, b);
    if (a.keep_out) a.keep_out[b] = keep ? 1 : 0;
    if (keep) {
      const int Lr = a.cache_len[b];
      if (Lr >= 0 && Lr < cap)
        a.cache_len[b] = Lr + 1;
      else if (a.err_flag)
        *a.err_flag = 1;
    }
  }
}

int pick_splits(int64_t n_bh, int max_pages) {
  static const int forced = [] {
    const char* e = getenv("DLLAVA_DECODE_SPLITS");
    return e ? atoi(e) : 0;
  }();
  int64_t S = forced > 0 ? forced : ceil_div(1536, n_bh);
  if (S > kMaxSplit) S = kMaxSplit;
  if (S > max_pages) S = max_pages;
  if (S < 1) S = 1;
  return static_cast<int>(S);
}

template <typename T, int DH>
int launch(const DecodeArgs& a, hipStream_t st) {
  dim3 grid(a.n_split, a.H, a.B);
  hipLaunchKernelGGL((decode_attn_kernel<T, DH>), grid, dim3(kThreads), 0, st, a);
  DLLAVA_CHECK_LAUNCH("decode_attn_kernel");
  return DLLAVA_OK;
}

size_t counter_bytes(int64_t B, int64_t H) { return round_up(static_cast<size_t>(B * H + B) * sizeof(int32_t), 256); }

}  // namespace
}  // namespace dllava

using namespace dllava;

extern "C" size_t dllava_decode_workspace(int32_t B, int32_t H, int32_t Dh, int32_t max_pages_per_seq) {
  if (B <= 0 || H <= 0 || Dh <= 0) return 256;
  (void)max_pages_per_seq;
  const size_t n = static_cast<size_t>(B) * H * kMaxSplit;
  return counter_bytes(B, H) + round_up(n * Dh * sizeof(float), 256) + round_up(n * 2 * sizeof(float), 256);
}

extern "C" int dllava_decode_attn_append(const void* q, const void* k_new, const void* v_new, int32_t B,
                                         const float* logits, float threshold, const uint8_t* keep_override,
                                         const dllava_kv_cache* cache, float scale, void* o, uint8_t* keep_out,
                                         int32_t* err_flag, void* workspace, size_t workspace_bytes,
                                         void* stream) {
  DLLAVA_REQUIRE(B >= 0, DLLAVA_EINVAL, "decode: B = %d < 0", B);
  if (int rc = check_cache(cache, "decode")) return rc;
  if (B == 0) return DLLAVA_OK;
  DLLAVA_REQUIRE(q && k_new && v_new && o, DLLAVA_ENULL, "decode: q, k_new, v_new and o are required");
  DLLAVA_REQUIRE(logits || keep_override, DLLAVA_ENULL, "decode: need logits or keep_override");
  DLLAVA_REQUIRE(threshold == threshold, DLLAVA_EINVAL, "decode: threshold is NaN");
  DLLAVA_REQUIRE(scale == scale && scale > 0.f && scale < INFINITY, DLLAVA_EINVAL, "decode: bad scale");
  DLLAVA_REQUIRE(aligned(q, 16) && aligned(k_new, 16) && aligned(v_new, 16) && aligned(o, 16), DLLAVA_EINVAL,
                 "decode: q, k_new, v_new, o must be 16-byte aligned");
  DLLAVA_REQUIRE(B <= 65535 && cache->H <= 65535, DLLAVA_ESHAPE, "decode: B and H must be <= 65535");
  const size_t need = dllava_decode_workspace(B, cache->H, cache->Dh, cache->max_pages_per_seq);
  DLLAVA_REQUIRE(workspace && aligned(workspace, 256) && workspace_bytes >= need, DLLAVA_EWORKSPACE,
                 "decode: workspace needs %zu bytes, 256-byte aligned (got %zu)", need, workspace_bytes);

  DecodeArgs a;
  a.q = q; a.k_new = k_new; a.v_new = v_new;
  a.logits = logits; a.keep_override = keep_override;
  a.threshold = threshold;
  a.scale_log2 = scale * 1.44269504088896340736f;
  a.pages = cache->pages; a.block_table = cache->block_table; a.cache_len = cache->cache_len;
  a.max_pages = cache->max_pages_per_seq; a.H = cache->H; a.B = B;
  a.n_split = pick_splits(static_cast<int64_t>(B) * cache->H, cache->max_pages_per_seq);
  const size_t n = static_cast<size_t>(B) * cache->H * kMaxSplit;
  char* ws = static_cast<char*>(workspace);
  a.cnt_bh = reinterpret_cast<int32_t*>(ws);
  a.cnt_b = a.cnt_bh + static_cast<size_t>(B) * cache->H;
  ws += counter_bytes(B, cache->H);
  a.part_acc = reinterpret_cast<float*>(ws);
  a.part_ml = reinterpret_cast<float*>(ws + round_up(n * cache->Dh * sizeof(float), 256));
  a.o = o; a.keep_out = keep_out; a.err_flag = err_flag;

  hipStream_t st = static_cast<hipStream_t>(stream);
  const bool bf = cache->dtype == DLLAVA_BF16;
  if (cache->Dh == 128) return bf ? launch<bf16_t, 128>(a, st) : launch<float, 128>(a, st);
  return bf ? launch<bf16_t, 64>(a, st) : launch<float, 64>(a, st);
}
