// dllava_decode_attn_append: one decode step with online KV-cache reduction (Eq. 6 of the paper).
//
// The step is a pure stream over the reduced cache: LLaVA-1.5 is plain multi-head attention, so every
// cached K/V byte is read by exactly one (sequence, head) query and there is one flop per byte.  The
// kernel therefore uses coalesced 16-byte loads and VALU arithmetic (see attend.h), not matrix cores.
//
// Launch shape.  Grid (n_split, H, B), 256 threads = 4 waves per block.  Block (s, h, b) owns pages
// [s*P/S, (s+1)*P/S) of the P = ceil(cache_len[b]/16) pages of sequence b; its waves take those pages
// round-robin and are merged through LDS.  Split 0 also folds in the current token (it always takes
// part in its own attention) and, when the token is kept, stores its K/V at position cache_len[b]
// (a slot no block reads).  cache_len itself is only advanced by the second kernel, after every block
// of the first has read it.  The second kernel also merges the S partial results per (b, h) in a fixed
// order, so results are bit-reproducible.
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
  float* part_acc;  // [B*H*S][DH]
  float* part_ml;   // [B*H*S][2]
  void* o;
  uint8_t* keep_out;
  int32_t* err_flag;
};

__device__ __forceinline__ bool decode_keep(const DecodeArgs& a, int b) {
  if (a.keep_override) return a.keep_override[b] != 0;
  return keep_from_logits(a.logits, b, a.threshold);
}

template <typename T, int DH>
__global__ __launch_bounds__(kThreads) void decode_split_kernel(DecodeArgs a) {
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

  float qs[C::E];
  load_query<T, DH>(qrow, a.scale_log2, qs);
  AttnState<C::E> st;
  st.clear();

  if (s == 0 && w == 0) attend_single<T, DH>(knew, vnew, qs, st);

  for (int p = p0 + w; p < p1; p += kWaves) {
    const int pg = bt[p];
    const T* kt = pages + (static_cast<size_t>(pg) * 2 * H + h) * tile;
    const T* vt = kt + static_cast<size_t>(H) * tile;
    const int nvalid = L - p * kPage;
    if (nvalid >= kPage)
      attend_chunk<T, DH, false>(kt, vt, DH, kPage, qs, st);
    else
      attend_chunk<T, DH, true>(kt, vt, DH, nvalid, qs, st);
  }
  merge_groups<T, DH>(st);

  __shared__ float sm_acc[kWaves][DH];
  __shared__ float sm_m[kWaves], sm_l[kWaves];
  if (lane < C::G) {
#pragma unroll
    for (int e = 0; e < C::E; ++e) sm_acc[w][lane * C::E + e] = st.acc[e];
    if (lane == 0) {
      sm_m[w] = st.m;
      sm_l[w] = st.l;
    }
  }
  __syncthreads();
  if (tid < DH) {
    float M = sm_m[0];
#pragma unroll
    for (int i = 1; i < kWaves; ++i) M = fmaxf(M, sm_m[i]);
    float l = 0.f, acc = 0.f;
#pragma unroll
    for (int i = 0; i < kWaves; ++i) {
      const float wgt = (sm_m[i] == -INFINITY) ? 0.f : exp2f(sm_m[i] - M);
      l += wgt * sm_l[i];
      acc += wgt * sm_acc[i][tid];
    }
    if (S == 1) {
      Elem<T>::store(static_cast<T*>(a.o) + bh * DH + tid, acc / l);  // split 0 holds the current token: l > 0
    } else {
      const size_t ps = bh * S + s;
      a.part_acc[ps * DH + tid] = acc;
      if (tid == 0) {
        a.part_ml[2 * ps] = M;
        a.part_ml[2 * ps + 1] = l;
      }
    }
  }

  // conditional append: position L is read by nobody in this launch
  if (s == 0 && L < cap && decode_keep(a, b)) {
    constexpr int kChunks = DH * sizeof(T) / 16;
    if (tid < 2 * kChunks) {
      const int kv = tid / kChunks, cc = tid % kChunks;
      const int pg = bt[L / kPage];
      T* dst = pages + ((static_cast<size_t>(pg) * 2 + kv) * H + h) * tile + static_cast<size_t>(L % kPage) * DH;
      const T* src = kv ? vnew : knew;
      reinterpret_cast<uint4*>(dst)[cc] = reinterpret_cast<const uint4*>(src)[cc];
    }
  }
}

// Merges the split partials of (b, h) in split order and commits the keep decision of sequence b.
template <typename T, int DH>
__global__ __launch_bounds__(DH) void decode_reduce_kernel(DecodeArgs a) {
  const int h = blockIdx.x, b = blockIdx.y, tid = threadIdx.x;
  const int S = a.n_split;
  const size_t bh = static_cast<size_t>(b) * a.H + h;
  if (S > 1) {
    const float* ml = a.part_ml + 2 * bh * S;
    float M = ml[0];
    for (int s = 1; s < S; ++s) M = fmaxf(M, ml[2 * s]);
    float l = 0.f, acc = 0.f;
    for (int s = 0; s < S; ++s) {
      const float m = ml[2 * s];
      const float wgt = (m == -INFINITY) ? 0.f : exp2f(m - M);
      l += wgt * ml[2 * s + 1];
      acc += wgt * a.part_acc[(bh * S + s) * DH + tid];
    }
    Elem<T>::store(static_cast<T*>(a.o) + bh * DH + tid, acc / l);
  }
  if (h == 0 && tid == 0) {
    const bool keep = decode_keep(a, b);
    if (a.keep_out) a.keep_out[b] = keep ? 1 : 0;
    if (keep) {
      const int cap = a.max_pages * kPage;
      const int L = a.cache_len[b];
      if (L >= 0 && L < cap)
        a.cache_len[b] = L + 1;
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
  hipLaunchKernelGGL((decode_split_kernel<T, DH>), grid, dim3(kThreads), 0, st, a);
  DLLAVA_CHECK_LAUNCH("decode_split_kernel");
  hipLaunchKernelGGL((decode_reduce_kernel<T, DH>), dim3(a.H, a.B), dim3(DH), 0, st, a);
  DLLAVA_CHECK_LAUNCH("decode_reduce_kernel");
  return DLLAVA_OK;
}

}  // namespace
}  // namespace dllava

using namespace dllava;

extern "C" size_t dllava_decode_workspace(int32_t B, int32_t H, int32_t Dh, int32_t max_pages_per_seq) {
  if (B <= 0 || H <= 0 || Dh <= 0) return 256;
  (void)max_pages_per_seq;
  const size_t n = static_cast<size_t>(B) * H * kMaxSplit;
  return round_up(n * Dh * sizeof(float), 256) + round_up(n * 2 * sizeof(float), 256);
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
  a.part_acc = static_cast<float*>(workspace);
  a.part_ml = reinterpret_cast<float*>(static_cast<char*>(workspace) + round_up(n * cache->Dh * sizeof(float), 256));
  a.o = o; a.keep_out = keep_out; a.err_flag = err_flag;

  hipStream_t st = static_cast<hipStream_t>(stream);
  const bool bf = cache->dtype == DLLAVA_BF16;
  if (cache->Dh == 128) return bf ? launch<bf16_t, 128>(a, st) : launch<float, 128>(a, st);
  return bf ? launch<bf16_t, 64>(a, st) : launch<float, 64>(a, st);
}
