// dllava_prefill_attn: causal attention over the reduced prefill set (Eq. 1 of the paper applied to S^{P*}).
//
// Precision-generic path: one wave per (compacted row, head) streams the keys 0..i of its sequence in
// 16-token chunks with the VALU routine of attend.h.  It serves float32 inputs and head sizes the
// matrix-core kernel does not cover.
#include "attend.h"
#include "prefill_args.h"

namespace dllava {

namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / kWave;

template <typename T, int DH>
__global__ __launch_bounds__(kThreads) void prefill_generic_kernel(PrefillArgs a) {
  using C = AttendCfg<T, DH>;
  const int j = blockIdx.x;
  const int lane = threadIdx.x & (kWave - 1), w = threadIdx.x / kWave;
  const int h = blockIdx.y * kWaves + w;
  const int total = a.off[a.B];
  if (j >= total || h >= a.H) return;
  int lo = 0, hi = a.B;
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (a.off[mid] <= j) lo = mid; else hi = mid;
  }
  const int b = lo, r0 = a.off[b], i = j - r0;
  const int H = a.H;
  const T* qrow = static_cast<const T*>(a.Q) + (static_cast<size_t>(j) * H + h) * DH;
  float qs[C::E];
  load_query<T, DH>(qrow, a.scale_log2, qs);
  AttnState<C::E> st;
  st.clear();
  const int nkeys = i + 1;
  const size_t tile = static_cast<size_t>(kPage) * DH;
  for (int c0 = 0; c0 < nkeys; c0 += kPage) {
    const int nvalid = nkeys - c0 < kPage ? nkeys - c0 : kPage;
    const T *kb, *vb;
    size_t stride;
    if (a.K) {
      const size_t o = (static_cast<size_t>(r0 + c0) * H + h) * DH;
      kb = static_cast<const T*>(a.K) + o;
      vb = static_cast<const T*>(a.V) + o;
      stride = static_cast<size_t>(H) * DH;
    } else {
      // clamped to the block table: beyond the capacity (flagged by the call that filled the cache) the reads stay
      // inside allocated pages
      const int pi = c0 / kPage < a.max_pages - 1 ? c0 / kPage : a.max_pages - 1;
      const int pg = a.block_table[static_cast<size_t>(b) * a.max_pages + pi];
      kb = static_cast<const T*>(a.pages) + (static_cast<size_t>(pg) * 2 * H + h) * tile;
      vb = kb + static_cast<size_t>(H) * tile;
      stride = DH;
    }
    if (nvalid == kPage)
      attend_chunk<T, DH, false>(kb, vb, stride, kPage, qs, st);
    else
      attend_chunk<T, DH, true>(kb, vb, stride, nvalid, qs, st);
  }
  merge_groups<T, DH>(st);
  if (lane < C::G) {
    T* orow = static_cast<T*>(a.O) + (static_cast<size_t>(j) * H + h) * DH + lane * C::E;
    const float inv = 1.f / st.l;
#pragma unroll
    for (int e = 0; e < C::E; ++e) Elem<T>::store(orow + e, st.acc[e] * inv);
  }
}

template <typename T, int DH>
int launch_generic(const PrefillArgs& a, int64_t rows, hipStream_t st) {
  dim3 grid(static_cast<unsigned>(rows), static_cast<unsigned>(ceil_div(a.H, kWaves)));
  hipLaunchKernelGGL((prefill_generic_kernel<T, DH>), grid, dim3(kThreads), 0, st, a);
  DLLAVA_CHECK_LAUNCH("prefill_generic_kernel");
  return DLLAVA_OK;
}

// Packs the per-token mask of Eq. 7 into one 32-bit word per key tile: thread = word slot; the words of sequence b
// start at slot off[b] / 32 + b (disjoint for any offsets, since ceil(n / 32) <= (off + n) / 32 - off / 32 + 1).
__global__ __launch_bounds__(256) void key_words_kernel(const uint8_t* __restrict__ keep, const int32_t* __restrict__ off,
                                                        int32_t B, int64_t n_slots, uint32_t* __restrict__ words) {
  const int64_t slot = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
  if (slot >= n_slots) return;
  int lo = 0, hi = B;  // the last sequence whose first slot is <= slot
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if ((off[mid] >> 5) + mid <= slot) lo = mid; else hi = mid;
  }
  const int b = lo, r0 = off[b], n = off[b + 1] - r0;
  const int64_t t = slot - ((r0 >> 5) + b);
  if (t < 0 || 32 * t >= n) return;  // a slot no tile uses
  uint32_t wd = 0;
#pragma unroll 8
  for (int i = 0; i < 32; ++i) {
    const int64_t j = 32 * t + i;
    if (j < n && keep[r0 + j] != 0) wd |= 1u << i;
  }
  words[slot] = wd;
}

}  // namespace

}  // namespace dllava

using namespace dllava;

extern "C" size_t dllava_masked_attn_workspace(int64_t rows, int32_t B) {
  return round_up((static_cast<size_t>(rows > 0 ? rows : 0) / 32 + static_cast<size_t>(B > 0 ? B : 0) + 2) * 4, 256);
}

extern "C" int dllava_masked_attn(const void* Q, const void* K, const void* V, int32_t B, const int32_t* off,
                                  int64_t rows, int32_t H, int32_t Dh, float scale, const uint8_t* keep_mask, void* O,
                                  int dtype, void* workspace, size_t workspace_bytes, void* stream) {
  DLLAVA_REQUIRE(dtype == DLLAVA_BF16, DLLAVA_EDTYPE, "masked_attn: only DLLAVA_BF16 is supported (got dtype %d)", dtype);
  DLLAVA_REQUIRE(B >= 0 && rows >= 0 && rows <= 0x7fffffffLL, DLLAVA_EINVAL, "masked_attn: B = %d, rows = %lld", B,
                 (long long)rows);
  DLLAVA_REQUIRE(Dh == 64 || Dh == 128, DLLAVA_ESHAPE, "masked_attn: Dh must be 64 or 128 (got %d)", Dh);
  DLLAVA_REQUIRE(H > 0 && H <= 65535, DLLAVA_ESHAPE, "masked_attn: bad H = %d", H);
  DLLAVA_REQUIRE(scale == scale && scale > 0.f && scale < INFINITY, DLLAVA_EINVAL, "masked_attn: bad scale");
  if (B == 0 || rows == 0) return DLLAVA_OK;
  DLLAVA_REQUIRE(Q && K && V && O && off && keep_mask, DLLAVA_ENULL, "masked_attn: Q, K, V, O, off and keep_mask are required");
  DLLAVA_REQUIRE(aligned(Q, 16) && aligned(O, 16) && aligned(K, 16) && aligned(V, 16), DLLAVA_EINVAL,
                 "masked_attn: Q, K, V, O must be 16-byte aligned");
  const size_t need = dllava_masked_attn_workspace(rows, B);
  DLLAVA_REQUIRE(workspace && aligned(workspace, 256) && workspace_bytes >= need, DLLAVA_EWORKSPACE,
                 "masked_attn: workspace needs %zu bytes, 256-byte aligned (got %zu)", need, workspace_bytes);
  hipStream_t st = static_cast<hipStream_t>(stream);
  uint32_t* words = static_cast<uint32_t*>(workspace);
  const int64_t n_slots = rows / 32 + B + 1;
  hipLaunchKernelGGL(key_words_kernel, dim3(static_cast<unsigned>(ceil_div(n_slots, 256))), dim3(256), 0, st, keep_mask,
                     off, B, n_slots, words);
  DLLAVA_CHECK_LAUNCH("key_words_kernel");
  PrefillArgs a{};
  a.Q = Q; a.K = K; a.V = V; a.O = O; a.off = off; a.B = B; a.H = H;
  a.scale_log2 = scale * 1.44269504088896340736f;
  a.key_words = words;
  const int rc = prefill_mfma_launch(a, rows, Dh, st);
  if (rc > 0) DLLAVA_FAIL(DLLAVA_ESHAPE, "masked_attn: too many rows or sequences");
  return rc;
}

extern "C" int dllava_prefill_attn(const void* Q, const void* K, const void* V, const dllava_kv_cache* cache,
                                   int32_t B, const int32_t* off, int64_t rows, int32_t H, int32_t Dh,
                                   float scale, void* O, int dtype, void* stream) {
  DLLAVA_REQUIRE(B >= 0 && rows >= 0, DLLAVA_EINVAL, "prefill_attn: B = %d, rows = %lld", B, (long long)rows);
  DLLAVA_REQUIRE(rows <= 0x7fffffffLL, DLLAVA_ESHAPE, "prefill_attn: rows must fit in int32");
  DLLAVA_REQUIRE(dtype == DLLAVA_F32 || dtype == DLLAVA_BF16, DLLAVA_EDTYPE, "prefill_attn: unknown dtype %d", dtype);
  DLLAVA_REQUIRE(Dh == 64 || Dh == 128, DLLAVA_ESHAPE, "prefill_attn: Dh must be 64 or 128 (got %d)", Dh);
  DLLAVA_REQUIRE(H > 0 && H <= 65535 * 4, DLLAVA_ESHAPE, "prefill_attn: bad H = %d", H);
  DLLAVA_REQUIRE(scale == scale && scale > 0.f && scale < INFINITY, DLLAVA_EINVAL, "prefill_attn: bad scale");
  DLLAVA_REQUIRE((K == nullptr) == (V == nullptr), DLLAVA_ENULL, "prefill_attn: K and V go together");
  if (!K) {
    if (int rc = check_cache(cache, "prefill_attn")) return rc;
    DLLAVA_REQUIRE(cache->dtype == dtype && cache->H == H && cache->Dh == Dh, DLLAVA_ESHAPE,
                   "prefill_attn: cache dtype/H/Dh differ from the call's");
  }
  if (B == 0 || rows == 0) return DLLAVA_OK;
  DLLAVA_REQUIRE(Q && O && off, DLLAVA_ENULL, "prefill_attn: Q, O and off are required");
  DLLAVA_REQUIRE(aligned(Q, 16) && aligned(O, 16) && aligned(K, 16) && aligned(V, 16), DLLAVA_EINVAL,
                 "prefill_attn: Q, K, V, O must be 16-byte aligned");

  PrefillArgs a{};
  a.Q = Q; a.K = K; a.V = V; a.O = O; a.off = off; a.B = B; a.H = H;
  a.scale_log2 = scale * 1.44269504088896340736f;
  if (!K) { a.pages = cache->pages; a.block_table = cache->block_table; a.max_pages = cache->max_pages_per_seq; }
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (dtype == DLLAVA_BF16) {
    const int rc = prefill_mfma_launch(a, rows, Dh, st);
    if (rc <= 0) return rc;
    return Dh == 128 ? launch_generic<bf16_t, 128>(a, rows, st) : launch_generic<bf16_t, 64>(a, rows, st);
  }
  return Dh == 128 ? launch_generic<float, 128>(a, rows, st) : launch_generic<float, 64>(a, rows, st);
}
