// dllava_qkv_project: Q, K, V of the REDUCED token set (Eq. 3 line 1 of the paper applied to S^{P*}): the
// projections of the decoder layer run over the kept rows only, which is where the paper's prefill saving comes
// from (Sec. 3.2: most of the cost is in the linear layers; Eq. 13: the 32 B N C^2 term).  Queries and keys are
// rotated by the ORIGINAL position of each kept token (rotary embedding of the LLaMA decoder; the paper does not
// mention positions), queries go to a compacted [rows, H, Dh] tensor, keys and values straight into the paged
// cache, so that compaction has to move hidden states only.
//
//  * qkv_gemm_kernel (bfloat16, Dh = 128): the transposed product W . x^T of gemm_tile.h, one block per
//    (128 features = one head of Q, K or V) x (128 compacted rows).  A wave holds features 32w' + [0,32) and
//    64 + 32w' + [0,32) of the head, i.e. both members of every rotary pair (i, i + 64), for 64 tokens: the
//    rotation happens in registers.  The tile is then transposed through LDS (chunk-swizzled) so that every
//    (token, head) row leaves as 256 contiguous bytes.  XCD-aware block order: an XCD owns a group of feature
//    tiles and walks the token tiles eight at a time, so that its share of W and the x tiles stay in its L2.
//  * qkv_ring_kernel (bfloat16, Dh = 128, many rows): the same on the large-tile product of gemm_ring.h, one block per
//    compute unit: 256 features = two heads of Q, K or V against 128 .. 256 compacted rows; wave w holds, of head
//    w/2, features 32*(w%2) + [0,32) and 64 + 32*(w%2) + [0,32) for all rows of the tile.
//  * qkv_generic_kernel: any dtype / head size, one thread per rotary pair of one row.
#include "dllava.h"
#include "gemm_ring.h"
#include "gemm_tile.h"

namespace dllava {

int check_cache(const dllava_kv_cache* c, const char* who);

namespace {

struct QkvArgs {
  const void* x;
  int64_t ldx, d;
  int32_t B;
  const int32_t* off;
  const int32_t* pos;  // nullptr: no rotation
  const void* W[3];
  int32_t H, Dh;
  void* Q_out;
  void* pages;
  const int32_t* block_table;
  int32_t* cache_len;
  int32_t max_pages;
  int32_t* err_flag;
};

// rotary angle per position of pair i, in revolutions, as float hi + lo (matrix-core kernel) and as a double in
// radians (generic kernel)
struct RopeTable {
  float hi[64], lo[64];
};
struct RopeTableD {
  double f[64];
};

// sequence of compacted row r: largest b with off[b] <= r
__device__ __forceinline__ int seq_of_row(const int32_t* off, int B, int r) {
  int lo = 0, hi = B;
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (off[mid] <= r) lo = mid; else hi = mid;
  }
  return lo;
}

// element offset of (token j of sequence b, head) inside the pages, K block; the V block is H*kPage*Dh further.
// -1 when j is beyond the capacity of the sequence.
__device__ __forceinline__ int64_t page_slot(const QkvArgs& a, int b, int j, int head) {
  if (j >= a.max_pages * kPage) return -1;
  const int pg = a.block_table[static_cast<size_t>(b) * a.max_pages + j / kPage];
  return ((static_cast<int64_t>(pg) * 2 * a.H + head) * kPage + j % kPage) * a.Dh;
}

// cache_len[b] = min(n_b, capacity); the flag reports an overflow
__device__ __forceinline__ void set_lengths(const QkvArgs& a, int tid, int nthreads) {
  const int cap = a.max_pages * kPage;
  for (int b = tid; b < a.B; b += nthreads) {
    const int n = a.off[b + 1] - a.off[b];
    a.cache_len[b] = n < cap ? n : cap;
    if (n > cap && a.err_flag) *a.err_flag = 1;
  }
}

constexpr int kXcds = 8;
constexpr int kTokGroup = 8;  // token tiles an XCD keeps in flight per feature tile group

__global__ __launch_bounds__(kGThreads) __attribute__((amdgpu_waves_per_eu(3, 4))) void qkv_gemm_kernel(
    QkvArgs a, RopeTable rt, int n_ft, int ft_per_xcd) {
  __shared__ __align__(16) bf16_t sAB[2 * kTileElems];  // W tile | x tile, then the transposed output tile
  __shared__ int64_t sm_dst[128];
  bf16_t* sA = sAB;
  bf16_t* sB = sAB + kTileElems;

  const int tid = threadIdx.x, lane = tid & (kWave - 1), w = tid / kWave;
  const int xcd = blockIdx.x % kXcds, jb = blockIdx.x / kXcds;
  const int per_group = ft_per_xcd * kTokGroup;
  const int local = jb % per_group;
  const int ft = xcd * ft_per_xcd + local % ft_per_xcd;          // feature tile (128 features)
  const int tt = (jb / per_group) * kTokGroup + local / ft_per_xcd;  // token tile (128 compacted rows)
  const int total = a.off[a.B];
  const int H = a.H;
  if (ft == H && tt == 0) set_lengths(a, tid, kGThreads);
  if (ft >= n_ft || tt * 128 >= total) return;
  const int which = ft / H, head = ft % H;  // Dh = 128: a feature tile is one head of Q (0), K (1) or V (2)
  const int64_t d = a.d;

  const int lc = tid & 7, lr = tid >> 3;
  const bf16_t* Wm = static_cast<const bf16_t*>(a.W[which]) + static_cast<int64_t>(head) * 128 * d;
  const bf16_t* X = static_cast<const bf16_t*>(a.x);
  const bf16_t *ga[4], *gb[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    ga[j] = Wm + static_cast<int64_t>(lr + 32 * j) * d + lc * 8;
    int r = tt * 128 + lr + 32 * j;
    if (r >= total) r = total - 1;  // such rows are computed and dropped
    gb[j] = X + static_cast<int64_t>(r) * a.ldx + lc * 8;
  }
  const int wf = (w >> 1) * 32, wm = (w & 1) * 64;  // features wf + [0,32) and wf + 64 + [0,32); tokens wm + [0,64)
  f32x16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
  gemm_tile_128x128<64>(ga[0], ga[1], ga[2], ga[3], gb[0], gb[1], gb[2], gb[3], static_cast<int>(d / kBK), sA, sB,
                        wf, wm, acc);

  // where the rows of this tile go (one thread per token)
  if (tid < 128) {
    const int r = tt * 128 + tid;
    int64_t dst = -1;
    if (r < total) {
      if (which == 0) {
        dst = (static_cast<int64_t>(r) * H + head) * 128;
      } else {
        const int b = seq_of_row(a.off, a.B, r);
        dst = page_slot(a, b, r - a.off[b], head);
        if (dst >= 0 && which == 2) dst += static_cast<int64_t>(H) * kPage * 128;
      }
    }
    sm_dst[tid] = dst;
  }

  // lane: token column wm + 32*j + lane%32; register r of fragment i: feature wf + 64*i + 8*(r/4) + 4*(lane/32) + r%4
  const int g = lane >> 5;
  bf16_t* sO = sAB;  // [128 tokens][16 chunks of 8 features], chunk c of token t at chunk position c ^ (t % 16)
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int t = wm + 32 * j + (lane & 31);
    if (which < 2 && a.pos) {
      int r = tt * 128 + t;
      if (r >= total) r = total - 1;
      const float p = static_cast<float>(a.pos[r]);
#pragma unroll
      for (int r16 = 0; r16 < 16; ++r16) {
        const int i = wf + 8 * (r16 >> 2) + 4 * g + (r16 & 3);  // rotary pair (i, i + 64)
        // angle in revolutions, reduced to its fraction without losing the low bits of the product
        const float hi = rt.hi[i];
        const float ph = p * hi;
        const float fr = __builtin_amdgcn_fractf(ph) + (__builtin_fmaf(p, hi, -ph) + p * rt.lo[i]);
        const float sn = __builtin_amdgcn_sinf(fr), cs = __builtin_amdgcn_cosf(fr);
        const float x0 = acc[0][j][r16], x1 = acc[1][j][r16];
        acc[0][j][r16] = x0 * cs - x1 * sn;
        acc[1][j][r16] = x1 * cs + x0 * sn;
      }
    }
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        const int c = (wf + 64 * i) / 8 + q4;  // chunk of features wf + 64*i + 8*q4 + [0,8); this lane's half: g
        uint2 v;
        v.x = pack_bf16x2(acc[i][j][4 * q4], acc[i][j][4 * q4 + 1]);
        v.y = pack_bf16x2(acc[i][j][4 * q4 + 2], acc[i][j][4 * q4 + 3]);
        *reinterpret_cast<uint2*>(sO + t * 128 + ((c ^ (t & 15)) * 8) + g * 4) = v;
      }
  }
  __syncthreads();
  bf16_t* out = static_cast<bf16_t*>(which == 0 ? a.Q_out : a.pages);
#pragma unroll
  for (int k = 0; k < 8; ++k) {
    const int idx = tid + kGThreads * k, t = idx >> 4, c = idx & 15;
    const int64_t dst = sm_dst[t];
    if (dst >= 0)
      *reinterpret_cast<uint4*>(out + dst + c * 8) = *reinterpret_cast<const uint4*>(sO + t * 128 + ((c ^ (t & 15)) * 8));
  }
}

// Large-tile form.  Feature tile f of matrix `which` = heads 2f and 2f+1 (the second may not exist when H is odd:
// its weight rows are clamped and nothing of it is stored).  tok_group: token tiles an XCD keeps in flight per group
// of its feature tiles (ft_per_xcd * tok_group is about the 32 compute units of an XCD).
template <int JB>
__global__ __launch_bounds__(kRingThreads, 1) void qkv_ring_kernel(QkvArgs a, RopeTable rt, int n_ft, int ft_per_xcd,
                                                                   int tok_group) {
  constexpr int kTok = 32 * JB;
  __shared__ __align__(1024) char smem_raw[kRingLdsBytes];
  DLLAVA_LDS char* smem = (DLLAVA_LDS char*)smem_raw;
  const int tid = threadIdx.x, lane = tid & (kWave - 1);
  const int w = __builtin_amdgcn_readfirstlane(tid / kWave);
  const int xcd = blockIdx.x % kXcds, jb = blockIdx.x / kXcds;
  const int per_group = ft_per_xcd * tok_group;
  const int local = jb % per_group;
  const int ft = xcd * ft_per_xcd + local % ft_per_xcd;             // feature tile (256 features)
  const int tt = (jb / per_group) * tok_group + local / ft_per_xcd;  // token tile (kTok compacted rows)
  const int total = a.off[a.B];
  const int H = a.H;
  if (blockIdx.x == 0) set_lengths(a, tid, kRingThreads);
  if (ft >= n_ft || tt * kTok >= total) return;
  const int tiles_per_matrix = (H + 1) / 2;
  const int which = ft / tiles_per_matrix, head0 = 2 * (ft % tiles_per_matrix);
  const int64_t d = a.d;

  uint32_t ga[kRingALoads], gb[JB];
#pragma unroll
  for (int j = 0; j < kRingALoads; ++j) {
    const int row = ring_load_row(w, j, lane);
    int64_t f = static_cast<int64_t>(head0) * 128 + row;
    if (f >= static_cast<int64_t>(H) * 128) f = static_cast<int64_t>(H) * 128 - 1;
    ga[j] = static_cast<uint32_t>(f * d * 2) + ring_load_chunk_bytes(row, lane);
  }
#pragma unroll
  for (int j = 0; j < JB; ++j) {
    const int row = ring_load_row(w, j, lane);
    int r = tt * kTok + row;
    if (r >= total) r = total - 1;  // such rows are computed and dropped
    gb[j] = static_cast<uint32_t>(static_cast<int64_t>(r) * a.ldx * 2) + ring_load_chunk_bytes(row, lane);
  }
  const int hh = w >> 1, sub = w & 1;  // head of the tile, and which 32 of its rotary pairs
  ring_f32x16 acc[2][JB];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < JB; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
  gemm_ring_256<JB, 64, uint32_t>(static_cast<const char*>(a.W[which]), ga, static_cast<const char*>(a.x), gb,
                                  static_cast<int>(d / kRingBK), smem, w, hh * 128 + sub * 32, acc);
  __syncthreads();  // the ring memory becomes the transposed output tile

  // where the rows of this tile go: one entry per (head of the tile, token)
  bf16_t* sO = reinterpret_cast<bf16_t*>(smem_raw);  // [kTok tokens][32 chunks of 8 features], chunk c of token t at c ^ (t % 16)
  int64_t* sm_dst = reinterpret_cast<int64_t*>(smem_raw + kTok * 512);  // [2][kTok]
  for (int e = tid; e < 2 * kTok; e += kRingThreads) {
    const int h2 = e / kTok, t = e % kTok;
    const int r = tt * kTok + t, head = head0 + h2;
    int64_t dst = -1;
    if (r < total && head < H) {
      if (which == 0) {
        dst = (static_cast<int64_t>(r) * H + head) * 128;
      } else {
        const int b = seq_of_row(a.off, a.B, r);
        dst = page_slot(a, b, r - a.off[b], head);
        if (dst >= 0 && which == 2) dst += static_cast<int64_t>(H) * kPage * 128;
      }
    }
    sm_dst[e] = dst;
  }

  // lane: token column 32*j + lane%32; register r of fragment i: feature 128*hh + 32*sub + 64*i + 8*(r/4) + 4*(lane/32) + r%4
  const int g = lane >> 5;
#pragma unroll
  for (int j = 0; j < JB; ++j) {
    const int t = 32 * j + (lane & 31);
    if (which < 2 && a.pos) {
      int r = tt * kTok + t;
      if (r >= total) r = total - 1;
      const float p = static_cast<float>(a.pos[r]);
#pragma unroll
      for (int r16 = 0; r16 < 16; ++r16) {
        const int i = 32 * sub + 8 * (r16 >> 2) + 4 * g + (r16 & 3);  // rotary pair (i, i + 64)
        const float hi = rt.hi[i];
        const float ph = p * hi;
        const float fr = __builtin_amdgcn_fractf(ph) + (__builtin_fmaf(p, hi, -ph) + p * rt.lo[i]);
        const float sn = __builtin_amdgcn_sinf(fr), cs = __builtin_amdgcn_cosf(fr);
        const float x0 = acc[0][j][r16], x1 = acc[1][j][r16];
        acc[0][j][r16] = x0 * cs - x1 * sn;
        acc[1][j][r16] = x1 * cs + x0 * sn;
      }
    }
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        const int c = (128 * hh + 32 * sub + 64 * i) / 8 + q4;  // chunk of 8 features; this lane's half of it: g
        uint2 v;
        v.x = pack_bf16x2(acc[i][j][4 * q4], acc[i][j][4 * q4 + 1]);
        v.y = pack_bf16x2(acc[i][j][4 * q4 + 2], acc[i][j][4 * q4 + 3]);
        *reinterpret_cast<uint2*>(sO + t * 256 + ((c ^ (t & 15)) * 8) + g * 4) = v;
      }
  }
  __syncthreads();
  bf16_t* out = static_cast<bf16_t*>(which == 0 ? a.Q_out : a.pages);
  for (int idx = tid; idx < kTok * 32; idx += kRingThreads) {
    const int t = idx >> 5, c = idx & 31;
    const int64_t dst = sm_dst[(c >> 4) * kTok + t];
    if (dst >= 0)
      *reinterpret_cast<uint4*>(out + dst + (c & 15) * 8) = *reinterpret_cast<const uint4*>(sO + t * 256 + ((c ^ (t & 15)) * 8));
  }
}

// generic path: thread = (compacted row, which of Q/K/V, head, rotary pair i)
template <typename T>
__global__ __launch_bounds__(256) void qkv_generic_kernel(QkvArgs a, RopeTableD rt) {
  const int r = blockIdx.x;
  const int total = a.off[a.B];
  if (r == 0 && blockIdx.y == 0) set_lengths(a, threadIdx.x, blockDim.x);
  if (r >= total) return;
  const int half = a.Dh / 2, H = a.H, Dh = a.Dh;
  const int e = blockIdx.y * blockDim.x + threadIdx.x;  // pair index over 3 * H * half
  if (e >= 3 * H * half) return;
  const int which = e / (H * half), head = (e / half) % H, i = e % half;
  const T* x = static_cast<const T*>(a.x) + static_cast<int64_t>(r) * a.ldx;
  const T* w0 = static_cast<const T*>(a.W[which]) + (static_cast<int64_t>(head) * Dh + i) * a.d;
  const T* w1 = w0 + static_cast<int64_t>(half) * a.d;
  float s0 = 0.f, s1 = 0.f;
  for (int64_t c = 0; c < a.d; ++c) {
    const float xv = Elem<T>::load(x + c);
    s0 = fmaf(xv, Elem<T>::load(w0 + c), s0);
    s1 = fmaf(xv, Elem<T>::load(w1 + c), s1);
  }
  if (which < 2 && a.pos) {
    const double ang = static_cast<double>(a.pos[r]) * rt.f[i];
    const float cs = static_cast<float>(cos(ang)), sn = static_cast<float>(sin(ang));
    const float y0 = s0 * cs - s1 * sn, y1 = s1 * cs + s0 * sn;
    s0 = y0;
    s1 = y1;
  }
  T* out;
  if (which == 0) {
    out = static_cast<T*>(a.Q_out) + (static_cast<int64_t>(r) * H + head) * Dh;
  } else {
    const int b = seq_of_row(a.off, a.B, r);
    int64_t dst = page_slot(a, b, r - a.off[b], head);
    if (dst < 0) return;
    if (which == 2) dst += static_cast<int64_t>(H) * kPage * Dh;
    out = static_cast<T*>(a.pages) + dst;
  }
  Elem<T>::store(out + i, s0);
  Elem<T>::store(out + i + half, s1);
}

template <typename T>
int launch_generic(const QkvArgs& a, int64_t rows, double base, hipStream_t st) {
  RopeTableD rt{};
  for (int i = 0; i < a.Dh / 2; ++i) rt.f[i] = base > 0 ? pow(base, -2.0 * i / a.Dh) : 0.0;
  const int pairs = 3 * a.H * (a.Dh / 2);
  dim3 grid(static_cast<unsigned>(rows), static_cast<unsigned>(ceil_div(pairs, 256)));
  hipLaunchKernelGGL(qkv_generic_kernel<T>, grid, dim3(256), 0, st, a, rt);
  DLLAVA_CHECK_LAUNCH("qkv_generic_kernel");
  return DLLAVA_OK;
}

// returns 1 if the shape is not handled by the matrix-core kernel
int launch_mfma(const QkvArgs& a, int64_t rows, double base, hipStream_t st) {
  if (a.Dh != 128 || a.d % 64 != 0 || a.ldx % 8 != 0) return 1;
  RopeTable rt{};
  const double two_pi = 6.283185307179586476925287;
  for (int i = 0; i < 64; ++i) {
    const double rev = base > 0 ? pow(base, -2.0 * i / 128.0) / two_pi : 0.0;
    rt.hi[i] = static_cast<float>(rev);
    rt.lo[i] = static_cast<float>(rev - static_cast<double>(rt.hi[i]));
  }
  // Many rows: the large-tile kernel (one block per compute unit), with the token-tile width that fills the XCDs'
  // 32 compute units most evenly; DLLAVA_LAUNCH_QKV_TILE forces a width (4..8) or the 128 x 128 kernel (1).
  {
    const int n_ft2 = 3 * ((a.H + 1) / 2);
    const int fpx = static_cast<int>(ceil_div(n_ft2, kXcds));
    int best = 0;
    int64_t best_cost = 0;
    for (int jb = 8; jb >= 4; --jb) {
      const int64_t per_xcd = ceil_div(rows, 32 * jb) * fpx;
      if (per_xcd < 24) continue;  // most of the chip would idle
      const int64_t cost = ceil_div(per_xcd, 32) * (256 * jb + 500);
      if (!best || cost < best_cost) best = jb, best_cost = cost;
    }
    const int forced = launch_override(DLLAVA_LAUNCH_QKV_TILE);
    if (forced == 1) best = 0;
    if (forced >= 4 && forced <= 8) best = forced;
    const bool fits = static_cast<int64_t>(a.H) * 128 * a.d * 2 < (int64_t{1} << 32) && rows * a.ldx * 2 < (int64_t{1} << 32);
    if (best && fits) {
      const int tok_group = fpx >= 32 ? 1 : 32 / fpx;
      const int64_t n_tt2 = ceil_div(rows, 32 * best);
      const int64_t blocks2 = ceil_div(n_tt2, tok_group) * tok_group * fpx * kXcds;
      if (blocks2 <= 0x7fffffffLL) {
        const dim3 grid(static_cast<unsigned>(blocks2)), block(kRingThreads);
        switch (best) {
          case 4: hipLaunchKernelGGL(qkv_ring_kernel<4>, grid, block, 0, st, a, rt, n_ft2, fpx, tok_group); break;
          case 5: hipLaunchKernelGGL(qkv_ring_kernel<5>, grid, block, 0, st, a, rt, n_ft2, fpx, tok_group); break;
          case 6: hipLaunchKernelGGL(qkv_ring_kernel<6>, grid, block, 0, st, a, rt, n_ft2, fpx, tok_group); break;
          case 7: hipLaunchKernelGGL(qkv_ring_kernel<7>, grid, block, 0, st, a, rt, n_ft2, fpx, tok_group); break;
          default: hipLaunchKernelGGL(qkv_ring_kernel<8>, grid, block, 0, st, a, rt, n_ft2, fpx, tok_group); break;
        }
        DLLAVA_CHECK_LAUNCH("qkv_ring_kernel");
        return DLLAVA_OK;
      }
    }
  }
  const int n_ft = 3 * a.H;
  const int ft_per_xcd = static_cast<int>(ceil_div(n_ft, kXcds));
  const int64_t n_tt = ceil_div(rows, 128);
  const int64_t blocks = ceil_div(n_tt, kTokGroup) * kTokGroup * ft_per_xcd * kXcds;
  if (blocks > 0x7fffffffLL) return 1;
  hipLaunchKernelGGL(qkv_gemm_kernel, dim3(static_cast<unsigned>(blocks)), dim3(kGThreads), 0, st, a, rt, n_ft,
                     ft_per_xcd);
  DLLAVA_CHECK_LAUNCH("qkv_gemm_kernel");
  return DLLAVA_OK;
}

}  // namespace

}  // namespace dllava

using namespace dllava;

extern "C" int dllava_qkv_project(const void* x, int64_t ldx, int64_t rows, int64_t d,
                                  int32_t B, const int32_t* off, const int32_t* pos,
                                  const void* Wq, const void* Wk, const void* Wv, float rope_base,
                                  void* Q_out, const dllava_kv_cache* cache, int32_t* err_flag,
                                  int dtype, void* stream) {
  DLLAVA_REQUIRE(B >= 0 && rows >= 0, DLLAVA_EINVAL, "qkv_project: B = %d, rows = %lld", B, (long long)rows);
  DLLAVA_REQUIRE(rows <= 0x7fffffffLL, DLLAVA_ESHAPE, "qkv_project: rows must fit in int32");
  DLLAVA_REQUIRE(dtype == DLLAVA_F32 || dtype == DLLAVA_BF16, DLLAVA_EDTYPE, "qkv_project: unknown dtype %d", dtype);
  if (int rc = check_cache(cache, "qkv_project")) return rc;
  DLLAVA_REQUIRE(cache->dtype == dtype, DLLAVA_EDTYPE, "qkv_project: cache dtype differs from the call's");
  DLLAVA_REQUIRE(d > 0 && ldx >= d, DLLAVA_EINVAL, "qkv_project: d = %lld, ldx = %lld", (long long)d, (long long)ldx);
  const int64_t esz = dtype == DLLAVA_BF16 ? 2 : 4;
  DLLAVA_REQUIRE((d * esz) % 16 == 0 && (ldx * esz) % 16 == 0, DLLAVA_ESHAPE,
                 "qkv_project: rows of x and of the weights must be multiples of 16 bytes");
  DLLAVA_REQUIRE(rope_base == rope_base && rope_base < INFINITY, DLLAVA_EINVAL, "qkv_project: bad rope_base");
  if (B == 0 || rows == 0) return DLLAVA_OK;
  DLLAVA_REQUIRE(x && off && Wq && Wk && Wv && Q_out, DLLAVA_ENULL, "qkv_project: x, off, Wq, Wk, Wv and Q_out are required");
  DLLAVA_REQUIRE(rope_base <= 0.f || pos, DLLAVA_ENULL, "qkv_project: pos is required when rope_base > 0");
  DLLAVA_REQUIRE(aligned(x, 16) && aligned(Wq, 16) && aligned(Wk, 16) && aligned(Wv, 16) && aligned(Q_out, 16),
                 DLLAVA_EINVAL, "qkv_project: x, Wq, Wk, Wv, Q_out must be 16-byte aligned");

  QkvArgs a{};
  a.x = x; a.ldx = ldx; a.d = d; a.B = B; a.off = off; a.pos = rope_base > 0.f ? pos : nullptr;
  a.W[0] = Wq; a.W[1] = Wk; a.W[2] = Wv;
  a.H = cache->H; a.Dh = cache->Dh; a.Q_out = Q_out;
  a.pages = cache->pages; a.block_table = cache->block_table; a.cache_len = cache->cache_len;
  a.max_pages = cache->max_pages_per_seq; a.err_flag = err_flag;
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (dtype == DLLAVA_BF16) {
    const int rc = launch_mfma(a, rows, rope_base, st);
    if (rc <= 0) return rc;
    return launch_generic<bf16_t>(a, rows, rope_base, st);
  }
  return launch_generic<float>(a, rows, rope_base, st);
}
