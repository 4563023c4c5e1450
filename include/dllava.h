/*
 * dllava — token sparsification followed by attention over the reduced context
 * (Dynamic-LLaVA, arXiv 2412.00876), as a C-ABI library for one AMD MI355X (gfx950).
 *
 * The entry points are the steps of the paper's sparsification inference
 * (Sec. 3.3.2; batch-parallel form in Appendix A.1):
 *   dllava_score               predictor logits D = P(S_l)                 (Eq. 5 line 1, Eq. 11 line 1)
 *   dllava_select_compact      keep decisions + reduced token set / cache  (Eq. 5 lines 2-3, Eq. 11 lines 2-3)
 *   dllava_prefill_attn        Attention over the reduced prefill set      (Eq. 1 with S^{P*}, Sec. 3.3.2)
 *   dllava_decode_attn_append  decode step with online KV-cache reduction  (Eq. 6)
 *   dllava_decode_step         the same step, scoring + attention in one launch, append deferred by one step
 *   dllava_qkv_project         Q, K, V of the reduced set, K/V into the cache (Eq. 3 line 1 with S^{P*})
 *   dllava_predict             predictor logits with the predictors of Appendix A.4.1 (in place of dllava_score)
 *   dllava_masked_attn         attention of the training form, mask inside the softmax (Eq. 7)
 *   dllava_compact             compaction of another layer's tensors with decisions already taken (Sec. 3.3)
 *
 * General conventions
 *   - Every pointer is a DEVICE pointer unless its comment says "host".  The caller
 *     allocates and frees every buffer; the library allocates nothing.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  All work is
 *     enqueued asynchronously on it; no entry point synchronises with the host, so the
 *     calls may be recorded into a HIP graph.
 *   - Floating tensors are stored in `dtype` (DLLAVA_F32 or DLLAVA_BF16), row-major, with
 *     the last index contiguous.  All accumulation is in float32.  Logits are float32.
 *   - Token layout of a batch: sequences are concatenated ("ragged"); sequence b owns rows
 *     [seq_off[b], seq_off[b+1]) and, inside them, one vision span
 *     [vis_start[b], vis_start[b] + vis_len[b]) in sequence-relative positions.  All other
 *     rows are text and are always kept in prefill (Fig. 2 of the paper).
 *   - Return value: DLLAVA_OK (0) or a negative dllava_status.  Argument errors are found on
 *     the host before anything is launched; dllava_last_error() then holds a message.
 *     Outputs are fully overwritten; inputs are never modified, except the KV cache
 *     (pages at newly written slots, cache_len).
 *   - Workspaces: the *_workspace() queries are pure host functions; the caller passes a
 *     device buffer of at least that many bytes, 256-byte aligned.  A workspace must be
 *     ZERO-FILLED once before its first use: it starts with device-scope counters that the
 *     kernels count up and return to zero before the call's work completes.  The same buffer
 *     may then be reused by later calls of the SAME entry point with the same sizes, ordered
 *     on one stream; it must not be shared with another entry point or written by the caller.
 */
#ifndef DLLAVA_H
#define DLLAVA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { DLLAVA_F32 = 0, DLLAVA_BF16 = 1 } dllava_dtype;

typedef enum {
  DLLAVA_OK = 0,
  DLLAVA_EINVAL = -1,     /* a scalar argument is out of range                     */
  DLLAVA_ENULL = -2,      /* a required pointer is NULL                            */
  DLLAVA_ESHAPE = -3,     /* a size is unsupported (see each call)                 */
  DLLAVA_EDTYPE = -4,     /* unknown dtype, or cache dtype differs from the call's */
  DLLAVA_ECAPACITY = -5,  /* a host-visible capacity is too small                  */
  DLLAVA_EWORKSPACE = -6, /* workspace missing, misaligned or too small            */
  DLLAVA_ELAUNCH = -7     /* the HIP runtime refused a launch                      */
} dllava_status;

typedef enum { DLLAVA_MODE_TOPK = 0, DLLAVA_MODE_THRESHOLD = 1, DLLAVA_MODE_THRESHOLD_KEEP_LAST = 2 } dllava_mode;

/*
 * Paged KV cache of ONE decoder layer; caller-owned (the per-sample caches {S^K(b), S^V(b)} of
 * Appendix A.1, stored ragged in pages instead of left-padded to a batch tensor).
 *   pages        [n_pages][2 (0 = K, 1 = V)][H][page_size][Dh], dtype
 *   block_table  [B][max_pages_per_seq] page ids; token t of sequence b lives in page
 *                block_table[b][t / page_size], slot t % page_size.  Every entry must be a
 *                valid page id in [0, n_pages) (capacity is pre-assigned by the caller).
 *   cache_len    [B] tokens currently cached per sequence; device-resident, read and
 *                written by the library.
 * page_size must be 16; Dh must be 64 or 128.  The struct itself lives in host memory.
 */
typedef struct dllava_kv_cache {
  void* pages;
  int32_t* block_table;
  int32_t* cache_len;
  int32_t n_pages;
  int32_t max_pages_per_seq;
  int32_t page_size;
  int32_t H;
  int32_t Dh;
  int32_t dtype; /* dllava_dtype */
} dllava_kv_cache;

/* Library version (major*10000 + minor*100 + patch).  Host, pure. */
int dllava_version(void);

/* Message of the last failing call made by this host thread ("" if none).  Host string
 * owned by the library, valid until the thread's next failing call. */
const char* dllava_last_error(void);

/*
 * Launch shapes.  The library picks the launch shape of its kernels from the problem size alone; results do not depend
 * on the shape (attention outputs agree to rounding, integer outputs exactly).  This call forces one of them for
 * the whole process, so that a test can run every kernel variant on one input; value 0 restores the automatic
 * choice, values a knob does not support are ignored.  Host, no GPU work; not meant for production callers.
 *   DLLAVA_LAUNCH_DECODE_WAVES   waves per block of the decode-attention kernels: 4 or 8
 *   DLLAVA_LAUNCH_DECODE_SPLITS  blocks per (sequence, head) of the decode-attention kernels: 1 .. 16
 *   DLLAVA_LAUNCH_PREFILL_WAVES  waves (of 32 queries each) per block of the matrix-core attention kernel: 1, 2 or 4
 *   DLLAVA_LAUNCH_PREFILL_BLOCKS blocks of the matrix-core attention kernel's launch (its blocks are persistent and
 *                                share the work items; by default as many as the chip holds at once): 1 .. 65535
 *   DLLAVA_LAUNCH_SCORE_TILE     tile of the many-rows scoring kernel: 1 = 128 units x 128 tokens, three blocks per
 *                                compute unit; 4 .. 8 = 256 units x 32*value tokens, one block per compute unit
 *   DLLAVA_LAUNCH_QKV_TILE       the same for the projection kernel of dllava_qkv_project
 *   DLLAVA_LAUNCH_SELECT_LAUNCHES 1 = dllava_select_compact in top-k mode as one launch (selection and copies side by
 *                                side; what it picks for up to 256 sequences), 2 = selection, then the copies,
 *                                3 = one launch in which the selection blocks stand back, so that a copying block
 *                                whose patience runs out (milliseconds) selects instead: the hand-off's fallback
 * The library reads no environment variables.
 */
typedef enum {
  DLLAVA_LAUNCH_DECODE_WAVES = 0,
  DLLAVA_LAUNCH_DECODE_SPLITS = 1,
  DLLAVA_LAUNCH_PREFILL_WAVES = 2,
  DLLAVA_LAUNCH_SCORE_TILE = 3,
  DLLAVA_LAUNCH_QKV_TILE = 4,
  DLLAVA_LAUNCH_PREFILL_BLOCKS = 5,
  DLLAVA_LAUNCH_SELECT_LAUNCHES = 6,
  DLLAVA_LAUNCH_KNOBS = 7
} dllava_launch_knob;
int dllava_set_launch_override(int knob, int value);

/*
 * Predictor scoring, D = P(S_l) (Eq. 5 line 1; Eq. 11 line 1), with the two-layer predictor
 *     h = GELU(x W1^T + b1)   (exact erf GELU),     D = h W2^T + b2,
 * one row per token, rows independent.  Column 0 of D is the "drop" logit, column 1 the "keep"
 * logit (a token is kept when the second value exceeds the first).
 *
 *   x        [*, d] dtype, row stride ldx elements (ldx >= d)
 *   M        number of rows scored = rows of `logits`
 *   B, seq_off [B+1], vis_start [B], vis_len [B]
 *            if seq_off is NULL, rows 0..M-1 of x are scored (decode: one row per sequence,
 *            B/vis_* ignored).  Otherwise the vision spans are scored: logits row
 *            sum_{b'<b} vis_len[b'] + i  <-  x row seq_off[b] + vis_start[b] + i,  i < vis_len[b];
 *            M must equal sum_b vis_len[b] (rows beyond that sum are left untouched).
 *   W1 [dh, d] dtype, W2 [2, dh] dtype;  b1 [dh], b2 [2] float32, either may be NULL (= 0)
 *   logits   [M, 2] float32, out
 * Sizes: d % 8 == 0, 1 <= dh, M >= 0 (M == 0 is a no-op).
 * dllava_score_workspace is non-decreasing in M: a workspace sized for the largest row count
 * serves every smaller one (same d, dh, dtype).
 */
int dllava_score(const void* x, int64_t ldx, int64_t M,
                 int32_t B, const int32_t* seq_off, const int32_t* vis_start, const int32_t* vis_len,
                 int64_t d, int64_t dh,
                 const void* W1, const float* b1, const void* W2, const float* b2,
                 int dtype, float* logits,
                 void* workspace, size_t workspace_bytes, void* stream);
size_t dllava_score_workspace(int64_t M, int64_t d, int64_t dh, int dtype);

/*
 * Keep decisions and order-preserving stream compaction (Eq. 5 lines 2-3; Eq. 11 lines 2-3).
 *
 * Decisions, per sequence b over its vision span (n = vis_len[b]):
 *   DLLAVA_MODE_TOPK       keep the k = floor(keep_ratio * n) rows (float64 product) with the largest
 *                          logits[:,1]; ties go to the lower index; NaN ranks below every
 *                          number; -0 equals +0.
 *   DLLAVA_MODE_THRESHOLD  keep row i iff logits[i,1] - logits[i,0] > threshold (float32,
 *                          strict; threshold 0 is the argmax rule of Eq. 5).
 *   DLLAVA_MODE_THRESHOLD_KEEP_LAST
 *                          the same, and the last row of the span is kept whatever its logits: decoding
 *                          WITHOUT KV cache (Sec. 3.3.2; Eq. 12), where the span is the output text S^OT
 *                          appended to the already reduced prompt, the mask entry of the last output token
 *                          is set to 1 because that token generates the next one, and dllava_prefill_attn
 *                          then runs over S^{P*} u S^{OT*}.
 * Text rows are always kept.  Kept rows keep their original relative order, which is what
 * makes causal attention over the reduced set equal the masked attention of Eq. 7.
 *
 *   logits     [sum_b vis_len[b], 2] float32, vision rows of all sequences back to back
 *   sumN       total rows = seq_off[B] (host copy of that value)
 *   hidden     [sumN, d] dtype -> hidden_out [sum N*, d]      (both NULL to skip)
 *   Q          [sumN, H*Dh] dtype -> Q_out [sum N*, H*Dh]     (both NULL to skip; H, Dh from `cache`,
 *              which is then required)
 *   K, V       [sumN, H, Dh] dtype -> written through cache->block_table into cache->pages at
 *              positions 0..N*(b)-1, and cache->cache_len[b] = N*(b)   (K, V, cache all NULL to skip)
 *   keep_mask  [sumN] uint8, out
 *   kept_idx   [sumN] capacity, out: sequence-relative original positions of the kept rows,
 *              ascending within each sequence, packed by out_off
 *   out_off    [B+1] out: offsets of each sequence in the compacted row order; out_off[B] = sum N*
 *   err_flag   device int32, may be NULL: set to 1 if some N*(b) exceeds the cache capacity
 *              max_pages_per_seq * page_size; the rows beyond capacity are then not written
 *              and cache_len[b] is clamped to the capacity.  Never cleared by the library.
 *              (2 if a copying block gave up waiting for its sequence's selection, which no dispatch order
 *              should produce: that row is then not written)
 *   workspace  device memory, 256-byte aligned, at least dllava_select_compact_workspace(B, sumN) bytes,
 *              zero-filled once by the caller before its first use: the library keeps hand-off words in it
 *              (at fixed offsets from its start) and leaves them zero at the end of every call, so one buffer
 *              sized for the largest (B, sumN) serves calls of smaller shapes too.  Calls that share a workspace
 *              must not overlap.
 * Output buffers hidden_out / Q_out need capacity for sum N* rows (sumN always suffices).
 * Errors: keep_ratio outside [0,1] or NaN, NaN threshold, d*sizeof(dtype) % 16 != 0.
 */
int dllava_select_compact(const float* logits,
                          int32_t B, const int32_t* seq_off, const int32_t* vis_start, const int32_t* vis_len,
                          int64_t sumN, int mode, double keep_ratio, float threshold,
                          const void* hidden, void* hidden_out, int64_t d,
                          const void* Q, void* Q_out,
                          const void* K, const void* V, const dllava_kv_cache* cache,
                          uint8_t* keep_mask, int32_t* kept_idx, int32_t* out_off,
                          int32_t* err_flag, int dtype,
                          void* workspace, size_t workspace_bytes, void* stream);
size_t dllava_select_compact_workspace(int32_t B, int64_t sumN);

/*
 * Compaction with decisions taken earlier (Sec. 3.3: the predictors run once, after decoder layer l, and their
 * decisions are shared by all subsequent layers): the gather half of dllava_select_compact, applied to the tensors
 * and the KV cache of another layer.  kept_idx and out_off are the outputs of the dllava_select_compact call that took
 * the decisions; everything else has the meaning it has there.  Sets cache->cache_len[b] = N*(b) (clamped to the
 * capacity, with err_flag raised) when K and V are given.  No workspace.
 *   Q needs `cache` too (it supplies H and Dh).  Any of the three tensor groups may be NULL.
 */
int dllava_compact(int32_t B, const int32_t* seq_off, const int32_t* kept_idx, const int32_t* out_off, int64_t sumN,
                   const void* hidden, void* hidden_out, int64_t d,
                   const void* Q, void* Q_out, const void* K, const void* V, const dllava_kv_cache* cache,
                   int32_t* err_flag, int dtype, void* stream);

/*
 * Causal scaled-dot-product attention over the reduced prefill set (Eq. 1 applied to S^{P*}):
 * for sequence b, head h and compacted row i,  O_i = softmax_{j<=i}(scale * q_i . k_j) V.
 *
 *   Q       [rows, H, Dh] dtype, compacted rows (rows >= off[B])
 *   K, V    [rows, H, Dh] dtype; or both NULL to read keys/values of sequence b from `cache`
 *           positions 0..n_b-1 (the cache must hold at least n_b = off[b+1]-off[b] tokens)
 *   off     [B+1] row offsets of the sequences (out_off of dllava_select_compact)
 *   rows    host upper bound on off[B] (capacity of Q and O); only rows < off[B] are written
 *   O       [rows, H, Dh] dtype, out
 * Sizes: Dh in {64, 128}.
 */
int dllava_prefill_attn(const void* Q, const void* K, const void* V, const dllava_kv_cache* cache,
                        int32_t B, const int32_t* off, int64_t rows,
                        int32_t H, int32_t Dh, float scale, void* O, int dtype, void* stream);

/*
 * One decode step with online KV-cache reduction (Eq. 6), for B sequences:
 *   o[b,h]  = softmax(scale * [K_cache(b,h); k_new[b,h]] q[b,h]) [V_cache(b,h); v_new[b,h]]
 *             -- the current token always takes part, whatever its keep decision;
 *   keep[b] = keep_override[b] != 0                      if keep_override != NULL
 *           = logits[b,1] - logits[b,0] > threshold      otherwise (float32, strict);
 *   if keep[b]: k_new[b], v_new[b] are stored at position cache_len[b] and cache_len[b] += 1.
 *
 *   q, k_new, v_new  [B, H, Dh] cache->dtype
 *   logits           [B, 2] float32 (output of dllava_score for the current tokens); may be NULL
 *                    only if keep_override is given
 *   o                [B, H, Dh] cache->dtype, out
 *   keep_out         [B] uint8 out, may be NULL
 *   err_flag         device int32, may be NULL: set to 1 when a kept token finds its sequence at
 *                    capacity (max_pages_per_seq * page_size); that append is skipped, cache_len
 *                    stays, keep_out still reports the decision.  Never cleared by the library.
 * Two calls that share a cache must be ordered on one stream (or otherwise serialised).
 */
int dllava_decode_attn_append(const void* q, const void* k_new, const void* v_new, int32_t B,
                              const float* logits, float threshold, const uint8_t* keep_override,
                              const dllava_kv_cache* cache, float scale,
                              void* o, uint8_t* keep_out, int32_t* err_flag,
                              void* workspace, size_t workspace_bytes, void* stream);
size_t dllava_decode_workspace(int32_t B, int32_t H, int32_t Dh, int32_t max_pages_per_seq);

/*
 * dllava_decode_attn_append for callers that cannot allocate device memory where they run, and so cannot bring a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments,
 * same kernels and same results as dllava_decode_attn_append, without `workspace`: the counters and partial results
 * live in a 4 MiB device array that is part of the library's code object (every GPU the library runs on holds its own
 * copy until the process ends).  The call itself allocates nothing and calls no allocating routine.
 *   Limits (DLLAVA_ECAPACITY beyond them, nothing launched): 2*B*H + B <= 12288 counters, and at most 1 MiB of
 *   partial results, B*H*splits*(Dh*4 + 8) bytes for the split count the library picks (none when B*H >= 512).
 *   The first call on a device resolves the array's device address (hipGetSymbolAddress); make that call outside a
 *   stream capture.  All calls on one GPU share the array: calls that overlap on one GPU (two streams, two host
 *   threads) race and must be serialised by the caller.  Between calls the array holds zeros where counters live (each
 *   launch returns its counters to zero) and stale partial results, which are always written before they are read.
 */
int dllava_decode_attn_append_static(const void* q, const void* k_new, const void* v_new, int32_t B,
                                     const float* logits, float threshold, const uint8_t* keep_override,
                                     const dllava_kv_cache* cache, float scale,
                                     void* o, uint8_t* keep_out, int32_t* err_flag, void* stream);

/*
 * The same decode step (Eq. 6) in DEFERRED form: scoring and attention of the current tokens in ONE launch.
 *
 * In dllava_decode_attn_append the append waits for the keep decision, so the predictor must run before the
 * attention kernel (two dependent launches per step).  Nothing else in the step needs the decision: the current
 * token takes part in its own attention whatever it is.  Here the decision of the token of step t is therefore
 * applied by the call of step t+1:
 *   logits[b]  = predictor logits of x[b]                          (as dllava_score, one row per sequence)
 *   keep_prev[b] = keep_prev_override[b] != 0                      if keep_prev_override != NULL
 *                = logits_prev[b,1] - logits_prev[b,0] > threshold if logits_prev != NULL   (float32, strict)
 *                = 0                                               otherwise (first step: nothing outstanding)
 *   if keep_prev[b]: k_prev[b], v_prev[b] are stored at position cache_len[b] and cache_len[b] += 1
 *   o[b,h] = softmax(scale * [K_cache(b,h); k_new[b,h]] q[b,h]) [V_cache(b,h); v_new[b,h]]   over the cache INCLUDING
 *            the previous token if it was kept -- exactly the o of dllava_decode_attn_append at the same step.
 * The current tokens are NOT in the cache when the call returns: pass their k_new, v_new and `logits` as k_prev,
 * v_prev, logits_prev of the next call (the buffers must stay untouched until then), and finish a generation
 * with dllava_decode_commit.  After that the cache equals the one dllava_decode_attn_append leaves, bit for bit.
 *
 *   x [B, d] dtype (row stride ldx), W1 [dh, d], W2 [2, dh] dtype, b1 [dh], b2 [2] float32 or NULL: as dllava_score.
 *                x may be NULL: then nothing is scored in this call (W1, W2, logits ignored; the logits of this step's
 *                tokens come from elsewhere, e.g. dllava_predict running beside this launch on another stream), the
 *                workspace of dllava_decode_workspace suffices, and the call is attention + deferred append only
 *   q, k_new, v_new, k_prev, v_prev  [B, H, Dh] cache->dtype
 *   logits       [B, 2] float32 out;  logits_prev [B, 2] float32 in (a different buffer) or NULL
 *   keep_prev_out [B] uint8 out, may be NULL: keep_prev, written only when a previous token is given
 *   err_flag     as in dllava_decode_attn_append (a kept previous token that finds its sequence at capacity is
 *                neither stored nor attended)
 *   workspace    dllava_decode_step_workspace(...) bytes, zero-filled once, private to this entry point
 * The single launch covers bfloat16 with B <= 64 and d % 64 == 0; other shapes run the predictor as a launch of its
 * own in front (same results).
 */
int dllava_decode_step(const void* x, int64_t ldx, int64_t d, int64_t dh,
                       const void* W1, const float* b1, const void* W2, const float* b2,
                       const void* q, const void* k_new, const void* v_new,
                       const void* k_prev, const void* v_prev, const float* logits_prev,
                       const uint8_t* keep_prev_override,
                       int32_t B, float threshold, const dllava_kv_cache* cache, float scale,
                       void* o, float* logits, uint8_t* keep_prev_out, int32_t* err_flag,
                       void* workspace, size_t workspace_bytes, void* stream);
size_t dllava_decode_step_workspace(int32_t B, int32_t H, int32_t Dh, int32_t max_pages_per_seq,
                                    int64_t d, int64_t dh, int dtype);

/* Applies the decision that the last dllava_decode_step left outstanding: if keep (from logits_prev and threshold, or
 * keep_prev_override), k_prev[b], v_prev[b] are stored at position cache_len[b] and cache_len[b] += 1.
 * keep_out [B] uint8 may be NULL; err_flag as above. */
int dllava_decode_commit(const void* k_prev, const void* v_prev, const float* logits_prev,
                         const uint8_t* keep_prev_override, int32_t B, float threshold,
                         const dllava_kv_cache* cache, uint8_t* keep_out, int32_t* err_flag, void* stream);

/*
 * Projections of the reduced prefill set (Eq. 3 line 1 applied to S^{P*}; Sec. 3.2: the linear layers carry
 * most of the prefill cost, so they run over the kept rows only):
 *     Q, K, V = W^Q x, W^K x, W^V x     for every compacted row x,
 * queries and keys then rotated by the ORIGINAL position p of their token: with half = Dh/2 and, per head,
 * the pair (i, i + half), i < half, angle = p * rope_base^(-2 i / Dh):
 *     y[i] = x[i] cos(angle) - x[i+half] sin(angle),   y[i+half] = x[i+half] cos(angle) + x[i] sin(angle)
 * (rotary position embedding in the pairing of the LLaMA decoder; the paper itself does not mention
 * positions).  Q goes to Q_out; K and V of token j of sequence b go through cache->block_table into
 * cache->pages at position j, and cache->cache_len[b] = n_b = off[b+1] - off[b].  With this call,
 * dllava_select_compact only has to gather the hidden states (its Q, K, V arguments NULL).
 *
 *   x        [rows, d] dtype, compacted hidden states (hidden_out of dllava_select_compact), row stride ldx
 *   rows     host upper bound on off[B] (capacity of x, pos and Q_out); only rows < off[B] are computed
 *   off      [B+1] row offsets of the sequences in the compacted order (out_off of dllava_select_compact)
 *   pos      [rows] int32 original sequence-relative position of every compacted row (kept_idx of
 *            dllava_select_compact), 0 <= pos < 2^24; may be NULL when rope_base <= 0
 *   Wq, Wk, Wv  [H*Dh, d] dtype, row-major (H, Dh from `cache`)
 *   rope_base   > 0: rotate as above (LLaMA uses 10000); <= 0: no rotation
 *   Q_out    [rows, H, Dh] dtype, out
 *   err_flag device int32, may be NULL: set to 1 if some n_b exceeds the cache capacity
 *            max_pages_per_seq * page_size; K/V rows beyond capacity are then not written and cache_len[b]
 *            is clamped to the capacity.  Never cleared by the library.
 * Sizes: d * sizeof(dtype) and ldx * sizeof(dtype) multiples of 16.  rows == 0 or B == 0 is a no-op.
 */
int dllava_qkv_project(const void* x, int64_t ldx, int64_t rows, int64_t d,
                       int32_t B, const int32_t* off, const int32_t* pos,
                       const void* Wq, const void* Wk, const void* Wv, float rope_base,
                       void* Q_out, const dllava_kv_cache* cache, int32_t* err_flag,
                       int dtype, void* stream);

/*
 * Predictors in the form of the paper's appendix (Appendix A.4.1, "Details of Predictor Architecture"):
 * one linear layer reduces the decoder width d to 512; the IMAGE predictor then runs n_blocks = 2
 * vision-transformer blocks over the image tokens of each sequence, the OUTPUT-TEXT predictor none
 * (n_blocks = 0: every row on its own); both end in the MLP 512 -> 256 -> 128 -> 2.  dllava_score is the
 * simplified two-layer form of the same step; the logits have the same meaning (column 1 = keep) and feed
 * dllava_select_compact / the decode steps unchanged.
 *
 * What the appendix leaves open is read as follows (all widths fixed):
 *   z   = x W_in^T + b_in                                          [M, 512], no activation
 *   per block (pre-norm):   z += MHA(LN1(z)) Wo^T + bo ,   z += GELU(LN2(z) Wfc1^T + bfc1) Wfc2^T + bfc2
 *       LN: per row, biased variance, eps 1e-6, scale g and shift b;  MHA: q|k|v = y Wqkv^T + bqkv (q first),
 *       8 heads of 64, softmax(q k^T / 8) v over ALL image tokens of the same sequence, no causal mask,
 *       no tokens of other sequences, no position term;  MLP width 2048;  exact (erf) GELU
 *   D   = GELU(GELU(z W_h1^T + b_h1) W_h2^T + b_h2) W_h3^T + b_h3   [M, 2]
 * Every tensor written between two layers (z, LN outputs, q/k/v, attention output, hidden activations) is
 * stored in dtype (rounded to nearest even); sums are float32; logits are float32.
 *
 * All matrices are [out, in] row-major in dtype; vectors are float32 and may be NULL (= 0 for biases and
 * LayerNorm shifts, = 1 for LayerNorm scales); matrices and vectors are 16-byte aligned (b_h3 and W_h3: 4).
 */
typedef struct dllava_vit_block {
  const float* ln1_g; const float* ln1_b;   /* [512] */
  const void* Wqkv; const float* bqkv;      /* [1536, 512], [1536]: rows 0..511 q, 512..1023 k, 1024..1535 v */
  const void* Wo; const float* bo;          /* [512, 512], [512] */
  const float* ln2_g; const float* ln2_b;   /* [512] */
  const void* Wfc1; const float* bfc1;      /* [2048, 512], [2048] */
  const void* Wfc2; const float* bfc2;      /* [512, 2048], [512] */
} dllava_vit_block;

#define DLLAVA_PREDICTOR_MAX_BLOCKS 4
typedef struct dllava_predictor {
  int64_t d;                                 /* input width; d % 64 == 0 */
  int32_t n_blocks;                          /* 0 .. DLLAVA_PREDICTOR_MAX_BLOCKS */
  const void* W_in; const float* b_in;       /* [512, d], [512] */
  dllava_vit_block blocks[DLLAVA_PREDICTOR_MAX_BLOCKS];
  const void* W_h1; const float* b_h1;       /* [256, 512], [256] */
  const void* W_h2; const float* b_h2;       /* [128, 256], [128] */
  const void* W_h3; const float* b_h3;       /* [2, 128], [2] */
} dllava_predictor;

/*
 *   x, ldx, M, B, seq_off, vis_start, vis_len, logits
 *            as in dllava_score: with seq_off the vision spans are scored (M = sum_b vis_len[b]) and, when
 *            n_blocks > 0, the rows of one span attend to one another; with seq_off == NULL rows 0..M-1 of x
 *            are scored and, when n_blocks > 0, form ONE span.
 *   p        host struct (device pointers inside), read during the call only
 *   dtype    DLLAVA_BF16 only (DLLAVA_EDTYPE otherwise)
 *   workspace  device, 256-byte aligned, dllava_predict_workspace(M, B, n_blocks) bytes; contents need not
 *            be initialised and are scratch (about 9.3 KB per row)
 * Sizes: ldx % 8 == 0, M < 2^31.  M == 0 is a no-op.
 */
int dllava_predict(const void* x, int64_t ldx, int64_t M,
                   int32_t B, const int32_t* seq_off, const int32_t* vis_start, const int32_t* vis_len,
                   const dllava_predictor* p, int dtype, float* logits,
                   void* workspace, size_t workspace_bytes, void* stream);
size_t dllava_predict_workspace(int64_t M, int32_t B, int32_t n_blocks);

/*
 * The layers dllava_predict is made of, as calls of their own (Appendix A.4.1 names the layers; the formulas are
 * the ones stated above), and the remaining layers of the LLaMA-family decoder the paper sparsifies.  DLLAVA_BF16
 * only; float32 sums; each output element is rounded once.  Pointers are device pointers, 16-byte aligned.
 */

/*
 * Linear layer:  y = act(x W^T + bias) + residual      (act 0 = none, 1 = exact GELU), or
 *                y = (x W^T + bias) * SiLU(residual)   (act 2: the gated unit of a SwiGLU feed-forward layer,
 *                                                       `residual` holding the gate x W_gate^T)
 *   x [M, K] row stride ldx;  W [N, K];  bias [N] float32 or NULL;
 *   residual [M, N] with y's row stride, or NULL (act 0, 1), may be y itself;  y [M, N] row stride ldy, out.
 * Sizes: K % 64 == 0, N % 8 == 0, ldx % 8 == 0, ldy % 8 == 0.
 */
int dllava_linear(const void* x, int64_t ldx, int64_t M, int64_t K, const void* W, const float* bias, int64_t N,
                  int act, const void* residual, void* y, int64_t ldy, int dtype, void* stream);

/*
 * LayerNorm of 512-wide rows:  y = (z - mean) / sqrt(var + 1e-6) * gamma + beta per row (biased variance).
 *   z, y [M, 512] contiguous;  gamma, beta [512] float32 or NULL (1 and 0).
 */
int dllava_layer_norm(const void* z, int64_t M, const float* gamma, const float* beta, void* y, int dtype,
                         void* stream);

/*
 * RMSNorm:  y = x / sqrt(mean(x^2) + eps) * weight per row of d.
 *   x [M, d] row stride ldx, y [M, d] row stride ldy;  weight [d] float32 or NULL (= 1);  d % 8 == 0, d <= 8192.
 */
int dllava_rms_norm(const void* x, int64_t ldx, int64_t M, int64_t d, const float* weight, float eps, void* y,
                    int64_t ldy, int dtype, void* stream);

/*
 * Attention without a causal mask inside row spans (the attention of the image predictor's blocks):
 *   O_i = softmax_j(scale * q_i . k_j) V over ALL rows j of the span of row i.
 *   Q, K, V, O [rows, H, Dh] contiguous;  off [B+1] row offsets of the spans;  rows = host upper bound on off[B];
 *   Dh in {64, 128}.
 */
int dllava_span_attn(const void* Q, const void* K, const void* V, int32_t B, const int32_t* off, int64_t rows,
                     int32_t H, int32_t Dh, float scale, void* O, int dtype, void* stream);

/*
 * Attention of the end-to-end sparsification training on the FULL token set (Sec. 3.3.3, Eq. 7): the keep mask acts
 * inside the softmax instead of removing tokens.  For sequence b, head h and row i:
 *     O_i = sum_{j<=i} w_ij V_j,   w_ij = exp(scale q_i.k_j) G_ij / sum_{k<=i} exp(scale q_i.k_k) G_ik,
 *     G_ij = keep_mask[j] for j < i,  G_ii = 1
 * (causal order of the decoder; the diagonal of the mask matrix is one).  Every row gets an output, also rows whose
 * own mask entry is 0; on the rows with mask 1 the result equals dllava_prefill_attn over the compacted sequence.
 *
 *   Q, K, V, O  [rows, H, Dh] dtype (DLLAVA_BF16 only), all tokens of the batch, sequences back to back
 *   off       [B+1] row offsets of the sequences;  rows = host upper bound on off[B]
 *   keep_mask [rows] uint8, 0 = dropped, anything else = kept (keep_mask of dllava_select_compact)
 *   workspace device, 256-byte aligned, dllava_masked_attn_workspace(rows, B) bytes, scratch (need not be initialised)
 * Sizes: Dh in {64, 128}, scale > 0.
 */
int dllava_masked_attn(const void* Q, const void* K, const void* V, int32_t B, const int32_t* off, int64_t rows,
                       int32_t H, int32_t Dh, float scale, const uint8_t* keep_mask, void* O, int dtype,
                       void* workspace, size_t workspace_bytes, void* stream);
size_t dllava_masked_attn_workspace(int64_t rows, int32_t B);

/*
 * dllava_linear for FEW rows (M <= 64: one row per sequence of a decode step), where the weight matrix is the
 * traffic: W is read once, spread over the chip (blocks of 32 output features x a part of K), in ONE launch: the
 * blocks of one feature group hand their sums over through `workspace` and the last to arrive adds them in a fixed
 * order and applies bias, activation and residual.  Arguments as dllava_linear; N % 32 == 0.
 *   workspace  dllava_linear_few_workspace(N, K) bytes, 256-byte aligned, ZERO-FILLED once before its first use (its
 *              first 4096 bytes are counters that every call returns to zero); one buffer of the largest size may
 *              serve all three few-rows entry points, calls ordered on one stream.
 */
int dllava_linear_few(const void* x, int64_t ldx, int64_t M, int64_t K, const void* W, const float* bias, int64_t N,
                      int act, const void* residual, void* y, int64_t ldy, int dtype,
                      void* workspace, size_t workspace_bytes, void* stream);
size_t dllava_linear_few_workspace(int64_t N, int64_t K);

/*
 * Rotary rotation IN PLACE of x [rows, H, Dh] at positions pos [rows] (int32), pairing and angles as in
 * dllava_qkv_project (feature i with i + Dh/2, angle pos * rope_base^(-2i/Dh)): q and k of the tokens of a decode step.
 */
int dllava_rope(void* x, const int32_t* pos, int64_t rows, int32_t H, int32_t Dh, float rope_base, int dtype, void* stream);

/*
 * q, k, v [M, H, Dh] = x Wq^T, x Wk^T, x Wv^T for few rows (M <= 64) with q and k rotated at pos[row] (as dllava_rope),
 * the three matrices [H*Dh, d] read once in one launch.  Dh % 32 == 0 (a block rotates 16 features of the lower half
 * of a head with their partners).
 *   workspace  dllava_decode_proj_workspace(3*H*Dh, d) bytes, as for dllava_linear_few.
 */
int dllava_qkv_few(const void* x, int64_t ldx, int64_t M, int64_t d, const void* Wq, const void* Wk, const void* Wv,
                   int32_t H, int32_t Dh, const int32_t* pos, float rope_base, void* q, void* k, void* v, int dtype,
                   void* workspace, size_t workspace_bytes, void* stream);

/*
 * y [M, F] = (x Wu^T) * SiLU(x Wg^T) for few rows (M <= 64), the gate rounded to dtype before the SiLU (as if it had
 * been stored), Wg and Wu [F, d] read once in one launch.  F % 32 == 0.
 *   workspace  dllava_decode_proj_workspace(2*F, d) bytes, as for dllava_linear_few.
 */
int dllava_gated_few(const void* x, int64_t ldx, int64_t M, int64_t d, const void* Wg, const void* Wu, int64_t F,
                     void* y, int64_t ldy, int dtype, void* workspace, size_t workspace_bytes, void* stream);

/* Workspace bytes of dllava_qkv_few (N_total = 3*H*Dh) and dllava_gated_few (N_total = 2*F).  Host, pure. */
size_t dllava_decode_proj_workspace(int64_t N_total, int64_t K);

#ifdef __cplusplus
}
#endif
#endif /* DLLAVA_H */
