/*
 * libsemanticache — C ABI of the SemantiCache compress-then-attend path for AMD MI355X (gfx950).
 *
 * Three operations, each a hand-written HIP kernel pipeline behind a plain C call:
 *
 *   sc_segment      Sec. 2.2, Eq. 1        delimiter mask            -> chunk offsets
 *   sc_gsc_merge    Sec. 2.3, Alg. 1/Eq. 2 keys/values + offsets     -> merged keys/values (semantic
 *                   Sec. 2.4, Eq. 3                                     cores), cluster sizes, lengths
 *   sc_decode_attn  Sec. 2.4, Eq. 4        query vs. merged cache with the log-size bias
 *
 * Conventions shared by all entry points
 *   - Every data pointer is DEVICE memory owned by the caller; the library neither allocates
 *     nor frees device memory.  Scratch memory is passed in as `ws` (size from the matching
 *     *_workspace_bytes query; 256-byte aligned).  `ws` contents are undefined afterwards.
 *   - Calls are asynchronous on `stream` (a hipStream_t passed as void*; NULL = default stream).
 *     No call synchronises with the host.  Calls that share a workspace must be stream-ordered.
 *   - Return value: SC_OK, or an error detected on the host BEFORE anything is launched
 *     (nothing is written in that case).  Conditions only the device can see (an output
 *     capacity that turns out too small) are reported in the outputs themselves: the affected
 *     length entry is set to -1 and no row is written out of bounds.
 *   - Shapes are row-major; "[B, H, N, d]" means d is the fastest dimension.
 *   - A "sequence" b has seq_lens[b] <= N_max tokens; positions beyond are never read.
 *   - Supported head dims: 64 and 128.  Supported element types: fp32 and bf16.
 */
#ifndef SEMANTICACHE_H
#define SEMANTICACHE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    SC_OK = 0,
    SC_ERR_INVALID_ARG = 1,   /* null pointer, non-positive size, misaligned pointer or stride */
    SC_ERR_UNSUPPORTED = 2,   /* head dim / dtype / head grouping the kernels do not cover */
    SC_ERR_CAPACITY = 3,      /* an output capacity that can never hold the result */
    SC_ERR_WORKSPACE = 4,     /* ws is NULL or smaller than *_workspace_bytes */
    SC_ERR_RUNTIME = 5        /* the HIP runtime refused a launch; see sc_last_runtime_error */
} sc_status;

typedef enum { SC_F32 = 0, SC_BF16 = 1 } sc_dtype;

/* Human-readable name of a status code (static storage, never NULL). */
const char *sc_status_string(sc_status status);

/* Text of the last HIP runtime error seen by this thread inside the library ("" if none). */
const char *sc_last_runtime_error(void);

/* Library version, "major.minor.patch". */
const char *sc_version(void);

/* ------------------------------------------------------------------------------------------------
 * sc_check_lengths — the one call that waits.  Overflow that only the device can see (more chunks than
 * offsets_cap, more merged rows than cap) is reported in band: the affected entry of num_chunks /
 * comp_lens is -1 and nothing is written out of bounds.  This helper copies `count` such entries to
 * the host on `stream`, waits for the stream, and returns SC_ERR_CAPACITY if any is negative
 * (*first_bad, if given, receives its index, else -1), SC_OK otherwise.  Not for the hot path.
 */
sc_status sc_check_lengths(const int32_t *lengths, int count, int *first_bad, void *stream);

/* ------------------------------------------------------------------------------------------------
 * sc_segment — semantic chunking (Sec. 2.2, Eq. 1).
 *
 * A sequence of n tokens with delimiters at positions p_1 < ... < p_{M-1} becomes the alternating
 * series (C_1, d_1, C_2, ..., d_{M-1}, C_M): M = (#delimiters + 1) possibly empty chunks separated
 * by single delimiters.  Encoding per sequence b (row b of `offsets`):
 *     offsets[0] = 0,  offsets[m] = p_m + 1 (1 <= m < M),  offsets[M] = n + 1,
 * so chunk m (0-based) covers positions [offsets[m], offsets[m+1] - 1) and the delimiter that closes
 * it, if any, is position offsets[m+1] - 1 (< n).  num_chunks[b] = M.
 *
 *   mask           device u8 [B, N_max] (row stride mask_stride_b bytes); nonzero = delimiter
 *   seq_lens       device i32 [B], or NULL meaning every sequence has N_max tokens
 *   offsets        device i32 [B, offsets_cap] (row stride offsets_stride_b elements); needs
 *                  offsets_cap >= M + 1; N_max + 2 always suffices
 *   num_chunks     device i32 [B]; set to -1 for a sequence whose M + 1 exceeds offsets_cap
 *                  (its offsets row is then unspecified but never overrun)
 *   ws, ws_bytes   unused by the current kernels (sc_segment_workspace_bytes returns 0); may be NULL
 *
 * Integer work: results are exact.  Host errors: NULL mask/offsets/num_chunks, B <= 0, N_max <= 0,
 * offsets_cap < 2, strides smaller than the row.
 */
size_t sc_segment_workspace_bytes(int B, int N_max);
sc_status sc_segment(const uint8_t *mask, int64_t mask_stride_b, const int32_t *seq_lens,
                     int B, int N_max,
                     int32_t *offsets, int64_t offsets_stride_b, int offsets_cap,
                     int32_t *num_chunks,
                     void *ws, size_t ws_bytes, void *stream);

/* ------------------------------------------------------------------------------------------------
 * sc_gsc_merge — Greedy Seed-Based Clustering inside every chunk (Sec. 2.3, Alg. 1 with the cosine
 * similarity of Eq. 2 on keys only) followed by clustered merging (Sec. 2.4, Eq. 3), independently
 * for every (sequence, KV head).
 *
 * Clustering: in each chunk the first unassigned token becomes a seed and absorbs every later
 * unassigned token whose key has cosine similarity to the SEED's key strictly greater than tau;
 * repeat until every token is assigned.  A similarity that is not a number (zero-norm key) never
 * exceeds tau.  Decisions are taken in fp32 and re-evaluated in fp64 whenever the fp32 value lies
 * within 1e-4 of tau, so they equal an fp64 evaluation except for similarities within ~1e-13 of tau.
 *
 * Merging: each cluster S_t becomes one row (mean of its keys, mean of its values, size |S_t|),
 * accumulated in fp32.  Output rows of a (sequence, head), in order: for each chunk, its clusters in
 * order of their seeds, then the chunk's closing delimiter with size 1.  Rows of size 1 (delimiters,
 * unmerged tokens) carry the values of their input row unchanged (widened exactly if out_dtype is
 * wider); the one liberty taken is that a negative zero may come out as a positive zero.
 * Inputs are expected to be finite: the sums run on matrix cores over groups of neighbouring chunks
 * with 0/1 weights, so a NaN or Inf element can turn the same column of other rows of its group into
 * NaN.  The clustering decisions themselves treat NaN similarities as "not above tau".
 * With bf16 inputs, bf16 or fp32 outputs and d = 128 the call runs two kernels (cluster + merge
 * into provisional rows; relocation to the final rows, which adds up the row counts itself), three
 * for sequences of more than 32768 tokens (an exclusive scan of the row counts in between); other
 * combinations run a generic three-kernel path with the same results.
 *
 *   K, V            device [B, Hkv, N_max, d] of in_dtype, addressed as
 *                   base + b*stride_b + h*stride_h + n*stride_n (+ e), strides in ELEMENTS;
 *                   the last dimension is contiguous; rows must be 16-byte aligned
 *   seq_lens        device i32 [B] or NULL (= N_max)
 *   offsets, num_chunks   as produced by sc_segment (shared by all heads); sequences with
 *                   num_chunks[b] < 0 are skipped and get comp_lens = -1
 *   tau             similarity threshold (any real value; the paper uses 0.5..0.9)
 *   Kc, Vc          device [B, Hkv, cap, d] of out_dtype, contiguous
 *   counts          device i32 [B, Hkv, cap]; cluster sizes (1 for delimiters)
 *   comp_lens       device i32 [B, Hkv]; number of rows produced N'(b,h), or -1 if N' > cap
 *                   (then only the first cap rows are written)
 *   cluster_id      device i32 [B, Hkv, N_max] or NULL; receives for every token the index of its
 *                   cluster inside its chunk (-1 for delimiters); positions >= seq_lens[b] untouched
 *   cap             rows available per (b, h); cap = N_max always suffices
 *
 * Host errors: NULL required pointer, B/Hkv/N_max/cap <= 0, d not in {64,128}, bad dtype,
 * misaligned base pointers or strides not multiples of 16 bytes, workspace too small.
 *
 * Workspace: sc_gsc_merge_workspace_bytes(B, Hkv, N_max, d) bytes serve either output type.  The
 * largest part holds the merged rows of Eq. 3 at provisional positions, in the output type:
 * sc_gsc_merge_workspace_bytes_for(..., out_dtype) is what a call with that out_dtype needs (for
 * bf16 about half: 544 instead of 1056 bytes per token and KV head at d = 128), and sc_gsc_merge and
 * sc_gsc_merge_append accept a workspace of that size.  0 for a non-positive size or an unknown type.
 */
size_t sc_gsc_merge_workspace_bytes(int B, int Hkv, int N_max, int d);
size_t sc_gsc_merge_workspace_bytes_for(int B, int Hkv, int N_max, int d, sc_dtype out_dtype);
sc_status sc_gsc_merge(const void *K, const void *V, sc_dtype in_dtype,
                       int64_t stride_b, int64_t stride_h, int64_t stride_n,
                       const int32_t *seq_lens,
                       const int32_t *offsets, int64_t offsets_stride_b, const int32_t *num_chunks,
                       int B, int Hkv, int N_max, int d, float tau,
                       void *Kc, void *Vc, sc_dtype out_dtype, int cap,
                       int32_t *counts, int32_t *comp_lens, int32_t *cluster_id,
                       void *ws, size_t ws_bytes, void *stream);

/* ------------------------------------------------------------------------------------------------
 * sc_decode_attn — Proportional Attention for one decode step (Sec. 2.4, Eq. 4):
 *     O[b,hq] = softmax_t( Q[b,hq] . Kc[b,h,t] * scale + ln(counts[b,h,t]) ) Vc[b,h,t],
 *     t in [0, comp_lens[b,h]),  h = hq / (Hq / Hkv)   (consecutive query heads share a KV head).
 * No mask: the query sees every row of the merged cache.  fp32 softmax and accumulation.
 *
 *   Q               device [B, Hq, d] of q_dtype, contiguous
 *   Kc, Vc, counts  device, layout as written by sc_gsc_merge ([B, Hkv, cap, d] of kv_dtype, [B, Hkv, cap])
 *   comp_lens       device i32 [B, Hkv]; entries <= 0 give O = 0 and lse = -inf for that head group
 *   scale           logit scale; 0 selects 1/sqrt(d)
 *   O               device [B, Hq, d] of o_dtype, contiguous, 16-byte aligned
 *   lse             device f32 [B, Hq] or NULL; natural-log-sum-exp of the biased logits
 *
 *   ws              workspace of sc_decode_attn_workspace_bytes.  Unlike the other workspaces it carries
 *                   state and must be initialised ONCE with sc_decode_attn_init_workspace (for the same
 *                   B and Hkv) after allocating; after that it can be reused by stream-ordered calls of
 *                   that shape without further care.  Two calls that overlap in time need two workspaces.
 *                   State: the rows of a (sequence, KV head) are cut into splits, one workgroup each,
 *                   and the workgroup of the last split folds the partial results of the others.  Per
 *                   (sequence, KV head) the workspace keeps an epoch counter and one flag per split;
 *                   a split publishes its partial by storing the current epoch + 1 in its flag, the
 *                   folding workgroup accepts only flags with that value and then raises the epoch, so
 *                   nothing has to be cleared between calls and a flag left over from an earlier call
 *                   can never be taken for a current one.
 *                   The folding workgroup waits for the flags for a bounded time.  Should the wait ever
 *                   run out (it cannot while workgroups start in grid order), the call fails visibly
 *                   and for good: that head group's O and lse are filled with NaN, the workspace's
 *                   status word is set, and every later call on the workspace also returns NaN for
 *                   that head group until the workspace is initialised again.  The status word is the
 *                   int32 at the start of the workspace (0, or -1 after a failure); it can be tested
 *                   with sc_check_lengths((const int32_t *)ws, 1, NULL, stream).
 *
 * Host errors: NULL required pointer, sizes <= 0, Hq not a multiple of Hkv or Hq/Hkv > 8,
 * d not in {64,128}, bad dtype, workspace too small.
 */
size_t sc_decode_attn_workspace_bytes(int B, int Hq, int Hkv, int cap, int d);
sc_status sc_decode_attn_init_workspace(void *ws, size_t ws_bytes, int B, int Hkv, void *stream);
sc_status sc_decode_attn(const void *Q, sc_dtype q_dtype,
                         const void *Kc, const void *Vc, sc_dtype kv_dtype, int cap,
                         const int32_t *counts, const int32_t *comp_lens,
                         int B, int Hq, int Hkv, int d, float scale,
                         void *O, sc_dtype o_dtype, float *lse,
                         void *ws, size_t ws_bytes, void *stream);

/* ------------------------------------------------------------------------------------------------
 * sc_decode_attn_static — sc_decode_attn for callers that cannot allocate device memory (code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc) and therefore cannot hand
 * in a workspace: same arguments without ws / ws_bytes, same kernels, same results bit for bit.  The
 * scratch is an array inside the library's code object (16 MiB for partial results plus 1 MiB of
 * hand-over state), one copy per GPU, held until the process ends; the call allocates and frees
 * nothing and needs no initialisation call (the array starts zeroed, which is the initialised state).
 *
 *   Limits: sc_decode_attn_workspace_bytes(B, Hq, Hkv, cap, d) must not exceed 16 MiB (16 777 216 B),
 *   e.g. B * Hkv <= 56 at Hq / Hkv = 4, d = 128, and B * Hkv must not exceed 1024; larger shapes are
 *   refused with SC_ERR_WORKSPACE and nothing is launched.  All other host errors as for sc_decode_attn.
 *   All calls on one GPU share that GPU's array, whatever their shapes: calls that overlap in time on
 *   one GPU race; order them on one stream or with events.  The first call on a device looks up the
 *   array's address (no allocation; do it once outside graph capture).  A failed hand-over (see
 *   sc_decode_attn) shows as NaN outputs, here too for every later call of that head group.
 */
sc_status sc_decode_attn_static(const void *Q, sc_dtype q_dtype,
                                const void *Kc, const void *Vc, sc_dtype kv_dtype, int cap,
                                const int32_t *counts, const int32_t *comp_lens,
                                int B, int Hq, int Hkv, int d, float scale,
                                void *O, sc_dtype o_dtype, float *lse, void *stream);

/* ------------------------------------------------------------------------------------------------
 * Decode-time growth.  The paper compresses the prefill cache once and leaves open what happens to the
 * tokens that arrive afterwards (Sec. 2.1 treats the cache as given).  These two calls follow from
 * its definitions without adding any: a token that has not been merged is a cluster of one, exactly
 * like a delimiter row (Sec. 2.4: s holds the cluster sizes, ln 1 = 0), and Alg. 1 never looks across
 * a delimiter (Sec. 2.3), so a stretch of new tokens that is cut at delimiters can be compressed by
 * itself and its rows appended.
 *
 * sc_decode_attn_tail — sc_decode_attn over the rows of the merged cache followed by the first
 * tail_lens[b] rows of an uncompressed tail, which attend with size 1:
 *     rows of (b, h) = Kc[b,h,0..comp_lens[b,h])  ++  Kt[b,h,0..tail_lens[b]).
 *   Kt, Vt          device [B, Hkv, tail_cap, d] of kv_dtype, contiguous, 16-byte aligned
 *   tail_lens       device i32 [B] (clamped to [0, tail_cap])
 * Everything else, the workspace included (same size query, same flags), as for sc_decode_attn.
 *
 * sc_gsc_merge_append — sc_gsc_merge of a further stretch of tokens whose rows are written behind the
 * rows already present: row r of the stretch's result goes to row base_lens[b,h] + r of Kc/Vc/counts,
 * and comp_lens[b,h] = base_lens[b,h] + (rows of the stretch), or -1 if that exceeds cap or
 * base_lens[b,h] is already negative or beyond cap (then nothing is written).  K, V, seq_lens,
 * offsets, num_chunks describe the stretch alone (its own sc_segment call, positions counted from its
 * first token).  If every earlier stretch ended with a delimiter, the result equals one sc_gsc_merge of
 * the whole sequence up to summation order.  base_lens is device i32 [B, Hkv] and must not be the
 * same array as comp_lens (all workgroups read the one while the other is written).
 */
sc_status sc_decode_attn_tail(const void *Q, sc_dtype q_dtype,
                              const void *Kc, const void *Vc, sc_dtype kv_dtype, int cap,
                              const int32_t *counts, const int32_t *comp_lens,
                              const void *Kt, const void *Vt, int tail_cap, const int32_t *tail_lens,
                              int B, int Hq, int Hkv, int d, float scale,
                              void *O, sc_dtype o_dtype, float *lse,
                              void *ws, size_t ws_bytes, void *stream);
sc_status sc_gsc_merge_append(const void *K, const void *V, sc_dtype in_dtype,
                              int64_t stride_b, int64_t stride_h, int64_t stride_n,
                              const int32_t *seq_lens, const int32_t *offsets, int64_t offsets_stride_b,
                              const int32_t *num_chunks,
                              int B, int Hkv, int N_max, int d, float tau,
                              void *Kc, void *Vc, sc_dtype out_dtype, int cap,
                              int32_t *counts, const int32_t *base_lens, int32_t *comp_lens, int32_t *cluster_id,
                              void *ws, size_t ws_bytes, void *stream);

/* ------------------------------------------------------------------------------------------------
 * sc_gsc_merge_global — sc_gsc_merge when the whole sequence of every (sequence, KV head) is ONE chunk:
 * Alg. 1 (Sec. 2.3) over all its tokens, no delimiter rows, then Eq. 3.  This is the "no chunking"
 * variant of the paper's chunking ablation (Sec. 3.4), for which the chunk-by-chunk kernels of
 * sc_gsc_merge are slow by construction; the result is what sc_segment on an all-zero mask followed by
 * sc_gsc_merge gives (same integers; sums in row order).  bf16 inputs with d = 128 and N_max <= 32768 run
 * a dedicated path (all pairwise comparisons on the matrix cores, a block-sequential resolution of the
 * seeds, a gather by cluster); other shapes are handed to sc_gsc_merge's kernels with one-chunk offsets.
 * Arguments, layouts, overflow behaviour (comp_lens = -1) and errors as for sc_gsc_merge, without offsets /
 * num_chunks;  ws: sc_gsc_merge_global_workspace_bytes(B, Hkv, N_max, d) bytes (about N_max^2 / 8 bytes
 * per (sequence, KV head) on the dedicated path: 1.1 GB for 8 heads of 32768 tokens).
 */
size_t sc_gsc_merge_global_workspace_bytes(int B, int Hkv, int N_max, int d);
sc_status sc_gsc_merge_global(const void *K, const void *V, sc_dtype in_dtype,
                              int64_t stride_b, int64_t stride_h, int64_t stride_n,
                              const int32_t *seq_lens,
                              int B, int Hkv, int N_max, int d, float tau,
                              void *Kc, void *Vc, sc_dtype out_dtype, int cap,
                              int32_t *counts, int32_t *comp_lens, int32_t *cluster_id,
                              void *ws, size_t ws_bytes, void *stream);

/* ------------------------------------------------------------------------------------------------
 * sc_gsc_merge_budget — sc_gsc_merge with the threshold chosen for a target cache size.  The paper
 * reports at cache budgets (Sec. 3.1: 20 / 35 / 50 % of the entries kept) without giving the rule
 * that turns a budget into the threshold of Alg. 1; this call takes the largest threshold a bisection
 * finds whose merged caches hold at most budget_rows rows in total (summed over all sequences and KV
 * heads of the call; a head whose rows exceed cap counts as over budget):
 *     lo = tau_lo, hi = tau_hi;  `iterations` times:  mid = 0.5f * (lo + hi) in fp32;
 *     rows(mid) <= budget_rows ? lo = mid : hi = mid;   result = lo.
 * tau_lo is assumed to meet the budget (-1.01 merges every chunk into one row and always does if
 * anything can); it is not probed unless iterations is 0.  Every probe clusters all chunks on the
 * caller's stream and only counts the rows (bf16 / d = 128: no values read, nothing merged; other
 * shapes run complete merges as probes); the bracket lives in device memory and is moved by a small
 * kernel between the probes: iterations + 1 launches of the clustering, no host synchronisation.  The
 * last one, at the result, is a complete sc_gsc_merge, so on completion Kc, Vc, counts, comp_lens,
 * cluster_id hold exactly what sc_gsc_merge(tau = result) gives.
 *
 *   budget_rows     target total of merged rows, e.g. round(0.35 * Hkv * sum of seq_lens)
 *   iterations      0..32 bisection steps (12 narrow [-1, 1] to 5e-4)
 *   tau_out         device f32 [1]: the threshold found
 *   rows_out        device i64 [1] or NULL: total rows at that threshold (-1 if a head overflowed cap);
 *                   larger than budget_rows if even tau_lo does not meet the budget
 *   ws              sc_gsc_merge_budget_workspace_bytes(B, Hkv, N_max, d) bytes
 * All other arguments and errors as for sc_gsc_merge; additionally iterations out of range,
 * tau_lo > tau_hi, negative budget_rows, NULL or misaligned tau_out.
 */
size_t sc_gsc_merge_budget_workspace_bytes(int B, int Hkv, int N_max, int d);
sc_status sc_gsc_merge_budget(const void *K, const void *V, sc_dtype in_dtype,
                              int64_t stride_b, int64_t stride_h, int64_t stride_n,
                              const int32_t *seq_lens, const int32_t *offsets, int64_t offsets_stride_b,
                              const int32_t *num_chunks,
                              int B, int Hkv, int N_max, int d,
                              int64_t budget_rows, float tau_lo, float tau_hi, int iterations,
                              void *Kc, void *Vc, sc_dtype out_dtype, int cap,
                              int32_t *counts, int32_t *comp_lens, int32_t *cluster_id,
                              float *tau_out, int64_t *rows_out,
                              void *ws, size_t ws_bytes, void *stream);

/* ------------------------------------------------------------------------------------------------
 * sc_multi_attn — Eq. 4 for several query rows at once (Sec. 2.4 states it for Q in R^{n x d}): every
 * query row attends to the whole merged cache of its KV head, no mask between the rows (they are all
 * later than the cache):
 *     O[j,b,hq] = softmax_t( Q[j,b,hq] . Kc[b,h,t] * scale + ln(counts[b,h,t]) ) Vc[b,h,t].
 * For a handful of speculative or freshly arrived tokens.
 *
 *   Q               device [nq, B, Hq, d] of q_dtype, contiguous (query-major, so that one row of the
 *                   call has the layout of an sc_decode_attn query)
 *   nq              number of query rows, 1..4096
 *   Kc, Vc, counts, comp_lens, scale    as for sc_decode_attn
 *   O               device [nq, B, Hq, d] of o_dtype;  lse  device f32 [nq, B, Hq] or NULL
 *   ws              sc_multi_attn_workspace_bytes(B, Hq, Hkv, nq, cap, d) bytes; carries no state
 *
 * bf16 queries and cache with d = 128 run on the matrix cores (probabilities enter the second product
 * as two bf16 parts, i.e. with 16 significant bits; fp32 accumulation); every other combination goes row by row through
 * the sc_decode_attn kernels.  Host errors as for sc_decode_attn, plus nq out of range.
 *
 * sc_multi_attn_tail — the same over the merged rows followed by the first tail_lens[b] rows of an
 * uncompressed tail (size 1, as for sc_decode_attn_tail).  With causal != 0 the last nq tail rows of a
 * sequence are the query rows' own tokens and query j sees the tail rows 0 .. tail_lens[b] - nq + j
 * (itself included; none if that is negative): the step that verifies nq speculative tokens, or a
 * chunk of prefill behind a compressed cache.  causal is supported on the matrix-core path only
 * (bf16, d = 128; SC_ERR_UNSUPPORTED otherwise).  Workspace: sc_multi_attn_workspace_bytes with
 * cap + tail_cap in place of cap.
 */
size_t sc_multi_attn_workspace_bytes(int B, int Hq, int Hkv, int nq, int cap, int d);
sc_status sc_multi_attn_tail(const void *Q, sc_dtype q_dtype, int nq,
                             const void *Kc, const void *Vc, sc_dtype kv_dtype, int cap,
                             const int32_t *counts, const int32_t *comp_lens,
                             const void *Kt, const void *Vt, int tail_cap, const int32_t *tail_lens, int causal,
                             int B, int Hq, int Hkv, int d, float scale,
                             void *O, sc_dtype o_dtype, float *lse,
                             void *ws, size_t ws_bytes, void *stream);
sc_status sc_multi_attn(const void *Q, sc_dtype q_dtype, int nq,
                        const void *Kc, const void *Vc, sc_dtype kv_dtype, int cap,
                        const int32_t *counts, const int32_t *comp_lens,
                        int B, int Hq, int Hkv, int d, float scale,
                        void *O, sc_dtype o_dtype, float *lse,
                        void *ws, size_t ws_bytes, void *stream);

/* ------------------------------------------------------------------------------------------------
 * sc_stream_read_probe — a measuring aid for benchmarks, not a step of the method: reads the first
 * `bytes` bytes (rounded down to a multiple of 16) of a device buffer once, 16 bytes per lane, fully
 * coalesced, eight non-temporal loads in flight per lane, one workgroup of twelve wavefronts per CU on a
 * contiguous slab of its own (the fastest of the shapes measured on MI355X), and nothing else to do.
 * Timing it on a buffer much larger than the caches gives the HBM read bandwidth
 * a kernel can attain on the device, to put beside the nominal peak the rooflines are quoted against.
 *   src             device buffer, 16-byte aligned
 *   sink            device scratch of at least 4 KiB that the kernel writes to (contents meaningless)
 * Host errors: NULL pointers, bytes < 16, misaligned pointers.
 */
sc_status sc_stream_read_probe(const void *src, size_t bytes, void *sink, void *stream);

/* ------------------------------------------------------------------------------------------------
 * Launch-shape knobs for experiments (process-wide, not thread-safe; results never depend on them
 * beyond floating-point summation order).  Keys:
 *   "decode_max_splits"    split-K workgroups per (sequence, KV head); <= 0 = chosen from B*Hkv
 *   "decode_min_rows"      rows of the merged cache a split should at least get
 *   "decode_local_handover" 0: split partials always travel through memory, also where all splits of a
 *                          head share one XCC and could use its L2 (the default, 1)
 *   "decode_poll_budget"   polls of the folding workgroup before it gives up (default 2^20); negative:
 *                          give up at once — a host-driven way to exercise the failure path in tests
 *   "decode_mfma_min_group" sc_decode_attn (bf16, d = 128): query heads per KV head from which the
 *                          kernel of sc_multi_attn is used for the single row; 9 = never (the default)
 *   "gsc_fast_path"        0 forces the generic kernels even for bf16 / d = 128
 *   "gsc_chunks_per_task"  fast path: chunks handled by one single-wave workgroup task (1..32);
 *                          <= 0 (the default) = 2, or 1 for a call of a few thousand tokens in all
 *   "gsc_chunks_per_item"  generic path: chunks per work item
 *   "gsc_grid_x"           workgroups per pass and (sequence, KV head); <= 0 = chosen from N_max
 *   "multi_block_rows"     sc_multi_attn: query rows per workgroup, 16 or 32; <= 0 = chosen from the shape
 *   "multi_target_wgs"     sc_multi_attn: workgroups the split count aims at (default 256)
 *                          (these two enter sc_multi_attn_workspace_bytes: set them before asking for the
 *                          size; a workspace that has become too small is refused with SC_ERR_WORKSPACE)
 * Return 0 / the value, or -1 for an unknown key.
 */
int sc_tune_set(const char *key, int value);
int sc_tune_get(const char *key);

#ifdef __cplusplus
}
#endif
#endif /* SEMANTICACHE_H */
