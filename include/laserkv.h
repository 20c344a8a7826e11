/*
 * laserkv.h - C-ABI of the MI355X (gfx950) LASER-KV prefill-selection library.
 *
 * One call of laserkv_select_block + laserkv_append processes one context block of one
 * layer for all KV heads: exact attention score of the block keys under the observation
 * window (Sec. 3.3 "Precision", Alg. 1 step 3), SimHash signatures and collision counts
 * (Sec. 3.3 "Recall", Alg. 1 step 6), the two-stage TopK of Alg. 1 steps 4-8 under the
 * protection-divisor partition of Sec. 3.1, and the append of the kept K/V rows onto the
 * accumulative per-layer cache (Sec. 3, first paragraph).
 *
 * Conventions for every function
 *   - returns LKV_OK (0) or a negative laserkv_status; nothing throws or aborts.
 *   - pointers marked DEVICE point to GPU memory owned by the caller; the library reads or
 *     writes them only during the call's kernels and keeps no reference afterwards.
 *   - all GPU work is enqueued on the caller's hipStream_t (passed as void*) and the call
 *     returns without synchronising; calls on one context must be issued on one stream at a
 *     time (the context's workspace is shared by consecutive calls).
 *   - strides are in ELEMENTS of the storage dtype; the head_dim axis is contiguous.
 *   - query head h*G + g (G = n_q_heads / n_kv_heads) belongs to KV head h.
 */
#ifndef LASERKV_H
#define LASERKV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct laserkv_ctx laserkv_ctx; /* opaque; owns only its own device workspace */

typedef enum { LKV_F32 = 0, LKV_BF16 = 1 } laserkv_dtype;

typedef enum {
  LKV_OK = 0,
  LKV_EINVAL = -1, /* bad shape, stride, budget or parameter; nothing was launched */
  LKV_ECAP = -2,   /* append would overflow the cache capacity */
  LKV_ENOMEM = -3, /* workspace allocation failed */
  LKV_EHIP = -4    /* a HIP runtime call failed; text in laserkv_last_error */
} laserkv_status;

/* q_pos0 value that places the window on the last w tokens of the block */
#define LKV_WINDOW_AT_BLOCK_END INT64_MIN

typedef struct {
  int32_t n_q_heads;   /* H_q */
  int32_t n_kv_heads;  /* H_kv, divides H_q */
  int32_t head_dim;    /* d: 64 or 128 */
  int32_t dtype;       /* laserkv_dtype: storage type of Q, K, V, cache and hyperplanes */
  int32_t lsh_tables;  /* L: number of hash functions h_r (tables), >= 1 */
  int32_t lsh_bits;    /* K: sign bits per table, 1..16; L*K <= 512 */
  int32_t max_block;   /* largest S_t (tokens per block) any call will pass, <= 16384 */
  int32_t max_window;  /* largest W (window queries per head); G*W <= 1024 */
  int32_t max_ctx_keys;/* largest T (look-back keys) */
} laserkv_config;

/* Create a context and allocate its device workspace (hipMalloc) on the current device.
 * *out is set only on success.  Host pointers. */
int laserkv_create(const laserkv_config* cfg, laserkv_ctx** out);

/* Free the workspace.  The caller must have synchronised the stream(s) it used. NULL is ignored. */
void laserkv_destroy(laserkv_ctx* ctx);

/* Text of the last error recorded on this context (or a process-wide one when ctx is NULL).
 * The string is owned by the library and valid until the next failing call. */
const char* laserkv_last_error(const laserkv_ctx* ctx);

/* Per-block budget B = floor(2 r S_block L_ctx / (S_block + L_ctx)), r = r_num / r_den,
 * evaluated in exact integer arithmetic (App. B equation).  Returns -1 on bad arguments.
 * Host only. */
int64_t laserkv_budget(int64_t s_block, int64_t l_ctx, int64_t r_num, int64_t r_den);

/* Partition of a block's budget (Sec. 3.1; Alg. 1 steps 4 and 7), host only:
 *   B_t = min(B, s_t); n_anchor = n_local = floor(B_t / n); B_long = B_t - 2 floor(B_t / n);
 *   k_exact = floor(alpha * B_long); k_lsh = B_long - k_exact.
 * Requires n >= 2, 0 <= alpha <= 1, B >= 0, s_t >= 1. */
int laserkv_partition(int32_t B, int32_t n, double alpha, int32_t s_t,
                      int32_t* n_anchor, int32_t* n_local, int32_t* k_exact, int32_t* k_lsh);

/* Steps a1-a4 for one block: score, hash, count, select.
 *
 *   q_win        DEVICE [H_q, w, d]      window queries; query j sits at position q_pos0 + j
 *   k_blk        DEVICE [H_kv, s_t, d]   block keys; key i sits at position block_pos0 + i
 *   k_ctx        DEVICE [H_kv, t_ctx, d] look-back keys (tail of the previous block, Sec. 3.2):
 *                always visible, they enter the softmax normaliser only; NULL iff t_ctx == 0
 *   hyperplanes  DEVICE [L*K, d] contiguous; row r*K + c decides bit c of table r (bit = proj >= 0)
 *   q_pos0       position of window query 0, or LKV_WINDOW_AT_BLOCK_END: the window is the block's last w
 *                tokens (q_pos0 = block_pos0 + s_t - w), the observation window of Sec. 3.3 "Precision"
 *   causal       non-zero: block key i is visible to query j iff block_pos0 + i <= q_pos0 + j; then
 *                q_pos0 >= block_pos0 is required (every query sees at least the block's first key).
 *                Look-back keys are visible to every query either way.
 *   n_anchor, n_local   first / last positions of the block that are always kept
 *   k_exact      candidates taken by (S_exact descending, index ascending)
 *   k_lsh        remaining candidates taken by (collision count descending, index ascending)
 *                n_anchor + n_local + k_exact + k_lsh = B_t <= s_t
 *   keep_idx     DEVICE out [H_kv, B_t] int32, block-local indices, ascending per head
 *   dbg_*        optional DEVICE outputs of the intermediate stages (NULL to skip):
 *                dbg_s_exact [H_kv, s_t] float, dbg_sig_k [H_kv, s_t, L] uint16,
 *                dbg_sig_q [H_q, w, L] uint16, dbg_count [H_kv, s_t] int32
 *
 * S_exact[h, i] = mean over the G*w window rows of KV head h of softmax(q.k / sqrt(d)) at key i.
 * Errors: LKV_EINVAL for shapes beyond the context's configuration, w < 1, budgets that do
 * not fit the block, misaligned pointers/strides (16-byte rows required), a causal window that
 * starts before the block, or a block with too few keys to spread the L tables' query-code job over. */
int laserkv_select_block(laserkv_ctx* ctx,
                         const void* q_win, int64_t q_stride_head, int64_t q_stride_tok,
                         const void* k_blk, int64_t k_stride_head, int64_t k_stride_tok,
                         const void* k_ctx, int64_t c_stride_head, int64_t c_stride_tok,
                         const void* hyperplanes,
                         int32_t s_t, int32_t w, int32_t t_ctx,
                         int64_t block_pos0, int64_t q_pos0, int32_t causal,
                         int32_t n_anchor, int32_t n_local, int32_t k_exact, int32_t k_lsh,
                         int32_t* keep_idx,
                         float* dbg_s_exact, uint16_t* dbg_sig_k, uint16_t* dbg_sig_q, int32_t* dbg_count,
                         void* hip_stream);

/* Step a5: copy the kept rows to the end of the append-only cache (Sec. 1, first contribution;
 * Sec. 3 first paragraph).
 *
 *   k_blk, v_blk DEVICE [H_kv, s_t, d]
 *   keep_idx     DEVICE [H_kv, b_t] int32 as written by laserkv_select_block (same stream: no sync needed)
 *   k_cache, v_cache DEVICE [H_kv, cache_cap, d], rows contiguous, head stride cache_stride_head
 *   cache_pos    DEVICE [H_kv, cache_cap] int64 absolute token positions, head stride pos_stride_head
 *   cache_len    rows already present per head (host-known: every block adds exactly b_t rows)
 * Rows [cache_len, cache_len + b_t) of every head are written; nothing else is touched.
 * Errors: LKV_ECAP when cache_len + b_t > cache_cap; LKV_EINVAL for bad arguments. */
int laserkv_append(laserkv_ctx* ctx,
                   const void* k_blk, int64_t k_stride_head, int64_t k_stride_tok,
                   const void* v_blk, int64_t v_stride_head, int64_t v_stride_tok,
                   const int32_t* keep_idx, int32_t b_t, int32_t s_t, int64_t block_pos0,
                   void* k_cache, void* v_cache, int64_t cache_stride_head,
                   int64_t* cache_pos, int64_t pos_stride_head,
                   int64_t cache_len, int64_t cache_cap,
                   void* hip_stream);

/* Steps a1-a5 in one call: laserkv_select_block followed by laserkv_append with the same arguments
 * (Alg. 1 and the Sec. 3.1 partition, then the append-only retention of Sec. 3, first paragraph),
 * but with the selection and the gather sharing one kernel, which saves a kernel boundary per block.
 * Results are identical to the two separate calls.  keep_idx still receives the kept indices.
 * Errors: those of both calls; nothing is launched when any check fails. */
int laserkv_compress_block(laserkv_ctx* ctx,
                           const void* q_win, int64_t q_stride_head, int64_t q_stride_tok,
                           const void* k_blk, int64_t k_stride_head, int64_t k_stride_tok,
                           const void* v_blk, int64_t v_stride_head, int64_t v_stride_tok,
                           const void* k_ctx, int64_t c_stride_head, int64_t c_stride_tok,
                           const void* hyperplanes,
                           int32_t s_t, int32_t w, int32_t t_ctx,
                           int64_t block_pos0, int64_t q_pos0, int32_t causal,
                           int32_t n_anchor, int32_t n_local, int32_t k_exact, int32_t k_lsh,
                           int32_t* keep_idx,
                           void* k_cache, void* v_cache, int64_t cache_stride_head,
                           int64_t* cache_pos, int64_t pos_stride_head,
                           int64_t cache_len, int64_t cache_cap,
                           void* hip_stream);

/* laserkv_compress_block for callers that cannot allocate device memory or hold a context: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, checks, kernels
 * and results as laserkv_compress_block on a context created from *cfg, but the workspace is a fixed
 * LKV_STATIC_SCRATCH_BYTES array inside the library (one copy per GPU, held until the process ends).
 * The call allocates nothing (no hipMalloc / hipFree, no events).  cfg is a HOST pointer read during the
 * call only.
 *   - Configurations whose workspace exceeds the array (laserkv_static_workspace_bytes(cfg) >
 *     LKV_STATIC_SCRATCH_BYTES) are rejected with LKV_EINVAL and a message; nothing is launched.
 *   - Every call on a GPU shares that GPU's array, which keeps the previous call's intermediates: each call
 *     rewrites all it reads, so no clearing is needed, but calls that overlap in time on one GPU (two
 *     streams, two threads) race.  Issue them on one stream.
 *   - laserkv_static_init does the once-per-device set-up (address of the array on the current device,
 *     kernel attributes) ahead of time, e.g. before a graph capture begins; otherwise the first
 *     laserkv_compress_block_static call on a device does it.
 *   - errors are reported through laserkv_last_error(NULL); the external log-sum-exp of
 *     laserkv_set_row_lse is not available here. */
#define LKV_STATIC_SCRATCH_BYTES (32u << 20)
int laserkv_static_init(void);
size_t laserkv_static_workspace_bytes(const laserkv_config* cfg); /* 0 for an invalid configuration */
int laserkv_compress_block_static(const laserkv_config* cfg,
                                  const void* q_win, int64_t q_stride_head, int64_t q_stride_tok,
                                  const void* k_blk, int64_t k_stride_head, int64_t k_stride_tok,
                                  const void* v_blk, int64_t v_stride_head, int64_t v_stride_tok,
                                  const void* k_ctx, int64_t c_stride_head, int64_t c_stride_tok,
                                  const void* hyperplanes,
                                  int32_t s_t, int32_t w, int32_t t_ctx,
                                  int64_t block_pos0, int64_t q_pos0, int32_t causal,
                                  int32_t n_anchor, int32_t n_local, int32_t k_exact, int32_t k_lsh,
                                  int32_t* keep_idx,
                                  void* k_cache, void* v_cache, int64_t cache_stride_head,
                                  int64_t* cache_pos, int64_t pos_stride_head,
                                  int64_t cache_len, int64_t cache_cap,
                                  void* hip_stream);

/* Boundary smoothing (Sec. 3.2) extended to context that is not re-read: keys outside a call (the rest
 * of the compressed cache, say) can join the softmax normaliser of Alg. 1 step 3 through one number per
 * window query, the natural-log sum of exp(q.k / sqrt(d)) over those keys, as an attention kernel
 * reports it.  They weigh in exactly as if they had been passed as look-back keys.
 *   row_lse  DEVICE [H_q, w] float, contiguous; NULL switches the feature off (the default).
 * The pointer is remembered by the context and read by the kernels of EVERY following
 * laserkv_select_block / laserkv_compress_block / laserkv_score_block call until it is replaced or reset;
 * it must stay valid until those calls' kernels have run.  Errors: LKV_EINVAL (null context, pointer
 * not 4-byte aligned). */
int laserkv_set_row_lse(laserkv_ctx* ctx, const float* row_lse);

/* The window rows' softmax statistics taken from the model's own attention kernel (Sec. 3.3 "Precision":
 * the exact score is the attention the model already computes; Sec. 3 first paragraph).  row_lse then
 * holds, per window query, the COMPLETE natural-log sum of exp(q.k / sqrt(d)) over every key the row
 * attends to (the block keys it sees, the look-back keys, the rest of the cache), exactly what a
 * flash-attention forward reports for those rows.  S_exact[h, i] = mean over the rows of
 * exp(q.k_i / sqrt(d) - row_lse) at the visible keys.  The library then computes no row statistics, and
 * k_ctx / t_ctx of the following calls are accepted but not read.  Where the shape allows it (G * w <= 512,
 * rows of at most 256 bytes, the query heads of a KV head within 2 GiB, K such that L * 2^K 16-bit bins fit 512 KiB)
 * a block then takes ONE sweep over its keys (hash, score and count from the same LDS rows) instead of two;
 * otherwise the first of the two sweeps only hashes.
 *   row_lse  DEVICE [H_q, w] float, contiguous; NULL switches back to the library's own statistics.
 * Lifetime and scope as for laserkv_set_row_lse, which it replaces (and which replaces it).
 * Errors: LKV_EINVAL (null context, pointer not 4-byte aligned). */
int laserkv_set_row_lse_complete(laserkv_ctx* ctx, const float* row_lse);

/* Attention over the compacted cache (Sec. 3 first paragraph: only the kept tokens remain for later tokens to
 * attend to).  For every query head hq and each of its n_q queries: l_i = q.k_i / sqrt(d) over the first
 * cache_len rows of KV head hq / G's cache (all visible: the cache holds earlier blocks only),
 * out = sum_i softmax(l)_i v_i and out_lse = log sum_i exp(l_i) (natural logarithm).  Serves decoding
 * (n_q = 1) and the window rows of the next block, whose out_lse is exactly what laserkv_set_row_lse takes:
 * the whole compressed cache then joins the normaliser of Alg. 1 step 3 without being read again by the
 * selection (Sec. 3.2); a caller merging this with its block-local attention uses out_lse as the weight.
 *   q          DEVICE [H_q, n_q, d], strides in elements, d contiguous, rows 16-byte aligned
 *   k_cache, v_cache  DEVICE [H_kv, cap, d] as written by laserkv_append (rows contiguous per head),
 *              cache_stride_head in elements; cache_len rows per head are read, 0 <= cache_len,
 *              cache_len * d * elem size < 2^31
 *   n_q        1 .. max_window of the context's configuration
 *   out        DEVICE [H_q, n_q, d] float, contiguous, 16-byte aligned; zero when cache_len == 0.  May be NULL:
 *              then only out_lse is computed (the values are not read; v_cache may be NULL too), by kernels that
 *              take a GQA group's whole window in one workgroup and read the keys once
 *   out_lse    DEVICE [H_q, n_q] float, contiguous; -inf when cache_len == 0
 *   workspace  DEVICE scratch of at least laserkv_attend_workspace_bytes(ctx, n_q, cache_len) bytes, 256-byte
 *              aligned, owned by the caller; partial results of the key splits, dead after the call's kernels
 * The call allocates nothing and is asynchronous on hip_stream.  Errors: LKV_EINVAL (null / misaligned
 * tensor, n_q or cache_len out of range, workspace too small), LKV_EHIP.
 * laserkv_attend_workspace_bytes returns -1 for arguments the call would reject. */
int64_t laserkv_attend_workspace_bytes(const laserkv_ctx* ctx, int32_t n_q, int64_t cache_len);
int laserkv_attend_cache(laserkv_ctx* ctx,
                         const void* q, int64_t q_stride_head, int64_t q_stride_tok, int32_t n_q,
                         const void* k_cache, const void* v_cache, int64_t cache_stride_head, int64_t cache_len,
                         float* out, float* out_lse,
                         void* workspace, int64_t workspace_bytes,
                         void* hip_stream);

/* The block's own prefill attention (Sec. 3 first paragraph: block t attends to the kept tokens of the earlier
 * blocks and, causally, to itself; Sec. 3.3 "Precision": the exact score is this attention's softmax).  Key
 * order per KV head: the first cache_len cache rows, all visible, then the block's s_t keys, key i (absolute
 * position block_pos0 + i) visible to query j (position q_pos0 + j) iff causal == 0 or block_pos0 + i <=
 * q_pos0 + j.  One softmax per query over both segments: out = sum_i p_i v_i, out_lse = log sum_i exp(q.k_i /
 * sqrt(d)) over the visible keys.  For the window rows out_lse is the COMPLETE statistic that
 * laserkv_set_row_lse_complete takes (call this with the window rows alone, or copy the rows of a whole-block
 * call into a contiguous [H_q, w] tensor): selection then takes one sweep over the block and reads no row
 * statistics of its own.  A query that sees no key gets zero and -inf.
 *   q          DEVICE [H_q, n_q, d], strides in elements, d contiguous, rows 16-byte aligned; 1 <= n_q <= max_block
 *   k_cache, v_cache, cache_stride_head, cache_len   as for laserkv_attend_cache
 *   k_blk, v_blk  DEVICE [H_kv, s_t, d], strides in elements, d contiguous, rows 16-byte aligned;
 *              0 <= s_t <= max_block (0: attention over the cache alone), (s_t + 256) * token stride * elem size < 2^31
 *   out        DEVICE [H_q, n_q, d] float, contiguous, 16-byte aligned (required)
 *   out_lse    DEVICE [H_q, n_q] float, contiguous
 *   workspace  DEVICE scratch of at least laserkv_attend_block_workspace_bytes(ctx, n_q, cache_len, s_t) bytes,
 *              256-byte aligned (256 bytes when a workgroup sees all keys of its rows: the kernel then writes
 *              the result itself; otherwise partial results of the key splits)
 * The call allocates nothing and is asynchronous on hip_stream.  Errors: LKV_EINVAL (null / misaligned tensor,
 * sizes out of range, workspace too small), LKV_EHIP.  laserkv_attend_block_workspace_bytes returns -1 for
 * arguments the call would reject. */
int64_t laserkv_attend_block_workspace_bytes(const laserkv_ctx* ctx, int32_t n_q, int64_t cache_len, int32_t s_t);
int laserkv_attend_block(laserkv_ctx* ctx,
                         const void* q, int64_t q_stride_head, int64_t q_stride_tok, int32_t n_q,
                         const void* k_cache, const void* v_cache, int64_t cache_stride_head, int64_t cache_len,
                         const void* k_blk, int64_t k_stride_head, int64_t k_stride_tok,
                         const void* v_blk, int64_t v_stride_head, int64_t v_stride_tok,
                         int32_t s_t, int64_t block_pos0, int64_t q_pos0, int32_t causal,
                         float* out, float* out_lse,
                         void* workspace, int64_t workspace_bytes,
                         void* hip_stream);

/* Global-consensus variant: Alg. 1 step 3 taken literally, with the exact score summed over every
 * layer and head (Sec. 3.3 "Precision") and, likewise, the collision counts of step 6, followed by
 * ONE two-stage TopK (steps 4-8) whose kept set serves every layer and head.  Three calls:
 *
 * laserkv_score_block: steps a1-a3 of laserkv_select_block for one layer's tensors (same arguments,
 *   same checks), then score_acc[i] (+)= sum over the layer's KV heads of S_exact[h, i] and
 *   count_acc[i] (+)= sum over heads of the collision counts.  accumulate == 0 overwrites the
 *   accumulators (first layer of a block), otherwise adds (every further layer, possibly through other
 *   contexts of the same block length on the same stream).
 *     score_acc  DEVICE [s_t] float, count_acc DEVICE [s_t] int32
 * laserkv_select_consensus: steps a4 on the accumulators; keep_idx DEVICE out [B_t] int32 ascending.
 * laserkv_append_shared: laserkv_append with one index list keep_idx DEVICE [b_t] for every KV head.
 * Errors: as for laserkv_select_block / laserkv_append; LKV_EINVAL for null accumulators. */
int laserkv_score_block(laserkv_ctx* ctx,
                        const void* q_win, int64_t q_stride_head, int64_t q_stride_tok,
                        const void* k_blk, int64_t k_stride_head, int64_t k_stride_tok,
                        const void* k_ctx, int64_t c_stride_head, int64_t c_stride_tok,
                        const void* hyperplanes,
                        int32_t s_t, int32_t w, int32_t t_ctx,
                        int64_t block_pos0, int64_t q_pos0, int32_t causal,
                        float* score_acc, int32_t* count_acc, int32_t accumulate,
                        void* hip_stream);

int laserkv_select_consensus(laserkv_ctx* ctx, const float* score_acc, const int32_t* count_acc, int32_t s_t,
                             int32_t n_anchor, int32_t n_local, int32_t k_exact, int32_t k_lsh,
                             int32_t* keep_idx, void* hip_stream);

int laserkv_append_shared(laserkv_ctx* ctx,
                          const void* k_blk, int64_t k_stride_head, int64_t k_stride_tok,
                          const void* v_blk, int64_t v_stride_head, int64_t v_stride_tok,
                          const int32_t* keep_idx, int32_t b_t, int32_t s_t, int64_t block_pos0,
                          void* k_cache, void* v_cache, int64_t cache_stride_head,
                          int64_t* cache_pos, int64_t pos_stride_head,
                          int64_t cache_len, int64_t cache_cap,
                          void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* LASERKV_H */
