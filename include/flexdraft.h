/*
 * flexdraft.h -- C ABI of the MI355X (gfx950) verify+draft hot path.
 *
 * One decoding step of the method runs a single target forward pass that
 * verifies the previous draft and drafts the next block at once (paper,
 * Sec. 4.1 "Inference").  This library provides the two operations of that
 * pass that are not plain GEMMs:
 *
 *   fd_verify_draft_attn   hybrid-mask attention over a paged KV cache
 *                          (Sec. 4.1 mask rules, Fig. 2b caption)
 *   fd_accept_greedy       lossless acceptance, temperature -> 0 (Sec. 3)
 *   fd_accept_sample       lossless acceptance by speculative sampling (Sec. 3)
 *
 * General conventions
 *   - Plain C.  Every pointer marked "device" is a HIP device pointer on the
 *     current device; pointers marked "host" are ordinary host memory.
 *   - The caller owns every buffer.  The library never allocates or frees device
 *     memory and never synchronises the stream.  The KV cache is read-only to every
 *     call except fd_append_kv, which receives it through separate, writable
 *     pointers.
 *   - All work is enqueued on `hip_stream` (a hipStream_t passed as void*; NULL
 *     is the default stream) and the call returns immediately.
 *   - The return value is the only host-side error channel.  Argument errors are
 *     detected on the host before anything is launched.  fd_last_error() returns
 *     a thread-local description of the last failure.
 *   - Device-side data that contradicts the host-side bounds (a kv_len above
 *     max_kv_len, a page id outside [0, num_pages), a page_indptr entry above
 *     page_indices_len, ...) is clamped by the kernels so that no access leaves
 *     the caller's buffers, and the matching bit is OR-ed into *status if the
 *     call has a status word and one was supplied.  The numerical result of such
 *     a call is unspecified.  The acceptance calls have no status word: a token
 *     id outside [0, vocab) is never used as an index, it counts as a draft that
 *     is not kept.
 *
 * Row convention (shared by all three calls)
 *   Sequence i feeds n_i = k_i + m_i new rows into the pass: first k_i verify
 *   rows (row 0 = the anchor, i.e. the previous step's bonus token, rows
 *   1..k_i-1 = the drafted tokens being verified), then m_i mask-token rows (the
 *   block being drafted).  Rows of all sequences are packed back to back.
 */
#ifndef FLEXDRAFT_H_
#define FLEXDRAFT_H_

#include <stddef.h>
#include <stdint.h>

/* exported symbol */
#define FD_API __attribute__((visibility("default")))

#ifdef __cplusplus
extern "C" {
#endif

typedef enum fd_status {
  FD_OK = 0,
  FD_ERR_INVALID_ARG = 1,         /* null pointer, negative size, inconsistent shapes        */
  FD_ERR_UNSUPPORTED = 2,         /* a shape / dtype this build has no kernel for            */
  FD_ERR_WORKSPACE_TOO_SMALL = 3, /* workspace_bytes below fd_*_workspace()                  */
  FD_ERR_HIP = 4                  /* a HIP runtime call failed (launch error)                */
} fd_status;

typedef enum fd_dtype { FD_F32 = 0, FD_BF16 = 1 } fd_dtype;

/* bits OR-ed into the optional device status word */
#define FD_DEV_KV_LEN_RANGE   1u  /* kv_len[i] < 0 or > max_kv_len                           */
#define FD_DEV_ROWS_RANGE     2u  /* n_i < 0, n_i > max_new_rows, k_i or v_i out of range    */
#define FD_DEV_PAGE_RANGE     4u  /* page id outside [0, num_pages) or page list too short   */

/* fd_attn_args.flags */
#define FD_ATTN_FORCE_GENERIC 1   /* use the scalar fp32-accumulate kernel even for bf16     */
#define FD_ATTN_PLANNED       2   /* the workspace holds fd_verify_draft_plan's plan for these
                                   * arguments: fd_verify_draft_attn starts from it           */

/*
 * Arguments of fd_verify_draft_attn.
 *
 * Operation (Sec. 4.1; Fig. 2b caption).  For sequence i with L_i = kv_len[i]
 * cached prefix tokens, keys are the L_i cached tokens followed by the n_i new
 * rows.  New row r may look at
 *     every cached token;
 *     if r < k_i  (verify row): new rows t <= r        (causal; never a mask token)
 *     if r >= k_i (mask row of block b): new rows t < v_ib, and the rows of its own
 *                               block (both directions); never another block
 * The n_i - k_i mask rows form nb_i = mask_blocks[i] (default 1) blocks of equal
 * length, one candidate draft per hypothetical number of accepted drafts (Sec. 3,
 * parallel speculative decoding; Sec. 4.1: blocks are isolated from one another).
 * Block b is conditioned on the first v_ib = min(v_i + b, k_i) verify rows, with
 * v_i = mask_vis[i] (default k_i - nb_i + 1, so that the last block sees every
 * verify row; with one block: all of them).  The output row is
 *     out[r,h] = sum_j softmax_j(sm_scale * q[r,h].k[j,h/G]) v[j,h/G]   over visible j,
 * G = num_q_heads / num_kv_heads; lse[r,h] (optional) is the natural-log
 * normaliser  log sum_j exp(sm_scale * q.k_j).
 *
 * Layouts (all innermost dimension = head_dim, contiguous):
 *   q, out        [total_rows][num_q_heads][head_dim]        dense
 *   k_new, v_new  [total_rows][num_kv_heads][head_dim]       dense; NOT appended to the cache
 *   k_cache, v_cache: element (page p, kv head g, slot s, d) at
 *       p*cache_stride_page + g*cache_stride_head + s*cache_stride_token + d
 *     strides in elements, each a multiple of 8.  A contiguous cache is the case
 *     page_indices = 0,1,2,...
 *   page_indices[page_indptr[i] .. page_indptr[i+1])  physical pages of sequence i,
 *     in logical order; token p of the sequence lives in page p / page_size,
 *     slot p % page_size.
 *   row_indptr[i] .. row_indptr[i+1]  packed rows of sequence i.
 * dtype applies to q, k_new, v_new, k_cache, v_cache and out.
 */
typedef struct fd_attn_args {
  int32_t batch;              /* B >= 0                                                       */
  int32_t num_q_heads;        /* Hq, multiple of num_kv_heads                                 */
  int32_t num_kv_heads;       /* Hkv                                                          */
  int32_t head_dim;           /* D: multiple of 8, <= 128 (MFMA kernel: 128 or 64)            */
  int32_t page_size;          /* tokens per page, >= 1 (MFMA kernel: power of two >= 16)      */
  int32_t dtype;              /* fd_dtype                                                     */
  float   sm_scale;           /* 0 => 1/sqrt(head_dim)                                        */
  int32_t flags;              /* FD_ATTN_*                                                    */
  /* host-side bounds that fix the launch shape (no device read-back is needed) */
  int32_t total_rows;         /* R = row_indptr[B]                                            */
  int32_t max_kv_len;         /* >= every kv_len[i]                                           */
  int32_t max_new_rows;       /* >= every n_i                                                 */
  int32_t num_pages;          /* physical pages in the pool; page ids are checked against it  */
  int32_t kv_chunk;           /* 0 => automatic.  > 0 (multiple of 64): keys of work handed to
                               * one work-group - the chunk of a sequence's prefix (fp32
                               * kernel) or the share of the batch's key tiles (MFMA kernel) */
  int32_t page_indices_len;   /* entries in page_indices; page_indptr is checked against it.
                               * 0 => not given: page_indptr is then trusted (the one device
                               * array whose extent the kernels cannot otherwise know)       */
  const void *k_cache;        /* device                                                       */
  const void *v_cache;        /* device                                                       */
  int64_t cache_stride_page, cache_stride_head, cache_stride_token;
  const int32_t *page_indptr; /* device [B+1]                                                 */
  const int32_t *page_indices;/* device [page_indptr[B]]                                      */
  const int32_t *kv_len;      /* device [B]                                                   */
  const int32_t *row_indptr;  /* device [B+1]                                                 */
  const int32_t *verify_len;  /* device [B]   k_i in [0, n_i]                                 */
  const int32_t *mask_vis;    /* device [B] or NULL (=> v_i = k_i - nb_i + 1); 0 <= v_i <= k_i */
  const int32_t *mask_blocks; /* device [B] or NULL (=> nb_i = 1); nb_i >= 1 divides n_i - k_i */
  const void *q;              /* device                                                       */
  const void *k_new;          /* device                                                       */
  const void *v_new;          /* device                                                       */
  void  *out;                 /* device                                                       */
  float *lse;                 /* device [total_rows][num_q_heads] or NULL                     */
  void  *workspace;           /* device, 256-byte aligned, >= fd_verify_draft_attn_workspace  */
  size_t workspace_bytes;
  uint32_t *status;           /* device uint32[1] or NULL; caller zeroes it                   */
} fd_attn_args;

/* Bytes of workspace fd_verify_draft_attn needs for these arguments (reads only the
 * host-side scalar fields).  Pure host function; returns 0 on invalid arguments. */
FD_API size_t fd_verify_draft_attn_workspace(const fd_attn_args *args);

/* Hybrid-mask verify+draft attention (Sec. 4.1).  Asynchronous on hip_stream.
 * Errors: FD_ERR_INVALID_ARG, FD_ERR_UNSUPPORTED, FD_ERR_WORKSPACE_TOO_SMALL, FD_ERR_HIP. */
FD_API fd_status fd_verify_draft_attn(const fd_attn_args *args, void *hip_stream);

/*
 * Planning for fd_verify_draft_attn, separated out because it depends on the lengths only and the
 * same lengths meet every layer of the model in one decoding step (Sec. 4.1: one forward pass
 * verifies and drafts; Sec. 4.3).  The bf16 kernel for head_dim 128 or 64 cuts the batch's key tiles into
 * equal shares for its persistent work-groups; the plan is, per work-group, where its share
 * starts (sequence, offset, the page ids of its first two tiles).  Without a plan every work-group
 * of fd_verify_draft_attn finds its share itself, by a scan over the batch, before it can request
 * its first tile; with args->flags & FD_ATTN_PLANNED it starts from the plan this call left in
 * args->workspace, and leaves it intact for the next call.
 *   Read here: the scalar fields, page_indptr, page_indices, kv_len, row_indptr, verify_len,
 *   mask_vis, mask_blocks, workspace, status.  q, k_new, v_new, out and the caches may be NULL.
 *   A planned attention call must pass the same scalar fields, the same (unchanged) length and
 *   page arrays and the same workspace, and needs page_indices_len > 0.  Calls that share a
 *   workspace must not overlap.  For shapes the fp32 kernel serves, planning does nothing and
 *   the flag is ignored.
 * Asynchronous on hip_stream.  Errors as fd_verify_draft_attn.
 */
FD_API fd_status fd_verify_draft_plan(const fd_attn_args *args, void *hip_stream);

/*
 * fd_verify_draft_attn for callers that cannot allocate device memory or hand over a workspace:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, same kernels, same result; args->workspace and args->workspace_bytes are ignored and
 * the split partials go to a buffer of FD_STATIC_SCRATCH_BYTES that is part of the library's device
 * image (every GPU the library runs on holds it until the process ends).  The call allocates and
 * frees nothing.  A call whose fd_verify_draft_attn_workspace() exceeds FD_STATIC_SCRATCH_BYTES is
 * rejected with FD_ERR_WORKSPACE_TOO_SMALL before anything is launched (the MFMA kernel's need is
 * independent of batch and lengths and always fits; the fp32 kernel's grows with rows x chunks).
 * All calls on one GPU share the one buffer: calls that may overlap on a GPU (different streams,
 * different threads) race on it and must be serialised by the caller; calls on one stream are safe.
 * FD_ATTN_PLANNED is ignored (every call finds its shares itself); nothing in the buffer has to
 * survive from call to call, and nothing in it has to start at zero.
 */
#define FD_STATIC_SCRATCH_BYTES ((size_t)44 << 20)
FD_API fd_status fd_verify_draft_attn_static(const fd_attn_args *args, void *hip_stream);

/*
 * Greedy lossless acceptance (Sec. 3, temperature -> 0).
 *
 * target_logits  device [total_rows][row_stride] of dtype dt; only the first
 *                `vocab` entries of a row are read.  Rows are the verify rows of
 *                all sequences, packed; row_indptr[B+1] (device) delimits them.
 * input_tokens   device [total_rows]: the token fed at each verify row.
 * For every row j:  a_j = lowest index attaining max_v target_logits[j][v].
 * For sequence i with k_i rows: accept_len[i] = r_i = number of leading
 * j in [0, k_i-2] with a_j == input_tokens[j+1]; bonus_token[i] = a_{r_i}.
 * The step commits r_i + 1 tokens.  k_i = 0 gives accept_len 0, bonus -1.
 * A token id outside [0, vocab) equals no arg-max: the draft is not kept.
 * row_argmax     device [total_rows] or NULL: receives every a_j.
 * Values are compared exactly as stored; NaN logits are undefined.
 */
FD_API fd_status fd_accept_greedy(const void *target_logits, fd_dtype dt, int64_t row_stride, int32_t vocab,
                           const int32_t *row_indptr, const int32_t *input_tokens,
                           int32_t batch, int32_t total_rows, int32_t max_rows_per_seq,
                           int32_t *accept_len, int32_t *bonus_token, int32_t *row_argmax,
                           void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Speculative-sampling acceptance with caller-supplied uniforms (Sec. 3).
 *
 * p_j = softmax(target_logits[j] / temperature), q_j = softmax(draft_logits[j] /
 * temperature); draft row j is the distribution the token fed at row j+1 was drawn
 * from.  Each sequence's last draft row judges no token and cannot change the result,
 * but it is read like the others: all total_rows rows of draft_logits must be
 * readable and free of NaN.  For j = 0 .. k_i-2 with
 * d = input_tokens[j+1]: keep d iff u_accept[j] * q_j(d) < p_j(d) (a token id outside
 * [0, vocab) is not kept); stop at the first row j* that fails.  The bonus token is drawn from the residual
 * max(0, p_j* - q_j*) (from p_{k_i-1} when every draft was kept; from p_j* if the
 * residual is identically zero) by inverse CDF in ascending token order: the first
 * token whose inclusive cumulative weight exceeds u_resample[j*] * total weight.
 * accept_len[i] = j*.  u_accept, u_resample: device [total_rows] float in [0,1).
 * Sums are accumulated in fp64 from fp32 exponentials; a decision whose exact
 * margin is below about 1e-6 (relative) may fall on either side.
 */
FD_API fd_status fd_accept_sample(const void *target_logits, const void *draft_logits, fd_dtype dt,
                           int64_t row_stride, int32_t vocab, float temperature,
                           const int32_t *row_indptr, const int32_t *input_tokens,
                           const float *u_accept, const float *u_resample,
                           int32_t batch, int32_t total_rows, int32_t max_rows_per_seq,
                           int32_t *accept_len, int32_t *bonus_token,
                           void *workspace, size_t workspace_bytes, void *hip_stream);

/* Workspace bytes for the acceptance calls (sampling != 0 for fd_accept_sample); 0 on invalid arguments. */
FD_API size_t fd_accept_workspace(int32_t batch, int32_t total_rows, int32_t vocab, int32_t sampling);

/*
 * Draft tokens of a mask block and how many of them are worth verifying: selective verification
 * (Sec. 4.3, Eq. 5) fused with the token pick, one pass over the drafter's logits.
 *   draft_logits  device [total_rows][vocab] (row stride in elements): row j of a sequence holds
 *                 the logits of draft position j+1; rows are packed per sequence by row_indptr
 *   draft_tokens  device int32 [total_rows]: arg-max of each row (lowest index on ties)
 *   confidence    device float [total_rows] or NULL: p_j = softmax(x_j / temperature)[token]
 *   keep_len      device int32 [B]: number of leading positions i with p_1 ... p_i >= threshold
 *                 (the estimate of P(accepted length >= i)); the first position below the
 *                 threshold and everything after it is pruned.  The next step verifies
 *                 1 + keep_len[i] rows: the anchor and the kept drafts.
 * temperature > 0; threshold in [0, 1] is useful (0 keeps everything), any finite value accepted.
 * Workspace: fd_draft_select_workspace(total_rows, vocab) bytes, device, 256-byte aligned.
 * Asynchronous on hip_stream.  Errors: FD_ERR_INVALID_ARG, FD_ERR_WORKSPACE_TOO_SMALL, FD_ERR_HIP.
 */
FD_API fd_status fd_draft_select(const void *draft_logits, fd_dtype dt, int64_t row_stride, int32_t vocab,
                                 float temperature, float threshold, const int32_t *row_indptr,
                                 int32_t batch, int32_t total_rows, int32_t max_rows_per_seq,
                                 int32_t *draft_tokens, float *confidence, int32_t *keep_len,
                                 void *workspace, size_t workspace_bytes, void *hip_stream);
FD_API size_t fd_draft_select_workspace(int32_t total_rows, int32_t vocab);

/*
 * Commit of the verified rows to the paged KV cache (Sec. 4.3, decoupled execution: the cache
 * written by target verification is what the next draft step reuses).  Sequence i commits its
 * anchor row and its first accept_len[i] drafts, i.e. new rows 0 .. accept_len[i] of
 * args->k_new / v_new; row j is written to logical position kv_len[i] + j (page
 * page_indices[page_indptr[i] + pos / page_size], slot pos % page_size), so the sequence's
 * page list must already hold the pages for them.  The bonus token has no K/V yet: it is the
 * next step's anchor.  Only verify rows are ever written (mask tokens stay invisible to the
 * clean prefix, Sec. 4.1): a sequence with k_i = 0 -- a mask-only draft pass -- commits nothing
 * and keeps its length.
 *   args          the fd_attn_args of the attention call that produced the rows; read here:
 *                 batch, num_kv_heads, head_dim, page_size, dtype, total_rows, max_new_rows,
 *                 num_pages, the three strides, page_indptr, page_indices, kv_len, row_indptr,
 *                 verify_len, k_new, v_new, status.  args->k_cache / v_cache are NOT used.
 *   k_cache, v_cache  device, WRITTEN: the cache the rows go to, in the layout the strides
 *                 describe (normally the buffers args->k_cache / v_cache point to)
 *   accept_len    device int32 [B], 0 <= accept_len[i] < k_i
 *   kv_len_out    device int32 [B]: kv_len[i] + accept_len[i] + 1 (kv_len[i] when k_i = 0);
 *                 may be args->kv_len itself
 * Out-of-range device data (a page list too short, a page id outside the pool, accept_len
 * outside [0, k_i)) is skipped or clamped and reported through args->status like in
 * fd_verify_draft_attn.  Asynchronous on hip_stream.  Errors: FD_ERR_INVALID_ARG, FD_ERR_HIP.
 */
FD_API fd_status fd_append_kv(const fd_attn_args *args, void *k_cache, void *v_cache,
                              const int32_t *accept_len, int32_t *kv_len_out, void *hip_stream);

/*
 * Branch selection of parallel speculative decoding (Sec. 3): the forward pass prepared one
 * candidate block per hypothetical number of accepted drafts; once acceptance has fixed that
 * number, the block drafted under it becomes the next draft.
 *   block_tokens  device int32 [total_tokens]: the drafted tokens of every block; sequence i
 *                 owns block_indptr[i] .. block_indptr[i+1], its nb_i = mask_blocks[i] blocks
 *                 of equal length back to back
 *   first_vis     device int32 [B] or NULL: verify rows block 0 was conditioned on, i.e. the
 *                 attention call's mask_vis; block b assumed first_vis[i] + b - 1 accepted drafts
 *   verify_len    device int32 [B], needed when first_vis is NULL (else may be NULL): the
 *                 attention call's verify_len.  first_vis then takes the attention call's own
 *                 default, max(k_i - nb_i + 1, 0), so that passing NULL to both calls pairs up
 *   accept_len    device int32 [B]: accepted drafts r_i (fd_accept_greedy / fd_accept_sample)
 *   out_tokens    device int32 [B][out_stride]: the chosen block, padded with -1
 *   out_block     device int32 [B] or NULL: index of the chosen block
 * The block index r_i + 1 - first_vis[i] is clamped to the blocks that exist.  A sequence
 * whose tokens do not split into nb_i >= 1 blocks, or whose block is longer than out_stride,
 * gets -1 everywhere.  Asynchronous on hip_stream.  Errors: FD_ERR_INVALID_ARG, FD_ERR_HIP.
 */
FD_API fd_status fd_select_branch(const int32_t *block_tokens, const int32_t *block_indptr,
                                  const int32_t *mask_blocks, const int32_t *accept_len,
                                  const int32_t *first_vis, const int32_t *verify_len,
                                  int32_t batch, int32_t total_tokens,
                                  int32_t out_stride, int32_t *out_tokens, int32_t *out_block,
                                  void *hip_stream);

/* Thread-local description of the last error returned on this thread ("" if none). */
FD_API const char *fd_last_error(void);

/* Library version string, e.g. "flexdraft-gfx950 0.1". */
FD_API const char *fd_version(void);

#ifdef __cplusplus
}
#endif
#endif /* FLEXDRAFT_H_ */
