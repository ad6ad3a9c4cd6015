/*
 * libskipkv — the periodic sentence-level KV-cache compression step of SkipKV
 * (Sec. 4.1 "Skipping KV Storage with Sentence-level Scoring", Alg. 1 eviction line)
 * and the steering-vector injection (Sec. 4.2), for AMD MI355X (gfx950).
 *
 * Conventions shared by every entry point
 * ---------------------------------------
 *  - Plain C ABI.  Every call returns an int status: SKIPKV_OK (0) or a negative code;
 *    skipkv_strerror() names it.  No exceptions, no global state, no environment variables.
 *  - Pointers marked "device" must be GPU-accessible memory owned by the caller and must
 *    stay valid until the work enqueued by the call has finished.  The library never
 *    allocates or frees device memory; scratch space comes from the caller's workspace
 *    (size from skipkv_workspace_bytes).
 *  - All GPU work is enqueued on the caller's stream (`stream` is a hipStream_t passed as
 *    void*; NULL is the default stream).  No call synchronises the device: outputs are
 *    valid after the caller synchronises the stream.  Argument structs are read before
 *    the call returns.
 *  - Arguments are validated on the host before anything is enqueued; on a validation
 *    error nothing has been launched.  Problems only visible on the device (non-monotone
 *    sentence offsets, more sentences per chunk of work than the kernels support) are
 *    reported by OR-ing SKIPKV_DEV_* bits into *params->dev_status when it is non-NULL.
 *  - Re-entrant for calls that use distinct buffers, workspaces and streams.
 *
 * Data layout
 * -----------
 *  A "head" is one (layer l, KV head h, sequence b) triple.  Sequences are stored
 *  unpadded, one after another along the token axis (CSR offsets seq_off), the same
 *  packing for every layer and head.  Element (l, h, t, d) of K (or V), t being the
 *  packed token index, lives at  base + l*stride_layer + h*stride_head + t*stride_tok + d
 *  (strides in elements, d contiguous, head_dim = 128).
 *  Sentence spans are per sequence and shared by all layers and heads: sequence b has
 *  S_b = sent_ptr[b+1]-sent_ptr[b]-1 sentences; sentence s is the half-open token span
 *  [o[s], o[s+1]) with o = sent_off + sent_ptr[b], relative to the start of the sequence,
 *  o[0] = 0, o[S_b] = N_b (the cache length of b), strictly ascending.
 *  Per-sentence arrays are laid out [n_layers, n_kv_heads, total_sentences]; sentence s of
 *  sequence b is at column sent_ptr[b] - b + s.  Per-token arrays are
 *  [n_layers, n_kv_heads, total_tokens] with column seq_off[b] + t.
 */
#ifndef SKIPKV_H
#define SKIPKV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SKIPKV_VERSION 101 /* major*10000 + minor*100 + patch */

enum {
  SKIPKV_OK = 0,
  SKIPKV_EINVAL = -1,     /* null pointer, bad shape, stride, alignment or dtype          */
  SKIPKV_EBUDGET = -2,    /* budget < protect_window, or obs_window > protect_window      */
  SKIPKV_ECAPACITY = -3,  /* shape outside what the kernels are built for (see limits)    */
  SKIPKV_EWORKSPACE = -4, /* workspace NULL, misaligned or smaller than required          */
  SKIPKV_EHIP = -5        /* a HIP runtime call failed (launch error)                     */
};

/* bits OR-ed into *dev_status by kernels */
enum {
  SKIPKV_DEV_BAD_OFFSETS = 1,  /* sentence offsets not strictly ascending from 0 to N_b   */
  SKIPKV_DEV_TOO_MANY_SENT = 2, /* a sequence has more than SKIPKV_MAX_SENTENCES sentences */
  SKIPKV_DEV_TIMEOUT = 4,       /* a bounded cross-workgroup wait ran out: the heads concerned were done by the two-pass scan (results valid, the call slower) */
  SKIPKV_DEV_TOO_MANY_TOK = 8,  /* skipkv_select_tokens: a sequence is longer than SKIPKV_MAX_TOKENS_TOKEN_SELECT */
  SKIPKV_DEV_BAD_BLOCK_TABLE = 16, /* paged cache: a block id outside [0, n_blocks); that sequence's K/V are left untouched */
  SKIPKV_DEV_BAD_BUDGET = 32,   /* a device budget below the protected window, negative, or too large for kept_stride */
  SKIPKV_DEV_BAD_SCORES = 64    /* selection: a candidate sentence's score is NaN                 */
};
/*
 * A head (layer, KV head, sequence) that one of these bits concerns is never compacted from
 * inputs the library could not trust: the selections give it new_len = N_b (everything kept),
 * kept_idx = the identity as far as the row reaches, sent_keep = 1 and unchanged ranges, and the
 * compaction leaves its K and V rows alone (it also skips any head whose new_len exceeds
 * kept_stride).  The other heads of the call are processed normally.
 */

typedef enum { SKIPKV_F32 = 0, SKIPKV_BF16 = 1 } skipkv_dtype;

/* Limits of this build. */
#define SKIPKV_HEAD_DIM 128
#define SKIPKV_MAX_GROUP 8        /* n = n_q_heads / n_kv_heads                           */
#define SKIPKV_MAX_OBS_WINDOW 32  /* alpha                                                */
#define SKIPKV_MAX_SENTENCES 4096 /* per sequence                                         */
#define SKIPKV_MAX_TOKENS_TOKEN_SELECT 131072 /* per sequence, token-level selection only   */

/* The KV cache and its ragged structure (Sec. 4.1: K, V in R^{bs x H_k x N' x d}). */
typedef struct skipkv_cache {
  void *k;               /* device, rewritten in place by skipkv_compact / skipkv_step    */
  void *v;               /* device, same layout as k                                      */
  int64_t stride_layer;  /* elements; multiples of 8 so that every row is 16-byte aligned */
  int64_t stride_head;
  int64_t stride_tok;    /* >= head_dim                                                   */
  int32_t dtype;         /* skipkv_dtype of k, v and the observation queries              */
  int32_t n_layers;
  int32_t n_kv_heads;    /* H_k                                                           */
  int32_t n_q_heads;     /* H_q, a multiple of H_k; query head i uses KV head i / n       */
  int32_t head_dim;      /* must be 128                                                   */
  int32_t batch;         /* number of sequences                                           */
  int32_t total_tokens;  /* host copy of seq_off[batch]                                   */
  int32_t total_sentences; /* host copy of sum_b S_b                                      */
  const int32_t *seq_off;  /* device [batch+1], seq_off[0] = 0                            */
  const int32_t *sent_ptr; /* device [batch+1], sent_ptr[0] = 0                           */
  const int32_t *sent_off; /* device [total_sentences + batch]                            */
} skipkv_cache;

/* Scalars of the method (Appendix "Hyper-parameters": sigma = 0.1, tau in [0.95, 0.99]). */
typedef struct skipkv_params {
  int32_t obs_window;     /* alpha: number of recent query positions that score the cache */
  int32_t protect_window; /* w >= alpha: the last min(w, N_b) tokens are never evicted     */
  float sigma;            /* weight of the importance term in the cumulative score (Eq. 6) */
  float tau;              /* similarity threshold of the redundant set (Eq. 3), strict >   */
  const int32_t *budget;  /* device [batch] per-sequence token budget, or NULL ...         */
  int32_t budget_scalar;  /* ... then this budget applies to every sequence                */
  int32_t max_budget;     /* host upper bound on any budget (sizes kept_idx rows)          */
  int32_t *dev_status;    /* device, nullable: SKIPKV_DEV_* bits are OR-ed into it         */
  void *profile;          /* nullable: handle from skipkv_profile_create                   */
  uint32_t flags;         /* SKIPKV_FLAG_* bits, 0 for the defaults                        */
  int32_t spin_limit;     /* polls that a cross-workgroup wait of the single-pass key scan may
                             take before it gives up: 0 = default (4000000), negative = give
                             up at the first poll (for tests of the time-out path)          */
} skipkv_params;
#define SKIPKV_FLAG_FORCE_TWO_PASS 1u /* read K twice: statistics pass + score pass, no waits across workgroups */

/* Bytes of device scratch that skipkv_score / skipkv_step need for this problem.         */
int skipkv_workspace_bytes(const skipkv_cache *cache, const skipkv_params *params, size_t *out_bytes);

/*
 * Scores (Sec. 4.1, Eq. 1-4 and Eq. 6).  Per head:
 *   token importance I[t]: softmax over the cached keys of q.k/sqrt(d) for each of the n
 *     query heads of the GQA group and each of the alpha window queries (window query a
 *     sits at cache position N-alpha+a and sees keys t <= N-alpha+a), max over the n heads,
 *     mean over the alpha queries;
 *   sentence embedding: mean of the head's keys over the sentence; lambda_s = largest
 *     cosine between sentence s and any LATER sentence (-inf for the last one);
 *   sent_score[s] = sigma * mean_t I[t] - (1-sigma) * mean_t R[t] - (lambda_s if lambda_s > tau),
 *     means over the part of s that lies before the protected window; +inf for sentences
 *     that start inside the protected window.
 * q_obs           device [n_layers, batch, n_q_heads, obs_window, 128], cache dtype.
 * tok_redundancy  device [n_layers, n_kv_heads, total_tokens] fp32 or NULL (R = 0).
 * sent_score, sent_lambda   device out [n_layers, n_kv_heads, total_sentences] fp32.
 * tok_importance  device out [n_layers, n_kv_heads, total_tokens] fp32, or NULL.
 * The key scan reads K once where it can (query rows n * obs_window <= 64 after padding, no
 * sentence longer than 128 tokens, at most 256 work items of up to 512 tokens per sequence, i.e.
 * about 120000 tokens) and twice otherwise.  Its single-pass form is a persistent grid that must
 * have the GPU's compute units to itself (work of other streams running at the same time can
 * only be waited out).  It waits across workgroups; the wait is bounded (params->spin_limit): on
 * expiry SKIPKV_DEV_TIMEOUT is OR-ed into dev_status, every later wait of the call gives up at
 * once, and the heads concerned are flagged and done again by the two-pass kernels that follow in
 * the stream: the call completes with valid results, only slower (the bit tells the caller that the
 * GPU was not the call's alone).  SKIPKV_FLAG_FORCE_TWO_PASS selects the two-pass form for every
 * sequence.
 * ws              device workspace, 256-byte aligned, >= skipkv_workspace_bytes().
 */
int skipkv_score(const skipkv_cache *cache, const skipkv_params *params, const void *q_obs,
                 const float *tok_redundancy, float *sent_score, float *sent_lambda,
                 float *tok_importance, void *ws, size_t ws_bytes, void *stream);

/*
 * Budgeted whole-sentence selection (Sec. 4.1 after Eq. 6: evict in increasing order of
 * the score until the budget is met; surviving index set P of the range-remap paragraph).
 * Per head: if N_b <= budget everything is kept.  Otherwise candidates (sentences that
 * start before the protected window, counted with their unprotected length) are ranked by
 * (score descending, sentence index descending) and the longest prefix of that ranking
 * whose lengths sum to <= budget - min(w, N_b) is kept, plus the protected window.
 * sent_keep     device out [n_layers, n_kv_heads, total_sentences] u8, nullable: 1 if the
 *               unprotected part of the sentence survives (1 for non-candidates).
 * kept_idx      device out [n_layers, n_kv_heads, batch, kept_stride] int32: ascending
 *               sequence-relative indices of the surviving tokens, new_len entries valid.
 * new_len       device out [n_layers, n_kv_heads, batch] int32.
 * new_sent_off  device out [n_layers, n_kv_heads, total_sentences + batch] int32, nullable:
 *               offsets of the surviving sentences in the compacted cache (Eq. 11), stored
 *               at column sent_ptr[b]; new_sent_cnt [n_layers, n_kv_heads, batch] holds
 *               their number (both NULL or both non-NULL).
 * kept_stride   row pitch of kept_idx, >= min(max_budget, total_tokens).
 */
int skipkv_select(const skipkv_cache *cache, const skipkv_params *params, const float *sent_score,
                  uint8_t *sent_keep, int32_t *kept_idx, int32_t *new_len, int32_t *new_sent_off,
                  int32_t *new_sent_cnt, int32_t kept_stride, void *stream);

/*
 * In-place compaction (Alg. 1 eviction line): for every head and k < new_len,
 * K[k] <- K[kept_idx[k]] and V[k] <- V[kept_idx[k]], bit for bit.  kept_idx rows must be
 * strictly ascending (so kept_idx[k] >= k).  Rows at and beyond new_len are unspecified
 * afterwards.  Only cache->k, v, strides, dtype, shape and seq_off are used.
 */
int skipkv_compact(const skipkv_cache *cache, const int32_t *kept_idx, const int32_t *new_len,
                   int32_t kept_stride, void *stream);

/* score + select + compact enqueued back to back with no host round trip in between.     */
int skipkv_step(const skipkv_cache *cache, const skipkv_params *params, const void *q_obs,
                const float *tok_redundancy, float *sent_score, float *sent_lambda,
                float *tok_importance, uint8_t *sent_keep, int32_t *kept_idx, int32_t *new_len,
                int32_t *new_sent_off, int32_t *new_sent_cnt, int32_t kept_stride, void *ws,
                size_t ws_bytes, void *stream);

/*
 * skipkv_step for callers that cannot allocate device memory or pass a workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same computation,
 * arguments and outputs as skipkv_step, but the scratch space is an array of
 * SKIPKV_STATIC_WS_BYTES that the library's code object holds on every GPU it is loaded on until the
 * process ends.  Nothing is allocated or freed, by this library or through it.  A problem whose
 * skipkv_workspace_bytes() exceeds SKIPKV_STATIC_WS_BYTES is refused with SKIPKV_EWORKSPACE and
 * nothing is enqueued.  The first call on a device looks the array's address up (not while a
 * stream is capturing: make one call before capture starts).  All calls on one GPU share the
 * array: calls whose enqueued work may overlap on that GPU race (serialise them on one stream,
 * or order the streams with events); the contents the previous call left are reset by the
 * step's own kernels where they matter.
 */
#define SKIPKV_STATIC_WS_BYTES (64u << 20)
int skipkv_step_static(const skipkv_cache *cache, const skipkv_params *params, const void *q_obs,
                       const float *tok_redundancy, float *sent_score, float *sent_lambda,
                       float *tok_importance, uint8_t *sent_keep, int32_t *kept_idx, int32_t *new_len,
                       int32_t *new_sent_off, int32_t *new_sent_cnt, int32_t kept_stride, void *stream);

/*
 * Token-level selection: Eq. 6 as printed and the rule after it ("evict tokens in increasing
 * order of the final score").  Per head and token t of sentence s:
 *   tok_score[t] = sigma * I[t] - (1 - sigma) * R[t] - (lambda_s if lambda_s > tau)
 * The last min(protect_window, N) tokens are kept; if N > budget, the other tokens are ranked by
 * (score descending, index descending) and exactly budget - window of them are kept.  Sentence
 * ranges follow Eq. 11: new_sent_off / new_sent_cnt list the sentences that still have a token.
 * The outputs have the layout of skipkv_select and feed skipkv_compact unchanged.
 * tok_importance  device [n_layers, n_kv_heads, total_tokens] fp32 (from skipkv_score).
 * tok_redundancy  device, same shape, or NULL (R = 0).   sent_lambda  device (from skipkv_score).
 * tok_score       device out, same shape, required (also the kernel's working copy).
 * tok_keep        device out [n_layers, n_kv_heads, total_tokens] u8, or NULL.
 * A sequence longer than SKIPKV_MAX_TOKENS_TOKEN_SELECT is reported (SKIPKV_DEV_TOO_MANY_TOK in
 * dev_status) and keeps everything, like any head whose inputs cannot be used (see SKIPKV_DEV_*).
 */
int skipkv_select_tokens(const skipkv_cache *cache, const skipkv_params *params, const float *tok_importance,
                         const float *tok_redundancy, const float *sent_lambda, float *tok_score,
                         uint8_t *tok_keep, int32_t *kept_idx, int32_t *new_len, int32_t *new_sent_off,
                         int32_t *new_sent_cnt, int32_t kept_stride, void *stream);

/*
 * Per-head sentence ranges across steps (Sec. 4.1 "KV Cache Sentence Range Monitoring Logic": the ranges M^(cs) and
 * cache lengths l_t^(cs) of Eq. 9-11 and Alg. 1).  After a step every (layer, KV head, sequence)
 * has evicted sentences of its own, so lengths and ranges are per head from then on:
 *   len       device [n_layers, n_kv_heads, batch]   cache length N of every head's sequence
 *   sent_cnt  device [n_layers, n_kv_heads, batch]   its number of sentences S
 *   sent_off  device [n_layers, n_kv_heads, total_sentences + batch]   its S+1 offsets, stored where
 *             the shared layout would keep those of sequence b (at sent_ptr[b] of the head's row)
 * These are exactly the new_len / new_sent_cnt / new_sent_off outputs of the previous step (Eq. 11
 * is applied there).  The cache's seq_off, sent_ptr, total_tokens and total_sentences keep their
 * meaning as ROOM: sequence b of every head lives in rows seq_off[b] .. seq_off[b+1] and may hold at
 * most sent_ptr[b+1]-sent_ptr[b]-1 sentences; cache->sent_off is not read.
 */
typedef struct skipkv_ranges {
  int32_t *len;
  int32_t *sent_cnt;
  int32_t *sent_off;
} skipkv_ranges;

/*
 * Eq. 10: n_new[b] tokens have been appended to sequence b of every head (the caller has written
 * their K and V rows at rows seq_off[b] + len .. of each head).  bnd_off[bnd_ptr[b] .. bnd_ptr[b+1])
 * lists, strictly ascending, the positions 0 <= p < n_new[b] inside the appended run at which a new
 * sentence starts (the token after a delimiter); tokens before the first such position continue
 * the head's last sentence.  Positions are cache positions: the shift by the number of evicted
 * tokens that the paper writes out is contained in len.  Updates ranges in place.  A head whose
 * room (tokens or sentences) would overflow, or bad boundaries, are reported in *dev_status
 * (SKIPKV_DEV_TOO_MANY_SENT / SKIPKV_DEV_BAD_OFFSETS) and that head is left unchanged.
 * n_new, bnd_ptr [batch+1], bnd_off: device.  dev_status: device, nullable.
 */
int skipkv_ranges_append(const skipkv_cache *cache, const skipkv_ranges *ranges, const int32_t *n_new,
                         const int32_t *bnd_ptr, const int32_t *bnd_off, int32_t *dev_status, void *stream);

/* Workspace of skipkv_step_ranges for this problem (larger than skipkv_workspace_bytes).       */
int skipkv_ranges_workspace_bytes(const skipkv_cache *cache, const skipkv_params *params, size_t *out_bytes);

/*
 * skipkv_step for caches with per-head ranges: same computation, outputs and layouts, with every
 * head's own length and sentence ranges as input.  Needs K and V contiguous over (layer, head,
 * token): stride_head = total_tokens * stride_tok, stride_layer = n_kv_heads * stride_head, else
 * SKIPKV_ECAPACITY.  params->budget, if not NULL, has one entry per (layer, KV head, sequence).
 * The outputs new_len / new_sent_off / new_sent_cnt must not alias the input ranges.
 */
int skipkv_step_ranges(const skipkv_cache *cache, const skipkv_ranges *ranges, const skipkv_params *params,
                       const void *q_obs, const float *tok_redundancy, float *sent_score, float *sent_lambda,
                       float *tok_importance, uint8_t *sent_keep, int32_t *kept_idx, int32_t *new_len,
                       int32_t *new_sent_off, int32_t *new_sent_cnt, int32_t kept_stride, void *ws, size_t ws_bytes,
                       void *stream);

/*
 * The token-level flow on per-head ranges (Sec. 4.1: Eq. 5, Eq. 6 as printed, ranges per Eq. 11,
 * repeated over the steps of a decode): the counterparts of skipkv_token_redundancy,
 * skipkv_score and skipkv_select_tokens that take every head's own length and sentence ranges.
 * Arguments, outputs and layouts are those of the shared-range calls; values at and beyond a
 * head's length (tokens) or count (sentences) are unspecified.  skipkv_compact serves per-head
 * ranges as it is (kept_idx and new_len are per head already).
 * skipkv_token_redundancy_ranges: R over the first ranges->len tokens of every head (only
 *   ranges->len is read); ws as for skipkv_token_redundancy.
 * skipkv_score_ranges: needs K contiguous over (layer, head, token) like skipkv_step_ranges; ws of
 *   at least skipkv_ranges_workspace_bytes, 256-byte aligned.
 * skipkv_select_ranges (the sentence-level selection of skipkv_step_ranges on its own, for scores
 *   that come from skipkv_score_ranges or skipkv_score_shared_ranges) and
 * skipkv_select_tokens_ranges: ws of at least skipkv_ranges_workspace_bytes (only its head is
 *   used), 256-byte aligned; params->budget, if not NULL, has one entry per (layer, KV head,
 *   sequence); new_len / new_sent_off / new_sent_cnt must not alias the input ranges.
 */
int skipkv_token_redundancy_ranges(const skipkv_cache *cache, const skipkv_ranges *ranges, float *tok_redundancy,
                                   void *ws, size_t ws_bytes, void *stream);
int skipkv_score_ranges(const skipkv_cache *cache, const skipkv_ranges *ranges, const skipkv_params *params,
                        const void *q_obs, const float *tok_redundancy, float *sent_score, float *sent_lambda,
                        float *tok_importance, void *ws, size_t ws_bytes, void *stream);
int skipkv_select_ranges(const skipkv_cache *cache, const skipkv_ranges *ranges, const skipkv_params *params,
                         const float *sent_score, uint8_t *sent_keep, int32_t *kept_idx, int32_t *new_len,
                         int32_t *new_sent_off, int32_t *new_sent_cnt, int32_t kept_stride, void *ws, size_t ws_bytes,
                         void *stream);
int skipkv_select_tokens_ranges(const skipkv_cache *cache, const skipkv_ranges *ranges, const skipkv_params *params,
                                const float *tok_importance, const float *tok_redundancy, const float *sent_lambda,
                                float *tok_score, uint8_t *tok_keep, int32_t *kept_idx, int32_t *new_len,
                                int32_t *new_sent_off, int32_t *new_sent_cnt, int32_t kept_stride, void *ws,
                                size_t ws_bytes, void *stream);

/*
 * Sentence similarity from the last layer's hidden states (Sec. 4.1 "Sentence Similarity Score",
 * Eq. 1-3 as printed): v_s = mean of the hidden states over the tokens of sentence s,
 * shared_lambda[s] = largest cosine between v_s and the embedding of a LATER sentence of the same
 * sequence (-inf for the last one): one value per sentence, shared by all layers and heads.
 * Uses cache->batch, seq_off, sent_ptr, sent_off, total_tokens, total_sentences (at most
 * SKIPKV_MAX_SENTENCES sentences per sequence; K and V are not touched).
 * hidden         device [total_tokens, d_model], rows packed like the cache's token axis; dtype is
 *                SKIPKV_BF16 or SKIPKV_F32; d_model a multiple of 128; 16-byte aligned.
 * shared_lambda  device out [total_sentences] fp32 (sentence s of sequence b at sent_ptr[b]-b+s).
 * ws             device workspace, 256-byte aligned, >= skipkv_similarity_workspace_bytes().
 */
int skipkv_similarity_workspace_bytes(const skipkv_cache *cache, int32_t d_model, size_t *out_bytes);
int skipkv_sentence_similarity(const skipkv_cache *cache, const void *hidden, int32_t d_model, int32_t dtype,
                               float *shared_lambda, void *ws, size_t ws_bytes, void *stream);

/*
 * skipkv_score with the similarity term taken from shared_lambda (one value per sentence of a
 * sequence, e.g. from skipkv_sentence_similarity) instead of per-head key embeddings: the key
 * scan only computes the token importance, no per-head Gram matrices are formed.  sent_lambda
 * (nullable) receives a per-head copy of shared_lambda.  Everything else as skipkv_score, same
 * workspace; follow with skipkv_select and skipkv_compact.
 */
int skipkv_score_shared(const skipkv_cache *cache, const skipkv_params *params, const void *q_obs,
                        const float *tok_redundancy, const float *shared_lambda, float *sent_score,
                        float *sent_lambda, float *tok_importance, void *ws, size_t ws_bytes, void *stream);

/*
 * The shared lambda on per-head ranges, i.e. skipkv_score_shared at every step after the first.
 * A head's surviving sentences are a subsequence of its sequence's own list of sentences (all
 * sentences generated so far, which is what the hidden-state similarity is computed over), so
 * every head carries the numbers its sentences have in that list:
 *   sent_id  device int32 [n_layers, n_kv_heads, total_sentences], laid out like sent_keep.
 * skipkv_ranges_ids_select: after a sentence-level selection, sent_id_out = the numbers of the
 *   sentences that survive it, in order: those with sent_keep != 0 and those that reach into the
 *   protected window (their tail stays).  ranges = the ranges the selection ran on (NULL: the
 *   shared ones of cache, the first step), protect_window that of the selection; sent_id_in
 *   NULL: a sentence's number is its position (the first step).  sent_id_out may be sent_id_in.
 *   As many numbers are written per head as the selection's new_sent_cnt says.
 * skipkv_ranges_ids_append: after skipkv_ranges_append, sentences old_cnt .. new_cnt-1 of every
 *   head continue the numbering after the head's last old sentence (which every selection keeps,
 *   so it is the sequence's last): old_cnt = a copy of the counts from before the append.
 * skipkv_score_shared_ranges: skipkv_score_shared with per-head ranges; lambda of a head's
 *   sentence is shared_lambda[lambda_ptr[b] + its number]; lambda_ptr is a device int32
 *   [batch + 1] CSR over the sequences' own lists (a number outside a sequence's list raises
 *   SKIPKV_DEV_BAD_OFFSETS and reads as -inf).  Needs K contiguous over (layer, head, token); ws
 *   of at least skipkv_ranges_workspace_bytes, 256-byte aligned.  skipkv_select_ranges and
 *   skipkv_compact complete the step.
 */
int skipkv_ranges_ids_select(const skipkv_cache *cache, const skipkv_ranges *ranges, int32_t protect_window,
                             const uint8_t *sent_keep, const int32_t *sent_id_in, int32_t *sent_id_out, void *stream);
int skipkv_ranges_ids_append(const skipkv_cache *cache, const int32_t *old_cnt, const int32_t *new_cnt, int32_t *sent_id,
                             void *stream);
int skipkv_score_shared_ranges(const skipkv_cache *cache, const skipkv_ranges *ranges, const int32_t *sent_id,
                               const int32_t *lambda_ptr, const skipkv_params *params, const void *q_obs,
                               const float *tok_redundancy, const float *shared_lambda, float *sent_score,
                               float *sent_lambda, float *tok_importance, void *ws, size_t ws_bytes, void *stream);

/*
 * Token redundancy (Sec. 4.1 "Token Redundancy Score", Eq. 5).  Per head, with Kbar the rows of
 * K scaled to unit length (1e-12 added to the norm):
 *   R[t] = mean over rows i of softmax_j(Kbar Kbar^T)[i, t]
 * (softmax along each row of the cosine matrix, mean over the rows; the diagonal is kept; no
 * causal mask).  R sums to 1 over the tokens of a head.  Cost is quadratic in the cache length:
 * 2 N^2 dot products of length 128 per head.  The dot products are taken in bf16 (fp32 caches
 * are rounded to bf16 for this call), accumulated in fp32.  The result can be handed to
 * skipkv_score / skipkv_step as tok_redundancy.
 * tok_redundancy  device out [n_layers, n_kv_heads, total_tokens] fp32.
 * ws, ws_bytes    device scratch of at least skipkv_redundancy_workspace_bytes, 256-byte aligned.
 * Uses cache->k, strides, dtype, n_layers, n_kv_heads, batch, total_tokens, seq_off only.
 */
int skipkv_redundancy_workspace_bytes(const skipkv_cache *cache, size_t *out_bytes);
int skipkv_token_redundancy(const skipkv_cache *cache, float *tok_redundancy, void *ws, size_t ws_bytes,
                            void *stream);

/*
 * Paged KV cache (Appendix, "System-Level Evaluation on vLLM": continuous batching with a paged
 * KV cache).  K and V are pools of blocks of block_size token slots, and logical token t of
 * sequence b lives in block block_table[b * table_stride + t / block_size] at slot
 * t % block_size:
 *   element offset of (layer l, KV head h, block p, slot s) =
 *       l * cache->stride_layer + h * cache->stride_head + p * stride_block + s * cache->stride_tok
 * with cache->k and cache->v pointing at the pools.  This covers [blocks, slots, heads, 128]
 * (stride_tok = heads * 128, stride_head = 128) as well as [blocks, heads, slots, 128].  Everything
 * else in skipkv_cache keeps its meaning: seq_off numbers the LOGICAL tokens of the batch
 * consecutively, and every per-token and per-sentence array uses that numbering.
 */
typedef struct skipkv_paging {
  const int32_t *block_table; /* device [batch, table_stride]; the first ceil(N_b / block_size) entries of row b are read */
  int32_t table_stride;       /* entries per row                                               */
  int32_t block_size;         /* token slots per block, >= 1                                   */
  int32_t n_blocks;           /* blocks in the pools: valid ids are 0 .. n_blocks-1            */
  int64_t stride_block;       /* elements; a multiple of cache->stride_tok                     */
} skipkv_paging;

/* Device scratch for skipkv_step_paged (the workspace of skipkv_step plus the row map).       */
int skipkv_paged_workspace_bytes(const skipkv_cache *cache, const skipkv_paging *paging, const skipkv_params *params,
                                 size_t *out_bytes);

/*
 * skipkv_step on a paged cache: same scores, same selection, and the compaction moves rows between
 * slots, K[slot of k] <- K[slot of kept_idx[k]] for k < new_len, bit for bit; the block table is
 * not changed (afterwards the caller may release the blocks that lie wholly beyond the new
 * lengths).  Outputs and their layouts are those of skipkv_step.  A row map (logical token ->
 * slot) is built first; a block id outside [0, n_blocks) raises SKIPKV_DEV_BAD_BLOCK_TABLE, is
 * read as block 0, and the sequence's K and V are not touched.  The key scan keeps its single-pass
 * form when block_size is a power of two >= 16 (a 16-token stage then spans at most two blocks)
 * and takes the two-pass form otherwise.
 */
int skipkv_step_paged(const skipkv_cache *cache, const skipkv_paging *paging, const skipkv_params *params,
                      const void *q_obs, const float *tok_redundancy, float *sent_score, float *sent_lambda,
                      float *tok_importance, uint8_t *sent_keep, int32_t *kept_idx, int32_t *new_len,
                      int32_t *new_sent_off, int32_t *new_sent_cnt, int32_t kept_stride, void *ws, size_t ws_bytes,
                      void *stream);

/*
 * The two halves of skipkv_step_paged that touch K and V, for callers that select in between
 * themselves (skipkv_select and skipkv_select_tokens only read scores and the ragged structure, so
 * they serve a paged cache as they are).
 * skipkv_score_paged: skipkv_score on a paged cache; ws as for skipkv_step_paged
 * (skipkv_paged_workspace_bytes).
 * skipkv_score_shared_paged: skipkv_score_shared on a paged cache (lambda from the hidden-state
 * similarity, which does not read K or V and so needs no paged form); same ws.
 * skipkv_compact_paged: skipkv_compact on a paged cache, K[slot of k] <- K[slot of kept_idx[k]]
 * for k < new_len <= kept_stride, bit for bit; a sequence with an invalid block id is left alone
 * and SKIPKV_DEV_BAD_BLOCK_TABLE is raised in dev_status (device int32, OR-ed into; may be NULL).
 * ws: device scratch of at least skipkv_compact_paged_workspace_bytes (row map + slot rows of the
 * kept tokens), 256-byte aligned.
 */
int skipkv_score_paged(const skipkv_cache *cache, const skipkv_paging *paging, const skipkv_params *params,
                       const void *q_obs, const float *tok_redundancy, float *sent_score, float *sent_lambda,
                       float *tok_importance, void *ws, size_t ws_bytes, void *stream);
int skipkv_score_shared_paged(const skipkv_cache *cache, const skipkv_paging *paging, const skipkv_params *params,
                              const void *q_obs, const float *tok_redundancy, const float *shared_lambda, float *sent_score,
                              float *sent_lambda, float *tok_importance, void *ws, size_t ws_bytes, void *stream);
int skipkv_compact_paged_workspace_bytes(const skipkv_cache *cache, const skipkv_paging *paging, int32_t kept_stride,
                                         size_t *out_bytes);
int skipkv_compact_paged(const skipkv_cache *cache, const skipkv_paging *paging, const int32_t *kept_idx,
                         const int32_t *new_len, int32_t kept_stride, int32_t *dev_status, void *ws, size_t ws_bytes,
                         void *stream);

/*
 * skipkv_token_redundancy on a paged cache (Eq. 5 with the key rows read through the block
 * table): same values, same layout of tok_redundancy.  A block id outside [0, n_blocks) raises
 * SKIPKV_DEV_BAD_BLOCK_TABLE in dev_status (device int32, OR-ed into; may be NULL) and is read as
 * block 0.  ws: device scratch of at least skipkv_redundancy_paged_workspace_bytes, 256-byte
 * aligned.
 */
int skipkv_redundancy_paged_workspace_bytes(const skipkv_cache *cache, const skipkv_paging *paging, size_t *out_bytes);
int skipkv_token_redundancy_paged(const skipkv_cache *cache, const skipkv_paging *paging, float *tok_redundancy,
                                  int32_t *dev_status, void *ws, size_t ws_bytes, void *stream);

/*
 * skipkv_step_ranges on a paged cache: the step of every decode-time compression after the
 * first, when the heads of a sequence have their own lengths and sentence ranges (Sec. 4.1
 * "KV Cache Sentence Range Monitoring Logic", Eq. 9-11) and the cache is paged (Appendix,
 * "System-Level Evaluation on vLLM").  ranges, the outputs and their layouts are those of
 * skipkv_step_ranges; paging is that of skipkv_step_paged, with the block table shared by the
 * layers and heads of a sequence and sized for the sequence's extent in cache->seq_off (a head
 * with len below the extent simply leaves the tail slots unused).  Instead of requiring K and V
 * contiguous over (layer, head, token), every (layer, head) gets a row map of its own in units
 * of one head row, so cache->stride_tok, stride_head, stride_layer and paging->stride_block must
 * all be multiples of head_dim, and the last slot row must fit 31 bits (SKIPKV_ECAPACITY).
 * Device errors are those of both calls; an invalid block id leaves K and V of all heads of that
 * sequence untouched.
 * ws, ws_bytes: device scratch of at least skipkv_ranges_paged_workspace_bytes, 256-byte aligned.
 */
int skipkv_ranges_paged_workspace_bytes(const skipkv_cache *cache, const skipkv_paging *paging,
                                        const skipkv_params *params, size_t *out_bytes);
int skipkv_step_ranges_paged(const skipkv_cache *cache, const skipkv_ranges *ranges, const skipkv_paging *paging,
                             const skipkv_params *params, const void *q_obs, const float *tok_redundancy,
                             float *sent_score, float *sent_lambda, float *tok_importance, uint8_t *sent_keep,
                             int32_t *kept_idx, int32_t *new_len, int32_t *new_sent_off, int32_t *new_sent_cnt,
                             int32_t kept_stride, void *ws, size_t ws_bytes, void *stream);

/*
 * The parts of skipkv_step_ranges_paged, for the token-level flow and for the shared lambda on
 * per-head ranges and pages.  The selections (skipkv_select_ranges, skipkv_select_tokens_ranges)
 * read neither K nor V and serve pages as they are; skipkv_compact_paged takes per-head kept_idx
 * and new_len as it is.
 * skipkv_score_ranges_paged: skipkv_score_ranges on pages; with shared_lambda != NULL it is
 *   skipkv_score_shared_ranges on pages (then sent_id and lambda_ptr are required and
 *   sent_lambda may be NULL), else sent_id / lambda_ptr are ignored.  ws as for
 *   skipkv_step_ranges_paged.
 * skipkv_token_redundancy_ranges_paged: skipkv_token_redundancy_ranges on pages; ws as for
 *   skipkv_token_redundancy_paged.
 */
int skipkv_score_ranges_paged(const skipkv_cache *cache, const skipkv_ranges *ranges, const skipkv_paging *paging,
                              const int32_t *sent_id, const int32_t *lambda_ptr, const float *shared_lambda,
                              const skipkv_params *params, const void *q_obs, const float *tok_redundancy,
                              float *sent_score, float *sent_lambda, float *tok_importance, void *ws, size_t ws_bytes,
                              void *stream);
int skipkv_token_redundancy_ranges_paged(const skipkv_cache *cache, const skipkv_ranges *ranges, const skipkv_paging *paging,
                                         float *tok_redundancy, int32_t *dev_status, void *ws, size_t ws_bytes,
                                         void *stream);

/*
 * Steering injection (Sec. 4.2): hidden[b, :] <- hidden[b, :] + coef_b * vec for every row b
 * with row_mask[b] != 0 (all rows when row_mask is NULL).  coef_b = coef[b] when coef is
 * non-NULL, else coef_scalar.  The sum is formed in fp64 and rounded once (nearest even)
 * to the storage dtype.
 * hidden   device in/out [rows, d_model], dtype; vec device [d_model], dtype;
 * coef     device [rows] fp32 or NULL; row_mask device [rows] u8 or NULL.
 */
int skipkv_steer_add(void *hidden, const void *vec, const float *coef, float coef_scalar,
                     const uint8_t *row_mask, int32_t rows, int32_t d_model, int32_t dtype,
                     void *stream);

/*
 * Adaptive steering strength (Sec. 4.2): coef[b] = alpha0 + gamma * n_nonexec[b], with n_nonexec[b]
 * the sample's running count of non-execution thoughts (kept by the caller, who labels the
 * thoughts).  coef is what skipkv_steer_add takes.  n_nonexec, coef: device [rows]; computed in fp32
 * with one rounding.
 */
int skipkv_steer_strength(const int32_t *n_nonexec, float alpha0, float gamma, float *coef, int32_t rows, void *stream);

/*
 * Optional per-kernel timing.  A profile owns HIP events; when params->profile is set the
 * library records one before and after each kernel it launches.  skipkv_profile_read
 * synchronises those events and returns, for slot i < *n, the kernel's name and the
 * milliseconds between its two events for the most recent call that used the profile.
 */
#define SKIPKV_PROFILE_SLOTS 16
int skipkv_profile_create(void **out_profile);
int skipkv_profile_read(void *profile, int32_t *n, const char **names, float *ms);
int skipkv_profile_destroy(void *profile);

const char *skipkv_strerror(int status);
int skipkv_version(void);

#ifdef __cplusplus
}
#endif
#endif /* SKIPKV_H */
