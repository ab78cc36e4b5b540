/*
 * spin.h -- C ABI of the batched verification step of speculative decoding on one MI355X.
 *
 * The step: every request of a batch brings its own number of draft (candidate) tokens from a
 * small speculative model; the large model checks them all in one pass.  This library holds the
 * data-parallel part of that pass:
 *
 *   spin_decompose    split requests into sub-requests                      (Sec. V-A)
 *   spin_verify_attn  attention of each request's draft queries over its cached prefix plus a
 *                     causal draft block, read through a page table, exact across sub-requests
 *                                                                (Sec. II-A1 Eq. (2), Sec. V-A Eq. (13))
 *   spin_accept       greedy-match or rejection-sampling acceptance of the draft tokens
 *                                                                (verification phase, Sec. II-A2)
 *   spin_append_kv    the draft tokens' K/V rows enter the paged cache just before that pass
 *                                                                (the KV cache of Sec. II-A1)
 *   spin_verify_attn_tree, spin_accept_tree   the same two steps for drafts that are token trees
 *                                                                (the related work named in Sec. I)
 *
 * Conventions
 *   - Plain C, no exceptions cross this boundary.  Every function returns SPIN_OK (0) or a
 *     negative SPIN_E* code; spin_last_error() gives the text of the last failure of a context.
 *   - "host" pointers are ordinary CPU memory, read during the call and free to go when it
 *     returns.  "device" pointers are HIP device memory of the context's GPU; the caller owns
 *     them, the library never frees or resizes them and never writes to an input.
 *   - Calls that take a stream only enqueue work on it (HIP stream handle passed as void*;
 *     NULL = the default stream).  All errors the host can see are reported before anything is
 *     launched.  Outputs are valid once the stream has been synchronised.  The calls do not wait
 *     for the stream; spin_verify_attn may hold the host for the few microseconds its own upload
 *     of the call's tables (a copy on a stream of the context) takes, so that nothing but kernels
 *     has to go onto the caller's stream.
 *   - Request i has prefix length p_i >= 0 (tokens whose K/V are cached and that ask nothing)
 *     and draft length g_i >= 1 (tokens whose K/V are ALSO already in the cache, at positions
 *     p_i .. p_i+g_i-1, and which each issue one query row).  Draft row t sees keys 0 .. p_i+t.
 *   - One context must not be used from two host threads at once, and its calls share one
 *     workspace (partial results, row statistics): give them one stream, or order the streams
 *     yourself.  Work that is meant to overlap on the GPU takes one context per stream.
 *   - "never writes to an input" has one exception, stated there: spin_append_kv writes the pools.
 */
#ifndef SPIN_H
#define SPIN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SPIN_OK 0
#define SPIN_EINVAL (-1)       /* null pointer, negative size, draft length < 1, ...            */
#define SPIN_ETABLE (-2)       /* inconsistent request table / page table / sub-request tiling  */
#define SPIN_ENOSPC (-3)       /* output capacity or reserved workspace too small               */
#define SPIN_EUNSUPPORTED (-4) /* a shape or type this build has no kernel for                  */
#define SPIN_EHIP (-5)         /* a HIP runtime call failed; text via spin_last_error           */

#define SPIN_DTYPE_BF16 1   /* bfloat16 */
#define SPIN_DTYPE_F16 2    /* IEEE binary16 */

typedef struct spin_ctx spin_ctx;

/* Ragged request table.  All arrays are host memory.
 *   prefix_len[n_req], draft_len[n_req]
 *   q_offset[n_req+1]   first packed query/output row of each request; q_offset[0] = 0 and
 *                       q_offset[i+1] - q_offset[i] = draft_len[i]
 *   pt_offset[n_req+1]  first page-table entry of each request (non-decreasing)
 *   page_table[pt_offset[n_req]]  physical page ids; request i needs at least
 *                       ceil((p_i+g_i)/page_size) entries; token j of the request lives in page
 *                       page_table[pt_offset[i] + j/page_size], slot j % page_size. */
typedef struct spin_req_table {
    int32_t n_req;
    const int32_t* prefix_len;
    const int32_t* draft_len;
    const int32_t* q_offset;
    const int32_t* pt_offset;
    const int32_t* page_table;
} spin_req_table;

/* Paged K/V cache.  k_pool / v_pool are device pointers to 16-bit elements of type `dtype`.  Element (page, kv
 * head, slot, c) sits at  page*page_stride + head*head_stride + slot*token_stride + c  (strides
 * in elements, the head dimension is contiguous, token_stride >= head_dim, a multiple of 8 and at most 2^24,
 * both pools 16-byte aligned).  page_size must be a power of two; from 16 tokens up, head-major
 * ([n_pages][n_kv_heads][page_size][head_dim]) and token-major ([n_pages][page_size][n_kv_heads][head_dim])
 * pages stream at full speed, smaller pages take a slower addressing path. */
typedef struct spin_kv_desc {
    const void* k_pool;
    const void* v_pool;
    int32_t n_pages;
    int32_t page_size;
    int32_t n_kv_heads;
    int32_t head_dim;          /* 64 or 128 */
    int64_t page_stride;
    int64_t head_stride;
    int64_t token_stride;
    int32_t dtype;             /* SPIN_DTYPE_BF16 or SPIN_DTYPE_F16: the type of K, V, Q and the output */
} spin_kv_desc;

/* A sub-request: a rectangle of its parent's (draft row x key) score matrix.  It refers to the
 * parent's query rows and pages by offset; nothing is copied or replicated (the replicated Q
 * rows of Sec. V-A exist only as these references).  Cells of the rectangle beyond the causal
 * edge (key > p + row) hold nothing. */
typedef struct spin_subreq {
    int32_t parent;            /* index into the request table                  */
    int32_t q_begin, q_len;    /* draft rows  [q_begin, q_begin+q_len)          */
    int32_t kv_begin, kv_len;  /* keys        [kv_begin, kv_begin+kv_len)       */
} spin_subreq;

#define SPIN_DECOMP_NONE 0      /* one sub-request per request                                     */
#define SPIN_DECOMP_Q_SPLIT 1   /* cut the draft block into pieces of q_width rows                 */
#define SPIN_DECOMP_KV_SPLIT 2  /* Sec. V-A: rows of a KV tensor of length kv_len; the whole draft
                                   block rides along with every piece                             */
#define SPIN_DECOMP_KV_SEARCH 3 /* Sec. V-A: cap the tensor width (number of rows) at max_subreq,
                                   pick the length L in [l_min, l_max] (multiples of l_step) with
                                   the fewest padding tokens, ties to the larger L; then KV_SPLIT  */

typedef struct spin_decomp_params {
    int32_t policy;
    int32_t q_width;     /* Q_SPLIT: draft rows per sub-request (>= 1)        */
    int32_t kv_len;      /* KV_SPLIT: L (>= 1)                                */
    int32_t max_subreq;  /* KV_SEARCH: width cap B                            */
    int32_t l_min, l_max, l_step; /* KV_SEARCH: candidate lengths             */
} spin_decomp_params;

/* ---- lifetime ---------------------------------------------------------------------------- */

/* Create a context on HIP device `device_id`.  Fails with SPIN_EHIP when no such device. */
int spin_create(spin_ctx** out, int device_id);

/* Allocate (or grow to) workspace for batches of up to max_req requests, max_rows draft rows in
 * total, max_pages page-table entries, max_items work pieces and max_part_slots partial result
 * rows.  This is the only call that allocates device or pinned memory; it synchronises the
 * device.  spin_verify_attn / spin_accept return SPIN_ENOSPC when the reservation is too small
 * and spin_required() then reports what the refused call needed. */
int spin_reserve(spin_ctx* ctx, int64_t max_req, int64_t max_rows, int64_t max_pages,
                 int64_t max_items, int64_t max_part_slots);

/* Sizes the last call on this context that returned SPIN_ENOSPC would have needed (any pointer
 * may be NULL). */
int spin_required(spin_ctx* ctx, int64_t* req, int64_t* rows, int64_t* pages, int64_t* items,
                  int64_t* part_slots);

/* Wait for outstanding work of this context, free everything it owns. NULL is allowed. */
void spin_destroy(spin_ctx* ctx);

const char* spin_strerror(int code);

/* Copy the text of the context's last error into buf (NUL-terminated, truncated to n). */
int spin_last_error(spin_ctx* ctx, char* buf, size_t n);

/* Number of wavefronts the attention kernel runs per launch: 0 (default) = as many as the GPU
 * holds at once, otherwise that many (for experiments and tests; results differ only in
 * summation order). */
int spin_set_waves(spin_ctx* ctx, int32_t n_waves);

/* ---- decomposition (host only, no GPU needed) -------------------------------------------- */

/* Sec. V-A.  Writes the sub-requests of `table` under `params` to out[0..cap) in the order
 * parent ascending, then q_begin, then kv_begin, and their number to *n_out.  If cap is too
 * small returns SPIN_ENOSPC with *n_out = the number needed (out may then be NULL).  With
 * KV_SEARCH, *kv_len_out (may be NULL) receives the chosen L; SPIN_ENOSPC with *n_out = 0 if no
 * candidate L fits under max_subreq.  Only prefix_len and draft_len of the table are read. */
int spin_decompose(const spin_req_table* table, const spin_decomp_params* params,
                   spin_subreq* out, int32_t cap, int32_t* n_out, int32_t* kv_len_out);

/* The padding-token count and row count of the B x L KV tensor of Sec. V-A for a given L. */
int spin_kv_padding(const spin_req_table* table, int32_t kv_len, int64_t* n_rows, int64_t* n_pad);

/* Check that subs tile every request exactly once (every visible (draft row, key) cell of every
 * request covered by exactly one sub-request).  SPIN_OK or SPIN_ETABLE.  Host only. */
int spin_check_tiling(const spin_req_table* table, const spin_subreq* subs, int32_t n_sub);

/* The scheduler's view of a batch, for inspection and tests (host only).  The attention kernel
 * runs a fixed number of wavefronts per launch; the key blocks (32 keys) of all (rectangle, KV
 * head) pairs form one sequence that is cut into equal shares, one per wavefront.  A piece is one
 * run of blocks of one (rectangle, KV head) inside one share.  The last part of the sequence is
 * cut into small chunks instead, which wavefronts take from a queue as they finish their share
 * (QUEUED).  `tile_class` 0/1/2 = launches for up to 16/32/64 (draft row x query head) rows;
 * `wave` numbers the shares of a class: first the per-wavefront ones, then the queued chunks.
 * Flags: CARRY_IN = continues the wavefront's previous piece, CARRY_OUT = continued by its next
 * piece (nothing written), DIRECT = ends a rectangle that one wavefront held entirely and that
 * holds every key its rows may see: final rows are written, no partial result.  `group` =
 * n_q_heads / n_kv_heads, n_waves = wavefronts per class.  Same cap/n_out protocol as
 * spin_decompose.  subs == NULL means one sub-request per request. */
#define SPIN_PIECE_CARRY_IN 1
#define SPIN_PIECE_CARRY_OUT 2
#define SPIN_PIECE_DIRECT 4
#define SPIN_PIECE_QUEUED 8
typedef struct spin_work_piece {
    int32_t parent, q_begin, q_len, kv_begin, kv_len;
    int32_t kv_head, tile_class, wave, flags;
} spin_work_piece;
int spin_schedule(const spin_req_table* table, const spin_subreq* subs, int32_t n_sub,
                  int32_t page_size, int32_t group, int32_t n_kv_heads, int32_t n_waves,
                  spin_work_piece* out, int32_t cap, int32_t* n_out);

/* ---- the verification step ---------------------------------------------------------------- */

/* Sec. II-A1 Eq. (2) with the normalisation of Sec. V-A Eq. (13).
 *   q_dev  device, kv->dtype [R][n_q_heads][head_dim], R = q_offset[n_req]   (read)
 *   o_dev  device, kv->dtype [R][n_q_heads][head_dim]                         (every row written once)
 *          both 16-byte aligned.  Products accumulate in fp32; the softmax weights are rounded
 *          to kv->dtype before they multiply V, the result rows once at the end.
 *   subs   host, n_sub sub-requests that tile the batch exactly once, or NULL for none
 *   softmax_scale  multiplies Q.K before exp; <= 0 selects 1/sqrt(head_dim); 1 is the literal
 *                  formula of Eq. (2)
 * Query head h uses KV head h / (n_q_heads / n_kv_heads).  Whatever the decomposition, the output
 * of a draft row is its attention over ALL keys it may see in the original request.
 * Errors: SPIN_EINVAL, SPIN_ETABLE (table or tiling inconsistent, page id outside the pool),
 * SPIN_EUNSUPPORTED (head_dim, dtype, page size, group > 64), SPIN_ENOSPC (reserve more),
 * SPIN_EHIP. */
int spin_verify_attn(spin_ctx* ctx, const spin_kv_desc* kv, const spin_req_table* table,
                     const spin_subreq* subs, int32_t n_sub, const void* q_dev, void* o_dev,
                     int32_t n_q_heads, float softmax_scale, void* hip_stream);

/* spin_verify_attn for tree-shaped drafts (the token trees of the speculative-inference systems the
 * paper's related work names): the draft tokens of a request are the nodes of a tree whose root hangs
 * below the last prefix token, numbered so that every node comes after its parent, and draft row t sees
 * the whole prefix plus its ancestors and itself instead of all earlier draft tokens.
 * tree_mask (host, [R], packed like Q): bit u of tree_mask[q_offset[i] + t] is set iff row t of request
 * i sees draft key p_i + u.  Bit t must be set and no bit above t; draft_len <= 64; violations give
 * SPIN_ETABLE.  A mask with bits 0..t set in every row is the linear draft of spin_verify_attn.
 * Sub-requests tile the same causal region as in spin_verify_attn; the mask only removes cells.
 * Everything else (arguments, layouts, asynchrony, errors) is as in spin_verify_attn. */
int spin_verify_attn_tree(spin_ctx* ctx, const spin_kv_desc* kv, const spin_req_table* table,
                          const spin_subreq* subs, int32_t n_sub, const uint64_t* tree_mask,
                          const void* q_dev, void* o_dev, int32_t n_q_heads, float softmax_scale,
                          void* hip_stream);

/* The step just before the attention: put the draft tokens' K and V rows into the paged cache, so
 * that the caller need not run a scatter of its own.  Row r of k_new_dev / v_new_dev (device, kv->dtype
 * [R][n_kv_heads][head_dim], packed like Q) is draft token t = r - q_offset[i] of its request i and goes
 * to position p_i + t: page page_table[pt_offset[i] + (p_i+t)/page_size], slot (p_i+t) % page_size.
 * kv->k_pool / kv->v_pool are WRITTEN by this call (and only by this call).  Rejected draft tokens
 * need no roll-back: their slots simply lie beyond the prefix the caller keeps.  Asynchronous on
 * the stream; same table checks and error codes as spin_verify_attn. */
int spin_append_kv(spin_ctx* ctx, const spin_kv_desc* kv, const spin_req_table* table,
                   const void* k_new_dev, const void* v_new_dev, void* hip_stream);

#define SPIN_ACCEPT_GREEDY 0
#define SPIN_ACCEPT_REJECTION 1

/* Verification phase of Sec. II-A2 (the paper prints no rule; this is the speculative-sampling
 * rule of the works it builds on), float64 arithmetic on fp32 logits.
 *   draft_len_host      host   int32 [n_req]
 *   draft_tokens_dev    device int32 [R]
 *   target_logits_dev   device fp32 [R+n_req][vocab]; request i owns rows q_offset[i]+i ..
 *                       q_offset[i]+i+g_i, the last one being the bonus row
 *   draft_logits_dev    device fp32 [R][vocab]            (REJECTION only, else may be NULL)
 *   u_accept_dev        device fp64 [R]  in [0,1)         (REJECTION only)
 *   u_sample_dev        device fp64 [n_req] in [0,1)      (REJECTION only)
 *   n_accepted_dev      device int32 [n_req]  out: number of leading draft tokens kept, 0..g_i
 *   next_token_dev      device int32 [n_req]  out: the token emitted after them
 * GREEDY: draft token t is kept iff it equals the arg-max (lowest id on ties) of target row t;
 * next token = arg-max of target row n.  REJECTION: with p, q the softmax of the target / draft
 * row, token d_t is kept iff u_t*q(d_t) < p(d_t); on the first rejection the next token is the
 * smallest k with sum_{x<=k} max(0,p-q)(x) > u'*Z (from p itself if Z = 0), otherwise the same
 * inverse CDF on the bonus row's p.  A draft token id outside [0, vocab) is never kept.
 * Errors: SPIN_EINVAL, SPIN_EUNSUPPORTED (vocab > 1048576), SPIN_ENOSPC (reserve more), SPIN_EHIP. */
int spin_accept(spin_ctx* ctx, int32_t mode, int32_t n_req, const int32_t* draft_len_host,
                const int32_t* draft_tokens_dev, const float* target_logits_dev,
                const float* draft_logits_dev, int32_t vocab, const double* u_accept_dev,
                const double* u_sample_dev, int32_t* n_accepted_dev, int32_t* next_token_dev,
                void* hip_stream);

/* spin_accept for callers that cannot allocate device memory: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  No context and no reservation: the row statistics live in a
 * static device array of the library (SPIN_NOALLOC_MAX_STAT_ROWS x 16 bytes = 512 KiB, held by every GPU
 * the library runs on until the process ends), and the call issues no hipMalloc / hipFree or any other
 * allocating routine.  It runs on the calling thread's current HIP device; hip_stream must belong to it.
 * Same arithmetic, kernels and outputs as spin_accept.  Differences in the arguments:
 *   n_rows          host: R, the total number of draft rows
 *   q_offset_dev    device int32 [n_req+1]: first draft row of each request (q_offset[0] = 0,
 *                   q_offset[n_req] = n_rows, every difference >= 1).  The host cannot read it, so the kernel
 *                   checks it: a request whose rows do not lie in [0, n_rows] gets n_accepted = next_token = -1.
 * Limit: 2*n_rows + n_req <= SPIN_NOALLOC_MAX_STAT_ROWS (rejection or greedy alike), else SPIN_ENOSPC.
 * Other errors: SPIN_EINVAL (null pointer, n_rows < n_req, unknown mode), SPIN_EUNSUPPORTED (vocab >
 * 1048576), SPIN_EHIP.  No error text is kept (there is no context).
 * All calls on one GPU share the one array, which keeps the previous call's contents (nothing in it has to
 * start at zero: every statistics row a call reads it has written first): calls that overlap on one GPU
 * -- two streams, two host threads -- race; order them on one stream or with events. */
#define SPIN_NOALLOC_MAX_STAT_ROWS 32768
int spin_accept_noalloc(int32_t mode, int32_t n_req, int32_t n_rows, const int32_t* q_offset_dev,
                        const int32_t* draft_tokens_dev, const float* target_logits_dev,
                        const float* draft_logits_dev, int32_t vocab, const double* u_accept_dev,
                        const double* u_sample_dev, int32_t* n_accepted_dev, int32_t* next_token_dev,
                        void* hip_stream);

/* Verification of token trees, the companion of spin_verify_attn_tree.  Draft token t of request i hangs
 * below token parent_host[q_offset[i] + t] of the same request (an earlier token, or -1 = the last prefix
 * token); draft_len <= 64.  Target row q_offset[i] + i is the model's output after the prefix, row
 * q_offset[i] + i + 1 + t its output after token t (for a chain this is the layout of spin_accept, and the
 * results are those of spin_accept); draft row q_offset[i] + t is the distribution token t was drawn from.
 * The walk starts below the last prefix token.
 *   SPIN_ACCEPT_GREEDY     move to the lowest-numbered child whose token equals the arg-max (lowest id on
 *                          ties) of the current node's target row, until no child does; next token = the
 *                          arg-max of the row of the last token reached.  draft_logits_dev, u_accept_dev and
 *                          u_sample_dev are not read and the vocabulary is not limited.
 *   SPIN_ACCEPT_REJECTION  multi-round speculative sampling (float64): with R_0 = p = softmax(target row of
 *                          the current node) and s_0 = 1, the children are tried in index order; child c with
 *                          token d and q_c = softmax(its draft row) is accepted iff
 *                          u_accept[c] * q_c(d) * s_k < R_k(d), and the walk moves on from c.  A rejected
 *                          child gives R_{k+1} = max(0, R_k - s_k q_c), s_{k+1} = sum R_{k+1}; if that sum is
 *                          zero the child is ignored.  A token id outside [0, vocab) is never accepted.  When
 *                          no child is accepted the next token is the smallest k with
 *                          sum_{x<=k} R_k(x) > u_sample[i] * s_k.  vocab <= 1048576.
 * Outputs:
 *   n_accepted_dev[i]            number of tokens on the accepted path
 *   path_dev[q_offset[i] + k]    its k-th token, k < n_accepted; -1 in the request's other entries
 *   next_token_dev[i]            the token that follows the path
 * Errors as for spin_accept, plus SPIN_ETABLE for a bad parent or more than 64 draft tokens. */
int spin_accept_tree(spin_ctx* ctx, int32_t mode, int32_t n_req, const int32_t* draft_len_host,
                     const int32_t* parent_host, const int32_t* draft_tokens_dev,
                     const float* target_logits_dev, const float* draft_logits_dev, int32_t vocab,
                     const double* u_accept_dev, const double* u_sample_dev, int32_t* n_accepted_dev,
                     int32_t* path_dev, int32_t* next_token_dev, void* hip_stream);

/* A transformer calls spin_verify_attn once per layer with the same request table.  The context
 * therefore keeps the tables of its most recent attention call on the device, with a copy of what they
 * were made from; a call whose request table, sub-requests, tree mask, head counts and page geometry are
 * equal in content (the caller's arrays are compared, never trusted to be unchanged) launches from them
 * again: no validation, scheduling or upload.  Pool, Q and O pointers, strides and the softmax scale may
 * differ between such calls.  On by default; enable = 0 makes every call plan afresh. */
int spin_set_plan_reuse(spin_ctx* ctx, int32_t enable);

/* ---- measurement aid ------------------------------------------------------------------------ */

/* Time the kernels of the next calls with HIP events handed to the kernel launches themselves: an event
 * pair receives the start and end time stamps of the kernel's own dispatch record, so nothing extra
 * is put on the stream and a timed call runs like an untimed one (nothing is synchronised until
 * spin_profile_end).  spin_profile_begin arms up to max_calls calls of spin_verify_attn and as many of
 * spin_accept; further calls run untimed.
 * spin_profile_end waits for the recorded events and returns the summed durations in
 * milliseconds: ms[0] attention kernels, ms[1] partial-join kernel (zero for a call that has no partial
 * results to join), ms[2] the first kernel of spin_accept (the logits row statistics; for a call small
 * enough to run as one kernel, the whole acceptance), ms[3] its second kernel (acceptance scan and
 * next-token draw; zero when there is none); calls[0] / calls[1] = timed calls of spin_verify_attn /
 * spin_accept.  It disarms the context. */
int spin_profile_begin(spin_ctx* ctx, int32_t max_calls);
/* While armed, time only every n-th call of each kind (n >= 1, default 1; the first call after
 * spin_profile_begin is timed).  The setting stays until changed.  max_calls of spin_profile_begin
 * counts timed calls. */
int spin_profile_every(spin_ctx* ctx, int32_t n);
int spin_profile_end(spin_ctx* ctx, double ms[4], int32_t calls[2]);

#ifdef __cplusplus
}
#endif
#endif /* SPIN_H */
