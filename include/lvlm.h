/*
 * lvlm.h -- C ABI of the LightVLM token-reduction path for AMD MI355X (gfx950).
 *
 * The library implements the per-layer step that LightVLM (arXiv 2509.00419)
 * adds to the language model of a vision-language model:
 *   prefill  (Sec. 3.2.1, pyramid token merging): score image tokens by the
 *            attention they receive, split them into P_unmerged / P_merged,
 *            merge P_merged into one token, compact every plane that shares
 *            the token axis;
 *   decode   (Sec. 3.2.2, KV-cache compression): evict cache entries per
 *            KV head and run grouped-query attention over what is left.
 *
 * General rules for every call below
 *   - Every tensor pointer is a DEVICE pointer owned by the caller and must be
 *     16-byte aligned (score_mean alone needs only 4 bytes, so that rows of a
 *     larger array can be passed).  Descriptors, plane tables and "host" outputs are HOST
 *     memory.  Strides are in elements; the innermost dimension is contiguous.
 *   - The calls of the path only enqueue kernels on the caller's stream
 *     (a hipStream_t passed as void*; NULL = the default stream).  They do not
 *     allocate, free or synchronise.  Scratch memory comes from the workspace
 *     the caller attached with lvlm_set_workspace; its size is queried with
 *     lvlm_workspace_bytes.  Calls that share one workspace must be ordered
 *     on one stream.
 *   - Arguments are validated on the host before anything is enqueued; on an
 *     error nothing has been launched and outputs are untouched.
 *     lvlm_last_error(ctx) returns a message for the last failing call.
 *   - One lvlm_ctx per host thread.  No global mutable state.
 */
#ifndef LVLM_H
#define LVLM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define LVLM_API __attribute__((visibility("default")))

typedef enum {
    LVLM_OK = 0,
    LVLM_ERR_INVALID_ARG = 1, /* null / misaligned pointer, inconsistent sizes */
    LVLM_ERR_UNSUPPORTED = 2, /* dtype or head_dim the kernels do not cover     */
    LVLM_ERR_WORKSPACE = 3,   /* no workspace attached, or it is too small      */
    LVLM_ERR_HIP = 4          /* a HIP runtime call failed                      */
} lvlm_status;

typedef enum { LVLM_BF16 = 0, LVLM_F32 = 1, LVLM_I32 = 2 } lvlm_dtype;

typedef enum {
    LVLM_OP_SCORE = 0,
    LVLM_OP_MERGE = 1,
    LVLM_OP_KV_COMPRESS = 2,
    LVLM_OP_DECODE_ATTN = 3,
    LVLM_OP_MERGE_SIMILAR = 4,
    LVLM_OP_SCORE_PROBS = 5,
    LVLM_OP_PREFILL_ATTN = 6
} lvlm_op;

/* Rank -> weight tables for the merged token (Sec. 3.2.1, par. 4). */
typedef enum {
    LVLM_MERGE_LINEAR_RANK = 0, /* W_v = {r+1,...,1} scaled to sum 1 (default)        */
    LVLM_MERGE_PAIRWISE = 1,    /* closed form of the iterated equal-weight tail merge */
    LVLM_MERGE_LINEAR_RAW = 2   /* W_v exactly as printed                              */
} lvlm_merge_mode;

typedef enum {
    LVLM_RULE_WEIGHTED = 0, /* new row = sum_k w_k * merged row k (hidden, K, V)       */
    LVLM_RULE_TOP = 1       /* new row = row of the most important merged token (ids)  */
} lvlm_merge_rule;

typedef enum {
    LVLM_KV_THRESHOLD = 0, /* Sec. 3.2.2: keep image entries until beta of their score mass */
    LVLM_KV_BUDGET = 1     /* fixed number of entries per head (not in the paper)           */
} lvlm_kv_mode;

typedef enum {
    LVLM_ORDER_STABLE = 0, /* survivors keep ascending slot order                        */
    LVLM_ORDER_FILL = 1    /* survivors below the new length stay; holes are filled from */
                           /* the survivors beyond it, both in ascending order           */
} lvlm_kv_order;

enum { LVLM_KIND_PROTECTED = 0, LVLM_KIND_IMAGE = 1, LVLM_KIND_GENERATED = 2 };

#define LVLM_MAX_PLANES 8

typedef struct lvlm_ctx lvlm_ctx;

/* ---- context, workspace, host helpers ------------------------------------ */

/* Creates a context bound to HIP device `device`.  Touches no GPU state until
 * the first launch.  *ctx is set to NULL on failure. */
LVLM_API lvlm_status lvlm_create(lvlm_ctx **ctx, int device);
LVLM_API lvlm_status lvlm_destroy(lvlm_ctx *ctx);
LVLM_API const char *lvlm_last_error(const lvlm_ctx *ctx);

/* Bytes of scratch the given call needs.  `desc` points to the lvlm_*_desc of
 * that op; for LVLM_OP_MERGE / LVLM_OP_MERGE_SIMILAR to an lvlm_merge_query (descriptor plus
 * plane table: only row_elems and dtype of each plane are read).  Pure host
 * arithmetic; the size never depends on pointer values.  It does not depend on
 * n_keep either, except for LVLM_OP_MERGE_SIMILAR (whose scratch holds one entry
 * per dominant token: there n_keep must already be the value of the call). */
LVLM_API lvlm_status lvlm_workspace_bytes(const lvlm_ctx *ctx, lvlm_op op, const void *desc, size_t *bytes);
/* Size limits, checked with the other descriptor fields (LVLM_ERR_INVALID_ARG beyond them): B <= 65536, Hq and
 * Hkv <= 1024, N <= 4194304 tokens, Lmax <= 16777216 slots, row_elems <= 1048576.  Within them no size or grid
 * computation of the library can overflow. */
/* Attaches caller-owned device scratch (256-byte aligned).  May be replaced at
 * any time between calls; the library never frees it. */
LVLM_API lvlm_status lvlm_set_workspace(lvlm_ctx *ctx, void *dev_ptr, size_t bytes);

/* Per-kernel timing for benchmarks (not on the hot path, not usable during
 * stream capture).  While enabled, every kernel the calls launch carries a HIP
 * event pair bound to the kernel itself (start of its first wave, end of its
 * last: the duration a kernel trace reports, without the gaps between
 * dispatches), at most 4096 launches between reads.  lvlm_profile_read waits
 * for those events, adds them up per kernel name into the caller's HOST array
 * and clears the record. */
typedef struct {
    char name[48];
    int32_t calls;
    float total_ms, min_ms, max_ms;
} lvlm_profile_entry;
LVLM_API lvlm_status lvlm_profile(lvlm_ctx *ctx, int enable);
LVLM_API lvlm_status lvlm_profile_read(lvlm_ctx *ctx, lvlm_profile_entry *out, int max_entries, int *n_entries);

/* Pyramid schedule (App. A.2: merge layers use a constant reduction ratio set
 * by the budget).  n_keep_out[s-1] = floor(n_img * final_keep^(s/n_stages) + 0.5)
 * for s = 1..n_stages, taken from the original n_img and clamped to [1, n_img].
 * Host only. */
LVLM_API lvlm_status lvlm_schedule(int n_img, double final_keep, int n_stages, int *n_keep_out);

/* Rank -> weight table of length m = r+1 (rank 0 = most important merged
 * token), written to HOST memory as fp32 (Sec. 3.2.1, par. 4). */
LVLM_API lvlm_status lvlm_merge_weights(lvlm_merge_mode mode, int m, float *w_host_out);

/* ---- step 1: token importance -------------------------------------------- */

/* Sec. 3.2.1: the importance of a token is the attention it receives -- the
 * column sum of the softmax probabilities ("cumsum attention score" A in R^N).
 * Query row i (0 <= i < T) sits at absolute position q_pos0 + i; its softmax
 * runs over every key j it may see (j <= q_pos0 + i if causal, else all N),
 * not only the image keys.  Softmax and sums are fp32. */
typedef struct {
    int32_t dtype;     /* LVLM_BF16 or LVLM_F32: element type of q and k          */
    int32_t B, N, T;   /* batch, keys per sequence, query rows                    */
    int32_t q_pos0;    /* absolute position of query row 0                        */
    int32_t Hq, Hkv;   /* query heads, KV heads (Hq % Hkv == 0)                   */
    int32_t hd;        /* head dimension: 64 or 128                               */
    int32_t img_begin; /* first image key                                         */
    int32_t n_img;     /* number of image keys; img_begin + n_img <= N            */
    int32_t causal;    /* 0 / 1                                                   */
    float scale;       /* logit scale >= 0, usually 1/sqrt(hd)                    */
    int64_t q_stride_b, q_stride_t, q_stride_h; /* q[b][i][h][0..hd)              */
    int64_t k_stride_b, k_stride_n, k_stride_h; /* k[b][j][g][0..hd)              */
    int64_t sh_stride_b, sh_stride_h; /* score_head[b][g][0..n_img); both 0 = dense
                                         [B,Hkv,n_img].  Lets the scores land in a
                                         cache's score array (stride Lmax per head) */
} lvlm_score_desc;

/* q, k: device, dtype above.  row_lse: optional device fp32 [B,Hq,T] holding
 * the natural-log sum-exp of each row's scaled logits (as an attention kernel
 * produces); when NULL the library computes it with one more pass over k.
 * score_head [B,Hkv,n_img] fp32 (strides above): mean over the G query heads of
 * each KV head.
 * score_mean [B,n_img] fp32: mean over the KV heads (= over all heads).
 * Both outputs are written in full.  Workspace: LVLM_OP_SCORE. */
LVLM_API lvlm_status lvlm_score_tokens(lvlm_ctx *ctx, void *stream, const lvlm_score_desc *d,
                              const void *q, const void *k, const float *row_lse,
                              float *score_head, float *score_mean);

/* Which kernels lvlm_score_tokens takes for a shape (host arithmetic; for benchmarks that credit work to
 * kernels by name): *form = 0 two passes over the keys in separate launches (normalisers, then column
 * sums), 1 both sweeps in one launch with one query chunk per workgroup, 2 both sweeps in one launch with
 * four query chunks per workgroup sharing the key tiles, 3 the kernel of form 2 with the keys cut into runs
 * (one launch per sweep, the runs' normaliser partials folded in between: launches of few workgroups). */
LVLM_API lvlm_status lvlm_score_plan(const lvlm_ctx *ctx, const lvlm_score_desc *d, int32_t *form);

/* The same scores from attention probabilities the caller already holds -- a
 * plain attention that materialises its matrix (Sec. 3.2.2 names both sources:
 * the full attention matrix or the cumulative score).  probs[b][h][i][j] is the
 * softmax probability of query row i (of the T rows to be summed, e.g. the
 * instruction rows) on key j, dtype bf16 or fp32, innermost axis contiguous,
 * strides in elements.  score_head[b][g][j] = (1/G)
 * sum over the G heads of group g and the T rows of probs[..][img_begin + j];
 * score_mean as in lvlm_score_tokens.  Sums are fp32 in a fixed order. */
typedef struct {
    int32_t dtype;     /* LVLM_BF16 or LVLM_F32: element type of probs            */
    int32_t B, N, T;   /* batch, keys per row, query rows                         */
    int32_t Hq, Hkv;   /* query heads, KV heads (Hq % Hkv == 0)                   */
    int32_t img_begin; /* first image key                                         */
    int32_t n_img;     /* number of image keys; img_begin + n_img <= N            */
    int64_t p_stride_b, p_stride_h, p_stride_t; /* probs[b][h][i][0..N)           */
    int64_t sh_stride_b, sh_stride_h; /* score_head strides; both 0 = dense       */
} lvlm_probs_desc;

/* probs: device.  score_head [B,Hkv,n_img] fp32, score_mean [B,n_img] fp32 (4-byte
 * aligned suffices), both written in full.  Workspace: LVLM_OP_SCORE_PROBS. */
LVLM_API lvlm_status lvlm_score_from_probs(lvlm_ctx *ctx, void *stream, const lvlm_probs_desc *d,
                                           const void *probs, float *score_head, float *score_mean);

/* The layer's own prefill attention with the scores as its by-product (Sec.
 * 3.2.1: the importance of a token is read off the attention of the layer, at
 * no cost of its own; Sec. 3.2.2: off the statistics its kernel keeps).  Row i
 * of q sits at position i; head h reads KV head h / (Hq/Hkv):
 *   out[b][i][h][:] = sum_j softmax_j(scale q[b][i][h] . k[b][j][g]) v[b][j][g][:]
 * over the keys the row may see (j <= i if causal, else all N), softmax and
 * sums in fp32; row_lse[b][h][i] = natural-log sum-exp of the row's scaled
 * logits.  With T > 0 the last T rows are the instruction rows: their scores
 * over the image keys are computed from these normalisers with the one
 * column-sum pass of lvlm_score_tokens (no normaliser pass), as
 * lvlm_score_tokens(q rows N-T.., q_pos0 = N-T, row_lse = these) would give. */
typedef struct {
    int32_t dtype;     /* LVLM_BF16 or LVLM_F32: element type of q, k, v, out     */
    int32_t B, N;      /* batch, tokens per sequence (query rows = keys)          */
    int32_t Hq, Hkv;   /* query heads, KV heads (Hq % Hkv == 0)                   */
    int32_t hd;        /* head dimension: 64 or 128                               */
    int32_t causal;    /* 0 / 1                                                   */
    float scale;       /* logit scale > 0, usually 1/sqrt(hd)                     */
    int32_t T;         /* instruction rows (the last T); 0 = attention only       */
    int32_t img_begin; /* first image key        (read only when T > 0)           */
    int32_t n_img;     /* number of image keys; img_begin + n_img <= N            */
    int64_t q_stride_b, q_stride_n, q_stride_h; /* q[b][i][h][0..hd), elements    */
    int64_t k_stride_b, k_stride_n, k_stride_h; /* k[b][j][g][0..hd)              */
    int64_t v_stride_b, v_stride_n, v_stride_h; /* v[b][j][g][0..hd)              */
    int64_t o_stride_b, o_stride_n, o_stride_h; /* out[b][i][h][0..hd)            */
    int64_t sh_stride_b, sh_stride_h; /* score_head strides; both 0 = dense       */
} lvlm_prefill_desc;

/* q, k, v: device, read only.  out: device, dtype above, must not overlap the
 * inputs.  row_lse: device fp32 [B,Hq,N], written in full.  score_head
 * [B,Hkv,n_img] and score_mean [B,n_img] fp32: written in full when T > 0 (then
 * both required), untouched when T == 0 (may be NULL).  All pointers 16-byte
 * aligned (score_mean: 4), strides multiples of 16 bytes.  Errors: invalid
 * descriptor or pointer -> LVLM_ERR_INVALID_ARG, nothing launched.
 * Workspace: LVLM_OP_PREFILL_ATTN. */
LVLM_API lvlm_status lvlm_prefill_attn(lvlm_ctx *ctx, void *stream, const lvlm_prefill_desc *d, const void *q,
                                       const void *k, const void *v, void *out, float *row_lse,
                                       float *score_head, float *score_mean);

/* ---- steps 2-4: partition, merge, compact -------------------------------- */

typedef struct {
    const void *src;      /* device [B, N, row_elems]                                 */
    void *dst;            /* device [B, N - r, row_elems]; must not overlap src       */
    int64_t src_stride_b; /* elements between batches of src (>= N * row_elems)       */
    int64_t dst_stride_b; /* elements between batches of dst (>= (N-r) * row_elems)   */
    int32_t row_elems;    /* elements per token row (rows are contiguous)             */
    int32_t dtype;        /* LVLM_BF16, LVLM_F32; LVLM_I32 only with LVLM_RULE_TOP    */
    int32_t merge_rule;   /* lvlm_merge_rule                                          */
    int32_t reserved;
} lvlm_plane;

typedef struct {
    int32_t B, N;      /* batch, tokens per sequence before the step            */
    int32_t img_begin; /* first image token                                     */
    int32_t n_img;     /* image tokens before the step                          */
    int32_t n_keep;    /* image tokens after it (1..n_img), merged slot included */
    int32_t n_planes;  /* 1..LVLM_MAX_PLANES                                    */
} lvlm_merge_desc;

typedef struct {
    const lvlm_merge_desc *desc;
    const lvlm_plane *planes; /* HOST array of desc->n_planes entries */
} lvlm_merge_query;

/* Sec. 3.2.1, par. 4.  With r = n_img - n_keep: P_unmerged = the n_img-(r+1)
 * highest-scoring image tokens, P_merged = the other r+1 ordered by importance
 * (ties: lower index first; NaN below every number).  The merged token is
 * P_new = sum_k w[k] * P_merged[k]; every plane is rewritten as
 *   [rows before the image span | P_unmerged in ascending original index |
 *    P_new | rows after the image span].
 * r == 0 copies every plane unchanged (nothing is merged or moved).
 * score_mean: device fp32 [B, n_img].
 * w: device fp32 [r+1] rank -> weight table, or NULL for LVLM_MERGE_LINEAR_RANK
 *    evaluated on the device.
 * planes: HOST array of n_planes entries.
 * keep_idx [B, n_keep-1] i32 ascending, merged_idx [B, r+1] i32 in rank order:
 *    device outputs, indices relative to img_begin (for r == 0 neither list is
 *    written: nothing was partitioned).  Either may be NULL.
 * Accumulation is fp32 in a fixed order; the result is rounded to the plane
 * dtype with round-to-nearest-even.  Workspace: LVLM_OP_MERGE. */
LVLM_API lvlm_status lvlm_merge_compact(lvlm_ctx *ctx, void *stream, const lvlm_merge_desc *d,
                               const float *score_mean, const float *w,
                               const lvlm_plane *planes,
                               int32_t *keep_idx, int32_t *merged_idx);

/* ---- step 3b: similarity merge -------------------------------------------- */

/* A merge by similarity instead of by rank weights.  This variant is named by the
 * task this library was built for, not by the paper (whose Sec. 3.2.1 deliberately
 * avoids clustering); its definition is this library's:
 *   dominant tokens = the n_keep highest-scoring image tokens (order as in
 *   lvlm_merge_compact); every other image token is assigned to the dominant token
 *   with the largest cosine similarity between their rows of planes[0] (bf16 / fp32
 *   plane whose row is a multiple of 16 bytes and whose image rows span less than
 *   2 GiB per batch row, else LVLM_ERR_UNSUPPORTED; ties: lower dominant position; the
 *   dot products run in the plane's dtype on the matrix cores with fp32
 *   accumulation); on LVLM_RULE_WEIGHTED planes each dominant token becomes
 *   sum(size * row) / sum(size) over itself and its assigned tokens (fp32, members in
 *   ascending index), on LVLM_RULE_TOP planes it keeps its own row.
 * Every plane is rewritten as [rows before the span | the n_keep dominant tokens in
 * ascending original index | rows after the span]; dst has N - (n_img - n_keep) rows.
 * size_in  [B, n_img] fp32 or NULL (all ones); size_out [B, n_keep] fp32 or NULL.
 * keep_idx [B, n_keep] i32: dominant tokens, ascending.  assign [B, n_img] i32: for
 * every token the position (0..n_keep-1) of the dominant token it ends up in.  Either
 * may be NULL.  n_keep == n_img copies every plane unchanged.
 * Workspace: LVLM_OP_MERGE_SIMILAR (queried with an lvlm_merge_query). */
LVLM_API lvlm_status lvlm_merge_similar(lvlm_ctx *ctx, void *stream, const lvlm_merge_desc *d,
                                        const float *score_mean, const lvlm_plane *planes,
                                        const float *size_in, float *size_out,
                                        int32_t *keep_idx, int32_t *assign);

/* ---- step 5: KV-cache compression ---------------------------------------- */

/* Cache layout (shared with lvlm_decode_attn), head-major so that each head's
 * ragged entry list is contiguous:
 *   k_cache, v_cache [B, Hkv, Lmax, hd]   dtype
 *   score            [B, Hkv, Lmax]       fp32  importance of each entry
 *   kind             [B, Hkv, Lmax]       u8    LVLM_KIND_*
 *   orig_pos         [B, Hkv, Lmax]       i32   position in the original sequence
 *   len              [B, Hkv]             i32   entries in use; slots >= len are free
 */
typedef struct {
    int32_t dtype;     /* LVLM_BF16 or LVLM_F32                                     */
    int32_t B, Hkv;
    int32_t hd;        /* 64 or 128                                                 */
    int32_t Lmax;      /* allocated slots per head                                  */
    int32_t len_bound; /* host-known upper bound of every len (0 = Lmax); sizes grids */
    int32_t mode;      /* lvlm_kv_mode                                              */
    int32_t order;     /* lvlm_kv_order                                             */
    int32_t budget;    /* LVLM_KV_BUDGET: entries to keep per head (>= 1)           */
    int32_t n_recent;  /* LVLM_KV_BUDGET: last n_recent slots are never evicted     */
    double beta;       /* LVLM_KV_THRESHOLD: score-mass fraction to keep            */
} lvlm_kv_desc;

/* Independently for every (batch, KV head) (Sec. 3.2.2):
 * LVLM_KV_THRESHOLD -- among entries of kind IMAGE, taken from the highest
 *   score down (ties: lower slot first), keep the shortest prefix whose
 *   accumulated score reaches beta * (sum of image scores), at least one;
 *   other kinds are always kept; beta >= 1 or a zero sum keeps everything.
 *   Sums are exact: each score is clamped to [0, 65536] (NaN -> 0), scaled by
 *   2^32 and truncated to an integer; target = ceil(beta * total) in fp64.
 * LVLM_KV_BUDGET -- if len > budget: keep kind PROTECTED and the last n_recent
 *   slots, then fill up to `budget` with the highest-scoring other entries
 *   (if the protected ones alone exceed the budget only they stay).
 * Survivors are then compacted in place in the chosen order, all five arrays
 * together, and len is updated.  n_evicted [B,Hkv] i32 (device, optional)
 * receives old len - new len.  Slots at or beyond the new len keep stale data.
 * len_bound is a promise the launch is sized by; a head that breaks it (len >
 * len_bound) is left exactly as it is, with n_evicted = 0.
 * A call that evicts nothing changes nothing; LVLM_KV_BUDGET with len_bound (or
 * Lmax) <= budget and no n_evicted launches nothing.  Workspace: LVLM_OP_KV_COMPRESS. */
LVLM_API lvlm_status lvlm_kv_compress(lvlm_ctx *ctx, void *stream, const lvlm_kv_desc *d,
                             void *k_cache, void *v_cache, float *score, uint8_t *kind,
                             int32_t *orig_pos, int32_t *len, int32_t *n_evicted);

/* ---- step 6: decode attention over the retained cache -------------------- */

typedef struct {
    int32_t dtype;     /* LVLM_BF16 or LVLM_F32: q, k_new, v_new, caches, out       */
    int32_t B, Hq, Hkv;
    int32_t hd;        /* 64 or 128                                                 */
    int32_t Lmax;
    int32_t len_bound; /* host-known upper bound of every len AFTER the append (0 = Lmax) */
    int32_t new_kind;  /* kind of the appended entry                                */
    int32_t new_pos;   /* orig_pos of the appended entry                            */
    float scale;       /* logit scale                                               */
    float score_decay; /* gamma in score <- gamma * score + mean_G(p)               */
    int32_t evict_budget; /* > 0: per-step compression in the same call (see below)  */
    int32_t evict_recent; /* the last evict_recent slots are never evicted           */
} lvlm_attn_desc;

/* Sec. 3.2.2: the current token attends only to the retained entries.
 * If k_new / v_new [B,Hkv,hd] are given, the entry is first appended at slot
 * len[b][g] (score 0, kind new_kind, orig_pos new_pos) and len += 1.  The
 * caller keeps len + 1 <= len_bound (<= Lmax); the lengths live on the device, so
 * a head that breaks this is handled there, without touching memory beyond the
 * bound: a head with len == len_bound is full -- the new entry is dropped
 * (nothing is overwritten, len stays) and the head attends to what it holds; a
 * head with len > len_bound attends to its first len_bound entries only, its
 * len is left alone and nothing is evicted from it.  A caller that cannot rule
 * this out compares len before and after.  Then for every query head h of KV head g:
 *   out[b][h] = sum_j softmax_j(scale * q[b][h] . k_j) * v_j,  j in [0, len[b][g])
 * with fp32 online softmax and accumulation, split over the entries and
 * recombined.  If `score` is not NULL every entry's importance is updated as
 *   score_j <- score_decay * score_j + (1/G) * sum_{h in g} p_j^h,
 * continuing the received-attention definition of Sec. 3.2.1 into decoding.
 * kind / orig_pos may be NULL when nothing is appended.  A head with len 0
 * writes zeros.
 * Per-step cache compression (Sec. 3.2.2 in steady state): with evict_budget > 0
 * (needs score, kind, orig_pos) a head whose length after the append exceeds
 * evict_budget then loses ONE entry, chosen on the updated scores exactly as
 * lvlm_kv_compress would with LVLM_KV_BUDGET, budget = that length - 1,
 * n_recent = evict_recent, LVLM_ORDER_FILL: the least important entry that is
 * not LVLM_KIND_PROTECTED and not among the last evict_recent slots (lowest
 * score, highest slot among equals); the last entry moves into its slot and
 * len drops by one.  A cache that is more than one entry over its budget
 * (e.g. right after prefill) is brought down with lvlm_kv_compress first.
 * Workspace: LVLM_OP_DECODE_ATTN. */
LVLM_API lvlm_status lvlm_decode_attn(lvlm_ctx *ctx, void *stream, const lvlm_attn_desc *d,
                             const void *q, const void *k_new, const void *v_new,
                             void *k_cache, void *v_cache, float *score, uint8_t *kind,
                             int32_t *orig_pos, int32_t *len, void *out);

/* How lvlm_decode_attn cuts a shape into launches (host arithmetic; for benchmarks and tests that reason about
 * the launch): every (batch, KV head) pair is split over *n_split workgroups of *split_len entries each (a multiple
 * of 32; a workgroup's four waves take 32-entry tiles in turn); *form = 0 every wave has at most one tile, 1 some
 * wave has a second tile (splits longer than 128 entries, or a remainder of up to one tile on the last split),
 * 2 whole 128-entry splits plus exactly one more entry, which one wave of the last split takes on its own (the
 * steady state of a cache at its budget, bf16 only). */
LVLM_API lvlm_status lvlm_decode_plan(const lvlm_ctx *ctx, const lvlm_attn_desc *d, int32_t *n_split, int32_t *split_len,
                                      int32_t *form);

/* The same call for callers that cannot allocate device memory or attach a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Arguments, results and error behaviour are those of
 * lvlm_decode_attn; the scratch (split partials, per-entry logits, lengths)
 * lives in a fixed array inside the library, LVLM_STATIC_SCRATCH_BYTES per GPU,
 * held from the first such call on that GPU until the process ends.  The
 * context's workspace is neither needed nor touched.  A shape whose scratch
 * (lvlm_workspace_bytes with LVLM_OP_DECODE_ATTN) exceeds the array is refused
 * with LVLM_ERR_WORKSPACE before anything is launched.  The call itself calls no
 * hipMalloc / hipFree.  All calls on one GPU share that GPU's array: calls that
 * may overlap in time (different streams, different threads) race; order them. */
#define LVLM_STATIC_SCRATCH_BYTES (8u << 20)
LVLM_API lvlm_status lvlm_decode_attn_static(lvlm_ctx *ctx, void *stream, const lvlm_attn_desc *d,
                                    const void *q, const void *k_new, const void *v_new,
                                    void *k_cache, void *v_cache, float *score, uint8_t *kind,
                                    int32_t *orig_pos, int32_t *len, void *out);

/* Diagnostic, not part of the path: one read-only pass over `bytes` (a multiple of 16) of device memory at src by
 * n_workgroups workgroups of 256 threads (contiguous shares, 16-byte loads, eight in flight per thread), timed like
 * any other kernel under lvlm_profile as "stream_probe".  It answers what a launch of a given size and shape can
 * stream on the device at hand -- the yardstick for the decode-attention launches, which move a few to a few tens of
 * MB each.  sink: one device word the kernel may write (it never does for ordinary data). */
LVLM_API lvlm_status lvlm_stream_probe(lvlm_ctx *ctx, void *stream, const void *src, size_t bytes, int32_t n_workgroups,
                                       uint32_t *sink);

#ifdef __cplusplus
}
#endif
#endif /* LVLM_H */
