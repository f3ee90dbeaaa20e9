/*
 * tri.h -- C ABI of the MI355X (gfx950) TriAttention KV-cache compression step.
 *
 * The step, per (sequence, layer, KV head) -- a "head-instance" -- over its N cached
 * pre-RoPE keys:
 *   1. score    S~(g)(k): trigonometric-series score + concentration-weighted norm score,
 *               averaged over the future offsets D, for each of the G query heads that share
 *               the KV head                                   (Sections 4.1, 4.2)
 *   2. reduce   z-score every head's scores over the N keys, take the maximum over the
 *               G heads -> S_final(k)                         (Section 4.3, GQA)
 *   3. select   the B keys with the largest S_final           (Section 4.3)
 *   4. compact  move the survivors' K, V and positions to the front of the cache
 *               ("evict the rest", Section 4.3)
 *
 * Conventions for every entry point
 *   - Every pointer is a DEVICE pointer owned by the caller, except tri_model itself, the
 *     tri_cache structs themselves and tri_model::offsets, which are HOST memory read during
 *     the call only.  The library allocates nothing and keeps no pointer after a call returns.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls only
 *     enqueue work on that stream; they never synchronise.  Arguments are validated on the
 *     host before anything is enqueued; on error nothing is enqueued.
 *   - Return value: TRI_OK or a negative tri_status.  Nothing aborts or throws.
 *     tri_last_error() returns a static string describing the last failure on the calling thread.
 *   - Non-finite key or statistics values: behaviour undefined.
 *   - Built geometries: head_dim 128 (64 frequency bands) and n_q_heads / n_kv_heads (= G) from 1 to 8; anything
 *     else returns TRI_ERR_UNSUPPORTED.  n_layers and n_seqs * n_kv_heads must each be below 65536, and
 *     head-instances x max(max_seq_len / 256, budget / 8) below 2^31 per call (TRI_ERR_UNSUPPORTED otherwise: split
 *     the batch).  Positions, cur_pos and cur_pos + max(offsets) must be below 2^62 in magnitude (positions
 *     and cur_pos are int32).
 */
#ifndef TRI_H
#define TRI_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    TRI_OK = 0,
    TRI_ERR_INVALID_ARG = -1, /* a NULL pointer, a size or stride out of range        */
    TRI_ERR_UNSUPPORTED = -2, /* a head_dim / group size / layout this build lacks   */
    TRI_ERR_WORKSPACE = -3,   /* workspace NULL, misaligned (256 B) or too small      */
    TRI_ERR_HIP = -4          /* a HIP launch reported an error                       */
} tri_status;

typedef enum { TRI_F32 = 0, TRI_BF16 = 1 } tri_dtype;

/* which two elements of a head vector form frequency band f */
typedef enum {
    TRI_PAIR_INTERLEAVED = 0, /* (x[2f], x[2f+1]) -- Section 2.1 Eq. 1                  */
    TRI_PAIR_HALF = 1         /* (x[f], x[f + head_dim/2]) -- half-split checkpoints  */
} tri_pair_layout;

/* which components the score is made of: the method, and the variants its ablation study removes a
 * component from (Section 5, ablations of the scoring components and of the adaptive weighting) */
typedef enum {
    TRI_SCORE_FULL = 0,           /* S_trig + S_norm (Sections 4.1-4.2)                          */
    TRI_SCORE_TRIG_ONLY = 1,      /* S_trig alone ("w/o S_norm")                                  */
    TRI_SCORE_NORM_ONLY = 2,      /* S_norm alone ("w/o S_trig")                                  */
    TRI_SCORE_NORM_UNWEIGHTED = 3 /* S_trig + S_norm^(0) = sum_f E||q_f|| ||k_f|| ("w/o R")       */
} tri_score_variant;

/* Model geometry and the scoring hyper-parameters (Section 2.1: omega_f = theta^(-2f/d);
 * Section 4.2: the offset set D, geometric in the paper). */
typedef struct tri_model {
    int32_t n_layers;
    int32_t n_q_heads;
    int32_t n_kv_heads;
    int32_t head_dim;
    double rope_theta;
    int32_t pairs;          /* tri_pair_layout */
    int32_t n_offsets;      /* |D| >= 1 */
    const int64_t *offsets; /* HOST array [n_offsets] */
    int32_t score_variant;  /* tri_score_variant; 0 = the method */
    const int32_t *head_budgets; /* NULL: every head-instance keeps `budget` keys (the paper's setting).  Else DEVICE
                               [n_layers][n_kv_heads]: the budget of each (layer, KV head), read into [0, budget]
                               (head-specific budgets, named as future work in Appendix A).  `budget` stays the
                               stride of kept_idx; kept_cnt holds min(N_s, the head's budget); new_seq_len
                               then reports layer 0, head 0 only */
} tri_model;

/*
 * A KV cache holding keys (pre-RoPE, or post-RoPE with k_rotated), values and key positions for n_layers x n_seqs x n_kv_heads
 * head-instances.  One descriptor covers both layouts:
 *   contiguous (block_size == 0): slot n of (layer l, sequence s, head h) is at element
 *       l*stride_layer + s*stride_seq_or_block + h*stride_head + n*stride_slot
 *   paged (block_size > 0, a power of two): with b = block_table[s*max_blocks_per_seq + n/block_size],
 *       l*stride_layer + b*stride_seq_or_block + h*stride_head + (n % block_size)*stride_slot
 * of k and of v (elements of `dtype`; a slot's head_dim elements are contiguous and 16-byte
 * aligned).  Positions use the same formula with the pos_* strides and a slot stride of 1;
 * they are stored per head because heads keep different tokens once compacted.
 */
typedef struct tri_cache {
    void *k;
    void *v; /* may be NULL for tri_score / tri_select_topk */
    int32_t *pos;
    int32_t dtype;                /* tri_dtype */
    int32_t n_seqs;               /* S */
    const int32_t *seq_len;       /* device [S]: N_s, number of occupied slots          */
    const int32_t *cur_pos;       /* device [S]: p_q, position of the current query      */
    int32_t max_seq_len;          /* host upper bound on every N_s (sizes grids and the N stride of score arrays);
                                     a seq_len entry outside [0, max_seq_len] is read as the nearer bound */
    int32_t block_size;           /* 0 = contiguous */
    const int32_t *block_table;   /* device [S][max_blocks_per_seq], paged only           */
    int32_t max_blocks_per_seq;
    int64_t stride_layer, stride_seq_or_block, stride_head, stride_slot;
    int64_t pos_stride_layer, pos_stride_seq_or_block, pos_stride_head;
    int32_t k_rotated;            /* 0: k holds pre-RoPE keys (the paper's setting).  1: k holds post-RoPE keys,
                                     each already rotated by its own position (Section 2.1 Eq. 1), as serving
                                     stacks usually store them; the scores are the same, the rotation of the key
                                     in the score kernel is skipped and pos is read by tri_compact only */
} tri_cache;

const char *tri_last_error(void);

/*
 * Offline calibration (Section 4.1 text under both score equations; Appendix B.5): per
 * (layer, query head, band f) the complex mean of the pre-RoPE query samples, E[q_f], and the
 * mean modulus E||q_f||.
 *   q_samples    device [n_tokens][n_layers][n_q_heads][head_dim], q_dtype, 16-byte aligned
 *   centers_out  device [n_layers][n_q_heads][head_dim/2][3] float = (Re E[q_f], Im E[q_f], E||q_f||)
 * Sums are accumulated in double in a fixed order (deterministic).  n_tokens >= 1.
 */
tri_status tri_build_centers(const tri_model *model, const void *q_samples, int32_t q_dtype,
                             int64_t n_tokens, float *centers_out, void *stream);

/*
 * The same calibration as a stream of chunks (Appendix H calibrates on 50 k to 960 k tokens, more than fits
 * beside a model): every call adds the sums of its chunk -- sum Re q_f, sum Im q_f, sum ||q_f|| -- to
 *   sums  device [n_layers][n_q_heads][head_dim/2][3] double
 * (first != 0: the chunk's sums overwrite `sums` instead, so no separate clearing is needed), and
 * tri_centers_finalize divides by the total number of tokens and writes the table tri_build_centers writes.
 * Chunks are accumulated in the order of the calls on the stream; within a chunk the order is fixed.
 */
tri_status tri_centers_accumulate(const tri_model *model, const void *q_samples, int32_t q_dtype,
                                  int64_t n_tokens, double *sums, int32_t first, void *stream);
tri_status tri_centers_finalize(const tri_model *model, const double *sums, int64_t total_tokens,
                                float *centers_out, void *stream);

/*
 * Concentration and dominant-band diagnostics of a statistics table (Appendix B.5, B.7):
 *   mrl_out        device [n_layers][n_q_heads][F] float: R_f = ||E[q_f]|| / E||q_f|| (0 for an all-zero band)
 *   contrib_out    NULL, or device [n_layers][n_q_heads][F] float: C_f = E||q_f|| * E||k_f||, the KV head of
 *                  query head h being h / G
 *   top_bands_out  NULL, or device [n_layers][n_q_heads][top_k] int32: the top_k bands by C_f, largest first,
 *                  equal contributions by ascending band
 *   k_centers      device [n_layers][n_kv_heads][F][3]: the table tri_build_centers writes for key samples
 *                  (built with a model whose n_q_heads is n_kv_heads); may be NULL when only mrl_out is wanted
 */
tri_status tri_band_diagnostics(const tri_model *model, const float *q_centers, const float *k_centers,
                                float *mrl_out, float *contrib_out, int32_t top_k,
                                int32_t *top_bands_out, void *stream);

/* Bytes of scratch tri_score / tri_select_topk / tri_compress_step need for this model, cache
 * geometry and budget (the maximum over the three).  0 on invalid arguments.
 * Where the workspace lies in physical memory relative to the K cache changes the score kernel's time by up to 8 %
 * on MI355X (its raw-score writes against its K reads; offsets inside one allocation do not matter, the allocation
 * does).  A caller that sets up once and runs many steps may allocate a few candidate workspaces some GB apart, time
 * one tri_score on each and keep the fastest. */
size_t tri_workspace_size(const tri_model *model, const tri_cache *cache, int32_t budget);

/*
 * Steps 1-2: scores of every cached key (Sections 4.1-4.3).
 *   centers    device [n_layers][n_q_heads][F][3], as written by tri_build_centers
 *   final_out  device [n_layers][n_seqs][n_kv_heads][max_seq_len] float: S_final; entries at
 *              n >= N_s are not written
 *   raw_out    NULL, or device [n_layers][n_seqs][n_q_heads][max_seq_len] float: S~(g), query
 *              head h*G+g belonging to KV head h
 *   workspace  device, 256-byte aligned, ws_bytes >= tri_workspace_size(); contents undefined after.
 *              It holds tables, partial sums and the score kernel's work list and item counter: calls that
 *              may overlap in time (different streams) need a workspace each
 * sigma is the population standard deviation; a head with sigma = 0 contributes 0 to the maximum.
 */
tri_status tri_score(const tri_model *model, const float *centers, const tri_cache *cache,
                     float *final_out, float *raw_out, void *workspace, size_t ws_bytes,
                     void *stream);

/*
 * Step 3: per head-instance the min(N_s, budget) keys with the largest final score, equal
 * scores resolved in favour of the lower slot index (-0.0 equals +0.0).
 *   final_scores  device [n_layers][n_seqs][n_kv_heads][max_seq_len] float
 *   kept_idx      device [n_layers][n_seqs][n_kv_heads][budget] int32: kept slots, ascending;
 *                 entries past the count are not written
 *   kept_cnt      device [n_layers][n_seqs][n_kv_heads] int32 = min(N_s, budget)
 */
tri_status tri_select_topk(const tri_model *model, const float *final_scores,
                           const tri_cache *cache, int32_t budget, int32_t *kept_idx,
                           int32_t *kept_cnt, void *workspace, size_t ws_bytes, void *stream);

/*
 * Step 4: slot j of dst <- slot kept_idx[j] of src, for K, V and positions, j < kept_cnt.
 * dst may describe the same memory as src (in-place compaction; also for the paged layout,
 * where the survivors fill the sequence's first blocks and the caller frees the rest): it must
 * then be the same mapping -- the same k, v, pos, strides and block table -- or the call returns
 * TRI_ERR_INVALID_ARG.  If dst is a different cache it must not overlap src; it uses its own strides / block
 * table, needs room for min(max_seq_len, budget) slots per sequence only, and takes src's n_seqs and dtype;
 * dst->seq_len, cur_pos and max_seq_len are ignored.
 *   new_seq_len  NULL or device [n_seqs] int32 <- min(N_s, budget)
 * kept_idx must be ascending and free of duplicates per head-instance (as tri_select_topk writes it);
 * otherwise the result is unspecified, but a count is read into [0, budget] and a slot index into
 * [0, src->max_seq_len - 1], so no memory outside the caches is touched.
 */
tri_status tri_compact(const tri_model *model, const tri_cache *src, const tri_cache *dst,
                       int32_t budget, const int32_t *kept_idx, const int32_t *kept_cnt,
                       int32_t *new_seq_len, void *stream);

/*
 * Step 4 for callers that do not need the survivors in slot order (attention treats the cached keys as a set;
 * each key carries its own position): in-place eviction that moves as few slots as possible.  Kept keys that
 * already sit in slots [0, kept_cnt) stay where they are; the i-th free slot below kept_cnt (ascending)
 * receives the i-th kept key stored at or beyond kept_cnt (ascending), with its V row and position.  In the
 * steady state of Section 4.3 (a budget of keys plus one window of 128 new tokens) this moves at most 128 slots
 * per head-instance instead of nearly all of them.  Arguments as tri_compact with dst = src = cache.
 */
tri_status tri_compact_fill(const tri_model *model, const tri_cache *cache, int32_t budget,
                            const int32_t *kept_idx, const int32_t *kept_cnt, int32_t *new_seq_len,
                            void *stream);

/*
 * Steps 1-4 in one call.  Same arguments and results as the three calls above; raw scores and
 * their statistics live in the workspace only and the selection forms the final scores itself.
 * dst == NULL evicts in place with tri_compact_fill (fewest moves, slot order not preserved).
 */
tri_status tri_compress_step(const tri_model *model, const float *centers, const tri_cache *src,
                             const tri_cache *dst, int32_t budget, int32_t *kept_idx,
                             int32_t *kept_cnt, int32_t *new_seq_len, void *workspace,
                             size_t ws_bytes, void *stream);

/*
 * tri_compress_step for callers that cannot allocate device memory and have no workspace to pass: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments (without the workspace)
 * and the same results as tri_compress_step; the scratch memory is an array inside the library,
 * tri_static_scratch_size() bytes (64 MiB) on every GPU the library is used on, held until the process ends.
 * The call allocates nothing (no hipMalloc / hipFree, no allocating library routine); a call whose
 * tri_workspace_size() exceeds the array returns TRI_ERR_WORKSPACE and enqueues nothing.  Every call on a GPU uses
 * that GPU's one array: two calls that may overlap in time on one GPU (different streams or threads) race --
 * serialise them, or give the second one tri_compress_step with a workspace of its own.
 */
size_t tri_static_scratch_size(void);
tri_status tri_compress_step_static(const tri_model *model, const float *centers, const tri_cache *src,
                                    const tri_cache *dst, int32_t budget, int32_t *kept_idx,
                                    int32_t *kept_cnt, int32_t *new_seq_len, void *stream);

/*
 * Measurement hook for benchmark harnesses (no counterpart in the paper).  After attaching, the
 * i-th launch of the score kernel made by the calling thread (i = 0, 1, ...) is bracketed by
 * hipEventRecord(events[2i]) before and hipEventRecord(events[2i+1]) after it, on the stream of
 * that launch, until n_pairs launches have been bracketed.  `events` is a HOST array of
 * 2*n_pairs hipEvent_t created by the caller with timing enabled; it must stay valid until
 * tri_timing_detach(), which returns the number of launches bracketed since the attach.
 */
tri_status tri_timing_attach(void **events, int32_t n_pairs);
int32_t tri_timing_detach(void);

#ifdef __cplusplus
}
#endif
#endif /* TRI_H */
