/*
 * mp.h -- C ABI of the MI355X (gfx950) Multipole Attention decode library.
 *
 * The library implements, on one GPU, the decode hot path of Multipole Attention
 * (arXiv 2506.13059): a clustered key/value index per (sequence, KV head), centroid scoring
 * (coarse level, then fine level), budgeted selection of clusters, exact softmax attention over
 * the selected clusters' keys, and one centroid term per remaining cluster inside the same softmax.
 *
 * General conventions
 *   - "unit" u = b * n_kv_heads + kv_head.  Query head h uses KV head h / G with
 *     G = n_q_heads / n_kv_heads (grouped-query attention, Sec. 3.1 last paragraph).
 *   - Every pointer documented "device" is a device pointer the caller owns (for instance the
 *     data_ptr() of a torch tensor); pointers documented "host" are ordinary host memory.
 *     Tensors are dense, row-major, in the stated shape.  bf16 = bfloat16.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  All device work is
 *     enqueued on it and the call returns without waiting for the GPU, unless stated otherwise.
 *   - Every function returns an mp_status; mp_last_error() gives a readable message.  Argument,
 *     state and capacity errors (MP_EINVAL, MP_ESTATE, MP_ECAPACITY, MP_ENOMEM) are found before
 *     anything is enqueued and leave the context unchanged.  MP_EHIP means a HIP runtime call
 *     failed, possibly after part of the call's work was enqueued: outputs are then undefined, and
 *     if the call was building or updating the index (mp_cluster_kv, mp_set_clustering,
 *     mp_update_clusters, a refreshing mp_decode_step) the context has no index any more (calls that
 *     need one return MP_ESTATE until the next successful mp_cluster_kv / mp_set_clustering).
 *     No C++ exception crosses this boundary.
 *   - head_dim must be 128.  1 <= G <= 8.
 *   - A context may be used from one host thread at a time; calls on the same context that
 *     overlap on the GPU (different streams without ordering) race on its workspace.
 */
#ifndef MP_H_
#define MP_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct mp_ctx mp_ctx;

typedef enum {
    MP_OK = 0,
    MP_EINVAL = 1,    /* bad argument: null pointer, size out of range, unsupported shape      */
    MP_ENOMEM = 2,    /* device or host allocation failed                                       */
    MP_ESTATE = 3,    /* call order: decode / update / getters before an index exists           */
    MP_ECAPACITY = 4, /* tokens or clusters beyond the capacities given at mp_create            */
    MP_EHIP = 5       /* a HIP runtime call failed; the message carries hipGetErrorString       */
} mp_status;

typedef struct {
    int32_t batch;         /* B >= 1                                                            */
    int32_t n_q_heads;     /* Hq, multiple of n_kv_heads                                        */
    int32_t n_kv_heads;    /* Hkv >= 1                                                          */
    int32_t head_dim;      /* must be 128                                                       */
    int32_t max_tokens;    /* capacity: clustered tokens per unit                               */
    int32_t levels;        /* 1 = fine clusters only (Sec. 3.1-3.2), 2 = coarse + fine (Sec. 3.4) */
    int32_t max_fine;      /* capacity: fine clusters per unit (<= 8192)                        */
    int32_t max_coarse;    /* capacity: coarse clusters per unit (0 allowed when levels == 1)   */
    int32_t block_w;       /* W of Sec. 3.3: clustering block length; 0 = one block             */
    int32_t block_alpha;   /* alpha of Sec. 3.3: the last block holds alpha .. W+alpha-1 tokens */
    int32_t max_tail;      /* capacity: unclustered newest tokens per unit passed to decode     */
    int32_t lookup_keys;   /* 1: clusters are formed on separate lookup keys (see mp_cluster_kv) */
    float softmax_scale;   /* multiplies every q.k and q.centroid product; 0 => 1/sqrt(head_dim) */
    int32_t kv_format;     /* storage of the clustered keys and values: MP_KV_BF16 or MP_KV_E4M3     */
} mp_config;

/* Storage formats of the clustered cache (the keys and values that are attended exactly).
 *
 * MP_KV_BF16  rows are kept as handed over.
 * MP_KV_E4M3  8-bit rows (KV quantisation is complementary to the method, Sec. 2.3).  A stored row is
 *             128 one-byte codes in the OCP e4m3 format (4 exponent bits, bias 7, 3 mantissa bits,
 *             subnormals, no infinities, largest magnitude 448) plus one fp32 scale:
 *               scale = fp32(max_d |x_d|) / 448 (fp32 division; 1 for an all-zero row),
 *               code_d = x_d / scale (fp32 division) rounded to the nearest e4m3 value, ties to
 *               the even code, magnitudes above 448 clamped,
 *             and stands for code * scale.  For a value row x is the row itself.  For a key row x is
 *             the residual from the key centroid c of the row's fine cluster, x_d = fp32(k_d) -
 *             fp32(c_d) (one fp32 subtraction), so that decode attends c + code * scale: the index
 *             already holds c and the scoring step already computes q.c, while e4m3's three
 *             mantissa bits on the key itself would put an error of several percent on every
 *             logit.  The centroid tables, the unclustered tail and every input stay bf16, and
 *             the centroids are means of the original rows, so the index is identical to the
 *             MP_KV_BF16 one.  Not available together with lookup_keys (MP_EINVAL: there the
 *             centroids are those of the lookup keys, not of the stored keys). */
#define MP_KV_BF16 0
#define MP_KV_E4M3 1

/* Create a context: allocates the clustered KV cache, the index tables and all workspaces on the
 * current HIP device (sizes follow the capacities in cfg).  *out receives the context.
 * Errors: MP_EINVAL (bad cfg, checked before any HIP call), MP_ENOMEM, MP_EHIP. */
mp_status mp_create(const mp_config* cfg, mp_ctx** out);

/* Free everything the context owns.  Synchronises the device first.  NULL is allowed. */
void mp_destroy(mp_ctx* ctx);

/* Message of the last failing call on this context (or, with ctx == NULL, of the last failing
 * mp_create / context-free call on this thread).  Never NULL; valid until the next call. */
const char* mp_last_error(const mp_ctx* ctx);

/* Device bytes the context holds (cache + tables + workspace). */
size_t mp_device_bytes(const mp_ctx* ctx);

/* ---------------------------------------------------------------------------------------------
 * Block plan (Sec. 3.3): clustering runs in blocks of block_w tokens; the last block holds the
 * remaining block_alpha .. block_w+block_alpha-1 tokens (all tokens if there are fewer than
 * block_w+block_alpha, or if block_w == 0).  n_fine / n_coarse (totals per unit) are split over
 * the blocks by cumulative integer division: block [t0,t1) owns fine ids
 * [n_fine*t0/n_tokens, n_fine*t1/n_tokens), coarse ids likewise.
 *
 * Writes up to max_blocks entries of 6 int32 {t0, t1, f0, f1, c0, c1} to `out` (host) and returns
 * the number of blocks (also when out == NULL); returns -1 on invalid arguments.
 * ------------------------------------------------------------------------------------------- */
int32_t mp_plan_blocks(int32_t n_tokens, int32_t block_w, int32_t block_alpha, int32_t n_fine,
                       int32_t n_coarse, int32_t* out, int32_t max_blocks);

/* ---------------------------------------------------------------------------------------------
 * mp_cluster_kv -- build the clustered index for tokens [0, n_tokens) of every unit
 * (Sec. 3.1: k-means on the keys, key centroid = mean of the member keys; Sec. 3.2: value
 * centroid = mean of the member values; Sec. 3.3: blockwise; Sec. 3.4: second level by k-means
 * on the fine centroids).
 *
 *   k, v        device bf16 [B, Hkv, n_tokens, 128], read-only; not referenced after the enqueued
 *               work has run (the context keeps its own cluster-contiguous copy).
 *   n_fine      fine clusters per unit (total over blocks), 1 <= n_fine <= max_fine,
 *               each block must get at least one and at most as many as it has tokens.
 *   n_coarse    coarse clusters per unit (levels == 2; each block needs 1 <= count <= its fine
 *               count); ignored when levels == 1.
 *   iters       Lloyd iterations (>= 1) at each level, no early stop (Sec. 5.1 uses 10).
 *   init_fine   host int32 [B*Hkv, n_fine]: seeds, block after block, each the index of a token
 *               inside its block (distinct per block, else MP_EINVAL).  NULL: drawn from `seed`.
 *   init_coarse host int32 [B*Hkv, n_coarse]: seeds of the coarse level, each the index of a fine
 *               cluster inside its block, numbered as produced by the fine k-means (= position of
 *               its seed in init_fine); distinct per block, else MP_EINVAL.  NULL: drawn from `seed`.
 *
 * Per block: centroids start at the seed keys; each iteration assigns every key to the nearest
 * centroid (squared Euclidean distance in fp64, equal distances -> lowest index) and replaces each
 * non-empty cluster's centroid by the bf16-rounded (nearest-even) fp64 mean of its members; empty
 * clusters keep their centroid.  The coarse level repeats this with the fine centroids as points.
 * Fine clusters are then renumbered so that the children of a coarse cluster are contiguous
 * (stable in the old number), tokens are stored cluster after cluster (sequence order inside a
 * cluster), and the stored tables hold, per cluster, N, bf16(mean key), bf16(mean value) (an empty
 * cluster keeps its k-means centroid as key centroid and a zero value centroid).
 *
 * Lookup keys (Sec. 3.1, last paragraph: keys rotated to a fixed relative position before
 * clustering, so that position-dependent rotation does not scatter similar keys).  A context
 * created with lookup_keys = 1 takes, wherever keys are handed over, a second array k_lookup of
 * the same shape: the clusters are formed on k_lookup and the key centroids are means of
 * k_lookup rows, while k is what is stored and attended exactly.  The rotation itself is the
 * caller's business.  k_lookup must be NULL for any other context (MP_EINVAL otherwise, and when
 * it is missing for a lookup context).
 *
 * Errors: MP_EINVAL, MP_ECAPACITY (n_tokens > max_tokens, n_fine > max_fine, ...), MP_EHIP.
 * Replaces any previous index of the context.
 * ------------------------------------------------------------------------------------------- */
mp_status mp_cluster_kv(mp_ctx* ctx, const void* k, const void* k_lookup, const void* v, int32_t n_tokens,
                        int32_t n_fine, int32_t n_coarse, int32_t iters, uint64_t seed, const int32_t* init_fine,
                        const int32_t* init_coarse, void* stream);

/* ---------------------------------------------------------------------------------------------
 * mp_set_clustering -- install an index from a given assignment instead of running k-means
 * (same stored tables and layout as mp_cluster_kv; one block).
 *
 *   fine_of_token   device int32 [B*Hkv, n_tokens], values in [0, n_fine)
 *   coarse_of_fine  device int32 [B*Hkv, n_fine], values in [0, n_coarse), NON-DECREASING in the
 *                   fine id (children contiguous); NULL when levels == 1.
 * Empty clusters get zero centroids and N = 0.  Out-of-range ids are undefined behaviour on the
 * device side (they are not read back to be checked).
 * ------------------------------------------------------------------------------------------- */
mp_status mp_set_clustering(mp_ctx* ctx, const void* k, const void* k_lookup, const void* v, int32_t n_tokens,
                            const int32_t* fine_of_token, int32_t n_fine,
                            const int32_t* coarse_of_fine, int32_t n_coarse, void* stream);

/* ---------------------------------------------------------------------------------------------
 * mp_update_clusters -- append n_new tokens per unit to the last block and refresh its clusters
 * (Sec. 3.3; the coarse level follows Sec. 3.4's remark that the blockwise update applies at every
 * level).  Per unit, with the last block's fine clusters [f0,f1) and coarse clusters [c0,c1):
 *
 *   1. n_new_fine new fine clusters are appended (ids f1..), each seeded with one appended key.
 *   2. one-shot step: every appended token is assigned to its nearest centroid among the block's
 *      stored fine key centroids and the new seeds (centroids frozen); every touched centroid moves
 *      to bf16((N c + sum of its newly assigned keys, sequence order) / (N + n)).
 *   3. refine_iters full Lloyd iterations over all tokens of the last block, from those centroids
 *      (refine_iters == 0: old tokens keep their cluster, appended ones keep the one-shot choice).
 *   4. two levels: n_new_coarse new coarse clusters are appended, each seeded with the working
 *      centroid of one NEW fine cluster; max(1, refine_iters) Lloyd iterations over the block's fine
 *      working centroids, starting from the stored coarse key centroids and the seeds.
 *   5. the last block is renumbered, re-stored and its tables recomputed exactly as in
 *      mp_cluster_kv (stored centroids = bf16 means of the members; empty clusters keep their
 *      working centroid).  Earlier blocks are untouched.
 *   6. if the last block now holds >= block_w + block_alpha tokens (block_w > 0), its first block_w
 *      tokens become a block of their own and the rest the new last block; both are clustered
 *      afresh (split_iters Lloyd iterations per level, Sec. 5.1 uses 10) with the block's kf fine
 *      and kc coarse clusters shared out as kf*block_w/nb (integer division) to the first part and
 *      the remainder to the second, nb = tokens in the block.
 *
 *   k_new, v_new   device bf16 [B, Hkv, n_new, 128]
 *   k_new_lookup   lookup keys of the appended tokens (same shape; contexts with lookup_keys only,
 *                  else NULL): every step above then works on lookup keys, k_new is only stored
 *   n_new_fine     0 <= n_new_fine <= n_new;  n_new_coarse: 0 <= n_new_coarse <= n_new_fine
 *   seeds          host int32 [B*Hkv, total], total and the six list lengths from
 *                  mp_update_seed_counts(): {n_new_fine indices into the appended tokens,
 *                  n_new_coarse indices into the new fine clusters, and -- only when step 6 applies --
 *                  fine seeds of the first part (token index inside it), fine seeds of the second
 *                  part, coarse seeds of the first part (fine-cluster index inside it), coarse seeds
 *                  of the second part}; every list holds distinct indices.  NULL: drawn from `seed`.
 * The last block may grow to at most 2*block_w tokens by one call (any size when block_w == 0, up
 * to max_tokens).  Errors: MP_ESTATE (no index yet), MP_ECAPACITY, MP_EINVAL, MP_EHIP.
 * ------------------------------------------------------------------------------------------- */
int32_t mp_update_seed_counts(const mp_ctx* ctx, int32_t n_new, int32_t n_new_fine, int32_t n_new_coarse,
                              int32_t* counts /* host int32 [6] */);   /* returns total, -1 on bad arguments */
mp_status mp_update_clusters(mp_ctx* ctx, const void* k_new, const void* k_new_lookup, const void* v_new,
                             int32_t n_new, int32_t n_new_fine, int32_t n_new_coarse, int32_t refine_iters,
                             int32_t split_iters, uint64_t seed, const int32_t* seeds, void* stream);

/* ---------------------------------------------------------------------------------------------
 * mp_decode_attention -- one decode step for every unit (Eq. 1, Eq. 2, Sec. 3.4, Sec. 4).
 *
 *   q               device bf16 [B, Hq, 128]
 *   q_lookup        device bf16 [B, Hq, 128] or NULL (= q): the query compared with the centroids
 *                   (Sec. 3.1, last paragraph: a query rotated to the fixed position that matches
 *                   the lookup keys).  It gives every centroid logit, including those of the Eq. 2
 *                   terms (Sec. 4: the replacement stage reuses the lookup's products); q itself
 *                   meets the stored keys and the tail.  Must be NULL for a context with
 *                   MP_KV_E4M3 (MP_EINVAL): its stored keys are residuals from the centroids, and
 *                   the centroid's share of an exact logit is the lookup's product.
 *   k_tail, v_tail  device bf16 [B, Hkv, tail_stride, 128], of which the first n_tail rows of every
 *                   unit are used: newest tokens that are not clustered yet (the local buffer of
 *                   Sec. 4); always attended exactly; NULL with n_tail == 0.
 *   tail_stride     rows between consecutive units in k_tail / v_tail (>= n_tail), so that a buffer
 *                   of fixed capacity can fill up in place; 0 means n_tail (densely packed).
 *   key_budget      keys of selected fine clusters per unit (>= 0; >= n_tokens => full attention;
 *                   0 => every cluster enters through its centroid).  Tail tokens do not count.
 *   coarse_budget   keys covered by the "promising" coarse clusters whose children are scored at
 *                   the fine level (levels == 2; ignored otherwise).
 *   flags           MP_DECODE_NO_MULTIPOLE drops the centroid terms of Eq. 2 (sparse attention
 *                   over the retrieved keys only).
 *   out             device bf16 [B, Hq, 128]
 *   lse             device fp32 [B, Hq], natural log of the softmax denominator; may be NULL.
 *
 * Per unit: coarse logits l = scale*q.Kc for clusters with N > 0, Eq. 1 per head with the
 * N-weighted denominator, averaged over the G heads of the group (ranked through its logarithm);
 * clusters ordered by that key (ties: lower id first) are taken while the running token count
 * stays <= the budget, stopping at the first that does not fit; the fine level repeats this over
 * the children of the promising coarse clusters, with the Eq. 1 denominator running over those
 * children and the unpromising coarse clusters.  The output is one softmax over the exact keys of
 * the selected clusters, the tail, and N*exp(l) terms carrying the value centroids of all other
 * clusters (unselected candidates at the fine level, unpromising clusters at the coarse level).
 * Centroid logits and rank keys are evaluated in fp64; exact attention uses bf16 inputs with
 * fp32 accumulation.
 *
 * Allocates nothing, never waits for the GPU, reads nothing back.
 * Errors: MP_ESTATE (no index), MP_EINVAL (null, negative sizes, 0 < tail_stride < n_tail),
 * MP_ECAPACITY (n_tail > max_tail).
 * ------------------------------------------------------------------------------------------- */
#define MP_DECODE_NO_MULTIPOLE 1u
mp_status mp_decode_attention(mp_ctx* ctx, const void* q, const void* q_lookup, const void* k_tail,
                              const void* v_tail, int32_t n_tail, int32_t tail_stride, int32_t key_budget,
                              int32_t coarse_budget, uint32_t flags, void* out, float* lse, void* stream);

/* ---------------------------------------------------------------------------------------------
 * Library-managed local buffer (Sec. 4 and Sec. 5.1: the newest L to 2L tokens are kept out of the
 * clusters and attended exactly at every step; every L steps the oldest L of them are appended to
 * the clusters; a few first "sink" tokens are never clustered).  Optional: callers that keep
 * their own tail buffer use mp_decode_attention and mp_update_clusters directly.
 *
 * mp_local_buffer_init sets the window L, copies n_sink sink tokens and the n_recent newest tokens
 * (0 <= n_recent < 2L, in sequence order) into the context's buffer.  k_* / v_*: device bf16
 * [B, Hkv, n, 128], read on the stream, may be NULL when n == 0.  Needs n_sink + 2L <= max_tail.
 * May be called again to reset the buffer.  Contexts with lookup_keys also take the lookup keys of
 * the recent tokens (they are needed when those tokens are clustered); sinks never are.
 *
 * mp_decode_step is one decoding step of a generation loop:
 *   1. the new token's key and value (device bf16 [B, Hkv, 1, 128]; k_new_lookup likewise for
 *      contexts with lookup_keys, else NULL) join the buffer;
 *   2. mp_decode_attention (q, q_lookup) with the buffer (sinks, then the recent tokens including
 *      the new one) as the tail;
 *   3. when the buffer holds 2L recent tokens, mp_update_clusters with the oldest L of them
 *      (n_new_fine, n_new_coarse, refine_iters, split_iters, seed, seeds as for that call; `seeds`
 *      is read only in such a step), and the newer L move to the front.
 * Whether a step will refresh is known beforehand: n_recent + 1 == 2L (mp_local_buffer_size).
 * Errors: those of the two calls it is made of; MP_ESTATE without an index or a local buffer.  If
 * the update of step 3 fails (e.g. MP_ECAPACITY), `out` is valid, the error is returned, and the
 * next call retries the update before anything else.
 * ------------------------------------------------------------------------------------------- */
mp_status mp_local_buffer_init(mp_ctx* ctx, int32_t window, const void* k_sink, const void* v_sink, int32_t n_sink,
                               const void* k_recent, const void* k_recent_lookup, const void* v_recent,
                               int32_t n_recent, void* stream);
mp_status mp_local_buffer_size(const mp_ctx* ctx, int32_t* window, int32_t* n_sink, int32_t* n_recent);
mp_status mp_decode_step(mp_ctx* ctx, const void* q, const void* q_lookup, const void* k_new, const void* k_new_lookup,
                         const void* v_new, int32_t key_budget, int32_t coarse_budget, uint32_t flags, int32_t n_new_fine,
                         int32_t n_new_coarse, int32_t refine_iters, int32_t split_iters, uint64_t seed,
                         const int32_t* seeds, void* out, float* lse, void* stream);

/* ---------------------------------------------------------------------------------------------
 * Stage timing (for benchmarks).  While enabled, mp_decode_attention records HIP events on the
 * call's own stream before and after each of its launches.  mp_get_stage_timing waits for the last
 * timed call and writes its four durations in milliseconds:
 * ms[0] = 0 (reserved), ms[1] scoring + selection (both levels, one launch),
 * ms[2] value pass (the kernel that streams the selected keys / values and the centroid terms),
 * ms[3] merge.  Errors: MP_ESTATE if no timed call has been made.
 * ------------------------------------------------------------------------------------------- */
mp_status mp_enable_stage_timing(mp_ctx* ctx, int32_t enable);
mp_status mp_get_stage_timing(mp_ctx* ctx, float* ms);

/* ---------------------------------------------------------------------------------------------
 * Introspection (for parity tests and accounting).  Outputs are device buffers of the stated
 * shape; NULL outputs are skipped.  Work is enqueued on `stream`.
 * ------------------------------------------------------------------------------------------- */

/* Sizes of the current index (host values, no GPU work). */
mp_status mp_get_sizes(const mp_ctx* ctx, int32_t* n_tokens, int32_t* n_fine, int32_t* n_coarse,
                       int32_t* n_blocks);

/* fine_of_token int32 [U, n_tokens] in sequence order; coarse_of_fine int32 [U, n_fine]. */
mp_status mp_get_assignments(mp_ctx* ctx, int32_t* fine_of_token, int32_t* coarse_of_fine, void* stream);

/* level 0 = fine, 1 = coarse.  kc, vc: bf16 [U, n, 128]; n_members: int32 [U, n]. */
mp_status mp_get_centroids(mp_ctx* ctx, int32_t level, void* kc, void* vc, int32_t* n_members, void* stream);

/* Selection of the last decode call: fine_selected uint8 [U, n_fine], coarse_promising uint8
 * [U, n_coarse]; rank keys of the last call (fp64, NaN where a cluster took no part):
 * r_fine [U, n_fine], r_coarse [U, n_coarse]. */
mp_status mp_get_selection(mp_ctx* ctx, uint8_t* fine_selected, uint8_t* coarse_promising,
                           double* r_fine, double* r_coarse, void* stream);

/* Per-unit counters of the last decode call, int32 [U, 4]:
 * {keys attended exactly (selected + tail), fine centroids scored, coarse centroids scored,
 *  centroid terms entering the softmax}. */
mp_status mp_get_counters(mp_ctx* ctx, int32_t* counters, void* stream);

/* Cluster-contiguous cache as stored: k_perm, v_perm bf16 [U, n_tokens, 128]; perm int32
 * [U, n_tokens] (sequence index of each stored row); fine_start int32 [U, n_fine+1] (first stored
 * row of each fine cluster).  A context with MP_KV_E4M3 holds no bf16 rows: k_perm and v_perm must
 * be NULL there (MP_EINVAL), see mp_get_kv_codes. */
mp_status mp_get_layout(mp_ctx* ctx, void* k_perm, void* v_perm, int32_t* perm, int32_t* fine_start,
                        void* stream);

/* The 8-bit cache of a context with MP_KV_E4M3, in stored order (MP_EINVAL for any other context):
 * k_codes (key residuals, see MP_KV_E4M3), v_codes uint8 [U, n_tokens, 128]; scales fp32
 * [U, n_tokens, 2] = {key scale, value scale} of each stored row.  Device pointers, each may be NULL. */
mp_status mp_get_kv_codes(mp_ctx* ctx, void* k_codes, void* v_codes, float* scales, void* stream);

/* ---------------------------------------------------------------------------------------------
 * Dense bf16 decode attention over all n keys (the comparison point: split-KV streaming pass and
 * an online-softmax merge, Sec. 4 / FlashDecoding), using the same inner loop as the exact pass
 * of mp_decode_attention.
 *
 *   q bf16 [B, Hq, 128]; k, v bf16 [B, Hkv, n, 128]; out bf16 [B, Hq, 128]; lse fp32 [B, Hq] or NULL
 *   workspace   device buffer of at least mp_dense_workspace_bytes(B, Hq, Hkv, n) bytes
 * Context-free; errors are reported through mp_last_error(NULL).
 * ------------------------------------------------------------------------------------------- */
size_t mp_dense_workspace_bytes(int32_t batch, int32_t n_q_heads, int32_t n_kv_heads, int32_t n);
mp_status mp_dense_attention(const void* q, const void* k, const void* v, int32_t batch,
                             int32_t n_q_heads, int32_t n_kv_heads, int32_t n, float softmax_scale,
                             void* out, float* lse, void* workspace, size_t workspace_bytes, void* stream);

/* ---------------------------------------------------------------------------------------------
 * mp_dense_attention_static -- mp_dense_attention for callers that cannot allocate: code under
 * HIP graph capture, serving loops with a fixed memory plan, harnesses that forbid hipMalloc.
 * Same arguments, same kernels and bit-identical results, but no workspace argument: the
 * partial results go to an array of MP_DENSE_STATIC_SCRATCH_BYTES bytes built into the library
 * (every GPU the library runs on holds its own copy until the process ends).  The call allocates
 * nothing and frees nothing.
 *
 * Limits: shapes with mp_dense_workspace_bytes(B, Hq, Hkv, n) > mp_dense_static_scratch_bytes()
 * are rejected with MP_ECAPACITY (nothing enqueued).  All calls on one GPU share that GPU's array:
 * calls that may overlap on the GPU (different streams without ordering, or another host thread)
 * race on it -- order them on one stream.  The array keeps the last call's contents; nothing in
 * it has to start at zero (every partial is written before it is read).
 * Other errors: as mp_dense_attention; MP_EHIP if the array's address cannot be resolved (done
 * once per device: by mp_create, else by the first call of this function on that device).
 * ------------------------------------------------------------------------------------------- */
#define MP_DENSE_STATIC_SCRATCH_BYTES (8u << 20)
size_t mp_dense_static_scratch_bytes(void);
mp_status mp_dense_attention_static(const void* q, const void* k, const void* v, int32_t batch,
                                    int32_t n_q_heads, int32_t n_kv_heads, int32_t n, float softmax_scale,
                                    void* out, float* lse, void* stream);

/* Library version string. */
const char* mp_version(void);

#ifdef __cplusplus
}
#endif
#endif /* MP_H_ */
