/*
 * krul.h -- C ABI of the MI355X (gfx950) cross-layer attention-similarity library.
 *
 * The library implements the data-parallel core of Krul's compression-strategy
 * search (arxiv 2507.08045): score how alike the attention patterns of adjacent
 * layers are for a conversation (Sec. 4.2, Sec. 5, Sec. 7) and pick disjoint layer
 * pairs under a budget (Alg. 1 second loop).
 *
 * Conventions for every entry point
 *   - All tensor arguments are DEVICE pointers unless stated; the caller owns every
 *     buffer.  The library allocates no device memory, keeps no state between
 *     calls and is re-entrant (krul_pair_similarity_static alone works in a scratch
 *     area of the library's own; see there).
 *   - Work is only enqueued on the caller's stream (hipStream_t passed as void*,
 *     NULL = the default stream); calls return without synchronising.
 *   - The return value is a krul_status_t.  Nothing throws or aborts across the ABI.
 *   - Tensors are dense, row-major, last index fastest.
 */
#ifndef KRUL_H
#define KRUL_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    KRUL_OK = 0,
    KRUL_EINVAL = -1,       /* null pointer, non-positive extent, bad head grouping, misalignment */
    KRUL_EDTYPE = -2,       /* dtype is not a krul_dtype_t */
    KRUL_EWORKSPACE = -3,   /* workspace missing, misaligned or shorter than the query says */
    KRUL_ELAUNCH = -4,      /* the HIP runtime refused a launch */
    KRUL_EUNSUPPORTED = -5, /* valid request with no kernel (head_dim, n_layers limits) */
    KRUL_ESCRATCH = -6      /* krul_pair_similarity_static: the shape needs more than KRUL_STATIC_SCRATCH_BYTES */
} krul_status_t;

typedef enum { KRUL_F32 = 0, KRUL_BF16 = 1, KRUL_F16 = 2 /* IEEE binary16 */ } krul_dtype_t;

/* flags of krul_shape_t */
enum {
    KRUL_FLAG_CAUSAL = 1 << 0,         /* the n_query rows are the LAST n_query tokens of the n_hist-token
                                          sequence held by k, and row t attends to the keys up to and
                                          including its own position, j <= n_hist - n_query + t (a decode
                                          step, n_query = 1, or a chunk of a prefill; Sec. 5).  Needs
                                          n_hist >= n_query.  Without it every row sees all n_hist keys. */
    /* test aids (see "Measurement and test aids" at the end of this file) */
    KRUL_FLAG_GENERIC_KERNEL = 1 << 8,
    KRUL_FLAG_SINGLE_SPLIT = 1 << 9
};

/*
 * Problem statement.  Alg. 1 takes the model's attention weights for a prompt; here
 * the forward pass is outside the library, so the attention weights are given by
 * their factors: per layer l the queries Q_l and keys K_l, from which
 * softmax(Q_l K_l^T * scale) of Sec. 2.1 is formed on the fly and never stored.
 */
typedef struct {
    int32_t batch;        /* B   independent conversations                         */
    int32_t n_layers;     /* L   transformer layers, >= 2                          */
    int32_t n_q_heads;    /* Hq  query heads                                       */
    int32_t n_kv_heads;   /* Hkv key heads, divides Hq; query head h reads kv head
                                 h / (Hq/Hkv)                                      */
    int32_t head_dim;     /* d   a multiple of 8: up to 128 for the matrix-core
                                 kernels (bf16, f16; sizes other than 64 and 128 ride
                                 zero-padded), up to 256 for the portable one       */
    int32_t n_hist;       /* S   history keys per layer (every query row sees all) */
    int32_t n_query;      /* Tq  query rows (tokens) per head                      */
    int32_t dtype;        /* krul_dtype_t of q and k                               */
    float   scale;        /* logit scale; 0 selects 1/sqrt(head_dim) (Sec. 2.1)    */
    int32_t flags;        /* 0, or KRUL_FLAG_* bits                                */
} krul_shape_t;

/*
 * Bytes of device workspace krul_pair_similarity needs for this
 * shape (a multiple of 256).  Returns 0 if the shape is invalid or unsupported.
 * Host-only: touches no GPU.
 */
size_t krul_pair_similarity_workspace(const krul_shape_t *shape);

/*
 * Token-wise cross-layer attention similarity (Sec. 5 and Sec. 7; distance of
 * Alg. 1 / Sec. 4.2 for adjacent layers).  For every conversation b, adjacent pair
 * l -> (l, l+1), query head h and query row t, with p = softmax(q_l K_l^T * scale)
 * and r = softmax(q_{l+1} K_{l+1}^T * scale) over the S history keys:
 *     cos  = <p, r> / (|p| |r|)            dist = |p - r|   (via p^2 + r^2 - 2pr, Sec. 7)
 * aggregated token-wise: mean over t, then mean over the Hq query heads.
 *
 *   q           [B][L][Hq][Tq][d]   device, 16-byte aligned, dtype as in shape
 *   k           [B][L][Hkv][S][d]   device, 16-byte aligned
 *   pair_score  [B][L-1] float      device, required: mean cosine per pair
 *   head_score  [B][L-1][Hq] float  device, may be NULL: mean cosine per pair and head
 *   pair_dist   [B][L-1] float      device, may be NULL: mean Euclidean distance per pair
 *   workspace   device, 256-byte aligned, at least krul_pair_similarity_workspace()
 *               bytes; contents are scratch, undefined afterwards
 *
 * Results are deterministic (fixed reduction order).  Non-finite inputs give
 * unspecified results.  Errors: KRUL_EINVAL, KRUL_EDTYPE, KRUL_EUNSUPPORTED,
 * KRUL_EWORKSPACE, KRUL_ELAUNCH; on error nothing has been enqueued unless the
 * code is KRUL_ELAUNCH.
 */
int krul_pair_similarity(const krul_shape_t *shape, const void *q, const void *k,
                         float *pair_score, float *head_score, float *pair_dist,
                         void *workspace, size_t workspace_bytes, void *stream);

/*
 * krul_pair_similarity for callers that cannot provide a workspace because they cannot allocate device
 * memory where they stand: code recorded into a HIP graph, tight serving loops, harnesses that forbid
 * hipMalloc.  Same arguments without the workspace, same results bit for bit.  The scratch memory is a
 * fixed area of KRUL_STATIC_SCRATCH_BYTES that the library's code object holds on every GPU it is loaded
 * on until the process ends; the call allocates nothing and frees nothing.
 *
 *   - Shapes whose krul_pair_similarity_workspace() exceeds KRUL_STATIC_SCRATCH_BYTES are refused with
 *     KRUL_ESCRATCH (nothing enqueued).  40 MiB holds every few-query and decode-step shape of the
 *     Llama-3-8B kind (64 query tokens over 4096 keys: 16 MiB; one token over 131072 keys: 32 MiB); the
 *     many-query shapes need hundreds of MiB and take krul_pair_similarity with a workspace.
 *   - The stream must belong to the CURRENT device.  The first call on a device looks up the area's
 *     address there (no allocation); make that first call outside graph capture.
 *   - All calls on one GPU share the one area: calls that overlap in time on one GPU (two streams, two
 *     threads) race.  Calls on one stream are ordered and safe.  Nothing in the area needs clearing
 *     between calls: every record read is written first by the same call.
 * Errors otherwise as for krul_pair_similarity.
 */
#define KRUL_STATIC_SCRATCH_BYTES (40u << 20)
int krul_pair_similarity_static(const krul_shape_t *shape, const void *q, const void *k,
                                float *pair_score, float *head_score, float *pair_dist, void *stream);

/*
 * krul_pair_similarity together with the Initial-Recent (I-R) layer test that precedes it in
 * Alg. 1 (first loop; Sec. 4.2, "Non-I-R Layer Extraction"), in the same pass over K.  With
 * T_initial = the first 10 % and T_recent = the last 10 % of the history -- keys
 * [0, floor(0.1 S)) and [floor(0.9 S), S) --
 *     ir_mass[b][l]  = mean over query heads and query rows of the softmax mass on T_initial and T_recent
 *     eligible[b][l] = (ir_mass[b][l] >= gamma): a layer whose mass stays below the threshold gamma
 *                      is not an I-R layer and is set aside (its byte is 0)
 * eligible can be handed to krul_select_pairs as is.
 *
 *   (not available together with KRUL_FLAG_CAUSAL: the test is stated for whole-sequence attention)
 *   gamma       threshold, finite and >= 0
 *   ir_mass     [B][L] float   device, may be NULL
 *   eligible    [B][L] uint8   device, may be NULL (not both NULL)
 *   workspace   at least krul_pair_similarity_ir_workspace() bytes (more than the plain call needs)
 * Everything else, and the error behaviour, is as for krul_pair_similarity.
 */
size_t krul_pair_similarity_ir_workspace(const krul_shape_t *shape);
int krul_pair_similarity_ir(const krul_shape_t *shape, const void *q, const void *k, float gamma,
                            float *pair_score, float *head_score, float *pair_dist,
                            float *ir_mass, uint8_t *eligible,
                            void *workspace, size_t workspace_bytes, void *stream);

/*
 * krul_pair_similarity (same scores: Sec. 5 and Sec. 7) on keys that stay where the inference engine
 * caches them (the KV caches of Sec. 2.1, which every layer keeps for its own attention): one
 * allocation per layer and arbitrary strides between conversations, kv heads and keys (e.g. a
 * [B][S][Hkv][d] cache), so the KV cache of a conversation is scored in place, without a gather.  q is dense as for krul_pair_similarity.
 *
 *   k_layers    DEVICE array (8-byte aligned) of n_layers device pointers; k_layers[l] = keys of layer l,
 *               16-byte aligned.  The array is read by the kernel: it must stay valid and unchanged until
 *               the call's work on the stream has finished.
 *   k_stride_b, k_stride_h, k_stride_s
 *               elements between conversations, kv heads and keys inside a layer: key (b, h, j) starts at
 *               k_layers[l] + b*k_stride_b + h*k_stride_h + j*k_stride_s; its head_dim elements are
 *               contiguous.  All > 0 and multiples of 8 elements (k_stride_b is ignored for batch 1),
 *               k_stride_s >= head_dim (else KRUL_EINVAL); for bf16 / f16 with head_dim up to 128,
 *               n_hist * k_stride_s * 2 bytes < 2 GiB and k_stride_s < 2^23 (else KRUL_EUNSUPPORTED).
 * The caller guarantees that every addressed key lies inside its layer's allocation.  Everything else
 * is as for krul_pair_similarity (same workspace size).
 */
typedef struct {
    const void *const *k_layers;
    int64_t k_stride_b, k_stride_h, k_stride_s;
} krul_k_layout_t;
int krul_pair_similarity_strided(const krul_shape_t *shape, const void *q, const krul_k_layout_t *k_layout,
                                 float *pair_score, float *head_score, float *pair_dist,
                                 void *workspace, size_t workspace_bytes, void *stream);

/*
 * krul_pair_similarity on keys kept in a paged cache (the KV caches of Sec. 2.1 as paged-attention
 * engines keep them): every layer owns a pool of fixed-size pages, a conversation's keys are spread over
 * pages named by its row of a block table (the same row for every layer), and are scored where they are.
 *
 *   k_layers     DEVICE array (8-byte aligned) of n_layers device pointers to the layers' pools, 16-byte aligned
 *   block_table  DEVICE int32 [batch][max_blocks]: page of keys [i*block_size, (i+1)*block_size) of conversation b
 *                at block_table[b][i]; entries from ceil(n_hist / block_size) on are not read
 *   block_size   keys per page: a power of two, >= 8
 *   max_blocks   row length of block_table, >= ceil(n_hist / block_size)
 *   k_stride_block, k_stride_h, k_stride_s
 *                elements between pages, kv heads and the keys of a page: key j of conversation b, kv head h starts
 *                at k_layers[l] + block_table[b][j / block_size]*k_stride_block + h*k_stride_h
 *                + (j % block_size)*k_stride_s; head_dim contiguous.  All > 0, multiples of 8, k_stride_s >=
 *                head_dim (else KRUL_EINVAL); for bf16 / f16 with head_dim up to 128, k_stride_s < 2^27 (else
 *                KRUL_EUNSUPPORTED).  E.g. a [num_blocks][block_size][Hkv][d] pool:
 *                (block_size*Hkv*d, d, Hkv*d).
 * Every page has room for block_size keys; the slots past the last key of a conversation may be read (their
 * contents do not matter, NaN included).
 * Tables and pools are read by the kernels: they must stay valid and unchanged until the call's work on the
 * stream has finished; the caller guarantees that every page index lies inside its pool.  Everything else is as
 * for krul_pair_similarity (same workspace size; KRUL_FLAG_CAUSAL is honoured).
 */
typedef struct {
    const void *const *k_layers;
    const int32_t *block_table;
    int32_t block_size, max_blocks;
    int64_t k_stride_block, k_stride_h, k_stride_s;
} krul_k_pages_t;
int krul_pair_similarity_paged(const krul_shape_t *shape, const void *q, const krul_k_pages_t *k_pages,
                               float *pair_score, float *head_score, float *pair_dist,
                               void *workspace, size_t workspace_bytes, void *stream);

/*
 * Token-wise accumulation over several calls (Sec. 5 and Sec. 7: the similarities of the tokens of
 * the prefill and of every decode step are added up).  krul_pair_similarity_accumulate adds, for every
 * (conversation, pair, query head), the SUM over this call's n_query rows of the row cosine to
 * head_sum, and of the row distance to head_dist_sum; the caller zeroes the sums before the first
 * call and counts the tokens.  Typical use: one call per prefill chunk or decode step with
 * KRUL_FLAG_CAUSAL, k holding the sequence so far.  krul_pair_scores_from_sums then turns the sums
 * into the scores krul_pair_similarity would give: head_score = head_sum / n_tokens,
 * pair_score = mean over heads (likewise pair_dist).
 *
 *   head_sum       [B][L-1][Hq] float  device, required, read and written (+=)
 *   head_dist_sum  [B][L-1][Hq] float  device, may be NULL
 *   n_tokens       rows accumulated per head so far (> 0)
 *   pair_score [B][L-1] required; head_score [B][L-1][Hq], pair_dist [B][L-1] may be NULL
 *   (pair_dist needs head_dist_sum)
 * Calls on one stream are ordered; concurrent calls that share sums race.  Errors as for
 * krul_pair_similarity.
 */
int krul_pair_similarity_accumulate(const krul_shape_t *shape, const void *q, const void *k,
                                    float *head_sum, float *head_dist_sum,
                                    void *workspace, size_t workspace_bytes, void *stream);
int krul_pair_scores_from_sums(const float *head_sum, const float *head_dist_sum,
                               int32_t batch, int32_t n_layers, int32_t n_q_heads, float n_tokens,
                               float *pair_score, float *head_score, float *pair_dist, void *stream);

/*
 * The accumulating call and the Initial-Recent call on keys read where a serving engine keeps them -- the
 * token-wise scoring of Sec. 5 as it would run beside decoding: one call per decode step or prefill chunk,
 * on the live cache.  keys names the source: exactly one of its members is set (else KRUL_EINVAL).
 *   dense    as krul_pair_similarity takes them
 *   strided  as for krul_pair_similarity_strided
 *   paged    as for krul_pair_similarity_paged
 * Everything else is as for krul_pair_similarity_accumulate and krul_pair_similarity_ir (same workspace
 * sizes); the Initial-Recent regions are positions of the conversation, wherever its keys lie.
 */
typedef struct {
    const void *dense;
    const krul_k_layout_t *strided;
    const krul_k_pages_t *paged;
} krul_keys_t;
int krul_pair_similarity_accumulate_in_place(const krul_shape_t *shape, const void *q, const krul_keys_t *keys,
                                             float *head_sum, float *head_dist_sum,
                                             void *workspace, size_t workspace_bytes, void *stream);
int krul_pair_similarity_ir_in_place(const krul_shape_t *shape, const void *q, const krul_keys_t *keys, float gamma,
                                     float *pair_score, float *head_score, float *pair_dist,
                                     float *ir_mass, uint8_t *eligible,
                                     void *workspace, size_t workspace_bytes, void *stream);
/* ... and krul_all_pairs_similarity (declared below; same outputs, workspace and limits) on such keys. */
int krul_all_pairs_similarity_in_place(const krul_shape_t *shape, const void *q, const krul_keys_t *keys,
                                       float *pair_score_all, float *pair_dist_all, float *head_score_all,
                                       void *workspace, size_t workspace_bytes, void *stream);

/*
 * Greedy disjoint pair selection (Alg. 1 second loop; Sec. 4.2).  Candidates are
 * the adjacent pairs l -> (l, l+1) whose two layers are both eligible.  They are
 * ordered by pair_score descending (= distance ascending), equal scores by lower l
 * first, and scanned once: a pair is taken iff neither of its layers is already in
 * a taken pair; the scan stops at n_select pairs.  A pair whose score is NaN is no candidate
 * (it is never taken and blocks no neighbour); +-infinity order as numbers.
 *
 *   pair_score [B][n_layers-1] float   device
 *   eligible   [B][n_layers] uint8     device, or NULL = every layer eligible
 *   out_pairs  [B][n_select] int32     device: lower layer index of each taken pair in
 *                                      the order taken, -1 after out_count[b]
 *   out_count  [B] int32               device: pairs taken (fewer than n_select when the
 *                                      candidates run out; that is not an error)
 * Limits: 2 <= n_layers <= 4096, 0 <= n_select <= n_layers/2.
 */
int krul_select_pairs(const float *pair_score, const uint8_t *eligible,
                      int32_t batch, int32_t n_layers, int32_t n_select,
                      int32_t *out_pairs, int32_t *out_count, void *stream);

/*
 * Alg. 1's scoring and greedy choice (Sec. 4.2) in one call: krul_pair_similarity followed by
 * krul_select_pairs on its pair_score, with the same results bit for bit.  Unless a conversation has more
 * than 16384 (pair, head) values, the averages over heads and the selection run in one kernel (a workgroup
 * per conversation), which saves a launch of a few microseconds; otherwise the same kernels run as for the
 * two calls.
 *
 *   eligible, n_select, out_pairs, out_count   as for krul_select_pairs (eligible is an input here: take it
 *                                              from an earlier krul_pair_similarity_ir, or pass NULL)
 *   event_begin, event_end                     caller-created HIP events (hipEvent_t as void*), either may be NULL,
 *                                              recorded on the stream just before and just after the
 *                                              similarity kernel (see krul_pair_similarity_timed)
 *   everything else                            as for krul_pair_similarity
 */
int krul_pair_similarity_select(const krul_shape_t *shape, const void *q, const void *k,
                                const uint8_t *eligible, int32_t n_select,
                                float *pair_score, float *head_score, float *pair_dist,
                                int32_t *out_pairs, int32_t *out_count,
                                void *workspace, size_t workspace_bytes, void *stream,
                                void *event_begin, void *event_end);

/*
 * Similarity of EVERY two layers i > j, as Alg. 1 is printed (its second loop runs over all two-layer
 * combinations of the remaining layers, Sec. 4.2; the layer-by-layer similarity map of Sec. 2.3), not only of
 * neighbours.  Same definitions as
 * krul_pair_similarity: per conversation, query head and query row the cosine and the Euclidean distance
 * between the attention rows that layers i and j give the row; mean over rows (Sec. 5, Sec. 7), then the
 * average over heads (Sec. 4.2).
 *
 *   q, k            as for krul_pair_similarity (dense layouts); KRUL_FLAG_CAUSAL is honoured
 *   pair_score_all  [B][L][L] float   device: mean cosine of layers i and j at [i][j] and [j][i]; 1 on the diagonal
 *   pair_dist_all   [B][L][L] float   device, may be NULL: mean distance, 0 on the diagonal
 *   head_score_all  [B][Hq][L][L] float  device, may be NULL: the cosines before the average over heads
 *   workspace       device, 256-byte aligned.  The attention weights of a batch of query rows are kept
 *                   in it (fp16), as the paper keeps them (Sec. 5), so its size sets how many rows one
 *                   batch holds: krul_all_pairs_workspace(shape, max_bytes) returns the bytes for the
 *                   largest batch that fits max_bytes (max_bytes 0: a default budget of 4 GiB; never
 *                   less than the bytes for the smallest batch, up to 256 rows of one kv head), or 0 if the
 *                   shape is not supported.  Any size from the smallest batch's up is accepted by the
 *                   call; more memory means fewer, larger launches.
 * Limits: n_layers <= 128.  bf16 or f16 with head_dim up to 128 runs on the matrix cores; other inputs take a
 * portable, slow kernel.  Exponentials are rounded to fp16 (2^-11 relative) before the products.
 * Results are deterministic.  Errors as for krul_pair_similarity.
 */
size_t krul_all_pairs_workspace(const krul_shape_t *shape, size_t max_bytes);
int krul_all_pairs_similarity(const krul_shape_t *shape, const void *q, const void *k,
                              float *pair_score_all, float *pair_dist_all, float *head_score_all,
                              void *workspace, size_t workspace_bytes, void *stream);

/*
 * Greedy disjoint pair selection over every two layers (Alg. 1 second loop as printed; Sec. 4.2).
 * Candidates are the pairs (j, i), j < i, of eligible layers, scored by score[b][i][j] (only the
 * entries below the diagonal are read).  closer_is_smaller != 0: the score is a distance, taken in
 * ascending order (Alg. 1's Euclidean distance); 0: a similarity, taken in descending order.  Equal
 * scores: lower j first, then lower i.  A pair is taken iff neither of its layers is in a taken pair;
 * the scan stops at n_select pairs.  A pair whose score is NaN is no candidate.
 *
 *   score      [B][n_layers][n_layers] float   device (e.g. pair_dist_all or pair_score_all)
 *   eligible   [B][n_layers] uint8             device, or NULL = every layer eligible
 *   out_pairs  [B][n_select][2] int32          device: (j, i) of each taken pair in the order taken,
 *                                              (-1, -1) after out_count[b]
 *   out_count  [B] int32                       device
 * Limits: 2 <= n_layers <= 1024, 0 <= n_select <= n_layers/2.
 */
int krul_select_pairs_all(const float *score, int32_t closer_is_smaller, const uint8_t *eligible,
                          int32_t batch, int32_t n_layers, int32_t n_select,
                          int32_t *out_pairs, int32_t *out_count, void *stream);

/*
 * Pairs to select for a compression ratio r_l: Alg. 1 stops once the shared-layer
 * set holds N * r_l layers, two per pair, so ceil(N * r_l / 2), clamped to
 * [0, N/2].  Host-only.
 */
int32_t krul_n_select_from_ratio(int32_t n_layers, float r_l);

/* Static description of a status code.  Host-only. */
const char *krul_strerror(int status);

/* ------------------------------------------------------------------------------------------------
 * Measurement and test aids.  Not part of the method: a benchmark harness and the parity tests use
 * them; a serving stack has no need to.
 * ------------------------------------------------------------------------------------------------
 *
 * KRUL_FLAG_GENERIC_KERNEL (flags of krul_shape_t): use the portable vector-ALU kernel even where the
 *     matrix-core kernel applies (results agree to rounding).
 * KRUL_FLAG_SINGLE_SPLIT: do not split a row's keys over several workgroups (less parallelism; drives
 *     the path that carries running sums from one key tile to the next).
 */

/*
 * krul_pair_similarity with two caller-created HIP events (hipEvent_t passed as void*,
 * either may be NULL) recorded on the stream immediately before and after the
 * similarity kernel -- the kernel that forms the logits and the softmax sums and
 * dominates the run time -- so that a harness can time that one kernel inside its own
 * timed region.  Everything else is as for krul_pair_similarity.
 */
int krul_pair_similarity_timed(const krul_shape_t *shape, const void *q, const void *k,
                               float *pair_score, float *head_score, float *pair_dist,
                               void *workspace, size_t workspace_bytes, void *stream,
                               void *event_begin, void *event_end);

/*
 * Measurement aid: a plain device-to-device copy kernel (src -> dst, both device, 16-byte
 * aligned, bytes a multiple of 16) on the caller's stream.  It reads `bytes` and writes
 * `bytes` of HBM and nothing else, which gives hardware traffic counters a known reference
 * to be scaled by when the similarity kernel's HBM traffic is measured.
 */
int krul_calibration_copy(const void *src, void *dst, size_t bytes, void *stream);

/*
 * Measurement aid: the inner step of the similarity kernels with no memory traffic, on 256 workgroups of 8
 * waves (one per CU, two waves per SIMD).  Per 32-key x 32-row block of logits (head_dim 128) and wave: a chain
 * of 8 MFMAs 32x32x16 bf16 (parts bit 0), the vector work of its 16 logits per lane -- scale-and-shift, exp2,
 * sum of squares, cross term, binary16 copy -- (bit 1), the 8 operand reads from LDS (bit 2); parts is one of
 * 1, 2, 3, 5, 7.  row_blocks (1 or 2): 32-row blocks per block of keys, as in the two forms of the kernel.  Every
 * wave takes 2 * row_blocks * iters blocks.  Timed by the caller (events around the call), it gives the floors
 * "matrix cores alone", "vector units alone", "both from one instruction stream" that the similarity kernels'
 * times are read against.
 *   out   device, 256 * 512 floats, scratch (keeps the work from being optimised away)
 */
int krul_calibration_block(int32_t row_blocks, int32_t parts, int32_t iters, float *out, void *stream);

/*
 * Measurement aid, host-only: which kernel form krul_pair_similarity takes for this shape on dense keys: 0 the
 * portable vector-ALU kernel; 1 to 7 the matrix-core kernel's tile shapes (1 wide 128 rows x 256 keys, 2 mid
 * 64 x 512, 3 slim 32 x 512, 4 slim with a deep ring, 5 / 6 / 7 the short forms of slim / mid / wide); 8 the
 * many-query kernel (256 x 256).  Negative: a krul_status_t.  n_workgroups, n_key_splits: may be NULL.
 */
int krul_pair_similarity_plan(const krul_shape_t *shape, int32_t *n_workgroups, int32_t *n_key_splits);


#ifdef __cplusplus
}
#endif
#endif /* KRUL_H */
