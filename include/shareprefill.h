/*
 * libshareprefill -- SharePrefill long-context prefill attention for one layer,
 * hand-written for AMD MI355X (gfx950).  C ABI: plain pointers and sizes only.
 *
 * The method (Sec. 5.2): inside every cluster of similar attention heads one
 * pivotal head runs dense causal attention; its exact attention is reduced to a
 * per-(query-block, key-block) score map; the map becomes a block mask (per
 * query-block row, the smallest set of key blocks whose cumulative score reaches
 * gamma -- Alg. 2 -- plus the sink block and the diagonal block); every other
 * head of the cluster then runs block-sparse attention A(Q,K,V,M) (Sec. 5.1)
 * over only those blocks (Alg. 4: pattern sharing).
 *
 * Conventions for every call
 *   - "device" pointers are HIP device memory owned by the caller; "host"
 *     pointers are ordinary host memory read synchronously during the call.
 *   - The library never allocates or frees device memory; scratch space comes in
 *     through `workspace` (size from sp_workspace_bytes, 256-byte aligned).
 *   - Work is enqueued on `hip_stream` (a hipStream_t passed as void*, NULL = the
 *     default stream) and the call returns without waiting for it.
 *   - Arguments are validated first; on any error nothing is launched, the
 *     status says why and sp_last_error() (thread-local) has the detail.
 *   - Results are deterministic: no floating-point atomics anywhere.
 *   - Q, K, V, O are bfloat16.  Element strides (not bytes) are given per batch,
 *     token and head; head_dim is contiguous; every row start must be 16-byte
 *     aligned (strides multiples of 8 elements).
 *   - Supported envelope: head_dim in {64,128}, block in {64,128},
 *     seq % block == 0, seq / block <= 32768 (an index limit: the workspace of a call that
 *     produces block-mass score maps grows as 2 * seq * (seq / block + 1) bytes per scored head,
 *     2.1 GB per head at seq 131072 / block 128, so memory binds long before it),
 *     n_q_heads % n_kv_heads == 0.  Query head h reads KV head h / (n_q_heads / n_kv_heads).
 */
#ifndef SHAREPREFILL_H
#define SHAREPREFILL_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  SP_OK = 0,
  SP_ERR_INVALID_ARG = 1, /* null pointer, bad size / stride / id, gamma out of (0,1] */
  SP_ERR_UNSUPPORTED = 2, /* outside the supported envelope above */
  SP_ERR_WORKSPACE = 3,   /* workspace missing, misaligned or too small */
  SP_ERR_HIP = 4          /* a HIP call or kernel launch failed */
} sp_status;

/* Geometry of one attention layer.  Strides are in elements. */
typedef struct {
  int32_t batch, seq, n_q_heads, n_kv_heads, head_dim, block;
  int64_t q_stride_b, q_stride_t, q_stride_h;
  int64_t kv_stride_b, kv_stride_t, kv_stride_h; /* shared by K and V */
  int64_t o_stride_b, o_stride_t, o_stride_h;
  float softmax_scale; /* 0 => 1/sqrt(head_dim) */
} sp_shape;

const char *sp_status_string(sp_status s);
const char *sp_last_error(void);

/*
 * Optional per-kernel timing for benchmarks (no counterpart in the paper; its protocol,
 * App. A.2 "Latency Benchmark", times whole runs).  While enabled, every kernel the calls
 * below launch is bracketed by two HIP events on the caller's stream.  After the caller has
 * synchronised that stream, sp_profile_read sums elapsed milliseconds and launch counts per
 * kernel kind into host arrays ms[6] / launches[6]: 0 = K/V packing, 1 = dense attention
 * (+ block-mass scores), 2 = mask builder, 3 = block-sparse attention, 4 = block-mean-logit
 * scores and the Alg. 3 gate, 5 = vertical-slash search; `reset` != 0 drops the records.
 * sp_profile_enable(1) creates a fixed pool of events (4096 launches between two reads; more are
 * reported as SP_ERR_UNSUPPORTED by the next read) and clears the records; nothing is created or
 * freed while launches are enqueued.  Process-wide; do not enable it under HIP graph capture.
 */
sp_status sp_profile_enable(int32_t on);
sp_status sp_profile_read(float *ms, int32_t *launches, int32_t reset);

/*
 * Bytes of device workspace that suffice for any of the attention calls below
 * (sp_dense_attn_with_block_scores, sp_block_sparse_attn, sp_block_sparse_attn_gated,
 * sp_prefill_layer, sp_prefill_layer_modes and sp_prefill_layer_gated in every mode)
 * for this shape when at most `n_dense_heads`
 * heads per batch entry produce a block score map in one call (0 if no scores are
 * ever requested).
 */
sp_status sp_workspace_bytes(const sp_shape *shape, int32_t n_dense_heads, size_t *bytes);

/* Workspace of sp_block_mean_logit_scores and of sp_determine_pattern for n_heads listed heads. */
sp_status sp_score_workspace_bytes(const sp_shape *shape, int32_t n_heads, size_t *bytes);

/* Workspace of sp_build_block_mask_global for n_maps maps of nqb x nqb blocks. */
sp_status sp_mask_workspace_bytes(int32_t n_maps, int32_t nqb, size_t *bytes);

/*
 * Dense causal attention A(Q,K,V) (Sec. 5.1) for the listed query heads, and the
 * block score map that Alg. 1 line 8 returns next to O, in the block-mass form:
 *   S[i][j] = (1/block) * sum_{t in query block i} sum_{s in key block j, s<=t} P[t][s]
 * (0 for j > i; every row sums to 1), P being the causal softmax of QK^T*scale.
 *   q,k,v        device bf16
 *   head_ids     host  [n_heads]  distinct query-head ids
 *   o            device bf16; only the listed heads' rows are written
 *   block_scores device fp32 [batch][n_heads][nqb][nkb] or NULL (no scores)
 */
sp_status sp_dense_attn_with_block_scores(const sp_shape *shape, const void *q, const void *k, const void *v,
                                          const int32_t *head_ids, int32_t n_heads, void *o,
                                          float *block_scores, void *workspace, size_t workspace_bytes,
                                          void *hip_stream);

/*
 * Alg. 2 (Construct Pivotal Pattern) applied to every query-block row of every map,
 * in exact integer arithmetic: u_j = rint(clamp(S[i][j],0,1) * 2^24) (NaN -> 0) for
 * j <= i; order by (u descending, j ascending); k* = the least k >= 1 whose prefix sum
 * times 2^24 reaches rint(gamma * 2^24) * sum_j u_j (k* = 0 when every u_j is 0);
 * the row's key-block set is that prefix plus block 0 (sink) and block i (diagonal).
 *   block_scores device fp32 [n_maps][nqb][nkb]   (nqb == nkb required)
 *   kb_idx       device int32 [n_maps][nqb][nkb]  ascending key blocks, tail = -1
 *   kb_cnt       device int32 [n_maps][nqb]
 *   bitmask      device uint64 [n_maps][nqb][ceil(nkb/64)] or NULL (bit j of word j/64)
 */
sp_status sp_build_block_mask(const float *block_scores, int32_t n_maps, int32_t nqb, int32_t nkb, float gamma,
                              int32_t *kb_idx, int32_t *kb_cnt, uint64_t *bitmask, void *hip_stream);

/*
 * Block-sparse causal attention A(Q,K,V,M) (Sec. 5.1) for the listed heads: query
 * block i of listed head n attends only to the key blocks
 * kb_idx[b][head_map[n]][i][0 .. kb_cnt[b][head_map[n]][i]) (ascending, each <= i;
 * blocks with M = 0 get weight exactly 0 and the softmax is renormalised).
 *   head_ids host [n_heads] distinct query heads; head_map host [n_heads] in [0,n_maps)
 *   kb_idx   device int32 [batch][n_maps][nqb][nkb]; kb_cnt device int32 [batch][n_maps][nqb]
 *   o        device bf16; only the listed heads' rows are written
 * Lists must be ascending, without repeats, every entry in [0, i]; the kernel clamps
 * entries into [0, i] (so the call stays memory-safe whatever the buffer holds, but
 * the output of a row whose list breaks the rule is unspecified).  A query block
 * whose count is 0 gets zeros.  The packed K/V copy lives in `workspace`.
 */
sp_status sp_block_sparse_attn(const sp_shape *shape, const void *q, const void *k, const void *v,
                               const int32_t *head_ids, const int32_t *head_map, int32_t n_heads,
                               const int32_t *kb_idx, const int32_t *kb_cnt, int32_t n_maps, void *o,
                               void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * The block score map as the paper prints it (Sec. 5.2, "Sparse Attention Computation"
 * and the first step of Alg. 2) for the listed heads: Abar[i][j] = the average of the
 * scaled logits q_t.k_s*scale over the entries of block (i,j) that exist under
 * causality (all block*block of them for j < i, the block(block+1)/2 with s <= t on
 * the diagonal, -inf for j > i), then a softmax over each row i.  Every row of the
 * result sums to 1; entries with j > i are 0.  No attention output is produced: the
 * averages are linear in Q and K and are formed from per-block sums.
 *   q, k         device bf16 (shape's strides; V is not read)
 *   head_ids     host [n_heads] distinct query-head ids
 *   block_scores device fp32 [batch][n_heads][nqb][nkb]   (output)
 *   workspace    sp_score_workspace_bytes(shape, n_heads)
 * Row nqb-1 of a head's map is the representative vector a~ that Alg. 2 stores.
 */
sp_status sp_block_mean_logit_scores(const sp_shape *shape, const void *q, const void *k, const int32_t *head_ids,
                                     int32_t n_heads, float *block_scores, void *workspace, size_t workspace_bytes,
                                     void *hip_stream);

/*
 * Alg. 2 (Construct Pivotal Pattern) as printed, one selection per map: the causal
 * entries (j <= i) of a map are quantised as in sp_build_block_mask, normalised by the
 * map's total, flattened row-major and ordered by (u descending, flat index ascending);
 * K = the least k >= 1 whose prefix sum times 2^24 reaches rint(gamma * 2^24) * total
 * (K = 0 for an all-zero map); entry (i, j) of that prefix puts key block j into row i's
 * list.  `forced` != 0 additionally gives every row its sink block 0 and diagonal block i
 * (not in the paper; without it a row's list may be empty and that query block then
 * attends to nothing).
 *   block_scores device fp32 [n_maps][nqb][nkb]  (nqb == nkb required; n_maps <= 65535)
 *   kb_idx       device int32 [n_maps][nqb][nkb] ascending key blocks, tail = -1
 *   kb_cnt       device int32 [n_maps][nqb]
 *   workspace    sp_mask_workspace_bytes(n_maps, nqb); contents are scratch
 */
sp_status sp_build_block_mask_global(const float *block_scores, int32_t n_maps, int32_t nqb, int32_t nkb, float gamma,
                                     int32_t forced, int32_t *kb_idx, int32_t *kb_cnt, void *workspace,
                                     size_t workspace_bytes, void *hip_stream);

/*
 * sp_build_block_mask_global for callers that cannot allocate or hand over device memory for scratch
 * (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): same arguments,
 * outputs, errors and results, bit for bit, but no workspace.  The selection's scratch (histograms, tie
 * counts) lives in a static device array inside the library, SP_STATIC_SCRATCH_BYTES per GPU, held until
 * the process ends; the call allocates and frees nothing and clears what it needs with a kernel.
 * Limit: n_maps * (65664 + 8 * nqb rounded up to 256) bytes must fit (e.g. 28 maps at nqb = 1024, 31 at
 * nqb = 256); larger requests return SP_ERR_UNSUPPORTED and launch nothing.
 * All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (different streams or
 * threads) race; calls on one stream, or ordered by events, are safe.
 */
#define SP_STATIC_SCRATCH_BYTES ((size_t)2 << 20)
sp_status sp_build_block_mask_global_static(const float *block_scores, int32_t n_maps, int32_t nqb, int32_t nkb,
                                            float gamma, int32_t forced, int32_t *kb_idx, int32_t *kb_cnt,
                                            void *hip_stream);

/*
 * Alg. 3 (Determine Sparse Pattern) for the listed heads.  For each listed head n:
 *   a_hat[n]  = softmax over key blocks of the pooled, scaled logits of the last `block`
 *               queries against every key block (causal inside the last block), i.e. row
 *               nqb-1 of the map sp_block_mean_logit_scores gives;
 *   d_sparse  = sqrt(JSD(a_hat[n] || uniform over the nkb key blocks)),
 *   d_sim     = sqrt(JSD(a_hat[n] || a_hat[ref_pos[n]])), 0 when ref_pos[n] < 0 (no pivotal
 *               representative exists yet); JSD with the natural logarithm, summed in fp64;
 *   the head shares its pivot's pattern iff d_sparse < delta and d_sim < tau (both strict).
 *   head_ids     host [n_heads] distinct query heads
 *   ref_pos      host [n_heads] position in head_ids of the head whose estimate serves as the
 *                pivotal representative a~ (the cluster's pivot; a head may name itself), or -1
 *   shared_map   host [n_heads] value stored for a head that passes (its cluster's list index)
 *   a_hat        device fp32 [batch][n_heads][nkb]        (output)
 *   dist         device fp32 [batch][n_heads][2]          (output: d_sparse, d_sim)
 *   head_pattern device int32 [batch][n_q_heads]          (output, indexed by query-head id; only
 *                the listed heads' entries are written: shared_map[n] if the head passes, else -1)
 *   workspace    sp_score_workspace_bytes(shape, n_heads)
 * The paper sends failing heads to the vertical-slash search (Alg. 5); in this library a head
 * whose entry is negative runs dense attention.
 */
sp_status sp_determine_pattern(const sp_shape *shape, const void *q, const void *k, const int32_t *head_ids,
                               int32_t n_heads, const int32_t *ref_pos, const int32_t *shared_map, float delta,
                               float tau, float *a_hat, float *dist, int32_t *head_pattern, void *workspace,
                               size_t workspace_bytes, void *hip_stream);

/*
 * sp_block_sparse_attn with the list of each head chosen on the device: listed head h of batch
 * entry b uses list head_pattern[b][h] (clamped to n_maps-1), or, if that entry is negative,
 * attends to every key block 0..i (dense causal attention).  head_pattern is the array
 * sp_determine_pattern writes, read by the kernel when it runs: no host round trip.
 *   head_pattern device int32 [batch][n_q_heads]
 */
sp_status sp_block_sparse_attn_gated(const sp_shape *shape, const void *q, const void *k, const void *v,
                                     const int32_t *head_ids, int32_t n_heads, const int32_t *kb_idx,
                                     const int32_t *kb_cnt, int32_t n_maps, const int32_t *head_pattern, void *o,
                                     void *workspace, size_t workspace_bytes, void *hip_stream);

/* How the pivot's block score map is formed / how Alg. 2 turns it into a pattern. */
enum { SP_SCORE_BLOCK_MASS = 0,   /* exact attention mass per block (sp_dense_attn_with_block_scores) */
       SP_SCORE_MEAN_LOGIT = 1 }; /* row softmax of block-mean logits (sp_block_mean_logit_scores) */
enum { SP_SELECT_PER_ROW = 0,     /* sp_build_block_mask */
       SP_SELECT_GLOBAL = 1 };    /* sp_build_block_mask_global with forced = 1 */

/*
 * One layer of pattern sharing (Alg. 1 with the pattern source of Alg. 4 and the
 * pattern construction of Alg. 2): pivot heads run dense attention with block
 * scores, each cluster's score map becomes its key-block lists, and every other
 * clustered head runs block-sparse attention over its cluster's lists.
 *   head_to_cluster host [n_q_heads]  cluster id in [0,n_clusters) or -1 (runs dense)
 *   pivot_heads     host [n_clusters] pivot_heads[c] must lie in cluster c
 *   o               device bf16, every head written
 *   block_scores    device fp32 [batch][n_clusters][nqb][nkb] (output), or NULL: the maps then
 *                   live in the workspace only and are not returned
 *   kb_idx, kb_cnt  device int32 [batch][n_clusters][nqb][nkb] / [..][nqb] (required, output)
 *   workspace       sized by sp_workspace_bytes(shape, n_clusters)
 */
sp_status sp_prefill_layer(const sp_shape *shape, const void *q, const void *k, const void *v,
                           const int32_t *head_to_cluster, const int32_t *pivot_heads, int32_t n_clusters,
                           float gamma, void *o, float *block_scores, int32_t *kb_idx, int32_t *kb_cnt,
                           void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * sp_prefill_layer with the pattern construction selectable: score_mode / select_mode =
 * (SP_SCORE_MEAN_LOGIT, SP_SELECT_GLOBAL) is Alg. 2 as the paper prints it (Sec. 5.2),
 * (SP_SCORE_BLOCK_MASS, SP_SELECT_PER_ROW) is sp_prefill_layer; the other two mix them.
 * All other arguments, outputs and errors as for sp_prefill_layer.
 */
sp_status sp_prefill_layer_modes(const sp_shape *shape, const void *q, const void *k, const void *v,
                                 const int32_t *head_to_cluster, const int32_t *pivot_heads, int32_t n_clusters,
                                 float gamma, int32_t score_mode, int32_t select_mode, void *o, float *block_scores,
                                 int32_t *kb_idx, int32_t *kb_cnt, void *workspace, size_t workspace_bytes,
                                 void *hip_stream);

/*
 * sp_prefill_layer_modes preceded by Alg. 3's gate (Alg. 1 with Alg. 3, Alg. 4 and Alg. 2):
 * every head's estimate a_hat is formed, the pivot's own serving as its cluster's representative
 * a~; a clustered non-pivot head shares its cluster's pattern iff d_sparse < delta and
 * d_sim < tau, and otherwise runs dense (the stand-in for the vertical-slash fallback).  Pivots
 * and heads outside every cluster run dense whatever their distances are.
 *   a_hat        device fp32 [batch][n_q_heads][nkb]   (output)
 *   dist         device fp32 [batch][n_q_heads][2]     (output)
 *   head_pattern device int32 [batch][n_q_heads]       (output: cluster id if shared, else -1)
 * One stream, no host synchronisation: the sparse kernel reads head_pattern on the device.
 */
sp_status sp_prefill_layer_gated(const sp_shape *shape, const void *q, const void *k, const void *v,
                                 const int32_t *head_to_cluster, const int32_t *pivot_heads, int32_t n_clusters,
                                 float gamma, float delta, float tau, int32_t score_mode, int32_t select_mode, void *o,
                                 float *block_scores, int32_t *kb_idx, int32_t *kb_cnt, float *a_hat, float *dist,
                                 int32_t *head_pattern, void *workspace, size_t workspace_bytes, void *hip_stream);

/* What a head does when Alg. 3 sends it to the fallback pattern. */
enum { SP_FALLBACK_DENSE = 0,                  /* dense causal attention (exact) */
       SP_FALLBACK_VERTICAL_SLASH = 1,         /* the pattern of Alg. 5 widened to whole key blocks
                                                  (sp_search_vertical_slash + block-sparse attention) */
       SP_FALLBACK_VERTICAL_SLASH_TOKEN = 2 }; /* the pattern of Alg. 5 token by token (sp_vertical_slash_attn) */

/* Workspace of sp_search_vertical_slash for n_heads listed heads (block * seq * 4 bytes per head and more). */
sp_status sp_vs_workspace_bytes(const sp_shape *shape, int32_t n_heads, size_t *bytes);

/*
 * Alg. 5 (Search Vertical Slash Pattern) for the listed heads, with Q_hat = the last `block`
 * queries: A_hat = causal softmax of their scaled logits against every key;
 *   a_v[s] = sum_t A_hat[t][s] / sum(A_hat),  a_s[o] = sum_t A_hat[t][t-o] / sum(A_hat);
 * each vector is quantised to 24 bits as in sp_build_block_mask, ordered by (value descending,
 * index ascending) and cut at the shortest prefix whose sum reaches gamma of its total; a token
 * pair (t, s), s <= t, belongs to the pattern iff key s or offset t-s is kept.  The result is
 * returned at block granularity: key block j is listed for query block i iff the block holds at
 * least one pair of the pattern (attention over the lists covers a superset of the token
 * pattern); `forced` != 0 adds the sink block 0 and the diagonal block i to every row.
 *   head_ids host [n_heads] distinct query heads
 *   sums     device fp32 [batch][n_heads][2][seq] or NULL  (output: a_v then a_s)
 *   kb_idx   device int32 [batch][n_heads][nqb][nkb]       (output, ascending, tail -1)
 *   kb_cnt   device int32 [batch][n_heads][nqb]            (output)
 *   workspace sp_vs_workspace_bytes(shape, n_heads)
 * Feed the lists to sp_block_sparse_attn with head_map[n] = n and n_maps = n_heads.
 */
sp_status sp_search_vertical_slash(const sp_shape *shape, const void *q, const void *k, const int32_t *head_ids,
                                   int32_t n_heads, float gamma, int32_t forced, float *sums, int32_t *kb_idx,
                                   int32_t *kb_cnt, void *workspace, size_t workspace_bytes, void *hip_stream);

/* Workspace of sp_vertical_slash_attn for n_heads listed heads (the search's, the packed K/V copy and one more
 * packed copy of K and V per listed head for its gathered keys). */
sp_status sp_vs_token_workspace_bytes(const sp_shape *shape, int32_t n_heads, size_t *bytes);

/*
 * Alg. 5 (Search Vertical Slash Pattern) for the listed heads, as sp_search_vertical_slash forms it (Q_hat = the
 * last `block` queries, the two vector selections at `gamma`), followed by attention A(Q,K,V,M) (Sec. 5.1) over
 * the mask M the algorithm builds from S = S_v U S_s, token by token: query t attends to key s <= t iff key s is
 * kept (a vertical line) or offset t - s is kept (a slash line) or -- forced != 0 -- s lies in the first block or
 * in t's own block (the sink and diagonal blocks every pattern of this library carries).  Pairs outside M get
 * weight exactly 0, the softmax is renormalised, a query without any allowed key gets zeros.
 * The kept keys are gathered into packed images of their own (64 keys each), the kept offsets are walked as bands
 * of key blocks with a bit mask inside every tile; no whole block is attended to because of one kept key.
 *   head_ids  host [n_heads] distinct query heads
 *   o         device bf16; only the listed heads' rows are written
 *   keep_bits device uint64 [batch][n_heads][2][seq/64] or NULL  (output: bit s of the first vector = key s kept,
 *             bit o of the second = offset o kept)
 *   pairs     device int64 [batch][n_heads] or NULL  (output: number of (query, key) pairs in M)
 *   workspace sp_vs_token_workspace_bytes(shape, n_heads)
 */
sp_status sp_vertical_slash_attn(const sp_shape *shape, const void *q, const void *k, const void *v,
                                 const int32_t *head_ids, int32_t n_heads, float gamma, int32_t forced, void *o,
                                 uint64_t *keep_bits, int64_t *pairs, void *workspace, size_t workspace_bytes,
                                 void *hip_stream);

/*
 * The dynamic pivotal pattern dictionary (Sec. 5.2, "Dynamic Pattern Construction and Sharing
 * during Inference"): for every cluster of the offline head dictionary, the pattern its first
 * qualifying head produced and that head's representative a~.  All arrays are caller-owned
 * device memory that lives across the layers of one prefill; `valid` must be zeroed before
 * the first layer.  Cluster ids are global: the same id in two layers means the same cluster.
 */
typedef struct {
  int32_t n_clusters;
  int32_t *valid;   /* device int32 [batch][n_clusters]            1 once the cluster has an entry */
  float *a_tilde;   /* device fp32  [batch][n_clusters][nkb]       representative (Alg. 2, "last row") */
  int32_t *kb_idx;  /* device int32 [batch][n_clusters][nqb][nkb]  key-block lists, ascending, tail -1 */
  int32_t *kb_cnt;  /* device int32 [batch][n_clusters][nqb] */
} sp_pattern_dict;

/*
 * One layer of Alg. 1 with the dictionary carried across layers (Alg. 3 decides, Alg. 4 shares,
 * Alg. 2 constructs).  Heads are taken in ascending index order.  For a head of cluster c:
 *   - c has an entry: the head shares the entry's pattern iff d_sparse < delta and
 *     d_sim(a_hat, entry's a~) < tau (role c), else it falls back (role -1);
 *   - c has no entry: the first head of c in this layer with d_sparse < delta (and 0 < tau: with
 *     no representative d_sim counts as 0) is elected pivot (role -2): it runs dense attention,
 *     its score map becomes the entry's pattern (Alg. 2 per score_mode / select_mode as in
 *     sp_prefill_layer_modes) and its estimate the entry's a~; the heads after it are tested
 *     against that estimate; heads before it, and all heads if none qualifies, fall back.
 *   Heads with cluster -1 and fallback heads (role -1) never touch the dictionary; with
 *   fallback_mode SP_FALLBACK_DENSE they run dense attention, with SP_FALLBACK_VERTICAL_SLASH
 *   each gets its own pattern from Alg. 5 (sp_search_vertical_slash with the layer's gamma, forced
 *   blocks on) and runs block-sparse over it, with SP_FALLBACK_VERTICAL_SLASH_TOKEN each runs
 *   sp_vertical_slash_attn's token-level attention over that pattern (vs_idx / vs_cnt unused).
 *   Everything is decided on the device: one stream, no
 *   host synchronisation; the roles can be read back afterwards.
 *   head_to_cluster host [n_q_heads] global cluster id in [0, dict->n_clusters) or -1
 *   block_scores    device fp32 [batch][n_slots][nqb][nkb], n_slots = number of distinct clusters
 *                   in head_to_cluster (ascending cluster id); slot s is written only if its
 *                   cluster elected a pivot in this call
 *   role            device int32 [batch][n_q_heads]      (output)
 *   a_hat, dist     device fp32 [batch][n_q_heads][nkb] / [batch][n_q_heads][2]   (outputs, Alg. 3; d_sim is 0
 *                   where no representative existed when the head was met: pivots, heads before their
 *                   cluster's new pivot, heads without a cluster -- these still get a_hat and d_sparse)
 *   vs_idx, vs_cnt  device int32 [batch][n_q_heads][nqb][nkb] / [batch][n_q_heads][nqb]: the lists of
 *                   the heads that took the vertical-slash fallback (other heads' entries are left
 *                   untouched); may be NULL with SP_FALLBACK_DENSE
 *   workspace       sp_workspace_bytes(shape, n_slots), plus sp_vs_workspace_bytes(shape, n_q_heads)
 *                   with SP_FALLBACK_VERTICAL_SLASH, or sp_vs_token_workspace_bytes(shape, n_q_heads)
 *                   with SP_FALLBACK_VERTICAL_SLASH_TOKEN
 */
sp_status sp_prefill_layer_dict(const sp_shape *shape, const void *q, const void *k, const void *v,
                                const int32_t *head_to_cluster, float gamma, float delta, float tau,
                                int32_t score_mode, int32_t select_mode, int32_t fallback_mode,
                                const sp_pattern_dict *dict, void *o, float *block_scores, int32_t *role, float *a_hat,
                                float *dist, int32_t *vs_idx, int32_t *vs_cnt, void *workspace, size_t workspace_bytes,
                                void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* SHAREPREFILL_H */
