/*
 * sgc.h -- C ABI of libsgc: cluster-shared KV-cache prefill attention for MI355X (gfx950).
 *
 * The library implements the GPU hot path of SubGCache (arXiv 2505.10951):
 *   - Sec. 3.4 "Subgraph-level Cache Reuse": for every query cluster the prompt of its
 *     representative subgraph is run ONCE and the per-layer attention K/V are kept in GPU
 *     memory as a cluster-wise KV cache (sgc_prefix_prefill); every query of the cluster then
 *     appends its own question tokens to that cached prompt (sgc_suffix_prefill_batched); when
 *     the cluster is served the cache is released (sgc_cache_free_cluster).
 *   - Sec. 3.2 "Query Clustering": clustering yields one cluster label per in-batch query;
 *     sgc_assign_clusters turns the labels into the grouping the kernels run on.
 * The paper processes clusters and queries one after another; this library runs all queries of
 * all clusters of a batch in one launch per layer.
 *
 * What is computed (the paper does not write attention down; this is the textbook form):
 *   scaled-dot-product attention, softmax over the visible keys, rotary position embedding in
 *   the rotate-half pairing (channel t pairs with t + head_dim/2, angle = position *
 *   rope_base^(-2t/head_dim)), grouped-query heads (KV head = query head / (n_q_heads /
 *   n_kv_heads)).  Prefix token j sits at position j.  Suffix token i of a query whose cluster
 *   has a prefix of P tokens sits at position P + i and sees all P cached keys plus suffix keys
 *   0..i of its own query; it never sees another query's tokens.
 *
 * Conventions
 *   - Every function returns SGC_OK (0) or a negative sgc_status.  Nothing throws, aborts or
 *     prints.  sgc_last_error() gives a readable message for the last failure on that context.
 *   - "dev" pointers are device (HBM) addresses, 16-byte aligned, owned by the caller (for
 *     example torch tensors); "host" pointers are ordinary host memory.  The library keeps no
 *     reference to q/k/v/o buffers after the call's work has been enqueued on the stream; the
 *     caller must keep them alive until that stream work has finished.
 *   - hip_stream is a hipStream_t passed as void* (NULL = the default stream).  Launches are
 *     asynchronous on it.  Use ONE stream for all the work of a context: the tables the library
 *     keeps on the device (page tables, rotary table, plan arrays, pages handed back by
 *     sgc_cache_free_cluster) are rewritten in stream order, behind the launches that read the
 *     old content on the same stream; work that still reads them on another stream is not waited
 *     for.  A caller that changes streams synchronises the old one first.
 *   - Argument checking happens on the host before anything is enqueued.
 *   - The library allocates small device-side metadata of its own (rotary table, page tables,
 *     plan arrays, fp8 scales) the first time a launch needs them; the big buffers (page pool,
 *     q/k/v/o) are always the caller's.
 *   - Token-major tensor layout everywhere at the boundary: [tokens][heads][head_dim], row-major,
 *     contiguous, element type io_dtype.
 *   - A context, its caches and plans are not thread-safe; use them from one host thread at a time.
 */
#ifndef SGC_H
#define SGC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    SGC_OK = 0,
    SGC_EINVAL = -1,       /* NULL / misaligned pointer, value out of range */
    SGC_ENOMEM = -2,       /* page pool exhausted, or a host/device allocation failed */
    SGC_ESHAPE = -3,       /* shapes inconsistent with the context or the cache */
    SGC_EUNSUPPORTED = -4, /* head_dim / dtype combination no kernel covers */
    SGC_EHIP = -5,         /* a HIP runtime call failed (message has the HIP error string) */
    SGC_ESTATE = -6        /* object used in the wrong state (cluster not allocated, ...) */
} sgc_status;

typedef enum { SGC_F32 = 0, SGC_BF16 = 1, SGC_FP8_E4M3 = 2 } sgc_dtype;

/* Which attention kernel family sgc_*_prefill use. */
typedef enum {
    SGC_KERNEL_AUTO = 0,    /* MFMA when it covers the shape, else generic */
    SGC_KERNEL_GENERIC = 1, /* fp32-arithmetic kernel, any supported shape/dtype */
    SGC_KERNEL_MFMA = 2,    /* matrix-core kernel: io bf16, kv bf16|fp8, head_dim 128; products on 16-bit operands
                               (an fp8 cache is widened exactly on its way into LDS) */
    SGC_KERNEL_MFMA_FP8 = 3 /* the same kernel with the FIRST product of the suffix prefill and of decode steps on the
                               e4m3 codes of an fp8 cache (fp8 matrix-core rate, twice the 16-bit one): each rotated,
                               scaled query row is rounded to e4m3 with a power-of-two scale of its own (3 significant
                               bits: a score moves by about 0.03 on unit-variance rows, well inside the 6e-2 the fp8
                               cache is held to on long prompts; peaked rows over short prompts are better served by
                               SGC_KERNEL_MFMA).  Weights, values and the second product stay bf16.  kv fp8 only. */
} sgc_kernel_kind;

/* Plain data, filled by the caller.  struct_size = sizeof(sgc_attn_params). */
typedef struct {
    uint32_t struct_size;
    int32_t n_q_heads;     /* Hq, multiple of n_kv_heads */
    int32_t n_kv_heads;    /* Hkv */
    int32_t head_dim;      /* d: 64 or 128 */
    int32_t n_layers;      /* layers the cache holds, >= 1 */
    int32_t page_tokens;   /* tokens per cache page: 16 */
    int32_t io_dtype;      /* sgc_dtype of q/k/v/o: SGC_F32 or SGC_BF16 */
    int32_t kv_dtype;      /* sgc_dtype of the cache: io_dtype, or SGC_FP8_E4M3 with io bf16 */
    float rope_base;       /* e.g. 10000, 500000; 0 = no rotation (inputs already rotated) */
    float softmax_scale;   /* 0 = 1/sqrt(head_dim) */
    int32_t max_position;  /* hint: largest prefix_len + suffix_len expected (rotary table size);
                              0 = grow on demand */
    int32_t kernel;        /* sgc_kernel_kind */
} sgc_attn_params;

typedef struct sgc_ctx sgc_ctx;
typedef struct sgc_cache sgc_cache;
typedef struct sgc_plan sgc_plan;

/* Sizes a caller can read back from a plan (all host integers). */
typedef struct {
    int32_t n_queries;
    int32_t n_clusters;
    int64_t total_tokens;   /* T = sum of suffix_len */
    int32_t max_position;   /* max over queries of prefix_len + suffix_len */
    int32_t tile_rows;      /* rows one workgroup handles (0 until uploaded) */
    int32_t n_tiles;        /* workgroups in the suffix launch (0 until uploaded) */
} sgc_plan_info;

const char *sgc_version(void);
const char *sgc_status_string(int status);

/* ---- context --------------------------------------------------------------------------------
 * Host-only: validates the parameters, touches no device.  SGC_EUNSUPPORTED for shapes/dtypes no
 * kernel covers, SGC_EINVAL for malformed values. */
int sgc_ctx_create(const sgc_attn_params *params, sgc_ctx **out);
int sgc_ctx_destroy(sgc_ctx *ctx); /* frees the context's device metadata; NULL is a no-op */
const char *sgc_last_error(const sgc_ctx *ctx);

/* ---- cluster-wise KV cache (Sec. 3.4: one cache per cluster, released after the cluster) -----
 *
 * The cache is a pool of fixed-size pages of page_tokens tokens.  One page id addresses one
 * slab in EVERY layer, holding that page's K and V for all KV heads:
 *     pool[layer][page][K|V][kv_head][page_tokens * head_dim]      (element type kv_dtype)
 * A cluster with a prefix of P tokens owns ceil(P / page_tokens) pages; token j lives in the
 * cluster's page j / page_tokens.  Inside a page K (after rotation) and V are stored in the
 * order the matrix-core operands are read in, not token-major; use sgc_cache_export /
 * sgc_cache_import to move between that and the canonical [P][Hkv][d] layout.
 * With kv_dtype = SGC_BF16 (a 16-bit cache) V is stored as given (bf16) and the rotated K, which has
 * no exact bf16 form, as IEEE binary16: 11 significant bits instead of 8 at the same size, which
 * keeps the stated 2e-2 output bar under keys with a few large channels.  The rotated, scaled query
 * is rounded to binary16 as well and the first product runs on binary16 operands.  A rotated key or
 * scaled query beyond 65504 in magnitude becomes an infinity and the rows that see it come out NaN.
 * With kv_dtype = SGC_FP8_E4M3 each (cluster, layer, kv head) has one fp32 scale for K and one
 * for V: stored code = round_to_nearest_even(x / scale), scale = max|x| / 448 (1 if all zero),
 * OCP E4M3 with saturation; K is scaled after rotation.
 */
size_t sgc_cache_page_bytes(const sgc_attn_params *params);                 /* one page, one layer */
size_t sgc_cache_pool_bytes(const sgc_attn_params *params, int64_t total_pages); /* all layers */

/* dev_pool: caller-owned device memory of pool_bytes bytes, 256-byte aligned; the library only
 * indexes it.  The number of pages is pool_bytes / (n_layers * page_bytes).  Host-only. */
int sgc_cache_create(sgc_ctx *ctx, void *dev_pool, size_t pool_bytes, int32_t max_clusters,
                     sgc_cache **out);
int sgc_cache_destroy(sgc_cache *cache);
/* Reserve pages for a cluster (host-only bookkeeping).  SGC_ENOMEM if the pool cannot hold it
 * (nothing is changed then), SGC_ESTATE if the cluster is already allocated. */
int sgc_cache_alloc_cluster(sgc_cache *cache, int32_t cluster_id, int32_t prefix_len);
/* Release a cluster's pages.  The caller must make sure no enqueued launch still reads them. */
int sgc_cache_free_cluster(sgc_cache *cache, int32_t cluster_id);
int64_t sgc_cache_total_pages(const sgc_cache *cache);
int64_t sgc_cache_free_pages(const sgc_cache *cache);
/* Copies up to cap page ids of the cluster into out_pages (may be NULL); returns the number of
 * pages the cluster owns (>= 0) or a negative status; *out_prefix_len (may be NULL) gets P. */
int sgc_cache_cluster_pages(const sgc_cache *cache, int32_t cluster_id, int32_t *out_pages,
                            int32_t cap, int32_t *out_prefix_len);

/* ---- prefix prefill (Sec. 3.4: run the representative prompt once, keep its K/V) -------------
 * One cluster, one layer.  dev_k, dev_v: [prefix_len][Hkv][d], before rotation.  Rotates K at
 * positions 0..prefix_len-1 and writes K and V into the cluster's pages (quantising when the
 * cache is fp8); the unused tail of the last page is zeroed.
 * dev_q / dev_o: [prefix_len][Hq][d] or both NULL.  When given, o receives the causal
 * self-attention of the prefix (row i sees keys 0..i, read back from the cache as stored) and
 * dev_lse (may be NULL) [Hq][prefix_len] fp32 the natural-log log-sum-exp of the scaled scores.
 * prefix_len must equal the length given to sgc_cache_alloc_cluster.
 * dev_k = dev_v = NULL (dev_q and dev_o given): the pages already hold this layer's keys and values
 * (sgc_project_qkv_prefix, sgc_cache_import, an earlier call); only the attention output is computed. */
int sgc_prefix_prefill(sgc_ctx *ctx, sgc_cache *cache, int32_t cluster_id, int32_t layer,
                       const void *dev_q, const void *dev_k, const void *dev_v, void *dev_o,
                       float *dev_lse, int32_t prefix_len, void *hip_stream);

/* The same for n clusters of one layer in one launch per kernel (Sec. 3.4 computes each cluster's
 * cache once; a batch of clusters is independent work).  cluster_ids[n]: distinct allocated
 * clusters.  dev_q, dev_k, dev_v, dev_o, dev_lse: HOST arrays of n device pointers, entry i shaped
 * as above for cluster_ids[i] with that cluster's prefix_len; dev_q and dev_o may both be NULL
 * (cache fill only) or hold NULL entries for clusters that need no attention output; dev_lse may be
 * NULL or hold NULL entries.  The pointer arrays are read before the call returns. */
int sgc_prefix_prefill_batched(sgc_ctx *ctx, sgc_cache *cache, int32_t n, const int32_t *cluster_ids,
                               int32_t layer, const void *const *dev_q, const void *const *dev_k,
                               const void *const *dev_v, void *const *dev_o, float *const *dev_lse,
                               void *hip_stream);

/* ---- query -> cluster -> cache mapping (Sec. 3.2 labels; Sec. 3.4 cluster-wise serving) ------
 * Host-only, deterministic.  labels[n] in [0, n_clusters) is query n's cluster, suffix_len[n]
 * >= 0 its number of question tokens.  Every cluster that has at least one query must be
 * allocated in `cache` (its prefix length is read from there).
 * Outputs (caller-allocated host arrays, int32):
 *   order[n_queries]        queries grouped by cluster, original order kept inside a cluster
 *   cluster_off[n_clusters+1]  order[cluster_off[c] .. cluster_off[c+1]) are cluster c's queries
 *   cu_seqlens[n_queries+1] first token row of each query in the packed q/k/v/o arrays, which
 *                           stay in ORIGINAL query order
 * *out_plan receives an opaque plan for sgc_suffix_prefill_batched; it stays valid while the
 * clusters it names keep their allocation. */
int sgc_assign_clusters(sgc_ctx *ctx, const sgc_cache *cache, int32_t n_queries,
                        const int32_t *labels, const int32_t *suffix_len, int32_t n_clusters,
                        int32_t *order, int32_t *cluster_off, int32_t *cu_seqlens,
                        sgc_plan **out_plan);
/* Copies the plan's work lists to the device (allocates them).  Optional: the first
 * sgc_suffix_prefill_batched call does it otherwise.  Asynchronous on the stream. */
int sgc_plan_upload(sgc_plan *plan, void *hip_stream);
int sgc_plan_get_info(const sgc_plan *plan, sgc_plan_info *out);
int sgc_plan_destroy(sgc_plan *plan);

/* ---- batched suffix prefill (Sec. 3.4: each query appends its tokens to the cached prompt) ---
 * One launch for every query of every cluster in the plan, one layer.
 * dev_q, dev_o: [T][Hq][d]; dev_k, dev_v: [T][Hkv][d]; packed in original query order by
 * cu_seqlens; before rotation.  dev_lse (may be NULL): [Hq][T] fp32, natural log.
 * o rows are written for every token of every query; nothing else is touched. */
int sgc_suffix_prefill_batched(sgc_ctx *ctx, const sgc_cache *cache, sgc_plan *plan, int32_t layer,
                               const void *dev_q, const void *dev_k, const void *dev_v,
                               void *dev_o, float *dev_lse, void *hip_stream);

/* ---- decode after the suffix prefill (App. A.2: generation is capped at 32 tokens per query) -----
 * Every generated token attends over the cluster's cached prompt, the query's question tokens and
 * the tokens generated before it.  The cached-prompt part of a step stacks the rows of all queries of
 * a cluster into shared row tiles, so the prompt's K/V are read once per cluster and step, not once
 * per query.  bf16 io, head_dim 128 only (SGC_EUNSUPPORTED otherwise).
 *
 * sgc_plan_enable_decode: host-only; call it before the plan's first suffix prefill.  Reserves room
 * for max_new_tokens more tokens in every query's suffix pages and keeps those pages per layer
 * (device memory: layers x pages of all queries).  A query's question plus generated tokens may not
 * exceed 1024.
 *
 * sgc_decode_step_batched: one layer, one step (0-based) for every query of the plan (a query without
 * question tokens generates from the cached prompt alone).  dev_q / dev_o: [n_queries][Hq][d], dev_k /
 * dev_v: [n_queries][Hkv][d], row n = query n in original order, the token generated at this step,
 * before rotation (position prefix_len + suffix_len + step).
 * dev_lse (may be NULL): [Hq][n_queries] fp32, natural log.  Appends the token's rotated K and V to
 * the query's pages of this layer, then attends.  For each layer the caller runs the suffix prefill
 * first and then steps 0, 1, 2, ... in order.  Asynchronous on hip_stream. */
int sgc_plan_enable_decode(sgc_plan *plan, int32_t max_new_tokens);
int sgc_decode_step_batched(sgc_ctx *ctx, const sgc_cache *cache, sgc_plan *plan, int32_t layer,
                            int32_t step, const void *dev_q, const void *dev_k, const void *dev_v,
                            void *dev_o, float *dev_lse, void *hip_stream);

/* sgc_decode_step_batched for callers that cannot allocate device memory: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels, same
 * results.  The call allocates nothing (no hipMalloc / hipFree / host allocation of the HIP runtime's):
 * the partial results of the step's cached-prompt part, which sgc_decode_step_batched keeps in a block
 * of the context's pool, go to a fixed 32 MiB device array inside the library (one copy per GPU, held
 * until the process ends).  SGC_ENOMEM if they need more: n_queries * Hq * d * 2 bytes plus n_queries *
 * Hq * 4, times the number of key ranges the plan splits long prompts into (at most 8).  Every table the
 * step reads must already be on the device and current, which is the case once the plan's suffix prefill
 * has run and no cluster was allocated or released since: SGC_ESTATE otherwise (rotary table too short --
 * set max_position to cover prefix + question + generated tokens --, page tables or tile lists stale).
 * All calls on one GPU share the array and it keeps the last call's contents; nothing in it needs
 * clearing (a step overwrites every entry it reads), but two calls whose kernels overlap on one GPU (two
 * streams, two host threads, two contexts) race on it. */
int sgc_decode_step_batched_noalloc(sgc_ctx *ctx, const sgc_cache *cache, sgc_plan *plan, int32_t layer,
                                    int32_t step, const void *dev_q, const void *dev_k, const void *dev_v,
                                    void *dev_o, float *dev_lse, void *hip_stream);

/* ---- query clustering (Sec. 3.2; App. A.2; linkages of Table 3) -------------------------------
 * Agglomerative hierarchical clustering of m query (subgraph) embeddings with Euclidean distance,
 * stopped when n_clusters clusters are left ("cutting the dendrogram at a predefined number of
 * clusters").  embeddings: HOST array [m][dim], row-major, finite.  labels: HOST array [m], receives
 * cluster ids 0 .. n_clusters-1, clusters numbered by their first (lowest-index) member; ready for
 * sgc_assign_clusters.  Equal distances: the pair whose clusters have the smallest first members is
 * merged.  Arithmetic in fp64.  ctx may be NULL (it only receives the error text).  Host-only;
 * O(m^2) memory.  m = 0 is allowed; otherwise 1 <= n_clusters <= m. */
typedef enum {
    SGC_LINKAGE_WARD = 0,      /* smallest growth of the within-cluster sum of squares */
    SGC_LINKAGE_SINGLE = 1,    /* closest pair of members */
    SGC_LINKAGE_AVERAGE = 2,   /* mean over member pairs */
    SGC_LINKAGE_COMPLETE = 3,  /* farthest pair of members */
    SGC_LINKAGE_CENTROID = 4   /* distance of the cluster means */
} sgc_linkage;
int sgc_cluster_queries(sgc_ctx *ctx, int32_t m, int32_t dim, const float *embeddings, int32_t linkage,
                        int32_t n_clusters, int32_t *labels);

/* ---- representative subgraph (Sec. 3.3) -----------------------------------------------------------
 * Per cluster, the union of all nodes and of all edges of the subgraphs retrieved by the cluster's
 * queries.  Query i's subgraph: node ids nodes[node_off[i] .. node_off[i+1]) and directed edges
 * (edges[2e], edges[2e+1]) for e in [edge_off[i], edge_off[i+1]); duplicates allowed.  Outputs, all
 * HOST arrays: out_node_off / out_edge_off [n_clusters + 1]; out_nodes with room for node_off[m] ids;
 * out_edges with room for edge_off[m] pairs.  Cluster k's distinct nodes come out ascending in
 * out_nodes[out_node_off[k] .. out_node_off[k+1]), its distinct edges ascending by (source,
 * destination).  (a, b) and (b, a) are different edges.  ctx may be NULL.  Host-only. */
int sgc_union_subgraphs(sgc_ctx *ctx, int32_t m, const int32_t *labels, int32_t n_clusters,
                        const int64_t *node_off, const int32_t *nodes, const int64_t *edge_off,
                        const int32_t *edges, int64_t *out_node_off, int32_t *out_nodes,
                        int64_t *out_edge_off, int32_t *out_edges);

/* ---- the attention layer's projections (Sec. 3.4) -------------------------------------------------
 * Sec. 3.4 feeds the representative prompt, and then every query's question tokens, through the LLM's
 * layers.  Inside a layer the hidden states x [rows][d_model] are projected to queries, keys and values,
 * and the attention output is projected back: y = Attention(x Wq^T, x Wk^T, x Wv^T) Wo^T.  Weights are
 * DEVICE arrays in io_dtype, stored "out features x in features", row-major:
 *   dev_w_qkv [(Hq + 2 Hkv) d][d_model]: rows are the Q heads, then the K heads, then the V heads, each
 *             head's d channels together;        dev_w_o [d_model][Hq d].
 * Products accumulate in fp32; q, keys, values and y are rounded to io_dtype (kv_dtype in the cache)
 * once, when stored.  Every row of x, q, y must start 16-byte aligned.  Normalisation and residual
 * connections are the caller's.
 *
 * sgc_project_qkv_prefix[_batched]: x of each cluster's prompt [prefix_len][d_model] -> keys rotated at
 * positions 0..prefix_len-1 and values written into the cluster's pages exactly as sgc_prefix_prefill
 * stores them (an fp8 cache takes its per-head scales from the projected keys and values), and, when
 * dev_q is given, the un-rotated queries [prefix_len][Hq][d] into dev_q (pass them to
 * sgc_prefix_prefill with dev_k = dev_v = NULL to get the prompt's attention output).  Batched form:
 * dev_x and dev_q are HOST arrays of n device pointers (dev_q may be NULL or hold NULL entries).
 *
 * sgc_project_qkv_suffix: x [T][d_model] packed like q of sgc_suffix_prefill_batched -> un-rotated queries
 * into dev_q [T][Hq][d]; keys (rotated at prefix_len + j) and values are kept with the plan for `layer`
 * until the next projection or until the plan changes.  Follow it with sgc_suffix_prefill_batched for the
 * same layer with dev_k = dev_v = NULL; without a projection for that layer that call returns SGC_ESTATE.
 *
 * sgc_project_out: dev_o [n_tokens][Hq][d] -> dev_y [n_tokens][d_model].
 * All three are asynchronous on hip_stream. */
int sgc_project_qkv_prefix(sgc_ctx *ctx, sgc_cache *cache, int32_t cluster_id, int32_t layer, const void *dev_x,
                           const void *dev_w_qkv, int32_t d_model, void *dev_q, int32_t prefix_len,
                           void *hip_stream);
int sgc_project_qkv_prefix_batched(sgc_ctx *ctx, sgc_cache *cache, int32_t n, const int32_t *cluster_ids,
                                   int32_t layer, const void *const *dev_x, const void *dev_w_qkv,
                                   int32_t d_model, void *const *dev_q, void *hip_stream);
int sgc_project_qkv_suffix(sgc_ctx *ctx, const sgc_cache *cache, sgc_plan *plan, int32_t layer,
                           const void *dev_x, const void *dev_w_qkv, int32_t d_model, void *dev_q,
                           void *hip_stream);
int sgc_project_out(sgc_ctx *ctx, const void *dev_o, const void *dev_w_o, int32_t d_model, int64_t n_tokens,
                    void *dev_y, void *hip_stream);

/* ---- kernel timing (measurement aid; no effect on results) -----------------------------------
 * With timing on, sgc_suffix_prefill_batched records HIP events on its launch stream around the
 * suffix K/V ingest kernel and around the attention kernel; the events of the last 128 timed launches
 * are kept, so a caller can enqueue many launches without waiting and read all durations afterwards.
 * sgc_timing_get waits for the launch recorded `back` timed launches before the last one (0 = the
 * last) to finish and returns the two durations in milliseconds (either pointer may be NULL);
 * SGC_ESTATE if timing is off or that launch was never recorded, SGC_EINVAL if back is outside
 * [0, 128).  sgc_timing_last is sgc_timing_get with back = 0.  sgc_timing_enable restarts the count;
 * on = 0 switches timing off, on = 1 times every launch, on = n > 1 every n-th launch, the first included
 * (three event records cost the stream about 8 us per launch; a loop that measures its own throughput
 * samples); negative: SGC_EINVAL.  Host-only calls. */
int sgc_timing_enable(sgc_ctx *ctx, int on);
int sgc_timing_get(sgc_ctx *ctx, int32_t back, float *ingest_ms, float *attention_ms);
int sgc_timing_last(sgc_ctx *ctx, float *ingest_ms, float *attention_ms);

/* ---- canonical view of a cluster's cache (tests, checkpointing) -----------------------------
 * dev_k, dev_v: [prefix_len][Hkv][d] as stored: fp32 for an fp32 cache; binary16 K and bf16 V for a
 * 16-bit cache; raw e4m3 codes for fp8.  K is the rotated K.
 * host_k_scale, host_v_scale: [Hkv] fp32 (written by export / read by import; ignored and may
 * be NULL unless the cache is fp8).  Export synchronises the stream before returning. */
int sgc_cache_export(sgc_ctx *ctx, const sgc_cache *cache, int32_t cluster_id, int32_t layer,
                     void *dev_k, void *dev_v, float *host_k_scale, float *host_v_scale,
                     void *hip_stream);
int sgc_cache_import(sgc_ctx *ctx, sgc_cache *cache, int32_t cluster_id, int32_t layer,
                     const void *dev_k, const void *dev_v, const float *host_k_scale,
                     const float *host_v_scale, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* SGC_H */
