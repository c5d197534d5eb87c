// Internal declarations shared by the host code and the kernels of libsgc.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <string>
#include <vector>

#include "sgc.h"

namespace sgc {

constexpr int kPageTokens = 16;

// ---- page-internal element order -------------------------------------------------------------
// A page holds 16 tokens of one KV head: a K part and a V part of 16 * d elements each.  Both
// are stored in the order the 32x32x16 matrix-core instruction reads its A operand in, so a
// page can be copied into LDS linearly and read back conflict-free as 1 KiB operand blocks.
//
// K part: [d/16][2][16 tokens][8 channels]; block (kb, h) holds channels kb*16 + h*8 .. +7.
//   A lane of the QK^T product (operand row = key, 8 consecutive channels) finds its 8
//   elements contiguous.
// V part: [d/32][2][32 channels][8 tokens]; block (db, h) holds channels db*32 .. +31 and the 8
//   tokens {4h + (i & 3) + 8 (i >> 2) : i = 0..7}.  This is the set of keys one lane of the
//   32x32 score accumulator holds in 8 consecutive registers, so the probabilities can feed the
//   PV product without any cross-lane movement, and V is already transposed (operand row =
//   channel, 8 keys contiguous).
__host__ __device__ inline int k_page_index(int tok, int c)
{
    return ((((c >> 4) * 2 + ((c >> 3) & 1)) * kPageTokens) + tok) * 8 + (c & 7);
}
__host__ __device__ inline int v_page_index(int tok, int c)
{
    const int h = (tok >> 2) & 1;
    const int i = (tok & 3) | ((tok >> 3) << 2);
    return ((((c >> 5) * 2 + h) * 32) + (c & 31)) * 8 + i;
}

// ---- element type of the rotated keys in 16-bit pages ------------------------------------------
// A rotated key is a sum of two products and has no exact bf16 form.  Rounded to bf16 (8 significant
// bits) the keys of a head with a few large channels move a score by up to 1e-2 and an output by more
// than the 2e-2 a bf16 result is held to; IEEE binary16 (11 significant bits) costs the same two bytes
// and the same matrix-core rate.  So in every 16-bit page (cluster caches with kv_dtype SGC_BF16 and
// the batch's suffix pages) K is binary16 and V, which is stored as given, stays bf16; the first
// product runs on binary16 operands (the rotated, scaled query is rounded to binary16 as well), the
// second on bf16.  Magnitudes beyond 65504 become infinities and poison the rows that see them.
typedef __attribute__((ext_vector_type(2))) _Float16 sgc_f16x2;
__device__ inline uint16_t f32_to_f16_bits(float x)
{
    const _Float16 h = (_Float16)x;
    return __builtin_bit_cast(uint16_t, h);
}
__device__ inline uint32_t pack2_f16(float a, float b)
{
    const sgc_f16x2 p = {(_Float16)a, (_Float16)b};
    return __builtin_bit_cast(uint32_t, p);
}
__device__ inline float f16_bits_to_f32(uint16_t b) { return (float)__builtin_bit_cast(_Float16, b); }
// internal element-type tag beside the sgc_dtype values: IEEE binary16
constexpr int kElemF16 = 16;
// the type K is stored in for a cache of type kv_dtype
__host__ __device__ inline int k_elem_type(int kv_dtype) { return kv_dtype == SGC_BF16 ? kElemF16 : kv_dtype; }

__host__ __device__ inline int dtype_bytes(int dt) { return dt == SGC_F32 ? 4 : (dt == SGC_BF16 ? 2 : 1); }

// Geometry of the page pool, passed by value to kernels.
struct PoolGeom {
    char *pool;            // device base of the whole pool
    int64_t total_pages;   // pages per layer
    int32_t n_kv_heads;
    int32_t head_dim;
    int32_t kv_dtype;
    int32_t kv_bytes;      // bytes per element
    int64_t head_part_bytes;   // 16 * d * kv_bytes: K (or V) of one head in one page
    int64_t page_bytes;        // 2 * Hkv * head_part_bytes
    int64_t layer_bytes;       // total_pages * page_bytes
    __host__ __device__ inline char *k_part(int layer, int page, int hk) const
    {
        return pool + layer * layer_bytes + (int64_t)page * page_bytes + (int64_t)hk * head_part_bytes;
    }
    __host__ __device__ inline char *v_part(int layer, int page, int hk) const
    {
        return pool + layer * layer_bytes + (int64_t)page * page_bytes +
               (int64_t)(n_kv_heads + hk) * head_part_bytes;
    }
};

// One workgroup's share of an attention launch, with everything the workgroup needs to start ALL its
// loads at once (one 160-byte scalar load instead of chains of dependent table look-ups).
constexpr int kTileQueries = 4;      // queries a tile record describes inline
struct TileQuery {
    int32_t tok0;    // first sorted token of the query (INT32_MAX in unused slots)
    int32_t src0;    // first row of the query in the caller's packed arrays
    int32_t len;     // suffix length
    int32_t page0;   // first page of the query in the suffix page pool
};
struct Tile {
    int32_t cluster;     // cluster id (index into the cache's per-cluster arrays)
    int32_t hk;          // KV head
    int32_t row0;        // first row inside the (cluster, hk) row space; row = token * g + head-in-group
    int32_t n_rows;      // valid rows in this tile (0 = padding tile, exit at once)
    int32_t prefix_len;  // cached tokens of the cluster
    int32_t pt_off;      // first entry of the cluster in the flat page table
    int32_t tok_base;    // first sorted token of the cluster (prefix mode: index of the job)
    int32_t sq_lo, sq_hi;   // sorted queries of the tile's first and last row
    int32_t last_qpos;   // position of the last row's token inside its query
    int32_t n_q;         // sq_hi - sq_lo + 1; the records q[] are valid when n_q <= kTileQueries
    int32_t pad;         // decode tiles: key range index << 24 | position offset (cached keys outside the range)
    int32_t first_pages[12];       // page ids of the cluster's first 12 pages (clamped to its last page)
    TileQuery q[kTileQueries];     // queries sq_lo, sq_lo + 1, ...
};
static_assert(sizeof(Tile) == 160, "tile record layout");

// What the host sends per tile; the device writes the tile record from it and from tables it already
// holds (a fifth of the record's bytes cross the host link).
struct TileSeed {
    int32_t cluster;     // suffix tiles: cluster id; prefix tiles: index of the job
    int32_t hk;
    int32_t row0;
    int32_t n_rows;      // 0 = padding tile
    int32_t sq_lo, sq_hi;
    int32_t last_qpos;
    int32_t pad;
};
static_assert(sizeof(TileSeed) == 32, "tile seed layout");

// Per sorted token: where it comes from and where it sits in its query.
struct TokInfo {
    int32_t src;    // row of the token in the caller's packed arrays
    int32_t qpos;   // index of the token inside its query
    int32_t sq;     // sorted query index
    int32_t pad;
};

// One cluster of a (batched) prefix prefill.
struct PrefixJob {
    const void *q, *k, *v;   // [P][Hq][d] (q may be null), [P][Hkv][d], io dtype, before rotation
    void *o;                 // [P][Hq][d] or null
    float *lse;              // [Hq][P] or null
    float *scale_kv;         // fp8 cache: the [2][Hkv] scales of this cluster and layer, else null
    int32_t cluster;
    int32_t prefix_len;
    int32_t pt_off;          // first entry of the cluster in the flat page table
    int32_t page0;           // first page of the job in the launch-wide page numbering
};

// One decode step of every (non-empty) query of a plan: arguments of the own-keys kernel.
constexpr int kDecodeMaxSplits = 8;       // key ranges the cached part of a decode step may be split into
constexpr int kDecodeMaxKeys = 1024;      // own keys (suffix + generated) a query may reach while decoding
struct DecodeArgs {
    const void *q, *k, *v;        // the new token of every query: [n_queries][Hq][d], [n_queries][Hkv][d], bf16
    void *o;                      // [n_queries][Hq][d] bf16
    float *lse;                   // [Hq][n_queries] natural log, or null
    const void *o_cached;         // cached-prefix part of the same rows: [n_queries][Hq][d] bf16 (normalised) ...
    const float *lse_cached;      // ... and its log-sum-exp [Hq][n_queries], natural log (-inf: no cached keys)
    int32_t n_splits;             // the cached part comes as n_splits partial results (key ranges), set s at ...
    int64_t split_o_elems, split_lse_elems;   // ... o_cached + s * split_o_elems, lse_cached + s * split_lse_elems
    char *spool;                  // the layer's suffix pages
    const int32_t *sq_query;      // [n_sq] original index of the sorted query
    const int32_t *sq_len, *sq_page0, *sq_cluster;
    const int32_t *cl_prefix_len;
    const float2 *rope;
    int32_t n_sq, n_queries, step, n_q_heads, n_kv_heads;
    int32_t key_cap;              // multiple of 16, >= every query's len + step + 1, <= kDecodeMaxKeys
    int32_t use_mfma;             // head_dim 128 and 16-bit rows: the matrix-core form of the own-keys kernel may run
    float scale_log2e;
};

// ---- projections around the attention (sgc_gemm.hip) -------------------------------------------
// One slab of up to 256 rows of a projection's left operand and where its results go.
struct GemmRowTile {
    const void *a;       // first row of the slab, [rows][K] bf16
    void *c;             // plain output (Q, or the whole product): first row of the slab, or null to store none
    void *ck, *cv;       // staged K / V outputs [rows][Hkv d] (first row of the slab), when keys are staged
    int32_t rows;        // valid rows, 1..256
    int32_t pos0;        // cache pages: position of the slab's first row inside its cluster (a multiple of 16)
    int32_t pt_off;      // cache pages: first page-table entry of the cluster
    int32_t dest0;       // suffix pages: index of the slab's first row in row_dest
};
static_assert(sizeof(GemmRowTile) == 48, "row tile record layout");

// C = A W^T on the matrix cores.  Columns [0, n_plain) are stored row-major with leading dimension ldc;
// with the QKV epilogue the columns after them are Hkv K heads and then Hkv V heads of 128 channels.
struct GemmArgs {
    const void *w;                // [N][K] bf16
    int32_t N, K;
    const GemmRowTile *tiles;     // [n_row_tiles], or null: slab r is rows 256 r .. of a / c below
    const void *a;
    void *c;
    int64_t M;
    int32_t n_row_tiles, n_col_tiles;
    int32_t ldc;
    int32_t n_plain;
    int32_t kv_dest;              // 0: the cache's pages (prompt), 1: the batch's suffix pages, 2: staging matrices
    int32_t n_kv_heads;
    char *kv_base;                // the layer's first page (cache pool or suffix pool)
    int64_t page_bytes;           // one page, every head, K and V
    int64_t part_bytes;           // K (or V) of one head in one page
    const int32_t *page_table;    // kv_dest 0: flat page ids
    const int2 *row_dest;         // kv_dest 1: per packed row {16 * page + slot, position}
    const float2 *rope;           // [position][64] (cos, sin), or null
};

enum { MODE_SUFFIX = 0, MODE_PREFIX = 1 };

// Everything an attention kernel needs, by value.
struct AttnArgs {
    const void *q, *k, *v;   // token-major q [*][Hq][d], k/v [*][Hkv][d] (io dtype), before rotation
    void *o;                 // [*][Hq][d]
    float *lse;              // [Hq][lse_stride] or null
    int64_t lse_stride;
    PoolGeom pool;
    int32_t layer;
    const int32_t *page_table;    // flat page ids
    const int32_t *cl_pt_off;     // [max_clusters] first entry of the cluster in page_table
    const int32_t *cl_prefix_len; // [max_clusters]
    const float *kv_scale;        // [max_clusters][n_layers][2][Hkv] or null (fp8 cache only)
    int32_t n_layers;
    const float2 *rope;           // [rope_len][d/2] (cos, sin) or null when rotation is off
    const Tile *tiles;
    int32_t n_tiles;
    // suffix mode: sorted-token and sorted-query tables (sorted = grouped by cluster; queries
    // without tokens are left out of the query tables)
    const int32_t *cl_tok_off;    // [n_clusters + 1] first sorted token of each cluster
    const int32_t *tok_src;       // [T] row of the token in the caller's packed arrays
    const int32_t *tok_qpos;      // [T] index of the token inside its query
    const int32_t *tok_sq;        // [T] sorted query index of the token
    const TokInfo *tok_info;      // [T] the three above in one record
    const int32_t *sq_src0;       // [n_queries] first packed row of the query
    const int32_t *sq_len;        // [n_queries] suffix length
    const int32_t *sq_tok0;       // [n_queries] first sorted token of the query
    const int32_t *sq_cluster;    // [n_queries]
    const int32_t *sq_page0;      // [n_queries] first page of the query in the suffix page pool
    const char *spool;            // suffix page pool (bf16 pages, same layout as cache pages) or null
    int64_t total_tokens;
    // prefix mode: the MFMA kernel takes its clusters from jobs (a tile's tok_base field is the job index),
    // the generic kernel works on one cluster per launch (prefix_cluster, prefix_len, q/k/v/o/lse above)
    const PrefixJob *jobs;
    int32_t prefix_cluster;
    int32_t prefix_len;
    int32_t mode;
    int32_t n_q_heads, n_kv_heads, group, head_dim;
    int32_t io_dtype;
    float scale_log2e;            // softmax_scale * log2(e)
    // decode: the one new token of a query sits pos_shift tokens behind the end of its suffix, and the MFMA
    // kernel only does the cached-prefix part (skip_self), leaving the own keys to the decode kernel
    int32_t pos_shift;
    int32_t skip_self;
    // a tile whose pad field names key range s (upper 8 bits) writes its rows to o + s * split_o_bytes and
    // lse + s * split_lse_elems; the low 24 bits of pad are added to the rows' positions
    int64_t split_o_bytes, split_lse_elems;
    // decode: blocks behind the tiles append the new token of each of the n_append sorted queries (k, v above: the
    // new tokens [n_queries][Hkv][d]; sq_query: original index of the sorted query) to the suffix pages
    const int32_t *sq_query;
    int32_t n_append;
    // fp8 cache: run the first product on the e4m3 codes, with the query quantised per row (suffix mode)
    int32_t fp8_first_product;
};

}  // namespace sgc

// ---- host objects behind the opaque handles --------------------------------------------------
struct sgc_dev_block {
    char *p = nullptr;
    size_t bytes = 0;
    hipStream_t last = nullptr;     // stream of the last launch that may still read the block
};

struct sgc_ctx {
    sgc_attn_params p;
    float scale;
    bool use_mfma;
    bool fp8_first_product; // SGC_KERNEL_MFMA_FP8: QK^T on the e4m3 codes of an fp8 cache (suffix prefill and decode)
    int tile_rows;         // rows per workgroup of the chosen attention kernel
    std::string err;
    float2 *d_rope = nullptr;
    int rope_len = 0;
    // Device blocks and pinned staging buffers are kept and reused: the per-batch tables are small and a
    // hipMalloc / hipFree pair per batch costs more than the copies themselves.
    std::vector<sgc_dev_block> dev_free;
    static constexpr int kStageSlots = 8;      // copies a caller can have in flight before the host waits for one
    char *h_stage[kStageSlots] = {};
    const char *h_stage_dev[kStageSlots] = {};   // the same buffers as kernels address them
    size_t h_stage_cap[kStageSlots] = {};
    hipEvent_t stage_ev[kStageSlots] = {};
    bool stage_pending[kStageSlots] = {};
    int stage_next = 0;
    bool timing = false;            // record events around the suffix launch's kernels
    int timing_period = 1;          // ... of every timing_period-th suffix launch
    uint64_t timing_launches = 0;   // suffix launches since timing was switched on
    // the last kTimingRing timed suffix launches: events before ingest, between, after attention
    static constexpr int kTimingRing = 128;
    hipEvent_t ev[kTimingRing][3] = {};
    uint64_t timing_count = 0;      // timed launches recorded since timing was switched on
};

struct sgc_cluster_entry {
    bool allocated = false;
    int32_t prefix_len = 0;
    std::vector<int32_t> pages;
};

struct sgc_cache {
    sgc_ctx *ctx;
    sgc::PoolGeom geom;
    size_t pool_bytes;
    int32_t max_clusters;
    std::vector<sgc_cluster_entry> cl;
    std::vector<int32_t> free_list;   // stack; back() is handed out next
    uint64_t generation = 0;          // bumped by alloc/free
    // device mirrors (built lazily): one allocation [page table: total_pages][pt_off: max_clusters][prefix_len: max_clusters]
    bool dirty = true;
    int32_t *d_tables = nullptr;
    int32_t *d_page_table = nullptr;
    int32_t *d_pt_off = nullptr;
    int32_t *d_prefix_len = nullptr;
    float *d_scale = nullptr;         // fp8 only: [max_clusters][n_layers][2][Hkv]
};

struct sgc_plan {
    sgc_ctx *ctx;
    const sgc_cache *cache;
    int32_t n_queries, n_clusters;
    int64_t total_tokens;
    int32_t max_position;
    std::vector<int32_t> order, cluster_off;
    std::vector<int32_t> cl_prefix_len;       // snapshot at assign time, [n_clusters]
    std::vector<int32_t> cl_tok_off;
    std::vector<int32_t> tok_src, tok_qpos, tok_sq;
    std::vector<int32_t> sq_src0, sq_len, sq_tok0, sq_cluster, sq_page0;   // non-empty queries only
    std::vector<int32_t> spage_sq;            // [total suffix pages] owning query of each suffix page
    std::vector<int32_t> sq_query;            // [non-empty queries] original index of the sorted query
    std::vector<int32_t> cl_sq_off;           // [n_clusters + 1] first sorted query of each cluster
    // decode (off unless sgc_plan_enable_decode was called): pages leave room for decode_cap more tokens per
    // query, the suffix page pool exists once per layer, and a second tile list stacks one row group per query
    int32_t decode_cap = 0;
    std::vector<sgc::Tile> dtiles;
    std::vector<int32_t> dtile_key0;          // first cached key of each decode tile's key range
    int32_t dec_splits = 1;                   // key ranges per row tile
    std::vector<sgc::TokInfo> dtok;
    size_t spool_layer_bytes = 0;
    sgc_dev_block dec_scratch;                // cached-prefix part of a decode step: O then LSE
    // projected keys of the batch (sgc_project_qkv_suffix): 1 = the suffix pages of proj_layer are written,
    // 2 = un-rotated K then V matrices [T][Hkv d] are kept in proj_kv for the suffix launch to ingest
    int32_t proj_state = 0, proj_layer = -1;
    sgc_dev_block proj_kv;
    std::vector<int32_t> row_dest;            // [T][2] per packed row: 16 * suffix page + slot, position
    const int2 *d_row_dest = nullptr;         // uploaded by the first projection on the plan
    sgc_dev_block row_dest_block;
    std::vector<sgc::Tile> tiles;
    std::vector<sgc::TokInfo> tok_info;
    uint64_t tiles_generation = 0;            // cache generation the tiles' page-table offsets belong to
    int32_t tile_rows = 0;
    bool uploaded = false;
    bool expand_pending = false;              // the device's tile records are to be (re)written before the next suffix launch
    sgc_dev_block blob, spool_block;          // device blocks behind d_blob / d_spool (from the context's pool)
    hipStream_t last_stream = nullptr;        // stream of the last launch that used the plan
    char *d_blob = nullptr;                   // one device allocation holding every array below
    const int32_t *d_cl_tok_off = nullptr, *d_tok_src = nullptr, *d_tok_qpos = nullptr, *d_tok_sq = nullptr;
    const int32_t *d_sq_src0 = nullptr, *d_sq_len = nullptr, *d_sq_tok0 = nullptr, *d_sq_cluster = nullptr;
    const int32_t *d_sq_page0 = nullptr, *d_spage_sq = nullptr;
    const sgc::Tile *d_tiles = nullptr;
    std::vector<sgc::TileSeed> seeds;         // one per entry of tiles
    const sgc::TileSeed *d_seeds = nullptr;
    const sgc::TokInfo *d_tok_info = nullptr;
    const int32_t *d_sq_query = nullptr;
    const sgc::Tile *d_dtiles = nullptr;
    const sgc::TokInfo *d_dtok = nullptr;
    char *d_spool = nullptr;                  // rotated suffix K / transposed V pages of the batch (MFMA path)
    size_t spool_bytes = 0;
};

// ---- kernel launchers (defined in the .hip files) --------------------------------------------
namespace sgc {

// Builds the (cos, sin) table for positions [0, n_pos) in double precision, stored as fp32.
hipError_t launch_rope_table(float2 *table, int n_pos, int head_dim, double base, hipStream_t s);

// Tile records from seeds.  jobs null: tiles of a suffix launch (per-cluster tables of the cache, per-query tables of
// the plan); jobs given: tiles of a batched prefix prefill.
struct ExpandArgs {
    const TileSeed *seeds;
    Tile *tiles;
    int32_t n;
    const PrefixJob *jobs;
    const int32_t *page_table, *pt_off, *prefix_len;      // the cache's device tables
    const int32_t *cl_tok_off, *sq_tok0, *sq_src0, *sq_len, *sq_page0;      // the plan's
};
hipError_t launch_expand_tiles(const ExpandArgs &e, hipStream_t s);

// Prefix ingest of n_jobs clusters: rotate K, (quantise), write K and V into the clusters' pages.
// d_page_job[p] is the job of launch-wide page p (n_pages of them).  expand (may be null): tile records to write in the
// same launch, by workgroups appended to the grid.
hipError_t launch_prefix_ingest(const PoolGeom &g, int layer, const int32_t *d_page_table, const PrefixJob *d_jobs,
                                int n_jobs, const int32_t *d_page_job, int n_pages, int io_dtype, const float2 *rope,
                                const ExpandArgs *expand, hipStream_t s);
hipError_t launch_cache_export(const PoolGeom &g, int layer, const int32_t *d_pages, int prefix_len,
                               void *k, void *v, hipStream_t s);
hipError_t launch_cache_import(const PoolGeom &g, int layer, const int32_t *d_pages, int prefix_len,
                               const void *k, const void *v, hipStream_t s);

// Suffix ingest: rotate every query's suffix K at prefix_len + j and write K and V as bf16 pages
// (cache page layout) into the suffix page pool; one workgroup per (suffix page, KV head).  expand: as above.
hipError_t launch_suffix_ingest(const AttnArgs &a, const int32_t *d_spage_sq, int n_spages, const ExpandArgs *expand,
                                hipStream_t s);

hipError_t launch_attn_generic(const AttnArgs &a, int64_t n_rows, hipStream_t s);
// Decode, per (query, head): attention over the query's own keys (the step's new token was appended to the suffix
// pages by the cached-part launch before) merged with the cached-prefix part.  head_dim 128, bf16.
hipError_t launch_decode_own_keys(const DecodeArgs &d, hipStream_t s);
hipError_t launch_fill_zero_bytes(void *p, size_t bytes, hipStream_t s);
// bytes (a multiple of 4, both pointers 16-byte aligned) from mapped host memory to device memory, read by a kernel;
// optionally a second piece in the same launch
hipError_t launch_copy_from_host(void *dst, const void *mapped_src, size_t bytes, hipStream_t s, void *dst2 = nullptr,
                                 const void *mapped_src2 = nullptr, size_t bytes2 = 0);
// Projections: the bf16 matrix-core kernel (K a multiple of 64, N a multiple of 128; qkv selects the fused
// epilogue) and a kernel for every other shape and type that deals columns [0, n0), [n0, n0 + n1) and the rest
// to three row-major matrices (c0 may be null to drop its columns).
hipError_t launch_proj_gemm(const GemmArgs &g, bool qkv, hipStream_t s);
hipError_t launch_proj_generic(const void *a, const void *w, int64_t M, int N, int K, int io_dtype, void *c0, int n0, void *c1,
                               int n1, void *c2, hipStream_t s);
hipError_t launch_zero_last_pages(char *spool, const int32_t *d_sq_len, const int32_t *d_sq_page0, int n_sq, int64_t page_bytes,
                                  hipStream_t s);
// Rows per workgroup of the MFMA attention kernel.
int mfma_tile_rows();
hipError_t launch_attn_mfma(const AttnArgs &a, hipStream_t s);

}  // namespace sgc
