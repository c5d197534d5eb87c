// Host side of libsgc: argument checking, the cluster-wise page allocator, the query->cluster
// planner and the C ABI.  Follows SubGCache (arXiv 2505.10951) Sec. 3.2 (cluster labels per
// query) and Sec. 3.4 (one KV cache per cluster: compute once, reuse for every query of the
// cluster, release).
#include <limits.h>
#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <algorithm>
#include <array>
#include <new>
#include <numeric>

#include "sgc_internal.h"

using namespace sgc;

namespace {

thread_local std::string g_err_noctx;

int fail(sgc_ctx *ctx, int code, const char *fmt, ...)
{
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof(buf), fmt, ap);
    va_end(ap);
    if (ctx)
        ctx->err = buf;
    else
        g_err_noctx = buf;
    return code;
}

int fail_hip(sgc_ctx *ctx, hipError_t e, const char *what)
{
    return fail(ctx, SGC_EHIP, "%s: %s", what, hipGetErrorString(e));
}

#define SGC_HIP(ctx, call)                                     \
    do {                                                       \
        hipError_t e__ = (call);                               \
        if (e__ != hipSuccess) return fail_hip(ctx, e__, #call); \
    } while (0)

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

bool mfma_covers(const sgc_attn_params &p)
{
    return p.io_dtype == SGC_BF16 && p.head_dim == 128 && (p.kv_dtype == SGC_BF16 || p.kv_dtype == SGC_FP8_E4M3);
}

int check_params(const sgc_attn_params *p, sgc_ctx *ctx)
{
    if (!p) return fail(ctx, SGC_EINVAL, "params is NULL");
    if (p->struct_size != sizeof(sgc_attn_params))
        return fail(ctx, SGC_EINVAL, "params.struct_size %u != %zu", p->struct_size, sizeof(sgc_attn_params));
    if (p->n_q_heads <= 0 || p->n_kv_heads <= 0 || p->n_q_heads % p->n_kv_heads != 0)
        return fail(ctx, SGC_EINVAL, "n_q_heads %d must be a positive multiple of n_kv_heads %d", p->n_q_heads,
                    p->n_kv_heads);
    if (p->n_q_heads > 1024) return fail(ctx, SGC_EINVAL, "n_q_heads %d too large", p->n_q_heads);
    if (p->head_dim != 64 && p->head_dim != 128)
        return fail(ctx, SGC_EUNSUPPORTED, "head_dim %d not supported (64 or 128)", p->head_dim);
    if (p->n_layers < 1) return fail(ctx, SGC_EINVAL, "n_layers %d < 1", p->n_layers);
    if (p->page_tokens != kPageTokens)
        return fail(ctx, SGC_EUNSUPPORTED, "page_tokens %d not supported (16)", p->page_tokens);
    if (p->io_dtype != SGC_F32 && p->io_dtype != SGC_BF16)
        return fail(ctx, SGC_EUNSUPPORTED, "io_dtype %d not supported (f32 or bf16)", p->io_dtype);
    if (!(p->kv_dtype == p->io_dtype || (p->kv_dtype == SGC_FP8_E4M3 && p->io_dtype == SGC_BF16)))
        return fail(ctx, SGC_EUNSUPPORTED, "kv_dtype %d not supported with io_dtype %d", p->kv_dtype, p->io_dtype);
    if (!(p->rope_base >= 0.0f) || !std::isfinite(p->rope_base))
        return fail(ctx, SGC_EINVAL, "rope_base must be finite and >= 0");
    if (!(p->softmax_scale >= 0.0f) || !std::isfinite(p->softmax_scale))
        return fail(ctx, SGC_EINVAL, "softmax_scale must be finite and >= 0");
    if (p->max_position < 0) return fail(ctx, SGC_EINVAL, "max_position < 0");
    if (p->kernel < SGC_KERNEL_AUTO || p->kernel > SGC_KERNEL_MFMA_FP8)
        return fail(ctx, SGC_EINVAL, "kernel %d unknown", p->kernel);
    if ((p->kernel == SGC_KERNEL_MFMA || p->kernel == SGC_KERNEL_MFMA_FP8) && !mfma_covers(*p))
        return fail(ctx, SGC_EUNSUPPORTED, "MFMA kernel needs io bf16, kv bf16|fp8, head_dim 128");
    if (p->kernel == SGC_KERNEL_MFMA_FP8 && p->kv_dtype != SGC_FP8_E4M3)
        return fail(ctx, SGC_EUNSUPPORTED, "the fp8 first product needs an fp8 cache");
    return SGC_OK;
}

size_t page_bytes_of(const sgc_attn_params &p)
{
    return (size_t)2 * p.n_kv_heads * kPageTokens * p.head_dim * dtype_bytes(p.kv_dtype);
}

// Makes sure the rotary table covers positions [0, need).
int ensure_rope(sgc_ctx *ctx, int need, hipStream_t s)
{
    if (!(ctx->p.rope_base > 0.0f)) return SGC_OK;
    if (need <= ctx->rope_len) return SGC_OK;
    int want = std::max(need, std::max(ctx->p.max_position, 1024));
    want = (want + 1023) / 1024 * 1024;
    float2 *t = nullptr;
    SGC_HIP(ctx, hipMalloc(&t, (size_t)want * (ctx->p.head_dim / 2) * sizeof(float2)));
    hipError_t e = launch_rope_table(t, want, ctx->p.head_dim, (double)ctx->p.rope_base, s);
    if (e != hipSuccess) {
        (void)hipFree(t);
        return fail_hip(ctx, e, "rope table kernel");
    }
    if (ctx->d_rope) {
        // earlier launches may still read the old table
        SGC_HIP(ctx, hipDeviceSynchronize());
        (void)hipFree(ctx->d_rope);
    }
    ctx->d_rope = t;
    ctx->rope_len = want;
    return SGC_OK;
}

// ---- reusable device blocks and pinned staging ------------------------------------------------
// A block handed back by dev_release may still be read by launches on the stream it was last used
// on; work enqueued later on that same stream is ordered behind them, any other stream waits first.
int dev_acquire(sgc_ctx *ctx, size_t bytes, hipStream_t s, sgc_dev_block *out)
{
    bytes = std::max<size_t>((bytes + 4095) / 4096 * 4096, 4096);
    int best = -1;
    for (int i = 0; i < (int)ctx->dev_free.size(); ++i) {
        const sgc_dev_block &b = ctx->dev_free[i];
        if (b.bytes >= bytes && b.bytes <= 4 * bytes && (best < 0 || b.bytes < ctx->dev_free[best].bytes)) best = i;
    }
    if (best >= 0) {
        *out = ctx->dev_free[best];
        ctx->dev_free.erase(ctx->dev_free.begin() + best);
        if (out->last != s) SGC_HIP(ctx, hipStreamSynchronize(out->last));
        out->last = s;
        return SGC_OK;
    }
    void *p = nullptr;
    SGC_HIP(ctx, hipMalloc(&p, bytes));
    out->p = static_cast<char *>(p);
    out->bytes = bytes;
    out->last = s;
    return SGC_OK;
}

void dev_release(sgc_ctx *ctx, sgc_dev_block b, hipStream_t last)
{
    if (!b.p) return;
    b.last = last;
    if (ctx->dev_free.size() >= 16) {        // keep the pool small: drop the oldest block
        (void)hipStreamSynchronize(ctx->dev_free.front().last);
        (void)hipFree(ctx->dev_free.front().p);
        ctx->dev_free.erase(ctx->dev_free.begin());
    }
    ctx->dev_free.push_back(b);
}

// Pinned host buffer of at least `bytes` whose previous copy, if any, has finished.
int stage_begin(sgc_ctx *ctx, size_t bytes, char **host, int *slot)
{
    const int i = ctx->stage_next;
    ctx->stage_next = (i + 1) % sgc_ctx::kStageSlots;
    if (!ctx->stage_ev[i]) SGC_HIP(ctx, hipEventCreateWithFlags(&ctx->stage_ev[i], hipEventDisableTiming));
    if (ctx->stage_pending[i]) {
        SGC_HIP(ctx, hipEventSynchronize(ctx->stage_ev[i]));
        ctx->stage_pending[i] = false;
    }
    if (ctx->h_stage_cap[i] < bytes) {
        if (ctx->h_stage[i]) SGC_HIP(ctx, hipHostFree(ctx->h_stage[i]));
        ctx->h_stage[i] = nullptr;
        ctx->h_stage_cap[i] = 0;
        const size_t cap = std::max<size_t>((bytes + 65535) / 65536 * 65536, 1 << 20);
        void *p = nullptr;
        SGC_HIP(ctx, hipHostMalloc(&p, cap, hipHostMallocMapped | hipHostMallocCoherent));
        void *dp = nullptr;
        hipError_t e = hipHostGetDevicePointer(&dp, p, 0);
        if (e != hipSuccess || !dp) {
            (void)hipHostFree(p);
            return fail_hip(ctx, e != hipSuccess ? e : hipErrorInvalidValue, "hipHostGetDevicePointer");
        }
        ctx->h_stage[i] = static_cast<char *>(p);
        ctx->h_stage_dev[i] = static_cast<const char *>(dp);
        ctx->h_stage_cap[i] = cap;
    }
    *host = ctx->h_stage[i];
    *slot = i;
    return SGC_OK;
}

// Copies `bytes` of the slot's buffer to `dev` (and, in the same launch, bytes2 from host_offset2 to dev2) and records the
// event that says the buffer has been read.
int stage_commit(sgc_ctx *ctx, int slot, void *dev, size_t bytes, hipStream_t s, void *dev2 = nullptr, size_t host_offset2 = 0,
                 size_t bytes2 = 0)
{
    if (bytes % 4 != 0 || bytes2 % 4 != 0 || (reinterpret_cast<uintptr_t>(dev) | reinterpret_cast<uintptr_t>(dev2) | host_offset2) % 16 != 0)
        return fail(ctx, SGC_EINVAL, "staged copy of %zu + %zu bytes is not aligned", bytes, bytes2);
    SGC_HIP(ctx, launch_copy_from_host(dev, ctx->h_stage_dev[slot], bytes, s, dev2, ctx->h_stage_dev[slot] + host_offset2, bytes2));
    SGC_HIP(ctx, hipEventRecord(ctx->stage_ev[slot], s));
    ctx->stage_pending[slot] = true;
    return SGC_OK;
}

// The device copy of the page tables is one array
// [page table: total_pages][first entry per cluster: max_clusters][prefix length per cluster: max_clusters].
int cache_tables_ensure(sgc_cache *c)
{
    sgc_ctx *ctx = c->ctx;
    const size_t n_pages = (size_t)c->geom.total_pages, n_cl = (size_t)c->max_clusters;
    if (c->d_tables) return SGC_OK;
    SGC_HIP(ctx, hipMalloc(&c->d_tables, sizeof(int32_t) * (n_pages + 2 * n_cl + 16)));
    c->d_page_table = c->d_tables;
    c->d_pt_off = c->d_tables + n_pages;
    c->d_prefix_len = c->d_pt_off + n_cl;
    if (ctx->p.kv_dtype == SGC_FP8_E4M3) {
        const size_t n = n_cl * ctx->p.n_layers * 2 * ctx->p.n_kv_heads;
        SGC_HIP(ctx, hipMalloc(&c->d_scale, sizeof(float) * n));
        SGC_HIP(ctx, hipMemset(c->d_scale, 0, sizeof(float) * n));
    }
    c->dirty = true;
    return SGC_OK;
}

size_t cache_tables_bytes(const sgc_cache *c) { return sizeof(int32_t) * ((size_t)c->geom.total_pages + 2 * (size_t)c->max_clusters); }

// The tables as the host allocator has them now.
void cache_tables_fill(const sgc_cache *c, int32_t *flat)
{
    const size_t n_pages = (size_t)c->geom.total_pages, n_cl = (size_t)c->max_clusters;
    int32_t *off = flat + n_pages, *plen = off + n_cl;
    size_t n = 0;
    for (size_t i = 0; i < n_cl; ++i) {
        off[i] = (int32_t)n;
        plen[i] = 0;
        if (c->cl[i].allocated) {
            plen[i] = c->cl[i].prefix_len;
            for (int32_t pg : c->cl[i].pages) flat[n++] = pg;
        }
    }
    for (; n < n_pages; ++n) flat[n] = 0;
}

// Brings the device copy of the page tables up to date with the host allocator: rewritten by one copy that is ordered on
// the stream behind the launches that read the old content.
int cache_sync(sgc_cache *c, hipStream_t s)
{
    sgc_ctx *ctx = c->ctx;
    int rc = cache_tables_ensure(c);
    if (rc != SGC_OK) return rc;
    if (!c->dirty) return SGC_OK;
    char *host = nullptr;
    int slot = 0;
    const size_t bytes = cache_tables_bytes(c);
    if ((rc = stage_begin(ctx, bytes, &host, &slot)) != SGC_OK) return rc;
    cache_tables_fill(c, reinterpret_cast<int32_t *>(host));
    if ((rc = stage_commit(ctx, slot, c->d_tables, bytes, s)) != SGC_OK) return rc;
    c->dirty = false;
    return SGC_OK;
}

int check_cluster(sgc_ctx *ctx, const sgc_cache *c, int32_t cluster_id, int32_t layer)
{
    if (cluster_id < 0 || cluster_id >= c->max_clusters)
        return fail(ctx, SGC_EINVAL, "cluster_id %d outside [0, %d)", cluster_id, c->max_clusters);
    if (!c->cl[cluster_id].allocated) return fail(ctx, SGC_ESTATE, "cluster %d is not allocated", cluster_id);
    if (layer < 0 || layer >= ctx->p.n_layers)
        return fail(ctx, SGC_EINVAL, "layer %d outside [0, %d)", layer, ctx->p.n_layers);
    return SGC_OK;
}

void fill_common_args(AttnArgs &a, sgc_ctx *ctx, const sgc_cache *c, int32_t layer)
{
    memset(&a, 0, sizeof(a));
    a.pool = c->geom;
    a.layer = layer;
    a.page_table = c->d_page_table;
    a.cl_pt_off = c->d_pt_off;
    a.cl_prefix_len = c->d_prefix_len;
    a.kv_scale = c->d_scale;
    a.n_layers = ctx->p.n_layers;
    a.rope = (ctx->p.rope_base > 0.0f) ? ctx->d_rope : nullptr;
    a.n_q_heads = ctx->p.n_q_heads;
    a.n_kv_heads = ctx->p.n_kv_heads;
    a.group = ctx->p.n_q_heads / ctx->p.n_kv_heads;
    a.head_dim = ctx->p.head_dim;
    a.io_dtype = ctx->p.io_dtype;
    a.scale_log2e = ctx->scale * 1.4426950408889634f;
    a.fp8_first_product = ctx->fp8_first_product ? 1 : 0;
}

// Workgroup b of a launch runs on XCD b % 8, and each XCD has an L2 of its own: units of work that read the same
// keys and values stay on one XCD.  Units are dealt, heaviest first (equal ones in their given order), each to the
// XCD with the least work so far; returned per XCD: the units' indices in the order they were dealt.
constexpr int kXcd = 8;
std::array<std::vector<int>, kXcd> deal_to_xcds(const std::vector<double> &work)
{
    std::vector<int> by_work(work.size());
    std::iota(by_work.begin(), by_work.end(), 0);
    std::stable_sort(by_work.begin(), by_work.end(), [&](int a, int b) { return work[a] > work[b]; });
    std::array<std::vector<int>, kXcd> of_xcd;
    double load[kXcd] = {0};
    for (int u : by_work) {
        int x = 0;
        for (int i = 1; i < kXcd; ++i)
            if (load[i] < load[x]) x = i;
        load[x] += work[u];
        of_xcd[x].push_back(u);
    }
    return of_xcd;
}

// Work list of the batched suffix launch.  One unit = (cluster, KV head): all rows of a unit read
// the same cached K/V.  Units are dealt, heaviest first, to the XCD with the least work so far;
// workgroup b runs on XCD b % 8, so slot-major interleaving keeps every tile of a unit on one
// XCD and that unit's K/V in one L2.
void build_tiles(sgc_plan *pl, int tile_rows)
{
    const sgc_ctx *ctx = pl->ctx;
    const int g = ctx->p.n_q_heads / ctx->p.n_kv_heads;
    struct Unit {
        int cluster, hk;
        int64_t rows;
    };
    std::vector<Unit> units;
    std::vector<double> work;
    for (int c = 0; c < pl->n_clusters; ++c) {
        const int64_t toks = pl->cl_tok_off[c + 1] - pl->cl_tok_off[c];
        if (toks == 0) continue;
        for (int hk = 0; hk < ctx->p.n_kv_heads; ++hk) {
            const int64_t rows = toks * g;
            const int64_t nt = (rows + tile_rows - 1) / tile_rows;
            units.push_back({c, hk, rows});
            work.push_back((double)nt * (pl->cl_prefix_len[c] + 64.0));
        }
    }
    struct Light {      // a tile before its record is written: unit and first row
        int32_t unit, row0;
    };
    std::vector<std::vector<Light>> lists(kXcd);
    const auto of_xcd = deal_to_xcds(work);
    for (int x = 0; x < kXcd; ++x)
        for (int ui : of_xcd[x])
            for (int64_t r = 0; r < units[ui].rows; r += tile_rows) lists[x].push_back({ui, (int32_t)r});
    size_t slots = 0;
    for (auto &l : lists) slots = std::max(slots, l.size());
    pl->tiles.resize(slots * kXcd);
    pl->seeds.assign(slots * kXcd, TileSeed{});
    for (int x = 0; x < kXcd; ++x) {
        for (size_t k = 0; k < slots; ++k) {
            Tile &t = pl->tiles[k * kXcd + x];
            if (k >= lists[x].size()) {
                t.n_rows = 0;            // padding: the workgroup exits at once and reads nothing else
                t.cluster = 0;
                continue;
            }
            const Unit &u = units[lists[x][k].unit];
            t.cluster = u.cluster;
            t.hk = u.hk;
            t.row0 = lists[x][k].row0;
            t.n_rows = (int32_t)std::min<int64_t>(tile_rows, u.rows - t.row0);
            t.prefix_len = pl->cl_prefix_len[u.cluster];
            t.pt_off = 0;
            t.tok_base = pl->cl_tok_off[u.cluster];
            const int32_t first_tok = t.tok_base + t.row0 / g, last_tok = t.tok_base + (t.row0 + t.n_rows - 1) / g;
            t.sq_lo = pl->tok_sq[first_tok];
            t.sq_hi = pl->tok_sq[last_tok];
            t.last_qpos = pl->tok_qpos[last_tok];
            t.n_q = t.sq_hi - t.sq_lo + 1;
            t.pad = 0;
            for (int q = 0; q < kTileQueries; ++q) {
                const int32_t sq = t.sq_lo + q;
                if (sq <= t.sq_hi)
                    t.q[q] = {pl->sq_tok0[sq], pl->sq_src0[sq], pl->sq_len[sq], pl->sq_page0[sq]};
                else
                    t.q[q] = {INT32_MAX, 0, 0, 0};
            }
            pl->seeds[k * kXcd + x] = {t.cluster, t.hk, t.row0, t.n_rows, t.sq_lo, t.sq_hi, t.last_qpos, 0};
        }
    }
    pl->tile_rows = tile_rows;
}

// first: first page of the tile's key range inside the cluster's page list; n: pages of the range
void fill_first_pages(Tile &t, const std::vector<int32_t> &pages, int first = 0, int n = -1)
{
    if (n < 0) n = (int)pages.size() - first;
    for (int i = 0; i < 12; ++i) t.first_pages[i] = n > 0 ? pages[first + std::min(i, n - 1)] : 0;
}

// Page-table offsets of the clusters as cache_sync lays the flat table out; they move when clusters
// are allocated or released, so the tiles carry the cache generation they were filled for.
void fill_tile_pt_off(sgc_plan *pl, const sgc_cache *c)
{
    std::vector<int32_t> off(c->max_clusters, 0);
    int32_t n = 0;
    for (int i = 0; i < c->max_clusters; ++i) {
        off[i] = n;
        if (c->cl[i].allocated) n += (int32_t)c->cl[i].pages.size();
    }
    for (Tile &t : pl->tiles) {
        if (t.n_rows == 0) continue;
        t.pt_off = off[t.cluster];
        fill_first_pages(t, c->cl[t.cluster].pages);
    }
    for (size_t i = 0; i < pl->dtiles.size(); ++i) {      // a decode tile covers the key range that starts at dtile_key0
        Tile &t = pl->dtiles[i];
        if (t.n_rows == 0) continue;
        const int first = pl->dtile_key0[i] / kPageTokens;
        t.pt_off = off[t.cluster] + first;
        fill_first_pages(t, c->cl[t.cluster].pages, first, (t.prefix_len + kPageTokens - 1) / kPageTokens);
    }
    pl->tiles_generation = c->generation;
}

// Pages of the suffix page pool: every query gets room for its suffix plus decode_cap more tokens.
void layout_suffix_pages(sgc_plan *pl)
{
    pl->spage_sq.clear();
    int32_t page = 0;
    for (size_t sq = 0; sq < pl->sq_len.size(); ++sq) {
        pl->sq_page0[sq] = page;
        const int32_t np = (pl->sq_len[sq] + pl->decode_cap + kPageTokens - 1) / kPageTokens;
        pl->spage_sq.insert(pl->spage_sq.end(), np, (int32_t)sq);
        page += np;
    }
}

// Decode work list: one row group (the g heads of a KV head) per query, all queries of a (cluster, KV head)
// stacked so that one tile of rows shares the cluster's cached K/V.  Same XCD dealing as build_tiles.
void build_decode_tiles(sgc_plan *pl, int tile_rows)
{
    const sgc_ctx *ctx = pl->ctx;
    const int g = ctx->p.n_q_heads / ctx->p.n_kv_heads;
    struct Light {
        int32_t cluster, hk, row0, split;
    };
    struct Unit {
        int32_t cluster, hk;
    };
    std::vector<Unit> units;
    std::vector<double> work;
    int64_t row_tiles = 0;
    int max_steps = 0;
    for (int c = 0; c < pl->n_clusters; ++c) {
        const int64_t nq = pl->cl_sq_off[c + 1] - pl->cl_sq_off[c];
        if (nq == 0) continue;
        const int64_t nt = (nq * g + tile_rows - 1) / tile_rows;
        row_tiles += nt * ctx->p.n_kv_heads;
        max_steps = std::max(max_steps, (pl->cl_prefix_len[c] + 63) / 64);
        for (int hk = 0; hk < ctx->p.n_kv_heads; ++hk) {
            units.push_back({c, hk});
            work.push_back((double)nt * (pl->cl_prefix_len[c] + 64.0));
        }
    }
    // A step has few rows (one per query and head), so few row tiles: the cached keys of every row tile are split
    // into S ranges of whole 64-key steps, each range a tile of its own whose partial result the own-keys kernel
    // merges.  A tile's fixed work (record, Q, store) costs about as much as eight steps, so S stays small: at
    // most one tile per CU, at least eight steps per range (measured on 80 row tiles x 16 steps: S = 2, 3, 4, 6
    // -> 42, 44, 45, 49 us per decode step).
    int S = row_tiles > 0 ? (int)std::min<int64_t>(kDecodeMaxSplits, 256 / row_tiles) : 1;
    S = std::max(1, std::min(S, max_steps / 8));
    if (max_steps >= (1 << 24) / 64) S = 1;      // the position offset travels in 24 bits of the tile record
    pl->dec_splits = S;
    std::vector<std::vector<Light>> lists(kXcd);
    const auto of_xcd = deal_to_xcds(work);
    for (int x = 0; x < kXcd; ++x)
        for (int ui : of_xcd[x]) {
            const Unit &u = units[ui];
            const int64_t rows = (int64_t)(pl->cl_sq_off[u.cluster + 1] - pl->cl_sq_off[u.cluster]) * g;
            for (int64_t r = 0; r < rows; r += tile_rows)
                for (int sp = 0; sp < S; ++sp) lists[x].push_back({u.cluster, u.hk, (int32_t)r, sp});
        }
    size_t slots = 0;
    for (auto &l : lists) slots = std::max(slots, l.size());
    pl->dtiles.assign(slots * kXcd, Tile{});
    pl->dtile_key0.assign(slots * kXcd, 0);
    for (int x = 0; x < kXcd; ++x)
        for (size_t k = 0; k < lists[x].size(); ++k) {
            Tile &t = pl->dtiles[k * kXcd + x];
            const Light &lt = lists[x][k];
            const int64_t rows = (int64_t)(pl->cl_sq_off[lt.cluster + 1] - pl->cl_sq_off[lt.cluster]) * g;
            const int P = pl->cl_prefix_len[lt.cluster], steps = (P + 63) / 64;
            const int key0 = std::min(P, 64 * (int)((int64_t)steps * lt.split / S));
            const int key1 = std::min(P, 64 * (int)((int64_t)steps * (lt.split + 1) / S));
            t.cluster = lt.cluster;
            t.hk = lt.hk;
            t.row0 = lt.row0;
            t.n_rows = (int32_t)std::min<int64_t>(tile_rows, rows - lt.row0);
            t.prefix_len = key1 - key0;                   // the tile's own key count ...
            t.pad = (lt.split << 24) | (P - t.prefix_len);   // ... its split index, and what positions start beyond it
            t.tok_base = pl->cl_sq_off[lt.cluster];      // "token" = the query's one new token
            t.sq_hi = -1;
            t.n_q = kTileQueries + 1;                     // row bookkeeping from the table, not from inline records
            pl->dtile_key0[k * kXcd + x] = key0;
        }
    pl->dtok.resize(pl->sq_len.size());
    for (size_t sq = 0; sq < pl->sq_len.size(); ++sq) pl->dtok[sq] = {pl->sq_query[sq], pl->sq_len[sq], (int32_t)sq, 0};
}

void plan_free_device(sgc_plan *pl)
{
    dev_release(pl->ctx, pl->dec_scratch, pl->last_stream);
    pl->dec_scratch = sgc_dev_block{};
    dev_release(pl->ctx, pl->proj_kv, pl->last_stream);
    pl->proj_kv = sgc_dev_block{};
    pl->proj_state = 0;
    dev_release(pl->ctx, pl->row_dest_block, pl->last_stream);
    pl->row_dest_block = sgc_dev_block{};
    pl->d_row_dest = nullptr;
    dev_release(pl->ctx, pl->blob, pl->last_stream);
    dev_release(pl->ctx, pl->spool_block, pl->last_stream);
    pl->blob = sgc_dev_block{};
    pl->spool_block = sgc_dev_block{};
    pl->d_blob = nullptr;
    pl->d_spool = nullptr;
    pl->spool_bytes = 0;
    pl->uploaded = false;
    pl->expand_pending = false;
}

}  // namespace

extern "C" {

const char *sgc_version(void) { return "libsgc 0.1 (gfx950)"; }

const char *sgc_status_string(int status)
{
    switch (status) {
        case SGC_OK: return "SGC_OK";
        case SGC_EINVAL: return "SGC_EINVAL";
        case SGC_ENOMEM: return "SGC_ENOMEM";
        case SGC_ESHAPE: return "SGC_ESHAPE";
        case SGC_EUNSUPPORTED: return "SGC_EUNSUPPORTED";
        case SGC_EHIP: return "SGC_EHIP";
        case SGC_ESTATE: return "SGC_ESTATE";
        default: return "SGC_UNKNOWN";
    }
}

const char *sgc_last_error(const sgc_ctx *ctx) { return ctx ? ctx->err.c_str() : g_err_noctx.c_str(); }

int sgc_ctx_create(const sgc_attn_params *params, sgc_ctx **out)
{
    if (!out) return fail(nullptr, SGC_EINVAL, "out is NULL");
    *out = nullptr;
    int rc = check_params(params, nullptr);
    if (rc != SGC_OK) return rc;
    sgc_ctx *ctx = new (std::nothrow) sgc_ctx();
    if (!ctx) return fail(nullptr, SGC_ENOMEM, "host allocation failed");
    ctx->p = *params;
    ctx->scale = params->softmax_scale > 0.0f ? params->softmax_scale : 1.0f / sqrtf((float)params->head_dim);
    ctx->use_mfma = params->kernel == SGC_KERNEL_MFMA || params->kernel == SGC_KERNEL_MFMA_FP8 ||
                    (params->kernel == SGC_KERNEL_AUTO && mfma_covers(*params));
    ctx->fp8_first_product = params->kernel == SGC_KERNEL_MFMA_FP8;
    ctx->tile_rows = ctx->use_mfma ? mfma_tile_rows() : 0;
    *out = ctx;
    return SGC_OK;
}

int sgc_ctx_destroy(sgc_ctx *ctx)
{
    if (!ctx) return SGC_OK;
    if (ctx->d_rope) (void)hipFree(ctx->d_rope);
    for (auto &triple : ctx->ev)
        for (hipEvent_t e : triple)
            if (e) (void)hipEventDestroy(e);
    (void)hipDeviceSynchronize();
    for (const sgc_dev_block &b : ctx->dev_free) (void)hipFree(b.p);
    for (int i = 0; i < sgc_ctx::kStageSlots; ++i) {
        if (ctx->h_stage[i]) (void)hipHostFree(ctx->h_stage[i]);
        if (ctx->stage_ev[i]) (void)hipEventDestroy(ctx->stage_ev[i]);
    }
    delete ctx;
    return SGC_OK;
}

size_t sgc_cache_page_bytes(const sgc_attn_params *params)
{
    if (check_params(params, nullptr) != SGC_OK) return 0;
    return page_bytes_of(*params);
}

size_t sgc_cache_pool_bytes(const sgc_attn_params *params, int64_t total_pages)
{
    if (check_params(params, nullptr) != SGC_OK || total_pages < 0) return 0;
    return page_bytes_of(*params) * (size_t)params->n_layers * (size_t)total_pages;
}

int sgc_cache_create(sgc_ctx *ctx, void *dev_pool, size_t pool_bytes, int32_t max_clusters, sgc_cache **out)
{
    if (!ctx) return fail(nullptr, SGC_EINVAL, "ctx is NULL");
    if (!out) return fail(ctx, SGC_EINVAL, "out is NULL");
    *out = nullptr;
    if (!dev_pool) return fail(ctx, SGC_EINVAL, "dev_pool is NULL");
    if (reinterpret_cast<uintptr_t>(dev_pool) & 255u) return fail(ctx, SGC_EINVAL, "dev_pool must be 256-byte aligned");
    if (max_clusters <= 0 || max_clusters > (1 << 20)) return fail(ctx, SGC_EINVAL, "max_clusters %d out of range", max_clusters);
    const size_t pb = page_bytes_of(ctx->p);
    const int64_t total_pages = (int64_t)(pool_bytes / (pb * (size_t)ctx->p.n_layers));
    if (total_pages < 1) return fail(ctx, SGC_EINVAL, "pool of %zu bytes holds no page (%zu bytes x %d layers)", pool_bytes, pb, ctx->p.n_layers);
    if (total_pages > INT32_MAX) return fail(ctx, SGC_EINVAL, "pool too large: %lld pages", (long long)total_pages);
    sgc_cache *c = new (std::nothrow) sgc_cache();
    if (!c) return fail(ctx, SGC_ENOMEM, "host allocation failed");
    c->ctx = ctx;
    c->pool_bytes = pool_bytes;
    c->max_clusters = max_clusters;
    c->geom.pool = static_cast<char *>(dev_pool);
    c->geom.total_pages = total_pages;
    c->geom.n_kv_heads = ctx->p.n_kv_heads;
    c->geom.head_dim = ctx->p.head_dim;
    c->geom.kv_dtype = ctx->p.kv_dtype;
    c->geom.kv_bytes = dtype_bytes(ctx->p.kv_dtype);
    c->geom.head_part_bytes = (int64_t)kPageTokens * ctx->p.head_dim * c->geom.kv_bytes;
    c->geom.page_bytes = (int64_t)pb;
    c->geom.layer_bytes = total_pages * (int64_t)pb;
    c->cl.resize(max_clusters);
    c->free_list.resize(total_pages);
    for (int64_t i = 0; i < total_pages; ++i) c->free_list[i] = (int32_t)(total_pages - 1 - i);  // page 0 first
    *out = c;
    return SGC_OK;
}

int sgc_cache_destroy(sgc_cache *c)
{
    if (!c) return SGC_OK;
    if (c->d_tables) (void)hipFree(c->d_tables);
    if (c->d_scale) (void)hipFree(c->d_scale);
    delete c;
    return SGC_OK;
}

int sgc_cache_alloc_cluster(sgc_cache *c, int32_t cluster_id, int32_t prefix_len)
{
    if (!c) return fail(nullptr, SGC_EINVAL, "cache is NULL");
    sgc_ctx *ctx = c->ctx;
    if (cluster_id < 0 || cluster_id >= c->max_clusters)
        return fail(ctx, SGC_EINVAL, "cluster_id %d outside [0, %d)", cluster_id, c->max_clusters);
    if (prefix_len < 0) return fail(ctx, SGC_EINVAL, "prefix_len %d < 0", prefix_len);
    sgc_cluster_entry &e = c->cl[cluster_id];
    if (e.allocated) return fail(ctx, SGC_ESTATE, "cluster %d is already allocated", cluster_id);
    const int64_t need = ((int64_t)prefix_len + kPageTokens - 1) / kPageTokens;
    if (need > (int64_t)c->free_list.size())
        return fail(ctx, SGC_ENOMEM, "cluster %d needs %lld pages, %zu free", cluster_id, (long long)need, c->free_list.size());
    e.pages.clear();
    e.pages.reserve(need);
    for (int64_t i = 0; i < need; ++i) {
        e.pages.push_back(c->free_list.back());
        c->free_list.pop_back();
    }
    e.prefix_len = prefix_len;
    e.allocated = true;
    c->dirty = true;
    c->generation++;
    return SGC_OK;
}

int sgc_cache_free_cluster(sgc_cache *c, int32_t cluster_id)
{
    if (!c) return fail(nullptr, SGC_EINVAL, "cache is NULL");
    sgc_ctx *ctx = c->ctx;
    if (cluster_id < 0 || cluster_id >= c->max_clusters)
        return fail(ctx, SGC_EINVAL, "cluster_id %d outside [0, %d)", cluster_id, c->max_clusters);
    sgc_cluster_entry &e = c->cl[cluster_id];
    if (!e.allocated) return fail(ctx, SGC_ESTATE, "cluster %d is not allocated", cluster_id);
    for (auto it = e.pages.rbegin(); it != e.pages.rend(); ++it) c->free_list.push_back(*it);
    e.pages.clear();
    e.prefix_len = 0;
    e.allocated = false;
    c->dirty = true;
    c->generation++;
    return SGC_OK;
}

int64_t sgc_cache_total_pages(const sgc_cache *c) { return c ? c->geom.total_pages : SGC_EINVAL; }
int64_t sgc_cache_free_pages(const sgc_cache *c) { return c ? (int64_t)c->free_list.size() : SGC_EINVAL; }

int sgc_cache_cluster_pages(const sgc_cache *c, int32_t cluster_id, int32_t *out_pages, int32_t cap, int32_t *out_prefix_len)
{
    if (!c) return fail(nullptr, SGC_EINVAL, "cache is NULL");
    if (cluster_id < 0 || cluster_id >= c->max_clusters)
        return fail(c->ctx, SGC_EINVAL, "cluster_id %d outside [0, %d)", cluster_id, c->max_clusters);
    const sgc_cluster_entry &e = c->cl[cluster_id];
    if (!e.allocated) return fail(c->ctx, SGC_ESTATE, "cluster %d is not allocated", cluster_id);
    if (out_prefix_len) *out_prefix_len = e.prefix_len;
    if (out_pages)
        for (int32_t i = 0; i < cap && i < (int32_t)e.pages.size(); ++i) out_pages[i] = e.pages[i];
    return (int)e.pages.size();
}

// ------------------------------------------------------------------------------------------------
int sgc_prefix_prefill_batched(sgc_ctx *ctx, sgc_cache *c, int32_t n, const int32_t *cluster_ids, int32_t layer,
                               const void *const *dev_q, const void *const *dev_k, const void *const *dev_v,
                               void *const *dev_o, float *const *dev_lse, void *hip_stream)
{
    if (!ctx) return fail(nullptr, SGC_EINVAL, "ctx is NULL");
    if (!c || c->ctx != ctx) return fail(ctx, SGC_EINVAL, "cache is NULL or belongs to another context");
    if (n < 0) return fail(ctx, SGC_EINVAL, "n %d < 0", n);
    if (n == 0) return SGC_OK;
    // dev_k and dev_v both NULL: the pages already hold this layer's keys (sgc_project_qkv_prefix*), attend only
    const bool attend_only = !dev_k && !dev_v;
    if (!cluster_ids || (!attend_only && (!dev_k || !dev_v))) return fail(ctx, SGC_EINVAL, "cluster_ids / dev_k / dev_v is NULL");
    if (attend_only && !dev_q) return fail(ctx, SGC_EINVAL, "neither keys to store nor queries to attend with");
    if ((dev_q == nullptr) != (dev_o == nullptr)) return fail(ctx, SGC_EINVAL, "dev_q and dev_o must both be given or both be NULL");
    if (dev_lse && !dev_o) return fail(ctx, SGC_EINVAL, "dev_lse given without dev_q/dev_o");
    const int Hkv = ctx->p.n_kv_heads, g = ctx->p.n_q_heads / Hkv;
    int rc;
    std::vector<char> seen(c->max_clusters, 0);
    int max_len = 0;
    for (int32_t i = 0; i < n; ++i) {
        if ((rc = check_cluster(ctx, c, cluster_ids[i], layer)) != SGC_OK) return rc;
        if (seen[cluster_ids[i]]) return fail(ctx, SGC_EINVAL, "cluster %d is named twice", cluster_ids[i]);
        seen[cluster_ids[i]] = 1;
        const int32_t P = c->cl[cluster_ids[i]].prefix_len;
        max_len = std::max(max_len, P);
        if (P == 0) continue;
        const void *q = dev_q ? dev_q[i] : nullptr;
        void *o = dev_o ? dev_o[i] : nullptr;
        const float *lse = dev_lse ? dev_lse[i] : nullptr;
        if (!attend_only && (!dev_k[i] || !dev_v[i])) return fail(ctx, SGC_EINVAL, "dev_k / dev_v of cluster %d is NULL", cluster_ids[i]);
        if ((q == nullptr) != (o == nullptr))
            return fail(ctx, SGC_EINVAL, "dev_q and dev_o of cluster %d must both be given or both be NULL", cluster_ids[i]);
        if (lse && !o) return fail(ctx, SGC_EINVAL, "dev_lse of cluster %d given without dev_q/dev_o", cluster_ids[i]);
        if ((!attend_only && (!aligned16(dev_k[i]) || !aligned16(dev_v[i]))) || !aligned16(q) || !aligned16(o) || !aligned16(lse))
            return fail(ctx, SGC_EINVAL, "device pointers must be 16-byte aligned");
    }
    if (max_len == 0) return SGC_OK;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    if ((rc = ensure_rope(ctx, max_len, s)) != SGC_OK) return rc;
    if ((rc = cache_tables_ensure(c)) != SGC_OK) return rc;      // (the tables themselves travel with this call's own copy)

    // jobs, the job of every page, and (MFMA attention) the tile list, in one device block
    std::vector<int32_t> pt_off(c->max_clusters, 0);
    for (int i = 0, acc = 0; i < c->max_clusters; ++i) {
        pt_off[i] = acc;
        if (c->cl[i].allocated) acc += (int32_t)c->cl[i].pages.size();
    }
    std::vector<PrefixJob> jobs;
    std::vector<int32_t> page_job;
    jobs.reserve(n);
    {
        size_t listed = 0;
        for (int32_t i = 0; i < n; ++i) listed += c->cl[cluster_ids[i]].pages.size();
        page_job.reserve(listed);
    }
    bool any_q = false;
    for (int32_t i = 0; i < n; ++i) {
        const int32_t id = cluster_ids[i], P = c->cl[id].prefix_len;
        if (P == 0) continue;
        PrefixJob j{};
        j.q = dev_q ? dev_q[i] : nullptr;
        j.k = attend_only ? nullptr : dev_k[i];
        j.v = attend_only ? nullptr : dev_v[i];
        j.o = dev_o ? dev_o[i] : nullptr;
        j.lse = dev_lse ? dev_lse[i] : nullptr;
        j.scale_kv = c->d_scale ? c->d_scale + ((size_t)id * ctx->p.n_layers + layer) * 2 * Hkv : nullptr;
        j.cluster = id;
        j.prefix_len = P;
        j.pt_off = pt_off[id];
        j.page0 = (int32_t)page_job.size();
        any_q = any_q || j.q != nullptr;
        page_job.insert(page_job.end(), c->cl[id].pages.size(), (int32_t)jobs.size());
        jobs.push_back(j);
    }
    // Tile list of the MFMA attention: units (job, KV head) are dealt, heaviest first, to the XCD with the
    // least work so far, each XCD's tiles longest first; workgroup b runs on XCD b % 8.
    struct Unit {
        int job, hk;
    };
    std::vector<Unit> units;
    std::vector<int> unit_tiles;
    std::array<std::vector<int>, kXcd> of_xcd;
    const int rows_per_tile = ctx->tile_rows;
    size_t slots = 0;
    if (any_q && ctx->use_mfma) {
        std::vector<double> work;
        units.reserve(jobs.size() * Hkv);
        unit_tiles.reserve(jobs.size() * Hkv);
        work.reserve(jobs.size() * Hkv);
        for (int ji = 0; ji < (int)jobs.size(); ++ji)
            if (jobs[ji].q)
                for (int hk = 0; hk < Hkv; ++hk) {
                    units.push_back({ji, hk});
                    unit_tiles.push_back((int)(((int64_t)jobs[ji].prefix_len * g + rows_per_tile - 1) / rows_per_tile));
                    work.push_back((double)jobs[ji].prefix_len * jobs[ji].prefix_len);
                }
        of_xcd = deal_to_xcds(work);
        for (int x = 0; x < kXcd; ++x) {
            size_t all = 0;
            for (int ui : of_xcd[x]) all += (size_t)unit_tiles[ui];
            slots = std::max(slots, all);
        }
    }
    // One block: [jobs][job of each page][tile seeds] from the host in one copy, then room for the tile records, which
    // are written on the device from the seeds, the jobs and the cache's page table.
    const size_t n_tiles = slots * kXcd;
    const size_t jobs_bytes = (jobs.size() * sizeof(PrefixJob) + 255) / 256 * 256;
    const size_t pj_bytes = (page_job.size() * sizeof(int32_t) + 255) / 256 * 256;
    const size_t seeds_bytes = (n_tiles * sizeof(TileSeed) + 255) / 256 * 256;
    const size_t copied = jobs_bytes + pj_bytes + seeds_bytes;
    const size_t total = copied + n_tiles * sizeof(Tile);
    sgc_dev_block blk;
    if ((rc = dev_acquire(ctx, total, s, &blk)) != SGC_OK) return rc;
    char *host = nullptr;
    int slot = 0;
    const size_t table_bytes = c->dirty ? cache_tables_bytes(c) : 0;      // the cache's page tables, when they are due
    if ((rc = stage_begin(ctx, copied + table_bytes, &host, &slot)) != SGC_OK) {
        dev_release(ctx, blk, s);
        return rc;
    }
    if (table_bytes) cache_tables_fill(c, reinterpret_cast<int32_t *>(host + copied));
    memcpy(host, jobs.data(), jobs.size() * sizeof(PrefixJob));
    memcpy(host + jobs_bytes, page_job.data(), page_job.size() * sizeof(int32_t));
    const PrefixJob *d_jobs = reinterpret_cast<const PrefixJob *>(blk.p);
    const int32_t *d_page_job = reinterpret_cast<const int32_t *>(blk.p + jobs_bytes);
    const TileSeed *d_seeds = reinterpret_cast<const TileSeed *>(blk.p + jobs_bytes + pj_bytes);
    const Tile *d_tiles = reinterpret_cast<const Tile *>(blk.p + copied);
    // a unit's tile t starts at row t * rows_per_tile; descending t, units in dealing order among equals; slot k of XCD x
    // is tile k * 8 + x of the launch (slots a short list does not fill stay padding tiles: n_rows = 0)
    TileSeed *hs = reinterpret_cast<TileSeed *>(host + jobs_bytes + pj_bytes);
    for (int x = 0; x < kXcd && n_tiles > 0; ++x) {
        int most = 0;
        for (int ui : of_xcd[x]) most = std::max(most, unit_tiles[ui]);
        size_t k = 0;
        for (int t = most - 1; t >= 0; --t)
            for (int ui : of_xcd[x]) {
                if (t >= unit_tiles[ui]) continue;
                const Unit &u = units[ui];
                const int32_t row0 = t * rows_per_tile;
                hs[k++ * kXcd + x] = TileSeed{u.job, u.hk, row0,
                                              (int32_t)std::min<int64_t>(rows_per_tile, (int64_t)jobs[u.job].prefix_len * g - row0),
                                              0, -1, 0, 0};
            }
        for (; k < slots; ++k) hs[k * kXcd + x] = TileSeed{};
    }
    // One copy for jobs, page jobs, seeds and page tables (with the event that says the staging buffer has been read); the tile records
    // are then written by workgroups appended to the ingest launch, or by a launch of their own when nothing is ingested.
    rc = stage_commit(ctx, slot, blk.p, copied, s, c->d_tables, copied, table_bytes);
    if (rc == SGC_OK) c->dirty = false;
    hipError_t e = hipSuccess;
    ExpandArgs x{};
    x.seeds = d_seeds;
    x.tiles = const_cast<Tile *>(d_tiles);
    x.n = (int32_t)n_tiles;
    x.jobs = d_jobs;
    x.page_table = c->d_page_table;
    const bool expand = n_tiles > 0;
    if (rc == SGC_OK && !attend_only)
        e = launch_prefix_ingest(c->geom, layer, c->d_page_table, d_jobs, (int)jobs.size(), d_page_job, (int)page_job.size(),
                                 ctx->p.io_dtype, ctx->p.rope_base > 0.0f ? ctx->d_rope : nullptr, expand ? &x : nullptr, s);
    else if (rc == SGC_OK && expand)
        e = launch_expand_tiles(x, s);
    if (rc == SGC_OK && e == hipSuccess && any_q) {
        AttnArgs a;
        fill_common_args(a, ctx, c, layer);
        a.mode = MODE_PREFIX;
        if (ctx->use_mfma) {
            a.jobs = d_jobs;
            a.tiles = d_tiles;
            a.n_tiles = (int32_t)n_tiles;
            e = launch_attn_mfma(a, s);
        } else {
            for (const PrefixJob &j : jobs) {      // the generic kernel works on one cluster per launch
                if (!j.q) continue;
                a.q = j.q;
                a.o = j.o;
                a.lse = j.lse;
                a.lse_stride = j.prefix_len;
                a.prefix_cluster = j.cluster;
                a.prefix_len = j.prefix_len;
                e = launch_attn_generic(a, (int64_t)j.prefix_len * ctx->p.n_q_heads, s);
                if (e != hipSuccess) break;
            }
        }
    }
    dev_release(ctx, blk, s);
    if (rc != SGC_OK) return rc;
    if (e != hipSuccess) return fail_hip(ctx, e, "prefix prefill launch");
    return SGC_OK;
}

int sgc_prefix_prefill(sgc_ctx *ctx, sgc_cache *c, int32_t cluster_id, int32_t layer, const void *dev_q,
                       const void *dev_k, const void *dev_v, void *dev_o, float *dev_lse, int32_t prefix_len,
                       void *hip_stream)
{
    if (!ctx) return fail(nullptr, SGC_EINVAL, "ctx is NULL");
    if (!c || c->ctx != ctx) return fail(ctx, SGC_EINVAL, "cache is NULL or belongs to another context");
    int rc = check_cluster(ctx, c, cluster_id, layer);
    if (rc != SGC_OK) return rc;
    if (prefix_len != c->cl[cluster_id].prefix_len)
        return fail(ctx, SGC_ESHAPE, "prefix_len %d differs from the %d the cluster was allocated with", prefix_len,
                    c->cl[cluster_id].prefix_len);
    if ((dev_q == nullptr) != (dev_o == nullptr)) return fail(ctx, SGC_EINVAL, "dev_q and dev_o must both be given or both be NULL");
    if (dev_lse && !dev_o) return fail(ctx, SGC_EINVAL, "dev_lse given without dev_q/dev_o");
    if (prefix_len == 0) return SGC_OK;
    if ((dev_k == nullptr) != (dev_v == nullptr)) return fail(ctx, SGC_EINVAL, "dev_k / dev_v is NULL");
    return sgc_prefix_prefill_batched(ctx, c, 1, &cluster_id, layer, dev_q ? &dev_q : nullptr, dev_k ? &dev_k : nullptr,
                                      dev_v ? &dev_v : nullptr,
                                      dev_o ? &dev_o : nullptr, dev_lse ? &dev_lse : nullptr, hip_stream);
}

// ------------------------------------------------------------------------------------------------
int sgc_assign_clusters(sgc_ctx *ctx, const sgc_cache *c, int32_t n_queries, const int32_t *labels,
                        const int32_t *suffix_len, int32_t n_clusters, int32_t *order, int32_t *cluster_off,
                        int32_t *cu_seqlens, sgc_plan **out_plan)
{
    if (!ctx) return fail(nullptr, SGC_EINVAL, "ctx is NULL");
    if (out_plan) *out_plan = nullptr;
    if (!c || c->ctx != ctx) return fail(ctx, SGC_EINVAL, "cache is NULL or belongs to another context");
    if (n_queries < 0) return fail(ctx, SGC_EINVAL, "n_queries %d < 0", n_queries);
    if (n_clusters <= 0 || n_clusters > c->max_clusters)
        return fail(ctx, SGC_EINVAL, "n_clusters %d outside [1, %d]", n_clusters, c->max_clusters);
    if (n_queries > 0 && (!labels || !suffix_len)) return fail(ctx, SGC_EINVAL, "labels / suffix_len is NULL");
    if (!order && n_queries > 0) return fail(ctx, SGC_EINVAL, "order is NULL");
    if (!cluster_off || !cu_seqlens) return fail(ctx, SGC_EINVAL, "cluster_off / cu_seqlens is NULL");

    // counting pass, with every check done before any output is written
    std::vector<int32_t> count(n_clusters, 0);
    int64_t total = 0;
    for (int32_t n = 0; n < n_queries; ++n) {
        const int32_t lab = labels[n];
        if (lab < 0 || lab >= n_clusters) return fail(ctx, SGC_EINVAL, "labels[%d] = %d outside [0, %d)", n, lab, n_clusters);
        if (suffix_len[n] < 0) return fail(ctx, SGC_EINVAL, "suffix_len[%d] = %d < 0", n, suffix_len[n]);
        if (!c->cl[lab].allocated) return fail(ctx, SGC_ESTATE, "query %d names cluster %d, which is not allocated", n, lab);
        count[lab]++;
        total += suffix_len[n];
    }
    if (total * (int64_t)(ctx->p.n_q_heads / ctx->p.n_kv_heads) > INT32_MAX || total > INT32_MAX / 2)
        return fail(ctx, SGC_EINVAL, "batch too large: %lld suffix tokens", (long long)total);

    cluster_off[0] = 0;
    for (int32_t k = 0; k < n_clusters; ++k) cluster_off[k + 1] = cluster_off[k] + count[k];
    std::vector<int32_t> cursor(cluster_off, cluster_off + n_clusters);
    for (int32_t n = 0; n < n_queries; ++n) order[cursor[labels[n]]++] = n;   // stable: ascending n inside a cluster
    cu_seqlens[0] = 0;
    for (int32_t n = 0; n < n_queries; ++n) cu_seqlens[n + 1] = cu_seqlens[n] + suffix_len[n];

    if (!out_plan) return SGC_OK;
    sgc_plan *pl = new (std::nothrow) sgc_plan();
    if (!pl) return fail(ctx, SGC_ENOMEM, "host allocation failed");
    pl->ctx = ctx;
    pl->cache = c;
    pl->n_queries = n_queries;
    pl->n_clusters = n_clusters;
    pl->total_tokens = total;
    pl->order.assign(order, order + n_queries);
    pl->cluster_off.assign(cluster_off, cluster_off + n_clusters + 1);
    pl->cl_prefix_len.resize(n_clusters);
    for (int32_t k = 0; k < n_clusters; ++k) pl->cl_prefix_len[k] = c->cl[k].allocated ? c->cl[k].prefix_len : 0;
    pl->cl_tok_off.assign(n_clusters + 1, 0);
    pl->tok_src.resize(total);
    pl->tok_qpos.resize(total);
    pl->tok_sq.resize(total);
    int32_t t = 0, maxpos = 0, spage = 0;
    pl->cl_sq_off.assign(n_clusters + 1, 0);
    for (int32_t k = 0; k < n_clusters; ++k) {
        pl->cl_tok_off[k] = t;
        pl->cl_sq_off[k] = (int32_t)pl->sq_len.size();
        for (int32_t i = cluster_off[k]; i < cluster_off[k + 1]; ++i) {
            const int32_t n = order[i];
            if (suffix_len[n] == 0) continue;             // queries without tokens follow behind the cluster's others
            const int32_t sq = (int32_t)pl->sq_len.size();
            pl->sq_query.push_back(n);
            pl->sq_src0.push_back(cu_seqlens[n]);
            pl->sq_len.push_back(suffix_len[n]);
            pl->sq_tok0.push_back(t);
            pl->sq_cluster.push_back(k);
            pl->sq_page0.push_back(spage);
            const int32_t np = (suffix_len[n] + kPageTokens - 1) / kPageTokens;
            for (int32_t pg = 0; pg < np; ++pg) pl->spage_sq.push_back(sq);
            spage += np;
            for (int32_t j = 0; j < suffix_len[n]; ++j, ++t) {
                pl->tok_src[t] = cu_seqlens[n] + j;
                pl->tok_qpos[t] = j;
                pl->tok_sq[t] = sq;
            }
            maxpos = std::max(maxpos, pl->cl_prefix_len[k] + suffix_len[n]);
        }
        // Queries without question tokens own no rows of the suffix prefill; they are numbered behind the cluster's
        // other queries, so that no row tile's query range ever contains one, and take part in decode steps only.
        for (int32_t i = cluster_off[k]; i < cluster_off[k + 1]; ++i) {
            const int32_t n = order[i];
            if (suffix_len[n] != 0) continue;
            pl->sq_query.push_back(n);
            pl->sq_src0.push_back(cu_seqlens[n]);
            pl->sq_len.push_back(0);
            pl->sq_tok0.push_back(t);
            pl->sq_cluster.push_back(k);
            pl->sq_page0.push_back(spage);
            maxpos = std::max(maxpos, pl->cl_prefix_len[k]);
        }
    }
    pl->cl_tok_off[n_clusters] = t;
    pl->cl_sq_off[n_clusters] = (int32_t)pl->sq_len.size();
    pl->max_position = maxpos;
    *out_plan = pl;
    return SGC_OK;
}

// What writes the plan's tile records on the device, from its seeds and the cache's current page tables (which the
// caller has brought up to date).
static ExpandArgs plan_expand_args(const sgc_plan *pl, const sgc_cache *c)
{
    ExpandArgs e{};
    e.seeds = pl->d_seeds;
    e.tiles = const_cast<Tile *>(pl->d_tiles);
    e.n = (int32_t)pl->tiles.size();
    e.jobs = nullptr;
    e.page_table = c->d_page_table;
    e.pt_off = c->d_pt_off;
    e.prefix_len = c->d_prefix_len;
    e.cl_tok_off = pl->d_cl_tok_off;
    e.sq_tok0 = pl->d_sq_tok0;
    e.sq_src0 = pl->d_sq_src0;
    e.sq_len = pl->d_sq_len;
    e.sq_page0 = pl->d_sq_page0;
    return e;
}

int sgc_plan_upload(sgc_plan *pl, void *hip_stream)
{
    if (!pl) return fail(nullptr, SGC_EINVAL, "plan is NULL");
    sgc_ctx *ctx = pl->ctx;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    const int want_rows = ctx->use_mfma ? ctx->tile_rows : 0;
    if (pl->uploaded && pl->tile_rows == want_rows) return SGC_OK;
    plan_free_device(pl);
    pl->tiles.clear();
    pl->seeds.clear();
    pl->tile_rows = 0;
    pl->dtiles.clear();
    pl->dtok.clear();
    if (want_rows > 0) {
        build_tiles(pl, want_rows);
        if (pl->decode_cap > 0) build_decode_tiles(pl, want_rows);
        fill_tile_pt_off(pl, pl->cache);
    }
    // The per-token records are only read by tiles that touch more queries than their own record describes.
    bool wide_tile = false;
    for (const Tile &t : pl->tiles) wide_tile = wide_tile || (t.n_rows > 0 && t.n_q > kTileQueries);
    pl->tok_info.clear();
    if (wide_tile) {
        pl->tok_info.resize(pl->tok_src.size());
        for (size_t i = 0; i < pl->tok_src.size(); ++i) pl->tok_info[i] = {pl->tok_src[i], pl->tok_qpos[i], pl->tok_sq[i], 0};
    }
    pl->row_dest.clear();      // made when a projection first asks for it

    // (src null: room on the device that no host data fills; such pieces come last and are not copied)
    struct Piece {
        const void *src;
        size_t bytes;
        const void **dst;
    };
    Piece pieces[] = {
        {pl->cl_tok_off.data(), pl->cl_tok_off.size() * 4, (const void **)&pl->d_cl_tok_off},
        // the three per-token arrays are only read by the generic attention kernel (the MFMA kernel has tok_info)
        {pl->tok_src.data(), want_rows > 0 ? 0 : pl->tok_src.size() * 4, (const void **)&pl->d_tok_src},
        {pl->tok_qpos.data(), want_rows > 0 ? 0 : pl->tok_qpos.size() * 4, (const void **)&pl->d_tok_qpos},
        {pl->tok_sq.data(), want_rows > 0 ? 0 : pl->tok_sq.size() * 4, (const void **)&pl->d_tok_sq},
        {pl->sq_src0.data(), pl->sq_src0.size() * 4, (const void **)&pl->d_sq_src0},
        {pl->sq_len.data(), pl->sq_len.size() * 4, (const void **)&pl->d_sq_len},
        {pl->sq_tok0.data(), pl->sq_tok0.size() * 4, (const void **)&pl->d_sq_tok0},
        {pl->sq_cluster.data(), pl->sq_cluster.size() * 4, (const void **)&pl->d_sq_cluster},
        {pl->sq_page0.data(), pl->sq_page0.size() * 4, (const void **)&pl->d_sq_page0},
        {pl->spage_sq.data(), pl->spage_sq.size() * 4, (const void **)&pl->d_spage_sq},
        {pl->seeds.data(), pl->seeds.size() * sizeof(TileSeed), (const void **)&pl->d_seeds},
        {pl->tok_info.data(), pl->tok_info.size() * sizeof(TokInfo), (const void **)&pl->d_tok_info},
        {pl->sq_query.data(), pl->sq_query.size() * 4, (const void **)&pl->d_sq_query},
        {pl->dtiles.data(), pl->dtiles.size() * sizeof(Tile), (const void **)&pl->d_dtiles},
        {pl->dtok.data(), pl->dtok.size() * sizeof(TokInfo), (const void **)&pl->d_dtok},
        // the tile records are written on the device, from the seeds
        {nullptr, pl->tiles.size() * sizeof(Tile), (const void **)&pl->d_tiles},
    };
    size_t total = 0, copied = 0;
    for (const Piece &p : pieces) {
        total += (p.bytes + 255) / 256 * 256 + 256;
        if (p.src || p.bytes == 0) copied = total;
    }
    int rc = dev_acquire(ctx, total, s, &pl->blob);
    if (rc != SGC_OK) return rc;
    pl->d_blob = pl->blob.p;
    pl->last_stream = s;
    char *host = nullptr;
    int slot = 0;
    if ((rc = stage_begin(ctx, copied, &host, &slot)) != SGC_OK) return rc;
    size_t off = 0;
    for (const Piece &p : pieces) {
        *p.dst = pl->d_blob + off;
        if (p.bytes && p.src) memcpy(host + off, p.src, p.bytes);
        off += (p.bytes + 255) / 256 * 256 + 256;
    }
    if ((rc = stage_commit(ctx, slot, pl->d_blob, copied, s)) != SGC_OK) return rc;
    pl->expand_pending = !pl->tiles.empty();      // the records are written with the next suffix launch's ingest
    if (want_rows > 0 && !pl->spage_sq.empty()) {
        // suffix page pool: bf16 pages of every query's rotated suffix K and transposed V
        // (decode: one pool per layer, since the pages have to outlive the layer's suffix launch; zeroed once,
        // so that pages no token has reached yet hold finite values)
        pl->spool_layer_bytes = pl->spage_sq.size() * (size_t)2 * ctx->p.n_kv_heads * kPageTokens * ctx->p.head_dim * 2;
        pl->spool_bytes = pl->spool_layer_bytes * (pl->decode_cap > 0 ? (size_t)ctx->p.n_layers : 1);
        if ((rc = dev_acquire(ctx, pl->spool_bytes, s, &pl->spool_block)) != SGC_OK) return rc;
        pl->d_spool = pl->spool_block.p;
        if (pl->decode_cap > 0) SGC_HIP(ctx, launch_fill_zero_bytes(pl->d_spool, pl->spool_bytes, s));
    }
    pl->uploaded = true;
    return SGC_OK;
}

int sgc_plan_get_info(const sgc_plan *pl, sgc_plan_info *out)
{
    if (!pl || !out) return fail(pl ? pl->ctx : nullptr, SGC_EINVAL, "plan / out is NULL");
    out->n_queries = pl->n_queries;
    out->n_clusters = pl->n_clusters;
    out->total_tokens = pl->total_tokens;
    out->max_position = pl->max_position;
    out->tile_rows = pl->tile_rows;
    out->n_tiles = (int32_t)pl->tiles.size();
    return SGC_OK;
}

int sgc_plan_destroy(sgc_plan *pl)
{
    if (!pl) return SGC_OK;
    plan_free_device(pl);
    delete pl;
    return SGC_OK;
}

// Clusters were allocated or released since the tiles were filled: refresh their page-table offsets and
// first page ids, on the host now and in the device copy with the next suffix launch (decode tiles: now).
static int refresh_tiles(sgc_plan *pl, const sgc_cache *c, hipStream_t s)
{
    sgc_ctx *ctx = pl->ctx;
    if (pl->tiles.empty() || pl->tiles_generation == c->generation) return SGC_OK;
    fill_tile_pt_off(pl, c);
    pl->expand_pending = true;
    for (int which = 1; which < 2; ++which) {
        const std::vector<Tile> &list = pl->dtiles;
        const Tile *dev = pl->d_dtiles;
        if (list.empty()) continue;
        const size_t bytes = list.size() * sizeof(Tile);
        char *host = nullptr;
        int slot = 0, rc;
        if ((rc = stage_begin(ctx, bytes, &host, &slot)) != SGC_OK) return rc;
        memcpy(host, list.data(), bytes);
        if ((rc = stage_commit(ctx, slot, const_cast<Tile *>(dev), bytes, s)) != SGC_OK) return rc;
    }
    return SGC_OK;
}

// ------------------------------------------------------------------------------------------------
int sgc_suffix_prefill_batched(sgc_ctx *ctx, const sgc_cache *cc, sgc_plan *pl, int32_t layer, const void *dev_q,
                               const void *dev_k, const void *dev_v, void *dev_o, float *dev_lse, void *hip_stream)
{
    if (!ctx) return fail(nullptr, SGC_EINVAL, "ctx is NULL");
    if (!cc || cc->ctx != ctx) return fail(ctx, SGC_EINVAL, "cache is NULL or belongs to another context");
    if (!pl || pl->ctx != ctx || pl->cache != cc) return fail(ctx, SGC_EINVAL, "plan is NULL or was made for another context/cache");
    if (layer < 0 || layer >= ctx->p.n_layers) return fail(ctx, SGC_EINVAL, "layer %d outside [0, %d)", layer, ctx->p.n_layers);
    sgc_cache *c = const_cast<sgc_cache *>(cc);   // device mirrors are refreshed lazily
    for (int32_t k = 0; k < pl->n_clusters; ++k) {
        if (pl->cluster_off[k + 1] == pl->cluster_off[k]) continue;
        if (!c->cl[k].allocated || c->cl[k].prefix_len != pl->cl_prefix_len[k])
            return fail(ctx, SGC_ESTATE, "cluster %d changed since the plan was made", k);
    }
    if (pl->total_tokens == 0) return SGC_OK;
    // dev_k and dev_v both NULL: take the keys sgc_project_qkv_suffix made for this layer
    const bool projected = !dev_k && !dev_v;
    if (projected) {
        if (pl->proj_state == 0 || pl->proj_layer != layer || !pl->uploaded)
            return fail(ctx, SGC_ESTATE, "no projected keys for layer %d: call sgc_project_qkv_suffix first", layer);
        if (pl->proj_state == 2) {
            dev_k = pl->proj_kv.p;
            dev_v = pl->proj_kv.p + (size_t)pl->total_tokens * ctx->p.n_kv_heads * ctx->p.head_dim * dtype_bytes(ctx->p.io_dtype);
        }
    }
    const bool skip_ingest = projected && pl->proj_state == 1;
    if (!dev_q || !dev_o || (!skip_ingest && (!dev_k || !dev_v))) return fail(ctx, SGC_EINVAL, "dev_q / dev_k / dev_v / dev_o is NULL");
    if (!aligned16(dev_q) || !aligned16(dev_k) || !aligned16(dev_v) || !aligned16(dev_o) || !aligned16(dev_lse))
        return fail(ctx, SGC_EINVAL, "device pointers must be 16-byte aligned");
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    int rc;
    if ((rc = ensure_rope(ctx, pl->max_position, s)) != SGC_OK) return rc;
    if ((rc = cache_sync(c, s)) != SGC_OK) return rc;
    if ((rc = sgc_plan_upload(pl, hip_stream)) != SGC_OK) return rc;
    if ((rc = refresh_tiles(pl, c, s)) != SGC_OK) return rc;
    pl->last_stream = s;

    AttnArgs a;
    fill_common_args(a, ctx, c, layer);
    a.q = dev_q;
    a.k = dev_k;
    a.v = dev_v;
    a.o = dev_o;
    a.lse = dev_lse;
    a.lse_stride = pl->total_tokens;
    a.mode = MODE_SUFFIX;
    a.tiles = pl->d_tiles;
    a.n_tiles = (int32_t)pl->tiles.size();
    a.cl_tok_off = pl->d_cl_tok_off;
    a.tok_src = pl->d_tok_src;
    a.tok_qpos = pl->d_tok_qpos;
    a.tok_sq = pl->d_tok_sq;
    a.tok_info = pl->d_tok_info;
    a.sq_src0 = pl->d_sq_src0;
    a.sq_len = pl->d_sq_len;
    a.sq_tok0 = pl->d_sq_tok0;
    a.sq_cluster = pl->d_sq_cluster;
    a.sq_page0 = pl->d_sq_page0;
    a.spool = pl->d_spool + (pl->decode_cap > 0 ? (size_t)layer * pl->spool_layer_bytes : 0);
    a.total_tokens = pl->total_tokens;
    hipEvent_t *tev = ctx->ev[ctx->timing_count % sgc_ctx::kTimingRing];
    const bool timed = ctx->timing && ctx->timing_launches++ % (uint64_t)ctx->timing_period == 0;
    if (timed) SGC_HIP(ctx, hipEventRecord(tev[0], s));
    // tile records that are due are written by workgroups appended to the ingest launch (they depend on nothing it writes)
    const ExpandArgs ex = plan_expand_args(pl, c);
    const bool expand = ctx->use_mfma && pl->expand_pending;
    if (ctx->use_mfma && !skip_ingest)
        SGC_HIP(ctx, launch_suffix_ingest(a, pl->d_spage_sq, (int)pl->spage_sq.size(), expand ? &ex : nullptr, s));
    else if (expand)
        SGC_HIP(ctx, launch_expand_tiles(ex, s));
    pl->expand_pending = false;
    if (timed) SGC_HIP(ctx, hipEventRecord(tev[1], s));
    if (ctx->use_mfma) {
        SGC_HIP(ctx, launch_attn_mfma(a, s));
    } else {
        SGC_HIP(ctx, launch_attn_generic(a, pl->total_tokens * ctx->p.n_q_heads, s));
    }
    if (timed) {
        SGC_HIP(ctx, hipEventRecord(tev[2], s));
        ++ctx->timing_count;
    }
    return SGC_OK;
}

// ------------------------------------------------------------------------------------------------
int sgc_plan_enable_decode(sgc_plan *pl, int32_t max_new_tokens)
{
    if (!pl) return fail(nullptr, SGC_EINVAL, "plan is NULL");
    sgc_ctx *ctx = pl->ctx;
    if (!ctx->use_mfma) return fail(ctx, SGC_EUNSUPPORTED, "decode needs the MFMA path (io bf16, head_dim 128)");
    if (max_new_tokens < 1 || max_new_tokens > 4096) return fail(ctx, SGC_EINVAL, "max_new_tokens %d outside [1, 4096]", max_new_tokens);
    for (int32_t len : pl->sq_len)
        if ((len + max_new_tokens + kPageTokens - 1) / kPageTokens * kPageTokens > kDecodeMaxKeys)
            return fail(ctx, SGC_EINVAL, "suffix %d + %d new tokens exceeds %d own keys per query", len, max_new_tokens, kDecodeMaxKeys);
    if (pl->decode_cap == max_new_tokens) return SGC_OK;
    plan_free_device(pl);          // page numbering changes: the device copy is rebuilt at the next upload
    pl->decode_cap = max_new_tokens;
    layout_suffix_pages(pl);
    return SGC_OK;
}

// ---- device scratch for callers that cannot allocate ------------------------------------------------
// sgc_decode_step_batched_noalloc keeps the partial results of a step's cached-prompt part here instead of in a
// block from the context's pool.  Every GPU the library runs on holds its own copy of the array until the process
// ends; host code never uses the array's name as an address, only what hipGetSymbolAddress returned for the
// device that was current.
constexpr size_t kNoAllocScratchBytes = (size_t)32 << 20;
static __device__ __align__(256) unsigned char g_noalloc_scratch[kNoAllocScratchBytes];
constexpr int kMaxDevices = 64;
static char *g_noalloc_scratch_ptr[kMaxDevices] = {};

// The array's address on the current device (looked up once per device).
static int noalloc_scratch(sgc_ctx *ctx, char **out)
{
    int dev = -1;
    SGC_HIP(ctx, hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return fail(ctx, SGC_EUNSUPPORTED, "device index %d outside [0, %d)", dev, kMaxDevices);
    if (!g_noalloc_scratch_ptr[dev]) {
        void *p = nullptr;
        SGC_HIP(ctx, hipGetSymbolAddress(&p, HIP_SYMBOL(g_noalloc_scratch)));
        if (!p) return fail(ctx, SGC_EHIP, "hipGetSymbolAddress returned a null address for the scratch array");
        g_noalloc_scratch_ptr[dev] = static_cast<char *>(p);
    }
    *out = g_noalloc_scratch_ptr[dev];
    return SGC_OK;
}

// One decode step.  no_alloc: nothing may be allocated, so every table the step reads must already be on the device
// and current (SGC_ESTATE otherwise) and the partial results go to the static scratch array (SGC_ENOMEM if they do
// not fit).
static int decode_step(sgc_ctx *ctx, const sgc_cache *cc, sgc_plan *pl, int32_t layer, int32_t step,
                       const void *dev_q, const void *dev_k, const void *dev_v, void *dev_o, float *dev_lse,
                       void *hip_stream, bool no_alloc)
{
    if (!ctx) return fail(nullptr, SGC_EINVAL, "ctx is NULL");
    if (!cc || cc->ctx != ctx) return fail(ctx, SGC_EINVAL, "cache is NULL or belongs to another context");
    if (!pl || pl->ctx != ctx || pl->cache != cc) return fail(ctx, SGC_EINVAL, "plan is NULL or was made for another context/cache");
    if (layer < 0 || layer >= ctx->p.n_layers) return fail(ctx, SGC_EINVAL, "layer %d outside [0, %d)", layer, ctx->p.n_layers);
    if (pl->decode_cap <= 0) return fail(ctx, SGC_ESTATE, "decode was not enabled on this plan");
    if (step < 0 || step >= pl->decode_cap) return fail(ctx, SGC_EINVAL, "step %d outside [0, %d)", step, pl->decode_cap);
    if (!pl->uploaded) return fail(ctx, SGC_ESTATE, "no suffix prefill has run on this plan: its suffix pages are empty");
    sgc_cache *c = const_cast<sgc_cache *>(cc);
    for (int32_t k = 0; k < pl->n_clusters; ++k) {
        if (pl->cluster_off[k + 1] == pl->cluster_off[k]) continue;
        if (!c->cl[k].allocated || c->cl[k].prefix_len != pl->cl_prefix_len[k])
            return fail(ctx, SGC_ESTATE, "cluster %d changed since the plan was made", k);
    }
    const int32_t n_sq = (int32_t)pl->sq_len.size();
    if (n_sq == 0) return SGC_OK;
    if (!dev_q || !dev_k || !dev_v || !dev_o) return fail(ctx, SGC_EINVAL, "dev_q / dev_k / dev_v / dev_o is NULL");
    if (!aligned16(dev_q) || !aligned16(dev_k) || !aligned16(dev_v) || !aligned16(dev_o) || !aligned16(dev_lse))
        return fail(ctx, SGC_EINVAL, "device pointers must be 16-byte aligned");
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    int rc;
    if (no_alloc) {
        // growing the rotary table, the first copy of the page tables and a refreshed tile list all allocate
        if (ctx->p.rope_base > 0.0f && pl->max_position + pl->decode_cap > ctx->rope_len)
            return fail(ctx, SGC_ESTATE, "the rotary table ends at position %d, the step needs %d: set max_position, or run "
                        "sgc_decode_step_batched once", ctx->rope_len, pl->max_position + pl->decode_cap);
        if (!c->d_tables || c->dirty || (!pl->tiles.empty() && pl->tiles_generation != c->generation))
            return fail(ctx, SGC_ESTATE, "clusters were allocated or released since the plan's last launch: the device "
                        "tables are stale and refreshing them allocates");
    } else {
        if ((rc = ensure_rope(ctx, pl->max_position + pl->decode_cap, s)) != SGC_OK) return rc;
        if ((rc = cache_sync(c, s)) != SGC_OK) return rc;
        if ((rc = refresh_tiles(pl, c, s)) != SGC_OK) return rc;
    }
    pl->last_stream = s;
    // scratch for the cached-prefix part of the step, one set per key range: O [S][n_queries][Hq][d] bf16, then
    // LSE [S][Hq][n_queries]
    const int S = std::max(1, pl->dec_splits);
    const size_t o_bytes = ((size_t)pl->n_queries * ctx->p.n_q_heads * ctx->p.head_dim * 2 + 255) / 256 * 256;
    const size_t lse_bytes = ((size_t)ctx->p.n_q_heads * pl->n_queries * sizeof(float) + 255) / 256 * 256;
    char *scratch = nullptr;
    if (no_alloc) {
        if (S * (o_bytes + lse_bytes) > kNoAllocScratchBytes)
            return fail(ctx, SGC_ENOMEM, "the step's partial results need %zu bytes, the static scratch array holds %zu",
                        S * (o_bytes + lse_bytes), kNoAllocScratchBytes);
        if ((rc = noalloc_scratch(ctx, &scratch)) != SGC_OK) return rc;
    } else {
        if (!pl->dec_scratch.p && (rc = dev_acquire(ctx, S * (o_bytes + lse_bytes), s, &pl->dec_scratch)) != SGC_OK) return rc;
        scratch = pl->dec_scratch.p;
    }
    char *spool = pl->d_spool + (size_t)layer * pl->spool_layer_bytes;

    DecodeArgs d{};
    d.q = dev_q;
    d.k = dev_k;
    d.v = dev_v;
    d.o = dev_o;
    d.lse = dev_lse;
    d.o_cached = scratch;
    d.lse_cached = reinterpret_cast<const float *>(scratch + S * o_bytes);
    d.n_splits = S;
    d.split_o_elems = (int64_t)(o_bytes / 2);
    d.split_lse_elems = (int64_t)(lse_bytes / sizeof(float));
    d.spool = spool;
    d.sq_query = pl->d_sq_query;
    d.sq_len = pl->d_sq_len;
    d.sq_page0 = pl->d_sq_page0;
    d.sq_cluster = pl->d_sq_cluster;
    d.cl_prefix_len = c->d_prefix_len;
    d.rope = (ctx->p.rope_base > 0.0f) ? ctx->d_rope : nullptr;
    d.n_sq = n_sq;
    d.n_queries = pl->n_queries;
    d.step = step;
    d.n_q_heads = ctx->p.n_q_heads;
    d.n_kv_heads = ctx->p.n_kv_heads;
    int32_t longest = 0;
    for (int32_t len : pl->sq_len) longest = std::max(longest, len);
    d.key_cap = (longest + pl->decode_cap + kPageTokens - 1) / kPageTokens * kPageTokens;
    d.scale_log2e = ctx->scale * 1.4426950408889634f;
    d.use_mfma = ctx->use_mfma ? 1 : 0;

    AttnArgs a;
    fill_common_args(a, ctx, c, layer);
    a.q = dev_q;
    a.o = scratch;
    a.lse = reinterpret_cast<float *>(scratch + S * o_bytes);
    a.split_o_bytes = (int64_t)o_bytes;
    a.split_lse_elems = (int64_t)(lse_bytes / sizeof(float));
    a.lse_stride = pl->n_queries;
    a.mode = MODE_SUFFIX;
    a.tiles = pl->d_dtiles;
    a.n_tiles = (int32_t)pl->dtiles.size();
    a.tok_info = pl->d_dtok;
    a.sq_len = pl->d_sq_len;
    a.sq_page0 = pl->d_sq_page0;
    a.spool = spool;
    a.pos_shift = step;
    a.skip_self = 1;
    a.k = dev_k;                 // the step's new tokens: appended by the blocks behind the tiles
    a.v = dev_v;
    a.sq_cluster = pl->d_sq_cluster;
    a.sq_query = pl->d_sq_query;
    a.n_append = n_sq;
    SGC_HIP(ctx, launch_attn_mfma(a, s));
    SGC_HIP(ctx, launch_decode_own_keys(d, s));
    return SGC_OK;
}

int sgc_decode_step_batched(sgc_ctx *ctx, const sgc_cache *cc, sgc_plan *pl, int32_t layer, int32_t step,
                            const void *dev_q, const void *dev_k, const void *dev_v, void *dev_o, float *dev_lse,
                            void *hip_stream)
{
    return decode_step(ctx, cc, pl, layer, step, dev_q, dev_k, dev_v, dev_o, dev_lse, hip_stream, false);
}

int sgc_decode_step_batched_noalloc(sgc_ctx *ctx, const sgc_cache *cc, sgc_plan *pl, int32_t layer, int32_t step,
                                    const void *dev_q, const void *dev_k, const void *dev_v, void *dev_o, float *dev_lse,
                                    void *hip_stream)
{
    return decode_step(ctx, cc, pl, layer, step, dev_q, dev_k, dev_v, dev_o, dev_lse, hip_stream, true);
}

int sgc_timing_enable(sgc_ctx *ctx, int on)
{
    if (!ctx) return fail(nullptr, SGC_EINVAL, "ctx is NULL");
    if (on < 0) return fail(ctx, SGC_EINVAL, "timing period %d is negative", on);
    if (on) {
        for (auto &triple : ctx->ev)
            for (hipEvent_t &e : triple)
                if (!e) SGC_HIP(ctx, hipEventCreate(&e));
    }
    ctx->timing = on != 0;
    ctx->timing_period = on > 0 ? on : 1;
    ctx->timing_launches = 0;
    ctx->timing_count = 0;
    return SGC_OK;
}

int sgc_timing_get(sgc_ctx *ctx, int32_t back, float *ingest_ms, float *attention_ms)
{
    if (!ctx) return fail(nullptr, SGC_EINVAL, "ctx is NULL");
    if (back < 0 || back >= sgc_ctx::kTimingRing) return fail(ctx, SGC_EINVAL, "back %d outside [0, %d)", back, sgc_ctx::kTimingRing);
    if (!ctx->timing || ctx->timing_count <= (uint64_t)back) return fail(ctx, SGC_ESTATE, "no such timed launch has been recorded");
    hipEvent_t *tev = ctx->ev[(ctx->timing_count - 1 - back) % sgc_ctx::kTimingRing];
    SGC_HIP(ctx, hipEventSynchronize(tev[2]));
    float a = 0.f, b = 0.f;
    SGC_HIP(ctx, hipEventElapsedTime(&a, tev[0], tev[1]));
    SGC_HIP(ctx, hipEventElapsedTime(&b, tev[1], tev[2]));
    if (ingest_ms) *ingest_ms = a;
    if (attention_ms) *attention_ms = b;
    return SGC_OK;
}

int sgc_timing_last(sgc_ctx *ctx, float *ingest_ms, float *attention_ms) { return sgc_timing_get(ctx, 0, ingest_ms, attention_ms); }

// ------------------------------------------------------------------------------------------------
static int export_import(sgc_ctx *ctx, sgc_cache *c, int32_t cluster_id, int32_t layer, void *dev_k, void *dev_v,
                         float *host_k_scale, float *host_v_scale, void *hip_stream, bool is_export)
{
    if (!ctx) return fail(nullptr, SGC_EINVAL, "ctx is NULL");
    if (!c || c->ctx != ctx) return fail(ctx, SGC_EINVAL, "cache is NULL or belongs to another context");
    int rc = check_cluster(ctx, c, cluster_id, layer);
    if (rc != SGC_OK) return rc;
    const int32_t P = c->cl[cluster_id].prefix_len;
    const bool fp8 = ctx->p.kv_dtype == SGC_FP8_E4M3;
    if (fp8 && (!host_k_scale || !host_v_scale)) return fail(ctx, SGC_EINVAL, "fp8 cache: scale arrays are NULL");
    if (P > 0 && (!dev_k || !dev_v)) return fail(ctx, SGC_EINVAL, "dev_k / dev_v is NULL");
    if (!aligned16(dev_k) || !aligned16(dev_v)) return fail(ctx, SGC_EINVAL, "device pointers must be 16-byte aligned");
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    if ((rc = cache_sync(c, s)) != SGC_OK) return rc;
    int32_t pt_off = 0;
    for (int i = 0; i < cluster_id; ++i)
        if (c->cl[i].allocated) pt_off += (int32_t)c->cl[i].pages.size();
    const int Hkv = ctx->p.n_kv_heads;
    float *d_sc = c->d_scale ? c->d_scale + ((size_t)cluster_id * ctx->p.n_layers + layer) * 2 * Hkv : nullptr;
    if (is_export) {
        if (P > 0) SGC_HIP(ctx, launch_cache_export(c->geom, layer, c->d_page_table + pt_off, P, dev_k, dev_v, s));
        if (fp8) {
            SGC_HIP(ctx, hipMemcpyAsync(host_k_scale, d_sc, sizeof(float) * Hkv, hipMemcpyDeviceToHost, s));
            SGC_HIP(ctx, hipMemcpyAsync(host_v_scale, d_sc + Hkv, sizeof(float) * Hkv, hipMemcpyDeviceToHost, s));
        }
        SGC_HIP(ctx, hipStreamSynchronize(s));
    } else {
        if (P > 0) SGC_HIP(ctx, launch_cache_import(c->geom, layer, c->d_page_table + pt_off, P, dev_k, dev_v, s));
        if (fp8) {
            SGC_HIP(ctx, hipMemcpyAsync(d_sc, host_k_scale, sizeof(float) * Hkv, hipMemcpyHostToDevice, s));
            SGC_HIP(ctx, hipMemcpyAsync(d_sc + Hkv, host_v_scale, sizeof(float) * Hkv, hipMemcpyHostToDevice, s));
            SGC_HIP(ctx, hipStreamSynchronize(s));
        }
    }
    return SGC_OK;
}

int sgc_cache_export(sgc_ctx *ctx, const sgc_cache *cache, int32_t cluster_id, int32_t layer, void *dev_k, void *dev_v,
                     float *host_k_scale, float *host_v_scale, void *hip_stream)
{
    return export_import(ctx, const_cast<sgc_cache *>(cache), cluster_id, layer, dev_k, dev_v, host_k_scale, host_v_scale,
                         hip_stream, true);
}

int sgc_cache_import(sgc_ctx *ctx, sgc_cache *cache, int32_t cluster_id, int32_t layer, const void *dev_k, const void *dev_v,
                     const float *host_k_scale, const float *host_v_scale, void *hip_stream)
{
    return export_import(ctx, cache, cluster_id, layer, const_cast<void *>(dev_k), const_cast<void *>(dev_v),
                         const_cast<float *>(host_k_scale), const_cast<float *>(host_v_scale), hip_stream, false);
}

// ------------------------------------------------------------------------------------------------
// The linear maps around the attention (SubGCache Sec. 3.4: prompt and question tokens pass through the LLM's
// layers; each layer projects its hidden states to Q, K, V and the attention output back to the model width).
static bool gemm_covers(const sgc_ctx *ctx, int64_t K, int64_t N)
{
    return ctx->p.io_dtype == SGC_BF16 && K >= 64 && K % 64 == 0 && K <= (1 << 20) && N >= 128 && N % 128 == 0;
}

int sgc_project_qkv_prefix_batched(sgc_ctx *ctx, sgc_cache *c, int32_t n, const int32_t *cluster_ids, int32_t layer,
                                   const void *const *dev_x, const void *dev_w_qkv, int32_t d_model, void *const *dev_q,
                                   void *hip_stream)
{
    if (!ctx) return fail(nullptr, SGC_EINVAL, "ctx is NULL");
    if (!c || c->ctx != ctx) return fail(ctx, SGC_EINVAL, "cache is NULL or belongs to another context");
    if (n < 0) return fail(ctx, SGC_EINVAL, "n %d < 0", n);
    if (n == 0) return SGC_OK;
    if (!cluster_ids || !dev_x || !dev_w_qkv) return fail(ctx, SGC_EINVAL, "cluster_ids / dev_x / dev_w_qkv is NULL");
    if (d_model <= 0) return fail(ctx, SGC_EINVAL, "d_model %d <= 0", d_model);
    if (!aligned16(dev_w_qkv) || ((int64_t)d_model * dtype_bytes(ctx->p.io_dtype)) % 16 != 0)
        return fail(ctx, SGC_EINVAL, "dev_w_qkv and every row of x must be 16-byte aligned");
    const int Hq = ctx->p.n_q_heads, Hkv = ctx->p.n_kv_heads, d = ctx->p.head_dim;
    const int nq = Hq * d, nkv = Hkv * d, N = nq + 2 * nkv, K = d_model;
    const size_t eb = (size_t)dtype_bytes(ctx->p.io_dtype);
    int rc;
    std::vector<char> seen(c->max_clusters, 0);
    int max_len = 0;
    int64_t total_rows = 0;
    bool any_q = false;
    for (int32_t i = 0; i < n; ++i) {
        if ((rc = check_cluster(ctx, c, cluster_ids[i], layer)) != SGC_OK) return rc;
        if (seen[cluster_ids[i]]) return fail(ctx, SGC_EINVAL, "cluster %d is named twice", cluster_ids[i]);
        seen[cluster_ids[i]] = 1;
        const int32_t P = c->cl[cluster_ids[i]].prefix_len;
        if (P == 0) continue;
        max_len = std::max(max_len, P);
        total_rows += P;
        if (!dev_x[i]) return fail(ctx, SGC_EINVAL, "dev_x of cluster %d is NULL", cluster_ids[i]);
        void *q = dev_q ? dev_q[i] : nullptr;
        if (!aligned16(dev_x[i]) || !aligned16(q)) return fail(ctx, SGC_EINVAL, "device pointers must be 16-byte aligned");
        any_q = any_q || q != nullptr;
    }
    if (max_len == 0) return SGC_OK;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    if ((rc = ensure_rope(ctx, max_len, s)) != SGC_OK) return rc;
    if ((rc = cache_sync(c, s)) != SGC_OK) return rc;
    const bool fused = gemm_covers(ctx, K, N) && d == 128;
    const bool to_pages = fused && ctx->p.kv_dtype == SGC_BF16;

    // keys and values that cannot go straight into pages are staged as [rows][Hkv d] matrices, K then V per cluster
    sgc_dev_block stg{};
    if (!to_pages && (rc = dev_acquire(ctx, (size_t)total_rows * 2 * nkv * eb, s, &stg)) != SGC_OK) return rc;
    std::vector<int32_t> ids;
    std::vector<const void *> kptr, vptr;
    std::vector<int32_t> pt_off(c->max_clusters, 0);
    for (int i = 0, acc = 0; i < c->max_clusters; ++i) {
        pt_off[i] = acc;
        if (c->cl[i].allocated) acc += (int32_t)c->cl[i].pages.size();
    }
    hipError_t e = hipSuccess;
    if (fused) {
        std::vector<GemmRowTile> tiles;
        int64_t row_base = 0;
        for (int32_t i = 0; i < n; ++i) {
            const int32_t id = cluster_ids[i], P = c->cl[id].prefix_len;
            if (P == 0) continue;
            char *ks = stg.p ? stg.p + (size_t)row_base * 2 * nkv * eb : nullptr;
            char *vs = ks ? ks + (size_t)P * nkv * eb : nullptr;
            if (ks) {
                ids.push_back(id);
                kptr.push_back(ks);
                vptr.push_back(vs);
            }
            for (int32_t r = 0; r < P; r += 256) {
                GemmRowTile t{};
                t.a = static_cast<const char *>(dev_x[i]) + (size_t)r * K * eb;
                t.c = (dev_q && dev_q[i]) ? static_cast<char *>(dev_q[i]) + (size_t)r * nq * eb : nullptr;
                t.ck = ks ? ks + (size_t)r * nkv * eb : nullptr;
                t.cv = vs ? vs + (size_t)r * nkv * eb : nullptr;
                t.rows = std::min(256, P - r);
                t.pos0 = r;
                t.pt_off = pt_off[id];
                tiles.push_back(t);
            }
            row_base += P;
        }
        const size_t bytes = tiles.size() * sizeof(GemmRowTile);
        sgc_dev_block blk;
        if ((rc = dev_acquire(ctx, bytes, s, &blk)) != SGC_OK) {
            dev_release(ctx, stg, s);
            return rc;
        }
        char *host = nullptr;
        int slot = 0;
        if ((rc = stage_begin(ctx, bytes, &host, &slot)) == SGC_OK) {
            memcpy(host, tiles.data(), bytes);
            rc = stage_commit(ctx, slot, blk.p, bytes, s);
        }
        if (rc == SGC_OK) {
            GemmArgs g{};
            // without any q output only the K and V rows of the weight are multiplied
            g.w = any_q ? dev_w_qkv : static_cast<const char *>(dev_w_qkv) + (size_t)nq * K * eb;
            g.N = any_q ? N : 2 * nkv;
            g.K = K;
            g.tiles = reinterpret_cast<const GemmRowTile *>(blk.p);
            g.n_row_tiles = (int32_t)tiles.size();
            g.n_col_tiles = (g.N + 255) / 256;
            g.ldc = nq;
            g.n_plain = any_q ? nq : 0;
            g.kv_dest = to_pages ? 0 : 2;
            g.n_kv_heads = Hkv;
            g.kv_base = c->geom.pool + (int64_t)layer * c->geom.layer_bytes;
            g.page_bytes = c->geom.page_bytes;
            g.part_bytes = c->geom.head_part_bytes;
            g.page_table = c->d_page_table;
            g.rope = ctx->p.rope_base > 0.0f ? ctx->d_rope : nullptr;
            e = launch_proj_gemm(g, true, s);
        }
        dev_release(ctx, blk, s);
    } else {
        int64_t row_base = 0;
        for (int32_t i = 0; i < n && e == hipSuccess; ++i) {
            const int32_t id = cluster_ids[i], P = c->cl[id].prefix_len;
            if (P == 0) continue;
            char *ks = stg.p + (size_t)row_base * 2 * nkv * eb, *vs = ks + (size_t)P * nkv * eb;
            ids.push_back(id);
            kptr.push_back(ks);
            vptr.push_back(vs);
            e = launch_proj_generic(dev_x[i], dev_w_qkv, P, N, K, ctx->p.io_dtype, dev_q ? dev_q[i] : nullptr, nq, ks, nkv, vs, s);
            row_base += P;
        }
    }
    if (rc == SGC_OK && e == hipSuccess && !ids.empty())
        rc = sgc_prefix_prefill_batched(ctx, c, (int32_t)ids.size(), ids.data(), layer, nullptr, kptr.data(), vptr.data(), nullptr,
                                        nullptr, hip_stream);
    dev_release(ctx, stg, s);
    if (rc != SGC_OK) return rc;
    if (e != hipSuccess) return fail_hip(ctx, e, "QKV projection launch");
    return SGC_OK;
}

int sgc_project_qkv_prefix(sgc_ctx *ctx, sgc_cache *c, int32_t cluster_id, int32_t layer, const void *dev_x,
                           const void *dev_w_qkv, int32_t d_model, void *dev_q, int32_t prefix_len, void *hip_stream)
{
    if (!ctx) return fail(nullptr, SGC_EINVAL, "ctx is NULL");
    if (!c || c->ctx != ctx) return fail(ctx, SGC_EINVAL, "cache is NULL or belongs to another context");
    int rc = check_cluster(ctx, c, cluster_id, layer);
    if (rc != SGC_OK) return rc;
    if (prefix_len != c->cl[cluster_id].prefix_len)
        return fail(ctx, SGC_ESHAPE, "prefix_len %d differs from the %d the cluster was allocated with", prefix_len,
                    c->cl[cluster_id].prefix_len);
    return sgc_project_qkv_prefix_batched(ctx, c, 1, &cluster_id, layer, &dev_x, dev_w_qkv, d_model, dev_q ? &dev_q : nullptr,
                                          hip_stream);
}

int sgc_project_qkv_suffix(sgc_ctx *ctx, const sgc_cache *cc, sgc_plan *pl, int32_t layer, const void *dev_x,
                           const void *dev_w_qkv, int32_t d_model, void *dev_q, void *hip_stream)
{
    if (!ctx) return fail(nullptr, SGC_EINVAL, "ctx is NULL");
    if (!cc || cc->ctx != ctx) return fail(ctx, SGC_EINVAL, "cache is NULL or belongs to another context");
    if (!pl || pl->ctx != ctx || pl->cache != cc) return fail(ctx, SGC_EINVAL, "plan is NULL or was made for another context/cache");
    if (layer < 0 || layer >= ctx->p.n_layers) return fail(ctx, SGC_EINVAL, "layer %d outside [0, %d)", layer, ctx->p.n_layers);
    if (d_model <= 0) return fail(ctx, SGC_EINVAL, "d_model %d <= 0", d_model);
    for (int32_t k = 0; k < pl->n_clusters; ++k) {
        if (pl->cluster_off[k + 1] == pl->cluster_off[k]) continue;
        if (!cc->cl[k].allocated || cc->cl[k].prefix_len != pl->cl_prefix_len[k])
            return fail(ctx, SGC_ESTATE, "cluster %d changed since the plan was made", k);
    }
    if (pl->total_tokens == 0) return SGC_OK;
    if (!dev_x || !dev_w_qkv || !dev_q) return fail(ctx, SGC_EINVAL, "dev_x / dev_w_qkv / dev_q is NULL");
    const size_t eb = (size_t)dtype_bytes(ctx->p.io_dtype);
    if (!aligned16(dev_x) || !aligned16(dev_w_qkv) || !aligned16(dev_q) || ((int64_t)d_model * eb) % 16 != 0)
        return fail(ctx, SGC_EINVAL, "device pointers and every row of x must be 16-byte aligned");
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    int rc;
    if ((rc = ensure_rope(ctx, pl->max_position, s)) != SGC_OK) return rc;
    if ((rc = sgc_plan_upload(pl, hip_stream)) != SGC_OK) return rc;
    pl->last_stream = s;
    const int Hq = ctx->p.n_q_heads, Hkv = ctx->p.n_kv_heads, d = ctx->p.head_dim;
    const int nq = Hq * d, nkv = Hkv * d, N = nq + 2 * nkv, K = d_model;
    const int64_t T = pl->total_tokens;
    if (ctx->use_mfma && gemm_covers(ctx, K, N) && pl->d_spool) {
        char *spool = pl->d_spool + (pl->decode_cap > 0 ? (size_t)layer * pl->spool_layer_bytes : 0);
        const int64_t page_bytes = (int64_t)2 * Hkv * kPageTokens * d * 2;
        if (!pl->d_row_dest) {          // first projection on this plan: the per-row destinations go to the device
            // where the epilogue puts the key and value of each packed row: {16 * page + slot, position}
            pl->row_dest.resize(2 * pl->tok_src.size());
            for (size_t i = 0; i < pl->tok_src.size(); ++i) {
                const int32_t sq = pl->tok_sq[i], qpos = pl->tok_qpos[i];
                pl->row_dest[2 * (size_t)pl->tok_src[i]] = (pl->sq_page0[sq] + qpos / kPageTokens) * kPageTokens + qpos % kPageTokens;
                pl->row_dest[2 * (size_t)pl->tok_src[i] + 1] = pl->cl_prefix_len[pl->sq_cluster[sq]] + qpos;
            }
            const size_t bytes = pl->row_dest.size() * sizeof(int32_t);
            if ((rc = dev_acquire(ctx, bytes, s, &pl->row_dest_block)) != SGC_OK) return rc;
            char *host = nullptr;
            int slot = 0;
            if ((rc = stage_begin(ctx, bytes, &host, &slot)) != SGC_OK) return rc;
            memcpy(host, pl->row_dest.data(), bytes);
            if ((rc = stage_commit(ctx, slot, pl->row_dest_block.p, bytes, s)) != SGC_OK) return rc;
            pl->d_row_dest = reinterpret_cast<const int2 *>(pl->row_dest_block.p);
        }
        SGC_HIP(ctx, launch_zero_last_pages(spool, pl->d_sq_len, pl->d_sq_page0, (int)pl->sq_len.size(), page_bytes, s));
        GemmArgs g{};
        g.w = dev_w_qkv;
        g.N = N;
        g.K = K;
        g.a = dev_x;
        g.c = dev_q;
        g.M = T;
        g.n_row_tiles = (int32_t)((T + 255) / 256);
        g.n_col_tiles = (N + 255) / 256;
        g.ldc = nq;
        g.n_plain = nq;
        g.kv_dest = 1;
        g.n_kv_heads = Hkv;
        g.kv_base = spool;
        g.page_bytes = page_bytes;
        g.part_bytes = (int64_t)kPageTokens * d * 2;
        g.row_dest = pl->d_row_dest;
        g.rope = ctx->p.rope_base > 0.0f ? ctx->d_rope : nullptr;
        SGC_HIP(ctx, launch_proj_gemm(g, true, s));
        pl->proj_state = 1;
    } else {
        const size_t need = (size_t)T * 2 * nkv * eb;
        if (pl->proj_kv.bytes < need) {
            dev_release(ctx, pl->proj_kv, s);
            pl->proj_kv = sgc_dev_block{};
            if ((rc = dev_acquire(ctx, need, s, &pl->proj_kv)) != SGC_OK) return rc;
        }
        SGC_HIP(ctx, launch_proj_generic(dev_x, dev_w_qkv, T, N, K, ctx->p.io_dtype, dev_q, nq, pl->proj_kv.p, nkv,
                                         pl->proj_kv.p + (size_t)T * nkv * eb, s));
        pl->proj_state = 2;
    }
    pl->proj_layer = layer;
    return SGC_OK;
}

int sgc_project_out(sgc_ctx *ctx, const void *dev_o, const void *dev_w_o, int32_t d_model, int64_t n_tokens, void *dev_y,
                    void *hip_stream)
{
    if (!ctx) return fail(nullptr, SGC_EINVAL, "ctx is NULL");
    if (n_tokens < 0) return fail(ctx, SGC_EINVAL, "n_tokens %lld < 0", (long long)n_tokens);
    if (d_model <= 0) return fail(ctx, SGC_EINVAL, "d_model %d <= 0", d_model);
    if (n_tokens == 0) return SGC_OK;
    if (!dev_o || !dev_w_o || !dev_y) return fail(ctx, SGC_EINVAL, "dev_o / dev_w_o / dev_y is NULL");
    const size_t eb = (size_t)dtype_bytes(ctx->p.io_dtype);
    const int K = ctx->p.n_q_heads * ctx->p.head_dim, N = d_model;
    if (!aligned16(dev_o) || !aligned16(dev_w_o) || !aligned16(dev_y) || ((int64_t)N * eb) % 16 != 0)
        return fail(ctx, SGC_EINVAL, "device pointers and every row of y must be 16-byte aligned");
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    if (gemm_covers(ctx, K, N)) {
        GemmArgs g{};
        g.w = dev_w_o;
        g.N = N;
        g.K = K;
        g.a = dev_o;
        g.c = dev_y;
        g.M = n_tokens;
        g.n_row_tiles = (int32_t)((n_tokens + 255) / 256);
        g.n_col_tiles = (N + 255) / 256;
        g.ldc = N;
        g.n_plain = N;
        SGC_HIP(ctx, launch_proj_gemm(g, false, s));
    } else {
        SGC_HIP(ctx, launch_proj_generic(dev_o, dev_w_o, n_tokens, N, K, ctx->p.io_dtype, dev_y, N, nullptr, 0, nullptr, s));
    }
    return SGC_OK;
}

}  // extern "C"
