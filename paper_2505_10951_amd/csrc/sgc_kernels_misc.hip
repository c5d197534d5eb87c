// Support kernels of libsgc (gfx950): rotary table, prefix K/V ingest into cache pages,
// canonical export/import of a cluster's cache, and the generic fp32-arithmetic attention kernel
// (one wavefront per output row) that serves shapes the MFMA kernel does not cover.
//
// SubGCache (arXiv 2505.10951) Sec. 3.4: the representative prompt's K/V are computed once per
// cluster and kept in GPU memory; each query's question tokens are appended to it.
#include <hip/hip_runtime.h>
#include <math.h>

#include <algorithm>

#include "sgc_internal.h"

namespace sgc {

namespace {

constexpr int kWave = 64;

// ---- element load/store helpers ------------------------------------------------------------
__device__ inline float bf16_to_f32(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }

__device__ inline uint16_t f32_to_bf16(float x)   // round to nearest even; NaN stays NaN
{
    uint32_t u = __float_as_uint(x);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((u >> 16) | 0x40);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

// OCP E4M3 (bias 7, largest finite 448, no infinities): nearest, ties to even, saturating.
__device__ inline uint8_t f32_to_e4m3(float x)
{
    const uint32_t u = __float_as_uint(x);
    const uint8_t sign = (uint8_t)((u >> 24) & 0x80u);
    const uint32_t au = u & 0x7FFFFFFFu;
    if (au > 0x7F800000u) return 0x7F;
    const float a = __uint_as_float(au);
    if (a >= 448.0f) return sign | 0x7E;
    if (a < 0.015625f) {                        // below 2^-6: fixed spacing 2^-9
        return sign | (uint8_t)__float2int_rn(a * 512.0f);
    }
    uint32_t r = au + 0x7FFFFu + ((au >> 20) & 1u);   // round 23 -> 3 mantissa bits
    r >>= 20;                                         // [exponent8 | mantissa3]
    uint32_t code = r - ((127u - 7u) << 3);
    if (code > 0x7Eu) code = 0x7Eu;
    return sign | (uint8_t)code;
}

__device__ inline float e4m3_to_f32(uint8_t c)
{
    const uint32_t e = (c >> 3) & 15u, m = c & 7u;
    float mag;
    if (e == 0)
        mag = (float)m * 0.001953125f;   // m * 2^-9
    else if (e == 15 && m == 7)
        mag = __uint_as_float(0x7FC00000u);
    else
        mag = __uint_as_float(((e + 120u) << 23) | (m << 20));
    return (c & 0x80) ? -mag : mag;
}

// 8 consecutive elements starting at element index `idx` (multiple of 8) of a typed array.
__device__ inline void load8(const void *base, int64_t idx, int dtype, float out[8])
{
    if (dtype == SGC_F32) {
        const float4 *p = reinterpret_cast<const float4 *>(static_cast<const float *>(base) + idx);
        const float4 a = p[0], b = p[1];
        out[0] = a.x; out[1] = a.y; out[2] = a.z; out[3] = a.w;
        out[4] = b.x; out[5] = b.y; out[6] = b.z; out[7] = b.w;
    } else if (dtype == SGC_BF16) {
        const uint4 a = *reinterpret_cast<const uint4 *>(static_cast<const uint16_t *>(base) + idx);
        const uint32_t w[4] = {a.x, a.y, a.z, a.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            out[2 * i] = __uint_as_float(w[i] << 16);
            out[2 * i + 1] = __uint_as_float(w[i] & 0xFFFF0000u);
        }
    } else if (dtype == kElemF16) {
        const uint4 a = *reinterpret_cast<const uint4 *>(static_cast<const uint16_t *>(base) + idx);
        const uint32_t w[4] = {a.x, a.y, a.z, a.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            out[2 * i] = f16_bits_to_f32((uint16_t)(w[i] & 0xFFFFu));
            out[2 * i + 1] = f16_bits_to_f32((uint16_t)(w[i] >> 16));
        }
    } else {
        const uint2 a = *reinterpret_cast<const uint2 *>(static_cast<const uint8_t *>(base) + idx);
        const uint32_t w[2] = {a.x, a.y};
#pragma unroll
        for (int i = 0; i < 8; ++i) out[i] = e4m3_to_f32((uint8_t)(w[i >> 2] >> (8 * (i & 3))));
    }
}

__device__ inline float load1(const void *base, int64_t idx, int dtype)
{
    if (dtype == SGC_F32) return static_cast<const float *>(base)[idx];
    if (dtype == SGC_BF16) return bf16_to_f32(static_cast<const uint16_t *>(base)[idx]);
    if (dtype == kElemF16) return f16_bits_to_f32(static_cast<const uint16_t *>(base)[idx]);
    return e4m3_to_f32(static_cast<const uint8_t *>(base)[idx]);
}

// Stores x into the cache element type; fp8 stores the code of x / scale.
__device__ inline void store1(void *base, int64_t idx, int dtype, float x, float scale)
{
    if (dtype == SGC_F32)
        static_cast<float *>(base)[idx] = x;
    else if (dtype == SGC_BF16)
        static_cast<uint16_t *>(base)[idx] = f32_to_bf16(x);
    else if (dtype == kElemF16)
        static_cast<uint16_t *>(base)[idx] = f32_to_f16_bits(x);
    else
        static_cast<uint8_t *>(base)[idx] = f32_to_e4m3(x / scale);
}

__device__ inline void store8(void *base, int64_t idx, int dtype, const float x[8], float scale)
{
    if (dtype == SGC_F32) {
        float4 *p = reinterpret_cast<float4 *>(static_cast<float *>(base) + idx);
        p[0] = make_float4(x[0], x[1], x[2], x[3]);
        p[1] = make_float4(x[4], x[5], x[6], x[7]);
    } else if (dtype == SGC_BF16) {
        uint32_t w[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) w[i] = (uint32_t)f32_to_bf16(x[2 * i]) | ((uint32_t)f32_to_bf16(x[2 * i + 1]) << 16);
        *reinterpret_cast<uint4 *>(static_cast<uint16_t *>(base) + idx) = make_uint4(w[0], w[1], w[2], w[3]);
    } else if (dtype == kElemF16) {
        *reinterpret_cast<uint4 *>(static_cast<uint16_t *>(base) + idx) =
            make_uint4(pack2_f16(x[0], x[1]), pack2_f16(x[2], x[3]), pack2_f16(x[4], x[5]), pack2_f16(x[6], x[7]));
    } else {
        uint32_t w[2] = {0, 0};
#pragma unroll
        for (int i = 0; i < 8; ++i) w[i >> 2] |= (uint32_t)f32_to_e4m3(x[i] / scale) << (8 * (i & 3));
        *reinterpret_cast<uint2 *>(static_cast<uint8_t *>(base) + idx) = make_uint2(w[0], w[1]);
    }
}

// Rotated pair of 8-channel chunks: x1 holds channels c0..c0+7, x2 channels c0+d/2.. of one head
// vector; tab points at the (cos, sin) entries of this position for channels c0..c0+7.
__device__ inline void rope8(float x1[8], float x2[8], const float2 *tab)
{
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const float2 cs = tab[i];
        const float a = x1[i], b = x2[i];
        x1[i] = a * cs.x - b * cs.y;
        x2[i] = b * cs.x + a * cs.y;
    }
}

// ---- rotary table ----------------------------------------------------------------------------
__global__ void rope_table_kernel(float2 *table, int n_pos, int half, double base, double inv_d)
{
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (int64_t)n_pos * half) return;
    const int pos = (int)(idx / half), t = (int)(idx % half);
    const double theta = pow(base, -2.0 * (double)t * inv_d);
    double s, c;
    sincos((double)pos * theta, &s, &c);
    table[idx] = make_float2((float)c, (float)s);
}

// ---- prefix ingest ---------------------------------------------------------------------------
// Linear copy of n bytes (a multiple of 16) from LDS to global memory, 16 bytes per thread and turn.
__device__ inline void copy_out_16(char *dst, const char *lds_src, int n)
{
    for (int off = threadIdx.x * 16; off < n; off += blockDim.x * 16)
        *reinterpret_cast<uint4 *>(dst + off) = *reinterpret_cast<const uint4 *>(lds_src + off);
}

// bf16 pages of 128-channel heads: V is a transpose (a page keeps, per channel, runs of 8 tokens), and element-sized
// scattered LDS writes of it collide in the banks.  The tokens' values go into a staging tile [16 tokens][128
// channels] instead, 16 bytes (8 channels) at a time, the sixteen chunks of token t's row at position
// vt_pos(chunk, t) so that the 16 lanes of a write cover all banks; the page's 16-byte units are then gathered from
// it column-wise (64 lanes read 64 neighbouring channels of one token) and stored straight to global memory.
__device__ inline int vt_pos(int chunk, int tok) { return chunk ^ ((tok & 1) << 3) ^ ((tok >> 1) & 7); }

__device__ inline void v_part_from_tile(char *vg, const uint16_t *vt)
{
    for (int u = threadIdx.x; u < 256; u += blockDim.x) {       // unit u = ((c / 32) * 2 + h) * 32 + c % 32, see v_page_index
        const int hh = (u >> 5) & 1, c = (u >> 6) * 32 + (u & 31);
        uint32_t w[4];
#pragma unroll
        for (int i2 = 0; i2 < 4; ++i2) {
            uint32_t e[2];
#pragma unroll
            for (int k = 0; k < 2; ++k) {
                const int i = 2 * i2 + k, t = 4 * hh + (i & 3) + 8 * (i >> 2);
                e[k] = vt[t * 128 + vt_pos(c >> 3, t) * 8 + (c & 7)];
            }
            w[i2] = e[0] | (e[1] << 16);
        }
        *reinterpret_cast<uint4 *>(vg + u * 16) = make_uint4(w[0], w[1], w[2], w[3]);
    }
}

// Pass 0 (fp8 only): per-head max |rotated K| and max |V| of every job into its scale slot
// amax[2][Hkv] via integer atomicMax on the bit patterns of non-negative floats.
__global__ void ingest_amax_kernel(const PrefixJob *jobs, const int32_t *page_job, int io_dtype, int Hkv, int d,
                                   const float2 *rope)
{
    const PrefixJob job = jobs[page_job[blockIdx.x]];
    const int pg = blockIdx.x - job.page0, hk = blockIdx.y;
    const int P = job.prefix_len;
    const int half = d / 2, pairs = d / 16;
    float mk = 0.f, mv = 0.f;
    for (int it = threadIdx.x; it < kPageTokens * pairs; it += blockDim.x) {
        const int tok = it / pairs, cc = it % pairs;
        const int j = pg * kPageTokens + tok;
        if (j >= P) continue;
        float x1[8], x2[8], y1[8], y2[8];
        const int64_t row = ((int64_t)j * Hkv + hk) * d;
        load8(job.k, row + cc * 8, io_dtype, x1);
        load8(job.k, row + half + cc * 8, io_dtype, x2);
        if (rope) rope8(x1, x2, rope + (int64_t)j * half + cc * 8);
        load8(job.v, row + cc * 8, io_dtype, y1);
        load8(job.v, row + half + cc * 8, io_dtype, y2);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            mk = fmaxf(mk, fmaxf(fabsf(x1[i]), fabsf(x2[i])));
            mv = fmaxf(mv, fmaxf(fabsf(y1[i]), fabsf(y2[i])));
        }
    }
    for (int o = 32; o > 0; o >>= 1) {
        mk = fmaxf(mk, __shfl_xor(mk, o));
        mv = fmaxf(mv, __shfl_xor(mv, o));
    }
    if ((threadIdx.x & 63) == 0) {
        atomicMax(reinterpret_cast<unsigned int *>(job.scale_kv + hk), __float_as_uint(mk));
        atomicMax(reinterpret_cast<unsigned int *>(job.scale_kv + Hkv + hk), __float_as_uint(mv));
    }
}

// One workgroup per job, 2 * Hkv values each: to_scale false clears the slot, true turns max|x| into the scale.
__global__ void scale_slot_kernel(const PrefixJob *jobs, int n, bool to_scale)
{
    float *p = jobs[blockIdx.x].scale_kv;
    for (int i = threadIdx.x; i < n; i += blockDim.x) p[i] = to_scale ? (p[i] > 0.f ? p[i] / 448.0f : 1.0f) : 0.f;
}

// ---- tile records -----------------------------------------------------------------------------
// The record the attention kernel reads for tile i, put together from the tile's seed and from the tables the device
// holds (the cluster's prompt length and pages, the plan's per-query records).
__device__ inline void expand_one_tile(const ExpandArgs &e, int i)
{
    const TileSeed sd = e.seeds[i];
    Tile t;
    t.cluster = sd.cluster;
    t.hk = sd.hk;
    t.row0 = sd.row0;
    t.n_rows = sd.n_rows;
    t.prefix_len = 0;
    t.pt_off = 0;
    t.tok_base = 0;
    t.sq_lo = sd.sq_lo;
    t.sq_hi = sd.sq_hi;
    t.last_qpos = sd.last_qpos;
    t.n_q = sd.sq_hi - sd.sq_lo + 1;
    t.pad = 0;
#pragma unroll
    for (int k = 0; k < 12; ++k) t.first_pages[k] = 0;
#pragma unroll
    for (int k = 0; k < kTileQueries; ++k) t.q[k] = {INT32_MAX, 0, 0, 0};
    if (sd.n_rows > 0) {
        if (e.jobs) {
            const PrefixJob &j = e.jobs[sd.cluster];
            t.cluster = j.cluster;
            t.prefix_len = j.prefix_len;
            t.pt_off = j.pt_off;
            t.tok_base = sd.cluster;          // prefix mode: the job index travels here
            t.sq_lo = 0;
            t.sq_hi = -1;
            t.last_qpos = 0;
            t.n_q = 0;
        } else {
            t.prefix_len = e.prefix_len[sd.cluster];
            t.pt_off = e.pt_off[sd.cluster];
            t.tok_base = e.cl_tok_off[sd.cluster];
#pragma unroll
            for (int k = 0; k < kTileQueries; ++k) {
                const int sq = sd.sq_lo + k;
                if (sq <= sd.sq_hi) t.q[k] = {e.sq_tok0[sq], e.sq_src0[sq], e.sq_len[sq], e.sq_page0[sq]};
            }
        }
        const int n_pages = (t.prefix_len + kPageTokens - 1) / kPageTokens;
        if (n_pages > 0) {
#pragma unroll
            for (int k = 0; k < 12; ++k) t.first_pages[k] = e.page_table[t.pt_off + min(k, n_pages - 1)];
        }
    } else {
        t.cluster = 0;
        t.n_q = 0;
    }
    e.tiles[i] = t;
}

// One thread per tile.
__global__ void expand_tiles_kernel(ExpandArgs e)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < e.n) expand_one_tile(e, i);
}

// The ingest kernels below run on (pages, KV heads) grids of 128 threads.  The tile records of the attention launch that
// follows depend on nothing the ingest writes, so they are written by workgroups appended to the same grid (columns
// blockIdx.x >= n_pages, 128 tiles per workgroup) instead of by a launch of their own between the two.
__device__ inline void expand_in_ingest_grid(const ExpandArgs &e, int n_pages)
{
    const int i = (((int)blockIdx.x - n_pages) * (int)gridDim.y + (int)blockIdx.y) * 128 + (int)threadIdx.x;
    if (i < e.n) expand_one_tile(e, i);
}
// grid columns to append for e.n tiles
inline unsigned expand_columns(int n_tiles, int n_kv_heads)
{
    const int groups = (n_tiles + 127) / 128;
    return (unsigned)((groups + n_kv_heads - 1) / n_kv_heads);
}

// One workgroup per (page, KV head): rotate K, convert, write K and V parts in page order.
// Tokens past the prefix end are written as zeros so that a whole page can always be read.
__global__ void ingest_write_kernel(PoolGeom g, int layer, const int32_t *page_table, const PrefixJob *jobs,
                                    const int32_t *page_job, int n_pages, int io_dtype, const float2 *rope, ExpandArgs ex)
{
    if ((int)blockIdx.x >= n_pages) {
        expand_in_ingest_grid(ex, n_pages);
        return;
    }
    const PrefixJob job = jobs[page_job[blockIdx.x]];
    const int pg = blockIdx.x - job.page0, hk = blockIdx.y;
    const int P = job.prefix_len;
    const void *k = job.k, *v = job.v;
    const int d = g.head_dim, Hkv = g.n_kv_heads, half = d / 2, pairs = d / 16;
    const int page = page_table[job.pt_off + pg];
    // The page images are put together in LDS (V is a transpose: element-sized scattered writes) and go out
    // as whole 16-byte rows.
    extern __shared__ __attribute__((aligned(16))) char page_img[];
    const int part_bytes = (int)g.head_part_bytes;
    char *kp = page_img, *vp = page_img + part_bytes;
    const bool via_tile = g.kv_dtype == SGC_BF16 && d == 128;     // V through the staging tile (see v_part_from_tile)
    float sc_k = 1.f, sc_v = 1.f;   // fp8: the per-head scales the codes are divided by
    if (g.kv_dtype == SGC_FP8_E4M3) {
        sc_k = job.scale_kv[hk];
        sc_v = job.scale_kv[Hkv + hk];
    }
    const bool v_as_given = via_tile && io_dtype == SGC_BF16;      // bf16 values into a bf16 cache: moved, not converted
    for (int it = threadIdx.x; it < kPageTokens * pairs; it += blockDim.x) {
        const int tok = it / pairs, cc = it % pairs;
        const int j = pg * kPageTokens + tok;
        float x1[8], x2[8], y1[8], y2[8];
        uint4 r1 = make_uint4(0, 0, 0, 0), r2 = r1;
        if (j < P) {
            const int64_t row = ((int64_t)j * Hkv + hk) * d;
            load8(k, row + cc * 8, io_dtype, x1);
            load8(k, row + half + cc * 8, io_dtype, x2);
            if (rope) rope8(x1, x2, rope + (int64_t)j * half + cc * 8);
            if (v_as_given) {
                r1 = *reinterpret_cast<const uint4 *>(static_cast<const uint16_t *>(v) + row + cc * 8);
                r2 = *reinterpret_cast<const uint4 *>(static_cast<const uint16_t *>(v) + row + half + cc * 8);
            } else {
                load8(v, row + cc * 8, io_dtype, y1);
                load8(v, row + half + cc * 8, io_dtype, y2);
            }
        } else {
#pragma unroll
            for (int i = 0; i < 8; ++i) x1[i] = x2[i] = y1[i] = y2[i] = 0.f;
        }
        store8(kp, k_page_index(tok, cc * 8), k_elem_type(g.kv_dtype), x1, sc_k);
        store8(kp, k_page_index(tok, half + cc * 8), k_elem_type(g.kv_dtype), x2, sc_k);
        if (v_as_given) {
            *reinterpret_cast<uint4 *>(reinterpret_cast<uint16_t *>(vp) + tok * 128 + vt_pos(cc, tok) * 8) = r1;
            *reinterpret_cast<uint4 *>(reinterpret_cast<uint16_t *>(vp) + tok * 128 + vt_pos(8 + cc, tok) * 8) = r2;
        } else if (via_tile) {
            store8(vp, tok * 128 + vt_pos(cc, tok) * 8, SGC_BF16, y1, 1.f);
            store8(vp, tok * 128 + vt_pos(8 + cc, tok) * 8, SGC_BF16, y2, 1.f);
        } else {
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                store1(vp, v_page_index(tok, cc * 8 + i), g.kv_dtype, y1[i], sc_v);
                store1(vp, v_page_index(tok, half + cc * 8 + i), g.kv_dtype, y2[i], sc_v);
            }
        }
    }
    __syncthreads();
    copy_out_16(g.k_part(layer, page, hk), kp, part_bytes);
    if (via_tile)
        v_part_from_tile(g.v_part(layer, page, hk), reinterpret_cast<const uint16_t *>(vp));
    else
        copy_out_16(g.v_part(layer, page, hk), vp, part_bytes);
}

// ---- suffix ingest ---------------------------------------------------------------------------
// Same page layout as the cache, 16-bit only (K binary16, V bf16), for the question tokens of every query of the batch
// (SubGCache Sec. 3.4: the question tokens are appended to the cached prompt, so suffix token j of a
// query whose cluster has P prefix tokens is rotated at position P + j).  One workgroup per
// (suffix page, KV head); tokens past the query's end are written as zeros.
__global__ void suffix_ingest_kernel(AttnArgs a, const int32_t *spage_sq, int n_spages, ExpandArgs ex)
{
    if ((int)blockIdx.x >= n_spages) {
        expand_in_ingest_grid(ex, n_spages);
        return;
    }
    const int page = blockIdx.x, hk = blockIdx.y;
    const int Hkv = a.n_kv_heads, d = a.head_dim, half = d / 2, pairs = d / 16;
    const int sq = spage_sq[page];
    const int S = a.sq_len[sq];
    const int64_t src0 = a.sq_src0[sq];
    const int P = a.cl_prefix_len[a.sq_cluster[sq]];
    const int tok0 = (page - a.sq_page0[sq]) * kPageTokens;
    if (tok0 >= S) return;      // a page kept free for decoded tokens: not this kernel's to write
    const int64_t part = (int64_t)kPageTokens * d * 2;
    char *kg = const_cast<char *>(a.spool) + (int64_t)page * 2 * Hkv * part + (int64_t)hk * part;
    char *vg = kg + (int64_t)Hkv * part;
    extern __shared__ __attribute__((aligned(16))) char page_img[];     // both images are built in LDS first
    char *kp = page_img, *vp = page_img + part;
    const bool via_tile = d == 128;          // V through the staging tile (see v_part_from_tile)
    const bool v_as_given = via_tile && a.io_dtype == SGC_BF16;      // bf16 values into bf16 pages: moved, not converted
    for (int it = threadIdx.x; it < kPageTokens * pairs; it += blockDim.x) {
        const int tok = it / pairs, cc = it % pairs;
        const int j = tok0 + tok;
        float x1[8], x2[8], y1[8], y2[8];
        uint4 r1 = make_uint4(0, 0, 0, 0), r2 = r1;
        if (j < S) {
            const int64_t row = ((src0 + j) * Hkv + hk) * d;
            load8(a.k, row + cc * 8, a.io_dtype, x1);
            load8(a.k, row + half + cc * 8, a.io_dtype, x2);
            if (a.rope) rope8(x1, x2, a.rope + (int64_t)(P + j) * half + cc * 8);
            if (v_as_given) {
                r1 = *reinterpret_cast<const uint4 *>(static_cast<const uint16_t *>(a.v) + row + cc * 8);
                r2 = *reinterpret_cast<const uint4 *>(static_cast<const uint16_t *>(a.v) + row + half + cc * 8);
            } else {
                load8(a.v, row + cc * 8, a.io_dtype, y1);
                load8(a.v, row + half + cc * 8, a.io_dtype, y2);
            }
        } else {
#pragma unroll
            for (int i = 0; i < 8; ++i) x1[i] = x2[i] = y1[i] = y2[i] = 0.f;
        }
        store8(kp, k_page_index(tok, cc * 8), kElemF16, x1, 1.f);
        store8(kp, k_page_index(tok, half + cc * 8), kElemF16, x2, 1.f);
        if (v_as_given) {
            *reinterpret_cast<uint4 *>(reinterpret_cast<uint16_t *>(vp) + tok * 128 + vt_pos(cc, tok) * 8) = r1;
            *reinterpret_cast<uint4 *>(reinterpret_cast<uint16_t *>(vp) + tok * 128 + vt_pos(8 + cc, tok) * 8) = r2;
        } else if (via_tile) {
            store8(vp, tok * 128 + vt_pos(cc, tok) * 8, SGC_BF16, y1, 1.f);
            store8(vp, tok * 128 + vt_pos(8 + cc, tok) * 8, SGC_BF16, y2, 1.f);
        } else {
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                store1(vp, v_page_index(tok, cc * 8 + i), SGC_BF16, y1[i], 1.f);
                store1(vp, v_page_index(tok, half + cc * 8 + i), SGC_BF16, y2[i], 1.f);
            }
        }
    }
    __syncthreads();
    copy_out_16(kg, kp, (int)part);
    if (via_tile)
        v_part_from_tile(vg, reinterpret_cast<const uint16_t *>(vp));
    else
        copy_out_16(vg, vp, (int)part);
}

// ---- decode ------------------------------------------------------------------------------------
// SubGCache App. A.2 caps generation at 32 tokens per query; every generated token attends over the
// cluster's cached prompt, the query's question tokens and the tokens generated before it (Sec. 3.4:
// all queries of a cluster reuse the same cache).  The cached-prompt part of a step runs in the MFMA
// kernel with the rows of all sibling queries stacked into one tile, so the prompt's K/V are read once
// per cluster instead of once per query (blocks behind that launch's tiles append the step's new tokens to the
// queries' suffix pages); the kernel here does what is per query.

// One wavefront per (sorted query, group of G query heads that share a KV head): scores of the new token
// against the query's own len + step + 1 keys (lane = key, each key read once for the G heads), softmax,
// weighted V sum (lane = channel pair), merged with the cached-prefix part by the log-sum-exp rule.
// Both products run on 16-bit pairs with fp32 accumulation (v_dot2_f32_f16 on the binary16 keys and the rotated
// query rounded to binary16; v_dot2_f32_bf16 on the bf16 values and the softmax weights rounded to bf16), the
// operands a matrix-core kernel would use; the row sum is taken over the rounded weights.  G divides the GQA
// group size.
typedef __attribute__((ext_vector_type(2))) __bf16 dec_bf16x2;

__device__ inline float dot8_f16(const uint4 &x, const uint4 &y, float acc)
{
    acc = __builtin_amdgcn_fdot2(__builtin_bit_cast(sgc_f16x2, x.x), __builtin_bit_cast(sgc_f16x2, y.x), acc, false);
    acc = __builtin_amdgcn_fdot2(__builtin_bit_cast(sgc_f16x2, x.y), __builtin_bit_cast(sgc_f16x2, y.y), acc, false);
    acc = __builtin_amdgcn_fdot2(__builtin_bit_cast(sgc_f16x2, x.z), __builtin_bit_cast(sgc_f16x2, y.z), acc, false);
    acc = __builtin_amdgcn_fdot2(__builtin_bit_cast(sgc_f16x2, x.w), __builtin_bit_cast(sgc_f16x2, y.w), acc, false);
    return acc;
}

__device__ inline float dot8_bf16(const uint4 &x, const uint4 &y, float acc)
{
    acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(dec_bf16x2, x.x), __builtin_bit_cast(dec_bf16x2, y.x), acc, false);
    acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(dec_bf16x2, x.y), __builtin_bit_cast(dec_bf16x2, y.y), acc, false);
    acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(dec_bf16x2, x.z), __builtin_bit_cast(dec_bf16x2, y.z), acc, false);
    acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(dec_bf16x2, x.w), __builtin_bit_cast(dec_bf16x2, y.w), acc, false);
    return acc;
}

template <int G>
__global__ void __launch_bounds__(64) decode_own_keys_kernel(DecodeArgs a)
{
    constexpr int d = 128, half = 64;
    // LDS: the G rotated query rows as binary16 [G][128]; G rows of key_cap scores (fp32); G rows of key_cap weights as
    // bf16 in the order the V pages hold their tokens (key_cap = the batch's largest key count, rounded up to a page;
    // sized at launch so that many wavefronts fit a CU)
    extern __shared__ __attribute__((aligned(16))) char dec_lds[];
    const int key_cap = a.key_cap;
    uint16_t *q_s = reinterpret_cast<uint16_t *>(dec_lds);                          // [G][d]
    float *p_base = reinterpret_cast<float *>(dec_lds + G * d * 2);                  // [G][key_cap]
    uint16_t *w_s = reinterpret_cast<uint16_t *>(dec_lds + G * d * 2 + G * key_cap * 4);   // [G][key_cap]
    const int lane = threadIdx.x;
    const int Hq = a.n_q_heads, Hkv = a.n_kv_heads, g = Hq / Hkv;
    const int units_per_query = Hq / G;
    const int sq = blockIdx.x / units_per_query;
    const int h0 = (blockIdx.x % units_per_query) * G;      // first head of the unit
    const int hk = h0 / g;
    const int n = a.sq_query[sq];
    const int n_keys = a.sq_len[sq] + a.step + 1;
    const int P = a.cl_prefix_len[a.sq_cluster[sq]];
    const int64_t io = ((int64_t)n * Hq + h0) * d;           // first of G consecutive rows
    for (int it = lane; it < G * (half / 8); it += kWave) {    // rotated query rows into LDS
        const int gi = it / (half / 8), cc = it % (half / 8);
        float x1[8], x2[8];
        load8(a.q, io + gi * d + cc * 8, SGC_BF16, x1);
        load8(a.q, io + gi * d + half + cc * 8, SGC_BF16, x2);
        if (a.rope) rope8(x1, x2, a.rope + (int64_t)(P + n_keys - 1) * half + cc * 8);
        uint32_t w1[4], w2[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            w1[i] = pack2_f16(x1[2 * i], x1[2 * i + 1]);
            w2[i] = pack2_f16(x2[2 * i], x2[2 * i + 1]);
        }
        *reinterpret_cast<uint4 *>(q_s + gi * d + cc * 8) = make_uint4(w1[0], w1[1], w1[2], w1[3]);
        *reinterpret_cast<uint4 *>(q_s + gi * d + half + cc * 8) = make_uint4(w2[0], w2[1], w2[2], w2[3]);
    }
    __syncthreads();
    const int64_t part = (int64_t)kPageTokens * d * 2;
    const char *pages = a.spool + (int64_t)a.sq_page0[sq] * 2 * Hkv * part + (int64_t)hk * part;
    const int64_t page_stride = 2 * Hkv * part;
    // scores (log2 units), lane = key
    float m[G], l[G];
#pragma unroll
    for (int gi = 0; gi < G; ++gi) m[gi] = -INFINITY;
    for (int j = lane; j < n_keys; j += kWave) {
        const char *kp = pages + (int64_t)(j / kPageTokens) * page_stride;
        const int tok = j % kPageTokens;
        uint4 raw[d / 8];                      // the key's 128 channels: all 16 loads in flight before any is used
#pragma unroll
        for (int cc = 0; cc < d / 8; ++cc)
            raw[cc] = *reinterpret_cast<const uint4 *>(kp + (int64_t)k_page_index(tok, cc * 8) * 2);
        float sc[G];
#pragma unroll
        for (int gi = 0; gi < G; ++gi) sc[gi] = 0.f;
#pragma unroll
        for (int cc = 0; cc < d / 8; ++cc) {
#pragma unroll
            for (int gi = 0; gi < G; ++gi)
                sc[gi] = dot8_f16(raw[cc], *reinterpret_cast<const uint4 *>(q_s + gi * d + cc * 8), sc[gi]);
        }
#pragma unroll
        for (int gi = 0; gi < G; ++gi) {
            sc[gi] *= a.scale_log2e;
            p_base[gi * key_cap + j] = sc[gi];
            m[gi] = fmaxf(m[gi], sc[gi]);
        }
    }
#pragma unroll
    for (int gi = 0; gi < G; ++gi) {
        for (int o = 32; o > 0; o >>= 1) m[gi] = fmaxf(m[gi], __shfl_xor(m[gi], o));
        l[gi] = 0.f;
    }
    // weights, rounded to bf16, stored where the V pages keep their tokens: a page holds, per channel, two runs of
    // 8 tokens; token t of a page is element (t & 3) | ((t >> 3) << 2) of run (t >> 2) & 1
    const int n_pages = (n_keys + kPageTokens - 1) / kPageTokens;
    for (int j = lane; j < n_pages * kPageTokens; j += kWave) {
        const int pg = j / kPageTokens, t = j % kPageTokens;
        const int slot = (pg * 2 + ((t >> 2) & 1)) * 8 + ((t & 3) | ((t >> 3) << 2));
#pragma unroll
        for (int gi = 0; gi < G; ++gi) {
            uint16_t wb = 0;                                    // the unused tail of the last page weighs nothing
            if (j < n_keys) {
                wb = f32_to_bf16(exp2f(p_base[gi * key_cap + j] - m[gi]));
                l[gi] += bf16_to_f32(wb);
            }
            w_s[gi * key_cap + slot] = wb;
        }
    }
#pragma unroll
    for (int gi = 0; gi < G; ++gi)
        for (int o = 32; o > 0; o >>= 1) l[gi] += __shfl_xor(l[gi], o);
    __syncthreads();
    // weighted V sum, lane = channels (lane, lane + 64)
    float acc[G][2];
#pragma unroll
    for (int gi = 0; gi < G; ++gi) acc[gi][0] = acc[gi][1] = 0.f;
    // (pages are taken four at a time: their sixteen 16-byte runs are all requested before the first is used)
    for (int pg0 = 0; pg0 < n_pages; pg0 += 4) {
        uint4 raw[4][4];
#pragma unroll
        for (int pi = 0; pi < 4; ++pi) {
            const int pg = min(pg0 + pi, n_pages - 1);           // a repeated page is skipped below
            const char *vp = pages + (int64_t)pg * page_stride + (int64_t)Hkv * part;
#pragma unroll
            for (int cI = 0; cI < 2; ++cI) {
                const int c = lane + cI * 64;
#pragma unroll
                for (int hh = 0; hh < 2; ++hh)
                    raw[pi][cI * 2 + hh] =
                        *reinterpret_cast<const uint4 *>(vp + (int64_t)((((c >> 5) * 2 + hh) * 32 + (c & 31)) * 8) * 2);
            }
        }
#pragma unroll
        for (int pi = 0; pi < 4; ++pi) {
            const int pg = pg0 + pi;
            if (pg >= n_pages) break;
#pragma unroll
            for (int hh = 0; hh < 2; ++hh) {
#pragma unroll
                for (int gi = 0; gi < G; ++gi) {
                    const uint4 wts = *reinterpret_cast<const uint4 *>(w_s + gi * key_cap + (pg * 2 + hh) * 8);
                    acc[gi][0] = dot8_bf16(raw[pi][hh], wts, acc[gi][0]);
                    acc[gi][1] = dot8_bf16(raw[pi][2 + hh], wts, acc[gi][1]);
                }
            }
        }
    }
    // merge with the cached-prefix part, which comes as n_splits partial results over key ranges (natural-log
    // LSE there, -inf for an empty range; log2 units here)
    uint16_t *og = static_cast<uint16_t *>(a.o);
    const uint16_t *oc = static_cast<const uint16_t *>(a.o_cached);
    const int S = a.n_splits;
#pragma unroll
    for (int gi = 0; gi < G; ++gi) {
        const int h = h0 + gi;
        const float lse_own = m[gi] + log2f(l[gi]);
        float lse_c[kDecodeMaxSplits];
        float M = lse_own;
#pragma unroll
        for (int sp = 0; sp < kDecodeMaxSplits; ++sp) {
            lse_c[sp] = -INFINITY;
            if (sp < S && a.lse_cached) lse_c[sp] = a.lse_cached[sp * a.split_lse_elems + (int64_t)h * a.n_queries + n] * 1.4426950408889634f;
            M = fmaxf(M, lse_c[sp]);
        }
        const float wo = exp2f(m[gi] - M);                       // weight of the unnormalised own sum
        float denom = exp2f(lse_own - M);
        float sum[2] = {wo * acc[gi][0], wo * acc[gi][1]};
#pragma unroll
        for (int sp = 0; sp < kDecodeMaxSplits; ++sp) {
            if (!(lse_c[sp] > -INFINITY)) continue;
            const float wc = exp2f(lse_c[sp] - M);
            denom += wc;
#pragma unroll
            for (int cI = 0; cI < 2; ++cI)
                sum[cI] += wc * bf16_to_f32(oc[sp * a.split_o_elems + io + gi * d + lane + cI * 64]);
        }
#pragma unroll
        for (int cI = 0; cI < 2; ++cI) og[io + gi * d + lane + cI * 64] = f32_to_bf16(sum[cI] / denom);
        if (a.lse && lane == 0) a.lse[(int64_t)h * a.n_queries + n] = (M + log2f(denom)) * 0.6931471805599453f;
    }
}

// The same step on the matrix cores, head_dim 128, groups of up to 16 query heads per KV head: one wavefront per (sorted
// query, KV head), no LDS.  v_mfma_f32_16x16x32: a page's 16 tokens are the 16 rows of the first product's left operand
// (32 channels per instruction are 1 KiB of the page, in lane order), the group's heads are its columns (the unused columns
// carry zeros), so lane (j, q) = (lane % 16, lane / 16) ends up with the scores of head j against tokens 4 q .. 4 q + 3 of
// every page.  Those four values of two neighbouring pages are, as they stand, the lane's eight contraction slots of the
// second product (keys x heads), whose left operand V^T takes, per lane, the 8-byte run of four tokens of channel
// 16 cb + lane % 16 from each of the two pages.  Keys come in chunks of 4 pages with an online softmax over the chunks.
typedef __attribute__((ext_vector_type(8))) _Float16 dec_f16x8;
typedef __attribute__((ext_vector_type(8))) __bf16 dec_bf16x8;
typedef __attribute__((ext_vector_type(4))) float dec_f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t dec_u32x4;

__global__ void __launch_bounds__(256, 3) decode_own_keys_mfma_kernel(DecodeArgs a)
{
    constexpr int d = 128, half = 64, CH = 4;        // CH: pages per chunk
    const int lane = threadIdx.x & 63;
    const int Hq = a.n_q_heads, Hkv = a.n_kv_heads, g = Hq / Hkv;
    const int unit = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (unit >= a.n_sq * Hkv) return;                 // (no barrier anywhere in this kernel)
    const int sq = unit / Hkv, hk = unit - sq * Hkv;
    const int j = lane & 15, q = lane >> 4;
    const int n = a.sq_query[sq];
    const int n_keys = a.sq_len[sq] + a.step + 1;
    const int P = a.cl_prefix_len[a.sq_cluster[sq]];
    const int n_pages = (n_keys + kPageTokens - 1) / kPageTokens;
    const bool live = j < g;                           // the lane's column is a head of the group
    const int h = hk * g + (live ? j : 0);
    const int64_t io = ((int64_t)n * Hq + h) * d;
    const int64_t part = (int64_t)kPageTokens * d * 2;
    const int64_t page_stride = 2 * Hkv * part;
    const char *pages = a.spool + (int64_t)a.sq_page0[sq] * page_stride + (int64_t)hk * part;

    // the query rows as right operands: chunk c8 = 4 cbk + q of 8 channels for cbk = 0..3; the rotation pairs chunk c8 with
    // chunk c8 + 8, both of which this lane holds (cbk and cbk + 2)
    dec_f16x8 qb[4];
    {
        float x1[2][8], x2[2][8];
#pragma unroll
        for (int cb = 0; cb < 2; ++cb) {
            const int c0 = 8 * (4 * cb + q);
            load8(a.q, io + c0, SGC_BF16, x1[cb]);
            load8(a.q, io + half + c0, SGC_BF16, x2[cb]);
            if (a.rope) rope8(x1[cb], x2[cb], a.rope + (int64_t)(P + n_keys - 1) * half + c0);
        }
        const float sc = live ? a.scale_log2e : 0.f;
#pragma unroll
        for (int cb = 0; cb < 2; ++cb)
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                qb[cb][e] = (_Float16)(x1[cb][e] * sc);
                qb[cb + 2][e] = (_Float16)(x2[cb][e] * sc);
            }
    }

    dec_f32x4 O[8];
#pragma unroll
    for (int cb = 0; cb < 8; ++cb) O[cb] = dec_f32x4{0.f, 0.f, 0.f, 0.f};
    float m_run = -INFINITY, l_run = 0.f;
    for (int pg0 = 0; pg0 < n_pages; pg0 += CH) {
        // scores of the chunk (log2 units): pages past the last are read as the last page again and masked
        dec_f32x4 S[CH];
        {
            dec_u32x4 ka[CH][4];
#pragma unroll
            for (int p = 0; p < CH; ++p) {
                const char *kp = pages + (int64_t)min(pg0 + p, n_pages - 1) * page_stride + lane * 16;
#pragma unroll
                for (int cbk = 0; cbk < 4; ++cbk) ka[p][cbk] = *reinterpret_cast<const dec_u32x4 *>(kp + cbk * 1024);
            }
#pragma unroll
            for (int p = 0; p < CH; ++p) {
                dec_f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int cbk = 0; cbk < 4; ++cbk)
                    acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(dec_f16x8, ka[p][cbk]), qb[cbk], acc, 0, 0, 0);
                S[p] = acc;
            }
        }
        float cmax = -INFINITY;
#pragma unroll
        for (int p = 0; p < CH; ++p)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int key = (pg0 + p) * kPageTokens + 4 * q + r;
                if (key >= n_keys) S[p][r] = -INFINITY;
                cmax = fmaxf(cmax, S[p][r]);
            }
        cmax = fmaxf(cmax, __shfl_xor(cmax, 16));
        cmax = fmaxf(cmax, __shfl_xor(cmax, 32));
        const float m_new = fmaxf(m_run, cmax);          // finite: every chunk holds at least one visible key
        const float alpha = exp2f(m_run - m_new);         // 0 on the first chunk
        m_run = m_new;
        l_run *= alpha;
#pragma unroll
        for (int cb = 0; cb < 8; ++cb)
#pragma unroll
            for (int r = 0; r < 4; ++r) O[cb][r] *= alpha;
        // weights, rounded to bf16 (the row sum adds the rounded values), two pages = one right operand
#pragma unroll
        for (int pp = 0; pp < CH / 2; ++pp) {
            if (pg0 + 2 * pp >= n_pages) break;            // (wave-uniform)
            uint16_t w[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                w[e] = f32_to_bf16(exp2f(S[2 * pp + (e >> 2)][e & 3] - m_new));
                l_run += bf16_to_f32(w[e]);
            }
            const dec_u32x4 wb = {(uint32_t)w[0] | ((uint32_t)w[1] << 16), (uint32_t)w[2] | ((uint32_t)w[3] << 16),
                                  (uint32_t)w[4] | ((uint32_t)w[5] << 16), (uint32_t)w[6] | ((uint32_t)w[7] << 16)};
            const char *va = pages + (int64_t)min(pg0 + 2 * pp, n_pages - 1) * page_stride + (int64_t)Hkv * part;
            const char *vb = pages + (int64_t)min(pg0 + 2 * pp + 1, n_pages - 1) * page_stride + (int64_t)Hkv * part;
            uint2 v0[8], v1[8];
#pragma unroll
            for (int cb = 0; cb < 8; ++cb) {
                // channel 16 cb + j: 32-channel group cb / 2, token block q & 1, channel (cb % 2) * 16 + j inside it, tokens
                // 4 q .. 4 q + 3 = the half 8 (q >> 1) of the 16-byte run
                const int off = ((((cb >> 1) * 2 + (q & 1)) * 32 + (cb & 1) * 16 + j) * 16) + 8 * (q >> 1);
                v0[cb] = *reinterpret_cast<const uint2 *>(va + off);
                v1[cb] = *reinterpret_cast<const uint2 *>(vb + off);
            }
#pragma unroll
            for (int cb = 0; cb < 8; ++cb) {
                const dec_u32x4 av = {v0[cb].x, v0[cb].y, v1[cb].x, v1[cb].y};
                O[cb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(dec_bf16x8, av), __builtin_bit_cast(dec_bf16x8, wb), O[cb], 0, 0, 0);
            }
        }
    }
    l_run += __shfl_xor(l_run, 16);
    l_run += __shfl_xor(l_run, 32);
    if (!live) return;
    // merge with the cached-prefix part (natural-log LSE there, -inf for an empty range; log2 units here); the lane holds
    // channels 16 cb + 4 q .. + 3 of its head
    const uint16_t *oc = static_cast<const uint16_t *>(a.o_cached);
    uint16_t *og = static_cast<uint16_t *>(a.o);
    const int S_n = a.n_splits;
    const float lse_own = m_run + log2f(l_run);
    float lse_c[kDecodeMaxSplits];
    float M = lse_own;
#pragma unroll
    for (int sp = 0; sp < kDecodeMaxSplits; ++sp) {
        lse_c[sp] = -INFINITY;
        if (sp < S_n && a.lse_cached) lse_c[sp] = a.lse_cached[sp * a.split_lse_elems + (int64_t)h * a.n_queries + n] * 1.4426950408889634f;
        M = fmaxf(M, lse_c[sp]);
    }
    const float wo = exp2f(m_run - M);                        // weight of the unnormalised own sum
    float denom = exp2f(lse_own - M);
    float sum[8][4];
#pragma unroll
    for (int cb = 0; cb < 8; ++cb)
#pragma unroll
        for (int r = 0; r < 4; ++r) sum[cb][r] = wo * O[cb][r];
#pragma unroll
    for (int sp = 0; sp < kDecodeMaxSplits; ++sp) {
        if (!(lse_c[sp] > -INFINITY)) continue;
        const float wc = exp2f(lse_c[sp] - M);
        denom += wc;
#pragma unroll
        for (int cb = 0; cb < 8; ++cb) {
            const uint2 raw = *reinterpret_cast<const uint2 *>(oc + sp * a.split_o_elems + io + cb * 16 + 4 * q);
            sum[cb][0] += wc * bf16_to_f32((uint16_t)(raw.x & 0xFFFF));
            sum[cb][1] += wc * bf16_to_f32((uint16_t)(raw.x >> 16));
            sum[cb][2] += wc * bf16_to_f32((uint16_t)(raw.y & 0xFFFF));
            sum[cb][3] += wc * bf16_to_f32((uint16_t)(raw.y >> 16));
        }
    }
    const float inv = 1.0f / denom;
#pragma unroll
    for (int cb = 0; cb < 8; ++cb) {
        uint2 out;
        out.x = (uint32_t)f32_to_bf16(sum[cb][0] * inv) | ((uint32_t)f32_to_bf16(sum[cb][1] * inv) << 16);
        out.y = (uint32_t)f32_to_bf16(sum[cb][2] * inv) | ((uint32_t)f32_to_bf16(sum[cb][3] * inv) << 16);
        *reinterpret_cast<uint2 *>(og + io + cb * 16 + 4 * q) = out;
    }
    if (a.lse && q == 0) a.lse[(int64_t)h * a.n_queries + n] = (M + log2f(denom)) * 0.6931471805599453f;
}

__global__ void fill_zero_bytes_kernel(uint4 *p, size_t n16)
{
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += (size_t)gridDim.x * blockDim.x)
        p[i] = make_uint4(0, 0, 0, 0);
}

// ---- export / import: raw element moves between page order and [P][Hkv][d] --------------------
template <typename T>
__global__ void cache_export_kernel(PoolGeom g, int layer, const int32_t *pages, int P, T *k, T *v)
{
    const int d = g.head_dim, Hkv = g.n_kv_heads;
    const int64_t n = (int64_t)P * Hkv * d;
    for (int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; idx < n; idx += (int64_t)gridDim.x * blockDim.x) {
        const int c = (int)(idx % d);
        const int hk = (int)((idx / d) % Hkv);
        const int j = (int)(idx / ((int64_t)d * Hkv));
        const int page = pages[j / kPageTokens], tok = j % kPageTokens;
        k[idx] = reinterpret_cast<const T *>(g.k_part(layer, page, hk))[k_page_index(tok, c)];
        v[idx] = reinterpret_cast<const T *>(g.v_part(layer, page, hk))[v_page_index(tok, c)];
    }
}

template <typename T>
__global__ void cache_import_kernel(PoolGeom g, int layer, const int32_t *pages, int P, const T *k, const T *v)
{
    const int d = g.head_dim, Hkv = g.n_kv_heads;
    const int n_pages = (P + kPageTokens - 1) / kPageTokens;
    const int64_t n = (int64_t)n_pages * kPageTokens * Hkv * d;   // whole pages: the tail is zeroed
    for (int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; idx < n; idx += (int64_t)gridDim.x * blockDim.x) {
        const int c = (int)(idx % d);
        const int hk = (int)((idx / d) % Hkv);
        const int j = (int)(idx / ((int64_t)d * Hkv));
        const int page = pages[j / kPageTokens], tok = j % kPageTokens;
        const T kk = j < P ? k[idx] : T(0);
        const T vv = j < P ? v[idx] : T(0);
        reinterpret_cast<T *>(g.k_part(layer, page, hk))[k_page_index(tok, c)] = kk;
        reinterpret_cast<T *>(g.v_part(layer, page, hk))[v_page_index(tok, c)] = vv;
    }
}

// ---- generic attention: one wavefront per (token, query head) row ----------------------------
// Lane l walks keys l, l + 64, ... keeping its own running (max, sum, weighted V); the 64 partial
// states are merged at the end.  All arithmetic is fp32; scores are kept in the log2 domain.
template <int D>
__global__ void __launch_bounds__(256) attn_generic_kernel(AttnArgs a)
{
    __shared__ float q_s[4][D];
    const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
    const int64_t row = (int64_t)blockIdx.x * 4 + wave;
    const int Hq = a.n_q_heads, Hkv = a.n_kv_heads, g = a.group, half = D / 2;
    const int64_t n_rows = (a.mode == MODE_SUFFIX ? a.total_tokens : (int64_t)a.prefix_len) * Hq;
    const bool live = row < n_rows;     // dead waves still reach the barrier below

    int h = 0, hk = 0, cluster = 0, P = 0, qpos = 0, n_cache = 0, n_self = 0;
    int64_t src = 0, self_src0 = 0;
    if (live) {
        const int64_t tau = row / Hq;
        h = (int)(row % Hq);
        hk = h / g;
        if (a.mode == MODE_SUFFIX) {
            const int sq = a.tok_sq[tau];
            cluster = a.sq_cluster[sq];
            P = a.cl_prefix_len[cluster];
            qpos = a.tok_qpos[tau];
            src = a.tok_src[tau];
            self_src0 = a.sq_src0[sq];
            n_cache = P;
            n_self = qpos + 1;
        } else {
            cluster = a.prefix_cluster;
            P = 0;                 // position of row = its own index
            qpos = (int)tau;
            src = tau;
            n_cache = qpos + 1;
            n_self = 0;
        }
    }
    const int pos = P + qpos;
    // rotated query row into LDS (lanes 0 .. D/16-1 handle one chunk pair each)
    if (live && lane < D / 16) {
        float x1[8], x2[8];
        const int64_t qrow = (src * Hq + h) * D;
        load8(a.q, qrow + lane * 8, a.io_dtype, x1);
        load8(a.q, qrow + half + lane * 8, a.io_dtype, x2);
        if (a.rope) rope8(x1, x2, a.rope + (int64_t)pos * half + lane * 8);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            q_s[wave][lane * 8 + i] = x1[i];
            q_s[wave][half + lane * 8 + i] = x2[i];
        }
    }
    __syncthreads();
    if (!live) return;

    float k_scale = 1.f, v_scale = 1.f;
    if (a.kv_scale) {
        const float *sc = a.kv_scale + ((int64_t)cluster * a.n_layers + a.layer) * 2 * Hkv;
        k_scale = sc[hk];
        v_scale = sc[Hkv + hk];
    }
    float m = -1e30f, l = 0.f, acc[D];
#pragma unroll
    for (int c = 0; c < D; ++c) acc[c] = 0.f;
    const int32_t *pt = a.page_table + a.cl_pt_off[cluster];
    const int kvd = a.pool.kv_dtype;

    // cached keys
    for (int j = lane; j < n_cache; j += kWave) {
        const int page = pt[j / kPageTokens], tok = j % kPageTokens;
        const char *kp = a.pool.k_part(a.layer, page, hk);
        const char *vp = a.pool.v_part(a.layer, page, hk);
        float s = 0.f;
#pragma unroll
        for (int cc = 0; cc < D / 8; ++cc) {
            float kk[8];
            load8(kp, k_page_index(tok, cc * 8), k_elem_type(kvd), kk);
#pragma unroll
            for (int i = 0; i < 8; ++i) s += q_s[wave][cc * 8 + i] * kk[i];
        }
        s *= a.scale_log2e * k_scale;
        float p, alpha = 1.f;
        if (s > m) {
            alpha = exp2f(m - s);
            m = s;
            p = 1.f;
        } else {
            p = exp2f(s - m);
        }
        l = l * alpha + p;
        const float pv = p * v_scale;
#pragma unroll
        for (int c = 0; c < D; ++c) acc[c] = acc[c] * alpha + pv * load1(vp, v_page_index(tok, c), kvd);
    }
    // the query's own suffix keys 0..qpos, rotated at P + j
    for (int j = lane; j < n_self; j += kWave) {
        const int64_t krow = ((self_src0 + j) * Hkv + hk) * D;
        float s = 0.f;
#pragma unroll
        for (int cc = 0; cc < D / 16; ++cc) {
            float x1[8], x2[8];
            load8(a.k, krow + cc * 8, a.io_dtype, x1);
            load8(a.k, krow + half + cc * 8, a.io_dtype, x2);
            if (a.rope) rope8(x1, x2, a.rope + (int64_t)(P + j) * half + cc * 8);
#pragma unroll
            for (int i = 0; i < 8; ++i) s += q_s[wave][cc * 8 + i] * x1[i] + q_s[wave][half + cc * 8 + i] * x2[i];
        }
        s *= a.scale_log2e;
        float p, alpha = 1.f;
        if (s > m) {
            alpha = exp2f(m - s);
            m = s;
            p = 1.f;
        } else {
            p = exp2f(s - m);
        }
        l = l * alpha + p;
#pragma unroll
        for (int cc = 0; cc < D / 8; ++cc) {
            float vv[8];
            load8(a.v, krow + cc * 8, a.io_dtype, vv);
#pragma unroll
            for (int i = 0; i < 8; ++i) acc[cc * 8 + i] = acc[cc * 8 + i] * alpha + p * vv[i];
        }
    }
    // merge the 64 partial states
    float M = m;
    for (int o = 32; o > 0; o >>= 1) M = fmaxf(M, __shfl_xor(M, o));
    const float f = exp2f(m - M);
    l *= f;
    for (int o = 32; o > 0; o >>= 1) l += __shfl_xor(l, o);
    const float inv_l = 1.0f / l;
    const int64_t orow = (src * Hq + h) * D;
#pragma unroll
    for (int c = 0; c < D; ++c) {
        float x = acc[c] * f;
        for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o);
        if (lane == (c & 63)) {
            const float y = x * inv_l;
            if (a.io_dtype == SGC_F32)
                static_cast<float *>(a.o)[orow + c] = y;
            else
                static_cast<uint16_t *>(a.o)[orow + c] = f32_to_bf16(y);
        }
    }
    if (a.lse && lane == 0) {
        const int64_t col = a.mode == MODE_SUFFIX ? src : (int64_t)qpos;
        a.lse[(int64_t)h * a.lse_stride + col] = (M + log2f(l)) * 0.6931471805599453f;
    }
}

}  // namespace

// ---- launchers -------------------------------------------------------------------------------
hipError_t launch_rope_table(float2 *table, int n_pos, int head_dim, double base, hipStream_t s)
{
    const int half = head_dim / 2;
    const int64_t n = (int64_t)n_pos * half;
    hipLaunchKernelGGL(rope_table_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, table, n_pos, half, base,
                       1.0 / (double)head_dim);
    return hipGetLastError();
}

hipError_t launch_prefix_ingest(const PoolGeom &g, int layer, const int32_t *d_page_table, const PrefixJob *d_jobs,
                                int n_jobs, const int32_t *d_page_job, int n_pages, int io_dtype, const float2 *rope,
                                const ExpandArgs *expand, hipStream_t s)
{
    if (n_pages == 0 || n_jobs == 0) return expand ? launch_expand_tiles(*expand, s) : hipSuccess;
    const dim3 grid(n_pages, g.n_kv_heads);
    if (g.kv_dtype == SGC_FP8_E4M3) {
        const int n = 2 * g.n_kv_heads;
        hipLaunchKernelGGL(scale_slot_kernel, dim3(n_jobs), dim3(64), 0, s, d_jobs, n, false);
        hipLaunchKernelGGL(ingest_amax_kernel, grid, dim3(128), 0, s, d_jobs, d_page_job, io_dtype, g.n_kv_heads, g.head_dim,
                           rope);
        hipLaunchKernelGGL(scale_slot_kernel, dim3(n_jobs), dim3(64), 0, s, d_jobs, n, true);
    }
    ExpandArgs ex{};
    if (expand) ex = *expand;
    const dim3 grid_all(n_pages + expand_columns(ex.n, g.n_kv_heads), g.n_kv_heads);
    hipLaunchKernelGGL(ingest_write_kernel, grid_all, dim3(128), 2 * (size_t)g.head_part_bytes, s, g, layer, d_page_table, d_jobs,
                       d_page_job, n_pages, io_dtype, rope, ex);
    return hipGetLastError();
}

hipError_t launch_expand_tiles(const ExpandArgs &e, hipStream_t s)
{
    if (e.n <= 0) return hipSuccess;
    hipLaunchKernelGGL(expand_tiles_kernel, dim3((e.n + 127) / 128), dim3(128), 0, s, e);
    return hipGetLastError();
}

hipError_t launch_suffix_ingest(const AttnArgs &a, const int32_t *d_spage_sq, int n_spages, const ExpandArgs *expand,
                                hipStream_t s)
{
    if (n_spages <= 0) return expand ? launch_expand_tiles(*expand, s) : hipSuccess;
    const size_t lds = 2 * (size_t)kPageTokens * a.head_dim * 2;
    ExpandArgs ex{};
    if (expand) ex = *expand;
    const dim3 grid(n_spages + expand_columns(ex.n, a.n_kv_heads), a.n_kv_heads);
    hipLaunchKernelGGL(suffix_ingest_kernel, grid, dim3(128), lds, s, a, d_spage_sq, n_spages, ex);
    return hipGetLastError();
}

hipError_t launch_decode_own_keys(const DecodeArgs &d, hipStream_t s)
{
    if (d.n_sq <= 0) return hipSuccess;
    const int g = d.n_q_heads / d.n_kv_heads;
    if (d.use_mfma && g <= 16) {                  // head_dim 128, bf16 rows: the matrix-core form
        const int units = d.n_sq * d.n_kv_heads;
        hipLaunchKernelGGL(decode_own_keys_mfma_kernel, dim3((units + 3) / 4), dim3(256), 0, s, d);
        return hipGetLastError();
    }
    const int G = g % 8 == 0 ? 8 : g % 4 == 0 ? 4 : g % 2 == 0 ? 2 : 1;      // heads per wavefront
    const dim3 grid((unsigned)((int64_t)d.n_sq * (d.n_q_heads / G)));
    const size_t lds = (size_t)G * (128 * 2 + (size_t)d.key_cap * (4 + 2));      // q rows (bf16), scores (fp32), weights (bf16)
    switch (G) {
        case 8: hipLaunchKernelGGL(decode_own_keys_kernel<8>, grid, dim3(64), lds, s, d); break;
        case 4: hipLaunchKernelGGL(decode_own_keys_kernel<4>, grid, dim3(64), lds, s, d); break;
        case 2: hipLaunchKernelGGL(decode_own_keys_kernel<2>, grid, dim3(64), lds, s, d); break;
        default: hipLaunchKernelGGL(decode_own_keys_kernel<1>, grid, dim3(64), lds, s, d); break;
    }
    return hipGetLastError();
}

// The tables a batch sends to the device are a few hundred KiB at most.  A copy engine transfer of that size spends most of
// its 25-35 us getting started; a kernel that reads the pinned, mapped staging buffer over the host link is done in
// the time the link needs.
// Up to two pieces per launch (a call's own tables and the cache's page tables, when both are due).
struct CopyPiece {
    uint4 *dst;
    const uint4 *src;
    size_t n16, n4;      // 16-byte chunks, then 4-byte words behind them
};
__device__ inline void copy_piece(const CopyPiece &p)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < p.n16; i += stride) p.dst[i] = p.src[i];
    uint32_t *d4 = reinterpret_cast<uint32_t *>(p.dst + p.n16);
    const uint32_t *s4 = reinterpret_cast<const uint32_t *>(p.src + p.n16);
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < p.n4; i += stride) d4[i] = s4[i];
}
__global__ void copy_from_host_kernel(CopyPiece a, CopyPiece b)
{
    copy_piece(a);
    copy_piece(b);
}

hipError_t launch_copy_from_host(void *dst, const void *mapped_src, size_t bytes, hipStream_t s, void *dst2,
                                 const void *mapped_src2, size_t bytes2)
{
    if (bytes == 0 && bytes2 == 0) return hipSuccess;
    const CopyPiece a{static_cast<uint4 *>(dst), static_cast<const uint4 *>(mapped_src), bytes / 16, (bytes % 16) / 4};
    const CopyPiece b{static_cast<uint4 *>(dst2), static_cast<const uint4 *>(mapped_src2), bytes2 / 16, (bytes2 % 16) / 4};
    const size_t most = std::max(a.n16, b.n16);
    const unsigned blocks = (unsigned)std::min<size_t>(std::max<size_t>((most + 255) / 256, 1), 1024);
    hipLaunchKernelGGL(copy_from_host_kernel, dim3(blocks), dim3(256), 0, s, a, b);
    return hipGetLastError();
}

hipError_t launch_fill_zero_bytes(void *p, size_t bytes, hipStream_t s)
{
    if (bytes == 0) return hipSuccess;
    const size_t n16 = bytes / 16;      // callers pass multiples of 16 bytes
    const unsigned blocks = (unsigned)std::min<size_t>((n16 + 255) / 256, 4096);
    hipLaunchKernelGGL(fill_zero_bytes_kernel, dim3(blocks), dim3(256), 0, s, static_cast<uint4 *>(p), n16);
    return hipGetLastError();
}

hipError_t launch_cache_export(const PoolGeom &g, int layer, const int32_t *d_pages, int prefix_len, void *k, void *v,
                               hipStream_t s)
{
    const int64_t n = (int64_t)prefix_len * g.n_kv_heads * g.head_dim;
    const unsigned blocks = (unsigned)std::min<int64_t>((n + 255) / 256, 65536);
    if (g.kv_bytes == 4)
        hipLaunchKernelGGL(cache_export_kernel<uint32_t>, dim3(blocks), dim3(256), 0, s, g, layer, d_pages, prefix_len,
                           (uint32_t *)k, (uint32_t *)v);
    else if (g.kv_bytes == 2)
        hipLaunchKernelGGL(cache_export_kernel<uint16_t>, dim3(blocks), dim3(256), 0, s, g, layer, d_pages, prefix_len,
                           (uint16_t *)k, (uint16_t *)v);
    else
        hipLaunchKernelGGL(cache_export_kernel<uint8_t>, dim3(blocks), dim3(256), 0, s, g, layer, d_pages, prefix_len,
                           (uint8_t *)k, (uint8_t *)v);
    return hipGetLastError();
}

hipError_t launch_cache_import(const PoolGeom &g, int layer, const int32_t *d_pages, int prefix_len, const void *k,
                               const void *v, hipStream_t s)
{
    const int n_pages = (prefix_len + kPageTokens - 1) / kPageTokens;
    const int64_t n = (int64_t)n_pages * kPageTokens * g.n_kv_heads * g.head_dim;
    const unsigned blocks = (unsigned)std::min<int64_t>((n + 255) / 256, 65536);
    if (g.kv_bytes == 4)
        hipLaunchKernelGGL(cache_import_kernel<uint32_t>, dim3(blocks), dim3(256), 0, s, g, layer, d_pages, prefix_len,
                           (const uint32_t *)k, (const uint32_t *)v);
    else if (g.kv_bytes == 2)
        hipLaunchKernelGGL(cache_import_kernel<uint16_t>, dim3(blocks), dim3(256), 0, s, g, layer, d_pages, prefix_len,
                           (const uint16_t *)k, (const uint16_t *)v);
    else
        hipLaunchKernelGGL(cache_import_kernel<uint8_t>, dim3(blocks), dim3(256), 0, s, g, layer, d_pages, prefix_len,
                           (const uint8_t *)k, (const uint8_t *)v);
    return hipGetLastError();
}

hipError_t launch_attn_generic(const AttnArgs &a, int64_t n_rows, hipStream_t s)
{
    if (n_rows <= 0) return hipSuccess;
    const unsigned blocks = (unsigned)((n_rows + 3) / 4);
    if (a.head_dim == 64)
        hipLaunchKernelGGL(attn_generic_kernel<64>, dim3(blocks), dim3(256), 0, s, a);
    else
        hipLaunchKernelGGL(attn_generic_kernel<128>, dim3(blocks), dim3(256), 0, s, a);
    return hipGetLastError();
}

}  // namespace sgc
