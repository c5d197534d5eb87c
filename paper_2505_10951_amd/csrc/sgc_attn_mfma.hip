// bf16 MFMA attention kernel of libsgc for gfx950 (MI355X), head_dim 128.
//
// SubGCache (arXiv 2505.10951) Sec. 3.4: every query of a cluster appends its question tokens to
// the cluster's cached prompt.  One workgroup takes a tile of rows that all belong to one
// (cluster, KV head): rows are (query, token, head-in-group) of ANY query of the cluster, so the
// cached prefix K/V tiles staged in LDS are shared by several queries at once.  After the
// prefix keys the same rows run causally over their own query's suffix keys, which a small
// ingest kernel has put into pages of the same layout beforehand.
//
// Matrix-core mapping (v_mfma_f32_32x32x16_bf16, 64-lane wavefronts):
//   S^T = K Q^T : A = 32 keys x 16 channels (from LDS), B = 16 channels x 32 rows (Q, registers).
//                 Lane (n, h) = (lane % 32, lane / 32) then owns row n and, in accumulator
//                 register r, key 8 (r / 4) + 4 h + r % 4: a row's scores sit in ONE lane pair, so
//                 the row max/sum need a single exchange between the two 32-lane halves.
//   O^T = V^T P^T : A = 32 channels x 16 keys (from LDS, V is stored transposed per 16-token page),
//                 B = 16 keys x 32 rows = the probabilities exactly as the score accumulator
//                 holds them (registers 8 kb .. 8 kb + 7), no cross-lane movement.
// A key tile is 64 keys = 4 pages; in LDS it is the linear image of those pages (8 parts of 4 KiB:
// K of the 4 pages, then V), copied global -> LDS without passing through registers.
//
// Softmax is online, fp32, base 2.  The reference maximum of a row is set from the first tile it
// sees and afterwards only raised (with a rescale of the accumulators) when a tile's weights
// against it would sum beyond 2^30, or in tiles that need masking; the result is the same
// softmax, since any reference that avoids overflow gives the same quotient.  The row sum adds
// the weights after their rounding to bf16, the values the second product uses.
#include <hip/hip_runtime.h>

#include "sgc_internal.h"

namespace sgc {

namespace {

#ifdef SGC_NO_SCHED_BARRIER
#define SGC_SCHED_FENCE() do { } while (0)
#else
#define SGC_SCHED_FENCE() __builtin_amdgcn_sched_barrier(0)
#endif

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

constexpr int D = 128;                       // head dim
constexpr int BN = 64;                       // keys per LDS tile (4 pages)
constexpr int PART_BYTES = kPageTokens * D * 2;   // one page's K (or V) of one head as bf16: 4 KiB
constexpr int BUF_BYTES = 8 * PART_BYTES;    // 4 K parts + 4 V parts
constexpr int V_TILE_OFF = 4 * PART_BYTES;
constexpr int MAX_TILE_QUERIES = 256;        // queries a row tile can touch (one row each at least)
constexpr float kKeepBelow = 1073741824.0f;  // 2^30: a tile's weights may sum to this against a stale maximum
constexpr float kNegBig = -1.0e30f;

#ifdef SGC_PHASE_TIMING
// Development aid (not built into the product library): per-phase cycle totals of the tile loop.
__device__ unsigned long long g_phase[2048 * 8 * 8];   // [block < 2048][wave < 8][phase < 8]
#define SGC_TS(i) do { const unsigned long long now__ = __builtin_readcyclecounter(); ph[i] += (unsigned)(now__ - tlast); tlast = __builtin_readcyclecounter(); } while (0)
#else
#define SGC_TS(i) do { } while (0)
#endif

__device__ inline float half_swap(float x) { return __shfl_xor(x, 32); }

// Unpacks 2 fp8 e4m3 codes (low or high half of w) to bf16 (exact: e4m3 is a subset of bf16).
__device__ inline uint32_t fp8x2_to_bf16x2(uint32_t w, bool high)
{
    const auto f = high ? __builtin_amdgcn_cvt_pk_f32_fp8((int)w, true) : __builtin_amdgcn_cvt_pk_f32_fp8((int)w, false);
    return (__float_as_uint(f[0]) >> 16) | (__float_as_uint(f[1]) & 0xFFFF0000u);
}

// 1 KiB global -> LDS, 16 bytes per lane, landing at lds + 16 * lane.
__device__ inline void copy_1k_to_lds(const char *src_lane, char *lds_block)
{
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)src_lane,
                                     (__attribute__((address_space(3))) void *)lds_block, 16, 0, 0);
}

struct TileDesc {
    int kind;      // 0: cached prefix keys, 1: the suffix keys of sorted query q
    int key0;      // first key of the tile (index inside the prefix / inside the query's suffix)
    int q;         // sorted query (kind 1)
    int page0;     // first suffix page of the tile (kind 1)
    int page_last; // last suffix page of the query (kind 1)
};

template <int NW, int MI, bool KV_FP8, int MODE>
__global__ void __launch_bounds__(NW * 64, (NW == 4 && MI == 1) ? 2 : 1) attn_mfma_kernel(const AttnArgs a)
{
    constexpr int BM = NW * MI * 32;
    extern __shared__ __attribute__((aligned(1024))) char smem[];
    char *const buf0 = smem;
    int2 *const qinfo = reinterpret_cast<int2 *>(smem + 2 * BUF_BYTES);   // (suffix length, first suffix page)

    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63;
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
    const int n = lane & 31, h = lane >> 5;
    const int Hq = a.n_q_heads, Hkv = a.n_kv_heads, g = a.group;

    // ---- which tile ----
    Tile t;
    if (MODE == MODE_SUFFIX) {
        t = a.tiles[blockIdx.x];
        if (t.n_rows == 0) return;
    } else {
        const int rows = a.prefix_len * g;
        const int tiles_per_head = (rows + BM - 1) / BM;
        t.cluster = a.prefix_cluster;
        t.hk = blockIdx.x % Hkv;
        const int ti = tiles_per_head - 1 - (int)(blockIdx.x / Hkv);   // longest rows first
        t.row0 = ti * BM;
        t.n_rows = min(BM, rows - t.row0);
    }
    // everything that steers the tile loop is made explicitly wave-uniform (scalar registers)
    const int cluster = __builtin_amdgcn_readfirstlane(t.cluster), hk = __builtin_amdgcn_readfirstlane(t.hk);
    t.row0 = __builtin_amdgcn_readfirstlane(t.row0);
    t.n_rows = __builtin_amdgcn_readfirstlane(t.n_rows);
    const int P = __builtin_amdgcn_readfirstlane((MODE == MODE_SUFFIX) ? a.cl_prefix_len[cluster] : a.prefix_len);
    const int n_pages = (P + kPageTokens - 1) / kPageTokens;
    const int32_t *pt = a.page_table + __builtin_amdgcn_readfirstlane(a.cl_pt_off[cluster]);
    const int tok_base = __builtin_amdgcn_readfirstlane((MODE == MODE_SUFFIX) ? a.cl_tok_off[cluster] : 0);
    const int last_row = t.row0 + t.n_rows - 1;

    // ---- the queries this tile touches (suffix mode): lengths and first pages into LDS ----
    int sq_lo = 0, sq_hi = -1, last_qpos = 0;
    if (MODE == MODE_SUFFIX) {
        const int last_tau = tok_base + last_row / g;
        sq_lo = __builtin_amdgcn_readfirstlane(a.tok_sq[tok_base + t.row0 / g]);
        sq_hi = __builtin_amdgcn_readfirstlane(a.tok_sq[last_tau]);
        last_qpos = __builtin_amdgcn_readfirstlane(a.tok_qpos[last_tau]);
        for (int i = tid; i <= sq_hi - sq_lo && i < MAX_TILE_QUERIES; i += NW * 64)
            qinfo[i] = make_int2(a.sq_len[sq_lo + i], a.sq_page0[sq_lo + i]);
    }

    float k_scale = 1.f, v_scale = 1.f;
    if (KV_FP8) {
        const float *sc = a.kv_scale + ((int64_t)cluster * a.n_layers + a.layer) * 2 * Hkv;
        k_scale = sc[hk];
        v_scale = sc[Hkv + hk];
    }
    const float c_cache = a.scale_log2e * k_scale;
    const float c_self = a.scale_log2e;

    // ---- per-lane row bookkeeping ----
    bool valid[MI];
    int64_t io_row[MI];     // element offset of the row in q / o
    int qpos[MI], sq[MI], lim[MI], src_tok[MI], head[MI];
#pragma unroll
    for (int mi = 0; mi < MI; ++mi) {
        const int r = t.row0 + (wave * MI + mi) * 32 + n;
        valid[mi] = r <= last_row;
        const int rc = valid[mi] ? r : last_row;
        const int tk = rc / g;
        head[mi] = hk * g + (rc - tk * g);
        if (MODE == MODE_SUFFIX) {
            const int tau = tok_base + tk;
            src_tok[mi] = a.tok_src[tau];
            qpos[mi] = a.tok_qpos[tau];
            sq[mi] = a.tok_sq[tau];
            lim[mi] = P;
        } else {
            src_tok[mi] = tk;
            qpos[mi] = tk;
            sq[mi] = 0;
            lim[mi] = tk + 1;
        }
        io_row[mi] = ((int64_t)src_tok[mi] * Hq + head[mi]) * D;
    }
    // wave-uniform bounds: visible cached keys, and the sorted queries / positions of this wave's rows
    int lim_min = lim[0], lim_max = lim[0], wsq_min = sq[0], wsq_max = sq[0];
#pragma unroll
    for (int mi = 1; mi < MI; ++mi) {
        lim_min = min(lim_min, lim[mi]);
        lim_max = max(lim_max, lim[mi]);
        wsq_min = min(wsq_min, sq[mi]);
        wsq_max = max(wsq_max, sq[mi]);
    }
    for (int o = 32; o > 0; o >>= 1) {
        lim_min = min(lim_min, __shfl_xor(lim_min, o));
        lim_max = max(lim_max, __shfl_xor(lim_max, o));
        wsq_min = min(wsq_min, __shfl_xor(wsq_min, o));
        wsq_max = max(wsq_max, __shfl_xor(wsq_max, o));
    }
    lim_min = __builtin_amdgcn_readfirstlane(lim_min);
    lim_max = __builtin_amdgcn_readfirstlane(lim_max);
    wsq_min = __builtin_amdgcn_readfirstlane(wsq_min);
    wsq_max = __builtin_amdgcn_readfirstlane(wsq_max);

    // ---- Q: load, rotate at position P + qpos (suffix) / qpos (prefix), keep as B operands ----
    bf16x8 qf[MI][8];
#pragma unroll
    for (int mi = 0; mi < MI; ++mi) {
        const uint16_t *qrow = static_cast<const uint16_t *>(a.q) + io_row[mi];
        const int pos = (MODE == MODE_SUFFIX ? P : 0) + qpos[mi];
#pragma unroll
        for (int kb = 0; kb < 4; ++kb) {
            const int c0 = kb * 16 + h * 8;
            const uint4 lo = *reinterpret_cast<const uint4 *>(qrow + c0);
            const uint4 hi = *reinterpret_cast<const uint4 *>(qrow + 64 + c0);
            const uint32_t wl[4] = {lo.x, lo.y, lo.z, lo.w}, wh[4] = {hi.x, hi.y, hi.z, hi.w};
            float x1[8], x2[8];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                x1[2 * i] = __uint_as_float(wl[i] << 16);
                x1[2 * i + 1] = __uint_as_float(wl[i] & 0xFFFF0000u);
                x2[2 * i] = __uint_as_float(wh[i] << 16);
                x2[2 * i + 1] = __uint_as_float(wh[i] & 0xFFFF0000u);
            }
            if (a.rope) {
                const float4 *tab = reinterpret_cast<const float4 *>(a.rope + (int64_t)pos * 64 + c0);
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const float4 cs = tab[i];   // (cos, sin) of two channels
                    const float a0 = x1[2 * i], b0 = x2[2 * i], a1 = x1[2 * i + 1], b1 = x2[2 * i + 1];
                    x1[2 * i] = a0 * cs.x - b0 * cs.y;
                    x2[2 * i] = b0 * cs.x + a0 * cs.y;
                    x1[2 * i + 1] = a1 * cs.z - b1 * cs.w;
                    x2[2 * i + 1] = b1 * cs.z + a1 * cs.w;
                }
            }
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                qf[mi][kb][i] = (__bf16)x1[i];
                qf[mi][kb + 4][i] = (__bf16)x2[i];
            }
        }
    }

    // ---- accumulators ----
    f32x16 oacc[MI][4];
    float m_ref[MI], l_part[MI];
#pragma unroll
    for (int mi = 0; mi < MI; ++mi) {
        m_ref[mi] = kNegBig;
        l_part[mi] = 0.f;
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) oacc[mi][db][r] = 0.f;
    }
    bool fresh = true;     // no tile processed yet by this wavefront
#ifdef SGC_PHASE_TIMING
    unsigned ph[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    unsigned long long tlast = 0;
    const unsigned long long blk_c0 = __builtin_readcyclecounter(), blk_r0 = __builtin_amdgcn_s_memrealtime();
#endif

    // Per-lane LDS offsets of the operand blocks.  K block (nb, kb): lane (m, hh) reads key m of the 32-key
    // group nb (page 2 nb + m / 16, token m % 16), channels kb * 16 + hh * 8 .. + 7.  Each 16-lane group
    // reads 256 contiguous bytes, which is conflict-free.  V block (pg, db) is 1 KiB contiguous.
    const int lane_koff = ((n >> 4) * PART_BYTES) + (h * kPageTokens + (n & 15)) * 16;
    const int lane_voff = V_TILE_OFF + lane * 16;

    // One 64-key tile from LDS buffer `buf`.  c is the score scale in log2 units.  `careful` forces the
    // exact running maximum and, with `masked`, masking through keep(mi, j) = "row mi may see key j of
    // the tile"; otherwise the weights are taken against the current reference maximum without
    // looking for the tile's maximum, and the careful step only runs when one of them turns out too
    // large to keep.
    auto process_tile = [&](const char *buf, const float c, bool careful, const bool masked, auto keep) {
        // LDS operand blocks are read through a rolling window of 8 register sets: 8 reads are in
        // flight, each matrix instruction is followed by the read that refills the block it used.
        bf16x8 frag[8];
        const char *kbase = buf + lane_koff;
        const char *vbase = buf + lane_voff;
#pragma unroll
        for (int i = 0; i < 8; ++i) frag[i] = *reinterpret_cast<const bf16x8 *>(kbase + i * 512);
        SGC_SCHED_FENCE();
        SGC_TS(1);
        f32x16 sacc[MI][2];
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
            for (int nb = 0; nb < 2; ++nb)
#pragma unroll
                for (int r = 0; r < 16; ++r) sacc[mi][nb][r] = 0.f;
        // S^T = K Q^T: block i = (32-key group nb = i / 8, 16-channel group kb = i % 8)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
#pragma unroll
            for (int mi = 0; mi < MI; ++mi)
                sacc[mi][i >> 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag[i & 7], qf[mi][i & 7], sacc[mi][i >> 3], 0, 0, 0);
            // refill: K block i + 8, then (while the softmax runs) the first 8 V blocks
            if (i < 8)
                frag[i & 7] = *reinterpret_cast<const bf16x8 *>(kbase + 2 * PART_BYTES + i * 512);
            else
                frag[i & 7] = *reinterpret_cast<const bf16x8 *>(vbase + (i - 8) * 1024);
            SGC_SCHED_FENCE();
        }
        SGC_TS(2);

        uint32_t pf[MI][4][4];     // weights as bf16 pairs: [row block][16-key group][register pair]
        careful = careful || fresh;
#ifdef SGC_ABLATE_SOFTMAX
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
            for (int pg = 0; pg < 4; ++pg)
#pragma unroll
                for (int i = 0; i < 4; ++i) pf[mi][pg][i] = __float_as_uint(sacc[mi][pg >> 1][(pg & 1) * 8 + i * 2]);
        if (false)
#endif
#pragma unroll
        for (int mi = 0; mi < MI; ++mi) {
            float psum = 0.f;
            auto weights = [&]() {
                psum = 0.f;
                bf16x2 ones;
                ones[0] = (__bf16)1.0f;
                ones[1] = (__bf16)1.0f;
#pragma unroll
                for (int nb = 0; nb < 2; ++nb)
#pragma unroll
                    for (int r = 0; r < 16; r += 2) {
                        bf16x2 pk;
                        pk[0] = (__bf16)__builtin_amdgcn_exp2f(sacc[mi][nb][r] * c - m_ref[mi]);
                        pk[1] = (__bf16)__builtin_amdgcn_exp2f(sacc[mi][nb][r + 1] * c - m_ref[mi]);
                        psum = __builtin_amdgcn_fdot2_f32_bf16(pk, ones, psum, false);   // sum of the ROUNDED weights
                        pf[mi][nb * 2 + (r >> 3)][(r & 7) >> 1] = __builtin_bit_cast(uint32_t, pk);
                    }
            };
            bool redo = careful;
            if (!careful) {
                weights();
                redo = __any(!(psum <= kKeepBelow));   // also catches inf / nan
            }
            if (redo) {
                if (masked) {
#pragma unroll
                    for (int nb = 0; nb < 2; ++nb)
#pragma unroll
                        for (int r = 0; r < 16; ++r) {
                            const int j = nb * 32 + 8 * (r >> 2) + 4 * h + (r & 3);
                            if (!keep(mi, j)) sacc[mi][nb][r] = -INFINITY;
                        }
                }
                float tmax = sacc[mi][0][0];
#pragma unroll
                for (int nb = 0; nb < 2; ++nb)
#pragma unroll
                    for (int r = 0; r < 16; ++r) tmax = fmaxf(tmax, sacc[mi][nb][r]);
                tmax = fmaxf(tmax, half_swap(tmax)) * c;
                if (__any(tmax > m_ref[mi])) {
                    const float m_new = fmaxf(m_ref[mi], tmax);
                    const float alpha = __builtin_amdgcn_exp2f(m_ref[mi] - m_new);
                    m_ref[mi] = m_new;
                    l_part[mi] *= alpha;
#pragma unroll
                    for (int db = 0; db < 4; ++db)
#pragma unroll
                        for (int r = 0; r < 16; ++r) oacc[mi][db][r] *= alpha;
                }
                weights();
            }
            l_part[mi] += psum;
        }
        fresh = false;
        SGC_SCHED_FENCE();
        SGC_TS(3);
        // O^T += V^T P^T: block i = (16-key page pg = i / 4, 32-channel group db = i % 4)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int pg = i >> 2, db = i & 3;
#pragma unroll
            for (int mi = 0; mi < MI; ++mi) {
                const u32x4 w = {pf[mi][pg][0], pf[mi][pg][1], pf[mi][pg][2], pf[mi][pg][3]};
                oacc[mi][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag[i & 7], __builtin_bit_cast(bf16x8, w), oacc[mi][db], 0, 0, 0);
            }
            if (i < 8) frag[i & 7] = *reinterpret_cast<const bf16x8 *>(vbase + (i + 8) * 1024);
            SGC_SCHED_FENCE();
        }
        SGC_TS(4);
    };

    // ---- copy machinery ----------------------------------------------------------------------------
    // A tile is 32 runs of 1 KiB (fp8 cache: 16 runs of 1 KiB of codes that widen to 2 KiB); run u = part * 4
    // + quarter with part 0..3 = K of page 0..3, part 4..7 = V of page 0..3.  Wavefront w moves runs
    // w, w + NW, ...  A run's address is a scalar base (source base + page offset) plus a per-lane 32-bit
    // offset that is fixed for the launch; page offsets travel as 32-bit counts of 256 bytes, one tile
    // ahead, in a vector register (lane j < 4 holds page j of the tile) and become scalars by readlane,
    // so no copy ever waits on a page-table load.
    constexpr int UNITS_BF16 = 32 / NW, UNITS_FP8 = 16 / NW;
    const char *cache_base = a.pool.pool + (int64_t)a.layer * a.pool.layer_bytes + (int64_t)hk * a.pool.head_part_bytes;
    const uint32_t cache_v_off = (uint32_t)(Hkv * a.pool.head_part_bytes);
    const uint32_t cache_page_256 = (uint32_t)(a.pool.page_bytes >> 8);
    const char *spool_base = a.spool + (int64_t)hk * PART_BYTES;
    const uint32_t spool_v_off = (uint32_t)Hkv * PART_BYTES;
    const uint32_t spool_page_256 = (2u * spool_v_off) >> 8;
    uint4 stage[KV_FP8 ? UNITS_FP8 : 1];

    // Page indices past the last page are clamped to it: such keys are masked out of the scores, and what
    // they multiply in the second product is finite cache content times a zero weight.
    auto cache_page_ids = [&](int kt) -> uint32_t {     // raw page ids; scaled to offsets when used
        if (n_pages == 0) return 0;       // no cached keys: nothing is ever copied from the cache
        return (uint32_t)pt[min(kt * 4 + (lane & 3), n_pages - 1)];
    };
    const uint32_t lane16 = lane * 16;
    auto issue_copy_bf16 = [&](uint32_t poff, char *buf, const char *base, uint32_t v_off) {
#pragma unroll
        for (int j = 0; j < UNITS_BF16; ++j) {
            const int u = wave_u + NW * j;
            const int part = u >> 2, quarter = u & 3;
            const uint32_t off256 = __builtin_amdgcn_readlane(poff, part & 3);
            const char *sbase = base + ((uint64_t)off256 << 8) + (part >= 4 ? v_off : 0u) + quarter * 1024;
            copy_1k_to_lds(sbase + lane16, buf + u * 1024);
        }
    };
    auto issue_load_fp8 = [&](uint32_t poff) {
#pragma unroll
        for (int j = 0; j < UNITS_FP8; ++j) {
            const int u = wave_u + NW * j;
            const int part = u >> 1, run = u & 1;       // a part is 2 KiB of codes
            const uint32_t off256 = __builtin_amdgcn_readlane(poff, part & 3);
            const char *sbase = cache_base + ((uint64_t)off256 << 8) + (part >= 4 ? cache_v_off : 0u) + run * 1024;
            stage[j] = *reinterpret_cast<const uint4 *>(sbase + lane16);
        }
    };
    auto store_fp8 = [&](char *buf) {
#pragma unroll
        for (int j = 0; j < UNITS_FP8; ++j) {
            const int u = wave_u + NW * j;
            const int part = u >> 1, run = u & 1;
            // 16 codes -> 16 bf16 = 32 bytes; chunk cp of the part lands at 32 * cp of its bf16 image
            const uint32_t w[4] = {stage[j].x, stage[j].y, stage[j].z, stage[j].w};
            uint4 o0, o1;
            o0.x = fp8x2_to_bf16x2(w[0], false); o0.y = fp8x2_to_bf16x2(w[0], true);
            o0.z = fp8x2_to_bf16x2(w[1], false); o0.w = fp8x2_to_bf16x2(w[1], true);
            o1.x = fp8x2_to_bf16x2(w[2], false); o1.y = fp8x2_to_bf16x2(w[2], true);
            o1.z = fp8x2_to_bf16x2(w[3], false); o1.w = fp8x2_to_bf16x2(w[3], true);
            char *dst = buf + part * PART_BYTES + (run * 64 + lane) * 32;
            *reinterpret_cast<uint4 *>(dst) = o0;
            *reinterpret_cast<uint4 *>(dst + 16) = o1;
        }
    };
    auto fetch_cache = [&](uint32_t poff, char *buf) {
        if (KV_FP8)
            issue_load_fp8(poff);
        else
            issue_copy_bf16(poff, buf, cache_base, cache_v_off);
    };
    auto land_cache = [&](char *buf) {      // make the fetched cached tile visible in LDS (before the barrier)
        if (KV_FP8) store_fp8(buf);
        __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): direct copies have landed
    };

    // Two wavefronts share each SIMD (wave w and w + 4).  Giving one of them standing priority breaks the
    // lock-step in which both want the matrix unit and then both want the vector unit.
    if (NW == 8) {
        if (wave_u < 4)
            __builtin_amdgcn_s_setprio(2);
        else
            __builtin_amdgcn_s_setprio(0);
    }

    // ---- cached prefix tiles, double buffered ------------------------------------------------------
    const int n_cache_keys = (MODE == MODE_SUFFIX) ? P : min(P, last_row / g + 1);
    const int n_kt = (n_cache_keys + BN - 1) / BN;
    int parity = 0;
    uint32_t pids = 0;          // page ids of the next cached tile, loaded one step before they are needed
    if (n_kt > 0) {
        pids = cache_page_ids(0);
        fetch_cache(pids * cache_page_256, buf0);
        pids = cache_page_ids(1);
        land_cache(buf0);
    }
    __syncthreads();       // also: qinfo is in LDS
#ifdef SGC_PHASE_TIMING
    tlast = __builtin_readcyclecounter();
#endif
    for (int kt = 0; kt < n_kt; ++kt) {
        char *buf = buf0 + parity * BUF_BYTES;
        char *other = buf0 + (parity ^ 1) * BUF_BYTES;
        const bool more = kt + 1 < n_kt;
        if (more) {
            fetch_cache(pids * cache_page_256, other);
            pids = cache_page_ids(kt + 2);       // lands before the end-of-step wait, used a step later
        }
        SGC_TS(0);
        const int key0 = kt * BN;
        if (key0 < lim_max) {                    // some row of this wave still sees keys of this tile
            const bool masked = key0 + BN > lim_min;
            process_tile(buf, c_cache, masked, masked, [&](int mi, int j) { return key0 + j < lim[mi]; });
        }
        if (more) land_cache(other);
        SGC_TS(5);
        __syncthreads();
        SGC_TS(6);
        parity ^= 1;
    }

    // ---- the suffix keys of every query this row tile touches, double buffered ------------------------
    bool v_scaled = !KV_FP8;
    if (MODE == MODE_SUFFIX) {
        if (!v_scaled) {        // fp8 cache: the accumulated cached part takes the V scale once
#pragma unroll
            for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                for (int db = 0; db < 4; ++db)
#pragma unroll
                    for (int r = 0; r < 16; ++r) oacc[mi][db][r] *= v_scale;
            v_scaled = true;
        }
        // scalar iterator over (query, 64-key tile); a query's LDS record is read when the stream reaches it
        int it_q = sq_lo - 1, it_jt = 0, it_njt = 0, it_pg0 = 0, it_pglast = 0;
#define SGC_NEXT_SELF(ok, d)                                                                        \
    do {                                                                                            \
        while (it_jt >= it_njt && it_q < sq_hi) {                                                   \
            ++it_q;                                                                                 \
            const int2 qi = qinfo[min(it_q - sq_lo, MAX_TILE_QUERIES - 1)];                         \
            const int S__ = __builtin_amdgcn_readfirstlane(qi.x);                                   \
            it_pg0 = __builtin_amdgcn_readfirstlane(qi.y);                                          \
            it_pglast = it_pg0 + (S__ - 1) / kPageTokens;                                           \
            it_njt = ((it_q == sq_hi ? last_qpos : S__ - 1) + BN) / BN;                             \
            it_jt = 0;                                                                              \
        }                                                                                           \
        (ok) = it_jt < it_njt;                                                                      \
        (d).key0 = it_jt * BN;                                                                      \
        (d).q = it_q;                                                                               \
        (d).page0 = it_pg0 + it_jt * 4;                                                             \
        (d).page_last = it_pglast;                                                                  \
        ++it_jt;                                                                                    \
    } while (0)
        auto fetch_self = [&](const TileDesc &d, char *buf) {
            const uint32_t po = (uint32_t)min(d.page0 + (lane & 3), d.page_last) * spool_page_256;
            issue_copy_bf16(po, buf, spool_base, spool_v_off);
        };
        TileDesc cur = {1, 0, 0, 0, 0}, nxt = {1, 0, 0, 0, 0};
        bool have, more;
        SGC_NEXT_SELF(have, cur);
        if (have) {
            fetch_self(cur, buf0 + parity * BUF_BYTES);
            __builtin_amdgcn_s_waitcnt(0x0F70);
        }
        __syncthreads();
        while (have) {
            char *buf = buf0 + parity * BUF_BYTES;
            char *other = buf0 + (parity ^ 1) * BUF_BYTES;
            SGC_NEXT_SELF(more, nxt);
            if (more) fetch_self(nxt, other);
            const int key0 = cur.key0, q = cur.q;
            bool mine = false;                  // does a row of this wave belong to query q and reach key0?
#pragma unroll
            for (int mi = 0; mi < MI; ++mi) mine |= valid[mi] && sq[mi] == q && qpos[mi] >= key0;
            if (q >= wsq_min && q <= wsq_max && __any(mine))
                process_tile(buf, c_self, true, true, [&](int mi, int j) { return sq[mi] == q && key0 + j <= qpos[mi]; });
            if (more) __builtin_amdgcn_s_waitcnt(0x0F70);
            __syncthreads();
            cur = nxt;
            have = more;
            parity ^= 1;
        }
#undef SGC_NEXT_SELF
    }
#ifdef SGC_PHASE_TIMING
    if (lane == 0 && blockIdx.x < 2048) {
        ph[7] = (unsigned)(__builtin_amdgcn_s_memrealtime() - blk_r0);      // 100 MHz ticks for the whole block so far
        ph[6] = (unsigned)(__builtin_readcyclecounter() - blk_c0);          // shader-clock ticks (overwrites the barrier slot)
#pragma unroll
        for (int i = 0; i < 8; ++i) g_phase[(blockIdx.x * 8 + wave) * 8 + i] = ph[i];
    }
#endif

    // ---- normalise and store ----
    uint16_t *og = static_cast<uint16_t *>(a.o);
#pragma unroll
    for (int mi = 0; mi < MI; ++mi) {
        const float l = l_part[mi] + half_swap(l_part[mi]);
        const float inv_l = (v_scaled ? 1.0f : v_scale) / l;
        if (valid[mi]) {
#pragma unroll
            for (int db = 0; db < 4; ++db)
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4) {
                    bf16x4 y;
#pragma unroll
                    for (int i = 0; i < 4; ++i) y[i] = (__bf16)(oacc[mi][db][q4 * 4 + i] * inv_l);
                    *reinterpret_cast<bf16x4 *>(og + io_row[mi] + db * 32 + q4 * 8 + h * 4) = y;
                }
            if (a.lse && h == 0) {
                const int64_t col = (MODE == MODE_SUFFIX) ? (int64_t)src_tok[mi] : (int64_t)qpos[mi];
                a.lse[(int64_t)head[mi] * a.lse_stride + col] = (m_ref[mi] + __builtin_amdgcn_logf(l)) * 0.6931471805599453f;
            }
        }
    }
}

constexpr size_t kDynLds = 2 * BUF_BYTES + MAX_TILE_QUERIES * sizeof(int2);

template <int NW, int MI, bool FP8, int MODE>
hipError_t launch_one(const AttnArgs &a, int blocks, hipStream_t s)
{
    static bool configured = false;     // raise the dynamic LDS limit once per instantiation
    auto kern = attn_mfma_kernel<NW, MI, FP8, MODE>;
    size_t lds = kDynLds;
#ifdef SGC_EXPERIMENT_LDS
    if (const char *e = getenv("SGC_EXTRA_LDS")) lds += (size_t)atoi(e);   // development aid: limit occupancy
#endif
    if (!configured) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        configured = true;
    }
    hipLaunchKernelGGL(kern, dim3(blocks), dim3(NW * 64), lds, s, a);
    return hipGetLastError();
}

template <int NW, int MI>
hipError_t launch_variant(const AttnArgs &a, hipStream_t s)
{
    constexpr int BM = NW * MI * 32;
    const bool fp8 = a.pool.kv_dtype == SGC_FP8_E4M3;
    if (a.mode == MODE_SUFFIX) {
        if (a.n_tiles <= 0) return hipSuccess;
        return fp8 ? launch_one<NW, MI, true, MODE_SUFFIX>(a, a.n_tiles, s) : launch_one<NW, MI, false, MODE_SUFFIX>(a, a.n_tiles, s);
    }
    const int rows = a.prefix_len * a.group;
    const int tiles = (rows + BM - 1) / BM * a.n_kv_heads;
    if (tiles <= 0) return hipSuccess;
    return fp8 ? launch_one<NW, MI, true, MODE_PREFIX>(a, tiles, s) : launch_one<NW, MI, false, MODE_PREFIX>(a, tiles, s);
}

}  // namespace

#ifdef SGC_PHASE_TIMING
extern "C" int sgc_debug_read_phases(unsigned long long *host, size_t n)
{
    return (int)hipMemcpyFromSymbol(host, HIP_SYMBOL(g_phase), n * sizeof(unsigned long long));
}
#endif

// variant 0: 8 waves x 32 rows (256-row tiles, one workgroup per CU);
//         1: 4 waves x 32 rows (128-row tiles, two workgroups per CU);
//         2: 4 waves x 64 rows (256-row tiles, one workgroup per CU)
int mfma_tile_rows(int variant)
{
    switch (variant) {
        case 0: return 256;
        case 1: return 128;
        case 2: return 256;
        default: return 0;
    }
}

hipError_t launch_attn_mfma(const AttnArgs &a, int variant, hipStream_t s)
{
    switch (variant) {
        case 0: return launch_variant<8, 1>(a, s);
        case 1: return launch_variant<4, 1>(a, s);
        case 2: return launch_variant<4, 2>(a, s);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace sgc
