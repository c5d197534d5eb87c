// Matrix-core attention kernel of libsgc for gfx950 (MI355X), head_dim 128: first product on binary16 operands
// (rotated keys and queries; on the e4m3 codes of an fp8 cache in the QK8 variant), second product on bf16.
//
// SubGCache (arXiv 2505.10951) Sec. 3.4: every query of a cluster appends its question tokens to
// the cluster's cached prompt.  One workgroup takes a tile of rows that all belong to one
// (cluster, KV head): rows are (query, token, head-in-group) of ANY query of the cluster, so the
// cached prefix K/V tiles staged in LDS are shared by several queries at once.  After the
// prefix keys the same rows run causally over their own query's suffix keys, which a small
// ingest kernel has put into pages of the same layout beforehand.
//
// Matrix-core mapping (v_mfma_f32_32x32x16_f16 / _bf16, 64-lane wavefronts):
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

#include <type_traits>

#include "sgc_internal.h"

namespace sgc {

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(8))) int i32x8;

constexpr int D = 128;                       // head dim
constexpr int BN = 64;                       // keys per LDS tile (4 pages)
constexpr int PART_BYTES = kPageTokens * D * 2;   // one page's K (or V) of one head as bf16: 4 KiB
constexpr int HALF_BYTES = 4 * PART_BYTES;   // the K (or V) of one 64-key tile: 16 KiB
constexpr int LDS_TILE_BYTES = 4 * HALF_BYTES;   // two K buffers, then two V buffers
constexpr int K8_PART_BYTES = kPageTokens * D;    // one page's K of one head as e4m3 codes: 2 KiB
constexpr int K8_PART_STRIDE = K8_PART_BYTES + 128;   // in LDS consecutive pages sit 2 KiB + 128 bytes apart: the two pages
                                                      // a 32-key operand read touches then fall into different banks
constexpr int MAX_TILE_QUERIES = 256;        // queries a row tile can touch (one row each at least)
constexpr float kKeepBelow = 1073741824.0f;  // 2^30: a tile's weights may sum to this against a stale maximum

// Combine a value with the one held by the lane 32 away (the other half of a score row), through
// v_permlane32_swap: with both operands x, the two results hold x's lower half and x's upper half, each
// in all 64 lanes.
__device__ inline float half_max(float x)
{
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ inline float half_sum(float x)
{
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// Unpacks 2 fp8 e4m3 codes (low or high half of w) to 16-bit floats: binary16 for keys, bf16 for values (both
// exact: e4m3 is a subset of either).
template <bool TO_F16>
__device__ inline uint32_t fp8x2_to_16x2(uint32_t w, bool high)
{
    if (TO_F16) {
        const auto r = high ? __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(w, 1.0f, true) : __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(w, 1.0f, false);
        return __builtin_bit_cast(uint32_t, r);
    }
    const auto r = high ? __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w, 1.0f, true) : __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w, 1.0f, false);
    return __builtin_bit_cast(uint32_t, r);
}

// 4 KiB global -> LDS as four 1 KiB instructions, 16 bytes per lane: byte 1024 q + 16 lane of the source
// lands at the same offset of lds_part.  The four share one address pair and differ in the immediate.
__device__ inline void copy_4k_to_lds(const char *src_lane, char *lds_part)
{
    const auto *g = (const __attribute__((address_space(1))) void *)src_lane;
    auto *l = (__attribute__((address_space(3))) void *)lds_part;
    __builtin_amdgcn_global_load_lds(g, l, 16, 0, 0);
    __builtin_amdgcn_global_load_lds(g, l, 16, 1024, 0);
    __builtin_amdgcn_global_load_lds(g, l, 16, 2048, 0);
    __builtin_amdgcn_global_load_lds(g, l, 16, 3072, 0);
}

// Rows 16 HF .. 16 HF + 15 of a wavefront's 32 x 128 block of bf16 query rows, from the lanes that loaded them whole
// (a_jj: 16-byte chunk lane % 16 of row 4 jj + lane / 16 of the half) to the lanes that use them as matrix operands (lane
// (n, h) of row n: chunks 2 kb + h and 8 + 2 kb + h), through 4 KiB of LDS that belongs to this wavefront alone.
// The chunks of row r sit permuted by r % 16, so that both the writes and the reads cover all banks.
template <int HF>
__device__ __forceinline__ void q_turn_half(char *qst, const uint4 &a0, const uint4 &a1, const uint4 &a2, const uint4 &a3, int lane, int n,
                                            int h, uint4 (&qlo)[4], uint4 (&qhi)[4])
{
    {
        const int r0 = lane >> 4, c = lane & 15;      // a_jj: chunk c of row 4 jj + r0 of the half
        *reinterpret_cast<uint4 *>(qst + (r0 + 0) * 256 + ((c ^ (r0 + 0)) * 16)) = a0;
        *reinterpret_cast<uint4 *>(qst + (r0 + 4) * 256 + ((c ^ (r0 + 4)) * 16)) = a1;
        *reinterpret_cast<uint4 *>(qst + (r0 + 8) * 256 + ((c ^ (r0 + 8)) * 16)) = a2;
        *reinterpret_cast<uint4 *>(qst + (r0 + 12) * 256 + ((c ^ (r0 + 12)) * 16)) = a3;
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront", "local");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront", "local");
    const int n16 = n & 15;
#pragma unroll
    for (int kb = 0; kb < 4; ++kb) {
        const uint4 lo = *reinterpret_cast<const uint4 *>(qst + n16 * 256 + (((2 * kb + h) ^ n16) * 16));
        const uint4 hi = *reinterpret_cast<const uint4 *>(qst + n16 * 256 + (((8 + 2 * kb + h) ^ n16) * 16));
        if ((n >> 4) == HF) {
            qlo[kb] = lo;
            qhi[kb] = hi;
        }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront", "local");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront", "local");
}

struct TileDesc {
    int kind;      // 0: cached prefix keys, 1: the suffix keys of sorted query q
    int key0;      // first key of the tile (index inside the prefix / inside the query's suffix)
    int q;         // sorted query (kind 1)
    int page0;     // first suffix page of the tile (kind 1)
    int page_last; // last suffix page of the query (kind 1)
};

// Decode (SubGCache App. A.2: up to 32 generated tokens per query): the blocks behind the tiles of a decode
// step's launch append the step's new token of every query to its suffix pages, K rotated at position
// P + len + step, V as given; 8 lanes per (sorted query, KV head), one 8-channel chunk of each half per lane.
// Nothing in the same launch reads those pages (the tiles of a decode step only read the cluster's cache).
__device__ inline void append_new_tokens(const AttnArgs &a, int blk)
{
    const int unit = blk * ((int)blockDim.x >> 3) + ((int)threadIdx.x >> 3), cc = (int)threadIdx.x & 7;
    const int Hkv = a.n_kv_heads;
    const int sq = unit / Hkv, hk = unit - sq * Hkv;
    if (sq >= a.n_append) return;
    const int j = a.sq_len[sq] + a.pos_shift;
    const int pos = a.cl_prefix_len[a.sq_cluster[sq]] + j;
    const int tok = j % kPageTokens;
    char *kp = const_cast<char *>(a.spool) + (int64_t)(a.sq_page0[sq] + j / kPageTokens) * 2 * Hkv * PART_BYTES + (int64_t)hk * PART_BYTES;
    char *vp = kp + (int64_t)Hkv * PART_BYTES;
    const int64_t row = ((int64_t)a.sq_query[sq] * Hkv + hk) * D;
    const uint16_t *kg = static_cast<const uint16_t *>(a.k) + row, *vg = static_cast<const uint16_t *>(a.v) + row;
    const uint4 k1 = *reinterpret_cast<const uint4 *>(kg + cc * 8), k2 = *reinterpret_cast<const uint4 *>(kg + D / 2 + cc * 8);
    const uint4 v1 = *reinterpret_cast<const uint4 *>(vg + cc * 8), v2 = *reinterpret_cast<const uint4 *>(vg + D / 2 + cc * 8);
    const uint32_t w1[4] = {k1.x, k1.y, k1.z, k1.w}, w2[4] = {k2.x, k2.y, k2.z, k2.w};
    uint32_t o1[4], o2[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        float x1[2] = {__uint_as_float(w1[i] << 16), __uint_as_float(w1[i] & 0xFFFF0000u)};
        float x2[2] = {__uint_as_float(w2[i] << 16), __uint_as_float(w2[i] & 0xFFFF0000u)};
        if (a.rope) {
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                const float2 cs = a.rope[(int64_t)pos * (D / 2) + cc * 8 + 2 * i + e];
                const float p = x1[e], q = x2[e];
                x1[e] = p * cs.x - q * cs.y;
                x2[e] = q * cs.x + p * cs.y;
            }
        }
        o1[i] = pack2_f16(x1[0], x1[1]);       // keys are kept as binary16
        o2[i] = pack2_f16(x2[0], x2[1]);
    }
    *reinterpret_cast<uint4 *>(kp + (int64_t)k_page_index(tok, cc * 8) * 2) = make_uint4(o1[0], o1[1], o1[2], o1[3]);
    *reinterpret_cast<uint4 *>(kp + (int64_t)k_page_index(tok, D / 2 + cc * 8) * 2) = make_uint4(o2[0], o2[1], o2[2], o2[3]);
    const uint32_t y1[4] = {v1.x, v1.y, v1.z, v1.w}, y2[4] = {v2.x, v2.y, v2.z, v2.w};
    uint16_t *vq = reinterpret_cast<uint16_t *>(vp);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        vq[v_page_index(tok, cc * 8 + i)] = (uint16_t)(y1[i >> 1] >> (16 * (i & 1)));
        vq[v_page_index(tok, D / 2 + cc * 8 + i)] = (uint16_t)(y2[i >> 1] >> (16 * (i & 1)));
    }
}

// QK8 (fp8 cache only): the first product runs on the cache's e4m3 codes as they are (v_mfma_scale_f32_32x32x64_f8f6f4,
// twice the bf16 rate): the rotated, scaled query row is quantised to e4m3 with a power-of-two scale of its own, which
// the instruction applies to the row's products in hardware, so scores come out in the same units as on the other
// paths.  K codes then go to LDS as they are (2 KiB per page part); V is still widened to bf16 for the second product.
template <int NW, int MI, bool KV_FP8, int MODE, bool QK8>
__global__ void __launch_bounds__(NW * 64, (NW == 4 && MI == 1) ? 2 : 1) attn_mfma_kernel(const AttnArgs a)
{
    static_assert(!QK8 || (KV_FP8 && MI == 1 && NW == 4), "the fp8 first product needs an fp8 cache");
    if (MODE == MODE_SUFFIX && (int)blockIdx.x >= a.n_tiles) {
        append_new_tokens(a, (int)blockIdx.x - a.n_tiles);
        return;
    }
    extern __shared__ __attribute__((aligned(1024))) char smem[];
    int2 *const qinfo = reinterpret_cast<int2 *>(smem + LDS_TILE_BYTES);   // (suffix length, first suffix page)

    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63;
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
    const int n = lane & 31, h = lane >> 5;
    const int Hq = a.n_q_heads, Hkv = a.n_kv_heads, g = a.group;

    // ---- which tile ----
    Tile t = a.tiles[blockIdx.x];
    if (t.n_rows == 0) return;
    // where the rows come from and go to: the batch's packed arrays, or (prefix mode) the job's
    const void *q_base = a.q;
    void *o_base = a.o;
    float *lse_base = a.lse;
    int64_t lse_stride = a.lse_stride;
    if (MODE == MODE_PREFIX) {
        const PrefixJob &job = a.jobs[__builtin_amdgcn_readfirstlane(t.tok_base)];
        q_base = job.q;
        o_base = job.o;
        lse_base = job.lse;
        lse_stride = t.prefix_len;
        t.tok_base = 0;
    }
    // decode tiles cover one key range of the cluster's cache: own output set, positions continue behind ALL cached keys
    const int key_range = __builtin_amdgcn_readfirstlane(t.pad) >> 24;
    const int pos_extra = __builtin_amdgcn_readfirstlane(t.pad) & 0xFFFFFF;
    if (MODE == MODE_SUFFIX) {
        o_base = static_cast<char *>(o_base) + key_range * a.split_o_bytes;
        if (lse_base) lse_base += key_range * a.split_lse_elems;
    }
    // everything that steers the tile loop is made explicitly wave-uniform (scalar registers)
    const int cluster = __builtin_amdgcn_readfirstlane(t.cluster), hk = __builtin_amdgcn_readfirstlane(t.hk);
    t.row0 = __builtin_amdgcn_readfirstlane(t.row0);
    t.n_rows = __builtin_amdgcn_readfirstlane(t.n_rows);
    const int P = __builtin_amdgcn_readfirstlane(t.prefix_len);
    const int n_pages = (P + kPageTokens - 1) / kPageTokens;
    const int32_t *pt = a.page_table + __builtin_amdgcn_readfirstlane(t.pt_off);
    const int tok_base = __builtin_amdgcn_readfirstlane(t.tok_base);
    const int last_row = t.row0 + t.n_rows - 1;
    const int sq_lo = __builtin_amdgcn_readfirstlane(t.sq_lo), sq_hi = __builtin_amdgcn_readfirstlane(t.sq_hi);
    const int last_qpos = __builtin_amdgcn_readfirstlane(t.last_qpos);

    // ---- copy machinery ----------------------------------------------------------------------------
    // A tile is 8 parts: K of its 4 pages, then V of its 4 pages; a part is 4 KiB of bf16 (2 KiB of fp8
    // codes that widen to 4 KiB).  With 4 wavefronts, wavefront w moves K and V of page w; with 8, wavefronts
    // 0..3 move K of page w and 4..7 move V of page w - 4.  A part's source is a scalar base (pool base +
    // page offset) plus a per-lane offset fixed for the launch; page offsets travel as 32-bit counts of 256
    // bytes, a step ahead, in a vector register (lane j < 4 holds page j of the tile) and become scalars by
    // readlane, so no copy ever waits on a page-table load.
    const int my_page = wave_u & 3;
    const bool moves_k = NW == 4 || wave_u < 4, moves_v = NW == 4 || wave_u >= 4;
    const char *cache_base = a.pool.pool + (int64_t)a.layer * a.pool.layer_bytes + (int64_t)hk * a.pool.head_part_bytes;
    const uint32_t cache_v_off = (uint32_t)(Hkv * a.pool.head_part_bytes);
    const uint32_t cache_page_256 = (uint32_t)(a.pool.page_bytes >> 8);
    const char *spool_base = a.spool + (int64_t)hk * PART_BYTES;
    const uint32_t spool_v_off = (uint32_t)Hkv * PART_BYTES;
    const uint32_t spool_page_256 = (2u * spool_v_off) >> 8;
    // fp8 cache only: codes on their way to LDS.  A 2 KiB part is fetched as four runs of 512 codes, 8 per lane; widened,
    // a lane's 8 codes are 16 bytes at 16 * lane of the run's 1 KiB image, so the stores cover all banks.
    uint2 stage[8];      // [K runs 0..3, V runs 0..3]
    bool staged_k = false, staged_v = false;

    // Page indices past the last page are clamped to it: such keys are masked out of the scores, and what
    // they multiply in the second product is finite cache content times a zero weight.
    auto cache_page_ids = [&](int kt) __attribute__((always_inline)) -> uint32_t {     // raw page ids; scaled to offsets when used
        if (n_pages == 0) return 0;       // no cached keys: nothing is ever copied from the cache
        return (uint32_t)pt[min(kt * 4 + (lane & 3), n_pages - 1)];
    };
    const uint32_t lane16 = lane * 16;
    // Copies K of one tile (page offsets poff_k, into kdst) and / or V of one tile (poff_v, into vdst); a null
    // destination skips that half.
    auto issue_copy_bf16 = [&](uint32_t poff_k, char *kdst, uint32_t poff_v, char *vdst, const char *base, uint32_t v_off) __attribute__((always_inline)) {
        if (moves_k && kdst) {
            const uint32_t off256 = __builtin_amdgcn_readlane(poff_k, my_page);
            copy_4k_to_lds(base + ((uint64_t)off256 << 8) + lane16, kdst + my_page * PART_BYTES);
        }
        if (moves_v && vdst) {
            const uint32_t off256 = __builtin_amdgcn_readlane(poff_v, my_page);
            copy_4k_to_lds(base + ((uint64_t)off256 << 8) + v_off + lane16, vdst + my_page * PART_BYTES);
        }
    };
    char *kdst_codes = nullptr;      // QK8: where the next K tile's codes go
    auto issue_load_fp8 = [&](uint32_t poff_k, bool want_k, uint32_t poff_v, bool want_v) __attribute__((always_inline)) {
        staged_k = moves_k && want_k;
        staged_v = moves_v && want_v;
        if (staged_k) {
            const uint32_t off256 = __builtin_amdgcn_readlane(poff_k, my_page);
            const char *src = cache_base + ((uint64_t)off256 << 8) + lane16;
            if (QK8) {      // the codes as they are, straight into LDS (kdst_codes: set by the caller)
                const auto *g = (const __attribute__((address_space(1))) void *)src;
                auto *l = (__attribute__((address_space(3))) void *)(kdst_codes + my_page * K8_PART_STRIDE);
                __builtin_amdgcn_global_load_lds(g, l, 16, 0, 0);
                __builtin_amdgcn_global_load_lds(g, l, 16, 1024, 0);
                staged_k = false;
            } else {
                const char *src8 = cache_base + ((uint64_t)off256 << 8) + lane * 8;
#pragma unroll
                for (int r = 0; r < 4; ++r) stage[r] = *reinterpret_cast<const uint2 *>(src8 + r * 512);
            }
        }
        if (staged_v) {
            const uint32_t off256 = __builtin_amdgcn_readlane(poff_v, my_page);
            const char *src8 = cache_base + ((uint64_t)off256 << 8) + cache_v_off + lane * 8;
#pragma unroll
            for (int r = 0; r < 4; ++r) stage[4 + r] = *reinterpret_cast<const uint2 *>(src8 + r * 512);
        }
    };
    // 8 codes -> 8 16-bit floats = 16 bytes
    auto widen_to_lds = [&](const uint2 &codes, char *dst, auto f16_tag) __attribute__((always_inline)) {
        constexpr bool F = decltype(f16_tag)::value;
        uint4 o;
        o.x = fp8x2_to_16x2<F>(codes.x, false); o.y = fp8x2_to_16x2<F>(codes.x, true);
        o.z = fp8x2_to_16x2<F>(codes.y, false); o.w = fp8x2_to_16x2<F>(codes.y, true);
        *reinterpret_cast<uint4 *>(dst) = o;
    };
    // Writes what the last issue_load_fp8 staged; a staged half is written once, and only to a real buffer.
    auto store_fp8 = [&](char *kdst, char *vdst) __attribute__((always_inline)) {
        if (staged_k && kdst) {
#pragma unroll
            for (int r = 0; r < 4; ++r) widen_to_lds(stage[r], kdst + my_page * PART_BYTES + r * 1024 + lane * 16, std::true_type{});
        }
        if (staged_v && vdst) {
#pragma unroll
            for (int r = 0; r < 4; ++r) widen_to_lds(stage[4 + r], vdst + my_page * PART_BYTES + r * 1024 + lane * 16, std::false_type{});
        }
        staged_k = false;
        staged_v = false;
    };
    // K of one cached tile and / or V of another: kdst / vdst null = none
    auto fetch_cache = [&](uint32_t ids_k, char *kdst, uint32_t ids_v, char *vdst) __attribute__((always_inline)) {
        if (KV_FP8) {
            kdst_codes = kdst;
            issue_load_fp8(ids_k * cache_page_256, kdst != nullptr, ids_v * cache_page_256, vdst != nullptr);
        } else
            issue_copy_bf16(ids_k * cache_page_256, kdst, ids_v * cache_page_256, vdst, cache_base, cache_v_off);
    };
    auto land_cache = [&](char *kdst, char *vdst) __attribute__((always_inline)) {   // make what was fetched visible in LDS (before the barrier)
        if (KV_FP8) store_fp8(kdst, vdst);
        __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): direct copies have landed
    };
    char *const kbuf0 = smem, *const vbuf0 = smem + 2 * HALF_BYTES;
    auto kbuf_of = [&](int i) __attribute__((always_inline)) -> char * { return kbuf0 + (i & 1) * HALF_BYTES; };
    auto vbuf_of = [&](int i) __attribute__((always_inline)) -> char * { return vbuf0 + (i & 1) * HALF_BYTES; };

    // The first cached tiles are requested before anything else: page ids now, the copies (bf16 cache) as soon
    // as the ids are there, so that they travel while Q is loaded and rotated.
    const int n_cache_keys = (MODE == MODE_SUFFIX) ? P : min(P, last_row / g + 1);
    const int n_kt = (n_cache_keys + BN - 1) / BN;
    // page ids of tiles 0, 1, 2 come with the tile record (lane j < 4 holds page j of a tile); later these
    // hold the ids of tiles kt + 1 and kt + 2
    auto spread4 = [&](const int32_t *p4) __attribute__((always_inline)) -> uint32_t {
        const int p0 = __builtin_amdgcn_readfirstlane(p4[0]), p1 = __builtin_amdgcn_readfirstlane(p4[1]);
        const int p2 = __builtin_amdgcn_readfirstlane(p4[2]), p3 = __builtin_amdgcn_readfirstlane(p4[3]);
        const int lo = (lane & 1) ? p1 : p0, hi = (lane & 1) ? p3 : p2;
        return (uint32_t)((lane & 2) ? hi : lo);
    };
    const uint32_t ids0 = spread4(t.first_pages);
    uint32_t ids1 = spread4(t.first_pages + 4), ids2 = spread4(t.first_pages + 8);
    float k_scale = 1.f, v_scale = 1.f;
    if (KV_FP8) {
        const float *sc = a.kv_scale + ((int64_t)cluster * a.n_layers + a.layer) * 2 * Hkv;
        k_scale = sc[hk];
        v_scale = sc[Hkv + hk];
    }
    // Scores are kept in log2 units.  Q carries the factor for cached keys; scores against the (unquantised)
    // suffix keys of the batch are brought to the same units by self_ratio.
    const float c_cache = a.scale_log2e * k_scale;
    const float self_ratio = KV_FP8 ? 1.0f / k_scale : 1.0f;

    // ---- per-lane row bookkeeping ----
    const bool inline_queries = MODE == MODE_SUFFIX && __builtin_amdgcn_readfirstlane(t.n_q) <= kTileQueries;
    int tq_tok0[kTileQueries], tq_src0[kTileQueries];
#pragma unroll
    for (int k = 0; k < kTileQueries; ++k) {
        tq_tok0[k] = __builtin_amdgcn_readfirstlane(t.q[k].tok0);
        tq_src0[k] = __builtin_amdgcn_readfirstlane(t.q[k].src0);
    }
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
            if (inline_queries) {        // which of the (at most 4) queries of the tile record the token belongs to
                const bool ge1 = tau >= tq_tok0[1], ge2 = tau >= tq_tok0[2], ge3 = tau >= tq_tok0[3];
                const int first = ge3 ? tq_tok0[3] : ge2 ? tq_tok0[2] : ge1 ? tq_tok0[1] : tq_tok0[0];
                const int src0 = ge3 ? tq_src0[3] : ge2 ? tq_src0[2] : ge1 ? tq_src0[1] : tq_src0[0];
                qpos[mi] = tau - first;
                src_tok[mi] = src0 + qpos[mi];
                sq[mi] = sq_lo + (int)ge1 + (int)ge2 + (int)ge3;
            } else {
                const TokInfo ti = a.tok_info[tau];
                src_tok[mi] = ti.src;
                qpos[mi] = ti.qpos;
                sq[mi] = ti.sq;
            }
            lim[mi] = P;
        } else {
            src_tok[mi] = tk;
            qpos[mi] = tk;
            sq[mi] = 0;
            lim[mi] = tk + 1;
        }
        io_row[mi] = ((int64_t)src_tok[mi] * Hq + head[mi]) * D;
    }
    // wave-uniform bounds: visible cached keys, and the sorted queries of this wave's rows.  Rows are in
    // sorted order (and rows past the tile's end repeat its last row), so the first lane holds the minima
    // and lane 31 of the last row block the maxima.
    const int lim_min = __builtin_amdgcn_readlane(lim[0], 0), lim_max = __builtin_amdgcn_readlane(lim[MI - 1], 31);
    const int wsq_min = __builtin_amdgcn_readlane(sq[0], 0), wsq_max = __builtin_amdgcn_readlane(sq[MI - 1], 31);

    if (!KV_FP8 && n_kt > 0) {
        fetch_cache(ids0, kbuf_of(0), ids0, vbuf_of(0));
        if (n_kt > 1) fetch_cache(ids1, kbuf_of(1), 0, nullptr);
    }
    // ---- Q: load, rotate at position P + qpos (suffix) / qpos (prefix), keep as B operands ----
    // All loads of the phase (Q row halves, then the rotation table entries) are issued before any of them is
    // used, so the phase costs one memory round trip and not one per channel group.
    f16x8 qf[MI][8];
    i32x8 q8[2];            // QK8: the row as e4m3 codes, operand t = channels 64 t .. 64 t + 63 in the order kc_block reads keys
    int qscale = 127;       // QK8: the row's scale as a biased power-of-two exponent (what the scaled product takes)
    {
        uint4 qlo[MI][4], qhi[MI][4];
        float4 cs[MI][4][4];            // (cos, sin) of two channels per entry
        if (NW == 4 && !KV_FP8) {       // (with an fp8 cache the registers for it are not there, and prompts are long)
            // The operand layout wants 16-byte pieces of 32 different rows per instruction.  Loaded that way the
            // requests are 32 scattered 32-byte runs each; instead instruction j fetches rows 4 j .. 4 j + 3 whole
            // (lane = 16-byte chunk lane % 16 of row 4 j + lane / 16), and the wavefront turns the block by
            // passing it, 16 rows at a time, through its 4 KiB share of the V buffer that nothing uses before the
            // first step (chunks of row r permuted by r % 16: writes and reads cover all banks).
            char *const qst = smem + 3 * HALF_BYTES + wave * 4096;
#pragma unroll
            for (int mi = 0; mi < MI; ++mi) {
                const int row_index = (int)(io_row[mi] / D);        // src_tok * Hq + head of this lane's row
                auto whole_row_chunk = [&](int j) __attribute__((always_inline)) -> uint4 {
                    const int64_t ro = (int64_t)__shfl(row_index, 4 * j + (lane >> 4)) * D;
                    return *reinterpret_cast<const uint4 *>(static_cast<const uint16_t *>(q_base) + ro + (lane & 15) * 8);
                };
                const uint4 r0 = whole_row_chunk(0), r1 = whole_row_chunk(1), r2 = whole_row_chunk(2), r3 = whole_row_chunk(3);
                const uint4 r4 = whole_row_chunk(4), r5 = whole_row_chunk(5), r6 = whole_row_chunk(6), r7 = whole_row_chunk(7);
                q_turn_half<0>(qst, r0, r1, r2, r3, lane, n, h, qlo[mi], qhi[mi]);
                q_turn_half<1>(qst, r4, r5, r6, r7, lane, n, h, qlo[mi], qhi[mi]);
            }
        } else {
#pragma unroll
            for (int mi = 0; mi < MI; ++mi) {
                const uint16_t *qrow = static_cast<const uint16_t *>(q_base) + io_row[mi];
#pragma unroll
                for (int kb = 0; kb < 4; ++kb) {
                    const int c0 = kb * 16 + h * 8;
                    qlo[mi][kb] = *reinterpret_cast<const uint4 *>(qrow + c0);
                    qhi[mi][kb] = *reinterpret_cast<const uint4 *>(qrow + 64 + c0);
                }
            }
        }
        const bool rotate = a.rope != nullptr;
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
            for (int kb = 0; kb < 4; ++kb)
#pragma unroll
                for (int i = 0; i < 4; ++i) cs[mi][kb][i] = make_float4(1.f, 0.f, 1.f, 0.f);
        if (rotate) {
#pragma unroll
            for (int mi = 0; mi < MI; ++mi) {
                const int pos = (MODE == MODE_SUFFIX ? P + pos_extra + a.pos_shift : 0) + qpos[mi];
#pragma unroll
                for (int kb = 0; kb < 4; ++kb) {
                    const float4 *tab = reinterpret_cast<const float4 *>(a.rope + (int64_t)pos * 64 + kb * 16 + h * 8);
#pragma unroll
                    for (int i = 0; i < 4; ++i) cs[mi][kb][i] = tab[i];
                }
            }
        }
#pragma unroll
        for (int mi = 0; mi < MI; ++mi) {
#pragma unroll
            for (int kb = 0; kb < 4; ++kb) {
                const uint32_t wl[4] = {qlo[mi][kb].x, qlo[mi][kb].y, qlo[mi][kb].z, qlo[mi][kb].w};
                const uint32_t wh[4] = {qhi[mi][kb].x, qhi[mi][kb].y, qhi[mi][kb].z, qhi[mi][kb].w};
                float x1[8], x2[8];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const float a0 = __uint_as_float(wl[i] << 16), a1 = __uint_as_float(wl[i] & 0xFFFF0000u);
                    const float b0 = __uint_as_float(wh[i] << 16), b1 = __uint_as_float(wh[i] & 0xFFFF0000u);
                    const float4 t4 = cs[mi][kb][i];
                    x1[2 * i] = a0 * t4.x - b0 * t4.y;
                    x2[2 * i] = b0 * t4.x + a0 * t4.y;
                    x1[2 * i + 1] = a1 * t4.z - b1 * t4.w;
                    x2[2 * i + 1] = b1 * t4.z + a1 * t4.w;
                }
#pragma unroll
                for (int i = 0; i < 8; ++i) {      // the score scale (log2 units, cached-K scale included) rides on Q
                    qf[mi][kb][i] = (_Float16)(x1[i] * c_cache);
                    qf[mi][kb + 4][i] = (_Float16)(x2[i] * c_cache);
                }
            }
        }
        if constexpr (QK8) {
            // The row as e4m3 codes with one power-of-two scale: largest magnitude of the row (both lanes of the pair)
            // = m 2^x with m in [0.5, 1); values times 2^(8 - x) lie below 256 (the format reaches 448), rounded to
            // nearest even by the conversion instruction.
            float amax = 0.f;
#pragma unroll
            for (int kb = 0; kb < 8; ++kb)
#pragma unroll
                for (int i = 0; i < 8; ++i) amax = fmaxf(amax, fabsf((float)qf[0][kb][i]));
            amax = half_max(amax);
            int e = __builtin_amdgcn_frexp_expf(amax) - 8;
            e = amax > 0.f ? max(-120, min(e, 120)) : 0;
            qscale = 127 + e;
            const float down = __uint_as_float((uint32_t)(127 - e) << 23);      // 2^-e
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int pc = 0; pc < 4; ++pc) {
                    const f16x8 v = qf[0][4 * t + pc];
                    int w0 = 0, w1 = 0;
                    w0 = __builtin_amdgcn_cvt_pk_fp8_f32((float)v[0] * down, (float)v[1] * down, w0, false);
                    w0 = __builtin_amdgcn_cvt_pk_fp8_f32((float)v[2] * down, (float)v[3] * down, w0, true);
                    w1 = __builtin_amdgcn_cvt_pk_fp8_f32((float)v[4] * down, (float)v[5] * down, w1, false);
                    w1 = __builtin_amdgcn_cvt_pk_fp8_f32((float)v[6] * down, (float)v[7] * down, w1, true);
                    q8[t][2 * pc] = w0;
                    q8[t][2 * pc + 1] = w1;
                }
        }
    }

    // ---- the queries this tile touches (suffix mode): lengths and first pages into LDS ----
    // (read by the own-suffix tile iterator after the first barrier; placed after the Q loads so that the
    // table look-ups of the rare many-queries case do not sit in front of them)
    if (MODE == MODE_SUFFIX) {
        if (inline_queries) {
            if (tid < kTileQueries) {
                const int len = tid == 0 ? t.q[0].len : tid == 1 ? t.q[1].len : tid == 2 ? t.q[2].len : t.q[3].len;
                const int pg0 = tid == 0 ? t.q[0].page0 : tid == 1 ? t.q[1].page0 : tid == 2 ? t.q[2].page0 : t.q[3].page0;
                qinfo[tid] = make_int2(len, pg0);
            }
        } else {
            for (int i = tid; i <= sq_hi - sq_lo && i < MAX_TILE_QUERIES; i += NW * 64)
                qinfo[i] = make_int2(a.sq_len[sq_lo + i], a.sq_page0[sq_lo + i]);
        }
    }

    // ---- accumulators ----
    // m_ref is the reference maximum of the row's softmax; the score products start from -m_ref (neg_ref, the
    // same value in all 16 accumulator registers of a lane, which all belong to one row), so finished scores
    // are already relative to it.  seen: the row has met at least one visible key.
    // (With 64 rows per wavefront the registers for neg_ref are not there: FOLD is off, the products start
    // from zero and the weights subtract m_ref themselves.)
    constexpr bool FOLD = MI == 1;
    f32x16 oacc[MI][4], neg_ref[MI];
    float m_ref[MI], l_part[MI];
    bool seen[MI];
#pragma unroll
    for (int mi = 0; mi < MI; ++mi) {
        m_ref[mi] = 0.f;
        l_part[mi] = 0.f;
        seen[mi] = false;
#pragma unroll
        for (int r = 0; r < 16; ++r) neg_ref[mi][r] = 0.f;
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) oacc[mi][db][r] = 0.f;
    }
    bool fresh = true;     // no tile processed yet by this wavefront

    // Per-lane LDS offsets of the operand blocks.  K block (nb, kb): lane (m, hh) reads key m of the 32-key
    // group nb (page 2 nb + m / 16, token m % 16), channels kb * 16 + hh * 8 .. + 7.  Each 16-lane group
    // reads 256 contiguous bytes, which is conflict-free.  V block (pg, db) is 1 KiB contiguous.
    const int lane_koff = ((n >> 4) * PART_BYTES) + (h * kPageTokens + (n & 15)) * 16;
    const int lane_voff = lane * 16;

    // ---- the pieces of one 32-key half step ---------------------------------------------------------
    // A 64-key tile is worked on as two 32-key halves (nb = 0, 1): half nb is K blocks 8 nb .. 8 nb + 7 of
    // the first product (one per 16 channels) and V blocks 8 nb .. 8 nb + 7 of the second (pages 2 nb and
    // 2 nb + 1, four 32-channel groups each).  LDS operand blocks are read through a rolling window of 8
    // register sets: each matrix instruction is followed by the read that refills the slot it used with a
    // block of the NEXT product, so that product never waits on LDS.
    bf16x8 frag[8];
    uint32_t pf[MI][2][4];     // weights of one half as bf16 pairs: [row block][page of the half][register pair]
    float psum[MI];
    auto k_block = [&](const char *kbuf, int nb, int kb) __attribute__((always_inline)) {
        return *reinterpret_cast<const bf16x8 *>(kbuf + lane_koff + nb * 2 * PART_BYTES + kb * 512);
    };
    auto v_block = [&](const char *vbuf, int nb, int i) __attribute__((always_inline)) {
        return *reinterpret_cast<const bf16x8 *>(vbuf + lane_voff + (nb * 8 + i) * 1024);
    };
    // Cached keys.  QK8: the 64-channel operand of the fp8 product is eight 8-byte pieces (lane (m, hh): key m, channels
    // 64 t + 16 p + 8 hh .. + 7 for p = 0..3; the contraction does not care which of its 64 slots a channel takes as
    // long as the query operand uses the same ones); window slot i < 4 holds pieces 2 (i % 2), 2 (i % 2) + 1 of operand
    // t = i / 2, slots 4..7 are not used by this product.
    const int lane_k8off = (n >> 4) * K8_PART_STRIDE + (h * kPageTokens + (n & 15)) * 8;
    auto kc_block = [&](const char *kbuf, int nb, int i) __attribute__((always_inline)) -> bf16x8 {
        if constexpr (QK8) {
            if (i >= 4) return frag[i];
            const char *p = kbuf + lane_k8off + nb * 2 * K8_PART_STRIDE + (4 * (i >> 1) + 2 * (i & 1)) * 256;
            const uint2 a0 = *reinterpret_cast<const uint2 *>(p), a1 = *reinterpret_cast<const uint2 *>(p + 256);
            const u32x4 w = {a0.x, a0.y, a1.x, a1.y};
            return __builtin_bit_cast(bf16x8, w);
        } else {
            return k_block(kbuf, nb, i);
        }
    };
    auto no_refill = [&](int) __attribute__((always_inline)) {};
    const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    // S^T = K Q^T - m_ref for the half whose K blocks the window holds; slot kb is refilled by refill(kb).
    auto qk_half = [&](f32x16 (&s)[MI], auto refill) __attribute__((always_inline)) {
#pragma unroll
        for (int kb = 0; kb < 8; ++kb) {
#pragma unroll
            for (int mi = 0; mi < MI; ++mi)
                s[mi] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, frag[kb]), qf[mi][kb], kb == 0 ? (FOLD ? neg_ref[mi] : zero16) : s[mi], 0, 0, 0);
            refill(kb);
        }
    };
    // The same against cached keys.  QK8: two 64-channel products on the codes; the query row's own scale (a power of two)
    // is applied by the instruction, so the scores leave it in the usual units with -m_ref already taken off.
    auto qk_half_cache = [&](f32x16 (&s)[MI], auto refill) __attribute__((always_inline)) {
        if constexpr (QK8) {
            refill(4);
            refill(5);
            refill(6);
            refill(7);
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                const u32x4 lo = __builtin_bit_cast(u32x4, frag[2 * t]), hi = __builtin_bit_cast(u32x4, frag[2 * t + 1]);
                const i32x8 kop = {(int)lo[0], (int)lo[1], (int)lo[2], (int)lo[3], (int)hi[0], (int)hi[1], (int)hi[2], (int)hi[3]};
                s[0] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(kop, q8[t], t == 0 ? neg_ref[0] : s[0], 0, 0, 0, 127, 0, qscale);
                refill(2 * t);
                refill(2 * t + 1);
            }
        } else {
            qk_half(s, refill);
        }
    };
    // O^T += V^T P^T for the half whose V blocks the window holds (slot i = page i / 4, channel group i % 4).
    auto pv_half = [&](auto refill) __attribute__((always_inline)) {
#pragma unroll
        for (int mi = 0; mi < MI; ++mi) l_part[mi] += psum[mi];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int pg = i >> 2, db = i & 3;
#pragma unroll
            for (int mi = 0; mi < MI; ++mi) {
                const u32x4 w = {pf[mi][pg][0], pf[mi][pg][1], pf[mi][pg][2], pf[mi][pg][3]};
                oacc[mi][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag[i], __builtin_bit_cast(bf16x8, w), oacc[mi][db], 0, 0, 0);
            }
            refill(i);
        }
    };
    // Weights of one half from scores relative to the reference maximum: one exp2 per score.
    auto weights = [&](const f32x16 (&s)[MI]) __attribute__((always_inline)) {
        bf16x2 ones;
        ones[0] = (__bf16)1.0f;
        ones[1] = (__bf16)1.0f;
#pragma unroll
        for (int mi = 0; mi < MI; ++mi) {
            float acc = 0.f;
#pragma unroll
            for (int r = 0; r < 16; r += 2) {
                bf16x2 pk;
                pk[0] = (__bf16)__builtin_amdgcn_exp2f(FOLD ? s[mi][r] : s[mi][r] - m_ref[mi]);
                pk[1] = (__bf16)__builtin_amdgcn_exp2f(FOLD ? s[mi][r + 1] : s[mi][r + 1] - m_ref[mi]);
                acc = __builtin_amdgcn_fdot2_f32_bf16(pk, ones, acc, false);   // sum of the ROUNDED weights
                pf[mi][r >> 3][(r & 7) >> 1] = __builtin_bit_cast(uint32_t, pk);
            }
            psum[mi] = acc;
        }
    };
    auto weights_overflow = [&]() __attribute__((always_inline)) {       // wave-uniform: some row's weights of this half summed beyond the limit
        bool bad = false;
#pragma unroll
        for (int mi = 0; mi < MI; ++mi) bad |= !(psum[mi] <= kKeepBelow);    // also catches inf / nan
        return __any(bad);
    };
    // The careful part of a softmax step, run before weights().  Masks the half through keep(mi, j) = "row mi
    // may see key j of the tile" when `masked`; raises the reference maximum to the half's own where that is
    // larger (rows that have seen no key yet take it as it is), rescales the accumulators and re-bases the
    // scores.  Returns nothing; m_ref, neg_ref, seen, l_part, oacc and s are updated.
    auto raise_reference = [&](f32x16 (&s)[MI], const int nb, const bool masked, auto keep) __attribute__((always_inline)) {
#pragma unroll
        for (int mi = 0; mi < MI; ++mi) {
            if (masked) {
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int j = nb * 32 + 8 * (r >> 2) + 4 * h + (r & 3);
                    if (!keep(mi, j)) s[mi][r] = -INFINITY;
                }
            }
            float tmax = s[mi][0];
#pragma unroll
            for (int r = 1; r < 16; ++r) tmax = fmaxf(tmax, s[mi][r]);
            tmax = half_max(tmax);
            const bool has = tmax > -INFINITY;
            if (!FOLD) tmax -= m_ref[mi];                      // relative to m_ref (FOLD: the scores already are)
            const float delta = seen[mi] ? fmaxf(tmax, 0.f) : (has ? tmax : 0.f);     // new m_ref - old m_ref
            if (__any(delta != 0.f)) {
                const float alpha = seen[mi] ? __builtin_amdgcn_exp2f(-delta) : 1.0f;
                m_ref[mi] += delta;
                l_part[mi] *= alpha;
#pragma unroll
                for (int db = 0; db < 4; ++db) {       // one accumulator block at a time keeps the temporaries few
#pragma unroll
                    for (int r = 0; r < 16; ++r) oacc[mi][db][r] *= alpha;
                    if (MI > 1) __builtin_amdgcn_sched_barrier(0);
                }
                if (FOLD) {
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        s[mi][r] -= delta;
                        neg_ref[mi][r] = -m_ref[mi];
                    }
                }
            }
            seen[mi] = seen[mi] || has;
        }
    };
    auto keep_all = [&](int, int) __attribute__((always_inline)) { return true; };
    // fp8 cache only: scores against suffix keys were formed with the cached-K scale on Q; undo it.  mb is the
    // reference maximum the product was started from.
    auto rescale_self = [&](f32x16 (&s)[MI], const float (&mb)[MI]) __attribute__((always_inline)) {
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
            for (int r = 0; r < 16; ++r) s[mi][r] = FOLD ? (s[mi][r] + mb[mi]) * self_ratio - mb[mi] : s[mi][r] * self_ratio;
    };

    // ---- cached prefix tiles, software pipelined ------------------------------------------------------
    // The two products of a half frame its softmax: while the vector unit turns the scores of half j into
    // weights, the matrix unit already forms the scores of half j + 1 (independent instruction streams in
    // one straight-line region); then comes the second product of half j.  So K runs one tile ahead of V:
    // during tile step kt, K of tile kt + 2 and V of tile kt + 1 are copied into LDS while K of tile kt + 1
    // and V of tile kt are read.  At the top of step kt a wavefront holds the scores of (kt, half 0) and, in
    // its window, the K blocks of (kt, half 1).
    const int n_my = min(n_kt, (lim_max + BN - 1) / BN);      // tiles this wavefront has rows for
    f32x16 s0[MI], s1[MI];
    if (n_kt > 0) {
        if (KV_FP8) {      // through registers: one tile's worth at a time
            fetch_cache(ids0, kbuf_of(0), ids0, vbuf_of(0));
            land_cache(kbuf_of(0), vbuf_of(0));
            if (n_kt > 1) {
                fetch_cache(ids1, kbuf_of(1), 0, nullptr);
                land_cache(kbuf_of(1), nullptr);
            }
        } else {
            land_cache(nullptr, nullptr);
        }
    }
    __syncthreads();       // also: qinfo is in LDS
    if (n_my > 0) {
        const char *k0 = kbuf_of(0);
#pragma unroll
        for (int i = 0; i < 8; ++i) frag[i] = kc_block(k0, 0, i);
        qk_half_cache(s0, [&](int i) __attribute__((always_inline)) { frag[i] = kc_block(k0, 1, i); });
    }
    __syncthreads();       // every wavefront has read K of tile 0 before step 0 overwrites it
    // ---- the stream of this row tile's own suffix key tiles ------------------------------------------------
    // Scalar iterator over (query, 64-key tile); a query's LDS record is read when the stream reaches it.  The
    // first tile is requested during the last cached step, into the buffers that step leaves free.
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
    auto fetch_self = [&](const TileDesc &d, char *kdst, char *vdst) __attribute__((always_inline)) {
        const uint32_t po = (uint32_t)min(d.page0 + (lane & 3), d.page_last) * spool_page_256;
        issue_copy_bf16(po, kdst, po, vdst, spool_base, spool_v_off);
    };
    TileDesc cur = {1, 0, 0, 0, 0}, nxt = {1, 0, 0, 0, 0};
    bool have = false, more = false;
    if (MODE == MODE_SUFFIX && !a.skip_self) SGC_NEXT_SELF(have, cur);      // qinfo is visible since the barriers above

    // One part's copy: per-lane source address and LDS destination.  Issued as four 1 KiB instructions that
    // the steady-state step spreads between its matrix instructions, so that a wavefront never sits on a
    // full memory-instruction queue while the matrix unit idles.
    struct PartCopy {
        const char *src;
        char *dst;
    };
    auto cache_part = [&](bool is_v, uint32_t ids, char *dst_half) __attribute__((always_inline)) -> PartCopy {
        const uint32_t off256 = (uint32_t)__builtin_amdgcn_readlane(ids, my_page) * cache_page_256;
        return {cache_base + ((uint64_t)off256 << 8) + (is_v ? cache_v_off : 0u) + lane16, dst_half + my_page * PART_BYTES};
    };
    auto copy_quarter = [&](const PartCopy &pc, int slot) __attribute__((always_inline)) {     // slot 0, 2, 4, 6 -> quarter 0..3; odd slots: nothing
        const auto *gp = (const __attribute__((address_space(1))) void *)pc.src;
        auto *lp = (__attribute__((address_space(3))) void *)pc.dst;
        switch (slot) {
            case 0: __builtin_amdgcn_global_load_lds(gp, lp, 16, 0, 0); break;
            case 2: __builtin_amdgcn_global_load_lds(gp, lp, 16, 1024, 0); break;
            case 4: __builtin_amdgcn_global_load_lds(gp, lp, 16, 2048, 0); break;
            case 6: __builtin_amdgcn_global_load_lds(gp, lp, 16, 3072, 0); break;
            default: break;
        }
    };
    // Step kt.  spread (a true_type / false_type tag): issue this step's copies between the matrix
    // instructions (needs a bf16 cache, both copies due and this wavefront computing) or at the top.
    auto cache_step = [&](const int kt, auto spread_tag) __attribute__((always_inline)) {
        constexpr bool spread = decltype(spread_tag)::value;
        char *kd = kt + 2 < n_kt ? kbuf_of(kt) : nullptr;
        char *vd = kt + 1 < n_kt ? vbuf_of(kt + 1) : nullptr;
        const uint32_t ids3 = cache_page_ids(kt + 3);    // issued before the copies, used a step later
        PartCopy first = {nullptr, nullptr}, second = {nullptr, nullptr};
        if (spread) {
            if (NW == 4) {
                first = cache_part(true, ids1, vd);      // V of tile kt + 1 is needed first
                second = cache_part(false, ids2, kd);
            } else {
                first = moves_v ? cache_part(true, ids1, vd) : cache_part(false, ids2, kd);
            }
        } else {
            if (kd || vd) fetch_cache(ids2, kd, ids1, vd);
            if (MODE == MODE_SUFFIX && kt == n_kt - 1 && have) fetch_self(cur, kbuf_of(kt), vbuf_of(kt + 1));
        }
        ids1 = ids2;
        ids2 = ids3;
        if (spread || MODE == MODE_SUFFIX || kt < n_my) {  // some row of this wave still sees keys of this tile
            const int key0 = kt * BN;
            const bool masked = key0 + BN > lim_min;
            const bool careful = masked || fresh;
            // Past this wave's last tile the "next" scores are formed from whatever the other K buffer holds
            // and never used; this keeps the step free of branches around the matrix instructions.
            const char *kn = kbuf_of(kt + 1), *vc = vbuf_of(kt);
            auto keep = [&](int mi, int j) __attribute__((always_inline)) { return key0 + j < lim[mi]; };
            // A reference raised after the next half's scores were started must be applied to those as well.
            auto redo = [&](f32x16 (&sc)[MI], f32x16 (&sn)[MI], int nb) __attribute__((always_inline)) {
                float before[MI];
#pragma unroll
                for (int mi = 0; mi < MI; ++mi) before[mi] = m_ref[mi];
                raise_reference(sc, nb, false, keep_all);
                weights(sc);
#pragma unroll
                for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        if (FOLD) sn[mi][r] -= m_ref[mi] - before[mi];
            };
            // half 0
            if (careful) raise_reference(s0, 0, masked, keep);
            qk_half_cache(s1, [&](int i) __attribute__((always_inline)) {
                frag[i] = v_block(vc, 0, i);
                if (spread) copy_quarter(first, i);
            });
            weights(s0);
            if (weights_overflow()) redo(s0, s1, 0);
            pv_half([&](int i) __attribute__((always_inline)) {
                frag[i] = kc_block(kn, 0, i);
                if (spread && NW == 4) copy_quarter(second, i);
            });
            // half 1
            if (careful) raise_reference(s1, 1, masked, keep);
            qk_half_cache(s0, [&](int i) __attribute__((always_inline)) { frag[i] = v_block(vc, 1, i); });
            weights(s1);
            if (weights_overflow()) redo(s1, s0, 1);
            pv_half([&](int i) __attribute__((always_inline)) { frag[i] = kc_block(kn, 1, i); });
            fresh = false;
        }
        land_cache(kd, vd);
        __syncthreads();
    };
    {
        int kt = 0;
        if (!KV_FP8) {
            const int n_spread = min(n_kt - 2, MODE == MODE_SUFFIX ? n_kt : n_my);
            for (; kt < n_spread; ++kt) cache_step(kt, std::true_type{});
        }
        for (; kt < n_kt; ++kt) cache_step(kt, std::false_type{});
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
        // own tile i: K in K buffer (kpar + i) & 1, V in V buffer (vpar + i) & 1
        int kpar = (n_kt + 1) & 1, vpar = n_kt & 1;
        if (n_kt == 0) {
            if (have) {
                fetch_self(cur, kbuf_of(kpar), vbuf_of(vpar));
                __builtin_amdgcn_s_waitcnt(0x0F70);
            }
            __syncthreads();
        }
        while (have) {
            SGC_NEXT_SELF(more, nxt);
            if (more) fetch_self(nxt, kbuf_of(kpar ^ 1), vbuf_of(vpar ^ 1));
            const int key0 = cur.key0, q = cur.q;
            bool mine = false;                  // does a row of this wave belong to query q and reach key0?
#pragma unroll
            for (int mi = 0; mi < MI; ++mi) mine |= valid[mi] && sq[mi] == q && qpos[mi] >= key0;
            if (q >= wsq_min && q <= wsq_max && __any(mine)) {
                const char *kc = kbuf_of(kpar), *vc = vbuf_of(vpar);
                // key j of the tile is visible to a row iff j <= reach (-1: another query's row); the 4 h of
                // the lane's key index is taken off once
                int reach[MI];
                bool far = false;
#pragma unroll
                for (int mi = 0; mi < MI; ++mi) {
                    const int r0 = (valid[mi] && sq[mi] == q) ? qpos[mi] - key0 : -1;
                    far |= r0 >= 32;
                    reach[mi] = r0 - 4 * h;
                }
                const bool second_half = __any(far);        // does any row of this wave see keys 32..63 of the tile?
                auto keep = [&](int mi, int j) __attribute__((always_inline)) { return j - 4 * h <= reach[mi]; };
#pragma unroll
                for (int i = 0; i < 8; ++i) frag[i] = k_block(kc, 0, i);
                // all products of the tile start from the same -m_ref; a raise by half 0 is passed on to half 1
                float before[MI];
#pragma unroll
                for (int mi = 0; mi < MI; ++mi) before[mi] = m_ref[mi];
                if (second_half) {
                    qk_half(s0, [&](int i) __attribute__((always_inline)) { frag[i] = k_block(kc, 1, i); });
                    qk_half(s1, [&](int i) __attribute__((always_inline)) { frag[i] = v_block(vc, 0, i); });
                } else {
                    qk_half(s0, [&](int i) __attribute__((always_inline)) { frag[i] = v_block(vc, 0, i); });
                }
                if (KV_FP8) rescale_self(s0, before);
                raise_reference(s0, 0, true, keep);
                weights(s0);
                if (second_half) {
                    pv_half([&](int i) __attribute__((always_inline)) { frag[i] = v_block(vc, 1, i); });
                    if (KV_FP8) rescale_self(s1, before);
#pragma unroll
                    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                        for (int r = 0; r < 16; ++r)
                            if (FOLD) s1[mi][r] -= m_ref[mi] - before[mi];
                    raise_reference(s1, 1, true, keep);
                    weights(s1);
                }
                pv_half(no_refill);
            }
            if (more) __builtin_amdgcn_s_waitcnt(0x0F70);
            __syncthreads();
            cur = nxt;
            have = more;
            kpar ^= 1;
            vpar ^= 1;
        }
#undef SGC_NEXT_SELF
    }

    // ---- normalise and store ----
    // A lane holds 4-channel pieces of its row; written out as they are they would make 8-byte stores scattered
    // over 32 rows per instruction.  The wavefront instead stages its 32 x 128 outputs in its own 8 KiB slice of
    // the tile buffers (idle now: every wavefront is past the last barrier behind its last read), the 16-byte
    // chunks of row n permuted by n % 16 so that the writes and the reads below spread over all banks, and stores
    // four whole rows of 256 bytes per instruction.
    uint16_t *og = static_cast<uint16_t *>(o_base);
    char *const ostage = smem + wave * MI * 8192;
#pragma unroll
    for (int mi = 0; mi < MI; ++mi) {
        const float l = half_sum(l_part[mi]);
        const float inv_l = (v_scaled ? 1.0f : v_scale) / l;
        char *st = ostage + mi * 8192 + n * 256 + h * 8;
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                bf16x4 y;
#pragma unroll
                for (int i = 0; i < 4; ++i) y[i] = (__bf16)(oacc[mi][db][q4 * 4 + i] * inv_l);
                *reinterpret_cast<bf16x4 *>(st + (((db * 4 + q4) ^ (n & 15)) * 16)) = y;
            }
        if (valid[mi] && lse_base && h == 0) {
            const int64_t col = (MODE == MODE_SUFFIX) ? (int64_t)src_tok[mi] : (int64_t)qpos[mi];
            lse_base[(int64_t)head[mi] * lse_stride + col] = (m_ref[mi] + __builtin_amdgcn_logf(l)) * 0.6931471805599453f;
        }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
    for (int mi = 0; mi < MI; ++mi) {
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const int r = 4 * k + (lane >> 4), c = lane & 15;     // row r of the block sits in lanes r and r + 32
            const uint4 y = *reinterpret_cast<const uint4 *>(ostage + mi * 8192 + r * 256 + ((c ^ (r & 15)) * 16));
            const int64_t row = __shfl(io_row[mi], r);
            const int ok = __shfl((int)valid[mi], r);
            if (ok) *reinterpret_cast<uint4 *>(og + row + c * 8) = y;
        }
    }
}

constexpr size_t kDynLds = LDS_TILE_BYTES + MAX_TILE_QUERIES * sizeof(int2);

template <int NW, int MI, bool FP8, int MODE, bool QK8>
hipError_t launch_one(const AttnArgs &a, int blocks, hipStream_t s)
{
    static bool configured = false;     // raise the dynamic LDS limit once per instantiation
    auto kern = attn_mfma_kernel<NW, MI, FP8, MODE, QK8>;
    size_t lds = kDynLds;
    if (!configured) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        configured = true;
    }
    hipLaunchKernelGGL(kern, dim3(blocks), dim3(NW * 64), lds, s, a);
    return hipGetLastError();
}

}  // namespace

// One kernel shape is built: 4 wavefronts x 32 rows, two workgroups per CU.  (8 wavefronts x 32 rows run in lock-step
// through the step barrier and lose the overlap two independent workgroups have; 64 rows per wavefront need more than
// 256 vector registers.  Both were measured slower and are not compiled.)
int mfma_tile_rows() { return 128; }

hipError_t launch_attn_mfma(const AttnArgs &a, hipStream_t s)
{
    constexpr int NW = 4, MI = 1;
    const bool fp8 = a.pool.kv_dtype == SGC_FP8_E4M3;
    if (a.n_tiles <= 0 && a.n_append <= 0) return hipSuccess;
    if (a.mode == MODE_SUFFIX) {
        // a decode step's launch carries, behind its tiles, the blocks that append the step's new tokens
        const int per_block = NW * 64 / 8;
        const int blocks = a.n_tiles + (a.n_append * a.n_kv_heads + per_block - 1) / per_block;
        if (fp8 && a.fp8_first_product) return launch_one<NW, MI, true, MODE_SUFFIX, true>(a, blocks, s);
        return fp8 ? launch_one<NW, MI, true, MODE_SUFFIX, false>(a, blocks, s) : launch_one<NW, MI, false, MODE_SUFFIX, false>(a, blocks, s);
    }
    // the prompt's own causal attention always takes the 16-bit first product
    return fp8 ? launch_one<NW, MI, true, MODE_PREFIX, false>(a, a.n_tiles, s) : launch_one<NW, MI, false, MODE_PREFIX, false>(a, a.n_tiles, s);
}

}  // namespace sgc
