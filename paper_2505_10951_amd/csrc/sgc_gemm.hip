// Projection kernels of libsgc for gfx950 (MI355X): the linear maps around the cached attention.
//
// SubGCache (arXiv 2505.10951) Sec. 3.4 feeds the representative prompt and then every query's question
// tokens through the LLM's layers.  In each layer the hidden states x [rows][K] are projected by the fused
// weight w_qkv [(Hq + 2 Hkv) d][K] ("out features x in features") to queries, keys and values, and the
// attention output is projected back by w_o.  Both are C = A B^T with A and B contiguous along the
// contraction, which is exactly what the 32x32x16 bf16 matrix-core instruction wants for both operands.
//
// bf16 kernel: a workgroup of 4 wavefronts computes a 256 x 256 tile of C; wavefront (wm, wn) owns the
// 128 x 128 quadrant and keeps it in 16 accumulators of 32 x 32 (256 registers, one wavefront per SIMD).
// The contraction runs in steps of 64: the 256 x 64 slabs of A and B (32 KiB each) are copied
// global -> LDS without passing through registers, double buffered, one barrier per step.  In LDS a slab is
// row-major with 128-byte rows whose eight 16-byte chunks are permuted by (row & 7) ^ ((row >> 3) & 1); the
// permutation is applied on the global side of the copy (the LDS side of such a copy is linear in the lane
// index), and it spreads the 16-byte operand reads of 32 consecutive rows over all banks.
//
// Epilogue of the QKV projection (a wavefront's 128 columns are exactly one head, d = 128):
//   Q heads: stored as they are (the attention kernel rotates Q itself);
//   K heads: rotated at the token's position (rotate-half pairs channel t with t + 64, which sit in the
//            same lane and register of accumulators pi and pi + 2) and written straight into the 16-token
//            pages in the cache's K order: 8 consecutive channels of a token are one 16-byte unit;
//   V heads: the matrix-core operands are swapped for these wavefronts so that a lane owns ONE channel and
//            16 tokens; when the 16 rows are one page this is the cache's V order (8 tokens of a channel
//            contiguous) and goes out as 16-byte stores, otherwise element by element.
// With an fp8 cache (the scale needs the maximum over the whole prompt first) K and V go to a staging
// matrix and the ingest kernels take it from there.
#include <hip/hip_runtime.h>

#include <type_traits>

#include "sgc_internal.h"

namespace sgc {

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr int TM = 256, TN = 256, TK = 64;
constexpr int SLAB_BYTES = TM * TK * 2;          // 32 KiB: 256 rows of 128 bytes
constexpr int STAGE_BYTES = 2 * SLAB_BYTES;      // A slab, then B slab
constexpr int GEMM_LDS = 2 * STAGE_BYTES;        // 128 KiB
constexpr int HD = 128;                          // head dim of the fused epilogue

__device__ inline uint32_t pack2(float a, float b)
{
    const bf16x2 p = {(__bf16)a, (__bf16)b};
    return __builtin_bit_cast(uint32_t, p);
}

// 1 KiB (64 lanes x 16 bytes) from per-lane global addresses to the LDS block at lds (wave-uniform).
__device__ inline void copy_1k_to_lds(const char *src_lane, char *lds)
{
    const auto *g = (const __attribute__((address_space(1))) void *)src_lane;
    auto *l = (__attribute__((address_space(3))) void *)lds;
    __builtin_amdgcn_global_load_lds(g, l, 16, 0, 0);
}

template <bool QKV>
__global__ void __launch_bounds__(256, 1) proj_gemm_kernel(const GemmArgs g)
{
    extern __shared__ __attribute__((aligned(1024))) char smem[];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 6);
    const int wm = wave >> 1, wn = wave & 1;
    const int h = lane >> 5, l31 = lane & 31;

    // ---- which tile: workgroup b runs on XCD b % 8; every XCD takes a contiguous run of tile ids, and ids
    // walk the tile grid in groups of 4 row tiles, column by column, so that the 32 workgroups an XCD runs
    // together cover about 4 x 8 tiles and share their A and B slabs in that XCD's L2.
    const int n_ct = g.n_col_tiles, n_rt = g.n_row_tiles;
    const int total = n_ct * n_rt;
    const int per = (total + 7) >> 3;
    const int local = (int)blockIdx.x >> 3;
    const int tid = ((int)blockIdx.x & 7) * per + local;
    if (local >= per || tid >= total) return;
    constexpr int GM = 4;
    const int grp = tid / (GM * n_ct);
    const int gsz = min(GM, n_rt - grp * GM);
    const int in = tid - grp * GM * n_ct;
    const int rt = __builtin_amdgcn_readfirstlane(grp * GM + in % gsz);
    const int ct = __builtin_amdgcn_readfirstlane(in / gsz);

    GemmRowTile t;
    if (g.tiles) {
        t = g.tiles[rt];
    } else {
        t.a = static_cast<const char *>(g.a) + (int64_t)rt * TM * g.K * 2;
        t.c = g.c ? static_cast<char *>(g.c) + (int64_t)rt * TM * g.ldc * 2 : nullptr;
        t.ck = t.cv = nullptr;
        t.rows = (int32_t)min<int64_t>(TM, g.M - (int64_t)rt * TM);
        t.pos0 = 0;
        t.pt_off = 0;
        t.dest0 = rt * TM;
    }
    const int rows = __builtin_amdgcn_readfirstlane(t.rows);
    const int K = g.K, N = g.N;
    const int n_steps = K / TK;

    // ---- copies: wavefront w moves rows [64 w, 64 w + 64) of both slabs, 8 rows (1 KiB) per instruction.
    // Lane (lr, slot) = (lane / 8, lane % 8) lands at LDS chunk `slot` of row 8 i + lr and therefore fetches the
    // global chunk slot ^ perm(row); rows past the operand's end are clamped (their results are never stored).
    const int lr = lane >> 3, slot = lane & 7;
    const char *a_base = static_cast<const char *>(t.a);
    const char *b_base = static_cast<const char *>(g.w) + (int64_t)ct * TN * K * 2;
    const int b_rows = min(TN, N - ct * TN);
    uint32_t a_off[8], b_off[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int row = 64 * wave + 8 * i + lr;
        const uint32_t chunk = (uint32_t)(slot ^ lr ^ (i & 1));
        a_off[i] = (uint32_t)min(row, rows - 1) * (uint32_t)(K * 2) + chunk * 16;
        b_off[i] = (uint32_t)min(row, b_rows - 1) * (uint32_t)(K * 2) + chunk * 16;
    }
    auto issue = [&](int kt, int stage) __attribute__((always_inline)) {
        char *as = smem + stage * STAGE_BYTES + wave * 8192;
        char *bs = as + SLAB_BYTES;
        const uint32_t k_off = (uint32_t)kt * (TK * 2);
#pragma unroll
        for (int i = 0; i < 8; ++i) copy_1k_to_lds(a_base + (a_off[i] + k_off), as + i * 1024);
#pragma unroll
        for (int i = 0; i < 8; ++i) copy_1k_to_lds(b_base + (b_off[i] + k_off), bs + i * 1024);
    };

    // ---- which output this wavefront makes
    const int col0 = ct * TN + wn * HD;              // first column of the wavefront's 128
    bool v_orient = false;
    int kind = 0, hk = 0;                            // 0 plain, 1 K head, 2 V head
    if (QKV && col0 >= g.n_plain) {
        const int kvh = (col0 - g.n_plain) / HD;
        kind = kvh < g.n_kv_heads ? 1 : 2;
        hk = kind == 1 ? kvh : kvh - g.n_kv_heads;
        v_orient = kind == 2 && g.kv_dest != 2;
    }

    // ---- operand reads: lane (l31, h) of block b reads row 32 b + l31, chunk 2 kk + h
    const uint32_t perm = (uint32_t)(h ^ (lane & 7) ^ ((lane >> 3) & 1));
    uint32_t r_off[4];
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) r_off[kk] = (uint32_t)l31 * 128 + (((uint32_t)kk * 32) ^ (perm * 16));
    const uint32_t x_region = (uint32_t)wm * 16384, w_region = SLAB_BYTES + (uint32_t)wn * 16384;
    // first operand: its rows land in the accumulator registers; second operand: its rows land in the lanes
    const uint32_t p_region = v_orient ? x_region : w_region;
    const uint32_t q_region = v_orient ? w_region : x_region;

    f32x16 acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    // Sub-step kk of a step multiplies the 16-wide slice kk of the slabs: 8 operand reads, 16 products.  The
    // reads run one sub-step ahead of the products, and the step's barrier sits in front of its LAST sub-step:
    // by then every wavefront holds that sub-step's operands in registers, so the buffer can be refilled (copy of
    // step kt + 2) and the first operands of step kt + 1 requested while the last 16 products still run.
    auto load_ops = [&](const char *st, int kk, bf16x8 (&p)[4], bf16x8 (&q)[4]) __attribute__((always_inline)) {
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            p[b] = *reinterpret_cast<const bf16x8 *>(st + p_region + b * 4096 + r_off[kk]);
            q[b] = *reinterpret_cast<const bf16x8 *>(st + q_region + b * 4096 + r_off[kk]);
        }
    };
    auto products = [&](const bf16x8 (&p)[4], const bf16x8 (&q)[4]) __attribute__((always_inline)) {
#pragma unroll
        for (int pi = 0; pi < 4; ++pi)
#pragma unroll
            for (int qj = 0; qj < 4; ++qj)
                acc[pi][qj] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(p[pi], q[qj], acc[pi][qj], 0, 0, 0);
    };
    // Issue order of a sub-step: the 8 reads of the next sub-step go out in the shadow of the first 4 products,
    // so that they have landed long before the next sub-step's first product asks for them.
    auto order_reads_under_products = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);     // one matrix-core instruction
            __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);     // two LDS reads
        }
        __builtin_amdgcn_sched_group_barrier(0x008, 12, 0);
        __builtin_amdgcn_sched_barrier(0);
    };
    bf16x8 p0[4], q0[4], p1[4], q1[4];
    issue(0, 0);
    __builtin_amdgcn_s_waitcnt(0x0F70);          // vmcnt(0): this wavefront's copies have landed
    __syncthreads();                             // everyone's have
    if (n_steps > 1) issue(1, 1);
    load_ops(smem, 0, p0, q0);
    __builtin_amdgcn_sched_barrier(0);
    // one step; NEXT: a step follows (barrier, first operands of it), NEXT2: two follow (refill this step's buffer)
    auto step = [&](int kt, auto next, auto next2) __attribute__((always_inline)) {
        constexpr bool NEXT = decltype(next)::value, NEXT2 = decltype(next2)::value;
        const char *st = smem + (kt & 1) * STAGE_BYTES;
        load_ops(st, 1, p1, q1);
        products(p0, q0);
        order_reads_under_products();
        load_ops(st, 2, p0, q0);
        products(p1, q1);
        order_reads_under_products();
        load_ops(st, 3, p1, q1);
        products(p0, q0);
        order_reads_under_products();
        if (NEXT) {
            __builtin_amdgcn_s_waitcnt(0x0F70);  // the copies of step kt + 1, requested a step ago
            __syncthreads();                  // every wavefront has read all of step kt out of LDS
            __builtin_amdgcn_sched_barrier(0);
            load_ops(smem + ((kt + 1) & 1) * STAGE_BYTES, 0, p0, q0);
            if (NEXT2) issue(kt + 2, kt & 1);
        }
        products(p1, q1);
        if (NEXT) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 1);
                __builtin_amdgcn_sched_group_barrier(0x100, 2, 1);
            }
        }
        if (NEXT2) {
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 1);
                __builtin_amdgcn_sched_group_barrier(0x010, 2, 1);     // two of the 16 copy instructions
            }
        }
        __builtin_amdgcn_sched_barrier(0);
    };
    int kt = 0;
    for (; kt + 2 < n_steps; ++kt) step(kt, std::true_type{}, std::true_type{});
    if (kt + 1 < n_steps) step(kt++, std::true_type{}, std::false_type{});
    step(kt, std::false_type{}, std::false_type{});

    if (col0 >= N) return;          // the second half of a ragged last column tile
    const int rows16 = (rows + 15) & ~15;

    if (!v_orient) {
        // lane = token 128 wm + 32 qj + l31; register r of accumulator pi = feature 32 pi + 8 (r / 4) + 4 h + r % 4
        const bool to_pages = QKV && kind == 1 && g.kv_dest != 2;
#pragma unroll
        for (int qj = 0; qj < 4; ++qj) {
            const int i = 128 * wm + 32 * qj + l31;
            const bool valid = i < rows;
            bool store = valid;
            char *dst = nullptr;
            int64_t chunk_stride = 16;
            if (to_pages) {
                int page, slot16, pos;
                if (g.kv_dest == 0) {
                    const int p = t.pos0 + i;
                    store = i < rows16;                          // the last page's unused slots are zeroed
                    page = store ? g.page_table[t.pt_off + (p >> 4)] : 0;
                    slot16 = p & 15;
                    pos = p;
                } else {
                    const int2 d = g.row_dest[t.dest0 + (valid ? i : 0)];
                    page = d.x >> 4;
                    slot16 = d.x & 15;
                    pos = d.y;
                }
                dst = g.kv_base + (int64_t)page * g.page_bytes + (int64_t)hk * g.part_bytes + slot16 * 16;
                chunk_stride = 256;
                if (g.rope) {
                    const float2 *tab = g.rope + (int64_t)(valid ? pos : 0) * (HD / 2);
#pragma unroll
                    for (int pi = 0; pi < 2; ++pi)
#pragma unroll
                        for (int q4 = 0; q4 < 4; ++q4) {
                            const float4 *cs = reinterpret_cast<const float4 *>(tab + 32 * pi + 8 * q4 + 4 * h);
                            const float4 c01 = cs[0], c23 = cs[1];
                            const float co[4] = {c01.x, c01.z, c23.x, c23.z}, si[4] = {c01.y, c01.w, c23.y, c23.w};
#pragma unroll
                            for (int e = 0; e < 4; ++e) {
                                const float x1 = acc[pi][qj][4 * q4 + e], x2 = acc[pi + 2][qj][4 * q4 + e];
                                acc[pi][qj][4 * q4 + e] = x1 * co[e] - x2 * si[e];
                                acc[pi + 2][qj][4 * q4 + e] = x2 * co[e] + x1 * si[e];
                            }
                        }
                }
            } else if (kind == 0) {
                store = valid && t.c != nullptr;
                dst = static_cast<char *>(t.c) + ((int64_t)i * g.ldc + col0) * 2;
            } else {
                char *base = static_cast<char *>(kind == 1 ? t.ck : t.cv);
                dst = base + ((int64_t)i * (g.n_kv_heads * HD) + hk * HD) * 2;
            }
#pragma unroll
            for (int pi = 0; pi < 4; ++pi)
#pragma unroll
                for (int u = 0; u < 2; ++u) {
                    // registers 8 u .. 8 u + 3 are features 16 u + 4 h + 0..3, registers 8 u + 4 .. + 7 features
                    // 16 u + 8 + 4 h + 0..3; after the swap between the two 32-lane halves lane h holds the eight
                    // consecutive features 16 u + 8 h .. + 7
                    float x[8];
#pragma unroll
                    for (int e = 0; e < 8; ++e) x[e] = valid ? acc[pi][qj][8 * u + e] : 0.f;
                    // keys that go straight into pages are binary16 there; everything else is bf16
                    const uint32_t a0 = to_pages ? pack2_f16(x[0], x[1]) : pack2(x[0], x[1]);
                    const uint32_t a1 = to_pages ? pack2_f16(x[2], x[3]) : pack2(x[2], x[3]);
                    const uint32_t b0 = to_pages ? pack2_f16(x[4], x[5]) : pack2(x[4], x[5]);
                    const uint32_t b1 = to_pages ? pack2_f16(x[6], x[7]) : pack2(x[6], x[7]);
                    const auto s0 = __builtin_amdgcn_permlane32_swap(a0, b0, false, false);
                    const auto s1 = __builtin_amdgcn_permlane32_swap(a1, b1, false, false);
                    const uint4 out = make_uint4(s0[0], s1[0], s0[1], s1[1]);
                    const int chunk = 4 * pi + 2 * u + h;
                    if (store) *reinterpret_cast<uint4 *>(dst + chunk * chunk_stride) = out;
                }
        }
    } else {
        // lane = channel 32 qj + l31 of the head; register r of accumulator pi = token 32 pi + 8 (r / 4) + 4 h + r % 4
#pragma unroll
        for (int pi = 0; pi < 4; ++pi)
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                const int r16 = 128 * wm + 32 * pi + 16 * e;      // first of the 16 rows registers 8 e .. 8 e + 7 belong to
                if (r16 >= rows16) continue;
                if (g.kv_dest == 0) {
                    // the 16 rows are one page; register 8 e + i is the page's token 4 h + (i & 3) + 8 (i >> 2)
                    const int page = g.page_table[t.pt_off + ((t.pos0 + r16) >> 4)];
                    char *vp = g.kv_base + (int64_t)page * g.page_bytes + (int64_t)(g.n_kv_heads + hk) * g.part_bytes;
#pragma unroll
                    for (int qj = 0; qj < 4; ++qj) {
                        float x[8];
#pragma unroll
                        for (int i = 0; i < 8; ++i) {
                            const int tok = r16 + 4 * h + (i & 3) + 8 * (i >> 2);
                            x[i] = tok < rows ? acc[pi][qj][8 * e + i] : 0.f;
                        }
                        const uint4 out = make_uint4(pack2(x[0], x[1]), pack2(x[2], x[3]), pack2(x[4], x[5]), pack2(x[6], x[7]));
                        *reinterpret_cast<uint4 *>(vp + (((qj * 2 + h) * 32) + l31) * 16) = out;
                    }
                } else {
#pragma unroll
                    for (int i = 0; i < 8; ++i) {
                        const int tok = r16 + 4 * h + (i & 3) + 8 * (i >> 2);
                        if (tok >= rows) continue;
                        const int2 d = g.row_dest[t.dest0 + tok];
                        __bf16 *vp = reinterpret_cast<__bf16 *>(g.kv_base + (int64_t)(d.x >> 4) * g.page_bytes +
                                                                (int64_t)(g.n_kv_heads + hk) * g.part_bytes);
#pragma unroll
                        for (int qj = 0; qj < 4; ++qj) vp[v_page_index(d.x & 15, 32 * qj + l31)] = (__bf16)acc[pi][qj][8 * e + i];
                    }
                }
            }
    }
}

// Any shape and both io types, one output element per thread, fp32 accumulation; columns are dealt to up to
// three row-major outputs (Q, K, V or just one).
__device__ inline float load_io(const void *p, int64_t i, int io_dtype)
{
    return io_dtype == SGC_F32 ? static_cast<const float *>(p)[i] : (float)static_cast<const __bf16 *>(p)[i];
}
__device__ inline void store_io(void *p, int64_t i, int io_dtype, float x)
{
    if (io_dtype == SGC_F32)
        static_cast<float *>(p)[i] = x;
    else
        static_cast<__bf16 *>(p)[i] = (__bf16)x;
}

__global__ void __launch_bounds__(256) proj_generic_kernel(const void *a, const void *w, int64_t M, int N, int K, int io_dtype,
                                                           void *c0, int n0, void *c1, int n1, void *c2)
{
    __shared__ float as[16][17], ws[16][17];
    const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
    const int64_t m = (int64_t)blockIdx.y * 16 + ty;
    const int n = blockIdx.x * 16 + tx;
    float sum = 0.f;
    for (int k0 = 0; k0 < K; k0 += 16) {
        const int64_t am = (int64_t)blockIdx.y * 16 + ty;
        const int wn_ = blockIdx.x * 16 + ty;
        as[ty][tx] = (am < M && k0 + tx < K) ? load_io(a, am * K + k0 + tx, io_dtype) : 0.f;
        ws[ty][tx] = (wn_ < N && k0 + tx < K) ? load_io(w, (int64_t)wn_ * K + k0 + tx, io_dtype) : 0.f;
        __syncthreads();
#pragma unroll
        for (int k = 0; k < 16; ++k) sum += as[ty][k] * ws[tx][k];
        __syncthreads();
    }
    if (m >= M || n >= N) return;
    if (n < n0) {
        if (c0) store_io(c0, m * n0 + n, io_dtype, sum);
    } else if (n < n0 + n1) {
        store_io(c1, m * n1 + (n - n0), io_dtype, sum);
    } else {
        store_io(c2, m * (N - n0 - n1) + (n - n0 - n1), io_dtype, sum);
    }
}

// Clears the last page (every head, K and V) of each query whose length is not a multiple of the page size:
// the projection only writes the slots of real tokens, and the attention kernel multiplies the rest by zero
// weights, which needs them finite.
__global__ void __launch_bounds__(256) zero_last_pages_kernel(char *spool, const int32_t *sq_len, const int32_t *sq_page0,
                                                              int64_t page_bytes)
{
    const int S = sq_len[blockIdx.x];
    if (S <= 0 || (S & 15) == 0) return;
    uint4 *p = reinterpret_cast<uint4 *>(spool + (int64_t)(sq_page0[blockIdx.x] + ((S - 1) >> 4)) * page_bytes);
    const int64_t n16 = page_bytes / 16;
    for (int64_t i = threadIdx.x; i < n16; i += blockDim.x) p[i] = make_uint4(0, 0, 0, 0);
}

}  // namespace


hipError_t launch_proj_gemm(const GemmArgs &g, bool qkv, hipStream_t s)
{
    const int total = g.n_row_tiles * g.n_col_tiles;
    if (total <= 0) return hipSuccess;
    static bool configured[2] = {false, false};
    const void *kern = qkv ? reinterpret_cast<const void *>(proj_gemm_kernel<true>) : reinterpret_cast<const void *>(proj_gemm_kernel<false>);
    if (!configured[qkv]) {
        hipError_t e = hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, GEMM_LDS);
        if (e != hipSuccess) return e;
        configured[qkv] = true;
    }
    const int per = (total + 7) / 8;
    if (qkv)
        hipLaunchKernelGGL(proj_gemm_kernel<true>, dim3(per * 8), dim3(256), GEMM_LDS, s, g);
    else
        hipLaunchKernelGGL(proj_gemm_kernel<false>, dim3(per * 8), dim3(256), GEMM_LDS, s, g);
    return hipGetLastError();
}

hipError_t launch_proj_generic(const void *a, const void *w, int64_t M, int N, int K, int io_dtype, void *c0, int n0, void *c1,
                               int n1, void *c2, hipStream_t s)
{
    if (M <= 0 || N <= 0) return hipSuccess;
    hipLaunchKernelGGL(proj_generic_kernel, dim3((N + 15) / 16, (unsigned)((M + 15) / 16)), dim3(256), 0, s, a, w, M, N, K, io_dtype,
                       c0, n0, c1, n1, c2);
    return hipGetLastError();
}

hipError_t launch_zero_last_pages(char *spool, const int32_t *d_sq_len, const int32_t *d_sq_page0, int n_sq, int64_t page_bytes,
                                  hipStream_t s)
{
    if (n_sq <= 0) return hipSuccess;
    hipLaunchKernelGGL(zero_last_pages_kernel, dim3(n_sq), dim3(256), 0, s, spool, d_sq_len, d_sq_page0, page_bytes);
    return hipGetLastError();
}

}  // namespace sgc
