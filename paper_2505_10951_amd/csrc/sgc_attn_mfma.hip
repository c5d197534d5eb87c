// bf16 MFMA attention kernel of libsgc for gfx950 (MI355X), head_dim 128.
//
// SubGCache (arXiv 2505.10951) Sec. 3.4: every query of a cluster appends its question tokens to
// the cluster's cached prompt.  One workgroup takes a tile of rows that all belong to one
// (cluster, KV head): rows are (query, token, head-in-group) of ANY query of the cluster, so the
// cached prefix K/V tiles staged in LDS are shared by several queries at once.  After the
// prefix keys the same rows run causally over their own query's suffix keys.
//
// Matrix-core mapping (v_mfma_f32_32x32x16_bf16, 64-lane wavefronts):
//   S^T = K Q^T : A = 32 keys x 16 channels (from LDS), B = 16 channels x 32 rows (Q, registers).
//                 Lane (n, h) = (lane % 32, lane / 32) then owns row n and, in accumulator
//                 register r, key 8 (r / 4) + 4 h + r % 4: a row's scores sit in ONE lane pair, so
//                 the row max/sum need a single exchange between the two 32-lane halves.
//   O^T = V^T P^T : A = 32 channels x 16 keys (from LDS, V is stored transposed per 16-token page),
//                 B = 16 keys x 32 rows = the probabilities exactly as the score accumulator
//                 holds them (registers 8 kb .. 8 kb + 7), no cross-lane movement.
// Softmax is online, fp32, base 2, with the running maximum only raised when it grows by more
// than 2^8 (the accumulators are rescaled at that moment only).
#include <hip/hip_runtime.h>

#include "sgc_internal.h"

namespace sgc {

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr int D = 128;         // head dim
constexpr int BN = 64;         // keys per LDS tile (4 pages)
constexpr int K_TILE_BYTES = BN * D * 2;   // 16 KiB of bf16
constexpr int BUF_BYTES = 2 * K_TILE_BYTES;
constexpr float kRescaleThreshold = 8.0f;   // log2 units
constexpr float kNegBig = -1.0e30f;

__device__ inline float half_swap(float x) { return __shfl_xor(x, 32); }

// Unpacks 2 fp8 e4m3 codes (low or high half of w) to bf16 (exact: e4m3 is a subset of bf16).
__device__ inline uint32_t fp8x2_to_bf16x2(uint32_t w, bool high)
{
    const auto f = high ? __builtin_amdgcn_cvt_pk_f32_fp8((int)w, true) : __builtin_amdgcn_cvt_pk_f32_fp8((int)w, false);
    return (__float_as_uint(f[0]) >> 16) | (__float_as_uint(f[1]) & 0xFFFF0000u);
}

template <int NW, int MI, bool KV_FP8, int MODE>
__global__ void __launch_bounds__(NW * 64) attn_mfma_kernel(const AttnArgs a)
{
    constexpr int NT = NW * 64;
    constexpr int BM = NW * MI * 32;
    __shared__ __attribute__((aligned(1024))) char smem[2][BUF_BYTES];

    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63;
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
    const int cluster = t.cluster, hk = t.hk;
    const int P = (MODE == MODE_SUFFIX) ? a.cl_prefix_len[cluster] : a.prefix_len;
    const int n_pages = (P + kPageTokens - 1) / kPageTokens;
    const int32_t *pt = a.page_table + a.cl_pt_off[cluster];
    const int tok_base = (MODE == MODE_SUFFIX) ? a.cl_tok_off[cluster] : 0;
    const int last_row = t.row0 + t.n_rows - 1;

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
    // wave-uniform bounds on the visible cached keys
    int lim_min = lim[0], lim_max = lim[0];
#pragma unroll
    for (int mi = 1; mi < MI; ++mi) {
        lim_min = min(lim_min, lim[mi]);
        lim_max = max(lim_max, lim[mi]);
    }
    for (int o = 32; o > 0; o >>= 1) {
        lim_min = min(lim_min, __shfl_xor(lim_min, o));
        lim_max = max(lim_max, __shfl_xor(lim_max, o));
    }
    lim_min = __builtin_amdgcn_readfirstlane(lim_min);
    lim_max = __builtin_amdgcn_readfirstlane(lim_max);

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

    // One 64-key tile from LDS buffer `buf`.  keep(mi, j) says whether row mi may see key j of the
    // tile (only consulted when `masked`); c is the score scale in log2 units.
    auto process_tile = [&](const char *buf, const float c, const bool masked, auto keep) {
        f32x16 sacc[MI][2];
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
            for (int nb = 0; nb < 2; ++nb)
#pragma unroll
                for (int r = 0; r < 16; ++r) sacc[mi][nb][r] = 0.f;
        // S^T = K Q^T
#pragma unroll
        for (int nb = 0; nb < 2; ++nb) {
#pragma unroll
            for (int kb = 0; kb < 8; ++kb) {
                const bf16x8 ka = *reinterpret_cast<const bf16x8 *>(buf + (nb * 8 + kb) * 1024 + h * 512 + n * 16);
#pragma unroll
                for (int mi = 0; mi < MI; ++mi)
                    sacc[mi][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, qf[mi][kb], sacc[mi][nb], 0, 0, 0);
            }
        }
        bf16x8 pf[MI][4];
#pragma unroll
        for (int mi = 0; mi < MI; ++mi) {
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
            // raise the reference maximum only when it grew by more than the threshold
            if (__any(tmax > m_ref[mi] + kRescaleThreshold)) {
                const float m_new = fmaxf(m_ref[mi], tmax);
                const float alpha = __builtin_amdgcn_exp2f(m_ref[mi] - m_new);
                m_ref[mi] = m_new;
                l_part[mi] *= alpha;
#pragma unroll
                for (int db = 0; db < 4; ++db)
#pragma unroll
                    for (int r = 0; r < 16; ++r) oacc[mi][db][r] *= alpha;
            }
            float psum = 0.f;
#pragma unroll
            for (int nb = 0; nb < 2; ++nb)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const float p = __builtin_amdgcn_exp2f(sacc[mi][nb][r] * c - m_ref[mi]);
                    psum += p;
                    pf[mi][nb * 2 + (r >> 3)][r & 7] = (__bf16)p;
                }
            l_part[mi] += psum;
        }
        // O^T += V^T P^T
        const char *vbuf = buf + K_TILE_BYTES;
#pragma unroll
        for (int pg = 0; pg < 4; ++pg) {
#pragma unroll
            for (int db = 0; db < 4; ++db) {
                const bf16x8 va = *reinterpret_cast<const bf16x8 *>(vbuf + (pg * 4 + db) * 1024 + h * 512 + n * 16);
#pragma unroll
                for (int mi = 0; mi < MI; ++mi)
                    oacc[mi][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va, pf[mi][pg], oacc[mi][db], 0, 0, 0);
            }
        }
    };

    // ---- cached prefix keys: global -> registers -> LDS, double buffered ----
    const int n_cache_keys = (MODE == MODE_SUFFIX) ? P : min(P, last_row / g + 1);
    const int n_kt = (n_cache_keys + BN - 1) / BN;

    // A tile is 8 page parts (K and V of 4 pages).  Each wavefront moves whole 1 KiB runs of a part, so
    // the page id and every address but the lane offset are wave-uniform (scalar loads, scalar
    // branches) and nothing in the prefetch waits on a vector load.
    constexpr int UNITS = KV_FP8 ? 16 : 32;           // 1 KiB global runs per tile
    constexpr int UPW = UNITS / NW;                   // per wavefront
    constexpr int RUNS_PER_PART = KV_FP8 ? 2 : 4;
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
    uint4 stage[UPW];

    auto load_tile = [&](int kt) {
#pragma unroll
        for (int j = 0; j < UPW; ++j) {
            const int u = wave_u + NW * j;
            const int part = u / RUNS_PER_PART, run = u % RUNS_PER_PART;   // part 0..3: K pages, 4..7: V pages
            const int p = part & 3;
            const int pn = kt * 4 + p;
            if (pn < n_pages) {
                const int page = pt[pn];
                const char *src = (part >= 4) ? a.pool.v_part(a.layer, page, hk) : a.pool.k_part(a.layer, page, hk);
                stage[j] = *reinterpret_cast<const uint4 *>(src + run * 1024 + lane * 16);
            } else {
                stage[j] = make_uint4(0, 0, 0, 0);
            }
        }
    };
    auto store_tile = [&](char *buf) {
#pragma unroll
        for (int j = 0; j < UPW; ++j) {
            const int u = wave_u + NW * j;
            const int part = u / RUNS_PER_PART, run = u % RUNS_PER_PART;
            const int p = part & 3;
            const bool is_v = part >= 4;
            const int cp = run * 64 + lane;               // 16-byte chunk inside the page part
            if (!KV_FP8) {
                int dst;
                if (is_v) {
                    dst = K_TILE_BYTES + p * 4096 + cp * 16;
                } else {
                    const int blk = cp >> 4, tok = cp & 15;     // blk = kb * 2 + hh
                    dst = (((p >> 1) * 8 + (blk >> 1)) * 2 + (blk & 1)) * 512 + ((p & 1) * 16 + tok) * 16;
                }
                *reinterpret_cast<uint4 *>(buf + dst) = stage[j];
            } else {
                // one 16-byte chunk = two adjacent 8-element groups; they land 16 bytes apart in LDS
                const uint32_t w[4] = {stage[j].x, stage[j].y, stage[j].z, stage[j].w};
                uint4 o0, o1;
                o0.x = fp8x2_to_bf16x2(w[0], false); o0.y = fp8x2_to_bf16x2(w[0], true);
                o0.z = fp8x2_to_bf16x2(w[1], false); o0.w = fp8x2_to_bf16x2(w[1], true);
                o1.x = fp8x2_to_bf16x2(w[2], false); o1.y = fp8x2_to_bf16x2(w[2], true);
                o1.z = fp8x2_to_bf16x2(w[3], false); o1.w = fp8x2_to_bf16x2(w[3], true);
                int dst;
                if (is_v) {
                    dst = K_TILE_BYTES + (p * 256 + cp * 2) * 16;
                } else {
                    const int blk = cp >> 3, tok = (cp & 7) * 2;
                    dst = (((p >> 1) * 8 + (blk >> 1)) * 2 + (blk & 1)) * 512 + ((p & 1) * 16 + tok) * 16;
                }
                *reinterpret_cast<uint4 *>(buf + dst) = o0;
                *reinterpret_cast<uint4 *>(buf + dst + 16) = o1;
            }
        }
    };

    if (n_kt > 0) {
        load_tile(0);
        store_tile(smem[0]);
    }
    __syncthreads();
    for (int kt = 0; kt < n_kt; ++kt) {
        const bool more = kt + 1 < n_kt;
        if (more) load_tile(kt + 1);
        const int key0 = kt * BN;
        if (key0 < lim_max) {   // some row of this wave still sees keys of this tile
            const bool masked = key0 + BN > lim_min;
            process_tile(smem[kt & 1], c_cache, masked, [&](int mi, int j) { return key0 + j < lim[mi]; });
        }
        if (more) store_tile(smem[(kt + 1) & 1]);
        __syncthreads();
    }

    // ---- the rows' own suffix keys (suffix mode only) ----
    if (MODE == MODE_SUFFIX) {
        if (KV_FP8) {
#pragma unroll
            for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                for (int db = 0; db < 4; ++db)
#pragma unroll
                    for (int r = 0; r < 16; ++r) oacc[mi][db][r] *= v_scale;
        }
        const int sq_lo = a.tok_sq[tok_base + t.row0 / g];
        const int last_tau = tok_base + last_row / g;
        const int sq_hi = a.tok_sq[last_tau];
        const int last_qpos = a.tok_qpos[last_tau];
        const uint16_t *kg = static_cast<const uint16_t *>(a.k);
        const uint16_t *vg = static_cast<const uint16_t *>(a.v);
        char *buf = smem[0];
        for (int q = sq_lo; q <= sq_hi; ++q) {
            const int S = a.sq_len[q];
            const int64_t src0 = a.sq_src0[q];
            const int jmax = (q == sq_hi) ? last_qpos : S - 1;
            for (int j0 = 0; j0 <= jmax; j0 += BN) {
                // stage 64 suffix keys: K rotated at P + j into operand order, V transposed
                for (int it = tid; it < BN * 8; it += NT) {
                    const int jj = it >> 3, cc = it & 7;
                    const int j = j0 + jj;
                    uint4 o1 = make_uint4(0, 0, 0, 0), o2 = o1;
                    if (j < S) {
                        const uint16_t *krow = kg + ((src0 + j) * Hkv + hk) * D;
                        const uint4 lo = *reinterpret_cast<const uint4 *>(krow + cc * 8);
                        const uint4 hi = *reinterpret_cast<const uint4 *>(krow + 64 + cc * 8);
                        if (a.rope) {
                            const uint32_t wl[4] = {lo.x, lo.y, lo.z, lo.w}, wh[4] = {hi.x, hi.y, hi.z, hi.w};
                            const float4 *tab = reinterpret_cast<const float4 *>(a.rope + (int64_t)(P + j) * 64 + cc * 8);
                            uint32_t r1[4], r2[4];
#pragma unroll
                            for (int i = 0; i < 4; ++i) {
                                const float4 cs = tab[i];
                                const float a0 = __uint_as_float(wl[i] << 16), a1 = __uint_as_float(wl[i] & 0xFFFF0000u);
                                const float b0 = __uint_as_float(wh[i] << 16), b1 = __uint_as_float(wh[i] & 0xFFFF0000u);
                                typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
                                bf16x2 y1, y2;
                                y1[0] = (__bf16)(a0 * cs.x - b0 * cs.y);
                                y1[1] = (__bf16)(a1 * cs.z - b1 * cs.w);
                                y2[0] = (__bf16)(b0 * cs.x + a0 * cs.y);
                                y2[1] = (__bf16)(b1 * cs.z + a1 * cs.w);
                                r1[i] = __builtin_bit_cast(uint32_t, y1);
                                r2[i] = __builtin_bit_cast(uint32_t, y2);
                            }
                            o1 = make_uint4(r1[0], r1[1], r1[2], r1[3]);
                            o2 = make_uint4(r2[0], r2[1], r2[2], r2[3]);
                        } else {
                            o1 = lo;
                            o2 = hi;
                        }
                    }
                    const int nb = jj >> 5, m = jj & 31;
                    // channels cc*8.. -> block (kb = cc/2, hh = cc%2); channels 64+cc*8.. -> kb + 4
                    *reinterpret_cast<uint4 *>(buf + ((nb * 8 + (cc >> 1)) * 2 + (cc & 1)) * 512 + m * 16) = o1;
                    *reinterpret_cast<uint4 *>(buf + ((nb * 8 + 4 + (cc >> 1)) * 2 + (cc & 1)) * 512 + m * 16) = o2;
                }
                for (int it = tid; it < BN * 16; it += NT) {
                    const int jj = it >> 4, cv = it & 15;
                    const int j = j0 + jj;
                    uint4 x = make_uint4(0, 0, 0, 0);
                    if (j < S) x = *reinterpret_cast<const uint4 *>(vg + ((src0 + j) * Hkv + hk) * D + cv * 8);
                    const uint32_t w[4] = {x.x, x.y, x.z, x.w};
                    const int pg = jj >> 4, tok = jj & 15;
                    const int hh = (tok >> 2) & 1, ii = (tok & 3) | ((tok >> 3) << 2);
                    const int db = cv >> 2, m0 = (cv & 3) * 8;
                    uint16_t *dst = reinterpret_cast<uint16_t *>(buf + K_TILE_BYTES + (((pg * 4 + db) * 2 + hh) * 32 + m0) * 16) + ii;
#pragma unroll
                    for (int i = 0; i < 8; ++i) dst[i * 8] = (uint16_t)(w[i >> 1] >> (16 * (i & 1)));
                }
                __syncthreads();
                // does any row of this wave belong to query q and reach key j0?
                bool mine = false;
#pragma unroll
                for (int mi = 0; mi < MI; ++mi) mine |= valid[mi] && sq[mi] == q && qpos[mi] >= j0;
                if (__any(mine)) {
                    process_tile(buf, c_self, true,
                                 [&](int mi, int j) { return sq[mi] == q && j0 + j <= qpos[mi]; });
                }
                __syncthreads();
            }
        }
    }

    // ---- normalise and store ----
    uint16_t *og = static_cast<uint16_t *>(a.o);
#pragma unroll
    for (int mi = 0; mi < MI; ++mi) {
        const float l = l_part[mi] + half_swap(l_part[mi]);
        const float inv_l = 1.0f / l;
        if (valid[mi]) {
#pragma unroll
            for (int db = 0; db < 4; ++db)
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4) {
                    typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
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

template <int NW, int MI>
hipError_t launch_variant(const AttnArgs &a, hipStream_t s)
{
    constexpr int BM = NW * MI * 32;
    const bool fp8 = a.pool.kv_dtype == SGC_FP8_E4M3;
    if (a.mode == MODE_SUFFIX) {
        if (a.n_tiles <= 0) return hipSuccess;
        if (fp8)
            hipLaunchKernelGGL((attn_mfma_kernel<NW, MI, true, MODE_SUFFIX>), dim3(a.n_tiles), dim3(NW * 64), 0, s, a);
        else
            hipLaunchKernelGGL((attn_mfma_kernel<NW, MI, false, MODE_SUFFIX>), dim3(a.n_tiles), dim3(NW * 64), 0, s, a);
    } else {
        const int rows = a.prefix_len * a.group;
        const int tiles = (rows + BM - 1) / BM * a.n_kv_heads;
        if (tiles <= 0) return hipSuccess;
        if (fp8)
            hipLaunchKernelGGL((attn_mfma_kernel<NW, MI, true, MODE_PREFIX>), dim3(tiles), dim3(NW * 64), 0, s, a);
        else
            hipLaunchKernelGGL((attn_mfma_kernel<NW, MI, false, MODE_PREFIX>), dim3(tiles), dim3(NW * 64), 0, s, a);
    }
    return hipGetLastError();
}

}  // namespace

// variant 0: 4 waves x 64 rows (256-row tiles); 1: 8 waves x 32 rows (256); 2: 4 waves x 32 rows (128)
int mfma_tile_rows(int variant)
{
    switch (variant) {
        case 0: return 256;
        case 1: return 256;
        case 2: return 128;
        default: return 0;
    }
}

hipError_t launch_attn_mfma(const AttnArgs &a, int variant, hipStream_t s)
{
    switch (variant) {
        case 0: return launch_variant<4, 2>(a, s);
        case 1: return launch_variant<8, 1>(a, s);
        case 2: return launch_variant<4, 1>(a, s);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace sgc
