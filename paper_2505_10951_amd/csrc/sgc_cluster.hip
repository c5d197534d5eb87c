// Host-side query clustering of libsgc.
//
// SubGCache (arXiv 2505.10951) Sec. 3.2: the subgraph embeddings of a batch's queries are grouped by
// hierarchical clustering; App. A.2: agglomerative, Euclidean distance, the dendrogram cut at a
// predefined number of clusters; Sec. 4.6 / Table 3: Ward (default), Single, Average, Complete and
// Centroid linkage.  The labels it produces are what sgc_assign_clusters takes.
//
// The batch is small (Table 4: 50-200 queries), so the whole inter-cluster distance matrix is kept in
// fp64 and updated after each merge with the Lance-Williams recurrence of the linkage; the closest
// pair is the one a full scan would find, read off per-slot nearest partners that a merge updates in place
// (centroid linkage, which can bring clusters closer, included: a changed row is scanned again).  O(m^2) memory,
// O(m^2) time unless many slots share one nearest partner, no device work.
#include <math.h>
#include <stdarg.h>
#include <stdio.h>

#include <algorithm>
#include <limits>
#include <new>
#include <vector>

#include "sgc_internal.h"

namespace {

int fail_cluster(sgc_ctx *ctx, int code, const char *fmt, ...)
{
    if (ctx) {
        char buf[256];
        va_list ap;
        va_start(ap, fmt);
        vsnprintf(buf, sizeof(buf), fmt, ap);
        va_end(ap);
        ctx->err = buf;
    }
    return code;
}

}  // namespace

extern "C" int sgc_cluster_queries(sgc_ctx *ctx, int32_t m, int32_t dim, const float *embeddings, int32_t linkage,
                                   int32_t n_clusters, int32_t *labels)
{
    if (m < 0 || dim < 0) return fail_cluster(ctx, SGC_EINVAL, "m %d / dim %d negative", m, dim);
    if (m == 0) return SGC_OK;
    if (!embeddings && dim > 0) return fail_cluster(ctx, SGC_EINVAL, "embeddings is NULL");
    if (!labels) return fail_cluster(ctx, SGC_EINVAL, "labels is NULL");
    if (linkage < SGC_LINKAGE_WARD || linkage > SGC_LINKAGE_CENTROID)
        return fail_cluster(ctx, SGC_EINVAL, "linkage %d unknown", linkage);
    if (n_clusters < 1 || n_clusters > m)
        return fail_cluster(ctx, SGC_EINVAL, "n_clusters %d outside [1, %d]", n_clusters, m);
    if (m > 32768) return fail_cluster(ctx, SGC_EINVAL, "m %d too large for the dense distance matrix", m);
    for (int64_t i = 0; i < (int64_t)m * dim; ++i)
        if (!std::isfinite(embeddings[i])) return fail_cluster(ctx, SGC_EINVAL, "embeddings[%lld] is not finite", (long long)i);

    // Ward and centroid recur on squared Euclidean distances, the other three on plain ones.
    const bool squared = linkage == SGC_LINKAGE_WARD || linkage == SGC_LINKAGE_CENTROID;
    std::vector<double> dist, xt, acc, near_d;
    std::vector<int32_t> size, parent, near_j;
    std::vector<char> alive;
    try {
        dist.assign((size_t)m * m, 0.0);
        xt.resize((size_t)dim * m);
        acc.resize(m);
        near_d.assign(m, std::numeric_limits<double>::infinity());
        near_j.assign(m, -1);
        size.assign(m, 1);
        parent.resize(m);
        alive.assign(m, 1);
    } catch (const std::bad_alloc &) {
        return fail_cluster(ctx, SGC_ENOMEM, "host allocation failed");
    }
    // Distances: every pair's sum runs over the coordinates in order (t = 0, 1, ...), as a scalar loop would; with the
    // embeddings transposed the inner loop runs over the partners j of one i and vectorises.
    for (int i = 0; i < m; ++i)
        for (int t = 0; t < dim; ++t) xt[(size_t)t * m + i] = (double)embeddings[(size_t)i * dim + t];
    for (int i = 0; i < m; ++i) {
        parent[i] = i;
        for (int j = i + 1; j < m; ++j) acc[j] = 0.0;
        int t = 0;
        for (; t + 4 <= dim; t += 4) {          // four coordinates per pass over the partners, added in order
            const double *c0 = &xt[(size_t)t * m], *c1 = c0 + m, *c2 = c1 + m, *c3 = c2 + m;
            const double x0 = c0[i], x1 = c1[i], x2 = c2[i], x3 = c3[i];
            for (int j = i + 1; j < m; ++j) {
                const double d0 = x0 - c0[j], d1 = x1 - c1[j], d2 = x2 - c2[j], d3 = x3 - c3[j];
                double a = acc[j];
                a += d0 * d0;
                a += d1 * d1;
                a += d2 * d2;
                a += d3 * d3;
                acc[j] = a;
            }
        }
        for (; t < dim; ++t) {
            const double *col = &xt[(size_t)t * m];
            const double xi = col[i];
            for (int j = i + 1; j < m; ++j) {
                const double d = xi - col[j];
                acc[j] += d * d;
            }
        }
        for (int j = i + 1; j < m; ++j) {
            const double v = squared ? acc[j] : sqrt(acc[j]);
            dist[(size_t)i * m + j] = dist[(size_t)j * m + i] = v;
        }
    }
    // A cluster lives in the slot of its smallest member.  The pair to merge is the one a scan over slots i < j in
    // order with strict minima would find (among equally close pairs the one with the smallest first members, then the
    // smallest second); the scan is not repeated for every merge: every slot keeps its nearest partner above it
    // (near_j[i] > i, the smallest such j among equals), which a merge of (bi, bj) can only change for slots below bj.
    auto rescan = [&](int i) {
        double best = std::numeric_limits<double>::infinity();
        int bj = -1;
        const double *row = &dist[(size_t)i * m];
        for (int j = i + 1; j < m; ++j)
            if (alive[j] && row[j] < best) {
                best = row[j];
                bj = j;
            }
        near_d[i] = best;
        near_j[i] = bj;
    };
    for (int i = 0; i < m; ++i) rescan(i);
    for (int remaining = m; remaining > n_clusters; --remaining) {
        double best = std::numeric_limits<double>::infinity();
        int bi = -1;
        for (int i = 0; i < m; ++i)
            if (alive[i] && near_d[i] < best) {
                best = near_d[i];
                bi = i;
            }
        const int bj = near_j[bi];
        const double ni = size[bi], nj = size[bj], dij = dist[(size_t)bi * m + bj];
        for (int k = 0; k < m; ++k) {
            if (!alive[k] || k == bi || k == bj) continue;
            const double dki = dist[(size_t)k * m + bi], dkj = dist[(size_t)k * m + bj], nk = size[k];
            double v;
            switch (linkage) {
                case SGC_LINKAGE_SINGLE: v = dki < dkj ? dki : dkj; break;
                case SGC_LINKAGE_COMPLETE: v = dki > dkj ? dki : dkj; break;
                case SGC_LINKAGE_AVERAGE: v = (ni * dki + nj * dkj) / (ni + nj); break;
                case SGC_LINKAGE_CENTROID:
                    v = (ni * dki + nj * dkj) / (ni + nj) - ni * nj * dij / ((ni + nj) * (ni + nj));
                    break;
                default:   // Ward
                    v = ((nk + ni) * dki + (nk + nj) * dkj - nk * dij) / (nk + ni + nj);
                    break;
            }
            dist[(size_t)k * m + bi] = dist[(size_t)bi * m + k] = v;
        }
        size[bi] += size[bj];
        alive[bj] = 0;
        parent[bj] = bi;
        // nearest partners: slot bi has a new row; a slot below bi sees a new distance to bi and loses bj; a slot
        // between them loses bj; slots above bj see nothing of the pair among their partners
        rescan(bi);
        for (int k = 0; k < bj; ++k) {
            if (!alive[k] || k == bi) continue;
            if (near_j[k] == bj || near_j[k] == bi) {
                rescan(k);
            } else if (k < bi) {
                const double v = dist[(size_t)k * m + bi];
                if (v < near_d[k] || (v == near_d[k] && bi < near_j[k])) {
                    near_d[k] = v;
                    near_j[k] = bi;
                }
            }
        }
    }
    // clusters are numbered by their first member
    std::vector<int32_t> id(m, -1);
    int32_t next = 0;
    for (int i = 0; i < m; ++i)
        if (alive[i]) id[i] = next++;
    for (int i = 0; i < m; ++i) {
        int r = i;
        while (parent[r] != r) r = parent[r];
        labels[i] = id[r];
    }
    return SGC_OK;
}

// ---- representative subgraph (Sec. 3.3) ---------------------------------------------------------
// For each cluster, the union of all nodes and of all edges of the subgraphs retrieved by the cluster's
// queries.  Lists come out ascending (edges by source, then destination), which fixes the order in which
// a caller textualises the representative subgraph and with it the prompt the cache is computed for.
extern "C" int sgc_union_subgraphs(sgc_ctx *ctx, int32_t m, const int32_t *labels, int32_t n_clusters,
                                   const int64_t *node_off, const int32_t *nodes, const int64_t *edge_off,
                                   const int32_t *edges, int64_t *out_node_off, int32_t *out_nodes, int64_t *out_edge_off,
                                   int32_t *out_edges)
{
    if (m < 0 || n_clusters < 1) return fail_cluster(ctx, SGC_EINVAL, "m %d / n_clusters %d out of range", m, n_clusters);
    if (!out_node_off || !out_edge_off) return fail_cluster(ctx, SGC_EINVAL, "out_node_off / out_edge_off is NULL");
    if (m > 0 && (!labels || !node_off || !edge_off)) return fail_cluster(ctx, SGC_EINVAL, "labels / node_off / edge_off is NULL");
    int64_t n_nodes = 0, n_edges = 0;
    if (m > 0) {
        if (node_off[0] != 0 || edge_off[0] != 0) return fail_cluster(ctx, SGC_EINVAL, "offsets must start at 0");
        for (int32_t i = 0; i < m; ++i) {
            if (labels[i] < 0 || labels[i] >= n_clusters)
                return fail_cluster(ctx, SGC_EINVAL, "labels[%d] = %d outside [0, %d)", i, labels[i], n_clusters);
            if (node_off[i + 1] < node_off[i] || edge_off[i + 1] < edge_off[i])
                return fail_cluster(ctx, SGC_EINVAL, "offsets of query %d decrease", i);
        }
        n_nodes = node_off[m];
        n_edges = edge_off[m];
    }
    if ((n_nodes > 0 && (!nodes || !out_nodes)) || (n_edges > 0 && (!edges || !out_edges)))
        return fail_cluster(ctx, SGC_EINVAL, "nodes / edges / out_nodes / out_edges is NULL");
    std::vector<std::vector<int32_t>> cn;
    std::vector<std::vector<uint64_t>> ce;      // edge as (src, dst) packed with a sign flip: sorts like the pair
    try {
        cn.resize(n_clusters);
        ce.resize(n_clusters);
        for (int32_t i = 0; i < m; ++i) {
            auto &vn = cn[labels[i]];
            vn.insert(vn.end(), nodes + node_off[i], nodes + node_off[i + 1]);
            auto &ve = ce[labels[i]];
            for (int64_t e = edge_off[i]; e < edge_off[i + 1]; ++e) {
                const uint64_t a = (uint32_t)edges[2 * e] ^ 0x80000000u, b = (uint32_t)edges[2 * e + 1] ^ 0x80000000u;
                ve.push_back((a << 32) | b);
            }
        }
    } catch (const std::bad_alloc &) {
        return fail_cluster(ctx, SGC_ENOMEM, "host allocation failed");
    }
    int64_t on = 0, oe = 0;
    for (int32_t k = 0; k < n_clusters; ++k) {
        out_node_off[k] = on;
        out_edge_off[k] = oe;
        auto &vn = cn[k];
        std::sort(vn.begin(), vn.end());
        vn.erase(std::unique(vn.begin(), vn.end()), vn.end());
        for (int32_t x : vn) out_nodes[on++] = x;
        auto &ve = ce[k];
        std::sort(ve.begin(), ve.end());
        ve.erase(std::unique(ve.begin(), ve.end()), ve.end());
        for (uint64_t x : ve) {
            out_edges[2 * oe] = (int32_t)((uint32_t)(x >> 32) ^ 0x80000000u);
            out_edges[2 * oe + 1] = (int32_t)((uint32_t)x ^ 0x80000000u);
            ++oe;
        }
    }
    out_node_off[n_clusters] = on;
    out_edge_off[n_clusters] = oe;
    return SGC_OK;
}
