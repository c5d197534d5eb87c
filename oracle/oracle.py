"""CPU fp64 oracle: Python face of ``sgc_oracle.c`` plus independent slow routines.

TEST INFRASTRUCTURE ONLY.  Imported by ``tests/``, by the smoke check and by the benchmark's
CPU-baseline leg.  The GPU library and its Python binding never import this package, and this
package imports nothing from them.

Three independent statements of the same result live here, written separately so that each
can be held against the others:

* the C routines (three-pass softmax, plain loops), reached through ``ctypes``;
* ``full_causal_numpy``: full causal attention over one whole sequence, done with dense numpy
  matrices and an explicit lower-triangular mask (used for the concatenation pin: suffix
  prefill over a cached prefix equals the last rows of causal attention over
  [prefix; suffix] -- SubGCache Sec. 3.4 and Sec. 1 Design 2);
* ``brute_force_suffix``: nested pure-Python loops with ``math.exp`` / ``math.cos`` on lists,
  for tiny shapes.

Integer bookkeeping (SubGCache Sec. 3.2: hierarchical clustering yields one label per query;
Sec. 3.4: each cluster's queries are served together from that cluster's cache) is
``assign_clusters``.
"""
from __future__ import annotations

import ctypes
import math
import os
import subprocess
from typing import List, Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "sgc_oracle.c")
_LIB = os.path.join(_HERE, "libsgc_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile ``sgc_oracle.c`` with gcc into ``libsgc_oracle.so`` beside it."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c99", "-fopenmp", "-fPIC", "-shared", _SRC, "-o", _LIB, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB)
        dp = ctypes.POINTER(ctypes.c_double)
        i64p = ctypes.POINTER(ctypes.c_int64)
        i32p = ctypes.POINTER(ctypes.c_int32)
        u8p = ctypes.POINTER(ctypes.c_uint8)
        f32p = ctypes.POINTER(ctypes.c_float)
        L.sgc_oracle_rope.argtypes = [dp, ctypes.c_int64, ctypes.c_int, ctypes.c_int, i64p, ctypes.c_double]
        L.sgc_oracle_rope.restype = None
        L.sgc_oracle_prefix_prefill.argtypes = [dp, dp, dp, ctypes.c_int64, ctypes.c_int, ctypes.c_int,
                                                ctypes.c_int, ctypes.c_double, ctypes.c_double, dp, dp, dp, dp]
        L.sgc_oracle_prefix_prefill.restype = None
        L.sgc_oracle_suffix_prefill.argtypes = [dp, dp, ctypes.c_int64, dp, dp, dp, ctypes.c_int64,
                                                ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_double,
                                                ctypes.c_double, dp, dp, dp, ctypes.c_int64, ctypes.c_int64]
        L.sgc_oracle_suffix_prefill.restype = None
        L.sgc_oracle_suffix_prefill_batched.argtypes = [ctypes.c_int, i32p, i64p, ctypes.POINTER(dp),
                                                        ctypes.POINTER(dp), i64p, dp, dp, dp, ctypes.c_int,
                                                        ctypes.c_int, ctypes.c_int, ctypes.c_double,
                                                        ctypes.c_double, dp, dp, dp]
        L.sgc_oracle_suffix_prefill_batched.restype = None
        L.sgc_oracle_suffix_prefill_head.argtypes = [dp, dp, ctypes.c_int64, dp, dp, dp, ctypes.c_int64,
                                                     ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                                     ctypes.c_double, ctypes.c_double, dp, dp]
        L.sgc_oracle_suffix_prefill_head.restype = None
        L.sgc_oracle_e4m3_decode.argtypes = [ctypes.c_uint8]
        L.sgc_oracle_e4m3_decode.restype = ctypes.c_double
        L.sgc_oracle_e4m3_encode.argtypes = [ctypes.c_double]
        L.sgc_oracle_e4m3_encode.restype = ctypes.c_uint8
        L.sgc_oracle_quantise_e4m3.argtypes = [dp, ctypes.c_int64, ctypes.c_int, ctypes.c_int, u8p, f32p, dp]
        L.sgc_oracle_quantise_e4m3.restype = None
        _lib = L
    return _lib


def _f64(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float64)


def _dp(a: Optional[np.ndarray]):
    if a is None:
        return None
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def n_threads() -> int:
    """Threads the C oracle's OpenMP loops use (OMP_NUM_THREADS, else the cores we may run on)."""
    env = os.environ.get("OMP_NUM_THREADS")
    if env:
        try:
            return max(1, int(env.split(",")[0]))
        except ValueError:
            pass
    try:
        return len(os.sched_getaffinity(0))
    except AttributeError:  # pragma: no cover
        return os.cpu_count() or 1


# ----------------------------------------------------------------------------------------------
# C routines
# ----------------------------------------------------------------------------------------------
def rope(x, pos, base: float) -> np.ndarray:
    """Rotate-half RoPE of x [n_tok][n_heads][d] at integer positions pos [n_tok]; returns a copy."""
    x = _f64(x).copy()
    pos = np.ascontiguousarray(pos, dtype=np.int64)
    n_tok, n_heads, d = x.shape
    assert pos.shape == (n_tok,)
    lib().sgc_oracle_rope(_dp(x), n_tok, n_heads, d, pos.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)), float(base))
    return x


def default_scale(d: int) -> float:
    return 1.0 / math.sqrt(d)


def prefix_prefill(q, k, v, rope_base: float, scale: Optional[float] = None, want_lse: bool = False):
    """One cluster's prefix prefill.  k, v [P][Hkv][d]; q [P][Hq][d] or None.

    Returns (cache_k, cache_v, o, lse): the cache as kept (K rotated at 0..P-1, V as is) and, when
    q is given, the causal self-attention output [P][Hq][d] and LSE [Hq][P] (else None).
    """
    k = _f64(k)
    v = _f64(v)
    P, Hkv, d = k.shape
    scale = default_scale(d) if scale is None else float(scale)
    cache_k = np.empty_like(k)
    cache_v = np.empty_like(v)
    o = lse = None
    Hq = Hkv
    if q is not None:
        q = _f64(q)
        Hq = q.shape[1]
        o = np.zeros_like(q)
        lse = np.zeros((Hq, P), dtype=np.float64) if want_lse else None
    lib().sgc_oracle_prefix_prefill(_dp(q), _dp(k), _dp(v), P, Hq, Hkv, d, float(rope_base), scale,
                                    _dp(cache_k), _dp(cache_v), _dp(o), _dp(lse))
    return cache_k, cache_v, o, lse


def suffix_prefill(cache_k, cache_v, q, k, v, rope_base: float, scale: Optional[float] = None):
    """One query over one cache.  Returns (o [S][Hq][d], lse [Hq][S], psum [Hq][S])."""
    cache_k = _f64(cache_k)
    cache_v = _f64(cache_v)
    q = _f64(q)
    k = _f64(k)
    v = _f64(v)
    P = cache_k.shape[0]
    S, Hq, d = q.shape
    Hkv = k.shape[1]
    scale = default_scale(d) if scale is None else float(scale)
    o = np.zeros_like(q)
    lse = np.zeros((Hq, S), dtype=np.float64)
    psum = np.zeros((Hq, S), dtype=np.float64)
    lib().sgc_oracle_suffix_prefill(_dp(cache_k), _dp(cache_v), P, _dp(q), _dp(k), _dp(v), S, Hq, Hkv, d,
                                    float(rope_base), scale, _dp(o), _dp(lse), _dp(psum), S, 0)
    return o, lse, psum


def suffix_prefill_batched(labels, cu_seqlens, caches_k: Sequence[np.ndarray], caches_v: Sequence[np.ndarray],
                           q, k, v, rope_base: float, scale: Optional[float] = None, want_psum: bool = False):
    """Whole batch in original query order.  caches_k[c], caches_v[c]: [P_c][Hkv][d] float64.

    Returns (o [T][Hq][d], lse [Hq][T]) and additionally psum [Hq][T] when want_psum.
    """
    labels = np.ascontiguousarray(labels, dtype=np.int32)
    cu = np.ascontiguousarray(cu_seqlens, dtype=np.int64)
    n = labels.shape[0]
    q = _f64(q)
    k = _f64(k)
    v = _f64(v)
    T, Hq, d = q.shape
    Hkv = k.shape[1]
    assert cu[-1] == T and cu.shape == (n + 1,)
    scale = default_scale(d) if scale is None else float(scale)
    cks = [_f64(a) for a in caches_k]
    cvs = [_f64(a) for a in caches_v]
    nc = len(cks)
    dp = ctypes.POINTER(ctypes.c_double)
    ck_arr = (dp * nc)(*[_dp(a) for a in cks])
    cv_arr = (dp * nc)(*[_dp(a) for a in cvs])
    plen = np.array([a.shape[0] for a in cks], dtype=np.int64)
    o = np.zeros_like(q)
    lse = np.zeros((Hq, T), dtype=np.float64)
    psum = np.zeros((Hq, T), dtype=np.float64) if want_psum else None
    lib().sgc_oracle_suffix_prefill_batched(
        n, labels.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)), cu.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)),
        ck_arr, cv_arr, plen.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)), _dp(q), _dp(k), _dp(v), Hq, Hkv, d,
        float(rope_base), scale, _dp(o), _dp(lse), _dp(psum))
    if want_psum:
        return o, lse, psum
    return o, lse


def suffix_prefill_head(cache_k, cache_v, q, k, v, head: int, rope_base: float, scale: Optional[float] = None):
    """One query, one query head (sampling huge workloads).  Returns (o [S][d], lse [S])."""
    cache_k = _f64(cache_k)
    cache_v = _f64(cache_v)
    q = _f64(q)
    k = _f64(k)
    v = _f64(v)
    P = cache_k.shape[0]
    S, Hq, d = q.shape
    Hkv = k.shape[1]
    scale = default_scale(d) if scale is None else float(scale)
    o = np.zeros((S, d), dtype=np.float64)
    lse = np.zeros((S,), dtype=np.float64)
    lib().sgc_oracle_suffix_prefill_head(_dp(cache_k), _dp(cache_v), P, _dp(q), _dp(k), _dp(v), S, Hq, Hkv, d,
                                         int(head), float(rope_base), scale, _dp(o), _dp(lse))
    return o, lse


def e4m3_decode(code: int) -> float:
    return float(lib().sgc_oracle_e4m3_decode(int(code) & 0xFF))


def e4m3_encode(x: float) -> int:
    return int(lib().sgc_oracle_e4m3_encode(float(x)))


def quantise_e4m3(x) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """Per-KV-head e4m3 quantisation of x [P][Hkv][d].  Returns (codes u8, scale f32 [Hkv], dequantised f64)."""
    x = _f64(x)
    P, Hkv, d = x.shape
    codes = np.zeros((P, Hkv, d), dtype=np.uint8)
    scale = np.zeros((Hkv,), dtype=np.float32)
    deq = np.zeros_like(x)
    lib().sgc_oracle_quantise_e4m3(_dp(x), P, Hkv, d, codes.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8)),
                                   scale.ctypes.data_as(ctypes.POINTER(ctypes.c_float)), _dp(deq))
    return codes, scale, deq


# ----------------------------------------------------------------------------------------------
# The attention layer around the cache (SubGCache Sec. 3.4: the representative prompt, and then each
# query's question tokens, pass through the LLM's transformer layers; in every layer the hidden states
# are projected to queries, keys and values, the keys and values of the prompt are what the cache
# keeps, and the attention output is projected back to the model width).  Weights are stored "out
# features x in features"; a projection is y[t][f] = sum_i x[t][i] w[f][i].  The matrix product is a
# library step (numpy, fp64); nothing is rounded between the steps.
# ----------------------------------------------------------------------------------------------
def project_qkv(x, w_qkv, n_q_heads: int, n_kv_heads: int, head_dim: int):
    """x [n][D], w_qkv [(Hq + 2 Hkv) d][D] (rows: Q heads, K heads, V heads, head-major).
    Returns q [n][Hq][d], k [n][Hkv][d], v [n][Hkv][d], before any rotation."""
    x = _f64(x)
    w = _f64(w_qkv)
    nq, nk = n_q_heads * head_dim, n_kv_heads * head_dim
    assert w.shape == (nq + 2 * nk, x.shape[1])
    y = x @ w.T
    n = x.shape[0]
    return (np.ascontiguousarray(y[:, :nq]).reshape(n, n_q_heads, head_dim),
            np.ascontiguousarray(y[:, nq:nq + nk]).reshape(n, n_kv_heads, head_dim),
            np.ascontiguousarray(y[:, nq + nk:]).reshape(n, n_kv_heads, head_dim))


def project_out(o, w_o) -> np.ndarray:
    """o [n][Hq][d] (heads concatenated head-major along the feature axis), w_o [D][Hq d] -> y [n][D]."""
    o = _f64(o)
    w = _f64(w_o)
    n = o.shape[0]
    flat = o.reshape(n, o.shape[1] * o.shape[2])
    assert w.shape[1] == flat.shape[1]
    return flat @ w.T


def attention_layer_prefix(x, w_qkv, w_o, n_q_heads: int, n_kv_heads: int, head_dim: int, rope_base: float,
                           scale: Optional[float] = None):
    """One layer over a cluster's prompt.  Returns (cache_k, cache_v, y [P][D]): the cache this layer keeps
    (projected K rotated at 0..P-1, projected V) and the layer's attention output projected back."""
    q, k, v = project_qkv(x, w_qkv, n_q_heads, n_kv_heads, head_dim)
    cache_k, cache_v, o, _ = prefix_prefill(q, k, v, rope_base, scale)
    return cache_k, cache_v, project_out(o, w_o)


def attention_layer_suffix(cache_k, cache_v, x, w_qkv, w_o, n_q_heads: int, n_kv_heads: int, head_dim: int,
                           rope_base: float, scale: Optional[float] = None) -> np.ndarray:
    """One layer over one query's question tokens appended to its cluster's cache: y [S][D]."""
    q, k, v = project_qkv(x, w_qkv, n_q_heads, n_kv_heads, head_dim)
    o, _, _ = suffix_prefill(cache_k, cache_v, q, k, v, rope_base, scale)
    return project_out(o, w_o)


# ----------------------------------------------------------------------------------------------
# Independent routine 1: dense numpy full-causal attention over one whole sequence
# ----------------------------------------------------------------------------------------------
def rope_numpy(x: np.ndarray, pos: np.ndarray, base: float) -> np.ndarray:
    """Rotate-half RoPE written with whole-array numpy operations (separate from the C loop)."""
    x = np.asarray(x, dtype=np.float64)
    if not base > 0:
        return x.copy()
    d = x.shape[-1]
    half = d // 2
    inv_freq = np.float64(base) ** (-np.arange(half, dtype=np.float64) * 2.0 / d)
    ang = np.asarray(pos, dtype=np.float64)[:, None] * inv_freq[None, :]       # [n_tok][half]
    c = np.cos(ang)[:, None, :]
    s = np.sin(ang)[:, None, :]
    x1, x2 = x[..., :half], x[..., half:]
    return np.concatenate([x1 * c - x2 * s, x2 * c + x1 * s], axis=-1)


def full_causal_numpy(q, k, v, rope_base: float, scale: Optional[float] = None):
    """Causal attention over ONE sequence of N tokens at positions 0..N-1.

    q [N][Hq][d], k, v [N][Hkv][d], all before rotation.  Returns (o [N][Hq][d], lse [Hq][N]).
    Dense score matrix, lower-triangular mask, softmax along keys.
    """
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    N, Hq, d = q.shape
    Hkv = k.shape[1]
    g = Hq // Hkv
    scale = default_scale(d) if scale is None else float(scale)
    pos = np.arange(N)
    qr = rope_numpy(q, pos, rope_base)
    kr = rope_numpy(k, pos, rope_base)
    kr_full = np.repeat(kr, g, axis=1)          # KV head h//g serves query head h
    v_full = np.repeat(v, g, axis=1)
    s = np.einsum("ihc,jhc->hij", qr, kr_full) * scale
    mask = np.tril(np.ones((N, N), dtype=bool))
    s = np.where(mask[None], s, -np.inf)
    mx = s.max(axis=-1, keepdims=True)
    e = np.exp(s - mx)
    z = e.sum(axis=-1, keepdims=True)
    p = e / z
    o = np.einsum("hij,jhc->ihc", p, v_full)
    lse = (mx + np.log(z))[..., 0]
    return o, lse


# ----------------------------------------------------------------------------------------------
# Independent routine 2: pure-Python brute force for tiny shapes
# ----------------------------------------------------------------------------------------------
def _bf_rope(vec: List[float], p: int, base: float) -> List[float]:
    d = len(vec)
    if not base > 0:
        return list(vec)
    half = d // 2
    out = [0.0] * d
    for t in range(half):
        a = p * (base ** (-2.0 * t / d))
        out[t] = vec[t] * math.cos(a) - vec[t + half] * math.sin(a)
        out[t + half] = vec[t + half] * math.cos(a) + vec[t] * math.sin(a)
    return out


def brute_force_suffix(prefix_k, prefix_v, q, k, v, rope_base: float, scale: Optional[float] = None):
    """Suffix prefill of one query from the *un-rotated* prefix K/V, by definition, in pure Python.

    prefix_k, prefix_v [P][Hkv][d] (before rotation); q [S][Hq][d]; k, v [S][Hkv][d].
    Returns nested lists o[S][Hq][d], lse[Hq][S].
    """
    prefix_k = np.asarray(prefix_k, dtype=np.float64).tolist()
    prefix_v = np.asarray(prefix_v, dtype=np.float64).tolist()
    q = np.asarray(q, dtype=np.float64).tolist()
    k = np.asarray(k, dtype=np.float64).tolist()
    v = np.asarray(v, dtype=np.float64).tolist()
    P = len(prefix_k)
    S = len(q)
    Hq = len(q[0]) if S else 0
    d = len(q[0][0]) if S else 0
    Hkv = len(k[0]) if S else 0
    g = Hq // Hkv if Hkv else 1
    scale = (1.0 / math.sqrt(d)) if scale is None else float(scale)
    o = [[[0.0] * d for _ in range(Hq)] for _ in range(S)]
    lse = [[0.0] * S for _ in range(Hq)]
    for i in range(S):
        for h in range(Hq):
            hk = h // g
            qi = _bf_rope(q[i][h], P + i, rope_base)
            keys = [(_bf_rope(prefix_k[j][hk], j, rope_base), prefix_v[j][hk]) for j in range(P)]
            keys += [(_bf_rope(k[j][hk], P + j, rope_base), v[j][hk]) for j in range(i + 1)]
            sc = [scale * sum(a * b for a, b in zip(qi, kk)) for kk, _ in keys]
            mx = max(sc)
            ex = [math.exp(x - mx) for x in sc]
            z = sum(ex)
            for c in range(d):
                o[i][h][c] = sum(ex[j] / z * keys[j][1][c] for j in range(len(keys)))
            lse[h][i] = mx + math.log(z)
    return o, lse


# ----------------------------------------------------------------------------------------------
# Integer bookkeeping
# ----------------------------------------------------------------------------------------------
def assign_clusters(labels: Sequence[int], suffix_len: Sequence[int], n_clusters: int):
    """Group queries by cluster label, keeping the original order inside each cluster.

    Returns (order, cluster_off, cu_seqlens) as int32 arrays:
      order[cluster_off[c] : cluster_off[c+1]] are the original indices of cluster c's queries,
      ascending; cu_seqlens[n] is the first token row of query n in the packed, original-order
      q/k/v/o arrays.
    """
    n = len(labels)
    buckets: List[List[int]] = [[] for _ in range(n_clusters)]
    for i in range(n):
        lab = int(labels[i])
        if lab < 0 or lab >= n_clusters:
            raise ValueError("label out of range")
        buckets[lab].append(i)
    order: List[int] = []
    cluster_off = [0]
    for b in buckets:
        order.extend(b)
        cluster_off.append(len(order))
    cu = [0]
    for i in range(n):
        if int(suffix_len[i]) < 0:
            raise ValueError("negative suffix length")
        cu.append(cu[-1] + int(suffix_len[i]))
    return (np.array(order, dtype=np.int32), np.array(cluster_off, dtype=np.int32), np.array(cu, dtype=np.int32))


def pages_needed(prefix_len: int, page_tokens: int = 16) -> int:
    """Pages a cluster's cache occupies in every layer: ceil(prefix_len / page_tokens)."""
    return -(-int(prefix_len) // int(page_tokens))


# ----------------------------------------------------------------------------------------------
# Query clustering (SubGCache Sec. 3.2; App. A.2: agglomerative hierarchical clustering with
# Euclidean distance, dendrogram cut at a predefined number of clusters; Sec. 4.6 / Table 3: Ward,
# Single, Average, Complete and Centroid linkage)
# ----------------------------------------------------------------------------------------------
LINKAGES = ("ward", "single", "average", "complete", "centroid")


def _linkage_distance(x: np.ndarray, a: List[int], b: List[int], linkage: str) -> float:
    """Distance between two clusters (member index lists) straight from the linkage's definition."""
    if linkage in ("single", "complete", "average"):
        d = np.sqrt(((x[a][:, None, :] - x[b][None, :, :]) ** 2).sum(axis=-1))     # all member pairs
        return float(d.min() if linkage == "single" else d.max() if linkage == "complete" else d.mean())
    ca, cb = x[a].mean(axis=0), x[b].mean(axis=0)
    gap2 = float(((ca - cb) ** 2).sum())
    if linkage == "centroid":
        return float(np.sqrt(gap2))
    if linkage == "ward":           # growth of the within-cluster sum of squares caused by the merge
        return len(a) * len(b) / (len(a) + len(b)) * gap2
    raise ValueError("unknown linkage")


def cluster_queries(embeddings: np.ndarray, n_clusters: int, linkage: str = "ward") -> np.ndarray:
    """Agglomerative clustering by its definition: start from singletons, repeatedly merge the two clusters
    at the smallest linkage distance (recomputed from the members every time) until n_clusters are left.

    Readings where the paper is silent: "cutting the dendrogram at c clusters" = the partition after m - c
    merges; equal distances are broken towards the pair whose clusters have the smallest first members
    (compare the smaller first member, then the larger); clusters are numbered by their first member.
    Returns int32 labels [m].
    """
    x = np.asarray(embeddings, dtype=np.float64)
    m = x.shape[0]
    if not 1 <= n_clusters <= max(m, 1):
        raise ValueError("n_clusters out of range")
    clusters: List[List[int]] = [[i] for i in range(m)]       # kept sorted by first member
    while len(clusters) > n_clusters:
        best = None
        for i in range(len(clusters)):
            for j in range(i + 1, len(clusters)):
                d = _linkage_distance(x, clusters[i], clusters[j], linkage)
                if best is None or d < best[0]:             # strict: the first (smallest-member) pair wins ties
                    best = (d, i, j)
        _, i, j = best
        clusters[i] = sorted(clusters[i] + clusters[j])
        del clusters[j]
    labels = np.empty(m, dtype=np.int32)
    for c, members in enumerate(clusters):
        labels[members] = c
    return labels


# ----------------------------------------------------------------------------------------------
# Representative subgraph (SubGCache Sec. 3.3): per cluster, the union of all nodes and all edges of the
# subgraphs its queries retrieved.
# ----------------------------------------------------------------------------------------------
def union_subgraphs(labels: Sequence[int], n_clusters: int, node_lists: Sequence[Sequence[int]],
                    edge_lists: Sequence[Sequence[Tuple[int, int]]]):
    """Returns (nodes, edges): per cluster the sorted list of distinct node ids and the sorted list of distinct
    directed edges (src, dst) over the cluster's queries.  Reading where the paper is silent: an edge is the
    ordered pair as retrieved; the order of the lists (ascending) only makes the prompt deterministic."""
    nodes = [set() for _ in range(n_clusters)]
    edges = [set() for _ in range(n_clusters)]
    for i, lab in enumerate(labels):
        lab = int(lab)
        if lab < 0 or lab >= n_clusters:
            raise ValueError("label out of range")
        nodes[lab].update(int(x) for x in node_lists[i])
        edges[lab].update((int(a), int(b)) for a, b in edge_lists[i])
    return [sorted(s) for s in nodes], [sorted(s) for s in edges]
