"""Test-side helpers: run the CPU oracle on a synthetic workload, and an emulation of the GPU's
rounding points (numpy, dense) used only to calibrate how tight a tolerance can be."""
from __future__ import annotations

import os
from typing import Dict, Optional, Sequence

import numpy as np

from oracle import oracle as orc
from paper_2505_10951_amd.workloads import Workload, round_to_bf16


def oracle_caches(w: Workload, layer: int = 0, clusters: Optional[Sequence[int]] = None, threads: int = 1) -> Dict[int, tuple]:
    """cluster -> (cache_k, cache_v) as the attention reads them (fp8: oracle-quantised, dequantised).  Clusters are
    independent; with threads > 1 several are prepared at once (the oracle's routines are called as they are)."""
    def one(c):
        k, v = w.prefix_kv(c, layer)
        ck, cv, _, _ = orc.prefix_prefill(None, k, v, w.rope_base)
        if w.kv_dtype == "fp8_e4m3":
            _, _, ck = orc.quantise_e4m3(ck)
            _, _, cv = orc.quantise_e4m3(cv)
        return c, (ck, cv)

    todo = list(range(w.n_clusters) if clusters is None else clusters)
    if threads > 1 and len(todo) > 1:
        from concurrent.futures import ThreadPoolExecutor
        with ThreadPoolExecutor(max_workers=min(threads, len(todo))) as ex:
            return dict(ex.map(one, todo))
    return dict(one(c) for c in todo)


def oracle_suffix(w: Workload, layer: int = 0, queries: Optional[Sequence[int]] = None, caches=None):
    """Oracle output for the chosen queries (default all).  Returns (rows, o_ref [len(rows)][Hq][d],
    lse_ref [Hq][len(rows)]): `rows` indexes the packed token rows of the full batch."""
    queries = list(range(w.n_queries)) if queries is None else list(queries)
    cu = w.cu_seqlens
    need = sorted({int(w.labels[n]) for n in queries})
    caches = oracle_caches(w, layer, need, threads=min(8, os.cpu_count() or 1)) if caches is None else caches
    nc = w.n_clusters
    empty = np.zeros((0, w.n_kv_heads, w.head_dim))
    cks = [caches[c][0] if c in caches else empty for c in range(nc)]
    cvs = [caches[c][1] if c in caches else empty for c in range(nc)]
    qs, ks, vs, rows, sub_cu = [], [], [], [], [0]
    for n in queries:
        q, k, v = w.suffix_qkv_query(n, layer)
        qs.append(q), ks.append(k), vs.append(v)
        rows.extend(range(int(cu[n]), int(cu[n + 1])))
        sub_cu.append(sub_cu[-1] + q.shape[0])
    if sub_cu[-1] == 0:
        return np.zeros(0, dtype=np.int64), np.zeros((0, w.n_q_heads, w.head_dim)), np.zeros((w.n_q_heads, 0))
    o, lse = orc.suffix_prefill_batched(w.labels[queries], np.array(sub_cu), cks, cvs, np.concatenate(qs),
                                        np.concatenate(ks), np.concatenate(vs), w.rope_base)
    return np.array(rows, dtype=np.int64), o, lse


def bf16_floor_arrays(pk, pv, q, k, v, rope_base: float, want_lse: bool = False):
    """max |o_rounded - o_exact| (and, with want_lse, the same for LSE) of one query's suffix prefill when the
    operands are rounded where a 16-bit matrix-core kernel has to round them: the rotated keys and the rotated,
    scaled queries to IEEE binary16 (what the library keeps and multiplies), the probabilities and the output to
    bf16 (dense numpy, fp64 otherwise).  A measure of the error any such kernel carries; used to set a
    tolerance, never as a reference."""
    P, S = pk.shape[0], q.shape[0]
    d = q.shape[-1]
    g = q.shape[1] // k.shape[1]
    r = lambda x: round_to_bf16(np.asarray(x, dtype=np.float32)).astype(np.float64)
    c_q = np.log2(np.e) / np.sqrt(d)      # the query carries the score scale in log2 units when it is rounded
    rh = lambda x: np.asarray(x, dtype=np.float32).astype(np.float16).astype(np.float64)
    kr = np.concatenate([orc.rope_numpy(pk, np.arange(P), rope_base), orc.rope_numpy(k, P + np.arange(S), rope_base)])
    qr = orc.rope_numpy(q, P + np.arange(S), rope_base)
    vv = np.concatenate([pv, v]).astype(np.float64)
    mask = np.arange(P + S)[None, :] <= (P + np.arange(S))[:, None]

    def attend(qx, kx, round_p):
        s = np.einsum("ihc,jhc->hij", qx, np.repeat(kx, g, axis=1)) / np.sqrt(d)
        s = np.where(mask[None], s, -np.inf)
        e = np.exp(s - s.max(axis=-1, keepdims=True))
        z = e.sum(axis=-1, keepdims=True)
        lse = (s.max(axis=-1, keepdims=True) + np.log(z))[..., 0]
        if round_p:
            e = r(e)
        return np.einsum("hij,jhc->ihc", e / z, np.repeat(vv, g, axis=1)), lse

    exact, lse_exact = attend(qr, kr, False)
    rounded, lse_rounded = attend(rh(qr * c_q) / c_q, rh(kr), True)
    o_floor = float(np.abs(r(rounded) - exact).max())
    if want_lse:
        return o_floor, float(np.abs(lse_rounded - lse_exact).max())
    return o_floor


def round_to_e4m3_pow2_rows(x: np.ndarray) -> np.ndarray:
    """Rows (last axis) rounded to e4m3 under a power-of-two scale of their own that puts the row's largest magnitude
    in [128, 256): nearest, ties to even, 3 fraction bits (numpy; the magnitudes stay far from the format's ends)."""
    x = np.asarray(x, dtype=np.float64)
    amax = np.abs(x).max(axis=-1, keepdims=True)
    _, e = np.frexp(np.where(amax > 0, amax, 1.0))
    y = x * np.exp2(8.0 - e)
    m, ex = np.frexp(y)
    step = np.maximum(np.exp2(ex - 4.0), 2.0 ** -9)          # 4 significant bits; fixed spacing below 2^-6
    return np.round(y / step) * step * np.exp2(e - 8.0)


def fp8_query_floor(cache_k, cache_v, q, k, v, rope_base: float) -> float:
    """max |o - o_exact| of one query's suffix prefill over an (already rotated, dequantised) cache when the rotated,
    scaled query rows are rounded to e4m3 as the fp8 first product does against cached keys (dense numpy, fp64
    otherwise; the query's own keys see the unrounded query).  A measure of what that rounding costs, for tolerances."""
    P, S = cache_k.shape[0], q.shape[0]
    d = q.shape[-1]
    g = q.shape[1] // k.shape[1]
    qr = orc.rope_numpy(q, P + np.arange(S), rope_base)
    kr = np.concatenate([cache_k, orc.rope_numpy(k, P + np.arange(S), rope_base)])
    vv = np.concatenate([cache_v, v]).astype(np.float64)
    mask = np.arange(P + S)[None, :] <= (P + np.arange(S))[:, None]
    q8 = round_to_e4m3_pow2_rows(qr)

    def attend(q_cache):
        kk = np.repeat(kr, g, axis=1)
        s = np.concatenate([np.einsum("ihc,jhc->hij", q_cache, kk[:P]), np.einsum("ihc,jhc->hij", qr, kk[P:])], axis=-1) / np.sqrt(d)
        s = np.where(mask[None], s, -np.inf)
        e = np.exp(s - s.max(axis=-1, keepdims=True))
        return np.einsum("hij,jhc->ihc", e / e.sum(axis=-1, keepdims=True), np.repeat(vv, g, axis=1))

    return float(np.abs(attend(q8) - attend(qr)).max())


def bf16_rounding_floor(w: Workload, n: int, layer: int = 0, want_lse: bool = False):
    """bf16_floor_arrays for query n of a workload."""
    pk, pv = w.prefix_kv(int(w.labels[n]), layer)
    q, k, v = w.suffix_qkv_query(n, layer)
    return bf16_floor_arrays(pk, pv, q, k, v, w.rope_base, want_lse)


def tight_bar(w: Workload, queries, layer: int = 0, factor: float = 4.0, floor_min: float = 5e-4):
    """(o_bar, lse_bar): `factor` times the largest bf16 rounding floor over the given queries."""
    fl = [bf16_rounding_floor(w, n, layer, want_lse=True) for n in queries if w.suffix_len[n] > 0]
    return factor * max([f[0] for f in fl] + [floor_min]), factor * max([f[1] for f in fl] + [floor_min])


def err_stats(o_gpu: np.ndarray, o_ref: np.ndarray) -> Dict[str, float]:
    d = np.abs(o_gpu.astype(np.float64) - o_ref)
    rms = float(np.sqrt(np.mean(o_ref ** 2))) if o_ref.size else 0.0
    return {"max_abs": float(d.max()) if d.size else 0.0, "rms_ref": rms,
            "rel": float(d.max() / rms) if d.size and rms > 0 else 0.0}
