"""Seeded synthetic workloads shaped like the paper's batches (inputs only, no attention math).

SubGCache (arXiv 2505.10951) is measured on two graph-RAG datasets that are not available
here; these generators stand in for them.  Shapes follow the paper's setup (Appendix A.2:
prompts of up to about a thousand tokens, one-sentence questions; Sec. 4.3 / Fig. 3: one to a
few tens of clusters per batch; Sec. 4.6 / Table 4: 50-200 queries per batch) and extend them
to longer prefixes and larger models.

This module only draws numbers and rounds them to the storage type the GPU receives.  Both the
GPU tests/benchmark and the CPU oracle's tests read their inputs from here; it imports neither.
Every tensor is drawn from ``numpy.random.Generator(PCG64(SeedSequence([seed, layer, kind,
index])))`` so any single cluster or query can be regenerated on its own.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, Optional, Tuple

import numpy as np

_KIND_PREFIX_Q, _KIND_PREFIX_K, _KIND_PREFIX_V = 1, 2, 3
_KIND_SUFFIX_Q, _KIND_SUFFIX_K, _KIND_SUFFIX_V = 4, 5, 6
_KIND_STRUCT, _KIND_OUTLIER = 7, 8
_KIND_EMBED_CENTRE, _KIND_EMBED_NOISE = 9, 10
_KIND_DECODE_Q, _KIND_DECODE_K, _KIND_DECODE_V = 11, 12, 13
_KIND_GRAPH = 14
_KIND_W_QKV, _KIND_W_O, _KIND_PREFIX_X, _KIND_SUFFIX_X = 15, 16, 17, 18


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round fp32 values to the nearest bfloat16 (ties to even); result is fp32 holding bf16 values."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    r = ((u + bias) & np.uint32(0xFFFF0000)).astype(np.uint32)
    return r.view(np.float32).reshape(x.shape)


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """Upper 16 bits of fp32 values that are already bf16-representable (uint16)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    return (x.view(np.uint32) >> np.uint32(16)).astype(np.uint16).reshape(x.shape)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32).reshape(b.shape)


@dataclass
class Workload:
    name: str
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    rope_base: float
    io_dtype: str                 # "f32" | "bf16"
    kv_dtype: str                 # "f32" | "bf16" | "fp8_e4m3"
    n_layers: int
    prefix_len: np.ndarray        # int32 [n_clusters]
    labels: np.ndarray            # int32 [n_queries], cluster of each query, original order
    suffix_len: np.ndarray        # int32 [n_queries]
    seed: int
    page_tokens: int = 16
    k_outlier_scale: float = 1.0  # >1: one seeded channel per KV head of every K is multiplied by it
    q_gain: float = 1.0           # multiplies Q (peaky-softmax test workloads)
    _outlier_cache: Dict[int, np.ndarray] = field(default_factory=dict, repr=False)

    # ---- structure -------------------------------------------------------------------------
    @property
    def n_clusters(self) -> int:
        return int(self.prefix_len.shape[0])

    @property
    def n_queries(self) -> int:
        return int(self.labels.shape[0])

    @property
    def cu_seqlens(self) -> np.ndarray:
        cu = np.zeros(self.n_queries + 1, dtype=np.int64)
        np.cumsum(self.suffix_len, out=cu[1:])
        return cu

    @property
    def total_suffix_tokens(self) -> int:
        return int(self.suffix_len.sum())

    def flops(self) -> float:
        """Algorithmic flop of one layer's batched suffix prefill: QK^T and PV over visible keys."""
        S = self.suffix_len.astype(np.float64)
        P = self.prefix_len[self.labels].astype(np.float64)
        return float(4.0 * self.n_q_heads * self.head_dim * np.sum(S * (P + (S + 1.0) / 2.0)))

    def io_bytes(self) -> int:
        return 4 if self.io_dtype == "f32" else 2

    def kv_bytes(self) -> int:
        return {"f32": 4, "bf16": 2, "fp8_e4m3": 1}[self.kv_dtype]

    def algorithmic_bytes(self) -> float:
        """Bytes one layer's batched suffix prefill must move: each cluster's cached prefix K+V once,
        Q in, O out, suffix K and V in."""
        T = self.total_suffix_tokens
        used = np.unique(self.labels)
        cache = 2.0 * float(self.prefix_len[used].sum()) * self.n_kv_heads * self.head_dim * self.kv_bytes()
        qo = 2.0 * T * self.n_q_heads * self.head_dim * self.io_bytes()
        skv = 2.0 * T * self.n_kv_heads * self.head_dim * self.io_bytes()
        return cache + qo + skv

    # ---- tensors ---------------------------------------------------------------------------
    def _rng(self, layer: int, kind: int, index: int) -> np.random.Generator:
        return np.random.Generator(np.random.PCG64(np.random.SeedSequence([self.seed, layer, kind, index])))

    def _store(self, x: np.ndarray) -> np.ndarray:
        return round_to_bf16(x) if self.io_dtype == "bf16" else np.ascontiguousarray(x, dtype=np.float32)

    def _outlier_channels(self, layer: int) -> np.ndarray:
        """One channel index per KV head (1 % of head_dim, at least one), fixed per layer."""
        if layer not in self._outlier_cache:
            n = max(1, int(round(0.01 * self.head_dim)))
            rng = self._rng(layer, _KIND_OUTLIER, 0)
            self._outlier_cache[layer] = np.stack(
                [rng.choice(self.head_dim, size=n, replace=False) for _ in range(self.n_kv_heads)])
        return self._outlier_cache[layer]

    def _k_post(self, k: np.ndarray, layer: int) -> np.ndarray:
        if self.k_outlier_scale != 1.0:
            ch = self._outlier_channels(layer)
            for h in range(self.n_kv_heads):
                k[:, h, ch[h]] *= np.float32(self.k_outlier_scale)
        return k

    def prefix_kv(self, cluster: int, layer: int = 0) -> Tuple[np.ndarray, np.ndarray]:
        """Un-rotated prefix K, V of one cluster: fp32 arrays [P_c][Hkv][d] holding storage-type values."""
        P = int(self.prefix_len[cluster])
        shp = (P, self.n_kv_heads, self.head_dim)
        k = self._rng(layer, _KIND_PREFIX_K, cluster).standard_normal(shp, dtype=np.float32)
        v = self._rng(layer, _KIND_PREFIX_V, cluster).standard_normal(shp, dtype=np.float32)
        return self._store(self._k_post(k, layer)), self._store(v)

    def prefix_q(self, cluster: int, layer: int = 0) -> np.ndarray:
        P = int(self.prefix_len[cluster])
        q = self._rng(layer, _KIND_PREFIX_Q, cluster).standard_normal(
            (P, self.n_q_heads, self.head_dim), dtype=np.float32)
        return self._store(q * np.float32(self.q_gain))

    def suffix_qkv_query(self, n: int, layer: int = 0) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
        """Un-rotated Q [S][Hq][d], K, V [S][Hkv][d] of query n."""
        S = int(self.suffix_len[n])
        q = self._rng(layer, _KIND_SUFFIX_Q, n).standard_normal((S, self.n_q_heads, self.head_dim), dtype=np.float32)
        k = self._rng(layer, _KIND_SUFFIX_K, n).standard_normal((S, self.n_kv_heads, self.head_dim), dtype=np.float32)
        v = self._rng(layer, _KIND_SUFFIX_V, n).standard_normal((S, self.n_kv_heads, self.head_dim), dtype=np.float32)
        return self._store(q * np.float32(self.q_gain)), self._store(self._k_post(k, layer)), self._store(v)

    def decode_qkv(self, step: int, layer: int = 0) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
        """Un-rotated Q [n_queries][Hq][d], K, V [n_queries][Hkv][d] of the token every query generates at
        decode step `step` (stand-ins for the projections of generated tokens; same recipe as the suffix)."""
        n = self.n_queries
        q = self._rng(layer, _KIND_DECODE_Q, step).standard_normal((n, self.n_q_heads, self.head_dim), dtype=np.float32)
        k = self._rng(layer, _KIND_DECODE_K, step).standard_normal((n, self.n_kv_heads, self.head_dim), dtype=np.float32)
        v = self._rng(layer, _KIND_DECODE_V, step).standard_normal((n, self.n_kv_heads, self.head_dim), dtype=np.float32)
        return self._store(q * np.float32(self.q_gain)), self._store(self._k_post(k, layer)), self._store(v)

    def query_embeddings(self, dim: int = 64, overlap: float = 0.15) -> np.ndarray:
        """Stand-in for the GNN embeddings of the queries' retrieved subgraphs: fp32 [n_queries][dim].  Queries
        of one cluster share a centre (a unit-scale Gaussian point); each adds Gaussian noise of standard
        deviation `overlap` per coordinate, so that the workload's labels are the clustering's ground truth
        for small overlap and become ambiguous as it grows."""
        centres = self._rng(0, _KIND_EMBED_CENTRE, 0).standard_normal((max(self.n_clusters, 1), dim), dtype=np.float32)
        noise = self._rng(0, _KIND_EMBED_NOISE, 0).standard_normal((self.n_queries, dim), dtype=np.float32)
        return np.ascontiguousarray(centres[self.labels] + np.float32(overlap) * noise, dtype=np.float32)

    def retrieved_subgraphs(self, graph_nodes: int = 5000, core: int = 24, extra: int = 4):
        """Stand-in for the subgraphs retrieved per query (the paper retrieves a few dozen nodes per query from the
        Scene Graph / OAG graphs): queries of a cluster draw most of their nodes from the cluster's `core` nodes
        and add `extra` nodes of their own; edges are random pairs among a query's nodes.  Returns (node_lists,
        edge_lists) with duplicates left in."""
        rng = self._rng(0, _KIND_GRAPH, 0)
        cores = [rng.choice(graph_nodes, size=core, replace=False) for _ in range(max(self.n_clusters, 1))]
        node_lists, edge_lists = [], []
        for n in range(self.n_queries):
            own = np.concatenate([rng.choice(cores[int(self.labels[n])], size=max(core * 3 // 4, 1), replace=True),
                                  rng.integers(0, graph_nodes, size=extra)])
            pairs = rng.choice(own, size=(2 * own.size, 2))
            node_lists.append(own.astype(np.int32))
            edge_lists.append(pairs.astype(np.int32))
        return node_lists, edge_lists

    # ---- the attention layer around the kernel (hidden states and projection weights) -------
    def layer_weights(self, d_model: int, layer: int = 0) -> Tuple[np.ndarray, np.ndarray]:
        """Random stand-ins for a trained layer's projections (the paper's backbones keep their weights in
        "out features x in features" order): w_qkv [(Hq + 2 Hkv) d][d_model], rows = Q heads, then K heads,
        then V heads, head-major; w_o [d_model][Hq d].  Entries are N(0, 1 / in_features), so projected Q, K, V
        have unit variance like the direct Q, K, V recipes above."""
        n_qkv = (self.n_q_heads + 2 * self.n_kv_heads) * self.head_dim
        n_o = self.n_q_heads * self.head_dim
        w_qkv = self._rng(layer, _KIND_W_QKV, 0).standard_normal((n_qkv, d_model), dtype=np.float32)
        w_qkv *= np.float32(1.0 / np.sqrt(d_model))
        w_qkv[: n_o] *= np.float32(self.q_gain)
        w_o = self._rng(layer, _KIND_W_O, 0).standard_normal((d_model, n_o), dtype=np.float32)
        w_o *= np.float32(1.0 / np.sqrt(n_o))
        return self._store(w_qkv), self._store(w_o)

    def prefix_x(self, cluster: int, d_model: int, layer: int = 0) -> np.ndarray:
        """Hidden states entering the layer for the cluster's prompt tokens: [P_c][d_model], N(0, 1)."""
        P = int(self.prefix_len[cluster])
        return self._store(self._rng(layer, _KIND_PREFIX_X, cluster).standard_normal((P, d_model), dtype=np.float32))

    def suffix_x_query(self, n: int, d_model: int, layer: int = 0) -> np.ndarray:
        S = int(self.suffix_len[n])
        return self._store(self._rng(layer, _KIND_SUFFIX_X, n).standard_normal((S, d_model), dtype=np.float32))

    def suffix_x(self, d_model: int, layer: int = 0) -> np.ndarray:
        """All queries' question-token hidden states packed in original order: [T][d_model]."""
        cu = self.cu_seqlens
        x = np.empty((self.total_suffix_tokens, d_model), dtype=np.float32)
        for n in range(self.n_queries):
            a, b = int(cu[n]), int(cu[n + 1])
            if b > a:
                x[a:b] = self.suffix_x_query(n, d_model, layer)
        return x

    def suffix_qkv(self, layer: int = 0, threads: int = 1) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
        """All queries packed in original order: Q [T][Hq][d], K, V [T][Hkv][d].  Every query has its own
        random stream, so `threads` > 1 draws them side by side and gives the same arrays."""
        T = self.total_suffix_tokens
        cu = self.cu_seqlens
        q = np.empty((T, self.n_q_heads, self.head_dim), dtype=np.float32)
        k = np.empty((T, self.n_kv_heads, self.head_dim), dtype=np.float32)
        v = np.empty((T, self.n_kv_heads, self.head_dim), dtype=np.float32)
        self._outlier_channels(layer)             # drawn once, before any worker asks for it

        def one(n: int) -> None:
            a, b = int(cu[n]), int(cu[n + 1])
            if b > a:
                q[a:b], k[a:b], v[a:b] = self.suffix_qkv_query(n, layer)

        if threads > 1:
            from concurrent.futures import ThreadPoolExecutor
            with ThreadPoolExecutor(max_workers=threads) as ex:
                list(ex.map(one, range(self.n_queries)))
        else:
            for n in range(self.n_queries):
                one(n)
        return q, k, v


# --------------------------------------------------------------------------------------------
# Structure helpers
# --------------------------------------------------------------------------------------------
def _struct_rng(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, 0, _KIND_STRUCT, 0])))


def zipf_cluster_sizes(n_clusters: int, total: int, exponent: float = 1.1) -> np.ndarray:
    """Cluster sizes proportional to k^-exponent (k = 1..n_clusters), largest-remainder rounding,
    each at least one, summing to `total`."""
    w = np.arange(1, n_clusters + 1, dtype=np.float64) ** (-exponent)
    ideal = total * w / w.sum()
    sizes = np.maximum(1, np.floor(ideal).astype(np.int64))
    while sizes.sum() > total:                      # only when the floor-of-one rule overshoots
        sizes[np.argmax(sizes)] -= 1
    rem = ideal - np.floor(ideal)
    order = np.argsort(-rem, kind="stable")
    i = 0
    while sizes.sum() < total:
        sizes[order[i % n_clusters]] += 1
        i += 1
    return sizes.astype(np.int32)


def _labels_from_sizes(sizes: np.ndarray, rng: np.random.Generator) -> np.ndarray:
    labels = np.repeat(np.arange(len(sizes), dtype=np.int32), sizes)
    rng.shuffle(labels)
    return labels


def custom(name: str, *, n_q_heads: int, n_kv_heads: int, head_dim: int, rope_base: float, io_dtype: str,
           kv_dtype: Optional[str] = None, prefix_len, queries_per_cluster=None, cluster_sizes=None,
           suffix_range=(16, 32), suffix_len=None, labels=None, n_layers: int = 1, seed: int = 0,
           k_outlier_scale: float = 1.0, q_gain: float = 1.0) -> Workload:
    """Build a workload from explicit structure (used by the scaled-down parity cases)."""
    rng = _struct_rng(seed)
    prefix_len = np.asarray(prefix_len, dtype=np.int32)
    nc = prefix_len.shape[0]
    if labels is None:
        if cluster_sizes is None:
            cluster_sizes = np.full(nc, int(queries_per_cluster), dtype=np.int32)
        labels = _labels_from_sizes(np.asarray(cluster_sizes, dtype=np.int32), rng)
    labels = np.asarray(labels, dtype=np.int32)
    if suffix_len is None:
        lo, hi = suffix_range
        suffix_len = rng.integers(lo, hi + 1, size=labels.shape[0]).astype(np.int32)
    suffix_len = np.asarray(suffix_len, dtype=np.int32)
    return Workload(name=name, n_q_heads=n_q_heads, n_kv_heads=n_kv_heads, head_dim=head_dim,
                    rope_base=float(rope_base), io_dtype=io_dtype, kv_dtype=kv_dtype or io_dtype,
                    n_layers=n_layers, prefix_len=prefix_len, labels=labels, suffix_len=suffix_len, seed=seed,
                    k_outlier_scale=k_outlier_scale, q_gain=q_gain)


def config(index: int, seed: Optional[int] = None, queries_per_cluster: Optional[int] = None) -> Workload:
    """The five benchmark workloads (index 0..4).  queries_per_cluster (configurations with equal clusters only: 0, 1, 3, 4)
    changes the batch size (and the workload's name) and nothing else: for sweeps of the launch size around the benchmark's own."""
    seed = (index + 1) * 1000 if seed is None else seed
    rng = _struct_rng(seed)
    if queries_per_cluster is not None:
        if index == 2:
            raise ValueError("configs[2] has Zipf cluster sizes; queries_per_cluster does not apply")
        base = config(index, seed)
        return custom(f"{base.name}_qpc{int(queries_per_cluster)}", n_q_heads=base.n_q_heads, n_kv_heads=base.n_kv_heads, head_dim=base.head_dim,
                      rope_base=base.rope_base, io_dtype=base.io_dtype, kv_dtype=base.kv_dtype, prefix_len=base.prefix_len,
                      queries_per_cluster=int(queries_per_cluster),
                      suffix_range=(int(base.suffix_len.min()), int(base.suffix_len.max())), n_layers=base.n_layers, seed=seed,
                      k_outlier_scale=base.k_outlier_scale, q_gain=base.q_gain)
    if index == 0:      # tiny fp32 MHA layer, the correctness case
        return custom("tiny_f32_mha", n_q_heads=4, n_kv_heads=4, head_dim=64, rope_base=10000.0, io_dtype="f32",
                      prefix_len=[256, 192], queries_per_cluster=8, suffix_range=(16, 32), seed=seed)
    if index == 1:      # Llama-3-8B-shaped GQA layer, bf16, K outlier channels
        return custom("llama3_8b_layer", n_q_heads=32, n_kv_heads=8, head_dim=128, rope_base=500000.0,
                      io_dtype="bf16", prefix_len=[1024] * 10, queries_per_cluster=32, suffix_range=(16, 64),
                      seed=seed, k_outlier_scale=8.0)
    if index == 2:      # Llama-2-7B-shaped MHA layer, variable prefixes, Zipf cluster sizes
        plen = rng.integers(1024, 4096 + 1, size=16).astype(np.int32)
        sizes = zipf_cluster_sizes(16, 1024, 1.1)
        rng.shuffle(sizes)                          # which prefix length meets which cluster size
        return custom("llama2_7b_ragged", n_q_heads=32, n_kv_heads=32, head_dim=128, rope_base=10000.0,
                      io_dtype="bf16", prefix_len=plen, cluster_sizes=sizes, suffix_range=(24, 96), seed=seed)
    if index == 3:      # 32-layer Llama-3-8B-shaped stack over a resident paged cache
        return custom("llama3_8b_stack32", n_q_heads=32, n_kv_heads=8, head_dim=128, rope_base=500000.0,
                      io_dtype="bf16", prefix_len=[4096] * 16, queries_per_cluster=16, suffix_range=(128, 128),
                      n_layers=32, seed=seed)
    if index == 4:      # 70B-shaped long-prefix layer, fp8 e4m3 cache
        return custom("llama70b_fp8_long", n_q_heads=64, n_kv_heads=8, head_dim=128, rope_base=500000.0,
                      io_dtype="bf16", kv_dtype="fp8_e4m3", prefix_len=[16384] * 8, queries_per_cluster=128,
                      suffix_range=(32, 256), seed=seed)
    raise ValueError("config index must be 0..4")
