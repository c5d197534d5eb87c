"""ctypes binding of ``libsgc.so``: the same entry points as ``include/sgc.h``, argument
marshalling only.  Device buffers are passed as integer addresses (``tensor.data_ptr()``) and the
stream as ``torch.cuda.current_stream().cuda_stream``; every step of the path runs inside the
library's kernels.  Loading fails loudly when the library has not been built."""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsgc.so")

SGC_OK, SGC_EINVAL, SGC_ENOMEM, SGC_ESHAPE, SGC_EUNSUPPORTED, SGC_EHIP, SGC_ESTATE = 0, -1, -2, -3, -4, -5, -6
SGC_F32, SGC_BF16, SGC_FP8_E4M3 = 0, 1, 2
SGC_KERNEL_AUTO, SGC_KERNEL_GENERIC, SGC_KERNEL_MFMA, SGC_KERNEL_MFMA_FP8 = 0, 1, 2, 3
DTYPES = {"f32": SGC_F32, "bf16": SGC_BF16, "fp8_e4m3": SGC_FP8_E4M3}

# every symbol include/sgc.h declares
EXPORTS = [
    "sgc_version", "sgc_status_string", "sgc_ctx_create", "sgc_ctx_destroy", "sgc_last_error",
    "sgc_cache_page_bytes", "sgc_cache_pool_bytes", "sgc_cache_create", "sgc_cache_destroy",
    "sgc_cache_alloc_cluster", "sgc_cache_free_cluster", "sgc_cache_total_pages", "sgc_cache_free_pages",
    "sgc_cache_cluster_pages", "sgc_prefix_prefill", "sgc_prefix_prefill_batched", "sgc_assign_clusters", "sgc_plan_upload",
    "sgc_plan_get_info", "sgc_plan_destroy", "sgc_suffix_prefill_batched", "sgc_cache_export", "sgc_cache_import",
    "sgc_timing_enable", "sgc_timing_last", "sgc_cluster_queries", "sgc_plan_enable_decode", "sgc_decode_step_batched",
    "sgc_union_subgraphs", "sgc_project_qkv_prefix", "sgc_project_qkv_prefix_batched", "sgc_project_qkv_suffix",
    "sgc_project_out", "sgc_timing_get", "sgc_decode_step_batched_noalloc",
]


class sgc_attn_params(ctypes.Structure):
    _fields_ = [
        ("struct_size", ctypes.c_uint32), ("n_q_heads", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32),
        ("head_dim", ctypes.c_int32), ("n_layers", ctypes.c_int32), ("page_tokens", ctypes.c_int32),
        ("io_dtype", ctypes.c_int32), ("kv_dtype", ctypes.c_int32), ("rope_base", ctypes.c_float),
        ("softmax_scale", ctypes.c_float), ("max_position", ctypes.c_int32), ("kernel", ctypes.c_int32),
    ]


class sgc_plan_info(ctypes.Structure):
    _fields_ = [
        ("n_queries", ctypes.c_int32), ("n_clusters", ctypes.c_int32), ("total_tokens", ctypes.c_int64),
        ("max_position", ctypes.c_int32), ("tile_rows", ctypes.c_int32), ("n_tiles", ctypes.c_int32),
    ]


class SgcError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"{status_string(status)}: {message}")
        self.status = status


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it first (python -c 'import __graft_entry__ as g; g.build()')")
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, i64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64
        i32p, f32p = ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_float)
        pp = ctypes.POINTER(sgc_attn_params)
        L.sgc_version.restype = ctypes.c_char_p
        L.sgc_status_string.argtypes = [ctypes.c_int]
        L.sgc_status_string.restype = ctypes.c_char_p
        L.sgc_ctx_create.argtypes = [pp, ctypes.POINTER(vp)]
        L.sgc_ctx_destroy.argtypes = [vp]
        L.sgc_last_error.argtypes = [vp]
        L.sgc_last_error.restype = ctypes.c_char_p
        L.sgc_cache_page_bytes.argtypes = [pp]
        L.sgc_cache_page_bytes.restype = ctypes.c_size_t
        L.sgc_cache_pool_bytes.argtypes = [pp, i64]
        L.sgc_cache_pool_bytes.restype = ctypes.c_size_t
        L.sgc_cache_create.argtypes = [vp, vp, ctypes.c_size_t, i32, ctypes.POINTER(vp)]
        L.sgc_cache_destroy.argtypes = [vp]
        L.sgc_cache_alloc_cluster.argtypes = [vp, i32, i32]
        L.sgc_cache_free_cluster.argtypes = [vp, i32]
        L.sgc_cache_total_pages.argtypes = [vp]
        L.sgc_cache_total_pages.restype = i64
        L.sgc_cache_free_pages.argtypes = [vp]
        L.sgc_cache_free_pages.restype = i64
        L.sgc_cache_cluster_pages.argtypes = [vp, i32, i32p, i32, i32p]
        L.sgc_prefix_prefill.argtypes = [vp, vp, i32, i32, vp, vp, vp, vp, vp, i32, vp]
        vpp = ctypes.POINTER(ctypes.c_void_p)
        L.sgc_prefix_prefill_batched.argtypes = [vp, vp, i32, i32p, i32, vpp, vpp, vpp, vpp, vpp, vp]
        L.sgc_assign_clusters.argtypes = [vp, vp, i32, i32p, i32p, i32, i32p, i32p, i32p, ctypes.POINTER(vp)]
        L.sgc_plan_upload.argtypes = [vp, vp]
        L.sgc_plan_get_info.argtypes = [vp, ctypes.POINTER(sgc_plan_info)]
        L.sgc_plan_destroy.argtypes = [vp]
        L.sgc_suffix_prefill_batched.argtypes = [vp, vp, vp, i32, vp, vp, vp, vp, vp, vp]
        L.sgc_cache_export.argtypes = [vp, vp, i32, i32, vp, vp, f32p, f32p, vp]
        L.sgc_cache_import.argtypes = [vp, vp, i32, i32, vp, vp, f32p, f32p, vp]
        L.sgc_plan_enable_decode.argtypes = [vp, i32]
        L.sgc_decode_step_batched.argtypes = [vp, vp, vp, i32, i32, vp, vp, vp, vp, vp, vp]
        L.sgc_decode_step_batched_noalloc.argtypes = [vp, vp, vp, i32, i32, vp, vp, vp, vp, vp, vp]
        i64p = ctypes.POINTER(ctypes.c_int64)
        L.sgc_union_subgraphs.argtypes = [vp, i32, i32p, i32, i64p, i32p, i64p, i32p, i64p, i32p, i64p, i32p]
        L.sgc_cluster_queries.argtypes = [vp, i32, i32, f32p, i32, i32, i32p]
        L.sgc_project_qkv_prefix.argtypes = [vp, vp, i32, i32, vp, vp, i32, vp, i32, vp]
        L.sgc_project_qkv_prefix_batched.argtypes = [vp, vp, i32, i32p, i32, vpp, vp, i32, vpp, vp]
        L.sgc_project_qkv_suffix.argtypes = [vp, vp, vp, i32, vp, vp, i32, vp, vp]
        L.sgc_project_out.argtypes = [vp, vp, vp, i32, i64, vp, vp]
        L.sgc_timing_enable.argtypes = [vp, ctypes.c_int]
        L.sgc_timing_last.argtypes = [vp, f32p, f32p]
        L.sgc_timing_get.argtypes = [vp, i32, f32p, f32p]
        for name in EXPORTS:
            fn = getattr(L, name)
            if fn.restype is ctypes.c_int and name not in ("sgc_version",):
                fn.restype = ctypes.c_int
        _lib = L
    return _lib


def version() -> str:
    return lib().sgc_version().decode()


def status_string(status: int) -> str:
    return lib().sgc_status_string(int(status)).decode()


def make_params(*, n_q_heads: int, n_kv_heads: int, head_dim: int, n_layers: int = 1, io_dtype="bf16",
                kv_dtype=None, rope_base: float = 10000.0, softmax_scale: float = 0.0, max_position: int = 0,
                kernel: int = SGC_KERNEL_AUTO, page_tokens: int = 16) -> sgc_attn_params:
    io = DTYPES[io_dtype] if isinstance(io_dtype, str) else int(io_dtype)
    kv = io if kv_dtype is None else (DTYPES[kv_dtype] if isinstance(kv_dtype, str) else int(kv_dtype))
    return sgc_attn_params(ctypes.sizeof(sgc_attn_params), n_q_heads, n_kv_heads, head_dim, n_layers, page_tokens,
                           io, kv, rope_base, softmax_scale, max_position, kernel)


def _check(ctx, rc: int):
    if rc < 0:
        raise SgcError(rc, sgc_last_error(ctx))
    return rc


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def _i32p(a: np.ndarray):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))


# ---- the entry points, same names as the header ---------------------------------------------------
def sgc_last_error(ctx) -> str:
    return lib().sgc_last_error(ctx).decode()


def sgc_ctx_create(params: sgc_attn_params):
    out = ctypes.c_void_p()
    rc = lib().sgc_ctx_create(ctypes.byref(params), ctypes.byref(out))
    _check(None, rc)
    return out


def sgc_ctx_destroy(ctx) -> None:
    lib().sgc_ctx_destroy(ctx)


def sgc_cache_page_bytes(params: sgc_attn_params) -> int:
    return int(lib().sgc_cache_page_bytes(ctypes.byref(params)))


def sgc_cache_pool_bytes(params: sgc_attn_params, total_pages: int) -> int:
    return int(lib().sgc_cache_pool_bytes(ctypes.byref(params), int(total_pages)))


def sgc_cache_create(ctx, dev_pool: int, pool_bytes: int, max_clusters: int):
    out = ctypes.c_void_p()
    _check(ctx, lib().sgc_cache_create(ctx, ctypes.c_void_p(dev_pool), pool_bytes, max_clusters, ctypes.byref(out)))
    return out


def sgc_cache_destroy(cache) -> None:
    lib().sgc_cache_destroy(cache)


def sgc_cache_alloc_cluster(ctx, cache, cluster_id: int, prefix_len: int) -> None:
    _check(ctx, lib().sgc_cache_alloc_cluster(cache, cluster_id, prefix_len))


def sgc_cache_free_cluster(ctx, cache, cluster_id: int) -> None:
    _check(ctx, lib().sgc_cache_free_cluster(cache, cluster_id))


def sgc_cache_total_pages(cache) -> int:
    return int(lib().sgc_cache_total_pages(cache))


def sgc_cache_free_pages(cache) -> int:
    return int(lib().sgc_cache_free_pages(cache))


def sgc_cache_cluster_pages(ctx, cache, cluster_id: int) -> Tuple[np.ndarray, int]:
    plen = ctypes.c_int32()
    n = _check(ctx, lib().sgc_cache_cluster_pages(cache, cluster_id, None, 0, ctypes.byref(plen)))
    pages = np.zeros(max(n, 1), dtype=np.int32)
    _check(ctx, lib().sgc_cache_cluster_pages(cache, cluster_id, _i32p(pages), n, None))
    return pages[:n], int(plen.value)


def sgc_prefix_prefill(ctx, cache, cluster_id: int, layer: int, dev_q: Optional[int], dev_k: int, dev_v: int,
                       dev_o: Optional[int], dev_lse: Optional[int], prefix_len: int, stream: int = 0) -> None:
    _check(ctx, lib().sgc_prefix_prefill(ctx, cache, cluster_id, layer, dev_q, dev_k, dev_v, dev_o, dev_lse,
                                         prefix_len, stream))


def _ptr_array(ptrs, n: int):
    """None, or a sequence of n device addresses (None entries allowed) -> ctypes array of void pointers."""
    if ptrs is None:
        return None
    if len(ptrs) != n:
        raise ValueError("pointer list and cluster list differ in length")
    return (ctypes.c_void_p * n)(*[None if p is None else int(p) for p in ptrs])


def sgc_prefix_prefill_batched(ctx, cache, cluster_ids: Sequence[int], layer: int, dev_q, dev_k, dev_v, dev_o,
                               dev_lse=None, stream: int = 0) -> None:
    """dev_q / dev_k / dev_v / dev_o / dev_lse: sequences of device addresses, one per cluster (or None)."""
    ids = _i32(cluster_ids)
    n = ids.shape[0]
    _check(ctx, lib().sgc_prefix_prefill_batched(ctx, cache, n, ids.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)), layer,
                                                 _ptr_array(dev_q, n), _ptr_array(dev_k, n), _ptr_array(dev_v, n),
                                                 _ptr_array(dev_o, n), _ptr_array(dev_lse, n), stream))


def sgc_assign_clusters(ctx, cache, labels: Sequence[int], suffix_len: Sequence[int], n_clusters: int,
                        want_plan: bool = True):
    """Returns (order, cluster_off, cu_seqlens, plan); plan is None when want_plan is False."""
    labels, suffix_len = _i32(labels), _i32(suffix_len)
    n = labels.shape[0]
    if suffix_len.shape[0] != n:
        raise ValueError("labels and suffix_len differ in length")
    order = np.zeros(max(n, 1), dtype=np.int32)
    cluster_off = np.zeros(max(n_clusters, 0) + 1, dtype=np.int32)
    cu = np.zeros(n + 1, dtype=np.int32)
    plan = ctypes.c_void_p()
    _check(ctx, lib().sgc_assign_clusters(ctx, cache, n, _i32p(labels), _i32p(suffix_len), n_clusters, _i32p(order),
                                          _i32p(cluster_off), _i32p(cu), ctypes.byref(plan) if want_plan else None))
    return order[:n], cluster_off, cu, (plan if want_plan else None)


def sgc_plan_upload(ctx, plan, stream: int = 0) -> None:
    _check(ctx, lib().sgc_plan_upload(plan, stream))


def sgc_plan_get_info(ctx, plan) -> sgc_plan_info:
    info = sgc_plan_info()
    _check(ctx, lib().sgc_plan_get_info(plan, ctypes.byref(info)))
    return info


def sgc_plan_destroy(plan) -> None:
    lib().sgc_plan_destroy(plan)


def sgc_suffix_prefill_batched(ctx, cache, plan, layer: int, dev_q: int, dev_k: int, dev_v: int, dev_o: int,
                               dev_lse: Optional[int] = None, stream: int = 0) -> None:
    _check(ctx, lib().sgc_suffix_prefill_batched(ctx, cache, plan, layer, dev_q, dev_k, dev_v, dev_o, dev_lse, stream))


def sgc_project_qkv_prefix(ctx, cache, cluster_id: int, layer: int, dev_x: int, dev_w_qkv: int, d_model: int,
                           dev_q: Optional[int], prefix_len: int, stream: int = 0) -> None:
    _check(ctx, lib().sgc_project_qkv_prefix(ctx, cache, cluster_id, layer, dev_x, dev_w_qkv, d_model, dev_q, prefix_len, stream))


def sgc_project_qkv_prefix_batched(ctx, cache, cluster_ids: Sequence[int], layer: int, dev_x, dev_w_qkv: int, d_model: int,
                                   dev_q=None, stream: int = 0) -> None:
    """dev_x / dev_q: sequences of device addresses, one per cluster (dev_q may be None or hold None entries)."""
    ids = _i32(cluster_ids)
    n = ids.shape[0]
    _check(ctx, lib().sgc_project_qkv_prefix_batched(ctx, cache, n, ids.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)), layer,
                                                     _ptr_array(dev_x, n), dev_w_qkv, d_model, _ptr_array(dev_q, n), stream))


def sgc_project_qkv_suffix(ctx, cache, plan, layer: int, dev_x: int, dev_w_qkv: int, d_model: int, dev_q: int,
                           stream: int = 0) -> None:
    _check(ctx, lib().sgc_project_qkv_suffix(ctx, cache, plan, layer, dev_x, dev_w_qkv, d_model, dev_q, stream))


def sgc_project_out(ctx, dev_o: int, dev_w_o: int, d_model: int, n_tokens: int, dev_y: int, stream: int = 0) -> None:
    _check(ctx, lib().sgc_project_out(ctx, dev_o, dev_w_o, d_model, n_tokens, dev_y, stream))


def sgc_plan_enable_decode(ctx, plan, max_new_tokens: int) -> None:
    _check(ctx, lib().sgc_plan_enable_decode(plan, int(max_new_tokens)))


def sgc_decode_step_batched(ctx, cache, plan, layer: int, step: int, dev_q: int, dev_k: int, dev_v: int, dev_o: int,
                            dev_lse: Optional[int] = None, stream: int = 0) -> None:
    _check(ctx, lib().sgc_decode_step_batched(ctx, cache, plan, layer, step, dev_q, dev_k, dev_v, dev_o, dev_lse, stream))


def sgc_decode_step_batched_noalloc(ctx, cache, plan, layer: int, step: int, dev_q: int, dev_k: int, dev_v: int, dev_o: int,
                                    dev_lse: Optional[int] = None, stream: int = 0) -> None:
    _check(ctx, lib().sgc_decode_step_batched_noalloc(ctx, cache, plan, layer, step, dev_q, dev_k, dev_v, dev_o, dev_lse,
                                                      stream))


LINKAGES = {"ward": 0, "single": 1, "average": 2, "complete": 3, "centroid": 4}


def sgc_cluster_queries(ctx, embeddings: np.ndarray, n_clusters: int, linkage="ward") -> np.ndarray:
    """Host embeddings [m][dim] -> int32 cluster labels [m] (ctx may be None)."""
    x = np.ascontiguousarray(embeddings, dtype=np.float32)
    if x.ndim != 2:
        raise ValueError("embeddings must be [m][dim]")
    m, dim = x.shape
    labels = np.zeros(m, dtype=np.int32)
    code = LINKAGES[linkage] if isinstance(linkage, str) else int(linkage)
    rc = lib().sgc_cluster_queries(ctx, m, dim, x.ctypes.data_as(ctypes.POINTER(ctypes.c_float)), code, int(n_clusters),
                                   labels.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)))
    if rc < 0:
        raise SgcError(rc, sgc_last_error(ctx) if ctx is not None else "sgc_cluster_queries failed")
    return labels


def sgc_union_subgraphs(ctx, labels: Sequence[int], n_clusters: int, node_lists, edge_lists):
    """node_lists[i]: node ids of query i's subgraph; edge_lists[i]: its (src, dst) pairs.  Returns (nodes,
    edges): per cluster an int32 array of node ids and an int32 [n][2] array of edges (ctx may be None)."""
    labels = _i32(labels)
    m = labels.shape[0]
    if len(node_lists) != m or len(edge_lists) != m:
        raise ValueError("one node list and one edge list per query")
    nl = [np.asarray(x, dtype=np.int32).reshape(-1) for x in node_lists]
    el = [np.asarray(x, dtype=np.int32).reshape(-1, 2) for x in edge_lists]
    node_off = np.zeros(m + 1, dtype=np.int64)
    edge_off = np.zeros(m + 1, dtype=np.int64)
    np.cumsum([x.shape[0] for x in nl], out=node_off[1:])
    np.cumsum([x.shape[0] for x in el], out=edge_off[1:])
    nodes = np.ascontiguousarray(np.concatenate(nl + [np.zeros(1, dtype=np.int32)]))        # (never empty)
    edges = np.ascontiguousarray(np.concatenate(el + [np.zeros((1, 2), dtype=np.int32)]))
    out_noff = np.zeros(n_clusters + 1, dtype=np.int64)
    out_eoff = np.zeros(n_clusters + 1, dtype=np.int64)
    out_nodes = np.zeros_like(nodes)
    out_edges = np.zeros_like(edges)
    i32p, i64p = ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_int64)
    rc = lib().sgc_union_subgraphs(ctx, m, labels.ctypes.data_as(i32p), int(n_clusters), node_off.ctypes.data_as(i64p),
                                   nodes.ctypes.data_as(i32p), edge_off.ctypes.data_as(i64p), edges.ctypes.data_as(i32p),
                                   out_noff.ctypes.data_as(i64p), out_nodes.ctypes.data_as(i32p),
                                   out_eoff.ctypes.data_as(i64p), out_edges.ctypes.data_as(i32p))
    if rc < 0:
        raise SgcError(rc, sgc_last_error(ctx) if ctx is not None else "sgc_union_subgraphs failed")
    return ([out_nodes[out_noff[k]:out_noff[k + 1]].copy() for k in range(n_clusters)],
            [out_edges[out_eoff[k]:out_eoff[k + 1]].copy() for k in range(n_clusters)])


def sgc_timing_enable(ctx, on) -> None:
    """on: False / 0 = off, True / 1 = every suffix launch, n > 1 = every n-th."""
    _check(ctx, lib().sgc_timing_enable(ctx, int(on)))


def sgc_timing_last(ctx) -> Tuple[float, float]:
    """(suffix ingest ms, attention kernel ms) of the last timed sgc_suffix_prefill_batched call."""
    a, b = ctypes.c_float(0), ctypes.c_float(0)
    _check(ctx, lib().sgc_timing_last(ctx, ctypes.byref(a), ctypes.byref(b)))
    return a.value, b.value


def sgc_timing_get(ctx, back: int) -> Tuple[float, float]:
    """The same for the launch `back` timed launches before the last one (the last 128 are kept)."""
    a, b = ctypes.c_float(0), ctypes.c_float(0)
    _check(ctx, lib().sgc_timing_get(ctx, int(back), ctypes.byref(a), ctypes.byref(b)))
    return a.value, b.value


def sgc_cache_export(ctx, cache, cluster_id: int, layer: int, dev_k: int, dev_v: int, n_kv_heads: int,
                     stream: int = 0) -> Tuple[np.ndarray, np.ndarray]:
    ks = np.zeros(n_kv_heads, dtype=np.float32)
    vs = np.zeros(n_kv_heads, dtype=np.float32)
    fp = ctypes.POINTER(ctypes.c_float)
    _check(ctx, lib().sgc_cache_export(ctx, cache, cluster_id, layer, dev_k, dev_v, ks.ctypes.data_as(fp),
                                       vs.ctypes.data_as(fp), stream))
    return ks, vs


def sgc_cache_import(ctx, cache, cluster_id: int, layer: int, dev_k: int, dev_v: int, k_scale=None, v_scale=None,
                     stream: int = 0) -> None:
    fp = ctypes.POINTER(ctypes.c_float)
    ks = None if k_scale is None else np.ascontiguousarray(k_scale, dtype=np.float32)
    vs = None if v_scale is None else np.ascontiguousarray(v_scale, dtype=np.float32)
    _check(ctx, lib().sgc_cache_import(ctx, cache, cluster_id, layer, dev_k, dev_v,
                                       None if ks is None else ks.ctypes.data_as(fp),
                                       None if vs is None else vs.ctypes.data_as(fp), stream))
