"""Driver used by the GPU tests, the smoke check and the benchmark: moves a synthetic workload
into HBM with torch (device memory and streams only) and calls the library's entry points in the
order SubGCache Sec. 3.4 prescribes: allocate a cluster's cache, prefill its prefix once, map
the batch's queries to their clusters, run every query's suffix prefill, release."""
from __future__ import annotations

import os
from concurrent.futures import ThreadPoolExecutor
from typing import Dict, List, Optional

import numpy as np
import torch

from . import sgc
from .workloads import Workload


def _torch_dtype(name: str):
    return {"f32": torch.float32, "bf16": torch.bfloat16}[name]


def to_device(x: np.ndarray, io_dtype: str, device="cuda:0") -> torch.Tensor:
    """fp32 host values (already representable in io_dtype) -> device tensor of io_dtype."""
    t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32))
    if io_dtype == "bf16":
        t = t.to(torch.bfloat16)
    return t.to(device)


def to_host_f32(t: torch.Tensor) -> np.ndarray:
    return t.detach().to(torch.float32).cpu().numpy()


class Session:
    """One context + one cache pool on cuda:0 for a workload's geometry."""

    def __init__(self, w: Workload, total_pages: Optional[int] = None, kernel: int = sgc.SGC_KERNEL_AUTO,
                 max_clusters: Optional[int] = None, device: str = "cuda:0"):
        if not torch.cuda.is_available():
            raise RuntimeError("no GPU: the sgc attention path only runs on a HIP device")
        self.w = w
        self.device = device
        self.params = sgc.make_params(n_q_heads=w.n_q_heads, n_kv_heads=w.n_kv_heads, head_dim=w.head_dim,
                                      n_layers=w.n_layers, io_dtype=w.io_dtype, kv_dtype=w.kv_dtype,
                                      rope_base=w.rope_base, kernel=kernel,
                                      max_position=int((w.prefix_len.max() if w.n_clusters else 0) +
                                                       (w.suffix_len.max() if w.n_queries else 0)))
        self.ctx = sgc.sgc_ctx_create(self.params)
        if total_pages is None:
            total_pages = int(sum(-(-int(p) // w.page_tokens) for p in w.prefix_len)) + 1
        self.total_pages = total_pages
        nbytes = sgc.sgc_cache_pool_bytes(self.params, total_pages)
        self.pool = torch.empty(nbytes, dtype=torch.uint8, device=device)
        self.cache = sgc.sgc_cache_create(self.ctx, self.pool.data_ptr(), nbytes, max_clusters or max(w.n_clusters, 1))
        self.plan = None
        self._keep: List[torch.Tensor] = []

    @property
    def stream(self) -> int:
        return torch.cuda.current_stream().cuda_stream

    # ---- Sec. 3.4: compute the cluster's cache once -------------------------------------------
    def alloc_cluster(self, c: int) -> None:
        sgc.sgc_cache_alloc_cluster(self.ctx, self.cache, c, int(self.w.prefix_len[c]))

    def free_cluster(self, c: int) -> None:
        sgc.sgc_cache_free_cluster(self.ctx, self.cache, c)

    def prefix_prefill(self, c: int, layer: int = 0, with_q: bool = False, want_lse: bool = False,
                       k: Optional[np.ndarray] = None, v: Optional[np.ndarray] = None, q: Optional[np.ndarray] = None):
        w = self.w
        P = int(w.prefix_len[c])
        if k is None:
            k, v = w.prefix_kv(c, layer)
        dk, dv = to_device(k, w.io_dtype, self.device), to_device(v, w.io_dtype, self.device)
        dq = do = dlse = None
        if with_q:
            if q is None:
                q = w.prefix_q(c, layer)
            dq = to_device(q, w.io_dtype, self.device)
            do = torch.empty_like(dq)
            if want_lse:
                dlse = torch.empty((w.n_q_heads, max(P, 1)), dtype=torch.float32, device=self.device)
        sgc.sgc_prefix_prefill(self.ctx, self.cache, c, layer, dq.data_ptr() if dq is not None else None,
                               dk.data_ptr(), dv.data_ptr(), do.data_ptr() if do is not None else None,
                               dlse.data_ptr() if dlse is not None else None, P, self.stream)
        torch.cuda.synchronize()
        return do, (dlse[:, :P] if dlse is not None else None)

    def prefix_prefill_batched(self, clusters, layer: int = 0, with_q: bool = False, want_lse: bool = False):
        """All the given clusters in one call; returns per-cluster (o, lse) device tensors (None without q)."""
        w = self.w
        dk, dv, dq, do, dl = [], [], [], [], []
        for c in clusters:
            P = int(w.prefix_len[c])
            k, v = w.prefix_kv(c, layer)
            dk.append(to_device(k, w.io_dtype, self.device))
            dv.append(to_device(v, w.io_dtype, self.device))
            if with_q:
                dq.append(to_device(w.prefix_q(c, layer), w.io_dtype, self.device))
                do.append(torch.empty_like(dq[-1]))
                dl.append(torch.empty((w.n_q_heads, max(P, 1)), dtype=torch.float32, device=self.device) if want_lse else None)
        ptr = lambda ts: [None if t is None else t.data_ptr() for t in ts]
        sgc.sgc_prefix_prefill_batched(self.ctx, self.cache, list(clusters), layer, ptr(dq) if with_q else None, ptr(dk), ptr(dv),
                                       ptr(do) if with_q else None, ptr(dl) if (with_q and want_lse) else None, self.stream)
        torch.cuda.synchronize()
        if not with_q:
            return [(None, None) for _ in clusters]
        return [(o, (l[:, :int(w.prefix_len[c])] if l is not None else None)) for c, o, l in zip(clusters, do, dl)]

    def fill_all_clusters(self, layer: int = 0) -> None:
        for c in range(self.w.n_clusters):
            self.prefix_prefill(c, layer)

    # ---- Sec. 3.2 / 3.4: map queries to their cluster's cache -----------------------------------
    def assign(self, labels=None, suffix_len=None):
        w = self.w
        if self.plan is not None:
            sgc.sgc_plan_destroy(self.plan)
            self.plan = None
        order, off, cu, plan = sgc.sgc_assign_clusters(self.ctx, self.cache, w.labels if labels is None else labels,
                                                       w.suffix_len if suffix_len is None else suffix_len, w.n_clusters)
        self.plan = plan
        return order, off, cu

    def upload_plan(self) -> None:
        sgc.sgc_plan_upload(self.ctx, self.plan, self.stream)

    # ---- Sec. 3.4: every query appends its tokens to the cached prompt --------------------------
    def suffix_prefill(self, dq: torch.Tensor, dk: torch.Tensor, dv: torch.Tensor, layer: int = 0,
                       do: Optional[torch.Tensor] = None, dlse: Optional[torch.Tensor] = None):
        if do is None:
            do = torch.empty_like(dq)
        sgc.sgc_suffix_prefill_batched(self.ctx, self.cache, self.plan, layer, dq.data_ptr(), dk.data_ptr(),
                                       dv.data_ptr(), do.data_ptr(), dlse.data_ptr() if dlse is not None else None,
                                       self.stream)
        return do

    # ---- Sec. 3.4: the layer around the attention (hidden states in, hidden states out) -------------
    def layer_prefix(self, clusters, d_model: int, dw_qkv: torch.Tensor, dw_o: torch.Tensor, layer: int = 0,
                     with_output: bool = True):
        """QKV projection of the given clusters' prompts into their pages; with_output also runs the prompt's
        causal attention and the output projection.  Returns per-cluster y device tensors (or None)."""
        w = self.w
        dx = [to_device(w.prefix_x(c, d_model, layer), w.io_dtype, self.device) for c in clusters]
        nq = w.n_q_heads * w.head_dim
        dq = [torch.empty((x.shape[0], nq), dtype=x.dtype, device=self.device) if with_output else None for x in dx]
        ptr = lambda ts: [None if t is None else t.data_ptr() for t in ts]
        sgc.sgc_project_qkv_prefix_batched(self.ctx, self.cache, list(clusters), layer, ptr(dx), dw_qkv.data_ptr(), d_model,
                                           ptr(dq) if with_output else None, self.stream)
        if not with_output:
            torch.cuda.synchronize()
            return [None for _ in clusters]
        do = [torch.empty_like(q) for q in dq]
        sgc.sgc_prefix_prefill_batched(self.ctx, self.cache, list(clusters), layer, ptr(dq), None, None, ptr(do), None, self.stream)
        ys = []
        for o in do:
            y = torch.empty((o.shape[0], d_model), dtype=o.dtype, device=self.device)
            sgc.sgc_project_out(self.ctx, o.data_ptr(), dw_o.data_ptr(), d_model, o.shape[0], y.data_ptr(), self.stream)
            ys.append(y)
        torch.cuda.synchronize()
        return ys

    def layer_suffix(self, dx: torch.Tensor, d_model: int, dw_qkv: torch.Tensor, dw_o: torch.Tensor, layer: int = 0,
                     bufs=None):
        """Whole batch: QKV projection, attention over cache + own tokens, output projection.  Returns y [T][d_model]."""
        w = self.w
        T = dx.shape[0]
        if bufs is None:
            nq = w.n_q_heads * w.head_dim
            bufs = (torch.empty((T, nq), dtype=dx.dtype, device=self.device), torch.empty((T, nq), dtype=dx.dtype, device=self.device),
                    torch.empty((T, d_model), dtype=dx.dtype, device=self.device))
        dq, do, dy = bufs
        sgc.sgc_project_qkv_suffix(self.ctx, self.cache, self.plan, layer, dx.data_ptr(), dw_qkv.data_ptr(), d_model,
                                   dq.data_ptr(), self.stream)
        sgc.sgc_suffix_prefill_batched(self.ctx, self.cache, self.plan, layer, dq.data_ptr(), None, None, do.data_ptr(), None,
                                       self.stream)
        sgc.sgc_project_out(self.ctx, do.data_ptr(), dw_o.data_ptr(), d_model, T, dy.data_ptr(), self.stream)
        return dy

    # ---- App. A.2: up to 32 generated tokens per query, attending over cache + question + earlier tokens ---
    def enable_decode(self, max_new_tokens: int) -> None:
        sgc.sgc_plan_enable_decode(self.ctx, self.plan, max_new_tokens)

    def decode_step(self, step: int, dq: torch.Tensor, dk: torch.Tensor, dv: torch.Tensor, layer: int = 0,
                    do: Optional[torch.Tensor] = None, dlse: Optional[torch.Tensor] = None):
        if do is None:
            do = torch.zeros_like(dq)
        sgc.sgc_decode_step_batched(self.ctx, self.cache, self.plan, layer, step, dq.data_ptr(), dk.data_ptr(), dv.data_ptr(),
                                    do.data_ptr(), dlse.data_ptr() if dlse is not None else None, self.stream)
        return do

    def export_cluster(self, c: int, layer: int = 0):
        """Canonical [P][Hkv][d] view of the cluster's cache: (k, v, k_scale, v_scale) on the host.
        k, v are fp32 values for f32/bf16 caches and raw uint8 e4m3 codes for fp8 caches.  (A 16-bit cache
        holds the rotated keys as IEEE binary16 and the values as bf16.)"""
        w = self.w
        P = int(w.prefix_len[c])
        shp = (max(P, 1), w.n_kv_heads, w.head_dim)
        tdt = {"f32": torch.float32, "bf16": torch.bfloat16, "fp8_e4m3": torch.uint8}[w.kv_dtype]
        dk = torch.zeros(shp, dtype=torch.float16 if w.kv_dtype == "bf16" else tdt, device=self.device)
        dv = torch.zeros(shp, dtype=tdt, device=self.device)
        ks, vs = sgc.sgc_cache_export(self.ctx, self.cache, c, layer, dk.data_ptr(), dv.data_ptr(), w.n_kv_heads,
                                      self.stream)
        torch.cuda.synchronize()
        if w.kv_dtype == "fp8_e4m3":
            return dk[:P].cpu().numpy(), dv[:P].cpu().numpy(), ks, vs
        return to_host_f32(dk[:P]), to_host_f32(dv[:P]), ks, vs

    def import_cluster(self, c: int, layer: int, k: np.ndarray, v: np.ndarray, k_scale=None, v_scale=None) -> None:
        w = self.w
        if w.kv_dtype == "fp8_e4m3":
            dk = torch.from_numpy(np.ascontiguousarray(k, dtype=np.uint8)).to(self.device)
            dv = torch.from_numpy(np.ascontiguousarray(v, dtype=np.uint8)).to(self.device)
        else:
            dk, dv = to_device(k, w.kv_dtype, self.device), to_device(v, w.kv_dtype, self.device)
            if w.kv_dtype == "bf16":      # keys of a 16-bit cache are binary16
                dk = torch.from_numpy(np.ascontiguousarray(k, dtype=np.float32)).to(torch.float16).to(self.device)
        sgc.sgc_cache_import(self.ctx, self.cache, c, layer, dk.data_ptr(), dv.data_ptr(), k_scale, v_scale, self.stream)
        torch.cuda.synchronize()

    def close(self) -> None:
        torch.cuda.synchronize()
        if self.plan is not None:
            sgc.sgc_plan_destroy(self.plan)
            self.plan = None
        if self.cache is not None:
            sgc.sgc_cache_destroy(self.cache)
            self.cache = None
        if self.ctx is not None:
            sgc.sgc_ctx_destroy(self.ctx)
            self.ctx = None
        self.pool = None

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()
        return False


def run_workload(w: Workload, layer: int = 0, kernel: int = sgc.SGC_KERNEL_AUTO, want_lse: bool = True) -> Dict:
    """Whole path for one layer: fill every cluster's cache, assign, batched suffix prefill.
    Returns host arrays: o [T][Hq][d] fp32, lse [Hq][T], order, cluster_off, cu_seqlens."""
    threads = min(16, os.cpu_count() or 1)
    with Session(w, kernel=kernel) as s:
        # the prompts' keys and values are generated on several threads (a cluster's values do not depend on that)
        with ThreadPoolExecutor(max_workers=threads) as ex:
            kvs = list(ex.map(lambda c: w.prefix_kv(c, layer), range(w.n_clusters)))
        for c in range(w.n_clusters):
            s.alloc_cluster(c)
            s.prefix_prefill(c, layer, k=kvs[c][0], v=kvs[c][1])
        del kvs
        order, off, cu = s.assign()
        q, k, v = w.suffix_qkv(layer, threads=threads)
        dq, dk, dv = (to_device(x, w.io_dtype) for x in (q, k, v))
        T = q.shape[0]
        dlse = torch.zeros((w.n_q_heads, max(T, 1)), dtype=torch.float32, device="cuda:0") if want_lse else None
        do = s.suffix_prefill(dq, dk, dv, layer, dlse=dlse)
        torch.cuda.synchronize()
        out = {"o": to_host_f32(do), "lse": dlse[:, :T].cpu().numpy() if want_lse else None, "order": order,
               "cluster_off": off, "cu_seqlens": cu, "q": q, "k": k, "v": v}
        for c in range(w.n_clusters):
            s.free_cluster(c)
        assert sgc.sgc_cache_free_pages(s.cache) == sgc.sgc_cache_total_pages(s.cache)
    return out
