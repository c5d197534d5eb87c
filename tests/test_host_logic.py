"""CPU-only checks of libsgc: the library loads, exports every declared symbol, validates its
arguments on the host, keeps the page accounting of the cluster-wise cache (SubGCache Sec. 3.4:
allocate, reuse, release) and produces bit-exact cluster bookkeeping (Sec. 3.2 labels).
No kernel is launched here."""
import ctypes
import os
import re

import numpy as np
import pytest

from oracle import oracle as orc
from paper_2505_10951_amd import sgc, workloads

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE_POOL = 0x7F0000000000      # never dereferenced by host-only calls


@pytest.fixture(scope="module", autouse=True)
def _built():
    if not os.path.exists(sgc.LIB_PATH):
        from paper_2505_10951_amd.build import build_lib
        build_lib()


def _params(**kw):
    base = dict(n_q_heads=32, n_kv_heads=8, head_dim=128, n_layers=2, io_dtype="bf16", rope_base=500000.0)
    base.update(kw)
    return sgc.make_params(**base)


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "sgc.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(sgc_[a-z0-9_]+)\s*\(", header))
    assert declared == set(sgc.EXPORTS)
    L = sgc.lib()
    for name in declared:
        assert hasattr(L, name), name
    assert "gfx950" in sgc.version()


def test_params_struct_matches_header_layout():
    assert ctypes.sizeof(sgc.sgc_attn_params) == 48
    assert ctypes.sizeof(sgc.sgc_plan_info) == 32


@pytest.mark.parametrize("kw,status", [
    (dict(n_q_heads=30), sgc.SGC_EINVAL), (dict(n_kv_heads=0), sgc.SGC_EINVAL), (dict(head_dim=96), sgc.SGC_EUNSUPPORTED),
    (dict(n_layers=0), sgc.SGC_EINVAL), (dict(page_tokens=32), sgc.SGC_EUNSUPPORTED),
    (dict(io_dtype="fp8_e4m3", kv_dtype="fp8_e4m3"), sgc.SGC_EUNSUPPORTED),
    (dict(io_dtype="f32", kv_dtype="bf16"), sgc.SGC_EUNSUPPORTED), (dict(io_dtype="f32", kv_dtype="fp8_e4m3"), sgc.SGC_EUNSUPPORTED),
    (dict(rope_base=-1.0), sgc.SGC_EINVAL), (dict(softmax_scale=float("nan")), sgc.SGC_EINVAL),
    (dict(kernel=7), sgc.SGC_EINVAL), (dict(head_dim=64, kernel=sgc.SGC_KERNEL_MFMA), sgc.SGC_EUNSUPPORTED),
    (dict(io_dtype="f32", kernel=sgc.SGC_KERNEL_MFMA), sgc.SGC_EUNSUPPORTED),
])
def test_ctx_create_rejects_bad_params(kw, status):
    with pytest.raises(sgc.SgcError) as e:
        sgc.sgc_ctx_create(_params(**kw))
    assert e.value.status == status


def test_ctx_create_rejects_wrong_struct_size():
    p = _params()
    p.struct_size = 12
    with pytest.raises(sgc.SgcError) as e:
        sgc.sgc_ctx_create(p)
    assert e.value.status == sgc.SGC_EINVAL


def test_pool_sizes():
    p = _params()                                    # bf16, 8 KV heads, d 128, 2 layers
    assert sgc.sgc_cache_page_bytes(p) == 2 * 8 * 16 * 128 * 2
    assert sgc.sgc_cache_pool_bytes(p, 100) == 2 * 8 * 16 * 128 * 2 * 2 * 100
    p8 = _params(kv_dtype="fp8_e4m3", n_layers=1)
    assert sgc.sgc_cache_page_bytes(p8) == 2 * 8 * 16 * 128
    # the 32-layer resident cache of the stack workload: 16 clusters x 4096 tokens = 8 GiB
    p32 = _params(n_layers=32)
    assert sgc.sgc_cache_pool_bytes(p32, 16 * 256) == 8 * 1024 ** 3


def test_cache_lifecycle_page_accounting():
    p = _params(n_layers=2)
    ctx = sgc.sgc_ctx_create(p)
    pages = 40
    nbytes = sgc.sgc_cache_pool_bytes(p, pages)
    cache = sgc.sgc_cache_create(ctx, FAKE_POOL, nbytes + 100, 8)     # slack bytes do not make a page
    assert sgc.sgc_cache_total_pages(cache) == pages and sgc.sgc_cache_free_pages(cache) == pages
    plen = {0: 100, 1: 16, 2: 0, 3: 255}
    owned = {}
    for c, P in plen.items():
        sgc.sgc_cache_alloc_cluster(ctx, cache, c, P)
        pg, got_len = sgc.sgc_cache_cluster_pages(ctx, cache, c)
        assert got_len == P and len(pg) == orc.pages_needed(P)
        owned[c] = set(pg.tolist())
    allp = [x for s in owned.values() for x in s]
    assert len(allp) == len(set(allp)) and all(0 <= x < pages for x in allp)          # no aliasing
    assert sgc.sgc_cache_free_pages(cache) == pages - len(allp)
    # pool exhaustion leaves everything as it was
    with pytest.raises(sgc.SgcError) as e:
        sgc.sgc_cache_alloc_cluster(ctx, cache, 4, 16 * (pages - len(allp)) + 1)
    assert e.value.status == sgc.SGC_ENOMEM
    assert sgc.sgc_cache_free_pages(cache) == pages - len(allp)
    with pytest.raises(sgc.SgcError) as e:
        sgc.sgc_cache_alloc_cluster(ctx, cache, 0, 5)
    assert e.value.status == sgc.SGC_ESTATE
    with pytest.raises(sgc.SgcError) as e:
        sgc.sgc_cache_free_cluster(ctx, cache, 5)
    assert e.value.status == sgc.SGC_ESTATE
    with pytest.raises(sgc.SgcError) as e:
        sgc.sgc_cache_alloc_cluster(ctx, cache, 8, 5)
    assert e.value.status == sgc.SGC_EINVAL
    # release, then the freed pages are reusable and nothing leaks (Sec. 3.4: release per cluster)
    sgc.sgc_cache_free_cluster(ctx, cache, 3)
    sgc.sgc_cache_alloc_cluster(ctx, cache, 5, 16 * 20)
    pg5, _ = sgc.sgc_cache_cluster_pages(ctx, cache, 5)
    assert not (set(pg5.tolist()) & (owned[0] | owned[1]))
    for c in (0, 1, 2, 5):
        sgc.sgc_cache_free_cluster(ctx, cache, c)
    assert sgc.sgc_cache_free_pages(cache) == pages
    sgc.sgc_cache_destroy(cache)
    sgc.sgc_ctx_destroy(ctx)


def test_cache_create_rejects_bad_pool():
    p = _params()
    ctx = sgc.sgc_ctx_create(p)
    for pool, nbytes, mc in [(0, 1 << 20, 4), (FAKE_POOL + 8, 1 << 20, 4), (FAKE_POOL, 100, 4), (FAKE_POOL, 1 << 20, 0)]:
        with pytest.raises(sgc.SgcError) as e:
            sgc.sgc_cache_create(ctx, pool, nbytes, mc)
        assert e.value.status == sgc.SGC_EINVAL
    sgc.sgc_ctx_destroy(ctx)


def _ctx_cache(n_clusters, prefix_len, **kw):
    p = _params(**kw)
    ctx = sgc.sgc_ctx_create(p)
    pages = sum(orc.pages_needed(x) for x in prefix_len) + 1
    cache = sgc.sgc_cache_create(ctx, FAKE_POOL, sgc.sgc_cache_pool_bytes(p, pages), n_clusters)
    for c, P in enumerate(prefix_len):
        sgc.sgc_cache_alloc_cluster(ctx, cache, c, int(P))
    return ctx, cache


def test_assign_clusters_bit_exact_vs_oracle():
    rng = np.random.default_rng(11)
    for n, nc in [(0, 1), (1, 1), (7, 3), (320, 10), (1024, 16), (200, 50)]:
        plen = rng.integers(0, 300, size=nc)
        ctx, cache = _ctx_cache(nc, plen)
        labels = rng.integers(0, nc, size=n).astype(np.int32)
        slen = rng.integers(0, 70, size=n).astype(np.int32)
        order, off, cu, plan = sgc.sgc_assign_clusters(ctx, cache, labels, slen, nc)
        o_ref, off_ref, cu_ref = orc.assign_clusters(labels, slen, nc)
        assert order.dtype == np.int32 and np.array_equal(order, o_ref)
        assert np.array_equal(off, off_ref) and np.array_equal(cu, cu_ref)
        info = sgc.sgc_plan_get_info(ctx, plan)
        assert (info.n_queries, info.n_clusters, info.total_tokens) == (n, nc, int(slen.sum()))
        expect_maxpos = max([int(plen[labels[i]] + slen[i]) for i in range(n) if slen[i] > 0], default=0)
        assert info.max_position == expect_maxpos
        sgc.sgc_plan_destroy(plan)
        sgc.sgc_cache_destroy(cache)
        sgc.sgc_ctx_destroy(ctx)


def test_assign_clusters_on_the_benchmark_workloads():
    for idx in range(5):
        w = workloads.config(idx)
        ctx, cache = _ctx_cache(w.n_clusters, w.prefix_len, n_q_heads=w.n_q_heads, n_kv_heads=w.n_kv_heads,
                                head_dim=w.head_dim, io_dtype=w.io_dtype, kv_dtype=w.kv_dtype, n_layers=1)
        order, off, cu, _ = sgc.sgc_assign_clusters(ctx, cache, w.labels, w.suffix_len, w.n_clusters, want_plan=False)
        o_ref, off_ref, cu_ref = orc.assign_clusters(w.labels, w.suffix_len, w.n_clusters)
        assert np.array_equal(order, o_ref) and np.array_equal(off, off_ref) and np.array_equal(cu, cu_ref)
        assert sorted(order.tolist()) == list(range(w.n_queries))
        sgc.sgc_cache_destroy(cache)
        sgc.sgc_ctx_destroy(ctx)


def test_assign_clusters_error_paths_leave_outputs_alone():
    ctx, cache = _ctx_cache(3, [10, 20, 30])
    sgc.sgc_cache_free_cluster(ctx, cache, 1)
    cases = [([0, 3], [1, 1], 3, sgc.SGC_EINVAL), ([0, -1], [1, 1], 3, sgc.SGC_EINVAL), ([0, 2], [1, -2], 3, sgc.SGC_EINVAL),
             ([0, 1], [1, 1], 3, sgc.SGC_ESTATE), ([0, 0], [1, 1], 4, sgc.SGC_EINVAL)]
    for labels, slen, nc, status in cases:
        with pytest.raises(sgc.SgcError) as e:
            sgc.sgc_assign_clusters(ctx, cache, labels, slen, nc)
        assert e.value.status == status
        assert sgc.sgc_last_error(ctx)
    # a cluster nobody asks for need not be allocated
    order, off, cu, plan = sgc.sgc_assign_clusters(ctx, cache, [2, 0, 2], [4, 5, 6], 3)
    assert order.tolist() == [1, 0, 2] and off.tolist() == [0, 1, 1, 3] and cu.tolist() == [0, 4, 9, 15]
    sgc.sgc_plan_destroy(plan)
    sgc.sgc_cache_destroy(cache)
    sgc.sgc_ctx_destroy(ctx)


def test_launch_entry_points_validate_before_touching_the_device():
    ctx, cache = _ctx_cache(2, [32, 48])
    _, _, _, plan = sgc.sgc_assign_clusters(ctx, cache, [0, 1], [4, 4], 2)
    bad = [
        lambda: sgc.sgc_prefix_prefill(ctx, cache, 5, 0, None, 256, 512, None, None, 32),          # cluster range
        lambda: sgc.sgc_prefix_prefill(ctx, cache, 0, 9, None, 256, 512, None, None, 32),          # layer range
        lambda: sgc.sgc_prefix_prefill(ctx, cache, 0, 0, None, 256, 512, None, None, 31),          # length mismatch
        lambda: sgc.sgc_prefix_prefill(ctx, cache, 0, 0, 256, 256, 512, None, None, 32),           # q without o
        lambda: sgc.sgc_prefix_prefill(ctx, cache, 0, 0, None, None, 512, None, None, 32),         # NULL k
        lambda: sgc.sgc_prefix_prefill(ctx, cache, 0, 0, None, 260, 512, None, None, 32),          # misaligned
        lambda: sgc.sgc_suffix_prefill_batched(ctx, cache, plan, 3, 256, 256, 256, 256),           # layer range
        lambda: sgc.sgc_suffix_prefill_batched(ctx, cache, plan, 0, None, 256, 256, 256),          # NULL q
        lambda: sgc.sgc_suffix_prefill_batched(ctx, cache, plan, 0, 256, 256, 264, 256),           # misaligned
        lambda: sgc.sgc_cache_export(ctx, cache, 7, 0, 256, 256, 8),
        lambda: sgc.sgc_prefix_prefill_batched(ctx, cache, [0, 0], 0, None, [256, 256], [512, 512], None),   # twice
        lambda: sgc.sgc_prefix_prefill_batched(ctx, cache, [0, 3], 0, None, [256, 256], [512, 512], None),   # range
        lambda: sgc.sgc_prefix_prefill_batched(ctx, cache, [0, 1], 0, None, [256, None], [512, 512], None),  # NULL k
        lambda: sgc.sgc_prefix_prefill_batched(ctx, cache, [0, 1], 0, [256, 256], [256, 256], [512, 512], None),  # q, no o
        lambda: sgc.sgc_prefix_prefill_batched(ctx, cache, [0, 1], 0, [256, None], [256, 256], [512, 512], [256, 256]),
        lambda: sgc.sgc_prefix_prefill_batched(ctx, cache, [0, 1], 0, None, [256, 264], [512, 512], None),   # misaligned
        lambda: sgc.sgc_timing_last(ctx),                                                                  # nothing timed
    ]
    expect = [sgc.SGC_EINVAL, sgc.SGC_EINVAL, sgc.SGC_ESHAPE, sgc.SGC_EINVAL, sgc.SGC_EINVAL, sgc.SGC_EINVAL,
              sgc.SGC_EINVAL, sgc.SGC_EINVAL, sgc.SGC_EINVAL, sgc.SGC_EINVAL,
              sgc.SGC_EINVAL, sgc.SGC_EINVAL, sgc.SGC_EINVAL, sgc.SGC_EINVAL, sgc.SGC_EINVAL, sgc.SGC_EINVAL,
              sgc.SGC_ESTATE]
    for fn, status in zip(bad, expect):
        with pytest.raises(sgc.SgcError) as e:
            fn()
        assert e.value.status == status
    # a plan goes stale when its cluster is released
    sgc.sgc_cache_free_cluster(ctx, cache, 1)
    with pytest.raises(sgc.SgcError) as e:
        sgc.sgc_suffix_prefill_batched(ctx, cache, plan, 0, 256, 256, 256, 256)
    assert e.value.status == sgc.SGC_ESTATE
    sgc.sgc_plan_destroy(plan)
    sgc.sgc_cache_destroy(cache)
    sgc.sgc_ctx_destroy(ctx)


def test_projection_entry_points_validate_before_touching_the_device():
    ctx, cache = _ctx_cache(2, [32, 48])
    _, _, _, plan = sgc.sgc_assign_clusters(ctx, cache, [0, 1], [4, 4], 2)
    E, S, T = sgc.SGC_EINVAL, sgc.SGC_ESHAPE, sgc.SGC_ESTATE
    bad = [
        (lambda: sgc.sgc_project_out(ctx, 256, 512, 4096, -1, 768), E),                         # negative rows
        (lambda: sgc.sgc_project_out(ctx, 256, 512, 0, 8, 768), E),                             # d_model
        (lambda: sgc.sgc_project_out(ctx, None, 512, 4096, 8, 768), E),                         # NULL o
        (lambda: sgc.sgc_project_out(ctx, 256, 520, 4096, 8, 768), E),                          # misaligned weight
        (lambda: sgc.sgc_project_out(ctx, 256, 512, 4100, 8, 768), E),                          # rows of y not 16-byte aligned
        (lambda: sgc.sgc_project_qkv_prefix(ctx, cache, 5, 0, 256, 512, 4096, None, 32), E),    # cluster range
        (lambda: sgc.sgc_project_qkv_prefix(ctx, cache, 0, 2, 256, 512, 4096, None, 32), E),    # layer range
        (lambda: sgc.sgc_project_qkv_prefix(ctx, cache, 0, 0, 256, 512, 4096, None, 31), S),    # length mismatch
        (lambda: sgc.sgc_project_qkv_prefix(ctx, cache, 0, 0, None, 512, 4096, None, 32), E),   # NULL x
        (lambda: sgc.sgc_project_qkv_prefix(ctx, cache, 0, 0, 256, None, 4096, None, 32), E),   # NULL weight
        (lambda: sgc.sgc_project_qkv_prefix(ctx, cache, 0, 0, 256, 512, 100, None, 32), E),     # rows of x not aligned
        (lambda: sgc.sgc_project_qkv_prefix_batched(ctx, cache, [1, 1], 0, [256, 256], 512, 4096), E),   # twice
        (lambda: sgc.sgc_project_qkv_prefix_batched(ctx, cache, [0, 1], 0, [256, None], 512, 4096), E),  # NULL x
        (lambda: sgc.sgc_project_qkv_prefix_batched(ctx, cache, [0, 1], 0, [256, 256], 512, 4096, [256, 260]), E),
        (lambda: sgc.sgc_project_qkv_suffix(ctx, cache, plan, 7, 256, 512, 4096, 768), E),      # layer range
        (lambda: sgc.sgc_project_qkv_suffix(ctx, cache, plan, 0, 256, 512, 4096, None), E),     # NULL q
        (lambda: sgc.sgc_project_qkv_suffix(ctx, cache, plan, 0, 256, 512, -4, 768), E),        # d_model
        (lambda: sgc.sgc_suffix_prefill_batched(ctx, cache, plan, 0, 256, None, None, 256), T),  # nothing projected yet
        (lambda: sgc.sgc_suffix_prefill_batched(ctx, cache, plan, 0, 256, None, 256, 256), E),   # only one of k, v
        (lambda: sgc.sgc_prefix_prefill(ctx, cache, 0, 0, None, None, None, None, None, 32), E),  # nothing to do
        (lambda: sgc.sgc_timing_get(ctx, 128), E),                                              # beyond the ring
        (lambda: sgc.sgc_timing_enable(ctx, -1), E),                                            # a negative period
    ]
    for i, (fn, status) in enumerate(bad):
        with pytest.raises(sgc.SgcError) as e:
            fn()
        assert e.value.status == status, (i, str(e.value))
    assert sgc.sgc_project_out(ctx, None, None, 4096, 0, None) is None            # zero rows: nothing to check or do
    sgc.sgc_cache_free_cluster(ctx, cache, 1)
    with pytest.raises(sgc.SgcError) as e:
        sgc.sgc_project_qkv_suffix(ctx, cache, plan, 0, 256, 512, 4096, 768)
    assert e.value.status == sgc.SGC_ESTATE
    sgc.sgc_plan_destroy(plan)
    sgc.sgc_cache_destroy(cache)
    sgc.sgc_ctx_destroy(ctx)


def test_workload_generators_are_deterministic_and_shaped():
    w = workloads.config(1)
    assert (w.n_clusters, w.n_queries) == (10, 320) and np.all(w.prefix_len == 1024)
    assert w.suffix_len.min() >= 16 and w.suffix_len.max() <= 64
    assert np.array_equal(np.bincount(w.labels, minlength=10), np.full(10, 32))
    q1, k1, v1 = w.suffix_qkv_query(5)
    q2, k2, v2 = workloads.config(1).suffix_qkv_query(5)
    assert np.array_equal(q1, q2) and np.array_equal(k1, k2) and np.array_equal(v1, v2)
    assert np.array_equal(workloads.round_to_bf16(k1), k1)            # already bf16-representable
    # one outlier channel per KV head, eight times the spread of the rest
    pk, _ = w.prefix_kv(0)
    std = pk.std(axis=0)
    assert np.all((std > 4).sum(axis=1) == 1) and abs(np.median(std) - 1) < 0.1
    w3 = workloads.config(2)
    sizes = np.bincount(w3.labels, minlength=16)
    assert sizes.sum() == 1024 and sorted(sizes.tolist(), reverse=True) == workloads.zipf_cluster_sizes(16, 1024).tolist()
    assert sizes.max() > 300 and sizes.min() >= 1
    assert w3.prefix_len.min() >= 1024 and w3.prefix_len.max() <= 4096
    assert abs(workloads.config(1).flops() / 2.2e11 - 1) < 0.1


def test_batch_size_knob_changes_the_batch_and_nothing_else():
    base = workloads.config(1)
    same = workloads.config(1, queries_per_cluster=32)
    assert np.array_equal(same.labels, base.labels) and np.array_equal(same.suffix_len, base.suffix_len)
    assert np.array_equal(same.prefix_len, base.prefix_len) and same.name != base.name      # no profiled constant applies
    wide = workloads.config(1, queries_per_cluster=40)
    assert wide.n_queries == 400 and np.array_equal(np.bincount(wide.labels), np.full(10, 40))
    assert (wide.n_q_heads, wide.n_kv_heads, wide.head_dim, wide.k_outlier_scale) == (32, 8, 128, 8.0)
    assert 16 <= wide.suffix_len.min() and wide.suffix_len.max() <= 64
    with pytest.raises(ValueError):
        workloads.config(2, queries_per_cluster=8)


def test_bf16_rounding_helper_is_round_to_nearest_even():
    x = np.array([1.0, 1.0 + 2 ** -8, 1.0 + 2 ** -7, 1.0 + 3 * 2 ** -8, -1.0 - 2 ** -8, 3.14159], dtype=np.float32)
    r = workloads.round_to_bf16(x)
    assert r.tolist()[:5] == [1.0, 1.0, 1.0 + 2 ** -7, 1.0 + 2 ** -6, -1.0]
    import torch
    assert np.array_equal(r, torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy())
    assert np.array_equal(workloads.bf16_bits_to_f32(workloads.bf16_bits(r)), r)
