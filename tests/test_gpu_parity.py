"""GPU parity: the HIP path, called through the C ABI, against the CPU fp64 oracle on the same
seeded inputs, element by element.  Tolerances: 2e-2 max-abs for bf16 in / fp32 accumulate,
6e-2 with an fp8 cache (the stated bars), 2e-5 for the fp32 path, plus a calibrated tighter bar
(a few times the error any bf16 kernel carries) so that a wrong mask or index cannot hide."""
import numpy as np
import pytest
import torch

from oracle import oracle as orc
from paper_2505_10951_amd import sgc, workloads
from paper_2505_10951_amd.harness import Session, run_workload, to_device, to_host_f32

from ref_util import (bf16_floor_arrays, bf16_rounding_floor, err_stats, fp8_query_floor, oracle_caches, oracle_suffix,
                      tight_bar)

pytestmark = pytest.mark.gpu

TOL_BF16, TOL_FP8, TOL_F32 = 2e-2, 6e-2, 2e-5


def _say(*a):
    print(*a, flush=True)


def _check_suffix(w, out, queries=None, tol=TOL_BF16, tight=None, lse_tol=None):
    rows, o_ref, lse_ref = oracle_suffix(w, 0, queries)
    st = err_stats(out["o"][rows], o_ref)
    _say(f"  {w.name}: rows {len(rows)} max_abs {st['max_abs']:.3e} rel {st['rel']:.3e} (tol {tol:g}, tight {tight})")
    assert np.isfinite(out["o"]).all()
    assert st["max_abs"] <= tol
    if tight is not None:
        assert st["max_abs"] <= tight
    if out.get("lse") is not None:
        # To first order an LSE error is the weighted mean of the row's score errors, so it is bounded by the largest
        # of them.  A score is scale * <q, k> on operands rounded to binary16 (relative 2^-11 each):
        # |ds| <= 2^-10 * scale * |q| |k|, which for unit-variance 128-channel rows (|q| |k| ~ 128, scale 0.088) is
        # 1.1e-2, plus the fp32 accumulation and exp2/log2 of the kernel (1e-3).  2e-2 unless the caller calibrated a
        # bound on its own data (workloads with scaled-up channels or queries do)
        lerr = np.abs(out["lse"][:, rows] - lse_ref).max() if len(rows) else 0.0
        _say(f"  lse max_abs {lerr:.3e}")
        assert lerr <= (lse_tol if lse_tol is not None else 2e-2)
    return st


def _check_bookkeeping(w, out):
    o_ref, off_ref, cu_ref = orc.assign_clusters(w.labels, w.suffix_len, w.n_clusters)
    assert np.array_equal(out["order"], o_ref) and np.array_equal(out["cluster_off"], off_ref)
    assert np.array_equal(out["cu_seqlens"], cu_ref)


# ---- configs[0]: tiny fp32 MHA layer, in full --------------------------------------------------
def test_config0_tiny_f32_full():
    w = workloads.config(0)
    _say("config 0", w.name, "T", w.total_suffix_tokens)
    out = run_workload(w)
    _check_bookkeeping(w, out)
    _check_suffix(w, out, tol=TOL_F32, lse_tol=2e-5)


@pytest.mark.parametrize("io,kv,d", [("f32", "f32", 128), ("bf16", "bf16", 64), ("bf16", "fp8_e4m3", 64)])
def test_generic_kernel_other_shapes(io, kv, d):
    w = workloads.custom(f"generic_{io}_{kv}_{d}", n_q_heads=4, n_kv_heads=2, head_dim=d, rope_base=10000.0, io_dtype=io,
                         kv_dtype=kv, prefix_len=[70, 33, 0], queries_per_cluster=3, suffix_range=(1, 20), seed=77)
    out = run_workload(w, kernel=sgc.SGC_KERNEL_GENERIC)
    _check_suffix(w, out, tol={"f32": TOL_F32, "bf16": TOL_BF16, "fp8_e4m3": TOL_FP8}[kv])


# ---- bf16 MFMA kernel: scaled-down cases spanning several tiles and ragged tails ----------------
def _small_gqa(seed=5, **kw):
    base = dict(n_q_heads=8, n_kv_heads=2, head_dim=128, rope_base=500000.0, io_dtype="bf16",
                prefix_len=[200, 71, 128], cluster_sizes=[5, 3, 4], suffix_range=(1, 70), seed=seed, k_outlier_scale=8.0)
    base.update(kw)
    return workloads.custom("small_gqa", **base)


def test_mfma_small_gqa_full():
    w = _small_gqa()
    _say("small gqa T", w.total_suffix_tokens, "suffix", w.suffix_len.tolist())
    out = run_workload(w, kernel=sgc.SGC_KERNEL_MFMA)
    _check_bookkeeping(w, out)
    tight, lse_bar = tight_bar(w, range(w.n_queries))
    _check_suffix(w, out, tol=TOL_BF16, tight=tight, lse_tol=lse_bar)


def test_mfma_small_mha_ragged():
    w = workloads.custom("small_mha", n_q_heads=4, n_kv_heads=4, head_dim=128, rope_base=10000.0, io_dtype="bf16",
                         prefix_len=[300, 17, 64, 1], cluster_sizes=[9, 1, 2, 4], suffix_range=(24, 96), seed=9)
    out = run_workload(w, kernel=sgc.SGC_KERNEL_MFMA)
    tight, lse_bar = tight_bar(w, range(w.n_queries))
    _check_suffix(w, out, tol=TOL_BF16, tight=tight, lse_tol=lse_bar)


@pytest.mark.parametrize("seed", [31, 33])
def test_mfma_small_gqa_three_prompt_lengths_both_cache_types(seed):
    """Prompts of 200, 71 and 300 tokens (four, two and five 64-key steps, the last ones ragged) without outlier channels,
    bf16 and fp8 cache, prompt and batch to the stated bars."""
    for kv in ("bf16", "fp8_e4m3"):
        w = _small_gqa(seed=seed, kv_dtype=kv, prefix_len=[200, 71, 300], k_outlier_scale=1.0)
        out = run_workload(w, kernel=sgc.SGC_KERNEL_MFMA)
        _check_bookkeeping(w, out)
        _check_suffix(w, out, tol=TOL_BF16 if kv == "bf16" else TOL_FP8)


def test_mfma_matches_generic_kernel():
    w = _small_gqa(seed=21)
    a = run_workload(w, kernel=sgc.SGC_KERNEL_MFMA)
    b = run_workload(w, kernel=sgc.SGC_KERNEL_GENERIC)
    d = np.abs(a["o"] - b["o"]).max()
    tight, lse_bar = tight_bar(w, range(w.n_queries))
    _say(f"  mfma vs generic max_abs {d:.3e} (bar {tight:.3e})")
    assert d <= tight
    assert np.abs(a["lse"] - b["lse"]).max() <= lse_bar


def test_mfma_edge_cases():
    # empty cluster, zero-length queries, P = 0, P one short of / one past a page and a 64-key tile,
    # single-token queries, a query longer than one key tile
    plen = [0, 15, 16, 17, 63, 64, 65, 1]
    labels = np.array([0, 0, 1, 2, 3, 4, 5, 6, 7, 7, 5, 3, 0], dtype=np.int32)
    slen = np.array([1, 70, 3, 0, 16, 17, 64, 65, 1, 130, 2, 1, 0], dtype=np.int32)
    w = workloads.custom("edges", n_q_heads=4, n_kv_heads=2, head_dim=128, rope_base=10000.0, io_dtype="bf16",
                         prefix_len=plen, labels=labels, suffix_len=slen, seed=13)
    tight, lse_bar = tight_bar(w, range(w.n_queries))
    for kernel in (sgc.SGC_KERNEL_MFMA, sgc.SGC_KERNEL_GENERIC):
        out = run_workload(w, kernel=kernel)
        _check_bookkeeping(w, out)
        _check_suffix(w, out, tol=TOL_BF16, tight=tight, lse_tol=lse_bar)


def test_mfma_row_tile_touching_dozens_of_queries():
    """Sixty queries of one to three tokens in one cluster, one KV head per query head: a 128-row tile then holds
    the rows of about sixty queries, far more than a tile record describes inline, so the kernel takes the
    per-token records and the per-tile query table; a second cluster of ordinary queries shares the batch."""
    rng = np.random.default_rng(5)
    slen = np.concatenate([rng.integers(1, 4, size=60), np.array([40, 17, 0, 64])]).astype(np.int32)
    labels = np.concatenate([np.zeros(60, dtype=np.int32), np.ones(4, dtype=np.int32)])
    perm = rng.permutation(labels.size)
    w = workloads.custom("many_tiny", n_q_heads=2, n_kv_heads=2, head_dim=128, rope_base=10000.0, io_dtype="bf16",
                         prefix_len=[150, 90], labels=labels[perm], suffix_len=slen[perm], seed=41)
    tight, lse_bar = tight_bar(w, range(w.n_queries))
    out = run_workload(w, kernel=sgc.SGC_KERNEL_MFMA)
    _check_bookkeeping(w, out)
    _check_suffix(w, out, tol=TOL_BF16, tight=tight, lse_tol=lse_bar)


def test_mfma_all_queries_empty_and_single_row():
    w = workloads.custom("empty", n_q_heads=4, n_kv_heads=4, head_dim=128, rope_base=10000.0, io_dtype="bf16",
                         prefix_len=[40], labels=[0, 0], suffix_len=[0, 0], seed=1)
    out = run_workload(w, kernel=sgc.SGC_KERNEL_MFMA)
    assert out["o"].shape[0] == 0
    w = workloads.custom("one", n_q_heads=1, n_kv_heads=1, head_dim=128, rope_base=10000.0, io_dtype="bf16",
                         prefix_len=[40], labels=[0], suffix_len=[1], seed=2)
    out = run_workload(w, kernel=sgc.SGC_KERNEL_MFMA)
    _check_suffix(w, out, tol=TOL_BF16, tight=tight_bar(w, [0])[0])


def test_mfma_peaky_softmax_one_hot_v_exposes_the_mask():
    # Q scaled so that softmax concentrates on a few keys; V rows are one-hot in (key index mod d):
    # channel c of the output is the total probability of keys j = c (mod d).  A key that must not
    # be seen (later suffix tokens, other queries) shows up as mass in the wrong channel.
    P, S = 100, 28
    w = workloads.custom("peaky", n_q_heads=2, n_kv_heads=1, head_dim=128, rope_base=10000.0, io_dtype="bf16",
                         prefix_len=[P], labels=[0, 0], suffix_len=[S, S], seed=31, q_gain=6.0)
    eye = np.eye(128, dtype=np.float32)

    with Session(w, kernel=sgc.SGC_KERNEL_MFMA) as s:
        s.alloc_cluster(0)
        pk, _ = w.prefix_kv(0)
        pv = eye[np.arange(P) % 128][:, None, :]
        s.prefix_prefill(0, 0, k=pk, v=pv)
        s.assign()
        q, k, _ = w.suffix_qkv()
        v = np.concatenate([eye[(P + np.arange(S)) % 128], eye[(P + np.arange(S)) % 128]])[:, None, :]
        do = s.suffix_prefill(to_device(q, "bf16"), to_device(k, "bf16"), to_device(v, "bf16"))
        torch.cuda.synchronize()
        o = to_host_f32(do)
    ck, cv, _, _ = orc.prefix_prefill(None, pk, pv, w.rope_base)
    o_ref, _ = orc.suffix_prefill_batched(w.labels, w.cu_seqlens, [ck], [cv], q, k, v, w.rope_base)
    assert np.abs(o - o_ref).max() <= 1e-2
    for n in range(2):
        for i in range(S):
            row = o[n * S + i]                       # [Hq][d]
            unseen = np.arange(P + i + 1, 128)       # keys i+1.. of the own suffix and nothing beyond
            assert np.all(row[:, unseen] == 0), (n, i)
            assert np.all(np.abs(row.sum(axis=-1) - 1) < 2e-2)


def test_batch_composition_does_not_change_a_query():
    w = _small_gqa(seed=41)
    full = run_workload(w, kernel=sgc.SGC_KERNEL_MFMA)
    cu = w.cu_seqlens
    keep = [1, 4, 6, 10][::-1]
    sub = workloads.custom("subset", n_q_heads=8, n_kv_heads=2, head_dim=128, rope_base=500000.0, io_dtype="bf16",
                           prefix_len=w.prefix_len, labels=w.labels[keep], suffix_len=w.suffix_len[keep], seed=41,
                           k_outlier_scale=8.0)
    with Session(sub, kernel=sgc.SGC_KERNEL_MFMA) as s:
        for c in range(sub.n_clusters):
            s.alloc_cluster(c)
            s.prefix_prefill(c)
        s.assign()
        qs, ks, vs = zip(*[w.suffix_qkv_query(n) for n in keep])
        do = s.suffix_prefill(*(to_device(np.concatenate(x), "bf16") for x in (qs, ks, vs)))
        torch.cuda.synchronize()
        o = to_host_f32(do)
    at = 0
    for n in keep:
        S = int(w.suffix_len[n])
        ref = full["o"][cu[n]:cu[n + 1]]
        assert np.abs(o[at:at + S] - ref).max() <= 4e-3, n     # same math, other tile packing
        at += S


def test_repeat_launch_is_bit_identical():
    w = _small_gqa(seed=43)
    a = run_workload(w, kernel=sgc.SGC_KERNEL_MFMA)
    b = run_workload(w, kernel=sgc.SGC_KERNEL_MFMA)
    assert np.array_equal(a["o"], b["o"]) and np.array_equal(a["lse"], b["lse"])


# ---- prefix prefill: cache contents and the prefix's own causal attention -----------------------
@pytest.mark.parametrize("kernel", [sgc.SGC_KERNEL_MFMA, sgc.SGC_KERNEL_GENERIC])
def test_prefix_prefill_cache_and_causal_output(kernel):
    w = workloads.custom("prefix", n_q_heads=8, n_kv_heads=2, head_dim=128, rope_base=500000.0, io_dtype="bf16",
                         prefix_len=[333, 64, 5], queries_per_cluster=1, suffix_range=(1, 1), seed=17)
    with Session(w, kernel=kernel) as s:
        for c in range(w.n_clusters):
            s.alloc_cluster(c)
            do, dlse = s.prefix_prefill(c, 0, with_q=True, want_lse=True)
            pk, pv = w.prefix_kv(c)
            ck, cv, o_ref, lse_ref = orc.prefix_prefill(w.prefix_q(c), pk, pv, w.rope_base, want_lse=True)
            ek, ev, _, _ = s.export_cluster(c)
            assert np.array_equal(ev, pv)                                     # V is stored as given
            assert np.all(np.abs(ek - ck) <= np.abs(ck) * 2.0 ** -11 + 1e-5)  # K: one binary16 rounding (+ fp32 rotation)
            st = err_stats(to_host_f32(do), o_ref)
            # the prefix's own attention is a suffix prefill over an empty cache
            e = np.zeros((0, w.n_kv_heads, w.head_dim))
            fl_o, fl_lse = bf16_floor_arrays(e, e, w.prefix_q(c), pk, pv, w.rope_base, want_lse=True)
            _say(f"  prefix cluster {c} P {w.prefix_len[c]} max_abs {st['max_abs']:.3e} (floor {fl_o:.3e})")
            assert st["max_abs"] <= TOL_BF16 and st["max_abs"] <= 4 * fl_o
            assert np.abs(dlse.cpu().numpy() - lse_ref).max() <= max(4 * fl_lse, 2e-3)


@pytest.mark.parametrize("kv", ["bf16", "fp8_e4m3"])
@pytest.mark.parametrize("kernel", [sgc.SGC_KERNEL_MFMA, sgc.SGC_KERNEL_GENERIC])
def test_prefix_prefill_batched_equals_one_by_one(kernel, kv):
    """One call for several clusters (given out of order, one of them empty) against a call per cluster:
    same kernels, same arithmetic, so caches, outputs and LSE are bit-identical; and against the oracle."""
    w = workloads.custom("prefix_batched", n_q_heads=8, n_kv_heads=2, head_dim=128, rope_base=500000.0, io_dtype="bf16",
                         kv_dtype=kv, prefix_len=[333, 64, 0, 5, 130], queries_per_cluster=1, suffix_range=(1, 1), seed=19)
    order = [3, 0, 4, 2, 1]
    with Session(w, kernel=kernel) as s1, Session(w, kernel=kernel) as s2:
        for c in range(w.n_clusters):
            s1.alloc_cluster(c)
            s2.alloc_cluster(c)
        single = {c: s1.prefix_prefill(c, 0, with_q=True, want_lse=True) for c in range(w.n_clusters) if w.prefix_len[c] > 0}
        batched = dict(zip(order, s2.prefix_prefill_batched(order, 0, with_q=True, want_lse=True)))
        for c in range(w.n_clusters):
            P = int(w.prefix_len[c])
            if P == 0:
                continue
            e1, e2 = s1.export_cluster(c), s2.export_cluster(c)
            for x, y in zip(e1, e2):
                assert np.array_equal(x, y)
            assert torch.equal(single[c][0], batched[c][0]) and torch.equal(single[c][1], batched[c][1])
            if kv == "bf16":
                pk, pv = w.prefix_kv(c)
                _, _, o_ref, lse_ref = orc.prefix_prefill(w.prefix_q(c), pk, pv, w.rope_base, want_lse=True)
                assert err_stats(to_host_f32(batched[c][0]), o_ref)["max_abs"] <= TOL_BF16
                assert np.abs(batched[c][1].cpu().numpy() - lse_ref).max() <= 2e-2


def test_prefix_prefill_f32_cache_exact_layout_roundtrip():
    w = workloads.config(0)
    with Session(w) as s:
        s.alloc_cluster(0)
        s.prefix_prefill(0)
        pk, pv = w.prefix_kv(0)
        ck, cv, _, _ = orc.prefix_prefill(None, pk, pv, w.rope_base)
        ek, ev, _, _ = s.export_cluster(0)
        assert np.array_equal(ev, pv) and np.abs(ek - ck).max() <= 2e-6
        # import(export) is the identity on the pages; shuffled physical pages do not matter
        s.alloc_cluster(1)
        s.import_cluster(1, 0, ek[:192], ev[:192])
        ek1, ev1, _, _ = s.export_cluster(1)
        assert np.array_equal(ek1, ek[:192]) and np.array_equal(ev1, ev[:192])


def test_physical_page_order_does_not_matter():
    w = _small_gqa(seed=47)
    ref = run_workload(w, kernel=sgc.SGC_KERNEL_MFMA)
    with Session(w, kernel=sgc.SGC_KERNEL_MFMA, total_pages=200, max_clusters=8) as s:
        # fragment the pool: interleave dummy allocations and free them again
        sgc.sgc_cache_alloc_cluster(s.ctx, s.cache, 5, 40)
        s.alloc_cluster(1)
        sgc.sgc_cache_alloc_cluster(s.ctx, s.cache, 6, 100)
        s.alloc_cluster(0)
        sgc.sgc_cache_free_cluster(s.ctx, s.cache, 5)
        s.alloc_cluster(2)
        sgc.sgc_cache_free_cluster(s.ctx, s.cache, 6)
        pages = [sgc.sgc_cache_cluster_pages(s.ctx, s.cache, c)[0] for c in range(3)]
        assert any(np.any(np.diff(p) != 1) for p in pages) or pages[0][0] != 0
        for c in range(3):
            s.prefix_prefill(c)
        s.assign()
        q, k, v = w.suffix_qkv()
        do = s.suffix_prefill(*(to_device(x, "bf16") for x in (q, k, v)))
        torch.cuda.synchronize()
        assert np.array_equal(to_host_f32(do), ref["o"])


def test_plan_outlives_a_reallocation_of_its_clusters():
    """A plan is launched, its clusters are released and allocated again on other pages (same prompts), and the same plan
    is launched once more: the tile records it keeps on the device have to follow the new page tables."""
    w = _small_gqa(seed=53)
    ref = run_workload(w, kernel=sgc.SGC_KERNEL_MFMA)
    with Session(w, kernel=sgc.SGC_KERNEL_MFMA, total_pages=300, max_clusters=8) as s:
        for c in range(3):
            s.alloc_cluster(c)
            s.prefix_prefill(c)
        s.assign()
        q, k, v = w.suffix_qkv()
        dq, dk, dv = (to_device(x, "bf16") for x in (q, k, v))
        do = s.suffix_prefill(dq, dk, dv)
        torch.cuda.synchronize()
        assert np.array_equal(to_host_f32(do), ref["o"])
        before = [sgc.sgc_cache_cluster_pages(s.ctx, s.cache, c)[0].copy() for c in range(3)]
        for c in range(3):
            s.free_cluster(c)
        sgc.sgc_cache_alloc_cluster(s.ctx, s.cache, 7, 50)          # takes the pages the first cluster had
        for c in (2, 0, 1):
            s.alloc_cluster(c)
        after = [sgc.sgc_cache_cluster_pages(s.ctx, s.cache, c)[0] for c in range(3)]
        assert all(not np.array_equal(a, b) for a, b in zip(before, after))
        for c in range(3):
            s.prefix_prefill(c)
        do.zero_()
        do = s.suffix_prefill(dq, dk, dv, do=do)
        torch.cuda.synchronize()
        assert np.array_equal(to_host_f32(do), ref["o"])


# ---- fp8 e4m3 cache --------------------------------------------------------------------------
def test_fp8_codec_and_quantised_cache_match_oracle():
    # all 256 codes decode as the oracle says; encoding agrees on every code point and midpoint
    d, Hkv = 128, 1
    vals = [orc.e4m3_decode(c) for c in range(0x7F)]
    mids = [(vals[i] + vals[i + 1]) / 2 for i in range(0x7E)]
    x = np.array(vals + mids + [448.0] * 3, dtype=np.float64)
    x = np.concatenate([x, -x])
    P = -(-x.size // d)
    flat = np.zeros(P * d)
    flat[: x.size] = x
    k = flat.reshape(P, Hkv, d).astype(np.float32)
    assert np.array_equal(workloads.round_to_bf16(k), k)       # representable: the GPU sees these exact values
    w = workloads.custom("codec", n_q_heads=1, n_kv_heads=1, head_dim=d, rope_base=0.0, io_dtype="bf16",
                         kv_dtype="fp8_e4m3", prefix_len=[P], labels=[0], suffix_len=[1], seed=3)
    with Session(w) as s:
        s.alloc_cluster(0)
        s.prefix_prefill(0, 0, k=k, v=k[::-1].copy())
        ek, ev, ks, vs = s.export_cluster(0)
    codes, scale, _ = orc.quantise_e4m3(k.astype(np.float64))
    assert ks[0] == scale[0] == 1.0 and vs[0] == 1.0         # amax = 448
    assert np.array_equal(ek, codes)
    assert np.array_equal(ev, codes[::-1])


@pytest.mark.parametrize("kernel", [sgc.SGC_KERNEL_MFMA, sgc.SGC_KERNEL_GENERIC, sgc.SGC_KERNEL_MFMA_FP8])
def test_fp8_cache_small(kernel):
    w = workloads.custom("fp8_small", n_q_heads=8, n_kv_heads=2, head_dim=128, rope_base=500000.0, io_dtype="bf16",
                         kv_dtype="fp8_e4m3", prefix_len=[260, 64, 31], cluster_sizes=[4, 2, 3], suffix_range=(1, 80),
                         seed=23)
    with Session(w, kernel=kernel) as s:
        for c in range(w.n_clusters):
            s.alloc_cluster(c)
            s.prefix_prefill(c)
        # the device's quantised cache against the oracle's: scales equal to an ulp, codes equal
        # except where fp32 rotation lands on the other side of a rounding boundary
        for c in range(w.n_clusters):
            pk, pv = w.prefix_kv(c)
            ck, cv, _, _ = orc.prefix_prefill(None, pk, pv, w.rope_base)
            kc, ksc, _ = orc.quantise_e4m3(ck)
            vc, vsc, _ = orc.quantise_e4m3(cv)
            ek, ev, ks, vs = s.export_cluster(c)
            assert np.allclose(ks, ksc, rtol=3e-7) and np.array_equal(vs, vsc)
            assert np.array_equal(ev, vc)           # V: same inputs, same fp32 quotient, same codes
            diff = ek != kc
            _say(f"  cluster {c}: K codes differing {diff.mean():.2e}")
            assert diff.mean() < 5e-3
            assert np.all(np.abs(ek.astype(np.int16)[diff] - kc.astype(np.int16)[diff]) == 1)
        s.assign()
        q, k, v = w.suffix_qkv()
        do = s.suffix_prefill(*(to_device(x, "bf16") for x in (q, k, v)))
        torch.cuda.synchronize()
        out = {"o": to_host_f32(do), "lse": None}
    # Against the oracle's own quantised cache the stated 6e-2 is the bar: where the GPU's fp32 rotation puts a key
    # element on the other side of a code boundary (counted above) a row that gives that key most of its weight moves by
    # up to p (1 - p) * scale * |q_c| * step * |v - o| ~ 2e-2, which no calibration on the CPU side predicts.  The tight
    # bound on the attention arithmetic itself is taken where both sides read identical codes (next test).
    tol = TOL_FP8
    if kernel == sgc.SGC_KERNEL_MFMA_FP8:
        # The fp8 first product rounds every rotated query row to e4m3 (3 significant bits).  Over prompts this short a
        # row's weight sits on few keys and that rounding alone moves outputs by several 1e-2 (emulated below on the
        # oracle's side); the stated 6e-2 is what this path is held to at the long prompts it is meant for (configs[4]).
        caches = oracle_caches(w)
        floor = max(fp8_query_floor(*caches[int(w.labels[n])], *w.suffix_qkv_query(n), w.rope_base)
                    for n in range(w.n_queries) if w.suffix_len[n] > 0)
        _say(f"  fp8 first product: e4m3 query floor {floor:.3e}")
        tol = 4 * floor + 6e-3
    _check_suffix(w, out, tol=tol)


@pytest.mark.parametrize("kernel", [sgc.SGC_KERNEL_MFMA, sgc.SGC_KERNEL_MFMA_FP8])
def test_fp8_imported_oracle_cache_isolates_the_attention(kernel):
    # load the ORACLE's quantised cache into the pages, so both sides read identical codes
    w = workloads.custom("fp8_import", n_q_heads=8, n_kv_heads=1, head_dim=128, rope_base=500000.0, io_dtype="bf16",
                         kv_dtype="fp8_e4m3", prefix_len=[150], cluster_sizes=[3], suffix_range=(5, 40), seed=29)
    pk, pv = w.prefix_kv(0)
    ck, cv, _, _ = orc.prefix_prefill(None, pk, pv, w.rope_base)
    kc, ksc, kdeq = orc.quantise_e4m3(ck)
    vc, vsc, vdeq = orc.quantise_e4m3(cv)
    with Session(w, kernel=kernel) as s:
        s.alloc_cluster(0)
        s.import_cluster(0, 0, kc, vc, ksc, vsc)
        s.assign()
        q, k, v = w.suffix_qkv()
        do = s.suffix_prefill(*(to_device(x, "bf16") for x in (q, k, v)))
        torch.cuda.synchronize()
        o = to_host_f32(do)
    o_ref, _ = orc.suffix_prefill_batched(w.labels, w.cu_seqlens, [kdeq], [vdeq], q, k, v, w.rope_base)
    st = err_stats(o, o_ref)
    _say(f"  fp8 import max_abs {st['max_abs']:.3e}")
    # identical codes on both sides: what is left is the rounding of the output to bf16 (half an ulp of values up to 2:
    # 3.9e-3) plus the binary16 query and bf16 weight roundings (about 1e-3 together on unit-variance data)
    if kernel == sgc.SGC_KERNEL_MFMA:
        assert st["max_abs"] <= 6e-3
    else:
        # the fp8 first product rounds the rotated query to e4m3 (3 significant bits) under a power-of-two row scale:
        # four times what that rounding alone costs on this very input (numpy emulation on the oracle's side)
        floor = max(fp8_query_floor(kdeq, vdeq, *w.suffix_qkv_query(n), w.rope_base) for n in range(w.n_queries))
        _say(f"  fp8 first product: e4m3 query floor {floor:.3e}")
        assert st["max_abs"] <= min(TOL_FP8, 4 * floor + 6e-3)


# ---- configs[1..4] at full size, in the benchmark's launch configuration ---------------------------
# configs[1] and configs[2] are checked on EVERY row against the oracle; configs[3] on a query and head of every
# (cluster, layer) pair, all rows of the pair; configs[4] on a query of every cluster, all heads and rows.
def _sampled_queries(w, per_cluster, seed=0):
    rng = np.random.default_rng(seed)
    picks = []
    for c in range(w.n_clusters):
        members = np.flatnonzero(w.labels == c)
        if members.size:
            picks.extend(rng.choice(members, size=min(per_cluster, members.size), replace=False).tolist())
    return sorted(picks)


def test_config1_llama3_8b_layer_full_size_every_row():
    w = workloads.config(1)
    _say("config 1", w.name, "T", w.total_suffix_tokens, "flop %.3e" % w.flops())
    out = run_workload(w)
    _check_bookkeeping(w, out)
    tight, lse_bar = tight_bar(w, _sampled_queries(w, 1)[:4])
    st = _check_suffix(w, out, queries=None, tol=TOL_BF16, lse_tol=lse_bar)       # all 320 queries, all heads, all rows
    # Outlier key channels make this the config with the peakiest softmax.  With the rotated keys and queries held
    # as binary16 the largest deviation an ideal kernel shows over the whole batch is 7.8e-3 (the bf16 rounding of
    # the output itself); the same emulation with bf16 keys and queries shows 2.6e-2.
    assert st["max_abs"] <= 1.2e-2
    assert np.isfinite(out["o"]).all() and np.abs(out["o"]).max() < 8


def test_config1_prefix_prefill_batched_full_size_every_row():
    """The first half of the benchmark's step as it is launched there: the ten 1024-token prompts of configs[1] in ONE
    batched call with their queries (ingest + causal attention, 2560 row tiles); every row of every cluster, its LSE and
    the exported cache against the oracle."""
    w = workloads.config(1)
    clusters = list(range(w.n_clusters))
    with Session(w) as s:
        for c in clusters:
            s.alloc_cluster(c)
        got = s.prefix_prefill_batched(clusters, 0, with_q=True, want_lse=True)
        worst = worst_lse = 0.0
        for c, (do, dlse) in zip(clusters, got):
            pk, pv = w.prefix_kv(c)
            ck, cv, o_ref, lse_ref = orc.prefix_prefill(w.prefix_q(c), pk, pv, w.rope_base, want_lse=True)
            ek, ev, _, _ = s.export_cluster(c)
            assert np.array_equal(ev, pv)
            assert np.all(np.abs(ek - ck) <= np.abs(ck) * 2.0 ** -11 + 1e-5)
            o = to_host_f32(do)
            assert np.isfinite(o).all()
            worst = max(worst, float(np.abs(o - o_ref).max()))
            worst_lse = max(worst_lse, float(np.abs(dlse.cpu().numpy() - lse_ref).max()))
        _say(f"  configs[1] prompts, {len(clusters)} x {int(w.prefix_len[0])} tokens x {w.n_q_heads} heads: max_abs {worst:.3e} lse {worst_lse:.3e}")
        assert worst <= TOL_BF16 and worst_lse <= 2e-2


def test_config2_llama2_7b_ragged_full_size_every_row():
    w = workloads.config(2)
    _say("config 2", w.name, "T", w.total_suffix_tokens, "flop %.3e" % w.flops())
    out = run_workload(w, want_lse=False)
    _check_bookkeeping(w, out)
    _check_suffix(w, out, queries=None, tol=TOL_BF16, tight=tight_bar(w, _sampled_queries(w, 1)[:3])[0])
    assert np.isfinite(out["o"]).all()


def test_config3_llama3_8b_stack32_every_cluster_and_layer():
    """32 layers over one resident paged cache (8 GiB of pages), every layer with the workload's own seeded data:
    all caches are filled before any suffix prefill runs; then each layer's whole batch runs in one launch and, for
    every (cluster, layer) pair, all rows of one of the cluster's queries under one query head are compared with
    the oracle (the head changes with the pair, so all 32 heads are visited)."""
    from concurrent.futures import ThreadPoolExecutor
    w = workloads.config(3)
    clusters = list(range(w.n_clusters))
    cu = w.cu_seqlens
    pick = {c: int(np.flatnonzero(w.labels == c)[c % 16]) for c in clusters}        # one query per cluster
    with Session(w) as s, ThreadPoolExecutor(max_workers=4) as pool:
        pool_gib = s.pool.numel() / 2 ** 30
        _say("config 3", w.name, "T/layer", w.total_suffix_tokens, "pool GiB %.2f" % pool_gib)
        assert pool_gib >= 8.0
        for c in clusters:
            s.alloc_cluster(c)
        ahead = [pool.submit(lambda l=l: [w.prefix_kv(c, l) for c in clusters]) for l in range(min(3, w.n_layers))]
        for layer in range(w.n_layers):                       # fill every layer of every cluster first
            kv = ahead.pop(0).result()
            if layer + 3 < w.n_layers:
                ahead.append(pool.submit(lambda l=layer + 3: [w.prefix_kv(c, l) for c in clusters]))
            dk = [to_device(k, "bf16") for k, _ in kv]
            dv = [to_device(v, "bf16") for _, v in kv]
            sgc.sgc_prefix_prefill_batched(s.ctx, s.cache, clusters, layer, None, [t.data_ptr() for t in dk],
                                           [t.data_ptr() for t in dv], None, None, s.stream)
            torch.cuda.synchronize()
            del kv, dk, dv
        order, off, cu_out = s.assign()
        _check_bookkeeping(w, {"order": order, "cluster_off": off, "cu_seqlens": cu_out})
        ahead = [pool.submit(w.suffix_qkv, l) for l in range(min(2, w.n_layers))]
        worst = 0.0
        for layer in range(w.n_layers):
            q, k, v = ahead.pop(0).result()
            if layer + 2 < w.n_layers:
                ahead.append(pool.submit(w.suffix_qkv, layer + 2))
            do = s.suffix_prefill(*(to_device(x, "bf16") for x in (q, k, v)), layer=layer)
            torch.cuda.synchronize()
            o = to_host_f32(do)
            assert np.isfinite(o).all()
            layer_worst = 0.0
            for c in clusters:
                n, head = pick[c], (5 * layer + 3 * c) % w.n_q_heads
                ck, cv, _, _ = orc.prefix_prefill(None, *w.prefix_kv(c, layer), w.rope_base)
                a, b = int(cu[n]), int(cu[n + 1])
                o_ref, _ = orc.suffix_prefill_head(ck, cv, q[a:b], k[a:b], v[a:b], head, w.rope_base)
                layer_worst = max(layer_worst, float(np.abs(o[a:b, head] - o_ref).max()))
            _say(f"  layer {layer}: 16 (cluster, head) pairs x 128 rows, max_abs {layer_worst:.3e}")
            assert layer_worst <= TOL_BF16
            worst = max(worst, layer_worst)
            del q, k, v, do, o
        _say(f"  config 3 worst over 512 (cluster, layer) pairs {worst:.3e}")


@pytest.mark.parametrize("kernel", [sgc.SGC_KERNEL_MFMA_FP8, sgc.SGC_KERNEL_MFMA])
def test_config4_llama70b_fp8_long_prefix_full_size_every_cluster(kernel):
    """fp8 e4m3 cache, 16 384-token prefixes, 1024 queries of 32-256 tokens: the whole batch in one launch,
    checked on one query of every cluster (all 64 heads, all rows) against the oracle reading its own quantised
    cache.  Both first products: on the e4m3 codes (the path bench.py times for this configuration) and on 16-bit
    operands."""
    w = workloads.config(4)
    _say("config 4", w.name, "T", w.total_suffix_tokens, "flop %.3e" % w.flops(), "kernel", kernel)
    out = run_workload(w, want_lse=False, kernel=kernel)
    _check_bookkeeping(w, out)
    qs = _sampled_queries(w, 1)                     # 8 queries, one per cluster
    assert sorted(int(w.labels[n]) for n in qs) == list(range(w.n_clusters))
    if "ref" not in _CONFIG4_ORACLE:                # the oracle's rows are the same for both kernels: computed once
        _CONFIG4_ORACLE["ref"] = oracle_suffix(w, 0, qs)
    rows, o_ref, _ = _CONFIG4_ORACLE["ref"]
    st = err_stats(out["o"][rows], o_ref)
    _say(f"  {w.name}: rows {len(rows)} max_abs {st['max_abs']:.3e} rel {st['rel']:.3e} (tol {TOL_FP8:g})")
    assert st["max_abs"] <= TOL_FP8
    assert np.isfinite(out["o"]).all()


_CONFIG4_ORACLE = {}


def test_streaming_schedule_release_after_each_cluster_equals_all_resident():
    """Sec. 3.4: clusters are served one after another, each cache released before the next is computed.  With
    a page pool that only holds the largest cluster, serving cluster by cluster gives bit-identical outputs to
    the all-resident batched run (a row tile never mixes clusters, so the arithmetic is the same)."""
    w = _small_gqa(seed=61)
    ref = run_workload(w, kernel=sgc.SGC_KERNEL_MFMA)
    q, k, v = w.suffix_qkv()
    cu = w.cu_seqlens
    largest = int(max(-(-int(p) // 16) for p in w.prefix_len))
    o = np.zeros_like(ref["o"])
    with Session(w, kernel=sgc.SGC_KERNEL_MFMA, total_pages=largest) as s:
        for c in range(w.n_clusters):
            members = np.flatnonzero(w.labels == c)
            s.alloc_cluster(c)
            assert sgc.sgc_cache_free_pages(s.cache) == largest - (-(-int(w.prefix_len[c]) // 16))
            if c + 1 < w.n_clusters and w.prefix_len[c + 1] > 16 * sgc.sgc_cache_free_pages(s.cache):
                with pytest.raises(sgc.SgcError) as e:      # the next cluster does not fit beside this one
                    s.alloc_cluster(c + 1)
                assert e.value.status == sgc.SGC_ENOMEM
            s.prefix_prefill(c)
            rows = np.concatenate([np.arange(cu[n], cu[n + 1]) for n in members])
            s.assign(np.full(members.size, c, dtype=np.int32), w.suffix_len[members])
            do = s.suffix_prefill(*(to_device(x[rows], "bf16") for x in (q, k, v)))
            torch.cuda.synchronize()
            o[rows] = to_host_f32(do)
            s.free_cluster(c)
            assert sgc.sgc_cache_free_pages(s.cache) == largest
    assert np.array_equal(o, ref["o"])


def test_steps_enqueued_back_to_back_equal_steps_run_one_at_a_time():
    """A serving loop enqueues batch after batch on one stream without waiting for the GPU: pages, plan tables and
    work lists of a step are recycled for the next one while earlier kernels are still running.  Every step's
    output must be bit-identical to the same
    step run alone with the GPU idle before and after (different batch composition and suffix lengths per step, so
    a table or page that is overwritten too early shows)."""
    w = workloads.custom("pipelined", n_q_heads=8, n_kv_heads=2, head_dim=128, rope_base=500000.0, io_dtype="bf16",
                         prefix_len=[700, 333, 129], cluster_sizes=[30, 20, 14], suffix_range=(1, 70), seed=77)
    rng = np.random.default_rng(5)
    n_steps = 8
    q, k, v = w.suffix_qkv()
    cu = w.cu_seqlens
    batches = []
    for _ in range(n_steps):                   # a random subset of the queries, in random order
        members = rng.permutation(w.n_queries)[: int(rng.integers(w.n_queries // 2, w.n_queries + 1))]
        rows = np.concatenate([np.arange(cu[n], cu[n + 1]) for n in members])
        batches.append((w.labels[members], w.suffix_len[members], [to_device(x[rows], "bf16") for x in (q, k, v)]))
    pk = [[to_device(a, "bf16") for a in w.prefix_kv(c)] for c in range(w.n_clusters)]
    clusters = list(range(w.n_clusters))

    def run(wait_each_step):
        outs = []
        with Session(w, kernel=sgc.SGC_KERNEL_MFMA) as s:
            for labels, slen, (dq, dk, dv) in batches:
                order = clusters
                for c in order:
                    s.alloc_cluster(c)
                sgc.sgc_prefix_prefill_batched(s.ctx, s.cache, order, 0, None, [pk[c][0].data_ptr() for c in order],
                                               [pk[c][1].data_ptr() for c in order], None, None, s.stream)
                s.assign(labels, slen)
                outs.append(s.suffix_prefill(dq, dk, dv))
                if wait_each_step:
                    torch.cuda.synchronize()
                for c in order:
                    s.free_cluster(c)
            torch.cuda.synchronize()
            return [to_host_f32(o) for o in outs]

    alone = run(True)
    together = run(False)
    for i, (a, b) in enumerate(zip(alone, together)):
        assert np.isfinite(a).all() and np.array_equal(a, b), f"step {i} differs"
    # and the first batch against the oracle, so that "identical" is not "identically wrong"
    labels, slen, (dq, dk, dv) = batches[0]
    caches = oracle_caches(w)
    sub_cu = np.concatenate([[0], np.cumsum(slen)])
    o_ref, _ = orc.suffix_prefill_batched(labels, sub_cu, [caches[c][0] for c in clusters], [caches[c][1] for c in clusters],
                                          to_host_f32(dq), to_host_f32(dk), to_host_f32(dv), w.rope_base)
    assert np.abs(alone[0] - o_ref).max() <= 2e-2


def test_kernel_timing_of_every_nth_launch():
    """sgc_timing_enable(ctx, n): the events go around the kernels of launches 0, n, 2 n, ... only; the durations are
    positive, launches beyond those recorded are refused, and timing never changes a result."""
    w = workloads.custom("timing", n_q_heads=8, n_kv_heads=2, head_dim=128, rope_base=500000.0, io_dtype="bf16",
                         prefix_len=[200, 77], cluster_sizes=[5, 3], suffix_range=(3, 40), seed=31)
    q, k, v = w.suffix_qkv()
    dq, dk, dv = (to_device(x, "bf16") for x in (q, k, v))
    with Session(w, kernel=sgc.SGC_KERNEL_MFMA) as s:
        for c in range(w.n_clusters):
            s.alloc_cluster(c)
            s.prefix_prefill(c)
        s.assign(w.labels, w.suffix_len)
        plain = to_host_f32(s.suffix_prefill(dq, dk, dv))
        sgc.sgc_timing_enable(s.ctx, 4)
        outs = [to_host_f32(s.suffix_prefill(dq, dk, dv)) for _ in range(9)]          # launches 0, 4 and 8 are timed
        for back in range(3):
            ingest_ms, attn_ms = sgc.sgc_timing_get(s.ctx, back)
            assert 0.0 < ingest_ms < 10.0 and 0.0 < attn_ms < 10.0
        with pytest.raises(sgc.SgcError) as e:
            sgc.sgc_timing_get(s.ctx, 3)
        assert e.value.status == sgc.SGC_ESTATE
        sgc.sgc_timing_enable(s.ctx, 1)                                                # restarts the count: every launch
        outs.append(to_host_f32(s.suffix_prefill(dq, dk, dv)))
        assert sgc.sgc_timing_last(s.ctx)[1] > 0.0
        with pytest.raises(sgc.SgcError):
            sgc.sgc_timing_get(s.ctx, 1)
        sgc.sgc_timing_enable(s.ctx, 0)
        with pytest.raises(sgc.SgcError):
            sgc.sgc_timing_last(s.ctx)
    for o in outs:
        assert np.array_equal(o, plain)


@pytest.mark.parametrize("seed", list(range(300, 312)))
def test_random_shapes_against_oracle(seed):
    """Seeded random small workloads: head counts and group sizes, one to four clusters with prompts of 0-400 tokens
    (page and tile multiples among them), empty clusters and empty queries, question lengths of 0-100 around the
    16 / 32 / 64 boundaries the own-suffix tiles split at; bf16 and fp8 caches."""
    rng = np.random.default_rng(seed)
    Hkv = int(rng.choice([1, 2, 4]))
    g = int(rng.choice([1, 2, 3, 4, 8]))
    nc = int(rng.integers(1, 5))
    edges = [0, 1, 15, 16, 17, 63, 64, 65, 127, 128, 129, 256]
    prefix = [int(rng.choice(edges)) if rng.random() < 0.5 else int(rng.integers(0, 401)) for _ in range(nc)]
    sizes = [int(rng.integers(0, 9)) for _ in range(nc)]
    if sum(sizes) == 0:
        sizes[0] = 3
    s_edges = [0, 1, 15, 16, 17, 31, 32, 33, 47, 48, 63, 64, 65, 96]
    slen = [int(rng.choice(s_edges)) if rng.random() < 0.5 else int(rng.integers(0, 101)) for _ in range(sum(sizes))]
    kv = "fp8_e4m3" if seed % 3 == 0 else "bf16"
    w = workloads.custom(f"random_{seed}", n_q_heads=Hkv * g, n_kv_heads=Hkv, head_dim=128, rope_base=500000.0, io_dtype="bf16",
                         kv_dtype=kv, prefix_len=prefix, cluster_sizes=sizes, suffix_len=slen, seed=seed)
    _say(f"random {seed}: Hq {Hkv * g} Hkv {Hkv} prefix {prefix} sizes {sizes} suffix {slen} kv {kv}")
    out = run_workload(w, kernel=sgc.SGC_KERNEL_MFMA)
    _check_bookkeeping(w, out)
    # stated bar, and for bf16 caches also four times what an ideal bf16 kernel's roundings cost on this very input
    tight = tight_bar(w, range(w.n_queries))[0] if kv == "bf16" else None
    _check_suffix(w, out, tol=TOL_FP8 if kv == "fp8_e4m3" else TOL_BF16, tight=tight)
