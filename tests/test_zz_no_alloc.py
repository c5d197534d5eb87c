"""The decode entry point for callers that cannot allocate (static device scratch) against the allocating one,
through the C ABI: same kernels, so outputs and log-sum-exps must be bit-identical; two calls in a row, the second
on a smaller batch, so that what the first call left in the shared scratch array cannot leak into the second."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

from oracle import oracle as orc
from paper_2505_10951_amd import sgc, workloads
from paper_2505_10951_amd.harness import Session, to_device, to_host_f32
from ref_util import oracle_caches

pytestmark = pytest.mark.gpu


def _prepare(w, cap):
    s = Session(w, kernel=sgc.SGC_KERNEL_MFMA)
    for c in range(w.n_clusters):
        s.alloc_cluster(c)
    s.prefix_prefill_batched(list(range(w.n_clusters)), 0)
    s.assign()
    s.enable_decode(cap)
    q, k, v = w.suffix_qkv(0)
    s.suffix_prefill(*(to_device(x, "bf16") for x in (q, k, v)), layer=0)
    torch.cuda.synchronize()
    return s


def _step(s, w, t, entry):
    dq, dk, dv = (to_device(x, "bf16") for x in w.decode_qkv(t, 0))
    do = torch.full_like(dq, 7.0)
    dlse = torch.full((w.n_q_heads, w.n_queries), 7.0, dtype=torch.float32, device="cuda:0")
    entry(s.ctx, s.cache, s.plan, 0, t, dq.data_ptr(), dk.data_ptr(), dv.data_ptr(), do.data_ptr(), dlse.data_ptr(), s.stream)
    torch.cuda.synchronize()
    return to_host_f32(do), dlse.cpu().numpy()


def test_noalloc_decode_step_equals_allocating_entry_point_two_calls_in_a_row():
    big = workloads.custom("noalloc_big", n_q_heads=8, n_kv_heads=2, head_dim=128, rope_base=500000.0, io_dtype="bf16",
                           prefix_len=[2100, 333, 0], cluster_sizes=[9, 6, 3], suffix_range=(0, 70), seed=91, k_outlier_scale=8.0)
    small = workloads.custom("noalloc_small", n_q_heads=8, n_kv_heads=2, head_dim=128, rope_base=500000.0, io_dtype="bf16",
                             prefix_len=[130, 40], cluster_sizes=[3, 2], suffix_range=(1, 20), seed=92)
    sb, ss = _prepare(big, 3), _prepare(small, 3)
    try:
        # the new entry point refuses what it cannot do without allocating: here the page tables are current, so it runs
        ref_big = [_step(sb, big, t, sgc.sgc_decode_step_batched) for t in range(2)]
        ref_small = [_step(ss, small, t, sgc.sgc_decode_step_batched) for t in range(2)]
        # the same steps again (a step rewrites the token it appends): big batch, then the small one right behind it
        for t in range(2):
            got_big = _step(sb, big, t, sgc.sgc_decode_step_batched_noalloc)
            got_small = _step(ss, small, t, sgc.sgc_decode_step_batched_noalloc)
            assert np.isfinite(got_big[0]).all() and np.isfinite(got_small[0]).all()
            assert np.array_equal(got_big[0], ref_big[t][0]) and np.array_equal(got_big[1], ref_big[t][1]), f"big batch, step {t}"
            assert np.array_equal(got_small[0], ref_small[t][0]) and np.array_equal(got_small[1], ref_small[t][1]), f"small batch, step {t}"
        # and against the oracle, so that "identical" is not "identically wrong": step 0 of the small batch
        caches = oracle_caches(small, 0)
        dec = small.decode_qkv(0, 0)
        worst = 0.0
        o0 = _step(ss, small, 0, sgc.sgc_decode_step_batched_noalloc)[0]
        for n in range(small.n_queries):
            S = int(small.suffix_len[n])
            q, k, v = small.suffix_qkv_query(n, 0)
            qe, ke, ve = (np.concatenate([a, b[n:n + 1]]) for a, b in zip((q, k, v), dec))
            ck, cv = caches[int(small.labels[n])]
            oo, _, _ = orc.suffix_prefill(ck, cv, qe, ke, ve, small.rope_base)
            worst = max(worst, float(np.abs(o0[n] - oo[S]).max()))
        print(f"  noalloc decode vs oracle: max_abs {worst:.3e}", flush=True)
        assert worst <= 2e-2
    finally:
        sb.close()
        ss.close()


def test_noalloc_decode_step_refuses_what_needs_an_allocation():
    w = workloads.custom("noalloc_state", n_q_heads=8, n_kv_heads=2, head_dim=128, rope_base=500000.0, io_dtype="bf16",
                         prefix_len=[130, 40], cluster_sizes=[3, 2], suffix_range=(1, 20), seed=93)
    s = _prepare(w, 2)
    try:
        dq, dk, dv = (to_device(x, "bf16") for x in w.decode_qkv(0, 0))
        do = torch.zeros_like(dq)
        args = (s.ctx, s.cache, s.plan, 0, 0, dq.data_ptr(), dk.data_ptr(), dv.data_ptr(), do.data_ptr(), None, s.stream)
        sgc.sgc_decode_step_batched_noalloc(*args)                  # fine: everything is resident
        torch.cuda.synchronize()
        with pytest.raises(sgc.SgcError) as e:                      # step outside the room reserved for decoding
            sgc.sgc_decode_step_batched_noalloc(s.ctx, s.cache, s.plan, 0, 5, dq.data_ptr(), dk.data_ptr(), dv.data_ptr(),
                                                do.data_ptr(), None, s.stream)
        assert e.value.status == sgc.SGC_EINVAL
        # releasing a cluster leaves the device page tables stale; bringing them up to date allocates staging memory
        s.free_cluster(1)
        with pytest.raises(sgc.SgcError) as e:
            sgc.sgc_decode_step_batched_noalloc(*args)
        assert e.value.status == sgc.SGC_ESTATE
    finally:
        s.close()
