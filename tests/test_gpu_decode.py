"""Decode steps after the suffix prefill (SubGCache App. A.2: up to 32 generated tokens; Sec. 3.4: every
query of a cluster reuses the cluster's cache) through the C ABI, against the fp64 oracle: the token a query
generates at step t is row S + t of the oracle's suffix prefill over [question tokens; generated tokens]."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

from oracle import oracle as orc
from paper_2505_10951_amd import sgc, workloads
from paper_2505_10951_amd.harness import Session, to_device, to_host_f32
from ref_util import oracle_caches

pytestmark = pytest.mark.gpu

TOL = {"bf16": 2e-2, "fp8_e4m3": 6e-2}


def _oracle_decode(w, layer, n_steps, caches, queries=None):
    """o_ref [n_steps][n_queries][Hq][d], lse_ref [n_steps][Hq][n_queries] (a query without question tokens
    generates from the cached prompt and its own earlier tokens alone).  queries: only these are filled in."""
    dec = [w.decode_qkv(t, layer) for t in range(n_steps)]
    o = np.zeros((n_steps, w.n_queries, w.n_q_heads, w.head_dim))
    lse = np.zeros((n_steps, w.n_q_heads, w.n_queries))
    for n in (range(w.n_queries) if queries is None else queries):
        S = int(w.suffix_len[n])
        q, k, v = w.suffix_qkv_query(n, layer)
        qe = np.concatenate([q] + [d[0][n:n + 1] for d in dec])
        ke = np.concatenate([k] + [d[1][n:n + 1] for d in dec])
        ve = np.concatenate([v] + [d[2][n:n + 1] for d in dec])
        ck, cv = caches[int(w.labels[n])]
        oo, ll, _ = orc.suffix_prefill(ck, cv, qe, ke, ve, w.rope_base)
        o[:, n] = oo[S:]
        lse[:, :, n] = ll[:, S:].T
    return o, lse


def _run_decode(w, n_steps, layers=(0,), cap=None, kernel=sgc.SGC_KERNEL_MFMA):
    out = {}
    with Session(w, kernel=kernel) as s:
        for c in range(w.n_clusters):
            s.alloc_cluster(c)
        for layer in layers:
            s.prefix_prefill_batched(list(range(w.n_clusters)), layer)
        s.assign()
        s.enable_decode(cap or n_steps)
        for layer in layers:                       # every layer's suffix prefill first: the pools are per layer
            q, k, v = w.suffix_qkv(layer)
            s.suffix_prefill(*(to_device(x, "bf16") for x in (q, k, v)), layer=layer)
        for layer in layers:
            os_, ls_ = [], []
            for t in range(n_steps):
                dq, dk, dv = (to_device(x, "bf16") for x in w.decode_qkv(t, layer))
                do = torch.full_like(dq, 7.0)
                dlse = torch.full((w.n_q_heads, w.n_queries), 7.0, dtype=torch.float32, device="cuda:0")
                s.decode_step(t, dq, dk, dv, layer, do=do, dlse=dlse)
                torch.cuda.synchronize()
                os_.append(to_host_f32(do))
                ls_.append(dlse.cpu().numpy())
            out[layer] = (np.stack(os_), np.stack(ls_))
    return out


@pytest.mark.parametrize("kv", ["bf16", "fp8_e4m3", "fp8_e4m3 with the first product on the codes"])
def test_decode_steps_match_oracle_small(kv):
    kernel = sgc.SGC_KERNEL_MFMA_FP8 if "codes" in kv else sgc.SGC_KERNEL_MFMA
    kv = kv.split()[0]
    # suffix lengths around the page size so that appended tokens cross page boundaries; one query without question tokens;
    # one cluster without any cached keys
    if kernel == sgc.SGC_KERNEL_MFMA_FP8:
        # the first product on the codes rounds the query to e4m3: meant for long prompts, where a row's weight is spread
        # over many keys (over prompts of a few hundred tokens the same rounding moves outputs by up to 1e-1)
        w = workloads.custom("decode_long_fp8", n_q_heads=8, n_kv_heads=2, head_dim=128, rope_base=500000.0, io_dtype="bf16",
                             kv_dtype=kv, prefix_len=[6000, 2500], labels=[0, 1, 0, 1, 1, 0], suffix_len=[14, 16, 1, 30, 0, 64],
                             seed=33)
    else:
        w = workloads.custom("decode_small", n_q_heads=8, n_kv_heads=2, head_dim=128, rope_base=500000.0, io_dtype="bf16",
                             kv_dtype=kv, prefix_len=[200, 71, 0], labels=[0, 1, 0, 2, 1, 0, 2, 0, 1, 0],
                             suffix_len=[14, 16, 1, 30, 47, 0, 15, 64, 33, 5], seed=31, k_outlier_scale=8.0)
    n_steps = 6
    got = _run_decode(w, n_steps, kernel=kernel)[0]
    o_ref, lse_ref = _oracle_decode(w, 0, n_steps, oracle_caches(w, 0))
    err = np.abs(got[0] - o_ref).max()
    lerr = np.abs(got[1] - lse_ref).max()
    print(f"  decode {kv}: max_abs {err:.3e} lse {lerr:.3e}", flush=True)
    assert np.isfinite(got[0]).all() and err <= TOL[kv] and lerr <= 5e-2


def test_decode_two_layers_keep_their_own_pages():
    w = workloads.custom("decode_layers", n_q_heads=8, n_kv_heads=2, head_dim=128, rope_base=10000.0, io_dtype="bf16",
                         prefix_len=[130, 64], cluster_sizes=[5, 4], suffix_range=(3, 40), n_layers=2, seed=37)
    got = _run_decode(w, 4, layers=(0, 1), cap=8)
    for layer in (0, 1):
        o_ref, lse_ref = _oracle_decode(w, layer, 4, oracle_caches(w, layer))
        assert np.abs(got[layer][0] - o_ref).max() <= TOL["bf16"]
        assert np.abs(got[layer][1] - lse_ref).max() <= 5e-2


def test_decode_many_queries_span_several_row_tiles():
    # 80 queries in one cluster: 80 x 4 rows per KV head = 320 rows = 3 row tiles sharing the cluster's cache
    w = workloads.custom("decode_wide", n_q_heads=8, n_kv_heads=2, head_dim=128, rope_base=500000.0, io_dtype="bf16",
                         prefix_len=[300, 40], cluster_sizes=[80, 3], suffix_range=(1, 50), seed=41)
    got = _run_decode(w, 3)[0]
    o_ref, lse_ref = _oracle_decode(w, 0, 3, oracle_caches(w, 0))
    assert np.abs(got[0] - o_ref).max() <= TOL["bf16"] and np.abs(got[1] - lse_ref).max() <= 5e-2


@pytest.mark.parametrize("kv", ["bf16", "fp8_e4m3"])
def test_decode_long_prompts_split_the_cached_keys_into_ranges(kv):
    # prompts of 17-40 key steps and few row tiles: the cached part of a step runs as several key ranges per row tile
    # (one of the clusters is too short to fill every range), merged with the own keys by log-sum-exp
    w = workloads.custom("decode_split", n_q_heads=8, n_kv_heads=2, head_dim=128, rope_base=500000.0, io_dtype="bf16",
                         kv_dtype=kv, prefix_len=[2500, 1100, 70], cluster_sizes=[3, 2, 2], suffix_range=(2, 35), seed=43)
    got = _run_decode(w, 3)[0]
    o_ref, lse_ref = _oracle_decode(w, 0, 3, oracle_caches(w, 0))
    err, lerr = np.abs(got[0] - o_ref).max(), np.abs(got[1] - lse_ref).max()
    print(f"  decode split {kv}: max_abs {err:.3e} lse {lerr:.3e}", flush=True)
    assert np.isfinite(got[0]).all() and err <= TOL[kv] and lerr <= 5e-2


@pytest.mark.parametrize("g", [16, 1])
def test_decode_long_questions_and_the_widest_head_group(g):
    """Questions of up to 330 tokens (21 pages of own keys: six chunks of the own-keys kernel's online softmax, the last one
    partly filled) and, with g = 16, as many query heads per KV head as the matrix-core form of that kernel takes."""
    w = workloads.custom(f"decode_long_q_g{g}", n_q_heads=2 * g, n_kv_heads=2, head_dim=128, rope_base=500000.0, io_dtype="bf16",
                         prefix_len=[90, 0], labels=[0, 1, 0, 1, 0], suffix_len=[330, 257, 63, 64, 129], seed=47)
    n_steps = 4
    got = _run_decode(w, n_steps)[0]
    o_ref, lse_ref = _oracle_decode(w, 0, n_steps, oracle_caches(w, 0))
    err, lerr = np.abs(got[0] - o_ref).max(), np.abs(got[1] - lse_ref).max()
    print(f"  decode long questions g {g}: max_abs {err:.3e} lse {lerr:.3e}", flush=True)
    assert np.isfinite(got[0]).all() and err <= TOL["bf16"] and lerr <= 5e-2


def test_decode_config1_llama3_8b_layer_full_size_sampled():
    """The decode measurement of the benchmark, as it is launched there: configs[1] whole (320 queries, ten 1024-token
    prompts in two key ranges each, 80 row tiles), all 32 steps; two queries of every cluster, all heads and steps, against
    the oracle."""
    w = workloads.config(1)
    n_steps = 32
    got = _run_decode(w, n_steps, kernel=sgc.SGC_KERNEL_AUTO)[0]
    rng = np.random.default_rng(9)
    picks = sorted(int(n) for c in range(w.n_clusters) for n in rng.choice(np.flatnonzero(w.labels == c), 2, replace=False))
    o_ref, lse_ref = _oracle_decode(w, 0, n_steps, oracle_caches(w, 0, threads=8), queries=picks)
    err = np.abs(got[0][:, picks] - o_ref[:, picks]).max()
    lerr = np.abs(got[1][:, :, picks] - lse_ref[:, :, picks]).max()
    print(f"  decode configs[1] full size, {len(picks)} queries x {n_steps} steps: max_abs {err:.3e} lse {lerr:.3e}", flush=True)
    assert np.isfinite(got[0]).all() and np.isfinite(got[1]).all()
    assert err <= TOL["bf16"] and lerr <= 5e-2


@pytest.mark.parametrize("seed", [400, 401, 402, 403, 404, 405])
def test_decode_random_shapes_against_oracle(seed):
    """Seeded random small workloads: group sizes 1-8, prompts of 0-1500 tokens (long ones split into key ranges),
    question lengths of 0-60 around page boundaries, 2-5 generated tokens."""
    rng = np.random.default_rng(seed)
    Hkv = int(rng.choice([1, 2, 4]))
    g = int(rng.choice([1, 2, 4, 8]))
    nc = int(rng.integers(1, 4))
    prefix = [int(rng.choice([0, 16, 64, 100, 700, 1500])) for _ in range(nc)]
    sizes = [int(rng.integers(1, 7)) for _ in range(nc)]
    slen = [int(rng.choice([0, 1, 14, 15, 16, 17, 31, 32, 33, 47, 60])) for _ in range(sum(sizes))]
    kv = "fp8_e4m3" if seed % 2 else "bf16"
    w = workloads.custom(f"decode_random_{seed}", n_q_heads=Hkv * g, n_kv_heads=Hkv, head_dim=128, rope_base=500000.0,
                         io_dtype="bf16", kv_dtype=kv, prefix_len=prefix, cluster_sizes=sizes, suffix_len=slen, seed=seed)
    n_steps = int(rng.integers(2, 6))
    got = _run_decode(w, n_steps)[0]
    o_ref, lse_ref = _oracle_decode(w, 0, n_steps, oracle_caches(w, 0))
    err = np.abs(got[0] - o_ref).max()
    lerr = np.abs(got[1] - lse_ref).max()
    print(f"  decode random {seed}: Hq {Hkv * g} Hkv {Hkv} prefix {prefix} suffix {slen} steps {n_steps} {kv}: max_abs {err:.3e} lse {lerr:.3e}", flush=True)
    assert np.isfinite(got[0]).all() and err <= TOL[kv] and lerr <= 5e-2


def test_decode_argument_checks():
    w = workloads.custom("decode_args", n_q_heads=8, n_kv_heads=2, head_dim=128, rope_base=10000.0, io_dtype="bf16",
                         prefix_len=[32], cluster_sizes=[2], suffix_range=(4, 4), seed=43)
    with Session(w, kernel=sgc.SGC_KERNEL_MFMA) as s:
        s.alloc_cluster(0)
        s.prefix_prefill(0)
        s.assign()
        t = torch.zeros((2, 8, 128), dtype=torch.bfloat16, device="cuda:0")
        kv = torch.zeros((2, 2, 128), dtype=torch.bfloat16, device="cuda:0")
        with pytest.raises(sgc.SgcError) as e:                    # not enabled
            s.decode_step(0, t, kv, kv)
        assert e.value.status == sgc.SGC_ESTATE
        with pytest.raises(sgc.SgcError):                         # question + new tokens beyond 1024 own keys
            s.enable_decode(2000)
        s.enable_decode(4)
        with pytest.raises(sgc.SgcError) as e:                    # no suffix prefill yet
            s.decode_step(0, t, kv, kv)
        assert e.value.status == sgc.SGC_ESTATE
        q, k, v = w.suffix_qkv()
        s.suffix_prefill(*(to_device(x, "bf16") for x in (q, k, v)))
        with pytest.raises(sgc.SgcError) as e:                    # step outside the reserved room
            s.decode_step(4, t, kv, kv)
        assert e.value.status == sgc.SGC_EINVAL
        s.decode_step(3, t, kv, kv)
        torch.cuda.synchronize()
