"""The paper's flow end to end through the C ABI on the GPU machine (SubGCache Sec. 3.2 -> 3.3 -> 3.4): embeddings of the
queries' retrieved subgraphs are clustered, each cluster's representative subgraph is the union of its queries'
subgraphs, its prompt is prefilled once into the cluster's cache, and every query appends its question tokens to it.
Labels, unions and bookkeeping must equal the oracle's bit for bit, the attention output within the stated bar.
Linkages are Table 3's.  (The prompt length of a cluster stands in for the tokenised text of its representative
subgraph: a fixed number of tokens per distinct node and per distinct edge, so it follows from the union.)"""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

from oracle import oracle as orc
from paper_2505_10951_amd import sgc, workloads
from paper_2505_10951_amd.harness import run_workload
from ref_util import err_stats, oracle_suffix, tight_bar

pytestmark = pytest.mark.gpu

TOKENS_PER_NODE, TOKENS_PER_EDGE = 3, 2


@pytest.mark.parametrize("linkage", orc.LINKAGES)
def test_cluster_union_assign_prefill_flow(linkage):
    n_clusters = 4
    base = workloads.custom("flow_base", n_q_heads=8, n_kv_heads=2, head_dim=128, rope_base=500000.0, io_dtype="bf16",
                            prefix_len=[1] * n_clusters, cluster_sizes=[17, 9, 13, 5], suffix_range=(3, 40), seed=404)
    # Sec. 3.2: cluster the queries by the embeddings of their retrieved subgraphs (noisy enough that linkages differ)
    emb = base.query_embeddings(dim=24, overlap=0.9)
    labels = sgc.sgc_cluster_queries(None, emb, n_clusters, linkage)
    assert np.array_equal(labels, orc.cluster_queries(emb, n_clusters, linkage))
    # Sec. 3.3: representative subgraph of a cluster = union of the nodes and edges its queries retrieved
    node_lists, edge_lists = base.retrieved_subgraphs(graph_nodes=400, core=12, extra=3)
    nodes, edges = sgc.sgc_union_subgraphs(None, labels, n_clusters, node_lists, edge_lists)
    rn, re = orc.union_subgraphs(labels, n_clusters, node_lists,
                                 [[tuple(e) for e in np.asarray(x).reshape(-1, 2).tolist()] for x in edge_lists])
    for k in range(n_clusters):
        assert nodes[k].tolist() == rn[k] and [tuple(e) for e in edges[k].tolist()] == re[k]
    prefix_len = [TOKENS_PER_NODE * len(rn[k]) + TOKENS_PER_EDGE * len(re[k]) for k in range(n_clusters)]
    # Sec. 3.4: one cache per cluster, filled once; every query of the cluster appends its question tokens
    w = workloads.custom(f"flow_{linkage}", n_q_heads=8, n_kv_heads=2, head_dim=128, rope_base=500000.0, io_dtype="bf16",
                         prefix_len=prefix_len, labels=labels, suffix_len=base.suffix_len, seed=405, k_outlier_scale=8.0)
    out = run_workload(w)
    o_ref, off_ref, cu_ref = orc.assign_clusters(labels, w.suffix_len, n_clusters)
    assert np.array_equal(out["order"], o_ref) and np.array_equal(out["cluster_off"], off_ref)
    assert np.array_equal(out["cu_seqlens"], cu_ref)
    rows, o_exp, _ = oracle_suffix(w, 0, None)
    st = err_stats(out["o"][rows], o_exp)
    bar = tight_bar(w, range(0, w.n_queries, 7))[0]
    print(f"  {linkage}: cluster sizes {np.bincount(labels, minlength=n_clusters).tolist()} prompts {prefix_len} "
          f"max_abs {st['max_abs']:.3e} (calibrated bar {bar:.3e})", flush=True)
    assert np.isfinite(out["o"]).all() and st["max_abs"] <= 2e-2 and st["max_abs"] <= bar
