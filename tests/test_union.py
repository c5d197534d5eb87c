"""sgc_union_subgraphs (host C++) against the representative-subgraph oracle: identical lists."""
import numpy as np
import pytest

from oracle import oracle as orc
from paper_2505_10951_amd import sgc, workloads


def _check(labels, c, node_lists, edge_lists):
    nodes, edges = sgc.sgc_union_subgraphs(None, labels, c, node_lists, edge_lists)
    rn, re = orc.union_subgraphs(labels, c, node_lists, [[tuple(e) for e in np.asarray(x).reshape(-1, 2).tolist()] for x in edge_lists])
    for k in range(c):
        assert nodes[k].dtype == np.int32 and nodes[k].tolist() == rn[k]
        assert [tuple(e) for e in edges[k].tolist()] == re[k]


@pytest.mark.parametrize("config", [1, 2])
def test_union_of_workload_subgraphs_equals_oracle(config):
    w = workloads.config(config)
    node_lists, edge_lists = w.retrieved_subgraphs()
    _check(w.labels, w.n_clusters, node_lists, edge_lists)
    # clustering the embeddings and taking the union per found cluster gives the same subgraphs, renumbered
    labels = sgc.sgc_cluster_queries(None, w.query_embeddings(), w.n_clusters)
    n1, _ = sgc.sgc_union_subgraphs(None, labels, w.n_clusters, node_lists, edge_lists)
    n0, _ = sgc.sgc_union_subgraphs(None, w.labels, w.n_clusters, node_lists, edge_lists)
    assert sorted(x.tolist() for x in n1) == sorted(x.tolist() for x in n0)


def test_edge_cases_negative_ids_empty_queries_empty_clusters():
    node_lists = [[-5, 7, 7], [], [2**31 - 1, -2**31, 0], [3]]
    edge_lists = [[(-5, 7), (7, -5), (-5, 7)], [], [(0, -2**31), (-2**31, 0)], []]
    _check([2, 0, 2, 0], 4, node_lists, edge_lists)
    nodes, edges = sgc.sgc_union_subgraphs(None, [2, 0, 2, 0], 4, node_lists, edge_lists)
    assert nodes[1].size == 0 and nodes[3].size == 0 and edges[0].shape == (0, 2)
    assert nodes[2].tolist() == [-2**31, -5, 0, 7, 2**31 - 1]
    assert [tuple(e) for e in edges[2].tolist()] == [(-2**31, 0), (-5, 7), (0, -2**31), (7, -5)]
    n, e = sgc.sgc_union_subgraphs(None, [], 2, [], [])
    assert len(n) == 2 and n[0].size == 0 and e[1].shape == (0, 2)


def test_argument_checks():
    with pytest.raises(sgc.SgcError):
        sgc.sgc_union_subgraphs(None, [0, 3], 2, [[1], [2]], [[], []])          # label out of range
    with pytest.raises(sgc.SgcError):
        sgc.sgc_union_subgraphs(None, [0], 0, [[1]], [[]])                      # no clusters
