"""Pins of the representative-subgraph oracle (SubGCache Sec. 3.3: union of all nodes and edges of a cluster's
retrieved subgraphs): the worked example of the section's Figure-1 walk-through shape, set-algebra
properties, and numpy's union as a library special case."""
import numpy as np

from oracle import oracle as orc


def test_two_clusters_by_hand():
    # queries 0,1,2 -> cluster 0, queries 3,4 -> cluster 1 (the grouping of the paper's running example)
    node_lists = [[3, 1], [1, 2], [5, 3], [9, 8], [8]]
    edge_lists = [[(3, 1)], [(1, 2), (2, 1)], [(5, 3), (3, 1)], [(9, 8)], []]
    nodes, edges = orc.union_subgraphs([0, 0, 0, 1, 1], 2, node_lists, edge_lists)
    assert nodes == [[1, 2, 3, 5], [8, 9]]
    assert edges == [[(1, 2), (2, 1), (3, 1), (5, 3)], [(9, 8)]]          # (1,2) and (2,1) are different edges


def test_properties_and_numpy_union():
    rng = np.random.default_rng(3)
    m, c = 40, 6
    labels = rng.integers(0, c, size=m)
    node_lists = [rng.integers(0, 60, size=rng.integers(0, 15)).tolist() for _ in range(m)]
    edge_lists = [[tuple(e) for e in rng.integers(0, 60, size=(rng.integers(0, 20), 2)).tolist()] for _ in range(m)]
    nodes, edges = orc.union_subgraphs(labels, c, node_lists, edge_lists)
    for k in range(c):
        members = np.flatnonzero(labels == k)
        ref = np.array([], dtype=np.int64)
        for i in members:
            ref = np.union1d(ref, np.asarray(node_lists[i], dtype=np.int64))      # library routine
        assert nodes[k] == ref.tolist()
        for i in members:                                                          # superset of every member
            assert set(node_lists[i]) <= set(nodes[k]) and set(edge_lists[i]) <= set(edges[k])
        assert edges[k] == sorted(set(e for i in members for e in edge_lists[i]))
        assert len(set(edges[k])) == len(edges[k])
    # idempotent: a query listed twice changes nothing; order of the queries does not matter
    perm = rng.permutation(m)
    n2, e2 = orc.union_subgraphs(labels[perm], c, [node_lists[i] for i in perm], [edge_lists[i] for i in perm])
    assert n2 == nodes and e2 == edges
    n3, e3 = orc.union_subgraphs(np.concatenate([labels, labels]), c, node_lists * 2, edge_lists * 2)
    assert n3 == nodes and e3 == edges
    # a cluster of one query is that query's own subgraph (Sec. 3.4: the method then degenerates to the baseline)
    n4, e4 = orc.union_subgraphs(np.arange(m), m, node_lists, edge_lists)
    assert all(n4[i] == sorted(set(node_lists[i])) and e4[i] == sorted(set(edge_lists[i])) for i in range(m))
