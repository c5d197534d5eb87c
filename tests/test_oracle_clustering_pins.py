"""Pins of the clustering oracle (SubGCache Sec. 3.2, App. A.2, Table 3) against things other than itself:
scipy's hierarchical clustering as a library special case, textbook special cases and invariances."""
import numpy as np
import pytest
from scipy.cluster.hierarchy import linkage as scipy_linkage

from oracle import oracle as orc


def _same_partition(a, b):
    a, b = np.asarray(a), np.asarray(b)
    pairs = set(zip(a.tolist(), b.tolist()))
    return len(pairs) == len(set(a.tolist())) == len(set(b.tolist()))


def _scipy_partition_after_merges(x, method, c):
    """Partition after the first m - c merges of scipy's linkage matrix (rows are in merge order, for the
    monotone linkages sorted by height, which is a valid merge order).  Centroid linkage can invert heights,
    so cutting by height would not be "the partition with c clusters on the way up"."""
    m = x.shape[0]
    z = scipy_linkage(x, method=method, metric="euclidean")
    members = {i: [i] for i in range(m)}
    for r in range(m - c):
        a, b = int(z[r, 0]), int(z[r, 1])
        members[m + r] = members.pop(a) + members.pop(b)
    labels = np.empty(m, dtype=np.int64)
    for k, (_, mem) in enumerate(sorted(members.items())):
        labels[mem] = k
    return labels


@pytest.mark.parametrize("linkage", orc.LINKAGES)
@pytest.mark.parametrize("m,dim,c,seed", [(12, 3, 4, 0), (25, 8, 5, 1), (30, 16, 1, 2), (30, 16, 30, 3), (40, 5, 7, 4)])
def test_matches_scipy_partition_on_generic_points(linkage, m, dim, c, seed):
    x = np.random.default_rng(seed).standard_normal((m, dim))
    mine = orc.cluster_queries(x, c, linkage)
    ref = _scipy_partition_after_merges(x, linkage, c)
    assert _same_partition(mine, ref)
    assert mine.max() + 1 == c and mine.min() == 0


@pytest.mark.parametrize("linkage", orc.LINKAGES)
def test_well_separated_blobs_are_recovered_and_numbered_by_first_member(linkage):
    rng = np.random.default_rng(7)
    truth = np.array([2, 0, 1, 1, 0, 2, 2, 1, 0, 0, 1, 2])
    centers = np.array([[0.0, 0.0], [50.0, 0.0], [0.0, 80.0]])
    x = centers[truth] + 0.5 * rng.standard_normal((truth.size, 2))
    labels = orc.cluster_queries(x, 3, linkage)
    assert _same_partition(labels, truth)
    first = [int(np.flatnonzero(labels == c)[0]) for c in range(3)]
    assert first == sorted(first) and labels[0] == 0


@pytest.mark.parametrize("linkage", orc.LINKAGES)
def test_invariances(linkage):
    rng = np.random.default_rng(11)
    x = rng.standard_normal((20, 6))
    base = orc.cluster_queries(x, 4, linkage)
    q, _ = np.linalg.qr(rng.standard_normal((6, 6)))                 # rotation + shift: distances unchanged
    assert _same_partition(orc.cluster_queries(x @ q + 3.0, 4, linkage), base)
    perm = rng.permutation(20)                                       # order of the queries does not matter
    assert _same_partition(orc.cluster_queries(x[perm], 4, linkage), base[perm])
    assert _same_partition(orc.cluster_queries(2.5 * x, 4, linkage), base)      # nor does the scale


def test_one_dimensional_hand_example_per_linkage():
    # points 0, 1, 3, 6.2, 10 on a line.  Single linkage chains neighbours: {0,1}, then 3 joins (gap 2),
    # then 6.2 (gap 3.2) -> at 2 clusters {0,1,3,6.2} | {10}.  Complete linkage: {0,1}; then 3 joins
    # (diameter 3) before {6.2,10} (3.8) -> at 2 clusters {0,1,3} | {6.2,10}.
    x = np.array([[0.0], [1.0], [3.0], [6.2], [10.0]])
    assert orc.cluster_queries(x, 2, "single").tolist() == [0, 0, 0, 0, 1]
    assert orc.cluster_queries(x, 2, "complete").tolist() == [0, 0, 0, 1, 1]
    assert orc.cluster_queries(x, 3, "complete").tolist() == [0, 0, 0, 1, 2]
    # Ward: merging {0,1} with 3 grows the sum of squares by 2*1/3 * 2.5^2 = 4.17, 6.2 with 10 by 7.22
    assert orc.cluster_queries(x, 3, "ward").tolist() == [0, 0, 0, 1, 2]


def test_ties_go_to_the_smallest_first_members():
    x = np.array([[0.0], [1.0], [2.0], [3.0]])            # all neighbour gaps equal
    assert orc.cluster_queries(x, 3, "single").tolist() == [0, 0, 1, 2]
    assert orc.cluster_queries(x, 2, "single").tolist() == [0, 0, 0, 1]
    assert orc.cluster_queries(x, 2, "complete").tolist() == [0, 0, 1, 1]
    dup = np.array([[5.0, 5.0], [1.0, 1.0], [5.0, 5.0], [1.0, 1.0]])
    assert orc.cluster_queries(dup, 2, "ward").tolist() == [0, 1, 0, 1]


def test_argument_checks():
    x = np.zeros((3, 2))
    for bad in (0, 4):
        with pytest.raises(ValueError):
            orc.cluster_queries(x, bad)
    with pytest.raises(ValueError):
        orc.cluster_queries(x, 2, "median")
