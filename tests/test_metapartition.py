"""The library's meta-partitioning (host code, runs without a GPU) against the oracle, entry by entry."""
import itertools

import numpy as np
import pytest

from oracle import metapartition as omp
from paper_2408_09697_amd import binding as hb


def _same(got: dict, want: omp.MetaPartition):
    assert got["sub_rel"] == want.sub_rel
    assert got["sub_weight"] == want.sub_weight
    assert got["sub_links"] == want.sub_links
    assert got["sub_part"] == want.sub_part
    assert got["part_weight"] == want.part_weight
    assert got["replica_of"] == want.replica_of
    assert got["rel_mask"] == want.rel_mask
    assert got["type_mask"] == want.type_mask


def _metagraph(seed, n_types, n_rels, big=False):
    r = np.random.default_rng(seed)
    pairs = [(int(r.integers(n_types)), int(r.integers(n_types))) for _ in range(n_rels)]
    hi = 2**40 if big else 50                      # small weights make equal sums (the tie rules) common
    return pairs, [int(x) for x in r.integers(0, hi, n_types)], [int(x) for x in r.integers(0, hi, n_rels)]


@pytest.mark.parametrize("seed", range(40))
def test_library_matches_oracle_on_random_metagraphs(seed):
    r = np.random.default_rng(1000 + seed)
    n_types, n_rels = int(r.integers(1, 7)), int(r.integers(0, 13))
    pairs, tw, rw = _metagraph(seed, n_types, n_rels, big=seed % 2 == 1)
    for root, k, p in itertools.product(range(n_types), (1, 2, 3), (1, 2, 3, 7)):
        got = hb.heta_meta_partition(tw, [s for s, _ in pairs], [t for _, t in pairs], rw, root, k, p)
        _same(got, omp.meta_partition(tw, pairs, rw, root, k, p))


@pytest.mark.parametrize("seed", range(10))
def test_library_matches_oracle_with_metapaths(seed):
    r = np.random.default_rng(2000 + seed)
    n_types, n_rels = 4, 9
    pairs, tw, rw = _metagraph(50 + seed, n_types, n_rels)
    root = int(r.integers(n_types))
    tree = omp.build_metatree(pairs, root, 3)
    walks = []
    for j in range(1, len(tree)):
        path, at = [], j
        while at > 0:
            path.append(tree[at].via)
            at = tree[at].parent
        walks.append(path[::-1])
    if not walks:
        walks = [[]]
    pick = [walks[int(i)] for i in r.integers(0, len(walks), 6)] + [[]]      # repeats, shared prefixes, an empty path
    for p in (1, 2, 4):
        got = hb.heta_meta_partition(tw, [s for s, _ in pairs], [t for _, t in pairs], rw, root, 3, p, metapaths=pick)
        _same(got, omp.meta_partition(tw, pairs, rw, root, 3, p, metapaths=pick))


def test_library_on_the_bibliographic_metagraph_of_the_papers_example():
    # structure of the paper's example (Section 5): target type 0 with three relations into it
    pairs = [(1, 0), (0, 0), (0, 3), (1, 2), (0, 1), (3, 0), (2, 1)]
    tw, rw = [7, 11, 1, 1], [71, 54, 75, 10, 71, 75, 10]
    got = hb.heta_meta_partition(tw, [s for s, _ in pairs], [t for _, t in pairs], rw, 0, 2, 2)
    _same(got, omp.meta_partition(tw, pairs, rw, 0, 2, 2))
    assert got["sub_rel"] == [0, 1, 5] and sum(got["rel_mask"][got["sub_part"][1]]) == 3


def test_root_without_in_relations_and_errors():
    got = hb.heta_meta_partition([5, 6], [0], [1], [9], root=0, k=2, p=3)
    _same(got, omp.meta_partition([5, 6], [(0, 1)], [9], 0, 2, 3))
    assert got["sub_rel"] == [] and got["replica_of"] == [-1, -1, -1] and got["type_mask"] == [[0, 0]] * 3
    for bad in (dict(root=2), dict(root=-1), dict(k=0), dict(p=0)):
        args = dict(root=0, k=1, p=1)
        args.update(bad)
        with pytest.raises(hb.HetaError) as e:
            hb.heta_meta_partition([5, 6], [0], [1], [9], **args)
        assert e.value.status == hb.HETA_ERR_INVALID_ARG
    with pytest.raises(hb.HetaError):
        hb.heta_meta_partition([5, 6], [2], [1], [9], 0, 1, 1)            # source type out of range
    with pytest.raises(hb.HetaError):
        hb.heta_meta_partition([5, -6], [0], [1], [9], 0, 1, 1)           # negative weight
    with pytest.raises(hb.HetaError):
        hb.heta_meta_partition([5, 6], [0], [1], [9], 0, 1, 1, metapaths=[[0]])   # relation 0 does not end in the root
    with pytest.raises(hb.HetaError):
        hb.heta_meta_partition([5, 6], [0], [1], [9], 1, 1, 1, metapaths=[[4]])   # no such relation
    # a metatree that would not fit is refused, not built: 12 self-loops, 7 levels = 12^7 walks
    with pytest.raises(hb.HetaError) as e:
        hb.heta_meta_partition([1], [0] * 12, [0] * 12, [1] * 12, 0, 7, 2)
    assert e.value.status == hb.HETA_ERR_UNSUPPORTED
