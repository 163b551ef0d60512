"""GPU parity of the device neighbour sampler against oracle/sampler.py: index work, so every array is
compared bit for bit (block row offsets, sampled global source ids in order, ascending unique source
sets, local ids), and the blocks the sequencer builds are checked against the oracle's blocks and then
run through a layer."""
import numpy as np
import pytest
import torch

import paper_2408_09697_amd as heta
from gen import rng, workloads
from gen.graphs import HetGraph, NodeType, power_law_relation, uniform_relation
from oracle import sampler as osampler
from tests.harness import make_graph

pytestmark = pytest.mark.gpu


def _graph(kind):
    wl = f"tests/sampler/{kind}"
    nts = [NodeType("s", 3000, 4, False), NodeType("t", 2500, 4, False)]
    G = HetGraph(nts)
    if kind == "uniform":
        G.relations.append(uniform_relation("r", 0, 1, 3000, 2500, 20000, wl))
    else:
        G.relations.append(power_law_relation("r", 0, 1, 3000, 2500, 80000, 1.6, wl))
    return G


@pytest.mark.parametrize("kind", ["uniform", "skew"])
@pytest.mark.parametrize("fanout", [1, 5, 25, 64])
def test_sample_neighbors_bit_exact(kind, fanout):
    G = _graph(kind)
    r = G.relations[0]
    hg = heta.heta_graph_create([(3000, 4, 0), (2500, 4, 0)], [(0, 1, r.rowptr, r.col)])
    g = rng.stream("tests", f"sampler/{kind}/{fanout}")
    deg = np.diff(r.rowptr)
    ids = np.concatenate([g.permutation(2500)[:700], [int(np.argmax(deg))] * 2, np.flatnonzero(deg == 0)[:3]]).astype(np.int64)
    for seed in (0, 0xDEADBEEFCAFEF00D):
        rowptr, src = heta.heta_sample_neighbors(hg, 0, torch.from_numpy(ids).cuda(), fanout, seed)
        ref_ptr, ref_src = osampler.sample_neighbors(r.rowptr, r.col, ids, fanout, seed)
        assert np.array_equal(rowptr.cpu().numpy(), ref_ptr)
        assert np.array_equal(src.cpu().numpy(), ref_src)
    # empty frontier, and ids out of range are refused
    rowptr, src = heta.heta_sample_neighbors(hg, 0, torch.zeros(0, dtype=torch.int64, device="cuda"), fanout, 1)
    assert rowptr.cpu().tolist() == [0] and src.numel() == 0
    with pytest.raises(heta.HetaError, match="outside"):
        heta.heta_sample_neighbors(hg, 0, torch.tensor([3, 2500], dtype=torch.int64, device="cuda"), fanout, 1)
    with pytest.raises(heta.HetaError, match="fanout"):
        heta.heta_sample_neighbors(hg, 0, torch.tensor([3], dtype=torch.int64, device="cuda"), 65, 1)
    hg.destroy()


def test_unique_relabel_bit_exact():
    g = rng.stream("tests", "sampler/unique")
    lists = [g.integers(0, 50000, 30000), np.zeros(0, dtype=np.int64), g.integers(0, 50000, 7), g.integers(49990, 50000, 5000)]
    uniq, local = heta.heta_unique_relabel([torch.from_numpy(l.astype(np.int64)).cuda() for l in lists], 50000)
    ref_u, ref_l = osampler.unique_relabel(lists)
    assert np.array_equal(uniq.cpu().numpy(), ref_u)
    for a, b in zip(local, ref_l):
        assert np.array_equal(a.cpu().numpy(), b)
    uniq, local = heta.heta_unique_relabel([torch.zeros(0, dtype=torch.int64, device="cuda")], 10)
    assert uniq.numel() == 0 and local[0].numel() == 0
    with pytest.raises(heta.HetaError, match="outside"):
        heta.heta_unique_relabel([torch.tensor([1, 10], dtype=torch.int64, device="cuda")], 10)


def test_sampled_blocks_match_the_oracle_and_run_a_layer():
    base = workloads.academic_graph(scale=0.02, workload="tests/sampler/blocks")
    T = len(base.ntypes)
    rels = [(r.src_type, r.dst_type, r.rowptr, r.col) for r in base.relations]
    hg = heta.heta_graph_create([(t.num_nodes, t.feat_dim, int(t.learnable)) for t in base.ntypes], rels)
    seeds = np.sort(rng.stream("tests", "sampler/seeds").choice(base.ntypes[0].num_nodes, 256, replace=False)).astype(np.int64)
    fanouts, seed = [25, 20], 20240809
    blocks = heta.sampler.sample_blocks(hg, 0, torch.from_numpy(seeds).cuda(), fanouts, seed)
    ref = osampler.sample_blocks(T, rels, 0, seeds, fanouts, seed)
    assert len(blocks) == len(ref) == 2
    for b, rb in zip(blocks, ref):
        for t in range(T):
            assert np.array_equal(b.src_ids[t].cpu().numpy(), rb["src_ids"][t])
            if rb["dst_ids"][t] is None:
                assert b.dst_ids[t] is None
            else:
                assert np.array_equal(b.dst_ids[t].cpu().numpy(), rb["dst_ids"][t])
        for i, (ptr, loc) in enumerate(rb["rels"]):
            assert np.array_equal(b.rowptr[i].cpu().numpy(), ptr)
            assert np.array_equal(b.col[i].cpu().numpy(), loc)
    # the outermost block drives one aggregation through its local -> global maps: sums of a table of
    # ones count the sampled in-edges of every destination
    b = blocks[0]
    for i, (s, t, _) in enumerate(hg.rels):
        n_dst = b.graph.n_dst(i)
        if n_dst == 0:
            continue
        table = torch.ones((hg.ntypes[s][0], 8), dtype=torch.float32, device="cuda")
        out = torch.empty((n_dst, 8), dtype=torch.float32, device="cuda")
        heta.heta_rel_aggregate_fwd(b.graph, i, heta.HETA_SUM, table, out, src_gid=b.src_ids[s])
        want = np.diff(ref[0]["rels"][i][0]).astype(np.float32)
        assert np.array_equal(out.cpu().numpy(), np.repeat(want[:, None], 8, axis=1))
    for b in blocks:
        b.graph.destroy()
    hg.destroy()


def test_batched_sampling_and_relabelling_match_the_oracle():
    """Several relations (and several id sets) in one call: item by item the results of the oracle, with an
    empty frontier, a repeated relation and different seeds in the batch; an id out of range in any item
    fails the call and names the relation."""
    wl = "tests/sampler/batch"
    nts = [NodeType("a", 3000, 4, False), NodeType("b", 2500, 4, False), NodeType("c", 40, 4, False)]
    G = HetGraph(nts)
    G.relations.append(uniform_relation("ab", 0, 1, 3000, 2500, 20000, wl))
    G.relations.append(power_law_relation("ba", 1, 0, 2500, 3000, 60000, 1.7, wl))
    G.relations.append(power_law_relation("ca", 2, 0, 40, 3000, 9000, 1.5, wl))
    hg = make_graph(type("P", (), {"graph": G})())
    g = rng.stream("tests", "sampler/batch")
    fr = [g.permutation(nts[t].num_nodes)[:k].astype(np.int64) for t, k in ((1, 600), (0, 900), (0, 0), (1, 37))]
    rels, seeds = [0, 1, 2, 0], [11, 0xFEEDFACE12345678, 13, 14]
    for fanout in (3, 20):
        got = heta.heta_sample_neighbors_batch(hg, rels, [torch.from_numpy(f).cuda() for f in fr], fanout, seeds)
        srcs = []
        for (rp, src), i, f, sd in zip(got, rels, fr, seeds):
            r = G.relations[i]
            ref_ptr, ref_src = osampler.sample_neighbors(r.rowptr, r.col, f, fanout, sd)
            assert np.array_equal(rp.cpu().numpy(), ref_ptr) and np.array_equal(src.cpu().numpy(), ref_src)
            srcs.append(src)
        # source sets per source type: relations 0 and 3 leave type a, 1 leaves b, 2 leaves c; plus an empty group
        groups = [[srcs[0], srcs[3]], [srcs[1]], [srcs[2]], []]
        out = heta.heta_unique_relabel_batch(groups, [3000, 2500, 40, 10])
        for grp, (uniq, local) in zip(groups, out):
            ref_u, ref_l = osampler.unique_relabel([x.cpu().numpy() for x in grp])
            assert np.array_equal(uniq.cpu().numpy(), ref_u)
            assert len(local) == len(ref_l)
            for a, b in zip(local, ref_l):
                assert np.array_equal(a.cpu().numpy(), b)
    bad = [torch.from_numpy(f).cuda() for f in fr]
    bad[1] = torch.tensor([5, 3000], dtype=torch.int64, device="cuda")      # relation 1's destinations are type a: 3000 is out
    with pytest.raises(heta.HetaError, match="relation 1"):
        heta.heta_sample_neighbors_batch(hg, rels, bad, 3, seeds)
    with pytest.raises(heta.HetaError, match="outside"):
        heta.heta_unique_relabel_batch([[srcs[0]], [srcs[1]]], [3000, 5])
    assert heta.heta_sample_neighbors_batch(hg, [], [], 3, []) == [] and heta.heta_unique_relabel_batch([], []) == []
    hg.destroy()


def test_batches_beyond_the_fused_limits_take_the_per_item_path():
    """More than 32 items in one sampling call, and id sets whose set index does not fit above the ids in a
    32-bit key (three sets with 2^31 possible ids each): same results, item by item."""
    wl = "tests/sampler/batch"
    nts = [NodeType("a", 3000, 4, False), NodeType("b", 2500, 4, False)]
    G = HetGraph(nts)
    G.relations.append(uniform_relation("ab", 0, 1, 3000, 2500, 20000, wl))
    G.relations.append(power_law_relation("ba", 1, 0, 2500, 3000, 60000, 1.7, wl))
    hg = make_graph(type("P", (), {"graph": G})())
    g = rng.stream("tests", "sampler/fallback")
    rels = [i % 2 for i in range(35)]
    fr = [g.permutation(nts[1 - r].num_nodes)[:(0 if i == 7 else 40 + 3 * i)].astype(np.int64) for i, r in enumerate(rels)]
    seeds = [1000 + i for i in range(35)]
    got = heta.heta_sample_neighbors_batch(hg, rels, [torch.from_numpy(f).cuda() for f in fr], 6, seeds)
    for (rp, src), i, f, sd in zip(got, rels, fr, seeds):
        ref_ptr, ref_src = osampler.sample_neighbors(G.relations[i].rowptr, G.relations[i].col, f, 6, sd)
        assert np.array_equal(rp.cpu().numpy(), ref_ptr) and np.array_equal(src.cpu().numpy(), ref_src)
    big = [np.array([2**31 - 1, 5, 5, 2**30, 0], dtype=np.int64), np.array([7, 7, 7], dtype=np.int64), np.array([2**31 - 2], dtype=np.int64)]
    out = heta.heta_unique_relabel_batch([[torch.from_numpy(x).cuda()] for x in big], [2**31] * 3)
    for x, (uniq, local) in zip(big, out):
        ref_u, ref_l = osampler.unique_relabel([x])
        assert np.array_equal(uniq.cpu().numpy(), ref_u) and np.array_equal(local[0].cpu().numpy(), ref_l[0])
    hg.destroy()
