"""GPU parity of the fused inference forward (aggregation + projection + cross-relation sum in one
kernel) against the oracle's forward, at the layer tolerances (1e-4 fp32, 2e-2 bf16 storage), and
against the unfused path of the library itself."""
import numpy as np
import pytest
import torch

import oracle
import paper_2408_09697_amd as heta
from gen import rng, workloads
from gen.graphs import HetGraph, NodeType, power_law_relation, uniform_relation
from tests.harness import assert_rows_close, dev_table, make_layer

pytestmark = pytest.mark.gpu
TOL = {"f32": 1e-4, "bf16": 2e-2}


def _check(p, relu=False):
    p.relu = relu
    layer = make_layer(p)
    H = layer.forward_inference()
    torch.cuda.synchronize()
    ref = oracle.layer_forward(p)
    assert set(H) == set(ref.H)
    for t, h in ref.H.items():
        assert_rows_close(H[t].float().cpu().numpy(), h, TOL[p.storage], f"H[{t}]")
    layer.g.destroy()


@pytest.mark.parametrize("storage", ["f32", "bf16"])
@pytest.mark.parametrize("relu", [False, True])
def test_fused_forward_config3_scaled(storage, relu):
    _check(workloads.config3(storage, scale=0.02), relu)


def test_fused_forward_config1_with_the_fixed_per_type_map():
    _check(workloads.config1())


@pytest.mark.parametrize("storage", ["f32", "bf16"])
@pytest.mark.parametrize("op", ["mean", "sum"])
@pytest.mark.parametrize("d_in,d_out", [(128, 256), (16, 64), (136, 200), (264, 96), (8, 8)])
def test_fused_forward_shapes_hubs_and_ragged_tiles(storage, op, d_in, d_out):
    """Two relations into one type: a skewed one with hub rows (>= 512 edges, the precomputed-row path)
    and a uniform one; 1,000 destinations = 15 full tiles and a ragged one; chunked and ragged widths."""
    wl = f"tests/fused/{d_in}/{d_out}"
    nts = [NodeType("s", 700, d_in, False), NodeType("t", 1000, d_in, False)]
    G = HetGraph(nts)
    G.relations.append(power_law_relation("skew", 0, 1, 700, 1000, 30000, 1.5, wl))
    G.relations.append(uniform_relation("uni", 1, 1, 1000, 1000, 5000, wl))
    assert np.diff(G.relations[0].rowptr).max() >= 512
    tabs = [rng.normal_table(t.num_nodes, d_in, wl, f"t/{t.name}") for t in nts]
    W = [workloads.glorot(d_in, d_out, wl, f"W/{r.name}") for r in G.relations]
    if storage == "bf16":
        tabs = [rng.round_to_bf16(x) for x in tabs]
        W = [rng.round_to_bf16(x) for x in W]
    p = workloads.LayerProblem("fused", G, op, storage, tabs, W, d_out, {})
    _check(p, relu=True)


def test_fused_forward_with_local_to_global_maps():
    """Sources read through src_gid from tables that hold more rows, in another order."""
    p = workloads.config3("f32", scale=0.02)
    g = rng.stream("tests", "fused/gid")
    p.src_gid = []
    for t, tab in enumerate(p.tables):
        n = tab.shape[0]
        where = g.permutation(n + 37)[:n].astype(np.int64)
        big = np.zeros((n + 37, tab.shape[1]), dtype=np.float32)
        big[where] = tab
        p.tables[t] = big
        p.src_gid.append(where)
    _check(p, relu=True)


def test_fused_forward_on_a_sampled_block():
    mb = workloads.config2(scale=0.02)
    _check(mb.layer_problem(0), relu=True)


def test_fused_forward_refuses_what_it_does_not_take():
    p = workloads.config4(scale=0.002)   # widths 7, 300, 789: rows that are not multiples of 16 bytes
    layer = make_layer(p, project_first=False)
    with pytest.raises(heta.HetaError) as e:
        layer.forward_inference()
    assert e.value.status == heta.HETA_ERR_UNSUPPORTED
    layer.g.destroy()
