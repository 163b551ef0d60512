"""Sampled 2-layer mini-batch models (configs 2 and 5) against the oracle, every layer's
embeddings, every weight gradient and every input / embedding gradient."""
import numpy as np
import pytest
import torch

from gen import rng, workloads
from tests.harness import compare_minibatch, dev_table, oracle_minibatch, run_minibatch_on_gpu

pytestmark = pytest.mark.gpu


def check_blocks(mb):
    """Structure every sampled model must have: layer l's destination sets are layer l+1's source sets."""
    T = mb.blocks[0].n_base_types
    for a, b in zip(mb.blocks[:-1], mb.blocks[1:]):
        for k in range(T):
            da = a.dst_gid[T + k]
            sb = b.src_gid[k]
            assert (da is None and sb.size == 0) or np.array_equal(da, sb)
    last = mb.blocks[-1]
    assert last.graph.ntypes[T + mb.seed_type].num_nodes == mb.G.shape[0]


@pytest.mark.parametrize("scale", [0.05, 1.0])
def test_config2_two_layer_minibatch(scale):
    mb = workloads.config2(scale)
    check_blocks(mb)
    tables = [dev_table(t, "f32", 4) for t in mb.tables]
    ref_fwd, ref_bwd, guards = oracle_minibatch(mb, 1e-4)
    layers, grads, graphs = run_minibatch_on_gpu(mb, tables, guards)
    compare_minibatch(mb, layers, grads, ref_fwd, ref_bwd, 1e-4)
    # the relation into a type outside the frontier is a no-op: it produced no output at all
    T = mb.blocks[0].n_base_types
    assert (T + 2) not in layers[0].H          # institution is no destination of the outer block
    for g in graphs:
        g.destroy()


def _device_tables(mb):
    tabs = []
    for t, nt in enumerate(mb.base.ntypes):
        buf = torch.empty((nt.num_nodes, nt.feat_dim), dtype=torch.bfloat16, device="cuda")
        rng.hashed_table_device(mb.table_keys[t], nt.num_nodes, nt.feat_dim, mb.table_kinds[t], buf)
        tabs.append(buf)
    return tabs


@pytest.mark.parametrize("scale", [0.01, 1.0])
def test_config5_two_layer_minibatch_bf16(scale):
    """768 -> 1024 -> 1024 on blocks sampled from the MAG240M-shaped partition; at scale 1 the
    tables (69 GB) are filled on the device and the host regenerates only the sampled rows."""
    mb = workloads.config5(scale)
    check_blocks(mb)
    tables = _device_tables(mb)
    # the device fill and the host replay agree bit for bit on the rows the batch reads
    for t in range(len(mb.base.ntypes)):
        ids = mb.blocks[0].src_gid[t][:2000]
        if ids.size:
            got = tables[t][torch.from_numpy(ids).cuda()].float().cpu().numpy()
            assert np.array_equal(got, mb.table_rows(t, ids))
    ref_fwd, ref_bwd, guards = oracle_minibatch(mb, 2e-2)
    layers, grads, graphs = run_minibatch_on_gpu(mb, tables, guards)
    compare_minibatch(mb, layers, grads, ref_fwd, ref_bwd, 2e-2)
    for g in graphs:
        g.destroy()
