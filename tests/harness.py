"""Shared helpers of the GPU parity tests: upload a gen.LayerProblem, run it through the
C-ABI binding, and compare with the oracle's fp64 results row by row."""
from __future__ import annotations

from typing import Dict, Optional

import numpy as np
import torch

import paper_2408_09697_amd as heta
from gen import rng  # noqa: F401
from paper_2408_09697_amd.problems import dev_table, make_graph, make_layer  # noqa: F401  (re-exported to the tests)


def run_layer_on_gpu(p, mode: str = "fused", project_first=None) -> Dict[str, dict]:
    """mode: "fused" (one projection per destination type), "per_relation" (one projection per
    relation accumulating with beta = 1) or "unfused" (explicit partials + cross-relation reduce)."""
    layer = make_layer(p, project_first=project_first)
    H = {"fused": layer.forward, "per_relation": layer.forward_per_relation, "unfused": layer.forward_unfused}[mode]()
    G = {t: torch.from_numpy(np.ascontiguousarray(g, dtype=np.float32)).cuda() for t, g in p.G.items()}
    dW, dH0, dT = layer.backward(G, per_relation=(mode != "fused"))
    torch.cuda.synchronize()
    f = lambda x: x.float().cpu().numpy()
    out = {"H": {t: f(h) for t, h in H.items()}, "M": {r: f(m) for r, m in layer.M.items() if r not in layer._pf_active},
           "dW": {r: f(w) for r, w in dW.items()}, "dH0": {s: f(x) for s, x in dH0.items()},
           "dT": {s: f(x) for s, x in dT.items()}}
    layer.g.destroy()
    return out


def row_err(got: np.ndarray, ref: np.ndarray) -> float:
    """max over rows i of max_j |got_ij - ref_ij| / max(1, max_j |ref_ij|)."""
    if ref.size == 0:
        return 0.0
    diff = np.abs(got.astype(np.float64) - ref).max(axis=1)
    scale = np.maximum(1.0, np.abs(ref).max(axis=1))
    return float((diff / scale).max())


def assert_rows_close(got, ref, tol, what=""):
    assert got.shape == ref.shape, (what, got.shape, ref.shape)
    assert np.isfinite(got).all(), f"{what}: non-finite values"
    e = row_err(got, ref)
    assert e <= tol, f"{what}: scaled row error {e:.3e} > {tol:.1e}"


def compare_layer(p, got, ref_f, ref_b, tol: float, tol_m: Optional[float] = None, observed_max: Optional[float] = None):
    """Forward embeddings, saved aggregations and all three gradient families against the oracle.
    Returns the largest observed scaled row error per family and prints it; with `observed_max` it must
    also stay below that (a regression guard well inside the contractual tolerance `tol`)."""
    tol_m = tol if tol_m is None else tol_m
    dW, dH0, dT = ref_b
    worst: Dict[str, float] = {}

    def check(g, r, t, what, family):
        assert_rows_close(g, r, t, what)
        worst[family] = max(worst.get(family, 0.0), row_err(g, r))

    assert set(got["H"]) == set(ref_f.H)
    for t, h in ref_f.H.items():
        check(got["H"][t], h, tol, f"H[{t}]", "H")
    for r, m in ref_f.M.items():
        if r in got["M"]:  # relations that were projected first have no M_r
            check(got["M"][r], m, tol_m, f"M[{r}]", "M")
    for r, w in dW.items():
        check(got["dW"][r], w, tol, f"dW[{r}]", "dW")
    assert set(got["dH0"]) == set(dH0)
    for s, x in dH0.items():
        check(got["dH0"][s], x, tol, f"dH0[{s}]", "dH0")
    for s, x in dT.items():
        check(got["dT"][s], x, tol, f"dtable[{s}]", "dtable")
    print(f"\n[observed] {p.name} {getattr(p, 'storage', '')}: " + " ".join(f"{k}={v:.2e}" for k, v in worst.items()))
    if observed_max is not None:
        assert max(worst.values()) <= observed_max, f"observed error {worst} above the guard {observed_max:.1e}"
    return worst


# ---- oracle values for sampled rows of a full-size problem ----------------------------------------

def oracle_forward_rows(p, t: int, rows: np.ndarray):
    """H_t[rows] (fp64) and the per-relation M_r[rows]: the oracle run on the sub-edge-lists whose
    destination is one of `rows` (degrees of those rows are complete, so means are unchanged)."""
    import oracle
    rows = np.asarray(rows, dtype=np.int64)
    remap = -np.ones(p.graph.ntypes[t].num_nodes, dtype=np.int64)
    remap[rows] = np.arange(rows.size)
    Z, Ms = [], {}
    for i in p.graph.rels_into(t):
        r = p.graph.relations[i]
        src, dst = r.edge_list()
        keep = remap[dst] >= 0
        gid = None if p.src_gid is None else p.src_gid[r.src_type]
        M = oracle.aggregate_fwd(src[keep], remap[dst[keep]].astype(np.int32), rows.size, p.tables[r.src_type],
                                 p.op, gid=gid)
        Ms[i] = M
        Z.append(oracle.project(M, p.W[i]))
    H = oracle.cross_rel_sum(Z, relu=p.relu)
    return H, Ms


def oracle_input_grad_rows(p, s: int, rows: np.ndarray, G):
    """dH0_s[rows] (fp64): for every relation out of type s, the edges leaving one of `rows`, the
    gradient rows dM_r = G_t W_r^T of their destinations, scattered with c_e = 1 or 1/deg_r(v_e)."""
    import oracle
    rows = np.asarray(rows, dtype=np.int64)
    remap = -np.ones(p.graph.ntypes[s].num_nodes, dtype=np.int64)
    remap[rows] = np.arange(rows.size)
    out = None
    for i in p.graph.rels_from(s):
        r = p.graph.relations[i]
        src, dst = r.edge_list()
        n_t = p.graph.ntypes[r.dst_type].num_nodes
        keep = remap[src] >= 0
        dsts, inv = np.unique(dst[keep], return_inverse=True)
        dM = np.asarray(G[r.dst_type][dsts], dtype=np.float64) @ np.asarray(p.W[i], dtype=np.float64).T
        if p.op == "mean":
            deg = oracle.in_degree(src, dst, n_t)
            dM = dM / deg[dsts][:, None]
        part = oracle.aggregate_bwd(remap[src[keep]].astype(np.int32), inv.astype(np.int32), rows.size, dsts.size,
                                    dM, "sum")
        out = part if out is None else out + part
    return out


# ---- sampled mini-batch models (several layers over blocks) -------------------------------------
# A ReLU between two layers makes the backward pass discontinuous in the forward values: an
# embedding whose magnitude is below the forward tolerance may legitimately come out on either
# side of zero, and a single flipped decision changes whole gradient entries.  As with finite
# differences, the check stays away from the kink: the upstream gradient handed to an inner
# layer is zeroed (on both sides, from the ORACLE's embeddings only) wherever the oracle's
# pre-activation magnitude is within the forward tolerance of zero.

def kink_guard(H_ref: np.ndarray, tol: float) -> np.ndarray:
    """True where the sign of the embedding is decidable at forward tolerance `tol`."""
    if H_ref.shape[0] == 0:
        return np.zeros(H_ref.shape, dtype=bool)
    scale = np.maximum(1.0, np.abs(H_ref).max(axis=1, keepdims=True))
    return np.abs(H_ref) > tol * scale


def oracle_minibatch(mb, tol: float):
    """Forward and backward of the whole k-layer model with the oracle.  Returns per layer the
    LayerResult, (dW, dH0), and the kink guards per layer and destination type."""
    import oracle
    fwd, probs = [], []
    prev = None
    for l in range(len(mb.blocks)):
        p = mb.layer_problem(l, prev)
        r = oracle.layer_forward(p)
        prev = r.H
        fwd.append(r)
        probs.append(p)
    guards = [{t: kink_guard(h, tol) for t, h in f.H.items()} for f in fwd]
    out = []
    T = mb.blocks[0].n_base_types
    G = None
    for l in reversed(range(len(mb.blocks))):
        p = probs[l]
        if G is None:
            G = dict(p.G)
        for t, nt in enumerate(p.graph.ntypes):      # destination roles without an upstream gradient
            if t >= T and t not in G:
                G[t] = np.zeros((nt.num_nodes, mb.d_hidden))
        dW, dH0, _ = oracle.layer_backward(p, fwd[l], G)
        out.append((dW, dH0))
        if l > 0:                                    # gradient of layer l-1's outputs, away from the kink
            G = {T + s: g * guards[l - 1][T + s] for s, g in dH0.items() if (T + s) in guards[l - 1]}
    out.reverse()
    return fwd, out, guards


def run_minibatch_on_gpu(mb, tables_dev, guards):
    """tables_dev: device tables per base node type (full size); guards: from oracle_minibatch.
    Returns the layers (holding H, M), per layer (dW, dH0), and the graph handles."""
    T = mb.blocks[0].n_base_types
    op = heta.HETA_MEAN if mb.op == "mean" else heta.HETA_SUM
    pad = 8 if mb.storage == "bf16" else 4
    layers, graphs = [], []
    prev_H = None
    for l, b in enumerate(mb.blocks):
        nts = [(t.num_nodes, t.feat_dim, int(t.learnable)) for t in b.graph.ntypes]
        hg = heta.heta_graph_create(nts, [(r.src_type, r.dst_type, r.rowptr, r.col) for r in b.graph.relations])
        graphs.append(hg)
        rels = [i for i, r in enumerate(b.graph.relations) if b.graph.ntypes[r.dst_type].num_nodes > 0]
        W = [dev_table(w, mb.storage, pad) for w in mb.W[l]]
        if l == 0:
            tabs = list(tables_dev) + [None] * T
            gid = [torch.from_numpy(g).cuda() for g in b.src_gid[:T]] + [None] * T
        else:
            tabs = [prev_H.get(T + k) for k in range(T)] + [None] * T
            gid = None
        for i in rels:                                # a source type nobody sampled still needs a (dummy) table
            s = b.graph.relations[i].src_type
            if tabs[s] is None:
                assert b.graph.ntypes[s].num_nodes == 0
                tabs[s] = torch.zeros((1, mb.W[l][i].shape[0]), dtype=torch.float32, device="cuda")
        layer = heta.RafLayer(hg, op, tabs, W, mb.d_hidden, src_gid=gid, relu=(l < len(mb.blocks) - 1), rels=rels)
        prev_H = layer.forward()
        layers.append(layer)
    G = {T + mb.seed_type: torch.from_numpy(mb.G).cuda()}
    grads = []
    for l in reversed(range(len(layers))):
        layer = layers[l]
        dW, dH0, _ = layer.backward(G)
        grads.append((dW, dH0))
        if l > 0:
            G = {}
            for s, g in dH0.items():
                if (T + s) in layers[l - 1].H:
                    keep = torch.from_numpy(guards[l - 1][T + s]).cuda()
                    G[T + s] = g * keep
            for t, h in layers[l - 1].H.items():      # destination types of the layer below that got no gradient
                if t not in G:
                    G[t] = torch.zeros_like(h)
    grads.reverse()
    torch.cuda.synchronize()
    return layers, grads, graphs


def compare_minibatch(mb, layers, grads, ref_fwd, ref_bwd, tol):
    for l, layer in enumerate(layers):
        for t, h in ref_fwd[l].H.items():
            if h.shape[0] == 0:
                continue
            assert_rows_close(layer.H[t].cpu().numpy(), h, tol, f"layer {l + 1} H[{t}]")
        dW_ref, dH0_ref = ref_bwd[l]
        dW, dH0 = grads[l]
        for r in layer.rels:
            assert_rows_close(dW[r].cpu().numpy(), dW_ref[r], tol, f"layer {l + 1} dW[{r}]")
        for s, g in dH0.items():
            if g.shape[0] == 0:
                continue
            assert_rows_close(g.cpu().numpy(), dH0_ref[s], tol, f"layer {l + 1} dH0[{s}]")
