"""Pins of the CPU oracle against things other than itself (CPU only).

Each test compares the oracle with what the paper and the mathematics fix: a dense
count-matrix formulation written with numpy matmul (Eq. 1 with AGG_r = GCN, AGG_all = sum),
closed forms on regular graphs, linearity, the adjoint identity, finite differences,
Proposition 1 (any split of the relation set gives the same embedding), and the buffer
shape implied by the communication example of Section 4.
"""
import math
import os

import numpy as np
import pytest

import oracle
from gen import rng, workloads
from gen.graphs import HetGraph, NodeType, Relation, csr_from_edges

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ---- a tiny random heterogeneous problem with every awkward feature ---------------------------

def tiny_problem(seed, op, relu=False, with_gid=False):
    g = np.random.default_rng(seed)
    n = [int(g.integers(3, 9)), int(g.integers(3, 9)), int(g.integers(2, 6))]
    d = [5, 3, 4]
    d_out = 6
    nts = [NodeType("a", n[0], d[0], False), NodeType("b", n[1], d[1], False), NodeType("c", n[2], d[2], True)]
    G = HetGraph(nts)
    for nm, s, t, e in [("aa", 0, 0, 11), ("ba", 1, 0, 7), ("ca", 2, 0, 9), ("ab", 0, 1, 13), ("cb", 2, 1, 0)]:
        src = g.integers(0, n[s], size=e).astype(np.int32)
        # leave the last destination row without edges: a zero-degree row in every relation
        dst = g.integers(0, max(1, n[t] - 1), size=e).astype(np.int32)
        rowptr, col = csr_from_edges(src, dst, n[t])
        G.relations.append(Relation(nm, s, t, rowptr, col))
    src_gid = None
    tables = []
    for t in range(3):
        rows = n[t] + 4 if with_gid else n[t]
        tables.append(g.standard_normal((rows, d[t])).astype(np.float32))
    if with_gid:
        src_gid = [g.permutation(n[t] + 4)[: n[t]].astype(np.int64) for t in range(3)]
    W = [g.standard_normal((d[r.src_type], d_out)).astype(np.float32) for r in G.relations]
    Gup = {0: g.standard_normal((n[0], d_out)).astype(np.float32),
           1: g.standard_normal((n[1], d_out)).astype(np.float32)}
    return workloads.LayerProblem("tiny", G, op, "f32", tables, W, d_out, Gup, src_gid=src_gid, relu=relu)


def dense_layer(p):
    """Textbook dense formulation: count matrix A_r[v,u], M = D^-1 A X, Z = M W, H = sum Z."""
    g = p.graph
    H, M, Acs = {}, {}, {}
    for i, r in enumerate(g.relations):
        n_s, n_t = g.ntypes[r.src_type].num_nodes, g.ntypes[r.dst_type].num_nodes
        A = np.zeros((n_t, n_s))
        src, dst = r.edge_list()
        for u, v in zip(src.tolist(), dst.tolist()):
            A[v, u] += 1.0
        if p.op == "mean":
            deg = A.sum(axis=1)
            A = A / np.where(deg > 0, deg, 1.0)[:, None]
        X = p.tables[r.src_type].astype(np.float64)
        if p.src_gid is not None:
            X = X[p.src_gid[r.src_type]]
        if p.pre_proj is not None:
            X = X @ p.pre_proj[r.src_type].astype(np.float64)
        Acs[i] = A
        M[i] = A @ X
        H[r.dst_type] = H.get(r.dst_type, 0.0) + M[i] @ p.W[i].astype(np.float64)
    pre = {t: h.copy() for t, h in H.items()}
    if p.relu:
        H = {t: np.maximum(h, 0.0) for t, h in H.items()}
    return Acs, M, H, pre


def dense_backward(p, Acs, M, pre):
    g = p.graph
    dW, dH0 = {}, {}
    for i, r in enumerate(g.relations):
        dZ = p.G[r.dst_type].astype(np.float64)
        if p.relu:
            dZ = dZ * (pre[r.dst_type] > 0)
        dW[i] = M[i].T @ dZ
        dM = dZ @ p.W[i].astype(np.float64).T
        dH0[r.src_type] = dH0.get(r.src_type, 0.0) + Acs[i].T @ dM
    return dW, dH0


@pytest.mark.parametrize("op", ["mean", "sum"])
@pytest.mark.parametrize("seed", [0, 1, 2, 3])
@pytest.mark.parametrize("relu", [False, True])
@pytest.mark.parametrize("with_gid", [False, True])
def test_layer_matches_dense_brute_force(seed, op, relu, with_gid):
    p = tiny_problem(seed, op, relu, with_gid)
    Acs, M, H, pre = dense_layer(p)
    res = oracle.layer_forward(p)
    for i in M:
        np.testing.assert_allclose(res.M[i], M[i], rtol=1e-13, atol=1e-13)
    assert set(res.H) == set(H)
    for t in H:
        np.testing.assert_allclose(res.H[t], H[t], rtol=1e-12, atol=1e-12)
    dW, dH0 = dense_backward(p, Acs, M, pre)
    odW, odH0, odT = oracle.layer_backward(p, res, p.G)
    for i in dW:
        np.testing.assert_allclose(odW[i], dW[i], rtol=1e-12, atol=1e-12)
    assert set(odH0) == set(dH0)
    for t in dH0:
        np.testing.assert_allclose(odH0[t], dH0[t], rtol=1e-12, atol=1e-12)
        np.testing.assert_allclose(odT[t], dH0[t], rtol=1e-12, atol=1e-12)


def test_config1_matches_dense_brute_force():
    p = workloads.config1()
    Acs, M, H, pre = dense_layer(p)
    res = oracle.layer_forward(p)
    for t in H:
        np.testing.assert_allclose(res.H[t], H[t], rtol=1e-11, atol=1e-11)
    dW, dH0 = dense_backward(p, Acs, M, pre)
    odW, odH0, odT = oracle.layer_backward(p, res, p.G)
    for i in dW:
        np.testing.assert_allclose(odW[i], dW[i], rtol=1e-11, atol=1e-11)
    for t in dH0:
        np.testing.assert_allclose(odH0[t], dH0[t], rtol=1e-11, atol=1e-11)
        np.testing.assert_allclose(odT[t], dH0[t] @ p.pre_proj[t].astype(np.float64).T, rtol=1e-11, atol=1e-11)
    # type C has no incoming relation: no output for it, only a gradient
    assert 2 not in res.H and 2 in odH0


# ---- closed forms ------------------------------------------------------------------------------

def test_closed_form_ring_and_star():
    n, d = 12, 3
    X = np.arange(n * d, dtype=np.float32).reshape(n, d)
    # ring: v receives from v-1 and v+1 -> mean is the midpoint, sum is twice it
    src = np.concatenate([(np.arange(n) - 1) % n, (np.arange(n) + 1) % n]).astype(np.int32)
    dst = np.concatenate([np.arange(n), np.arange(n)]).astype(np.int32)
    M = oracle.aggregate_fwd(src, dst, n, X, "mean")
    expect = (X[(np.arange(n) - 1) % n].astype(np.float64) + X[(np.arange(n) + 1) % n]) / 2
    np.testing.assert_array_equal(M, expect)
    np.testing.assert_array_equal(oracle.aggregate_fwd(src, dst, n, X, "sum"), 2 * expect)
    # star: node 0 receives from everybody once, node 1 three times from node 5 (multi-edge)
    src = np.array(list(range(n)) + [5, 5, 5], dtype=np.int32)
    dst = np.array([0] * n + [1, 1, 1], dtype=np.int32)
    S = oracle.aggregate_fwd(src, dst, n, X, "sum")
    np.testing.assert_array_equal(S[0], X.astype(np.float64).sum(0))
    np.testing.assert_array_equal(S[1], 3.0 * X[5])
    np.testing.assert_array_equal(S[2:], 0.0)
    Mn = oracle.aggregate_fwd(src, dst, n, X, "mean")
    np.testing.assert_allclose(Mn[0], X.astype(np.float64).mean(0), rtol=1e-15)
    np.testing.assert_array_equal(Mn[1], X[5])            # mean of three copies of one row
    np.testing.assert_array_equal(oracle.in_degree(src, dst, n), [n, 3] + [0] * (n - 2))


def test_all_ones_gives_degree_and_unit_vectors_count_indices():
    p = workloads.config1()
    r = p.graph.relations[1]  # B->A
    src, dst = r.edge_list()
    n_s, n_t = 1000, 2000
    deg = oracle.in_degree(src, dst, n_t)
    assert deg.sum() == 5000
    ones = np.ones((n_s, 4), dtype=np.float32)
    S = oracle.aggregate_fwd(src, dst, n_t, ones, "sum")
    np.testing.assert_array_equal(S, np.repeat(deg[:, None], 4, axis=1).astype(np.float64))
    d = 16
    E = np.zeros((n_s, d), dtype=np.float32)
    E[np.arange(n_s), np.arange(n_s) % d] = 1.0
    S = oracle.aggregate_fwd(src, dst, n_t, E, "sum")
    cnt = np.zeros((n_t, d))
    np.add.at(cnt, (dst, src % d), 1.0)
    np.testing.assert_array_equal(S, cnt)


def test_zero_degree_and_empty_relation():
    X = np.random.default_rng(0).standard_normal((5, 3)).astype(np.float32)
    e = np.zeros(0, dtype=np.int32)
    for op in ("sum", "mean"):
        M = oracle.aggregate_fwd(e, e, 4, X, op)
        assert M.shape == (4, 3) and not M.any() and np.isfinite(M).all()
        g = oracle.aggregate_bwd(e, e, 5, 4, np.ones((4, 3)), op)
        assert g.shape == (5, 3) and not g.any()
    src = np.array([0, 1], dtype=np.int32)
    dst = np.array([2, 2], dtype=np.int32)
    M = oracle.aggregate_fwd(src, dst, 4, X, "mean")
    assert not M[[0, 1, 3]].any()
    # zero destinations: no output rows
    assert oracle.aggregate_fwd(e, e, 0, X, "mean").shape == (0, 3)


# ---- invariants --------------------------------------------------------------------------------

@pytest.mark.parametrize("op", ["mean", "sum"])
def test_linearity_aggregate_then_project_equals_project_then_aggregate(op):
    p = workloads.config1()
    r = p.graph.relations[3]  # A->B
    src, dst = r.edge_list()
    X = p.tables[0]
    W = np.random.default_rng(1).standard_normal((64, 20))
    lhs = oracle.project(oracle.aggregate_fwd(src, dst, 1000, X, op), W)
    XW = X.astype(np.float64) @ W
    rhs = oracle.aggregate_fwd(src, dst, 1000, XW, op)
    np.testing.assert_allclose(lhs, rhs, rtol=1e-11, atol=1e-11)


@pytest.mark.parametrize("op", ["mean", "sum"])
def test_adjoint_identity(op):
    p = workloads.config1()
    rs = np.random.default_rng(2)
    for i, r in enumerate(p.graph.relations):
        src, dst = r.edge_list()
        n_s, n_t = p.graph.ntypes[r.src_type].num_nodes, p.graph.ntypes[r.dst_type].num_nodes
        X = rs.standard_normal((n_s, 7)).astype(np.float32)
        Gm = rs.standard_normal((n_t, 7))
        lhs = np.vdot(Gm, oracle.aggregate_fwd(src, dst, n_t, X, op))
        rhs = np.vdot(X.astype(np.float64), oracle.aggregate_bwd(src, dst, n_s, n_t, Gm, op))
        assert abs(lhs - rhs) <= 1e-10 * max(1.0, abs(lhs))


def test_backward_of_sum_is_forward_of_transpose():
    p = workloads.config1()
    r = p.graph.relations[1]
    src, dst = r.edge_list()
    Gm = np.random.default_rng(3).standard_normal((2000, 5)).astype(np.float32)
    bwd = oracle.aggregate_bwd(src, dst, 1000, 2000, Gm.astype(np.float64), "sum")
    fwd_T = oracle.aggregate_fwd(dst, src, 1000, Gm, "sum")   # transposed edge list
    np.testing.assert_allclose(bwd, fwd_T, rtol=1e-13, atol=1e-13)


def test_finite_differences_config1():
    """L = <G, H> is linear in each of tables, embeddings and W_r separately (no ReLU), so a
    central difference reproduces the gradient up to rounding."""
    p = workloads.config1()
    res = oracle.layer_forward(p)
    dW, dH0, dT = oracle.layer_backward(p, res, p.G)

    def loss(q):
        out = oracle.layer_forward(q)
        return sum(np.vdot(q.G[t].astype(np.float64), out.H[t]) for t in out.H)

    rs = np.random.default_rng(4)
    eps = 2.0 ** -7
    for t in range(3):
        for _ in range(3):
            i, j = int(rs.integers(p.tables[t].shape[0])), int(rs.integers(p.tables[t].shape[1]))
            old = p.tables[t][i, j]
            p.tables[t][i, j] = old + np.float32(eps)
            up = loss(p)
            p.tables[t][i, j] = old - np.float32(eps)
            dn = loss(p)
            p.tables[t][i, j] = old
            step = float(np.float32(old + np.float32(eps)) - np.float32(old - np.float32(eps)))
            fd = (up - dn) / step
            assert abs(fd - dT[t][i, j]) <= 1e-8 * max(1.0, abs(fd)), (t, i, j, fd, dT[t][i, j])
    for r in range(4):
        for _ in range(3):
            i, j = int(rs.integers(32)), int(rs.integers(32))
            old = p.W[r][i, j]
            p.W[r][i, j] = old + np.float32(eps)
            up = loss(p)
            p.W[r][i, j] = old - np.float32(eps)
            dn = loss(p)
            p.W[r][i, j] = old
            step = float(np.float32(old + np.float32(eps)) - np.float32(old - np.float32(eps)))
            fd = (up - dn) / step
            assert abs(fd - dW[r][i, j]) <= 1e-8 * max(1.0, abs(fd)), (r, i, j, fd, dW[r][i, j])


def test_finite_differences_with_relu_tiny():
    p = tiny_problem(5, "mean", relu=True)
    res = oracle.layer_forward(p)
    dW, dH0, dT = oracle.layer_backward(p, res, p.G)
    # stay away from the kink: every pre-activation must be far from zero compared with the step
    pre = dense_layer(p)[3]
    # (rows without any incoming edge are exactly 0 and no input can move them)
    margin = min(np.abs(h[h != 0.0]).min() for h in pre.values())
    eps = 2.0 ** -20
    assert margin > 100 * eps * 50

    def loss(q):
        out = oracle.layer_forward(q)
        return sum(np.vdot(q.G[t].astype(np.float64), out.H[t]) for t in out.H)

    for t in range(3):
        for i in range(p.tables[t].shape[0]):
            for j in range(p.tables[t].shape[1]):
                old = p.tables[t][i, j]
                hi, lo = np.float32(old + np.float32(eps)), np.float32(old - np.float32(eps))
                p.tables[t][i, j] = hi
                up = loss(p)
                p.tables[t][i, j] = lo
                dn = loss(p)
                p.tables[t][i, j] = old
                fd = (up - dn) / (float(hi) - float(lo))
                assert abs(fd - dT[t][i, j]) <= 1e-6 * max(1.0, abs(fd))


def test_proposition1_any_split_of_relations():
    """Partial aggregations over any partition of the relation set, summed, equal the embedding
    over all relations (Proposition 1); the same holds for the gradients."""
    p = workloads.config1()
    full = oracle.layer_forward(p)
    for split in ([[0], [1], [2], [3]], [[0, 2], [1, 3]], [[3, 1, 0], [2]]):
        parts = [oracle.layer_forward(p, rels=s) for s in split]
        for t in full.H:
            tot = oracle.cross_rel_sum([q.H[t] for q in parts if t in q.H])
            np.testing.assert_allclose(tot, full.H[t], rtol=1e-12, atol=1e-12)
    dW, dH0, _ = oracle.layer_backward(p, full, p.G)
    acc = {}
    for s in [[0, 2], [1, 3]]:
        part = oracle.layer_forward(p, rels=s)
        pdW, pdH0, _ = oracle.layer_backward(p, part, p.G, rels=s)
        for i in s:
            np.testing.assert_allclose(pdW[i], dW[i], rtol=1e-12, atol=1e-12)
        for t, gH in pdH0.items():
            acc[t] = acc.get(t, 0.0) + gH
    for t in dH0:
        np.testing.assert_allclose(acc[t], dH0[t], rtol=1e-12, atol=1e-12)


def test_integer_inputs_are_exact():
    p = workloads.config1(exact=True)
    p.op = "sum"
    res = oracle.layer_forward(p)
    for h in res.H.values():
        assert np.array_equal(h, np.rint(h)) and np.abs(h).max() < 2 ** 24
    Acs, M, H, _ = dense_layer(p)
    for t in H:
        np.testing.assert_array_equal(res.H[t], H[t])


# ---- CSC (stable transpose) -------------------------------------------------------------------

@pytest.mark.parametrize("seed", [0, 1, 2])
def test_csc_is_the_stable_transpose(seed):
    g = np.random.default_rng(seed)
    n_s, n_t, E = 37, 23, 400
    src = g.integers(0, n_s, size=E).astype(np.int32)
    dst = np.sort(g.integers(0, n_t, size=E)).astype(np.int32)
    colptr, row = oracle.csc(src, dst, n_s)
    order = np.lexsort((np.arange(E), src))      # by source, ties by original position
    np.testing.assert_array_equal(row, dst[order])
    np.testing.assert_array_equal(colptr, np.concatenate([[0], np.cumsum(np.bincount(src, minlength=n_s))]))
    # brute force per column
    for u in range(n_s):
        np.testing.assert_array_equal(row[colptr[u]:colptr[u + 1]], dst[src == u])


def test_csc_empty():
    e = np.zeros(0, dtype=np.int32)
    colptr, row = oracle.csc(e, e, 5)
    assert colptr.tolist() == [0] * 6 and row.size == 0


# ---- the one place the paper prints numbers that touch this path -------------------------------

def test_partial_aggregation_buffer_shape_from_communication_example():
    """Section 4 prints 8.0 MB (partials and gradients of 14,568 one-hop nodes plus 1,024 seeds)
    and 0.5 MB (1,024 seeds only) at hidden size 64: both are reproduced by one [n, hidden]
    4-byte buffer forward and one of the same shape backward."""
    vals = {}
    with open(os.path.join(GOLDEN, "comm_example.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                k, v = line.split()
                vals[k] = float(v)
    hidden, seeds, hop1 = int(vals["hidden"]), int(vals["seeds"]), int(vals["one_hop_nodes"])
    fwd_bwd = 2
    assert round((hop1 + seeds) * hidden * 4 * fwd_bwd / 1e6, 1) == vals["raf_megabytes"]
    assert round(seeds * hidden * 4 * fwd_bwd / 2 ** 20, 1) == vals["raf_meta_partitioning_megabytes"]
    # the oracle's partial aggregation has exactly that shape: one row per destination, hidden wide
    e = np.zeros(0, dtype=np.int32)
    Z = oracle.project(oracle.aggregate_fwd(e, e, seeds, np.zeros((1, 8), np.float32), "mean"),
                       np.zeros((8, hidden)))
    assert Z.shape == (seeds, hidden)



# ---- sparse Adam on learnable tables (Sections 2.2 and 6: learnable vectors and their optimizer states) ----

def _adam_case(seed=0, n_rows=40, d=5, n_ids=17):
    g = np.random.default_rng(seed)
    theta = g.standard_normal((n_rows, d))
    ids = g.permutation(n_rows)[:n_ids]
    grads = [g.standard_normal((n_ids, d)) for _ in range(4)]
    return theta, ids, grads


def test_adam_first_step_is_a_signed_step_of_size_lr():
    """From zero states, mhat = g and vhat = g^2 after the first step, so every touched element moves by
    lr * g / (|g| + eps) (Adam paper, Section 2.1: the effective step is bounded by lr)."""
    theta, ids, grads = _adam_case()
    z = np.zeros_like(theta)
    lr, eps = 0.01, 1e-8
    t1, m1, v1 = oracle.sparse_adam_step(theta, z, z, ids, grads[0], lr, 0.9, 0.999, eps, 1)
    g = grads[0]
    np.testing.assert_allclose(t1[ids], theta[ids] - lr * g / (np.abs(g) + eps), rtol=1e-12, atol=0)
    np.testing.assert_allclose(m1[ids], 0.1 * g, rtol=1e-12)
    np.testing.assert_allclose(v1[ids], 0.001 * g * g, rtol=1e-12)
    untouched = np.setdiff1d(np.arange(theta.shape[0]), ids)
    assert np.array_equal(t1[untouched], theta[untouched]) and not m1[untouched].any() and not v1[untouched].any()


def test_adam_constant_gradient_has_a_closed_form():
    """A constant gradient keeps mhat = g and vhat = g^2 at every step (the bias corrections cancel the
    geometric sums exactly), so after T steps theta = theta0 - T lr g / (|g| + eps)."""
    theta, ids, grads = _adam_case(1)
    m = np.zeros_like(theta)
    v = np.zeros_like(theta)
    lr, eps, T = 0.003, 1e-8, 25
    x = theta
    for t in range(1, T + 1):
        x, m, v = oracle.sparse_adam_step(x, m, v, ids, grads[0], lr, 0.9, 0.999, eps, t)
    g = grads[0]
    np.testing.assert_allclose(x[ids], theta[ids] - T * lr * g / (np.abs(g) + eps), rtol=1e-9, atol=1e-12)


def test_adam_matches_the_library_optimizer_when_every_row_is_touched():
    """With all rows touched at every step the sparse step is the dense Adam of torch.optim (fp64)."""
    import torch
    g0 = np.random.default_rng(2)
    n, d, T = 12, 7, 6
    theta0 = g0.standard_normal((n, d))
    grads = [g0.standard_normal((n, d)) for _ in range(T)]
    lr, b1, b2, eps = 0.02, 0.8, 0.95, 1e-6
    p = torch.nn.Parameter(torch.tensor(theta0, dtype=torch.float64))
    opt = torch.optim.Adam([p], lr=lr, betas=(b1, b2), eps=eps)
    x, m, v = theta0, np.zeros_like(theta0), np.zeros_like(theta0)
    for t in range(1, T + 1):
        perm = g0.permutation(n)                       # ids in any order: rows are independent
        p.grad = torch.tensor(grads[t - 1], dtype=torch.float64)
        opt.step()
        x, m, v = oracle.sparse_adam_step(x, m, v, perm, grads[t - 1][perm], lr, b1, b2, eps, t)
        np.testing.assert_allclose(x, p.detach().numpy(), rtol=1e-10, atol=1e-13)


def test_adam_rows_skipped_for_a_step_keep_state_and_are_not_decayed():
    """Lazy semantics: a row absent from `ids` is bit-for-bit unchanged, states included, and on its next
    visit it sees the global step counter (not a per-row one)."""
    theta, ids, grads = _adam_case(3)
    z = np.zeros_like(theta)
    a, b = ids[:9], ids[5:]
    x1, m1, v1 = oracle.sparse_adam_step(theta, z, z, a, grads[0][:9], 0.01, 0.9, 0.999, 1e-8, 1)
    x2, m2, v2 = oracle.sparse_adam_step(x1, m1, v1, b, grads[1][5:], 0.01, 0.9, 0.999, 1e-8, 2)
    only_a = np.setdiff1d(a, b)
    assert np.array_equal(x2[only_a], x1[only_a]) and np.array_equal(m2[only_a], m1[only_a]) and np.array_equal(v2[only_a], v1[only_a])
    only_b = np.setdiff1d(b, a)                        # first visit at t = 2: m = 0.1 g, divided by 1 - 0.9^2
    g = grads[1][5:][np.isin(b, only_b)]
    r = b[np.isin(b, only_b)]
    mhat, vhat = 0.1 * g / (1 - 0.81), 0.001 * g * g / (1 - 0.999 ** 2)
    np.testing.assert_allclose(x2[r], theta[r] - 0.01 * mhat / (np.sqrt(vhat) + 1e-8), rtol=1e-12)
    with pytest.raises(AssertionError):
        oracle.sparse_adam_step(theta, z, z, np.array([1, 1]), grads[0][:2], 0.01, 0.9, 0.999, 1e-8, 1)


# ---- R-GAT (graph attention as AGG_r): pins of oracle/rgat.py --------------------------------------

from oracle import rgat


def _tiny_rgat(seed, heads=2, relu=True, gain=2.0):
    p = tiny_problem(seed, "sum", relu=relu)
    g = np.random.default_rng(seed + 100)
    F = p.d_out // heads
    a = [gain * g.standard_normal((heads, F)) for _ in p.graph.relations]
    q = [gain * g.standard_normal((p.tables[r.dst_type].shape[1], heads)) for r in p.graph.relations]
    return p, a, q


def _dense_rgat_torch(p, a, q, slope):
    """GAT written densely for autograd: per relation a count matrix C[v, u] (multi-edges are
    repeated softmax terms), logits for every (v, u) pair, softmax weights
    C exp(s) / sum_u C exp(s), output = weights @ Z per head.  Returns H per type and the leaves."""
    import torch
    g = p.graph
    T = [torch.tensor(np.asarray(t, np.float64), requires_grad=True) for t in p.tables]
    W = [torch.tensor(np.asarray(w, np.float64), requires_grad=True) for w in p.W]
    A = [torch.tensor(np.asarray(x, np.float64), requires_grad=True) for x in a]
    Q = [torch.tensor(np.asarray(x, np.float64), requires_grad=True) for x in q]
    acc = {}
    for i, r in enumerate(g.relations):
        n_s, n_t = g.ntypes[r.src_type].num_nodes, g.ntypes[r.dst_type].num_nodes
        C = np.zeros((n_t, n_s))
        src, dst = r.edge_list()
        for u, v in zip(src.tolist(), dst.tolist()):
            C[v, u] += 1.0
        C = torch.tensor(C)
        K, F = A[i].shape
        Z = (T[r.src_type] @ W[i]).reshape(n_s, K, F)
        el = (Z * A[i][None]).sum(-1)                 # [n_s, K]
        er = T[r.dst_type] @ Q[i]                     # [n_t, K]
        heads = []
        for k in range(K):
            s = torch.nn.functional.leaky_relu(er[:, k][:, None] + el[:, k][None, :], slope)   # [n_t, n_s]
            wgt = C * torch.exp(s)
            den = wgt.sum(1, keepdim=True)
            wgt = torch.where(den > 0, wgt / torch.where(den > 0, den, torch.ones_like(den)), torch.zeros_like(wgt))
            heads.append(wgt @ Z[:, k, :])
        O = torch.cat(heads, dim=1)
        acc[r.dst_type] = O if r.dst_type not in acc else acc[r.dst_type] + O
    H = {t: (torch.relu(h) if p.relu else h) for t, h in acc.items()}
    return H, T, W, A, Q


@pytest.mark.parametrize("seed", [0, 1, 2])
@pytest.mark.parametrize("heads", [1, 2, 3])
def test_rgat_matches_dense_autograd(seed, heads):
    import torch
    p, a, q = _tiny_rgat(seed, heads)
    slope = 0.2
    fwd = rgat.rgat_forward(p, a, q, slope)
    dW, da, dq, dH0 = rgat.rgat_backward(p, a, q, fwd, p.G, slope)
    H, T, W, A, Q = _dense_rgat_torch(p, a, q, slope)
    loss = sum((torch.tensor(np.asarray(p.G[t], np.float64)) * H[t]).sum() for t in H)
    loss.backward()
    for t in H:
        np.testing.assert_allclose(fwd.H[t], H[t].detach().numpy(), rtol=1e-11, atol=1e-12)
    for i in range(len(p.graph.relations)):
        np.testing.assert_allclose(dW[i], W[i].grad.numpy(), rtol=1e-9, atol=1e-11)
        np.testing.assert_allclose(da[i], A[i].grad.numpy(), rtol=1e-9, atol=1e-11)
        np.testing.assert_allclose(dq[i], Q[i].grad.numpy(), rtol=1e-9, atol=1e-11)
    for t in range(len(p.tables)):
        ref = T[t].grad.numpy() if T[t].grad is not None else np.zeros_like(p.tables[t])
        np.testing.assert_allclose(dH0.get(t, np.zeros_like(ref)), ref, rtol=1e-9, atol=1e-11)


def test_rgat_with_zero_attention_parameters_is_the_mean_aggregation():
    """a = 0 and q = 0 give equal logits, so alpha = 1/deg and the module is the R-GCN mean:
    o_r = mean_agg(H0_s) W_r, which the first oracle computes through its own C edge loop."""
    p, a, q = _tiny_rgat(3, heads=2, relu=False)
    a = [np.zeros_like(x) for x in a]
    q = [np.zeros_like(x) for x in q]
    fwd = rgat.rgat_forward(p, a, q)
    p.op = "mean"
    ref = oracle.layer_forward(p)
    for t in ref.H:
        np.testing.assert_allclose(fwd.H[t], ref.H[t], rtol=1e-12, atol=1e-12)


def test_edge_softmax_against_the_library_softmax_row_by_row():
    from scipy.special import softmax
    g = np.random.default_rng(5)
    n_src, n_dst, E, K = 9, 7, 40, 3
    src = g.integers(0, n_src, E)
    dst = g.integers(0, n_dst - 1, E)           # last row stays empty
    el = 3.0 * g.standard_normal((n_src, K))
    er = 3.0 * g.standard_normal((n_dst, K))
    alpha = rgat.edge_softmax(src, dst, n_dst, el, er, 0.2)
    for v in range(n_dst):
        sel = np.nonzero(dst == v)[0]
        if sel.size == 0:
            continue
        x = el[src[sel]] + er[v]
        s = np.where(x > 0, x, 0.2 * x)
        np.testing.assert_allclose(alpha[sel], softmax(s, axis=0), rtol=1e-12)
        np.testing.assert_allclose(alpha[sel].sum(0), 1.0, rtol=1e-12)


def test_gat_single_in_edge_copies_the_source_row_and_empty_rows_are_zero():
    g = np.random.default_rng(6)
    K, F = 2, 3
    Z = g.standard_normal((5, K * F))
    src = np.array([4, 1, 1], dtype=np.int64)
    dst = np.array([0, 2, 3], dtype=np.int64)
    el, er = g.standard_normal((5, K)), g.standard_normal((5, K))
    O, alpha = rgat.gat_aggregate_fwd(src, dst, 5, Z, el, er)
    assert np.array_equal(alpha, np.ones((3, K)))
    assert np.array_equal(O[0], Z[4]) and np.array_equal(O[2], Z[1]) and np.array_equal(O[3], Z[1])
    assert not O[1].any() and not O[4].any()
    # with a single term the softmax is constant: no gradient reaches the scores
    dZ, d_el, d_er = rgat.gat_aggregate_bwd(src, dst, 5, 5, Z, el, er, alpha, g.standard_normal((5, K * F)))
    assert not d_el.any() and not d_er.any()


def test_gat_with_slope_one_ignores_the_destination_score():
    """LeakyReLU with slope 1 is the identity; then er[v] shifts every logit of row v alike,
    the softmax drops it, and its gradient is exactly the sum of a softmax Jacobian row: 0."""
    g = np.random.default_rng(7)
    n_src, n_dst, E, K, F = 8, 6, 30, 2, 4
    src, dst = g.integers(0, n_src, E), g.integers(0, n_dst, E)
    Z = g.standard_normal((n_src, K * F))
    el, er = g.standard_normal((n_src, K)), g.standard_normal((n_dst, K))
    O1, al1 = rgat.gat_aggregate_fwd(src, dst, n_dst, Z, el, er, slope=1.0)
    O2, al2 = rgat.gat_aggregate_fwd(src, dst, n_dst, Z, el, 5.0 * er + 1.0, slope=1.0)
    np.testing.assert_allclose(O1, O2, rtol=1e-12, atol=1e-13)
    _, _, d_er = rgat.gat_aggregate_bwd(src, dst, n_src, n_dst, Z, el, er, al1, g.standard_normal((n_dst, K * F)), slope=1.0)
    np.testing.assert_allclose(d_er, 0.0, atol=1e-13)


def test_rgat_finite_differences_on_the_tiny_workload():
    p = workloads.rgat_tiny()
    ap = workloads.attention_params(p, 4, gain=2.0)
    a = [np.asarray(x, np.float64) for x in ap.a]
    q = [np.asarray(x, np.float64) for x in ap.q]
    p.tables = [np.asarray(t, np.float64) for t in p.tables]
    p.W = [np.asarray(w, np.float64) for w in p.W]
    fwd = rgat.rgat_forward(p, a, q, ap.slope)
    dW, da, dq, dH0 = rgat.rgat_backward(p, a, q, fwd, p.G, ap.slope)

    def loss():
        f = rgat.rgat_forward(p, a, q, ap.slope)
        return sum(float((np.asarray(p.G[t], np.float64) * f.H[t]).sum()) for t in f.H)

    g = np.random.default_rng(11)
    eps = 1e-6
    checks = []
    for i in range(len(p.W)):
        checks.append((p.W[i], dW[i]))
        checks.append((a[i], da[i]))
        checks.append((q[i], dq[i]))
    for t in range(len(p.tables)):
        checks.append((p.tables[t], dH0[t]))
    for arr, grad in checks:
        for _ in range(2):
            idx = tuple(int(g.integers(0, s)) for s in arr.shape)
            old = arr[idx]
            arr[idx] = old + eps
            up = loss()
            arr[idx] = old - eps
            dn = loss()
            arr[idx] = old
            fd = (up - dn) / (2 * eps)
            assert abs(fd - grad[idx]) <= 1e-5 * max(1.0, abs(fd)), (idx, fd, grad[idx])


# ---- neighbour sampling: pins of oracle/sampler.py ---------------------------------------------------

from oracle import sampler as osampler


def test_splitmix64_matches_the_published_outputs():
    with open(os.path.join(GOLDEN, "splitmix64.txt")) as f:
        want = [int(l, 16) for l in f if l.strip() and not l.startswith("#")]
    state, got = 0, []
    for _ in want:
        got.append(osampler.mix(state))
        state = (state + osampler.GAMMA) & osampler.MASK64
    assert got == want


def test_below_covers_the_range_evenly():
    assert osampler.below(0, 7) == 0 and osampler.below(osampler.MASK64, 7) == 6
    counts = np.zeros(7, dtype=np.int64)
    prev = 0
    for i in range(1 << 14):
        b = osampler.below(i << 50, 7)
        assert b >= prev
        prev = b
        counts[b] += 1
    assert counts.max() - counts.min() <= 1


@pytest.mark.parametrize("deg,k", [(5, 2), (6, 3), (4, 3), (7, 1)])
def test_floyd_subsets_are_uniform_over_all_draws(deg, k):
    """Feeding every possible sequence of draws (each equally likely) must produce every k-subset of the
    slots equally often: the defining property of sampling without replacement."""
    import itertools
    ranges = [range(j + 1) for j in range(deg - k, deg)]
    counts = {}
    for draws in itertools.product(*ranges):
        s = tuple(osampler.sample_slots(0, deg, k, 0, draw=lambda step, n: draws[step]))
        assert len(set(s)) == k and list(s) == sorted(s) and 0 <= s[0] and s[-1] < deg
        counts[s] = counts.get(s, 0) + 1
    n_subsets = len(list(itertools.combinations(range(deg), k)))
    assert len(counts) == n_subsets and len(set(counts.values())) == 1


def test_sampled_slots_are_uniform_with_the_generator():
    deg, k, n = 10, 3, 20000
    hits = np.zeros(deg)
    for v in range(n):
        for s in osampler.sample_slots(v, deg, k, 12345):
            hits[s] += 1
    p = k / deg
    sigma = np.sqrt(n * p * (1 - p))
    assert np.all(np.abs(hits - n * p) < 4.5 * sigma), hits
    # and a different seed gives a different draw for most destinations
    same = sum(osampler.sample_slots(v, deg, k, 12345) == osampler.sample_slots(v, deg, k, 54321) for v in range(2000))
    assert same < 2000 * 0.05


def test_sample_neighbors_invariants_and_unique_relabel():
    g = np.random.default_rng(3)
    n_src, n_dst, E = 50, 40, 600
    src = g.integers(0, n_src, E).astype(np.int32)
    dst = np.sort(g.integers(0, n_dst - 3, E)).astype(np.int32)     # the last rows stay empty
    rowptr, col = csr_from_edges(src, dst, n_dst)
    ids = g.permutation(n_dst)[:25]
    for fanout in (1, 5, 64):
        ptr, out = osampler.sample_neighbors(rowptr, col, ids, fanout, 7)
        for i, v in enumerate(ids):
            nb = col[rowptr[v]:rowptr[v + 1]]
            got = out[ptr[i]:ptr[i + 1]]
            assert got.size == min(nb.size, fanout)
            if nb.size <= fanout:
                assert np.array_equal(got, nb)
            else:   # a sub-multiset of the neighbourhood, in edge order: match greedily
                j = 0
                for x in got:
                    while nb[j] != x:
                        j += 1
                    j += 1
                assert j <= nb.size
    lists = [g.integers(0, 30, 17), g.integers(0, 30, 0), g.integers(0, 30, 40)]
    uniq, loc = osampler.unique_relabel(lists)
    ref_u, ref_inv = np.unique(np.concatenate(lists), return_inverse=True)
    assert np.array_equal(uniq, ref_u)
    assert np.array_equal(np.concatenate(loc), ref_inv.astype(np.int32))


def test_sample_blocks_link_up():
    p = workloads.academic_graph(scale=0.002, workload="tests/sampler")
    rels = [(r.src_type, r.dst_type, r.rowptr, r.col) for r in p.relations]
    seeds = np.arange(0, p.ntypes[0].num_nodes, 7, dtype=np.int64)[:64]
    blocks = osampler.sample_blocks(len(p.ntypes), rels, 0, seeds, [5, 3], 99)
    assert len(blocks) == 2 and np.array_equal(blocks[1]["dst_ids"][0], seeds)
    for t in range(len(p.ntypes)):
        inner_src = blocks[1]["src_ids"][t]
        outer_dst = blocks[0]["dst_ids"][t]
        assert (outer_dst is None and inner_src.size == 0) or np.array_equal(outer_dst, inner_src)
    for b, fanout in zip(blocks, [5, 3]):
        for (s, t, rowptr, col), (ptr, loc) in zip(rels, b["rels"]):
            n_dst = 0 if b["dst_ids"][t] is None else b["dst_ids"][t].size
            assert ptr.size == n_dst + 1 and ptr[-1] == loc.size and np.all(np.diff(ptr) <= fanout)
            if loc.size:
                assert loc.max() < b["src_ids"][s].size


# ---- meta-partitioning (Section 5, Algorithm 2) ---------------------------------------------------

import itertools

from oracle import metapartition as omp


def _read_metapartition_example():
    types, rels, out = {}, [], {}
    for line in open(os.path.join(GOLDEN, "metapartition_example.txt")):
        f = line.split()
        if not f or f[0].startswith("#"):
            continue
        if f[0] == "type":
            types[f[1]] = (len(types), int(f[2]))
        elif f[0] == "rel":
            rels.append((f[1], types[f[2]][0], types[f[3]][0], int(f[4])))
        else:
            out[f[0]] = [float(x) for x in f[1:]]
    return types, rels, out


def test_metapartition_reproduces_the_papers_worked_example():
    types, rels, want = _read_metapartition_example()
    tw = [w for _, w in sorted(types.values())]
    pairs = [(s, t) for _, s, t, _ in rels]
    rw = [w for *_, w in rels]
    mp = omp.meta_partition(tw, pairs, rw, root=types["paper"][0], k=2, p=2)
    names = [rels[i][0] for i in mp.sub_rel]
    assert sorted(names) == ["cites", "rev_has_topic", "writes"]          # the root has three children
    assert sorted(round(w / 1e6) for w in mp.sub_weight) == want["sub_weights_millions"]
    heavy = int(np.argmax(mp.sub_weight))
    assert names[heavy] == "cites"
    light = [c for c in range(3) if c != heavy]
    assert mp.sub_part[light[0]] == mp.sub_part[light[1]] != mp.sub_part[heavy]
    for key, q, subs in (("partition_light_pair", mp.sub_part[light[0]], light), ("partition_heavy", mp.sub_part[heavy], [heavy])):
        n_rel, nodes_m, edges_m = want[key]
        assert sum(mp.rel_mask[q]) == n_rel
        nodes = sum(tw[t] for t in range(len(tw)) if mp.type_mask[q][t])
        assert round(nodes / 1e6, 1) == nodes_m
        # the printed edge counts are those of the sub-metatrees' links before a repeated relation
        # is dropped (the heavy partition holds "cites" twice: 25 million with it, 20 without)
        assert round(sum(mp.sub_links[c] for c in subs) / 1e6) == edges_m
    q = mp.sub_part[heavy]
    assert round(sum(rw[i] for i in range(len(rw)) if mp.rel_mask[q][i]) / 1e6) == 20
    assert sorted(rels[i][0] for i in range(len(rels)) if mp.rel_mask[q][i]) == ["cites", "rev_has_topic", "writes"]


def _random_metagraph(seed, n_types, n_rels):
    r = np.random.default_rng(seed)
    pairs = [(int(r.integers(n_types)), int(r.integers(n_types))) for _ in range(n_rels)]
    return pairs, [int(x) for x in r.integers(1, 1000, n_types)], [int(x) for x in r.integers(1, 5000, n_rels)]


@pytest.mark.parametrize("seed", range(6))
def test_metatree_levels_count_the_walks(seed):
    """Level l of the tree holds one vertex per walk of l relations from the root: e_root^T B^l 1,
    B[t, s] = number of relations from s into t."""
    pairs, _, _ = _random_metagraph(seed, 5, 9)
    B = np.zeros((5, 5), dtype=np.int64)
    for s, t in pairs:
        B[t, s] += 1
    for root in range(5):
        tree = omp.build_metatree(pairs, root, 4)
        for l in range(5):
            walks = int(np.linalg.matrix_power(B, l)[root].sum())
            assert sum(1 for v in tree if v.depth == l) == walks
        for j, v in enumerate(tree[1:], 1):
            s, t = pairs[v.via]
            assert (v.ntype, tree[v.parent].ntype, v.depth) == (s, t, tree[v.parent].depth + 1) and v.parent < j


def test_lpt_on_grahams_tight_instance_and_against_the_optimum():
    # Graham 1969: 2m+1 jobs {2m-1, 2m-1, ..., m+1, m+1, m, m, m}; LPT ends at 4m-1, the optimum is 3m
    part, sums = omp.lpt([5, 5, 4, 4, 3, 3, 3], 3)
    assert sums == [11, 8, 8] and part == [0, 1, 2, 2, 0, 1, 0]
    assert part[:2] == [0, 1] and part[2] == 2                  # heaviest first, lowest free index first
    r = np.random.default_rng(3)
    for _ in range(60):
        n, p = int(r.integers(1, 8)), int(r.integers(1, 4))
        w = [int(x) for x in r.integers(1, 30, n)]
        part, sums = omp.lpt(w, p)
        assert sorted(part + list(range(p)))[-1] < p and sum(sums) == sum(w)
        assert all(sums[q] == sum(w[i] for i in range(n) if part[i] == q) for q in range(p))
        best = min(max(sum(w[i] for i in range(n) if a[i] == q) for q in range(p)) for a in itertools.product(range(p), repeat=n))
        assert best <= max(sums) <= (4.0 / 3.0 - 1.0 / (3 * p)) * best + 1e-9


@pytest.mark.parametrize("seed", range(8))
def test_metapartition_invariants_on_random_metagraphs(seed):
    n_types, n_rels = 5, 8
    pairs, tw, rw = _random_metagraph(100 + seed, n_types, n_rels)
    for root, k, p in itertools.product(range(n_types), (1, 2, 3), (1, 2, 3)):
        mp = omp.meta_partition(tw, pairs, rw, root, k, p)
        into_root = [i for i, (s, t) in enumerate(pairs) if t == root]
        assert mp.sub_rel == into_root
        n_real = min(p, len(into_root))
        assert sum(mp.part_weight) == sum(mp.sub_weight) and all(0 <= q < max(n_real, 1) for q in mp.sub_part)
        # relations within k steps of the root (a plain frontier sweep): held by some partition; no others
        reach, frontier = set(), {root}
        for _ in range(k):
            step = {i for i, (s, t) in enumerate(pairs) if t in frontier}
            reach |= step
            frontier = {pairs[i][0] for i in step}
        held = {i for q in range(p) for i in range(n_rels) if mp.rel_mask[q][i]}
        assert held == reach
        for q in range(p):
            rels_q = [i for i in range(n_rels) if mp.rel_mask[q][i]]
            if q >= n_real:
                assert (mp.replica_of[q] >= 0) == (n_real > 0)
                continue
            assert mp.replica_of[q] == -1 and mp.type_mask[q][root] == 1
            # closed: both end types of every relation are in the partition, and no type is idle
            ends = {root} | {x for i in rels_q for x in pairs[i]}
            assert ends == {t for t in range(n_types) if mp.type_mask[q][t]}
            # the aggregation path stays inside: every relation is reached from the root through the
            # partition's own relations
            got, frontier = set(), {root}
            for _ in range(k):
                step = {i for i in rels_q if pairs[i][1] in frontier}
                got |= step
                frontier = {pairs[i][0] for i in step}
            assert got == set(rels_q)


def test_metapartition_one_hop_closed_form_and_metapaths():
    pairs = [(1, 0), (2, 0), (0, 0), (0, 1), (1, 0)]
    tw, rw = [10, 20, 30], [1, 2, 3, 4, 5]
    mp = omp.meta_partition(tw, pairs, rw, root=0, k=1, p=2)
    assert mp.sub_rel == [0, 1, 2, 4]
    assert mp.sub_weight == [10 + 20 + 1, 10 + 30 + 2, 10 + 3, 10 + 20 + 5]      # a self-loop counts its type once
    # 42 -> 0, 35 -> 1, 31 -> 1 (35 < 42), 13 -> 0 (42 < 66)
    assert mp.sub_part == [1, 0, 0, 1] and mp.part_weight == [42 + 13, 35 + 31]
    # every walk of at most k relations given as a metapath = the breadth-first tree
    k = 3
    tree = omp.build_metatree(pairs, 0, k)
    paths = []
    for j in range(1, len(tree)):
        path, at = [], j
        while at > 0:
            path.append(tree[at].via)
            at = tree[at].parent
        paths.append(path[::-1])
    a = omp.meta_partition(tw, pairs, rw, 0, k, 2)
    b = omp.meta_partition(tw, pairs, rw, 0, k, 2, metapaths=paths)
    assert (a.sub_weight, a.sub_part, a.rel_mask, a.type_mask) == (b.sub_weight, b.sub_part, b.rel_mask, b.type_mask)
    # two metapaths sharing their first relation make one sub-metatree
    c = omp.meta_partition(tw, pairs, rw, 0, k, 2, metapaths=[[0, 3], [0, 3, 2], [2]])
    assert c.sub_rel == [0, 2] and c.sub_weight == [10 + 20 + 1 + 4 + 3, 10 + 3]
    with pytest.raises(ValueError):
        omp.meta_partition(tw, pairs, rw, 0, k, 2, metapaths=[[3]])


def test_metapartition_replicates_the_heaviest_partition_per_replica():
    pairs = [(1, 0), (2, 0)]
    mp = omp.meta_partition([0, 0, 0], pairs, [90, 40], root=0, k=1, p=5)
    assert mp.part_weight == [90, 40, 0, 0, 0]
    assert mp.replica_of == [-1, -1, 0, 0, 1]        # 90 vs 40; 45 vs 40; 30 vs 40
    assert mp.rel_mask[2] == mp.rel_mask[0] == [1, 0] and mp.rel_mask[4] == [0, 1]


def test_error_scale_of_a_plain_float32_loop_on_a_long_row():
    """Why the oracle accumulates in fp64 and what the 1e-4 bound of the fp32 parity tests means: a hub row of
    2^17 N(0,1) neighbours summed edge after edge in float32 is off by a few 1e-6 of the row's largest
    entry, the fp64 loop by less than 1e-12: a tree-ordered float32 sum (the GPU's) has room to spare under
    1e-4, and the oracle's own rounding is invisible at that scale."""
    g = rng.stream("tests", "pins/f32scale")
    n, d = 1 << 17, 8
    X = g.standard_normal((n, d)).astype(np.float32)
    src = np.arange(n, dtype=np.int64)
    dst = np.zeros(n, dtype=np.int64)
    ref = oracle.aggregate_fwd(src, dst, 1, X, "sum")
    exact = np.array([math.fsum(X[:, j].astype(np.float64)) for j in range(d)])
    assert np.abs(ref[0] - exact).max() <= 1e-12 * np.abs(exact).max() + 1e-9
    plain = oracle.aggregate_fwd_f32_sequential(src, dst, 1, X, "sum")
    err = np.abs(plain[0].astype(np.float64) - exact).max() / max(1.0, np.abs(exact).max())
    assert 1e-9 < err < 1e-4
