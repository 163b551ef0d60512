"""R-GAT: graph attention as the relation-specific aggregation.  TEST INFRASTRUCTURE ONLY.

The paper names R-GAT as its second model (Section 2.1 and the model-architecture figure of
the introduction): one GAT module per mono-relation subgraph, the modules' outputs summed
over the relations into a destination type (AGG_all = summation, Eq. 1) and activated by
ReLU.  It prints no formula for the module, so the module below is the graph attention layer
of the GAT paper (Velickovic et al., ICLR 2018, Eqs. 1-4 and the multi-head concatenation),
written for a bipartite relation r from source type s to destination type t with K heads of
width F (d_out = K F):

    z_u        = W_r^T h_u                       z_u in R^{K x F}, u of type s
    el[u, k]   = <z_u[k, :], a_r[k, :]>          source half of  a^T [W h_i || W h_j]
    er[v, k]   = <h_v, q_r[:, k]>                destination half; q_r[:, k] is the product of the
                                                 destination-side weight matrix and its half of a,
                                                 kept as one d_t x K matrix because s and t have
                                                 different widths and cannot share W
    s_e[k]     = LeakyReLU(el[u_e, k] + er[v_e, k])          (negative slope 0.2 in GAT)
    alpha_e[k] = exp(s_e[k]) / sum_{e': v_e' = v_e} exp(s_e'[k])   softmax over the in-edges of v
    o_{v,r}    = concat_k sum_{e: v_e = v} alpha_e[k] z_{u_e}[k, :]
    h_v        = ReLU(sum_r o_{v,r})

Multi-edges are separate terms of the softmax; a destination without in-edges gets o = 0.
Everything is fp64 numpy over the explicit edge list (np.add.at / np.maximum.at in edge
order); the backward pass is the chain rule of the lines above written out term by term.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence

import numpy as np


def leaky_relu(x: np.ndarray, slope: float) -> np.ndarray:
    return np.where(x > 0.0, x, slope * x)


def source_scores(Z: np.ndarray, a: np.ndarray) -> np.ndarray:
    """el[u, k] = sum_f Z[u, k F + f] a[k, f]."""
    K, F = a.shape
    Z = np.asarray(Z, dtype=np.float64)
    return np.einsum("ukf,kf->uk", Z.reshape(Z.shape[0], K, F), np.asarray(a, dtype=np.float64))


def destination_scores(H0_t: np.ndarray, q: np.ndarray) -> np.ndarray:
    """er[v, k] = sum_j H0_t[v, j] q[j, k]."""
    return np.asarray(H0_t, dtype=np.float64) @ np.asarray(q, dtype=np.float64)


def edge_softmax(src, dst, n_dst: int, el: np.ndarray, er: np.ndarray, slope: float) -> np.ndarray:
    """alpha[e, k]: softmax of LeakyReLU(el[u_e] + er[v_e]) over the edges sharing v_e."""
    src = np.asarray(src, dtype=np.int64)
    dst = np.asarray(dst, dtype=np.int64)
    K = el.shape[1]
    s = leaky_relu(el[src] + er[dst], slope)                   # [E, K]
    top = np.full((n_dst, K), -np.inf)
    np.maximum.at(top, dst, s)                                 # the usual shift; it cancels in alpha
    p = np.exp(s - top[dst])
    den = np.zeros((n_dst, K))
    np.add.at(den, dst, p)
    return p / den[dst]


def gat_aggregate_fwd(src, dst, n_dst: int, Z: np.ndarray, el: np.ndarray, er: np.ndarray,
                      slope: float = 0.2):
    """o[v] = concat_k sum_{e into v} alpha_e[k] Z[u_e, head k].  Returns (o, alpha)."""
    src = np.asarray(src, dtype=np.int64)
    dst = np.asarray(dst, dtype=np.int64)
    Z = np.asarray(Z, dtype=np.float64)
    K = el.shape[1]
    F = Z.shape[1] // K
    assert Z.shape[1] == K * F
    alpha = edge_softmax(src, dst, n_dst, np.asarray(el, np.float64), np.asarray(er, np.float64), slope)
    o = np.zeros((n_dst, K, F))
    np.add.at(o, dst, alpha[:, :, None] * Z[src].reshape(-1, K, F))
    return o.reshape(n_dst, K * F), alpha


def gat_aggregate_bwd(src, dst, n_src: int, n_dst: int, Z: np.ndarray, el: np.ndarray, er: np.ndarray,
                      alpha: np.ndarray, dO: np.ndarray, slope: float = 0.2):
    """Chain rule of gat_aggregate_fwd for L = <dO, o>.  Returns (dZ, del, der):

        dZ[u, k, :]  = sum_{e: u_e = u} alpha_e[k] dO[v_e, k, :]
        dalpha_e[k]  = <dO[v_e, k, :], Z[u_e, k, :]>
        ds_e[k]      = alpha_e[k] (dalpha_e[k] - sum_{e' into v_e} alpha_e'[k] dalpha_e'[k])   (softmax)
        dx_e[k]      = ds_e[k] * (1 if el[u_e,k] + er[v_e,k] > 0 else slope)                   (LeakyReLU)
        del[u, k]    = sum_{e: u_e = u} dx_e[k] ;  der[v, k] = sum_{e: v_e = v} dx_e[k]
    """
    src = np.asarray(src, dtype=np.int64)
    dst = np.asarray(dst, dtype=np.int64)
    Z = np.asarray(Z, dtype=np.float64)
    dO = np.asarray(dO, dtype=np.float64)
    K = alpha.shape[1]
    F = Z.shape[1] // K
    Zs = Z[src].reshape(-1, K, F)
    Gd = dO[dst].reshape(-1, K, F)
    dZ = np.zeros((n_src, K, F))
    np.add.at(dZ, src, alpha[:, :, None] * Gd)
    dalpha = np.einsum("ekf,ekf->ek", Gd, Zs)
    mean = np.zeros((n_dst, K))
    np.add.at(mean, dst, alpha * dalpha)
    ds = alpha * (dalpha - mean[dst])
    x = np.asarray(el, np.float64)[src] + np.asarray(er, np.float64)[dst]
    dx = ds * np.where(x > 0.0, 1.0, slope)
    d_el = np.zeros((n_src, K))
    np.add.at(d_el, src, dx)
    d_er = np.zeros((n_dst, K))
    np.add.at(d_er, dst, dx)
    return dZ.reshape(n_src, K * F), d_el, d_er


@dataclass
class RgatResult:
    Z: Dict[int, np.ndarray] = field(default_factory=dict)       # per relation [n_src, K F]
    el: Dict[int, np.ndarray] = field(default_factory=dict)      # per relation [n_src, K]
    er: Dict[int, np.ndarray] = field(default_factory=dict)      # per relation [n_dst, K]
    alpha: Dict[int, np.ndarray] = field(default_factory=dict)   # per relation [E, K], edge-list order
    O: Dict[int, np.ndarray] = field(default_factory=dict)       # per relation [n_dst, K F]
    H: Dict[int, np.ndarray] = field(default_factory=dict)       # per destination type


def rgat_forward(problem, a: Sequence[np.ndarray], q: Sequence[np.ndarray], slope: float = 0.2,
                 rels: Optional[Sequence[int]] = None) -> RgatResult:
    """One R-GAT layer over a LayerProblem (its W are the W_r; `a[i]` is [K, F], `q[i]` is
    [d_t, K] for relation i); ReLU after the cross-relation sum when problem.relu."""
    g = problem.graph
    rels = list(range(len(g.relations))) if rels is None else list(rels)
    res = RgatResult()
    acc: Dict[int, np.ndarray] = {}
    for i in rels:
        r = g.relations[i]
        src, dst = r.edge_list()
        n_dst = g.ntypes[r.dst_type].num_nodes
        Z = np.asarray(problem.tables[r.src_type], np.float64) @ np.asarray(problem.W[i], np.float64)
        el = source_scores(Z, a[i])
        er = destination_scores(problem.tables[r.dst_type], q[i])
        O, alpha = gat_aggregate_fwd(src, dst, n_dst, Z, el, er, slope)
        res.Z[i], res.el[i], res.er[i], res.alpha[i], res.O[i] = Z, el, er, alpha, O
        acc[r.dst_type] = O.copy() if r.dst_type not in acc else acc[r.dst_type] + O
    for t, h in acc.items():
        res.H[t] = np.maximum(h, 0.0) if problem.relu else h
    return res


def rgat_backward(problem, a: Sequence[np.ndarray], q: Sequence[np.ndarray], fwd: RgatResult,
                  G: Dict[int, np.ndarray], slope: float = 0.2, rels: Optional[Sequence[int]] = None):
    """Backward of rgat_forward for L = sum_t <G_t, H_t>.  Returns (dW, da, dq, dH0):
    per relation dW_r, da_r, dq_r; per node type the gradient of its table, which collects
    the source side of every relation leaving the type and the destination-score side of
    every relation entering it."""
    g = problem.graph
    rels = list(range(len(g.relations))) if rels is None else list(rels)
    dW: Dict[int, np.ndarray] = {}
    da: Dict[int, np.ndarray] = {}
    dq: Dict[int, np.ndarray] = {}
    dH0: Dict[int, np.ndarray] = {}

    def table_grad(t: int) -> np.ndarray:
        if t not in dH0:
            dH0[t] = np.zeros(np.asarray(problem.tables[t]).shape, dtype=np.float64)
        return dH0[t]

    for i in rels:
        r = g.relations[i]
        src, dst = r.edge_list()
        n_src = g.ntypes[r.src_type].num_nodes
        n_dst = g.ntypes[r.dst_type].num_nodes
        dO = np.asarray(G[r.dst_type], dtype=np.float64)
        if problem.relu:
            dO = dO * (fwd.H[r.dst_type] > 0.0)
        dZ, d_el, d_er = gat_aggregate_bwd(src, dst, n_src, n_dst, fwd.Z[i], fwd.el[i], fwd.er[i],
                                           fwd.alpha[i], dO, slope)
        ai = np.asarray(a[i], np.float64)
        K, F = ai.shape
        # el = <z_k, a_k>: its gradient reaches z and a
        dZt = (dZ.reshape(n_src, K, F) + d_el[:, :, None] * ai[None]).reshape(n_src, K * F)
        da[i] = np.einsum("uk,ukf->kf", d_el, fwd.Z[i].reshape(n_src, K, F))
        H0s = np.asarray(problem.tables[r.src_type], np.float64)
        H0t = np.asarray(problem.tables[r.dst_type], np.float64)
        Wi = np.asarray(problem.W[i], np.float64)
        dW[i] = H0s.T @ dZt
        table_grad(r.src_type)[...] += dZt @ Wi.T
        dq[i] = H0t.T @ d_er
        table_grad(r.dst_type)[...] += d_er @ np.asarray(q[i], np.float64).T
    return dW, da, dq, dH0
