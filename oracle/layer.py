"""The layer as the paper defines it, composed from the edge-loop oracle and fp64 matmuls.

TEST INFRASTRUCTURE ONLY (see the package docstring).  Notation follows Eq. 1 of the
paper: for relation r with source type s and destination type t,

    h_{v,r} = AGG_r({h_u : u in N_r(v)}) = (sum | mean)_{e: v_e = v} H0_s[u_e] . W_r
    h_v     = AGG_all({h_{v,r}})         = sum over relations r into t of h_{v,r}

with AGG_r the GCN-style normalised neighbour sum times a per-relation weight matrix
(Section 2.1, R-GCN) and AGG_all the summation (Section 2.1; Algorithm 1, the
cross-relation aggregation on the designated worker).  H0 of a node type is its feature
table, or its table of learnable vectors when the type has no features (Section 2.1).
The backward pass is what Algorithm 1 calls local backpropagation with the gradients of
the partial aggregations: dZ_r = G_t, dW_r = M_r^T dZ_r, dM_r = dZ_r W_r^T, and a
per-edge scatter dH0_s[u_e] += c_e dM_r[v_e].
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_HERE, "liboracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile heta_oracle.c with gcc into liboracle.so next to it."""
    src = os.path.join(_HERE, "heta_oracle.c")
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(src):
        subprocess.check_call(["gcc", "-O2", "-fPIC", "-shared", "-std=c11", "-Wall", "-Wextra",
                               "-o", _SO, src])
    return _SO


def _load():
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_SO)
        i64, i32, vp = ctypes.c_int64, ctypes.c_int32, ctypes.c_void_p
        L.oracle_in_degree.argtypes = [i64, vp, i64, vp]
        L.oracle_aggregate_fwd.argtypes = [i64, vp, vp, i64, vp, i64, i32, vp, i32, vp]
        L.oracle_aggregate_fwd_f64.argtypes = [i64, vp, vp, i64, vp, i64, i32, vp, i32, vp]
        L.oracle_aggregate_fwd_f64.restype = None
        L.oracle_aggregate_bwd.argtypes = [i64, vp, vp, i64, vp, i32, i32, vp]
        L.oracle_csc.argtypes = [i64, vp, vp, i64, vp, vp]
        for f in (L.oracle_in_degree, L.oracle_aggregate_fwd, L.oracle_aggregate_bwd, L.oracle_csc):
            f.restype = None
        _lib = L
    return _lib


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data


def _edges(src, dst):
    src = np.ascontiguousarray(src, dtype=np.int32)
    dst = np.ascontiguousarray(dst, dtype=np.int32)
    assert src.shape == dst.shape and src.ndim == 1
    return src, dst


# ---- single steps -----------------------------------------------------------------------------

def in_degree(src, dst, n_dst: int) -> np.ndarray:
    """deg_r(v): edges into v, multi-edges counted."""
    src, dst = _edges(src, dst)
    assert dst.size == 0 or (dst.min() >= 0 and dst.max() < n_dst)
    deg = np.zeros(n_dst, dtype=np.int64)
    _load().oracle_in_degree(dst.size, _p(dst), n_dst, _p(deg))
    return deg


def aggregate_fwd(src, dst, n_dst: int, H0: np.ndarray, op: str,
                  gid: Optional[np.ndarray] = None, d: Optional[int] = None) -> np.ndarray:
    """M_r [n_dst, d] fp64: neighbour sum (op == "sum") or mean (op == "mean", zero-degree rows 0).
    H0 is a float32 (or fp64) [rows, >=d] table; gid optionally maps source ids to table rows."""
    assert op in ("sum", "mean")
    src, dst = _edges(src, dst)
    H0 = np.asarray(H0)
    assert H0.dtype in (np.float32, np.float64) and H0.ndim == 2
    if H0.shape[0] == 0:          # an empty table (a source type nobody sampled): strides carry no meaning
        H0 = np.zeros((0, H0.shape[1]), dtype=H0.dtype)
        ld = H0.shape[1]
    else:
        assert H0.strides[1] == H0.itemsize
        ld = H0.strides[0] // H0.itemsize
    d = H0.shape[1] if d is None else d
    if gid is not None:
        gid = np.ascontiguousarray(gid, dtype=np.int64)
        assert src.size == 0 or src.max() < gid.size
        assert gid.size == 0 or (gid.min() >= 0 and gid.max() < H0.shape[0])
    else:
        assert src.size == 0 or (src.min() >= 0 and src.max() < H0.shape[0])
    assert dst.size == 0 or (dst.min() >= 0 and dst.max() < n_dst)
    M = np.zeros((n_dst, d), dtype=np.float64)
    fn = _load().oracle_aggregate_fwd if H0.dtype == np.float32 else _load().oracle_aggregate_fwd_f64
    fn(src.size, _p(src), _p(dst), n_dst, _p(H0), ld, d, _p(gid), 1 if op == "mean" else 0, _p(M))
    return M


def aggregate_fwd_f32_sequential(src, dst, n_dst: int, H0: np.ndarray, op: str) -> np.ndarray:
    """The same neighbour sum accumulated in float32, edge after edge in list order: NOT the oracle, only a
    yardstick for the error a plain single-precision loop makes on long rows (the tolerances of the parity
    tests are judged against it)."""
    src, dst = _edges(src, dst)
    H0 = np.asarray(H0, dtype=np.float32)
    M = np.zeros((n_dst, H0.shape[1]), dtype=np.float32)
    for u, v in zip(src.tolist(), dst.tolist()):
        M[v] += H0[u]
    if op == "mean":
        deg = np.bincount(dst, minlength=n_dst).astype(np.float32)
        M = np.where(deg[:, None] > 0, M / np.maximum(deg, 1)[:, None], np.float32(0))
    return M


def aggregate_bwd(src, dst, n_src: int, n_dst: int, dM: np.ndarray, op: str,
                  out: Optional[np.ndarray] = None) -> np.ndarray:
    """dH0 [n_src, d] fp64 (+)= per-edge scatter of c_e * dM[v_e]; accumulates into `out` if given."""
    assert op in ("sum", "mean")
    src, dst = _edges(src, dst)
    dM = np.ascontiguousarray(dM, dtype=np.float64)
    assert dM.shape[0] == n_dst
    d = dM.shape[1]
    assert src.size == 0 or (src.min() >= 0 and src.max() < n_src)
    assert dst.size == 0 or (dst.min() >= 0 and dst.max() < n_dst)
    if out is None:
        out = np.zeros((n_src, d), dtype=np.float64)
    assert out.dtype == np.float64 and out.shape == (n_src, d) and out.flags.c_contiguous
    _load().oracle_aggregate_bwd(src.size, _p(src), _p(dst), n_dst, _p(dM), d,
                                 1 if op == "mean" else 0, _p(out))
    return out


def csc(src, dst, n_src: int):
    """(colptr int64 [n_src+1], row int32 [E]): transposed adjacency, rows of a column in
    ascending original edge position."""
    src, dst = _edges(src, dst)
    assert src.size == 0 or (src.min() >= 0 and src.max() < n_src)
    colptr = np.zeros(n_src + 1, dtype=np.int64)
    row = np.zeros(src.size, dtype=np.int32)
    _load().oracle_csc(src.size, _p(src), _p(dst), n_src, _p(colptr), _p(row))
    return colptr, row


def project(M: np.ndarray, W: np.ndarray) -> np.ndarray:
    """Z_r = M_r W_r in fp64 (library matmul as the step)."""
    return np.asarray(M, dtype=np.float64) @ np.asarray(W, dtype=np.float64)


def project_bwd(M: np.ndarray, dZ: np.ndarray, W: np.ndarray):
    """(dM_r, dW_r) = (dZ_r W_r^T, M_r^T dZ_r) in fp64."""
    M = np.asarray(M, dtype=np.float64)
    dZ = np.asarray(dZ, dtype=np.float64)
    W = np.asarray(W, dtype=np.float64)
    return dZ @ W.T, M.T @ dZ


def cross_rel_sum(partials: Sequence[np.ndarray], relu: bool = False) -> np.ndarray:
    """H_t = sum of the per-relation partial embeddings in the given order (optional ReLU)."""
    H = np.zeros_like(np.asarray(partials[0], dtype=np.float64))
    for Z in partials:
        H = H + np.asarray(Z, dtype=np.float64)
    return np.maximum(H, 0.0) if relu else H


# ---- the whole layer --------------------------------------------------------------------------

@dataclass
class LayerResult:
    H0: List[Optional[np.ndarray]]            # per node type: table @ P (fp64) when a fixed map is given
    M: Dict[int, np.ndarray]                  # per relation [n_dst, d_r] fp64
    H: Dict[int, np.ndarray]                  # per destination type [n_t, d_out] fp64
    Z: Dict[int, np.ndarray] = field(default_factory=dict)   # kept only on request


def layer_forward(problem, rels: Optional[Sequence[int]] = None, keep_Z: bool = False) -> LayerResult:
    """Forward of one layer over the relations in `rels` (default: all), in list order."""
    g = problem.graph
    rels = list(range(len(g.relations))) if rels is None else list(rels)
    n_types = len(g.ntypes)
    H0: List[Optional[np.ndarray]] = [None] * n_types
    if problem.pre_proj is not None:
        for t in range(n_types):
            H0[t] = np.asarray(problem.tables[t], dtype=np.float64) @ \
                np.asarray(problem.pre_proj[t], dtype=np.float64)
    M: Dict[int, np.ndarray] = {}
    Z: Dict[int, np.ndarray] = {}
    acc: Dict[int, List[np.ndarray]] = {}
    for i in rels:
        r = g.relations[i]
        src, dst = r.edge_list()
        n_dst = g.ntypes[r.dst_type].num_nodes
        gid = None if problem.src_gid is None else problem.src_gid[r.src_type]
        table = H0[r.src_type] if problem.pre_proj is not None else problem.tables[r.src_type]
        M[i] = aggregate_fwd(src, dst, n_dst, table, problem.op, gid=gid)
        z = project(M[i], problem.W[i])
        acc.setdefault(r.dst_type, []).append(z)
        if keep_Z:
            Z[i] = z
    H = {t: cross_rel_sum(zs, relu=problem.relu) for t, zs in acc.items()}
    return LayerResult(H0=H0, M=M, H=H, Z=Z)


def layer_backward(problem, fwd: LayerResult, G: Dict[int, np.ndarray],
                   rels: Optional[Sequence[int]] = None):
    """Backward of one layer.  Returns (dW per relation, dH0 per node type, dtable per node
    type); dtable == dH0 unless a fixed per-type map P is present, in which case
    dtable = dH0 P^T.  With a local->global map, dH0 rows are per local source row."""
    g = problem.graph
    rels = list(range(len(g.relations))) if rels is None else list(rels)
    dW: Dict[int, np.ndarray] = {}
    dH0: Dict[int, np.ndarray] = {}
    for i in rels:
        r = g.relations[i]
        src, dst = r.edge_list()
        n_src = g.ntypes[r.src_type].num_nodes
        n_dst = g.ntypes[r.dst_type].num_nodes
        dZ = np.asarray(G[r.dst_type], dtype=np.float64)
        if problem.relu:
            dZ = dZ * (fwd.H[r.dst_type] > 0.0)
        dM, dW[i] = project_bwd(fwd.M[i], dZ, problem.W[i])
        if r.src_type not in dH0:
            n_rows = n_src
            d = dM.shape[1]
            dH0[r.src_type] = np.zeros((n_rows, d), dtype=np.float64)
        aggregate_bwd(src, dst, n_src, n_dst, dM, problem.op, out=dH0[r.src_type])
    dtable: Dict[int, np.ndarray] = {}
    for t, gH in dH0.items():
        if problem.pre_proj is not None:
            dtable[t] = gH @ np.asarray(problem.pre_proj[t], dtype=np.float64).T
        else:
            dtable[t] = gH
    return dW, dH0, dtable
