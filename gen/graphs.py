"""Synthetic heterogeneous graphs: containers and structure generators.

A heterogeneous graph is a list of node types (each with a node count, a feature
width and a flag saying whether its input vectors are learnable embeddings) and a
list of relations, each a bipartite mono-relation subgraph stored as a CSR over
its destination rows (Section 2.1 of the paper: HetG, relation triple,
mono-relation subgraph).  Nothing here computes any part of the layer.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional, List, Tuple

import numpy as np

from . import rng

MAX_DEGREE_SUPPORT = 1 << 20


@dataclass
class NodeType:
    name: str
    num_nodes: int
    feat_dim: int
    learnable: bool


@dataclass
class Relation:
    name: str
    src_type: int
    dst_type: int
    rowptr: np.ndarray  # int64 [n_dst + 1], CSR over destination rows
    col: np.ndarray     # int32 [E], source node ids (duplicates allowed, any order)
    reverse_of: Optional[str] = None  # name of the relation this one is the exact transpose of, if it was built as one

    @property
    def num_edges(self) -> int:
        return int(self.col.shape[0])

    def edge_list(self) -> Tuple[np.ndarray, np.ndarray]:
        """(src[e], dst[e]) in CSR edge order; a plain re-statement of the CSR."""
        n_dst = self.rowptr.shape[0] - 1
        deg = np.diff(self.rowptr)
        dst = np.repeat(np.arange(n_dst, dtype=np.int32), deg)
        return self.col.astype(np.int32, copy=False), dst


@dataclass
class HetGraph:
    ntypes: List[NodeType]
    relations: List[Relation] = field(default_factory=list)

    def ntype_index(self, name: str) -> int:
        return [t.name for t in self.ntypes].index(name)

    def rel_index(self, name: str) -> int:
        return [r.name for r in self.relations].index(name)

    def rels_into(self, dst_type: int) -> List[int]:
        return [i for i, r in enumerate(self.relations) if r.dst_type == dst_type]

    def rels_from(self, src_type: int) -> List[int]:
        return [i for i, r in enumerate(self.relations) if r.src_type == src_type]


def csr_from_edges(src: np.ndarray, dst: np.ndarray, n_dst: int) -> Tuple[np.ndarray, np.ndarray]:
    """CSR over destinations of an edge list; edges of one row keep their input order."""
    order = np.argsort(dst, kind="stable")
    counts = np.bincount(dst, minlength=n_dst).astype(np.int64)
    rowptr = np.zeros(n_dst + 1, dtype=np.int64)
    np.cumsum(counts, out=rowptr[1:])
    return rowptr, np.ascontiguousarray(src[order], dtype=np.int32)


def uniform_relation(name: str, src_type: int, dst_type: int, n_src: int, n_dst: int,
                     n_edges: int, workload: str) -> Relation:
    """Sources and destinations uniform with replacement (multi-edges kept)."""
    g = rng.stream(workload, f"{name}/edges")
    src = g.integers(0, n_src, size=n_edges, dtype=np.int32)
    dst = g.integers(0, n_dst, size=n_edges, dtype=np.int32)
    rowptr, col = csr_from_edges(src, dst, n_dst)
    return Relation(name, src_type, dst_type, rowptr, col)


def power_law_degrees(n_rows: int, n_edges: int, exponent: float, g: np.random.Generator,
                      k_max: int = MAX_DEGREE_SUPPORT) -> np.ndarray:
    """In-degrees whose distribution follows P(k) ~ k**-exponent on 1..k_max, rescaled so
    that they sum to n_edges: weights are drawn i.i.d., scaled to the target total, rounded
    up or down at random in proportion to the fraction, and the remaining difference is put
    on the largest row.  Many rows end at 0-2 edges and a few at 1e5 and more."""
    if n_rows == 0:
        return np.zeros(0, dtype=np.int64)
    k = np.arange(1, k_max + 1, dtype=np.float64)
    cdf = np.cumsum(k ** (-exponent))
    cdf /= cdf[-1]
    z = (np.searchsorted(cdf, g.random(n_rows), side="left") + 1).astype(np.float64)
    w = z * (n_edges / z.sum())
    fl = np.floor(w)
    deg = (fl + (g.random(n_rows) < (w - fl))).astype(np.int64)
    diff = n_edges - int(deg.sum())
    hub = int(np.argmax(deg))
    if deg[hub] + diff < 0:  # cannot happen for the workloads here; keep the total exact anyway
        raise ValueError("power_law_degrees: fix-up would make a degree negative")
    deg[hub] += diff
    return deg


def power_law_relation(name: str, src_type: int, dst_type: int, n_src: int, n_dst: int,
                       n_edges: int, exponent: float, workload: str) -> Relation:
    """Power-law destination in-degree, sources uniform with replacement."""
    g = rng.stream(workload, f"{name}/edges")
    deg = power_law_degrees(n_dst, n_edges, exponent, g)
    rowptr = np.zeros(n_dst + 1, dtype=np.int64)
    np.cumsum(deg, out=rowptr[1:])
    col = g.integers(0, n_src, size=n_edges, dtype=np.int32)
    return Relation(name, src_type, dst_type, rowptr, col)


def reverse_relation(name: str, base: Relation, n_src_of_base: int) -> Relation:
    """The exact transpose of `base`: an edge u->v becomes v->u.  Its rows are the base's
    sources, so here the *sources* carry the skew."""
    src, dst = base.edge_list()
    rowptr, col = csr_from_edges(dst, src, n_src_of_base)
    return Relation(name, base.dst_type, base.src_type, rowptr, col, reverse_of=base.name)
