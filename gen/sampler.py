"""Host-side k-hop neighbour sampling into per-layer blocks (input generator only).

The paper samples a fixed number of k-hop neighbours of a mini-batch of target nodes
(Section 2.2; Algorithm 1, "sample k-hop neighbors for nodes in B") with fanouts {25, 20}
(Section 8.1).  This module produces such blocks from a synthetic graph so that the layer can
be exercised on mini-batch shaped inputs; it is not part of the measured path.

Rule per (destination node, relation): all in-edges if the degree is at most the fanout,
otherwise `fanout` distinct edge slots uniformly without replacement.  Blocks are returned
outermost first: block[0] reads the feature tables through its `src_gid` lists, block[l]'s
destination sets equal block[l+1]'s source sets (same order).
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Optional

import numpy as np

from . import rng
from .graphs import HetGraph, NodeType, Relation


@dataclass
class Block:
    """A bipartite layer graph.  Its node types are the base graph's types twice: index t is
    type t in the source role, index n_types + t is type t in the destination role."""
    graph: HetGraph
    src_gid: List[Optional[np.ndarray]]   # per block node type: global ids of the source sets (None for dst roles)
    dst_gid: List[Optional[np.ndarray]]   # per block node type: global ids of the destination sets (None for src roles)
    n_base_types: int


def _sample_relation(rel: Relation, dst_ids: np.ndarray, fanout: int, g: np.random.Generator):
    """(owner, src_global): sampled in-edges of the destinations `dst_ids` (owner = position in dst_ids),
    ordered by owner and, within one owner, by original edge position."""
    if dst_ids.size == 0 or rel.num_edges == 0:
        return np.zeros(0, dtype=np.int64), np.zeros(0, dtype=np.int64)
    starts = rel.rowptr[dst_ids]
    degs = rel.rowptr[dst_ids + 1] - starts
    total = int(degs.sum())
    if total == 0:
        return np.zeros(0, dtype=np.int64), np.zeros(0, dtype=np.int64)
    owner = np.repeat(np.arange(dst_ids.size, dtype=np.int64), degs)
    first = np.cumsum(degs) - degs
    pos_in_row = np.arange(total, dtype=np.int64) - np.repeat(first, degs)
    edge_pos = np.repeat(starts, degs) + pos_in_row
    big = np.repeat(degs > fanout, degs)
    keep = ~big
    if big.any():
        idx = np.flatnonzero(big)
        key = g.random(idx.size)
        order = np.lexsort((key, owner[idx]))          # by owner, then by random key
        o_sorted = owner[idx][order]
        run_start = np.flatnonzero(np.r_[True, o_sorted[1:] != o_sorted[:-1]])
        run_len = np.diff(np.r_[run_start, o_sorted.size])
        rank = np.arange(o_sorted.size) - np.repeat(run_start, run_len)
        keep[idx[order[rank < fanout]]] = True
    sel = np.flatnonzero(keep)
    return owner[sel], rel.col[edge_pos[sel]].astype(np.int64)


def sample_blocks(graph: HetGraph, seed_type: int, seeds: np.ndarray, fanouts: List[int], workload: str) -> List[Block]:
    """fanouts are listed outermost hop first (e.g. [25, 20]: the seed hop uses 20)."""
    T = len(graph.ntypes)
    frontier: List[Optional[np.ndarray]] = [None] * T
    frontier[seed_type] = np.asarray(seeds, dtype=np.int64)
    blocks: List[Block] = []
    for hop, fanout in enumerate(reversed(fanouts)):
        level = len(fanouts) - hop          # 1-based layer this block feeds
        sampled = []
        src_sets = [[] for _ in range(T)]
        for i, r in enumerate(graph.relations):
            dst_ids = frontier[r.dst_type]
            if dst_ids is None:
                dst_ids = np.zeros(0, dtype=np.int64)
            g = rng.stream(workload, f"sample/L{level}/{r.name}")
            owner, src = _sample_relation(r, dst_ids, fanout, g)
            sampled.append((owner, src, dst_ids.size))
            if src.size:
                src_sets[r.src_type].append(src)
        src_gid = [np.unique(np.concatenate(s)) if s else np.zeros(0, dtype=np.int64) for s in src_sets]
        nts = [NodeType(f"{t.name}/src", int(src_gid[k].size), t.feat_dim, t.learnable) for k, t in enumerate(graph.ntypes)]
        nts += [NodeType(f"{t.name}/dst", 0 if frontier[k] is None else int(frontier[k].size), t.feat_dim, t.learnable)
                for k, t in enumerate(graph.ntypes)]
        bg = HetGraph(nts)
        for i, r in enumerate(graph.relations):
            owner, src, n_dst = sampled[i]
            local = np.searchsorted(src_gid[r.src_type], src).astype(np.int32)
            counts = np.bincount(owner, minlength=n_dst).astype(np.int64)
            rowptr = np.zeros(n_dst + 1, dtype=np.int64)
            np.cumsum(counts, out=rowptr[1:])
            bg.relations.append(Relation(r.name, r.src_type, T + r.dst_type, rowptr, local))
        blocks.append(Block(bg, list(src_gid) + [None] * T,
                            [None] * T + [None if f is None else f.copy() for f in frontier], T))
        frontier = [s if s.size else None for s in src_gid]
    blocks.reverse()
    return blocks
