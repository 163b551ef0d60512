"""Sequencing of the device sampler for a k-hop mini-batch (Section 2.2 and the sampling step of
Algorithm 1 of the paper): hop by hop from the seeds outwards, per relation a call of
`heta_sample_neighbors` on the current frontier of its destination type, then per source type one
`heta_unique_relabel` over the relations leaving it (each hop issues them as one batched call of each
kind, synchronising twice); the handles of all hops' blocks are then built by one `heta_graph_create_batch` on
the hops' device arrays.  No arithmetic here beyond the seed given to each (hop, relation) pair.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Optional, Sequence

import torch

from . import binding as hb

_MASK64 = (1 << 64) - 1


def relation_seed(seed: int, hop: int, rel: int) -> int:
    """Seed of one (hop, relation) pair; hop 0 is the hop next to the seeds."""
    return (seed + 0x100000001B3 * (hop * 4096 + rel + 1)) & _MASK64


@dataclass
class DeviceBlock:
    """One bipartite layer graph on the device.  Node types are the base graph's types twice: index t is
    type t in the source role, index n_types + t is type t in the destination role."""
    graph: hb.Graph
    src_ids: List[torch.Tensor]             # per base type: ascending global ids of the block's sources
    dst_ids: List[Optional[torch.Tensor]]   # per base type: global ids of the block's destinations, or None
    rowptr: List[torch.Tensor]              # per relation, device int64
    col: List[torch.Tensor]                 # per relation, device int32 local source ids


def sample_blocks(base: hb.Graph, seed_type: int, seeds: torch.Tensor, fanouts: Sequence[int], seed: int,
                  stream=None) -> List[DeviceBlock]:
    """Blocks outermost first; fanouts are listed outermost hop first ([25, 20]: the seeds' hop uses 20)."""
    T = len(base.ntypes)
    frontier: List[Optional[torch.Tensor]] = [None] * T
    frontier[seed_type] = seeds
    empty = torch.zeros(0, dtype=torch.int64, device=seeds.device)
    specs = []
    parts = []
    for hop, fanout in enumerate(reversed(list(fanouts))):
        n_rels = len(base.rels)
        sampled = hb.heta_sample_neighbors_batch(
            base, list(range(n_rels)), [frontier[t] if frontier[t] is not None else empty for _, t, _ in base.rels], fanout,
            [relation_seed(seed, hop, i) for i in range(n_rels)], stream=stream)
        rowptrs = [rp for rp, _ in sampled]
        srcs = [src for _, src in sampled]
        by_type = [[i for i, r in enumerate(base.rels) if r[0] == s] for s in range(T)]
        relabelled = hb.heta_unique_relabel_batch([[srcs[i] for i in rs] for rs in by_type],
                                                  [base.ntypes[s][0] for s in range(T)], stream=stream)
        src_ids: List[torch.Tensor] = []
        cols: List[Optional[torch.Tensor]] = [None] * n_rels
        for rs, (uniq, local) in zip(by_type, relabelled):
            src_ids.append(uniq)
            for i, l in zip(rs, local):
                cols[i] = l
        nts = [(int(src_ids[k].numel()), base.ntypes[k][1], base.ntypes[k][2]) for k in range(T)]
        nts += [(0 if frontier[k] is None else int(frontier[k].numel()), base.ntypes[k][1], base.ntypes[k][2]) for k in range(T)]
        rels = [(s, T + t, rowptrs[i], cols[i]) for i, (s, t, _) in enumerate(base.rels)]
        specs.append((nts, rels))
        parts.append((src_ids, list(frontier), rowptrs, cols))
        frontier = [u if u.numel() else None for u in src_ids]
    # the blocks' handles (CSC, 1/deg, schedules of every relation of every hop) in one build
    graphs = hb.heta_graph_create_batch(specs, flags=hb.HETA_PTRS_ON_DEVICE)
    blocks = [DeviceBlock(g, *p) for g, p in zip(graphs, parts)]
    blocks.reverse()
    return blocks
