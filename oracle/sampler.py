"""k-hop neighbour sampling into per-layer blocks.  TEST INFRASTRUCTURE ONLY.

The paper's workers sample a fixed number of k-hop neighbours for the nodes of a mini-batch
(Section 2.2; Algorithm 1, the sampling step of every iteration) with per-relation fan-outs
such as {25, 20} (Section 8.1).  It does not say how the neighbours are drawn; the rule here is
the usual one: per (destination node, relation) all in-edges if the in-degree is at most the
fan-out, otherwise `fanout` distinct edge slots uniformly without replacement.

So that a GPU implementation can be compared bit for bit, the draw is fixed completely:
  * random numbers come from a counter-based generator, SplitMix64 (Steele, Lea, Flood,
    "Fast splittable pseudorandom number generators", OOPSLA 2014): the stream of destination v
    has the key mix(seed XOR mix(v)) and its j-th number is mix(key + j), where mix is
    SplitMix64's output function applied to (x + golden gamma);
  * a number r is mapped to an integer below n by taking the high 32 bits of r and the high half
    of their 64-bit product with n (n < 2^32);
  * the subset is built by Floyd's algorithm (Bentley & Floyd, "A sample of brilliant random
    samples", CACM 1987): for j = deg - fanout, ..., deg - 1 draw t uniform on [0, j]; take t
    unless it is already in the subset, in which case take j;
  * the sampled in-edges of a destination are listed by ascending edge slot, the unique source
    ids of a node type in ascending order, and local ids are positions in that list.

Plain Python integers and loops; no vectorisation.
"""
from __future__ import annotations

from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

MASK64 = (1 << 64) - 1
GAMMA = 0x9E3779B97F4A7C15


def mix(x: int) -> int:
    """SplitMix64's next(): state += gamma, then the two multiply-xorshift rounds; `x` is the state before."""
    z = (x + GAMMA) & MASK64
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & MASK64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & MASK64
    return z ^ (z >> 31)


def below(r: int, n: int) -> int:
    """Maps a 64-bit random number to [0, n), n < 2^32: high half of (high 32 bits of r) * n."""
    return ((r >> 32) * n) >> 32


def sample_slots(v: int, deg: int, fanout: int, seed: int, draw=None) -> List[int]:
    """Edge slots (0-based positions within v's in-edge list) chosen for destination v, ascending.
    `draw(j, n)`, if given, replaces the generator (used to enumerate Floyd's algorithm exhaustively)."""
    if deg <= fanout:
        return list(range(deg))
    key = mix((seed ^ mix(v)) & MASK64)
    chosen: List[int] = []
    for step, j in enumerate(range(deg - fanout, deg)):
        t = draw(step, j + 1) if draw is not None else below(mix((key + step) & MASK64), j + 1)
        chosen.append(j if t in chosen else t)
    return sorted(chosen)


def sample_neighbors(rowptr: np.ndarray, col: np.ndarray, dst_ids: Sequence[int], fanout: int, seed: int):
    """(block_rowptr [n+1], src_ids [total]) for the destinations dst_ids of one relation's CSR."""
    out_ptr = [0]
    out_src: List[int] = []
    for v in dst_ids:
        v = int(v)
        start, deg = int(rowptr[v]), int(rowptr[v + 1] - rowptr[v])
        for s in sample_slots(v, deg, fanout, seed):
            out_src.append(int(col[start + s]))
        out_ptr.append(len(out_src))
    return np.asarray(out_ptr, dtype=np.int64), np.asarray(out_src, dtype=np.int64)


def unique_relabel(lists: Sequence[np.ndarray]) -> Tuple[np.ndarray, List[np.ndarray]]:
    """Ascending unique ids over all lists, and each list rewritten as positions in that array."""
    seen = sorted({int(x) for l in lists for x in l})
    where = {x: i for i, x in enumerate(seen)}
    return (np.asarray(seen, dtype=np.int64),
            [np.asarray([where[int(x)] for x in l], dtype=np.int32) for l in lists])


def relation_seed(seed: int, hop: int, rel: int) -> int:
    """The seed of one (hop, relation) pair of a mini-batch: hop = 0 is the hop next to the seeds."""
    return (seed + 0x100000001B3 * (hop * 4096 + rel + 1)) & MASK64


def sample_blocks(n_types: int, relations: Sequence[Tuple[int, int, np.ndarray, np.ndarray]], seed_type: int,
                  seeds: Sequence[int], fanouts: Sequence[int], seed: int):
    """Blocks of a k-hop mini-batch, outermost first.  `relations`: (src_type, dst_type, rowptr, col).
    fanouts are listed outermost hop first ([25, 20]: the hop next to the seeds uses 20).  Each block
    is a dict: dst_ids[t] (the destinations per type, None if absent), src_ids[t] (ascending unique
    sampled sources per type), and per relation (rowptr, col_local)."""
    frontier: List[Optional[np.ndarray]] = [None] * n_types
    frontier[seed_type] = np.asarray(seeds, dtype=np.int64)
    blocks = []
    for hop, fanout in enumerate(reversed(list(fanouts))):
        sampled = []
        per_type: Dict[int, List[int]] = {}
        for i, (s, t, rowptr, col) in enumerate(relations):
            dst = frontier[t] if frontier[t] is not None else np.zeros(0, dtype=np.int64)
            ptr, src = sample_neighbors(rowptr, col, dst, fanout, relation_seed(seed, hop, i))
            sampled.append((ptr, src))
            per_type.setdefault(s, []).append(i)
        src_ids: List[np.ndarray] = []
        local: Dict[int, np.ndarray] = {}
        for s in range(n_types):
            rs = per_type.get(s, [])
            uniq, loc = unique_relabel([sampled[i][1] for i in rs])
            src_ids.append(uniq)
            for i, l in zip(rs, loc):
                local[i] = l
        blocks.append({"dst_ids": [None if f is None else f.copy() for f in frontier], "src_ids": src_ids,
                       "rels": [(sampled[i][0], local[i]) for i in range(len(relations))]})
        frontier = [u if u.size else None for u in src_ids]
    blocks.reverse()
    return blocks
