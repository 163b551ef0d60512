"""Meta-partitioning of a heterogeneous graph by its metagraph.  TEST INFRASTRUCTURE ONLY.

Section 5 and Algorithm 2 of the paper: the relations of a heterogeneous graph are dealt to p
partitions by working on the weighted metagraph alone (vertex weight = nodes of the type, link
weight = edges of the relation), in four steps.

  1. Metatree.  Sampling starts at the target type and can only follow relations that end in the
     type it stands on, so the computation depends on the walks of at most k relations that
     start at the target type.  The metatree is the tree of those walks (a type or relation
     appears once per walk that reaches it: the paper's example shows the target type as root,
     child and grandchild).  With user-given metapaths the tree holds exactly those walks,
     merged on common prefixes.
  2. Split.  One sub-metatree per child of the root: the root, the child and all its
     descendants.  Its weight is the sum of the weights of its vertices and links.  The
     example's three weights (16, 17 and 27 million) are reproduced by counting a node type
     once per sub-metatree and a link once per occurrence in it; counting the types per
     occurrence gives 17, 18 and 29.
  3. Assignment: longest-processing-time-first (Graham 1969).  Sub-metatrees by descending
     weight (equal weights: the lower relation index first), each to the partition with the
     smallest sum so far (equal sums: the lowest partition index).
  4. Deduplication: a partition holds every relation and every node type of its sub-metatrees
     once.

When there are more partitions than sub-metatrees the paper replicates partitions, whose
replicas split the target nodes (end of Section 5); which one it replicates is not said.  Here
each further partition becomes a replica of the partition whose weight per replica is largest
at that moment (equal: the lowest index).

A relation is (src_type, dst_type): messages flow from src to dst, sampling walks from dst to
src.  Plain Python lists and loops.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Sequence, Tuple


@dataclass
class TreeVertex:
    ntype: int
    parent: int        # index into the tree, -1 for the root
    via: int           # relation followed from the parent's type to this one, -1 for the root
    depth: int


def build_metatree(relations: Sequence[Tuple[int, int]], root: int, k: int,
                   metapaths: Optional[Sequence[Sequence[int]]] = None) -> List[TreeVertex]:
    """Breadth-first list of the metatree's vertices; vertex 0 is the root."""
    tree = [TreeVertex(root, -1, -1, 0)]
    if metapaths is None:
        head = 0
        while head < len(tree):                      # plain BFS queue over walks
            v = tree[head]
            if v.depth < k:
                for i, (s, t) in enumerate(relations):
                    if t == v.ntype:
                        tree.append(TreeVertex(s, head, i, v.depth + 1))
            head += 1
        return tree
    for path in metapaths:                           # a trie of the given walks
        at = 0
        for i in path:
            s, t = relations[i]
            if t != tree[at].ntype:
                raise ValueError("metapath does not follow the metagraph from the root")
            nxt = [j for j, w in enumerate(tree) if w.parent == at and w.via == i]
            if nxt:
                at = nxt[0]
            else:
                tree.append(TreeVertex(s, at, i, tree[at].depth + 1))
                at = len(tree) - 1
    return tree


def sub_metatrees(tree: Sequence[TreeVertex]) -> List[List[int]]:
    """For each child of the root, in tree order: the indices of the child and its descendants."""
    owner = [-1] * len(tree)
    subs: List[List[int]] = []
    for j, v in enumerate(tree):
        if v.parent == 0:
            owner[j] = len(subs)
            subs.append([j])
        elif v.parent > 0:
            owner[j] = owner[v.parent]               # parents precede children in the list
            subs[owner[j]].append(j)
    return subs


def sub_weight(tree: Sequence[TreeVertex], sub: Sequence[int], type_weight: Sequence[int],
               rel_weight: Sequence[int]) -> Tuple[int, int, int]:
    """(weight, vertex part, link part) of the sub-metatree {root} + sub."""
    types = {tree[0].ntype} | {tree[j].ntype for j in sub}
    nodes = sum(int(type_weight[t]) for t in types)
    links = sum(int(rel_weight[tree[j].via]) for j in sub)
    return nodes + links, nodes, links


def lpt(weights: Sequence[int], p: int) -> Tuple[List[int], List[int]]:
    """Longest-processing-time-first: (partition of each item, partition sums)."""
    order = sorted(range(len(weights)), key=lambda i: (-int(weights[i]), i))
    sums = [0] * p
    part = [-1] * len(weights)
    for i in order:
        j = min(range(p), key=lambda q: (sums[q], q))
        part[i] = j
        sums[j] += int(weights[i])
    return part, sums


@dataclass
class MetaPartition:
    sub_rel: List[int] = field(default_factory=list)       # relation from the root to each child
    sub_weight: List[int] = field(default_factory=list)
    sub_links: List[int] = field(default_factory=list)     # link part of the weight (per occurrence)
    sub_part: List[int] = field(default_factory=list)
    part_weight: List[int] = field(default_factory=list)   # LPT sums (0 for replicas)
    replica_of: List[int] = field(default_factory=list)    # -1, or the partition this one copies
    rel_mask: List[List[int]] = field(default_factory=list)    # [p][n_rels] 0/1
    type_mask: List[List[int]] = field(default_factory=list)   # [p][n_types] 0/1


def meta_partition(type_weight: Sequence[int], relations: Sequence[Tuple[int, int]], rel_weight: Sequence[int],
                   root: int, k: int, p: int, metapaths: Optional[Sequence[Sequence[int]]] = None) -> MetaPartition:
    n_types, n_rels = len(type_weight), len(relations)
    tree = build_metatree(relations, root, k, metapaths)
    subs = sub_metatrees(tree)
    res = MetaPartition()
    for sub in subs:
        w, _, links = sub_weight(tree, sub, type_weight, rel_weight)
        res.sub_rel.append(tree[sub[0]].via)
        res.sub_weight.append(w)
        res.sub_links.append(links)
    n_real = min(p, len(subs)) if subs else 0
    res.sub_part, sums = lpt(res.sub_weight, n_real) if n_real else ([], [])
    res.part_weight = sums + [0] * (p - n_real)
    res.replica_of = [-1] * p
    res.rel_mask = [[0] * n_rels for _ in range(p)]
    res.type_mask = [[0] * n_types for _ in range(p)]
    for c, sub in enumerate(subs):
        q = res.sub_part[c]
        res.type_mask[q][root] = 1
        for j in sub:
            res.rel_mask[q][tree[j].via] = 1
            res.type_mask[q][tree[j].ntype] = 1
    copies = [1] * n_real
    for q in range(n_real, p):
        if n_real == 0:
            break
        # weight per replica compared exactly: a / ca > b / cb  <=>  a * cb > b * ca
        best = 0
        for j in range(1, n_real):
            if sums[j] * copies[best] > sums[best] * copies[j]:
                best = j
        copies[best] += 1
        res.replica_of[q] = best
        res.rel_mask[q] = list(res.rel_mask[best])
        res.type_mask[q] = list(res.type_mask[best])
    return res
