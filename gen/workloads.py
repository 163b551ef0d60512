"""The benchmark workloads as seeded synthetic inputs.

Shapes follow the paper's datasets (Table 1 and Section 8.1): an academic graph with
four node types of which only one has features (ogbn-mag-like), a seven-type graph with
feature widths from 7 to 789 (Donor-like), and a three-type graph with 768-wide vectors
(MAG240M-like).  None of those datasets is used: structure, features, weights and upstream
gradients are all drawn from `gen.rng` streams.  `scale` shrinks node and edge counts
proportionally so that the same recipe gives CPU-sized instances.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional

import numpy as np

from . import rng
from .graphs import (HetGraph, NodeType, Relation, power_law_relation, reverse_relation,
                     uniform_relation)


@dataclass
class LayerProblem:
    """Inputs of one layer: H_t = sum_r AGG_r(H0_s) W_r, plus the upstream gradient G_t."""
    name: str
    graph: HetGraph
    op: str                              # "mean" | "sum"
    storage: str                         # "f32" | "bf16": storage type of tables and weights
    tables: List[np.ndarray]             # per node type [N, d] float32 (bf16-exact if storage == "bf16")
    W: List[np.ndarray]                  # per relation [d_src, d_out] float32
    d_out: int
    G: Dict[int, np.ndarray]             # per destination type with >=1 incoming relation: [N_t, d_out]
    pre_proj: Optional[List[np.ndarray]] = None   # per node type fixed [d_table, d_shared], or None
    src_gid: Optional[List[Optional[np.ndarray]]] = None  # per node type local->global row map (int64)
    relu: bool = False
    notes: Dict[str, object] = field(default_factory=dict)

    def edge_features(self) -> int:
        """sum_r E_r * d_r, where d_r is the width the aggregation of relation r runs at."""
        tot = 0
        for r in self.graph.relations:
            d = self.W[self.graph.relations.index(r)].shape[0]
            tot += r.num_edges * d
        return tot


def _maybe_bf16(x: np.ndarray, storage: str) -> np.ndarray:
    return rng.round_to_bf16(x) if storage == "bf16" else x


def glorot(d_in: int, d_out: int, workload: str, name: str) -> np.ndarray:
    a = float(np.sqrt(6.0 / (d_in + d_out)))
    return rng.uniform_table(d_in, d_out, -a, a, workload, name)


def _upstream(graph: HetGraph, d_out: int, workload: str, exact: bool) -> Dict[int, np.ndarray]:
    G = {}
    for t, nt in enumerate(graph.ntypes):
        if graph.rels_into(t):
            G[t] = (rng.small_int_table(nt.num_nodes, d_out, -2, 2, workload, f"G/{nt.name}") if exact
                    else rng.normal_table(nt.num_nodes, d_out, workload, f"G/{nt.name}"))
    return G


def _tables(graph: HetGraph, workload: str, storage: str, exact: bool) -> List[np.ndarray]:
    tabs = []
    for nt in graph.ntypes:
        if exact:
            t = rng.small_int_table(nt.num_nodes, nt.feat_dim, -2, 2, workload, f"table/{nt.name}")
        elif nt.learnable:
            t = rng.uniform_table(nt.num_nodes, nt.feat_dim, -0.1, 0.1, workload, f"table/{nt.name}")
        else:
            t = rng.normal_table(nt.num_nodes, nt.feat_dim, workload, f"table/{nt.name}")
        tabs.append(_maybe_bf16(t, storage))
    return tabs


def _weights(graph: HetGraph, d_in_of_rel, d_out: int, workload: str, storage: str, exact: bool):
    Ws = []
    for i, r in enumerate(graph.relations):
        d = d_in_of_rel(i)
        w = (rng.small_int_table(d, d_out, -1, 1, workload, f"W/{r.name}") if exact
             else glorot(d, d_out, workload, f"W/{r.name}"))
        Ws.append(_maybe_bf16(w, storage))
    return Ws


# ---- config 1: tiny RGCN layer ----------------------------------------------------------------

def config1(exact: bool = False) -> LayerProblem:
    """Types A (2,000 x 64 features), B (1,000 x 16 features), C (500 featureless, 32-wide
    embeddings); relations A->A, B->A, C->A, A->B with 5,000 uniform random edges each; a fixed
    per-type matrix maps every table to a shared 32-wide input; mean aggregation; W_r 32 x 32."""
    wl = "config1" + ("/exact" if exact else "")
    nts = [NodeType("A", 2000, 64, False), NodeType("B", 1000, 16, False), NodeType("C", 500, 32, True)]
    g = HetGraph(nts)
    for nm, s, t in [("A->A", 0, 0), ("B->A", 1, 0), ("C->A", 2, 0), ("A->B", 0, 1)]:
        g.relations.append(uniform_relation(nm, s, t, nts[s].num_nodes, nts[t].num_nodes, 5000, wl))
    tabs = _tables(g, wl, "f32", exact)
    P = []
    for nt in nts:
        if exact:
            P.append(rng.small_int_table(nt.feat_dim, 32, -1, 1, wl, f"P/{nt.name}"))
        else:
            a = 1.0 / float(np.sqrt(nt.feat_dim))
            P.append(rng.uniform_table(nt.feat_dim, 32, -a, a, wl, f"P/{nt.name}"))
    W = _weights(g, lambda i: 32, 32, wl, "f32", exact)
    return LayerProblem("config1", g, "mean", "f32", tabs, W, 32, _upstream(g, 32, wl, exact), pre_proj=P)


# ---- R-GAT parameters and a tiny R-GAT problem ----------------------------------------------

@dataclass
class AttentionParams:
    """Per relation: `a[i]` [heads, d_out / heads] (source half of the attention vector) and
    `q[i]` [d_dst_table, heads] (destination half, already multiplied into the table's width)."""
    heads: int
    slope: float
    a: List[np.ndarray]
    q: List[np.ndarray]


def attention_params(problem: LayerProblem, heads: int, slope: float = 0.2, gain: float = 1.0) -> AttentionParams:
    """Seeded attention parameters for every relation of a layer problem: uniform with the
    Glorot bound of their shape times `gain` (larger gains give sharper softmaxes)."""
    assert problem.d_out % heads == 0
    F = problem.d_out // heads
    wl = problem.name + f"/attn{heads}"
    a, q = [], []
    for r in problem.graph.relations:
        ba = gain * float(np.sqrt(6.0 / (F + 1)))
        d_t = problem.tables[r.dst_type].shape[1]
        bq = gain * float(np.sqrt(6.0 / (d_t + 1)))
        a.append(rng.uniform_table(heads, F, -ba, ba, wl, f"a/{r.name}"))
        q.append(rng.uniform_table(d_t, heads, -bq, bq, wl, f"q/{r.name}"))
    return AttentionParams(heads, slope, a, q)


def rgat_tiny(storage: str = "f32", d_out: int = 32) -> LayerProblem:
    """Config 1's graph as an R-GAT problem: every relation maps its source table's own
    width (64, 16, 32) to `d_out` with its W_r; ReLU after the cross-relation sum."""
    wl = "rgat_tiny"
    nts = [NodeType("A", 2000, 64, False), NodeType("B", 1000, 16, False), NodeType("C", 500, 32, True)]
    g = HetGraph(nts)
    for nm, s, t in [("A->A", 0, 0), ("B->A", 1, 0), ("C->A", 2, 0), ("A->B", 0, 1)]:
        g.relations.append(uniform_relation(nm, s, t, nts[s].num_nodes, nts[t].num_nodes, 5000, wl))
    tabs = _tables(g, wl, storage, False)
    W = _weights(g, lambda i: nts[g.relations[i].src_type].feat_dim, d_out, wl, storage, False)
    return LayerProblem("rgat_tiny", g, "sum", storage, tabs, W, d_out, _upstream(g, d_out, wl, False), relu=True)


# ---- the academic-shaped graph of configs 2 and 3 ----------------------------------------------

def academic_graph(scale: float = 1.0, exponent: float = 2.1, workload: str = "academic") -> HetGraph:
    """paper / author / institution / field; four base relations with power-law destination
    in-degree and uniform sources, plus the exact transposes of three of them (7 relations)."""
    n = lambda x: max(4, int(round(x * scale)))
    nts = [NodeType("paper", n(700_000), 128, False), NodeType("author", n(1_100_000), 128, True),
           NodeType("institution", n(9_000), 128, True), NodeType("field", n(60_000), 128, True)]
    P, A, I, F = 0, 1, 2, 3
    g = HetGraph(nts)
    N = [t.num_nodes for t in nts]

    def base(nm, s, t, e):
        return power_law_relation(nm, s, t, N[s], N[t], n(e), exponent, workload)

    writes = base("writes", A, P, 4_000_000)
    cites = base("cites", P, P, 4_000_000)
    has_topic = base("has_topic", P, F, 4_000_000)
    affiliated = base("affiliated", A, I, 500_000)
    g.relations += [writes, cites, has_topic, affiliated,
                    reverse_relation("rev_writes", writes, N[A]),
                    reverse_relation("rev_has_topic", has_topic, N[P]),
                    reverse_relation("rev_affiliated", affiliated, N[A])]
    return g


def config3(storage: str = "f32", scale: float = 1.0, exact: bool = False, upstream: bool = True) -> LayerProblem:
    """Full-graph single layer on the academic-shaped graph (~21 M edges at scale 1):
    128-wide inputs, 256-wide output, mean aggregation."""
    wl = f"config3/{scale:g}" + ("/exact" if exact else "")
    g = academic_graph(scale, 2.1, wl)
    tabs = _tables(g, wl, storage, exact)
    W = _weights(g, lambda i: 128, 256, wl, storage, exact)
    return LayerProblem(f"config3-{storage}", g, "mean", storage, tabs, W, 256,
                        _upstream(g, 256, wl, exact) if upstream else {})


# ---- config 4: mixed widths --------------------------------------------------------------------

def config4(scale: float = 1.0, exact: bool = False, upstream: bool = True) -> LayerProblem:
    """Seven node types with widths {7, 24, 64e, 64e, 300, 512, 789} (e = learnable embedding),
    twelve independent power-law relations through the hub type T5, sum aggregation, per-relation
    W_r of shape d_src x 256, bf16 storage."""
    wl = f"config4/{scale:g}" + ("/exact" if exact else "")
    n = lambda x: max(4, int(round(x * scale)))
    spec = [("T1", 1_500_000, 7, False), ("T2", 1_200_000, 24, False), ("T3", 800_000, 64, True),
            ("T4", 600_000, 64, True), ("T5", 500_000, 300, False), ("T6", 300_000, 512, False),
            ("T7", 100_000, 789, False)]
    nts = [NodeType(nm, n(c), d, l) for nm, c, d, l in spec]
    g = HetGraph(nts)
    N = [t.num_nodes for t in nts]
    T5 = 4
    edges = {0: 5_000_000, 1: 4_000_000, 2: 4_000_000, 3: 3_000_000, 5: 2_000_000, 6: 2_000_000}
    for s, e in edges.items():
        g.relations.append(power_law_relation(f"{nts[s].name}->T5", s, T5, N[s], N[T5], n(e), 2.0, wl))
    for t, e in edges.items():
        g.relations.append(power_law_relation(f"T5->{nts[t].name}", T5, t, N[T5], N[t], n(e), 2.0, wl))
    tabs = _tables(g, wl, "bf16", exact)
    W = _weights(g, lambda i: nts[g.relations[i].src_type].feat_dim, 256, wl, "bf16", exact)
    return LayerProblem("config4", g, "sum", "bf16", tabs, W, 256, _upstream(g, 256, wl, exact) if upstream else {})


# ---- sampled mini-batch problems (configs 2 and 5) ---------------------------------------------

@dataclass
class MiniBatchProblem:
    """A k-layer model over sampled blocks: layer l runs on blocks[l]; layer 0 reads the node-type
    tables through the block's src_gid lists, layer l > 0 reads layer l-1's output embeddings.
    ReLU follows every layer but the last.  The upstream gradient G is given on the seeds."""
    name: str
    base: HetGraph
    blocks: list                          # gen.sampler.Block, outermost first
    op: str
    storage: str
    W: List[List[np.ndarray]]             # per layer, per relation: [d_in(l), d_hidden]
    d_hidden: int
    seed_type: int
    G: np.ndarray                         # [n_seeds, d_hidden]
    tables: Optional[List[np.ndarray]] = None          # host tables per base type, or None when counter-based
    table_keys: Optional[List[int]] = None             # counter-based tables (gen.rng.hashed_rows)
    table_kinds: Optional[List[str]] = None

    def table_rows(self, t: int, ids: np.ndarray) -> np.ndarray:
        """float32 rows `ids` of base type t's table, as stored (bf16-exact when storage is bf16)."""
        if self.tables is not None:
            return self.tables[t][ids]
        x = rng.hashed_rows(self.table_keys[t], ids, self.base.ntypes[t].feat_dim, self.table_kinds[t])
        return _maybe_bf16(x, self.storage)

    def layer_problem(self, l: int, prev_H: Optional[Dict[int, np.ndarray]] = None) -> LayerProblem:
        """The LayerProblem of layer l with compact host tables (row i = i-th source of the block).
        prev_H: layer l-1's output per block node type (destination roles), needed for l > 0."""
        b = self.blocks[l]
        T = b.n_base_types
        tabs = []
        for k in range(2 * T):
            if k >= T:
                tabs.append(np.zeros((0, 1), dtype=np.float32))
            elif l == 0:
                tabs.append(self.table_rows(k, b.src_gid[k]))
            else:
                h = prev_H.get(T + k)
                n = b.graph.ntypes[k].num_nodes
                assert h is not None or n == 0, "a source type of an inner layer has no embedding"
                tabs.append(h if h is not None else np.zeros((0, self.d_hidden)))
        last = l == len(self.blocks) - 1
        G = {T + self.seed_type: self.G} if last else {}
        return LayerProblem(f"{self.name}/L{l + 1}", b.graph, self.op, self.storage, tabs, self.W[l], self.d_hidden,
                            G, relu=not last)


def _minibatch(name: str, base: HetGraph, seed_type: int, n_seeds: int, fanouts: List[int], d_hidden: int,
               storage: str, wl: str, tables, keys, kinds) -> MiniBatchProblem:
    from .sampler import sample_blocks
    g = rng.stream(wl, "seeds")
    seeds = np.sort(g.choice(base.ntypes[seed_type].num_nodes, size=n_seeds, replace=False)).astype(np.int64)
    blocks = sample_blocks(base, seed_type, seeds, fanouts, wl)
    W = []
    for l in range(len(fanouts)):
        d_in = lambda i, l=l: base.ntypes[base.relations[i].src_type].feat_dim if l == 0 else d_hidden
        W.append(_weights(base, d_in, d_hidden, f"{wl}/L{l + 1}", storage, False))
    G = rng.normal_table(n_seeds, d_hidden, wl, "G/seeds")
    return MiniBatchProblem(name, base, blocks, "mean", storage, W, d_hidden, seed_type, G,
                            tables=tables, table_keys=keys, table_kinds=kinds)


def config2(scale: float = 1.0) -> MiniBatchProblem:
    """Sampled 2-layer mini-batch on the academic-shaped graph of config 3: 1,024 seed papers,
    fanouts [25, 20] (seed hop 20), hidden 256, mean, fp32."""
    gwl = f"config3/{scale:g}"
    base = academic_graph(scale, 2.1, gwl)
    tabs = _tables(base, gwl, "f32", False)
    n_seeds = min(1024, base.ntypes[0].num_nodes // 2)
    return _minibatch("config2", base, 0, n_seeds, [25, 20], 256, "f32", f"config2/{scale:g}", tabs, None, None)


def mag_graph(scale: float = 1.0, workload: str = "config5") -> HetGraph:
    """paper / author / institution with 768-wide vectors; cites, writes, affiliated with power-law
    destination in-degree (exponent 1.9) and uniform sources, plus the exact transposes of the
    latter two (5 relations, 400 M edges at scale 1)."""
    n = lambda x: max(4, int(round(x * scale)))
    nts = [NodeType("paper", n(30_000_000), 768, False), NodeType("author", n(15_000_000), 768, True),
           NodeType("institution", n(100_000), 768, True)]
    P, A, I = 0, 1, 2
    N = [t.num_nodes for t in nts]
    g = HetGraph(nts)
    cites = power_law_relation("cites", P, P, N[P], N[P], n(240_000_000), 1.9, workload)
    writes = power_law_relation("writes", A, P, N[A], N[P], n(70_000_000), 1.9, workload)
    affiliated = power_law_relation("affiliated", A, I, N[A], N[I], n(10_000_000), 1.9, workload)
    g.relations += [cites, writes, affiliated, reverse_relation("rev_writes", writes, N[A]),
                    reverse_relation("rev_affiliated", affiliated, N[A])]
    return g


def config5(scale: float = 1.0) -> MiniBatchProblem:
    """One GPU's partition of a 240 M-node-shaped graph: sampled 2-layer mini-batch, 4,096 seed
    papers, fanouts [25, 15], 768 -> 1024 -> 1024, mean, bf16 tables.  The tables are
    counter-based (filled on the device; the host regenerates the rows it needs)."""
    wl = f"config5/{scale:g}"
    base = mag_graph(scale, wl)
    keys = [rng.table_key(wl, f"table/{t.name}") for t in base.ntypes]
    kinds = ["embedding" if t.learnable else "normal" for t in base.ntypes]
    n_seeds = min(4096, base.ntypes[0].num_nodes // 2)
    return _minibatch("config5", base, 0, n_seeds, [25, 15], 1024, "bf16", wl, None, keys, kinds)
