"""Sequencing of the library calls for one R-GAT layer on one GPU (forward and backward).

R-GAT (Section 2.1 of the paper) uses a GAT module as the relation-specific aggregation and
sums the modules' outputs over the relations into a destination type, followed by ReLU.  This
module allocates device buffers with torch and issues the C-ABI calls; it computes nothing
itself.  Per relation r from source type s to destination type t:

    Z_r  = H0_s W_r                         heta_project_batch (all relations leaving s in one launch)
    el_r = <Z_r[u, head k], a_r[k]>         = <H0_s[u], (W_r a_r)[k]>: heta_attn_fold, then a score of the input
                                            table (narrower than Z_r, and never rounded to the storage type)
    er_r = <H0_t[v], q_r[k]>                a score of the destination type's table; all scores of one table in
                                            one pass (heta_attn_score_multi)
    O_r  = edge-softmax weighted sum of Z_r heta_rel_attn_fwd
    H_t  = ReLU(sum_r O_r)                  heta_cross_rel_reduce

and the backward runs the same chain in reverse (heta_act_bwd, heta_rel_attn_bwd,
heta_attn_score_bwd_multi, heta_project_wgrad_batch, heta_attn_fold_bwd, heta_project_sum).
"""
from __future__ import annotations

from typing import Dict, List, Optional, Sequence

import torch

from . import binding as hb

_MAX_BATCH = 8  # products per batched projection launch
_MAX_SETS = 8   # score vector sets per one-pass score call


class RgatLayer:
    """Device-resident state of one R-GAT layer over a `binding.Graph`.

    tables[t] : device [N_t, d_t] (fp32 or bf16)
    W[r]      : device [d_s, d_out] in the storage dtype
    a[r]      : device fp32 [heads, d_out / heads]   (source half of the attention vector)
    q[r]      : device fp32 [heads, d_t]             (destination half, in the table's width)
    """

    def __init__(self, graph: hb.Graph, tables: Sequence[torch.Tensor], W: Sequence[torch.Tensor],
                 a: Sequence[torch.Tensor], q: Sequence[torch.Tensor], d_out: int, heads: int, slope: float = 0.2,
                 relu: bool = True, rels: Optional[Sequence[int]] = None):
        self.g = graph
        self.tables = list(tables)
        self.W, self.a, self.q = list(W), list(a), list(q)
        self.d_out, self.heads, self.slope = d_out, heads, float(slope)
        self.act = hb.HETA_ACT_RELU if relu else hb.HETA_ACT_NONE
        self.relu = relu
        self.rels = list(range(len(graph.rels))) if rels is None else list(rels)
        dev = self.W[self.rels[0]].device
        self.rels_into: Dict[int, List[int]] = {}
        self.rels_from: Dict[int, List[int]] = {}
        for r in self.rels:
            s, t, _ = graph.rels[r]
            self.rels_into.setdefault(t, []).append(r)
            self.rels_from.setdefault(s, []).append(r)
        # (relation, is the source side) for every score taken off a node type's table
        self._score_sets: Dict[int, List] = {}
        for r in self.rels:
            s, t, _ = graph.rels[r]
            self._score_sets.setdefault(s, []).append((r, True))
            self._score_sets.setdefault(t, []).append((r, False))
        store = self.W[self.rels[0]].dtype
        self.two_terms = store == torch.bfloat16

        def padded(n, d, dtype):
            qd = 16 // dtype.itemsize
            return torch.empty((n, (d + qd - 1) // qd * qd), dtype=dtype, device=dev)[:, :d]

        f32 = torch.float32
        n_src, n_dst = graph.n_src, graph.n_dst
        self.Z = {r: padded(n_src(r), d_out, store) for r in self.rels}
        self.el = {r: torch.empty((n_src(r), heads), dtype=f32, device=dev) for r in self.rels}
        self.er = {r: torch.empty((n_dst(r), heads), dtype=f32, device=dev) for r in self.rels}
        self.smax = {r: torch.empty((n_dst(r), heads), dtype=f32, device=dev) for r in self.rels}
        self.sinv = {r: torch.empty((n_dst(r), heads), dtype=f32, device=dev) for r in self.rels}
        self.O = {r: padded(n_dst(r), d_out, f32) for r in self.rels}
        # the same sums over the edges with a positive logit: saved so that the backward gathers no
        # feature row on the destination side
        self.Opos = {r: padded(n_dst(r), d_out, f32) for r in self.rels}
        self.H = {t: torch.empty((graph.ntypes[t][0], d_out), dtype=f32, device=dev) for t in self.rels_into}
        self._Gact = {t: torch.empty_like(h) for t, h in self.H.items()} if relu else {}
        self.dZ = {r: padded(n_src(r), d_out, f32) for r in self.rels}
        self.d_el = {r: torch.empty((n_src(r), heads), dtype=f32, device=dev) for r in self.rels}
        self.d_er = {r: torch.empty((n_dst(r), heads), dtype=f32, device=dev) for r in self.rels}
        self.dW = {r: torch.empty((self.W[r].shape[0], d_out), dtype=f32, device=dev) for r in self.rels}
        self.da = {r: torch.empty_like(self.a[r]) for r in self.rels}
        # wa_r = W_r a_r per head ([heads, d_s]) and its gradient
        self.wa = {r: torch.empty((heads, self.W[r].shape[0]), dtype=f32, device=dev) for r in self.rels}
        self.dwa = {r: torch.empty_like(self.wa[r]) for r in self.rels}
        self.dq = {r: torch.empty_like(self.q[r]) for r in self.rels}
        touched = set(self.rels_from) | set(self.rels_into)
        self.dH0 = {t: padded(graph.ntypes[t][0], self.tables[t].shape[1], f32) for t in sorted(touched)}

    # ---- forward ------------------------------------------------------------------------------------
    def forward(self, stream=None) -> Dict[int, torch.Tensor]:
        g = self.g
        for s, rs in self.rels_from.items():
            for i in range(0, len(rs), _MAX_BATCH):
                part = rs[i:i + _MAX_BATCH]
                hb.heta_project_batch([self.tables[s]] * len(part), [self.W[r] for r in part],
                                      [self.Z[r] for r in part], stream=stream, graph=self.g)
        for r in self.rels:
            hb.heta_attn_fold(self.W[r], self.a[r], self.wa[r], stream=stream)
        # every score of a node type's table in one pass over it: el of the relations leaving the type, er of
        # those entering it
        for t, sets in self._score_sets.items():
            for i in range(0, len(sets), _MAX_SETS):
                part = sets[i:i + _MAX_SETS]
                hb.heta_attn_score_multi(self.tables[t], [self.wa[r] if src else self.q[r] for r, src in part],
                                         [self.el[r] if src else self.er[r] for r, src in part], stream=stream)
        for r in self.rels:
            s, t, _ = g.rels[r]
            hb.heta_rel_attn_fwd(g, r, self.Z[r], self.el[r], self.er[r], self.slope, self.O[r], beta=0.0,
                                 smax=self.smax[r], sinv=self.sinv[r], out_pos=self.Opos[r], stream=stream)
        for t, rs in self.rels_into.items():
            hb.heta_cross_rel_reduce(g, t, [self.O[r] for r in rs], self.H[t], act=self.act, stream=stream)
        return self.H

    # ---- backward -----------------------------------------------------------------------------------
    def backward(self, G: Dict[int, torch.Tensor], stream=None):
        """G[t]: upstream gradient of H_t (fp32).  Fills dW, da, dq per relation and dH0 per node type."""
        g = self.g
        grads = {}
        for t in self.rels_into:
            grads[t] = hb.heta_act_bwd(self.act, self.H[t], G[t], self._Gact[t], stream=stream) if self.relu else G[t]
        written = set()
        for r in self.rels:
            s, t, _ = g.rels[r]
            hb.heta_rel_attn_bwd(g, r, self.Z[r], self.el[r], self.er[r], self.slope, self.smax[r], self.sinv[r],
                                 self.O[r], grads[t], self.dZ[r], self.d_el[r], self.d_er[r], o_pos=self.Opos[r],
                                 stream=stream)
        # el = <H0_s, wa> reaches the source type's table and, through wa, W_r and a_r; er = <H0_t, q> reaches the
        # destination type's table and gives dq: per node type, all of them in one pass over its table
        for t, sets in self._score_sets.items():
            for i in range(0, len(sets), _MAX_SETS):
                part = sets[i:i + _MAX_SETS]
                hb.heta_attn_score_bwd_multi(g, self.tables[t], [self.wa[r] if src else self.q[r] for r, src in part],
                                             [self.d_el[r] if src else self.d_er[r] for r, src in part], dx=self.dH0[t],
                                             beta=1.0 if t in written else 0.0,
                                             dvecs=[self.dwa[r] if src else self.dq[r] for r, src in part], stream=stream)
                written.add(t)
        for s, rs in self.rels_from.items():
            for i in range(0, len(rs), _MAX_BATCH):
                part = rs[i:i + _MAX_BATCH]
                hb.heta_project_wgrad_batch(g, [self.tables[s]] * len(part), [self.dZ[r] for r in part],
                                            [self.dW[r] for r in part], gout_two_terms=self.two_terms, stream=stream)
                for r in part:
                    hb.heta_attn_fold_bwd(self.W[r], self.a[r], self.dwa[r], dW=self.dW[r], beta=1.0, da=self.da[r],
                                          stream=stream)
                hb.heta_project_sum([self.dZ[r] for r in part], [self.W[r] for r in part], self.dH0[s], trans_w=True,
                                    beta=1.0 if s in written else 0.0, stream=stream, graph=self.g)
                written.add(s)
        return self.dW, self.da, self.dq, self.dH0
