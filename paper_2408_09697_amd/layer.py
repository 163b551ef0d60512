"""Sequencing of the library calls for one RAF layer on one GPU (forward and backward).

This module allocates device buffers with torch and issues the C-ABI calls in the order of
Algorithm 1 of the paper, one worker's share: relation-specific aggregation per relation,
projection of all relations into a destination type fused with the cross-relation sum, and
the local backward.  It computes nothing itself.
"""
from __future__ import annotations

from typing import Dict, List, Optional, Sequence

import torch

from . import binding as hb


def project_first_pays(n_src: int, n_dst: int, n_edges: int, d_r: int, d_out: int, elt_bytes: int) -> bool:
    """Whether relation r is cheaper projected first (Z'_r = H0_s W_r over the n_src source rows, aggregated
    at width d_out straight into H_t) than aggregated first (M_r over the n_dst destination rows, then
    projected).  Both orders give the same result (Eq. 1 is linear in H0); this is an estimate of the time
    of forward + backward from flops and bytes alone:

      aggregate first: 3 contractions over n_dst rows; gathers of d_r-wide rows per edge, forward and backward
      project first  : 3 contractions over n_src rows; gathers of d_out-wide rows per edge, the forward one
                       accumulating into H_t (rows with in-edges only), the backward one reading fp32 G_t

    priced at 5 TB/s (what the gather kernels reach), a gather from a table of at most 64 MB at twice
    that (it stays in the last-level cache), fp32 contractions at 120 TFLOP/s and bf16 ones at 500.
    Wider-than-output relations are always projected first (measured on the mixed-width workload, where
    the contraction over d_r > d_out is the slower one at any row count).  The typical case it finds:
    few source rows feeding many destination rows through few edges, where aggregating first spends
    three contractions on mostly empty rows of M_r."""
    if d_r > d_out:
        return True
    bw, flops = 5e12, (120e12 if elt_bytes == 4 else 500e12)
    b = float(elt_bytes)

    def contraction(rows, byt):
        return max(2.0 * rows * d_r * d_out / flops, byt / bw)

    def gather(table_rows, width, elt):
        return n_edges * width * elt / (bw * (2.0 if table_rows * width * elt <= 64e6 else 1.0))

    agg_first = (3.0 * contraction(n_dst, n_dst * d_r * b)
                 + gather(n_src, d_r, b) + n_dst * d_r * b / bw
                 + gather(n_dst, d_r, b) + n_src * d_r * 4.0 / bw)
    proj_first = (contraction(n_src, n_src * (d_r * b + d_out * b)) + contraction(n_src, n_src * (d_r * b + d_out * 4.0))
                  + contraction(n_src, n_src * (d_out * 4.0 + 2.0 * d_r * 4.0))
                  + gather(n_src, d_out, b) + 2.0 * min(n_edges, n_dst) * d_out * 4.0 / bw
                  + gather(n_dst, d_out, 4.0) + n_src * d_out * 4.0 / bw)
    return proj_first < agg_first


class RafLayer:
    """Device-resident state of one layer over a `binding.Graph`.

    tables[t]   : device [N_t, d_t] (fp32 or bf16), or None for types that are never a source
    W[r]        : device [d_r, d_out] in the storage dtype
    pre_proj[t] : optional fixed fp32 [d_t, d_shared] map applied to every table first
    src_gid[t]  : optional int64 map local source id -> table row (sampled blocks)
    """

    def __init__(self, graph: hb.Graph, op: int, tables: Sequence[Optional[torch.Tensor]],
                 W: Sequence[torch.Tensor], d_out: int, pre_proj: Optional[Sequence[torch.Tensor]] = None,
                 src_gid: Optional[Sequence[Optional[torch.Tensor]]] = None, relu: bool = False,
                 m_dtype: Optional[torch.dtype] = None, rels: Optional[Sequence[int]] = None,
                 project_first=None):
        self.g = graph
        self.op = op
        self.tables = list(tables)
        self.W = list(W)
        self.d_out = d_out
        self.pre_proj = None if pre_proj is None else list(pre_proj)
        self.src_gid = None if src_gid is None else list(src_gid)
        self.relu = relu
        self.act = hb.HETA_ACT_RELU if relu else hb.HETA_ACT_NONE
        self.rels = list(range(len(graph.rels))) if rels is None else list(rels)
        dev = self.W[self.rels[0]].device
        self.dev = dev
        n_types = len(graph.ntypes)
        self.rels_into: Dict[int, List[int]] = {}
        self.rels_from: Dict[int, List[int]] = {}
        for r in self.rels:
            s, t, _ = graph.rels[r]
            self.rels_into.setdefault(t, []).append(r)
            self.rels_from.setdefault(s, []).append(r)
        # width the aggregation of relation r runs at
        self.d_rel = {r: self.W[r].shape[0] for r in self.rels}
        if m_dtype is None:
            m_dtype = torch.bfloat16 if self.W[self.rels[0]].dtype == torch.bfloat16 else torch.float32
        self.m_dtype = m_dtype
        # H0 buffers only when a fixed per-type map produces them
        self.H0: List[Optional[torch.Tensor]] = [None] * n_types
        if self.pre_proj is not None:
            for t in range(n_types):
                if self.tables[t] is not None:
                    self.H0[t] = torch.empty((self.tables[t].shape[0], self.pre_proj[t].shape[1]),
                                             dtype=torch.float32, device=dev)
        # rows of every intermediate start on 16-byte boundaries (padded leading dimension), which
        # keeps awkward widths (7, 300, 789, ...) on the library's 128-bit paths
        def padded(n, d, dtype):
            q = 16 // dtype.itemsize
            return torch.empty((n, (d + q - 1) // q * q), dtype=dtype, device=dev)[:, :d]

        # Aggregation and projection commute (Eq. 1 is linear in H0).  A relation can be projected
        # first: Z'_r = H0_s W_r over the source rows, then aggregated at the output width straight
        # into H_t - no M_r, and the contraction runs over the source rows instead of the destination
        # rows.  project_first: None = per relation by project_first_pays (whole-table sources only: no
        # src_gid, no pre_proj); True = the relations wider than the output; False = none; or an
        # explicit collection of relations.
        auto = src_gid is None and pre_proj is None
        elt = self.W[self.rels[0]].element_size()
        if project_first is None:
            self.pf = set(r for r in self.rels if project_first_pays(graph.n_src(r), graph.n_dst(r), graph.rels[r][2],
                                                                    self.d_rel[r], d_out, elt)) if auto else set()
        elif isinstance(project_first, bool):
            self.pf = set(r for r in self.rels if self.d_rel[r] > d_out) if project_first else set()
        else:
            self.pf = set(int(r) for r in project_first) & set(self.rels)
        if self.pf and not auto:
            # the project-first calls below run over whole source tables: with a row map or a fixed per-type
            # map in front they would project the wrong rows
            raise hb.HetaError(hb.HETA_ERR_UNSUPPORTED, "project_first needs whole-table sources (no src_gid, no pre_proj)")
        self._pf_active = set()  # what the last forward actually used (the other call paths aggregate first)
        self._padded = padded
        self._m_shapes = {r: (graph.n_dst(r), self.d_rel[r]) for r in self.rels}
        self.M = {r: padded(graph.n_dst(r), self.d_rel[r], m_dtype) for r in self.rels if r not in self.pf}
        # dM_r, like the saved M_r, is an [n x d] intermediate that the backward aggregation re-reads once
        # per edge: it is kept in the storage type (bf16 tables -> bf16 dM_r, fp32 accumulation around it)
        self.dM = {r: padded(graph.n_dst(r), self.d_rel[r], m_dtype) for r in self.rels if r not in self.pf}
        self._dM32 = None  # fp32 dM_r for the per-relation call path, whose projection writes fp32
        self.Zp = {r: padded(graph.n_src(r), d_out, m_dtype) for r in self.pf}
        self.Ghat = {r: padded(graph.n_src(r), d_out, torch.float32) for r in self.pf}
        self.H = {t: torch.empty((graph.ntypes[t][0], d_out), dtype=torch.float32, device=dev)
                  for t in self.rels_into}
        self.dW = {r: torch.empty((self.d_rel[r], d_out), dtype=torch.float32, device=dev) for r in self.rels}
        self.dH0 = {s: padded(graph.ntypes[s][0], self.d_rel[rs[0]], torch.float32)
                    for s, rs in self.rels_from.items()}
        self.dtable: Dict[int, torch.Tensor] = {}
        if self.pre_proj is not None:
            for s in self.rels_from:
                self.dtable[s] = torch.empty((self.tables[s].shape[0], self.pre_proj[s].shape[0]),
                                             dtype=torch.float32, device=dev)
        self._Gact = ({t: torch.empty_like(h) for t, h in self.H.items()} if relu else {})

    def source(self, s: int) -> torch.Tensor:
        return self.H0[s] if self.pre_proj is not None else self.tables[s]

    def _pre_project(self, stream):
        if self.pre_proj is not None:
            for t, h0 in enumerate(self.H0):
                if h0 is not None:
                    hb.heta_project(self.tables[t], self.pre_proj[t], h0, stream=stream)

    def _aggregate_first_everywhere(self):
        """The per-relation and unfused call paths aggregate first: give every relation its M_r / dM_r."""
        self._pf_active = set()
        for r in self.rels:
            if r not in self.M:
                self.M[r] = self._padded(*self._m_shapes[r], self.m_dtype)
                self.dM[r] = self._padded(*self._m_shapes[r], self.m_dtype)

    def _aggregate(self, r: int, stream):
        s = self.g.rels[r][0]
        gid = None if self.src_gid is None else self.src_gid[s]
        hb.heta_rel_aggregate_fwd(self.g, r, self.op, self.source(s), self.M[r], d=self.d_rel[r], src_gid=gid,
                                  stream=stream)

    def _aggregate_all(self, rs: Sequence[int], stream):
        if len(rs) == 1:
            return self._aggregate(rs[0], stream)
        srcs = [self.g.rels[r][0] for r in rs]
        hb.heta_rel_aggregate_fwd_multi(self.g, rs, self.op, [self.source(s) for s in srcs], [self.M[r] for r in rs],
                                        d=[self.d_rel[r] for r in rs],
                                        src_gids=None if self.src_gid is None else [self.src_gid[s] for s in srcs],
                                        stream=stream)

    # ---- forward ------------------------------------------------------------------------------------
    def forward(self, stream=None) -> Dict[int, torch.Tensor]:
        """aggregate every relation, then one fused projection + cross-relation sum per type."""
        self._pre_project(stream)
        self._pf_active = set(self.pf)
        for s, rs in self.rels_from.items():  # Z'_r = H0_s W_r for all project-first relations out of s, one launch
            pfs = [r for r in rs if r in self.pf]
            for c in range(0, len(pfs), 8):
                part = pfs[c:c + 8]
                hb.heta_project_batch([self.source(s)] * len(part), [self.W[r] for r in part], [self.Zp[r] for r in part],
                                      n_rows=self.g.ntypes[s][0], stream=stream, graph=self.g)
        # the relation-specific aggregations of a layer do not depend on each other: one call for all of them
        # (relations of one shape class share launches, which is what a sampled block's small relations need)
        self._aggregate_all([r for r in self.rels if r not in self.pf], stream)
        for t, all_rs in self.rels_into.items():
            rs = [r for r in all_rs if r not in self.pf]
            pfs = [r for r in all_rs if r in self.pf]
            wrote = False
            for c in range(0, len(rs), 8):  # the library takes up to 8 relations per call
                part = rs[c:c + 8]
                last = c + 8 >= len(rs) and not pfs
                hb.heta_cross_rel_project(self.g, t, [self.M[r] for r in part], [self.W[r] for r in part], self.H[t],
                                          act=self.act if last else hb.HETA_ACT_NONE, beta=0.0 if c == 0 else 1.0,
                                          stream=stream)
                wrote = True
            for r in pfs:  # projected over the source rows above; aggregate at the output width into H_t
                hb.heta_rel_aggregate_fwd(self.g, r, self.op, self.Zp[r], self.H[t], d=self.d_out,
                                          beta=1.0 if wrote else 0.0, stream=stream)
                wrote = True
            if pfs and self.relu:
                hb.heta_cross_rel_reduce(self.g, t, [self.H[t]], self.H[t], act=hb.HETA_ACT_RELU, stream=stream)
        return self.H

    def forward_per_relation(self, stream=None) -> Dict[int, torch.Tensor]:
        """Same result with one projection per relation accumulating into H (beta = 1)."""
        self._aggregate_first_everywhere()
        self._pre_project(stream)
        for t, rs in self.rels_into.items():
            for k, r in enumerate(rs):
                self._aggregate(r, stream)
                hb.heta_rel_project(self.g, r, self.M[r], self.W[r], self.H[t], beta=0.0 if k == 0 else 1.0,
                                    stream=stream)
            if self.relu:
                hb.heta_cross_rel_reduce(self.g, t, [self.H[t]], self.H[t], act=hb.HETA_ACT_RELU, stream=stream)
        return self.H

    def forward_inference(self, stream=None) -> Dict[int, torch.Tensor]:
        """Forward only, one fused kernel per destination type (aggregation, projection, cross-relation sum
        and activation; no M_r is written, so no backward can follow).  Raises HetaError UNSUPPORTED for
        shapes the fused kernel does not take (d_out > 256, rows that are not 16-byte aligned)."""
        self._pre_project(stream)
        for t, rs in self.rels_into.items():
            if self.g.ntypes[t][0] == 0:
                continue
            for i in range(0, len(rs), 16):
                part = rs[i:i + 16]
                if i > 0:
                    raise hb.HetaError(hb.HETA_ERR_UNSUPPORTED, "more than 16 relations into one node type")
                srcs = [self.g.rels[r][0] for r in part]
                gids = None if self.src_gid is None else [self.src_gid[s] for s in srcs]
                hb.heta_cross_rel_aggregate_project(self.g, t, part, self.op, [self.source(s) for s in srcs],
                                                    [self.W[r] for r in part], self.H[t], act=self.act, src_gid=gids,
                                                    stream=stream)
        return self.H

    def forward_unfused(self, stream=None) -> Dict[int, torch.Tensor]:
        """Same result through explicit per-relation partials Z_r and heta_cross_rel_reduce."""
        self._aggregate_first_everywhere()
        self._pre_project(stream)
        for t, rs in self.rels_into.items():
            Z = []
            for r in rs:
                self._aggregate(r, stream)
                z = torch.empty_like(self.H[t])
                hb.heta_rel_project(self.g, r, self.M[r], self.W[r], z, stream=stream)
                Z.append(z)
            hb.heta_cross_rel_reduce(self.g, t, Z, self.H[t], act=self.act, stream=stream)
        return self.H

    # ---- backward: dZ = G; dW = M^T dZ; dM = dZ W^T; dH0 += CSC gather of dM ---------------------------
    def backward(self, G: Dict[int, torch.Tensor], stream=None, per_relation: bool = False):
        first_for_src = {s: True for s in self.rels_from}
        per_src: Dict[int, list] = {}  # source type -> [(relation, dM_r)] in the order of the sum
        for t, all_rs in self.rels_into.items():
            rs = [r for r in all_rs if r not in self._pf_active]
            pfs = [r for r in all_rs if r in self._pf_active]
            g = G[t]
            if self.relu:
                g = hb.heta_act_bwd(hb.HETA_ACT_RELU, self.H[t], G[t], self._Gact[t], stream=stream)
            dM = self.dM
            if per_relation:
                if self.m_dtype != torch.float32:
                    if self._dM32 is None:
                        self._dM32 = {r: self._padded(self.g.n_dst(r), self.d_rel[r], torch.float32) for r in self.rels}
                    dM = self._dM32
                for r in rs:
                    hb.heta_rel_project_wgrad(self.g, r, self.M[r], g, self.dW[r], stream=stream)
                    hb.heta_rel_project(self.g, r, g, self.W[r], dM[r], trans_w=True, stream=stream)
            else:
                for c in range(0, len(rs), 8):
                    part = rs[c:c + 8]
                    hb.heta_cross_rel_project_wgrad(self.g, t, [self.M[r] for r in part], g,
                                                    [self.dW[r] for r in part], stream=stream)
                    hb.heta_cross_rel_project_bwd(self.g, t, g, [self.W[r] for r in part],
                                                  [self.dM[r] for r in part], stream=stream)
            for r in rs:
                per_src.setdefault(self.g.rels[r][0], []).append((r, dM[r]))
            for r in pfs:  # dZ'_r = CSC gather of G_t over the source rows
                hb.heta_rel_aggregate_bwd(self.g, r, self.op, g, self.Ghat[r], d=self.d_out, stream=stream)
        # dH0_s = sum over the relations leaving s of the CSC gather of dM_r.  Round k takes the k-th relation
        # of every source type (their outputs are distinct, so one call covers them); the rounds follow each
        # other on the stream, which keeps the order of the sum over the relations of a type fixed.
        for k in range(max((len(v) for v in per_src.values()), default=0)):
            items = [(s, v[k]) for s, v in per_src.items() if k < len(v)]
            if len(items) == 1:
                s, (r, dm) = items[0]
                hb.heta_rel_aggregate_bwd(self.g, r, self.op, dm, self.dH0[s], beta=0.0 if k == 0 else 1.0, stream=stream)
            else:
                hb.heta_rel_aggregate_bwd_multi(self.g, [r for _, (r, _) in items], self.op, [dm for _, (_, dm) in items],
                                                [self.dH0[s] for s, _ in items], betas=[0.0 if k == 0 else 1.0] * len(items),
                                                stream=stream)
        for s in per_src:
            first_for_src[s] = False
        for s, rs in self.rels_from.items():  # per source type: dW_r = H0_s^T dZ'_r ; dH0_s += sum_r dZ'_r W_r^T
            pfs = [r for r in rs if r in self._pf_active]
            for c in range(0, len(pfs), 8):
                part = pfs[c:c + 8]
                # dZ'_r sums G over a source's out-edges: fed to the bf16 MFMA as two terms so that its size does not show in dW
                hb.heta_project_wgrad_batch(self.g, [self.source(s)] * len(part), [self.Ghat[r] for r in part],
                                            [self.dW[r] for r in part], gout_two_terms=True, n_rows=self.g.ntypes[s][0],
                                            stream=stream)
                hb.heta_project_sum([self.Ghat[r] for r in part], [self.W[r] for r in part], self.dH0[s], trans_w=True,
                                    beta=0.0 if first_for_src[s] else 1.0, n_rows=self.g.ntypes[s][0], stream=stream,
                                    graph=self.g)
                first_for_src[s] = False
        if self.pre_proj is not None:
            for s, gh in self.dH0.items():
                hb.heta_project(gh, self.pre_proj[s], self.dtable[s], trans_w=True, stream=stream)
        return self.dW, self.dH0, (self.dtable if self.pre_proj is not None else self.dH0)
