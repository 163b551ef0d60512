"""Uploading a generated problem (gen.workloads.LayerProblem) to the device: tables and weights in their
storage type with 16-byte aligned rows, the graph handle, and a RafLayer over them.  Used by the
benchmark, the smoke check and the tests; no arithmetic of the method here."""
from __future__ import annotations

from typing import Optional

import numpy as np
import torch

from . import binding as heta
from .layer import RafLayer


def dev_table(x: np.ndarray, storage: str, pad_to: int = 1) -> torch.Tensor:
    """Uploads a float32 host table as fp32 or bf16; `pad_to` pads the leading dimension (in
    elements) so that rows start on 16-byte boundaries; the returned tensor is the [:, :d] view."""
    n, d = x.shape
    ld = (d + pad_to - 1) // pad_to * pad_to
    if storage == "bf16":
        from gen import rng  # the generators' rounding: the values are bf16-exact already, this only re-encodes them
        bits = rng.f32_to_bf16_bits(x)
        buf = torch.zeros((n, ld), dtype=torch.bfloat16, device="cuda")
        buf[:, :d] = torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)
    else:
        buf = torch.zeros((n, ld), dtype=torch.float32, device="cuda")
        buf[:, :d] = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).cuda()
    return buf[:, :d]


def relation_tuples(graph, declare_reverses: bool = True):
    """(src_type, dst_type, rowptr, col[, extras]) per relation for heta_graph_create; a relation the
    generator built as the exact transpose of an earlier one is declared as its reverse, so that the
    handle shares the index arrays of the pair."""
    names = [r.name for r in graph.relations]
    out = []
    for i, r in enumerate(graph.relations):
        base = getattr(r, "reverse_of", None)
        if declare_reverses and base in names[:i]:
            out.append((r.src_type, r.dst_type, r.rowptr, r.col, {"reverse_of": names.index(base)}))
        else:
            out.append((r.src_type, r.dst_type, r.rowptr, r.col))
    return out


def make_graph(p, declare_reverses: bool = True) -> heta.Graph:
    nts = [(t.num_nodes, t.feat_dim, int(t.learnable)) for t in p.graph.ntypes]
    return heta.heta_graph_create(nts, relation_tuples(p.graph, declare_reverses))


def make_layer(p, graph: Optional[heta.Graph] = None, rels=None, project_first=None) -> RafLayer:
    graph = make_graph(p) if graph is None else graph
    pad = 8 if p.storage == "bf16" else 4
    tables = [dev_table(t, p.storage, pad) for t in p.tables]
    W = [dev_table(w, p.storage, pad) for w in p.W]
    P = None if p.pre_proj is None else [dev_table(m, "f32", 4) for m in p.pre_proj]
    gid = None
    if p.src_gid is not None:
        gid = [None if g is None else torch.from_numpy(np.ascontiguousarray(g, dtype=np.int64)).cuda()
               for g in p.src_gid]
    op = heta.HETA_MEAN if p.op == "mean" else heta.HETA_SUM
    return RafLayer(graph, op, tables, W, p.d_out, pre_proj=P, src_gid=gid, relu=p.relu, rels=rels,
                         project_first=project_first)
