"""ctypes binding of libheta.so: the same entry points as include/heta.h, argument
marshalling only.  Device buffers are torch tensors (PyTorch-ROCm is used for device memory
and streams, nothing else); host index arrays are numpy arrays.  Every step of the path runs
inside the library's HIP kernels; there is no fallback: a missing library is an error.
"""
from __future__ import annotations

import ctypes
import struct
import os
from typing import List, Optional, Sequence

import numpy as np
import torch  # noqa: F401  (also makes sure the HIP runtime torch ships is the one in the process)

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "lib", "libheta.so")

HETA_OK = 0
HETA_ERR_INVALID_ARG, HETA_ERR_BAD_CSR, HETA_ERR_SHAPE = 1, 2, 3
HETA_ERR_UNSUPPORTED, HETA_ERR_OOM, HETA_ERR_DEVICE = 4, 5, 6
HETA_F32, HETA_BF16 = 0, 1
HETA_SUM, HETA_MEAN = 0, 1
HETA_ACT_NONE, HETA_ACT_RELU = 0, 1
HETA_PTRS_ON_DEVICE = 1

EXPORTS = ["heta_graph_create", "heta_graph_create_batch", "heta_graph_destroy", "heta_graph_get_csc", "heta_graph_get_degrees",
           "heta_feature_gather", "heta_check_ids", "heta_rel_aggregate_fwd", "heta_rel_aggregate_bwd",
           "heta_rel_aggregate_fwd_multi", "heta_rel_aggregate_bwd_multi",
           "heta_project", "heta_rel_project", "heta_rel_project_wgrad", "heta_cross_rel_reduce",
           "heta_act_bwd", "heta_sparse_adam_multi", "heta_last_error", "heta_version", "heta_profile_enable", "heta_profile_reset",
           "heta_profile_read", "heta_calibration_copy", "heta_calibration_mfma", "heta_cross_rel_project", "heta_cross_rel_project_bwd",
           "heta_cross_rel_project_wgrad", "heta_sparse_adam", "heta_project_batch",
           "heta_project_sum", "heta_project_wgrad_batch", "heta_attn_score", "heta_attn_score_bwd", "heta_attn_score_multi", "heta_attn_score_bwd_multi",
           "heta_rel_attn_fwd", "heta_rel_attn_bwd", "heta_sample_neighbors", "heta_unique_relabel",
           "heta_cross_rel_aggregate_project", "heta_meta_partition", "heta_sample_neighbors_batch",
           "heta_unique_relabel_batch", "heta_rel_aggregate_fwd_noalloc", "heta_attn_fold", "heta_attn_fold_bwd",
           "heta_graph_index_bytes"]
# process-wide switches for tests and measurements, declared in csrc/heta_test_hooks.h (not in the public header)
TEST_HOOKS = ["heta_projection_force_staged", "heta_ingest_force", "heta_projection_f32_native"]
HETA_NOALLOC_SCRATCH_BYTES = 32 << 20


class HetaError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"heta status {status}: {message}")
        self.status = status
        self.message = message


class _NType(ctypes.Structure):
    _fields_ = [("num_nodes", ctypes.c_int64), ("feat_dim", ctypes.c_int32), ("learnable", ctypes.c_int32)]


class _Relation(ctypes.Structure):
    _fields_ = [("src_type", ctypes.c_int32), ("dst_type", ctypes.c_int32), ("num_edges", ctypes.c_int64),
                ("csr_rowptr", ctypes.c_void_p), ("csr_col", ctypes.c_void_p),
                ("csc_colptr", ctypes.c_void_p), ("csc_row", ctypes.c_void_p), ("reverse_of", ctypes.c_int32)]


class _AdamItem(ctypes.Structure):
    _fields_ = [("table", ctypes.c_void_p), ("dt", ctypes.c_int32), ("ld_table", ctypes.c_int64), ("d", ctypes.c_int32),
                ("n_table_rows", ctypes.c_int64), ("m", ctypes.c_void_p), ("v", ctypes.c_void_p), ("ld_state", ctypes.c_int64),
                ("ids", ctypes.c_void_p), ("n", ctypes.c_int64), ("grad", ctypes.c_void_p), ("ld_grad", ctypes.c_int64)]


class _AggItem(ctypes.Structure):
    _fields_ = [("rel", ctypes.c_int32), ("d", ctypes.c_int32), ("inp", ctypes.c_void_p), ("ld_in", ctypes.c_int64),
                ("n_table_rows", ctypes.c_int64), ("src_gid", ctypes.c_void_p), ("out", ctypes.c_void_p),
                ("ld_out", ctypes.c_int64), ("beta", ctypes.c_float)]


_lib = None


def load_library() -> ctypes.CDLL:
    """Loads libheta.so (built in-tree by `paper_2408_09697_amd.build`); raises if it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is not built: run `python -m paper_2408_09697_amd.build` "
                          "(or __graft_entry__.build()) first; there is no fallback path")
    L = ctypes.CDLL(LIB_PATH)
    i32, i64, u32, vp, f32 = ctypes.c_int32, ctypes.c_int64, ctypes.c_uint32, ctypes.c_void_p, ctypes.c_float
    L.heta_graph_create.argtypes = [vp, i32, vp, i32, u32, ctypes.POINTER(vp)]
    L.heta_graph_destroy.argtypes = [vp]
    L.heta_graph_get_csc.argtypes = [vp, i32, vp, vp]
    L.heta_graph_get_degrees.argtypes = [vp, i32, vp]
    L.heta_feature_gather.argtypes = [vp, i32, i64, i32, i64, vp, i64, vp, i64, vp]
    L.heta_check_ids.argtypes = [vp, i64, i64, vp]
    L.heta_rel_aggregate_fwd.argtypes = [vp, i32, i32, vp, i32, i64, i32, i64, vp, vp, i32, i64, f32, vp]
    L.heta_rel_aggregate_fwd_noalloc.argtypes = L.heta_rel_aggregate_fwd.argtypes
    L.heta_rel_aggregate_bwd.argtypes = [vp, i32, i32, vp, i32, i64, i32, vp, i64, f32, vp]
    L.heta_rel_aggregate_fwd_multi.argtypes = [vp, i32, ctypes.POINTER(_AggItem), i32, i32, i32, vp]
    L.heta_rel_aggregate_bwd_multi.argtypes = [vp, i32, ctypes.POINTER(_AggItem), i32, i32, vp]
    L.heta_project.argtypes = [i64, vp, i32, i64, i32, vp, i32, i64, i32, i32, vp, vp, i32, i64, f32, vp]
    L.heta_rel_project.argtypes = [vp, i32, vp, i32, i64, i32, vp, i32, i64, i32, i32, vp, vp, i32, i64, f32, vp]
    L.heta_rel_project_wgrad.argtypes = [vp, i32, vp, i32, i64, i32, vp, i64, i32, vp, i64, f32, vp]
    L.heta_cross_rel_reduce.argtypes = [vp, i32, vp, i32, i64, i32, i32, vp, i64, vp]
    L.heta_act_bwd.argtypes = [i64, i32, i32, vp, i64, vp, i64, vp, i64, vp]
    for name in EXPORTS + TEST_HOOKS:
        getattr(L, name).restype = ctypes.c_int
    L.heta_last_error.restype = ctypes.c_char_p
    L.heta_last_error.argtypes = []
    L.heta_version.restype = ctypes.c_char_p
    L.heta_version.argtypes = []
    _lib = L
    return L


def _check(st: int) -> None:
    if st != HETA_OK:
        raise HetaError(st, load_library().heta_last_error().decode())


def _dt(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return HETA_F32
    if t.dtype == torch.bfloat16:
        return HETA_BF16
    raise TypeError(f"unsupported tensor dtype {t.dtype}")


def _dev(t: Optional[torch.Tensor], name: str, dtype=None) -> Optional[int]:
    """Device pointer of a tensor whose last dimension is contiguous."""
    if t is None:
        return None
    if not t.is_cuda:
        raise TypeError(f"{name} must be a device tensor")
    if t.numel() and t.dim() >= 1 and t.shape[-1] > 1 and t.stride(-1) != 1:
        raise TypeError(f"{name}: last dimension must be contiguous")
    if dtype is not None and t.dtype != dtype:
        raise TypeError(f"{name} must be {dtype}, got {t.dtype}")
    return t.data_ptr()


def _ld(t: torch.Tensor) -> int:
    return t.stride(0) if t.dim() == 2 else t.shape[-1]


def _stream(stream) -> Optional[int]:
    if stream is None:  # torch's current stream on the current device, without building a Stream object (3 us a call)
        return torch._C._cuda_getCurrentRawStream(torch.cuda.current_device())
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


class Graph:
    """Owner of a heta_graph handle."""

    def __init__(self, handle: int, ntypes, rel_meta):
        self._h = ctypes.c_void_p(handle)
        self.ntypes = ntypes          # [(num_nodes, feat_dim, learnable)]
        self.rels = rel_meta          # [(src_type, dst_type, num_edges)]

    @property
    def handle(self):
        if self._h is None:
            raise HetaError(HETA_ERR_INVALID_ARG, "graph already destroyed")
        return self._h

    def n_src(self, rel: int) -> int:
        return self.ntypes[self.rels[rel][0]][0]

    def n_dst(self, rel: int) -> int:
        return self.ntypes[self.rels[rel][1]][0]

    def meta_partition(self, root: int, k: int, p: int, metapaths=None) -> dict:
        """heta_meta_partition on this graph's own metagraph (nodes per type, edges per relation)."""
        return heta_meta_partition([n for n, _, _ in self.ntypes], [s for s, _, _ in self.rels],
                                   [t for _, t, _ in self.rels], [e for _, _, e in self.rels], root, k, p, metapaths)

    def destroy(self) -> None:
        if self._h is not None:
            heta_graph_destroy(self)

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def heta_version() -> str:
    return load_library().heta_version().decode()


def heta_last_error() -> str:
    return load_library().heta_last_error().decode()


_NT_PACK = struct.Struct("=qii")            # heta_ntype
_REL_PACK = struct.Struct("=iiqQQQQi4x")     # heta_relation
assert _NT_PACK.size == ctypes.sizeof(_NType) and _REL_PACK.size == ctypes.sizeof(_Relation)


def _marshal_graph(ntypes: Sequence[Sequence[int]], relations: Sequence[Sequence], flags: int):
    """The C arrays of one heta_graph_create call (packed byte buffers laid out as heta_ntype[] and
    heta_relation[]), what keeps their memory alive, and the relations' (s, t, E)."""
    nt = ctypes.create_string_buffer(_NT_PACK.size * max(1, len(ntypes)))
    for i, (n, d, l) in enumerate(ntypes):
        _NT_PACK.pack_into(nt, i * _NT_PACK.size, int(n), int(d), int(l))
    rl = ctypes.create_string_buffer(_REL_PACK.size * max(1, len(relations)))
    keep = []
    meta = []
    on_device = bool(flags & HETA_PTRS_ON_DEVICE)
    for i, relation in enumerate(relations):
        s, t, rowptr, col = relation[:4]
        extras = relation[4] if len(relation) > 4 else None
        csc = extras.get("csc") if extras else None
        ccp = crp = 0
        if on_device:
            rp = _dev(rowptr, "rowptr", torch.int64)
            cp = _dev(col, "col", torch.int32)
            n_e = int(col.numel())
            if csc is not None:
                ccp, crp = _dev(csc[0], "csc colptr", torch.int64), _dev(csc[1], "csc row", torch.int32)
                keep += list(csc)
        else:
            rowptr = np.ascontiguousarray(rowptr, dtype=np.int64)
            col = np.ascontiguousarray(col, dtype=np.int32)
            rp, cp, n_e = rowptr.__array_interface__["data"][0], col.__array_interface__["data"][0], int(col.size)
            if csc is not None:
                c0, c1 = np.ascontiguousarray(csc[0], dtype=np.int64), np.ascontiguousarray(csc[1], dtype=np.int32)
                ccp, crp = c0.__array_interface__["data"][0], c1.__array_interface__["data"][0]
                keep += [c0, c1]
        keep += [rowptr, col]
        s, t = int(s), int(t)
        _REL_PACK.pack_into(rl, i * _REL_PACK.size, s, t, n_e, rp or 0, cp or 0, ccp or 0, crp or 0,
                            int(extras.get("reverse_of", -1)) if extras else -1)
        meta.append((s, t, n_e))
    return nt, rl, keep, meta


def heta_graph_create(ntypes: Sequence[Sequence[int]], relations: Sequence[Sequence], flags: int = 0) -> Graph:
    """ntypes: (num_nodes, feat_dim, learnable) per node type.  relations: (src_type, dst_type,
    rowptr, col[, extras]) per relation, rowptr int64 [n_dst+1] and col int32 [E]; numpy arrays, or device
    tensors when flags has HETA_PTRS_ON_DEVICE.  extras: a dict with "csc": (colptr int64 [n_src+1], row int32 [E])
    and / or "reverse_of": index of the earlier relation this one is the exact transpose of."""
    L = load_library()
    nt, rl, keep, meta = _marshal_graph(ntypes, relations, flags)
    out = ctypes.c_void_p()
    _check(L.heta_graph_create(ctypes.addressof(nt) if len(ntypes) else None, len(ntypes),
                               ctypes.addressof(rl) if len(relations) else None, len(relations),
                               flags, ctypes.byref(out)))
    del keep
    return Graph(out.value, [tuple(int(x) for x in t) for t in ntypes], meta)


def heta_graph_create_batch(graphs: Sequence[Sequence], flags: int = 0) -> List[Graph]:
    """Several graphs (the blocks of one mini-batch) in one call: graphs[i] = (ntypes, relations) as for
    heta_graph_create; their small relations are built together on the device."""
    L = load_library()
    n = len(graphs)
    if n == 0:
        return []
    parts = [_marshal_graph(nts, rels, flags) for nts, rels in graphs]
    vp, i32 = ctypes.c_void_p, ctypes.c_int32
    L.heta_graph_create_batch.argtypes = [i32, vp, vp, vp, vp, ctypes.c_uint32, vp]
    nt_ptrs = (vp * n)(*[ctypes.addressof(p[0]) for p in parts])
    rl_ptrs = (vp * n)(*[ctypes.addressof(p[1]) for p in parts])
    n_nt = (i32 * n)(*[len(g[0]) for g in graphs])
    n_rl = (i32 * n)(*[len(g[1]) for g in graphs])
    outs = (vp * n)()
    _check(L.heta_graph_create_batch(n, nt_ptrs, n_nt, rl_ptrs, n_rl, flags, outs))
    return [Graph(outs[i], [tuple(int(x) for x in t) for t in graphs[i][0]], parts[i][3]) for i in range(n)]


def heta_graph_destroy(g: Graph) -> None:
    h, g._h = g._h, None
    if h is not None:
        _check(load_library().heta_graph_destroy(h))


def heta_graph_get_csc(g: Graph, rel: int):
    n_src, n_e = g.n_src(rel), g.rels[rel][2]
    colptr = np.zeros(n_src + 1, dtype=np.int64)
    row = np.zeros(n_e, dtype=np.int32)
    _check(load_library().heta_graph_get_csc(g.handle, rel, colptr.ctypes.data, row.ctypes.data))
    return colptr, row


def heta_graph_index_bytes(g: Graph) -> int:
    """Device bytes the handle holds for index data; arrays shared through reverse_of count once."""
    L = load_library()
    L.heta_graph_index_bytes.argtypes = [ctypes.c_void_p, ctypes.POINTER(ctypes.c_int64)]
    out = ctypes.c_int64()
    _check(L.heta_graph_index_bytes(g.handle, ctypes.byref(out)))
    return int(out.value)


def heta_graph_get_degrees(g: Graph, rel: int) -> np.ndarray:
    deg = np.zeros(g.n_dst(rel), dtype=np.int64)
    _check(load_library().heta_graph_get_degrees(g.handle, rel, deg.ctypes.data))
    return deg


def heta_feature_gather(table: torch.Tensor, gid: torch.Tensor, out: torch.Tensor, d: Optional[int] = None,
                        stream=None) -> torch.Tensor:
    d = table.shape[1] if d is None else d
    if table.dtype != out.dtype:
        raise TypeError("heta_feature_gather: table and out must have the same dtype")
    _check(load_library().heta_feature_gather(_dev(table, "table"), _dt(table), _ld(table), d, table.shape[0],
                                              _dev(gid, "gid", torch.int64), gid.numel(), _dev(out, "out"),
                                              _ld(out), _stream(stream)))
    return out


def heta_check_ids(ids: torch.Tensor, limit: int, stream=None) -> None:
    _check(load_library().heta_check_ids(_dev(ids, "ids", torch.int64), ids.numel(), limit, _stream(stream)))


def heta_rel_aggregate_fwd(g: Graph, rel: int, op: int, src_table: torch.Tensor, out: torch.Tensor,
                           d: Optional[int] = None, src_gid: Optional[torch.Tensor] = None, beta: float = 0.0,
                           stream=None) -> torch.Tensor:
    d = src_table.shape[1] if d is None else d
    if out.shape[0] < g.n_dst(rel):
        raise HetaError(HETA_ERR_SHAPE, "out has fewer rows than the relation has destinations")
    if src_gid is not None and src_gid.numel() < g.n_src(rel):
        raise HetaError(HETA_ERR_SHAPE, "src_gid has fewer entries than the relation has sources")
    _check(load_library().heta_rel_aggregate_fwd(
        g.handle, rel, op, _dev(src_table, "src_table"), _dt(src_table), _ld(src_table), d, src_table.shape[0],
        _dev(src_gid, "src_gid", torch.int64), _dev(out, "out"), _dt(out), _ld(out), beta, _stream(stream)))
    return out


def heta_rel_aggregate_fwd_noalloc(g: Graph, rel: int, op: int, src_table: torch.Tensor, out: torch.Tensor,
                                   d: Optional[int] = None, src_gid: Optional[torch.Tensor] = None,
                                   beta: float = 0.0, stream=None) -> torch.Tensor:
    """heta_rel_aggregate_fwd for callers that cannot allocate: fixed scratch, errors when it does not fit."""
    d = src_table.shape[1] if d is None else d
    if out.shape[0] < g.n_dst(rel):
        raise HetaError(HETA_ERR_SHAPE, "out has fewer rows than the relation has destinations")
    if src_gid is not None and src_gid.numel() < g.n_src(rel):
        raise HetaError(HETA_ERR_SHAPE, "src_gid has fewer entries than the relation has sources")
    _check(load_library().heta_rel_aggregate_fwd_noalloc(
        g.handle, rel, op, _dev(src_table, "src_table"), _dt(src_table), _ld(src_table), d, src_table.shape[0],
        _dev(src_gid, "src_gid", torch.int64), _dev(out, "out"), _dt(out), _ld(out), beta, _stream(stream)))
    return out


def heta_rel_aggregate_bwd(g: Graph, rel: int, op: int, grad_out: torch.Tensor, grad_src: torch.Tensor,
                           beta: float = 0.0, d: Optional[int] = None, stream=None) -> torch.Tensor:
    d = grad_out.shape[1] if d is None else d
    if grad_out.shape[0] < g.n_dst(rel) or grad_src.shape[0] < g.n_src(rel):
        raise HetaError(HETA_ERR_SHAPE, "gradient buffers have fewer rows than the relation needs")
    _check(load_library().heta_rel_aggregate_bwd(
        g.handle, rel, op, _dev(grad_out, "grad_out"), _dt(grad_out), _ld(grad_out), d,
        _dev(grad_src, "grad_src", torch.float32), _ld(grad_src), beta, _stream(stream)))
    return grad_src


def heta_rel_aggregate_fwd_multi(g: Graph, rels: Sequence[int], op: int, src_tables: Sequence[torch.Tensor],
                                 outs: Sequence[torch.Tensor], d: Optional[Sequence[int]] = None,
                                 src_gids: Optional[Sequence[Optional[torch.Tensor]]] = None,
                                 betas: Optional[Sequence[float]] = None, stream=None) -> None:
    """heta_rel_aggregate_fwd for several relations at once (relations of equal shape class share launches)."""
    n = len(rels)
    if n == 0:
        return
    items = (_AggItem * n)()
    for i, r in enumerate(rels):
        x, o = src_tables[i], outs[i]
        gid = None if src_gids is None else src_gids[i]
        if o.shape[0] < g.n_dst(r):
            raise HetaError(HETA_ERR_SHAPE, "out has fewer rows than the relation has destinations")
        if gid is not None and gid.numel() < g.n_src(r):
            raise HetaError(HETA_ERR_SHAPE, "src_gid has fewer entries than the relation has sources")
        if x.dtype != src_tables[0].dtype or o.dtype != outs[0].dtype:
            raise HetaError(HETA_ERR_INVALID_ARG, "the items of one call share their element types")
        it = items[i]
        it.rel, it.d = r, (x.shape[1] if d is None else d[i])
        it.inp, it.ld_in, it.n_table_rows = _dev(x, "src_table"), _ld(x), x.shape[0]
        it.src_gid = _dev(gid, "src_gid", torch.int64)
        it.out, it.ld_out = _dev(o, "out"), _ld(o)
        it.beta = 0.0 if betas is None else betas[i]
    _check(load_library().heta_rel_aggregate_fwd_multi(g.handle, n, items, op, _dt(src_tables[0]), _dt(outs[0]),
                                                       _stream(stream)))


def heta_rel_aggregate_bwd_multi(g: Graph, rels: Sequence[int], op: int, grad_outs: Sequence[torch.Tensor],
                                 grad_srcs: Sequence[torch.Tensor], betas: Optional[Sequence[float]] = None,
                                 d: Optional[Sequence[int]] = None, stream=None) -> None:
    """heta_rel_aggregate_bwd for several relations at once; no two items may share a grad_src."""
    n = len(rels)
    if n == 0:
        return
    items = (_AggItem * n)()
    for i, r in enumerate(rels):
        x, o = grad_outs[i], grad_srcs[i]
        if x.shape[0] < g.n_dst(r) or o.shape[0] < g.n_src(r):
            raise HetaError(HETA_ERR_SHAPE, "gradient buffers have fewer rows than the relation needs")
        if x.dtype != grad_outs[0].dtype:
            raise HetaError(HETA_ERR_INVALID_ARG, "the items of one call share their element types")
        it = items[i]
        it.rel, it.d = r, (x.shape[1] if d is None else d[i])
        it.inp, it.ld_in, it.n_table_rows, it.src_gid = _dev(x, "grad_out"), _ld(x), 0, None
        it.out, it.ld_out = _dev(o, "grad_src", torch.float32), _ld(o)
        it.beta = 0.0 if betas is None else betas[i]
    _check(load_library().heta_rel_aggregate_bwd_multi(g.handle, n, items, op, _dt(grad_outs[0]), _stream(stream)))


def _w_ld(W: torch.Tensor) -> int:
    return W.stride(0)


def heta_project(inp: torch.Tensor, W: torch.Tensor, out: torch.Tensor, trans_w: bool = False,
                 row_scale: Optional[torch.Tensor] = None, beta: float = 0.0, n_rows: Optional[int] = None,
                 stream=None) -> torch.Tensor:
    """out = beta*out + row_scale * inp @ (W^T if trans_w else W)."""
    n_rows = inp.shape[0] if n_rows is None else n_rows
    d_in = inp.shape[1]
    d_out = W.shape[0] if trans_w else W.shape[1]
    if (W.shape[1] if trans_w else W.shape[0]) != d_in:
        raise HetaError(HETA_ERR_SHAPE, "W does not match the input width")
    if out.shape[0] < n_rows or out.shape[1] < d_out or inp.shape[0] < n_rows:
        raise HetaError(HETA_ERR_SHAPE, "buffers too small for the projection")
    if row_scale is not None and row_scale.numel() < n_rows:
        raise HetaError(HETA_ERR_SHAPE, "row_scale too short")
    _check(load_library().heta_project(
        n_rows, _dev(inp, "in"), _dt(inp), _ld(inp), d_in, _dev(W, "W"), _dt(W), _w_ld(W), d_out, int(trans_w),
        _dev(row_scale, "row_scale", torch.float32), _dev(out, "out"), _dt(out), _ld(out), beta, _stream(stream)))
    return out


def heta_rel_project(g: Graph, rel: int, inp: torch.Tensor, W: torch.Tensor, out: torch.Tensor,
                     trans_w: bool = False, row_scale: Optional[torch.Tensor] = None, beta: float = 0.0,
                     stream=None) -> torch.Tensor:
    n = g.n_dst(rel)
    d_in = inp.shape[1]
    d_out = W.shape[0] if trans_w else W.shape[1]
    if (W.shape[1] if trans_w else W.shape[0]) != d_in:
        raise HetaError(HETA_ERR_SHAPE, "W does not match the input width")
    if inp.shape[0] < n or out.shape[0] < n or out.shape[1] < d_out:
        raise HetaError(HETA_ERR_SHAPE, "buffers too small for the projection")
    if row_scale is not None and row_scale.numel() < n:
        raise HetaError(HETA_ERR_SHAPE, "row_scale too short")
    _check(load_library().heta_rel_project(
        g.handle, rel, _dev(inp, "in"), _dt(inp), _ld(inp), d_in, _dev(W, "W"), _dt(W), _w_ld(W), d_out,
        int(trans_w), _dev(row_scale, "row_scale", torch.float32), _dev(out, "out"), _dt(out), _ld(out),
        beta, _stream(stream)))
    return out


def heta_rel_project_wgrad(g: Graph, rel: int, inp: torch.Tensor, gout: torch.Tensor, dW: torch.Tensor,
                           beta: float = 0.0, stream=None) -> torch.Tensor:
    n = g.n_dst(rel)
    d_in, d_out = inp.shape[1], gout.shape[1]
    if inp.shape[0] < n or gout.shape[0] < n or dW.shape[0] < d_in or dW.shape[1] < d_out:
        raise HetaError(HETA_ERR_SHAPE, "buffers too small for the weight gradient")
    _check(load_library().heta_rel_project_wgrad(
        g.handle, rel, _dev(inp, "in"), _dt(inp), _ld(inp), d_in, _dev(gout, "gout", torch.float32), _ld(gout),
        d_out, _dev(dW, "dW", torch.float32), _ld(dW), beta, _stream(stream)))
    return dW


def _ptr_array(ts, name, dtype=None):
    return (ctypes.c_void_p * len(ts))(*[_dev(t, name, dtype) for t in ts])


def _i64_array(vals):
    return (ctypes.c_int64 * len(vals))(*[int(v) for v in vals])


def _i32_array(vals):
    return (ctypes.c_int32 * len(vals))(*[int(v) for v in vals])


def heta_cross_rel_project(g: Graph, dst_type: int, ins: List[torch.Tensor], Ws: List[torch.Tensor],
                           out: torch.Tensor, act: int = HETA_ACT_NONE, beta: float = 0.0, stream=None) -> torch.Tensor:
    """out = act(beta*out + sum_p ins[p] @ Ws[p]) over the rows of dst_type."""
    n_rows = g.ntypes[dst_type][0]
    d_out = Ws[0].shape[1]
    if len(ins) != len(Ws) or not ins:
        raise HetaError(HETA_ERR_INVALID_ARG, "need one weight per input")
    for x, w in zip(ins, Ws):
        if x.shape[0] < n_rows or w.shape[0] != x.shape[1] or w.shape[1] != d_out or x.dtype != ins[0].dtype \
                or w.dtype != Ws[0].dtype:
            raise HetaError(HETA_ERR_SHAPE, "inputs / weights do not match")
    if out.shape[0] < n_rows or out.shape[1] < d_out:
        raise HetaError(HETA_ERR_SHAPE, "out too small")
    L = load_library()
    vp, i32, i64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64
    L.heta_cross_rel_project.argtypes = [vp, i32, i32, vp, i32, vp, vp, vp, i32, vp, i32, i32, vp, i64,
                                         ctypes.c_float, vp]
    a_in, a_w = _ptr_array(ins, "in"), _ptr_array(Ws, "W")
    ld_in, d_in, ld_w = _i64_array([_ld(x) for x in ins]), _i32_array([x.shape[1] for x in ins]), \
        _i64_array([w.stride(0) for w in Ws])
    _check(L.heta_cross_rel_project(g.handle, dst_type, len(ins), a_in, _dt(ins[0]), ld_in, d_in, a_w, _dt(Ws[0]),
                                    ld_w, d_out, act, _dev(out, "out", torch.float32), _ld(out), beta,
                                    _stream(stream)))
    return out


def heta_project_batch(ins: List[torch.Tensor], Ws: List[torch.Tensor], outs: List[torch.Tensor], trans_w: bool = False,
                       n_rows: Optional[int] = None, stream=None, graph: Optional["Graph"] = None) -> List[torch.Tensor]:
    """outs[p] = ins[p] @ (Ws[p]^T if trans_w else Ws[p]), independent products in one launch; graph: optional
    handle whose packing buffer the call may use."""
    n_rows = ins[0].shape[0] if n_rows is None else n_rows
    d_out = Ws[0].shape[0] if trans_w else Ws[0].shape[1]
    if not ins or len(ins) != len(Ws) or len(ins) != len(outs):
        raise HetaError(HETA_ERR_SHAPE, "bad arguments")
    for x, w, o in zip(ins, Ws, outs):
        if (w.shape[1] if trans_w else w.shape[0]) != x.shape[1] or (w.shape[0] if trans_w else w.shape[1]) != d_out \
                or x.shape[0] < n_rows or o.shape[0] < n_rows or o.shape[1] < d_out or x.dtype != ins[0].dtype \
                or w.dtype != Ws[0].dtype or o.dtype != outs[0].dtype:
            raise HetaError(HETA_ERR_SHAPE, "inputs / weights / outputs do not match")
    L = load_library()
    vp, i32, i64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64
    L.heta_project_batch.argtypes = [vp, i64, i32, vp, i32, vp, vp, vp, i32, vp, i32, i32, vp, i32, vp, vp]
    _check(L.heta_project_batch(graph.handle if graph is not None else None, n_rows, len(ins), _ptr_array(ins, "in"), _dt(ins[0]), _i64_array([_ld(x) for x in ins]),
                                _i32_array([x.shape[1] for x in ins]), _ptr_array(Ws, "W"), _dt(Ws[0]),
                                _i64_array([w.stride(0) for w in Ws]), d_out, int(trans_w), _ptr_array(outs, "out"),
                                _dt(outs[0]), _i64_array([_ld(o) for o in outs]), _stream(stream)))
    return outs


def heta_project_sum(ins: List[torch.Tensor], Ws: List[torch.Tensor], out: torch.Tensor, trans_w: bool = False,
                     beta: float = 0.0, n_rows: Optional[int] = None, stream=None, graph: Optional["Graph"] = None) -> torch.Tensor:
    """out = beta*out + sum_p ins[p] @ (Ws[p]^T if trans_w else Ws[p]), one contraction; graph: optional handle whose
    packing buffer the call may use."""
    n_rows = ins[0].shape[0] if n_rows is None else n_rows
    d_out = Ws[0].shape[0] if trans_w else Ws[0].shape[1]
    if not ins or len(ins) != len(Ws) or out.shape[0] < n_rows or out.shape[1] < d_out:
        raise HetaError(HETA_ERR_SHAPE, "bad arguments")
    for x, w in zip(ins, Ws):
        if (w.shape[1] if trans_w else w.shape[0]) != x.shape[1] or (w.shape[0] if trans_w else w.shape[1]) != d_out \
                or x.shape[0] < n_rows or x.dtype != ins[0].dtype or w.dtype != Ws[0].dtype:
            raise HetaError(HETA_ERR_SHAPE, "inputs / weights do not match")
    L = load_library()
    vp, i32, i64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64
    L.heta_project_sum.argtypes = [vp, i64, i32, vp, i32, vp, vp, vp, i32, vp, i32, i32, vp, i64, ctypes.c_float, vp]
    _check(L.heta_project_sum(graph.handle if graph is not None else None, n_rows, len(ins), _ptr_array(ins, "in"), _dt(ins[0]), _i64_array([_ld(x) for x in ins]),
                              _i32_array([x.shape[1] for x in ins]), _ptr_array(Ws, "W"), _dt(Ws[0]),
                              _i64_array([w.stride(0) for w in Ws]), d_out, int(trans_w), _dev(out, "out", torch.float32),
                              _ld(out), beta, _stream(stream)))
    return out


def heta_project_wgrad_batch(g: Graph, ins: List[torch.Tensor], gouts: List[torch.Tensor], dW: List[torch.Tensor],
                             beta: float = 0.0, gout_two_terms: bool = False, n_rows: Optional[int] = None,
                             stream=None) -> List[torch.Tensor]:
    """dW[p] = beta*dW[p] + ins[p]^T @ gouts[p] over n_rows rows, one launch."""
    n_rows = ins[0].shape[0] if n_rows is None else n_rows
    d_out = gouts[0].shape[1]
    if not ins or len(ins) != len(gouts) or len(ins) != len(dW):
        raise HetaError(HETA_ERR_SHAPE, "bad arguments")
    for x, go, w in zip(ins, gouts, dW):
        if x.shape[0] < n_rows or go.shape[0] < n_rows or go.shape[1] != d_out or w.shape[0] < x.shape[1] \
                or w.shape[1] < d_out or x.dtype != ins[0].dtype:
            raise HetaError(HETA_ERR_SHAPE, "inputs / gradients do not match")
    L = load_library()
    vp, i32, i64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64
    L.heta_project_wgrad_batch.argtypes = [vp, i64, i32, vp, i32, vp, vp, vp, vp, i32, vp, vp, ctypes.c_float, i32, vp]
    _check(L.heta_project_wgrad_batch(g.handle, n_rows, len(ins), _ptr_array(ins, "in"), _dt(ins[0]),
                                      _i64_array([_ld(x) for x in ins]), _i32_array([x.shape[1] for x in ins]),
                                      _ptr_array(gouts, "gout", torch.float32), _i64_array([_ld(x) for x in gouts]), d_out,
                                      _ptr_array(dW, "dW", torch.float32), _i64_array([_ld(w) for w in dW]), beta,
                                      int(gout_two_terms), _stream(stream)))
    return dW


def heta_cross_rel_project_bwd(g: Graph, dst_type: int, gout: torch.Tensor, Ws: List[torch.Tensor],
                               dM: List[torch.Tensor], stream=None) -> List[torch.Tensor]:
    """dM[p] = gout @ Ws[p]^T for every relation p into dst_type, one launch."""
    n_rows = g.ntypes[dst_type][0]
    d_out = gout.shape[1]
    if len(Ws) != len(dM) or not Ws or gout.shape[0] < n_rows:
        raise HetaError(HETA_ERR_SHAPE, "bad arguments")
    for w, m in zip(Ws, dM):
        if w.shape[1] != d_out or m.shape[0] < n_rows or m.shape[1] < w.shape[0] or w.dtype != Ws[0].dtype:
            raise HetaError(HETA_ERR_SHAPE, "weights / outputs do not match")
    L = load_library()
    vp, i32, i64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64
    L.heta_cross_rel_project_bwd.argtypes = [vp, i32, i32, vp, i64, i32, vp, i32, vp, vp, vp, i32, vp, vp]
    a_w, a_m = _ptr_array(Ws, "W"), _ptr_array(dM, "dM", dM[0].dtype)
    ld_w, d_in, ld_dm = _i64_array([w.stride(0) for w in Ws]), _i32_array([w.shape[0] for w in Ws]), \
        _i64_array([_ld(m) for m in dM])
    _check(L.heta_cross_rel_project_bwd(g.handle, dst_type, len(Ws), _dev(gout, "gout", torch.float32), _ld(gout),
                                        d_out, a_w, _dt(Ws[0]), ld_w, d_in, a_m, _dt(dM[0]), ld_dm, _stream(stream)))
    return dM


def heta_cross_rel_project_wgrad(g: Graph, dst_type: int, ins: List[torch.Tensor], gout: torch.Tensor,
                                 dW: List[torch.Tensor], beta: float = 0.0, gout_two_terms: bool = False,
                                 stream=None) -> List[torch.Tensor]:
    """dW[p] = beta*dW[p] + ins[p]^T @ gout for every relation p into dst_type, one launch."""
    n_rows = g.ntypes[dst_type][0]
    d_out = gout.shape[1]
    if len(ins) != len(dW) or not ins or gout.shape[0] < n_rows:
        raise HetaError(HETA_ERR_SHAPE, "bad arguments")
    for x, w in zip(ins, dW):
        if x.shape[0] < n_rows or w.shape[0] < x.shape[1] or w.shape[1] < d_out or x.dtype != ins[0].dtype:
            raise HetaError(HETA_ERR_SHAPE, "inputs / gradients do not match")
    L = load_library()
    vp, i32, i64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64
    L.heta_cross_rel_project_wgrad.argtypes = [vp, i32, i32, vp, i32, vp, vp, vp, i64, i32, vp, vp,
                                               ctypes.c_float, i32, vp]
    a_in, a_dw = _ptr_array(ins, "in"), _ptr_array(dW, "dW", torch.float32)
    ld_in, d_in, ld_dw = _i64_array([_ld(x) for x in ins]), _i32_array([x.shape[1] for x in ins]), \
        _i64_array([_ld(w) for w in dW])
    _check(L.heta_cross_rel_project_wgrad(g.handle, dst_type, len(ins), a_in, _dt(ins[0]), ld_in, d_in,
                                          _dev(gout, "gout", torch.float32), _ld(gout), d_out, a_dw, ld_dw, beta,
                                          int(gout_two_terms), _stream(stream)))
    return dW


def heta_cross_rel_reduce(g: Graph, dst_type: int, partials: List[torch.Tensor], out: torch.Tensor,
                          act: int = HETA_ACT_NONE, stream=None) -> torch.Tensor:
    n = g.ntypes[dst_type][0]
    d_out = partials[0].shape[1]
    ld = _ld(partials[0])
    for p in partials:
        if p.shape[0] < n or p.shape[1] != d_out or _ld(p) != ld:
            raise HetaError(HETA_ERR_SHAPE, "partials must share shape and leading dimension")
    if out.shape[0] < n or out.shape[1] < d_out:
        raise HetaError(HETA_ERR_SHAPE, "out too small")
    arr = (ctypes.c_void_p * len(partials))(*[_dev(p, "partial", torch.float32) for p in partials])
    _check(load_library().heta_cross_rel_reduce(g.handle, dst_type, ctypes.addressof(arr), len(partials), ld,
                                                d_out, act, _dev(out, "out", torch.float32), _ld(out),
                                                _stream(stream)))
    return out


def heta_act_bwd(act: int, h: Optional[torch.Tensor], grad_out: torch.Tensor, grad_in: torch.Tensor,
                 stream=None) -> torch.Tensor:
    n, d = grad_out.shape
    if grad_in.shape[0] < n or grad_in.shape[1] < d or (h is not None and (h.shape[0] < n or h.shape[1] < d)):
        raise HetaError(HETA_ERR_SHAPE, "buffers too small")
    _check(load_library().heta_act_bwd(n, d, act, _dev(h, "h", torch.float32), _ld(h) if h is not None else d,
                                       _dev(grad_out, "grad_out", torch.float32), _ld(grad_out),
                                       _dev(grad_in, "grad_in", torch.float32), _ld(grad_in), _stream(stream)))
    return grad_in


class _KernelStat(ctypes.Structure):
    _fields_ = [("name", ctypes.c_char * 48), ("launches", ctypes.c_int64), ("total_ms", ctypes.c_double),
                ("algorithmic_bytes", ctypes.c_double), ("flops", ctypes.c_double)]


def heta_profile_enable(on: bool) -> None:
    L = load_library()
    L.heta_profile_enable.argtypes = [ctypes.c_int32]
    _check(L.heta_profile_enable(int(bool(on))))


def heta_sparse_adam(table: torch.Tensor, m: torch.Tensor, v: torch.Tensor, grad: torch.Tensor,
                     ids: Optional[torch.Tensor] = None, lr: float = 1e-3, beta1: float = 0.9, beta2: float = 0.999,
                     eps: float = 1e-8, step: int = 1, d: Optional[int] = None, stream=None) -> torch.Tensor:
    """One Adam step on the rows `ids` (distinct) of a learnable table, in place."""
    d = table.shape[1] if d is None else d
    n = grad.shape[0]
    if ids is not None and ids.numel() < n:
        raise HetaError(HETA_ERR_SHAPE, "fewer ids than gradient rows")
    if m.shape[0] < table.shape[0] or v.shape[0] < table.shape[0]:
        raise HetaError(HETA_ERR_SHAPE, "optimizer states have fewer rows than the table")
    L = load_library()
    vp, i32, i64, f32 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_float
    L.heta_sparse_adam.argtypes = [vp, i32, i64, i32, i64, vp, vp, i64, vp, i64, vp, i64, f32, f32, f32, f32, i64, vp]
    _check(L.heta_sparse_adam(_dev(table, "table"), _dt(table), _ld(table), d, table.shape[0],
                              _dev(m, "m", torch.float32), _dev(v, "v", torch.float32), _ld(m),
                              _dev(ids, "ids", torch.int64), n, _dev(grad, "grad", torch.float32), _ld(grad),
                              lr, beta1, beta2, eps, int(step), _stream(stream)))
    return table


def heta_sparse_adam_multi(items: Sequence[Sequence], lr: float = 1e-3, beta1: float = 0.9, beta2: float = 0.999,
                           eps: float = 1e-8, step: int = 1, stream=None) -> None:
    """One Adam step on several tables in one call: items[i] = (table, m, v, grad, ids or None), each as for
    heta_sparse_adam (whole rows: d = table.shape[1])."""
    n = len(items)
    if n == 0:
        return
    arr = (_AdamItem * n)()
    for i, (table, m, v, grad, ids) in enumerate(items):
        rows = grad.shape[0]
        if ids is not None and ids.numel() < rows:
            raise HetaError(HETA_ERR_SHAPE, "fewer ids than gradient rows")
        if m.shape[0] < table.shape[0] or v.shape[0] < table.shape[0]:
            raise HetaError(HETA_ERR_SHAPE, "optimizer states have fewer rows than the table")
        arr[i] = _AdamItem(_dev(table, "table"), _dt(table), _ld(table), table.shape[1], table.shape[0],
                           _dev(m, "m", torch.float32), _dev(v, "v", torch.float32), _ld(m), _dev(ids, "ids", torch.int64),
                           rows, _dev(grad, "grad", torch.float32), _ld(grad))
    L = load_library()
    vp, i32, i64, f32 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_float
    L.heta_sparse_adam_multi.argtypes = [i32, vp, f32, f32, f32, f32, i64, vp]
    _check(L.heta_sparse_adam_multi(n, ctypes.addressof(arr), lr, beta1, beta2, eps, int(step), _stream(stream)))


def _scores(t: torch.Tensor, name: str, rows: int, heads: int) -> int:
    """Device pointer of a contiguous fp32 [rows, heads] score array."""
    if t.dtype != torch.float32 or not t.is_contiguous() or t.dim() != 2 or t.shape[0] < rows or t.shape[1] != heads:
        raise HetaError(HETA_ERR_SHAPE, f"{name} must be a contiguous fp32 [>= {rows}, {heads}] tensor")
    return _dev(t, name, torch.float32)


def heta_attn_score(x: torch.Tensor, vec: torch.Tensor, per_head: bool, score: torch.Tensor,
                    d: Optional[int] = None, stream=None) -> torch.Tensor:
    """score[i, k] = <x[i, head k's columns], vec[k]> (per_head) or <x[i, :], vec[k]>; vec is [heads, F] or [heads, d]."""
    d = x.shape[1] if d is None else d
    heads = vec.shape[0]
    if not vec.is_contiguous() or vec.shape[1] != (d // heads if per_head else d):
        raise HetaError(HETA_ERR_SHAPE, "vec must be contiguous [heads, d / heads] (per_head) or [heads, d]")
    L = load_library()
    vp, i32, i64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64
    L.heta_attn_score.argtypes = [vp, i32, i64, i64, i32, vp, i32, i32, vp, vp]
    _check(L.heta_attn_score(_dev(x, "x"), _dt(x), _ld(x), x.shape[0], d, _dev(vec, "vec", torch.float32), heads,
                             int(bool(per_head)), _scores(score, "score", x.shape[0], heads), _stream(stream)))
    return score


def heta_attn_fold(W: torch.Tensor, a: torch.Tensor, wa: torch.Tensor, stream=None) -> torch.Tensor:
    """wa[k, j] = sum_f W[j, k F + f] a[k, f]: the vector that turns the source score into a product with the input table."""
    d_in, d_out = W.shape
    heads = a.shape[0]
    if not a.is_contiguous() or a.shape[1] * heads != d_out or not wa.is_contiguous() or tuple(wa.shape) != (heads, d_in):
        raise HetaError(HETA_ERR_SHAPE, "a must be contiguous [heads, d_out / heads] and wa contiguous [heads, d_in]")
    L = load_library()
    vp, i32, i64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64
    L.heta_attn_fold.argtypes = [vp, i32, i64, i32, i32, vp, i32, vp, vp]
    _check(L.heta_attn_fold(_dev(W, "W"), _dt(W), _w_ld(W), d_in, d_out, _dev(a, "a", torch.float32), heads,
                            _dev(wa, "wa", torch.float32), _stream(stream)))
    return wa


def heta_attn_fold_bwd(W: torch.Tensor, a: torch.Tensor, dwa: torch.Tensor, dW: Optional[torch.Tensor] = None,
                       beta: float = 0.0, da: Optional[torch.Tensor] = None, stream=None) -> None:
    d_in, d_out = W.shape
    heads = a.shape[0]
    if not a.is_contiguous() or a.shape[1] * heads != d_out or not dwa.is_contiguous() or tuple(dwa.shape) != (heads, d_in):
        raise HetaError(HETA_ERR_SHAPE, "a must be contiguous [heads, d_out / heads] and dwa contiguous [heads, d_in]")
    if dW is not None and (dW.shape[0] < d_in or dW.shape[1] < d_out):
        raise HetaError(HETA_ERR_SHAPE, "dW is smaller than W")
    if da is not None and (not da.is_contiguous() or da.shape != a.shape):
        raise HetaError(HETA_ERR_SHAPE, "da must be contiguous and shaped like a")
    L = load_library()
    vp, i32, i64, f32 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_float
    L.heta_attn_fold_bwd.argtypes = [vp, i32, i64, i32, i32, vp, i32, vp, vp, i64, f32, vp, vp]
    _check(L.heta_attn_fold_bwd(_dev(W, "W"), _dt(W), _w_ld(W), d_in, d_out, _dev(a, "a", torch.float32), heads,
                                _dev(dwa, "dwa", torch.float32), _dev(dW, "dW", torch.float32),
                                _w_ld(dW) if dW is not None else 0, beta, _dev(da, "da", torch.float32), _stream(stream)))


def heta_attn_score_bwd(g: Graph, x: torch.Tensor, vec: torch.Tensor, per_head: bool, dscore: torch.Tensor,
                        dx: Optional[torch.Tensor] = None, beta: float = 0.0, dvec: Optional[torch.Tensor] = None,
                        d: Optional[int] = None, stream=None) -> None:
    d = x.shape[1] if d is None else d
    heads = vec.shape[0]
    if not vec.is_contiguous() or vec.shape[1] != (d // heads if per_head else d):
        raise HetaError(HETA_ERR_SHAPE, "vec must be contiguous [heads, d / heads] (per_head) or [heads, d]")
    if dvec is not None and (not dvec.is_contiguous() or dvec.shape != vec.shape):
        raise HetaError(HETA_ERR_SHAPE, "dvec must be contiguous and shaped like vec")
    if dx is not None and (dx.shape[0] < x.shape[0] or dx.shape[1] < d):
        raise HetaError(HETA_ERR_SHAPE, "dx is smaller than x")
    L = load_library()
    vp, i32, i64, f32 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_float
    L.heta_attn_score_bwd.argtypes = [vp, vp, i32, i64, i64, i32, vp, i32, i32, vp, vp, i64, f32, vp, vp]
    _check(L.heta_attn_score_bwd(g.handle, _dev(x, "x"), _dt(x), _ld(x), x.shape[0], d, _dev(vec, "vec", torch.float32),
                                 heads, int(bool(per_head)), _scores(dscore, "dscore", x.shape[0], heads),
                                 _dev(dx, "dx", torch.float32), _ld(dx) if dx is not None else 0, beta,
                                 _dev(dvec, "dvec", torch.float32), _stream(stream)))


def heta_attn_score_multi(x: torch.Tensor, vecs: Sequence[torch.Tensor], scores: Sequence[torch.Tensor],
                          d: Optional[int] = None, stream=None) -> None:
    """scores[s] = x @ vecs[s]^T for every set s in one pass over x (vecs[s]: [heads, d] fp32)."""
    if not vecs:
        return
    d = x.shape[1] if d is None else d
    heads = vecs[0].shape[0]
    for v in vecs:
        if not v.is_contiguous() or tuple(v.shape) != (heads, d):
            raise HetaError(HETA_ERR_SHAPE, "every vec must be contiguous [heads, d]")
    L = load_library()
    vp, i32, i64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64
    L.heta_attn_score_multi.argtypes = [vp, i32, i64, i64, i32, i32, vp, i32, vp, vp]
    sc = (ctypes.c_void_p * len(vecs))(*[_scores(t, "score", x.shape[0], heads) for t in scores])
    _check(L.heta_attn_score_multi(_dev(x, "x"), _dt(x), _ld(x), x.shape[0], d, len(vecs),
                                   _ptr_array(vecs, "vec", torch.float32), heads, sc, _stream(stream)))


def heta_attn_score_bwd_multi(g: Graph, x: torch.Tensor, vecs: Sequence[torch.Tensor], dscores: Sequence[torch.Tensor],
                              dx: Optional[torch.Tensor] = None, beta: float = 0.0,
                              dvecs: Optional[Sequence[Optional[torch.Tensor]]] = None, d: Optional[int] = None,
                              stream=None) -> None:
    """dx = beta dx + sum_s dscores[s] @ vecs[s];  dvecs[s] = dscores[s]^T @ x, all in one pass over x."""
    if not vecs:
        return
    d = x.shape[1] if d is None else d
    heads = vecs[0].shape[0]
    for v in vecs:
        if not v.is_contiguous() or tuple(v.shape) != (heads, d):
            raise HetaError(HETA_ERR_SHAPE, "every vec must be contiguous [heads, d]")
    if dvecs is not None:
        for v, dv in zip(vecs, dvecs):
            if dv is not None and (not dv.is_contiguous() or dv.shape != v.shape):
                raise HetaError(HETA_ERR_SHAPE, "dvec must be contiguous and shaped like vec")
    if dx is not None and (dx.shape[0] < x.shape[0] or dx.shape[1] < d):
        raise HetaError(HETA_ERR_SHAPE, "dx is smaller than x")
    L = load_library()
    vp, i32, i64, f32 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_float
    L.heta_attn_score_bwd_multi.argtypes = [vp, vp, i32, i64, i64, i32, i32, vp, i32, vp, vp, i64, f32, vp, vp]
    ds = (ctypes.c_void_p * len(vecs))(*[_scores(t, "dscore", x.shape[0], heads) for t in dscores])
    dv = None if dvecs is None else (ctypes.c_void_p * len(vecs))(*[_dev(t, "dvec", torch.float32) for t in dvecs])
    _check(L.heta_attn_score_bwd_multi(g.handle, _dev(x, "x"), _dt(x), _ld(x), x.shape[0], d, len(vecs),
                                       _ptr_array(vecs, "vec", torch.float32), heads, ds,
                                       _dev(dx, "dx", torch.float32), _ld(dx) if dx is not None else 0, beta, dv,
                                       _stream(stream)))


def heta_rel_attn_fwd(g: Graph, rel: int, z: torch.Tensor, el: torch.Tensor, er: torch.Tensor, slope: float,
                      out: torch.Tensor, beta: float = 0.0, smax: Optional[torch.Tensor] = None,
                      sinv: Optional[torch.Tensor] = None, out_pos: Optional[torch.Tensor] = None,
                      d: Optional[int] = None, stream=None) -> torch.Tensor:
    d = z.shape[1] if d is None else d
    heads = el.shape[1]
    if z.shape[0] < g.n_src(rel) or out.shape[0] < g.n_dst(rel):
        raise HetaError(HETA_ERR_SHAPE, "z / out have fewer rows than the relation needs")
    if out_pos is not None and (out_pos.shape[0] < g.n_dst(rel) or out_pos.dtype != out.dtype):
        raise HetaError(HETA_ERR_SHAPE, "out_pos must match out")
    L = load_library()
    vp, i32, i64, f32 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_float
    L.heta_rel_attn_fwd.argtypes = [vp, i32, vp, i32, i64, i32, i32, vp, vp, f32, vp, i32, i64, f32, vp, vp, vp, i64, vp]
    _check(L.heta_rel_attn_fwd(g.handle, rel, _dev(z, "z"), _dt(z), _ld(z), d, heads,
                               _scores(el, "el", g.n_src(rel), heads), _scores(er, "er", g.n_dst(rel), heads), slope,
                               _dev(out, "out"), _dt(out), _ld(out), beta,
                               None if smax is None else _scores(smax, "smax", g.n_dst(rel), heads),
                               None if sinv is None else _scores(sinv, "sinv", g.n_dst(rel), heads),
                               _dev(out_pos, "out_pos"), _ld(out_pos) if out_pos is not None else 0, _stream(stream)))
    return out


def heta_rel_attn_bwd(g: Graph, rel: int, z: torch.Tensor, el: torch.Tensor, er: torch.Tensor, slope: float,
                      smax: torch.Tensor, sinv: torch.Tensor, o: torch.Tensor, grad_out: torch.Tensor,
                      dz: torch.Tensor, d_el: torch.Tensor, d_er: torch.Tensor, o_pos: Optional[torch.Tensor] = None,
                      d: Optional[int] = None, stream=None) -> None:
    d = z.shape[1] if d is None else d
    heads = el.shape[1]
    n_src, n_dst = g.n_src(rel), g.n_dst(rel)
    if z.shape[0] < n_src or dz.shape[0] < n_src or o.shape[0] < n_dst or grad_out.shape[0] < n_dst:
        raise HetaError(HETA_ERR_SHAPE, "a buffer has fewer rows than the relation needs")
    if o_pos is not None and (o_pos.shape[0] < n_dst or o_pos.dtype != o.dtype or _ld(o_pos) != _ld(o)):
        raise HetaError(HETA_ERR_SHAPE, "o_pos must match o (rows, dtype, leading dimension)")
    L = load_library()
    vp, i32, i64, f32 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_float
    L.heta_rel_attn_bwd.argtypes = [vp, i32, vp, i32, i64, i32, i32, vp, vp, f32, vp, vp, vp, vp, i32, i64, vp, i64,
                                    vp, i64, vp, vp, vp]
    _check(L.heta_rel_attn_bwd(g.handle, rel, _dev(z, "z"), _dt(z), _ld(z), d, heads,
                               _scores(el, "el", n_src, heads), _scores(er, "er", n_dst, heads), slope,
                               _scores(smax, "smax", n_dst, heads), _scores(sinv, "sinv", n_dst, heads),
                               _dev(o, "o"), _dev(o_pos, "o_pos"), _dt(o), _ld(o),
                               _dev(grad_out, "grad_out", torch.float32), _ld(grad_out),
                               _dev(dz, "dz", torch.float32), _ld(dz), _scores(d_el, "del", n_src, heads),
                               _scores(d_er, "der", n_dst, heads), _stream(stream)))


def heta_cross_rel_aggregate_project(g: Graph, dst_type: int, rels: List[int], op: int, tables: List[torch.Tensor],
                                     Ws: List[torch.Tensor], out: torch.Tensor, act: int = HETA_ACT_NONE,
                                     src_gid: Optional[List[Optional[torch.Tensor]]] = None, stream=None) -> torch.Tensor:
    """out = act(sum_p agg_{rels[p]}(tables[p]) @ Ws[p]) over the rows of dst_type, one fused kernel (inference)."""
    n = len(rels)
    if n == 0 or len(tables) != n or len(Ws) != n or (src_gid is not None and len(src_gid) != n):
        raise HetaError(HETA_ERR_SHAPE, "bad arguments")
    d_out = Ws[0].shape[1]
    for t, w in zip(tables, Ws):
        if w.shape[0] != t.shape[1] or w.shape[1] != d_out or t.dtype != tables[0].dtype or w.dtype != tables[0].dtype:
            raise HetaError(HETA_ERR_SHAPE, "tables / weights do not match")
    if out.shape[0] < g.ntypes[dst_type][0] or out.shape[1] < d_out:
        raise HetaError(HETA_ERR_SHAPE, "out too small")
    L = load_library()
    vp, i32, i64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64
    L.heta_cross_rel_aggregate_project.argtypes = [vp, i32, i32, vp, i32, vp, i32, vp, vp, vp, vp, vp, vp, i32, i32, vp, i64, vp]
    gids = None
    if src_gid is not None:
        gids = (ctypes.c_void_p * n)(*[_dev(x, "src_gid", torch.int64) for x in src_gid])
    _check(L.heta_cross_rel_aggregate_project(
        g.handle, dst_type, n, _i32_array(rels), op, _ptr_array(tables, "table"), _dt(tables[0]),
        _i64_array([_ld(t) for t in tables]), _i32_array([t.shape[1] for t in tables]),
        _i64_array([t.shape[0] for t in tables]),
        None if gids is None else ctypes.addressof(gids), _ptr_array(Ws, "W"), _i64_array([w.stride(0) for w in Ws]),
        d_out, act, _dev(out, "out", torch.float32), _ld(out), _stream(stream)))
    return out


def heta_sample_neighbors(g: Graph, rel: int, dst_ids: torch.Tensor, fanout: int, seed: int, stream=None):
    """Samples up to `fanout` in-edges of every destination in dst_ids (device int64).  Returns
    (rowptr [n + 1] device int64, src_ids [n_sampled] device int64 global source ids)."""
    n = int(dst_ids.numel())
    rowptr = torch.empty(n + 1, dtype=torch.int64, device=dst_ids.device)
    src = torch.empty(max(1, n * fanout), dtype=torch.int64, device=dst_ids.device)
    n_sampled = ctypes.c_int64(0)
    L = load_library()
    vp, i32, i64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64
    L.heta_sample_neighbors.argtypes = [vp, i32, vp, i64, i32, ctypes.c_uint64, vp, vp, ctypes.POINTER(i64), vp]
    _check(L.heta_sample_neighbors(g.handle, rel, _dev(dst_ids, "dst_ids", torch.int64), n, fanout,
                                   ctypes.c_uint64(seed & ((1 << 64) - 1)), _dev(rowptr, "rowptr"), _dev(src, "src_ids"),
                                   ctypes.byref(n_sampled), _stream(stream)))
    return rowptr, src[:n_sampled.value]


def heta_sample_neighbors_batch(g: Graph, rels: Sequence[int], dst_ids: Sequence[torch.Tensor], fanout: int,
                                seeds: Sequence[int], stream=None):
    """heta_sample_neighbors for several relations in one call (one synchronisation).  Returns a list of
    (rowptr, src_ids) pairs, one per item."""
    n = len(rels)
    if n == 0:
        return []
    dev = dst_ids[0].device
    sizes = [int(d.numel()) for d in dst_ids]
    # one allocation for all row offsets and one for all source ids, cut into per-item views
    rp_all = torch.empty(sum(sizes) + n, dtype=torch.int64, device=dev)
    src_all = torch.empty(max(1, sum(sizes) * fanout), dtype=torch.int64, device=dev)
    rowptr, src, o_r, o_s = [], [], 0, 0
    for k in sizes:
        rowptr.append(rp_all[o_r:o_r + k + 1])
        src.append(src_all[o_s:o_s + k * fanout])
        o_r += k + 1
        o_s += k * fanout
    vp, i32, i64, u64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_uint64
    a_rels = (i32 * n)(*[int(r) for r in rels])
    a_dst = (vp * n)(*[_dev(d, "dst_ids", torch.int64) if d.numel() else None for d in dst_ids])
    a_n = (i64 * n)(*sizes)
    a_seed = (u64 * n)(*[int(x) & ((1 << 64) - 1) for x in seeds])
    a_rp = (vp * n)(*[r.data_ptr() for r in rowptr])
    a_src = (vp * n)(*[x.data_ptr() if x.numel() else None for x in src])
    a_cnt = (i64 * n)()
    L = load_library()
    L.heta_sample_neighbors_batch.argtypes = [vp, i32, vp, vp, vp, i32, vp, vp, vp, vp, vp]
    _check(L.heta_sample_neighbors_batch(g.handle, n, ctypes.addressof(a_rels), ctypes.addressof(a_dst), ctypes.addressof(a_n),
                                         int(fanout), ctypes.addressof(a_seed), ctypes.addressof(a_rp), ctypes.addressof(a_src),
                                         ctypes.addressof(a_cnt), _stream(stream)))
    return [(rowptr[i], src[i][:a_cnt[i]]) for i in range(n)]


def heta_unique_relabel_batch(groups: Sequence[Sequence[torch.Tensor]], id_limits: Sequence[int], stream=None):
    """heta_unique_relabel for several id sets in one call (one synchronisation).  groups[j] is the list of
    device int64 tensors of set j.  Returns a list of (unique_ids, [local per list]) pairs."""
    n = len(groups)
    if n == 0:
        return []
    dev = next((l.device for grp in groups for l in grp), torch.device("cuda"))
    totals = [sum(int(l.numel()) for l in grp) for grp in groups]
    uniq_all = torch.empty(max(1, sum(totals)), dtype=torch.int64, device=dev)
    local_all = torch.empty(max(1, sum(totals)), dtype=torch.int32, device=dev)
    uniq, local, lists, ptr, o_u, o_l = [], [], [], [0], 0, 0
    for grp, tot in zip(groups, totals):
        uniq.append(uniq_all[o_u:o_u + tot])
        o_u += tot
        loc = []
        for l in grp:
            k = int(l.numel())
            loc.append(local_all[o_l:o_l + k])
            o_l += k
            lists.append(l)
        local.append(loc)
        ptr.append(len(lists))
    m = max(1, len(lists))
    vp, i32, i64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64
    a_ptr = (i32 * (n + 1))(*ptr)
    a_lists = (vp * m)(*[_dev(l, "list", torch.int64) if l.numel() else None for l in lists])
    a_lens = (i64 * m)(*[int(l.numel()) for l in lists])
    a_local = (vp * m)(*[x.data_ptr() if x.numel() else None for loc in local for x in loc])
    a_lim = (i64 * n)(*[int(x) for x in id_limits])
    a_uniq = (vp * n)(*[u.data_ptr() if u.numel() else None for u in uniq])
    a_cnt = (i64 * n)()
    L = load_library()
    L.heta_unique_relabel_batch.argtypes = [i32, vp, vp, vp, vp, vp, vp, vp, vp]
    _check(L.heta_unique_relabel_batch(n, ctypes.addressof(a_ptr), ctypes.addressof(a_lists), ctypes.addressof(a_lens),
                                       ctypes.addressof(a_lim), ctypes.addressof(a_uniq), ctypes.addressof(a_cnt),
                                       ctypes.addressof(a_local), _stream(stream)))
    return [(uniq[j][:a_cnt[j]], local[j]) for j in range(n)]


def heta_unique_relabel(lists: List[torch.Tensor], id_limit: int, stream=None):
    """Ascending unique ids over all lists (device int64) and, per list, the positions of its entries in
    that array (device int32)."""
    dev = lists[0].device if lists else torch.device("cuda")
    total = sum(int(l.numel()) for l in lists)
    uniq = torch.empty(max(1, total), dtype=torch.int64, device=dev)
    local = [torch.empty(int(l.numel()), dtype=torch.int32, device=dev) for l in lists]
    n_unique = ctypes.c_int64(0)
    L = load_library()
    vp, i32, i64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64
    L.heta_unique_relabel.argtypes = [i32, vp, vp, i64, vp, ctypes.POINTER(i64), vp, vp]
    a_lists = (ctypes.c_void_p * max(1, len(lists)))(*[_dev(l, "list", torch.int64) for l in lists])
    a_local = (ctypes.c_void_p * max(1, len(lists)))(*[_dev(l, "local") for l in local])
    a_lens = (ctypes.c_int64 * max(1, len(lists)))(*[int(l.numel()) for l in lists])
    _check(L.heta_unique_relabel(len(lists), ctypes.addressof(a_lists), ctypes.addressof(a_lens), int(id_limit),
                                 _dev(uniq, "unique_ids"), ctypes.byref(n_unique), ctypes.addressof(a_local),
                                 _stream(stream)))
    return uniq[:n_unique.value], local


def heta_meta_partition(type_weight: Sequence[int], rel_src: Sequence[int], rel_dst: Sequence[int],
                        rel_weight: Sequence[int], root: int, k: int, p: int,
                        metapaths: Optional[Sequence[Sequence[int]]] = None) -> dict:
    """Meta-partitioning of the weighted metagraph (host only, no device needed).  Returns a dict of
    plain lists: sub_rel, sub_weight, sub_links, sub_part (per sub-metatree), part_weight, replica_of
    (per partition), rel_mask [p][n_rels], type_mask [p][n_types]."""
    n_types, n_rels = len(type_weight), len(rel_src)
    if len(rel_dst) != n_rels or len(rel_weight) != n_rels:
        raise HetaError(HETA_ERR_SHAPE, "rel_src, rel_dst and rel_weight must have one entry per relation")
    i32, i64, u8 = ctypes.c_int32, ctypes.c_int64, ctypes.c_uint8
    a_tw = (i64 * max(1, n_types))(*[int(x) for x in type_weight])
    a_rs = (i32 * max(1, n_rels))(*[int(x) for x in rel_src])
    a_rd = (i32 * max(1, n_rels))(*[int(x) for x in rel_dst])
    a_rw = (i64 * max(1, n_rels))(*[int(x) for x in rel_weight])
    paths = [list(m) for m in metapaths] if metapaths else []
    ptr = [0]
    for m in paths:
        ptr.append(ptr[-1] + len(m))
    flat = [int(i) for m in paths for i in m]
    a_mp = (i32 * len(ptr))(*ptr)
    a_mr = (i32 * max(1, len(flat)))(*flat)
    n_sub = i32(0)
    sub_rel, sub_part = (i32 * max(1, n_rels))(), (i32 * max(1, n_rels))()
    sub_weight, sub_links = (i64 * max(1, n_rels))(), (i64 * max(1, n_rels))()
    np_ = max(1, int(p))
    part_weight, replica_of = (i64 * np_)(), (i32 * np_)()
    rel_mask, type_mask = (u8 * max(1, np_ * n_rels))(), (u8 * max(1, np_ * n_types))()
    L = load_library()
    vp = ctypes.c_void_p
    L.heta_meta_partition.argtypes = [i32, vp, i32, vp, vp, vp, i32, i32, i32, i32, vp, vp, ctypes.POINTER(i32),
                                      vp, vp, vp, vp, vp, vp, vp, vp]
    _check(L.heta_meta_partition(n_types, ctypes.addressof(a_tw), n_rels, ctypes.addressof(a_rs), ctypes.addressof(a_rd),
                                 ctypes.addressof(a_rw), int(root), int(k), int(p), len(paths), ctypes.addressof(a_mp),
                                 ctypes.addressof(a_mr), ctypes.byref(n_sub), ctypes.addressof(sub_rel),
                                 ctypes.addressof(sub_weight), ctypes.addressof(sub_links), ctypes.addressof(sub_part),
                                 ctypes.addressof(part_weight), ctypes.addressof(replica_of), ctypes.addressof(rel_mask),
                                 ctypes.addressof(type_mask)))
    n = n_sub.value
    return {"sub_rel": list(sub_rel[:n]), "sub_weight": list(sub_weight[:n]), "sub_links": list(sub_links[:n]),
            "sub_part": list(sub_part[:n]), "part_weight": list(part_weight[:p]), "replica_of": list(replica_of[:p]),
            "rel_mask": [list(rel_mask[q * n_rels:(q + 1) * n_rels]) for q in range(p)],
            "type_mask": [list(type_mask[q * n_types:(q + 1) * n_types]) for q in range(p)]}


def heta_ingest_force(mode: int) -> None:
    L = load_library()
    L.heta_ingest_force.argtypes = [ctypes.c_int32]
    _check(L.heta_ingest_force(int(mode)))


def heta_projection_force_staged(on: bool) -> None:
    L = load_library()
    L.heta_projection_force_staged.argtypes = [ctypes.c_int32]
    _check(L.heta_projection_force_staged(1 if on else 0))


def heta_projection_f32_native(on: bool) -> None:
    L = load_library()
    L.heta_projection_f32_native.argtypes = [ctypes.c_int32]
    _check(L.heta_projection_f32_native(1 if on else 0))


def heta_calibration_copy(dst: torch.Tensor, src: torch.Tensor, stream=None) -> None:
    n_bytes = src.numel() * src.element_size()
    if dst.numel() * dst.element_size() < n_bytes or not src.is_contiguous() or not dst.is_contiguous():
        raise HetaError(HETA_ERR_SHAPE, "calibration copy needs contiguous buffers, dst at least as large as src")
    L = load_library()
    L.heta_calibration_copy.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p]
    _check(L.heta_calibration_copy(_dev(dst, "dst"), _dev(src, "src"), n_bytes, _stream(stream)))


def heta_calibration_mfma(dtype: int, iters: int, sink: torch.Tensor, stream=None, varying: bool = False) -> float:
    """Launches the register-only MFMA kernel (varying: operands that change from instruction to instruction); returns
    the flops of the launch."""
    L = load_library()
    L.heta_calibration_mfma.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_int64, ctypes.c_void_p, ctypes.c_int64,
                                        ctypes.POINTER(ctypes.c_double), ctypes.c_void_p]
    flops = ctypes.c_double(0.0)
    _check(L.heta_calibration_mfma(dtype, int(varying), iters, _dev(sink, "sink", torch.float32), sink.numel(),
                                   ctypes.byref(flops), _stream(stream)))
    return flops.value


def heta_profile_reset() -> None:
    _check(load_library().heta_profile_reset())


def heta_profile_read():
    """Per-kernel records: {name: {launches, total_ms, algorithmic_bytes, flops}}."""
    L = load_library()
    L.heta_profile_read.argtypes = [ctypes.c_void_p, ctypes.c_int32, ctypes.POINTER(ctypes.c_int32)]
    cap = 64
    arr = (_KernelStat * cap)()
    n = ctypes.c_int32(0)
    _check(L.heta_profile_read(ctypes.addressof(arr), cap, ctypes.byref(n)))
    out = {}
    for i in range(min(cap, n.value)):
        s = arr[i]
        out[s.name.decode()] = {"launches": int(s.launches), "total_ms": float(s.total_ms),
                                "algorithmic_bytes": float(s.algorithmic_bytes), "flops": float(s.flops)}
    return out
