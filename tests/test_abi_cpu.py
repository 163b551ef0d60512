"""CPU-only checks of the C-ABI library: it loads, exports every symbol the header declares,
and rejects bad arguments on the host before any device call."""
import os
import re

import numpy as np
import pytest

import paper_2408_09697_amd as heta
from paper_2408_09697_amd import binding as hb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols(header=os.path.join("include", "heta.h")):
    text = open(os.path.join(ROOT, header)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(heta_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = hb.load_library()
    names = declared_symbols()
    assert len(names) >= 15
    for n in names:
        assert hasattr(lib, n), f"{n} declared in heta.h but not exported"
    assert sorted(hb.EXPORTS) == names
    # the process-wide test switches live in an internal header, outside the public ABI, and are exported too
    hooks = declared_symbols(os.path.join("paper_2408_09697_amd", "csrc", "heta_test_hooks.h"))
    assert sorted(hb.TEST_HOOKS) == hooks and not set(hooks) & set(names)
    for n in hooks:
        assert hasattr(lib, n), n
    assert heta.heta_version() == "0.1"


def test_binding_has_the_same_names():
    for n in declared_symbols():
        assert callable(getattr(heta, n)), n


NT = [(4, 8, 0), (3, 8, 1)]


def _create(rels, nts=NT):
    return heta.heta_graph_create(nts, rels)


@pytest.mark.parametrize("rowptr,col,status,needle", [
    ([1, 1, 2, 2], [0, 1], hb.HETA_ERR_BAD_CSR, "rowptr[0]"),
    ([0, 2, 1, 2], [0, 1], hb.HETA_ERR_BAD_CSR, "decreases"),
    ([0, 1, 1, 3], [0, 1], hb.HETA_ERR_BAD_CSR, "num_edges"),
    ([0, 1, 2, 2], [0, 4], hb.HETA_ERR_BAD_CSR, "outside"),
    ([0, 1, 2, 2], [-1, 0], hb.HETA_ERR_BAD_CSR, "outside"),
])
def test_malformed_csr_is_rejected_on_the_host(rowptr, col, status, needle):
    # relation from type 0 (4 nodes) into type 1 (3 nodes)
    with pytest.raises(heta.HetaError) as ei:
        _create([(0, 1, np.array(rowptr, dtype=np.int64), np.array(col, dtype=np.int32))])
    assert ei.value.status == status
    assert needle in ei.value.message


def test_bad_node_types_and_counts():
    rp, col = np.array([0, 0, 0, 0], dtype=np.int64), np.zeros(0, dtype=np.int32)
    with pytest.raises(heta.HetaError) as ei:
        _create([(0, 2, rp, col)])
    assert ei.value.status == hb.HETA_ERR_INVALID_ARG
    with pytest.raises(heta.HetaError) as ei:
        _create([(0, 1, rp, col)], nts=[(-1, 8, 0), (3, 8, 0)])
    assert ei.value.status == hb.HETA_ERR_INVALID_ARG
    with pytest.raises(heta.HetaError) as ei:
        _create([(0, 1, rp, col)], nts=[(1 << 31, 8, 0), (3, 8, 0)])
    assert ei.value.status == hb.HETA_ERR_INVALID_ARG
    with pytest.raises(heta.HetaError) as ei:
        heta.heta_graph_create([], [])
    assert ei.value.status == hb.HETA_ERR_INVALID_ARG
    with pytest.raises(heta.HetaError) as ei:
        heta.heta_graph_create(NT, [(0, 1, rp, col)], flags=8)
    assert ei.value.status == hb.HETA_ERR_INVALID_ARG


def test_null_handle_calls_fail_cleanly():
    lib = hb.load_library()
    assert lib.heta_graph_destroy(None) == hb.HETA_OK
    assert lib.heta_graph_get_csc(None, 0, None, None) == hb.HETA_ERR_INVALID_ARG
    assert lib.heta_graph_get_degrees(None, 0, None) == hb.HETA_ERR_INVALID_ARG
    assert lib.heta_rel_aggregate_fwd(None, 0, 0, None, 0, 0, 0, 0, None, None, 0, 0, 0.0, None) == hb.HETA_ERR_INVALID_ARG
    assert lib.heta_rel_aggregate_bwd(None, 0, 0, None, 0, 0, 0, None, 0, 0.0, None) == hb.HETA_ERR_INVALID_ARG
    assert lib.heta_project(0, None, 0, 0, 0, None, 0, 0, 0, 0, None, None, 0, 0, 0.0, None) == hb.HETA_ERR_INVALID_ARG
    assert lib.heta_rel_project(None, 0, None, 0, 0, 0, None, 0, 0, 0, 0, None, None, 0, 0, 0.0, None) == hb.HETA_ERR_INVALID_ARG
    assert lib.heta_rel_project_wgrad(None, 0, None, 0, 0, 0, None, 0, 0, None, 0, 0.0, None) == hb.HETA_ERR_INVALID_ARG
    assert lib.heta_cross_rel_reduce(None, 0, None, 0, 0, 0, 0, None, 0, None) == hb.HETA_ERR_INVALID_ARG
    assert lib.heta_act_bwd(0, 0, 0, None, 0, None, 0, None, 0, None) == hb.HETA_ERR_INVALID_ARG
    assert lib.heta_feature_gather(None, 0, 0, 0, 0, None, 0, None, 0, None) == hb.HETA_ERR_INVALID_ARG
    assert b"null" in lib.heta_last_error().lower()


def test_project_shape_checks_happen_before_any_launch():
    lib = hb.load_library()
    one = 16  # fake, 4-byte aligned non-null addresses: rejected before they are ever dereferenced
    assert lib.heta_project(4, one, 0, 2, 8, one, 0, 8, 8, 0, None, one, 0, 8, 0.0, None) == hb.HETA_ERR_SHAPE   # ld_in < d_in
    assert lib.heta_project(4, one, 7, 8, 8, one, 0, 8, 8, 0, None, one, 0, 8, 0.0, None) == hb.HETA_ERR_INVALID_ARG  # dtype
    assert lib.heta_project(4, one + 2, 0, 8, 8, one, 0, 8, 8, 0, None, one, 0, 8, 0.0, None) == hb.HETA_ERR_INVALID_ARG  # align
    assert lib.heta_act_bwd(4, 8, 5, one, 8, one, 8, one, 8, None) == hb.HETA_ERR_INVALID_ARG


def test_null_arguments_of_the_later_entry_points_fail_cleanly():
    """Attention, sampler, fused forward, optimizer: a null handle or pointer is refused on the host."""
    import ctypes
    lib = hb.load_library()
    vp, i32, i64, f32, u64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_float, ctypes.c_uint64
    lib.heta_attn_score.argtypes = [vp, i32, i64, i64, i32, vp, i32, i32, vp, vp]
    assert lib.heta_attn_score(None, 0, 8, 4, 8, None, 2, 1, None, None) == hb.HETA_ERR_INVALID_ARG
    lib.heta_attn_score_bwd.argtypes = [vp, vp, i32, i64, i64, i32, vp, i32, i32, vp, vp, i64, f32, vp, vp]
    assert lib.heta_attn_score_bwd(None, None, 0, 8, 4, 8, None, 2, 1, None, None, 0, 0.0, None, None) == hb.HETA_ERR_INVALID_ARG
    lib.heta_rel_attn_fwd.argtypes = [vp, i32, vp, i32, i64, i32, i32, vp, vp, f32, vp, i32, i64, f32, vp, vp, vp, i64, vp]
    assert lib.heta_rel_attn_fwd(None, 0, None, 0, 8, 8, 2, None, None, 0.2, None, 0, 8, 0.0, None, None, None, 0, None) \
        == hb.HETA_ERR_INVALID_ARG
    lib.heta_rel_attn_bwd.argtypes = [vp, i32, vp, i32, i64, i32, i32, vp, vp, f32, vp, vp, vp, vp, i32, i64, vp, i64, vp, i64,
                                      vp, vp, vp]
    assert lib.heta_rel_attn_bwd(None, 0, None, 0, 8, 8, 2, None, None, 0.2, None, None, None, None, 0, 8, None, 8, None, 8,
                                 None, None, None) == hb.HETA_ERR_INVALID_ARG
    lib.heta_sample_neighbors.argtypes = [vp, i32, vp, i64, i32, u64, vp, vp, vp, vp]
    assert lib.heta_sample_neighbors(None, 0, None, 4, 5, 1, None, None, None, None) == hb.HETA_ERR_INVALID_ARG
    lib.heta_unique_relabel.argtypes = [i32, vp, vp, i64, vp, vp, vp, vp]
    assert lib.heta_unique_relabel(1, None, None, 10, None, None, None, None) == hb.HETA_ERR_INVALID_ARG
    n_unique = ctypes.c_int64(-1)
    assert lib.heta_unique_relabel(0, None, None, 10, None, ctypes.byref(n_unique), None, None) == hb.HETA_OK and n_unique.value == 0
    assert lib.heta_unique_relabel(0, None, None, (1 << 31) + 1, None, ctypes.byref(n_unique), None, None) == hb.HETA_ERR_SHAPE
    lib.heta_cross_rel_aggregate_project.argtypes = [vp, i32, i32, vp, i32, vp, i32, vp, vp, vp, vp, vp, vp, i32, i32, vp, i64, vp]
    assert lib.heta_cross_rel_aggregate_project(None, 0, 1, None, 0, None, 0, None, None, None, None, None, None, 8, 0, None, 8,
                                                None) == hb.HETA_ERR_INVALID_ARG
    lib.heta_sparse_adam.argtypes = [vp, i32, i64, i32, i64, vp, vp, i64, vp, i64, vp, i64, f32, f32, f32, f32, i64, vp]
    assert lib.heta_sparse_adam(None, 0, 8, 8, 4, None, None, 8, None, 2, None, 8, 1e-3, 0.9, 0.999, 1e-8, 1, None) \
        == hb.HETA_ERR_INVALID_ARG
    lib.heta_meta_partition.argtypes = [i32, vp, i32, vp, vp, vp, i32, i32, i32, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp]
    assert lib.heta_meta_partition(2, None, 1, None, None, None, 0, 1, 1, 0, None, None, None, None, None, None, None, None,
                                   None, None, None) == hb.HETA_ERR_INVALID_ARG
    assert "null argument" in hb.heta_last_error()
    lib.heta_sample_neighbors_batch.argtypes = [vp, i32, vp, vp, vp, i32, vp, vp, vp, vp, vp]
    assert lib.heta_sample_neighbors_batch(None, 2, None, None, None, 5, None, None, None, None, None) == hb.HETA_ERR_INVALID_ARG
    lib.heta_unique_relabel_batch.argtypes = [i32, vp, vp, vp, vp, vp, vp, vp, vp]
    assert lib.heta_unique_relabel_batch(2, None, None, None, None, None, None, None, None) == hb.HETA_ERR_INVALID_ARG
    assert lib.heta_unique_relabel_batch(0, None, None, None, None, None, None, None, None) == hb.HETA_OK


def test_relation_order_rule_on_the_shapes_it_was_measured_on():
    """Host logic: which relations the layer projects before aggregating.  On the academic-shaped graph
    (128 -> 256) only the relations from few sources into many, mostly empty, destination rows; every
    relation wider than the output; never a narrow relation into fewer rows."""
    from paper_2408_09697_amd.layer import project_first_pays as pays
    A, P, F, I = 1_100_000, 700_000, 60_000, 9_000
    c3 = [(A, P, 4_000_000), (P, P, 4_000_000), (P, F, 4_000_000), (A, I, 500_000), (P, A, 4_000_000), (F, P, 4_000_000),
          (I, A, 500_000)]
    assert [i for i, (s, t, e) in enumerate(c3) if pays(s, t, e, 128, 256, 4)] == [5, 6]
    assert [i for i, (s, t, e) in enumerate(c3) if pays(s, t, e, 128, 256, 2)] == [6]
    assert pays(500_000, 1_500_000, 5_000_000, 300, 256, 2) and pays(100_000, 500_000, 2_000_000, 789, 256, 2)
    assert not pays(1_500_000, 500_000, 5_000_000, 7, 256, 2) and not pays(800_000, 500_000, 4_000_000, 64, 256, 2)


def test_csc_and_reverse_arguments_are_checked_on_the_host():
    rp = np.array([0, 1, 2, 2], dtype=np.int64)           # type 0 (4 nodes) -> type 1 (3 nodes), 2 edges
    col = np.array([0, 3], dtype=np.int32)
    trp = np.array([0, 1, 1, 1, 2], dtype=np.int64)        # its transpose: type 1 -> type 0
    tcol = np.array([0, 1], dtype=np.int32)
    L = hb.load_library()
    import ctypes
    nt = (hb._NType * 2)(hb._NType(4, 8, 0), hb._NType(3, 8, 1))

    def create(structs):
        arr = (hb._Relation * len(structs))(*structs)
        out = ctypes.c_void_p()
        st = L.heta_graph_create(ctypes.addressof(nt), 2, ctypes.addressof(arr), len(structs), 0, ctypes.byref(out))
        return st, L.heta_last_error().decode(), out.value

    base = hb._Relation(0, 1, 2, rp.ctypes.data, col.ctypes.data, None, None, -1)
    # one CSC pointer without the other
    st, msg, h = create([hb._Relation(0, 1, 2, rp.ctypes.data, col.ctypes.data, trp.ctypes.data, None, -1)])
    assert st == hb.HETA_ERR_INVALID_ARG and "come together" in msg and h is None
    # reverse_of must name an earlier relation
    st, msg, h = create([hb._Relation(0, 1, 2, rp.ctypes.data, col.ctypes.data, None, None, 0)])
    assert st == hb.HETA_ERR_INVALID_ARG and "earlier relation" in msg and h is None
    # ... that is not itself a declared reverse
    rev = hb._Relation(1, 0, 2, trp.ctypes.data, tcol.ctypes.data, None, None, 0)
    st, msg, h = create([base, rev, hb._Relation(0, 1, 2, rp.ctypes.data, col.ctypes.data, None, None, 1)])
    assert st == hb.HETA_ERR_INVALID_ARG and "itself declared a reverse" in msg and h is None
    # node types that are not swapped
    st, msg, h = create([base, hb._Relation(0, 1, 2, rp.ctypes.data, col.ctypes.data, None, None, 0)])
    assert st == hb.HETA_ERR_BAD_CSR and "node types or edge counts" in msg and h is None
