"""GPU parity of the sparse Adam step of learnable tables against the fp64 oracle.

fp32 table: the kernel evaluates Adam's Algorithm 1 in fp32 (one sqrt, one division per element):
|got - ref| <= 1e-5 * max(1, |ref|) per element after several steps.  bf16 table: the parameter is
rounded to bf16 after every step, so after T steps it may differ from the fp64 trajectory by T
roundings of 2^-9 relative: checked to 2e-2 (the storage tolerance) and, tightly, against the oracle
stepped from the GPU's own previous bf16 state.  States (fp32) are checked to 1e-5 in both modes.
"""
import numpy as np
import pytest
import torch

import oracle
import paper_2408_09697_amd as heta
from gen import rng
from tests.harness import dev_table

pytestmark = pytest.mark.gpu


def close(got, ref, tol, what):
    err = np.abs(got.astype(np.float64) - ref) / np.maximum(1.0, np.abs(ref))
    assert np.isfinite(got).all() and err.max() <= tol, f"{what}: {err.max():.3e} > {tol:.1e}"


@pytest.mark.parametrize("n_rows,d,n_ids,pad", [(3000, 128, 1700, 4), (500, 768, 500, 4), (1000, 7, 333, 1), (64, 300, 1, 4),
                                                (4096, 64, 0, 4)])
@pytest.mark.parametrize("storage", ["f32", "bf16"])
def test_sparse_adam_matches_the_oracle(n_rows, d, n_ids, pad, storage):
    g = rng.stream("tests", f"adam{n_rows}x{d}")
    theta0 = rng.uniform_table(n_rows, d, -0.1, 0.1, "tests", f"adam-theta{n_rows}")
    if storage == "bf16":
        theta0 = rng.round_to_bf16(theta0)
    table = dev_table(theta0, storage, 8 if storage == "bf16" and pad > 1 else pad)
    m = torch.zeros((n_rows, (d + pad - 1) // pad * pad), dtype=torch.float32, device="cuda")[:, :d]
    v = torch.zeros_like(m)
    ref_t, ref_m, ref_v = theta0.astype(np.float64), np.zeros((n_rows, d)), np.zeros((n_rows, d))
    lr, b1, b2, eps = 0.01, 0.9, 0.999, 1e-8
    for t in range(1, 5):
        ids = g.permutation(n_rows)[:n_ids].astype(np.int64)
        grad = g.standard_normal((n_ids, d)).astype(np.float32)
        before = table.float().cpu().numpy().astype(np.float64)
        heta.heta_sparse_adam(table, m, v, dev_table(grad, "f32", pad if d % pad == 0 else 1) if n_ids else torch.zeros((0, d), device="cuda"),
                              ids=torch.from_numpy(ids).cuda(), lr=lr, beta1=b1, beta2=b2, eps=eps, step=t)
        ref_t, ref_m, ref_v = oracle.sparse_adam_step(ref_t, ref_m, ref_v, ids, grad, lr, b1, b2, eps, t)
        got_t = table.float().cpu().numpy()
        close(m.cpu().numpy(), ref_m, 1e-5, "moment")
        close(v.cpu().numpy(), ref_v, 1e-5, "variance")
        if storage == "f32":
            close(got_t, ref_t, 1e-5, "table")
        else:
            close(got_t, ref_t, 2e-2, "table (trajectory)")
            # one step from the GPU's own previous state: only this step's rounding to bf16 remains
            one, _, _ = oracle.sparse_adam_step(before, ref_m_prev if t > 1 else np.zeros((n_rows, d)),
                                                ref_v_prev if t > 1 else np.zeros((n_rows, d)), ids, grad, lr, b1, b2, eps, t)
            assert np.abs(got_t - one).max() <= 2.0 ** -8 * max(1.0, np.abs(one).max())
        untouched = np.setdiff1d(np.arange(n_rows), ids)
        assert np.array_equal(got_t[untouched], before[untouched].astype(np.float32))
        ref_m_prev, ref_v_prev = ref_m, ref_v


def test_sparse_adam_identity_ids_and_argument_checks():
    n, d = 257, 32
    theta0 = rng.normal_table(n, d, "tests", "adam-id")
    table = dev_table(theta0, "f32", 4)
    m = torch.zeros((n, d), dtype=torch.float32, device="cuda")
    v = torch.zeros_like(m)
    grad = rng.normal_table(100, d, "tests", "adam-idg")
    heta.heta_sparse_adam(table, m, v, dev_table(grad, "f32", 4), ids=None, lr=0.05, step=1)
    ref, _, _ = oracle.sparse_adam_step(theta0, np.zeros((n, d)), np.zeros((n, d)), np.arange(100), grad, 0.05, 0.9, 0.999, 1e-8, 1)
    close(table.cpu().numpy(), ref, 1e-5, "identity ids")
    with pytest.raises(heta.HetaError):
        heta.heta_sparse_adam(table, m, v, dev_table(grad, "f32", 4), step=0)
    with pytest.raises(heta.HetaError):
        heta.heta_sparse_adam(table, m, v, dev_table(grad, "f32", 4), beta1=1.0)
    with pytest.raises(heta.HetaError):   # more gradient rows than table rows without ids
        heta.heta_sparse_adam(table, m, v, torch.zeros((n + 1, d), device="cuda"))


def test_sparse_adam_skips_row_ids_outside_the_table():
    """An id outside [0, n_table_rows) is ignored by the kernel: the listed valid rows are updated as if the
    bad entries were absent, nothing else changes (heta_check_ids is the call that reports such ids)."""
    n, d = 64, 16
    theta0 = rng.normal_table(n, d, "tests", "adam-oob")
    grad = rng.normal_table(6, d, "tests", "adam-oobg")
    ids = np.array([3, -1, 10, n, 1 << 40, 20], dtype=np.int64)
    table = dev_table(theta0, "f32", 4)
    guard = torch.full((4 * n, d), 7.0, dtype=torch.float32, device="cuda")   # m lives in the middle of a guarded buffer
    m, v = guard[n:2 * n], torch.zeros((n, d), dtype=torch.float32, device="cuda")
    m.zero_()
    heta.heta_sparse_adam(table, m, v, dev_table(grad, "f32", 4), ids=torch.from_numpy(ids).cuda(), lr=0.05, step=1)
    torch.cuda.synchronize()
    ok = np.array([0, 2, 5])
    ref, ref_m, _ = oracle.sparse_adam_step(theta0, np.zeros((n, d)), np.zeros((n, d)), ids[ok], grad[ok], 0.05, 0.9, 0.999, 1e-8, 1)
    close(table.cpu().numpy(), ref, 1e-5, "valid rows updated, others untouched")
    close(m.cpu().numpy(), ref_m, 1e-5, "moments")
    assert bool((guard[:n] == 7.0).all()) and bool((guard[2 * n:] == 7.0).all())
    with pytest.raises(heta.HetaError):
        heta.heta_check_ids(torch.from_numpy(ids).cuda(), n)


def test_sparse_adam_multi_equals_the_single_calls_bit_for_bit():
    """Twenty updates in one call (two launches' worth: fp32 and bf16 tables, with and without ids, widths that take the
    128-bit path and widths that do not, an empty one) against the same updates one by one, over three steps."""
    g = rng.stream("tests", "adam-multi")
    shapes = [(256, 128, None), (300, 768, 120), (128, 7, 50), (64, 300, None), (1000, 64, 0), (512, 256, 512)] * 3 + \
             [(1024, 1024, None), (77, 33, 20)]
    assert len(shapes) > 16

    def fresh():
        out = []
        for k, (n_rows, d, n_ids) in enumerate(shapes):
            storage = "bf16" if k % 2 else "f32"
            theta = rng.uniform_table(n_rows, d, -0.1, 0.1, "tests", f"adam-multi-theta{k}")
            table = dev_table(rng.round_to_bf16(theta) if storage == "bf16" else theta, storage, 8 if d % 8 == 0 else 1)
            pad = 4 if d % 4 == 0 else 1
            m = torch.zeros((n_rows, (d + pad - 1) // pad * pad), dtype=torch.float32, device="cuda")[:, :d]
            out.append((table, m, torch.zeros_like(m)))
        return out

    one, multi = fresh(), fresh()
    for step in range(1, 4):
        updates_one, updates_multi = [], []
        for k, (n_rows, d, n_ids) in enumerate(shapes):
            n = n_rows if n_ids is None else n_ids
            ids = None if n_ids is None else torch.from_numpy(g.permutation(n_rows)[:n_ids].astype(np.int64)).cuda()
            grad = dev_table(rng.normal_table(n, d, "tests", f"adam-multi-g{k}-{step}"), "f32", 4 if d % 4 == 0 else 1)
            updates_one.append((*one[k], grad, ids))
            updates_multi.append((*multi[k], grad, ids))
        for table, m, v, grad, ids in updates_one:
            heta.heta_sparse_adam(table, m, v, grad, ids=ids, lr=0.01, step=step)
        heta.heta_sparse_adam_multi(updates_multi, lr=0.01, step=step)
    torch.cuda.synchronize()
    for k in range(len(shapes)):
        for a, b, what in zip(one[k], multi[k], ("table", "m", "v")):
            assert torch.equal(a, b), f"item {k} {shapes[k]}: {what} differs"
    with pytest.raises(heta.HetaError):   # a bad item anywhere: nothing is launched, the call fails
        bad = list(updates_multi)
        t, m, v, grad, ids = bad[3]
        bad[3] = (t, m[: t.shape[0] // 2], v, grad, ids)
        heta.heta_sparse_adam_multi(bad, lr=0.01, step=1)
