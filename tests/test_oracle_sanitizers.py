"""The C part of the oracle under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only): the file is
compiled, unchanged, with `-fsanitize=address,undefined` into a small driver program, run in a subprocess
on inputs of the kinds the pin tests use (multi-edges, empty rows, an empty relation, a row map, padded
tables, both reductions) with every buffer allocated at its exact size, and its outputs must equal those
of the ordinary build bit for bit."""
import os
import shutil
import struct
import subprocess

import numpy as np
import pytest

import oracle
from gen import rng

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def driver(tmp_path_factory):
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no gcc")
    exe = str(tmp_path_factory.mktemp("sanitize") / "oracle_sanitized")
    cmd = [gcc, "-std=c11", "-g", "-O1", "-fno-omit-frame-pointer", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           os.path.join(ROOT, "oracle", "heta_oracle.c"), os.path.join(ROOT, "oracle", "sanitize_driver.c"), "-o", exe]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0 and ("asan" in r.stderr or "ubsan" in r.stderr or "sanitize" in r.stderr):
        pytest.skip("this gcc has no sanitizer runtime: " + r.stderr[-200:])
    assert r.returncode == 0, r.stderr
    return exe


def _case(name, n_src, n_dst, n_edges, d, ld, mean, with_gid):
    g = rng.stream("tests/sanitize", name)
    src = g.integers(0, max(n_src, 1), size=n_edges, dtype=np.int32)
    dst = np.sort(g.integers(0, max(n_dst, 1), size=n_edges, dtype=np.int32))
    n_rows = 3 * n_src + 1 if with_gid else n_src
    table = g.standard_normal((n_rows, ld)).astype(np.float32)
    gid = g.permutation(n_rows)[:n_src].astype(np.int64) if with_gid else None
    dM = g.standard_normal((n_dst, d))
    return dict(name=name, n_src=n_src, n_dst=n_dst, src=src, dst=dst, d=d, ld=ld, mean=mean, table=table, gid=gid, dM=dM)


CASES = [
    _case("multi-edges-mean", 40, 30, 500, 7, 7, 1, False),
    _case("padded-rows-sum", 25, 60, 200, 5, 8, 0, False),          # many empty destination rows, ld > d
    _case("row-map", 30, 20, 300, 12, 16, 1, True),
    _case("empty-relation", 10, 10, 0, 4, 4, 1, False),
    _case("one-destination-hub", 50, 1, 2000, 3, 3, 1, False),
    _case("no-destinations", 5, 0, 0, 4, 4, 0, False),
]


@pytest.mark.parametrize("c", CASES, ids=[c["name"] for c in CASES])
def test_oracle_c_code_is_clean_under_asan_and_ubsan(driver, tmp_path, c):
    n_edges = c["src"].size
    fin, fout = str(tmp_path / "in.bin"), str(tmp_path / "out.bin")
    with open(fin, "wb") as f:
        f.write(struct.pack("8q", n_edges, c["n_src"], c["n_dst"], c["table"].shape[0], c["ld"], c["d"], int(c["gid"] is not None), c["mean"]))
        f.write(c["src"].tobytes()); f.write(c["dst"].tobytes()); f.write(c["table"].tobytes())
        if c["gid"] is not None:
            f.write(c["gid"].tobytes())
        f.write(np.ascontiguousarray(c["dM"], dtype=np.float64).tobytes())
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")
    r = subprocess.run([driver, fin, fout], capture_output=True, text=True, env=env, timeout=120)
    assert r.returncode == 0 and "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr, r.stderr[-2000:]
    raw = open(fout, "rb").read()
    n_s, n_t, d = c["n_src"], c["n_dst"], c["d"]
    off = 0

    def take(dtype, count):
        nonlocal off
        a = np.frombuffer(raw, dtype=dtype, count=count, offset=off)
        off += a.nbytes
        return a
    deg, M, dH0 = take(np.int64, n_t), take(np.float64, n_t * d).reshape(n_t, d), take(np.float64, n_s * d).reshape(n_s, d)
    colptr, row = take(np.int64, n_s + 1), take(np.int32, n_edges)
    op = "mean" if c["mean"] else "sum"
    assert np.array_equal(deg, oracle.in_degree(c["src"], c["dst"], n_t))
    assert np.array_equal(M, oracle.aggregate_fwd(c["src"], c["dst"], n_t, c["table"], op, gid=c["gid"], d=d))
    assert np.array_equal(dH0, oracle.aggregate_bwd(c["src"], c["dst"], n_s, n_t, c["dM"], op))
    rc, rr = oracle.csc(c["src"], c["dst"], n_s)
    assert np.array_equal(colptr, rc) and np.array_equal(row, rr)
