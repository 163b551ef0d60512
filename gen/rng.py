"""Seeded, stateless random streams for the synthetic inputs.

Every array of every workload is drawn from its own Philox stream whose key is a
hash of (master seed, workload name, array name, block index), so an array's
bytes do not depend on what else was generated, in which order, or on how many
threads filled it.  This module holds no arithmetic of the layer itself: it only
produces input data, and is the one piece shared by the CPU oracle's tests and
the GPU path's tests.
"""
from __future__ import annotations

import hashlib
from concurrent.futures import ThreadPoolExecutor

import numpy as np

MASTER_SEED = 20240809
_BLOCK_ROWS = 1 << 16


def _key(workload: str, name: str, block: int = 0, seed: int = MASTER_SEED) -> int:
    h = hashlib.sha256(f"{seed}|{workload}|{name}|{block}".encode()).digest()
    return int.from_bytes(h[:16], "little")


def stream(workload: str, name: str, block: int = 0, seed: int = MASTER_SEED) -> np.random.Generator:
    """A generator that depends only on (seed, workload, name, block)."""
    return np.random.Generator(np.random.Philox(key=_key(workload, name, block, seed)))


def _fill_blocks(n_rows: int, n_cols: int, workload: str, name: str, draw, seed: int) -> np.ndarray:
    out = np.empty((n_rows, n_cols), dtype=np.float32)
    n_blocks = (n_rows + _BLOCK_ROWS - 1) // _BLOCK_ROWS

    def work(b: int) -> None:
        r0 = b * _BLOCK_ROWS
        r1 = min(n_rows, r0 + _BLOCK_ROWS)
        g = stream(workload, name, b, seed)
        out[r0:r1] = draw(g, (r1 - r0, n_cols))

    if n_blocks <= 1:
        for b in range(n_blocks):
            work(b)
    else:
        with ThreadPoolExecutor(max_workers=8) as ex:
            list(ex.map(work, range(n_blocks)))
    return out


def normal_table(n_rows: int, n_cols: int, workload: str, name: str, seed: int = MASTER_SEED) -> np.ndarray:
    """[n_rows, n_cols] float32, i.i.d. N(0,1); filled block-wise (thread-count independent)."""
    return _fill_blocks(n_rows, n_cols, workload, name,
                        lambda g, shp: g.standard_normal(shp, dtype=np.float32), seed)


def uniform_table(n_rows: int, n_cols: int, lo: float, hi: float, workload: str, name: str,
                  seed: int = MASTER_SEED) -> np.ndarray:
    """[n_rows, n_cols] float32, i.i.d. U(lo, hi)."""
    lo32, w32 = np.float32(lo), np.float32(hi - lo)
    return _fill_blocks(n_rows, n_cols, workload, name,
                        lambda g, shp: g.random(shp, dtype=np.float32) * w32 + lo32, seed)


def small_int_table(n_rows: int, n_cols: int, lo: int, hi: int, workload: str, name: str,
                    seed: int = MASTER_SEED) -> np.ndarray:
    """[n_rows, n_cols] float32 holding integers in [lo, hi]: sums of such values are exact
    in fp32 (and the values themselves exact in bf16) while partial sums stay below 2**24,
    so results do not depend on the order of summation."""
    return _fill_blocks(n_rows, n_cols, workload, name,
                        lambda g, shp: g.integers(lo, hi + 1, size=shp).astype(np.float32), seed)


# ---- bf16 storage helpers (format conversion only) -------------------------------------------

def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest, ties to even); returns the uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    nan = (u & 0x7FFFFFFF) > 0x7F800000
    r = (u + (0x7FFF + ((u >> 16) & 1))) >> 16
    r = np.where(nan, (u >> 16) | 0x40, r)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bfloat16 bit patterns (uint16) to float32 exactly."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """float32 array whose every value is exactly representable in bfloat16."""
    return bf16_bits_to_f32(f32_to_bf16_bits(x))


# ---- counter-based tables: value = f(key, row, column), identical on host and device -----------
# Tables too large to build on the host (tens of GB) are filled on the GPU with torch integer
# ops; the host regenerates only the rows a test touches.  Integer mixing (splitmix64), one
# int -> float conversion and one fp32 multiply: no transcendental function, so both sides
# produce the same bits.  "normal": sum of four 16-bit uniforms, centred and scaled to unit
# variance; "embedding": one 16-bit uniform mapped to (-0.1, 0.1).

_SM_A, _SM_B, _SM_C = 0x9E3779B97F4A7C15, 0xBF58476D1CE4E5B9, 0x94D049BB133111EB
_NORMAL_SCALE = np.float32(1.0 / 37837.0)       # 1 / std of the sum of four uniforms on [0, 65535]
_EMB_SCALE = np.float32(0.1 / 65535.0)


def table_key(workload: str, name: str, seed: int = MASTER_SEED) -> int:
    return _key(workload, name, 0, seed) & ((1 << 63) - 1)


def hashed_rows(key: int, rows: np.ndarray, d: int, kind: str) -> np.ndarray:
    """float32 [len(rows), d] of the counter-based table `key` (host side)."""
    rows = np.asarray(rows, dtype=np.uint64)
    x = rows[:, None] * np.uint64(d) + np.arange(d, dtype=np.uint64)[None, :] + np.uint64(key)
    with np.errstate(over="ignore"):
        z = x + np.uint64(_SM_A)
        z = (z ^ (z >> np.uint64(30))) * np.uint64(_SM_B)
        z = (z ^ (z >> np.uint64(27))) * np.uint64(_SM_C)
        z = z ^ (z >> np.uint64(31))
    m = np.uint64(0xFFFF)
    if kind == "normal":
        s = (z & m) + ((z >> np.uint64(16)) & m) + ((z >> np.uint64(32)) & m) + ((z >> np.uint64(48)) & m)
        return (s.astype(np.int64) - 131070).astype(np.float32) * _NORMAL_SCALE
    if kind == "embedding":
        a = (z & m).astype(np.int64)
        return (2 * a - 65535).astype(np.float32) * _EMB_SCALE
    raise ValueError(kind)


def hashed_table_device(key: int, n_rows: int, d: int, kind: str, out, chunk_elems: int = 1 << 27) -> None:
    """Fills the torch device tensor `out[:n_rows, :d]` (fp32 or bf16) with the same table."""
    import torch

    def s64(v: int) -> int:                      # the same 64 bits as a signed integer
        return v - (1 << 64) if v >= (1 << 63) else v

    def lsr(z, s: int):                          # logical shift right on int64
        return (z >> s) & ((1 << (64 - s)) - 1)

    dev = out.device
    cols = torch.arange(d, dtype=torch.int64, device=dev)[None, :]
    rows_per = max(1, chunk_elems // d)
    for r0 in range(0, n_rows, rows_per):
        r1 = min(n_rows, r0 + rows_per)
        x = torch.arange(r0, r1, dtype=torch.int64, device=dev)[:, None] * d + cols + s64(key)
        z = x + s64(_SM_A)
        z = (z ^ lsr(z, 30)) * s64(_SM_B)
        z = (z ^ lsr(z, 27)) * s64(_SM_C)
        z = z ^ lsr(z, 31)
        if kind == "normal":
            s = (z & 0xFFFF) + (lsr(z, 16) & 0xFFFF) + (lsr(z, 32) & 0xFFFF) + (lsr(z, 48) & 0xFFFF)
            v = (s - 131070).to(torch.float32) * float(_NORMAL_SCALE)
        elif kind == "embedding":
            v = (2 * (z & 0xFFFF) - 65535).to(torch.float32) * float(_EMB_SCALE)
        else:
            raise ValueError(kind)
        out[r0:r1, :d] = v.to(out.dtype)
        del x, z, v
