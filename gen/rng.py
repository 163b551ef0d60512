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
