"""Seeded synthetic inputs shared by the tests, the bench and the smoke check.

This module draws numbers and converts them to IEEE binary16; it contains none
of the reduction / scan arithmetic.  The device library and the CPU oracle both
receive the *same* fp16 bit patterns produced here.

Generator: ``numpy.random.default_rng(seed)`` (PCG64) drawing in float64, then
``astype(float16)`` (round to nearest even).  Large arrays are drawn in fixed
chunks of ``_CHUNK`` elements from one generator, so an array of n elements is a
prefix of the array of any larger n with the same seed and distribution.

Workload shapes follow the paper's evaluation (Section 6): a fixed number of
half-precision elements swept over power-of-two segment sizes, plus full
(unsegmented) reduction and scan.
"""
from __future__ import annotations

import hashlib
from dataclasses import dataclass
from typing import Iterator, Tuple

import numpy as np

_CHUNK = 1 << 22


def _draw(rng: np.random.Generator, dist: str, m: int) -> np.ndarray:
    if dist == "uniform_pm1":          # i.i.d. uniform[-1, 1)
        return rng.uniform(-1.0, 1.0, m)
    if dist == "uniform_01":           # i.i.d. uniform[0, 1)
        return rng.uniform(0.0, 1.0, m)
    if dist == "normal":               # i.i.d. N(0, 1)
        return rng.standard_normal(m)
    if dist.startswith("int"):         # "int8" -> integers uniform on {-8..8}
        r = int(dist[3:])
        return rng.integers(-r, r, m, endpoint=True).astype(np.float64)
    if dist == "ones":
        return np.ones(m)
    if dist == "subnormal":            # integer multiples of 2^-24 below the fp16 normal range
        return rng.integers(-1023, 1023, m, endpoint=True).astype(np.float64) * 2.0 ** -24
    raise ValueError(f"unknown distribution {dist!r}")


def make_input(n: int, dist: str, seed) -> np.ndarray:
    """Return n fp16 values (numpy float16, C-contiguous) for (dist, seed)."""
    rng = np.random.default_rng(seed)
    out = np.empty(n, dtype=np.float16)
    for lo in range(0, n, _CHUNK):
        m = min(_CHUNK, n - lo)
        out[lo:lo + m] = _draw(rng, dist, m).astype(np.float16)
    return out


def sha256(x: np.ndarray) -> str:
    return hashlib.sha256(np.ascontiguousarray(x).view(np.uint8)).hexdigest()


@dataclass(frozen=True)
class Workload:
    name: str
    op: str            # "segmented_reduce" | "segmented_scan" | "reduce" | "scan"
    n: int
    seg_len: int       # == n for the full operations
    dist: str
    seed: object
    exact: bool        # integer-valued input: fp32 results must equal the oracle bit for bit


def configs() -> Iterator[Workload]:
    """The five evaluation configurations (segment-size sweeps at fixed n, full reduce, full scan)."""
    yield Workload("cfg1_segreduce_n2^20_L256", "segmented_reduce", 1 << 20, 256, "uniform_pm1", 0, False)
    for L in (16, 64, 256, 1024, 4096):
        yield Workload(f"cfg2_segscan_n2^24_L{L}", "segmented_scan", 1 << 24, L, "uniform_pm1", 1, False)
    yield Workload("cfg3a_reduce_n2^28_normal", "reduce", 1 << 28, 1 << 28, "normal", 2, False)
    yield Workload("cfg3b_reduce_n2^28_int8", "reduce", 1 << 28, 1 << 28, "int8", (2, 1), True)
    yield Workload("cfg4_scan_n2^28_int4", "scan", 1 << 28, 1 << 28, "int4", 3, True)
    for e in (4, 6, 8, 10, 12, 14, 16, 20):
        yield Workload(f"cfg5_segreduce_n2^28_L2^{e}", "segmented_reduce", 1 << 28, 1 << e, "uniform_01", 4, False)
    for e in (4, 6, 8, 10, 12, 14, 16, 20):
        yield Workload(f"cfg5_segscan_n2^28_L2^{e}", "segmented_scan", 1 << 28, 1 << e, "uniform_01", 4, False)


def algorithmic_bytes(op: str, n: int, seg_len: int) -> Tuple[int, int]:
    """(bytes read, bytes written) the operation must move: fp16 in, fp32 out."""
    if op in ("segmented_reduce", "reduce"):
        return 2 * n, 4 * (n // seg_len)
    return 2 * n, 4 * n
