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


def make_offsets(n: int, recipe: str, seed) -> np.ndarray:
    """Return uint64 offsets[nseg + 1] (offsets[0] = 0, offsets[-1] = n, non-decreasing) cutting n elements
    into irregular segments.  The paper evaluates regular segments only; these recipes give the
    irregular entry points length mixes of the same scale as its sweep:

    * ``"uniform<M>"``   lengths i.i.d. uniform on {0..2M} (mean M, empty segments included);
    * ``"lognormal<M>"`` lengths i.i.d. log-normal with median M and sigma 2 (heavy tail: most segments are
      short, most elements lie in a few long ones);
    * ``"few<K>"``       K - 1 cut points i.i.d. uniform on {0..n} (K very long segments).
    """
    rng = np.random.default_rng(seed)
    if recipe.startswith("few"):
        cuts = np.sort(rng.integers(0, n, int(recipe[3:]) - 1, endpoint=True).astype(np.uint64))
        return np.concatenate(([0], cuts, [n])).astype(np.uint64)
    if recipe.startswith("uniform"):
        m = int(recipe[7:])
        draw = lambda k: rng.integers(0, 2 * m, k, endpoint=True)
    elif recipe.startswith("lognormal"):
        m = int(recipe[9:])
        draw = lambda k: np.floor(rng.lognormal(np.log(m), 2.0, k)).astype(np.int64)
    else:
        raise ValueError(f"unknown offsets recipe {recipe!r}")
    parts, total = [], 0
    while total < n:
        lens = draw(max(1024, n // max(m, 1) // 4 + 1))
        parts.append(lens)
        total += int(lens.sum())
    ends = np.cumsum(np.concatenate(parts))
    ends = ends[: int(np.searchsorted(ends, n, side="left"))]      # cut points strictly below n
    return np.concatenate(([0], ends, [n])).astype(np.uint64)


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
