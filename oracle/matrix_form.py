"""The paper's matrix-product algorithms, step by step, in binary64 numpy.

TEST INFRASTRUCTURE ONLY (see ``oracle/__init__.py``).  Where ``tcr_oracle.c`` writes
out the *definition* of reduction and scan, this module carries out the *method* of
Sections 4 and 5 of the paper in the paper's notation: 16x16 tiles, the constant
matrices P, U, L and the all-ones matrix, and the accumulator matrices V and S.  A
"matrix unit" operation ``A . B + C`` is ``A @ B + C`` on float64 arrays, so the only
difference from the definition is the order of additions.  Tests require the two to
agree, which pins the readings listed below.

Readings taken where the text is garbled (each is forced by the displayed equations):

* Section 5 stores a 256-vector "in row-major order" but prints the column-major index
  formula; the displayed result matrix has the plain running sums along its first row,
  so row-major is meant:  A[r, c] = V[16 r + c].
* The closing sentence of the derivation in Section 5 swaps the two inequalities that
  define U and L.  The displayed matrices are used: U has ones on and above the
  diagonal (A.U is the inclusive scan of each row) and L has ones strictly below the
  diagonal (L.A is the exclusive scan of each column).
* G (Section 5) is L.A times the all-ones matrix: every entry of row j equals the sum
  of all elements in rows before j.
* The block-level scan listing (Algorithm 7) adds the running carry S inside every
  tile's product *and* scans tile totals that already contain S, and its final
  broadcast uses an exclusive prefix that omits the last tile.  Implemented here as
  what its prose describes: scan each tile, exclusive-scan the tile totals, add the
  offsets, and carry the block total into the next round.
* Algorithm 3 (coalesced 16N reduction) accumulates *contiguous* tiles and then stores
  16 values; with contiguous tiles those are 16 partial sums of one segment, so the
  listing only makes sense as the 256N reduction applied to each segment.  It is not
  reproduced; the strided 16N form of Section 4 is.

Inputs are float64 arrays holding the exactly widened binary16 values.
"""
from __future__ import annotations

import numpy as np

T = 16            # tile edge assumed throughout the paper
TT = T * T

# Section 4: P has ones in its first row and zeros elsewhere.
P = np.zeros((T, T))
P[0, :] = 1.0
# Section 5 (displayed matrices): U upper triangular including the diagonal,
# L strictly lower triangular, ONES the matrix of all ones.
U = np.triu(np.ones((T, T)))
L = np.tril(np.ones((T, T)), k=-1)
ONES = np.ones((T, T))
ZERO = np.zeros((T, T))


def load_tile(mem: np.ndarray, offset: int, layout: str = "rowmajor", stride: int = T) -> np.ndarray:
    """LoadTile (Section 4): a 16x16 tile whose consecutive rows (row-major) or
    consecutive columns (column-major) start ``stride`` elements apart in memory."""
    a = np.empty((T, T))
    for major in range(T):
        line = mem[offset + major * stride: offset + major * stride + T]
        if layout == "rowmajor":
            a[major, :] = line
        elif layout == "colmajor":
            a[:, major] = line
        else:
            raise ValueError(layout)
    return a


def broadcast(value: float) -> np.ndarray:
    return np.full((T, T), float(value))


# ----------------------------------------------------------------------------- reduction

def reduction_16(x: np.ndarray) -> np.ndarray:
    """Algorithm 1: 256 elements = 16 segments of 16; column c of the tile is segment c;
    the first row of P.A holds the 16 segment sums."""
    assert x.size % TT == 0
    out = np.empty(x.size // T)
    for idx in range(0, x.size, TT):
        a = load_tile(x, idx, "colmajor")
        v = P @ a + ZERO
        out[idx // T: idx // T + T] = v[0, :]
    return out


def reduction_256(x: np.ndarray) -> np.ndarray:
    """Algorithm 2: row 0 of P.A holds the column sums; multiplying by P^T folds that
    row into element (0, 0)."""
    assert x.size % TT == 0
    out = np.empty(x.size // TT)
    for idx in range(0, x.size, TT):
        a = load_tile(x, idx, "colmajor")
        v = P @ a + ZERO
        v = v @ P.T + ZERO
        out[idx // TT] = v[0, 0]
    return out


def reduction_256n(x: np.ndarray, seg_len: int) -> np.ndarray:
    """Work-efficient 256N reduction (Section 4): V_i = P.A_i + V_{i-1}, V_0 = 0, and one
    final product with P^T."""
    assert seg_len % TT == 0 and x.size % seg_len == 0
    out = np.empty(x.size // seg_len)
    for s in range(x.size // seg_len):
        v = ZERO.copy()
        for i in range(seg_len // TT):
            a = load_tile(x, s * seg_len + TT * i, "colmajor")
            v = P @ a + v
        r = v @ P.T + ZERO
        out[s] = r[0, 0]
    return out


def reduction_16n_strided(x: np.ndarray, seg_len: int) -> np.ndarray:
    """Strided 16N reduction (Section 4): a wave owns 16 segments of length 16N; in
    iteration i column c of the tile is the i-th run of 16 elements of segment c (leading
    dimension 16N); the first row of V accumulates the 16 segment sums."""
    assert seg_len % T == 0 and x.size % (T * seg_len) == 0
    n16 = seg_len // T
    out = np.empty(x.size // seg_len)
    for g in range(0, x.size, T * seg_len):
        v = ZERO.copy()
        for i in range(n16):
            a = load_tile(x, g + T * i, "colmajor", stride=seg_len)
            v = P @ a + v
        out[g // seg_len: g // seg_len + T] = v[0, :]
    return out


def _reduction_small(vals: np.ndarray) -> float:
    """Reduction_wpb of Algorithm 4: at most 256 partials, zero padded into one tile."""
    assert vals.size <= TT
    buf = np.zeros(TT)
    buf[:vals.size] = vals
    return float(reduction_256(buf)[0])


def block_reduction_256n(x: np.ndarray, seg_len: int, wpb: int) -> np.ndarray:
    """Algorithm 4: each of wpb waves reduces a slice of 256.N/wpb elements, the partials
    go to shared memory, and the first wave reduces the partials on the matrix unit."""
    assert seg_len % (TT * wpb) == 0 and x.size % seg_len == 0
    slice_len = seg_len // wpb
    out = np.empty(x.size // seg_len)
    for s in range(x.size // seg_len):
        prtls = np.empty(wpb)
        for w in range(wpb):
            lo = s * seg_len + w * slice_len
            prtls[w] = reduction_256n(x[lo: lo + slice_len], slice_len)[0]
        out[s] = _reduction_small(prtls)
    return out


def grid_reduction(x: np.ndarray, block_len: int, wpb: int = 4) -> float:
    """Device-level reduction (Section 4): one kernel writes a list of per-block partials
    (a segmented reduction), a second reduces that list."""
    assert x.size % block_len == 0
    partials = block_reduction_256n(x, block_len, wpb)
    while partials.size > 1:
        pad = (-partials.size) % TT
        padded = np.concatenate([partials, np.zeros(pad)])
        partials = reduction_256(padded)
    return float(partials[0])


# ----------------------------------------------------------------------------------- scan

def scan_16(x: np.ndarray) -> np.ndarray:
    """Scan_16 (Section 5): each row of the row-major tile is one segment; A.U is the
    inclusive scan of every row."""
    assert x.size % TT == 0
    out = np.empty(x.size)
    for idx in range(0, x.size, TT):
        a = load_tile(x, idx)
        out[idx: idx + TT] = (a @ U + ZERO).reshape(-1)
    return out


def _scan_256_tile(a: np.ndarray, s: np.ndarray) -> np.ndarray:
    """The three products of Scan_256 / Algorithm 6's loop body."""
    au = a @ U + s
    la = L @ a + ZERO
    return la @ ONES + au


def scan_256n(x: np.ndarray, seg_len: int) -> np.ndarray:
    """Algorithm 6: scan 256-element tiles in order; the last element of each result is
    broadcast into S and enters the next tile through the accumulator."""
    assert seg_len % TT == 0 and x.size % seg_len == 0
    out = np.empty(x.size)
    for g in range(0, x.size, seg_len):
        s = ZERO.copy()
        for i in range(seg_len // TT):
            idx = g + TT * i
            r = _scan_256_tile(load_tile(x, idx), s)
            out[idx: idx + TT] = r.reshape(-1)
            s = broadcast(r[T - 1, T - 1])
    return out


def scan_16n(x: np.ndarray, seg_len: int) -> np.ndarray:
    """Algorithm 5: a wave owns 16 segments of length 16N, one per tile row (rows are 16N
    apart in memory); after each product the last column of R, one running total per
    segment, is broadcast along its row into S."""
    assert seg_len % T == 0 and x.size % (T * seg_len) == 0
    out = np.empty(x.size)
    for g in range(0, x.size, T * seg_len):
        s = ZERO.copy()
        for i in range(seg_len // T):
            idx = g + T * i
            r = load_tile(x, idx, stride=seg_len) @ U + s
            s = np.repeat(r[:, T - 1:T], T, axis=1)
            for lid in range(T):
                oi = idx + lid * seg_len
                out[oi: oi + T] = r[lid, :]
    return out


def block_scan_256n(x: np.ndarray, seg_len: int, wpb: int) -> np.ndarray:
    """Block-level scan (Algorithm 7, as its prose describes it): in every round each of
    wpb waves scans one 256-element tile, the first wave exclusive-scans the tile totals,
    every wave adds its offset plus the carry of earlier rounds, and the round's total
    becomes the carry."""
    assert 1 <= wpb <= T and seg_len % (TT * wpb) == 0 and x.size % seg_len == 0
    out = np.empty(x.size)
    for g in range(0, x.size, seg_len):
        carry = 0.0
        for i in range(0, seg_len // TT, wpb):
            sout = np.empty((wpb, TT))
            for w in range(wpb):
                idx = g + TT * (i + w)
                sout[w] = _scan_256_tile(load_tile(x, idx), ZERO).reshape(-1)
            # tile totals (last element of each tile), zero padded into one row of a tile;
            # E.U - E is the exclusive scan of that row.
            e = np.zeros((T, T))
            e[0, :wpb] = sout[:, TT - 1]
            prtls = (e @ U - e)[0, :]
            for w in range(wpb):
                idx = g + TT * (i + w)
                out[idx: idx + TT] = sout[w] + prtls[w] + carry
            carry += prtls[wpb - 1] + sout[wpb - 1, TT - 1]
    return out


def grid_scan(x: np.ndarray, block_len: int, wpb: int = 4) -> np.ndarray:
    """Device-level scan (Section 5): scan-then-propagate with three kernels -- a segmented
    scan that also yields each block's total, a scan of those totals, and a uniform add
    of the preceding total to every element of a block."""
    assert x.size % block_len == 0
    local = block_scan_256n(x, block_len, wpb)                      # kernel 1
    totals = local[block_len - 1:: block_len]
    offsets = np.concatenate([[0.0], np.cumsum(totals)[:-1]])        # kernel 2 (exclusive)
    return (local.reshape(-1, block_len) + offsets[:, None]).reshape(-1)   # kernel 3
