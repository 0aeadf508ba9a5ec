"""Pins for the definition oracle (oracle/tcr_oracle.c): it is checked against things
other than itself -- hand-evaluated closed forms, exact rational arithmetic, exact
integer arithmetic on scaled inputs, invariants, and numpy's float64 routines on the
special cases they cover."""
import os
from fractions import Fraction

import numpy as np
import pytest

from paper_1811_09736_amd import workloads

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "closed_forms.txt")


# ------------------------------------------------------------------ binary16 decoder

def test_half_decoder_hand_values(oracle):
    # bit patterns worked out from the binary16 format (1 sign, 5 exponent, 10 fraction)
    cases = {
        0x0000: 0.0, 0x3C00: 1.0, 0xC000: -2.0, 0x3800: 0.5, 0x7BFF: 65504.0,
        0x0001: 2.0 ** -24, 0x03FF: 1023 * 2.0 ** -24, 0x0400: 2.0 ** -14,
        0x3555: 1365.0 / 4096.0, 0x4248: 3.140625, 0xFBFF: -65504.0, 0x6800: 2048.0,
    }
    for bits, val in cases.items():
        assert oracle.half_to_double(bits) == val, hex(bits)
    assert oracle.half_to_double(0x8000) == 0.0
    assert np.signbit(oracle.half_to_double(0x8000))
    assert oracle.half_to_double(0x7C00) == np.inf
    assert oracle.half_to_double(0xFC00) == -np.inf
    assert np.isnan(oracle.half_to_double(0x7E00))


def test_half_decoder_all_patterns_vs_numpy(oracle):
    bits = np.arange(65536, dtype=np.uint16)
    ref = bits.view(np.float16).astype(np.float64)
    got = np.array([oracle.half_to_double(int(b)) for b in bits])
    fin = np.isfinite(ref)
    assert np.array_equal(got[fin], ref[fin])
    assert np.array_equal(np.signbit(got[fin]), np.signbit(ref[fin]))
    assert np.array_equal(np.isnan(got), np.isnan(ref))
    assert np.array_equal(np.isinf(got), np.isinf(ref))


# ------------------------------------------------------------------ hand-evaluated fixtures

def _golden_cases():
    with open(GOLDEN) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            head, xin, xscan, xred = [p.strip() for p in line.split("|")]
            n, seg = (int(t) for t in head.split())
            yield (n, seg, [float(t) for t in xin.split()], [float(t) for t in xscan.split()],
                   [float(t) for t in xred.split()])


@pytest.mark.parametrize("case", list(_golden_cases()), ids=lambda c: f"n{c[0]}_L{c[1]}")
def test_golden_closed_forms(oracle, case):
    n, seg, xin, xscan, xred = case
    x = np.array(xin, dtype=np.float16)
    assert x.astype(np.float64).tolist() == xin          # fixture is exactly representable
    assert oracle.segmented_scan(x, seg).tolist() == xscan
    assert oracle.segmented_reduce(x, seg).tolist() == xred


# ------------------------------------------------------------------ closed forms

@pytest.mark.parametrize("n,seg", [(4096, 16), (4096, 256), (1 << 16, 1 << 12), (1 << 20, 1 << 20), (3000, 1000)])
def test_all_ones(oracle, n, seg):
    x = np.ones(n, dtype=np.float16)
    scan = oracle.segmented_scan(x, seg)
    assert np.array_equal(scan, (np.arange(n) % seg + 1).astype(np.float64))
    assert np.array_equal(oracle.segmented_reduce(x, seg), np.full(n // seg, float(seg)))


def test_all_ones_past_fp32_integer_range(oracle):
    # binary64 holds every integer up to 2^53, so the oracle stays exact where fp32 cannot
    n = (1 << 24) + 4096
    x = np.ones(n, dtype=np.float16)
    assert oracle.reduce(x) == float(n)
    assert oracle.segmented_scan_at(x, n, [n - 1, 1 << 24, 5])[0] == float(n)


@pytest.mark.parametrize("m,reps", [(1, 7), (16, 3), (255, 2), (2048, 2)])
def test_arithmetic_ramp(oracle, m, reps):
    # 1, 2, ..., m per segment: reduce = m(m+1)/2, scan = triangular numbers (m <= 2048 is exact in binary16)
    ramp = np.arange(1, m + 1, dtype=np.float64)
    x = np.tile(ramp, reps).astype(np.float16)
    assert np.array_equal(x.astype(np.float64), np.tile(ramp, reps))
    assert np.array_equal(oracle.segmented_reduce(x, m), np.full(reps, m * (m + 1) / 2.0))
    tri = ramp * (ramp + 1) / 2.0
    assert np.array_equal(oracle.segmented_scan(x, m), np.tile(tri, reps))


def test_alternating_signs(oracle):
    # +1, -1, +1, ... : scan is 1, 0, 1, 0, ...; reduce is 0 for even lengths, 1 for odd
    x = np.where(np.arange(30) % 2 == 0, 1.0, -1.0).astype(np.float16)
    assert np.array_equal(oracle.scan(x), (np.arange(30) % 2 == 0).astype(np.float64))
    assert oracle.reduce(x) == 0.0
    assert np.array_equal(oracle.segmented_reduce(x, 3), np.tile([1.0, -1.0], 5))


# ------------------------------------------------------------------ brute force, exact rationals

def _fraction_scan(vals, seg):
    out = []
    for s in range(0, len(vals), seg):
        for k in range(seg):
            out.append(sum((Fraction(v) for v in vals[s: s + k + 1]), Fraction(0)))   # O(L^2)
    return out


@pytest.mark.parametrize("n", [1, 2, 3, 5, 12, 16, 17, 34, 48, 60, 64])
def test_brute_force_tiny(oracle, n):
    x = workloads.make_input(n, "uniform_pm1", 100 + n)
    vals = [float(v) for v in x.astype(np.float64)]
    for seg in [d for d in range(1, n + 1) if n % d == 0]:
        ref = _fraction_scan(vals, seg)
        scan = oracle.segmented_scan(x, seg)
        red = oracle.segmented_reduce(x, seg)
        # binary64 sums of <= 64 binary16 values in [-1, 1] are exact (all are multiples of 2^-24)
        assert [Fraction(v) for v in scan.tolist()] == ref
        assert [Fraction(v) for v in red.tolist()] == ref[seg - 1:: seg]


# ------------------------------------------------------------------ exact fixed point at scale

@pytest.mark.parametrize("dist,seed", [("uniform_pm1", 0), ("normal", 2), ("int8", (2, 1)), ("uniform_01", 4), ("subnormal", 9)])
@pytest.mark.parametrize("seg", [16, 256, 4096, 1 << 18])
def test_fixed_point_int64(oracle, dist, seed, seg):
    # every binary16 value with |x| < 2^5 is an integer multiple of 2^-24; their int64 sums are
    # exact and so are the binary64 sums (|sum| * 2^24 < 2^53), hence equality must be exact.
    n = 1 << 18
    x = workloads.make_input(n, dist, seed)
    q = np.rint(x.astype(np.float64) * 2.0 ** 24).astype(np.int64)
    assert np.array_equal(q.astype(np.float64) * 2.0 ** -24, x.astype(np.float64))
    qs = np.cumsum(q.reshape(-1, seg), axis=1)
    scan = oracle.segmented_scan(x, seg)
    assert np.array_equal(np.rint(scan * 2.0 ** 24).astype(np.int64), qs.reshape(-1))
    assert np.array_equal(scan * 2.0 ** 24, qs.reshape(-1).astype(np.float64))
    red = oracle.segmented_reduce(x, seg)
    assert np.array_equal(red * 2.0 ** 24, qs[:, -1].astype(np.float64))


# ------------------------------------------------------------------ invariants

@pytest.mark.parametrize("n,seg", [(1 << 12, 1), (1 << 12, 16), (1 << 12, 64), (1 << 14, 1 << 10), (1 << 14, 1 << 14), (3 * 5 * 7 * 8, 35)])
def test_invariants(oracle, n, seg):
    x = workloads.make_input(n, "normal", 7)
    xd = x.astype(np.float64)
    scan = oracle.segmented_scan(x, seg)
    red = oracle.segmented_reduce(x, seg)
    # last scan element of a segment is that segment's reduction
    assert np.array_equal(scan[seg - 1:: seg], red)
    # first differences inside a segment give back the input (values are exact multiples of 2^-24)
    d = np.diff(scan.reshape(-1, seg), axis=1, prepend=0.0)
    assert np.array_equal(d.reshape(-1), xd)
    # negating the input negates every output
    assert np.array_equal(oracle.segmented_scan(-x, seg), -scan)
    assert np.array_equal(oracle.segmented_reduce(-x, seg), -red)
    # segments are independent: scanning one segment alone gives the same values
    s = (n // seg) // 2
    assert np.array_equal(oracle.scan(np.ascontiguousarray(x[s * seg:(s + 1) * seg])), scan[s * seg:(s + 1) * seg])
    # seg_len == 1 is the identity
    if seg == 1:
        assert np.array_equal(scan, xd) and np.array_equal(red, xd)
    # seg_len == n is the full operation
    if seg == n:
        assert np.array_equal(oracle.scan(x), scan)
        assert oracle.reduce(x) == red[0]


# ------------------------------------------------------------------ exclusive scan

def test_exclusive_scan_hand_values(oracle):
    # worked by hand from the definition: each output leaves out its own element
    x = np.array([1, 2, 3, 4, 5, 6, 7, 8], dtype=np.float16)
    assert oracle.segmented_scan_exclusive(x, 8).tolist() == [0, 1, 3, 6, 10, 15, 21, 28]
    assert oracle.segmented_scan_exclusive(x, 4).tolist() == [0, 1, 3, 6, 0, 5, 11, 18]
    assert oracle.segmented_scan_exclusive(x, 1).tolist() == [0] * 8
    y = np.array([0.5, -0.25, 8, -8], dtype=np.float16)
    assert oracle.segmented_scan_exclusive(y, 2).tolist() == [0, 0.5, 0, 8]
    assert oracle.segmented_scan_exclusive(np.ones(6, dtype=np.float16), 3).tolist() == [0, 1, 2, 0, 1, 2]


@pytest.mark.parametrize("n,seg", [(1 << 12, 16), (1 << 12, 1 << 12), (3 * 5 * 7 * 8, 35), (60, 1)])
def test_exclusive_scan_relations(oracle, n, seg):
    x = workloads.make_input(n, "uniform_pm1", 3)
    xd = x.astype(np.float64)
    ex = oracle.segmented_scan_exclusive(x, seg).reshape(-1, seg)
    inc = oracle.segmented_scan(x, seg).reshape(-1, seg)
    assert not ex[:, 0].any()                                   # starts at zero
    assert np.array_equal(ex[:, 1:], inc[:, :-1])               # shifted inclusive scan
    assert np.array_equal(ex + xd.reshape(-1, seg), inc)        # exact: values are multiples of 2^-24
    q = np.rint(xd * 2.0 ** 24).astype(np.int64).reshape(-1, seg)
    exq = np.cumsum(q, axis=1) - q                              # exact integer arithmetic
    assert np.array_equal(ex * 2.0 ** 24, exq.astype(np.float64))


# ------------------------------------------------------------------ irregular segments

def test_irregular_hand_values(oracle):
    x = np.array([1, 2, 3, 4, 5, 6, 7, 8], dtype=np.float16)
    off = [0, 3, 3, 4, 8]                                    # lengths 3, 0, 1, 4 -- worked by hand
    assert oracle.irregular_reduce(x, off).tolist() == [6, 0, 4, 26]
    assert oracle.irregular_scan(x, off).tolist() == [1, 3, 6, 4, 5, 11, 18, 26]
    assert oracle.irregular_scan_exclusive(x, off).tolist() == [0, 1, 3, 0, 0, 5, 11, 18]
    a, q = oracle.irregular_moments(x, off)                  # squares 1 4 9 | | 16 | 25 36 49 64
    assert a.tolist() == [6, 0, 4, 26] and q.tolist() == [14, 0, 16, 174]
    # segments need not cover the input: untouched outputs stay zero
    assert oracle.irregular_scan(x, [2, 5]).tolist() == [0, 0, 3, 7, 12, 0, 0, 0]
    assert oracle.irregular_reduce(x, [2, 5]).tolist() == [12]
    assert oracle.irregular_reduce(x, [0]).size == 0
    with pytest.raises(ValueError):
        oracle.irregular_reduce(x, [0, 9])
    with pytest.raises(ValueError):
        oracle.irregular_scan(x, [4, 2])


def test_irregular_equals_per_piece_definition(oracle):
    rng = np.random.default_rng(8)
    x = workloads.make_input(5000, "uniform_pm1", 8)
    cuts = np.sort(rng.integers(0, 5001, 40))
    off = np.concatenate([[0], cuts, [5000]])
    red = oracle.irregular_reduce(x, off)
    scan = oracle.irregular_scan(x, off)
    xd = x.astype(np.float64)
    q = np.rint(xd * 2.0 ** 24).astype(np.int64)
    for s in range(off.size - 1):
        a, b = int(off[s]), int(off[s + 1])
        piece = np.ascontiguousarray(x[a:b])
        assert red[s] * 2.0 ** 24 == float(q[a:b].sum())                       # exact integer arithmetic
        if b > a:
            assert np.array_equal(scan[a:b], oracle.scan(piece))               # the definition, piece by piece
            assert np.array_equal(scan[a:b] * 2.0 ** 24, np.cumsum(q[a:b]).astype(np.float64))
    # uniform offsets are the regular segmented forms
    reg = np.arange(0, 5001, 125)
    assert np.array_equal(oracle.irregular_reduce(x, reg), oracle.segmented_reduce(x, 125))
    assert np.array_equal(oracle.irregular_scan(x, reg), oracle.segmented_scan(x, 125))
    assert np.array_equal(oracle.irregular_scan_exclusive(x, reg), oracle.segmented_scan_exclusive(x, 125))
    ra, rq = oracle.segmented_moments(x, 125)
    ia, iq = oracle.irregular_moments(x, reg)
    assert np.array_equal(ia, ra) and np.array_equal(iq, rq)
    ia, iq = oracle.irregular_moments(x, off)
    assert np.array_equal(ia, red)
    q2 = q * q                                                # exact integers: the squares times 2^48
    for s in range(off.size - 1):
        assert iq[s] * 2.0 ** 48 == float(q2[int(off[s]):int(off[s + 1])].sum())
    # exclusive + own element = inclusive (exact: every term is a multiple of 2^-24 far below 2^53)
    covered = slice(int(off[0]), int(off[-1]))
    assert np.array_equal((oracle.irregular_scan_exclusive(x, off) + xd)[covered], scan[covered])


def test_reduce_is_permutation_invariant_on_integers(oracle):
    x = workloads.make_input(1 << 12, "int8", 5)
    rng = np.random.default_rng(11)
    red = oracle.segmented_reduce(x, 256)
    y = x.reshape(-1, 256).copy()
    for row in y:
        rng.shuffle(row)
    assert np.array_equal(oracle.segmented_reduce(np.ascontiguousarray(y.reshape(-1)), 256), red)


def test_numpy_float64_cross_check(oracle):
    # numpy's float64 cumsum / reduceat are sequential, so integer-valued data must agree exactly
    # and real-valued data to a few ulps of the running magnitude
    x = workloads.make_input(1 << 16, "int4", 3)
    xd = x.astype(np.float64)
    assert np.array_equal(oracle.scan(x), np.cumsum(xd))
    assert np.array_equal(oracle.segmented_reduce(x, 64), np.add.reduceat(xd, np.arange(0, x.size, 64)))
    y = workloads.make_input(1 << 16, "uniform_01", 4)
    assert np.allclose(oracle.scan(y), np.cumsum(y.astype(np.float64)), rtol=1e-13, atol=0)


def test_sampled_scan_matches_full_scan(oracle):
    x = workloads.make_input(1 << 14, "uniform_pm1", 1)
    idx = np.array([0, 1, 255, 256, 4095, 4096, (1 << 14) - 1], dtype=np.uint64)
    for seg in (16, 256, 4096, 1 << 14):
        assert np.array_equal(oracle.segmented_scan_at(x, seg, idx), oracle.segmented_scan(x, seg)[idx.astype(np.int64)])


def test_argument_errors(oracle):
    x = workloads.make_input(12, "ones", 0)
    with pytest.raises(ValueError):
        oracle.segmented_reduce(x, 5)
    with pytest.raises(ValueError):
        oracle.segmented_scan(x, 0)
    with pytest.raises(TypeError):
        oracle.segmented_scan(x.astype(np.float32), 4)
    assert oracle.reduce(np.empty(0, dtype=np.float16)) == 0.0
    assert oracle.scan(np.empty(0, dtype=np.float16)).size == 0
    with pytest.raises(ValueError):
        oracle.segmented_scan_at(x, 4, [12])


# ------------------------------------------------------------------ first two moments

def test_moments_hand_values_and_closed_forms(oracle):
    x = np.array([1, 2, 3, 4, -5, 6, -7, 8], dtype=np.float16)
    a, q = oracle.segmented_moments(x, 4)
    assert a.tolist() == [10, 2] and q.tolist() == [30, 174]               # 1+4+9+16, 25+36+49+64
    a, q = oracle.segmented_moments(x, 8)
    assert a.tolist() == [12] and q.tolist() == [204]
    a, q = oracle.segmented_moments(np.array([0.5, -0.25], dtype=np.float16), 1)
    assert a.tolist() == [0.5, -0.25] and q.tolist() == [0.25, 0.0625]
    for m in (1, 7, 16, 300, 2048):                                         # 1..m: m(m+1)/2 and m(m+1)(2m+1)/6
        ramp = np.arange(1, m + 1, dtype=np.float16)
        a, q = oracle.segmented_moments(ramp, m)
        assert a[0] == m * (m + 1) // 2 and q[0] == m * (m + 1) * (2 * m + 1) // 6
    ones = workloads.make_input(4096, "ones", 0)
    a, q = oracle.segmented_moments(ones, 256)
    assert np.all(a == 256) and np.all(q == 256)


def test_moments_exact_rational_and_invariants(oracle):
    from fractions import Fraction
    x = workloads.make_input(60, "uniform_pm1", 12)
    fx = [Fraction(float(v)) for v in x]
    for seg in (1, 2, 3, 4, 5, 6, 10, 12, 15, 20, 30, 60):
        a, q = oracle.segmented_moments(x, seg)
        for s in range(60 // seg):
            piece = fx[s * seg:(s + 1) * seg]
            assert Fraction(a[s]) == sum(piece)
            assert Fraction(q[s]) == sum(v * v for v in piece)          # < 2^53 of 2^-48 units: exact in binary64
    y = workloads.make_input(1 << 14, "normal", 3)
    for seg in (16, 1000 if (1 << 14) % 1000 == 0 else 1024, 1 << 14):
        a, q = oracle.segmented_moments(y, seg)
        assert np.array_equal(a, oracle.segmented_reduce(y, seg))           # the first moment is the reduction
        a2, q2 = oracle.segmented_moments(-y, seg)
        assert np.array_equal(a2, -a) and np.array_equal(q2, q)             # squares do not see the sign
        assert np.all(q * seg >= a * a * (1 - 1e-12))                       # Cauchy-Schwarz: variance >= 0
        yd = y.astype(np.float64).reshape(-1, seg)
        assert np.allclose(q, (yd * yd).sum(axis=1), rtol=1e-12, atol=0)    # numpy float64 cross-check
    z = workloads.make_input(1 << 12, "int8", 2)                            # integers: numpy must agree exactly
    a, q = oracle.segmented_moments(z, 64)
    zd = z.astype(np.float64).reshape(-1, 64)
    assert np.array_equal(q, (zd * zd).sum(axis=1))
    with pytest.raises(ValueError):
        oracle.segmented_moments(z, 7)


def test_openmp_build_equals_the_sequential_one(oracle):
    # the multi-core build that bench.py also times.  Segments up to 131072 elements: every segment is the same
    # sequential loop, shared among threads, so bit-identical.
    omp = oracle.openmp()
    x = workloads.make_input(1 << 18, "uniform_pm1", 21)
    for seg in (1, 16, 100, 256, 4096, 1 << 17):
        n = (x.size // seg) * seg
        assert np.array_equal(omp.segmented_reduce(x[:n], seg), oracle.segmented_reduce(x[:n], seg))
        assert np.array_equal(omp.segmented_scan(x[:n], seg), oracle.segmented_scan(x[:n], seg))


@pytest.mark.parametrize("seg", [(1 << 17) + 8, 3 * 65536 + 17, 1 << 20])
def test_openmp_build_chunks_long_segments(oracle, seg):
    # longer segments (and the one-segment operations): chunks of 65536 elements side by side -- partial sums for
    # the reduction, the two-pass form for the scan.  Only the order of binary64 additions changes: identical on
    # integer-valued data, within parts in 10^12 of the sums' scale otherwise.
    omp = oracle.openmp()
    n = 2 * seg
    xi = workloads.make_input(n, "int8", 5)
    assert np.array_equal(omp.segmented_reduce(xi, seg), oracle.segmented_reduce(xi, seg))
    assert np.array_equal(omp.segmented_scan(xi, seg), oracle.segmented_scan(xi, seg))
    assert np.array_equal(omp.scan(xi), oracle.scan(xi)) and omp.reduce(xi) == oracle.reduce(xi)
    xr = workloads.make_input(n, "normal", 6)
    scale = np.cumsum(np.abs(xr.astype(np.float64)).reshape(-1, seg), axis=1)
    assert np.all(np.abs(omp.segmented_scan(xr, seg) - oracle.segmented_scan(xr, seg)) <= 1e-12 * scale.reshape(-1))
    assert np.all(np.abs(omp.segmented_reduce(xr, seg) - oracle.segmented_reduce(xr, seg)) <= 1e-12 * scale[:, -1])
