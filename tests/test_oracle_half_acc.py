"""Pins for the binary16-accumulate part of the oracle (oracle_double_to_half, oracle_segmented_scan_half_acc):
hand-evaluated fixtures, the rounding rule checked at every midpoint between neighbouring binary16 values, numpy's
correctly rounded binary64 -> binary16 conversion, exact rational brute force on tiny inputs, and the cases in
which a binary16 accumulator must agree with the exact scan."""
import os
import subprocess
from fractions import Fraction

import numpy as np
import pytest

import oracle as oracle_pkg
from paper_1811_09736_amd import workloads

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "half_accumulate.txt")


def _cases():
    with open(GOLDEN) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            head, xin, xscan = [p.strip() for p in line.split("|")]
            n, seg = (int(t) for t in head.split())
            yield n, seg, [float(t) for t in xin.split()], [float(t) for t in xscan.split()]


def _pins(o):
    """Compact pin set; raises AssertionError on a wrong oracle (also used on the planted mistakes below)."""
    # the rounding rule, straight from the format: spacing 2 above 2048, 2^-24 in the subnormal range
    hand = {1.0: 0x3C00, 2049.0: 0x6800, 2051.0: 0x6802, 2050.999: 0x6801, 2049.001: 0x6801, -2049.0: 0xE800,
            65504.0: 0x7BFF, 65519.999: 0x7BFF, 65520.0: 0x7C00, -65520.0: 0xFC00, 1e30: 0x7C00,
            2.0 ** -24: 0x0001, 2.0 ** -25: 0x0000, 2.0 ** -25 * 1.0001: 0x0001, 1.5 * 2.0 ** -24: 0x0002,
            2.5 * 2.0 ** -24: 0x0002, 1023.5 * 2.0 ** -24: 0x0400, 2.0 ** -14: 0x0400, 0.0: 0x0000, 1.0 / 3.0: 0x3555}
    for v, bits in hand.items():
        assert o.double_to_half(v) == bits, (v, hex(o.double_to_half(v)), hex(bits))
    assert o.double_to_half(-0.0) == 0x8000
    for n, seg, xin, want in _cases():
        x = np.array(xin, dtype=np.float16)
        assert x.astype(np.float64).tolist() == xin, "fixture inputs must be binary16 values"
        got = o.segmented_scan_half_acc(x, seg).astype(np.float64).tolist()
        assert got == want, (xin, got, want)
        excl = o.segmented_scan_half_acc(x, seg, True).astype(np.float64).reshape(-1, seg)
        inc = np.array(want).reshape(-1, seg)
        assert np.array_equal(excl[:, 1:], inc[:, :-1]) and not excl[:, 0].any()


def test_hand_values_and_fixtures(oracle):
    _pins(oracle._get())


def test_every_binary16_value_survives_the_round_trip(oracle):
    for b in range(65536):
        v = oracle.half_to_double(b)
        if not np.isnan(v):
            assert oracle.double_to_half(v) == b, hex(b)


def test_midpoints_go_to_the_even_neighbour(oracle):
    # consecutive finite positive patterns are consecutive values; their midpoint is exact in binary64
    for b in range(0, 0x7BFF):
        lo, hi = oracle.half_to_double(b), oracle.half_to_double(b + 1)
        mid = (lo + hi) / 2
        even = b if b % 2 == 0 else b + 1
        assert oracle.double_to_half(mid) == even, hex(b)
        assert oracle.double_to_half(np.nextafter(mid, 0.0)) == b
        assert oracle.double_to_half(np.nextafter(mid, np.inf)) == b + 1
        assert oracle.double_to_half(-mid) == (even | 0x8000)


def test_conversion_against_numpy(oracle):
    rng = np.random.default_rng(7)
    d = rng.standard_normal(50000) * 10.0 ** rng.integers(-9, 6, 50000)
    with np.errstate(over="ignore"):
        ref = d.astype(np.float16).view(np.uint16)
    got = np.array([oracle.double_to_half(v) for v in d], dtype=np.uint16)
    assert np.array_equal(got, ref)


def _round16(fr: Fraction) -> float:
    """Nearest binary16 value of an exact rational that binary64 holds exactly (numpy's conversion rounds once)."""
    f = float(fr)
    assert Fraction(f) == fr
    with np.errstate(over="ignore"):
        return float(np.float64(f).astype(np.float16))


@pytest.mark.parametrize("dist", ["uniform_pm1", "normal", "int8", "subnormal", "uniform_01"])
def test_brute_force_on_tiny_inputs(oracle, dist):
    for n in (1, 2, 5, 12, 30):
        x = workloads.make_input(n, dist, 100 + n)
        if dist == "normal":
            x = (x * np.float16(300.0)).astype(np.float16)           # reach the coarse end of the format
        for seg in [d for d in range(1, n + 1) if n % d == 0]:
            inc = oracle.segmented_scan_half_acc(x, seg).astype(np.float64)
            exc = oracle.segmented_scan_half_acc(x, seg, True).astype(np.float64)
            for s in range(n // seg):
                acc = 0.0
                for k in range(seg):
                    assert exc[s * seg + k] == acc
                    acc = _round16(Fraction(acc) + Fraction(float(x[s * seg + k])))
                    assert inc[s * seg + k] == acc, (dist, n, seg, s, k)


def test_equals_the_exact_scan_while_nothing_is_rounded(oracle):
    # integers whose partial sums stay within +-2048 are binary16 values: no addition rounds
    rng = np.random.default_rng(3)
    x = rng.integers(-4, 4, 4096, endpoint=True).astype(np.float16)
    for seg in (16, 256, 4096):
        exact = oracle.segmented_scan(x, seg)
        assert np.max(np.abs(exact)) <= 2048
        assert np.array_equal(oracle.segmented_scan_half_acc(x, seg).astype(np.float64), exact)
        assert np.array_equal(oracle.segmented_scan_half_acc(x, seg, True).astype(np.float64), oracle.segmented_scan_exclusive(x, seg))


def test_all_ones_stall_at_2048(oracle):
    # 2048 + 1 lies halfway between 2048 and 2050 and goes to the even one: the running count stops there
    x = np.ones(5000, dtype=np.float16)
    got = oracle.segmented_scan_half_acc(x, 5000).astype(np.float64)
    assert np.array_equal(got[:2048], np.arange(1, 2049)) and np.all(got[2048:] == 2048)


def test_error_bound_of_a_rounded_accumulator(oracle):
    # every step rounds once: |acc - exact| <= sum over the steps of half a spacing of that step's result
    x = workloads.make_input(2048, "uniform_01", 4)
    exact = oracle.segmented_scan(x, 2048)
    got = oracle.segmented_scan_half_acc(x, 2048).astype(np.float64)
    half_spacing = 2.0 ** (np.floor(np.log2(np.maximum(got, 2.0 ** -14))) - 11)
    assert np.all(np.abs(got - exact) <= np.cumsum(half_spacing))


MUTANTS = {
    "ties_away_from_zero": ("(rest == 0.5 && fmod(whole, 2.0) == 1.0)", "(rest == 0.5)"),
    "truncation": ("if (rest > 0.5 || (rest == 0.5 && fmod(whole, 2.0) == 1.0)) whole += 1.0;", ""),
    "one_bit_too_many": ("int ulp_exp = e - 1 - 10;", "int ulp_exp = e - 1 - 11;"),
    "subnormals_flushed": ("if (ulp_exp < -24) ulp_exp = -24;", "if (ulp_exp < -24) return sign;"),
    "overflow_saturates": ("if (r >= 65536.0) return (uint16_t)(sign | 0x7c00u);", "if (r >= 65536.0) return (uint16_t)(sign | 0x7bffu);"),
    "sign_lost": ("const uint16_t sign = signbit(v) ? 0x8000u : 0u;", "const uint16_t sign = 0u;"),
    "half_acc_carry_not_reset": ("        uint16_t acc = 0;", "        static uint16_t acc = 0;"),
    "half_acc_exclusive_swapped": ("out[s * seg_len + k] = exclusive ? acc : next;", "out[s * seg_len + k] = exclusive ? next : acc;"),
    "half_acc_adds_unrounded_sum": ("uint16_t acc = 0;\n        for (uint64_t k = 0; k < seg_len; ++k) {\n            const uint16_t next = oracle_double_to_half(oracle_half_to_double(acc) + oracle_half_to_double(in[s * seg_len + k]));",
                                    "uint16_t acc = 0; double wide = 0.0;\n        for (uint64_t k = 0; k < seg_len; ++k) {\n            wide += oracle_half_to_double(in[s * seg_len + k]);\n            const uint16_t next = oracle_double_to_half(wide);"),
}


def _build(tmp_path, name, text):
    c = tmp_path / f"{name}.c"
    so = tmp_path / f"{name}.so"
    c.write_text(text)
    subprocess.check_call(["gcc", "-O1", "-std=c11", "-fPIC", "-shared", "-o", str(so), str(c), "-lm"])
    return str(so)


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_planted_mistake_is_rejected(tmp_path, name):
    src = os.path.join(os.path.dirname(oracle_pkg.__file__), "tcr_oracle.c")
    old, new = MUTANTS[name]
    text = open(src).read()
    assert text.count(old) >= 1, "mutation site not found; update the table"
    with pytest.raises(AssertionError):
        _pins(oracle_pkg.Oracle(_build(tmp_path, name, text.replace(old, new, 1))))
