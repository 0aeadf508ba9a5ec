"""The pins must be able to tell a wrong oracle from a right one.  Each case below plants
one plausible mistake in a copy of the C source (on the CPU, in a temporary file), builds
it, and requires the compact pin set to reject it; the untouched source must pass."""
import os
import subprocess

import numpy as np
import pytest

import oracle as oracle_pkg
from paper_1811_09736_amd import workloads

SRC = os.path.join(os.path.dirname(oracle_pkg.__file__), "tcr_oracle.c")

MUTANTS = {
    "scan_made_exclusive": ("            acc += oracle_half_to_double(in[s * seg_len + k]);\n            out[s * seg_len + k] = acc;",
                            "            out[s * seg_len + k] = acc;\n            acc += oracle_half_to_double(in[s * seg_len + k]);"),
    "reduce_drops_last_term": ("for (uint64_t k = 0; k < seg_len; ++k)\n            acc += ", "for (uint64_t k = 0; k + 1 < seg_len; ++k)\n            acc += "),
    "reduce_wrong_segment_base": ("acc += oracle_half_to_double(in[s * seg_len + k]);\n        out[s] = acc;", "acc += oracle_half_to_double(in[s + k]);\n        out[s] = acc;"),
    "scan_carry_not_reset": ("        double acc = 0.0;\n        for (uint64_t k = 0; k < seg_len; ++k) {", "        static double acc = 0.0;\n        for (uint64_t k = 0; k < seg_len; ++k) {"),
    "subnormal_scale": ("ldexp((double)frac, -24)", "ldexp((double)frac, -25)"),
    "normal_exponent_bias": ("expo - 25", "expo - 24"),
    "hidden_bit": ("(double)(1024 + frac)", "(double)(1023 + frac)"),
    "sign_dropped": ("return sign ? -v : v;", "return v;"),
    "sign_bit_position": ("(h >> 15) & 1", "(h >> 14) & 1"),
    "fraction_mask": ("h & 0x3ff", "h & 0x1ff"),
    "scan_wrong_output_index": ("out[s * seg_len + k] = acc;", "out[s + k] = acc;"),
    "exclusive_made_inclusive": ("            out[s * seg_len + k] = acc;\n            acc += oracle_half_to_double(in[s * seg_len + k]);",
                                 "            acc += oracle_half_to_double(in[s * seg_len + k]);\n            out[s * seg_len + k] = acc;"),
    "irregular_reduce_includes_end": ("for (uint64_t k = offsets[s]; k < offsets[s + 1]; ++k)\n            acc += ",
                                      "for (uint64_t k = offsets[s]; k <= offsets[s + 1]; ++k)\n            acc += "),
    "irregular_scan_carry_not_reset": ("        double acc = 0.0;\n        for (uint64_t k = offsets[s]; k < offsets[s + 1]; ++k) {",
                                       "        static double acc = 0.0;\n        for (uint64_t k = offsets[s]; k < offsets[s + 1]; ++k) {"),
    "irregular_exclusive_includes_own_element": ("            out[k] = acc;\n            acc += oracle_half_to_double(in[k]);",
                                                 "            acc += oracle_half_to_double(in[k]);\n            out[k] = acc;"),
    "irregular_exclusive_carry_not_reset": ("        double acc = 0.0;\n        for (uint64_t k = offsets[s]; k < offsets[s + 1]; ++k) {\n            out[k] = acc;",
                                            "        static double acc = 0.0;\n        for (uint64_t k = offsets[s]; k < offsets[s + 1]; ++k) {\n            out[k] = acc;"),
    "irregular_moments_square_of_sum": ("            a += v;\n            q += v * v;\n        }\n        sum[s] = a;\n        sumsq[s] = q;\n    }\n    return 0;\n}\n\n/*\n * binary64",
                                        "            a += v;\n            q += v;\n        }\n        sum[s] = a;\n        sumsq[s] = q;\n    }\n    return 0;\n}\n\n/*\n * binary64"),
    "moments_square_of_sum": ("            q += v * v;", "            q += v;"),
    "moments_sum_of_abs": ("            a += v;\n            q += v * v;", "            a += v < 0 ? -v : v;\n            q += v * v;"),
    "moments_carry_not_reset": ("        double a = 0.0, q = 0.0;", "        double a = 0.0; static double q = 0.0;"),
    "sampled_scan_starts_at_zero": ("const uint64_t first = idx[q] - idx[q] % seg_len;", "const uint64_t first = 0;"),
    "sampled_scan_exclusive": ("k <= idx[q]; ++k)", "k < idx[q]; ++k)"),
}


def _pins(o) -> None:
    """A compact version of the pins in test_oracle.py; raises AssertionError on a wrong oracle."""
    for bits, val in {0x3C00: 1.0, 0xC000: -2.0, 0x0001: 2.0 ** -24, 0x03FF: 1023 * 2.0 ** -24,
                      0x0400: 2.0 ** -14, 0x3555: 1365.0 / 4096.0, 0x7BFF: 65504.0}.items():
        assert o.half_to_double(bits) == val
    x = np.array([1, 2, 3, 4, 5, 6, 7, 8], dtype=np.float16)
    assert o.segmented_scan(x, 4).tolist() == [1, 3, 6, 10, 5, 11, 18, 26]
    assert o.segmented_reduce(x, 4).tolist() == [10, 26]
    assert o.segmented_reduce(x, 2).tolist() == [3, 7, 11, 15]
    assert o.scan(x).tolist() == [1, 3, 6, 10, 15, 21, 28, 36]
    assert o.segmented_scan_exclusive(x, 4).tolist() == [0, 1, 3, 6, 0, 5, 11, 18]
    assert o.irregular_reduce(x, [0, 3, 3, 4, 7]).tolist() == [6, 0, 4, 18]
    assert o.irregular_scan(x, [0, 3, 3, 4, 8]).tolist() == [1, 3, 6, 4, 5, 11, 18, 26]
    assert o.irregular_scan_exclusive(x, [0, 3, 3, 4, 8]).tolist() == [0, 1, 3, 0, 0, 5, 11, 18]
    ia, iq = o.irregular_moments(x, [0, 3, 3, 4, 8])
    assert ia.tolist() == [6, 0, 4, 26] and iq.tolist() == [14, 0, 16, 174]
    assert o.reduce(x) == 36.0
    a, q = o.segmented_moments(np.array([1, -2, 3, 4, -5, 6], dtype=np.float16), 3)
    assert a.tolist() == [2, 5] and q.tolist() == [14, 77]
    for dist, seed in (("uniform_pm1", 0), ("subnormal", 9)):
        y = workloads.make_input(1 << 12, dist, seed)
        q = np.rint(y.astype(np.float64) * 2.0 ** 24).astype(np.int64)
        for seg in (16, 256, 1 << 12):
            qs = np.cumsum(q.reshape(-1, seg), axis=1)
            assert np.array_equal(o.segmented_scan(y, seg) * 2.0 ** 24, qs.reshape(-1).astype(np.float64))
            assert np.array_equal(o.segmented_reduce(y, seg) * 2.0 ** 24, qs[:, -1].astype(np.float64))
            idx = np.array([0, seg - 1, seg, 4095], dtype=np.uint64) % (1 << 12)
            assert np.array_equal(o.segmented_scan_at(y, seg, idx) * 2.0 ** 24,
                                  qs.reshape(-1)[idx.astype(np.int64)].astype(np.float64))


def _build(tmp_path, name, text):
    c = tmp_path / f"{name}.c"
    so = tmp_path / f"{name}.so"
    c.write_text(text)
    subprocess.check_call(["gcc", "-O1", "-std=c11", "-fPIC", "-shared", "-o", str(so), str(c), "-lm"])
    return str(so)


def test_unmodified_source_passes(tmp_path):
    _pins(oracle_pkg.Oracle(_build(tmp_path, "clean", open(SRC).read())))


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_planted_mistake_is_rejected(tmp_path, name):
    old, new = MUTANTS[name]
    text = open(SRC).read()
    assert text.count(old) >= 1, "mutation site not found; update the table"
    mutated = text.replace(old, new, 1)
    with pytest.raises(AssertionError):
        _pins(oracle_pkg.Oracle(_build(tmp_path, name, mutated)))
