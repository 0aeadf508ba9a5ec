"""Host-side checks that need no GPU: the shared library loads, exports every symbol the
header declares, rejects bad arguments before touching a device, and its dispatch table
names the kernels expected for each segment-length class."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "tcr.h")


@pytest.fixture(scope="module")
def lib():
    from paper_1811_09736_amd import build as b
    if not os.path.exists(b.LIB_PATH):
        b.build_library()
    from paper_1811_09736_amd import binding
    return binding


def _declared_symbols():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(tcr_[a-z_]+)\s*\(", text)))


def test_header_symbols_are_exported(lib):
    names = _declared_symbols()
    assert len(names) >= 10
    raw = lib.raw()
    for name in names:
        assert hasattr(raw, name), name
    assert sorted(lib.EXPORTS) == names


def test_status_strings(lib):
    raw = lib.raw()
    seen = {raw.tcr_status_string(i).decode() for i in range(5)}
    assert len(seen) == 5 and "ok" in seen
    assert raw.tcr_status_string(99).decode() == "unknown status"


def test_argument_validation_happens_before_any_device_work(lib):
    raw = lib.raw()
    buf = ctypes.create_string_buffer(4096 + 64)
    base = (ctypes.addressof(buf) + 63) & ~63           # a 64-byte aligned host address (never dereferenced)
    inv = lib.ERR_INVALID_ARG
    assert raw.tcr_segmented_reduce(base, base + 2048, 64, 0, None) == inv       # seg_len == 0
    assert raw.tcr_segmented_reduce(base, base + 2048, 100, 16, None) == inv     # n % seg_len != 0
    assert raw.tcr_segmented_scan(base, base + 2048, 64, 0, None) == inv
    assert raw.tcr_segmented_scan(base, base + 2048, 65, 16, None) == inv
    assert raw.tcr_segmented_reduce(None, base, 64, 16, None) == inv             # null input
    assert raw.tcr_segmented_scan(base, None, 64, 16, None) == inv               # null output
    assert raw.tcr_segmented_scan(base + 1, base + 2048, 64, 16, None) == inv    # input not aligned to its elements
    assert raw.tcr_segmented_scan(base, base + 2048 + 2, 64, 16, None) == inv    # output not aligned to its elements
    assert raw.tcr_segmented_reduce(base, base + 2048 + 2, 64, 16, None) == inv
    assert raw.tcr_reduce(base, None, 64, None) == inv
    assert raw.tcr_scan(base + 3, base + 2048, 64, None) == inv
    assert raw.tcr_segmented_scan_ex(base, base + 2048 + 1, 64, 16, 2, None) == inv      # binary16 output at an odd address
    # unknown flag bits of the scan variants
    assert raw.tcr_segmented_scan_ex(base, base + 2048, 64, 16, 4, None) == inv
    assert raw.tcr_scan_ex(base, base + 2048, 64, 8, None) == inv
    assert raw.tcr_segmented_scan_ex(base, base + 2048, 65, 16, 1, None) == inv
    assert raw.tcr_scan_ex(None, None, 0, 3, None) == lib.OK
    # n == 0 is a no-op for everything that writes no output
    assert raw.tcr_segmented_reduce(None, None, 0, 16, None) == lib.OK
    assert raw.tcr_segmented_scan(None, None, 0, 16, None) == lib.OK
    assert raw.tcr_scan(None, None, 0, None) == lib.OK
    # sizes without a kernel
    assert raw.tcr_segmented_scan(base, base + 2048, 1 << 39, 1 << 39, None) == lib.ERR_UNSUPPORTED


def test_variant_switch(lib):
    with pytest.raises(lib.TcrError):
        lib.set_variant("formulation", "tensor")
    with pytest.raises(lib.TcrError):
        lib.set_variant("nonsense", "x")
    try:
        lib.set_variant("formulation", "dpp")
        assert "dpp" in lib.kernel_name(lib.OP_SEGMENTED_SCAN, 1 << 20, 256)
        lib.set_variant("scan_carry", "reduce_then_scan")
        assert "table" in lib.kernel_name(lib.OP_SCAN, 1 << 28, 1 << 28)
        lib.set_variant("scan_carry", "scan_then_propagate")
        assert "uniform_add_kernel" in lib.kernel_name(lib.OP_SCAN, 1 << 28, 1 << 28)
    finally:
        lib.set_variant("reset")
    assert "mfma" in lib.kernel_name(lib.OP_SEGMENTED_SCAN, 1 << 20, 256)
    assert lib.kernel_name(lib.OP_SCAN, 1 << 28, 1 << 28) == "scan_chain_kernel<mfma>"


def test_dispatch_by_segment_length(lib):
    n = 1 << 28
    k = lib.kernel_name
    for e in range(4, 10):
        assert k(lib.OP_SEGMENTED_REDUCE, n, 1 << e).startswith("reduce_small_kernel")
        assert k(lib.OP_SEGMENTED_SCAN, n, 1 << e).startswith("scan_small_kernel")
    for e in (10, 12, 16):
        assert k(lib.OP_SEGMENTED_REDUCE, n, 1 << e) == "reduce_span_kernel<mfma,wave>"
    for e in (13, 14, 15):                                 # segments split over 2 or 4 wavefronts of a workgroup
        assert k(lib.OP_SEGMENTED_REDUCE, n, 1 << e) == "reduce_span_kernel<mfma,block>"
    for e in (10, 11, 12):
        assert k(lib.OP_SEGMENTED_SCAN, n, 1 << e) == "scan_block_kernel<mfma,nocarry>"
    for e in (13, 14):
        assert k(lib.OP_SEGMENTED_SCAN, n, 1 << e) == "scan_block_kernel<mfma,ticket>"
    for e in (15, 16, 20, 24):                             # the persistent, pipelined chain
        assert k(lib.OP_SEGMENTED_SCAN, n, 1 << e) == "scan_chain_kernel<mfma>"
    assert k(lib.OP_SEGMENTED_REDUCE, n, 1 << 17) == "reduce_span_kernel<mfma,block>"
    assert k(lib.OP_SEGMENTED_REDUCE, n, 1 << 18) == "reduce_span_kernel<mfma,wave>+reduce_final_kernel"
    assert k(lib.OP_SEGMENTED_REDUCE, n, 1 << 20) == "reduce_span_kernel<mfma,wave>+reduce_final_kernel"
    assert k(lib.OP_SEGMENTED_REDUCE, n, 1 << 24).endswith("+reduce_final_kernel")
    lib.set_variant("reduce_finish", "fused")
    assert k(lib.OP_SEGMENTED_REDUCE, n, 1 << 20) == "reduce_span_kernel<mfma,wave,finish>"
    assert k(lib.OP_SEGMENTED_REDUCE, 1 << 36, 1 << 24).endswith("+reduce_final_kernel")   # 2^18 partials: too many for one workgroup
    lib.set_variant("reset")
    assert k(lib.OP_REDUCE, n, n).endswith("+reduce_final_kernel")
    assert k(lib.OP_REDUCE, 1000, 1000) == "reduce_span_kernel<mfma,wave>"
    assert k(lib.OP_SCAN, n, n) == "scan_chain_kernel<mfma>"
    assert k(lib.OP_SCAN, n - 3, n - 3) == "scan_chain_kernel<mfma>+scan_tail_kernel"      # n not a multiple of 8
    assert k(lib.OP_SCAN, 40003, 40003).startswith("scan_block_kernel<mfma,")              # ... under two chain tiles: one kernel
    lib.set_variant("formulation", "dpp")
    try:
        assert k(lib.OP_SCAN, n, n) == "scan_chain_kernel<dpp>"
        assert k(lib.OP_SEGMENTED_SCAN, n, 1 << 16) == "scan_chain_kernel<dpp>"
        assert k(lib.OP_SEGMENTED_SCAN, n, 1 << 14) == "scan_block_kernel<dpp,ticket>"
        assert k(lib.OP_SEGMENTED_SCAN, 3 << 24, 3 << 20) == "irregular_scan_kernel<regular>"   # other lengths: fixed tiles
    finally:
        lib.set_variant("reset")
    assert k(lib.OP_SCAN, 5000, 5000) == "scan_block_kernel<mfma,nocarry>"
    assert k(lib.OP_SCAN, 8192, 8192) == "scan_block_kernel<mfma,nocarry>"
    assert k(lib.OP_SEGMENTED_SCAN, 48000, 48) == "irregular_scan_kernel<regular>"     # untuned lengths: fixed tiles
    assert k(lib.OP_SEGMENTED_SCAN, 48000, 1) == "tiny_scan_kernel"
    assert k(lib.OP_SEGMENTED_SCAN, 48000, 8) == "tiny_scan_kernel"
    assert k(lib.OP_SEGMENTED_REDUCE, 48000, 2) == "tiny_reduce_kernel"
    for seg in (3, 4, 5, 6, 7, 8, 9, 12, 15, 18, 24, 30):        # rows of whole segments, an even number of at most 32 elements
        assert k(lib.OP_SEGMENTED_REDUCE, seg * 1000, seg) == "packed_rows_reduce_kernel"
    for seg in (17, 25, 31, 33, 48, 999, 1001, 8160):      # masked rows of the array, whole segments per workgroup
        assert k(lib.OP_SEGMENTED_REDUCE, seg * 5, seg) == "rows_reduce_kernel"
    assert k(lib.OP_SEGMENTED_REDUCE, 8168 * 5, 8168) == "masked_wave_reduce_kernel"
    lib.set_variant("untuned_reduce", "tiles")
    assert k(lib.OP_SEGMENTED_REDUCE, 48000, 3) == "generic_thread_kernel"
    assert k(lib.OP_SEGMENTED_REDUCE, 48000, 8) == "tiny_reduce_kernel"
    assert k(lib.OP_SEGMENTED_REDUCE, 48000, 6).startswith("irregular_reduce_kernel<regular>")
    assert k(lib.OP_SEGMENTED_REDUCE, 48000, 12).startswith("irregular_reduce_kernel<regular>+")
    assert k(lib.OP_SEGMENTED_REDUCE, 48000, 48).startswith("irregular_reduce_kernel<regular>+")
    assert k(lib.OP_SEGMENTED_REDUCE, 1001 * 5, 1001) == "masked_wave_reduce_kernel"
    lib.set_variant("reset")
    assert k(lib.OP_IRREGULAR_REDUCE, 1 << 20, 0).startswith("irregular_bounds_kernel+irregular_reduce_kernel")
    assert k(lib.OP_IRREGULAR_SCAN, 1 << 20, 0) == "irregular_bounds_kernel+irregular_scan_kernel"
    assert k(lib.OP_SEGMENTED_REDUCE, 3 << 20, 3 << 10) == "rows_reduce_kernel"
    assert k(lib.OP_SEGMENTED_REDUCE, 3 << 20, 3 << 12) == "masked_wave_reduce_kernel"
    assert k(lib.OP_SEGMENTED_REDUCE, 3 << 24, 3 << 20) == "masked_span_reduce_kernel+reduce_final_kernel"
    assert k(lib.OP_SEGMENTED_SCAN, 3 << 24, 3 << 20) == "scan_chain_kernel<mfma>"        # long, a multiple of 8
    assert k(lib.OP_SEGMENTED_SCAN, 100003 * 5, 100003) == "irregular_scan_kernel<regular>"   # long, odd
    assert k(lib.OP_SEGMENTED_SCAN, 40000 * 5, 40000) == "irregular_scan_kernel<regular>"   # under two chain tiles
    assert k(lib.OP_SEGMENTED_SCAN, 3584 * 7, 3584) == "scan_segment_kernel"             # aligned, fills its workgroup: one each
    assert k(lib.OP_SEGMENTED_SCAN, 3000 * 7, 3000) == "irregular_scan_kernel<regular>"   # a multiple of 8 that does not
    assert k(lib.OP_SEGMENTED_SCAN, 4160 * 7, 4160) == "irregular_scan_kernel<regular>"   # aligned, two thirds of 12 tiles
    assert k(lib.OP_SEGMENTED_SCAN, 3001 * 7, 3001) == "irregular_scan_kernel<regular>"
    assert k(lib.OP_SEGMENTED_SCAN, 200 * 7, 200) == "irregular_scan_kernel<regular>"
    assert k(lib.OP_SEGMENTED_SCAN, n, 3) == ""           # 3 does not divide n: the call reports an invalid argument
    assert k(lib.OP_SEGMENTED_SCAN, 0, 16) == ""


def test_tuning_table_text_round_trip(lib):
    assert lib.tuning_export() == ""
    try:
        lib.tuning_import("scan:14=8;reduce:20=1;scan:41=9;")
        assert lib.tuning_export() == "scan:14=8;scan:41=9;reduce:20=1;"           # table by table, class by class
        # the dispatcher follows the table where the choice is valid for the segment length ...
        assert lib.kernel_name(lib.OP_SEGMENTED_SCAN, 1 << 28, 1 << 14) == "scan_block_kernel<mfma,ticket>"
        lib.tuning_import("scan:14=4;")
        assert lib.kernel_name(lib.OP_SEGMENTED_SCAN, 1 << 28, 1 << 14) == "scan_block_kernel<mfma,nocarry>"
        lib.tuning_import("reduce:20=0;")
        assert lib.kernel_name(lib.OP_SEGMENTED_REDUCE, 1 << 28, 1 << 20) == "reduce_span_kernel<mfma,block>+reduce_final_kernel"
        # ... and ignores a shape whose share cannot hold the segment
        lib.tuning_import("scan:16=0;")
        assert lib.kernel_name(lib.OP_SEGMENTED_SCAN, 1 << 28, 1 << 16) == "scan_chain_kernel<mfma>"
        lib.tuning_import("scan:16=8;scan:14=10;")           # the pipelined shapes need a segment of a whole share at least
        assert lib.kernel_name(lib.OP_SEGMENTED_SCAN, 1 << 28, 1 << 16) == "scan_block_kernel<mfma,lookback>"
        assert lib.kernel_name(lib.OP_SEGMENTED_SCAN, 1 << 28, 1 << 14) == "scan_block_kernel<mfma,ticket>"
        lib.tuning_import("scan:16=0;")
        for bad in ("scan:14", "scan:99=1;", "scan:14=15;", "reduce:20=4;", "sort:3=1;", "scan:14=8", "scan:14=64;",
                    "scan_any:6=32;", "reduce_any:6=6;", "irregular:2=0;", "irregular:0=3;", "scan_an:6=1;"):
            with pytest.raises(lib.TcrError):
                lib.tuning_import(bad)
        assert lib.tuning_export() == "scan:16=0;"       # a rejected text leaves the table untouched
        # the wider tables: formulation per class (+32), carry strategies (12, 13), kernels for untuned lengths
        n = 1 << 28
        lib.tuning_import("scan:8=33;reduce:8=34;scan:20=12;scan:41=13;reduce:41=32;scan_any:6=1;reduce_any:9=1;irregular:0=1;irregular:1=1;")
        assert lib.tuning_export() == "scan:8=33;scan:20=12;scan:41=13;reduce:8=34;reduce:41=32;scan_any:6=1;reduce_any:9=1;irregular:0=1;irregular:1=1;"
        assert lib.kernel_name(lib.OP_SEGMENTED_SCAN, n, 256) == "scan_small_kernel<dpp>"
        assert lib.kernel_name(lib.OP_SEGMENTED_SCAN, n, 512) == "scan_small_kernel<mfma>"
        assert lib.kernel_name(lib.OP_SEGMENTED_REDUCE, n, 256) == "reduce_small_kernel<dpp>"
        assert lib.kernel_name(lib.OP_SEGMENTED_SCAN, n, 1 << 20).startswith("reduce_span_kernel+scan_partials_kernel+")
        assert lib.kernel_name(lib.OP_SCAN, n, 0).endswith("+uniform_add_kernel")
        assert lib.kernel_name(lib.OP_REDUCE, n, 0) == "reduce_span_kernel<dpp,block>+reduce_final_kernel"
        assert lib.kernel_name(lib.OP_SEGMENTED_REDUCE, 600 * 7, 600).startswith("irregular_reduce_kernel<regular>")
        lib.tuning_import("reduce_any:9=3;scan_any:11=0;scan_any:17=0;scan:12=12;")
        assert lib.kernel_name(lib.OP_SEGMENTED_REDUCE, 600 * 7, 600) == "masked_wave_reduce_kernel"
        assert lib.kernel_name(lib.OP_SEGMENTED_SCAN, 3000 * 7, 3000) == "irregular_scan_kernel<regular>"
        assert lib.kernel_name(lib.OP_SEGMENTED_SCAN, 3 << 20, 3 << 16) == "irregular_scan_kernel<regular>"
        assert lib.kernel_name(lib.OP_SEGMENTED_SCAN, n, 1 << 12) == "scan_block_kernel<mfma,nocarry>"   # a strategy needs long segments
        lib.tuning_import("reduce_any:3=1;reduce_any:4=0;reduce_any:6=4;")
        assert lib.kernel_name(lib.OP_SEGMENTED_REDUCE, 12 * 500, 12).startswith("irregular_reduce_kernel<regular>")
        assert lib.kernel_name(lib.OP_SEGMENTED_REDUCE, 24 * 500, 24) == "rows_reduce_kernel"
        assert lib.kernel_name(lib.OP_SEGMENTED_REDUCE, 100 * 500, 100) == "rows_reduce_kernel"    # no packed rows of 100: the default stays
        lib.tuning_import("reduce_any:5=1;")                 # tiles are for 8 .. 999 elements; 33 fits, ...
        assert lib.kernel_name(lib.OP_SEGMENTED_REDUCE, 33 * 5, 33).startswith("irregular_reduce_kernel<regular>")
        lib.tuning_import("reduce_any:12=1;")                # ... 5000 does not: the default stays
        assert lib.kernel_name(lib.OP_SEGMENTED_REDUCE, 5000 * 5, 5000) == "rows_reduce_kernel"
    finally:
        lib.tuning_import("")
    assert lib.tuning_export() == ""


def test_workspace_bytes_is_a_host_side_bound(lib):
    wb = lib.workspace_bytes
    assert wb(lib.OP_SEGMENTED_SCAN, 0, 16) == 0
    assert wb(lib.OP_SEGMENTED_SCAN, 48, 5) == 0            # 5 does not divide 48
    assert wb(8, 1 << 20, 16) == 0
    small, big = wb(lib.OP_SCAN, 1 << 20, 0), wb(lib.OP_SCAN, 1 << 28, 0)
    assert 768 <= small < big
    # header + two areas of one size: descriptors, one per 16384 elements (8 bytes), and partials, one binary32 per
    # 4096 elements (what the one-segment reduction leaves when every wavefront writes its own)
    exact = 256 + 2 * max((1 << 28) // 16384 * 8, (1 << 28) // 4096 * 4)
    assert exact <= big <= exact + 512                      # (+ one tile for an array that starts 7 elements into a tile)
    assert big % 256 == 0
    # irregular segments: look-up tables and per-tile pairs (reduce), one descriptor per 32768-element tile (scan)
    ired, iscan = wb(lib.OP_IRREGULAR_REDUCE, 1 << 28, 0), wb(lib.OP_IRREGULAR_SCAN, 1 << 28, 0)
    assert ired % 256 == 0 and iscan % 256 == 0
    assert ired >= 256 + 2 * 8 * (4 * (1 << 14) + 2) and iscan >= 256 + 2 * 8 * ((1 << 13) + 1)
    assert ired < 4 << 20 and iscan < 1 << 20
    assert wb(lib.OP_IRREGULAR_SCAN, 0, 0) == 0


def _tiled_reduce_words(n, channels):
    """8-byte words the tiled reduction keeps in the partials area for an array of n elements laid out from the
    16-byte boundary below it (up to 7 elements more): two look-up tables of tiles + 1 entries, one carried-segment
    index per tile, and per channel one pair per tile and per group of 64 tiles."""
    tiles = -(-(n + 7) // 16384)
    groups = -(-tiles // 64)
    return 2 * (tiles + 1) + tiles + channels * (tiles + groups)


@pytest.mark.parametrize("n", [1, 9, 16384, 16385, (1 << 20) - 7, 1 << 20, (1 << 28) + 24])
def test_workspace_bytes_covers_the_tiled_kernels_behind_regular_calls(lib, n):
    # A regular call lands on the tiled kernels of the irregular calls for some lengths (reductions of 5 .. 15
    # elements that are no power of two) and for every length when `in` is not 16-byte aligned; the bound must
    # hold for those too, for both moments as well, and one area must hold the scan's descriptors.
    wb = lib.workspace_bytes
    area = lambda op, seg: (wb(op, n, seg) - 256) // 2
    assert area(lib.OP_SEGMENTED_REDUCE, 1) >= 8 * _tiled_reduce_words(n, 1)
    assert area(lib.OP_REDUCE, 0) >= 8 * _tiled_reduce_words(n, 1)
    assert area(lib.OP_IRREGULAR_REDUCE, 0) >= 8 * _tiled_reduce_words(n, 1)
    assert area(lib.OP_SEGMENTED_MOMENTS, 1) >= 8 * _tiled_reduce_words(n, 2)
    assert area(lib.OP_IRREGULAR_MOMENTS, 0) >= 8 * _tiled_reduce_words(n, 2)
    scan_tiles = -(-(n + 7) // 32768)
    for op in (lib.OP_SEGMENTED_SCAN, lib.OP_SCAN, lib.OP_IRREGULAR_SCAN):
        assert area(op, 1) >= 8 * scan_tiles
    assert area(lib.OP_IRREGULAR_SCAN, 0) >= 8 * (scan_tiles + 1)         # its look-up table
    # the long power-of-two paths: a descriptor per 16384-element share, a partial per 65536-element span
    assert area(lib.OP_SEGMENTED_SCAN, 1) >= 8 * -(-n // 16384)
    assert area(lib.OP_SEGMENTED_REDUCE, 1) >= 4 * -(-n // 65536) * 2
    assert area(lib.OP_REDUCE, 0) >= 4 * -(-n // 4096)                     # one segment: a partial per wavefront span


def test_cxx_header_compiles_and_forwards_every_call(lib, tmp_path):
    # include/tcr.hpp: the paper's API names (Section 6) as inline calls of the C ABI; C++11, warnings as errors
    import shutil
    import subprocess
    from paper_1811_09736_amd import build as b
    if shutil.which("g++") is None:
        pytest.skip("no g++")
    exe = str(tmp_path / "cxx_api")
    cmd = ["g++", "-std=c++11", "-Wall", "-Wextra", "-Werror", "-I" + os.path.join(ROOT, "include"), "-o", exe,
           os.path.join(ROOT, "tests", "sanitize", "cxx_api_driver.cpp"), b.LIB_PATH, "-Wl,-rpath," + os.path.dirname(b.LIB_PATH)]
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert proc.returncode == 0, proc.stdout[-3000:]
    run = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert run.returncode == 0 and run.stdout.strip().endswith("ok"), run.stdout[-3000:]
    # every entry point of the operations has a wrapper
    text = open(os.path.join(ROOT, "include", "tcr.hpp")).read()
    for name in ("tcr_segmented_reduce", "tcr_reduce", "tcr_segmented_scan", "tcr_scan", "tcr_segmented_scan_ex", "tcr_scan_ex",
                 "tcr_irregular_reduce", "tcr_irregular_scan", "tcr_irregular_scan_ex", "tcr_segmented_moments", "tcr_irregular_moments"):
        assert name + "(" in text, name
