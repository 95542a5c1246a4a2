"""CPU-only checks of the boundary: the shared library loads, exports every symbol the header
declares, and rejects bad arguments on the host before any GPU work."""
import os
import re

import pytest

from paper_2311_06281_amd import binding as hb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "heinsen.h")


def _declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(heinsen_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = hb.load()
    declared = _declared_functions()
    assert "heinsen_scan" in declared and len(declared) >= 5
    for name in declared:
        assert hasattr(lib, name), f"{name} declared in heinsen.h but not exported"
    assert sorted(hb.EXPORTS) == declared


def test_header_constants_match_binding():
    text = open(HEADER).read()
    for name, value in hb.FLAGS.items():
        m = re.search(rf"HEINSEN_{name}\s*=\s*1u\s*<<\s*(\d+)", text)
        assert m and (1 << int(m.group(1))) == value
    assert re.search(r"HEINSEN_LAYOUT_BND\s*=\s*0", text) and re.search(r"HEINSEN_LAYOUT_BDN\s*=\s*1", text)


def test_version_and_status_strings():
    assert hb.heinsen_version() >= 100
    for st in range(0, 7):
        assert hb.heinsen_status_string(st) not in ("", "unknown status")
    assert hb.heinsen_status_string(99) == "unknown status"


P = 4096  # a non-null, aligned fake address: validation must fail before it is ever dereferenced


@pytest.mark.parametrize("args,expect", [
    ((0, P, P, P, 1, 1, 8, 0, 0), hb.HEINSEN_ERR_INVALID_ARG),          # null a
    ((P, 0, P, P, 1, 1, 8, 0, 0), hb.HEINSEN_ERR_INVALID_ARG),          # null b
    ((P, P, 0, P, 1, 1, 8, 0, 0), hb.HEINSEN_ERR_INVALID_ARG),          # null x0
    ((P, P, P, 0, 1, 1, 8, 0, 0), hb.HEINSEN_ERR_INVALID_ARG),          # null out
    ((P, P, P, P, 0, 1, 8, 0, 0), hb.HEINSEN_ERR_INVALID_ARG),          # B < 1
    ((P, P, P, P, 1, -3, 8, 0, 0), hb.HEINSEN_ERR_INVALID_ARG),         # D < 1
    ((P, P, P, P, 1, 1, 0, 0, 0), hb.HEINSEN_ERR_INVALID_ARG),          # n < 1
    ((P, P, P, P, 1, 1, 8, 2, 0), hb.HEINSEN_ERR_INVALID_ARG),          # unknown layout
    ((P, P, P, P, 1, 1, 8, 0, 1 << 9), hb.HEINSEN_ERR_INVALID_ARG),     # unknown flag bit
    ((P, P, P, P, 1 << 31, 1 << 31, 1 << 10, 0, 0), hb.HEINSEN_ERR_INVALID_ARG),  # B*D*n overflow
    ((P, P, P, P, 1, 1, 1 << 42, 1, 0), hb.HEINSEN_ERR_UNSUPPORTED),    # more elements than 32-bit tile counters cover
    ((P + 2, P, P, P, 1, 1, 8, 0, 0), hb.HEINSEN_ERR_INVALID_ARG),      # misaligned float32 input
    ((P + 1, P, P, P, 1, 1, 8, 0, hb.HEINSEN_IN_BF16), hb.HEINSEN_ERR_INVALID_ARG),  # misaligned bf16 input
    ((P, P, P, P + 2, 1, 1, 8, 0, 0), hb.HEINSEN_ERR_INVALID_ARG),      # misaligned out
    ((P, P, P, P, 1, 1, 8, 0, hb.HEINSEN_LOG_OUTPUT), hb.HEINSEN_ERR_UNSUPPORTED),  # real log of a signed result
    ((P, P, P, P, 1, 1, 8, 0, hb.HEINSEN_OUT_COMPLEX), hb.HEINSEN_ERR_INVALID_ARG),  # complex output of a linear result
    ((P, P, P, P, 1, 1, 8, 0, hb.HEINSEN_OUT_COMPLEX | hb.HEINSEN_LOG_OUTPUT | hb.HEINSEN_LOG_INPUTS),
     hb.HEINSEN_ERR_UNSUPPORTED),                                       # complex output of log-domain inputs
    ((P, P, P, P, 1, 1, 8, 0, hb.HEINSEN_LINEAR | hb.HEINSEN_LOG_INPUTS), hb.HEINSEN_ERR_INVALID_ARG),  # linear path on log data
    ((P, P, P, P + 4, 1, 1, 8, 0, hb.HEINSEN_OUT_COMPLEX | hb.HEINSEN_LOG_OUTPUT), hb.HEINSEN_ERR_INVALID_ARG),  # misaligned complex out
])
def test_bad_arguments_are_rejected_on_the_host(args, expect):
    assert hb.heinsen_scan_status(*args) == expect


def test_tile_shape_of_the_benchmark_workloads():
    assert hb.heinsen_tile_shape(16, 2048, 16384, hb.HEINSEN_LAYOUT_BND, 0) == (128, 128)  # wide tile
    assert hb.heinsen_tile_shape(8, 1024, 4096, hb.HEINSEN_LAYOUT_BND, 0) == (64, 256)
    assert hb.heinsen_tile_shape(2, 16384, 1229, hb.HEINSEN_LAYOUT_BND, hb.HEINSEN_POSITIVE) == (128, 128)
    assert hb.heinsen_tile_shape(2, 16384, 1000, hb.HEINSEN_LAYOUT_BND, 0) == (64, 256)    # too short for the wide tile
    assert hb.heinsen_tile_shape(1, 1, 1 << 26, hb.HEINSEN_LAYOUT_BDN, 8) == (1, 16384)
    assert hb.heinsen_tile_shape(1, 1, 4096, hb.HEINSEN_LAYOUT_BDN, 8) == (1, 4096)
    assert hb.heinsen_tile_shape(64, 4096, 2048, hb.HEINSEN_LAYOUT_BDN, 7) == (4, 2048)
    with pytest.raises(hb.HeinsenError):
        hb.heinsen_tile_shape(1, 1, 0, 0, 0)


def test_kernel_name_follows_layout_and_length():
    assert hb.heinsen_kernel_name(8, 1024, 4096, hb.HEINSEN_LAYOUT_BND, 0) == "heinsen_scan_bnd"
    assert hb.heinsen_kernel_name(64, 4096, 2048, hb.HEINSEN_LAYOUT_BDN, 7) == "heinsen_scan_rows_wave"
    assert hb.heinsen_kernel_name(1, 1, 1 << 26, hb.HEINSEN_LAYOUT_BDN, 8) == "heinsen_scan_tiles"
    assert hb.heinsen_kernel_name(64, 64, 64, hb.HEINSEN_LAYOUT_BDN, 0) == "heinsen_scan_rows_packed"
    with pytest.raises(hb.HeinsenError):
        hb.heinsen_kernel_name(1, 1, 0, 0, 0)


def test_bench_refuses_more_than_one_gpu():
    """bench.py is a one-GPU measurement; asking for more must end with a message, not a wrong number."""
    import subprocess
    import sys

    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""
