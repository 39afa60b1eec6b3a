"""The C-ABI library loads without a GPU and exports every symbol include/pipad.h declares."""
import ctypes
import os
import re

import paper_2301_00391_amd as pipad
from paper_2301_00391_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    names = set()
    for header in sorted(os.listdir(os.path.join(ROOT, "include"))):
        text = open(os.path.join(ROOT, "include", header)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(pipad_[a-z_]+)\s*\(", text))
    return sorted(names - {"pipad_alloc_fn"})


def test_header_symbols_are_exported_and_bound():
    lib = pipad.load_library()
    names = declared_symbols()
    assert "pipad_frame_build_overlap" in names and "pipad_frame_aggregate" in names
    for name in names:
        assert hasattr(lib, name), f"{name} is declared in pipad.h but not exported"
        assert name in binding.SIGNATURES, f"{name} has no binding signature"
    assert sorted(binding.SIGNATURES) == names


def test_host_only_calls():
    lib = pipad.load_library()
    assert lib.pipad_strerror(0) == b"ok"
    assert lib.pipad_strerror(-2).startswith(b"snapshot")
    assert lib.pipad_strerror(12345) == b"unknown status"
    assert lib.pipad_last_hip_error() == b""
    before = pipad.get_option("agg_nt")
    pipad.set_option("agg_nt", 2)
    assert pipad.get_option("agg_nt") == 2
    pipad.set_option("agg_nt", before)
    assert lib.pipad_set_option(b"no_such_key", 1) == -1
    # argument checks that need no device
    out = ctypes.c_void_p()
    assert lib.pipad_frame_build_overlap(4, 0, None, 0, None, None, None, ctypes.byref(out)) == -1
    assert lib.pipad_frame_aggregate(None, 4, None, 4, None, 4, None) == -1
    lib.pipad_frame_destroy(None)


def test_coalescent_row_bytes_match_the_paper(golden_dir):
    """Section 5.3: 16 bytes for two graphs at F = 2, 256 bytes for four graphs at F = 16."""
    for line in open(os.path.join(golden_dir, "coalescent_row_bytes.txt")):
        if line.startswith("#") or not line.strip():
            continue
        snaps, feat, nbytes = map(int, line.split())
        assert pipad.coalescent_row_bytes(snaps, feat) == nbytes


def test_padded_row_stride():
    """Rows within one 128-byte line: the next power of two (no row straddles two lines); longer
    rows: an odd number of 128-byte lines."""
    import paper_2301_00391_amd as pipad
    for feat in (33, 64, 96, 128, 130, 256):
        stride = pipad.padded_row_stride(feat)
        assert stride >= feat and stride % 32 == 0 and (stride // 32) % 2 == 1
        assert stride - feat < 64  # never more than two lines of padding
    for feat in range(1, 33):
        stride = pipad.padded_row_stride(feat)
        assert feat <= stride < 2 * feat and stride & (stride - 1) == 0
    assert pipad.padded_row_stride(64) == 96 and pipad.padded_row_stride(32) == 32
    assert pipad.padded_row_stride(6) == 8 and pipad.padded_row_stride(16) == 16
