"""The C-ABI library loads and exports every function include/vardrop.h declares (no GPU needed)."""
import ctypes
import os
import re

import paper_2501_14183_amd as vd
from paper_2501_14183_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "vardrop.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(vardrop_[a-z0-9_]+)\s*\(", text)))


def test_header_declares_the_five_hot_path_calls():
    names = declared_functions()
    for need in ("vardrop_hash", "vardrop_sample", "vardrop_gather", "vardrop_attn_fwd", "vardrop_attn_bwd"):
        assert need in names


def test_library_exports_every_declared_symbol():
    lib = ctypes.CDLL(vd.library_path())
    for name in declared_functions():
        assert hasattr(lib, name), name


def test_binding_covers_every_declared_symbol():
    assert sorted(binding._SIGNATURES) == declared_functions()


def test_host_only_calls():
    lib = vd.load_library()
    assert lib.vardrop_strerror(0) == b"ok"
    assert lib.vardrop_strerror(-1) == b"invalid argument"
    assert lib.vardrop_strerror(-77) == b"unknown error code"
    # saved = q, k, v, o in bf16 + log-sum-exp in fp32, rounded up to 256 bytes
    assert lib.vardrop_attn_saved_bytes(32, 130, 512, 8, vd.BF16) == 4 * 32 * 130 * 512 * 2 + 32 * 8 * 130 * 4
    assert lib.vardrop_attn_saved_bytes(4, 10, 64, 2, vd.F32) == 4 * 4 * 10 * 64 * 4 + 4 * 2 * 10 * 4 + 192
    assert lib.vardrop_attn_saved_bytes(4, 10, 64, 3, vd.F32) == 0            # H does not divide d
    assert lib.vardrop_attn_workspace_bytes(1, 1, 64, 1, vd.BF16) >= 4 * 64 * 2 + 4
