"""C-ABI checks that need no GPU: the library loads, exports every symbol the
header declares, and rejects bad arguments before launching anything."""
import ctypes
import os
import re

import pytest

from paper_2509_13523_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_exports_match_header():
    text = open(os.path.join(ROOT, "include", "aeris_winattn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(aeris_winattn_[a-z_]+)\s*\(", text))
    assert declared == set(B.EXPORTS)
    lib = B.load()
    for name in declared:
        assert getattr(lib, name) is not None


def test_version_and_strerror():
    assert B.aeris_winattn_version() >= 100
    assert B.aeris_winattn_strerror(0) == "ok"
    for code in range(-11, 0):
        assert B.aeris_winattn_strerror(code) != "unknown error code"
    assert B.aeris_winattn_strerror(-99) == "unknown error code"


def good():
    return dict(shape=(1, 64, 128, 4, 32), win=(8, 8), shift=(4, 4), mask=B.AERIS_MASK_SWIN)


@pytest.mark.parametrize("change,code", [
    ({}, 0),
    ({"shape": (1, 64, 128, 4, 48)}, -6),
    ({"shape": (1, 64, 128, 4, 256)}, -6),
    ({"shape": (0, 64, 128, 4, 32)}, -2),
    ({"shape": (1, 64, 128, 0, 32)}, -2),
    ({"win": (7, 8)}, -3),
    ({"win": (8, 12)}, -3),
    ({"shift": (8, 0)}, -4),
    ({"shift": (0, -1)}, -4),
    ({"mask": 3}, -5),
    ({"out_dtype": 2}, -10),
    ({"shape": (1, 128, 128, 1, 32), "win": (128, 128), "shift": (0, 0)}, -9),
    ({"qkv_strides": (4 * 32 * 3 + 4, 32)}, -7),
    ({"qkv_strides": (64, 32)}, -2),
    ({"o_strides": (128, 16)}, -2),
    ({"qkv_strides": (3 * 4 * 32, 32)}, 0),
])
def test_validate(change, code):
    kw = good()
    kw.update(change)
    assert B.aeris_winattn_validate(B.make_params(**kw)) == code


def test_null_and_misaligned_pointers_rejected_before_launch():
    lib = B.load()
    p = B.make_params(**good())
    fake = 0x1000   # never dereferenced: validation fails first
    assert lib.aeris_winattn_fwd(None, fake, fake, fake, fake, fake, None) == -1
    assert lib.aeris_winattn_fwd(ctypes.byref(p), fake, None, fake, fake, fake, None) == -1
    assert lib.aeris_winattn_fwd(ctypes.byref(p), fake, fake, fake + 8, fake, fake, None) == -7
    args = [fake] * 10
    assert lib.aeris_winattn_bwd(ctypes.byref(p), *args[:9], None, 1 << 30, None) == -1
    need = B.aeris_winattn_bwd_workspace_bytes(p)
    assert need == 2 * (1 * 4 * 64 * 128 + 64) * 4
    assert lib.aeris_winattn_bwd(ctypes.byref(p), *args, need - 1, None) == -8
    bad = B.make_params(**dict(good(), win=(7, 8)))
    assert B.aeris_winattn_bwd_workspace_bytes(bad) == 0
    assert lib.aeris_winattn_bwd(ctypes.byref(bad), *args, need, None) == -3
