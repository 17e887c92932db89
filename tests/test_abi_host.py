"""C-ABI checks that need no GPU: the library loads, exports every symbol the
header declares, and rejects bad arguments before launching anything."""
import ctypes
import os
import re

import pytest

from paper_2509_13523_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_exports_match_header():
    declared = set()
    for header in sorted(os.listdir(os.path.join(ROOT, "include"))):
        text = open(os.path.join(ROOT, "include", header)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        declared |= set(re.findall(r"\b(aeris_[a-z0-9_]+)\s*\(", text))
    assert declared == set(B.EXPORTS)
    lib = B.load()
    for name in declared:
        assert getattr(lib, name) is not None


def test_version_and_strerror():
    v = B.aeris_winattn_version()          # major * 10000 + minor * 100 + patch
    assert v >= 20000 and v % 100 < 100 and (v // 100) % 100 < 100
    assert B.aeris_winattn_strerror(0) == "ok"
    for code in range(-14, 0):
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


def test_static_scratch_backward_rejects_before_launch():
    """The allocation-free backward validates like aeris_winattn_bwd and refuses problems whose
    statistics do not fit its static array, all before any HIP call."""
    lib = B.load()
    fake = 0x1000
    args = [fake] * 9
    p = B.make_params(**good())
    assert lib.aeris_winattn_bwd_static(None, *args, None) == -1
    assert lib.aeris_winattn_bwd_static(ctypes.byref(p), *args[:8], None, None) == -1
    assert lib.aeris_winattn_bwd_static(ctypes.byref(p), fake + 2, *args[1:], None) == -7
    bad = B.make_params(**dict(good(), shift=(8, 0)))
    assert lib.aeris_winattn_bwd_static(ctypes.byref(bad), *args, None) == -4
    # 97 windows of 60x60 x 24 heads still fit 64 MiB; 98 do not
    fits = B.make_params((1, 60, 97 * 60, 24, 128), (60, 60), (30, 30), B.AERIS_MASK_SWIN)
    assert B.aeris_winattn_bwd_workspace_bytes(fits) <= B.AERIS_BWD_STATIC_SCRATCH_BYTES
    big = B.make_params((1, 60, 98 * 60, 24, 128), (60, 60), (30, 30), B.AERIS_MASK_SWIN)
    assert B.aeris_winattn_bwd_workspace_bytes(big) > B.AERIS_BWD_STATIC_SCRATCH_BYTES
    assert lib.aeris_winattn_bwd_static(ctypes.byref(big), *args, None) == -13
    header = open(os.path.join(ROOT, "include", "aeris_winattn.h")).read()
    m = re.search(r"#define AERIS_BWD_STATIC_SCRATCH_BYTES \((\d+)u << (\d+)\)", header)
    assert int(m.group(1)) << int(m.group(2)) == B.AERIS_BWD_STATIC_SCRATCH_BYTES


def test_rope_arguments_rejected_before_launch():
    lib = B.load()
    p = B.make_params((1, 64, 128, 4, 32), (8, 8), (4, 4))
    buf = (ctypes.c_char * 64)()
    a = ctypes.addressof(buf)
    a += (-a) % 16
    for base, pos, code in ((1.0, 0, -12), (0.0, 0, -12), (-5.0, 1, -12), (100.0, 2, -12),
                            (float("inf"), 0, -12)):
        r = B.aeris_rope_params(base, pos)
        assert lib.aeris_rope2d_apply(ctypes.byref(p), ctypes.byref(r), a, a, 0, None) == code
        assert lib.aeris_winattn_rope_fwd(ctypes.byref(p), ctypes.byref(r), a, a, a, a, a, a,
                                          1 << 40, None) == code
    r = B.aeris_rope_params(100.0, 0)
    assert lib.aeris_rope2d_apply(ctypes.byref(p), None, a, a, 0, None) == -1
    assert lib.aeris_rope2d_apply(ctypes.byref(p), ctypes.byref(r), None, a, 0, None) == -1
    assert lib.aeris_rope2d_apply(ctypes.byref(p), ctypes.byref(r), a + 2, a, 0, None) == -7
    # workspace sizes: two compact bf16 tensors forward (rotated k and q, kept for the backward
    # pass); backward two of them plus the statistics, or the statistics alone with `saved`
    half = 1 * 64 * 128 * 4 * 32 * 2
    tensor = 2 * half
    stats = B.aeris_winattn_bwd_workspace_bytes(p)
    assert B.aeris_winattn_rope_fwd_workspace_bytes(p) == tensor
    assert B.aeris_winattn_rope_bwd_workspace_bytes(p) == 2 * half + stats
    assert lib.aeris_winattn_rope_fwd(ctypes.byref(p), ctypes.byref(r), a, a, a, a, a, a,
                                      tensor - 1, None) == -8
    P, R = ctypes.byref(p), ctypes.byref(r)
    assert lib.aeris_winattn_rope_bwd(P, R, a, a, a, a, a, a, a, a, a, None, a, 2 * half, None) == -8
    assert lib.aeris_winattn_rope_bwd(P, R, a, a, a, a, a, a, a, a, a, a, a, stats - 1, None) == -8
    assert lib.aeris_winattn_rope_bwd(P, R, None, a, a, a, a, a, a, a, a, None, a, 1 << 40, None) == -1
    assert lib.aeris_winattn_rope_bwd(P, R, None, None, a, a, a, a, a, a, a, a + 4, a, 1 << 40,
                                      None) == -7
    # the same calls on a list of windows
    P, R = ctypes.byref(p), ctypes.byref(r)
    assert lib.aeris_winattn_rope_fwd_windows(P, R, None, 4, a, a, a, a, a, a, tensor, None) == -1
    assert lib.aeris_winattn_rope_fwd_windows(P, R, a, 0, a, a, a, a, a, a, tensor, None) == -2
    assert lib.aeris_winattn_rope_fwd_windows(P, R, a, 8 * 16 + 1, a, a, a, a, a, a, tensor, None) == -2
    assert lib.aeris_winattn_rope_fwd_windows(P, R, a + 2, 4, a, a, a, a, a, a, tensor, None) == -7
    assert lib.aeris_winattn_rope_fwd_windows(P, R, a, 4, a, a, a, a, a, a, tensor - 1, None) == -8
    assert lib.aeris_winattn_rope_fwd_windows(P, None, a, 4, a, a, a, a, a, a, tensor, None) == -1
    assert lib.aeris_winattn_rope_bwd_windows(P, R, a, 4, a, a, a, a, a, a, a, a, a, None, a,
                                              2 * half, None) == -8
    assert lib.aeris_winattn_rope_bwd_windows(P, R, a, 4, a, a, a, a, a, a, a, None, a, None, a,
                                              1 << 40, None) == -1


def test_window_list_arguments_rejected_before_launch():
    lib = B.load()
    p = B.make_params((1, 64, 128, 4, 32), (8, 8), (4, 4))      # 8 x 16 = 128 windows
    buf = (ctypes.c_char * 64)()
    a = ctypes.addressof(buf)
    a += (-a) % 16
    fwd = lambda lst, n: lib.aeris_winattn_fwd_windows(ctypes.byref(p), lst, n, a, a, a, a, a, None)
    assert fwd(None, 4) == -1
    assert fwd(a, 0) == -2
    assert fwd(a, -3) == -2
    assert fwd(a, 129) == -2
    assert fwd(a + 2, 4) == -7
    assert lib.aeris_winattn_bwd_windows(ctypes.byref(p), None, 4, a, a, a, a, a, a, a, a, a, a,
                                         1 << 30, None) == -1
    # four of 128 windows need 1/32 of the full workspace (plus padding): 16 bytes are too few
    assert lib.aeris_winattn_bwd_windows(ctypes.byref(p), a, 4, a, a, a, a, a, a, a, a, a, a,
                                         16, None) == -8


def test_header_is_plain_c_and_callable_from_c(tmp_path):
    """Compiles tests/c/abi_check.c as C99 against include/aeris_winattn.h, links it to the
    library and runs it: struct layout as the binding assumes, host-only calls work from C."""
    import subprocess
    B.load()
    exe = str(tmp_path / "abi_check")
    lib_dir = os.path.dirname(B.LIB_PATH)
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Werror", "-pedantic", "-I", os.path.join(ROOT, "include"),
                    os.path.join(ROOT, "tests", "c", "abi_check.c"), "-o", exe,
                    "-L", lib_dir, "-laeris_winattn", "-Wl,-rpath," + lib_dir,
                    "-Wl,-rpath,/opt/rocm/lib", "-Wl,--allow-shlib-undefined"], check=True)
    out = subprocess.run([exe], check=True, capture_output=True, text=True).stdout
    got = dict(l.split(" ", 1) for l in out.strip().splitlines())
    assert int(got["sizeof_params"]) == ctypes.sizeof(B.aeris_winattn_params)
    assert int(got["offset_strides"]) == B.aeris_winattn_params.qkv_tok_stride.offset
    assert int(got["sizeof_rope"]) == ctypes.sizeof(B.aeris_rope_params)
    assert int(got["version"]) == B.aeris_winattn_version()
    assert got["validate"] == "0"
    assert got["validate_bad"].startswith("-3 window does not divide")
    assert int(got["bwd_ws"]) == 2 * (1 * 128 * 4 * 64 + 64) * 4
    assert int(got["rope_fwd_ws"]) == 2 * 64 * 128 * 4 * 32 * 2
    assert got["null_fwd"] == "-1" and got["null_rope"] == "-1"


# ------------------------------------------------------------------ include/aeris_layer_ops.h
def test_layer_ops_reject_bad_arguments_before_launching():
    lib = B.load()
    a = ctypes.c_void_p(4096)          # a non-null, aligned address that is never dereferenced
    odd = ctypes.c_void_p(4096 + 8)
    ok = (a, a, a, a, 1e-6, 8, 4, 64, a, a, None)
    assert lib.aeris_rmsnorm_adaln_fwd(None, a, a, a, 1e-6, 8, 4, 64, a, a, None) == -1
    assert lib.aeris_rmsnorm_adaln_fwd(a, a, a, a, 1e-6, 8, 4, 64, None, a, None) == -1
    assert lib.aeris_rmsnorm_adaln_fwd(a, a, a, a, 1e-6, 0, 4, 64, a, a, None) == -2
    assert lib.aeris_rmsnorm_adaln_fwd(a, a, a, a, 1e-6, 8, 4, 4104, a, a, None) == -2   # too wide
    assert lib.aeris_rmsnorm_adaln_fwd(a, a, a, a, 1e-6, 8, 4, 4, a, a, None) == -2      # too narrow
    assert lib.aeris_rmsnorm_adaln_fwd(a, a, a, a, 1e-6, 8, 4, 60, a, a, None) == -3     # 60 % 8
    assert lib.aeris_rmsnorm_adaln_fwd(a, a, a, a, 1e-6, 8, 3, 64, a, a, None) == -3     # 8 % 3
    assert lib.aeris_rmsnorm_adaln_fwd(a, a, a, a, -1.0, 8, 4, 64, a, a, None) == -2
    assert lib.aeris_rmsnorm_adaln_fwd(odd, a, a, a, 1e-6, 8, 4, 64, a, a, None) == -7
    assert len(ok) == 11
    need = lib.aeris_rmsnorm_adaln_bwd_workspace_bytes(8, 4, 64)
    assert need == 2 * 1 * 2 * 64 * 4           # two samples, one chunk each, two rows of 64 floats
    assert lib.aeris_rmsnorm_adaln_bwd_workspace_bytes(8, 3, 64) == 0
    assert lib.aeris_rmsnorm_adaln_bwd(a, a, a, a, a, 8, 4, 64, a, None, None, None, a, need - 1,
                                       None) == -8
    assert lib.aeris_rmsnorm_adaln_bwd(a, a, a, a, a, 8, 4, 64, a, None, None, None, None, need,
                                       None) == -1
    # the residual form: same checks, dres optional but aligned
    assert lib.aeris_rmsnorm_adaln_bwd_residual(a, a, a, a, a, None, 8, 4, 64, a, None, None, None, a,
                                                need - 1, None) == -8
    assert lib.aeris_rmsnorm_adaln_bwd_residual(a, a, a, a, a, odd, 8, 4, 64, a, None, None, None, a,
                                                need, None) == -7
    assert lib.aeris_rmsnorm_adaln_bwd_residual(a, a, a, a, None, a, 8, 4, 64, a, None, None, None, a,
                                                need, None) == -1
    assert lib.aeris_gate_residual_fwd(a, None, a, 8, 4, 64, a, None) == -1
    assert lib.aeris_gate_residual_fwd(a, a, a, 8, 4, 64, odd, None) == -7
    assert lib.aeris_gate_residual_bwd_workspace_bytes(8, 4, 64) == 2 * 64 * 4
    assert lib.aeris_gate_residual_bwd(a, a, a, 8, 4, 64, a, None, a, 8, None) == -8
    assert lib.aeris_swiglu_fwd(a, 8, 12, a, None) == -3
    assert lib.aeris_swiglu_fwd(a, 0, 16, a, None) == -2
    assert lib.aeris_swiglu_fwd(None, 8, 16, a, None) == -1
    assert lib.aeris_swiglu_bwd(a, odd, 8, 16, a, None) == -7


def test_layer_ops_workspace_grows_with_the_number_of_chunks():
    lib = B.load()
    # 4 samples of 1,036,800 rows: 512 chunks per sample (2048 workgroups in all)
    assert lib.aeris_rmsnorm_adaln_bwd_workspace_bytes(4 * 1036800, 1036800, 2048) == 2048 * 2 * 2048 * 4
    # tiny samples: at most one chunk per four rows
    assert lib.aeris_gate_residual_bwd_workspace_bytes(6, 6, 8) == 2 * 8 * 4


def test_projections_reject_bad_arguments_before_launching():
    lib = B.load()
    a = ctypes.c_void_p(4096)
    odd = ctypes.c_void_p(4096 + 8)
    need = lib.aeris_norm_linear_workspace_bytes(512, 256, 128, 384)
    # folded weights (2 samples x 384 x 128 bf16) + biases (2 x 384 fp32) + r (512 fp32), each
    # rounded up to 256 bytes
    assert need == 2 * 384 * 128 * 2 + 2 * 384 * 4 + 512 * 4
    assert lib.aeris_norm_linear_workspace_bytes(512, 256, 96, 384) == 0       # 96 % 64
    ok = lambda **kw: lib.aeris_norm_linear_fwd(
        kw.get("x", a), a, a, a, kw.get("eps", 1e-6), a, kw.get("n", 512), kw.get("rps", 256),
        kw.get("c", 128), kw.get("f", 384), kw.get("y", a), a, kw.get("ws", need), None)
    assert ok(x=None) == -1 and ok(y=None) == -1
    assert ok(c=96) == -3 and ok(f=12) == -3 and ok(rps=100) == -3
    assert ok(c=32) == -2 and ok(c=16384) == -2 and ok(n=0) == -2 and ok(eps=-1.0) == -2
    assert ok(x=odd) == -7
    assert ok(ws=need - 1) == -8
    sw = lambda **kw: lib.aeris_norm_linear_swiglu_fwd(
        a, a, a, a, 1e-6, a, 512, 256, 128, kw.get("h", 192), kw.get("g", a), kw.get("uv", None),
        a, kw.get("ws", need), None)
    assert sw(g=None) == -1 and sw(h=100) == -3 and sw(h=0) == -2 and sw(ws=need - 1) == -8
    lin = lambda **kw: lib.aeris_linear_fwd(kw.get("x", a), a, kw.get("n", 512), kw.get("c", 128),
                                            kw.get("f", 384), kw.get("y", a), None)
    assert lin(x=None) == -1 and lin(c=100) == -3 and lin(f=4) == -2 and lin(y=odd) == -7


def test_linear_bwd_rejects_bad_arguments_before_launching():
    lib = B.load()
    a = ctypes.c_void_p(4096)
    odd = ctypes.c_void_p(4096 + 8)
    # 2048 rows, 256 channels, 512 features: 2 output tiles, 32 steps -> 2 row ranges of 16 steps;
    # transposed weight (512 x 256 bf16) + 2 partial results (512 x 256 fp32)
    need = lib.aeris_linear_bwd_workspace_bytes(2048, 256, 512)
    assert need == 512 * 256 * 2 + 2 * 512 * 256 * 4
    # the headline QKV shape: 192 tiles in 6 units of 32; 64800 steps in 12 row ranges (72 units:
    # nine for each XCD)
    assert lib.aeris_linear_bwd_workspace_bytes(4 * 720 * 1440, 2048, 6144) == 6144 * 2048 * (2 + 12 * 4)
    # 2000 rows: 31 whole steps in 2 row ranges; the 16 rows left over are added with them
    assert lib.aeris_linear_bwd_workspace_bytes(2000, 256, 512) == need
    # one row range and nothing left over: the tile kernel writes dW itself
    assert lib.aeris_linear_bwd_workspace_bytes(1024, 256, 512) == 512 * 256 * 2
    assert lib.aeris_linear_bwd_workspace_bytes(1000, 256, 512) == 512 * 256 * 2 + 512 * 256 * 4
    assert lib.aeris_linear_bwd_workspace_bytes(2048, 256, 520) == 0          # 520 % 64
    call = lambda **kw: lib.aeris_linear_bwd(
        kw.get("x", a), kw.get("w", a), kw.get("dy", a), kw.get("n", 2048), kw.get("c", 256),
        kw.get("f", 512), kw.get("dx", a), kw.get("dw", a), kw.get("wsp", a), kw.get("ws", need), None)
    assert call(dy=None) == -1 and call(wsp=None) == -1 and call(dx=None, dw=None) == -1
    assert call(w=None) == -1 and call(x=None) == -1            # needed by the outputs asked for
    assert call(c=96) == -3 and call(f=520) == -3
    assert call(n=0) == -2 and call(c=0) == -2
    assert call(dx=odd) == -7 and call(dy=odd) == -7
    assert call(ws=need - 1) == -8
