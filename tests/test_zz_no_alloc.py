"""The allocation-free backward entry point against aeris_winattn_bwd (which the parity tests
hold to the oracle): same kernels, scratch in the library's static device array instead of the
caller's workspace, so results must be bit-identical.  Two calls in a row on the same device,
the second with a smaller problem (the array keeps the first call's contents), then the first
again."""
import ctypes

import numpy as np
import pytest
import torch

from paper_2509_13523_amd import binding as B
from paper_2509_13523_amd import synth

pytestmark = pytest.mark.gpu


def dev(bits):
    return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)


def bits_of(t):
    return t.view(torch.int16) if t.dtype == torch.bfloat16 else t.view(torch.int32)


def run_pair(shape, win, shift, mask, seed, out_dtype):
    """Returns True if the static entry point reproduced aeris_winattn_bwd bit for bit."""
    Bn, H, W, nh, d = shape
    tq, tk, tv, tdo = [dev(b) for b in synth.make_inputs("blend", seed, shape, 4)]
    o, lse = B.aeris_winattn_fwd(tq, tk, tv, win, shift, mask, out_dtype=out_dtype)
    want = B.aeris_winattn_bwd(tq, tk, tv, o, lse, tdo, win, shift, mask, out_dtype=out_dtype)
    got = [torch.full_like(w, float("nan")) for w in want]
    torch.cuda.synchronize()
    # straight through the C ABI: plain pointers, no workspace argument
    p = B.make_params(shape, win, shift, mask, out_dtype=out_dtype)
    rc = B.load().aeris_winattn_bwd_static(
        ctypes.byref(p), tq.data_ptr(), tk.data_ptr(), tv.data_ptr(), o.data_ptr(),
        lse.data_ptr(), tdo.data_ptr(), got[0].data_ptr(), got[1].data_ptr(), got[2].data_ptr(),
        torch.cuda.current_stream().cuda_stream)
    assert rc == 0, B.aeris_winattn_strerror(rc)
    torch.cuda.synchronize()
    for g, w in zip(got, want):
        assert torch.isfinite(g.float()).all()
        assert torch.equal(bits_of(g), bits_of(w))


def test_static_scratch_backward_two_calls_second_smaller():
    big = ((2, 60, 90, 3, 128), (30, 30), (15, 15), B.AERIS_MASK_SWIN)     # T = 900, ragged tiles
    small = ((1, 24, 36, 2, 64), (12, 12), (6, 6), B.AERIS_MASK_LAT)
    run_pair(*big, seed=8101, out_dtype=B.AERIS_DT_BF16)
    run_pair(*small, seed=8102, out_dtype=B.AERIS_DT_F32)
    run_pair(*big, seed=8103, out_dtype=B.AERIS_DT_BF16)


def test_static_scratch_backward_rejects_what_does_not_fit():
    # 288 windows of 60x60 x 16 heads: 16.6 million (token, head) entries, twice the array
    shape, win, shift = (1, 720, 1440, 16, 128), (60, 60), (30, 30)
    p = B.make_params(shape, win, shift, B.AERIS_MASK_SWIN)
    assert B.aeris_winattn_bwd_workspace_bytes(p) > B.AERIS_BWD_STATIC_SCRATCH_BYTES
    t = torch.zeros(8, dtype=torch.bfloat16, device="cuda")       # never touched: rejected first
    f = torch.zeros(8, dtype=torch.float32, device="cuda")
    rc = B.load().aeris_winattn_bwd_static(
        ctypes.byref(p), t.data_ptr(), t.data_ptr(), t.data_ptr(), t.data_ptr(), f.data_ptr(),
        t.data_ptr(), t.data_ptr(), t.data_ptr(), t.data_ptr(), None)
    assert rc == -13
    assert "AERIS_BWD_STATIC_SCRATCH_BYTES" in B.aeris_winattn_strerror(rc)
