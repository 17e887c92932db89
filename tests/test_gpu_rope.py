"""GPU parity of the rotary-embedding entry points against oracle/rope_oracle.py.

The kernels multiply in bf16, so the rotated queries and keys are rounded to bf16 before the
logits; the oracle rounds nothing (fp64 throughout).  That extra operand rounding stays inside
the attention tolerances of tests/test_gpu_parity.py, which apply unchanged here.  The rotation
itself is checked element by element: a rotated pair may differ from the fp64 value by the bf16
rounding of its components (2^-9 relative each) plus the error of the hardware sine and cosine,
together bounded by 2^-8 of the pair's length.
"""
import numpy as np
import pytest
import torch

from oracle import rope_oracle as ro
from oracle import winattn_oracle as orc
from paper_2509_13523_amd import binding as B
from paper_2509_13523_amd import synth
from test_gpu_parity import LSE_ABS, check, check_lse, to_dev, to_f64

pytestmark = pytest.mark.gpu

MODES = [B.AERIS_ROPE_POS_WINDOW, B.AERIS_ROPE_POS_GRID]


def pair_error_ok(got, ref):
    err2 = (got[..., 0::2] - ref[..., 0::2]) ** 2 + (got[..., 1::2] - ref[..., 1::2]) ** 2
    len2 = ref[..., 0::2] ** 2 + ref[..., 1::2] ** 2
    return bool((err2 <= (2.0 ** -8) ** 2 * len2 + 1e-12).all())


@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("shape,win,shift", [
    ((2, 24, 36, 3, 32), (12, 12), (6, 6)),
    ((1, 60, 1440, 1, 64), (60, 60), (30, 30)),     # longitude positions up to 1439
    ((1, 40, 60, 2, 128), (20, 20), (0, 0)),
])
def test_rope2d_apply_elementwise(mode, shape, win, shift):
    (bits,) = synth.make_inputs("normal", 4001, shape, 1)
    x64 = synth.bf16_bits_to_f64(bits)
    tx = to_dev(bits)
    Bn, H, W, nh, d = shape
    phi = ro.angles(H, W, d, win, shift, 100.0, ro.POS_GRID if mode else ro.POS_WINDOW)
    ty = B.aeris_rope2d_apply(tx, win, shift, 100.0, mode)
    torch.cuda.synchronize()
    assert pair_error_ok(to_f64(ty), ro.rotate(x64, phi))
    # inverse, in place: back to the input within two roundings
    tz = ty.clone()
    B.aeris_rope2d_apply(tz, win, shift, 100.0, mode, inverse=True, y=tz)
    torch.cuda.synchronize()
    back = to_f64(tz)
    assert pair_error_ok(back, ro.rotate(to_f64(ty), phi, inverse=True))
    err2 = (back[..., 0::2] - x64[..., 0::2]) ** 2 + (back[..., 1::2] - x64[..., 1::2]) ** 2
    len2 = x64[..., 0::2] ** 2 + x64[..., 1::2] ** 2
    assert (err2 <= (2.0 ** -7) ** 2 * len2 + 1e-12).all()


def test_rope2d_apply_other_base_and_origin_identity():
    shape, win, shift = (1, 16, 16, 2, 32), (8, 8), (4, 4)
    (bits,) = synth.make_inputs("normal", 4002, shape, 1)
    x64 = synth.bf16_bits_to_f64(bits)
    ty = B.aeris_rope2d_apply(to_dev(bits), win, shift, 10000.0, B.AERIS_ROPE_POS_GRID)
    torch.cuda.synchronize()
    phi = ro.angles(16, 16, 32, win, shift, 10000.0, ro.POS_GRID)
    got = to_f64(ty)
    assert pair_error_ok(got, ro.rotate(x64, phi))
    np.testing.assert_array_equal(got[0, 0, 0], x64[0, 0, 0])     # position (0, 0): untouched


def run_rope_case(shape, win, shift, mask, mode, base=100.0, kind="normal", seed=4100,
                  outs=(B.AERIS_DT_F32, B.AERIS_DT_BF16)):
    bits = synth.make_inputs(kind, seed, shape, 4)
    q64, k64, v64, do64 = [synth.bf16_bits_to_f64(b) for b in bits]
    tq, tk, tv, tdo = [to_dev(b) for b in bits]
    pm = ro.POS_GRID if mode == B.AERIS_ROPE_POS_GRID else ro.POS_WINDOW
    o_ref, lse_ref = ro.winattn_rope_fwd(q64, k64, v64, win, shift, mask, base, pm)
    dq_ref, dk_ref, dv_ref = ro.winattn_rope_bwd(q64, k64, v64, do64, win, shift, mask, base, pm)
    # the embedding must matter in this case, or the test proves nothing
    o_plain, _ = orc.winattn_fwd(q64, k64, v64, win, shift, mask)
    assert np.linalg.norm(o_plain - o_ref) > 0.05 * np.linalg.norm(o_ref)
    for out in outs:
        bf = out == B.AERIS_DT_BF16
        o, lse, saved = B.aeris_winattn_rope_fwd(tq, tk, tv, win, shift, base, mode, mask,
                                                 out_dtype=out, return_saved=True)
        torch.cuda.synchronize()
        check("o", o, o_ref, bf)
        check_lse(lse, lse_ref)
        # with the rotated operands the forward call left behind, and rotating again: same bits
        dq, dk, dv = B.aeris_winattn_rope_bwd(tq, tk, tv, o, lse, tdo, win, shift, base, mode, mask,
                                              out_dtype=out, saved=saved)
        again = B.aeris_winattn_rope_bwd(tq, tk, tv, o, lse, tdo, win, shift, base, mode, mask,
                                         out_dtype=out)
        torch.cuda.synchronize()
        for a, b in zip((dq, dk, dv), again):
            assert torch.equal(a, b)
        check("dq", dq, dq_ref, bf)
        check("dk", dk, dk_ref, bf)
        check("dv", dv, dv_ref, bf)


@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("shape,win,shift,mask", [
    ((1, 64, 128, 4, 32), (8, 8), (4, 4), B.AERIS_MASK_SWIN),
    ((1, 36, 72, 2, 64), (12, 12), (6, 6), B.AERIS_MASK_LAT),
    ((1, 40, 60, 2, 128), (20, 20), (10, 10), B.AERIS_MASK_NONE),
    ((1, 40, 60, 2, 128), (20, 20), (0, 0), B.AERIS_MASK_NONE),
])
def test_rope_attention_fwd_bwd(mode, shape, win, shift, mask):
    run_rope_case(shape, win, shift, mask, mode)


def test_rope_attention_ragged_30x30_windows():
    # T = 900: several resident tiles with a ragged tail; window-local positions
    run_rope_case((1, 30, 60, 1, 128), (30, 30), (15, 15), B.AERIS_MASK_SWIN,
                  B.AERIS_ROPE_POS_WINDOW, outs=(B.AERIS_DT_BF16,))


def test_rope_attention_matches_two_step_composition():
    """Rotating q and k with aeris_rope2d_apply and calling the plain forward gives the same
    result as the fused call, bit for bit: both multiply the same bf16 operands."""
    shape, win, shift, mask = (1, 36, 72, 2, 64), (12, 12), (6, 6), B.AERIS_MASK_SWIN
    bits = synth.make_inputs("normal", 4200, shape, 3)
    tq, tk, tv = [to_dev(b) for b in bits]
    for mode in MODES:
        o1, l1 = B.aeris_winattn_rope_fwd(tq, tk, tv, win, shift, 100.0, mode, mask)
        qr = B.aeris_rope2d_apply(tq, win, shift, 100.0, mode)
        kr = B.aeris_rope2d_apply(tk, win, shift, 100.0, mode)
        o2, l2 = B.aeris_winattn_fwd(qr, kr, tv, win, shift, mask)
        torch.cuda.synchronize()
        assert torch.equal(o1, o2) and torch.equal(l1, l2)


def test_rope_band_share_full_size_sampled():
    """Config-4 launch shape (48 windows of 60x60, 24 heads x 128) with grid positions, whose
    longitude positions reach 1439: sampled (window, head) pairs against the oracle."""
    shape, win, shift, mask = (1, 120, 1440, 24, 128), (60, 60), (30, 30), B.AERIS_MASK_SWIN
    Bn, H, W, nh, d = shape
    base, mode = 100.0, B.AERIS_ROPE_POS_GRID
    tq, tk, tv, tdo = synth.make_inputs_device("blend", 4301, shape, 4)
    o, lse, saved = B.aeris_winattn_rope_fwd(tq, tk, tv, win, shift, base, mode, mask,
                                             out_dtype=B.AERIS_DT_F32, return_saved=True)
    dq, dk, dv = B.aeris_winattn_rope_bwd(tq, tk, tv, o, lse, tdo, win, shift, base, mode, mask,
                                          out_dtype=B.AERIS_DT_F32, saved=saved)
    torch.cuda.synchronize()
    phi = ro.angles(H, W, d, win, shift, base, ro.POS_GRID)

    def turn(x_hwd, inverse=False):
        return ro.rotate(x_hwd[None, :, :, None, :], phi, inverse=inverse)[0, :, :, 0, :]

    for (wy, wx, h) in [(0, 4, 0), (1, 23, 17)]:           # interior window, corner window
        sl = lambda t: to_f64(t[0, :, :, h, :])
        qr, kr = turn(sl(tq)), turn(sl(tk))
        res = orc.winattn_pair(qr, kr, sl(tv), sl(tdo), H, W, win, shift, mask, None, wy, wx)
        y, x = res["y"], res["x"]
        check("o", sl(o)[y, x], res["o"], False)
        check_lse(to_f64(lse[0, h])[y, x], res["lse"])
        check("dv", sl(dv)[y, x], res["dv"], False)
        for name, got, ref_rot in (("dq", dq, res["dq"]), ("dk", dk, res["dk"])):
            full = np.zeros((H, W, d))
            full[y, x] = ref_rot
            check(name, sl(got)[y, x], turn(full, inverse=True)[y, x], False)


def test_rope_seeded_sweep_of_small_shapes():
    """Twelve seeded random small problems with the rotary embedding: any window shape and shift,
    both position modes, bases from 10 to 10000, every mask policy and head_dim."""
    rng = np.random.default_rng(20240608)
    for case in range(12):
        wh, ww = int(rng.integers(2, 21)), int(rng.integers(2, 21))
        nwy, nwx = int(rng.integers(1, 4)), int(rng.integers(1, 4))
        sh, sw = int(rng.integers(0, wh)), int(rng.integers(0, ww))
        d = int(rng.choice([32, 64, 128]))
        shape = (int(rng.integers(1, 3)), wh * nwy, ww * nwx, int(rng.integers(1, 3)), d)
        mask = int(rng.choice([B.AERIS_MASK_NONE, B.AERIS_MASK_LAT, B.AERIS_MASK_SWIN]))
        mode = int(rng.choice(MODES))
        base = float(rng.choice([10.0, 100.0, 10000.0]))
        out = B.AERIS_DT_F32 if rng.random() < 0.5 else B.AERIS_DT_BF16
        print("case", case, shape, (wh, ww), (sh, sw), mask, mode, base, out, flush=True)
        run_rope_case(shape, (wh, ww), (sh, sw), mask, mode, base=base, seed=7100 + case,
                      outs=(out,))


def test_rope_attention_on_packed_qkv_is_bitwise_the_contiguous_result():
    """Queries, keys and values interleaved per token, as a fused QKV projection writes them
    ([B,H,W,3,heads,d]), gradients written into the same packing: the rotary entry points must
    give exactly what they give on separate contiguous tensors (which the cases above hold to the
    oracle)."""
    import ctypes
    shape, win, shift, mask = (2, 24, 36, 3, 64), (12, 12), (6, 6), B.AERIS_MASK_SWIN
    Bn, H, W, nh, d = shape
    bits = synth.make_inputs("normal", 4300, shape, 4)
    tq, tk, tv, tdo = [to_dev(b) for b in bits]
    mode = B.AERIS_ROPE_POS_WINDOW
    o_ref, lse_ref = B.aeris_winattn_rope_fwd(tq, tk, tv, win, shift, 100.0, mode, mask)
    dq_ref, dk_ref, dv_ref = B.aeris_winattn_rope_bwd(tq, tk, tv, o_ref, lse_ref, tdo, win, shift,
                                                      100.0, mode, mask)
    packed = torch.stack([tq, tk, tv], dim=3).contiguous()
    dpacked = torch.full_like(packed, float("nan"))
    o = torch.empty_like(tq)
    lse = torch.empty_like(lse_ref)
    p = B.make_params(shape, win, shift, mask, qkv_strides=(3 * nh * d, d))
    r = B.aeris_rope_params(100.0, mode)
    lib = B.load()
    ptr = lambda t, i: t.data_ptr() + i * nh * d * 2
    stream = torch.cuda.current_stream().cuda_stream
    fws = torch.empty(B.aeris_winattn_rope_fwd_workspace_bytes(p), dtype=torch.uint8, device="cuda")
    ws = torch.empty(B.aeris_winattn_rope_bwd_workspace_bytes(p), dtype=torch.uint8, device="cuda")
    rc = lib.aeris_winattn_rope_fwd(ctypes.byref(p), ctypes.byref(r), ptr(packed, 0), ptr(packed, 1),
                                    ptr(packed, 2), o.data_ptr(), lse.data_ptr(), fws.data_ptr(),
                                    fws.numel(), stream)
    assert rc == 0
    for saved in (None, fws.data_ptr()):      # rotating again, then from the forward's workspace
        dpacked.fill_(float("nan"))
        rc = lib.aeris_winattn_rope_bwd(ctypes.byref(p), ctypes.byref(r), ptr(packed, 0),
                                        ptr(packed, 1), ptr(packed, 2), o.data_ptr(), lse.data_ptr(),
                                        tdo.data_ptr(), ptr(dpacked, 0), ptr(dpacked, 1),
                                        ptr(dpacked, 2), saved, ws.data_ptr(), ws.numel(), stream)
        assert rc == 0
        torch.cuda.synchronize()
        assert torch.equal(o, o_ref) and torch.equal(lse, lse_ref)
        for i, ref in enumerate((dq_ref, dk_ref, dv_ref)):
            assert torch.equal(dpacked[:, :, :, i].contiguous().view(torch.int16),
                               ref.view(torch.int16))
