"""GPU parity of the window-list launches (a rank's share of the windows under window
parallelism, SWiPe section): the listed windows match the oracle of the whole grid, and
nothing outside them is written."""
import numpy as np
import pytest
import torch

from oracle import rope_oracle as ro
from oracle import winattn_oracle as orc
from paper_2509_13523_amd import binding as B
from paper_2509_13523_amd import synth
from test_gpu_parity import LSE_ABS, check, to_dev, to_f64

pytestmark = pytest.mark.gpu


def window_token_mask(H, W, win, shift, windows):
    """[H, W] bool: grid points that belong to the listed windows."""
    m = np.zeros((H, W), dtype=bool)
    nWx = W // win[1]
    for w in windows:
        y, x, _, _ = orc.window_tokens(H, W, win, shift, w // nWx, w % nWx)
        m[y, x] = True
    return m


@pytest.mark.parametrize("shape,win,shift,mask,picks", [
    # round-robin share: every 3rd window, including seam and corner windows
    ((2, 48, 72, 2, 64), (12, 12), (6, 6), B.AERIS_MASK_SWIN, list(range(1, 24, 3)) + [23]),
    ((1, 40, 60, 2, 128), (20, 20), (10, 10), B.AERIS_MASK_LAT, [5, 0]),
    ((1, 64, 128, 4, 32), (8, 8), (0, 0), B.AERIS_MASK_NONE, [127, 64, 3, 17, 90]),
])
def test_window_subset_fwd_bwd(shape, win, shift, mask, picks):
    Bn, H, W, nh, d = shape
    bits = synth.make_inputs("normal", 6001, shape, 4)
    q64, k64, v64, do64 = [synth.bf16_bits_to_f64(b) for b in bits]
    tq, tk, tv, tdo = [to_dev(b) for b in bits]
    o_ref, lse_ref = orc.winattn_fwd(q64, k64, v64, win, shift, mask)
    dq_ref, dk_ref, dv_ref, _ = orc.winattn_bwd(q64, k64, v64, do64, win, shift, mask)
    inside = window_token_mask(H, W, win, shift, picks)
    assert 0 < inside.sum() < H * W
    # the list also carries an index outside the grid of windows: it must be skipped
    lst = torch.tensor(picks + [(H // win[0]) * (W // win[1]) + 7], dtype=torch.int32, device="cuda")
    o = torch.full(shape, float("nan"), dtype=torch.float32, device="cuda")
    lse = torch.full((Bn, nh, H, W), float("nan"), dtype=torch.float32, device="cuda")
    B.aeris_winattn_fwd_windows(tq, tk, tv, win, shift, lst, o, lse, mask, out_dtype=B.AERIS_DT_F32)
    torch.cuda.synchronize()
    o_h, lse_h = to_f64(o), to_f64(lse)
    check("o", o_h[:, inside], o_ref[:, inside], False)
    assert np.abs(lse_h[:, :, inside] - lse_ref[:, :, inside]).max() <= LSE_ABS
    assert np.isnan(o_h[:, ~inside]).all() and np.isnan(lse_h[:, :, ~inside]).all()
    # backward needs o and lse only inside the listed windows
    grads = [torch.full(shape, float("nan"), dtype=torch.float32, device="cuda") for _ in range(3)]
    B.aeris_winattn_bwd_windows(tq, tk, tv, o, lse, tdo, win, shift, lst, *grads, mask=mask,
                                out_dtype=B.AERIS_DT_F32)
    torch.cuda.synchronize()
    for name, g, ref in zip(("dq", "dk", "dv"), grads, (dq_ref, dk_ref, dv_ref)):
        g_h = to_f64(g)
        check(name, g_h[:, inside], ref[:, inside], False)
        assert np.isnan(g_h[:, ~inside]).all(), name


def test_full_list_equals_plain_call_bitwise():
    shape, win, shift, mask = (1, 36, 72, 2, 64), (12, 12), (6, 6), B.AERIS_MASK_SWIN
    bits = synth.make_inputs("normal", 6002, shape, 4)
    tq, tk, tv, tdo = [to_dev(b) for b in bits]
    o1, l1 = B.aeris_winattn_fwd(tq, tk, tv, win, shift, mask)
    g1 = B.aeris_winattn_bwd(tq, tk, tv, o1, l1, tdo, win, shift, mask)
    perm = torch.randperm(18, generator=torch.Generator().manual_seed(3)).to(torch.int32).cuda()
    o2, l2 = torch.empty_like(o1), torch.empty_like(l1)
    B.aeris_winattn_fwd_windows(tq, tk, tv, win, shift, perm, o2, l2, mask)
    g2 = [torch.empty_like(g) for g in g1]
    B.aeris_winattn_bwd_windows(tq, tk, tv, o2, l2, tdo, win, shift, perm, *g2, mask=mask)
    torch.cuda.synchronize()
    assert torch.equal(o1, o2) and torch.equal(l1, l2)
    for a, b in zip(g1, g2):
        assert torch.equal(a, b)


@pytest.mark.parametrize("mode", [B.AERIS_ROPE_POS_WINDOW, B.AERIS_ROPE_POS_GRID])
def test_rotary_attention_on_a_window_subset(mode):
    """A rank's share with the rotary embedding: inside the listed windows the result matches the
    fp64 rotary oracle of the whole grid (and is bit for bit that of the full-grid rotary calls);
    nothing outside them is written, and q, k outside them are never read (NaN there)."""
    shape, win, shift, mask = (2, 36, 72, 2, 64), (12, 12), (6, 6), B.AERIS_MASK_SWIN
    Bn, H, W, nh, d = shape
    picks = [17, 0, 5, 11, 6]          # corner, seam and interior windows of the 3 x 6 grid
    bits = synth.make_inputs("normal", 6003, shape, 4)
    tq, tk, tv, tdo = [to_dev(b) for b in bits]
    o_ref, lse_ref = B.aeris_winattn_rope_fwd(tq, tk, tv, win, shift, 100.0, mode, mask)
    g_ref = B.aeris_winattn_rope_bwd(tq, tk, tv, o_ref, lse_ref, tdo, win, shift, 100.0, mode, mask)
    inside = torch.from_numpy(window_token_mask(H, W, win, shift, picks)).cuda()
    assert 0 < int(inside.sum()) < H * W
    # poison everything outside the share
    def share(t):
        out = torch.full_like(t, float("nan"))
        out[:, inside] = t[:, inside]
        return out
    sq, sk, sv, sdo = share(tq), share(tk), share(tv), share(tdo)
    lst = torch.tensor(picks, dtype=torch.int32, device="cuda")
    o = torch.full_like(o_ref, float("nan"))
    lse = torch.full_like(lse_ref, float("nan"))
    p = B.make_params(shape, win, shift, mask)
    fws = torch.empty(B.aeris_winattn_rope_fwd_workspace_bytes(p), dtype=torch.uint8, device="cuda")
    fws.fill_(0xFF)                     # bf16 NaN everywhere the forward call does not write
    B.aeris_winattn_rope_fwd_windows(sq, sk, sv, win, shift, 100.0, mode, lst, o, lse, mask,
                                     workspace=fws)
    torch.cuda.synchronize()
    assert torch.equal(o[:, inside], o_ref[:, inside])
    assert torch.equal(lse[:, :, inside], lse_ref[:, :, inside])
    assert torch.isnan(o[:, ~inside]).all() and torch.isnan(lse[:, :, ~inside]).all()
    # against the oracle (not only against the full-grid HIP call)
    q64, k64, v64, do64 = [synth.bf16_bits_to_f64(b) for b in bits]
    pm = ro.POS_GRID if mode == B.AERIS_ROPE_POS_GRID else ro.POS_WINDOW
    o_orc, lse_orc = ro.winattn_rope_fwd(q64, k64, v64, win, shift, mask, 100.0, pm)
    g_orc = ro.winattn_rope_bwd(q64, k64, v64, do64, win, shift, mask, 100.0, pm)
    ins = inside.cpu().numpy()
    check("o", to_f64(o)[:, ins], o_orc[:, ins], True)
    assert np.abs(to_f64(lse)[:, :, ins] - lse_orc[:, :, ins]).max() <= LSE_ABS
    for saved in (None, fws):           # rotating the share again, then from the forward's copies
        grads = [torch.full_like(tq, float("nan")) for _ in range(3)]
        B.aeris_winattn_rope_bwd_windows(sq, sk, sv, o, lse, sdo, win, shift, 100.0, mode, lst,
                                         *grads, mask=mask, saved=saved)
        torch.cuda.synchronize()
        for name, g, ref, want in zip(("dq", "dk", "dv"), grads, g_ref, g_orc):
            assert torch.equal(g[:, inside], ref[:, inside])
            assert torch.isnan(g[:, ~inside]).all()
            check(name, to_f64(g)[:, ins], want[:, ins], True)
