"""Pins for the fp64 oracle: everything here runs on the CPU.

The paper prints no numbers for window attention, so the oracle is tied to
what the mathematics fixes: scalar brute force built a different way (roll,
reshape, label image), textbook global attention through torch autograd,
equivariances, closed forms, conservation identities, finite differences and
closed-form counts of unmasked pairs.
"""
import itertools
import math
import os

import numpy as np
import pytest
import torch

from oracle import winattn_oracle as orc

POLICIES = [orc.MASK_NONE, orc.MASK_LAT, orc.MASK_SWIN]


def rand_qkv(seed, shape, n=3):
    rng = np.random.default_rng(seed)
    return [rng.standard_normal(shape) for _ in range(n)]


# ----------------------------------------------------------------------------
# 1. brute force, constructed differently from the oracle: the field is rolled
#    explicitly, cut into windows by slicing, and the mask comes from a label
#    image painted with slices in the shifted frame.
# ----------------------------------------------------------------------------
def label_image(H, W, win, shift, mask):
    lab = np.zeros((H, W), dtype=np.int64)
    if mask == orc.MASK_NONE:
        return lab
    hs = [(0, H - win[0]), (H - win[0], H - shift[0]), (H - shift[0], H)]
    wsl = [(0, W - win[1]), (W - win[1], W - shift[1]), (W - shift[1], W)]
    if mask == orc.MASK_LAT:
        wsl = [(0, W)]
    n = 0
    for (h0, h1) in hs:
        for (w0, w1) in wsl:
            lab[h0:h1, w0:w1] = n
            n += 1
    return lab


def brute_fwd(q, k, v, win, shift, mask, scale):
    B, H, W, nh, d = q.shape
    qr, kr, vr = [np.roll(a, (-shift[0], -shift[1]), axis=(1, 2)) for a in (q, k, v)]
    lab = label_image(H, W, win, shift, mask)
    o_r = np.zeros_like(q)
    lse_r = np.zeros((B, nh, H, W))
    for b, h in itertools.product(range(B), range(nh)):
        for y0 in range(0, H, win[0]):
            for x0 in range(0, W, win[1]):
                cells = [(y0 + r, x0 + c) for r in range(win[0]) for c in range(win[1])]
                for (yi, xi) in cells:
                    logits = []
                    for (yj, xj) in cells:
                        if lab[yi, xi] != lab[yj, xj]:
                            continue
                        s = 0.0
                        for e in range(d):
                            s += qr[b, yi, xi, h, e] * kr[b, yj, xj, h, e]
                        logits.append((scale * s, yj, xj))
                    z = sum(math.exp(s) for (s, _, _) in logits)
                    lse_r[b, h, yi, xi] = math.log(z)
                    for e in range(d):
                        o_r[b, yi, xi, h, e] = sum(math.exp(s) / z * vr[b, yj, xj, h, e]
                                                   for (s, yj, xj) in logits)
    o = np.roll(o_r, (shift[0], shift[1]), axis=(1, 2))
    lse = np.roll(lse_r, (shift[0], shift[1]), axis=(2, 3))
    return o, lse


@pytest.mark.parametrize("mask", POLICIES)
@pytest.mark.parametrize("shift", [(0, 0), (1, 1), (2, 2), (3, 3), (1, 3)])
def test_brute_force_fwd(mask, shift):
    q, k, v = rand_qkv(11 + shift[0], (1, 8, 12, 2, 3))
    scale = 0.7
    o, lse = orc.winattn_fwd(q, k, v, (4, 4), shift, mask, scale)
    ob, lb = brute_fwd(q, k, v, (4, 4), shift, mask, scale)
    np.testing.assert_allclose(o, ob, rtol=0, atol=1e-12)
    np.testing.assert_allclose(lse, lb, rtol=0, atol=1e-12)


def torch_windowed(q, k, v, win, shift, mask, scale):
    """Windowed attention via roll + reshape + masked_fill in torch (double)."""
    B, H, W, nh, d = q.shape
    lab = torch.from_numpy(label_image(H, W, win, shift, mask))

    def part(t):  # [B,H,W,nh,d] -> [B, nWy, nWx, nh, T, d]
        t = torch.roll(t, (-shift[0], -shift[1]), dims=(1, 2))
        t = t.reshape(B, H // win[0], win[0], W // win[1], win[1], nh, d)
        return t.permute(0, 1, 3, 5, 2, 4, 6).reshape(B, H // win[0], W // win[1], nh, -1, d)

    labw = lab.reshape(H // win[0], win[0], W // win[1], win[1]).permute(0, 2, 1, 3)
    labw = labw.reshape(H // win[0], W // win[1], -1)
    allowed = labw[..., :, None] == labw[..., None, :]           # [nWy,nWx,T,T]
    S = scale * part(q) @ part(k).transpose(-1, -2)
    S = S.masked_fill(~allowed[None, :, :, None], float("-inf"))
    O = torch.softmax(S, dim=-1) @ part(v)
    O = O.reshape(B, H // win[0], W // win[1], nh, win[0], win[1], d)
    O = O.permute(0, 1, 4, 2, 5, 3, 6).reshape(B, H, W, nh, d)
    return torch.roll(O, (shift[0], shift[1]), dims=(1, 2))


@pytest.mark.parametrize("mask", POLICIES)
@pytest.mark.parametrize("shift", [(0, 0), (2, 3), (3, 1)])
def test_autograd_windowed_bwd(mask, shift):
    """dQ, dK, dV of the oracle against torch autograd on an independently
    built windowed attention (non-square window, every mask policy)."""
    shape = (2, 8, 15, 2, 4)
    win = (4, 5)
    q, k, v, do = rand_qkv(5, shape, 4)
    tq, tk, tv = [torch.tensor(a, requires_grad=True) for a in (q, k, v)]
    out = torch_windowed(tq, tk, tv, win, shift, mask, 0.5)
    out.backward(torch.tensor(do))
    o, _ = orc.winattn_fwd(q, k, v, win, shift, mask, 0.5)
    dq, dk, dv, delta = orc.winattn_bwd(q, k, v, do, win, shift, mask, 0.5)
    np.testing.assert_allclose(o, out.detach().numpy(), atol=1e-12)
    np.testing.assert_allclose(dq, tq.grad.numpy(), atol=1e-12)
    np.testing.assert_allclose(dk, tk.grad.numpy(), atol=1e-12)
    np.testing.assert_allclose(dv, tv.grad.numpy(), atol=1e-12)
    np.testing.assert_allclose(delta, np.einsum("bhwnd,bhwnd->bnhw", do, o), atol=1e-12)


# ----------------------------------------------------------------------------
# 2. one window covering the grid = textbook global attention
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("shift", [(0, 0), (2, 5)])
def test_global_attention_special_case(shift):
    shape = (2, 6, 10, 3, 8)
    q, k, v, do = rand_qkv(3, shape, 4)
    B, H, W, nh, d = shape
    tq, tk, tv = [torch.tensor(a.reshape(B, H * W, nh, d).transpose(0, 2, 1, 3).copy(),
                               requires_grad=True) for a in (q, k, v)]
    out = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv)   # 1/sqrt(d)
    tdo = torch.tensor(do.reshape(B, H * W, nh, d).transpose(0, 2, 1, 3).copy())
    out.backward(tdo)
    back = lambda t: t.detach().numpy().transpose(0, 2, 1, 3).reshape(shape)
    o, lse = orc.winattn_fwd(q, k, v, (H, W), shift, orc.MASK_NONE)
    dq, dk, dv, _ = orc.winattn_bwd(q, k, v, do, (H, W), shift, orc.MASK_NONE)
    np.testing.assert_allclose(o, back(out), atol=1e-12)
    np.testing.assert_allclose(dq, back(tq.grad), atol=1e-12)
    np.testing.assert_allclose(dk, back(tk.grad), atol=1e-12)
    np.testing.assert_allclose(dv, back(tv.grad), atol=1e-12)
    S = torch.einsum("bnid,bnjd->bnij", tq, tk).detach() / math.sqrt(d)
    ref_lse = torch.logsumexp(S, dim=-1).numpy().reshape(B, nh, H, W)
    np.testing.assert_allclose(lse, ref_lse, atol=1e-12)


# ----------------------------------------------------------------------------
# 3. roll equivariance
# ----------------------------------------------------------------------------
def test_shift_is_roll_conjugation():
    """NONE: F_s(x) = roll(F_0(roll(x, -s)), +s)."""
    q, k, v = rand_qkv(21, (1, 12, 18, 2, 4))
    win, s = (4, 6), (1, 4)
    o_s, lse_s = orc.winattn_fwd(q, k, v, win, s, orc.MASK_NONE)
    r = lambda a: np.roll(a, (-s[0], -s[1]), axis=(1, 2))
    o0, lse0 = orc.winattn_fwd(r(q), r(k), r(v), win, (0, 0), orc.MASK_NONE)
    np.testing.assert_allclose(o_s, np.roll(o0, s, axis=(1, 2)), atol=1e-13)
    np.testing.assert_allclose(lse_s, np.roll(lse0, s, axis=(2, 3)), atol=1e-13)


@pytest.mark.parametrize("mask,axis,commutes", [
    (orc.MASK_NONE, 1, True), (orc.MASK_NONE, 2, True),
    (orc.MASK_LAT, 2, True), (orc.MASK_LAT, 1, False),
    (orc.MASK_SWIN, 1, False), (orc.MASK_SWIN, 2, False)])
def test_window_multiple_roll(mask, axis, commutes):
    """Rolling the inputs by one window commutes with the operator exactly
    where no seam is pinned to the grid."""
    q, k, v = rand_qkv(22, (1, 12, 12, 1, 4))
    win, s = (4, 4), (2, 2)
    o, _ = orc.winattn_fwd(q, k, v, win, s, mask)
    r = lambda a: np.roll(a, 4, axis=axis)
    o_r, _ = orc.winattn_fwd(r(q), r(k), r(v), win, s, mask)
    same = np.allclose(o_r, r(o), atol=1e-12)
    assert same == commutes


def test_half_window_shift_direction_irrelevant():
    """With s = ws/2 the set of windows is the same for +s and -s (= ws - s)."""
    q, k, v = rand_qkv(23, (1, 8, 8, 1, 4))
    a, _ = orc.winattn_fwd(q, k, v, (4, 4), (2, 2), orc.MASK_NONE)
    b, _ = orc.winattn_fwd(q, k, v, (4, 4), (4 - 2, 4 - 2), orc.MASK_NONE)
    np.testing.assert_array_equal(a, b)


# ----------------------------------------------------------------------------
# 4. permutation of tokens inside a window
# ----------------------------------------------------------------------------
def test_within_window_permutation():
    H, W, win, s = 8, 8, (4, 4), (0, 0)
    q, k, v, do = rand_qkv(31, (1, H, W, 2, 4), 4)
    rng = np.random.default_rng(0)
    src_y = np.empty((H, W), dtype=np.int64)
    src_x = np.empty((H, W), dtype=np.int64)
    for wy in range(2):
        for wx in range(2):
            y, x, _, _ = orc.window_tokens(H, W, win, s, wy, wx)
            p = rng.permutation(16)
            src_y[y, x] = y[p]
            src_x[y, x] = x[p]
    perm = lambda a: a[:, src_y, src_x]
    permL = lambda a: a[:, :, src_y, src_x]
    o, lse = orc.winattn_fwd(q, k, v, win, s)
    dq, dk, dv, _ = orc.winattn_bwd(q, k, v, do, win, s)
    o2, lse2 = orc.winattn_fwd(perm(q), perm(k), perm(v), win, s)
    dq2, dk2, dv2, _ = orc.winattn_bwd(perm(q), perm(k), perm(v), perm(do), win, s)
    np.testing.assert_allclose(o2, perm(o), atol=1e-13)
    np.testing.assert_allclose(lse2, permL(lse), atol=1e-13)
    np.testing.assert_allclose(dq2, perm(dq), atol=1e-13)
    np.testing.assert_allclose(dk2, perm(dk), atol=1e-13)
    np.testing.assert_allclose(dv2, perm(dv), atol=1e-13)


# ----------------------------------------------------------------------------
# 5. closed forms
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("mask", POLICIES)
def test_zero_query_gives_region_mean(mask):
    H, W, win, s = 8, 12, (4, 4), (1, 2)
    _, k, v = rand_qkv(41, (1, H, W, 1, 3))
    q = np.zeros_like(k)
    o, lse = orc.winattn_fwd(q, k, v, win, s, mask)
    lab = label_image(H, W, win, s, mask)
    vr = np.roll(v, (-s[0], -s[1]), axis=(1, 2))
    exp_o = np.zeros_like(v)
    exp_l = np.zeros((1, 1, H, W))
    for y0 in range(0, H, 4):
        for x0 in range(0, W, 4):
            for r in range(4):
                for c in range(4):
                    same = lab[y0:y0 + 4, x0:x0 + 4] == lab[y0 + r, x0 + c]
                    exp_o[0, y0 + r, x0 + c, 0] = vr[0, y0:y0 + 4, x0:x0 + 4, 0][same].mean(axis=0)
                    exp_l[0, 0, y0 + r, x0 + c] = math.log(same.sum())
    np.testing.assert_allclose(o, np.roll(exp_o, s, axis=(1, 2)), atol=1e-13)
    np.testing.assert_allclose(lse, np.roll(exp_l, s, axis=(2, 3)), atol=1e-13)


def test_constant_v_and_zero_do():
    q, k, v, do = rand_qkv(42, (1, 8, 8, 2, 4), 4)
    vc = np.broadcast_to(np.array([1.5, -2.0, 0.25, 3.0]), v.shape).copy()
    o, _ = orc.winattn_fwd(q, k, vc, (4, 4), (2, 2), orc.MASK_SWIN)
    np.testing.assert_allclose(o, vc, atol=1e-13)
    dq, dk, dv, delta = orc.winattn_bwd(q, k, v, np.zeros_like(do), (4, 4), (2, 2), orc.MASK_SWIN)
    assert not dq.any() and not dk.any() and not dv.any() and not delta.any()
    # constant V: P dV-contraction has dP_ij independent of j, so dS = 0
    dq, dk, _, _ = orc.winattn_bwd(q, k, vc, do, (4, 4), (2, 2), orc.MASK_SWIN)
    np.testing.assert_allclose(dq, 0, atol=1e-12)
    np.testing.assert_allclose(dk, 0, atol=1e-12)


def test_huge_scale_selects_argmax_key():
    q, k, v = rand_qkv(43, (1, 4, 8, 1, 4))
    o, _ = orc.winattn_fwd(q, k, v, (4, 4), (0, 0), orc.MASK_NONE, scale=1e4)
    for wx in range(2):
        y, x, _, _ = orc.window_tokens(4, 8, (4, 4), (0, 0), 0, wx)
        S = q[0, y, x, 0] @ k[0, y, x, 0].T
        j = S.argmax(axis=1)
        np.testing.assert_allclose(o[0, y, x, 0], v[0, y[j], x[j], 0], atol=1e-9)


def test_no_mask_when_unshifted():
    q, k, v = rand_qkv(44, (1, 8, 8, 1, 4))
    ref, _ = orc.winattn_fwd(q, k, v, (4, 4), (0, 0), orc.MASK_NONE)
    for mask in (orc.MASK_LAT, orc.MASK_SWIN):
        o, _ = orc.winattn_fwd(q, k, v, (4, 4), (0, 0), mask)
        np.testing.assert_array_equal(o, ref)


# ----------------------------------------------------------------------------
# 6. conservation identities (also used at full size on the GPU outputs)
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("mask", POLICIES)
def test_conservation_identities(mask):
    H, W, win, s = 8, 12, (4, 6), (2, 3)
    q, k, v, do = rand_qkv(51, (1, H, W, 2, 5), 4)
    o, _ = orc.winattn_fwd(q, k, v, win, s, mask)
    dq, dk, dv, _ = orc.winattn_bwd(q, k, v, do, win, s, mask)
    for wy in range(H // win[0]):
        for wx in range(W // win[1]):
            y, x, yh, xh = orc.window_tokens(H, W, win, s, wy, wx)
            reg = orc.token_regions(H, W, win, s, mask, yh, xh)
            for g in np.unique(reg):
                m = reg == g
                yy, xx = y[m], x[m]
                # columns of P over a region sum dO into dV
                np.testing.assert_allclose(dv[0, yy, xx].sum(axis=0), do[0, yy, xx].sum(axis=0),
                                           atol=1e-12)
                vv = v[0, yy, xx]
                assert (o[0, yy, xx] <= vv.max(axis=0) + 1e-12).all()
                assert (o[0, yy, xx] >= vv.min(axis=0) - 1e-12).all()
            # sum_i <Q_i, dQ_i> = sum_j <K_j, dK_j> = scale * sum_ij dS_ij S_ij / scale
            a = np.einsum("thd,thd->h", q[0, y, x], dq[0, y, x])
            b = np.einsum("thd,thd->h", k[0, y, x], dk[0, y, x])
            np.testing.assert_allclose(a, b, atol=1e-12)


# ----------------------------------------------------------------------------
# 7. finite differences
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("mask", POLICIES)
def test_finite_differences(mask):
    H, W, win, s = 6, 6, (3, 3), (1, 1)
    q, k, v, do = rand_qkv(61, (1, H, W, 2, 4), 4)
    dq, dk, dv, _ = orc.winattn_bwd(q, k, v, do, win, s, mask, 0.6)

    def loss(q_, k_, v_):
        o, _ = orc.winattn_fwd(q_, k_, v_, win, s, mask, 0.6)
        return float((o * do).sum())

    rng = np.random.default_rng(0)
    eps = 1e-6
    for which, grad in ((0, dq), (1, dk), (2, dv)):
        for _ in range(12):
            idx = tuple(rng.integers(0, n) for n in q.shape)
            args = [q.copy(), k.copy(), v.copy()]
            args[which][idx] += eps
            up = loss(*args)
            args[which][idx] -= 2 * eps
            dn = loss(*args)
            fd = (up - dn) / (2 * eps)
            assert abs(fd - grad[idx]) <= 1e-7 * max(1.0, abs(grad[idx])), (which, idx)


# ----------------------------------------------------------------------------
# 8. number of unmasked pairs: closed form from the region sizes
# ----------------------------------------------------------------------------
def read_golden_counts():
    path = os.path.join(os.path.dirname(__file__), "golden", "unmasked_pairs.txt")
    rows = []
    with open(path) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if line:
                rows.append([float(t) for t in line.split()])
    return rows


def test_unmasked_pair_counts():
    names = {0: orc.MASK_NONE, 1: orc.MASK_LAT, 2: orc.MASK_SWIN}
    for H, W, ws, s, pol, windows_equiv in read_golden_counts():
        H, W, ws, s = int(H), int(W), int(ws), int(s)
        got = orc.unmasked_pairs(H, W, (ws, ws), (s, s), names[int(pol)])
        assert got == round(windows_equiv * ws ** 4), (H, W, ws, s, pol)


def test_unmasked_pair_formula_general_shift():
    """Seam windows split an axis into ws-s and s: ((ws-s)^2 + s^2)/ws^2 survives."""
    H, W, ws = 12, 20, 4
    for s in range(ws):
        f = ((ws - s) ** 2 + s ** 2) / ws ** 2
        nwy, nwx = H // ws, W // ws
        T2 = ws ** 4
        lat = ((nwy - 1) * nwx + nwx * f) * T2
        swin = ((nwy - 1) * (nwx - 1) + (nwy - 1) * f + (nwx - 1) * f + f * f) * T2
        assert orc.unmasked_pairs(H, W, (ws, ws), (s, s), orc.MASK_LAT) == round(lat)
        assert orc.unmasked_pairs(H, W, (ws, ws), (s, s), orc.MASK_SWIN) == round(swin)
        assert orc.unmasked_pairs(H, W, (ws, ws), (s, s), orc.MASK_NONE) == nwy * nwx * T2


# ----------------------------------------------------------------------------
# 9. the sampled-pair entry (what the full-size GPU cases are compared with) is the
#    whole-grid oracle restricted to one (batch, window, head); and an independent
#    brute-force pin that does not go through the whole-grid functions at all
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("mask", POLICIES)
@pytest.mark.parametrize("with_do", [False, True])
def test_sampled_pair_equals_whole_grid_slices(mask, with_do):
    """Non-square grid and window, unequal shifts: a swapped wy/wx, H/W or slice order,
    a wrong default scale or a wrong key in the result would all show."""
    shape, win, shift = (2, 8, 15, 3, 4), (4, 5), (1, 3)
    Bn, H, W, nh, d = shape
    q, k, v, do = rand_qkv(71, shape, 4)
    for scale in (None, 0.37):
        o, lse = orc.winattn_fwd(q, k, v, win, shift, mask, scale)
        dq, dk, dv, delta = orc.winattn_bwd(q, k, v, do, win, shift, mask, scale)
        for b, h in itertools.product(range(Bn), range(nh)):
            for wy, wx in itertools.product(range(H // win[0]), range(W // win[1])):
                res = orc.winattn_pair(q[b, :, :, h], k[b, :, :, h], v[b, :, :, h],
                                       do[b, :, :, h] if with_do else None, H, W, win, shift,
                                       mask, scale, wy, wx)
                y, x = res["y"], res["x"]
                # the window's grid points, built here by hand
                ey = [(wy * win[0] + r + shift[0]) % H for r in range(win[0]) for _ in range(win[1])]
                ex = [(wx * win[1] + c + shift[1]) % W for _ in range(win[0]) for c in range(win[1])]
                assert list(y) == ey and list(x) == ex
                np.testing.assert_allclose(res["o"], o[b, y, x, h], rtol=0, atol=1e-13)
                np.testing.assert_allclose(res["lse"], lse[b, h, y, x], rtol=0, atol=1e-13)
                if with_do:
                    np.testing.assert_allclose(res["dq"], dq[b, y, x, h], rtol=0, atol=1e-13)
                    np.testing.assert_allclose(res["dk"], dk[b, y, x, h], rtol=0, atol=1e-13)
                    np.testing.assert_allclose(res["dv"], dv[b, y, x, h], rtol=0, atol=1e-13)
                    np.testing.assert_allclose(res["delta"], delta[b, h, y, x], rtol=0, atol=1e-13)
                else:
                    assert set(res) == {"y", "x", "o", "lse"}


@pytest.mark.parametrize("wy,wx", [(0, 0), (1, 0), (0, 2), (1, 2)])
def test_sampled_pair_against_brute_force(wy, wx):
    """Interior, lat-seam, lon-seam and corner window of a SWIN-masked shifted grid against the
    scalar-loop brute force (which rolls, slices and paints labels: no shared step)."""
    shape, win, shift = (1, 8, 12, 2, 3), (4, 4), (2, 1)
    q, k, v = rand_qkv(72, shape)
    ob, lb = brute_fwd(q, k, v, win, shift, orc.MASK_SWIN, 0.7)
    res = orc.winattn_pair(q[0, :, :, 1], k[0, :, :, 1], v[0, :, :, 1], None, 8, 12, win, shift,
                           orc.MASK_SWIN, 0.7, wy, wx)
    np.testing.assert_allclose(res["o"], ob[0, res["y"], res["x"], 1], rtol=0, atol=1e-12)
    np.testing.assert_allclose(res["lse"], lb[0, 1, res["y"], res["x"]], rtol=0, atol=1e-12)


def test_bench_flop_count_uses_the_oracle_pair_count():
    """bench.py credits FLOPs per unmasked (query, key) pair through a closed form of its own;
    it must agree with the oracle's enumeration for general, one-axis and zero shifts."""
    import bench
    for (H, W, win) in [(12, 20, (4, 4)), (12, 18, (4, 6)), (8, 8, (8, 8))]:
        for shift in [(0, 0), (1, 0), (0, 3), (2, 2), (3, 1)]:
            if shift[0] >= win[0] or shift[1] >= win[1]:
                continue
            for mask in POLICIES:
                want = orc.unmasked_pairs(H, W, win, shift, mask)
                assert abs(bench.unmasked_pairs(H, W, win, shift, mask) - want) < 1e-6 * want
