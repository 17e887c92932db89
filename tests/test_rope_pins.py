"""Pins of oracle/rope_oracle.py against things other than itself: hand-computed angles,
the complex-exponential route written with explicit loops, invariants of rotations,
identity cases, and torch autograd through an independent complex-number implementation.
(AERIS paper, Model Architecture section: axial-frequency 2-D rotary embedding of queries
and keys.)"""
import os

import numpy as np
import pytest
import torch

from oracle import rope_oracle as ro
from oracle import winattn_oracle as wa

HERE = os.path.dirname(os.path.abspath(__file__))


def rng_fields(seed, shape, n):
    g = np.random.default_rng(seed)
    return [g.standard_normal(shape) for _ in range(n)]


def test_angles_match_hand_computed_table():
    rows = [l.split() for l in open(os.path.join(HERE, "golden", "rope_angles.txt"))
            if l.strip() and not l.startswith("#")]
    assert len(rows) == 7
    for mode, y, x, *phi in rows:
        pm = ro.POS_GRID if mode == "grid" else ro.POS_WINDOW
        got = ro.angles(8, 8, 8, (4, 4), (2, 2), 100.0, pm)[int(y), int(x)]
        np.testing.assert_allclose(got, [float(p) for p in phi], rtol=0, atol=1e-12)


@pytest.mark.parametrize("pos_mode", [ro.POS_WINDOW, ro.POS_GRID])
def test_rotation_is_complex_multiplication_scalar_loops(pos_mode):
    B, H, W, nh, d = 1, 6, 4, 2, 8
    win, shift, base = (3, 2), (1, 1), 50.0
    (t,) = rng_fields(3, (B, H, W, nh, d), 1)
    phi = ro.angles(H, W, d, win, shift, base, pos_mode)
    got = ro.rotate(t, phi)
    for y in range(H):
        for x in range(W):
            if pos_mode == ro.POS_GRID:
                p_lat, p_lon = y, x
            else:
                p_lat, p_lon = ((y - shift[0]) % H) % win[0], ((x - shift[1]) % W) % win[1]
            for h in range(nh):
                for tt in range(d // 4):
                    theta = base ** (-tt / (d / 4))
                    for axis, pos in ((0, p_lon), (1, p_lat)):
                        j = 2 * tt + axis
                        z = complex(t[0, y, x, h, 2 * j], t[0, y, x, h, 2 * j + 1])
                        z *= np.exp(1j * theta * pos)
                        assert abs(got[0, y, x, h, 2 * j] - z.real) < 1e-12
                        assert abs(got[0, y, x, h, 2 * j + 1] - z.imag) < 1e-12


def test_pair_norms_are_preserved_and_inverse_undoes():
    B, H, W, nh, d = 2, 8, 12, 3, 16
    (t,) = rng_fields(5, (B, H, W, nh, d), 1)
    phi = ro.angles(H, W, d, (4, 6), (2, 3), 100.0, ro.POS_GRID)
    r = ro.rotate(t, phi)
    np.testing.assert_allclose(r[..., 0::2] ** 2 + r[..., 1::2] ** 2,
                               t[..., 0::2] ** 2 + t[..., 1::2] ** 2, rtol=1e-12)
    assert np.abs(r - t).max() > 0.1                       # it does turn something
    np.testing.assert_allclose(ro.rotate(r, phi, inverse=True), t, atol=1e-12)


def test_identity_where_all_positions_are_zero():
    (t,) = rng_fields(6, (1, 4, 4, 1, 8), 1)
    # 1 x 1 windows: every window-local position is (0, 0)
    phi = ro.angles(4, 4, 8, (1, 1), (0, 0), 100.0, ro.POS_WINDOW)
    np.testing.assert_array_equal(ro.rotate(t, phi), t)
    # grid mode: the origin is not turned, other points are
    phi = ro.angles(4, 4, 8, (2, 2), (0, 0), 100.0, ro.POS_GRID)
    r = ro.rotate(t, phi)
    np.testing.assert_array_equal(r[0, 0, 0], t[0, 0, 0])
    assert np.abs(r[0, 1, 1] - t[0, 1, 1]).max() > 1e-3


def test_logits_depend_on_position_differences_only():
    # the same two vectors placed at two point pairs with equal offsets give equal logits
    d, H, W = 16, 16, 16
    g = np.random.default_rng(7)
    qv, kv = g.standard_normal(d), g.standard_normal(d)
    phi = ro.angles(H, W, d, (16, 16), (0, 0), 100.0, ro.POS_GRID)

    def logit(pq, pk):
        t = np.zeros((1, H, W, 1, d))
        t[0, pq[0], pq[1], 0] = qv
        qr = ro.rotate(t, phi)[0, pq[0], pq[1], 0]
        t[:] = 0
        t[0, pk[0], pk[1], 0] = kv
        kr = ro.rotate(t, phi)[0, pk[0], pk[1], 0]
        return qr @ kr

    a = logit((2, 3), (5, 1))
    b = logit((9, 12), (12, 10))
    c = logit((2, 3), (5, 2))
    assert abs(a - b) < 1e-12
    assert abs(a - c) > 1e-3


def test_window_and_grid_positions_agree_inside_unwrapped_windows():
    # without shift, positions inside a window differ from grid positions by a constant per
    # window, so the attention output is the same in both modes
    B, H, W, nh, d = 1, 8, 12, 2, 8
    q, k, v = rng_fields(8, (B, H, W, nh, d), 3)
    o1, l1 = ro.winattn_rope_fwd(q, k, v, (4, 6), (0, 0), wa.MASK_NONE, 100.0, ro.POS_WINDOW)
    o2, l2 = ro.winattn_rope_fwd(q, k, v, (4, 6), (0, 0), wa.MASK_NONE, 100.0, ro.POS_GRID)
    np.testing.assert_allclose(o1, o2, atol=1e-12)
    np.testing.assert_allclose(l1, l2, atol=1e-12)
    # with a shift, windows that wrap around the grid see different position differences
    o3, _ = ro.winattn_rope_fwd(q, k, v, (4, 6), (2, 3), wa.MASK_NONE, 100.0, ro.POS_WINDOW)
    o4, _ = ro.winattn_rope_fwd(q, k, v, (4, 6), (2, 3), wa.MASK_NONE, 100.0, ro.POS_GRID)
    assert np.abs(o3 - o4).max() > 1e-3


def _torch_rope(t, pos_lat, pos_lon, base):
    """Independent route: channel pairs as torch complex numbers times e^{i theta p}."""
    d = t.shape[-1]
    n = d // 4
    theta = base ** (-torch.arange(n, dtype=torch.float64) / n)
    z = torch.view_as_complex(t.reshape(*t.shape[:-1], d // 2, 2).contiguous())
    ang = torch.empty(t.shape[1], t.shape[2], d // 2, dtype=torch.float64)
    ang[:, :, 0::2] = pos_lon[:, :, None] * theta
    ang[:, :, 1::2] = pos_lat[:, :, None] * theta
    z = z * torch.polar(torch.ones_like(ang), ang)[None, :, :, None, :]
    return torch.view_as_real(z).reshape(t.shape)


@pytest.mark.parametrize("pos_mode", [ro.POS_WINDOW, ro.POS_GRID])
def test_forward_and_backward_against_torch_autograd_global_window(pos_mode):
    # one window covering the grid, no shift: plain global attention on rotated q, k
    B, H, W, nh, d = 2, 5, 6, 2, 8
    base = 100.0
    q, k, v, do = rng_fields(9, (B, H, W, nh, d), 4)
    tq, tk, tv = [torch.tensor(a, requires_grad=True) for a in (q, k, v)]
    yy, xx = torch.meshgrid(torch.arange(H, dtype=torch.float64),
                            torch.arange(W, dtype=torch.float64), indexing="ij")
    qr, kr = _torch_rope(tq, yy, xx, base), _torch_rope(tk, yy, xx, base)

    def flat(t):
        return t.reshape(B, H * W, nh, d).permute(0, 2, 1, 3)

    o = torch.nn.functional.scaled_dot_product_attention(flat(qr), flat(kr), flat(tv))
    o = o.permute(0, 2, 1, 3).reshape(B, H, W, nh, d)
    o.backward(torch.tensor(do))
    o_ref, _ = ro.winattn_rope_fwd(q, k, v, (H, W), (0, 0), wa.MASK_NONE, base, pos_mode)
    dq, dk, dv = ro.winattn_rope_bwd(q, k, v, do, (H, W), (0, 0), wa.MASK_NONE, base, pos_mode)
    np.testing.assert_allclose(o_ref, o.detach().numpy(), atol=1e-10)
    np.testing.assert_allclose(dq, tq.grad.numpy(), atol=1e-10)
    np.testing.assert_allclose(dk, tk.grad.numpy(), atol=1e-10)
    np.testing.assert_allclose(dv, tv.grad.numpy(), atol=1e-10)


def test_backward_finite_differences_shifted_masked_windows():
    B, H, W, nh, d = 1, 4, 6, 1, 4
    win, shift, mask, base = (2, 3), (1, 1), wa.MASK_SWIN, 20.0
    q, k, v, do = rng_fields(10, (B, H, W, nh, d), 4)
    dq, dk, dv = ro.winattn_rope_bwd(q, k, v, do, win, shift, mask, base, ro.POS_WINDOW)

    def loss(qq, kk):
        o, _ = ro.winattn_rope_fwd(qq, kk, v, win, shift, mask, base, ro.POS_WINDOW)
        return (o * do).sum()

    g = np.random.default_rng(11)
    eps = 1e-6
    for _ in range(12):
        idx = tuple(g.integers(0, s) for s in q.shape)
        e = np.zeros_like(q)
        e[idx] = eps
        assert abs((loss(q + e, k) - loss(q - e, k)) / (2 * eps) - dq[idx]) < 1e-6
        assert abs((loss(q, k + e) - loss(q, k - e)) / (2 * eps) - dk[idx]) < 1e-6
