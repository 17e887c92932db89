"""Pins of oracle/block_oracle.py against things other than itself: rows worked by hand, the
invariants RMSNorm and SiLU have, limits, torch's own rms_norm / silu routines, central finite
differences in fp64 and torch autograd through separately written forward expressions.
(AERIS paper, Model Architecture section: pre-RMSNorm, adaptive layer norm values alpha, beta,
gamma, SwiGLU; formulas from the works that section cites.)"""
import math

import numpy as np
import pytest
import torch

from oracle import block_oracle as bo


def _rand(rng, *shape):
    return rng.standard_normal(shape)


# ---------------------------------------------------------------- forward: RMSNorm + modulation
def test_rmsnorm_row_worked_by_hand():
    # x = (3, 4): mean square 12.5, r = 1/sqrt(12.5); n = (3, 4) r
    x = np.array([[3.0, 4.0]])
    w = np.array([2.0, 0.5])
    gamma = np.array([[0.5, -1.0]])
    beta = np.array([[1.0, 2.0]])
    h, r = bo.rmsnorm_adaln_fwd(x, w, gamma, beta, 0.0, 1)
    assert r[0] == pytest.approx(0.28284271247461900976, abs=1e-15)
    # channel 0: 3 r * 2 * 1.5 + 1; channel 1: scale (1 + gamma) = 0 leaves the shift
    assert h[0, 0] == pytest.approx(9.0 / math.sqrt(12.5) + 1.0, abs=1e-14)
    assert h[0, 1] == pytest.approx(2.0, abs=1e-14)


def test_rmsnorm_unit_rms_and_scale_invariance():
    rng = np.random.default_rng(1)
    x = _rand(rng, 6, 40) * 3.0
    w = np.ones(40)
    z = np.zeros((2, 40))
    h, _ = bo.rmsnorm_adaln_fwd(x, w, z, z, 0.0, 3)
    np.testing.assert_allclose(np.mean(h * h, axis=1), 1.0, rtol=1e-13)
    h2, r2 = bo.rmsnorm_adaln_fwd(7.5 * x, w, z, z, 0.0, 3)
    np.testing.assert_allclose(h2, h, rtol=1e-13)
    # a negative factor flips the sign of every normalised value
    h3, _ = bo.rmsnorm_adaln_fwd(-x, w, z, z, 0.0, 3)
    np.testing.assert_allclose(h3, -h, rtol=1e-13)


def test_rmsnorm_zero_row_gives_the_shift_and_eps_bounds_r():
    x = np.zeros((2, 8))
    rng = np.random.default_rng(2)
    w, gamma, beta = _rand(rng, 8), _rand(rng, 2, 8), _rand(rng, 2, 8)
    h, r = bo.rmsnorm_adaln_fwd(x, w, gamma, beta, 1e-6, 1)
    np.testing.assert_array_equal(h, beta)
    np.testing.assert_allclose(r, 1e3, rtol=1e-12)


def test_rmsnorm_rows_take_their_own_samples_vectors():
    rng = np.random.default_rng(3)
    C, rows, B = 5, 4, 3
    x = _rand(rng, B * rows, C)
    w, gamma, beta = _rand(rng, C), _rand(rng, B, C), _rand(rng, B, C)
    h, r = bo.rmsnorm_adaln_fwd(x, w, gamma, beta, 1e-5, rows)
    for i in range(B * rows):
        smp = i // rows
        ms = sum(x[i, c] ** 2 for c in range(C)) / C
        ri = 1.0 / math.sqrt(ms + 1e-5)
        assert r[i] == pytest.approx(ri, rel=1e-13)
        for c in range(C):
            want = x[i, c] * ri * w[c] * (1.0 + gamma[smp, c]) + beta[smp, c]
            assert h[i, c] == pytest.approx(want, rel=1e-12, abs=1e-14)


def test_rmsnorm_matches_torch_rms_norm_when_modulation_is_off():
    rng = np.random.default_rng(4)
    x, w = _rand(rng, 10, 32), _rand(rng, 32)
    z = np.zeros((5, 32))
    h, _ = bo.rmsnorm_adaln_fwd(x, w, z, z, 1e-6, 2)
    ref = torch.nn.functional.rms_norm(torch.from_numpy(x), (32,), torch.from_numpy(w), 1e-6)
    np.testing.assert_allclose(h, ref.numpy(), rtol=1e-12, atol=1e-14)


# ---------------------------------------------------------------- backward: RMSNorm + modulation
def _loss_fwd(x, w, gamma, beta, eps, rows, g):
    h, _ = bo.rmsnorm_adaln_fwd(x, w, gamma, beta, eps, rows)
    return float(np.sum(h * g))


def _central(f, arr, idx, step=1e-6):
    old = arr[idx]
    arr[idx] = old + step
    up = f()
    arr[idx] = old - step
    dn = f()
    arr[idx] = old
    return (up - dn) / (2 * step)


def test_rmsnorm_backward_against_finite_differences():
    rng = np.random.default_rng(5)
    C, rows, B, eps = 6, 3, 2, 1e-3
    x = _rand(rng, B * rows, C)
    w, gamma, beta = _rand(rng, C), _rand(rng, B, C), _rand(rng, B, C)
    g = _rand(rng, B * rows, C)
    dx, dw, dgamma, dbeta = bo.rmsnorm_adaln_bwd(x, w, gamma, beta, eps, rows, g)
    f = lambda: _loss_fwd(x, w, gamma, beta, eps, rows, g)
    for i in range(B * rows):
        for c in range(C):
            assert dx[i, c] == pytest.approx(_central(f, x, (i, c)), rel=1e-6, abs=1e-8)
    for c in range(C):
        assert dw[c] == pytest.approx(_central(f, w, (c,)), rel=1e-6, abs=1e-8)
    for smp in range(B):
        for c in range(C):
            assert dgamma[smp, c] == pytest.approx(_central(f, gamma, (smp, c)), rel=1e-6, abs=1e-8)
            assert dbeta[smp, c] == pytest.approx(_central(f, beta, (smp, c)), rel=1e-6, abs=1e-8)


def test_rmsnorm_backward_against_torch_autograd():
    rng = np.random.default_rng(6)
    C, rows, B, eps = 48, 5, 3, 1e-6
    x = _rand(rng, B * rows, C)
    w, gamma, beta = _rand(rng, C), 0.3 * _rand(rng, B, C), _rand(rng, B, C)
    g = _rand(rng, B * rows, C)
    tx, tw, tg, tb = [torch.tensor(a, requires_grad=True) for a in (x, w, gamma, beta)]
    y = torch.nn.functional.rms_norm(tx, (C,), tw, eps)
    h = torch.addcmul(tb.repeat_interleave(rows, dim=0), y, 1.0 + tg.repeat_interleave(rows, dim=0))
    (h * torch.tensor(g)).sum().backward()
    dx, dw, dgamma, dbeta = bo.rmsnorm_adaln_bwd(x, w, gamma, beta, eps, rows, g)
    np.testing.assert_allclose(dx, tx.grad.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(dw, tw.grad.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(dgamma, tg.grad.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(dbeta, tb.grad.numpy(), rtol=1e-10, atol=1e-12)


def test_rmsnorm_input_gradient_is_orthogonal_to_the_row_without_eps():
    # h(c x) = h(x) for every c > 0 when eps = 0, so the directional derivative along x vanishes
    rng = np.random.default_rng(7)
    x, g = _rand(rng, 4, 16), _rand(rng, 4, 16)
    w, gamma, beta = _rand(rng, 16), _rand(rng, 2, 16), _rand(rng, 2, 16)
    dx, _, _, _ = bo.rmsnorm_adaln_bwd(x, w, gamma, beta, 0.0, 2, g)
    np.testing.assert_allclose(np.sum(dx * x, axis=1), 0.0, atol=1e-12)


def test_rmsnorm_shift_gradient_is_the_column_sum_per_sample():
    g = np.arange(24, dtype=np.float64).reshape(6, 4)
    x = np.ones((6, 4))
    z = np.zeros((2, 4))
    _, _, _, dbeta = bo.rmsnorm_adaln_bwd(x, np.ones(4), z, z, 0.0, 3, g)
    np.testing.assert_array_equal(dbeta[0], [0 + 4 + 8, 1 + 5 + 9, 2 + 6 + 10, 3 + 7 + 11])
    np.testing.assert_array_equal(dbeta[1], [12 + 16 + 20, 13 + 17 + 21, 14 + 18 + 22, 15 + 19 + 23])


# ---------------------------------------------------------------- gated residual
def test_gate_residual_by_hand_and_limits():
    x = np.array([[1.0, 2.0], [3.0, 4.0]])
    y = np.array([[10.0, 20.0], [30.0, 40.0]])
    alpha = np.array([[0.5, -1.0], [2.0, 0.0]])
    out = bo.gate_residual_fwd(x, y, alpha, 1)
    np.testing.assert_array_equal(out, [[6.0, -18.0], [63.0, 4.0]])
    np.testing.assert_array_equal(bo.gate_residual_fwd(x, y, np.zeros((1, 2)), 2), x)
    np.testing.assert_array_equal(bo.gate_residual_fwd(x, y, np.ones((1, 2)), 2), x + y)


def test_gate_residual_backward_by_hand():
    y = np.array([[1.0, 2.0], [3.0, 4.0], [5.0, 6.0], [7.0, 8.0]])
    dout = np.array([[1.0, 1.0], [2.0, 0.5], [-1.0, 3.0], [0.0, 2.0]])
    alpha = np.array([[2.0, 3.0], [-1.0, 0.5]])
    dx, dy, dalpha = bo.gate_residual_bwd(y, alpha, dout, 2)
    np.testing.assert_array_equal(dx, dout)
    np.testing.assert_array_equal(dy, [[2.0, 3.0], [4.0, 1.5], [1.0, 1.5], [0.0, 1.0]])
    np.testing.assert_array_equal(dalpha, [[1 * 1 + 2 * 3, 1 * 2 + 0.5 * 4], [-1 * 5 + 0 * 7, 3 * 6 + 2 * 8]])


def test_gate_residual_backward_against_torch_autograd():
    rng = np.random.default_rng(8)
    rows, B, C = 4, 3, 7
    x, y, g = _rand(rng, B * rows, C), _rand(rng, B * rows, C), _rand(rng, B * rows, C)
    alpha = _rand(rng, B, C)
    tx, ty, ta = [torch.tensor(a, requires_grad=True) for a in (x, y, alpha)]
    out = tx + ta.repeat_interleave(rows, dim=0) * ty
    np.testing.assert_allclose(bo.gate_residual_fwd(x, y, alpha, rows), out.detach().numpy(), rtol=1e-14)
    (out * torch.tensor(g)).sum().backward()
    dx, dy, dalpha = bo.gate_residual_bwd(y, alpha, g, rows)
    np.testing.assert_allclose(dx, tx.grad.numpy(), rtol=1e-12)
    np.testing.assert_allclose(dy, ty.grad.numpy(), rtol=1e-12)
    np.testing.assert_allclose(dalpha, ta.grad.numpy(), rtol=1e-12, atol=1e-13)


# ---------------------------------------------------------------- SwiGLU gate
def test_swiglu_known_values_and_identities():
    u = np.array([[0.0, 1.0, -1.0, 30.0, -30.0, -800.0]])
    v = np.ones_like(u)
    g = bo.swiglu_fwd(np.concatenate([u, v], axis=1))
    assert g[0, 0] == 0.0
    assert g[0, 1] == pytest.approx(1.0 / (1.0 + math.exp(-1.0)), rel=1e-15)
    # silu(u) - silu(-u) = u, since the two logistic values add up to one
    assert g[0, 1] - g[0, 2] == pytest.approx(1.0, abs=1e-15)
    assert g[0, 3] - g[0, 4] == pytest.approx(30.0, abs=1e-13)
    assert g[0, 3] == pytest.approx(30.0, rel=1e-12)          # silu(u) -> u
    assert abs(g[0, 4]) < 1e-11 and g[0, 5] == 0.0           # silu(u) -> 0 without overflow
    rng = np.random.default_rng(9)
    uu, vv = _rand(rng, 5, 12) * 4, _rand(rng, 5, 12)
    ref = torch.nn.functional.silu(torch.from_numpy(uu)).numpy() * vv
    np.testing.assert_allclose(bo.swiglu_fwd(np.concatenate([uu, vv], axis=1)), ref, rtol=1e-13, atol=1e-15)


def test_swiglu_u_is_the_first_half_of_the_packed_row():
    uv = np.array([[2.0, 0.0, 5.0, 7.0]])      # u = (2, 0), v = (5, 7)
    g = bo.swiglu_fwd(uv)
    assert g[0, 0] == pytest.approx(2.0 / (1.0 + math.exp(-2.0)) * 5.0, rel=1e-15)
    assert g[0, 1] == 0.0


def test_swiglu_backward_known_slope_and_autograd():
    # d silu / du at 0 is 1/2; with v = 3 and dg = 2 the u-gradient is 3
    d = bo.swiglu_bwd(np.array([[0.0, 3.0]]), np.array([[2.0]]))
    assert d[0, 0] == pytest.approx(3.0, abs=1e-15) and d[0, 1] == 0.0
    rng = np.random.default_rng(10)
    uv, dg = _rand(rng, 6, 20) * 3, _rand(rng, 6, 10)
    t = torch.tensor(uv, requires_grad=True)
    (torch.nn.functional.silu(t[:, :10]) * t[:, 10:] * torch.tensor(dg)).sum().backward()
    np.testing.assert_allclose(bo.swiglu_bwd(uv, dg), t.grad.numpy(), rtol=1e-12, atol=1e-14)


def test_swiglu_backward_against_finite_differences():
    rng = np.random.default_rng(11)
    uv, dg = _rand(rng, 3, 8) * 2, _rand(rng, 3, 4)
    d = bo.swiglu_bwd(uv, dg)
    f = lambda: float(np.sum(bo.swiglu_fwd(uv) * dg))
    for i in range(3):
        for c in range(8):
            assert d[i, c] == pytest.approx(_central(f, uv, (i, c)), rel=1e-6, abs=1e-8)


def test_rows_must_be_whole_samples():
    with pytest.raises(ValueError):
        bo.rmsnorm_adaln_fwd(np.ones((5, 4)), np.ones(4), np.zeros((2, 4)), np.zeros((2, 4)), 0.0, 2)
    with pytest.raises(ValueError):
        bo.swiglu_fwd(np.ones((2, 5)))


# ---------------------------------------------------------------- projections of the normalised rows
def test_norm_linear_row_worked_by_hand():
    # the row of test_rmsnorm_row_worked_by_hand: h = (9/sqrt(12.5) + 1, 2)
    x = np.array([[3.0, 4.0]])
    w = np.array([2.0, 0.5])
    gamma = np.array([[0.5, -1.0]])
    beta = np.array([[1.0, 2.0]])
    weight = np.array([[1.0, 0.0], [0.0, 1.0], [2.0, -3.0]])       # [F = 3, C = 2]
    y = bo.norm_linear_fwd(x, w, gamma, beta, 0.0, 1, weight)
    h0 = 9.0 / math.sqrt(12.5) + 1.0
    np.testing.assert_allclose(y, [[h0, 2.0, 2.0 * h0 - 6.0]], rtol=0, atol=1e-14)
    # SwiGLU on a 4-row weight: u = (y0, y1), v = (y2, y0 + y1)
    w4 = np.array([[1.0, 0.0], [0.0, 1.0], [2.0, -3.0], [1.0, 1.0]])
    g, uv = bo.norm_linear_swiglu_fwd(x, w, gamma, beta, 0.0, 1, w4)
    np.testing.assert_allclose(uv, [[h0, 2.0, 2.0 * h0 - 6.0, h0 + 2.0]], rtol=0, atol=1e-14)
    silu = lambda t: t / (1.0 + math.exp(-t))
    np.testing.assert_allclose(g, [[silu(h0) * (2.0 * h0 - 6.0), silu(2.0) * (h0 + 2.0)]],
                               rtol=0, atol=1e-14)


def test_norm_linear_against_scalar_loops_and_torch():
    rng = np.random.default_rng(31)
    B, rows, C, F = 2, 3, 6, 4                                    # F != C: a transposed W cannot pass
    x = _rand(rng, B * rows, C)
    w, gamma, beta = 1.0 + 0.1 * _rand(rng, C), 0.3 * _rand(rng, B, C), _rand(rng, B, C)
    weight = _rand(rng, 2 * F, C)
    eps = 1e-5
    g, uv = bo.norm_linear_swiglu_fwd(x, w, gamma, beta, eps, rows, weight)
    # scalar loops, nothing shared with the oracle
    for i in range(B * rows):
        b = i // rows
        ms = sum(x[i, c] ** 2 for c in range(C)) / C
        r = 1.0 / math.sqrt(ms + eps)
        h = [x[i, c] * r * w[c] * (1.0 + gamma[b, c]) + beta[b, c] for c in range(C)]
        for f in range(2 * F):
            want = sum(h[c] * weight[f, c] for c in range(C))
            assert uv[i, f] == pytest.approx(want, abs=1e-13)
        for f in range(F):
            u, v = uv[i, f], uv[i, F + f]
            assert g[i, f] == pytest.approx(u / (1.0 + math.exp(-u)) * v, abs=1e-13)
    np.testing.assert_allclose(bo.norm_linear_fwd(x, w, gamma, beta, eps, rows, weight), uv,
                               rtol=0, atol=0)
    # torch's own routines in double
    tx = torch.tensor(x)
    n = torch.nn.functional.rms_norm(tx, (C,), weight=torch.tensor(w), eps=eps)
    bidx = torch.arange(B * rows) // rows
    th = n * (1.0 + torch.tensor(gamma)[bidx]) + torch.tensor(beta)[bidx]
    tuv = torch.nn.functional.linear(th, torch.tensor(weight))
    np.testing.assert_allclose(uv, tuv.numpy(), rtol=0, atol=1e-13)
    tg = torch.nn.functional.silu(tuv[:, :F]) * tuv[:, F:]
    np.testing.assert_allclose(g, tg.numpy(), rtol=0, atol=1e-13)
    np.testing.assert_allclose(bo.linear_fwd(x, weight), x @ weight.T, rtol=0, atol=0)
    with pytest.raises(ValueError):
        bo.linear_fwd(x, weight.T)


def test_norm_linear_invariants():
    rng = np.random.default_rng(32)
    B, rows, C, F = 2, 4, 8, 5
    x = _rand(rng, B * rows, C)
    w, gamma, beta = _rand(rng, C), 0.2 * _rand(rng, B, C), _rand(rng, B, C)
    weight = _rand(rng, F, C)
    y = bo.norm_linear_fwd(x, w, gamma, beta, 0.0, rows, weight)
    # without eps the projection does not see the scale of a row
    np.testing.assert_allclose(bo.norm_linear_fwd(3.0 * x, w, gamma, beta, 0.0, rows, weight), y,
                               rtol=1e-12)
    # zero rows leave the shift alone: y = beta_b W^T
    y0 = bo.norm_linear_fwd(np.zeros_like(x), w, gamma, beta, 1e-6, rows, weight)
    np.testing.assert_allclose(y0[:rows], np.tile(beta[0] @ weight.T, (rows, 1)), rtol=1e-13)
    np.testing.assert_allclose(y0[rows:], np.tile(beta[1] @ weight.T, (rows, 1)), rtol=1e-13)
    # linear in W; and the folded form the kernels use is the same map:
    #   y_i = r_i * x_i (W diag(w (1 + gamma_b)))^T + beta_b W^T
    np.testing.assert_allclose(bo.norm_linear_fwd(x, w, gamma, beta, 0.0, rows, 2.0 * weight), 2.0 * y,
                               rtol=1e-13)
    _, r = bo.rmsnorm_adaln_fwd(x, w, gamma, beta, 0.0, rows)
    for b in range(B):
        sl = slice(b * rows, (b + 1) * rows)
        folded = weight * (w * (1.0 + gamma[b]))[None, :]
        np.testing.assert_allclose(r[sl, None] * (x[sl] @ folded.T) + beta[b] @ weight.T, y[sl],
                                   rtol=0, atol=1e-12)


# ---------------------------------------------------------------- backward of a projection
def test_linear_bwd_worked_by_hand():
    # y = x W^T with x = (1, 2), W = [[3, 4], [5, 6], [7, 8]], dy = (1, 0, -1):
    # dx = dy W = (3 - 7, 4 - 8); dW = dy^T x = rows (1, 2), (0, 0), (-1, -2)
    x = np.array([[1.0, 2.0]])
    weight = np.array([[3.0, 4.0], [5.0, 6.0], [7.0, 8.0]])
    dy = np.array([[1.0, 0.0, -1.0]])
    dx, dw = bo.linear_bwd(x, weight, dy)
    np.testing.assert_array_equal(dx, [[-4.0, -4.0]])
    np.testing.assert_array_equal(dw, [[1.0, 2.0], [0.0, 0.0], [-1.0, -2.0]])


def test_linear_bwd_against_scalar_loops_autograd_and_differences():
    rng = np.random.default_rng(77)
    n, c, f = 7, 5, 4                       # all different: a transposed operand changes a shape
    x, weight, dy = _rand(rng, n, c), _rand(rng, f, c), _rand(rng, n, f)
    dx, dw = bo.linear_bwd(x, weight, dy)
    assert dx.shape == (n, c) and dw.shape == (f, c)
    for i in range(n):
        for k in range(c):
            assert dx[i, k] == pytest.approx(sum(dy[i, j] * weight[j, k] for j in range(f)), abs=1e-13)
    for j in range(f):
        for k in range(c):
            assert dw[j, k] == pytest.approx(sum(dy[i, j] * x[i, k] for i in range(n)), abs=1e-13)
    tx = torch.tensor(x, requires_grad=True)
    tw = torch.tensor(weight, requires_grad=True)
    torch.nn.functional.linear(tx, tw).backward(torch.tensor(dy))
    np.testing.assert_allclose(dx, tx.grad.numpy(), rtol=0, atol=1e-13)
    np.testing.assert_allclose(dw, tw.grad.numpy(), rtol=0, atol=1e-13)
    # central differences of L = <y, dy> through the forward oracle (L is bilinear: exact up to rounding)
    loss = lambda xx, ww: float(np.sum(bo.linear_fwd(xx, ww) * dy))
    h = 1e-3
    for (i, k) in [(0, 0), (3, 4), (6, 2)]:
        e = np.zeros_like(x); e[i, k] = h
        assert (loss(x + e, weight) - loss(x - e, weight)) / (2 * h) == pytest.approx(dx[i, k], abs=1e-9)
    for (j, k) in [(0, 0), (3, 4), (1, 2)]:
        e = np.zeros_like(weight); e[j, k] = h
        assert (loss(x, weight + e) - loss(x, weight - e)) / (2 * h) == pytest.approx(dw[j, k], abs=1e-9)
    # the two gradients pair up: <dx, x> = <dW, W> = <y, dy>
    assert np.sum(dx * x) == pytest.approx(np.sum(dw * weight), rel=1e-13)
    assert np.sum(dx * x) == pytest.approx(loss(x, weight), rel=1e-13)
    with pytest.raises(ValueError):
        bo.linear_bwd(x, weight, dy.T)
    with pytest.raises(ValueError):
        bo.linear_bwd(x, weight.T, dy)


def test_rmsnorm_bwd_residual_against_autograd_of_a_residual_layer():
    """out = x + c * h(x) (a branch that scales the normalised rows): the gradient of
    <out, dout> with respect to x is dout + the normalisation's backward of c * dout."""
    rng = np.random.default_rng(91)
    n, c, rows, eps = 6, 24, 3, 1e-5
    x, dout = _rand(rng, n, c), _rand(rng, n, c)
    w = 1.0 + 0.1 * _rand(rng, c)
    gamma, beta = 0.3 * _rand(rng, 2, c), _rand(rng, 2, c)
    scale = 0.7
    dx, dw, dgamma, dbeta = bo.rmsnorm_adaln_bwd_residual(x, w, gamma, beta, eps, rows, scale * dout, dout)
    tx = torch.tensor(x, requires_grad=True)
    tw = torch.tensor(w, requires_grad=True)
    tg = torch.tensor(gamma, requires_grad=True)
    tb = torch.tensor(beta, requires_grad=True)
    b = torch.arange(n) // rows
    th = tx * torch.rsqrt((tx * tx).mean(dim=1, keepdim=True) + eps) * tw * (1 + tg[b]) + tb[b]
    ((tx + scale * th) * torch.tensor(dout)).sum().backward()
    np.testing.assert_allclose(dx, tx.grad.numpy(), rtol=0, atol=1e-12)
    np.testing.assert_allclose(dw, tw.grad.numpy(), rtol=0, atol=1e-12)
    np.testing.assert_allclose(dgamma, tg.grad.numpy(), rtol=0, atol=1e-12)
    np.testing.assert_allclose(dbeta, tb.grad.numpy(), rtol=0, atol=1e-12)
    # no residual gradient: the plain backward
    plain = bo.rmsnorm_adaln_bwd(x, w, gamma, beta, eps, rows, dout)
    again = bo.rmsnorm_adaln_bwd_residual(x, w, gamma, beta, eps, rows, dout, np.zeros_like(x))
    for a_, b_ in zip(plain, again):
        np.testing.assert_array_equal(a_, b_)
