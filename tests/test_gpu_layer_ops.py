"""GPU parity of include/aeris_layer_ops.h (pre-RMSNorm with adaptive modulation, gated
residual, SwiGLU gate; AERIS paper, Model Architecture section) against oracle/block_oracle.py.

Both sides start from the same bf16 activations (exchanged as bit patterns) and fp32 parameters.
The kernels compute in fp32 and round results to bf16 (nearest even), the oracle computes in fp64
and does not round.  A bf16 result may therefore differ from the fp64 value by one rounding
(2^-8 relative at worst) plus, where the fp32 value falls next to a rounding boundary, one more
step: the element-wise bound is 2^-7 |ref| plus an absolute slack for cancelling terms (and
1e-37, under the smallest normal bf16, where the kernels flush to zero); the
relative L2 error of a whole tensor is bounded by 3e-3.  fp32 sums over tokens: 2e-5 relative L2.
"""
import numpy as np
import pytest
import torch

from oracle import block_oracle as bo
from paper_2509_13523_amd import binding as B
from paper_2509_13523_amd import synth

pytestmark = pytest.mark.gpu

REL_L2_BF16 = 3e-3
REL_L2_SUM = 2e-5


def to_dev(bits):
    return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)


def to_f64(t):
    return t.float().cpu().numpy().astype(np.float64)


def activations(seed, n_rows, channels, spread=1.0):
    """bf16 bits and their exact fp64 values: N(0,1) times a per-channel gain (log-normal, a few
    channels 30 times larger, as the outlier channels of transformer activations)."""
    rng = np.random.default_rng(seed)
    gain = np.exp(spread * 0.5 * rng.standard_normal(channels))
    gain[rng.integers(0, channels, size=max(1, channels // 64))] *= 30.0
    a = synth.normal_field(seed + 1, (n_rows, channels)) * gain.astype(np.float32)
    bits = synth.f32_to_bf16_bits(a)
    return bits, synth.bf16_bits_to_f64(bits)


def vectors(seed, n_samples, channels, scale):
    v = (scale * np.random.default_rng(seed).standard_normal((n_samples, channels))).astype(np.float32)
    return v, torch.from_numpy(v).cuda()


def bf16_close(name, got, ref, slack):
    got = to_f64(got)
    assert np.isfinite(got).all(), name
    err = np.abs(got - ref)
    bound = 2.0 ** -7 * np.abs(ref) + slack + 1e-37   # below the smallest normal bf16: flushed to zero
    worst = np.argmax(err - bound)
    assert (err <= bound).all(), "%s: err %.3e > bound %.3e at %d" % (
        name, err.flat[worst], np.broadcast_to(bound, err.shape).flat[worst], worst)
    rel = np.linalg.norm(got - ref) / max(np.linalg.norm(ref), 1e-30)
    assert rel <= REL_L2_BF16, "%s rel_l2 %.3e" % (name, rel)


def sum_close(name, got, ref):
    got = got.cpu().numpy().astype(np.float64)
    assert np.isfinite(got).all(), name
    rel = np.linalg.norm(got - ref) / max(np.linalg.norm(ref), 1e-30)
    assert rel <= REL_L2_SUM, "%s rel_l2 %.3e" % (name, rel)


ROW_CASES = [
    # samples, rows per sample, channels
    (2, 37, 96),        # one vector per lane, 12 of 64 lanes used
    (3, 5, 520),        # 65 vectors: second vector of lane 0 only
    (1, 300, 2048),     # the headline width (16 heads x 128)
    (2, 33, 4096),      # the widest supported row
    (4, 1, 8),          # one-row samples, one vector
    (1, 1, 64),
    (2, 1000, 1024),
    (5, 3, 1536),       # three of four vectors per lane
]


@pytest.mark.parametrize("nb,rps,C", ROW_CASES)
def test_rmsnorm_adaln_forward_and_backward(nb, rps, C):
    n = nb * rps
    eps = 1e-6
    xb, x64 = activations(100 + C, n, C)
    gb, g64 = activations(200 + C, n, C, spread=0.5)
    w = (1.0 + 0.2 * np.random.default_rng(C).standard_normal(C)).astype(np.float32)
    gamma, tgamma = vectors(C + 1, nb, C, 0.3)
    beta, tbeta = vectors(C + 2, nb, C, 0.5)
    tw = torch.from_numpy(w).cuda()
    tx, tdh = to_dev(xb), to_dev(gb)

    th, tr = B.aeris_rmsnorm_adaln_fwd(tx, tw, tgamma, tbeta, eps, rps)
    tdx, tdw, tdgamma, tdbeta = B.aeris_rmsnorm_adaln_bwd(tx, tw, tgamma, tr, tdh, rps)
    torch.cuda.synchronize()

    w64, gamma64, beta64 = w.astype(np.float64), gamma.astype(np.float64), beta.astype(np.float64)
    h, r = bo.rmsnorm_adaln_fwd(x64, w64, gamma64, beta64, eps, rps)
    np.testing.assert_allclose(tr.cpu().numpy(), r, rtol=2e-6)
    # h = n s + beta cancels when the two terms are opposite: slack from the fp32 terms
    smp = np.arange(n) // rps
    term = np.abs(x64 * r[:, None] * w64 * (1 + gamma64[smp])) + np.abs(beta64[smp])
    bf16_close("h", th, h, 2.0 ** -20 * term)

    dx, dw, dgamma, dbeta = bo.rmsnorm_adaln_bwd(x64, w64, gamma64, beta64, eps, rps, g64)
    dn = g64 * w64 * (1 + gamma64[smp])
    nrm = x64 * r[:, None]
    term = r[:, None] * (np.abs(dn) + np.abs(nrm) * np.abs(np.mean(dn * nrm, axis=1, keepdims=True)))
    # the row mean of dn * n is itself an fp32 sum of C cancelling products
    mean_err = 2.0 ** -21 * np.mean(np.abs(dn * nrm), axis=1, keepdims=True) * np.sqrt(C)
    bf16_close("dx", tdx, dx, 2.0 ** -20 * term + r[:, None] * np.abs(nrm) * mean_err)
    sum_close("dw", tdw, dw)
    sum_close("dgamma", tdgamma, dgamma)
    sum_close("dbeta", tdbeta, dbeta)

    # with the residual connection closed in the same pass: dx + dres, rounded once; the
    # parameter gradients do not change by a bit
    rb_, r64 = activations(300 + C, n, C, spread=0.5)
    tdx2, tdw2, tdgamma2, tdbeta2 = B.aeris_rmsnorm_adaln_bwd(tx, tw, tgamma, tr, tdh, rps, dres=to_dev(rb_))
    torch.cuda.synchronize()
    dx2, _, _, _ = bo.rmsnorm_adaln_bwd_residual(x64, w64, gamma64, beta64, eps, rps, g64, r64)
    bf16_close("dx+dres", tdx2, dx2, 2.0 ** -20 * (term + np.abs(r64)) + r[:, None] * np.abs(nrm) * mean_err)
    assert torch.equal(tdw, tdw2) and torch.equal(tdgamma, tdgamma2) and torch.equal(tdbeta, tdbeta2)


def test_rmsnorm_adaln_without_r_and_without_parameter_gradients():
    nb, rps, C = 2, 50, 256
    xb, _ = activations(1, nb * rps, C)
    gb, _ = activations(2, nb * rps, C)
    tw = torch.ones(C, device="cuda")
    _, tgamma = vectors(3, nb, C, 0.3)
    _, tbeta = vectors(4, nb, C, 0.3)
    tx, tdh = to_dev(xb), to_dev(gb)
    h1, r1 = B.aeris_rmsnorm_adaln_fwd(tx, tw, tgamma, tbeta, 1e-5, rps)
    h2, r2 = B.aeris_rmsnorm_adaln_fwd(tx, tw, tgamma, tbeta, 1e-5, rps, want_r=False)
    assert r2 is None and torch.equal(h1.view(torch.int16), h2.view(torch.int16))
    full = B.aeris_rmsnorm_adaln_bwd(tx, tw, tgamma, r1, tdh, rps)
    only_dx = B.aeris_rmsnorm_adaln_bwd(tx, tw, tgamma, r1, tdh, rps, want=(False, False, False))
    assert only_dx[1] is None and only_dx[2] is None and only_dx[3] is None
    assert torch.equal(full[0].view(torch.int16), only_dx[0].view(torch.int16))
    some = B.aeris_rmsnorm_adaln_bwd(tx, tw, tgamma, r1, tdh, rps, want=(False, True, False))
    assert torch.equal(some[2], full[2])


def test_sums_over_tokens_are_bitwise_reproducible_and_span_many_chunks():
    nb, rps, C = 2, 20000, 512
    n = nb * rps
    xb, x64 = activations(11, n, C)
    gb, g64 = activations(12, n, C, spread=0.5)
    w = np.random.default_rng(13).standard_normal(C).astype(np.float32)
    gamma, tgamma = vectors(14, nb, C, 0.3)
    tw = torch.from_numpy(w).cuda()
    tx, tdh = to_dev(xb), to_dev(gb)
    _, tr = B.aeris_rmsnorm_adaln_fwd(tx, tw, tgamma, tgamma, 1e-6, rps)
    a = B.aeris_rmsnorm_adaln_bwd(tx, tw, tgamma, tr, tdh, rps)
    b = B.aeris_rmsnorm_adaln_bwd(tx, tw, tgamma, tr, tdh, rps)
    torch.cuda.synchronize()
    for u, v in zip(a[1:], b[1:]):
        assert torch.equal(u, v)
    assert torch.equal(a[0].view(torch.int16), b[0].view(torch.int16))
    _, dw, dgamma, dbeta = bo.rmsnorm_adaln_bwd(x64, w.astype(np.float64), gamma.astype(np.float64),
                                                gamma.astype(np.float64), 1e-6, rps, g64)
    sum_close("dw", a[1], dw)
    sum_close("dgamma", a[2], dgamma)
    sum_close("dbeta", a[3], dbeta)
    # the gate's sums take the same route
    _, talpha = vectors(15, nb, C, 1.0)
    d1 = B.aeris_gate_residual_bwd(tx, talpha, tdh, rps)
    d2 = B.aeris_gate_residual_bwd(tx, talpha, tdh, rps)
    assert torch.equal(d1[1], d2[1])
    _, _, dalpha = bo.gate_residual_bwd(x64, talpha.cpu().numpy().astype(np.float64), g64, rps)
    sum_close("dalpha", d1[1], dalpha)


@pytest.mark.parametrize("nb,rps,C", ROW_CASES)
def test_gate_residual_forward_and_backward(nb, rps, C):
    n = nb * rps
    xb, x64 = activations(300 + C, n, C)
    yb, y64 = activations(400 + C, n, C)
    gb, g64 = activations(500 + C, n, C, spread=0.5)
    alpha, talpha = vectors(C + 3, nb, C, 1.0)
    a64 = alpha.astype(np.float64)
    tx, ty, tg = to_dev(xb), to_dev(yb), to_dev(gb)
    tout = B.aeris_gate_residual_fwd(tx, ty, talpha, rps)
    tdy, tdalpha = B.aeris_gate_residual_bwd(ty, talpha, tg, rps)
    torch.cuda.synchronize()
    smp = np.arange(n) // rps
    out = bo.gate_residual_fwd(x64, y64, a64, rps)
    bf16_close("out", tout, out, 2.0 ** -22 * (np.abs(x64) + np.abs(a64[smp] * y64)))
    _, dy, dalpha = bo.gate_residual_bwd(y64, a64, g64, rps)
    bf16_close("dy", tdy, dy, 0.0)
    sum_close("dalpha", tdalpha, dalpha)
    # in place: out over x, dy over dout
    x2, g2 = tx.clone(), tg.clone()
    B.aeris_gate_residual_fwd(x2, ty, talpha, rps, out=x2)
    B.aeris_gate_residual_bwd(ty, talpha, g2, rps, dy=g2, want_dalpha=False)
    torch.cuda.synchronize()
    assert torch.equal(x2.view(torch.int16), tout.view(torch.int16))
    assert torch.equal(g2.view(torch.int16), tdy.view(torch.int16))


@pytest.mark.parametrize("n,F", [(7, 8), (33, 24), (100, 520), (64, 2048), (3, 8192), (1000, 1024)])
def test_swiglu_forward_and_backward(n, F):
    uvb, uv64 = activations(600 + F, n, 2 * F)
    gb, g64 = activations(700 + F, n, F, spread=0.5)
    tuv, tdg = to_dev(uvb), to_dev(gb)
    tg = B.aeris_swiglu_fwd(tuv)
    tduv = B.aeris_swiglu_bwd(tuv, tdg)
    torch.cuda.synchronize()
    g = bo.swiglu_fwd(uv64)
    duv = bo.swiglu_bwd(uv64, g64)
    # the logistic value s = 1 / (1 + exp(-u)) is an fp32 number in the kernels: below the smallest
    # normal fp32 (u < -87) it is flushed to zero, which moves results by at most TINY times
    # their other factors
    TINY = 1.2e-38
    u, v = uv64[:, :F], uv64[:, F:]
    bf16_close("g", tg, g, TINY * np.abs(u * v))
    # du = dg v s (1 + u (1 - s)): the bracket cancels near u = -1.28; slack from its terms
    s = 1.0 / (1.0 + np.exp(-np.clip(u, -700, 700)))
    slack = np.concatenate([(2.0 ** -20 * s + TINY) * np.abs(g64 * v) * (1 + np.abs(u)),
                            TINY * np.abs(g64 * u)], axis=1)
    bf16_close("duv", tduv, duv, slack)
    # in place over uv
    uv2 = tuv.clone()
    B.aeris_swiglu_bwd(uv2, tdg, duv=uv2)
    torch.cuda.synchronize()
    assert torch.equal(uv2.view(torch.int16), tduv.view(torch.int16))


def test_swiglu_extreme_gate_inputs():
    F = 16
    u = np.array([0.0, -0.0, 1.0, -1.0, 20.0, -20.0, 60.0, -60.0, 88.0, -88.0, 120.0, -120.0,
                  300.0, -300.0, 1e-3, -1e-3], dtype=np.float32)
    v = np.linspace(-2.0, 2.0, F, dtype=np.float32)
    uv = np.concatenate([u, v])[None, :].repeat(3, axis=0)
    bits = synth.f32_to_bf16_bits(uv)
    uv64 = synth.bf16_bits_to_f64(bits)
    dgb = synth.f32_to_bf16_bits(np.ones((3, F), dtype=np.float32))
    tg = B.aeris_swiglu_fwd(to_dev(bits))
    tduv = B.aeris_swiglu_bwd(to_dev(bits), to_dev(dgb))
    torch.cuda.synchronize()
    u64, v64 = uv64[:, :F], uv64[:, F:]
    bf16_close("g", tg, bo.swiglu_fwd(uv64), 1.2e-38 * np.abs(u64 * v64))
    bf16_close("duv", tduv, bo.swiglu_bwd(uv64, np.ones((3, F))),
               1.2e-38 * np.concatenate([np.abs(v64) * (1 + np.abs(u64)), np.abs(u64)], axis=1))


def test_headline_size_rows_sampled():
    """4 x 720 x 1440 tokens x 2048 channels (the headline grid with 16 heads x 128): sampled rows
    of h and dx against the oracle row by row, the shift gradient against a plain fp64 column sum."""
    nb, rps, C = 4, 720 * 1440, 2048
    n = nb * rps
    gen = torch.Generator(device="cuda").manual_seed(77)
    tx = torch.randn(n, C, device="cuda", dtype=torch.bfloat16, generator=gen)
    tdh = torch.randn(n, C, device="cuda", dtype=torch.bfloat16, generator=gen)
    w = (1.0 + 0.1 * np.random.default_rng(78).standard_normal(C)).astype(np.float32)
    gamma, tgamma = vectors(79, nb, C, 0.3)
    beta, tbeta = vectors(80, nb, C, 0.5)
    tw = torch.from_numpy(w).cuda()
    th, tr = B.aeris_rmsnorm_adaln_fwd(tx, tw, tgamma, tbeta, 1e-6, rps)
    tdx, tdw, tdgamma, tdbeta = B.aeris_rmsnorm_adaln_bwd(tx, tw, tgamma, tr, tdh, rps)
    torch.cuda.synchronize()
    rows = np.unique(np.concatenate([[0, 1, rps - 1, rps, n - 1],
                                     np.random.default_rng(81).integers(0, n, size=59)]))
    idx = torch.from_numpy(rows).cuda()
    x64, g64 = to_f64(tx[idx]), to_f64(tdh[idx])
    hs, dxs, rs = to_f64(th[idx]), to_f64(tdx[idx]), tr[idx].cpu().numpy()
    w64 = w.astype(np.float64)
    for j, row in enumerate(rows):
        smp = int(row // rps)
        gm, bt = gamma[smp:smp + 1].astype(np.float64), beta[smp:smp + 1].astype(np.float64)
        h, r = bo.rmsnorm_adaln_fwd(x64[j:j + 1], w64, gm, bt, 1e-6, 1)
        assert abs(rs[j] - r[0]) <= 2e-6 * r[0]
        assert (np.abs(hs[j] - h[0]) <= 2.0 ** -7 * np.abs(h[0]) + 1e-5).all(), row
        dx, _, _, _ = bo.rmsnorm_adaln_bwd(x64[j:j + 1], w64, gm, bt, 1e-6, 1, g64[j:j + 1])
        assert (np.abs(dxs[j] - dx[0]) <= 2.0 ** -7 * np.abs(dx[0]) + 1e-5).all(), row
    ref = tdh.view(nb, rps, C).sum(dim=1, dtype=torch.float64)
    rel = (tdbeta.double() - ref).norm() / ref.norm()
    assert rel.item() <= REL_L2_SUM
    del th, tdx
    # gated residual and SwiGLU at the same number of tokens (hidden = channels here)
    _, talpha = vectors(82, nb, C, 1.0)
    tout = B.aeris_gate_residual_fwd(tx, tdh, talpha, rps)
    tg = B.aeris_swiglu_fwd(tx)
    torch.cuda.synchronize()
    xs, ys = to_f64(tx[idx]), to_f64(tdh[idx])
    outs, gs = to_f64(tout[idx]), to_f64(tg[idx])
    alpha64 = talpha.cpu().numpy().astype(np.float64)
    for j, row in enumerate(rows):
        smp = int(row // rps)
        out = bo.gate_residual_fwd(xs[j:j + 1], ys[j:j + 1], alpha64[smp:smp + 1], 1)
        assert (np.abs(outs[j] - out[0]) <= 2.0 ** -7 * np.abs(out[0]) + 1e-5).all(), row
        g = bo.swiglu_fwd(xs[j:j + 1])
        assert (np.abs(gs[j] - g[0]) <= 2.0 ** -7 * np.abs(g[0]) + 1e-30).all(), row


def test_errors_are_reported():
    t = torch.zeros(8, 64, device="cuda", dtype=torch.bfloat16)
    f = torch.zeros(2, 64, device="cuda")
    w = torch.zeros(64, device="cuda")
    with pytest.raises(B.AerisError):
        B.aeris_rmsnorm_adaln_fwd(t, w, f, f, 1e-6, 3)          # 8 rows are not whole samples of 3
    r = torch.zeros(8, device="cuda")
    small = torch.zeros(16, dtype=torch.uint8, device="cuda")
    with pytest.raises(B.AerisError):
        B.aeris_rmsnorm_adaln_bwd(t, w, f, r, t, 4, workspace=small)
