"""GPU parity of the fused projections of include/aeris_layer_ops.h (RMSNorm + adaptive modulation
folded into the QKV / SwiGLU up-projection GEMM, SwiGLU gate as its epilogue, plain output
projection; AERIS paper, Model Architecture section) against oracle/block_oracle.py.

Both sides start from the same bf16 activations and weights (exchanged as bit patterns) and fp32
parameters; the oracle is fp64 throughout and rounds nothing.  The kernels multiply in bf16: the
raw rows x are bf16 as given, the folded weight W_fc w_c (1 + gamma_bc) is rounded to bf16 once
(half an ulp, 2^-8 relative at worst, per element), products accumulate in fp32, the row scale and
the bias are applied in fp32 and the result is rounded to bf16.  Tolerances, written out in
`close`: relative L2 of a whole tensor <= 3e-3 (the bound of the other layer operations; the
folded-weight rounding and the output rounding are each uniform within half an ulp, 2^-9 / sqrt 3
= 1.1e-3 in relative L2, together 1.6e-3, measured 1.6e-3 to 2.4e-3), 4e-3 for the gated output
g = silu(u) v, which multiplies two such values and is rounded once more (expected
sqrt(2 * 1.6e-3^2 + 1.1e-3^2) = 2.5e-3, measured 2.7e-3 to 3.0e-3), and per
element  |err| <= 2^-7 |ref| (output rounding, with a boundary step)
                  + 2^-8 r_i sum_c |x_ic| |Wf_fc|  (first-order effect of rounding the folded weight)
                  + 1e-5 |x_i|.|Wf_f| r_i          (fp32 accumulation of 2^11 terms).
"""
import numpy as np
import pytest
import torch

from oracle import block_oracle as bo
from oracle import winattn_oracle as orc
from paper_2509_13523_amd import binding as B
from paper_2509_13523_amd import synth
import parity_log

pytestmark = pytest.mark.gpu

REL_L2 = 3e-3
REL_L2_GATED = 4e-3


def to_dev(bits):
    return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)


def to_f64(t):
    return t.float().cpu().numpy().astype(np.float64)


def bf16_pair(a):
    """bf16 bit patterns of an fp32/fp64 array and their exact fp64 values."""
    bits = synth.f32_to_bf16_bits(np.asarray(a, dtype=np.float32))
    return bits, synth.bf16_bits_to_f64(bits)


def make_case(seed, n_samples, rows, channels, features):
    rng = np.random.default_rng(seed)
    gain = np.exp(0.5 * rng.standard_normal(channels))
    gain[rng.integers(0, channels, size=max(1, channels // 64))] *= 10.0   # outlier channels
    xb, x = bf16_pair(rng.standard_normal((n_samples * rows, channels)) * gain)
    wb, weight = bf16_pair(rng.standard_normal((features, channels)) / np.sqrt(channels))
    w = (1.0 + 0.1 * rng.standard_normal(channels)).astype(np.float32)
    gamma = (0.3 * rng.standard_normal((n_samples, channels))).astype(np.float32)
    beta = (0.5 * rng.standard_normal((n_samples, channels))).astype(np.float32)
    dev = lambda a: torch.from_numpy(a).cuda()
    return dict(x=x, weight=weight, w=w.astype(np.float64), gamma=gamma.astype(np.float64),
                beta=beta.astype(np.float64), tx=to_dev(xb), tweight=to_dev(wb), tw=dev(w),
                tgamma=dev(gamma), tbeta=dev(beta))


def rounding_bound(c, eps, rows):
    """2^-8 r_i sum_c |x_ic| |Wf_fc| + fp32 accumulation slack, per output element [N, F]."""
    n = c["x"].shape[0]
    _, r = bo.rmsnorm_adaln_fwd(c["x"], c["w"], c["gamma"], c["beta"], eps, rows)
    out = np.empty((n, c["weight"].shape[0]))
    for b in range(n // rows):
        sl = slice(b * rows, (b + 1) * rows)
        folded = np.abs(c["weight"] * (c["w"] * (1.0 + c["gamma"][b]))[None, :])
        out[sl] = r[sl, None] * (np.abs(c["x"][sl]) @ folded.T)
    return (2.0 ** -8 + 1e-5) * out


def close(name, got, ref, bound, rel_l2=REL_L2):
    got = to_f64(got)
    assert np.isfinite(got).all(), name
    err = np.abs(got - ref)
    rel = np.linalg.norm(got - ref) / np.linalg.norm(ref)
    allow = 2.0 ** -7 * np.abs(ref) + bound + 1e-30
    parity_log.add(name, "bf16", rel, err.max(), np.abs(ref).max(), (allow).max(),
                   np.linalg.norm(bound) / np.linalg.norm(ref))
    worst = np.argmax(err - allow)
    assert (err <= allow).all(), "%s: err %.3e > %.3e at %d" % (name, err.flat[worst],
                                                                allow.flat[worst], worst)
    assert rel <= rel_l2, "%s rel_l2 %.3e" % (name, rel)


PROJ_CASES = [
    # samples, rows per sample, channels, out features
    (1, 256, 64, 8),          # one step of 64 channels, eight features: most of the tile is padding
    (2, 300, 128, 384),       # ragged second token tile (44 rows), ragged second feature tile
    (3, 70, 256, 520),        # every sample smaller than a tile, three feature tiles
    (1, 1000, 192, 256),      # four token tiles, odd number of 64-channel steps
    (2, 513, 2048, 264),      # the headline width; one row spills into a third token tile
]


@pytest.mark.parametrize("n_samples,rows,channels,features", PROJ_CASES)
def test_norm_linear_fwd(n_samples, rows, channels, features):
    eps = 1e-6
    c = make_case(100 + features, n_samples, rows, channels, features)
    y = B.aeris_norm_linear_fwd(c["tx"], c["tw"], c["tgamma"], c["tbeta"], eps, c["tweight"], rows)
    torch.cuda.synchronize()
    ref = bo.norm_linear_fwd(c["x"], c["w"], c["gamma"], c["beta"], eps, rows, c["weight"])
    close("y", y, ref, rounding_bound(c, eps, rows))
    # bitwise reproducible (no atomics, fixed summation order)
    y2 = B.aeris_norm_linear_fwd(c["tx"], c["tw"], c["tgamma"], c["tbeta"], eps, c["tweight"], rows)
    torch.cuda.synchronize()
    assert torch.equal(y.view(torch.int16), y2.view(torch.int16))


@pytest.mark.parametrize("n_samples,rows,channels,hidden", [
    (1, 256, 64, 8), (2, 300, 128, 200), (3, 70, 256, 128), (2, 260, 1024, 392)])
def test_norm_linear_swiglu_fwd(n_samples, rows, channels, hidden):
    eps = 1e-6
    c = make_case(200 + hidden, n_samples, rows, channels, 2 * hidden)
    g, uv = B.aeris_norm_linear_swiglu_fwd(c["tx"], c["tw"], c["tgamma"], c["tbeta"], eps,
                                           c["tweight"], rows)
    torch.cuda.synchronize()
    g_ref, uv_ref = bo.norm_linear_swiglu_fwd(c["x"], c["w"], c["gamma"], c["beta"], eps, rows,
                                              c["weight"])
    bound = rounding_bound(c, eps, rows)
    close("uv", uv, uv_ref, bound)
    # g = silu(u) v: |d g| <= |silu'(u)| |v| |d u| + |silu(u)| |d v|, |silu'| <= 1.1
    u, v = uv_ref[:, :hidden], uv_ref[:, hidden:]
    silu_u = u / (1.0 + np.exp(-u))
    close("g", g, g_ref, 1.1 * np.abs(v) * bound[:, :hidden] + np.abs(silu_u) * bound[:, hidden:],
          rel_l2=REL_L2_GATED)
    # without the packed up-projection: same g, nothing else written
    g2, none = B.aeris_norm_linear_swiglu_fwd(c["tx"], c["tw"], c["tgamma"], c["tbeta"], eps,
                                              c["tweight"], rows, want_uv=False)
    torch.cuda.synchronize()
    assert none is None and torch.equal(g.view(torch.int16), g2.view(torch.int16))


@pytest.mark.parametrize("n,channels,features", [(515, 192, 264), (256, 64, 8), (1030, 2048, 2048)])
def test_linear_fwd(n, channels, features):
    rng = np.random.default_rng(300 + n)
    xb, x = bf16_pair(rng.standard_normal((n, channels)))
    wb, weight = bf16_pair(rng.standard_normal((features, channels)) / np.sqrt(channels))
    y = B.aeris_linear_fwd(to_dev(xb), to_dev(wb))
    torch.cuda.synchronize()
    ref = bo.linear_fwd(x, weight)
    # exact bf16 operands: only fp32 accumulation and the output rounding remain
    close("y", y, ref, 1e-5 * (np.abs(x) @ np.abs(weight).T))


def test_qkv_projection_at_the_headline_size_on_sampled_rows():
    """4 x 720 x 1440 token rows x 2048 channels -> 6144 features (the QKV projection of the
    headline workload, in the launch configuration bench.py times): sampled rows against the
    oracle, which needs only those rows of x and the whole weight."""
    n_samples, rows, channels, features = 4, 720 * 1440, 2048, 6144
    eps = 1e-6
    n = n_samples * rows
    gen = torch.Generator(device="cuda").manual_seed(4100)
    tx = torch.randn(n, channels, device="cuda", dtype=torch.bfloat16, generator=gen)
    tweight = (torch.randn(features, channels, device="cuda", generator=gen) / channels ** 0.5).to(torch.bfloat16)
    tw = 1.0 + 0.1 * torch.randn(channels, device="cuda", generator=gen)
    tgamma = 0.3 * torch.randn(n_samples, channels, device="cuda", generator=gen)
    tbeta = 0.5 * torch.randn(n_samples, channels, device="cuda", generator=gen)
    y = B.aeris_norm_linear_fwd(tx, tw, tgamma, tbeta, eps, tweight, rows)
    torch.cuda.synchronize()
    f64 = lambda t: t.float().cpu().numpy().astype(np.float64)
    weight, w, gamma, beta = f64(tweight), f64(tw), f64(tgamma), f64(tbeta)
    picks = [0, 255, 256, rows - 1, rows, 2 * rows + 12345, 3 * rows + 777777, n - 1]
    for i in picks:
        b = i // rows
        xi = f64(tx[i:i + 1])
        ref = bo.norm_linear_fwd(xi, w, gamma[b:b + 1], beta[b:b + 1], eps, 1, weight)
        c = dict(x=xi, weight=weight, w=w, gamma=gamma[b:b + 1], beta=beta[b:b + 1])
        close("y", y[i:i + 1], ref, rounding_bound(c, eps, 1))


def test_attention_branch_from_the_fused_projections():
    """The attention half of a layer with this library's own projections: fused norm + QKV
    projection -> packed [B,H,W,3,heads,d] -> window attention on the packed buffer -> output
    projection -> gated residual, against the chained fp64 oracles with no rounding anywhere."""
    Bn, H, W, nh, d = 2, 24, 36, 2, 64
    C, rows = nh * d, H * W
    win, shift, mask = (12, 12), (6, 6), B.AERIS_MASK_SWIN
    eps = 1e-6
    c = make_case(400, Bn, rows, C, 3 * C)
    rng = np.random.default_rng(401)
    wob, wo = bf16_pair(rng.standard_normal((C, C)) / np.sqrt(C))
    alpha = (0.8 * rng.standard_normal((Bn, C))).astype(np.float32)
    # reference
    qkv = bo.norm_linear_fwd(c["x"], c["w"], c["gamma"], c["beta"], eps, rows, c["weight"])
    q, k, v = [qkv.reshape(Bn, H, W, 3, nh, d)[:, :, :, i] for i in range(3)]
    a, _ = orc.winattn_fwd(q, k, v, win, shift, mask)
    y = bo.linear_fwd(a.reshape(Bn * rows, C), wo)
    out = bo.gate_residual_fwd(c["x"], y, alpha.astype(np.float64), rows)
    # GPU
    tqkv = B.aeris_norm_linear_fwd(c["tx"], c["tw"], c["tgamma"], c["tbeta"], eps, c["tweight"], rows)
    import ctypes
    p = B.make_params((Bn, H, W, nh, d), win, shift, mask, qkv_strides=(3 * C, d))
    ta = torch.empty(Bn * rows, C, dtype=torch.bfloat16, device="cuda")
    tlse = torch.empty(Bn, nh, H, W, dtype=torch.float32, device="cuda")
    part = lambda i: tqkv.data_ptr() + i * C * 2
    rc = B.load().aeris_winattn_fwd(ctypes.byref(p), part(0), part(1), part(2), ta.data_ptr(),
                                    tlse.data_ptr(), torch.cuda.current_stream().cuda_stream)
    assert rc == 0
    ty = B.aeris_linear_fwd(ta, to_dev(wob))
    tout = B.aeris_gate_residual_fwd(c["tx"], ty, torch.from_numpy(alpha).cuda(), rows)
    torch.cuda.synchronize()
    rel = lambda got, ref: np.linalg.norm(to_f64(got) - ref) / np.linalg.norm(ref)
    errs = dict(qkv=rel(tqkv, qkv), a=rel(ta, a.reshape(Bn * rows, C)), y=rel(ty, y), out=rel(tout, out))
    for name, e in errs.items():
        parity_log.add(name, "bf16", e, 0.0, 0.0, 0.0)
    assert errs["qkv"] <= 3e-3 and errs["a"] <= 5e-3 and errs["y"] <= 6e-3 and errs["out"] <= 3e-3, errs


def test_projection_errors_are_reported():
    x = torch.zeros(256, 64, dtype=torch.bfloat16, device="cuda")
    wt = torch.zeros(16, 64, dtype=torch.bfloat16, device="cuda")
    f = torch.zeros(1, 64, device="cuda")
    ws = torch.empty(1 << 20, dtype=torch.uint8, device="cuda")
    with pytest.raises(B.AerisError) as e:
        B.aeris_norm_linear_fwd(x, f[0], f, f, 1e-6, wt, 100, workspace=ws)   # 256 % 100
    assert e.value.code == -3
    x96 = torch.zeros(256, 96, dtype=torch.bfloat16, device="cuda")     # 96 % 64
    with pytest.raises(B.AerisError) as e:
        B.aeris_linear_fwd(x96, torch.zeros(16, 96, dtype=torch.bfloat16, device="cuda"))
    assert e.value.code == -3
