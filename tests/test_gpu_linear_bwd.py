"""GPU parity of aeris_linear_bwd (include/aeris_layer_ops.h: the gradients dx = dy W and
dW = dy^T x of a projection y = x W^T; AERIS paper, Model Architecture section: the projections
of a transformer layer, whose backward pass training runs) against oracle/block_oracle.py.

Both sides start from the same bf16 operands (exchanged as bit patterns); the oracle is fp64 and
rounds nothing.  On the GPU the products of bf16 values are exact in fp32 and accumulate in fp32.
Tolerances, written out in `close_dx` / `close_dw`:
  dx (bf16 out):  |err| <= 2^-7 |ref| (output rounding, with a boundary step)
                          + 1e-5 sum_f |dy_if| |W_fc|         (fp32 accumulation, up to 11008 terms)
                  relative L2 <= 3e-3 (output rounding alone is 2^-9 / sqrt 3 = 1.1e-3).
  dW (fp32 out):  |err| <= slack * sum_i |dy_if| |x_ic|,  slack = max(1e-5, 4 sqrt(N) 2^-24):
                  a running fp32 sum of N terms picks up about sqrt(N) roundings of 2^-24 of the
                  partial sum, which the sum of magnitudes bounds; relative L2 <= 1e-4 at the
                  sizes the oracle runs whole (measured 2e-7), also on the sampled entries of the
                  headline size (N = 4.1 million rows; measured 4.6e-6).
"""
import numpy as np
import pytest
import torch

from oracle import block_oracle as bo
from paper_2509_13523_amd import binding as B
from paper_2509_13523_amd import synth
import parity_log

pytestmark = pytest.mark.gpu


def to_dev(bits):
    return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)


def to_f64(t):
    return t.float().cpu().numpy().astype(np.float64)


def bf16_pair(a):
    bits = synth.f32_to_bf16_bits(np.asarray(a, dtype=np.float32))
    return bits, synth.bf16_bits_to_f64(bits)


def close_dx(got, ref, mag):
    got = to_f64(got)
    assert np.isfinite(got).all()
    err = np.abs(got - ref)
    allow = 2.0 ** -7 * np.abs(ref) + 1e-5 * mag + 1e-30
    rel = np.linalg.norm(got - ref) / np.linalg.norm(ref)
    parity_log.add("dx", "bf16", rel, err.max(), np.abs(ref).max(), allow.max())
    assert (err <= allow).all(), "dx: err %.3e at %d" % (err.max(), np.argmax(err - allow))
    assert rel <= 3e-3, rel


def close_dw(got, ref, mag, n_rows, rel_l2=1e-4):
    got = got.double().cpu().numpy() if torch.is_tensor(got) else got
    assert np.isfinite(got).all()
    err = np.abs(got - ref)
    slack = max(1e-5, 4.0 * np.sqrt(n_rows) * 2.0 ** -24)
    allow = slack * mag + 1e-30
    rel = np.linalg.norm(got - ref) / np.linalg.norm(ref)
    parity_log.add("dweight", "f32", rel, err.max(), np.abs(ref).max(), allow.max())
    assert (err <= allow).all(), "dW: err %.3e at %d" % (err.max(), np.argmax(err - allow))
    assert rel <= rel_l2, rel


CASES = [
    # rows, channels, out features
    (64, 64, 64),             # one step, one tile that is mostly padding
    (1024, 192, 320),         # ragged channel tile, ragged second feature tile, one row range
    (4096, 256, 512),         # two feature tiles, four row ranges added by the second kernel
    (2112, 2048, 448),        # the headline width; 33 steps: the last row range holds one step
    (8256, 128, 6144),        # 24 feature tiles (three per XCD), nine row ranges
    (1000, 192, 320),         # 15 whole steps and 40 rows left over
    (40, 64, 128),            # fewer rows than one step: everything is "left over"
    (4159, 256, 512),         # four row ranges and 63 rows left over
    (1024, 64, 11008),        # the SwiGLU width: 43 feature tiles (empty slots on five XCDs);
                              # dx contracts over 11008 features
]


@pytest.mark.parametrize("n,channels,features", CASES)
def test_linear_bwd(n, channels, features):
    rng = np.random.default_rng(500 + features + n)
    gain = np.exp(0.5 * rng.standard_normal(channels))
    xb, x = bf16_pair(rng.standard_normal((n, channels)) * gain)
    wb, weight = bf16_pair(rng.standard_normal((features, channels)) / np.sqrt(channels))
    dyb, dy = bf16_pair(rng.standard_normal((n, features)) * np.exp(0.5 * rng.standard_normal(features)))
    tx, tw, tdy = to_dev(xb), to_dev(wb), to_dev(dyb)
    dx, dw = B.aeris_linear_bwd(tx, tw, tdy)
    torch.cuda.synchronize()
    dx_ref, dw_ref = bo.linear_bwd(x, weight, dy)
    close_dx(dx, dx_ref, np.abs(dy) @ np.abs(weight))
    close_dw(dw, dw_ref, np.abs(dy).T @ np.abs(x), n)
    # each output alone gives the same bits, and nothing depends on the schedule
    dx2, none = B.aeris_linear_bwd(None, tw, tdy, want_dweight=False)
    none2, dw2 = B.aeris_linear_bwd(tx, tw, tdy, want_dx=False)
    torch.cuda.synchronize()
    assert none is None and none2 is None
    assert torch.equal(dx.view(torch.int16), dx2.view(torch.int16))
    assert torch.equal(dw.view(torch.int32), dw2.view(torch.int32))


def test_linear_bwd_undoes_the_forward_pairing():
    """<dx, x> = <dW, W> = <y, dy> with y from this library's own forward projection: the three
    GEMMs (forward, dx, dW) agree with each other, not only each with the oracle."""
    rng = np.random.default_rng(77)
    n, channels, features = 2048, 256, 384
    xb, x = bf16_pair(rng.standard_normal((n, channels)))
    wb, weight = bf16_pair(rng.standard_normal((features, channels)) / 16.0)
    dyb, dy = bf16_pair(rng.standard_normal((n, features)))
    tx, tw, tdy = to_dev(xb), to_dev(wb), to_dev(dyb)
    y = B.aeris_linear_fwd(tx, tw)
    dx, dw = B.aeris_linear_bwd(tx, tw, tdy)
    torch.cuda.synchronize()
    a = float(np.sum(to_f64(dx) * x))
    b = float(np.sum(dw.double().cpu().numpy() * weight))
    c = float(np.sum(to_f64(y) * dy))
    exact = float(np.sum(bo.linear_fwd(x, weight) * dy))
    scale = float(np.sum(np.abs(bo.linear_fwd(np.abs(x), np.abs(weight))) * np.abs(dy)))
    assert abs(b - exact) <= 1e-6 * scale          # fp32 accumulation only
    assert abs(a - exact) <= 1e-4 * scale and abs(c - exact) <= 1e-4 * scale   # bf16 outputs, errors average out


def test_qkv_projection_backward_at_the_headline_size_on_samples():
    """4 x 720 x 1440 token rows, 2048 channels, 6144 features (the QKV projection of the headline
    workload, in the launch configuration bench.py times): sampled rows of dx and sampled entries
    of dW against the oracle, which needs one row of dy and the weight, or one column of dy and
    one of x."""
    n, channels, features = 4 * 720 * 1440, 2048, 6144
    gen = torch.Generator(device="cuda").manual_seed(5100)
    tx = torch.randn(n, channels, device="cuda", dtype=torch.bfloat16, generator=gen)
    tw = (torch.randn(features, channels, device="cuda", generator=gen) / channels ** 0.5).to(torch.bfloat16)
    tdy = torch.empty(n, features, device="cuda", dtype=torch.bfloat16)
    for i in range(0, n, n // 8):                       # filled in pieces: no fp32 copy of 51 GB
        tdy[i:i + n // 8] = torch.randn(n // 8, features, device="cuda", dtype=torch.bfloat16, generator=gen)
    dx, dw = B.aeris_linear_bwd(tx, tw, tdy)
    torch.cuda.synchronize()
    weight = to_f64(tw)
    rows = [0, 63, 64, 255, 256, 720 * 1440 - 1, 2 * 720 * 1440 + 12345, n - 1]
    for i in rows:
        dyi = to_f64(tdy[i:i + 1])
        ref, _ = bo.linear_bwd(np.zeros((1, channels)), weight, dyi)
        close_dx(dx[i:i + 1], ref, np.abs(dyi) @ np.abs(weight))
    entries = [(0, 0), (255, 255), (256, 256), (6143, 2047), (1000, 77), (4097, 1999), (31, 2016), (5888, 5)]
    got, ref, mag = [], [], []
    for f, c in entries:
        dcol = tdy[:, f].double().cpu().numpy()
        xcol = tx[:, c].double().cpu().numpy()
        _, r = bo.linear_bwd(xcol[:, None], np.zeros((1, 1)), dcol[:, None])
        got.append(float(dw[f, c])); ref.append(r[0, 0]); mag.append(float(np.abs(dcol) @ np.abs(xcol)))
    close_dw(np.array(got), np.array(ref), np.array(mag), n)


def test_linear_bwd_errors_are_reported():
    bf = lambda *s: torch.zeros(*s, dtype=torch.bfloat16, device="cuda")
    ws = torch.empty(1 << 20, dtype=torch.uint8, device="cuda")
    with pytest.raises(B.AerisError) as e:                       # 96 channels: not a multiple of 64
        B.aeris_linear_bwd(bf(128, 96), bf(64, 96), bf(128, 64), workspace=ws)
    assert e.value.code == -3
    with pytest.raises(B.AerisError) as e:                       # 72 features: not a multiple of 64
        B.aeris_linear_bwd(bf(128, 64), bf(72, 64), bf(128, 72), workspace=ws)
    assert e.value.code == -3
    with pytest.raises(B.AerisError) as e:                       # workspace too small
        B.aeris_linear_bwd(bf(128, 64), bf(64, 64), bf(128, 64),
                           workspace=torch.empty(256, dtype=torch.uint8, device="cuda"))
    assert e.value.code == -8
