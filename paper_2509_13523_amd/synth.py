"""Seeded synthetic inputs shared by the tests, the benchmark and the smoke run.

Holds no attention arithmetic: only random draws, smooth large-scale fields
that imitate the structure of gridded atmospheric data (the paper's 0.25-degree
ERA5 fields are not available), and the bf16 <-> float conversions that define
the exchanged bit patterns.  Both the GPU binding and the CPU oracle's tests
read their operands from here, as raw bf16 bits, so they see identical values.
"""
import numpy as np


# ----------------------------------------------------------------------------
# bf16 bit patterns (numpy has no bfloat16 dtype: uint16 carries the bits)
# ----------------------------------------------------------------------------
def f32_to_bf16_bits(a):
    """Round float32 -> bf16 (round to nearest even), returned as uint16 bits."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    rounding = ((u >> 16) & 1) + np.uint32(0x7FFF)
    return ((u + rounding) >> 16).astype(np.uint16)


def bf16_bits_to_f64(bits):
    """Widen bf16 bit patterns (uint16) exactly to float64."""
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def bf16_bits_to_f32(bits):
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    return (bits.astype(np.uint32) << 16).view(np.float32)


# ----------------------------------------------------------------------------
# value recipes
# ----------------------------------------------------------------------------
def normal_field(seed, shape):
    """i.i.d. N(0,1), float32."""
    return np.random.default_rng(seed).standard_normal(shape, dtype=np.float32)


def smooth_field(seed, shape, n_modes=8, noise=0.1):
    """Unit-variance sum of low-order lat/lon Fourier modes plus white noise.

    shape = [B, H, W, heads, d].  Per (batch, head, channel):
        sum_m a_m sin(2 pi (k_m y/H + l_m x/W) + phi_m),  k_m, l_m in 0..3 not
    both zero, a_m ~ N(0, 1/4) (eight modes give unit variance), phi_m uniform,
    then + noise * N(0,1).  Peaked softmax rows result, as on smooth fields.
    """
    B, H, W, nh, d = shape
    rng = np.random.default_rng(seed)
    y = np.arange(H, dtype=np.float64)[:, None] / H
    x = np.arange(W, dtype=np.float64)[None, :] / W
    out = np.empty(shape, dtype=np.float32)
    for b in range(B):
        for h in range(nh):
            k = rng.integers(0, 4, size=(n_modes, d))
            l = rng.integers(0, 4, size=(n_modes, d))
            both_zero = (k == 0) & (l == 0)
            k = np.where(both_zero, 1, k)
            a = rng.normal(0.0, 0.5, size=(n_modes, d))
            phi = rng.uniform(0.0, 2.0 * np.pi, size=(n_modes, d))
            acc = np.zeros((H, W, d), dtype=np.float64)
            for m in range(n_modes):
                phase = 2.0 * np.pi * (k[m][None, None, :] * y[:, :, None]
                                       + l[m][None, None, :] * x[:, :, None])
                acc += a[m][None, None, :] * np.sin(phase + phi[m][None, None, :])
            out[b, :, :, h, :] = acc.astype(np.float32)
    if noise:
        out += noise * rng.standard_normal(shape, dtype=np.float32)
    return out


def blend_field(seed, shape, sigma):
    """(1 - sigma) * smooth + sigma * N(0,1): a diffusion-style noisy member."""
    return ((1.0 - sigma) * smooth_field(seed, shape, noise=0.0)
            + sigma * normal_field(seed + 7919, shape)).astype(np.float32)


def make_inputs(kind, seed, shape, n_tensors=4, sigma=0.5):
    """n_tensors bf16-bit arrays (uint16) of ``shape``: Q, K, V, dO in that order.

    kind: "normal" | "smooth" | "blend".  Tensor i uses seed + i.
    """
    outs = []
    for i in range(n_tensors):
        if kind == "normal":
            a = normal_field(seed + i, shape)
        elif kind == "smooth":
            a = smooth_field(seed + i, shape)
        elif kind == "blend":
            a = blend_field(seed + i, shape, sigma)
        else:
            raise ValueError("unknown input kind %r" % (kind,))
        outs.append(f32_to_bf16_bits(a))
    return outs


# ----------------------------------------------------------------------------
# on-device generation for grids too large for host memory (torch is plumbing)
# ----------------------------------------------------------------------------
def make_inputs_device(kind, seed, shape, n_tensors=4, sigmas=None, device="cuda"):
    """Same recipes drawn with torch on the device; returns torch.bfloat16 tensors.

    ``sigmas`` (one per batch member) selects the per-member blend of the
    diffusion-ensemble workload; None means sigma = 0.5 for "blend".
    The oracle reads these very bits back from the device for its samples.
    """
    import torch
    B, H, W, nh, d = shape
    g = torch.Generator(device=device)
    outs = []
    for i in range(n_tensors):
        g.manual_seed(seed + i)
        t = torch.empty(shape, dtype=torch.bfloat16, device=device)
        for b in range(B):
            if kind == "normal":
                t[b] = torch.randn((H, W, nh, d), generator=g, device=device,
                                   dtype=torch.float32).to(torch.bfloat16)
                continue
            sig = 0.5 if sigmas is None else float(sigmas[b])
            if kind == "smooth":
                sig_noise, sig_smooth = 0.1, 1.0
            else:
                sig_noise, sig_smooth = sig, 1.0 - sig
            yy = torch.arange(H, device=device, dtype=torch.float32)[:, None, None, None] / H
            xx = torch.arange(W, device=device, dtype=torch.float32)[None, :, None, None] / W
            acc = torch.zeros((H, W, nh, d), device=device, dtype=torch.float32)
            for _ in range(8):
                kk = torch.randint(0, 4, (nh, d), generator=g, device=device)
                ll = torch.randint(0, 4, (nh, d), generator=g, device=device)
                kk = torch.where((kk == 0) & (ll == 0), torch.ones_like(kk), kk)
                aa = 0.5 * torch.randn((nh, d), generator=g, device=device)
                ph = 2.0 * torch.pi * torch.rand((nh, d), generator=g, device=device)
                acc += aa * torch.sin(2.0 * torch.pi * (kk * yy + ll * xx) + ph)
            acc *= sig_smooth
            acc += sig_noise * torch.randn((H, W, nh, d), generator=g, device=device,
                                           dtype=torch.float32)
            t[b] = acc.to(torch.bfloat16)
            del acc
        outs.append(t)
    return outs
