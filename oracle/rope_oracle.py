"""fp64 CPU oracle for the axial-frequency 2-D rotary position embedding of
queries and keys in AERIS window attention.

TEST INFRASTRUCTURE ONLY.  Nothing on the product path may import this file; it
shares no code with the GPU library and imports nothing from the package.

What it computes (AERIS paper, Model Architecture section: queries and keys
pass through an axial-frequency 2-D rotary embedding, citing Heo et al. 2024,
in place of relative position biases, before the dot-product attention of a
window).  The AERIS text gives no formula; the readings taken here follow the
axial-frequency variant of the cited work:

  * the d channels of a head are d/2 pairs (x[2j], x[2j+1]); d % 4 == 0;
  * frequencies theta_t = base**(-t / (d/4)), t = 0 .. d/4-1;
  * pair j = 2t turns with the LONGITUDE position, pair j = 2t+1 with the
    LATITUDE position: angle phi_j = theta_t * position;
  * a pair is turned as a complex number:
        (a, b) -> (a cos phi - b sin phi,  a sin phi + b cos phi);
  * positions, selected by ``pos_mode`` (the paper is silent):
        POS_WINDOW  coordinates inside the attention window, in the shifted
                    frame: r = ((y - s_h) mod H) mod ws_h, c likewise;
        POS_GRID    grid coordinates (y, x);
  * ``base`` is a parameter (the paper is silent; the cited work uses 100 for
    the axial variant and 10000 is the language-model habit);
  * the backward pass treats the embedding as the linear map it is:
        dQ = R(phi)^T dQ',  i.e. the rotation by -phi.

Nothing is rounded anywhere: fp64 throughout.

Parity pins: tests/test_rope_pins.py (hand-computed angles, the complex
exponential route written with explicit loops, norm and relative-position
invariants, identity cases, inverse, torch autograd through an independent
complex-number implementation).  All functions here are pinned by those tests.
"""
import numpy as np

from . import winattn_oracle as wa

POS_WINDOW = 0
POS_GRID = 1


def positions(H, W, win, shift, pos_mode):
    """(p_lat [H,W], p_lon [H,W]) of every grid point."""
    y, x = np.meshgrid(np.arange(H), np.arange(W), indexing="ij")
    if pos_mode == POS_GRID:
        return y.astype(np.float64), x.astype(np.float64)
    if pos_mode != POS_WINDOW:
        raise ValueError("unknown position mode")
    r = ((y - shift[0]) % H) % win[0]
    c = ((x - shift[1]) % W) % win[1]
    return r.astype(np.float64), c.astype(np.float64)


def angles(H, W, d, win, shift, base, pos_mode):
    """phi[H, W, d/2]: angle of channel pair j at each grid point."""
    if d % 4:
        raise ValueError("head_dim must be a multiple of 4")
    p_lat, p_lon = positions(H, W, win, shift, pos_mode)
    n = d // 4
    theta = np.asarray(base, dtype=np.float64) ** (-np.arange(n, dtype=np.float64) / n)
    phi = np.empty((H, W, d // 2), dtype=np.float64)
    phi[:, :, 0::2] = p_lon[:, :, None] * theta          # pairs 2t:   longitude
    phi[:, :, 1::2] = p_lat[:, :, None] * theta          # pairs 2t+1: latitude
    return phi


def rotate(t, phi, inverse=False):
    """Turn the channel pairs of t [B,H,W,heads,d] by phi [H,W,d/2] (by -phi if inverse)."""
    a, b = t[..., 0::2], t[..., 1::2]
    c = np.cos(phi)[None, :, :, None, :]
    s = np.sin(phi)[None, :, :, None, :]
    if inverse:
        s = -s
    out = np.empty_like(t)
    out[..., 0::2] = a * c - b * s
    out[..., 1::2] = a * s + b * c
    return out


def winattn_rope_fwd(q, k, v, win, shift, mask, base, pos_mode, scale=None):
    """Window attention on rotated queries and keys.  Returns (O, LSE)."""
    B, H, W, nh, d = q.shape
    phi = angles(H, W, d, win, shift, base, pos_mode)
    return wa.winattn_fwd(rotate(q, phi), rotate(k, phi), v, win, shift, mask, scale)


def winattn_rope_bwd(q, k, v, do, win, shift, mask, base, pos_mode, scale=None):
    """Gradients with respect to the UNROTATED q, k (and v).  Returns (dQ, dK, dV)."""
    B, H, W, nh, d = q.shape
    phi = angles(H, W, d, win, shift, base, pos_mode)
    dq_r, dk_r, dv, _ = wa.winattn_bwd(rotate(q, phi), rotate(k, phi), v, do, win, shift, mask,
                                       scale)
    return rotate(dq_r, phi, inverse=True), rotate(dk_r, phi, inverse=True), dv
