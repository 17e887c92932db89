"""fp64 CPU oracle for AERIS shifted-window multi-head self-attention.

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
HIP kernels are checked against.  Nothing on the product path may import it;
it shares no code with the GPU library and imports nothing from the package.

What it computes (AERIS paper, Model Architecture section: the embedded image
is partitioned into non-overlapping square windows, the window grid is shifted
on alternating layers, and ordinary multi-head dot-product attention runs
inside each window; SWiPe section, Overview: windows are disjoint and need no
halo).  The paper is silent on the shift amount/direction, on wrapping and on
a boundary mask; the readings taken here are

  * the shifted frame is the field rolled by -shift on both axes (cyclic),
    i.e. window (wy, wx), local token (r, c) sits at grid point
        y = (wy*ws_h + r + s_h) mod H,   x = (wx*ws_w + c + s_w) mod W
    (Fig. 2a, right panel: the shifted grid overhangs the image top-left);
  * three mask policies, selected by ``mask``:
        NONE  no mask (pure periodic wrap),
        LAT   keys are visible only within the same latitude region (the
              longitude seam is physically periodic on the globe, the
              pole-to-pole seam is not),
        SWIN  the masked shifted-window attention of the Swin paper the
              authors cite: latitude and longitude regions both separate.
    Regions are defined in the shifted frame: along an axis of length L with
    window side ws and shift s, coordinate u-hat is in region 0 if
    u-hat < L-ws, region 1 if L-ws <= u-hat < L-s, region 2 otherwise;
  * masked logits are excluded exactly (weight zero);
  * softmax scale defaults to 1/sqrt(head_dim); natural-log LSE.

Every array is float64.  Callers widen the bf16 input bits to float64 first,
so the oracle and the GPU see identical operands.  There is no tiling, no
running maximum carried across blocks, no fusion: one window and one head at a
time, the textbook formulas in order.

Parity pins: tests/test_oracle_pins.py (brute-force scalar loops on tiny
grids, global attention through torch autograd, roll and permutation
equivariance, closed forms, invariants, finite differences, mask-pair counts).
All functions here are pinned by those tests.
"""
import numpy as np

MASK_NONE = 0
MASK_LAT = 1
MASK_SWIN = 2


def axis_region(u_hat, L, ws, s):
    """Region id (0, 1 or 2) of shifted-frame coordinates ``u_hat`` on one axis."""
    u_hat = np.asarray(u_hat)
    rho = np.zeros(u_hat.shape, dtype=np.int64)
    rho[u_hat >= L - ws] = 1
    rho[u_hat >= L - s] = 2
    return rho


def window_tokens(H, W, win, shift, wy, wx):
    """Grid coordinates and shifted-frame coordinates of one window's tokens.

    Returns (y, x, y_hat, x_hat), each of shape [T] with T = ws_h*ws_w, the
    token order being row-major in the window (r major, c minor).
    """
    ws_h, ws_w = win
    s_h, s_w = shift
    r, c = np.meshgrid(np.arange(ws_h), np.arange(ws_w), indexing="ij")
    y_hat = (wy * ws_h + r).reshape(-1)
    x_hat = (wx * ws_w + c).reshape(-1)
    y = (y_hat + s_h) % H
    x = (x_hat + s_w) % W
    return y, x, y_hat, x_hat


def token_regions(H, W, win, shift, mask, y_hat, x_hat):
    """Region id per token under a mask policy (tokens attend only within equal ids)."""
    if mask == MASK_NONE:
        return np.zeros(y_hat.shape, dtype=np.int64)
    rho_y = axis_region(y_hat, H, win[0], shift[0])
    if mask == MASK_LAT:
        return rho_y
    if mask == MASK_SWIN:
        rho_x = axis_region(x_hat, W, win[1], shift[1])
        return 3 * rho_y + rho_x
    raise ValueError("unknown mask policy %r" % (mask,))


def _check(q, k, v, win, shift):
    if q.ndim != 5 or q.shape != k.shape or q.shape != v.shape:
        raise ValueError("q, k, v must share a [B,H,W,heads,d] shape")
    B, H, W, nh, d = q.shape
    if H % win[0] or W % win[1]:
        raise ValueError("window must divide the grid")
    if not (0 <= shift[0] < win[0] and 0 <= shift[1] < win[1]):
        raise ValueError("need 0 <= shift < window")
    return B, H, W, nh, d


def window_pair_fwd(qw, kw, vw, reg, scale):
    """Attention of one (batch, window, head): qw,kw,vw are [T,d], reg is [T].

    Returns (O [T,d], LSE [T], P [T,T]).
    """
    S = scale * (qw @ kw.T)                                  # logits
    allowed = reg[:, None] == reg[None, :]
    S = np.where(allowed, S, -np.inf)                        # exact exclusion
    m = S.max(axis=1, keepdims=True)                         # finite: i sees itself
    lse = m[:, 0] + np.log(np.exp(S - m).sum(axis=1))        # ln sum_j e^{S_ij}
    P = np.exp(S - lse[:, None])                             # softmax rows
    O = P @ vw
    return O, lse, P


def window_pair_bwd(qw, kw, vw, dow, reg, scale):
    """Gradients of one (batch, window, head) given dO [T,d].

    Returns (dQ, dK, dV, delta) with delta_i = sum_j P_ij dP_ij.
    """
    _, _, P = window_pair_fwd(qw, kw, vw, reg, scale)
    dV = P.T @ dow
    dP = dow @ vw.T
    delta = (P * dP).sum(axis=1)
    dS = P * (dP - delta[:, None])
    dQ = scale * (dS @ kw)
    dK = scale * (dS.T @ qw)
    return dQ, dK, dV, delta


def winattn_fwd(q, k, v, win, shift, mask=MASK_NONE, scale=None):
    """Forward over the whole grid.

    q, k, v: float64 [B, H, W, heads, d].  win=(ws_h, ws_w), shift=(s_h, s_w).
    Returns O [B, H, W, heads, d] and LSE [B, heads, H, W], both at the
    original (unshifted) grid coordinates.
    """
    B, H, W, nh, d = _check(q, k, v, win, shift)
    if scale is None:
        scale = 1.0 / np.sqrt(d)
    o = np.zeros_like(q)
    lse = np.zeros((B, nh, H, W), dtype=np.float64)
    for wy in range(H // win[0]):
        for wx in range(W // win[1]):
            y, x, y_hat, x_hat = window_tokens(H, W, win, shift, wy, wx)
            reg = token_regions(H, W, win, shift, mask, y_hat, x_hat)
            for b in range(B):
                for h in range(nh):
                    O, l, _ = window_pair_fwd(q[b, y, x, h], k[b, y, x, h],
                                              v[b, y, x, h], reg, scale)
                    o[b, y, x, h] = O
                    lse[b, h, y, x] = l
    return o, lse


def winattn_bwd(q, k, v, do, win, shift, mask=MASK_NONE, scale=None):
    """Backward over the whole grid: returns dQ, dK, dV ([B,H,W,heads,d]) and
    delta [B, heads, H, W]."""
    B, H, W, nh, d = _check(q, k, v, win, shift)
    if do.shape != q.shape:
        raise ValueError("dO must have the shape of Q")
    if scale is None:
        scale = 1.0 / np.sqrt(d)
    dq = np.zeros_like(q)
    dk = np.zeros_like(q)
    dv = np.zeros_like(q)
    delta = np.zeros((B, nh, H, W), dtype=np.float64)
    for wy in range(H // win[0]):
        for wx in range(W // win[1]):
            y, x, y_hat, x_hat = window_tokens(H, W, win, shift, wy, wx)
            reg = token_regions(H, W, win, shift, mask, y_hat, x_hat)
            for b in range(B):
                for h in range(nh):
                    dQ, dK, dV, dl = window_pair_bwd(q[b, y, x, h], k[b, y, x, h],
                                                     v[b, y, x, h], do[b, y, x, h],
                                                     reg, scale)
                    dq[b, y, x, h] = dQ
                    dk[b, y, x, h] = dK
                    dv[b, y, x, h] = dV
                    delta[b, h, y, x] = dl
    return dq, dk, dv, delta


def winattn_pair(qs, ks, vs, dos, H, W, win, shift, mask, scale, wy, wx):
    """One sampled (batch, window, head) of a grid too large to run whole.

    qs, ks, vs (and dos, or None) are the [H, W, d] float64 slices of one batch
    member and head.  Returns a dict with the window's grid coordinates y, x
    and O, LSE (and dQ, dK, dV, delta when dos is given), each indexed by
    window-local token.
    """
    d = qs.shape[-1]
    if scale is None:
        scale = 1.0 / np.sqrt(d)
    y, x, y_hat, x_hat = window_tokens(H, W, win, shift, wy, wx)
    reg = token_regions(H, W, win, shift, mask, y_hat, x_hat)
    O, l, _ = window_pair_fwd(qs[y, x], ks[y, x], vs[y, x], reg, scale)
    out = {"y": y, "x": x, "o": O, "lse": l}
    if dos is not None:
        dQ, dK, dV, dl = window_pair_bwd(qs[y, x], ks[y, x], vs[y, x], dos[y, x],
                                         reg, scale)
        out.update(dq=dQ, dk=dK, dv=dV, delta=dl)
    return out


def unmasked_pairs(H, W, win, shift, mask):
    """Number of (query, key) pairs with non-zero weight, summed over the
    windows of one grid (per batch member and head)."""
    total = 0
    for wy in range(H // win[0]):
        for wx in range(W // win[1]):
            _, _, y_hat, x_hat = window_tokens(H, W, win, shift, wy, wx)
            reg = token_regions(H, W, win, shift, mask, y_hat, x_hat)
            total += int((reg[:, None] == reg[None, :]).sum())
    return total
