"""fp64 CPU oracle for the element-wise operations that surround the window
attention inside an AERIS transformer layer: pre-RMSNorm with adaptive
modulation, the gated residual connection, and the SwiGLU gate.

TEST INFRASTRUCTURE ONLY.  Nothing on the product path may import this file; it
shares no code with the GPU library and imports nothing from the package.

What it computes (AERIS paper, Model Architecture section).  Every transformer
layer normalises its input with a pre-RMSNorm (Zhang & Sennrich 2019) in place
of LayerNorm, its fully connected part is a SwiGLU (Shazeer 2020), and a
layer-specific linear map of the diffusion-time embedding supplies the values
alpha, beta, gamma of an adaptive layer norm (Perez et al. 2018; Peebles & Xie
2023).  The AERIS text prints none of the formulas; the readings taken here are
the ones of the cited works:

  * RMSNorm over the C channels of a token:
        r = (mean_c x_c^2 + eps)^(-1/2),   n_c = x_c r,   y_c = n_c w_c;
  * adaptive modulation with per-sample vectors (one diffusion time per sample,
    so all tokens of a sample share them), in the scale/shift form of the
    diffusion-transformer work:
        h_c = y_c (1 + gamma_{b,c}) + beta_{b,c};
  * the branch output (attention or SwiGLU, after its output projection) is
    gated by alpha before it joins the residual stream:
        out_c = x_c + alpha_{b,c} branch_c;
  * SwiGLU gate on the packed up-projection uv = [u | v] (u = first F columns):
        g_f = silu(u_f) v_f,   silu(u) = u / (1 + exp(-u)).

  * the branches' input projections act on the normalised, modulated rows
    (the paper: RMSNorm precedes the projection of queries, keys and values,
    and the fully connected part): with a weight W [F, C] (one row per output
    feature, as a linear layer stores it)
        y_f = sum_c h_c W_{f,c};
    the SwiGLU up-projection has 2F' rows, the first F' giving u, the rest v.

Rows are tokens; the sample of row i is i // rows_per_sample.  The backward
functions are the exact derivatives of these maps (sums over the tokens of a
sample for gamma, beta, alpha; over all tokens for w).

Parity pins: tests/test_block_pins.py (hand-computed rows, unit-RMS and scale
invariance, the identity silu(u) - silu(-u) = u, limits, central finite
differences of the forward maps in fp64, and torch autograd through separately
written forward expressions).  All functions here are pinned by those tests.
"""
import numpy as np


def _sample_of_row(n_rows, rows_per_sample):
    if rows_per_sample <= 0 or n_rows % rows_per_sample:
        raise ValueError("rows must be a whole number of samples")
    return np.arange(n_rows) // rows_per_sample


def rmsnorm_adaln_fwd(x, w, gamma, beta, eps, rows_per_sample):
    """x [N, C], w [C], gamma/beta [B, C] -> (h [N, C], r [N])."""
    x = np.asarray(x, dtype=np.float64)
    b = _sample_of_row(x.shape[0], rows_per_sample)
    r = 1.0 / np.sqrt(np.mean(x * x, axis=1) + eps)
    n = x * r[:, None]
    h = n * w[None, :] * (1.0 + gamma[b]) + beta[b]
    return h, r


def rmsnorm_adaln_bwd(x, w, gamma, beta, eps, rows_per_sample, dh):
    """Gradients of sum(h * dh_const): (dx [N,C], dw [C], dgamma [B,C], dbeta [B,C])."""
    x = np.asarray(x, dtype=np.float64)
    dh = np.asarray(dh, dtype=np.float64)
    n_rows, n_ch = x.shape
    n_samples = n_rows // rows_per_sample
    b = _sample_of_row(n_rows, rows_per_sample)
    r = 1.0 / np.sqrt(np.mean(x * x, axis=1) + eps)
    n = x * r[:, None]
    s = w[None, :] * (1.0 + gamma[b])                 # d h / d n
    dn = dh * s
    # n = x r with r a function of the row: d n_c / d x_k = r (delta_ck - n_c n_k / C)
    dx = r[:, None] * (dn - n * np.mean(dn * n, axis=1, keepdims=True))
    dhn = dh * n
    dbeta = np.zeros((n_samples, n_ch))
    a = np.zeros((n_samples, n_ch))                    # sum over a sample's tokens of dh * n
    for smp in range(n_samples):
        rows = slice(smp * rows_per_sample, (smp + 1) * rows_per_sample)
        dbeta[smp] = dh[rows].sum(axis=0)
        a[smp] = dhn[rows].sum(axis=0)
    dgamma = a * w[None, :]
    dw = (a * (1.0 + gamma)).sum(axis=0)
    return dx, dw, dgamma, dbeta


def rmsnorm_adaln_bwd_residual(x, w, gamma, beta, eps, rows_per_sample, dh, dres):
    """The same for a layer out = x + branch(h(x)): x also receives the gradient dres that
    arrives along the residual path (the chain rule adds the two paths)."""
    dx, dw, dgamma, dbeta = rmsnorm_adaln_bwd(x, w, gamma, beta, eps, rows_per_sample, dh)
    return dx + np.asarray(dres, dtype=np.float64), dw, dgamma, dbeta


def gate_residual_fwd(x, y, alpha, rows_per_sample):
    """out = x + alpha_b * y."""
    x = np.asarray(x, dtype=np.float64)
    b = _sample_of_row(x.shape[0], rows_per_sample)
    return x + alpha[b] * np.asarray(y, dtype=np.float64)


def gate_residual_bwd(y, alpha, dout, rows_per_sample):
    """(dx, dy, dalpha [B, C]) for out = x + alpha_b * y."""
    y = np.asarray(y, dtype=np.float64)
    dout = np.asarray(dout, dtype=np.float64)
    n_rows, n_ch = y.shape
    n_samples = n_rows // rows_per_sample
    b = _sample_of_row(n_rows, rows_per_sample)
    dy = alpha[b] * dout
    prod = dout * y
    dalpha = np.zeros((n_samples, n_ch))
    for smp in range(n_samples):
        dalpha[smp] = prod[smp * rows_per_sample:(smp + 1) * rows_per_sample].sum(axis=0)
    return dout.copy(), dy, dalpha


def _sigmoid(u):
    # 1 / (1 + exp(-u)) without overflow for large negative u
    e = np.exp(-np.abs(u))
    return np.where(u >= 0, 1.0 / (1.0 + e), e / (1.0 + e))


def swiglu_fwd(uv):
    """uv [N, 2F] = [u | v] -> g [N, F] = silu(u) * v."""
    uv = np.asarray(uv, dtype=np.float64)
    f = uv.shape[1] // 2
    if uv.shape[1] != 2 * f:
        raise ValueError("packed width must be even")
    u, v = uv[:, :f], uv[:, f:]
    return u * _sigmoid(u) * v


def swiglu_bwd(uv, dg):
    """d uv [N, 2F] for g = silu(u) * v."""
    uv = np.asarray(uv, dtype=np.float64)
    dg = np.asarray(dg, dtype=np.float64)
    f = uv.shape[1] // 2
    u, v = uv[:, :f], uv[:, f:]
    sg = _sigmoid(u)
    dsilu = sg * (1.0 + u * (1.0 - sg))                # d silu / d u
    return np.concatenate([dg * v * dsilu, dg * u * sg], axis=1)


def linear_fwd(x, weight):
    """y [N, F] = x [N, C] W^T for W [F, C] (the output projection of a branch)."""
    x = np.asarray(x, dtype=np.float64)
    weight = np.asarray(weight, dtype=np.float64)
    if weight.ndim != 2 or weight.shape[1] != x.shape[1]:
        raise ValueError("weight must be [out_features, channels]")
    return x @ weight.T


def linear_bwd(x, weight, dy):
    """Gradients of y = x W^T (the chain rule on a bilinear map):
    dx [N, C] = dy W,   dW [F, C] = dy^T x   for dy [N, F]."""
    x = np.asarray(x, dtype=np.float64)
    weight = np.asarray(weight, dtype=np.float64)
    dy = np.asarray(dy, dtype=np.float64)
    if weight.ndim != 2 or weight.shape[1] != x.shape[1] or dy.shape != (x.shape[0], weight.shape[0]):
        raise ValueError("x [N, C], weight [F, C] and dy [N, F] do not fit")
    return dy @ weight, dy.T @ x


def norm_linear_fwd(x, w, gamma, beta, eps, rows_per_sample, weight):
    """Projection of the normalised, modulated rows: y = h W^T, h as in rmsnorm_adaln_fwd."""
    h, _ = rmsnorm_adaln_fwd(x, w, gamma, beta, eps, rows_per_sample)
    return linear_fwd(h, weight)


def norm_linear_swiglu_fwd(x, w, gamma, beta, eps, rows_per_sample, weight):
    """SwiGLU up-projection of the normalised, modulated rows and its gate:
    uv = h W^T with W [2F, C] = [u rows ; v rows];  returns (g [N, F], uv [N, 2F])."""
    uv = norm_linear_fwd(x, w, gamma, beta, eps, rows_per_sample, weight)
    return swiglu_fwd(uv), uv
