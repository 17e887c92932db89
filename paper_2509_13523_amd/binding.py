"""ctypes binding of libaeris_winattn.so: same names as the C entry points.

Argument marshalling only.  PyTorch supplies device memory and the current HIP
stream; every step of the computation runs in the library's kernels.  There is
no fallback: if the library is missing or a call fails, an exception is raised.
"""
import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libaeris_winattn.so")

AERIS_MASK_NONE, AERIS_MASK_LAT, AERIS_MASK_SWIN = 0, 1, 2
AERIS_DT_BF16, AERIS_DT_F32 = 0, 1
AERIS_BWD_DELTA, AERIS_BWD_DQ, AERIS_BWD_DKDV, AERIS_BWD_ALL = 1, 2, 4, 7
AERIS_ROPE_POS_WINDOW, AERIS_ROPE_POS_GRID = 0, 1
AERIS_BWD_STATIC_SCRATCH_BYTES = 64 << 20

EXPORTS = ("aeris_winattn_fwd", "aeris_winattn_bwd", "aeris_winattn_bwd_stages",
           "aeris_winattn_bwd_workspace_bytes", "aeris_winattn_bwd_static",
           "aeris_winattn_validate", "aeris_winattn_strerror", "aeris_winattn_version",
           "aeris_winattn_fwd_windows", "aeris_winattn_bwd_windows",
           "aeris_mfma_loop_probe", "aeris_rope2d_apply", "aeris_winattn_rope_fwd_workspace_bytes",
           "aeris_winattn_rope_bwd_workspace_bytes", "aeris_winattn_rope_fwd",
           "aeris_winattn_rope_bwd", "aeris_winattn_rope_fwd_windows",
           "aeris_winattn_rope_bwd_windows",
           # include/aeris_layer_ops.h
           "aeris_rmsnorm_adaln_fwd", "aeris_rmsnorm_adaln_bwd_workspace_bytes",
           "aeris_rmsnorm_adaln_bwd", "aeris_rmsnorm_adaln_bwd_residual", "aeris_gate_residual_fwd",
           "aeris_gate_residual_bwd_workspace_bytes", "aeris_gate_residual_bwd",
           "aeris_swiglu_fwd", "aeris_swiglu_bwd", "aeris_norm_linear_workspace_bytes",
           "aeris_norm_linear_fwd", "aeris_norm_linear_swiglu_fwd", "aeris_linear_fwd",
           "aeris_linear_bwd_workspace_bytes", "aeris_linear_bwd")


class aeris_winattn_params(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int32), ("H_lat", ctypes.c_int32), ("W_lon", ctypes.c_int32),
                ("heads", ctypes.c_int32), ("head_dim", ctypes.c_int32),
                ("win_h", ctypes.c_int32), ("win_w", ctypes.c_int32),
                ("shift_h", ctypes.c_int32), ("shift_w", ctypes.c_int32),
                ("mask_policy", ctypes.c_int32), ("softmax_scale", ctypes.c_float),
                ("out_dtype", ctypes.c_int32),
                ("qkv_tok_stride", ctypes.c_int64), ("qkv_head_stride", ctypes.c_int64),
                ("o_tok_stride", ctypes.c_int64), ("o_head_stride", ctypes.c_int64)]


class aeris_rope_params(ctypes.Structure):
    _fields_ = [("base", ctypes.c_float), ("positions", ctypes.c_int32)]


class AerisError(RuntimeError):
    def __init__(self, code, where):
        self.code = code
        super().__init__("%s failed: %d (%s)" % (where, code, aeris_winattn_strerror(code)))


_lib = None


def load():
    """Load the shared library (once).  Raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError("libaeris_winattn.so is not built: run "
                          "`python -c 'import __graft_entry__ as g; g.build()'` "
                          "(expected at %s)" % LIB_PATH)
    lib = ctypes.CDLL(LIB_PATH)
    P = ctypes.POINTER(aeris_winattn_params)
    vp = ctypes.c_void_p
    lib.aeris_winattn_fwd.argtypes = [P, vp, vp, vp, vp, vp, vp]
    lib.aeris_winattn_fwd.restype = ctypes.c_int
    lib.aeris_winattn_bwd.argtypes = [P, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp,
                                      ctypes.c_size_t, vp]
    lib.aeris_winattn_bwd.restype = ctypes.c_int
    lib.aeris_winattn_bwd_static.argtypes = [P, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp]
    lib.aeris_winattn_bwd_static.restype = ctypes.c_int
    lib.aeris_winattn_bwd_stages.argtypes = [P, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp,
                                             ctypes.c_size_t, vp, ctypes.c_uint]
    lib.aeris_winattn_bwd_stages.restype = ctypes.c_int
    lib.aeris_winattn_bwd_workspace_bytes.argtypes = [P]
    lib.aeris_winattn_bwd_workspace_bytes.restype = ctypes.c_size_t
    lib.aeris_winattn_validate.argtypes = [P]
    lib.aeris_winattn_validate.restype = ctypes.c_int
    lib.aeris_winattn_strerror.argtypes = [ctypes.c_int]
    lib.aeris_winattn_strerror.restype = ctypes.c_char_p
    lib.aeris_winattn_version.argtypes = []
    lib.aeris_winattn_version.restype = ctypes.c_int
    lib.aeris_winattn_fwd_windows.argtypes = [P, vp, ctypes.c_int32, vp, vp, vp, vp, vp, vp]
    lib.aeris_winattn_fwd_windows.restype = ctypes.c_int
    lib.aeris_winattn_bwd_windows.argtypes = [P, vp, ctypes.c_int32, vp, vp, vp, vp, vp, vp, vp, vp,
                                              vp, vp, ctypes.c_size_t, vp]
    lib.aeris_winattn_bwd_windows.restype = ctypes.c_int
    lib.aeris_mfma_loop_probe.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, vp, vp]
    lib.aeris_mfma_loop_probe.restype = ctypes.c_int
    R = ctypes.POINTER(aeris_rope_params)
    lib.aeris_rope2d_apply.argtypes = [P, R, vp, vp, ctypes.c_int32, vp]
    lib.aeris_rope2d_apply.restype = ctypes.c_int
    lib.aeris_winattn_rope_fwd_workspace_bytes.argtypes = [P]
    lib.aeris_winattn_rope_fwd_workspace_bytes.restype = ctypes.c_size_t
    lib.aeris_winattn_rope_bwd_workspace_bytes.argtypes = [P]
    lib.aeris_winattn_rope_bwd_workspace_bytes.restype = ctypes.c_size_t
    lib.aeris_winattn_rope_fwd.argtypes = [P, R, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
    lib.aeris_winattn_rope_fwd.restype = ctypes.c_int
    lib.aeris_winattn_rope_bwd.argtypes = [P, R, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp,
                                           ctypes.c_size_t, vp]
    lib.aeris_winattn_rope_bwd.restype = ctypes.c_int
    lib.aeris_winattn_rope_fwd_windows.argtypes = [P, R, vp, ctypes.c_int32, vp, vp, vp, vp, vp, vp,
                                                   ctypes.c_size_t, vp]
    lib.aeris_winattn_rope_fwd_windows.restype = ctypes.c_int
    lib.aeris_winattn_rope_bwd_windows.argtypes = [P, R, vp, ctypes.c_int32, vp, vp, vp, vp, vp, vp, vp,
                                                   vp, vp, vp, vp, ctypes.c_size_t, vp]
    lib.aeris_winattn_rope_bwd_windows.restype = ctypes.c_int
    i64, i32, f32, sz = ctypes.c_int64, ctypes.c_int32, ctypes.c_float, ctypes.c_size_t
    lib.aeris_rmsnorm_adaln_fwd.argtypes = [vp, vp, vp, vp, f32, i64, i64, i32, vp, vp, vp]
    lib.aeris_rmsnorm_adaln_fwd.restype = ctypes.c_int
    lib.aeris_rmsnorm_adaln_bwd_workspace_bytes.argtypes = [i64, i64, i32]
    lib.aeris_rmsnorm_adaln_bwd_workspace_bytes.restype = sz
    lib.aeris_rmsnorm_adaln_bwd.argtypes = [vp, vp, vp, vp, vp, i64, i64, i32, vp, vp, vp, vp,
                                            vp, sz, vp]
    lib.aeris_rmsnorm_adaln_bwd.restype = ctypes.c_int
    lib.aeris_rmsnorm_adaln_bwd_residual.argtypes = [vp, vp, vp, vp, vp, vp, i64, i64, i32, vp, vp,
                                                     vp, vp, vp, sz, vp]
    lib.aeris_rmsnorm_adaln_bwd_residual.restype = ctypes.c_int
    lib.aeris_gate_residual_fwd.argtypes = [vp, vp, vp, i64, i64, i32, vp, vp]
    lib.aeris_gate_residual_fwd.restype = ctypes.c_int
    lib.aeris_gate_residual_bwd_workspace_bytes.argtypes = [i64, i64, i32]
    lib.aeris_gate_residual_bwd_workspace_bytes.restype = sz
    lib.aeris_gate_residual_bwd.argtypes = [vp, vp, vp, i64, i64, i32, vp, vp, vp, sz, vp]
    lib.aeris_gate_residual_bwd.restype = ctypes.c_int
    lib.aeris_swiglu_fwd.argtypes = [vp, i64, i32, vp, vp]
    lib.aeris_swiglu_fwd.restype = ctypes.c_int
    lib.aeris_swiglu_bwd.argtypes = [vp, vp, i64, i32, vp, vp]
    lib.aeris_swiglu_bwd.restype = ctypes.c_int
    lib.aeris_norm_linear_workspace_bytes.argtypes = [i64, i64, i32, i32]
    lib.aeris_norm_linear_workspace_bytes.restype = sz
    lib.aeris_norm_linear_fwd.argtypes = [vp, vp, vp, vp, f32, vp, i64, i64, i32, i32, vp, vp, sz, vp]
    lib.aeris_norm_linear_fwd.restype = ctypes.c_int
    lib.aeris_norm_linear_swiglu_fwd.argtypes = [vp, vp, vp, vp, f32, vp, i64, i64, i32, i32, vp, vp,
                                                 vp, sz, vp]
    lib.aeris_norm_linear_swiglu_fwd.restype = ctypes.c_int
    lib.aeris_linear_fwd.argtypes = [vp, vp, i64, i32, i32, vp, vp]
    lib.aeris_linear_fwd.restype = ctypes.c_int
    lib.aeris_linear_bwd_workspace_bytes.argtypes = [i64, i32, i32]
    lib.aeris_linear_bwd_workspace_bytes.restype = sz
    lib.aeris_linear_bwd.argtypes = [vp, vp, vp, i64, i32, i32, vp, vp, vp, sz, vp]
    lib.aeris_linear_bwd.restype = ctypes.c_int
    _lib = lib
    return lib


def make_params(shape, win, shift, mask=AERIS_MASK_NONE, scale=0.0, out_dtype=AERIS_DT_BF16,
                qkv_strides=(0, 0), o_strides=(0, 0)):
    B, H, W, nh, d = shape
    return aeris_winattn_params(B, H, W, nh, d, win[0], win[1], shift[0], shift[1], mask,
                                float(scale or 0.0), out_dtype,
                                qkv_strides[0], qkv_strides[1], o_strides[0], o_strides[1])


def aeris_winattn_version():
    return load().aeris_winattn_version()


def aeris_winattn_strerror(code):
    return load().aeris_winattn_strerror(int(code)).decode()


def aeris_winattn_validate(params):
    return load().aeris_winattn_validate(ctypes.byref(params))


def aeris_winattn_bwd_workspace_bytes(params):
    return load().aeris_winattn_bwd_workspace_bytes(ctypes.byref(params))


def _stream():
    import torch
    return torch.cuda.current_stream().cuda_stream


def _torch_out_dtype(out_dtype):
    import torch
    return torch.float32 if out_dtype == AERIS_DT_F32 else torch.bfloat16


def aeris_winattn_fwd(q, k, v, win, shift, mask=AERIS_MASK_NONE, scale=None,
                      out_dtype=AERIS_DT_BF16, o=None, lse=None):
    """q, k, v: contiguous torch.bfloat16 device tensors [B,H,W,heads,d].
    Returns (o, lse); buffers are allocated with torch unless passed in."""
    import torch
    B, H, W, nh, d = q.shape
    for t in (q, k, v):
        assert t.is_cuda and t.dtype == torch.bfloat16 and t.is_contiguous() and t.shape == q.shape
    p = make_params(q.shape, win, shift, mask, scale, out_dtype)
    if o is None:
        o = torch.empty(q.shape, dtype=_torch_out_dtype(out_dtype), device=q.device)
    if lse is None:
        lse = torch.empty((B, nh, H, W), dtype=torch.float32, device=q.device)
    rc = load().aeris_winattn_fwd(ctypes.byref(p), q.data_ptr(), k.data_ptr(), v.data_ptr(),
                                  o.data_ptr(), lse.data_ptr(), _stream())
    if rc != 0:
        raise AerisError(rc, "aeris_winattn_fwd")
    return o, lse


def aeris_winattn_bwd(q, k, v, o, lse, d_o, win, shift, mask=AERIS_MASK_NONE, scale=None,
                      out_dtype=AERIS_DT_BF16, dq=None, dk=None, dv=None, workspace=None):
    """Returns (dq, dk, dv).  o must be the forward output in ``out_dtype``."""
    return aeris_winattn_bwd_stages(q, k, v, o, lse, d_o, win, shift, mask, scale, out_dtype,
                                    dq, dk, dv, workspace, AERIS_BWD_ALL)


def aeris_winattn_bwd_stages(q, k, v, o, lse, d_o, win, shift, mask=AERIS_MASK_NONE, scale=None,
                             out_dtype=AERIS_DT_BF16, dq=None, dk=None, dv=None, workspace=None,
                             stages=AERIS_BWD_ALL):
    """Subset of the backward kernels (see the header); returns (dq, dk, dv)."""
    import torch
    p = make_params(q.shape, win, shift, mask, scale, out_dtype)
    odt = _torch_out_dtype(out_dtype)
    assert o.dtype == odt and d_o.dtype == torch.bfloat16 and lse.dtype == torch.float32
    for t in (q, k, v, o, d_o, lse):
        assert t.is_cuda and t.is_contiguous()
    if dq is None:
        dq = torch.empty(q.shape, dtype=odt, device=q.device)
    if dk is None:
        dk = torch.empty(q.shape, dtype=odt, device=q.device)
    if dv is None:
        dv = torch.empty(q.shape, dtype=odt, device=q.device)
    need = aeris_winattn_bwd_workspace_bytes(p)
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=q.device)
    lib = load()
    args = (ctypes.byref(p), q.data_ptr(), k.data_ptr(), v.data_ptr(), o.data_ptr(),
            lse.data_ptr(), d_o.data_ptr(), dq.data_ptr(), dk.data_ptr(), dv.data_ptr(),
            workspace.data_ptr(), workspace.numel() * workspace.element_size(), _stream())
    if stages == AERIS_BWD_ALL:
        rc = lib.aeris_winattn_bwd(*args)
    else:
        rc = lib.aeris_winattn_bwd_stages(*args, stages)
    if rc != 0:
        raise AerisError(rc, "aeris_winattn_bwd")
    return dq, dk, dv


def aeris_winattn_bwd_static(q, k, v, o, lse, d_o, win, shift, mask=AERIS_MASK_NONE, scale=None,
                             out_dtype=AERIS_DT_BF16, dq=None, dk=None, dv=None):
    """aeris_winattn_bwd with the kernels' scratch in the library's static device array: the
    C call allocates nothing.  Pass dq, dk, dv to keep torch from allocating them here."""
    import torch
    p = make_params(q.shape, win, shift, mask, scale, out_dtype)
    odt = _torch_out_dtype(out_dtype)
    assert o.dtype == odt and d_o.dtype == torch.bfloat16 and lse.dtype == torch.float32
    for t in (q, k, v, o, d_o, lse):
        assert t.is_cuda and t.is_contiguous()
    if dq is None:
        dq = torch.empty(q.shape, dtype=odt, device=q.device)
    if dk is None:
        dk = torch.empty(q.shape, dtype=odt, device=q.device)
    if dv is None:
        dv = torch.empty(q.shape, dtype=odt, device=q.device)
    rc = load().aeris_winattn_bwd_static(ctypes.byref(p), q.data_ptr(), k.data_ptr(), v.data_ptr(),
                                         o.data_ptr(), lse.data_ptr(), d_o.data_ptr(),
                                         dq.data_ptr(), dk.data_ptr(), dv.data_ptr(), _stream())
    if rc != 0:
        raise AerisError(rc, "aeris_winattn_bwd_static")
    return dq, dk, dv


def aeris_rope2d_apply(x, win, shift, base, positions, inverse=False, y=None):
    """Rotary embedding of one contiguous bf16 [B,H,W,heads,d] device tensor; returns y."""
    import torch
    assert x.is_cuda and x.dtype == torch.bfloat16 and x.is_contiguous()
    p = make_params(x.shape, win, shift)
    r = aeris_rope_params(float(base), int(positions))
    if y is None:
        y = torch.empty_like(x)
    rc = load().aeris_rope2d_apply(ctypes.byref(p), ctypes.byref(r), x.data_ptr(), y.data_ptr(),
                                   1 if inverse else 0, _stream())
    if rc != 0:
        raise AerisError(rc, "aeris_rope2d_apply")
    return y


def aeris_winattn_rope_fwd_workspace_bytes(params):
    return load().aeris_winattn_rope_fwd_workspace_bytes(ctypes.byref(params))


def aeris_winattn_rope_bwd_workspace_bytes(params):
    return load().aeris_winattn_rope_bwd_workspace_bytes(ctypes.byref(params))


def aeris_winattn_rope_fwd(q, k, v, win, shift, base, positions, mask=AERIS_MASK_NONE, scale=None,
                           out_dtype=AERIS_DT_BF16, o=None, lse=None, workspace=None,
                           return_saved=False):
    """Attention on rotated queries and keys.  Returns (o, lse), or (o, lse, workspace) with
    return_saved: the workspace then holds the rotated k and q for aeris_winattn_rope_bwd."""
    import torch
    B, H, W, nh, d = q.shape
    for t in (q, k, v):
        assert t.is_cuda and t.dtype == torch.bfloat16 and t.is_contiguous() and t.shape == q.shape
    p = make_params(q.shape, win, shift, mask, scale, out_dtype)
    r = aeris_rope_params(float(base), int(positions))
    if o is None:
        o = torch.empty(q.shape, dtype=_torch_out_dtype(out_dtype), device=q.device)
    if lse is None:
        lse = torch.empty((B, nh, H, W), dtype=torch.float32, device=q.device)
    need = aeris_winattn_rope_fwd_workspace_bytes(p)
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=q.device)
    rc = load().aeris_winattn_rope_fwd(ctypes.byref(p), ctypes.byref(r), q.data_ptr(),
                                       k.data_ptr(), v.data_ptr(), o.data_ptr(), lse.data_ptr(),
                                       workspace.data_ptr(), workspace.numel(), _stream())
    if rc != 0:
        raise AerisError(rc, "aeris_winattn_rope_fwd")
    return (o, lse, workspace) if return_saved else (o, lse)


def aeris_winattn_rope_bwd(q, k, v, o, lse, d_o, win, shift, base, positions,
                           mask=AERIS_MASK_NONE, scale=None, out_dtype=AERIS_DT_BF16,
                           workspace=None, saved=None, dq=None, dk=None, dv=None):
    """Gradients with respect to the unrotated q, k and v.  Returns (dq, dk, dv).  saved: the
    workspace of the matching forward call (nothing is rotated again)."""
    import torch
    p = make_params(q.shape, win, shift, mask, scale, out_dtype)
    r = aeris_rope_params(float(base), int(positions))
    odt = _torch_out_dtype(out_dtype)
    assert o.dtype == odt and d_o.dtype == torch.bfloat16 and lse.dtype == torch.float32
    for t in (q, k, v, o, d_o, lse):
        assert t.is_cuda and t.is_contiguous()
    dq, dk, dv = [torch.empty(q.shape, dtype=odt, device=q.device) if t is None else t
                  for t in (dq, dk, dv)]
    need = (aeris_winattn_rope_bwd_workspace_bytes(p) if saved is None
            else aeris_winattn_bwd_workspace_bytes(p))
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=q.device)
    rc = load().aeris_winattn_rope_bwd(ctypes.byref(p), ctypes.byref(r), q.data_ptr(),
                                       k.data_ptr(), v.data_ptr(), o.data_ptr(), lse.data_ptr(),
                                       d_o.data_ptr(), dq.data_ptr(), dk.data_ptr(),
                                       dv.data_ptr(), None if saved is None else saved.data_ptr(),
                                       workspace.data_ptr(), workspace.numel(), _stream())
    if rc != 0:
        raise AerisError(rc, "aeris_winattn_rope_bwd")
    return dq, dk, dv


def aeris_winattn_fwd_windows(q, k, v, win, shift, windows, o, lse, mask=AERIS_MASK_NONE,
                              scale=None, out_dtype=AERIS_DT_BF16):
    """Forward over the listed windows only.  windows: int32 device tensor of indices
    wy * (W/win_w) + wx; o and lse are caller-provided and written only inside those windows."""
    import torch
    assert windows.is_cuda and windows.dtype == torch.int32 and windows.is_contiguous()
    for t in (q, k, v):
        assert t.is_cuda and t.dtype == torch.bfloat16 and t.is_contiguous() and t.shape == q.shape
    p = make_params(q.shape, win, shift, mask, scale, out_dtype)
    rc = load().aeris_winattn_fwd_windows(ctypes.byref(p), windows.data_ptr(), windows.numel(),
                                          q.data_ptr(), k.data_ptr(), v.data_ptr(), o.data_ptr(),
                                          lse.data_ptr(), _stream())
    if rc != 0:
        raise AerisError(rc, "aeris_winattn_fwd_windows")
    return o, lse


def aeris_winattn_bwd_windows(q, k, v, o, lse, d_o, win, shift, windows, dq, dk, dv,
                              mask=AERIS_MASK_NONE, scale=None, out_dtype=AERIS_DT_BF16,
                              workspace=None):
    """Backward over the listed windows only; dq, dk, dv are written only inside them."""
    import torch
    assert windows.is_cuda and windows.dtype == torch.int32 and windows.is_contiguous()
    p = make_params(q.shape, win, shift, mask, scale, out_dtype)
    if workspace is None:
        workspace = torch.empty(aeris_winattn_bwd_workspace_bytes(p), dtype=torch.uint8,
                                device=q.device)
    rc = load().aeris_winattn_bwd_windows(ctypes.byref(p), windows.data_ptr(), windows.numel(),
                                          q.data_ptr(), k.data_ptr(), v.data_ptr(), o.data_ptr(),
                                          lse.data_ptr(), d_o.data_ptr(), dq.data_ptr(),
                                          dk.data_ptr(), dv.data_ptr(), workspace.data_ptr(),
                                          workspace.numel(), _stream())
    if rc != 0:
        raise AerisError(rc, "aeris_winattn_bwd_windows")
    return dq, dk, dv


def aeris_winattn_rope_fwd_windows(q, k, v, win, shift, base, positions, windows, o, lse,
                                   mask=AERIS_MASK_NONE, scale=None, out_dtype=AERIS_DT_BF16,
                                   workspace=None):
    """Rotary attention over the listed windows only; o and lse are written only inside them."""
    import torch
    assert windows.is_cuda and windows.dtype == torch.int32 and windows.is_contiguous()
    for t in (q, k, v):
        assert t.is_cuda and t.dtype == torch.bfloat16 and t.is_contiguous() and t.shape == q.shape
    p = make_params(q.shape, win, shift, mask, scale, out_dtype)
    r = aeris_rope_params(float(base), int(positions))
    if workspace is None:
        workspace = torch.empty(aeris_winattn_rope_fwd_workspace_bytes(p), dtype=torch.uint8,
                                device=q.device)
    rc = load().aeris_winattn_rope_fwd_windows(ctypes.byref(p), ctypes.byref(r), windows.data_ptr(),
                                               windows.numel(), q.data_ptr(), k.data_ptr(),
                                               v.data_ptr(), o.data_ptr(), lse.data_ptr(),
                                               workspace.data_ptr(), workspace.numel(), _stream())
    if rc != 0:
        raise AerisError(rc, "aeris_winattn_rope_fwd_windows")
    return o, lse


def aeris_winattn_rope_bwd_windows(q, k, v, o, lse, d_o, win, shift, base, positions, windows,
                                   dq, dk, dv, mask=AERIS_MASK_NONE, scale=None,
                                   out_dtype=AERIS_DT_BF16, workspace=None, saved=None):
    """Backward of the call above; dq, dk, dv are written only inside the listed windows.
    saved: the workspace of the forward call over the same list."""
    import torch
    assert windows.is_cuda and windows.dtype == torch.int32 and windows.is_contiguous()
    p = make_params(q.shape, win, shift, mask, scale, out_dtype)
    r = aeris_rope_params(float(base), int(positions))
    if workspace is None:
        need = (aeris_winattn_rope_bwd_workspace_bytes(p) if saved is None
                else aeris_winattn_bwd_workspace_bytes(p))
        workspace = torch.empty(need, dtype=torch.uint8, device=q.device)
    rc = load().aeris_winattn_rope_bwd_windows(ctypes.byref(p), ctypes.byref(r), windows.data_ptr(),
                                               windows.numel(), q.data_ptr(), k.data_ptr(),
                                               v.data_ptr(), o.data_ptr(), lse.data_ptr(),
                                               d_o.data_ptr(), dq.data_ptr(), dk.data_ptr(),
                                               dv.data_ptr(),
                                               None if saved is None else saved.data_ptr(),
                                               workspace.data_ptr(), workspace.numel(), _stream())
    if rc != 0:
        raise AerisError(rc, "aeris_winattn_rope_bwd_windows")
    return dq, dk, dv


def aeris_mfma_loop_probe(blocks, iters, random_operands, sink):
    """Measurement aid: register-operand MFMA loop; sink is a float32 device tensor of blocks*256."""
    import torch
    assert sink.is_cuda and sink.dtype == torch.float32 and sink.numel() >= blocks * 256
    rc = load().aeris_mfma_loop_probe(int(blocks), int(iters), 1 if random_operands else 0,
                                      sink.data_ptr(), _stream())
    if rc != 0:
        raise AerisError(rc, "aeris_mfma_loop_probe")
    return blocks * 4 * iters * 8 * 32768.0


# ---------------------------------------------------------------------------------------------
# include/aeris_layer_ops.h: element-wise operations of a transformer layer.  Activations are
# contiguous bf16 CUDA tensors [n_rows, channels]; w, alpha, beta, gamma are fp32.
# ---------------------------------------------------------------------------------------------
def _rows(t):
    import torch
    assert t.is_cuda and t.is_contiguous() and t.dtype == torch.bfloat16 and t.dim() == 2
    return t.shape[0], t.shape[1]


def _f32(*ts):
    import torch
    for t in ts:
        assert t is None or (t.is_cuda and t.is_contiguous() and t.dtype == torch.float32)


def _ptr(t):
    return None if t is None else t.data_ptr()


def aeris_rmsnorm_adaln_fwd(x, w, gamma, beta, eps, rows_per_sample, h=None, r=None,
                            want_r=True):
    """Returns (h, r): h = RMSNorm(x; w) * (1 + gamma_b) + beta_b, r the reciprocal RMS per row."""
    import torch
    n, c = _rows(x)
    _f32(w, gamma, beta, r)
    if h is None:
        h = torch.empty_like(x)
    if r is None and want_r:
        r = torch.empty(n, dtype=torch.float32, device=x.device)
    rc = load().aeris_rmsnorm_adaln_fwd(x.data_ptr(), w.data_ptr(), gamma.data_ptr(),
                                        beta.data_ptr(), float(eps), n, rows_per_sample, c,
                                        h.data_ptr(), _ptr(r), _stream())
    if rc != 0:
        raise AerisError(rc, "aeris_rmsnorm_adaln_fwd")
    return h, r


def aeris_rmsnorm_adaln_bwd_workspace_bytes(n_rows, rows_per_sample, channels):
    return load().aeris_rmsnorm_adaln_bwd_workspace_bytes(n_rows, rows_per_sample, channels)


def aeris_rmsnorm_adaln_bwd(x, w, gamma, r, dh, rows_per_sample, workspace=None,
                            want=(True, True, True), dres=None):
    """Returns (dx, dw, dgamma, dbeta); entries of `want` switch dw, dgamma, dbeta off (None).
    dres: the gradient arriving along the residual path, added into dx in the same pass."""
    import torch
    n, c = _rows(x)
    assert _rows(dh) == (n, c) and (dres is None or _rows(dres) == (n, c))
    _f32(w, gamma, r)
    nb = n // rows_per_sample
    dx = torch.empty_like(x)
    dw = torch.empty(c, dtype=torch.float32, device=x.device) if want[0] else None
    dgamma = torch.empty(nb, c, dtype=torch.float32, device=x.device) if want[1] else None
    dbeta = torch.empty(nb, c, dtype=torch.float32, device=x.device) if want[2] else None
    if workspace is None:
        need = aeris_rmsnorm_adaln_bwd_workspace_bytes(n, rows_per_sample, c)
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=x.device)
    rc = load().aeris_rmsnorm_adaln_bwd_residual(x.data_ptr(), w.data_ptr(), gamma.data_ptr(),
                                                 r.data_ptr(), dh.data_ptr(), _ptr(dres), n,
                                                 rows_per_sample, c, dx.data_ptr(), _ptr(dw),
                                                 _ptr(dgamma), _ptr(dbeta), workspace.data_ptr(),
                                                 workspace.numel(), _stream())
    if rc != 0:
        raise AerisError(rc, "aeris_rmsnorm_adaln_bwd")
    return dx, dw, dgamma, dbeta


def aeris_gate_residual_fwd(x, y, alpha, rows_per_sample, out=None):
    """out = x + alpha_b * y (out may be x or y)."""
    import torch
    n, c = _rows(x)
    assert _rows(y) == (n, c)
    _f32(alpha)
    if out is None:
        out = torch.empty_like(x)
    rc = load().aeris_gate_residual_fwd(x.data_ptr(), y.data_ptr(), alpha.data_ptr(), n,
                                        rows_per_sample, c, out.data_ptr(), _stream())
    if rc != 0:
        raise AerisError(rc, "aeris_gate_residual_fwd")
    return out


def aeris_gate_residual_bwd_workspace_bytes(n_rows, rows_per_sample, channels):
    return load().aeris_gate_residual_bwd_workspace_bytes(n_rows, rows_per_sample, channels)


def aeris_gate_residual_bwd(y, alpha, dout, rows_per_sample, dy=None, workspace=None,
                            want_dalpha=True):
    """Returns (dy, dalpha) for out = x + alpha_b * y (dy may be dout)."""
    import torch
    n, c = _rows(y)
    assert _rows(dout) == (n, c)
    _f32(alpha)
    if dy is None:
        dy = torch.empty_like(y)
    dalpha = (torch.empty(n // rows_per_sample, c, dtype=torch.float32, device=y.device)
              if want_dalpha else None)
    if workspace is None:
        need = aeris_gate_residual_bwd_workspace_bytes(n, rows_per_sample, c)
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=y.device)
    rc = load().aeris_gate_residual_bwd(y.data_ptr(), alpha.data_ptr(), dout.data_ptr(), n,
                                        rows_per_sample, c, dy.data_ptr(), _ptr(dalpha),
                                        workspace.data_ptr(), workspace.numel(), _stream())
    if rc != 0:
        raise AerisError(rc, "aeris_gate_residual_bwd")
    return dy, dalpha


def aeris_swiglu_fwd(uv, g=None):
    """g = silu(u) * v for uv = [u | v]."""
    import torch
    n, c2 = _rows(uv)
    assert c2 % 2 == 0
    if g is None:
        g = torch.empty(n, c2 // 2, dtype=torch.bfloat16, device=uv.device)
    rc = load().aeris_swiglu_fwd(uv.data_ptr(), n, c2 // 2, g.data_ptr(), _stream())
    if rc != 0:
        raise AerisError(rc, "aeris_swiglu_fwd")
    return g


def aeris_swiglu_bwd(uv, dg, duv=None):
    """duv = [du | dv] (duv may be uv)."""
    import torch
    n, c2 = _rows(uv)
    assert _rows(dg) == (n, c2 // 2)
    if duv is None:
        duv = torch.empty_like(uv)
    rc = load().aeris_swiglu_bwd(uv.data_ptr(), dg.data_ptr(), n, c2 // 2, duv.data_ptr(),
                                 _stream())
    if rc != 0:
        raise AerisError(rc, "aeris_swiglu_bwd")
    return duv


def aeris_norm_linear_workspace_bytes(n_rows, rows_per_sample, channels, out_features):
    return load().aeris_norm_linear_workspace_bytes(n_rows, rows_per_sample, channels, out_features)


def _check_projection(x, w, gamma, beta, weight):
    import torch
    n, c = _rows(x)
    assert weight.is_cuda and weight.dtype == torch.bfloat16 and weight.is_contiguous()
    assert weight.dim() == 2 and weight.shape[1] == c
    for t in (w, gamma, beta):
        assert t.is_cuda and t.dtype == torch.float32 and t.is_contiguous()
    return n, c


def aeris_norm_linear_fwd(x, w, gamma, beta, eps, weight, rows_per_sample, y=None, workspace=None):
    """y = (RMSNorm(x; w) (1 + gamma_b) + beta_b) weight^T without writing the normalised rows.
    x [N, C] bf16, weight [F, C] bf16; returns y [N, F] bf16."""
    import torch
    n, c = _check_projection(x, w, gamma, beta, weight)
    f = weight.shape[0]
    if y is None:
        y = torch.empty((n, f), dtype=torch.bfloat16, device=x.device)
    if workspace is None:
        workspace = torch.empty(aeris_norm_linear_workspace_bytes(n, rows_per_sample, c, f),
                                dtype=torch.uint8, device=x.device)
    rc = load().aeris_norm_linear_fwd(x.data_ptr(), w.data_ptr(), gamma.data_ptr(), beta.data_ptr(),
                                      float(eps), weight.data_ptr(), n, rows_per_sample, c, f,
                                      y.data_ptr(), workspace.data_ptr(), workspace.numel(),
                                      _stream())
    if rc != 0:
        raise AerisError(rc, "aeris_norm_linear_fwd")
    return y


def aeris_norm_linear_swiglu_fwd(x, w, gamma, beta, eps, weight, rows_per_sample, g=None, uv=None,
                                 want_uv=True, workspace=None):
    """SwiGLU up-projection of the normalised rows with the gate in the epilogue.
    weight [2*hidden, C] = [u rows ; v rows]; returns (g [N, hidden], uv [N, 2*hidden] or None)."""
    import torch
    n, c = _check_projection(x, w, gamma, beta, weight)
    f2 = weight.shape[0]
    assert f2 % 2 == 0
    if g is None:
        g = torch.empty((n, f2 // 2), dtype=torch.bfloat16, device=x.device)
    if uv is None and want_uv:
        uv = torch.empty((n, f2), dtype=torch.bfloat16, device=x.device)
    if workspace is None:
        workspace = torch.empty(aeris_norm_linear_workspace_bytes(n, rows_per_sample, c, f2),
                                dtype=torch.uint8, device=x.device)
    rc = load().aeris_norm_linear_swiglu_fwd(x.data_ptr(), w.data_ptr(), gamma.data_ptr(),
                                             beta.data_ptr(), float(eps), weight.data_ptr(), n,
                                             rows_per_sample, c, f2 // 2, g.data_ptr(),
                                             None if uv is None else uv.data_ptr(),
                                             workspace.data_ptr(), workspace.numel(), _stream())
    if rc != 0:
        raise AerisError(rc, "aeris_norm_linear_swiglu_fwd")
    return g, uv


def aeris_linear_fwd(x, weight, y=None):
    """y = x weight^T (bf16 in and out, fp32 accumulation)."""
    import torch
    n, c = _rows(x)
    assert weight.is_cuda and weight.dtype == torch.bfloat16 and weight.is_contiguous()
    assert weight.dim() == 2 and weight.shape[1] == c
    if y is None:
        y = torch.empty((n, weight.shape[0]), dtype=torch.bfloat16, device=x.device)
    rc = load().aeris_linear_fwd(x.data_ptr(), weight.data_ptr(), n, c, weight.shape[0],
                                 y.data_ptr(), _stream())
    if rc != 0:
        raise AerisError(rc, "aeris_linear_fwd")
    return y


def aeris_linear_bwd_workspace_bytes(n_rows, channels, out_features):
    return load().aeris_linear_bwd_workspace_bytes(n_rows, channels, out_features)


def aeris_linear_bwd(x, weight, dy, want_dx=True, want_dweight=True, dx=None, dweight=None,
                     workspace=None):
    """Gradients of y = x weight^T: dx = dy weight (bf16), dweight = dy^T x (fp32)."""
    import torch
    n, f = _rows(dy)
    assert weight.is_cuda and weight.dtype == torch.bfloat16 and weight.is_contiguous()
    assert weight.dim() == 2 and weight.shape[0] == f
    c = weight.shape[1]
    if want_dweight:
        assert _rows(x) == (n, c)
    if want_dx and dx is None:
        dx = torch.empty((n, c), dtype=torch.bfloat16, device=dy.device)
    if want_dweight and dweight is None:
        dweight = torch.empty((f, c), dtype=torch.float32, device=dy.device)
    if workspace is None:
        workspace = torch.empty(max(aeris_linear_bwd_workspace_bytes(n, c, f), 16), dtype=torch.uint8,
                                device=dy.device)
    rc = load().aeris_linear_bwd(x.data_ptr() if want_dweight else None, weight.data_ptr(),
                                 dy.data_ptr(), n, c, f,
                                 dx.data_ptr() if want_dx else None,
                                 dweight.data_ptr() if want_dweight else None,
                                 workspace.data_ptr(), workspace.numel(), _stream())
    if rc != 0:
        raise AerisError(rc, "aeris_linear_bwd")
    return (dx if want_dx else None), (dweight if want_dweight else None)
