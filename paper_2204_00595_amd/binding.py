"""Thin ctypes binding over libmonarch.so: argument marshalling only.

Every function has the name of the C entry point it calls (``include/monarch.h``).
PyTorch supplies device memory and the current HIP stream; all arithmetic runs in
the library's kernels.  There is no fallback: if the library is missing, loading
fails with an error that says how to build it.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmonarch.so")

MONARCH_F32 = 0
MONARCH_BF16 = 1
MONARCH_OK = 0
MONARCH_ERR_INVALID = -1
MONARCH_ERR_UNSUPPORTED = -2
MONARCH_ERR_WORKSPACE = -3
MONARCH_ERR_HIP = -4
MONARCH_FLAG_WGRAD_F32 = 1
MONARCH_FLAG_PERM_B = 2
MONARCH_FLAG_GENERIC = 4
MONARCH_FLAG_WS_PACKED = 8

# every symbol include/monarch.h declares
EXPORTS = (
    "monarch_fwd", "monarch_fwd_ex", "monarch_fwd_ws", "monarch_fwd_static", "monarch_fwd_bias", "monarch_fwd_workspace_bytes", "monarch_bwd",
    "monarch_bwd_bias", "monarch_fwd_bias_gelu", "monarch_bwd_bias_gelu_in",
    "monarch_bwd_workspace_bytes",
    "monarch_fwd_t", "monarch_fwd_t_workspace_bytes", "monarch_saved_bytes", "monarch_fwd_save", "monarch_bwd_saved", "monarch_fwd_c64", "monarch_fwd_h_c64", "monarch_bwd_c64", "monarch_fwd_c64_ws", "monarch_fwd_h_c64_ws", "monarch_bwd_c64_ws", "monarch_c64_workspace_bytes", "monarch_dft_factors", "monarch_to_dense", "monarch_project", "monarch_kernel_name", "monarch_status_string", "monarch_version", "monarch_stream_copy", "monarch_launch_probe",
)

_lib = None


class MonarchError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s failed: %d (%s)" % (where, status, monarch_status_string(status)))


def lib() -> ctypes.CDLL:
    """Load libmonarch.so (built in-tree by ``paper_2204_00595_amd.build``)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(
                "%s is missing: build it with `python -m paper_2204_00595_amd.build` "
                "(or __graft_entry__.build()); there is no fallback path" % LIB_PATH)
        L = ctypes.CDLL(LIB_PATH)
        vp, i64, ci, cu, sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_uint, ctypes.c_size_t
        L.monarch_fwd.restype = ci
        L.monarch_fwd.argtypes = [vp, vp, vp, vp, i64, ci, ci, ci, ci, ci, vp]
        L.monarch_fwd_ex.restype = ci
        L.monarch_fwd_ex.argtypes = [vp, vp, vp, vp, i64, ci, ci, ci, ci, ci, vp, cu]
        L.monarch_fwd_ws.restype = ci
        L.monarch_fwd_ws.argtypes = [vp, vp, vp, vp, i64, ci, ci, ci, ci, ci, vp, vp, sz, cu]
        L.monarch_fwd_static.restype = ci
        L.monarch_fwd_static.argtypes = [vp, vp, vp, vp, i64, ci, ci, ci, ci, ci, vp, cu]
        L.monarch_fwd_bias.restype = ci
        L.monarch_fwd_bias.argtypes = [vp, vp, vp, vp, vp, i64, ci, ci, ci, ci, ci, vp, vp, sz, cu]
        L.monarch_bwd_bias.restype = ci
        L.monarch_bwd_bias.argtypes = [vp] * 8 + [i64, ci, ci, ci, ci, ci, vp, vp, sz, cu]
        L.monarch_fwd_bias_gelu.restype = ci
        L.monarch_fwd_bias_gelu.argtypes = [vp] * 6 + [i64, ci, ci, ci, ci, ci, vp, vp, sz, cu]
        L.monarch_bwd_bias_gelu_in.restype = ci
        L.monarch_bwd_bias_gelu_in.argtypes = [vp] * 9 + [i64, ci, ci, ci, ci, ci, vp, vp, sz, cu]
        L.monarch_fwd_workspace_bytes.restype = sz
        L.monarch_fwd_workspace_bytes.argtypes = [i64, ci, ci, ci, ci, ci, cu]
        L.monarch_bwd.restype = ci
        L.monarch_bwd.argtypes = [vp] * 7 + [i64, ci, ci, ci, ci, ci, vp, vp, sz, cu]
        L.monarch_bwd_workspace_bytes.restype = sz
        L.monarch_bwd_workspace_bytes.argtypes = [i64, ci, ci, ci, ci, ci, cu]
        L.monarch_to_dense.restype = ci
        L.monarch_to_dense.argtypes = [vp, vp, vp, ci, ci, ci, ci, ci, vp, cu]
        L.monarch_fwd_t.restype = ci
        L.monarch_fwd_t.argtypes = [vp, vp, vp, vp, i64, ci, ci, ci, ci, ci, vp, vp, sz, cu]
        L.monarch_fwd_t_workspace_bytes.restype = sz
        L.monarch_fwd_t_workspace_bytes.argtypes = [i64, ci, ci, ci, ci, ci, cu]
        L.monarch_saved_bytes.restype = sz
        L.monarch_saved_bytes.argtypes = [i64, ci, ci, ci, ci, ci, cu]
        L.monarch_fwd_save.restype = ci
        L.monarch_fwd_save.argtypes = [vp, vp, vp, vp, vp, sz, i64, ci, ci, ci, ci, ci, vp, cu]
        L.monarch_bwd_saved.restype = ci
        L.monarch_bwd_saved.argtypes = [vp, vp, vp, sz, vp, vp, vp, vp, vp, vp, i64, ci, ci, ci, ci, ci, vp, vp, sz, cu]
        L.monarch_fwd_c64.restype = ci
        L.monarch_fwd_c64.argtypes = [vp, vp, vp, vp, i64, ci, ci, ci, ci, vp, cu]
        L.monarch_fwd_h_c64.restype = ci
        L.monarch_fwd_h_c64.argtypes = [vp, vp, vp, vp, i64, ci, ci, ci, ci, vp, cu]
        L.monarch_bwd_c64.restype = ci
        L.monarch_bwd_c64.argtypes = [vp] * 7 + [i64, ci, ci, ci, ci, vp, cu]
        L.monarch_bwd_c64_ws.restype = ci
        L.monarch_bwd_c64_ws.argtypes = [vp] * 7 + [i64, ci, ci, ci, ci, vp, vp, sz, cu]
        L.monarch_fwd_c64_ws.restype = ci
        L.monarch_fwd_c64_ws.argtypes = [vp, vp, vp, vp, i64, ci, ci, ci, ci, vp, vp, sz, cu]
        L.monarch_fwd_h_c64_ws.restype = ci
        L.monarch_fwd_h_c64_ws.argtypes = [vp, vp, vp, vp, i64, ci, ci, ci, ci, vp, vp, sz, cu]
        L.monarch_c64_workspace_bytes.restype = sz
        L.monarch_c64_workspace_bytes.argtypes = [ci, i64, ci, ci, ci, ci, cu]
        L.monarch_dft_factors.restype = ci
        L.monarch_dft_factors.argtypes = [vp, vp, ci, ci, vp]
        L.monarch_project.restype = ci
        L.monarch_project.argtypes = [vp, vp, vp, ci, ci, ci, vp, cu]
        L.monarch_kernel_name.restype = ctypes.c_char_p
        L.monarch_kernel_name.argtypes = [ci, ci, ci, ci, ci, ci, cu]
        L.monarch_status_string.restype = ctypes.c_char_p
        L.monarch_status_string.argtypes = [ci]
        L.monarch_version.restype = ci
        L.monarch_version.argtypes = []
        L.monarch_stream_copy.restype = ci
        L.monarch_stream_copy.argtypes = [vp, vp, sz, vp]
        L.monarch_launch_probe.restype = ci
        L.monarch_launch_probe.argtypes = [vp]
        _lib = L
    return _lib


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return MONARCH_F32
    if t.dtype == torch.bfloat16:
        return MONARCH_BF16
    raise TypeError("dtype must be float32 or bfloat16, got %s" % t.dtype)


def _check(t: torch.Tensor, name: str, shape, dtype, device):
    if not t.is_cuda or t.device != device:
        raise ValueError("%s must live on %s" % (name, device))
    if t.dtype != dtype:
        raise TypeError("%s: dtype %s, expected %s" % (name, t.dtype, dtype))
    if tuple(t.shape) != tuple(shape):
        raise ValueError("%s: shape %s, expected %s" % (name, tuple(t.shape), tuple(shape)))
    if not t.is_contiguous():
        raise ValueError("%s must be contiguous" % name)


def _scratch(nbytes: int, dev, stream) -> torch.Tensor:
    """A temporary buffer for kernels that run on `stream`.  It is allocated with `stream` current, so the
    caching allocator hands its block, once released, only to later work of that same stream: a buffer
    released on return while the kernels are still running cannot be given to another stream."""
    if stream is None:
        return torch.empty(nbytes, dtype=torch.uint8, device=dev)
    with torch.cuda.stream(stream):
        return torch.empty(nbytes, dtype=torch.uint8, device=dev)


def _stream_ptr(stream) -> int:
    st = torch.cuda.current_stream() if stream is None else stream
    return int(st.cuda_stream)


def monarch_stream_copy(dst: torch.Tensor, src: torch.Tensor, stream=None) -> torch.Tensor:
    """Plain streaming copy src -> dst (same byte size, contiguous, on one GPU): the measured HBM roof."""
    nbytes = src.numel() * src.element_size()
    if dst.numel() * dst.element_size() != nbytes or not (dst.is_cuda and src.is_cuda and dst.device == src.device):
        raise ValueError("dst and src must be GPU tensors of the same byte size on one device")
    if not (dst.is_contiguous() and src.is_contiguous()):
        raise ValueError("dst and src must be contiguous")
    with torch.cuda.device(src.device):
        rc = lib().monarch_stream_copy(dst.data_ptr(), src.data_ptr(), nbytes, _stream_ptr(stream))
    if rc != MONARCH_OK:
        raise MonarchError(rc, "monarch_stream_copy")
    return dst


def monarch_launch_probe(stream=None) -> None:
    """Enqueue one empty kernel on the stream (the launch floor of the machine, for the benchmark)."""
    rc = lib().monarch_launch_probe(_stream_ptr(stream))
    if rc != MONARCH_OK:
        raise MonarchError(rc, "monarch_launch_probe")


def monarch_version() -> int:
    return int(lib().monarch_version())


def monarch_status_string(status: int) -> str:
    return lib().monarch_status_string(int(status)).decode()


def monarch_kernel_name(pass_: int, n_in: int, k: int, q: int, s: int, dtype: int, flags: int = 0) -> str:
    return lib().monarch_kernel_name(pass_, n_in, k, q, s, dtype, flags).decode()


def monarch_bwd_workspace_bytes(batch: int, n_in: int, k: int, q: int, s: int, dtype: int, flags: int = 0) -> int:
    return int(lib().monarch_bwd_workspace_bytes(batch, n_in, k, q, s, dtype, flags))


def monarch_fwd_workspace_bytes(batch: int, n_in: int, k: int, q: int, s: int, dtype: int, flags: int = 0) -> int:
    return int(lib().monarch_fwd_workspace_bytes(batch, n_in, k, q, s, dtype, flags))


def monarch_fwd_ws(x: torch.Tensor, R: torch.Tensor, L: torch.Tensor, y: torch.Tensor | None = None,
                   workspace: torch.Tensor | None = None, flags: int = 0, stream=None) -> torch.Tensor:
    """y = x M^T through monarch_fwd_ws.  The workspace is allocated when not given."""
    k, q, p = R.shape
    s = L.shape[1]
    B = x.shape[0]
    dev, dt = x.device, x.dtype
    _check(x, "x", (B, k * p), dt, dev)
    _check(R, "R", (k, q, p), dt, dev)
    _check(L, "L", (k, s, q), dt, dev)
    if y is None:
        y = torch.empty((B, k * s), dtype=dt, device=dev)
    _check(y, "y", (B, k * s), dt, dev)
    need = monarch_fwd_workspace_bytes(B, k * p, k, q, s, _dtype_code(x), flags)
    if workspace is None and need:
        if flags & MONARCH_FLAG_WS_PACKED:
            raise ValueError("MONARCH_FLAG_WS_PACKED needs the workspace of the earlier call")
        workspace = _scratch(need, dev, stream)
    ws_ptr = workspace.data_ptr() if workspace is not None else 0
    ws_len = workspace.numel() * workspace.element_size() if workspace is not None else 0
    with torch.cuda.device(dev):
        rc = lib().monarch_fwd_ws(x.data_ptr(), R.data_ptr(), L.data_ptr(), y.data_ptr(), B, k * p, k, q, s,
                                  _dtype_code(x), _stream_ptr(stream), ws_ptr, ws_len, flags)
    if rc != MONARCH_OK:
        raise MonarchError(rc, "monarch_fwd_ws")
    return y


MONARCH_STATIC_WORKSPACE_BYTES = 8 << 20


def monarch_fwd_static(x: torch.Tensor, R: torch.Tensor, L: torch.Tensor, y: torch.Tensor, flags: int = 0,
                       stream=None) -> torch.Tensor:
    """y = x M^T through monarch_fwd_static (the library's own static workspace; nothing is allocated,
    so `y` must be given)."""
    k, q, p = R.shape
    s = L.shape[1]
    B = x.shape[0]
    dev, dt = x.device, x.dtype
    _check(x, "x", (B, k * p), dt, dev)
    _check(R, "R", (k, q, p), dt, dev)
    _check(L, "L", (k, s, q), dt, dev)
    _check(y, "y", (B, k * s), dt, dev)
    with torch.cuda.device(dev):
        rc = lib().monarch_fwd_static(x.data_ptr(), R.data_ptr(), L.data_ptr(), y.data_ptr(), B, k * p, k, q, s,
                                      _dtype_code(x), _stream_ptr(stream), flags)
    if rc != MONARCH_OK:
        raise MonarchError(rc, "monarch_fwd_static")
    return y


def monarch_fwd(x: torch.Tensor, R: torch.Tensor, L: torch.Tensor, y: torch.Tensor | None = None,
                flags: int = 0, stream=None) -> torch.Tensor:
    """y = x M^T.  x (B, k*p), R (k, q, p), L (k, s, q) on the GPU; returns y (B, k*s)."""
    k, q, p = R.shape
    s = L.shape[1]
    B = x.shape[0]
    dev, dt = x.device, x.dtype
    _check(x, "x", (B, k * p), dt, dev)
    _check(R, "R", (k, q, p), dt, dev)
    _check(L, "L", (k, s, q), dt, dev)
    if y is None:
        y = torch.empty((B, k * s), dtype=dt, device=dev)
    _check(y, "y", (B, k * s), dt, dev)
    with torch.cuda.device(dev):
        if flags:
            rc = lib().monarch_fwd_ex(x.data_ptr(), R.data_ptr(), L.data_ptr(), y.data_ptr(), B, k * p, k, q, s,
                                      _dtype_code(x), _stream_ptr(stream), flags)
        else:
            rc = lib().monarch_fwd(x.data_ptr(), R.data_ptr(), L.data_ptr(), y.data_ptr(), B, k * p, k, q, s,
                                   _dtype_code(x), _stream_ptr(stream))
    if rc != MONARCH_OK:
        raise MonarchError(rc, "monarch_fwd")
    return y


def monarch_to_dense(R: torch.Tensor, L: torch.Tensor, M: torch.Tensor | None = None, flags: int = 0,
                     stream=None) -> torch.Tensor:
    """M = P L P^T R as a dense (k*s, k*p) matrix.  R (k, q, p), L (k, s, q) on the GPU."""
    k, q, p = R.shape
    s = L.shape[1]
    dev, dt = R.device, R.dtype
    _check(R, "R", (k, q, p), dt, dev)
    _check(L, "L", (k, s, q), dt, dev)
    if M is None:
        M = torch.empty((k * s, k * p), dtype=dt, device=dev)
    _check(M, "M", (k * s, k * p), dt, dev)
    with torch.cuda.device(dev):
        rc = lib().monarch_to_dense(R.data_ptr(), L.data_ptr(), M.data_ptr(), k * p, k, q, s, _dtype_code(R),
                                    _stream_ptr(stream), flags)
    if rc != MONARCH_OK:
        raise MonarchError(rc, "monarch_to_dense")
    return M


def monarch_bwd(dy: torch.Tensor, x: torch.Tensor, R: torch.Tensor, L: torch.Tensor,
                dx: torch.Tensor | None = None, dR: torch.Tensor | None = None, dL: torch.Tensor | None = None,
                workspace: torch.Tensor | None = None, flags: int = 0, stream=None):
    """(dx, dR, dL) for upstream gradient dy (B, k*s).  Buffers are allocated when not given."""
    k, q, p = R.shape
    s = L.shape[1]
    B = x.shape[0]
    dev, dt = x.device, x.dtype
    _check(x, "x", (B, k * p), dt, dev)
    _check(dy, "dy", (B, k * s), dt, dev)
    _check(R, "R", (k, q, p), dt, dev)
    _check(L, "L", (k, s, q), dt, dev)
    gdt = torch.float32 if (flags & MONARCH_FLAG_WGRAD_F32) else dt
    if dx is None:
        dx = torch.empty_like(x)
    if dR is None:
        dR = torch.empty((k, q, p), dtype=gdt, device=dev)
    if dL is None:
        dL = torch.empty((k, s, q), dtype=gdt, device=dev)
    _check(dx, "dx", (B, k * p), dt, dev)
    _check(dR, "dR", (k, q, p), gdt, dev)
    _check(dL, "dL", (k, s, q), gdt, dev)
    need = monarch_bwd_workspace_bytes(B, k * p, k, q, s, _dtype_code(x), flags)
    if workspace is None and need:
        workspace = _scratch(need, dev, stream)
    ws_ptr = workspace.data_ptr() if workspace is not None else 0
    ws_len = workspace.numel() * workspace.element_size() if workspace is not None else 0
    with torch.cuda.device(dev):
        rc = lib().monarch_bwd(dy.data_ptr(), x.data_ptr(), R.data_ptr(), L.data_ptr(), dx.data_ptr(),
                               dR.data_ptr(), dL.data_ptr(), B, k * p, k, q, s, _dtype_code(x),
                               _stream_ptr(stream), ws_ptr, ws_len, flags)
    if rc != MONARCH_OK:
        raise MonarchError(rc, "monarch_bwd")
    return dx, dR, dL


def monarch_fwd_bias(x: torch.Tensor, R: torch.Tensor, L: torch.Tensor, bias: torch.Tensor,
                     y: torch.Tensor | None = None, workspace: torch.Tensor | None = None, flags: int = 0,
                     stream=None) -> torch.Tensor:
    """y = x M^T + bias.  bias (k*s,) of the same dtype; the workspace is allocated when not given."""
    k, q, p = R.shape
    s = L.shape[1]
    B = x.shape[0]
    dev, dt = x.device, x.dtype
    _check(x, "x", (B, k * p), dt, dev)
    _check(R, "R", (k, q, p), dt, dev)
    _check(L, "L", (k, s, q), dt, dev)
    _check(bias, "bias", (k * s,), dt, dev)
    if y is None:
        y = torch.empty((B, k * s), dtype=dt, device=dev)
    _check(y, "y", (B, k * s), dt, dev)
    need = monarch_fwd_workspace_bytes(B, k * p, k, q, s, _dtype_code(x), flags)
    if workspace is None and need:
        if flags & MONARCH_FLAG_WS_PACKED:
            raise ValueError("MONARCH_FLAG_WS_PACKED needs the workspace of the earlier call")
        workspace = _scratch(need, dev, stream)
    ws_ptr = workspace.data_ptr() if workspace is not None else 0
    ws_len = workspace.numel() * workspace.element_size() if workspace is not None else 0
    with torch.cuda.device(dev):
        rc = lib().monarch_fwd_bias(x.data_ptr(), R.data_ptr(), L.data_ptr(), bias.data_ptr(), y.data_ptr(), B, k * p,
                                    k, q, s, _dtype_code(x), _stream_ptr(stream), ws_ptr, ws_len, flags)
    if rc != MONARCH_OK:
        raise MonarchError(rc, "monarch_fwd_bias")
    return y


def monarch_bwd_bias(dy: torch.Tensor, x: torch.Tensor, R: torch.Tensor, L: torch.Tensor,
                     dx: torch.Tensor | None = None, dR: torch.Tensor | None = None, dL: torch.Tensor | None = None,
                     dbias: torch.Tensor | None = None, workspace: torch.Tensor | None = None, flags: int = 0,
                     stream=None):
    """(dx, dR, dL, dbias) for upstream gradient dy (B, k*s).  Buffers are allocated when not given."""
    k, q, p = R.shape
    s = L.shape[1]
    B = x.shape[0]
    dev, dt = x.device, x.dtype
    _check(x, "x", (B, k * p), dt, dev)
    _check(dy, "dy", (B, k * s), dt, dev)
    _check(R, "R", (k, q, p), dt, dev)
    _check(L, "L", (k, s, q), dt, dev)
    gdt = torch.float32 if (flags & MONARCH_FLAG_WGRAD_F32) else dt
    if dx is None:
        dx = torch.empty_like(x)
    if dR is None:
        dR = torch.empty((k, q, p), dtype=gdt, device=dev)
    if dL is None:
        dL = torch.empty((k, s, q), dtype=gdt, device=dev)
    if dbias is None:
        dbias = torch.empty((k * s,), dtype=gdt, device=dev)
    _check(dx, "dx", (B, k * p), dt, dev)
    _check(dR, "dR", (k, q, p), gdt, dev)
    _check(dL, "dL", (k, s, q), gdt, dev)
    _check(dbias, "dbias", (k * s,), gdt, dev)
    need = monarch_bwd_workspace_bytes(B, k * p, k, q, s, _dtype_code(x), flags)
    if workspace is None and need:
        workspace = _scratch(need, dev, stream)
    ws_ptr = workspace.data_ptr() if workspace is not None else 0
    ws_len = workspace.numel() * workspace.element_size() if workspace is not None else 0
    with torch.cuda.device(dev):
        rc = lib().monarch_bwd_bias(dy.data_ptr(), x.data_ptr(), R.data_ptr(), L.data_ptr(), dx.data_ptr(),
                                    dR.data_ptr(), dL.data_ptr(), dbias.data_ptr(), B, k * p, k, q, s,
                                    _dtype_code(x), _stream_ptr(stream), ws_ptr, ws_len, flags)
    if rc != MONARCH_OK:
        raise MonarchError(rc, "monarch_bwd_bias")
    return dx, dR, dL, dbias


def monarch_fwd_bias_gelu(x: torch.Tensor, R: torch.Tensor, L: torch.Tensor, bias: torch.Tensor | None = None,
                          y_pre: torch.Tensor | None = None, y: torch.Tensor | None = None, want_pre: bool = True,
                          workspace: torch.Tensor | None = None, flags: int = 0, stream=None):
    """(y_pre, y) with y_pre = x M^T + bias and y = gelu(y_pre) (tanh form).  `want_pre=False` and no y_pre
    buffer: the pre-activation is not written and None is returned in its place."""
    k, q, p = R.shape
    s = L.shape[1]
    B = x.shape[0]
    dev, dt = x.device, x.dtype
    _check(x, "x", (B, k * p), dt, dev)
    _check(R, "R", (k, q, p), dt, dev)
    _check(L, "L", (k, s, q), dt, dev)
    if bias is not None:
        _check(bias, "bias", (k * s,), dt, dev)
    if y is None:
        y = torch.empty((B, k * s), dtype=dt, device=dev)
    if y_pre is None and want_pre:
        y_pre = torch.empty((B, k * s), dtype=dt, device=dev)
    _check(y, "y", (B, k * s), dt, dev)
    if y_pre is not None:
        _check(y_pre, "y_pre", (B, k * s), dt, dev)
    need = monarch_fwd_workspace_bytes(B, k * p, k, q, s, _dtype_code(x), flags)
    if workspace is None and need:
        if flags & MONARCH_FLAG_WS_PACKED:
            raise ValueError("MONARCH_FLAG_WS_PACKED needs the workspace of the earlier call")
        workspace = _scratch(need, dev, stream)
    ws_ptr = workspace.data_ptr() if workspace is not None else 0
    ws_len = workspace.numel() * workspace.element_size() if workspace is not None else 0
    with torch.cuda.device(dev):
        rc = lib().monarch_fwd_bias_gelu(x.data_ptr(), R.data_ptr(), L.data_ptr(),
                                         bias.data_ptr() if bias is not None else 0,
                                         y_pre.data_ptr() if y_pre is not None else 0, y.data_ptr(), B, k * p,
                                         k, q, s, _dtype_code(x), _stream_ptr(stream), ws_ptr, ws_len, flags)
    if rc != MONARCH_OK:
        raise MonarchError(rc, "monarch_fwd_bias_gelu")
    return y_pre, y


def monarch_bwd_bias_gelu_in(dy: torch.Tensor, x: torch.Tensor, x_pre: torch.Tensor, R: torch.Tensor, L: torch.Tensor,
                             dx_pre: torch.Tensor | None = None, dR: torch.Tensor | None = None,
                             dL: torch.Tensor | None = None, dbias: torch.Tensor | None = None, want_dbias: bool = True,
                             workspace: torch.Tensor | None = None, flags: int = 0, stream=None):
    """(dx_pre, dR, dL, dbias) of the layer y = x M^T + bias whose input is x = gelu(x_pre): dx_pre is the
    gradient with respect to x_pre.  Buffers are allocated when not given."""
    k, q, p = R.shape
    s = L.shape[1]
    B = x.shape[0]
    dev, dt = x.device, x.dtype
    _check(x, "x", (B, k * p), dt, dev)
    _check(x_pre, "x_pre", (B, k * p), dt, dev)
    _check(dy, "dy", (B, k * s), dt, dev)
    _check(R, "R", (k, q, p), dt, dev)
    _check(L, "L", (k, s, q), dt, dev)
    gdt = torch.float32 if (flags & MONARCH_FLAG_WGRAD_F32) else dt
    if dx_pre is None:
        dx_pre = torch.empty_like(x)
    if dR is None:
        dR = torch.empty((k, q, p), dtype=gdt, device=dev)
    if dL is None:
        dL = torch.empty((k, s, q), dtype=gdt, device=dev)
    if dbias is None and want_dbias:
        dbias = torch.empty((k * s,), dtype=gdt, device=dev)
    _check(dx_pre, "dx_pre", (B, k * p), dt, dev)
    _check(dR, "dR", (k, q, p), gdt, dev)
    _check(dL, "dL", (k, s, q), gdt, dev)
    if dbias is not None:
        _check(dbias, "dbias", (k * s,), gdt, dev)
    need = monarch_bwd_workspace_bytes(B, k * p, k, q, s, _dtype_code(x), flags)
    if workspace is None and need:
        workspace = _scratch(need, dev, stream)
    ws_ptr = workspace.data_ptr() if workspace is not None else 0
    ws_len = workspace.numel() * workspace.element_size() if workspace is not None else 0
    with torch.cuda.device(dev):
        rc = lib().monarch_bwd_bias_gelu_in(dy.data_ptr(), x.data_ptr(), x_pre.data_ptr(), R.data_ptr(), L.data_ptr(),
                                            dx_pre.data_ptr(), dR.data_ptr(), dL.data_ptr(),
                                            dbias.data_ptr() if dbias is not None else 0, B, k * p, k, q, s,
                                            _dtype_code(x), _stream_ptr(stream), ws_ptr, ws_len, flags)
    if rc != MONARCH_OK:
        raise MonarchError(rc, "monarch_bwd_bias_gelu_in")
    return dx_pre, dR, dL, dbias


def monarch_project(A: torch.Tensor, R: torch.Tensor | None = None, L: torch.Tensor | None = None, stream=None):
    """(L, R): factors of the square Monarch matrix closest to the dense A (n, n), n = m*m, m <= 64."""
    n = A.shape[0]
    m = int(round(n ** 0.5))
    dev, dt = A.device, A.dtype
    if m * m != n:
        raise ValueError("A must be n x n with n a perfect square, got %s" % (tuple(A.shape),))
    _check(A, "A", (n, n), dt, dev)
    if R is None:
        R = torch.empty((m, m, m), dtype=dt, device=dev)
    if L is None:
        L = torch.empty((m, m, m), dtype=dt, device=dev)
    _check(R, "R", (m, m, m), dt, dev)
    _check(L, "L", (m, m, m), dt, dev)
    with torch.cuda.device(dev):
        rc = lib().monarch_project(A.data_ptr(), R.data_ptr(), L.data_ptr(), n, m, _dtype_code(A), _stream_ptr(stream), 0)
    if rc != MONARCH_OK:
        raise MonarchError(rc, "monarch_project")
    return L, R


def monarch_fwd_t_workspace_bytes(batch: int, n_in: int, k: int, q: int, s: int, dtype: int, flags: int = 0) -> int:
    return int(lib().monarch_fwd_t_workspace_bytes(batch, n_in, k, q, s, dtype, flags))


def monarch_fwd_t(x: torch.Tensor, R: torch.Tensor, L: torch.Tensor, y: torch.Tensor | None = None,
                  workspace: torch.Tensor | None = None, flags: int = 0, stream=None) -> torch.Tensor:
    """y = x M (the transposed Monarch matrix applied to the rows).  x (B, k*s) -> y (B, k*p)."""
    k, q, p = R.shape
    s = L.shape[1]
    B = x.shape[0]
    dev, dt = x.device, x.dtype
    _check(x, "x", (B, k * s), dt, dev)
    _check(R, "R", (k, q, p), dt, dev)
    _check(L, "L", (k, s, q), dt, dev)
    if y is None:
        y = torch.empty((B, k * p), dtype=dt, device=dev)
    _check(y, "y", (B, k * p), dt, dev)
    need = monarch_fwd_t_workspace_bytes(B, k * p, k, q, s, _dtype_code(x), flags)
    if workspace is None and need:
        workspace = _scratch(need, dev, stream)
    ws_ptr = workspace.data_ptr() if workspace is not None else 0
    ws_len = workspace.numel() * workspace.element_size() if workspace is not None else 0
    with torch.cuda.device(dev):
        rc = lib().monarch_fwd_t(x.data_ptr(), R.data_ptr(), L.data_ptr(), y.data_ptr(), B, k * p, k, q, s,
                                 _dtype_code(x), _stream_ptr(stream), ws_ptr, ws_len, flags)
    if rc != MONARCH_OK:
        raise MonarchError(rc, "monarch_fwd_t")
    return y


def monarch_saved_bytes(batch: int, n_in: int, k: int, q: int, s: int, dtype: int, flags: int = 0) -> int:
    return int(lib().monarch_saved_bytes(batch, n_in, k, q, s, dtype, flags))


def monarch_fwd_save(x: torch.Tensor, R: torch.Tensor, L: torch.Tensor, y: torch.Tensor | None = None,
                     saved: torch.Tensor | None = None, flags: int = 0, stream=None):
    """(y, saved): y = x M^T, and the buffer monarch_bwd_saved reads instead of recomputing (None when
    the shape has no such path)."""
    k, q, p = R.shape
    s = L.shape[1]
    B = x.shape[0]
    dev, dt = x.device, x.dtype
    _check(x, "x", (B, k * p), dt, dev)
    _check(R, "R", (k, q, p), dt, dev)
    _check(L, "L", (k, s, q), dt, dev)
    if y is None:
        y = torch.empty((B, k * s), dtype=dt, device=dev)
    _check(y, "y", (B, k * s), dt, dev)
    need = monarch_saved_bytes(B, k * p, k, q, s, _dtype_code(x), flags)
    if saved is None and need:
        saved = torch.empty(need, dtype=torch.uint8, device=dev)
    sv_ptr = saved.data_ptr() if saved is not None else 0
    sv_len = saved.numel() * saved.element_size() if saved is not None else 0
    with torch.cuda.device(dev):
        rc = lib().monarch_fwd_save(x.data_ptr(), R.data_ptr(), L.data_ptr(), y.data_ptr(), sv_ptr, sv_len, B, k * p,
                                    k, q, s, _dtype_code(x), _stream_ptr(stream), flags)
    if rc != MONARCH_OK:
        raise MonarchError(rc, "monarch_fwd_save")
    return y, (saved if need else None)


def monarch_bwd_saved(dy: torch.Tensor, x: torch.Tensor, saved: torch.Tensor | None, R: torch.Tensor, L: torch.Tensor,
                      dx: torch.Tensor | None = None, dR: torch.Tensor | None = None, dL: torch.Tensor | None = None,
                      dbias: torch.Tensor | None = None, want_dbias: bool = False,
                      workspace: torch.Tensor | None = None, flags: int = 0, stream=None):
    """(dx, dR, dL, dbias or None) with the vector saved by monarch_fwd_save (None: recompute)."""
    k, q, p = R.shape
    s = L.shape[1]
    B = x.shape[0]
    dev, dt = x.device, x.dtype
    _check(x, "x", (B, k * p), dt, dev)
    _check(dy, "dy", (B, k * s), dt, dev)
    _check(R, "R", (k, q, p), dt, dev)
    _check(L, "L", (k, s, q), dt, dev)
    gdt = torch.float32 if (flags & MONARCH_FLAG_WGRAD_F32) else dt
    if dx is None:
        dx = torch.empty_like(x)
    if dR is None:
        dR = torch.empty((k, q, p), dtype=gdt, device=dev)
    if dL is None:
        dL = torch.empty((k, s, q), dtype=gdt, device=dev)
    if dbias is None and want_dbias:
        dbias = torch.empty((k * s,), dtype=gdt, device=dev)
    _check(dx, "dx", (B, k * p), dt, dev)
    _check(dR, "dR", (k, q, p), gdt, dev)
    _check(dL, "dL", (k, s, q), gdt, dev)
    if dbias is not None:
        _check(dbias, "dbias", (k * s,), gdt, dev)
    need = monarch_bwd_workspace_bytes(B, k * p, k, q, s, _dtype_code(x), flags)
    if workspace is None and need:
        workspace = _scratch(need, dev, stream)
    ws_ptr = workspace.data_ptr() if workspace is not None else 0
    ws_len = workspace.numel() * workspace.element_size() if workspace is not None else 0
    sv_ptr = saved.data_ptr() if saved is not None else 0
    sv_len = saved.numel() * saved.element_size() if saved is not None else 0
    with torch.cuda.device(dev):
        rc = lib().monarch_bwd_saved(dy.data_ptr(), x.data_ptr(), sv_ptr, sv_len, R.data_ptr(), L.data_ptr(),
                                     dx.data_ptr(), dR.data_ptr(), dL.data_ptr(),
                                     dbias.data_ptr() if dbias is not None else 0, B, k * p, k, q, s,
                                     _dtype_code(x), _stream_ptr(stream), ws_ptr, ws_len, flags)
    if rc != MONARCH_OK:
        raise MonarchError(rc, "monarch_bwd_saved")
    return dx, dR, dL, dbias


def monarch_fwd_c64(x: torch.Tensor, R: torch.Tensor, L: torch.Tensor, y: torch.Tensor | None = None,
                    flags: int = 0, stream=None) -> torch.Tensor:
    """y = x M^T for complex64 tensors (same shapes as monarch_fwd)."""
    k, q, p = R.shape
    s = L.shape[1]
    B = x.shape[0]
    dev, dt = x.device, torch.complex64
    _check(x, "x", (B, k * p), dt, dev)
    _check(R, "R", (k, q, p), dt, dev)
    _check(L, "L", (k, s, q), dt, dev)
    if y is None:
        y = torch.empty((B, k * s), dtype=dt, device=dev)
    _check(y, "y", (B, k * s), dt, dev)
    with torch.cuda.device(dev):
        rc = lib().monarch_fwd_c64(x.data_ptr(), R.data_ptr(), L.data_ptr(), y.data_ptr(), B, k * p, k, q, s,
                                   _stream_ptr(stream), flags)
    if rc != MONARCH_OK:
        raise MonarchError(rc, "monarch_fwd_c64")
    return y


def monarch_fwd_h_c64(x: torch.Tensor, R: torch.Tensor, L: torch.Tensor, y: torch.Tensor | None = None,
                      flags: int = 0, stream=None) -> torch.Tensor:
    """y = x conj(M) (the conjugate transpose applied to every row) for complex64 tensors: x (B, k*s) -> y (B, k*p)."""
    k, q, p = R.shape
    s = L.shape[1]
    B = x.shape[0]
    dev, dt = x.device, torch.complex64
    _check(x, "x", (B, k * s), dt, dev)
    _check(R, "R", (k, q, p), dt, dev)
    _check(L, "L", (k, s, q), dt, dev)
    if y is None:
        y = torch.empty((B, k * p), dtype=dt, device=dev)
    _check(y, "y", (B, k * p), dt, dev)
    with torch.cuda.device(dev):
        rc = lib().monarch_fwd_h_c64(x.data_ptr(), R.data_ptr(), L.data_ptr(), y.data_ptr(), B, k * p, k, q, s,
                                     _stream_ptr(stream), flags)
    if rc != MONARCH_OK:
        raise MonarchError(rc, "monarch_fwd_h_c64")
    return y


def monarch_bwd_c64(dy: torch.Tensor, x: torch.Tensor, R: torch.Tensor, L: torch.Tensor, flags: int = 0, stream=None):
    """(dx, dR, dL) for complex64 tensors, gradients in the dRe + i dIm convention."""
    k, q, p = R.shape
    s = L.shape[1]
    B = x.shape[0]
    dev, dt = x.device, torch.complex64
    _check(x, "x", (B, k * p), dt, dev)
    _check(dy, "dy", (B, k * s), dt, dev)
    _check(R, "R", (k, q, p), dt, dev)
    _check(L, "L", (k, s, q), dt, dev)
    dx, dR, dL = torch.empty_like(x), torch.empty_like(R), torch.empty_like(L)
    with torch.cuda.device(dev):
        rc = lib().monarch_bwd_c64(dy.data_ptr(), x.data_ptr(), R.data_ptr(), L.data_ptr(), dx.data_ptr(),
                                   dR.data_ptr(), dL.data_ptr(), B, k * p, k, q, s, _stream_ptr(stream), flags)
    if rc != MONARCH_OK:
        raise MonarchError(rc, "monarch_bwd_c64")
    return dx, dR, dL


C64_FWD, C64_BWD, C64_FWD_H = 0, 1, 2


def monarch_c64_workspace_bytes(pass_: int, batch: int, n_in: int, k: int, q: int, s: int, flags: int = 0) -> int:
    """Workspace of monarch_fwd_c64_ws (C64_FWD), monarch_bwd_c64_ws (C64_BWD), monarch_fwd_h_c64_ws (C64_FWD_H)."""
    return int(lib().monarch_c64_workspace_bytes(pass_, batch, n_in, k, q, s, flags))


def _c64_apply_ws(name: str, pass_: int, x, R, L, y, workspace, flags, stream):
    k, q, p = R.shape
    s = L.shape[1]
    B = x.shape[0]
    n_from, n_to = (k * s, k * p) if pass_ == C64_FWD_H else (k * p, k * s)
    dev, dt = x.device, torch.complex64
    _check(x, "x", (B, n_from), dt, dev)
    _check(R, "R", (k, q, p), dt, dev)
    _check(L, "L", (k, s, q), dt, dev)
    if y is None:
        y = torch.empty((B, n_to), dtype=dt, device=dev)
    _check(y, "y", (B, n_to), dt, dev)
    if workspace is None:
        workspace = _scratch(max(monarch_c64_workspace_bytes(pass_, B, k * p, k, q, s, flags), 256), dev, stream)
    with torch.cuda.device(dev):
        rc = getattr(lib(), name)(x.data_ptr(), R.data_ptr(), L.data_ptr(), y.data_ptr(), B, k * p, k, q, s,
                                  _stream_ptr(stream), workspace.data_ptr(),
                                  workspace.numel() * workspace.element_size(), flags)
    if rc != MONARCH_OK:
        raise MonarchError(rc, name)
    return y


def monarch_fwd_c64_ws(x: torch.Tensor, R: torch.Tensor, L: torch.Tensor, y: torch.Tensor | None = None,
                       workspace: torch.Tensor | None = None, flags: int = 0, stream=None) -> torch.Tensor:
    """monarch_fwd_c64 with a workspace (allocated when not given): matrix-core kernels for square blocks."""
    return _c64_apply_ws("monarch_fwd_c64_ws", C64_FWD, x, R, L, y, workspace, flags, stream)


def monarch_fwd_h_c64_ws(x: torch.Tensor, R: torch.Tensor, L: torch.Tensor, y: torch.Tensor | None = None,
                         workspace: torch.Tensor | None = None, flags: int = 0, stream=None) -> torch.Tensor:
    """monarch_fwd_h_c64 with a workspace (allocated when not given): matrix-core kernels for square blocks."""
    return _c64_apply_ws("monarch_fwd_h_c64_ws", C64_FWD_H, x, R, L, y, workspace, flags, stream)


def monarch_bwd_c64_ws(dy: torch.Tensor, x: torch.Tensor, R: torch.Tensor, L: torch.Tensor,
                       dx: torch.Tensor | None = None, dR: torch.Tensor | None = None, dL: torch.Tensor | None = None,
                       workspace: torch.Tensor | None = None, flags: int = 0, stream=None):
    """monarch_bwd_c64 with a workspace (allocated when not given): matrix-core kernels for square blocks, else
    the weight gradients contracted by a GEMM over operands kept in the workspace."""
    k, q, p = R.shape
    s = L.shape[1]
    B = x.shape[0]
    dev, dt = x.device, torch.complex64
    _check(x, "x", (B, k * p), dt, dev)
    _check(dy, "dy", (B, k * s), dt, dev)
    _check(R, "R", (k, q, p), dt, dev)
    _check(L, "L", (k, s, q), dt, dev)
    dx = torch.empty_like(x) if dx is None else dx
    dR = torch.empty_like(R) if dR is None else dR
    dL = torch.empty_like(L) if dL is None else dL
    _check(dx, "dx", (B, k * p), dt, dev)
    _check(dR, "dR", (k, q, p), dt, dev)
    _check(dL, "dL", (k, s, q), dt, dev)
    need = monarch_c64_workspace_bytes(C64_BWD, B, k * p, k, q, s, flags)
    if workspace is None:
        workspace = _scratch(max(need, 256), dev, stream)
    with torch.cuda.device(dev):
        rc = lib().monarch_bwd_c64_ws(dy.data_ptr(), x.data_ptr(), R.data_ptr(), L.data_ptr(), dx.data_ptr(),
                                      dR.data_ptr(), dL.data_ptr(), B, k * p, k, q, s, _stream_ptr(stream),
                                      workspace.data_ptr(), workspace.numel() * workspace.element_size(), flags)
    if rc != MONARCH_OK:
        raise MonarchError(rc, "monarch_bwd_c64_ws")
    return dx, dR, dL


def monarch_dft_factors(m: int, inverse: bool = False, device="cuda", stream=None):
    """(R, L): complex64 factors with P L P^T R = F_n P (n = m*m), or its inverse."""
    dev = torch.device(device)
    R = torch.empty((m, m, m), dtype=torch.complex64, device=dev)
    L = torch.empty((m, m, m), dtype=torch.complex64, device=dev)
    with torch.cuda.device(dev):
        rc = lib().monarch_dft_factors(R.data_ptr(), L.data_ptr(), m, 1 if inverse else 0, _stream_ptr(stream))
    if rc != MONARCH_OK:
        raise MonarchError(rc, "monarch_dft_factors")
    return R, L
