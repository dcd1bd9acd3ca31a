"""Thin ctypes binding of the C ABI in include/lmkan.h.

Argument marshalling only: every step of the layer runs in the HIP kernels of
liblmkan.so.  PyTorch appears here only as the owner of device memory and of
the current stream.  There is no CPU fallback: if the library is missing or a
call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "liblmkan.so")

LMKAN_F32, LMKAN_F16, LMKAN_BF16 = 0, 1, 2
LMKAN_LAYOUT_PAPER, LMKAN_LAYOUT_PACKED = 0, 1
LMKAN_FLAG_ACCUMULATE_GRAD_COEF = 1
LMKAN_FLAG_WORKSPACE_HAS_RECORDS = 2
LMKAN_PACK_TILE = 64
LMKAN_MAX_GRID = 64
LMKAN_STATIC_SCRATCH_BYTES = 32 << 20

_TORCH_DTYPE = {LMKAN_F32: torch.float32, LMKAN_F16: torch.float16, LMKAN_BF16: torch.bfloat16}
_DTYPE_CODE = {v: k for k, v in _TORCH_DTYPE.items()}


class LmkanError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = lib().lmkan_status_string(status).decode()
        super().__init__(f"{where}: {msg} (status {status})")


class _Desc(C.Structure):
    _fields_ = [("n_in", C.c_int32), ("n_out", C.c_int32), ("grid", C.c_int32),
                ("spline_order", C.c_int32), ("coef_dtype", C.c_int32),
                ("coef_layout", C.c_int32), ("flags", C.c_int32)]


class _Conv2d(C.Structure):
    _fields_ = [("n", C.c_int32), ("h", C.c_int32), ("w", C.c_int32), ("c_in", C.c_int32),
                ("kh", C.c_int32), ("kw", C.c_int32), ("stride", C.c_int32)]


@dataclass
class Conv2d:
    """Mirror of ``lmkan_conv2d``: channels-last image [n][h][w][c_in], kh x kw windows, no padding."""
    n: int
    h: int
    w: int
    c_in: int
    kh: int
    kw: int
    stride: int

    def c(self) -> _Conv2d:
        return _Conv2d(self.n, self.h, self.w, self.c_in, self.kh, self.kw, self.stride)

    def image_shape(self):
        return (self.n, self.h, self.w, self.c_in)


@dataclass
class LayerDesc:
    """Mirror of ``lmkan_desc``."""
    n_in: int
    n_out: int
    grid: int
    spline_order: int = 2
    coef_dtype: int = LMKAN_F32
    coef_layout: int = LMKAN_LAYOUT_PAPER
    flags: int = 0

    def c(self) -> _Desc:
        return _Desc(self.n_in, self.n_out, self.grid, self.spline_order, self.coef_dtype,
                     self.coef_layout, self.flags)

    @property
    def pairs(self) -> int:
        return self.n_in // 2

    def coef_shape(self):
        return (self.grid + 1, self.grid + 1, self.pairs, self.n_out)


_lib = None


def lib() -> C.CDLL:
    """Load liblmkan.so (built in-tree by ``build.py``); fail loudly if it is absent."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: run `python -m paper_2509_07103_amd.build` "
                          "(the layer has no fallback implementation)")
    L = C.CDLL(LIB_PATH)
    dp = C.POINTER(_Desc)
    L.lmkan_version.restype = C.c_int
    L.lmkan_version.argtypes = []
    L.lmkan_status_string.restype = C.c_char_p
    L.lmkan_status_string.argtypes = [C.c_int]
    L.lmkan_grid.restype = C.c_int
    L.lmkan_grid.argtypes = [C.c_int32, C.c_void_p, C.c_void_p]
    L.lmkan_packed_bytes.restype = C.c_size_t
    L.lmkan_packed_bytes.argtypes = [dp]
    L.lmkan_workspace_bytes.restype = C.c_size_t
    L.lmkan_workspace_bytes.argtypes = [dp, C.c_int64, C.c_int32]
    L.lmkan_pack.restype = C.c_int
    L.lmkan_pack.argtypes = [dp, C.c_void_p, C.c_void_p, C.c_void_p]
    L.lmkan_locate.restype = C.c_int
    L.lmkan_locate.argtypes = [dp, C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p]
    L.lmkan_forward.restype = C.c_int
    L.lmkan_forward.argtypes = [dp, C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                C.c_size_t, C.c_void_p]
    L.lmkan_forward_static.restype = C.c_int
    L.lmkan_forward_static.argtypes = [dp, C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
    L.lmkan_fold.restype = C.c_int
    L.lmkan_fold.argtypes = [dp, C.c_void_p, C.c_float, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
    L.lmkan_hessian_reg.restype = C.c_int
    L.lmkan_hessian_reg.argtypes = [dp, C.c_void_p, C.c_float, C.c_void_p, C.c_void_p, C.c_void_p]
    L.lmkan_backward.restype = C.c_int
    L.lmkan_backward.argtypes = [dp, C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                 C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    L.lmkan_time_next_kernel.restype = C.c_int
    L.lmkan_time_next_kernel.argtypes = [C.c_void_p, C.c_void_p]
    L.lmkan_microbench.restype = C.c_int
    L.lmkan_microbench.argtypes = [C.c_int32, C.c_void_p, C.c_size_t, C.POINTER(C.c_double), C.c_void_p]
    cp = C.POINTER(_Conv2d)
    L.lmkan_conv2d_rows.restype = C.c_int64
    L.lmkan_conv2d_rows.argtypes = [cp, C.POINTER(C.c_int32), C.POINTER(C.c_int32)]
    L.lmkan_conv2d_forward.restype = C.c_int
    L.lmkan_conv2d_forward.argtypes = [dp, cp, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t,
                                       C.c_void_p]
    L.lmkan_conv2d_backward.restype = C.c_int
    L.lmkan_conv2d_backward.argtypes = [dp, cp, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                        C.c_void_p, C.c_size_t, C.c_void_p]
    _lib = L
    return L


def _check(status: int, where: str) -> None:
    if status != 0:
        raise LmkanError(status, where)


def _stream(stream) -> int:
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


def _used_on(stream, *tensors) -> None:
    """Tells torch's caching allocator that `tensors` (what a call allocated itself: the workspace it
    frees on return, the outputs it hands back) are in use on `stream` when that is not the current
    stream: their memory is then not given out again before the work queued there has finished."""
    if stream is None:
        return
    handle = _stream(stream)
    if handle == torch.cuda.current_stream().cuda_stream:
        return
    s = stream if isinstance(stream, torch.cuda.Stream) else torch.cuda.ExternalStream(handle)
    for t in tensors:
        if t is not None:
            t.record_stream(s)


def _dev(t: torch.Tensor | None, dtype, shape, name: str) -> int | None:
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous() or t.dtype != dtype or tuple(t.shape) != tuple(shape):
        raise ValueError(f"{name}: expected contiguous device tensor {dtype} {tuple(shape)}, got "
                         f"{t.dtype} {tuple(t.shape)} on {t.device}")
    return t.data_ptr()


def lmkan_version() -> int:
    return lib().lmkan_version()


def lmkan_status_string(status: int) -> str:
    return lib().lmkan_status_string(status).decode()


def lmkan_grid(grid: int):
    """(nodes[G+1], inv_h[G]) as float32 numpy arrays."""
    n = max(int(grid), 0)
    nodes = np.zeros(n + 1, dtype=np.float32)
    inv_h = np.zeros(n, dtype=np.float32)
    _check(lib().lmkan_grid(grid, nodes.ctypes.data, inv_h.ctypes.data), "lmkan_grid")
    return nodes, inv_h


def lmkan_packed_bytes(desc: LayerDesc) -> int:
    return lib().lmkan_packed_bytes(C.byref(desc.c()))


def lmkan_workspace_bytes(desc: LayerDesc, batch: int, backward: bool, need_grad_x: bool = True,
                          need_grad_coef: bool = True) -> int:
    """Workspace of a forward call, or of a backward call for the gradients it is asked for."""
    if not backward:
        code = 0
    else:
        code = 1 if (need_grad_x and need_grad_coef) else (2 if need_grad_x else 3)
    return lib().lmkan_workspace_bytes(C.byref(desc.c()), batch, code)


def _workspace(desc: LayerDesc, batch: int, backward: bool, device, workspace: torch.Tensor | None = None,
               need_grad_x: bool = True, need_grad_coef: bool = True):
    """(tensor or None, bytes): the caller's workspace when given (any dtype, contiguous, on the device;
    its size goes to the library, which checks it), else a fresh allocation of the size the library asks for."""
    if workspace is not None:
        if not workspace.is_cuda or not workspace.is_contiguous():
            raise ValueError("workspace: expected a contiguous device tensor")
        return workspace, workspace.numel() * workspace.element_size()
    need = lmkan_workspace_bytes(desc, batch, backward, need_grad_x, need_grad_coef)
    if need == 0:
        return None, 0
    ws = torch.empty(need, dtype=torch.uint8, device=device)
    return ws, need


def lmkan_pack(desc: LayerDesc, coef: torch.Tensor, stream=None) -> torch.Tensor:
    """Coefficients [G+1][G+1][K][n_out] -> packed tensor (flat, same dtype)."""
    dt = _TORCH_DTYPE[desc.coef_dtype]
    src = _dev(coef, dt, desc.coef_shape(), "coef")
    nbytes = lmkan_packed_bytes(desc)
    out = torch.empty(nbytes // coef.element_size(), dtype=dt, device=coef.device)
    _check(lib().lmkan_pack(C.byref(desc.c()), src, out.data_ptr(), _stream(stream)), "lmkan_pack")
    _used_on(stream, out)
    return out


def _coef_ptr(desc: LayerDesc, coef: torch.Tensor | None) -> int | None:
    if coef is None:
        return None
    dt = _TORCH_DTYPE[desc.coef_dtype]
    if desc.coef_layout == LMKAN_LAYOUT_PACKED:
        shape = (lmkan_packed_bytes(desc) // (4 if desc.coef_dtype == LMKAN_F32 else 2),)
    else:
        shape = desc.coef_shape()
    return _dev(coef, dt, shape, "coef")


def lmkan_locate(desc: LayerDesc, x: torch.Tensor, stream=None) -> torch.Tensor:
    batch = x.shape[0]
    xp = _dev(x, torch.float32, (batch, desc.n_in), "x")
    cell = torch.empty((batch, desc.pairs), dtype=torch.int32, device=x.device)
    _check(lib().lmkan_locate(C.byref(desc.c()), batch, xp, cell.data_ptr(), _stream(stream)),
           "lmkan_locate")
    _used_on(stream, cell)
    return cell


def lmkan_forward(desc: LayerDesc, x: torch.Tensor, coef: torch.Tensor, y: torch.Tensor | None = None,
                  stream=None, workspace: torch.Tensor | None = None) -> torch.Tensor:
    batch = x.shape[0]
    xp = _dev(x, torch.float32, (batch, desc.n_in), "x")
    cp = _coef_ptr(desc, coef)
    if y is None:
        y = torch.empty((batch, desc.n_out), dtype=torch.float32, device=x.device)
    yp = _dev(y, torch.float32, (batch, desc.n_out), "y")
    ws, wsz = _workspace(desc, batch, False, x.device, workspace)
    _check(lib().lmkan_forward(C.byref(desc.c()), batch, xp, cp, yp,
                               ws.data_ptr() if ws is not None else None, wsz, _stream(stream)),
           "lmkan_forward")
    _used_on(stream, ws, y)
    return y


def lmkan_forward_static(desc: LayerDesc, x: torch.Tensor, coef: torch.Tensor, y: torch.Tensor,
                         stream=None) -> torch.Tensor:
    """lmkan_forward on the library's own static scratch: the caller brings x, coef and y, nothing is allocated."""
    batch = x.shape[0]
    xp = _dev(x, torch.float32, (batch, desc.n_in), "x")
    cp = _coef_ptr(desc, coef)
    yp = _dev(y, torch.float32, (batch, desc.n_out), "y")
    _check(lib().lmkan_forward_static(C.byref(desc.c()), batch, xp, cp, yp, _stream(stream)),
           "lmkan_forward_static")
    return y


def lmkan_backward(desc: LayerDesc, x: torch.Tensor, coef: torch.Tensor | None, grad_y: torch.Tensor,
                   need_grad_x: bool = True, need_grad_coef: bool = True,
                   grad_x: torch.Tensor | None = None, grad_coef: torch.Tensor | None = None,
                   stream=None, workspace: torch.Tensor | None = None):
    """Returns (grad_x or None, grad_coef or None); grad_coef is float32 in the layout of Alg. 1."""
    batch = x.shape[0]
    xp = _dev(x, torch.float32, (batch, desc.n_in), "x")
    cp = _coef_ptr(desc, coef)
    gyp = _dev(grad_y, torch.float32, (batch, desc.n_out), "grad_y")
    if need_grad_x and grad_x is None:
        grad_x = torch.empty((batch, desc.n_in), dtype=torch.float32, device=x.device)
    if need_grad_coef and grad_coef is None:
        if desc.flags & LMKAN_FLAG_ACCUMULATE_GRAD_COEF:
            raise ValueError("accumulating into grad_coef needs an existing grad_coef tensor")
        grad_coef = torch.empty(desc.coef_shape(), dtype=torch.float32, device=x.device)
    gxp = _dev(grad_x, torch.float32, (batch, desc.n_in), "grad_x") if need_grad_x else None
    gcp = _dev(grad_coef, torch.float32, desc.coef_shape(), "grad_coef") if need_grad_coef else None
    ws, wsz = _workspace(desc, batch, True, x.device, workspace, need_grad_x, need_grad_coef)
    _check(lib().lmkan_backward(C.byref(desc.c()), batch, xp, cp, gyp, gxp, gcp,
                                ws.data_ptr() if ws is not None else None, wsz, _stream(stream)),
           "lmkan_backward")
    _used_on(stream, ws, grad_x, grad_coef)
    return (grad_x if need_grad_x else None), (grad_coef if need_grad_coef else None)


def lmkan_time_next_kernel(start: torch.cuda.Event | None, stop: torch.cuda.Event | None) -> None:
    """Arms two timing events (already created: record them once beforehand) for the main kernel of
    the next compute call of this thread; (None, None) disarms."""
    hs = None if start is None else start.cuda_event
    he = None if stop is None else stop.cuda_event
    if (start is not None and not hs) or (stop is not None and not he):
        raise ValueError("the events must exist already: record each once before arming them")
    _check(lib().lmkan_time_next_kernel(hs, he), "lmkan_time_next_kernel")


MICROBENCH = {"hbm_copy_GBps": 0, "hbm_read_GBps": 1, "fma_per_clk_cu": 2, "mfma_fma_per_clk_cu": 3,
              "lds_read_B_per_clk_cu": 4, "lds_write_B_per_clk_cu": 5, "l2_row_gather_B_per_clk_cu": 6,
              "nominal_clock_GHz": 7}


def lmkan_microbench(which: int, scratch: torch.Tensor, stream=None) -> float:
    """One of the machine measurements of ``lmkan_microbench`` (waits for its kernels)."""
    if not scratch.is_cuda or not scratch.is_contiguous():
        raise ValueError("scratch: expected a contiguous device tensor")
    out = C.c_double(0.0)
    _check(lib().lmkan_microbench(which, scratch.data_ptr(), scratch.numel() * scratch.element_size(),
                                  C.byref(out), _stream(stream)), "lmkan_microbench")
    return out.value


def lmkan_conv2d_rows(conv: Conv2d):
    """(rows, out_h, out_w) of the equivalent fully connected layer."""
    oh, ow = C.c_int32(0), C.c_int32(0)
    rows = lib().lmkan_conv2d_rows(C.byref(conv.c()), C.byref(oh), C.byref(ow))
    if rows < 0:
        raise ValueError(f"invalid convolution geometry {conv}")
    return rows, oh.value, ow.value


def lmkan_conv2d_forward(desc: LayerDesc, conv: Conv2d, x: torch.Tensor, coef: torch.Tensor,
                         y: torch.Tensor | None = None, stream=None,
                         workspace: torch.Tensor | None = None) -> torch.Tensor:
    """x[n][h][w][c_in] -> y[n][out_h][out_w][n_out]."""
    rows, oh, ow = lmkan_conv2d_rows(conv)
    xp = _dev(x, torch.float32, conv.image_shape(), "x")
    cp = _coef_ptr(desc, coef)
    if y is None:
        y = torch.empty((conv.n, oh, ow, desc.n_out), dtype=torch.float32, device=x.device)
    yp = _dev(y, torch.float32, (conv.n, oh, ow, desc.n_out), "y")
    ws, wsz = _workspace(desc, rows, False, x.device, workspace)
    _check(lib().lmkan_conv2d_forward(C.byref(desc.c()), C.byref(conv.c()), xp, cp, yp,
                                      ws.data_ptr() if ws is not None else None, wsz, _stream(stream)),
           "lmkan_conv2d_forward")
    _used_on(stream, ws, y)
    return y


def lmkan_conv2d_backward(desc: LayerDesc, conv: Conv2d, x: torch.Tensor, coef: torch.Tensor | None,
                          grad_y: torch.Tensor, need_grad_x: bool = True, need_grad_coef: bool = True,
                          grad_x: torch.Tensor | None = None, grad_coef: torch.Tensor | None = None, stream=None,
                          workspace: torch.Tensor | None = None):
    """Returns (grad_x in the shape of the image or None, grad_coef in the layout of Alg. 1 or None)."""
    rows, oh, ow = lmkan_conv2d_rows(conv)
    xp = _dev(x, torch.float32, conv.image_shape(), "x")
    cp = _coef_ptr(desc, coef)
    gyp = _dev(grad_y, torch.float32, (conv.n, oh, ow, desc.n_out), "grad_y")
    if need_grad_x and grad_x is None:
        grad_x = torch.empty(conv.image_shape(), dtype=torch.float32, device=x.device)
    if need_grad_coef and grad_coef is None:
        if desc.flags & LMKAN_FLAG_ACCUMULATE_GRAD_COEF:
            raise ValueError("accumulating into grad_coef needs an existing grad_coef tensor")
        grad_coef = torch.empty(desc.coef_shape(), dtype=torch.float32, device=x.device)
    gxp = _dev(grad_x, torch.float32, conv.image_shape(), "grad_x") if need_grad_x else None
    gcp = _dev(grad_coef, torch.float32, desc.coef_shape(), "grad_coef") if need_grad_coef else None
    ws, wsz = _workspace(desc, rows, True, x.device, workspace, need_grad_x, need_grad_coef)
    _check(lib().lmkan_conv2d_backward(C.byref(desc.c()), C.byref(conv.c()), xp, cp, gyp, gxp, gcp,
                                       ws.data_ptr() if ws is not None else None, wsz, _stream(stream)),
           "lmkan_conv2d_backward")
    _used_on(stream, ws, grad_x, grad_coef)
    return (grad_x if need_grad_x else None), (grad_coef if need_grad_coef else None)


def lmkan_hessian_reg(desc: LayerDesc, coef: torch.Tensor, scale: float = 1.0, need_value: bool = True,
                      need_grad: bool = True, grad_coef: torch.Tensor | None = None, stream=None):
    """Returns (value tensor of one float64 or None, scale * gradient float32 in the layout of Alg. 1 or None)."""
    cp = _coef_ptr(desc, coef)
    value = torch.empty(1, dtype=torch.float64, device=coef.device) if need_value else None
    if need_grad and grad_coef is None:
        if desc.flags & LMKAN_FLAG_ACCUMULATE_GRAD_COEF:
            raise ValueError("accumulating into grad_coef needs an existing grad_coef tensor")
        grad_coef = torch.empty(desc.coef_shape(), dtype=torch.float32, device=coef.device)
    gcp = _dev(grad_coef, torch.float32, desc.coef_shape(), "grad_coef") if need_grad else None
    _check(lib().lmkan_hessian_reg(C.byref(desc.c()), cp, float(scale),
                                   value.data_ptr() if need_value else None, gcp, _stream(stream)),
           "lmkan_hessian_reg")
    _used_on(stream, value, grad_coef)
    return value, (grad_coef if need_grad else None)


def lmkan_fold(desc: LayerDesc, coef: torch.Tensor, gamma: float = 1.0, lin_w: torch.Tensor | None = None,
               lin_b: torch.Tensor | None = None, out_scale: torch.Tensor | None = None,
               out_shift: torch.Tensor | None = None, stream=None) -> torch.Tensor:
    """Folds, in place, the ReLU-first preconditioning and an output affine into a float32 table."""
    cp = _coef_ptr(desc, coef)
    wp = _dev(lin_w, torch.float32, (desc.n_out, desc.n_in), "lin_w") if lin_w is not None else None
    bp = _dev(lin_b, torch.float32, (desc.n_out,), "lin_b") if lin_b is not None else None
    sp = _dev(out_scale, torch.float32, (desc.n_out,), "out_scale") if out_scale is not None else None
    tp = _dev(out_shift, torch.float32, (desc.n_out,), "out_shift") if out_shift is not None else None
    _check(lib().lmkan_fold(C.byref(desc.c()), cp, float(gamma), wp, bp, sp, tp, _stream(stream)), "lmkan_fold")
    return coef
