"""ctypes access to the CPU oracle in ``lmkan_oracle.c``.

TEST INFRASTRUCTURE ONLY: the tests, the smoke check and the benchmark's
CPU-baseline leg may import this package; the GPU library never does.  This
file only marshals numpy arrays into the C functions; every piece of the
method's arithmetic lives in the C file.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "lmkan_oracle.c")

F32, F16, BF16 = 0, 1, 2


def _lib_path(variant: str) -> str:
    return os.path.join(_HERE, f"liblmkan_oracle{variant}.so")


def build(variant: str = "", force: bool = False) -> str:
    """Compile the oracle with gcc.  ``variant='_clip'`` builds the rejected
    edge-cell reading (-DORACLE_CLIP_EDGE) that one test uses as a foil."""
    out = _lib_path(variant)
    if not force and os.path.exists(out) and os.path.getmtime(out) >= os.path.getmtime(_SRC):
        return out
    cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
           "-Wall", "-Wextra", "-o", out, _SRC, "-lm"]
    if variant == "_clip":
        cmd.insert(1, "-DORACLE_CLIP_EDGE")
    elif variant != "":
        raise ValueError(variant)
    subprocess.run(cmd, check=True)
    return out


_dp = C.POINTER(C.c_double)
_fp = C.POINTER(C.c_float)
_ip = C.POINTER(C.c_int32)


def _ptr(a: np.ndarray, t):
    return a.ctypes.data_as(t)


def _f32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float32)


def _f64(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float64)


class Oracle:
    """One loaded build of the oracle."""

    def __init__(self, variant: str = ""):
        self.lib = C.CDLL(build(variant))
        L = self.lib
        L.oracle_sigma.restype = C.c_double
        L.oracle_sigma.argtypes = [C.c_double]
        L.oracle_grid.argtypes = [C.c_int, _dp]
        L.oracle_grid_f32.argtypes = [C.c_int, _fp]
        L.oracle_locate.argtypes = [C.c_int, _fp, C.c_float]
        L.oracle_locate_sigma.argtypes = [C.c_int, C.c_double]
        L.oracle_basis.restype = C.c_double
        L.oracle_basis.argtypes = [C.c_int, _dp, C.c_int, C.c_double]
        L.oracle_eval2d_def.restype = C.c_double
        L.oracle_eval2d_def.argtypes = [C.c_int, _dp, _dp, C.c_double, C.c_double]
        L.oracle_preamble.argtypes = [C.c_int, _fp, C.c_float, C.c_float, _dp]
        L.oracle_eval2d.restype = C.c_double
        L.oracle_eval2d.argtypes = [C.c_int, _fp, _dp, C.c_float, C.c_float]
        L.oracle_half_bits_to_double.restype = C.c_double
        L.oracle_half_bits_to_double.argtypes = [C.c_uint16]
        L.oracle_bf16_bits_to_double.restype = C.c_double
        L.oracle_bf16_bits_to_double.argtypes = [C.c_uint16]
        L.oracle_forward.argtypes = [C.c_int64, C.c_int, C.c_int, C.c_int, _fp, C.c_void_p,
                                     C.c_int, _dp, C.c_int]
        L.oracle_forward_def.argtypes = [C.c_int64, C.c_int, C.c_int, C.c_int, _fp, C.c_void_p,
                                         C.c_int, _dp]
        L.oracle_locate_batch.argtypes = [C.c_int64, C.c_int, C.c_int, _fp, _ip]
        L.oracle_backward_input.argtypes = [C.c_int64, C.c_int, C.c_int, C.c_int, _fp, C.c_void_p,
                                            C.c_int, _fp, _dp, C.c_int]
        L.oracle_backward_coef_pair.argtypes = [C.c_int64, C.c_int, C.c_int, C.c_int, C.c_int,
                                                _fp, _fp, _dp]
        L.oracle_fold.argtypes = [C.c_int, C.c_int, C.c_int, _fp, C.c_double, _dp, _dp, _dp, _dp, _dp]
        L.oracle_hessian_reg_2d.restype = C.c_double
        L.oracle_hessian_reg_2d.argtypes = [C.c_int, _dp, _dp, _dp]
        L.oracle_hessian_reg.argtypes = [C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_int, _dp, _dp]
        L.oracle_conv2d_patches.argtypes = [C.c_int] * 7 + [_fp, _fp]
        L.oracle_conv2d_patches_adjoint.argtypes = [C.c_int] * 7 + [_dp, _dp]

    # ---- scalars and small pieces -------------------------------------
    def sigma(self, x: float) -> float:
        return self.lib.oracle_sigma(float(x))

    def grid(self, G: int) -> np.ndarray:
        E = np.empty(G + 1, dtype=np.float64)
        if self.lib.oracle_grid(G, _ptr(E, _dp)):
            raise ValueError("oracle_grid rejected G=%d" % G)
        return E

    def grid_f32(self, G: int) -> np.ndarray:
        E = np.empty(G + 1, dtype=np.float32)
        if self.lib.oracle_grid_f32(G, _ptr(E, _fp)):
            raise ValueError("oracle_grid_f32 rejected G=%d" % G)
        return E

    def locate(self, G: int, E32: np.ndarray, x: float) -> int:
        E32 = _f32(E32)
        return self.lib.oracle_locate(G, _ptr(E32, _fp), float(np.float32(x)))

    def locate_sigma(self, G: int, x: float) -> int:
        return self.lib.oracle_locate_sigma(G, float(x))

    def basis(self, G: int, E: np.ndarray, a: int, x: float) -> float:
        E = _f64(E)
        return self.lib.oracle_basis(G, _ptr(E, _dp), a, float(x))

    def eval2d_def(self, G: int, E: np.ndarray, P2: np.ndarray, x1: float, x2: float) -> float:
        E, P2 = _f64(E), _f64(P2)
        assert P2.shape == (G + 1, G + 1)
        return self.lib.oracle_eval2d_def(G, _ptr(E, _dp), _ptr(P2, _dp), float(x1), float(x2))

    def preamble(self, G: int, E32: np.ndarray, x1: float, x2: float):
        E32 = _f32(E32)
        out = np.empty(4, dtype=np.float64)
        cell = self.lib.oracle_preamble(G, _ptr(E32, _fp), float(np.float32(x1)),
                                        float(np.float32(x2)), _ptr(out, _dp))
        return cell, out

    def eval2d(self, G: int, E32: np.ndarray, P2: np.ndarray, x1: float, x2: float) -> float:
        E32, P2 = _f32(E32), _f64(P2)
        assert P2.shape == (G + 1, G + 1)
        return self.lib.oracle_eval2d(G, _ptr(E32, _fp), _ptr(P2, _dp), float(np.float32(x1)),
                                      float(np.float32(x2)))

    def half_bits_to_double(self, h: int) -> float:
        return self.lib.oracle_half_bits_to_double(h)

    def bf16_bits_to_double(self, b: int) -> float:
        return self.lib.oracle_bf16_bits_to_double(b)

    # ---- layer --------------------------------------------------------
    @staticmethod
    def _coef(P: np.ndarray, dtype: int, G: int, K: int, N_out: int) -> np.ndarray:
        want = {F32: np.float32, F16: np.uint16, BF16: np.uint16}[dtype]
        if dtype == F16 and P.dtype == np.float16:
            P = P.view(np.uint16)
        P = np.ascontiguousarray(P)
        assert P.dtype == want, (P.dtype, want)
        assert P.shape == (G + 1, G + 1, K, N_out), P.shape
        return P

    def forward(self, x, P, G: int, dtype: int = F32, threads: int = 1) -> np.ndarray:
        x = _f32(x)
        B, N_in = x.shape
        N_out = P.shape[-1]
        P = self._coef(P, dtype, G, N_in // 2, N_out)
        y = np.empty((B, N_out), dtype=np.float64)
        if self.lib.oracle_forward(B, N_in, N_out, G, _ptr(x, _fp), P.ctypes.data, dtype,
                                   _ptr(y, _dp), threads):
            raise ValueError("oracle_forward rejected its arguments")
        return y

    def forward_def(self, x, P, G: int, dtype: int = F32) -> np.ndarray:
        x = _f32(x)
        B, N_in = x.shape
        N_out = P.shape[-1]
        P = self._coef(P, dtype, G, N_in // 2, N_out)
        y = np.empty((B, N_out), dtype=np.float64)
        if self.lib.oracle_forward_def(B, N_in, N_out, G, _ptr(x, _fp), P.ctypes.data, dtype,
                                       _ptr(y, _dp)):
            raise ValueError("oracle_forward_def rejected its arguments")
        return y

    def locate_batch(self, x, G: int) -> np.ndarray:
        x = _f32(x)
        B, N_in = x.shape
        cell = np.empty((B, N_in // 2), dtype=np.int32)
        if self.lib.oracle_locate_batch(B, N_in, G, _ptr(x, _fp), _ptr(cell, _ip)):
            raise ValueError("oracle_locate_batch rejected its arguments")
        return cell

    def backward_input(self, x, P, gy, G: int, dtype: int = F32, threads: int = 1) -> np.ndarray:
        x, gy = _f32(x), _f32(gy)
        B, N_in = x.shape
        N_out = P.shape[-1]
        assert gy.shape == (B, N_out)
        P = self._coef(P, dtype, G, N_in // 2, N_out)
        gx = np.empty((B, N_in), dtype=np.float64)
        if self.lib.oracle_backward_input(B, N_in, N_out, G, _ptr(x, _fp), P.ctypes.data, dtype,
                                          _ptr(gy, _fp), _ptr(gx, _dp), threads):
            raise ValueError("oracle_backward_input rejected its arguments")
        return gx

    def backward_coef_pair(self, x, gy, G: int, k: int) -> np.ndarray:
        x, gy = _f32(x), _f32(gy)
        B, N_in = x.shape
        N_out = gy.shape[1]
        assert gy.shape[0] == B
        gPk = np.empty((G + 1, G + 1, N_out), dtype=np.float64)
        if self.lib.oracle_backward_coef_pair(B, N_in, N_out, G, k, _ptr(x, _fp), _ptr(gy, _fp),
                                              _ptr(gPk, _dp)):
            raise ValueError("oracle_backward_coef_pair rejected its arguments")
        return gPk

    def fold(self, P, G: int, gamma: float = 1.0, lin_w=None, lin_b=None, scale=None, shift=None) -> np.ndarray:
        """Table of the single layer equal to  scale * (gamma lmKAN + Linear(ReLU(x))) + shift  (float64)."""
        P = _f32(P)
        K, N_out = P.shape[2], P.shape[3]
        opt = lambda v: (None, None) if v is None else (lambda arr: (arr, _ptr(arr, _dp)))(_f64(v))
        (w, wp), (b, bp), (s, sp), (t, tp) = opt(lin_w), opt(lin_b), opt(scale), opt(shift)
        if w is not None:
            assert w.shape == (N_out, 2 * K)
        out = np.empty(P.shape, dtype=np.float64)
        if self.lib.oracle_fold(2 * K, N_out, G, _ptr(P, _fp), float(gamma), wp, bp, sp, tp, _ptr(out, _dp)):
            raise ValueError("oracle_fold rejected its arguments")
        return out

    def hessian_reg_2d(self, G: int, E: np.ndarray, p2: np.ndarray, want_grad: bool = False):
        """Regulariser of one 2-D table p2[G+1][G+1] on the grid E (any increasing points)."""
        E, p2 = _f64(E), _f64(p2)
        assert E.shape == (G + 1,) and p2.shape == (G + 1, G + 1)
        if not want_grad:
            return self.lib.oracle_hessian_reg_2d(G, _ptr(E, _dp), _ptr(p2, _dp), None)
        g = np.zeros((G + 1, G + 1), dtype=np.float64)
        v = self.lib.oracle_hessian_reg_2d(G, _ptr(E, _dp), _ptr(p2, _dp), _ptr(g, _dp))
        return v, g

    def hessian_reg(self, P, G: int, dtype: int = F32, want_grad: bool = True):
        """Regulariser of a layer (sum over pairs and outputs) and its gradient w.r.t. P."""
        K, N_out = P.shape[2], P.shape[3]
        P = self._coef(P, dtype, G, K, N_out)
        value = np.zeros(1, dtype=np.float64)
        grad = np.empty((G + 1, G + 1, K, N_out), dtype=np.float64) if want_grad else None
        if self.lib.oracle_hessian_reg(2 * K, N_out, G, P.ctypes.data, dtype, _ptr(value, _dp),
                                       _ptr(grad, _dp) if want_grad else None):
            raise ValueError("oracle_hessian_reg rejected its arguments")
        return float(value[0]), grad

    # ---- convolution = fully connected layer on patches (Sec. 5) -------

    @staticmethod
    def conv2d_out_hw(H: int, W: int, kh: int, kw: int, stride: int):
        return (H - kh) // stride + 1, (W - kw) // stride + 1

    def conv2d_patches(self, x, kh: int, kw: int, stride: int) -> np.ndarray:
        """x[N][H][W][C] -> patches[N*OH*OW][kh*kw*C] (float32 copy of the inputs, no arithmetic)."""
        x = _f32(x)
        N, H, W, Cc = x.shape
        OH, OW = self.conv2d_out_hw(H, W, kh, kw, stride)
        out = np.empty((N * OH * OW, kh * kw * Cc), dtype=np.float32)
        if self.lib.oracle_conv2d_patches(N, H, W, Cc, kh, kw, stride, _ptr(x, _fp), _ptr(out, _fp)):
            raise ValueError("oracle_conv2d_patches rejected its arguments")
        return out

    def conv2d_patches_adjoint(self, g_patches, shape, kh: int, kw: int, stride: int) -> np.ndarray:
        """Gradient w.r.t. the image from the gradient w.r.t. its patches (float64)."""
        N, H, W, Cc = shape
        g = _f64(g_patches)
        OH, OW = self.conv2d_out_hw(H, W, kh, kw, stride)
        assert g.shape == (N * OH * OW, kh * kw * Cc)
        out = np.empty((N, H, W, Cc), dtype=np.float64)
        if self.lib.oracle_conv2d_patches_adjoint(N, H, W, Cc, kh, kw, stride, _ptr(g, _dp), _ptr(out, _dp)):
            raise ValueError("oracle_conv2d_patches_adjoint rejected its arguments")
        return out

    def conv2d_forward(self, x, P, G: int, kh: int, kw: int, stride: int, dtype: int = F32,
                       threads: int = 1) -> np.ndarray:
        """y[N][OH][OW][C_out]: the layer applied to every window."""
        N, H, W, _ = np.shape(x)
        OH, OW = self.conv2d_out_hw(H, W, kh, kw, stride)
        y = self.forward(self.conv2d_patches(x, kh, kw, stride), P, G, dtype=dtype, threads=threads)
        return y.reshape(N, OH, OW, -1)

    def conv2d_backward_input(self, x, P, gy, G: int, kh: int, kw: int, stride: int, dtype: int = F32,
                              threads: int = 1) -> np.ndarray:
        shape = np.shape(x)
        gy2 = _f32(gy).reshape(-1, np.shape(gy)[-1])
        gp = self.backward_input(self.conv2d_patches(x, kh, kw, stride), P, gy2, G, dtype=dtype, threads=threads)
        return self.conv2d_patches_adjoint(gp, shape, kh, kw, stride)

    def conv2d_backward_coef(self, x, gy, G: int, kh: int, kw: int, stride: int) -> np.ndarray:
        gy2 = _f32(gy).reshape(-1, np.shape(gy)[-1])
        return self.backward_coef(self.conv2d_patches(x, kh, kw, stride), gy2, G)

    def backward_coef(self, x, gy, G: int) -> np.ndarray:
        """All pairs, assembled into the layout of Alg. 1: [G+1][G+1][K][N_out]."""
        x = _f32(x)
        K = x.shape[1] // 2
        slabs = [self.backward_coef_pair(x, gy, G, k) for k in range(K)]
        return np.stack(slabs, axis=2)


_default = None


def get() -> Oracle:
    global _default
    if _default is None:
        _default = Oracle("")
    return _default
