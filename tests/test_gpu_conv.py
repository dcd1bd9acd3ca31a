"""GPU parity of the convolution (Sec. 5: a kh x kw lmKAN convolution is the layer applied to
every window) against the oracle, which gathers the windows into rows and calls its fully
connected functions.  The library never writes the rows out, so these tests are what checks
its window map: forward, the input gradient (summed over overlapping windows, zero outside
every window) and the coefficient gradient, on every kernel family the dispatch can pick."""
import os

import numpy as np
import pytest
import torch

import paper_2509_07103_amd as pkg
from paper_2509_07103_amd import workloads as wl
from parity_util import ORACLE_DTYPE, TOL_F32, TOL_HALF, bits, pair_slice_rel_err, rowwise_rel_err

pytestmark = pytest.mark.gpu

DT_CODE = {"f32": pkg.LMKAN_F32, "f16": pkg.LMKAN_F16, "bf16": pkg.LMKAN_BF16}


@pytest.fixture(scope="module")
def dev():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    pkg.lib()
    return torch.device("cuda:0")


CASES = [
    # N, H, W, C, kh, kw, stride, n_out, G          rows  kernels
    (4, 32, 32, 6, 2, 2, 2, 16, 8),     # 1024  slab; the 2x2 stride-2 stage of the CIFAR-like backbone
    (5, 32, 32, 3, 2, 2, 2, 12, 12),    # 1280  slab; odd channel count: pairs straddle pixels
    (3, 27, 27, 4, 3, 3, 3, 20, 16),    # 243   generic (few rows); the 3x3 stride-3 stage
    (7, 27, 27, 4, 3, 3, 3, 20, 16),    # 567   slab
    (2, 13, 11, 2, 3, 3, 1, 8, 8),      # 198   small outputs, overlapping windows
    (6, 12, 14, 4, 3, 2, 2, 5, 6),      # 180   small outputs, ragged: last row / column outside every window
    (2, 20, 20, 2, 3, 3, 1, 24, 10),    # 648   slab, overlapping windows
    (3, 9, 10, 2, 2, 2, 1, 10, 5),      # 216   generic (10 outputs), overlapping: atomics into the image
    (2, 16, 16, 8, 1, 1, 1, 32, 16),    # 512   1x1: the layer on pixel rows
    (1, 4, 4, 2, 4, 4, 4, 6, 4),        # 1     one window
    (5, 18, 18, 4, 3, 3, 1, 20, 20),    # 1280  16-output slabs (G > 16), overlapping windows
    (3, 20, 20, 2, 2, 2, 2, 24, 24),    # 300   16-output slabs, rows not a multiple of 64
    (3, 21, 20, 2, 2, 2, 2, 64, 8),     # 300   64-output slabs, rows not a multiple of 64, a row of pixels left over
    (4, 32, 32, 6, 2, 2, 2, 10, 8),     # 1024  slab with a ten-way head (packed table), generic in the layout of Alg. 1
    (2, 24, 24, 4, 3, 3, 1, 18, 20),    # 968   16-output slabs, output count not a multiple of four, overlapping windows
]


def _inputs(case, seed, dev):
    N, H, W, C, kh, kw, stride, n_out, G = case
    g = torch.Generator(device="cpu").manual_seed(seed)
    x = torch.randn((N, H, W, C), generator=g)
    K = kh * kw * C // 2
    P = torch.randn((G + 1, G + 1, K, n_out), generator=g) * 0.1
    conv = pkg.Conv2d(N, H, W, C, kh, kw, stride)
    rows, oh, ow = pkg.lmkan_conv2d_rows(conv)
    gy = torch.randn((N, oh, ow, n_out), generator=g)
    return conv, x.to(dev), P.to(dev), gy.to(dev)


def _image_rel_err(got, want):
    """Per image, max |got - want| / max |want|."""
    return rowwise_rel_err(got.reshape(got.shape[0], -1), want.reshape(want.shape[0], -1))


@pytest.mark.parametrize("layout", [pkg.LMKAN_LAYOUT_PAPER, pkg.LMKAN_LAYOUT_PACKED])
@pytest.mark.parametrize("case", CASES)
def test_conv2d_f32(dev, oracle, case, layout):
    N, H, W, C, kh, kw, stride, n_out, G = case
    conv, x, P, gy = _inputs(case, 21, dev)
    desc = pkg.LayerDesc(kh * kw * C, n_out, G, coef_layout=layout)
    Pd = pkg.lmkan_pack(pkg.LayerDesc(kh * kw * C, n_out, G), P) if layout == pkg.LMKAN_LAYOUT_PACKED else P
    xh, Ph, gyh = x.cpu().numpy(), P.cpu().numpy(), gy.cpu().numpy()

    y = pkg.lmkan_conv2d_forward(desc, conv, x, Pd)
    torch.cuda.synchronize()
    want = oracle.conv2d_forward(xh, Ph, G, kh, kw, stride)
    assert tuple(y.shape) == want.shape
    got = y.cpu().numpy().reshape(-1, n_out)
    want2 = want.reshape(-1, n_out)
    if n_out >= 16:
        assert rowwise_rel_err(got, want2) <= TOL_F32
    else:
        assert np.abs(got - want2).max() <= TOL_F32 * np.abs(want2).max()

    gx, gP = pkg.lmkan_conv2d_backward(desc, conv, x, Pd, gy)
    torch.cuda.synchronize()
    want_gx = oracle.conv2d_backward_input(xh, Ph, gyh, G, kh, kw, stride)
    assert tuple(gx.shape) == (N, H, W, C)
    assert _image_rel_err(gx.cpu().numpy(), want_gx) <= TOL_F32
    # elements outside every window: exact zeros
    assert np.all(gx.cpu().numpy()[want_gx == 0.0] == 0.0)
    want_gP = oracle.conv2d_backward_coef(xh, gyh, G, kh, kw, stride)
    got_gP = gP.cpu().numpy()
    for k in range(want_gP.shape[2]):
        assert pair_slice_rel_err(got_gP[:, :, k, :], want_gP[:, :, k, :]) <= TOL_F32
    assert np.all(got_gP[want_gP == 0.0] == 0.0)


@pytest.mark.parametrize("storage", ["f16", "bf16"])
@pytest.mark.parametrize("case", [CASES[0], CASES[1], CASES[3], CASES[4], CASES[7],
                                  (3, 20, 20, 2, 2, 2, 2, 24, 24)])   # 16-output slabs (G = 24)
def test_conv2d_half_storage(dev, oracle, case, storage):
    N, H, W, C, kh, kw, stride, n_out, G = case
    conv, x, P, gy = _inputs(case, 22, dev)
    paper = pkg.LayerDesc(kh * kw * C, n_out, G, coef_dtype=DT_CODE[storage])
    packed = pkg.LayerDesc(kh * kw * C, n_out, G, coef_dtype=DT_CODE[storage], coef_layout=pkg.LMKAN_LAYOUT_PACKED)
    Ps = wl.store(P, storage).contiguous()
    Pp = pkg.lmkan_pack(paper, Ps)
    xh, gyh = x.cpu().numpy(), gy.cpu().numpy()
    code = ORACLE_DTYPE[storage]

    y = pkg.lmkan_conv2d_forward(packed, conv, x, Pp)
    gx, gP = pkg.lmkan_conv2d_backward(packed, conv, x, Pp, gy)
    torch.cuda.synchronize()
    want = oracle.conv2d_forward(xh, bits(Ps), G, kh, kw, stride, dtype=code).reshape(-1, n_out)
    master = oracle.conv2d_forward(xh, P.cpu().numpy(), G, kh, kw, stride).reshape(-1, n_out)
    got = y.cpu().numpy().reshape(-1, n_out)
    assert np.abs(got - want).max() <= TOL_F32 * np.abs(want).max()
    assert np.abs(got - master).max() <= TOL_HALF * np.abs(master).max()
    want_gx = oracle.conv2d_backward_input(xh, bits(Ps), gyh, G, kh, kw, stride, dtype=code)
    assert _image_rel_err(gx.cpu().numpy(), want_gx) <= TOL_F32
    want_gP = oracle.conv2d_backward_coef(xh, gyh, G, kh, kw, stride)
    got_gP = gP.cpu().numpy()
    for k in range(want_gP.shape[2]):
        assert pair_slice_rel_err(got_gP[:, :, k, :], want_gP[:, :, k, :]) <= TOL_F32


def test_conv2d_equals_the_layer_on_gathered_rows(dev, oracle):
    """The library against itself: convolution = lmkan_forward / lmkan_backward on the rows the
    oracle's gathering writes out (which the library never does)."""
    case = (4, 24, 24, 4, 3, 3, 3, 32, 16)
    N, H, W, C, kh, kw, stride, n_out, G = case
    conv, x, P, gy = _inputs(case, 23, dev)
    desc = pkg.LayerDesc(kh * kw * C, n_out, G)
    rows = torch.from_numpy(oracle.conv2d_patches(x.cpu().numpy(), kh, kw, stride)).to(dev)
    y = pkg.lmkan_conv2d_forward(desc, conv, x, P)
    y_rows = pkg.lmkan_forward(desc, rows, P)
    gx, gP = pkg.lmkan_conv2d_backward(desc, conv, x, P, gy)
    gx_rows, gP_rows = pkg.lmkan_backward(desc, rows, P, gy.reshape(-1, n_out).contiguous())
    torch.cuda.synchronize()
    assert torch.equal(y.reshape(-1, n_out), y_rows)
    # stride = window: every image element sits in exactly one window, so grad_x is a permutation
    back = oracle.conv2d_patches_adjoint(gx_rows.cpu().numpy(), (N, H, W, C), kh, kw, stride)
    np.testing.assert_array_equal(gx.cpu().numpy().astype(np.float64), back)
    np.testing.assert_allclose(gP.cpu().numpy(), gP_rows.cpu().numpy(), rtol=0, atol=1e-5 * float(gP_rows.abs().max()))


def test_conv2d_image_smaller_than_window(dev):
    conv = pkg.Conv2d(2, 2, 5, 2, 3, 3, 1)
    desc = pkg.LayerDesc(18, 4, 8)
    x = torch.randn((2, 2, 5, 2), device=dev)
    P = torch.randn(desc.coef_shape(), device=dev)
    y = pkg.lmkan_conv2d_forward(desc, conv, x, P)
    assert tuple(y.shape) == (2, 0, 3, 4)
    gy = torch.empty((2, 0, 3, 4), device=dev)
    gx = torch.full((2, 2, 5, 2), 7.0, device=dev)
    gP = torch.full(desc.coef_shape(), 7.0, device=dev)
    pkg.lmkan_conv2d_backward(desc, conv, x, P, gy, grad_x=gx, grad_coef=gP)
    torch.cuda.synchronize()
    assert float(gx.abs().max()) == 0.0 and float(gP.abs().max()) == 0.0


def test_conv2d_accumulates_coefficient_gradient(dev, oracle):
    case = CASES[0]
    N, H, W, C, kh, kw, stride, n_out, G = case
    conv, x, P, gy = _inputs(case, 24, dev)
    acc = pkg.LayerDesc(kh * kw * C, n_out, G, flags=pkg.LMKAN_FLAG_ACCUMULATE_GRAD_COEF)
    base = torch.randn(acc.coef_shape(), device=dev)
    gP = base.clone()
    pkg.lmkan_conv2d_backward(acc, conv, x, P, gy, need_grad_x=False, grad_coef=gP)
    torch.cuda.synchronize()
    want = base.cpu().numpy().astype(np.float64) + oracle.conv2d_backward_coef(x.cpu().numpy(), gy.cpu().numpy(), G, kh, kw, stride)
    assert np.abs(gP.cpu().numpy() - want).max() <= TOL_F32 * np.abs(want).max()


def _random_geometries(n, seed):
    """Seeded draws of image, window, stride, output count, grid, storage and layout.  A third of
    the draws have enough windows (256 and more) for the slab kernels."""
    rng = np.random.RandomState(seed)
    out = []
    while len(out) < n:
        kh, kw = int(rng.randint(1, 5)), int(rng.randint(1, 5))
        C = int(rng.randint(1, 9))
        if (kh * kw * C) % 2:
            continue
        stride = int(rng.randint(1, 4))
        H, W = kh + int(rng.randint(0, 22)), kw + int(rng.randint(0, 22))
        N = int(rng.randint(1, 7)) if len(out) % 3 else int(rng.randint(6, 12))
        n_out = int(rng.choice([1, 3, 4, 8, 10, 16, 20, 33, 64, 72]))
        G = int(rng.choice([4, 8, 12, 16, 20, 24, 40]))
        storage = str(rng.choice(["f32", "f32", "f16", "bf16"]))
        layout = int(rng.choice([pkg.LMKAN_LAYOUT_PAPER, pkg.LMKAN_LAYOUT_PACKED]))
        out.append((N, H, W, C, kh, kw, stride, n_out, G, storage, layout))
    return out


GEOMETRIES = _random_geometries(int(os.environ.get("LMKAN_TEST_DRAWS", "48")),
                                int(os.environ.get("LMKAN_TEST_SEED", "20250907")))


@pytest.mark.parametrize("geo", GEOMETRIES, ids=lambda g: "N%d_%dx%dx%d_w%dx%ds%d_to%d_G%d_%s_%s" % (
    g[:10] + ("packed" if g[10] == pkg.LMKAN_LAYOUT_PACKED else "paper",)))
def test_conv2d_random_geometry(dev, oracle, geo):
    N, H, W, C, kh, kw, stride, n_out, G, storage, layout = geo
    conv, x, P, gy = _inputs(geo[:9], 25, dev)
    n_in = kh * kw * C
    desc = pkg.LayerDesc(n_in, n_out, G, coef_dtype=DT_CODE[storage], coef_layout=layout)
    Ps = wl.store(P, storage).contiguous()
    Pd = pkg.lmkan_pack(pkg.LayerDesc(n_in, n_out, G, coef_dtype=DT_CODE[storage]), Ps) \
        if layout == pkg.LMKAN_LAYOUT_PACKED else Ps
    xh, gyh = x.cpu().numpy(), gy.cpu().numpy()
    code = ORACLE_DTYPE[storage]

    y = pkg.lmkan_conv2d_forward(desc, conv, x, Pd)
    gx, gP = pkg.lmkan_conv2d_backward(desc, conv, x, Pd, gy)
    torch.cuda.synchronize()
    want = oracle.conv2d_forward(xh, bits(Ps), G, kh, kw, stride, dtype=code)
    assert tuple(y.shape) == want.shape
    assert np.abs(y.cpu().numpy() - want).max() <= TOL_F32 * np.abs(want).max()
    want_gx = oracle.conv2d_backward_input(xh, bits(Ps), gyh, G, kh, kw, stride, dtype=code)
    assert tuple(gx.shape) == (N, H, W, C)
    assert np.abs(gx.cpu().numpy() - want_gx).max() <= TOL_F32 * np.abs(want_gx).max()
    assert np.all(gx.cpu().numpy()[want_gx == 0.0] == 0.0)
    want_gP = oracle.conv2d_backward_coef(xh, gyh, G, kh, kw, stride)
    got_gP = gP.cpu().numpy()
    for k in range(want_gP.shape[2]):
        assert pair_slice_rel_err(got_gP[:, :, k, :], want_gP[:, :, k, :]) <= TOL_F32
    assert np.all(got_gP[want_gP == 0.0] == 0.0)
