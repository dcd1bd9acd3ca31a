"""Pins for the oracle's convolution (Sec. 5, "lmKAN-based Convolutional Neural Networks": a
kh x kw convolution is a fully connected layer R^{kh kw C_in} -> R^{C_out} on every window).

The oracle gathers patches with explicit loops and then calls its fully connected functions;
these tests fix the gathering and its adjoint against formulations that do not share those
loops: numpy reshapes for non-overlapping windows, numpy's sliding-window view for
overlapping ones, the inner-product identity of an adjoint, a direct per-window evaluation
through the 2-D evaluator, and finite differences of the convolution output."""
import numpy as np
import pytest
from numpy.lib.stride_tricks import sliding_window_view


def test_1x1_convolution_is_the_layer_on_pixel_rows(oracle):
    rng = np.random.default_rng(0)
    x = rng.normal(size=(2, 3, 5, 4)).astype(np.float32)
    np.testing.assert_array_equal(oracle.conv2d_patches(x, 1, 1, 1), x.reshape(-1, 4))


@pytest.mark.parametrize("k,H,W", [(2, 8, 6), (3, 9, 9), (2, 7, 5), (3, 10, 8)])
def test_stride_k_windows_are_a_reshape(oracle, k, H, W):
    """Non-overlapping windows (the backbones of Sec. 5: 2x2 stride 2, 3x3 stride 3); rows or
    columns that do not fill a window are dropped."""
    rng = np.random.default_rng(k * 100 + H)
    N, C = 3, 4
    x = rng.normal(size=(N, H, W, C)).astype(np.float32)
    OH, OW = H // k, W // k
    want = (x[:, :OH * k, :OW * k].reshape(N, OH, k, OW, k, C).transpose(0, 1, 3, 2, 4, 5)
            .reshape(N * OH * OW, k * k * C))
    np.testing.assert_array_equal(oracle.conv2d_patches(x, k, k, k), want)


@pytest.mark.parametrize("kh,kw,stride", [(3, 3, 1), (3, 2, 2), (2, 3, 1), (4, 4, 3)])
def test_overlapping_windows_match_the_sliding_window_view(oracle, kh, kw, stride):
    rng = np.random.default_rng(kh * 10 + kw + stride)
    N, H, W, C = 2, 9, 8, 2
    x = rng.normal(size=(N, H, W, C)).astype(np.float32)
    v = sliding_window_view(x, (kh, kw), axis=(1, 2))[:, ::stride, ::stride]   # [N][OH][OW][C][kh][kw]
    want = v.transpose(0, 1, 2, 4, 5, 3).reshape(-1, kh * kw * C)
    got = oracle.conv2d_patches(x, kh, kw, stride)
    assert got.shape == want.shape == (N * np.prod(oracle.conv2d_out_hw(H, W, kh, kw, stride)), kh * kw * C)
    np.testing.assert_array_equal(got, want)


@pytest.mark.parametrize("kh,kw,stride,H,W", [(3, 3, 1, 7, 6), (2, 2, 2, 7, 5), (3, 2, 2, 8, 9), (3, 3, 3, 9, 9)])
def test_adjoint_identity(oracle, kh, kw, stride, H, W):
    """<patches(x), g> = <x, adjoint(g)> for arbitrary x and g, and the adjoint counts how many
    windows contain each element (g = 1)."""
    rng = np.random.default_rng(H * 10 + W)
    N, C = 2, 4
    x = rng.normal(size=(N, H, W, C)).astype(np.float32)
    p = oracle.conv2d_patches(x, kh, kw, stride).astype(np.float64)
    g = rng.normal(size=p.shape)
    a = oracle.conv2d_patches_adjoint(g, x.shape, kh, kw, stride)
    assert np.sum(p * g) == pytest.approx(np.sum(x.astype(np.float64) * a), rel=1e-12)
    count = oracle.conv2d_patches_adjoint(np.ones_like(g), x.shape, kh, kw, stride)
    OH, OW = oracle.conv2d_out_hw(H, W, kh, kw, stride)
    cy = np.zeros(H)
    for oy in range(OH):
        cy[oy * stride:oy * stride + kh] += 1
    cx = np.zeros(W)
    for ox in range(OW):
        cx[ox * stride:ox * stride + kw] += 1
    np.testing.assert_array_equal(count, np.broadcast_to((cy[:, None] * cx[None, :])[None, :, :, None], x.shape))


def test_forward_equals_direct_window_evaluation(oracle):
    """One output pixel at a time: the sum over window positions and channel pairs of the 2-D
    functions, with the window read straight from the image."""
    rng = np.random.default_rng(5)
    G, N, H, W, C, kh, kw, stride, n_out = 6, 2, 5, 6, 2, 2, 3, 1, 3
    x = rng.normal(size=(N, H, W, C)).astype(np.float32)
    K = kh * kw * C // 2
    P = rng.normal(size=(G + 1, G + 1, K, n_out)).astype(np.float32)
    y = oracle.conv2d_forward(x, P, G, kh, kw, stride)
    OH, OW = oracle.conv2d_out_hw(H, W, kh, kw, stride)
    assert y.shape == (N, OH, OW, n_out)
    E32 = oracle.grid_f32(G)
    for img, oy, ox in [(0, 0, 0), (1, OH - 1, OW - 1), (0, 2, 1), (1, 0, 3)]:
        for j in range(n_out):
            acc = 0.0
            for ky in range(kh):
                for kx in range(kw):
                    for cp in range(C // 2):
                        k = ((ky * kw + kx) * C + 2 * cp) // 2
                        px = x[img, oy * stride + ky, ox * stride + kx]
                        acc += oracle.eval2d(G, E32, np.ascontiguousarray(P[:, :, k, j].astype(np.float64)),
                                             float(px[2 * cp]), float(px[2 * cp + 1]))
            assert y[img, oy, ox, j] == pytest.approx(acc, rel=1e-12, abs=1e-12)


def test_input_gradient_by_finite_differences(oracle):
    """Overlapping windows: an image element feeds several outputs and its gradient is their sum."""
    rng = np.random.default_rng(6)
    G, N, H, W, C, kh, kw, stride, n_out = 8, 1, 5, 5, 2, 3, 3, 1, 2
    x = (0.6 * rng.normal(size=(N, H, W, C))).astype(np.float32)
    P = rng.normal(size=(G + 1, G + 1, kh * kw * C // 2, n_out)).astype(np.float32)
    OH, OW = oracle.conv2d_out_hw(H, W, kh, kw, stride)
    gy = rng.normal(size=(N, OH, OW, n_out)).astype(np.float32)
    gx = oracle.conv2d_backward_input(x, P, gy, G, kh, kw, stride)
    E = oracle.grid_f32(G).astype(np.float64)
    h = 2.0 ** -12
    checked = 0
    for idx in [(0, 2, 2, 0), (0, 0, 0, 1), (0, 4, 3, 0), (0, 1, 3, 1), (0, 2, 0, 0)]:
        if np.min(np.abs(E - x[idx])) < 4 * h:      # a kink inside the difference stencil
            continue
        xp, xm = x.copy(), x.copy()
        xp[idx] += h
        xm[idx] -= h
        step = float(xp[idx]) - float(xm[idx])
        d = (oracle.conv2d_forward(xp, P, G, kh, kw, stride) - oracle.conv2d_forward(xm, P, G, kh, kw, stride)) / step
        assert gx[idx] == pytest.approx(np.sum(d * gy.astype(np.float64)), rel=1e-6, abs=1e-9)
        checked += 1
    assert checked >= 3


def test_coefficient_gradient_is_the_adjoint_of_forward(oracle):
    """The output is linear in the table: <conv(x; Q), gy> = <Q, grad_P> for any table Q."""
    rng = np.random.default_rng(7)
    G, N, H, W, C, kh, kw, stride, n_out = 5, 2, 4, 6, 2, 2, 2, 2, 3
    x = rng.normal(size=(N, H, W, C)).astype(np.float32)
    OH, OW = oracle.conv2d_out_hw(H, W, kh, kw, stride)
    gy = rng.normal(size=(N, OH, OW, n_out)).astype(np.float32)
    gP = oracle.conv2d_backward_coef(x, gy, G, kh, kw, stride)
    Q = rng.normal(size=gP.shape).astype(np.float32)
    lhs = np.sum(oracle.conv2d_forward(x, Q, G, kh, kw, stride) * gy.astype(np.float64))
    assert lhs == pytest.approx(np.sum(Q.astype(np.float64) * gP), rel=1e-10)
