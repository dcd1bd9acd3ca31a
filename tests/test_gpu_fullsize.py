"""GPU parity at the full sizes of the five benchmark configurations, in the launch
configuration bench.py times (packed tables, workspace from lmkan_workspace_bytes).

The oracle cannot finish whole tensors of these sizes in seconds, so it computes sampled
outputs one by one: random rows for forward and the input gradient, random pair slices
(over all rows: a slice of the coefficient gradient depends on one pair only) for the
coefficient gradient.  Cell indices are compared bit for bit on every element.
Tolerances as in the small-shape parity tests (row-wise max norm)."""
import dataclasses

import numpy as np
import pytest
import torch

import paper_2509_07103_amd as pkg
from paper_2509_07103_amd import workloads as wl
from parity_util import ORACLE_DTYPE, TOL_F32, TOL_HALF, bits, pair_slice_rel_err, rowwise_rel_err

pytestmark = pytest.mark.gpu

DT_CODE = {"f32": pkg.LMKAN_F32, "f16": pkg.LMKAN_F16, "bf16": pkg.LMKAN_BF16}
THREADS = 8


@pytest.fixture(scope="module")
def dev():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    pkg.lib()
    return torch.device("cuda:0")


def _descs(w, storage):
    code = DT_CODE[storage]
    return (pkg.LayerDesc(w.n_in, w.n_out, w.grid, coef_dtype=code),
            pkg.LayerDesc(w.n_in, w.n_out, w.grid, coef_dtype=code, coef_layout=pkg.LMKAN_LAYOUT_PACKED))


def _rel_err(got, want):
    """Row-wise max norm; a row of fewer than 16 outputs is too short for its own maximum to be a
    scale (one output is a sum that can cancel to nothing), so such layers take the maximum of
    the whole sampled block as the scale."""
    if want.shape[1] >= 16:
        return rowwise_rel_err(got, want)
    return float(np.abs(got.astype(np.float64) - want).max() / max(np.abs(want).max(), 1e-30))


def _rows(w, count, seed):
    return np.sort(np.random.default_rng(seed).choice(w.batch, size=min(count, w.batch), replace=False))


def _check_layer(w, storage, dev, oracle, n_rows, n_pairs, backward=True, master=True):
    x = wl.make_x(w, dev)
    gy = wl.make_grad_y(w, dev)
    P = wl.make_coef(w, dev)
    Ps = wl.store(P, storage).contiguous()
    paper, packed = _descs(w, storage)
    Pp = pkg.lmkan_pack(paper, Ps)
    G, K = w.grid, w.n_in // 2

    xh = x.cpu().numpy()
    cell = pkg.lmkan_locate(packed, x)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(cell.cpu().numpy(), oracle.locate_batch(xh, G))
    del cell

    rows = _rows(w, n_rows, 100 + w.seed)
    Pbits = bits(Ps)
    Pm = P.cpu().numpy() if (storage != "f32" and master) else None
    code = ORACLE_DTYPE[storage]

    y = pkg.lmkan_forward(packed, x, Pp)
    torch.cuda.synchronize()
    got = y.cpu().numpy()[rows]
    want = oracle.forward(xh[rows], Pbits, G, dtype=code, threads=THREADS)
    assert _rel_err(got, want) <= TOL_F32
    if Pm is not None:
        assert _rel_err(got, oracle.forward(xh[rows], Pm, G, threads=THREADS)) <= TOL_HALF
    if not backward:
        return

    gx, gP = pkg.lmkan_backward(packed, x, Pp, gy)
    torch.cuda.synchronize()
    gyh = gy.cpu().numpy()
    got = gx.cpu().numpy()[rows]
    want = oracle.backward_input(xh[rows], Pbits, gyh[rows], G, dtype=code, threads=THREADS)
    assert rowwise_rel_err(got, want) <= TOL_F32
    if Pm is not None:
        ref = oracle.backward_input(xh[rows], Pm, gyh[rows], G, threads=THREADS)
        assert np.linalg.norm(got.astype(np.float64) - ref) <= TOL_HALF * np.linalg.norm(ref)
    assert tuple(gP.shape) == (G + 1, G + 1, K, w.n_out)
    pairs = np.random.default_rng(200 + w.seed).choice(K, size=min(n_pairs, K), replace=False)
    for k in pairs:
        got_k = gP[:, :, int(k), :].cpu().numpy()
        want_k = oracle.backward_coef_pair(xh, gyh, G, int(k))
        assert pair_slice_rel_err(got_k, want_k) <= TOL_F32
        assert np.all(got_k[want_k == 0.0] == 0.0)   # untouched entries: exact zeros (Sec. 3.5)


def test_cfg1_whole(dev, oracle):
    w = wl.CFG1
    _check_layer(w, "f32", dev, oracle, n_rows=w.batch, n_pairs=w.n_in // 2)


@pytest.mark.parametrize("layer", range(len(wl.CFG2_LAYERS)))
def test_cfg2_layers_forward(dev, oracle, layer):
    # each layer of the stack on its own seeded input; batch normalisation between the layers
    # is outside the library
    _check_layer(wl.CFG2_LAYERS[layer], "f32", dev, oracle, n_rows=512, n_pairs=0, backward=False)


def test_cfg2_last_layer_backward(dev, oracle):
    # n_out = 1: the shapes the tuned kernels do not take
    _check_layer(wl.CFG2_LAYERS[3], "f32", dev, oracle, n_rows=256, n_pairs=4)


@pytest.mark.parametrize("storage", ["f32", "f16"])
def test_cfg3_headline(dev, oracle, storage):
    _check_layer(wl.CFG3, storage, dev, oracle, n_rows=256 if storage == "f32" else 128, n_pairs=8)


@pytest.mark.parametrize("grid", [20, 24])
def test_cfg3_shape_on_the_papers_finer_grids(dev, oracle, grid):
    """The cfg3 layer on G = 20 (the grid of the paper's kernel benchmark, appendix on the CUDA
    kernels) and on the largest grid whose float32 table still takes 32-output tiles, in the
    launch configuration `bench.py --grid` times."""
    w = dataclasses.replace(wl.CFG3, grid=grid, name=f"{wl.CFG3.name}@G={grid}")
    _check_layer(w, "f32", dev, oracle, n_rows=128, n_pairs=4)


def test_cfg3_hessian_regulariser(dev, oracle):
    """The regulariser over the whole 606 MB table; the oracle walks all 524288 functions."""
    w = wl.CFG3
    P = wl.make_coef(w, dev)
    paper, packed = _descs(w, "f32")
    Pp = pkg.lmkan_pack(paper, P)
    value, grad = pkg.lmkan_hessian_reg(packed, Pp, scale=1.0)
    torch.cuda.synchronize()
    want_v, want_g = oracle.hessian_reg(P.cpu().numpy(), w.grid)
    assert float(value.cpu()[0]) == pytest.approx(want_v, rel=1e-5)
    got = grad.cpu().numpy()
    for k in np.random.default_rng(300).choice(w.n_in // 2, size=16, replace=False):
        assert pair_slice_rel_err(got[:, :, int(k), :], want_g[:, :, int(k), :]) <= TOL_F32
    # over the whole tensor: the regulariser is a quadratic form of the table, so <grad, P> = 2 value
    euler = float((grad.double() * P.double()).sum())
    assert euler == pytest.approx(2.0 * want_v, rel=1e-5)


def test_cfg4_rows(dev, oracle):
    _check_layer(wl.CFG4, "f32", dev, oracle, n_rows=1024, n_pairs=4)


def test_cfg5_large_table_bf16(dev, oracle):
    """4096 -> 4096, G = 32, bfloat16 table of 18 GB generated on the device; the coefficient
    gradient (36 GB, float32) never leaves the device except for the sampled pair slices."""
    w = wl.CFG5
    torch.cuda.empty_cache()
    free, _ = torch.cuda.mem_get_info()
    if free < 120 * 2**30:
        pytest.skip("needs about 120 GB of free device memory")
    x = wl.make_x(w, dev)
    gy = wl.make_grad_y(w, dev)
    Ps = wl.make_coef_bf16_chunked(w, dev)
    paper, packed = _descs(w, "bf16")
    Pp = pkg.lmkan_pack(paper, Ps)
    G, K = w.grid, w.n_in // 2
    xh, gyh = x.cpu().numpy(), gy.cpu().numpy()

    cell = pkg.lmkan_locate(packed, x)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(cell.cpu().numpy(), oracle.locate_batch(xh, G))
    del cell

    Pbits = bits(Ps)
    del Ps
    rows = _rows(w, 32, 100 + w.seed)
    y = pkg.lmkan_forward(packed, x, Pp)
    torch.cuda.synchronize()
    want = oracle.forward(xh[rows], Pbits, G, dtype=ORACLE_DTYPE["bf16"], threads=THREADS)
    assert rowwise_rel_err(y.cpu().numpy()[rows], want) <= TOL_F32
    del y

    gx, gP = pkg.lmkan_backward(packed, x, Pp, gy)
    torch.cuda.synchronize()
    want = oracle.backward_input(xh[rows], Pbits, gyh[rows], G, dtype=ORACLE_DTYPE["bf16"], threads=THREADS)
    assert rowwise_rel_err(gx.cpu().numpy()[rows], want) <= TOL_F32
    del Pbits
    for k in np.random.default_rng(200 + w.seed).choice(K, size=4, replace=False):
        got_k = gP[:, :, int(k), :].cpu().numpy()
        want_k = oracle.backward_coef_pair(xh, gyh, G, int(k))
        assert pair_slice_rel_err(got_k, want_k) <= TOL_F32
        assert np.all(got_k[want_k == 0.0] == 0.0)
    # every element of the 36 GB gradient enters its moments over the nodes (see the property tests
    # below), taken 128 pairs at a time
    E = torch.from_numpy(pkg.lmkan_grid(G)[0]).to(dev).double()
    gyd = gy.double()
    s0 = gyd.abs().sum(0)[None]
    for k0 in range(0, K, 128):
        g = gP[:, :, k0:k0 + 128, :].double()
        m0 = g.sum(dim=(0, 1))
        m1 = (g * E[:, None, None, None]).sum(dim=(0, 1))
        x1 = x[:, 2 * k0:2 * (k0 + 128):2].double()
        assert float(((m0 - gyd.sum(0)[None]).abs() / s0).max()) <= 1e-5
        assert float(((m1 - x1.T @ gyd).abs() / (x1.abs().T @ gyd.abs())).max()) <= 1e-5
        del g, m0, m1


def test_cfg2_inference_stack_with_folded_normalisation(dev, oracle):
    """The four layers chained for inference (App. F.1): the evaluation-mode batch normalisation
    after each hidden layer, a per-output scale and shift, is folded into that layer's table, so
    the device runs lmKAN -> lmKAN -> lmKAN -> lmKAN with nothing in between; the oracle applies
    the normalisation explicitly in double precision on sampled rows.  The statistics are
    seeded stand-ins for running statistics (scale ~ 1 / expected output deviation)."""
    layers = wl.CFG2_LAYERS
    g = torch.Generator(device="cpu").manual_seed(77)
    x = wl.make_x(layers[0], dev)
    rows = _rows(layers[0], 384, 177)
    a_dev = x
    a_ref = x.cpu().numpy()[rows]
    worst = 0.0
    for i, w in enumerate(layers):
        P = wl.make_coef(w, dev)
        paper, packed = _descs(w, "f32")
        last = i == len(layers) - 1
        if not last:
            scale = (torch.rand((w.n_out,), generator=g) * 0.4 + 0.8) / (w.coef_std * (w.n_in / 2) ** 0.5)
            shift = torch.randn((w.n_out,), generator=g) * 0.2
            folded = P.clone()
            pkg.lmkan_fold(paper, folded, 1.0, None, None, scale.to(dev), shift.to(dev))
        else:
            folded = P
        a_in = a_dev.cpu().numpy()[rows]    # what this layer was given on the device
        a_dev = pkg.lmkan_forward(packed, a_dev, pkg.lmkan_pack(paper, folded))
        torch.cuda.synchronize()
        y = oracle.forward(a_ref, P.cpu().numpy(), w.grid, threads=THREADS)
        # every layer on its own, to the single-layer bar: the oracle is fed the device's own
        # activations, so nothing of the earlier layers' rounding enters the comparison
        y_own = oracle.forward(a_in, P.cpu().numpy(), w.grid, threads=THREADS)
        if not last:
            y = y * scale.numpy().astype(np.float64) + shift.numpy().astype(np.float64)
            y_own = y_own * scale.numpy().astype(np.float64) + shift.numpy().astype(np.float64)
        assert _rel_err(a_dev.cpu().numpy()[rows], y_own) <= TOL_F32, i
        err = _rel_err(a_dev.cpu().numpy()[rows], y)
        worst = max(worst, err)
        # float32 rounding of one layer is ~1e-6 of the row scale; later layers see it magnified by
        # the slope of the next layer's functions summed over its pairs, hence the wider bound
        assert err <= (TOL_F32 if i == 0 else 2e-4), (i, err)
        a_ref = y.astype(np.float32)     # the oracle's own activations feed its next layer
    assert np.isfinite(worst)


# ---------------------------------------------------------------------------------------------
# Properties that hold at any size, checked on EVERY element of the full-size tensors (the sampled
# rows above cover a fraction).  A table that samples an affine function,
#     P[a][b][k][j] = alpha[k][j] E[a] + beta[k][j] E[b] + gamma[k][j],
# is reproduced exactly by piecewise-linear interpolation, inside the grid and beyond the ghost
# points (Sec. 3.1, App. B: every function continues linearly to infinity), so the layer is the
# dense affine map  y = x1 alpha + x2 beta + sum_k gamma,  its input gradient is  gy alpha^T / gy beta^T,
# and, because the four weights of a sample sum to one and interpolate the coordinates,
#     sum_ab gP[a][b][k][j] = sum_n gy[n][j],   sum_ab E[a] gP[a][b][k][j] = sum_n x[n][2k] gy[n][j]
# (and likewise with E[b], x[n][2k+1]) for every table.  The right-hand sides are float64 matrix
# products of the inputs: nothing of the library enters them.
# ---------------------------------------------------------------------------------------------
def _affine_table(w, dev, seed):
    g = torch.Generator(device=dev)
    g.manual_seed(seed)
    K = w.n_in // 2
    alpha = torch.randn((K, w.n_out), generator=g, device=dev) * 0.3
    beta = torch.randn((K, w.n_out), generator=g, device=dev) * 0.3
    gamma = torch.randn((K, w.n_out), generator=g, device=dev) * 0.1
    E = torch.from_numpy(pkg.lmkan_grid(w.grid)[0]).to(dev).double()
    P = (alpha.double()[None, None] * E[:, None, None, None] + beta.double()[None, None] * E[None, :, None, None]
         + gamma.double()[None, None])
    return alpha, beta, gamma, E, P.float().contiguous()


@pytest.mark.parametrize("w", [wl.CFG3, wl.CFG4, wl.CFG2_LAYERS[1]], ids=lambda w: w.name)
def test_affine_table_makes_the_layer_a_dense_affine_map_everywhere(dev, w):
    alpha, beta, gamma, E, P = _affine_table(w, dev, 500 + w.seed)
    paper, packed = _descs(w, "f32")
    Pp = pkg.lmkan_pack(paper, P)
    x = wl.make_x(w, dev) * 1.5            # a good share of the inputs beyond the ghost points
    gy = wl.make_grad_y(w, dev)
    y = pkg.lmkan_forward(packed, x, Pp)
    gx, _ = pkg.lmkan_backward(packed, x, Pp, gy, need_grad_coef=False)
    torch.cuda.synchronize()
    # the table itself is rounded to float32: use the rounded coefficients' own affine law where
    # it matters (interpolation of rounded samples of an affine function is affine up to rounding)
    x1, x2 = x[:, 0::2].double(), x[:, 1::2].double()
    want = x1 @ alpha.double() + x2 @ beta.double() + gamma.double().sum(0)[None]
    scale = want.abs().amax(dim=1, keepdim=True).clamp_min(1e-30)
    assert float(((y.double() - want).abs() / scale).max()) <= 2e-5
    want_g1, want_g2 = gy.double() @ alpha.double().T, gy.double() @ beta.double().T
    got_g1, got_g2 = gx[:, 0::2].double(), gx[:, 1::2].double()
    gscale = torch.maximum(want_g1.abs().amax(dim=1, keepdim=True), want_g2.abs().amax(dim=1, keepdim=True))
    assert float(((got_g1 - want_g1).abs() / gscale).max()) <= 2e-5
    assert float(((got_g2 - want_g2).abs() / gscale).max()) <= 2e-5


@pytest.mark.parametrize("w", [wl.CFG3, wl.CFG4, wl.CFG2_LAYERS[1]], ids=lambda w: w.name)
def test_coefficient_gradient_moments_over_the_whole_tensor(dev, w):
    paper, packed = _descs(w, "f32")
    x = wl.make_x(w, dev)
    gy = wl.make_grad_y(w, dev)
    _, gP = pkg.lmkan_backward(packed, x, None, gy, need_grad_x=False)
    torch.cuda.synchronize()
    E = torch.from_numpy(pkg.lmkan_grid(w.grid)[0]).to(dev).double()
    g = gP.double()
    m0 = g.sum(dim=(0, 1))                                     # [K][n_out]
    m1 = (g * E[:, None, None, None]).sum(dim=(0, 1))
    m2 = (g * E[None, :, None, None]).sum(dim=(0, 1))
    gyd = gy.double()
    want0 = gyd.sum(0)[None].expand_as(m0)
    want1 = x[:, 0::2].double().T @ gyd
    want2 = x[:, 1::2].double().T @ gyd
    # scale: the sum of absolute contributions, which is what float32 rounding acts on
    s0 = gyd.abs().sum(0)[None]
    s1 = x[:, 0::2].double().abs().T @ gyd.abs()
    s2 = x[:, 1::2].double().abs().T @ gyd.abs()
    assert float(((m0 - want0).abs() / s0).max()) <= 1e-5
    assert float(((m1 - want1).abs() / s1).max()) <= 1e-5
    assert float(((m2 - want2).abs() / s2).max()) <= 1e-5


@pytest.mark.parametrize("w", [wl.CONV_2X2, wl.CONV_3X3_S1], ids=lambda w: w.name)
def test_convolution_stages_at_full_size(dev, oracle, w):
    """The bench's convolution stages: every window of a few sampled images against the oracle."""
    x = wl.make_image(w, dev)
    P = wl.make_coef(w, dev)
    oh, ow = w.out_hw
    gy = wl.make_grad_y(w, dev).reshape(w.n, oh, ow, w.n_out)
    conv = pkg.Conv2d(w.n, w.h, w.w, w.c_in, w.kh, w.kw, w.stride)
    paper = pkg.LayerDesc(w.n_in, w.n_out, w.grid)
    packed = pkg.LayerDesc(w.n_in, w.n_out, w.grid, coef_layout=pkg.LMKAN_LAYOUT_PACKED)
    Pp = pkg.lmkan_pack(paper, P)
    y = pkg.lmkan_conv2d_forward(packed, conv, x, Pp)
    gx, gP = pkg.lmkan_conv2d_backward(packed, conv, x, Pp, gy)
    torch.cuda.synchronize()
    imgs = np.sort(np.random.default_rng(w.seed).choice(w.n, size=3, replace=False))
    xh, Ph, gyh = x[imgs].cpu().numpy(), P.cpu().numpy(), gy[imgs].cpu().numpy()
    want = oracle.conv2d_forward(xh, Ph, w.grid, w.kh, w.kw, w.stride, threads=THREADS)
    assert rowwise_rel_err(y[imgs].cpu().numpy().reshape(-1, w.n_out), want.reshape(-1, w.n_out)) <= TOL_F32
    want_gx = oracle.conv2d_backward_input(xh, Ph, gyh, w.grid, w.kh, w.kw, w.stride, threads=THREADS)
    assert rowwise_rel_err(gx[imgs].cpu().numpy().reshape(3, -1), want_gx.reshape(3, -1)) <= TOL_F32
    # the coefficient gradient sums over all images: its zeroth moment is checked over the whole tensor
    m0 = gP.double().sum(dim=(0, 1))
    gyd = gy.reshape(-1, w.n_out).double()
    assert float(((m0 - gyd.sum(0)[None]).abs() / gyd.abs().sum(0)[None]).max()) <= 1e-5
