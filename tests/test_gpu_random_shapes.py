"""GPU parity on shapes drawn at random (seeded): every draw picks a batch, a layer, a grid, a
storage type, a table layout, which gradients are asked for and whether the coefficient gradient
is added to an existing one, so that combinations nobody listed by hand meet the dispatch
(which kernel, which workspace layout) and the oracle.  Sizes are small enough for the oracle;
a quarter of the draws are wide enough (pairs x outputs >= 8192) for the slab kernels to take
short batches, a quarter are middling layers (16 to 158 inputs, 1 to 260 outputs) on either side
of the batch and work thresholds.

LMKAN_TEST_DRAWS and LMKAN_TEST_SEED in the environment replace the number of draws and the seed
(the committed run uses 144 draws of seed 20240917)."""
import os

import numpy as np
import pytest
import torch

import paper_2509_07103_amd as pkg
from paper_2509_07103_amd import workloads as wl
from parity_util import ORACLE_DTYPE, TOL_F32, bits, pair_slice_rel_err, rowwise_rel_err

pytestmark = pytest.mark.gpu

DT_CODE = {"f32": pkg.LMKAN_F32, "f16": pkg.LMKAN_F16, "bf16": pkg.LMKAN_BF16}


def _draws(n, seed):
    rng = np.random.RandomState(seed)
    out = []
    for i in range(n):
        G = int(rng.choice([3, 4, 5, 8, 12, 16, 17, 20, 24, 32, 34, 35, 40, 48, 49, 64]))
        if i % 4 == 0:       # wide enough for the slab kernels whatever the batch
            n_in = 2 * int(rng.randint(33, 70))
            n_out = int(rng.randint(8192 // (n_in // 2) + 1, 8192 // (n_in // 2) + 40))
            B = int(rng.choice([1, 2, 17, 64, 200, 300]))
        elif i % 4 == 2:     # middling layers around the batch and work thresholds of the dispatch
            n_in = 2 * int(rng.randint(8, 80))
            n_out = int(rng.choice([1, 2, 5, 8, 16, 24, 64, 72, 128, 136, 256, 260]))
            B = int(rng.choice([1, 30, 255, 256, 300, 1024, 1025, 2300]))
        else:
            n_in = 2 * int(rng.randint(1, 12))
            n_out = int(rng.choice([1, 2, 3, 4, 7, 8, 9, 10, 12, 16, 17, 60, 64, 65, 100, 130, 193]))
            B = int(rng.choice([1, 5, 63, 255, 256, 257, 700, 1300, 2500, 4200, 9000]))
        if G >= 48 and B > 3000:
            B = 3000         # keeps the oracle's table walk short
        storage = str(rng.choice(["f32", "f32", "f16", "bf16"]))
        layout = int(rng.choice([pkg.LMKAN_LAYOUT_PAPER, pkg.LMKAN_LAYOUT_PACKED, pkg.LMKAN_LAYOUT_PACKED]))
        grads = str(rng.choice(["both", "both", "x", "coef"]))
        accumulate = bool(rng.randint(0, 2)) and grads != "x"
        out.append((B, n_in, n_out, G, storage, layout, grads, accumulate))
    return out


DRAWS = _draws(int(os.environ.get("LMKAN_TEST_DRAWS", "144")), int(os.environ.get("LMKAN_TEST_SEED", "20240917")))


@pytest.fixture(scope="module")
def dev():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    pkg.lib()
    return torch.device("cuda:0")


@pytest.mark.parametrize("draw", DRAWS, ids=lambda d: "B%d_%dto%d_G%d_%s_%s_%s%s" % (
    d[0], d[1], d[2], d[3], d[4], "packed" if d[5] == pkg.LMKAN_LAYOUT_PACKED else "paper", d[6], "_acc" if d[7] else ""))
def test_random_shape_matches_oracle(dev, oracle, draw):
    B, n_in, n_out, G, storage, layout, grads, accumulate = draw
    g = torch.Generator(device="cpu").manual_seed(B * 7919 + n_in * 131 + n_out * 17 + G)
    x = torch.randn((B, n_in), generator=g) * (1.0 + 3.0 * torch.rand((B, n_in), generator=g) ** 4)
    P = torch.randn((G + 1, G + 1, n_in // 2, n_out), generator=g) * 0.1
    gy = torch.randn((B, n_out), generator=g)
    x, P, gy = x.to(dev), P.to(dev), gy.to(dev)
    flags = pkg.LMKAN_FLAG_ACCUMULATE_GRAD_COEF if accumulate else 0
    desc = pkg.LayerDesc(n_in, n_out, G, coef_dtype=DT_CODE[storage], coef_layout=layout, flags=flags)
    Ps = wl.store(P, storage).contiguous()
    Pdev = pkg.lmkan_pack(desc, Ps) if layout == pkg.LMKAN_LAYOUT_PACKED else Ps
    xh, gyh = x.cpu().numpy(), gy.cpu().numpy()
    dt = ORACLE_DTYPE[storage]

    y = pkg.lmkan_forward(desc, x, Pdev)
    base = torch.full((G + 1, G + 1, n_in // 2, n_out), 0.5, device=dev) if accumulate else None
    gx, gP = pkg.lmkan_backward(desc, x, Pdev, gy, need_grad_x=grads != "coef", need_grad_coef=grads != "x",
                                grad_coef=base)
    torch.cuda.synchronize()

    # (row by row where a row has enough entries for its largest one to set a scale; over the whole
    # tensor for the few-output layers, where a row is one or two sums that may cancel to nothing)
    def rel_err(got, want):
        if want.shape[1] >= 8:
            return rowwise_rel_err(got, want)
        return np.abs(got.astype(np.float64) - want).max() / np.abs(want).max()

    want_y = oracle.forward(xh, bits(Ps), G, dtype=dt)
    if B * n_out >= 8:
        assert rel_err(y.cpu().numpy(), want_y) <= TOL_F32
    else:
        # a handful of outputs, each a sum over the pairs that may cancel to nothing (one row of one
        # output is a single number): the scale is what float32 rounding acts on, the sum of the
        # terms' magnitudes, which the oracle gives with |coefficients| (the weights are positive
        # inside the grid; beyond the ghost points the bound is what the largest output needs anyway)
        Pabs = wl.store(P.abs(), storage).contiguous()
        scale = max(np.abs(oracle.forward(xh, bits(Pabs), G, dtype=dt)).max(), np.abs(want_y).max())
        assert np.abs(y.cpu().numpy() - want_y).max() <= TOL_F32 * scale
    if grads != "coef":
        want = oracle.backward_input(xh, bits(Ps), gyh, G, dtype=dt)
        assert rel_err(gx.cpu().numpy(), want) <= TOL_F32
    else:
        assert gx is None
    if grads != "x":
        got = gP.cpu().numpy().astype(np.float64) - (0.5 if accumulate else 0.0)
        for k in range(n_in // 2):
            want = oracle.backward_coef_pair(xh, gyh, G, k)
            # (added to 0.5, the sum is rounded to float32 at 0.5's magnitude)
            slack = 2.0 ** -23 * (0.5 + np.abs(want).max()) / max(np.abs(want).max(), 1e-30) if accumulate else 0.0
            assert pair_slice_rel_err(got[:, :, k, :], want) <= TOL_F32 + slack
            if not accumulate:
                assert np.all(got[:, :, k, :][want == 0.0] == 0.0)
    else:
        assert gP is None
