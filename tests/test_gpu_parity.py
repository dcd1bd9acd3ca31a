"""GPU parity: the HIP library (through its C ABI) against the CPU oracle, element by
element on the same seeded inputs.  Cell indices must agree bit for bit; values within
1e-5 (float32 tables, and half tables against the oracle reading the stored bits) and
2e-2 (half tables against the oracle on the float32 master), in the row-wise max norm."""
import numpy as np
import pytest
import torch

import paper_2509_07103_amd as pkg
from paper_2509_07103_amd import workloads as wl
from parity_util import (ORACLE_DTYPE, TOL_F32, TOL_HALF, bits, output_rel_err, pair_slice_rel_err,
                         rowwise_rel_err)

pytestmark = pytest.mark.gpu

DT_CODE = {"f32": pkg.LMKAN_F32, "f16": pkg.LMKAN_F16, "bf16": pkg.LMKAN_BF16}


@pytest.fixture(scope="module")
def dev():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    pkg.lib()   # fails loudly if liblmkan.so was not built
    return torch.device("cuda:0")


def _inputs(B, n_in, n_out, G, seed, dev, heavy=False, std=0.1):
    g = torch.Generator(device="cpu").manual_seed(seed)
    x = torch.randn((B, n_in), generator=g)
    if heavy:
        x = x * (1.0 + 4.0 * torch.rand((B, n_in), generator=g) ** 4)
    P = torch.randn((G + 1, G + 1, n_in // 2, n_out), generator=g) * std
    gy = torch.randn((B, n_out), generator=g)
    return x.to(dev), P.to(dev), gy.to(dev)


def _desc(n_in, n_out, G, storage="f32", layout=pkg.LMKAN_LAYOUT_PAPER, flags=0):
    return pkg.LayerDesc(n_in, n_out, G, coef_dtype=DT_CODE[storage], coef_layout=layout, flags=flags)


def _stored(P, storage, desc, layout):
    Ps = wl.store(P, storage).contiguous()
    if layout == pkg.LMKAN_LAYOUT_PACKED:
        return Ps, pkg.lmkan_pack(desc, Ps)
    return Ps, Ps


SHAPES = [
    # B, n_in, n_out, G
    (1, 2, 1, 3),
    (7, 4, 3, 4),
    (33, 6, 65, 5),
    (256, 16, 16, 8),
    (257, 18, 100, 8),
    (130, 34, 64, 16),
    (513, 130, 129, 12),
    (100, 260, 256, 16),
    (64, 8, 200, 33),
    (40, 6, 70, 64),
    # large enough for the LDS-slab forward: ragged sample tile, ragged output tile, pair split
    (1100, 140, 132, 16),
    (2053, 64, 64, 12),
    (300, 10, 260, 3),
    # grids too fine for 64-output slabs: 16-output slabs (16-bit tables), ragged everything,
    # more samples than one workgroup takes
    (700, 12, 72, 20),
    (4200, 6, 40, 32),
    (300, 8, 20, 34),
    # a batch long enough for the coefficient gradient to sort it block by block
    (13000, 6, 68, 5),
    # rows wide enough for the sorted kernels to gather gy from a tile-by-tile copy (ragged last tile)
    (600, 4, 2116, 9),
    # the finest grids whose 16-output slab fits LDS once (forward walks one slab at a time), and
    # the first one beyond
    (4300, 6, 40, 48),
    (300, 4, 24, 49),
    # either side of the thresholds at which the dispatch changes kernels: 256 rows, 8 and 9
    # outputs, G = 16 / 17 and 34 / 35, 12288 rows
    (255, 6, 12, 8),
    (256, 6, 12, 8),
    (1024, 66, 4, 16),
    (2049, 130, 8, 12),
    (300, 4, 9, 16),
    (300, 6, 12, 17),
    (300, 6, 12, 35),
    (12289, 4, 12, 6),
    # both gradients from one walk over the cell-sorted samples: grids too fine for any slab
    # (ragged output tile, more than one trip per cell, a batch long enough to be sorted block by
    # block), and the 16-output slab range with enough samples per cell
    (2100, 10, 132, 40),
    (600, 4, 64, 64),
    (13000, 6, 68, 36),
    (7000, 12, 72, 20),
    # output counts that are not a multiple of four on the tuned kernels (packed tables): a ten-way
    # head, a last tile of one output, 16-output slabs, the single-slab forward, the sorted walk
    # with dense cells, a pair split; and few outputs on a grid too fine for their own
    # coefficient-gradient kernel
    (1000, 16, 10, 16),
    (2200, 40, 193, 8),
    (700, 6, 21, 24),
    (600, 4, 18, 40),
    (7000, 6, 70, 20),
    (1100, 140, 66, 16),
    (300, 4, 8, 64),
    (300, 4, 3, 64),
    # 32-output tiles with the pairs split over several workgroups (partial sums, atomics)
    (2100, 64, 40, 22),
    # batches under 256 rows on layers wide enough for the slab kernels anyway (pairs x outputs
    # >= 8192), down to a single row; 16-output slabs, the single-slab forward, a ragged head
    (1, 128, 128, 16),
    (3, 64, 256, 8),
    (37, 130, 140, 20),
    (5, 140, 132, 40),
    (100, 1100, 10, 12),
    # one output: the forward kernel that keeps the tables in LDS and locates by itself (all pairs
    # in one chunk; chunks of 128 and of 64 pairs with a ragged last one; the finest grid it takes
    # and the first one beyond, with more and fewer pairs than fit; one pair on the finest grid; a
    # batch long enough for workgroups to take more than eight rounds)
    (5000, 256, 1, 16),
    (700, 600, 1, 16),
    (300, 200, 1, 23),
    (300, 200, 1, 24),
    (300, 200, 1, 25),
    (300, 100, 1, 25),
    (3, 2, 1, 64),
    (300000, 4, 1, 4),
]


@pytest.mark.parametrize("shape", SHAPES)
def test_cell_indices_are_bit_exact(dev, oracle, shape):
    B, n_in, n_out, G = shape
    x, _, _ = _inputs(B, n_in, n_out, G, 11, dev, heavy=True)
    nodes = torch.from_numpy(oracle.grid_f32(G))
    flat = x.flatten().cpu()
    # plant every grid point, its float neighbours, and non-finite / huge values
    special = torch.cat([nodes, torch.nextafter(nodes, torch.tensor(-1e30)),
                         torch.nextafter(nodes, torch.tensor(1e30)),
                         torch.tensor([float("inf"), float("-inf"), float("nan"), 3e38, -3e38,
                                       0.0, -0.0, 1e-45, 17.0, -17.0, 88.0, -104.0])])
    m = min(len(special), flat.numel())
    flat[:m] = special[:m]
    x = flat.reshape(B, n_in).to(dev)
    cell = pkg.lmkan_locate(_desc(n_in, n_out, G), x)
    torch.cuda.synchronize()
    want = oracle.locate_batch(x.cpu().numpy(), G)
    np.testing.assert_array_equal(cell.cpu().numpy(), want)


@pytest.mark.parametrize("layout", [pkg.LMKAN_LAYOUT_PAPER, pkg.LMKAN_LAYOUT_PACKED])
@pytest.mark.parametrize("storage", ["f32", "f16", "bf16"])
@pytest.mark.parametrize("shape", SHAPES)
def test_forward_matches_oracle(dev, oracle, shape, storage, layout):
    B, n_in, n_out, G = shape
    x, P, _ = _inputs(B, n_in, n_out, G, 21, dev, heavy=True)
    desc = _desc(n_in, n_out, G, storage, layout)
    Ps, Pdev = _stored(P, storage, desc, layout)
    y = pkg.lmkan_forward(desc, x, Pdev)
    torch.cuda.synchronize()
    xh = x.cpu().numpy()
    want = oracle.forward(xh, bits(Ps), G, dtype=ORACLE_DTYPE[storage])
    assert output_rel_err(y.cpu().numpy(), want) <= TOL_F32
    if storage != "f32":
        master = oracle.forward(xh, P.cpu().numpy(), G)
        assert output_rel_err(y.cpu().numpy(), master) <= TOL_HALF


@pytest.mark.parametrize("layout", [pkg.LMKAN_LAYOUT_PAPER, pkg.LMKAN_LAYOUT_PACKED])
@pytest.mark.parametrize("storage", ["f32", "f16", "bf16"])
@pytest.mark.parametrize("shape", SHAPES)
def test_backward_matches_oracle(dev, oracle, shape, storage, layout):
    B, n_in, n_out, G = shape
    x, P, gy = _inputs(B, n_in, n_out, G, 31, dev, heavy=True)
    desc = _desc(n_in, n_out, G, storage, layout)
    Ps, Pdev = _stored(P, storage, desc, layout)
    gx, gP = pkg.lmkan_backward(desc, x, Pdev, gy)
    torch.cuda.synchronize()
    xh, gyh = x.cpu().numpy(), gy.cpu().numpy()
    want_gx = oracle.backward_input(xh, bits(Ps), gyh, G, dtype=ORACLE_DTYPE[storage])
    assert rowwise_rel_err(gx.cpu().numpy(), want_gx) <= TOL_F32
    gPh = gP.cpu().numpy()
    assert gPh.shape == (G + 1, G + 1, n_in // 2, n_out)
    for k in range(n_in // 2):
        want = oracle.backward_coef_pair(xh, gyh, G, k)
        assert pair_slice_rel_err(gPh[:, :, k, :], want) <= TOL_F32
        # entries no sample touches must be exactly zero (Sec. 3.5)
        assert np.all(gPh[:, :, k, :][want == 0.0] == 0.0)
    if storage != "f32":
        # against the float32 master the input gradient sees *differences* of rounded
        # coefficients, so its worst single element is not a fair yardstick; the bound is
        # taken on the whole tensor (relative Frobenius norm)
        master = oracle.backward_input(xh, P.cpu().numpy(), gyh, G)
        diff = np.linalg.norm(gx.cpu().numpy().astype(np.float64) - master)
        assert diff <= TOL_HALF * np.linalg.norm(master)
        # element by element, to the bound the arithmetic gives: an input gradient is 1/h times a
        # weighted sum over j of gy[n][j] times differences of two stored coefficients, each of
        # which is off by at most one unit roundoff u of the storage format times |P|max
        # (the two differences enter with weights 1 - t and t of the pair's *other* coordinate,
        # |1 - t| + |t| = 1 inside the grid and 1 + 2 (distance past the outermost point) / h beyond it,
        # where every function continues linearly)
        u = 2.0 ** -11 if storage == "f16" else 2.0 ** -8
        E = oracle.grid_f32(G).astype(np.float64)
        inv_h = 1.0 / np.diff(E).min()
        beyond = np.maximum(np.abs(xh.astype(np.float64)) - E[G], 0.0) / (E[G] - E[G - 1])
        other = (1.0 + 2.0 * beyond).reshape(B, n_in // 2, 2)[:, :, ::-1].reshape(B, n_in)
        bound = 2.0 * u * float(P.abs().max()) * inv_h * other * np.abs(gyh.astype(np.float64)).sum(axis=1, keepdims=True)
        assert np.all(np.abs(gx.cpu().numpy().astype(np.float64) - master) <= bound + 1e-30)


# one shape per way the coefficient gradient can be formed: float32 atomics in the generic
# kernel (n_out not a multiple of 4), the cell-sorted stream written row by row, the same
# stream cut into runs that meet through atomics (long batch, few pairs), the LDS-privatised
# kernel of narrow layers
# and the walk that forms both gradients at once (a grid too fine for the slab kernels)
@pytest.mark.parametrize("shape", [(90, 12, 70, 8), (90, 12, 72, 8), (2100, 12, 72, 8), (90, 12, 3, 8),
                                   (2100, 10, 132, 40)])
def test_backward_pieces_and_accumulate_flag(dev, oracle, shape):
    B, n_in, n_out, G = shape
    x, P, gy = _inputs(B, n_in, n_out, G, 41, dev)
    desc = _desc(n_in, n_out, G)
    gx_only, none = pkg.lmkan_backward(desc, x, P, gy, need_grad_coef=False)
    assert none is None
    none, gP_only = pkg.lmkan_backward(desc, x, None, gy, need_grad_x=False)
    assert none is None
    gx, gP = pkg.lmkan_backward(desc, x, P, gy)
    torch.cuda.synchronize()
    # same kernel, same inputs; only the order of a few float atomics may differ
    assert rowwise_rel_err(gx.cpu().numpy(), gx_only.cpu().numpy().astype(np.float64)) <= 1e-6
    want = oracle.backward_coef(x.cpu().numpy(), gy.cpu().numpy(), G)
    for got in (gP, gP_only):
        assert np.abs(got.cpu().numpy() - want).max() <= TOL_F32 * np.abs(want).max()
    # accumulate: start from a known tensor, expect tensor + gradient
    acc = torch.full_like(gP, 0.5)
    dacc = _desc(n_in, n_out, G, flags=pkg.LMKAN_FLAG_ACCUMULATE_GRAD_COEF)
    pkg.lmkan_backward(dacc, x, P, gy, need_grad_x=False, grad_coef=acc)
    torch.cuda.synchronize()
    assert np.abs(acc.cpu().numpy() - (want + 0.5)).max() <= 2e-5 * max(1.0, np.abs(want).max())
    # the same with both gradients in one call
    acc = torch.full_like(gP, 0.5)
    gx_acc, _ = pkg.lmkan_backward(dacc, x, P, gy, grad_coef=acc)
    torch.cuda.synchronize()
    assert np.abs(acc.cpu().numpy() - (want + 0.5)).max() <= 2e-5 * max(1.0, np.abs(want).max())
    assert rowwise_rel_err(gx_acc.cpu().numpy(), gx.cpu().numpy().astype(np.float64)) <= 1e-6
    # overwrite really overwrites stale contents
    stale = torch.full_like(gP, 123.0)
    pkg.lmkan_backward(desc, x, P, gy, need_grad_x=False, grad_coef=stale)
    torch.cuda.synchronize()
    assert np.abs(stale.cpu().numpy() - want).max() <= TOL_F32 * np.abs(want).max()


@pytest.mark.parametrize("shape", [(1100, 140, 132, 16), (1024, 66, 4, 16), (4200, 6, 40, 32), (2100, 10, 132, 40)])
def test_calls_can_reuse_the_records_in_the_workspace(dev, oracle, shape):
    """LMKAN_FLAG_WORKSPACE_HAS_RECORDS: a backward (or forward) call on the workspace an earlier call
    on the same x left behind skips the preamble pass and gives what the full call gives."""
    B, n_in, n_out, G = shape
    x, P, gy = _inputs(B, n_in, n_out, G, 55, dev)
    desc = _desc(n_in, n_out, G)
    reuse = _desc(n_in, n_out, G, flags=pkg.LMKAN_FLAG_WORKSPACE_HAS_RECORDS)
    need = max(pkg.lmkan_workspace_bytes(desc, B, False), pkg.lmkan_workspace_bytes(desc, B, True))
    assert pkg.lmkan_workspace_bytes(desc, B, False) > 0
    ws = torch.empty(need, dtype=torch.uint8, device=dev)
    want_y = pkg.lmkan_forward(desc, x, P)
    want_gx, want_gp = pkg.lmkan_backward(desc, x, P, gy)
    ws.fill_(0xFF)                                   # nothing usable in the workspace yet
    y = pkg.lmkan_forward(desc, x, P, workspace=ws)  # writes the records
    gx, gp = pkg.lmkan_backward(reuse, x, P, gy, workspace=ws)
    y2 = pkg.lmkan_forward(reuse, x, P, workspace=ws)
    gx2, gp2 = pkg.lmkan_backward(reuse, x, P, gy, workspace=ws)
    torch.cuda.synchronize()
    for got in (y, y2):     # (the kernel for narrow outputs adds its pair splits with atomics: not bit-equal)
        assert rowwise_rel_err(got.cpu().numpy(), want_y.cpu().numpy().astype(np.float64)) <= 1e-6
    for a, b in ((gx, gp), (gx2, gp2)):
        assert rowwise_rel_err(a.cpu().numpy(), want_gx.cpu().numpy().astype(np.float64)) <= 1e-6
        assert torch.allclose(b, want_gp, rtol=1e-5, atol=1e-6 * float(want_gp.abs().max()))
    want = oracle.backward_input(x.cpu().numpy(), P.cpu().numpy(), gy.cpu().numpy(), G)
    assert rowwise_rel_err(gx.cpu().numpy(), want) <= TOL_F32


def test_sorted_paths_repeat_bit_for_bit(dev):
    """What the header promises about run-to-run variation: the counting sort leaves the samples of
    a cell in the order of their indices, so a coefficient gradient that one wave writes row by
    row (stream not cut into runs) is the same float32 sum in every run, and so is the input
    gradient of the walk over the sorted samples (its tiles are added in a fixed order).  Paths
    that meet through float32 atomics are only held to the tolerance (other tests)."""
    # a short stream: one run per (pair, tile)
    B, n_in, n_out, G = 30, 12, 72, 4
    x, P, gy = _inputs(B, n_in, n_out, G, 51, dev)
    desc = _desc(n_in, n_out, G)
    runs = [pkg.lmkan_backward(desc, x, None, gy, need_grad_x=False)[1] for _ in range(3)]
    torch.cuda.synchronize()
    assert torch.equal(runs[0], runs[1]) and torch.equal(runs[0], runs[2])
    # both gradients from the sorted walk: grad_x repeats exactly
    B, n_in, n_out, G = 2100, 10, 132, 40
    x, P, gy = _inputs(B, n_in, n_out, G, 52, dev)
    desc = _desc(n_in, n_out, G)
    gxs = [pkg.lmkan_backward(desc, x, P, gy)[0] for _ in range(3)]
    torch.cuda.synchronize()
    assert torch.equal(gxs[0], gxs[1]) and torch.equal(gxs[0], gxs[2])
    # enough (pair, tile) streams to fill the chip, so that none is cut into runs (256 pairs x 16
    # tiles), many trips per wave, several waves per CU
    B, n_in, n_out, G = 2000, 512, 1024, 8
    x, P, gy = _inputs(B, n_in, n_out, G, 53, dev)
    desc = _desc(n_in, n_out, G)
    runs = [pkg.lmkan_backward(desc, x, None, gy, need_grad_x=False)[1] for _ in range(2)]
    torch.cuda.synchronize()
    assert torch.equal(runs[0], runs[1])


def test_empty_batch(dev):
    desc = _desc(8, 5, 4)
    x = torch.empty((0, 8), device=dev)
    P = torch.randn(desc.coef_shape(), device=dev)
    y = pkg.lmkan_forward(desc, x, P)
    assert y.shape == (0, 5)
    gy = torch.empty((0, 5), device=dev)
    gP = torch.full(desc.coef_shape(), 7.0, device=dev)
    gx, gP = pkg.lmkan_backward(desc, x, P, gy, grad_coef=gP)
    torch.cuda.synchronize()
    assert gx.shape == (0, 8) and torch.all(gP == 0)
    assert pkg.lmkan_locate(desc, x).shape == (0, 4)


def test_pack_layout(dev):
    n_in, n_out, G = 6, 70, 4
    desc = _desc(n_in, n_out, G)
    P = torch.randn(desc.coef_shape(), device=dev)
    packed = pkg.lmkan_pack(desc, P).cpu().reshape(2, 3, 25, 64)
    Ph = P.cpu().reshape(25, 3, n_out)
    for jt in range(2):
        for k in range(3):
            cols = min(64, n_out - jt * 64)
            assert torch.equal(packed[jt, k, :, :cols], Ph[:, k, jt * 64: jt * 64 + cols])
            assert torch.all(packed[jt, k, :, cols:] == 0)


def test_nonfinite_inputs_stay_memory_safe(dev, oracle):
    B, n_in, n_out, G = 16, 8, 10, 8
    x, P, gy = _inputs(B, n_in, n_out, G, 51, dev)
    x[0, 0] = float("nan")
    x[1, 3] = float("inf")
    x[2, 4] = float("-inf")
    x[3, 5] = 1e30
    desc = _desc(n_in, n_out, G)
    y = pkg.lmkan_forward(desc, x, P)
    gx, gP = pkg.lmkan_backward(desc, x, P, gy)
    torch.cuda.synchronize()
    # rows without a non-finite input are unaffected
    want = oracle.forward(x[4:].cpu().numpy(), P.cpu().numpy(), G)
    assert rowwise_rel_err(y[4:].cpu().numpy(), want) <= TOL_F32
    assert torch.isnan(y[0]).all()
    # the huge but finite input is a valid far extrapolation
    want3 = oracle.forward(x[3:4].cpu().numpy(), P.cpu().numpy(), G)
    assert rowwise_rel_err(y[3:4].cpu().numpy(), want3) <= TOL_F32


def test_results_do_not_depend_on_the_stream(dev, oracle):
    B, n_in, n_out, G = 300, 20, 96, 8
    x, P, _ = _inputs(B, n_in, n_out, G, 61, dev)
    desc = _desc(n_in, n_out, G)
    y0 = pkg.lmkan_forward(desc, x, P)
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        y1 = pkg.lmkan_forward(desc, x, P)
    s.synchronize()
    torch.cuda.synchronize()
    assert torch.equal(y0, y1)
    # a stream passed by argument while another one is current: the binding's own allocations
    # (the workspace it frees on return, the outputs) must survive allocations made meanwhile on
    # the current stream
    B, n_in, n_out, G = 4000, 64, 128, 12      # large enough for a workspace
    x, P, gy = _inputs(B, n_in, n_out, G, 62, dev)
    desc = _desc(n_in, n_out, G)
    want_y = pkg.lmkan_forward(desc, x, P)
    want_gx, want_gp = pkg.lmkan_backward(desc, x, P, gy)
    torch.cuda.synchronize()
    s.wait_stream(torch.cuda.current_stream())
    y2 = pkg.lmkan_forward(desc, x, P, stream=s)
    gx2, gp2 = pkg.lmkan_backward(desc, x, P, gy, stream=s)
    junk = [torch.full((1 << 20,), float(i), device=dev) for i in range(16)]   # current stream
    s.synchronize()
    torch.cuda.synchronize()
    assert torch.equal(want_y, y2)
    assert rowwise_rel_err(gx2.cpu().numpy(), want_gx.cpu().numpy().astype(np.float64)) <= TOL_F32
    assert torch.allclose(gp2, want_gp, rtol=1e-4, atol=1e-5)
    del junk


@pytest.mark.parametrize("G", list(range(3, 65)))
def test_layer_every_grid(dev, oracle, G):
    """Forward and both gradients at every grid size the library takes, on a batch long enough for
    the tiled kernels: the tile (64 or 16 outputs, one or two slabs in LDS), the fused and the
    generic kernels all change over with G.  Storage, layout and output count rotate with G."""
    storage = ["f32", "f16", "bf16"][G % 3]
    layout = [pkg.LMKAN_LAYOUT_PACKED, pkg.LMKAN_LAYOUT_PAPER][(G // 3) % 2]
    B, n_in = 330, 6
    n_out = [20, 64, 18, 72][G % 4] if layout == pkg.LMKAN_LAYOUT_PACKED else [20, 64, 16, 72][G % 4]
    x, P, gy = _inputs(B, n_in, n_out, G, 41 + G, dev, heavy=True)
    desc = _desc(n_in, n_out, G, storage, layout)
    Ps, Pdev = _stored(P, storage, desc, layout)
    y = pkg.lmkan_forward(desc, x, Pdev)
    gx, gP = pkg.lmkan_backward(desc, x, Pdev, gy)
    torch.cuda.synchronize()
    xh, gyh = x.cpu().numpy(), gy.cpu().numpy()
    code = ORACLE_DTYPE[storage]
    assert rowwise_rel_err(y.cpu().numpy(), oracle.forward(xh, bits(Ps), G, dtype=code)) <= TOL_F32
    assert rowwise_rel_err(gx.cpu().numpy(), oracle.backward_input(xh, bits(Ps), gyh, G, dtype=code)) <= TOL_F32
    gPh = gP.cpu().numpy()
    for k in range(n_in // 2):
        want = oracle.backward_coef_pair(xh, gyh, G, k)
        assert pair_slice_rel_err(gPh[:, :, k, :], want) <= TOL_F32
        assert np.all(gPh[:, :, k, :][want == 0.0] == 0.0)


# ---- Hessian regulariser (Sec. 3.5, App. C) ---------------------------------------------------
@pytest.mark.parametrize("layout", [pkg.LMKAN_LAYOUT_PAPER, pkg.LMKAN_LAYOUT_PACKED])
@pytest.mark.parametrize("storage", ["f32", "f16", "bf16"])
# grids on either side of every band count of the kernel (bands of nine columns: G + 1 = 9, 10, 18, 19 ...),
# output counts that leave the last tile ragged, a single tile, several tiles
@pytest.mark.parametrize("shape", [(4, 3, 3), (6, 70, 4), (4, 64, 8), (4, 65, 9), (6, 130, 12), (18, 132, 16),
                                   (4, 64, 17), (4, 20, 18), (4, 96, 20), (4, 70, 32), (8, 200, 33), (4, 64, 40),
                                   (6, 5, 64)])
def test_hessian_reg_matches_oracle(dev, oracle, shape, storage, layout):
    n_in, n_out, G = shape
    g = torch.Generator(device="cpu").manual_seed(71)
    P = (torch.randn((G + 1, G + 1, n_in // 2, n_out), generator=g) * 0.1).to(dev)
    desc = _desc(n_in, n_out, G, storage, layout)
    Ps, Pdev = _stored(P, storage, desc, layout)
    value, grad = pkg.lmkan_hessian_reg(desc, Pdev, scale=0.5)
    torch.cuda.synchronize()
    want_v, want_g = oracle.hessian_reg(bits(Ps), G, dtype=ORACLE_DTYPE[storage])
    assert float(value.cpu()[0]) == pytest.approx(want_v, rel=1e-5)
    got = grad.cpu().numpy()
    for k in range(n_in // 2):
        assert pair_slice_rel_err(got[:, :, k, :], 0.5 * want_g[:, :, k, :]) <= TOL_F32
    # accumulate on top of an existing gradient; value alone; gradient alone
    acc = torch.full_like(grad, 0.25)
    dacc = _desc(n_in, n_out, G, storage, layout, flags=pkg.LMKAN_FLAG_ACCUMULATE_GRAD_COEF)
    v2, _ = pkg.lmkan_hessian_reg(dacc, Pdev, scale=0.5, grad_coef=acc)
    only_v, none = pkg.lmkan_hessian_reg(desc, Pdev, need_grad=False)
    torch.cuda.synchronize()
    assert none is None
    assert np.abs(acc.cpu().numpy() - (0.5 * want_g + 0.25)).max() <= 2e-5 * max(1.0, np.abs(want_g).max())
    assert float(v2.cpu()[0]) == pytest.approx(want_v, rel=1e-5)
    assert float(only_v.cpu()[0]) == pytest.approx(want_v, rel=1e-5)


@pytest.mark.parametrize("G", list(range(3, 65)))
def test_hessian_reg_every_grid(dev, oracle, G):
    """Every grid size the library takes: the kernel's bands, its three-row steps and the rows left
    over after them all change with G.  Storage, layout and output count rotate with G."""
    storage = ["f32", "f16", "bf16"][G % 3]
    layout = [pkg.LMKAN_LAYOUT_PAPER, pkg.LMKAN_LAYOUT_PACKED][(G // 3) % 2]
    n_in, n_out = 4, [5, 64, 66, 1][G % 4]
    g = torch.Generator(device="cpu").manual_seed(72 + G)
    P = (torch.randn((G + 1, G + 1, n_in // 2, n_out), generator=g) * 0.1).to(dev)
    desc = _desc(n_in, n_out, G, storage, layout)
    Ps, Pdev = _stored(P, storage, desc, layout)
    value, grad = pkg.lmkan_hessian_reg(desc, Pdev, scale=2.0)
    torch.cuda.synchronize()
    want_v, want_g = oracle.hessian_reg(bits(Ps), G, dtype=ORACLE_DTYPE[storage])
    assert float(value.cpu()[0]) == pytest.approx(want_v, rel=1e-5)
    got = grad.cpu().numpy()
    for k in range(n_in // 2):
        assert np.abs(got[:, :, k, :] - 2.0 * want_g[:, :, k, :]).max() <= TOL_F32 * np.abs(2.0 * want_g[:, :, k, :]).max()


def test_hessian_reg_is_zero_on_linear_tables(dev, oracle):
    n_in, n_out, G = 6, 40, 12
    E = torch.from_numpy(oracle.grid_f32(G).astype(np.float32))
    lin = 0.3 + 1.5 * E[:, None] - 0.7 * E[None, :]
    P = lin[:, :, None, None].expand(G + 1, G + 1, n_in // 2, n_out).contiguous().to(dev)
    value, grad = pkg.lmkan_hessian_reg(_desc(n_in, n_out, G), P)
    torch.cuda.synchronize()
    # Exactly zero for an exactly linear table; what is left is rounding.  The table itself is
    # linear only up to float32 rounding of its entries (a relative 2^-24 of values up to
    # |P|max), and a second difference divides such an error by a product of two spacings:
    # derivative errors up to 4 * 2^-24 |P|max / hmin^2 on either side, squared and averaged in the
    # value, times the same 1 / h^2 factors (over the (G-1)^2 interior nodes) in the gradient.
    Pmax = float(P.abs().max())
    h = np.diff(E.numpy().astype(np.float64))
    d_err = 4.0 * 2.0 ** -24 * Pmax / h.min() ** 2
    assert float(value.cpu()[0]) <= 4.0 * d_err ** 2 * (n_in // 2) * n_out
    assert float(grad.abs().max()) <= 16.0 * d_err / h.min() ** 2 / (G - 1) ** 2
    # and the double-precision oracle, on the same float32 table, agrees to the same bound
    want_v, want_g = oracle.hessian_reg(P.cpu().numpy(), G)
    assert np.abs(grad.cpu().numpy() - want_g).max() <= 16.0 * d_err / h.min() ** 2 / (G - 1) ** 2
    assert want_v <= 4.0 * d_err ** 2 * (n_in // 2) * n_out


# ---- inference-time folds (App. E Eq. 4b, App. F.1) -------------------------------------------
@pytest.mark.parametrize("layout", [pkg.LMKAN_LAYOUT_PAPER, pkg.LMKAN_LAYOUT_PACKED])
@pytest.mark.parametrize("shape", [(4, 3, 4), (10, 70, 8), (34, 132, 16)])
def test_fold_matches_oracle_and_the_unfolded_layer(dev, oracle, shape, layout):
    n_in, n_out, G = shape
    g = torch.Generator(device="cpu").manual_seed(81)
    P = torch.randn((G + 1, G + 1, n_in // 2, n_out), generator=g) * 0.1
    lin_w = torch.randn((n_out, n_in), generator=g) * 0.3
    lin_b = torch.randn((n_out,), generator=g)
    scale = torch.rand((n_out,), generator=g) + 0.5
    shift = torch.randn((n_out,), generator=g)
    x = (torch.randn((200, n_in), generator=g) * 2.0).to(dev)
    desc = _desc(n_in, n_out, G, "f32", layout)
    _, table = _stored(P.to(dev), "f32", desc, layout)
    table = table.clone()
    y_plain = pkg.lmkan_forward(desc, x, table)
    pkg.lmkan_fold(desc, table, 0.3, lin_w.to(dev), lin_b.to(dev), scale.to(dev), shift.to(dev))
    y_folded = pkg.lmkan_forward(desc, x, table)
    torch.cuda.synchronize()
    # the folded table itself against the oracle's (paper layout only: it can be read back as is)
    want_table = oracle.fold(P.numpy(), G, 0.3, lin_w.numpy(), lin_b.numpy(), scale.numpy(), shift.numpy())
    if layout == pkg.LMKAN_LAYOUT_PAPER:
        got = table.cpu().numpy().astype(np.float64)
        assert np.abs(got - want_table).max() <= 1e-6 * np.abs(want_table).max()
    # and the identity it stands for: one folded layer == scale (gamma layer + Linear(ReLU x)) + shift
    want_y = scale.to(dev) * (0.3 * y_plain + torch.relu(x) @ lin_w.to(dev).T + lin_b.to(dev)) + shift.to(dev)
    assert rowwise_rel_err(y_folded.cpu().numpy(), want_y.double().cpu().numpy()) <= 2e-5
    # the oracle's forward on the oracle's folded table agrees too
    want = oracle.forward(x.cpu().numpy(), want_table.astype(np.float32), G)
    assert rowwise_rel_err(y_folded.cpu().numpy(), want) <= TOL_F32


def _shifted(t, elems=1):
    """A contiguous copy of t whose storage starts `elems` elements past an aligned allocation."""
    buf = torch.empty(t.numel() + elems, dtype=t.dtype, device=t.device)
    out = buf[elems:].view(t.shape)
    out.copy_(t)
    return out


def test_one_output_layer_takes_rows_and_tables_on_any_element_boundary(dev, oracle):
    """The forward kernel of a layer with one output reads its rows eight bytes at a time; rows on a
    4-byte boundary go through the general kernel instead, a table or y off the 16-byte grid
    change nothing."""
    B, n_in, n_out, G = 500, 40, 1, 12
    x, P, _ = _inputs(B, n_in, n_out, G, 33, dev)
    desc = _desc(n_in, n_out, G)
    want = oracle.forward(x.cpu().numpy(), P.cpu().numpy(), G)
    xu, Pu = _shifted(x), _shifted(P)
    assert xu.data_ptr() % 8 == 4 and Pu.data_ptr() % 16 != 0
    for xq, Pq, yq in ((x, Pu, _shifted(torch.empty((B, 1), device=dev))), (xu, P, torch.empty((B, 1), device=dev)),
                       (xu, Pu, _shifted(torch.empty((B, 1), device=dev)))):
        yq.fill_(float("nan"))
        pkg.lmkan_forward(desc, xq, Pq, y=yq)
        torch.cuda.synchronize()
        assert np.abs(yq.cpu().numpy() - want).max() <= TOL_F32 * np.abs(want).max()


@pytest.mark.parametrize("storage", ["f32", "bf16"])
def test_buffers_off_the_16_byte_grid_take_the_general_kernels(dev, oracle, storage):
    """The tuned kernels move 16 bytes per lane; buffers that are only element-aligned must still
    give the same results (the dispatch falls back); that includes x and grad_x on a 4-byte
    boundary, which are read and written element by element."""
    B, n_in, n_out, G = 600, 12, 72, 8
    x, P, gy = _inputs(B, n_in, n_out, G, 31, dev)
    desc = _desc(n_in, n_out, G, storage)
    Ps = wl.store(P, storage).contiguous()
    Pu, gyu = _shifted(Ps), _shifted(gy)
    y = _shifted(torch.empty((B, n_out), device=dev))
    gx = torch.empty((B, n_in), device=dev)
    gP = _shifted(torch.empty(desc.coef_shape(), device=dev))
    assert Pu.data_ptr() % 16 != 0 and gyu.data_ptr() % 16 != 0 and y.data_ptr() % 16 != 0
    pkg.lmkan_forward(desc, x, Pu, y=y)
    pkg.lmkan_backward(desc, x, Pu, gyu, grad_x=gx, grad_coef=gP)
    torch.cuda.synchronize()
    xh, gyh = x.cpu().numpy(), gy.cpu().numpy()
    code = ORACLE_DTYPE[storage]
    assert rowwise_rel_err(y.cpu().numpy(), oracle.forward(xh, bits(Ps), G, dtype=code)) <= TOL_F32
    assert rowwise_rel_err(gx.cpu().numpy(), oracle.backward_input(xh, bits(Ps), gyh, G, dtype=code)) <= TOL_F32
    want = oracle.backward_coef(xh, gyh, G)
    got = gP.cpu().numpy()
    for k in range(n_in // 2):
        assert pair_slice_rel_err(got[:, :, k, :], want[:, :, k, :]) <= TOL_F32
    # x and grad_x on a 4-byte boundary only, everything else aligned; then everything shifted
    xu, gxu = _shifted(x), _shifted(torch.empty((B, n_in), device=dev))
    assert xu.data_ptr() % 8 == 4 and gxu.data_ptr() % 8 == 4
    want_y = oracle.forward(xh, bits(Ps), G, dtype=code)
    want_gx = oracle.backward_input(xh, bits(Ps), gyh, G, dtype=code)
    for Pq, gyq, yq, gPq in ((Ps, gy, torch.empty((B, n_out), device=dev), torch.empty(desc.coef_shape(), device=dev)),
                             (Pu, gyu, y, gP)):
        yq.fill_(float("nan"))
        gxu.fill_(float("nan"))
        pkg.lmkan_forward(desc, xu, Pq, y=yq)
        pkg.lmkan_backward(desc, xu, Pq, gyq, grad_x=gxu, grad_coef=gPq)
        torch.cuda.synchronize()
        assert rowwise_rel_err(yq.cpu().numpy(), want_y) <= TOL_F32
        assert rowwise_rel_err(gxu.cpu().numpy(), want_gx) <= TOL_F32
        got = gPq.cpu().numpy()
        for k in range(n_in // 2):
            assert pair_slice_rel_err(got[:, :, k, :], want[:, :, k, :]) <= TOL_F32
    assert np.array_equal(pkg.lmkan_locate(desc, xu).cpu().numpy(), oracle.locate_batch(xh, G))
    # a pointer off its element size is an error, not a fault
    L = pkg.lib()
    import ctypes as C
    d = desc.c()
    assert L.lmkan_forward(C.byref(d), B, C.c_void_p(x.data_ptr() + 2), C.c_void_p(Ps.data_ptr()),
                           C.c_void_p(y.data_ptr()), None, 0, None) == 5
