"""The forward entry point that allocates nothing (lmkan_forward_static) against lmkan_forward
and the oracle: two calls in a row on the library's static scratch, the second on a smaller
input, so that whatever the first call left in the buffer is seen not to matter."""
import numpy as np
import pytest
import torch

import paper_2509_07103_amd as pkg
from parity_util import TOL_F32, rowwise_rel_err

pytestmark = pytest.mark.gpu


def _inputs(B, n_in, n_out, G, seed, dev):
    g = torch.Generator(device="cpu").manual_seed(seed)
    x = torch.randn((B, n_in), generator=g) * (1.0 + 4.0 * torch.rand((B, n_in), generator=g) ** 4)
    P = torch.randn((G + 1, G + 1, n_in // 2, n_out), generator=g) * 0.1
    return x.to(dev), P.to(dev)


def test_static_scratch_forward_twice_second_call_smaller(oracle):
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    pkg.lib()
    dev = torch.device("cuda:0")
    # first: slab kernels with a pair split (records and partial outputs in the scratch, 5.6 MB);
    # second: fewer rows, fewer pairs, another grid (records only) -- both well under the limit
    for i, (B, n_in, n_out, G) in enumerate([(1100, 140, 132, 16), (300, 10, 260, 3)]):
        desc = pkg.LayerDesc(n_in, n_out, G)
        need = pkg.lmkan_workspace_bytes(desc, B, False)
        assert 0 < need <= pkg.LMKAN_STATIC_SCRATCH_BYTES
        x, P = _inputs(B, n_in, n_out, G, 900 + i, dev)
        print(f"lmkan_forward_static call {i}: B={B} n_in={n_in} n_out={n_out} G={G} scratch={need}", flush=True)
        y_static = torch.full((B, n_out), float("nan"), device=dev)
        pkg.lmkan_forward_static(desc, x, P, y_static)
        y_ref = pkg.lmkan_forward(desc, x, P)
        torch.cuda.synchronize()
        got, ref = y_static.cpu().numpy(), y_ref.cpu().numpy()
        assert rowwise_rel_err(got, ref.astype(np.float64)) <= TOL_F32
        want = oracle.forward(x.cpu().numpy(), P.cpu().numpy(), G)
        assert rowwise_rel_err(got, want) <= TOL_F32


def test_static_scratch_forward_refuses_a_batch_beyond_its_buffer():
    dev = torch.device("cuda:0")
    desc = pkg.LayerDesc(64, 64, 16)
    B = 200000   # 32 pairs x 12 bytes x 200000 rows = 77 MB of records
    x = torch.zeros((B, 64), device=dev)
    P = torch.zeros(desc.coef_shape(), device=dev)
    y = torch.zeros((B, 64), device=dev)
    with pytest.raises(pkg.LmkanError) as e:
        pkg.lmkan_forward_static(desc, x, P, y)
    assert e.value.status == 7
