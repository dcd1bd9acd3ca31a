"""The library under HIP graph capture: it never allocates, never synchronises and clears memory
with fill kernels only, so forward + backward can be recorded once and replayed (what a
launch-bound small layer or a serving loop wants).  Every replay is checked against the eager
result for the same inputs, with the program's own eager work and synchronisations between the
replays."""
import numpy as np
import pytest
import torch

import paper_2509_07103_amd as pkg

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def dev():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    pkg.lib()
    return torch.device("cuda:0")


def _rand(shape, seed, dev, scale=1.0):
    g = torch.Generator(device="cpu").manual_seed(seed)
    return (torch.randn(shape, generator=g) * scale).to(dev)


@pytest.mark.parametrize("shape", [(256, 16, 16, 8),        # cfg1: launch-bound
                                   (1100, 140, 132, 16),    # pair splits, partial outputs, ragged tiles
                                   (300, 8, 20, 34),        # 16-output slabs
                                   (513, 10, 5, 6)])        # small-output kernels
def test_forward_backward_replay_matches_eager(dev, shape):
    B, n_in, n_out, G = shape
    desc = pkg.LayerDesc(n_in, n_out, G)
    P = _rand(desc.coef_shape(), 1, dev, 0.1)
    x, gy = torch.empty((B, n_in), device=dev), torch.empty((B, n_out), device=dev)
    y, gx, gP = torch.empty((B, n_out), device=dev), torch.empty((B, n_in), device=dev), torch.empty_like(P)
    need = max(pkg.lmkan_workspace_bytes(desc, B, False), pkg.lmkan_workspace_bytes(desc, B, True), 256)
    ws = torch.empty(need, dtype=torch.uint8, device=dev)

    def step():
        pkg.lmkan_forward(desc, x, P, y=y, workspace=ws)
        pkg.lmkan_backward(desc, x, P, gy, grad_x=gx, grad_coef=gP, workspace=ws)

    x.copy_(_rand((B, n_in), 10, dev))
    gy.copy_(_rand((B, n_out), 11, dev))
    step()                      # one eager call first: kernel attributes are set outside the capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for rep in range(3):
        xs, gys = _rand((B, n_in), 20 + rep, dev), _rand((B, n_out), 30 + rep, dev)
        # eager result on separate buffers (also the "other work" between replays)
        y_e = pkg.lmkan_forward(desc, xs, P)
        gx_e, gP_e = pkg.lmkan_backward(desc, xs, P, gys)
        torch.cuda.synchronize()
        x.copy_(xs)
        gy.copy_(gys)
        y.fill_(float("nan"))
        gx.fill_(float("nan"))
        gP.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        if n_out > 8:
            assert torch.equal(y, y_e), rep             # the forward sums in a fixed order
        else:
            torch.testing.assert_close(y, y_e, rtol=0, atol=1e-5 * float(y_e.abs().max()))
        # gradients are sums whose order may differ between runs (atomics, order inside a cell)
        torch.testing.assert_close(gx, gx_e, rtol=0, atol=1e-5 * float(gx_e.abs().max()))
        torch.testing.assert_close(gP, gP_e, rtol=0, atol=1e-5 * float(gP_e.abs().max()))


def test_convolution_and_regulariser_replay(dev):
    conv = pkg.Conv2d(3, 12, 12, 4, 3, 3, 1)
    rows, oh, ow = pkg.lmkan_conv2d_rows(conv)
    desc = pkg.LayerDesc(36, 16, 8)
    P = _rand(desc.coef_shape(), 2, dev, 0.1)
    x = torch.empty(conv.image_shape(), device=dev)
    gy = torch.empty((3, oh, ow, 16), device=dev)
    y, gx, gP = torch.empty_like(gy), torch.empty_like(x), torch.empty_like(P)
    need = max(pkg.lmkan_workspace_bytes(desc, rows, False), pkg.lmkan_workspace_bytes(desc, rows, True), 256)
    ws = torch.empty(need, dtype=torch.uint8, device=dev)
    acc = pkg.LayerDesc(36, 16, 8, flags=pkg.LMKAN_FLAG_ACCUMULATE_GRAD_COEF)

    def step():
        pkg.lmkan_conv2d_forward(desc, conv, x, P, y=y, workspace=ws)
        pkg.lmkan_conv2d_backward(desc, conv, x, P, gy, grad_x=gx, grad_coef=gP, workspace=ws)
        pkg.lmkan_hessian_reg(acc, P, scale=0.5, need_value=False, grad_coef=gP)   # adds into the same gradient

    x.copy_(_rand(conv.image_shape(), 40, dev))
    gy.copy_(_rand(tuple(gy.shape), 41, dev))
    step()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for rep in range(3):
        xs, gys = _rand(conv.image_shape(), 50 + rep, dev), _rand(tuple(gy.shape), 60 + rep, dev)
        y_e = pkg.lmkan_conv2d_forward(desc, conv, xs, P)
        gx_e, gP_e = pkg.lmkan_conv2d_backward(desc, conv, xs, P, gys)
        pkg.lmkan_hessian_reg(acc, P, scale=0.5, need_value=False, grad_coef=gP_e)
        torch.cuda.synchronize()
        x.copy_(xs)
        gy.copy_(gys)
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(y, y_e)
        torch.testing.assert_close(gx, gx_e, rtol=0, atol=1e-5 * float(gx_e.abs().max()))
        torch.testing.assert_close(gP, gP_e, rtol=0, atol=1e-5 * float(gP_e.abs().max()))


def test_time_next_kernel_brackets_only_the_main_kernel(dev):
    """The measurement aid: armed events are recorded around the main kernel of the next call and
    used once; the kernel's time is positive and no longer than the whole call's."""
    B, n_in, n_out, G = 4096, 64, 64, 16
    desc = pkg.LayerDesc(n_in, n_out, G)
    P = _rand(desc.coef_shape(), 3, dev, 0.1)
    x, gy = _rand((B, n_in), 4, dev), _rand((B, n_out), 5, dev)
    pkg.lmkan_forward(desc, x, P)           # warm-up
    pkg.lmkan_backward(desc, x, P, gy)
    torch.cuda.synchronize()

    def armed(call):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        c0, c1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        e1.record()
        pkg.lmkan_time_next_kernel(e0, e1)
        c0.record()
        call()
        c1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1), c0.elapsed_time(c1)

    for call in (lambda: pkg.lmkan_forward(desc, x, P),
                 lambda: pkg.lmkan_backward(desc, x, P, gy, need_grad_coef=False),
                 lambda: pkg.lmkan_backward(desc, x, P, gy, need_grad_x=False),
                 lambda: pkg.lmkan_backward(desc, x, P, gy)):
        kernel, whole = armed(call)
        assert 0.0 < kernel <= whole
    # used once: a second call leaves fresh events untouched (stop is not after start by a kernel's time)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    e1.record()
    pkg.lmkan_time_next_kernel(e0, e1)
    pkg.lmkan_forward(desc, x, P)
    torch.cuda.synchronize()
    first = e0.elapsed_time(e1)
    pkg.lmkan_forward(desc, x, P)           # not armed any more
    torch.cuda.synchronize()
    assert e0.elapsed_time(e1) == first
    with pytest.raises(pkg.LmkanError):
        pkg.lib().lmkan_time_next_kernel  # attribute exists
        pkg.binding._check(pkg.lib().lmkan_time_next_kernel(e0.cuda_event, None), "lmkan_time_next_kernel")
    pkg.lmkan_time_next_kernel(None, None)
