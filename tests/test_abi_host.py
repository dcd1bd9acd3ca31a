"""Host-side checks of the C ABI that need no GPU: the library loads, exports every
symbol the header declares, and turns bad arguments into status codes."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import paper_2509_07103_amd as pkg
from paper_2509_07103_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    names = set()
    for fn in os.listdir(os.path.join(ROOT, "include")):
        if fn.endswith(".h"):
            text = open(os.path.join(ROOT, "include", fn)).read()
            text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
            names |= set(re.findall(r"\b(lmkan_[a-z_0-9]+)\s*\(", text))
    return names


def test_library_exports_every_declared_symbol():
    L = pkg.lib()
    declared = _declared_functions()
    assert {"lmkan_forward", "lmkan_backward", "lmkan_locate", "lmkan_pack", "lmkan_grid",
            "lmkan_version", "lmkan_status_string", "lmkan_packed_bytes",
            "lmkan_workspace_bytes", "lmkan_hessian_reg", "lmkan_fold", "lmkan_conv2d_rows",
            "lmkan_conv2d_forward", "lmkan_conv2d_backward", "lmkan_time_next_kernel",
            "lmkan_forward_static", "lmkan_microbench"} <= declared
    for name in declared:
        assert hasattr(L, name), name
        assert hasattr(pkg, name), f"python binding lacks {name}"


def test_version_and_status_strings():
    assert pkg.lmkan_version() == 1
    seen = {pkg.lmkan_status_string(s) for s in range(8)}
    assert len(seen) == 8 and "ok" in seen
    assert pkg.lmkan_status_string(99) == "unknown status"


@pytest.mark.parametrize("G", [3, 4, 8, 16, 32, 64])
def test_grid_table_matches_oracle_bit_for_bit(oracle, G):
    nodes, inv_h = pkg.lmkan_grid(G)
    E32 = oracle.grid_f32(G)
    np.testing.assert_array_equal(nodes, E32)
    want = (1.0 / (E32[1:].astype(np.float64) - E32[:-1].astype(np.float64))).astype(np.float32)
    np.testing.assert_array_equal(inv_h, want)


def test_grid_rejects_bad_sizes():
    for G in (-3, 0, 2, 65, 1000):
        with pytest.raises(pkg.LmkanError) as e:
            pkg.lmkan_grid(G)
        assert e.value.status == 2


def _desc(**kw):
    d = dict(n_in=8, n_out=4, grid=8)
    d.update(kw)
    return pkg.LayerDesc(**d)


BAD_DESCS = [
    (dict(n_in=7), 2), (dict(n_in=0), 2), (dict(n_in=131072), 2), (dict(n_out=4194241), 2), (dict(n_out=0), 2), (dict(grid=2), 2), (dict(grid=65), 2),
    (dict(spline_order=3), 3), (dict(coef_dtype=7), 3), (dict(coef_layout=2), 3), (dict(flags=4), 3),
]


@pytest.mark.parametrize("kw,status", BAD_DESCS)
def test_bad_descriptors_are_rejected_before_any_launch(kw, status):
    L = pkg.lib()
    d = _desc(**kw).c()
    fake = C.c_void_p(0x1000)   # never dereferenced: validation comes first
    assert L.lmkan_forward(C.byref(d), 4, fake, fake, fake, None, 0, None) == status
    assert L.lmkan_backward(C.byref(d), 4, fake, fake, fake, fake, fake, None, 0, None) == status
    assert L.lmkan_locate(C.byref(d), 4, fake, fake, None) == status
    assert L.lmkan_pack(C.byref(d), fake, fake, None) == status
    assert L.lmkan_packed_bytes(C.byref(d)) == 0


def test_null_misaligned_and_negative_arguments():
    L = pkg.lib()
    d = _desc().c()
    ok = C.c_void_p(0x1000)
    odd = C.c_void_p(0x1002)
    assert L.lmkan_forward(None, 4, ok, ok, ok, None, 0, None) == 1
    assert L.lmkan_forward(C.byref(d), 4, None, ok, ok, None, 0, None) == 1
    assert L.lmkan_forward(C.byref(d), 4, ok, None, ok, None, 0, None) == 1
    assert L.lmkan_forward(C.byref(d), 4, ok, ok, None, None, 0, None) == 1
    assert L.lmkan_forward(C.byref(d), -1, ok, ok, ok, None, 0, None) == 2
    assert L.lmkan_forward(C.byref(d), 4, odd, ok, ok, None, 0, None) == 5
    assert L.lmkan_forward(C.byref(d), 4, ok, odd, ok, None, 0, None) == 5
    assert L.lmkan_backward(C.byref(d), 4, ok, None, ok, ok, None, None, 0, None) == 1
    assert L.lmkan_backward(C.byref(d), 4, ok, ok, None, ok, ok, None, 0, None) == 1
    assert L.lmkan_backward(C.byref(d), -5, ok, ok, ok, ok, ok, None, 0, None) == 2
    assert L.lmkan_backward(C.byref(d), 4, ok, ok, ok, odd, ok, None, 0, None) == 5
    assert L.lmkan_locate(C.byref(d), 4, None, ok, None) == 1
    assert L.lmkan_pack(C.byref(d), None, ok, None) == 1
    # nothing to do: empty batch, or no gradient requested
    assert L.lmkan_forward(C.byref(d), 0, None, None, None, None, 0, None) == 0
    assert L.lmkan_locate(C.byref(d), 0, None, None, None) == 0
    assert L.lmkan_backward(C.byref(d), 4, ok, ok, ok, None, None, None, 0, None) == 0


def test_static_scratch_forward_rejects_what_does_not_fit_before_any_launch():
    """The entry point that allocates nothing: a batch whose records and partial outputs exceed the
    library's static buffer is an error of its own, found on the host (the pointers are never read)."""
    L = pkg.lib()
    ok = C.c_void_p(0x1000)
    big = _desc(n_in=1024, n_out=1024, grid=16)
    assert pkg.lmkan_workspace_bytes(big, 8192, False) > pkg.LMKAN_STATIC_SCRATCH_BYTES
    assert L.lmkan_forward_static(C.byref(big.c()), 8192, ok, ok, ok, None) == 7
    assert "static" in pkg.lmkan_status_string(7)
    d = _desc().c()
    assert L.lmkan_forward_static(C.byref(d), 0, None, None, None, None) == 0
    assert L.lmkan_forward_static(C.byref(d), -1, ok, ok, ok, None) == 2
    assert L.lmkan_forward_static(C.byref(d), 4, None, ok, ok, None) == 1
    assert L.lmkan_forward_static(None, 4, ok, ok, ok, None) == 1
    assert L.lmkan_forward_static(C.byref(_desc(grid=2).c()), 4, ok, ok, ok, None) == 2


def test_workspace_sizes_follow_the_limits_of_the_sorted_path():
    """The cell-sorted kernels index stream positions with 32 bits and launch one workgroup per 4096
    samples in the second grid dimension (at most 65535): batches beyond that go to the generic
    kernels, and the workspace no longer holds a sorted stream.  Sizes are size_t: no overflow up
    to the largest batch the header admits."""
    d = _desc(n_in=4, n_out=64, grid=4)
    limit = 65535 * 4096                       # the longest batch the sort takes
    records = 3 * 2 * 4                        # bytes per row: (node, u, v) for each of the 2 pairs
    with_sort = pkg.lmkan_workspace_bytes(d, limit, True, need_grad_x=False)
    without = pkg.lmkan_workspace_bytes(d, limit + 1, True, need_grad_x=False)
    assert with_sort >= limit * (records + 2 * 16)          # records + one 16-byte entry per pair and sample
    assert (limit + 1) * records <= without < (limit + 1) * records + 4096
    assert pkg.lmkan_workspace_bytes(d, limit, True) > with_sort    # grad_x adds its scratch
    max_batch = 2147483647                     # LMKAN_MAX_BATCH
    top = pkg.lmkan_workspace_bytes(d, max_batch, True)
    assert top >= max_batch * records
    # forward only: the records alone, whatever the batch
    assert pkg.lmkan_workspace_bytes(d, limit + 1, False) >= (limit + 1) * records


def test_workspace_holds_a_sorted_stream_whenever_a_gradient_needs_one():
    """Layers with few outputs take kernels of their own, but their coefficient gradient needs the
    cell-sorted stream once a pair's slice of it no longer fits LDS (fine grids): the workspace of
    a call for both gradients must then hold the stream, as the call for the coefficient gradient
    alone does."""
    B = 1000
    entry = 16                                  # bytes per pair and sample in the sorted stream
    fine = _desc(n_in=4, n_out=8, grid=64)      # 65^2 nodes x 8 outputs x 4 bytes > 64 KiB
    coarse = _desc(n_in=4, n_out=1, grid=8)     # one output: the kernels for few outputs throughout
    for d, needs_stream in ((fine, True), (coarse, False)):
        both = pkg.lmkan_workspace_bytes(d, B, True)
        gx_only = pkg.lmkan_workspace_bytes(d, B, True, need_grad_coef=False)
        gp_only = pkg.lmkan_workspace_bytes(d, B, True, need_grad_x=False)
        assert (both - gx_only >= 2 * B * entry) == needs_stream
        assert (gp_only >= 2 * B * (entry + 12)) == needs_stream
    # an output count that is not a multiple of four: sorted as well, with room for the copy of gy
    ragged = _desc(n_in=4, n_out=10, grid=8)
    assert pkg.lmkan_workspace_bytes(ragged, B, True, need_grad_x=False) >= 2 * B * (entry + 12) + B * 64 * 4


def test_packed_size_pads_outputs_to_the_tile():
    for n_out, tiles in ((1, 1), (64, 1), (65, 2), (1024, 16)):
        for dt, sz in ((binding.LMKAN_F32, 4), (binding.LMKAN_F16, 2), (binding.LMKAN_BF16, 2)):
            d = _desc(n_in=10, n_out=n_out, grid=5, coef_dtype=dt)
            assert pkg.lmkan_packed_bytes(d) == tiles * 5 * 36 * 64 * sz


def test_binding_refuses_host_tensors():
    import torch
    d = _desc()
    x = torch.zeros((4, 8))
    P = torch.zeros(d.coef_shape())
    with pytest.raises(ValueError):
        pkg.lmkan_forward(d, x, P)


def test_conv2d_rows_and_geometry_checks():
    """Output size by the floor rule; geometry that does not fit the layer is a shape error
    before any launch (the pointers are never dereferenced)."""
    assert pkg.lmkan_conv2d_rows(pkg.Conv2d(4, 32, 32, 6, 2, 2, 2)) == (4 * 16 * 16, 16, 16)
    assert pkg.lmkan_conv2d_rows(pkg.Conv2d(2, 9, 8, 3, 3, 2, 2)) == (2 * 4 * 4, 4, 4)
    assert pkg.lmkan_conv2d_rows(pkg.Conv2d(2, 7, 5, 2, 3, 3, 1)) == (2 * 5 * 3, 5, 3)
    assert pkg.lmkan_conv2d_rows(pkg.Conv2d(2, 2, 5, 2, 3, 3, 1)) == (0, 0, 3)   # image smaller than the window
    with pytest.raises(ValueError):
        pkg.lmkan_conv2d_rows(pkg.Conv2d(2, 8, 8, 2, 2, 2, 0))
    L = pkg.lib()
    fake = C.c_void_p(0x1000)
    d = _desc(n_in=8).c()
    good = pkg.Conv2d(1, 4, 4, 2, 2, 2, 2).c()
    for bad in (pkg.Conv2d(1, 4, 4, 3, 2, 2, 2), pkg.Conv2d(1, 4, 4, 2, 2, 2, 0), pkg.Conv2d(1, 0, 4, 2, 2, 2, 2),
                pkg.Conv2d(-1, 4, 4, 2, 2, 2, 2)):
        b = bad.c()
        assert L.lmkan_conv2d_forward(C.byref(d), C.byref(b), fake, fake, fake, None, 0, None) == 2
        assert L.lmkan_conv2d_backward(C.byref(d), C.byref(b), fake, fake, fake, fake, fake, None, 0, None) == 2
    assert L.lmkan_conv2d_forward(C.byref(d), None, fake, fake, fake, None, 0, None) == 1
    assert L.lmkan_conv2d_forward(C.byref(d), C.byref(good), None, fake, fake, None, 0, None) == 1
    odd = _desc(n_in=7).c()
    assert L.lmkan_conv2d_forward(C.byref(odd), C.byref(good), fake, fake, fake, None, 0, None) == 2


# ---- the check of the generated code of the kernels that issue their own loads and waits ----
_ASM_OK = """
kern:                                   ; @kern
\ts_load_dwordx2 s[0:1], s[4:5], 0x0
.LBB0_1:
\t;;#ASMSTART
\tglobal_load_dwordx4 v[4:7], v1, s[0:1]
\t;;#ASMEND
\tv_add_u32_e32 v1, 16, v1
\ts_cbranch_scc1 .LBB0_3
\tv_mov_b32_e32 v9, v2
.LBB0_3:
\t;;#ASMSTART
\ts_waitcnt vmcnt(1) ; landed v[4:7]
\t;;#ASMEND
\tv_add_f32_e32 v8, v4, v5
\ts_cbranch_scc0 .LBB0_1
\ts_endpgm
"""


def test_codegen_check_accepts_a_load_first_touched_by_its_wait():
    from paper_2509_07103_amd import check_codegen
    assert check_codegen.check_assembly(_ASM_OK) == {"kern": 1}


@pytest.mark.parametrize("planted", [
    "\tv_mov_b32_e32 v9, v5",            # a copy of a register still in flight
    "\tv_mov_b32_e32 v6, 0",             # the register handed to something else
    "\tv_add_f32_e32 v8, v[4:5], v2",    # named inside a register range
])
def test_codegen_check_rejects_a_touch_before_the_wait(planted):
    from paper_2509_07103_amd import check_codegen
    # on the branch that skips nothing: only the control flow graph reaches it from the load
    bad = _ASM_OK.replace("\tv_mov_b32_e32 v9, v2", planted)
    with pytest.raises(RuntimeError, match="touched before their wait"):
        check_codegen.check_assembly(bad)
    # and a wait that names other registers than the load's does not end the path
    other = _ASM_OK.replace("landed v[4:7]", "landed v[10:13]")
    with pytest.raises(RuntimeError, match="touched before their wait"):
        check_codegen.check_assembly(other)


def test_codegen_check_passes_on_the_library_sources():
    from paper_2509_07103_amd import check_codegen
    counts = check_codegen.check()
    assert len(counts) == 2 and all(n == 34 for n in counts.values()), counts


_REPORT = """\
a.hip:10:1: remark: Function Name: _ZN5lmkan12_GLOBAL__N_126backward_input_lane_kernelILi17EEEvNS_10GradInArgsE [-Rpass-analysis=kernel-resource-usage]
a.hip:10:1: remark:     VGPRs: 120 [-Rpass-analysis=kernel-resource-usage]
a.hip:10:1: remark:     ScratchSize [bytes/lane]: 0 [-Rpass-analysis=kernel-resource-usage]
a.hip:90:1: remark: Function Name: _ZN5lmkan12_GLOBAL__N_133backward_input_slab_narrow_kernelIfLi16ELi4EEEvNS_10GradInArgsE [-Rpass-analysis=kernel-resource-usage]
a.hip:90:1: remark:     VGPRs: 128 [-Rpass-analysis=kernel-resource-usage]
a.hip:90:1: remark:     ScratchSize [bytes/lane]: 56 [-Rpass-analysis=kernel-resource-usage]
"""


def test_resource_check_accepts_a_clean_report_and_catches_spills():
    """The build reads the compiler's resource report: a hot kernel with any scratch, any kernel
    with a spilled loop, or a report without kernels must raise (mistakes planted in the text)."""
    from paper_2509_07103_amd import check_codegen
    got = check_codegen.check_resources(_REPORT)
    assert sorted(got.values()) == [0, 56]
    with pytest.raises(RuntimeError, match="backward_input_lane_kernel"):
        check_codegen.check_resources(_REPORT.replace("[bytes/lane]: 0", "[bytes/lane]: 8"))
    with pytest.raises(RuntimeError, match="narrow"):
        check_codegen.check_resources(_REPORT.replace("[bytes/lane]: 56", "[bytes/lane]: 1132"))
    with pytest.raises(RuntimeError, match="no kernel"):
        check_codegen.check_resources("warning: nothing here")
