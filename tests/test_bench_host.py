"""Host-side checks of bench.py and the workload recipes that need no GPU."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_bench_refuses_more_than_one_gpu():
    """This build measures one GPU; asking for more must end with a message, not a number."""
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                         capture_output=True, text=True, timeout=120)
    assert res.returncode != 0
    assert "one GPU" in res.stderr
    assert res.stdout.strip() == ""


def test_workload_shapes_match_the_configurations():
    from paper_2509_07103_amd import workloads as wl
    assert (wl.CFG1.n_in, wl.CFG1.n_out, wl.CFG1.grid, wl.CFG1.batch) == (16, 16, 8, 256)
    assert [(w.n_in, w.n_out) for w in wl.CFG2_LAYERS] == [(64, 256), (256, 256), (256, 256), (256, 1)]
    assert (wl.CFG3.n_in, wl.CFG3.n_out, wl.CFG3.grid, wl.CFG3.batch) == (1024, 1024, 16, 8192)
    assert (wl.CFG4.n_in, wl.CFG4.n_out, wl.CFG4.grid, wl.CFG4.batch) == (128, 128, 12, 262144)
    assert (wl.CFG5.n_in, wl.CFG5.n_out, wl.CFG5.grid, wl.CFG5.batch) == (4096, 4096, 32, 4096)
    for w in wl.CONV_BY_NAME.values():
        oh, ow = w.out_hw
        assert w.n_in == w.kh * w.kw * w.c_in and w.n_in % 2 == 0
        assert w.batch == w.n * oh * ow


@pytest.mark.parametrize("name", ["cfg1_16x16_G8", "conv_3x3s1_16x16x32_to_64_G12"])
def test_inputs_are_seeded(name):
    import torch
    from paper_2509_07103_amd import workloads as wl
    w = wl.BY_NAME.get(name) or wl.CONV_BY_NAME[name]
    make = wl.make_image if name in wl.CONV_BY_NAME else wl.make_x
    a, b = make(w, torch.device("cpu")), make(w, torch.device("cpu"))
    assert torch.equal(a, b)
    assert torch.equal(wl.make_coef(w, "cpu"), wl.make_coef(w, "cpu"))


def test_the_product_never_touches_the_oracle():
    """The oracle is test infrastructure: nothing under the package may import or load it, and the
    package has no CPU path to fall back on (a missing library is an ImportError)."""
    import re
    pkg_dir = os.path.join(ROOT, "paper_2509_07103_amd")
    for dirpath, _, files in os.walk(pkg_dir):
        for fn in files:
            if fn.endswith((".py", ".hip", ".h")):
                text = open(os.path.join(dirpath, fn)).read()
                assert not re.search(r"^\s*(import|from)\s+oracle\b|oracle\.(get|build)|liblmkan_oracle", text, re.M), \
                    f"{fn} uses the oracle"
    # bench.py imports it in one place only: the CPU-baseline leg, which runs after every timed region
    bench = open(os.path.join(ROOT, "bench.py")).read()
    assert bench.count("import oracle") == 1
    assert bench.index("import oracle") > bench.index("def cpu_baseline(")
    assert bench.index("b.cpu_baseline(") > bench.index('out["configs"] = configs')


def test_traffic_figures_name_kernels_that_exist():
    """bench.py takes roofline.traffic from the counter summaries under profiles/, looked up by kernel name.
    A summary that names a kernel the sources no longer define is stale: fail here rather than print it."""
    import re
    import bench
    src = ""
    csrc = os.path.join(ROOT, "paper_2509_07103_amd", "csrc")
    for fn in os.listdir(csrc):
        src += open(os.path.join(csrc, fn)).read()
    seen = 0
    for fn in sorted(os.listdir(os.path.join(ROOT, "profiles"))):
        m = re.fullmatch(r"bench_(.+)_(f32|f16|bf16)_hbm_counters\.md", fn)
        if not m:
            continue
        for line in open(os.path.join(ROOT, "profiles", fn)):
            cells = [c.strip() for c in line.strip().strip("|").split("|")]
            if len(cells) >= 2 and re.fullmatch(r"[a-z_0-9]+_kernel", cells[0]):
                assert re.search(r"\b%s\b" % cells[0], src), f"{fn} names {cells[0]}, which no source defines"
                got, where = bench.profile_traffic(m.group(1), m.group(2), cells[0])
                assert got is not None and got > 0, (fn, cells[0], where)
                seen += 1
    assert seen >= 3
    assert bench.profile_traffic("cfg3_1024x1024_G16", "f32", "no_such_kernel")[0] is None


def test_missing_library_is_a_loud_error(tmp_path, monkeypatch):
    from paper_2509_07103_amd import binding
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", str(tmp_path / "liblmkan.so"))
    with pytest.raises(ImportError):
        binding.lib()
