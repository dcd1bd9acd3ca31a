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
    bench = open(os.path.join(ROOT, "bench.py")).read()
    assert bench.count("import oracle") == 1 and bench.index("import oracle") > bench.index("if not args.no_cpu_baseline")


def test_missing_library_is_a_loud_error(tmp_path, monkeypatch):
    from paper_2509_07103_amd import binding
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", str(tmp_path / "liblmkan.so"))
    with pytest.raises(ImportError):
        binding.lib()
