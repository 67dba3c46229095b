"""Host-side checks that need no GPU: the library loads, exports what the header declares, and its
pure host functions agree with exact arithmetic."""
import math
import os
import re
from fractions import Fraction

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def pac():
    import paper_2505_18563_amd as pac_mod
    pac_mod.load_library()
    return pac_mod


def declared_functions():
    text = open(os.path.join(ROOT, "include", "pactrain.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(pac_[a-z_0-9]+)\s*\(", text)))


def test_header_declares_the_four_path_calls():
    names = declared_functions()
    for must in ("pac_build_mask", "pac_compress", "pac_reduce_local", "pac_decompress",
                 "pac_create", "pac_destroy", "pac_keep_count", "pac_mask_words", "pac_last_error"):
        assert must in names


def test_library_exports_every_declared_symbol(pac):
    lib = pac.load_library()
    for name in declared_functions():
        assert hasattr(lib, name), f"{name} declared in pactrain.h but not exported"


def test_library_is_built_from_hip_sources_in_tree(pac):
    path = pac.library_path()
    assert os.path.dirname(path) == os.path.join(ROOT, "paper_2505_18563_amd")
    assert os.path.exists(path)


def test_keep_count_host_rule(pac):
    rng = np.random.default_rng(3)
    for _ in range(2000):
        n = int(rng.integers(0, 2**32 - 1))
        ppm = int(rng.integers(0, 1000001))
        s_text = f"{ppm / 1e6:.6f}"
        assert pac.pac_keep_count(n, float(s_text)) == math.ceil((1 - Fraction(s_text)) * n)
    rows = [l.split() for l in open(os.path.join(ROOT, "tests", "golden", "keep_counts.txt"))
            if l.strip() and not l.startswith("#")]
    for n, s, k in rows:
        assert pac.pac_keep_count(int(n), float(s)) == int(k)
    assert pac.pac_keep_count(10, 1.5) == 0 and pac.pac_keep_count(10, float("nan")) == 0


def test_mask_words(pac):
    for n, w in ((0, 0), (1, 1), (64, 1), (65, 2), (2**32 - 1, 2**26)):
        assert pac.pac_mask_words(n) == w


def test_create_without_gpu_fails_with_status_not_crash(pac):
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    with pytest.raises(pac.PacError) as e:
        pac.pac_create(0, 1000, 1)
    assert e.value.status in (-5, -1)


def test_product_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2505_18563_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.lower(), f"{f} mentions the oracle"


def test_per_tensor_keep_totals_of_the_configurations(pac):
    """nnz of a per-tensor prune = sum of the tensors' keep counts: the library's host rule and the oracle's
    against the totals worked by exact arithmetic (tests/golden/keep_totals_per_tensor.txt)."""
    import oracle
    from synth.shapes import config_shapes, flat_size
    rows = [l.split() for l in open(os.path.join(ROOT, "tests", "golden", "keep_totals_per_tensor.txt"))
            if l.strip() and not l.startswith("#")]
    assert len(rows) >= 9
    for cid, n, s, total in rows:
        specs = config_shapes(int(cid))
        assert flat_size(specs) == int(n)
        assert sum(pac.pac_keep_count(t.numel, float(s)) for t in specs) == int(total)
        assert sum(oracle.keep_count(t.numel, float(s)) for t in specs) == int(total)


def test_bench_refuses_more_than_one_gpu_before_touching_a_device():
    """The benchmark is a one-GPU program: --gpus above 1 ends with a message and a non-zero status, on a
    machine without a GPU as well (it decides before anything initialises a device)."""
    import subprocess
    import sys
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert p.returncode != 0
    assert "ONE GPU" in (p.stdout + p.stderr)
    assert not any(line.startswith("{") for line in p.stdout.splitlines())


def test_committed_traffic_summary_is_what_the_bench_line_quotes():
    """roofline.traffic comes from the committed counter summary: the file must carry the figure, within a few
    percent of the kernel's algorithmic bytes (a summary of some other kernel or workload would not be)."""
    sys_path_bench = os.path.join(ROOT, "bench.py")
    import importlib.util
    spec = importlib.util.spec_from_file_location("bench_for_test", sys_path_bench)
    bench = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(bench)
    t = bench.measured_traffic(bench.HEADLINE)
    assert t is not None
    n, k = 354823168, 35482317
    algorithmic = 2 * n + 3 * ((n + 63) // 64) * 4 + 2 * k      # bf16 gradient + mask and prefix words + compact buffer
    assert algorithmic == 847140314
    assert 1.0 <= t / algorithmic < 1.03
    assert bench.measured_traffic(3) is None
