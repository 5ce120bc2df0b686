"""The shared library loads without a GPU and exports every symbol declared in include/kimad.h."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "kimad.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(kimad_[a-z_0-9]+)\s*\(", text)))


def test_header_declares_the_three_calls_of_the_path():
    names = _declared()
    for need in ("kimad_profile", "kimad_allocate", "kimad_compress_ef", "kimad_workspace_bytes", "kimad_strerror"):
        assert need in names


def test_library_exports_every_declared_symbol():
    import paper_2312_08053_amd as kimad
    if not os.path.exists(kimad.LIB_PATH):
        pytest.fail("libkimad.so is not built: run `python -m paper_2312_08053_amd.build`")
    lib = ctypes.CDLL(kimad.LIB_PATH)
    for name in _declared():
        assert hasattr(lib, name), f"{name} declared in kimad.h but not exported"
    assert sorted(kimad.EXPORTED_SYMBOLS) == _declared()


def test_host_side_argument_checks_need_no_gpu():
    import paper_2312_08053_amd as kimad
    assert kimad.kimad_workspace_bytes([100, 20000], 8) > 0
    with pytest.raises(kimad.KimadError) as e:
        kimad.kimad_workspace_bytes([100, 0], 8)                 # empty layer
    assert e.value.code == -1
    with pytest.raises(kimad.KimadError):
        kimad.kimad_workspace_bytes([100], 65)                   # too many ratios
    with pytest.raises(kimad.KimadError):
        kimad.kimad_workspace_bytes([], 4)
    assert kimad.kimad_strerror(-6).startswith("budget")
    # the exact cost axis without a budget limit would need L * d bytes of tables: refused above 4 GiB, not asked for
    gpt2_like = [38_597_376, 786_432] + [2_359_296] * 40
    with pytest.raises(kimad.KimadError) as e:
        kimad.kimad_workspace_bytes(gpt2_like, 64)
    assert e.value.code == -14
    assert kimad.kimad_workspace_bytes(gpt2_like, 64, D=1000) > 0
    assert kimad.kimad_workspace_bytes(gpt2_like, 64, D=0, max_budget_bytes=8 * 600_000) > 0
    # the exact-knapsack table grows with the largest budget the plan must serve
    small = kimad.kimad_workspace_bytes([100000] * 4, 8, D=0, max_budget_bytes=8 * 1000)
    large = kimad.kimad_workspace_bytes([100000] * 4, 8, D=0, max_budget_bytes=8 * 100000)
    assert large > small


def test_budget_rule_matches_the_oracle_on_the_host():
    """kimad_budget_bytes is host arithmetic (Section 3.1, Eq. budget): same integers as the oracle."""
    import numpy as np
    import paper_2312_08053_amd as kimad
    from oracle import kimad_oracle as ko
    rng = np.random.default_rng(9)
    for _ in range(2000):
        B = float(rng.choice([0.0, -1.0, np.nan, np.inf, rng.uniform(1e3, 4e11)], p=[.02, .02, .02, .02, .92]))
        tc = float(rng.uniform(0.0, 0.3))
        t = float(rng.choice([tc, tc - 0.1, tc + rng.uniform(1e-6, 2.0)], p=[.05, .05, .9]))
        alpha = float(rng.choice([1.0, 0.0, 0.5, 3.0, -1.0], p=[.6, .1, .1, .1, .1]))
        cap = int(rng.choice([0, 1, 12345, 4 * 124_439_808]))
        assert kimad.kimad_budget_bytes(B, t, tc, alpha, cap) == ko.budget_bytes(B, t, tc, alpha, cap), (B, t, tc, alpha, cap)
    # the paper's setting: alpha = 1, 30..330 Mbps, a 50 ms step of which 10 ms is computation
    assert kimad.kimad_budget_bytes(330e6, 0.05, 0.01) == 825000


def test_benchmark_refuses_more_than_one_gpu():
    """One worker is one GPU: bench.py --gpus N with N above 1 exits with a message, before any device work."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode == 2 and "one GPU" in r.stderr and r.stdout == ""


def test_product_package_never_imports_the_oracle():
    """The oracle is test infrastructure: no source line of the package or of the input generators imports it."""
    for pkg in ("paper_2312_08053_amd", "kimad_synth"):
        for dirpath, _, files in os.walk(os.path.join(ROOT, pkg)):
            for f in files:
                if not f.endswith((".py", ".h", ".hip")):
                    continue
                for line in open(os.path.join(dirpath, f)):
                    if "oracle" in line:
                        assert "import" not in line and "#include" not in line, (dirpath, f, line)


def test_workspace_is_a_quarter_of_the_gradient_buffers_at_most():
    """The candidate region of a tiled layer holds about a sixth of it, not all of it: a plan's workspace stays below a
    quarter of the bytes of g and h on the two benchmark shapes (host arithmetic only)."""
    import kimad_synth.shapes as shapes
    import paper_2312_08053_amd as kimad
    for sizes in (shapes.gpt2_small_shapes(), shapes.llama_shapes()):
        n = [shapes.numel(s) for s in sizes]
        ws = kimad.kimad_workspace_bytes(n, 64, D=1000)
        assert ws <= 0.25 * 8 * sum(n), (ws, 8 * sum(n))
