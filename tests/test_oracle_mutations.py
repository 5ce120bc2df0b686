"""Do the pins bite?  Plausible slips are planted in a copy of the oracle's source (on the CPU, never
in the library), and the pin tests are run against each mutant: every one of them must turn some pin red.

A mutant is one textual replacement in oracle/kimad_oracle.py, loaded under the oracle's module name in a
child interpreter that then runs the pin files.  The list names the kind of mistake each stands for.
Two replacements are known to be equivalent (the dynamic programme started from a row of zeros computes "cost
at most c" instead of "cost exactly c", and every output the oracle returns is the same; a uniform ratio above 1
is clamped by the grid-size rule): they are kept here as such, and must stay green.
"""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SOURCE = os.path.join(ROOT, "oracle", "kimad_oracle.py")
PIN_FILES = ["tests/test_oracle_topk.py", "tests/test_oracle_ef.py", "tests/test_oracle_alloc.py",
             "tests/test_oracle_server.py", "tests/test_oracle_budget.py", "tests/test_oracle_variants.py"]

MUTANTS = [
    ("tie in the DP goes to the later candidate", "better = t < cur[wij:]", "better = t <= cur[wij:]"),
    ("final argmin takes the largest cost", "c = int(np.argmax(prev == best))",
     "c = int(len(prev)-1-np.argmax(prev[::-1] == best))"),
    ("operand g + h", "np.subtract(g, h, dtype=np.float32)", "np.add(g, h, dtype=np.float32)"),
    ("unstable sort: ties in any order", 'return np.argsort(-key, kind="stable")', "return np.argsort(-key)"),
    ("sign kept in the magnitude key", "& np.uint32(0x7FFFFFFF)", "& np.uint32(0xFFFFFFFF)"),
    ("errors summed from the largest entry", "sq = x[pi[::-1]]", "sq = x[pi]"),
    ("grid size one too small", "out[j] = min(int(n), max(1, k))", "out[j] = min(int(n), max(1, k-1))"),
    ("costs rounded down", "w = -(-np.asarray(K_table, dtype=np.int64) // unit)",
     "w = np.asarray(K_table, dtype=np.int64) // unit"),
    ("estimator set to g on the support", "h_new[idx] = np.add(h_new[idx], val, dtype=np.float32)",
     "h_new[idx] = g[idx]"),
    ("walk back with the first candidate's cost", "c -= int(w[i, j_out[i]])", "c -= int(w[i, 0])"),
    ("payload in magnitude order", "idx = np.sort(topk_support(x, int(K))).astype(np.uint32)",
     "idx = topk_support(x, int(K)).astype(np.uint32)"),
    ("capacity rounded up", "cap = P // unit", "cap = -(-P // unit)"),
    ("one dropped entry too few", "dropped = n - int(K)", "dropped = n - int(K) - 1 if K < n else 0"),
    ("server sum accumulated in fp32", "acc = acc + np.float64(weights[m]) * new_hats[m].astype(np.float64)",
     "acc = (acc + np.float32(weights[m]) * new_hats[m]).astype(np.float32)"),
    ("server overwrites the estimator entry", "u[where] = u[where] + v", "u[where] = v"),
    ("budget rule without the down-link share", "c_bits = B * (t - t_comp) / (1.0 + alpha)",
     "c_bits = B * (t - t_comp) / 2.0"),
    ("dense fallback only beyond the break-even", "dense = K_table * int(pair_bytes) >= n * int(value_bytes)",
     "dense = K_table * int(pair_bytes) > n * int(value_bytes)"),
    ("dense layer charged rounded down", "dense_pairs = -(-(n * int(value_bytes)) // int(pair_bytes))",
     "dense_pairs = (n * int(value_bytes)) // int(pair_bytes)"),
    ("half-precision values saturate to infinity", "np.clip(v, np.float32(-65504.0), np.float32(65504.0))",
     "np.clip(v, np.float32(-1e30), np.float32(1e30))"),
    ("uniform ratio from the budget in bytes", "rho = min(1.0, P / d)", "rho = min(1.0, int(budget_bytes) / d)"),
    ("whole-model selection ignores the estimator", "x = np.concatenate([operand(g, h) for g, h in zip(g_layers, h_layers)])",
     "x = np.concatenate([np.asarray(g, dtype=np.float32) for g, h in zip(g_layers, h_layers)])"),
    ("whole-model count of the next layer", "out.append(int(kept[pos:pos + len(g)].sum()))",
     "out.append(int(kept[pos + 1:pos + 1 + len(g)].sum()))"),
]
EQUIVALENT = [
    ("DP started from a row of zeros", "prev[0] = 0.0", "prev[:] = 0.0"),
    ("uniform ratio not capped at 1 (the grid-size rule clamps K to the layer anyway)", "rho = min(1.0, P / d)", "rho = P / d"),
]

_DRIVER = r"""
import importlib.util, sys, types
src, a, b = sys.argv[1], sys.argv[2], sys.argv[3]
text = open(src).read()
assert text.count(a) == 1, "anchor of the mutation must occur exactly once"
import oracle
spec = importlib.util.spec_from_loader("oracle.kimad_oracle", loader=None)
mod = types.ModuleType("oracle.kimad_oracle")
mod.__file__ = src
mod.__package__ = "oracle"
sys.modules["oracle.kimad_oracle"] = mod
exec(compile(text.replace(a, b), src + " (mutant)", "exec"), mod.__dict__)
oracle.kimad_oracle = mod
import pytest
sys.exit(pytest.main(["-x", "-q", "-p", "no:cacheprovider", "-m", "not gpu"] + sys.argv[4:]))
"""


def _run(a, b):
    env = dict(os.environ, PYTHONPATH=ROOT + os.pathsep + os.environ.get("PYTHONPATH", ""))
    return subprocess.run([sys.executable, "-c", _DRIVER, SOURCE, a, b] + PIN_FILES, cwd=ROOT, env=env,
                          capture_output=True, text=True, timeout=300)


@pytest.mark.parametrize("what,a,b", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_a_planted_mistake_fails_a_pin(what, a, b):
    r = _run(a, b)
    assert "anchor of the mutation" not in r.stderr, r.stderr[-400:]
    assert r.returncode == 1 and (" failed" in r.stdout or " error" in r.stdout), (what, r.stdout[-600:], r.stderr[-300:])


@pytest.mark.parametrize("what,a,b", EQUIVALENT, ids=[m[0] for m in EQUIVALENT])
def test_the_known_equivalent_rewrite_stays_green(what, a, b):
    r = _run(a, b)
    assert r.returncode == 0, (what, r.stdout[-600:], r.stderr[-300:])
