"""The three allocators of the paper's Kimad+ comparison (Section 4.3) through the library, against
totals assembled from the oracle's pinned functions."""
import numpy as np
import pytest

import kimad_synth as ks
from oracle import kimad_oracle as ko
from tests import gpu_harness as gh

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name,kw", [("resnet18", {}), ("gpt2", dict(n_layer=1, vocab=2053))])
def test_allocator_comparison_matches_the_oracle(name, kw):
    from paper_2312_08053_amd.baselines import allocator_errors
    work = ks.make_workload(name, **kw)
    g, h = gh.to_device(work)
    got = allocator_errors(g, h, work.sizes.tolist(), work.ratios.tolist(), work.budget_bytes,
                           work.pair_bytes, work.cost_units_D)
    gL, hL = gh.oracle_layers(work)
    # Kimad+: the oracle's allocation on the oracle's table
    E, Kt = ko.profile(gL, hL, work.ratios)
    st, j, K, off = ko.allocate(E, Kt, work.budget_bytes, work.pair_bytes, work.cost_units_D)
    assert st == ko.OK and got["kimad_plus"]["status"] == 0
    want_plus = float(sum(E[i, j[i]] for i in range(work.L)))
    assert got["kimad_plus"]["pairs"] == int(off[-1])
    assert abs(got["kimad_plus"]["error"] - want_plus) <= 1e-5 * want_plus
    # uniform ratio: K_i = ceil(rho d_i)
    P = work.budget_bytes // work.pair_bytes
    rho = P / work.d
    Ku = [int(ko.grid_sizes([rho], len(x))[0]) for x in gL]
    want_uni = float(sum(ko.topk_error_profile(ko.operand(gL[i], hL[i]), [Ku[i]])[0] for i in range(work.L)))
    assert got["uniform_ratio"]["pairs"] == sum(Ku)
    assert abs(got["uniform_ratio"]["error"] - want_uni) <= 1e-5 * want_uni
    # whole model: one TopK over the concatenation
    xall = ko.operand(work.g, work.h)
    Kw = int(ko.grid_sizes([rho], work.d)[0])
    want_whole = float(ko.topk_error_profile(xall, [Kw])[0])
    assert got["whole_model"]["pairs"] == Kw
    assert abs(got["whole_model"]["error"] - want_whole) <= 1e-5 * want_whole
    # what the paper's figure shows: the whole-model TopK is the floor for its own number of pairs
    assert got["whole_model"]["error"] <= got["uniform_ratio"]["error"] * (1 + 1e-9)
    assert np.array_equal(h.cpu().numpy().view(np.uint32), work.h.view(np.uint32))
