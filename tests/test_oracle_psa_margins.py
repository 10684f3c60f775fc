"""The index-set parity protocol on the CPU: the margin function by hand, the seed search (a tie is rejected and the
next seed taken), and the stored search log of the named inputs is what the search gives today."""
import os

import numpy as np

import psa_inputs
from paper_2501_15021_amd import synth

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def test_topk_margins_by_hand(orc):
    m = np.array([[0.5, 4.0, 1.0, 2.0, 0.25],
                  [3.0, 3.0, 1.0, 0.0, 0.0]])
    assert np.allclose(orc.topk_margins(m, 1), [(4 - 2) / 4, 0.0])          # second row: a tie at the top
    assert np.allclose(orc.topk_margins(m, 2), [(2 - 1) / 2, (3 - 1) / 3])
    assert np.allclose(orc.topk_margins(m, 3), [(1 - 0.5) / 1, 1.0])
    assert np.allclose(orc.topk_margins(m, 4), [0.5, 0.0])                  # second row: k-th mass is zero -> no gap
    assert np.isinf(orc.topk_margins(m, 5)).all()                           # nothing is left out: any set is the set
    assert orc.topk_margins(m[None], 2).shape == (1, 2)


def test_margin_is_that_of_the_oracles_own_selection(orc):
    """The set the oracle stores is the k largest masses, and the margin is the gap to the best one left out."""
    w = synth.small("margin", B=2, Hq=4, Hkv=2, T=150, W=16, top_k=6)
    d = {k: v.numpy() for k, v in synth.generate(w, seed=31).items()}
    oc, mass = psa_inputs.oracle_masses(orc, w, d, 6)
    margins = psa_inputs.margins_of(orc, mass, 6)
    for b in range(w.B):
        for h in range(w.Hkv):
            chosen = oc.sal_idx[b, h, :6]
            rest = np.setdiff1d(np.arange(w.T), chosen)
            lo, hi = mass[b, h, chosen].min(), mass[b, h, rest].max()
            assert lo > hi
            assert np.isclose(margins[b, h], (lo - hi) / lo, rtol=1e-12)


def test_seed_search_rejects_a_tie_and_moves_on(orc):
    w = synth.small("tie", B=1, Hq=2, Hkv=2, T=120, W=16, top_k=1)
    first = 41

    def generate(w_, seed):
        d = synth.generate(w_, seed=seed)
        if seed == first:                       # two identical dominant keys, both visible to every scoring row
            d["k"][:, :, 7] = d["k"][:, :, 0]
        return d

    log = []
    d, seed, oc, mass, m = psa_inputs.margin_checked(orc, generate, w, first, 1, log=log.append)
    assert seed == first + 1 and len(log) == 2
    assert "rejected" in log[0] and "min margin 0.000e+00" in log[0] and "accepted" in log[1]
    assert (m >= psa_inputs.MIN_MARGIN).all()


def test_stored_seed_search_log_is_current(orc):
    import importlib.util
    spec = importlib.util.spec_from_file_location("make_psa_seed_log", os.path.join(GOLDEN, "make_psa_seed_log.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    stored = [l.rstrip("\n") for l in open(os.path.join(GOLDEN, "psa_seed_search.txt")) if not l.startswith("#")]
    assert stored == mod.search_log()
    assert any("[cfg1 top_k=8]" in l and "accepted" in l for l in stored)
