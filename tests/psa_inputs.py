"""Inputs for exact comparison of pivot index sets (not a test module).

The attention-mass pivot set of a (batch, kv-head) is the top-k of sums of softmax weights.  An fp32 implementation
reproduces the fp64 oracle's set only when the k-th and (k+1)-th masses are further apart than summation noise, so an
input is accepted for index-set parity only if the oracle's own fp64 margin (m_k - m_{k+1}) / m_k is at least
MIN_MARGIN in EVERY (batch, kv-head); otherwise the next seed is tried.  The search runs on the CPU, calls only the
oracle and the input generator, is deterministic, and is logged (printed; the searches of the named CPU test inputs are
also stored in tests/golden/psa_seed_search.txt by tests/golden/make_psa_seed_log.py).  Comparison is then exact set
equality.  Units whose margin is below REPORT_MARGIN are listed in the log.
"""
import numpy as np

MIN_MARGIN = 1e-4
REPORT_MARGIN = 1e-3
MAX_TRIES = 16


def _np(d):
    return {k: (v.cpu().numpy() if hasattr(v, "cpu") else v) for k, v in d.items()}


def oracle_masses(orc, w, d, top_k, share_heads=False, T=None):
    """The oracle's selection on host inputs d: (its cache with sal_idx / sal_cnt filled, fp64 masses [B,Hkv,T])."""
    T = T or d["k"].shape[2]
    oc = orc.OracleCache(w.B, w.Hkv, w.G, (T + 63) // 64 * 64, max(64, (top_k + 63) // 64 * 64))
    mass = oc.select_psa(d["q_tail"], d["k"][:, :, :T], top_k, w.sm_scale, want_mass=True, share_heads=share_heads)
    return oc, mass


def margins_of(orc, mass, top_k, share_heads=False):
    """[B,Hkv] margins (token-level pivots: one per batch element, on the masses added over its kv-heads)."""
    if share_heads:
        return orc.topk_margins(mass.sum(axis=1), top_k)
    return orc.topk_margins(mass, top_k)


def describe(margins):
    m = np.asarray(margins)
    tight = [(tuple(int(x) for x in ix), float(m[ix])) for ix in zip(*np.nonzero(m < REPORT_MARGIN))]
    return f"min margin {m.min():.3e}" + (f", below {REPORT_MARGIN:g}: " + ", ".join(
        f"{ix} {v:.2e}" for ix, v in tight) if tight else "")


def margin_checked(orc, generate, w, seed, top_k, share_heads=False, T=None, log=print, **gen_kw):
    """Draw generate(w, seed=s, **gen_kw) for s = seed, seed + 1, ... until every unit's margin is >= MIN_MARGIN.
    Returns (host inputs, accepted seed, oracle cache, masses, margins)."""
    for s in range(seed, seed + MAX_TRIES):
        d = _np(generate(w, seed=s, **gen_kw))
        oc, mass = oracle_masses(orc, w, d, top_k, share_heads, T)
        m = margins_of(orc, mass, top_k, share_heads)
        ok = bool((m >= MIN_MARGIN).all())
        log(f"psa seed search [{w.name} top_k={top_k}{' shared' if share_heads else ''}]: seed {s}: {describe(m)}: "
            + ("accepted" if ok else "rejected"))
        if ok:
            return d, s, oc, mass, m
    raise AssertionError(f"no seed in [{seed}, {seed + MAX_TRIES}) gives every unit of {w.name} a margin >= {MIN_MARGIN}")
