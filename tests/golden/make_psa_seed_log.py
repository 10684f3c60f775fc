#!/usr/bin/env python3
"""Writes tests/golden/psa_seed_search.txt: the seed search of the index-set parity protocol (tests/psa_inputs.py) for
the pivot-selection inputs that are generated on the CPU (configuration 1, the smoke input and the named small cases
of tests/test_gpu_parity.py).  Calls the oracle and the input generator only; no GPU, no GPU library.

    python tests/golden/make_psa_seed_log.py
"""
import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.dirname(HERE))

import psa_inputs  # noqa: E402
from oracle import pyoracle as orc  # noqa: E402
from paper_2501_15021_amd import synth  # noqa: E402


def cases():
    """(workload, first seed, top_k, token-level) of every named CPU-generated pivot-selection input."""
    w = synth.WORKLOADS["cfg1"]
    yield w, synth.BASE_SEED, w.top_k, False
    yield synth.small("smoke", B=2, Hq=4, Hkv=4, T=200, G=128, n_text_head=20, n_text_tail=12, top_k=8, W=16), 7, 8, False
    yield synth.small("psa", B=2, Hq=4, Hkv=2, T=300, W=16, top_k=8), 106, 8, False
    long = synth.small("psa_long", B=1, Hq=2, Hkv=1, T=33111, W=16, top_k=12, n_text_head=40, n_text_tail=31)
    yield long, 161, 12, False
    yield long, 161, 300, False
    for Hq, Hkv, T, top_k in ((6, 3, 500, 7), (8, 8, 2100, 16), (14, 2, 333, 4)):
        yield synth.small(f"psa_sh{Hq}", B=2, Hq=Hq, Hkv=Hkv, T=T, W=16, top_k=top_k, n_text_head=9, n_text_tail=4), \
            221, top_k, True


def search_log():
    lines = []
    for w, seed, top_k, shared in cases():
        psa_inputs.margin_checked(orc, synth.generate, w, seed, top_k, shared, log=lines.append)
    return lines


if __name__ == "__main__":
    out = os.path.join(HERE, "psa_seed_search.txt")
    with open(out, "w") as f:
        f.write("# Seed search of the pivot index-set parity protocol: a seed is accepted when the oracle's fp64 masses leave\n"
                "# (m_k - m_{k+1}) / m_k >= 1e-4 in every (batch, kv-head); units below 1e-3 are listed.  Written by\n"
                "# tests/golden/make_psa_seed_log.py (oracle and input generator only).\n")
        for line in search_log():
            f.write(line + "\n")
    print(open(out).read())
