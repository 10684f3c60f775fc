"""Pins of the oracle's massive-activation pivot identification (Section III-B.2)."""
import numpy as np

from paper_2501_15021_amd import synth


def test_planted_massive_activations_are_the_pivots(orc):
    w = synth.small("ma", B=3, Hq=4, Hkv=2, T=300)
    d = synth.generate(w, seed=7)
    hid = synth.hidden_states(w, d["pivots"], d_model=256, seed=7).numpy()
    oc = orc.OracleCache(w.B, w.Hkv, w.G, 320, 64)
    score = oc.select_massive(hid, 15, floor=100.0, want_score=True)
    for b in range(w.B):
        want = sorted(set(int(x) for x in d["pivots"][b]))
        for h in range(w.Hkv):
            assert oc.sal_cnt[b, h] == len(want)                      # fewer than 15 pass the floor
            assert oc.sal_idx[b, h, :len(want)].tolist() == want
        assert np.array_equal(score[b], np.abs(hid[b].astype(np.float64)).max(axis=-1))


def test_top_k_by_full_sort_ties_and_floor(orc):
    rng = np.random.default_rng(3)
    B, T, dm = 2, 90, 64
    hid = rng.standard_normal((B, T, dm)).astype(np.float16)
    hid[0, 10, 3] = hid[0, 40, 9] = 77.0          # a tie: the lower position wins when only one fits
    hid[0, 70, 0] = -90.0
    oc = orc.OracleCache(B, 2, 128, 128, 64)
    oc.select_massive(hid, 2, floor=0.0)
    assert oc.sal_idx[0, 0, :2].tolist() == [10, 70] and oc.sal_cnt[0, 1] == 2
    for k in (1, 5, 17):
        oc.select_massive(hid, k, floor=0.0)
        for b in range(B):
            sc = np.abs(hid[b].astype(np.float64)).max(axis=-1)
            order = sorted(range(T), key=lambda t: (-sc[t], t))[:k]
            assert oc.sal_idx[b, 0, :k].tolist() == sorted(order)
    oc.select_massive(hid, 8, floor=80.0)
    assert oc.sal_cnt[0, 0] == 1 and oc.sal_idx[0, 0, 0] == 70 and oc.sal_cnt[1, 0] == 0
