"""Pins of the oracle's offline fold of the rotation into projection weights (Section III-C.2, Fig. 7)."""
import numpy as np


def test_fold_equals_dense_hadamard_product(orc):
    rng = np.random.default_rng(5)
    H = orc.hadamard_dense(128)
    w = rng.standard_normal((96, 256)).astype(np.float16)          # like W_V: [d_model, Hkv*128]
    got = orc.fold_hadamard(w, 1).astype(np.float64)
    want = np.concatenate([w[:, :128].astype(np.float64) @ H, w[:, 128:].astype(np.float64) @ H], axis=1)
    assert np.abs(got - want).max() <= 2 ** -10 * np.abs(want).max() * 1.01
    w2 = rng.standard_normal((256, 80)).astype(np.float16)         # like W_O: [Hq*128, d_model]
    got2 = orc.fold_hadamard(w2, 0).astype(np.float64)
    want2 = np.concatenate([H @ w2[:128].astype(np.float64), H @ w2[128:].astype(np.float64)], axis=0)
    assert np.abs(got2 - want2).max() <= 2 ** -10 * np.abs(want2).max() * 1.01
    # H is its own inverse: folding twice returns the weights within two roundings
    back = orc.fold_hadamard(orc.fold_hadamard(w, 1), 1).astype(np.float64)
    assert np.abs(back - w.astype(np.float64)).max() <= 3 * 2 ** -10 * np.abs(w.astype(np.float64)).max()


def test_folded_projections_give_the_same_layer_output(orc):
    """x W_V H == x (W_V folded) and (o H)(W_O folded) == o W_O: the identities the offline mode relies on."""
    rng = np.random.default_rng(6)
    x = rng.standard_normal((7, 64))
    wv = (rng.standard_normal((64, 128)) / 8).astype(np.float16)
    wo = (rng.standard_normal((128, 64)) / 11).astype(np.float16)
    H = orc.hadamard_dense(128)
    v_rot = (x @ wv.astype(np.float64)) @ H
    assert np.abs(x @ orc.fold_hadamard(wv, 1).astype(np.float64) - v_rot).max() <= 5e-3 * np.abs(v_rot).max()
    o = rng.standard_normal((7, 128))
    ref = o @ wo.astype(np.float64)
    assert np.abs((o @ H) @ orc.fold_hadamard(wo, 0).astype(np.float64) - ref).max() <= 5e-3 * np.abs(ref).max()
