"""Pins of the oracle's rotary position embedding in front of the rotation (Section III-C.2 / Fig. 6 of
arXiv 2501.15021: Q and K are rotated after RoPE).  No GPU needed."""
import numpy as np

from paper_2501_15021_amd import synth

D = 128


def _rows(seed, n, B=1, H=2, scale=1.0):
    rng = np.random.default_rng(seed)
    return (rng.standard_normal((B, H, n, D)) * scale).astype(np.float16)


def test_position_zero_is_the_identity(orc):
    x = _rows(1, 3)
    cos, sin = synth.rope_tables(np.zeros(3))
    assert np.array_equal(orc.rope_rows(x, cos, sin).view(np.uint16), x.view(np.uint16))


def test_pairing_and_sign_hand_cases(orc):
    """Quarter turn (cos 0, sin 1): channel i moves to i + 64 with its sign, channel i + 64 moves to i negated."""
    x = np.zeros((1, 1, 2, D), dtype=np.float16)
    x[0, 0, 0, 5] = 2.0
    x[0, 0, 1, 64 + 9] = 3.0
    cos = np.zeros((2, 64), dtype=np.float16)
    sin = np.ones((2, 64), dtype=np.float16)
    y = orc.rope_rows(x, cos, sin)
    want = np.zeros_like(x)
    want[0, 0, 0, 64 + 5] = 2.0
    want[0, 0, 1, 9] = -3.0
    assert np.array_equal(y, want)
    # only channel i's own table entry is used
    cos = np.ones((2, 64), dtype=np.float16)
    sin = np.zeros((2, 64), dtype=np.float16)
    cos[0, 5], sin[0, 5] = 0.0, 1.0
    y = orc.rope_rows(x, cos, sin)
    want = x.copy()
    want[0, 0, 0, 5], want[0, 0, 0, 69] = 0.0, 2.0
    assert np.array_equal(y, want)


def test_against_complex_multiplication(orc):
    """(x_i + j x_{i+64}) * (cos + j sin) in complex128, with the same fp16 tables: within one rounding to binary32
    followed by one to binary16 (at most half an fp16 ulp plus the double rounding slack)."""
    n = 40
    x = _rows(2, n, B=2, H=3, scale=4.0)
    cos, sin = synth.rope_tables(np.arange(100, 100 + n))
    y = orc.rope_rows(x, cos, sin).astype(np.float64)
    z = (x[..., :64].astype(np.float64) + 1j * x[..., 64:].astype(np.float64)) * \
        (cos.astype(np.float64) + 1j * sin.astype(np.float64))
    exact = np.concatenate([z.real, z.imag], axis=-1)
    ulp = np.spacing(np.abs(exact).astype(np.float16)).astype(np.float64)
    assert np.all(np.abs(y - exact) <= 0.5 * ulp * (1 + 2 ** -10))
    # and bit-exact against the two roundings written out
    two_step = exact.astype(np.float32).astype(np.float16)
    assert np.array_equal(y.astype(np.float16).view(np.uint16), two_step.view(np.uint16))


def test_per_batch_tables(orc):
    x = _rows(3, 4, B=3, H=2)
    pos = np.array([[0, 1, 2, 3], [10, 11, 12, 13], [7, 7, 7, 7]])
    cos, sin = synth.rope_tables(pos)                       # [3, 4, 64]
    y = orc.rope_rows(x, cos, sin)
    for b in range(3):
        yb = orc.rope_rows(x[b:b + 1], cos[b], sin[b])      # shared-table form on one batch entry
        assert np.array_equal(y[b:b + 1].view(np.uint16), yb.view(np.uint16))


def test_relative_position_property(orc):
    """The point of the embedding: <rope(q, m), rope(k, n)> depends on m - n only (up to fp16 rounding of the rows)."""
    q = _rows(4, 1, H=1)
    k = _rows(5, 1, H=1)
    dots = []
    for shift in (0, 17, 300):
        cq, sq = synth.rope_tables(np.array([50 + shift]))
        ck, sk = synth.rope_tables(np.array([20 + shift]))
        a = orc.rope_rows(q, cq, sq).astype(np.float64).ravel()
        b = orc.rope_rows(k, ck, sk).astype(np.float64).ravel()
        dots.append(a @ b)
    scale = np.linalg.norm(q.astype(np.float64)) * np.linalg.norm(k.astype(np.float64))
    assert max(dots) - min(dots) <= 4e-3 * scale
    # and the norm of every (i, i + 64) pair is kept
    cq, sq = synth.rope_tables(np.array([123]))
    y = orc.rope_rows(q, cq, sq).astype(np.float64).ravel()
    x = q.astype(np.float64).ravel()
    assert np.allclose(y[:64] ** 2 + y[64:] ** 2, x[:64] ** 2 + x[64:] ** 2, rtol=4e-3, atol=1e-4)


def test_fused_write_path_is_rope_then_append(orc):
    """Handing pre-RoPE K to the write path equals applying the embedding first: the cache holds the rotation of the
    embedded rows (checked on the 16-bit rows of an all-salient cache against the dense transform)."""
    w = synth.small("rope", B=1, Hq=2, Hkv=2, T=20)
    d = synth.generate(w, seed=9)
    k, v = d["k"].numpy(), d["v"].numpy()
    cos, sin = synth.rope_tables(np.arange(20))
    c = orc.OracleCache(1, 2, 128, 64, 64)
    c.select_tsa(np.ones((1, 20), dtype=np.uint8))
    c.quantize_append(orc.rope_rows(k, cos, sin), v, 0.8)
    H = orc.hadamard_dense(D)
    want = orc.rope_rows(k, cos, sin).astype(np.float64) @ H
    got = orc.bf16_bits_to_f64(c.k_sal[0, :, :20])
    assert np.all(np.abs(got - want[0]) <= 2 ** -8 * np.abs(want[0]) + 1e-6)
