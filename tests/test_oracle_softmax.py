"""Pins for the oracle's row softmax (scale, optional causal mask; Alg. 2)."""
import numpy as np
import scipy.special

from oracle import ref, workloads


def test_against_scipy_and_closed_forms():
    rng = np.random.default_rng(1)
    x = rng.standard_normal((7, 13)) * 3
    got = ref.softmax_rows(x, scale=0.7)
    assert np.allclose(got, scipy.special.softmax(0.7 * x, axis=1), rtol=1e-14, atol=0)
    assert np.allclose(got.sum(axis=1), 1.0, rtol=1e-15)
    # a constant row is uniform; adding a constant to a row changes nothing
    assert np.array_equal(ref.softmax_rows(np.full((3, 8), 2.5)), np.full((3, 8), 0.125))
    assert np.allclose(ref.softmax_rows(x + 11.0, scale=0.7), got, rtol=1e-12)
    # two-element row: logistic function of the difference
    two = ref.softmax_rows(np.array([[1.0, 3.0]]))
    assert abs(two[0, 1] - 1.0 / (1.0 + np.exp(-2.0))) < 1e-16
    # huge entries do not overflow, one dominant entry takes everything
    big = ref.softmax_rows(np.array([[1000.0, 0.0, -1000.0]]))
    assert big[0, 0] == 1.0 and big[0, 2] == 0.0


def test_causal_mask():
    rng = np.random.default_rng(2)
    x = rng.standard_normal((5, 5))
    got = ref.softmax_rows(x, scale=2.0, causal=True)
    assert np.array_equal(np.triu(got, 1), np.zeros((5, 5)))          # future keys get exactly 0
    assert got[0, 0] == 1.0
    for i in range(5):
        assert np.allclose(got[i, :i + 1], scipy.special.softmax(2.0 * x[i, :i + 1]), rtol=1e-14)
    # rectangular: the last row sees every column
    r = ref.softmax_rows(rng.standard_normal((2, 6)), causal=True)
    assert np.all(r[1] > 0) and r[0, 5] == 0.0 and r[0, 4] > 0


def test_attention_with_softmax_matches_numpy():
    rng = np.random.default_rng(3)
    Q, K, V = (rng.standard_normal((2, 9, 16)) for _ in range(3))
    out = workloads.attention({"Q": Q, "K": K, "V": V}, softmax=True, causal=True, keep_s=True)
    for h in range(2):
        logits = Q[h] @ K[h].T / 4.0
        logits = np.where(np.tril(np.ones((9, 9), dtype=bool)), logits, -np.inf)
        P = scipy.special.softmax(logits, axis=1)
        assert np.allclose(out["S"][h], P, rtol=1e-13, atol=1e-300)
        assert ref.rel_frobenius(out["O"][h], P @ V[h]) <= 1e-13
