"""Pins for the CPU oracle's GEMM and chain (Eq. 1, Eq. 2).

Each test checks the oracle against something other than itself: a hand-worked
example, exact rational arithmetic on every small shape, numpy's einsum, closed
forms, identity/permutation matrices, integer-valued associativity, and numpy's
own fp64 matmul.
"""
import itertools
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import ref, workloads

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _read_blocks(path):
    blocks, cur = [], []
    for line in open(path):
        line = line.strip()
        if not line:
            continue
        if line.startswith("#"):
            if cur:
                blocks.append(np.array(cur, dtype=np.float64))
                cur = []
            continue
        cur.append([float(t) for t in line.split()])
    if cur:
        blocks.append(np.array(cur, dtype=np.float64))
    return blocks


def test_hand_worked_example():
    A, B, C, ab, AB, full = _read_blocks(os.path.join(GOLDEN, "gemm_hand_2x3x2.txt"))
    alpha, beta = ab[0]
    assert np.array_equal(ref.gemm(A, B), AB)
    assert np.array_equal(ref.gemm(A, B, alpha=alpha, beta=beta, C=C), full)


SIZES = (1, 2, 3, 5, 8, 17, 33)


def test_against_einsum_all_small_shapes():
    """Every shape in SIZES^3 (the degenerate 1s, odd sizes, one past a power of two) against the
    definition written as a single einsum in fp64."""
    rng = np.random.default_rng(7)
    for m, n, k in itertools.product(SIZES, SIZES, SIZES):
        A = rng.uniform(-1, 1, (m, k))
        B = rng.uniform(-1, 1, (k, n))
        C = rng.uniform(-1, 1, (m, n))
        got = ref.gemm(A, B, alpha=0.75, beta=-1.5, C=C)
        want = 0.75 * np.einsum("il,lj->ij", A, B) - 1.5 * C
        # two summation orders of k terms: a few ulps of the magnitudes involved
        bound = 4 * (k + 2) * np.finfo(np.float64).eps * (np.abs(A) @ np.abs(B) + np.abs(C) * 1.5)
        assert np.all(np.abs(got - want) <= bound), (m, n, k)


def test_against_exact_rational_arithmetic():
    """Brute force: every element of every shape in {1, 2, 3, 5, 8}^3 recomputed in exact rational
    arithmetic from Eq. 1 (a wrong index, a transposed operand or a dropped term cannot pass)."""
    rng = np.random.default_rng(11)
    small = (1, 2, 3, 5, 8)
    for m, n, k in itertools.product(small, small, small):
        A = rng.uniform(-1, 1, (m, k))
        B = rng.uniform(-1, 1, (k, n))
        C = rng.uniform(-1, 1, (m, n))
        alpha, beta = 1.25, 0.5
        got = ref.gemm(A, B, alpha=alpha, beta=beta, C=C)
        fa = [[Fraction(x) for x in row] for row in A]
        fb = [[Fraction(x) for x in row] for row in B]
        for i in range(m):
            for j in range(n):
                exact = Fraction(alpha) * sum(fa[i][l] * fb[l][j] for l in range(k)) + Fraction(beta) * Fraction(C[i, j])
                mag = alpha * sum(abs(A[i, l] * B[l, j]) for l in range(k)) + abs(beta * C[i, j])
                assert abs(Fraction(got[i, j]) - exact) <= (k + 3) * np.finfo(np.float64).eps * mag, (m, n, k, i, j)


def test_identity_and_permutation_are_exact():
    rng = np.random.default_rng(3)
    A = rng.standard_normal((13, 9))
    assert np.array_equal(ref.gemm(A, np.eye(9)), A)
    assert np.array_equal(ref.gemm(np.eye(13), A), A)
    perm = rng.permutation(13)
    P = np.eye(13)[perm]
    assert np.array_equal(ref.gemm(P, A), A[perm])            # P*A permutes rows
    cperm = rng.permutation(9)
    assert np.array_equal(ref.gemm(A, np.eye(9)[:, cperm]), A[:, cperm])


def test_closed_forms():
    m, k, n = 6, 37, 5
    assert np.array_equal(ref.gemm(np.ones((m, k)), np.ones((k, n))), np.full((m, n), float(k)))
    # rank one times rank one: (u v^T)(w z^T) = (v.w) u z^T, integer-valued so exact
    u, v = np.arange(1, 5.0), np.arange(-3, 4.0)
    w, z = np.arange(2, 9.0), np.arange(1, 4.0)
    got = ref.gemm(np.outer(u, v), np.outer(w, z))
    assert np.array_equal(got, float(v @ w) * np.outer(u, z))
    # diagonal scaling
    A = np.arange(12.0).reshape(3, 4)
    d = np.array([2.0, -1.0, 0.5, 4.0])
    assert np.array_equal(ref.gemm(A, np.diag(d)), A * d)
    assert np.array_equal(ref.gemm(np.diag([3.0, 0.0, -2.0]), A), A * np.array([[3.0], [0.0], [-2.0]]))
    # chain of all-ones matrices: product of the inner dimensions
    out = ref.chain(np.ones((2, 3)), [np.ones((3, 4)), np.ones((4, 5)), np.ones((5, 2))])
    assert np.array_equal(out, np.full((2, 2), 3.0 * 4.0 * 5.0))


def test_agrees_with_numpy_matmul():
    rng = np.random.default_rng(5)
    A = rng.standard_normal((67, 129))
    B = rng.standard_normal((129, 45))
    C = rng.standard_normal((67, 45))
    assert ref.rel_frobenius(ref.gemm(A, B), A @ B) <= 1e-13
    assert ref.rel_frobenius(ref.gemm(A, B, 0.3, -2.0, C), 0.3 * (A @ B) - 2.0 * C) <= 1e-13


def test_alpha_beta_semantics():
    rng = np.random.default_rng(9)
    A = rng.integers(-2, 3, (7, 11)).astype(np.float64)
    B = rng.integers(-2, 3, (11, 4)).astype(np.float64)
    C = rng.integers(-5, 6, (7, 4)).astype(np.float64)
    assert np.array_equal(ref.gemm(A, B, alpha=0.0, beta=3.0, C=C), 3.0 * C)
    nan_c = np.full((7, 4), np.nan)
    assert np.array_equal(ref.gemm(A, B, alpha=1.0, beta=0.0, C=nan_c), ref.gemm(A, B))
    assert np.array_equal(ref.gemm(A, B, alpha=2.0, beta=-1.0, C=C), 2.0 * ref.gemm(A, B) - C)
    assert np.array_equal(ref.gemm(A, B, alpha=1.0, beta=1.0, C=C), ref.gemm(A, B) + C)
    with pytest.raises(ValueError):
        ref.gemm(A, B, beta=1.0)
    with pytest.raises(ValueError):
        ref.gemm(A, A)


def test_integer_valued_associativity_is_bit_exact():
    rng = np.random.default_rng(21)
    A = rng.integers(-2, 3, (40, 64)).astype(np.float64)
    B = rng.integers(-2, 3, (64, 48)).astype(np.float64)
    C = rng.integers(-2, 3, (48, 24)).astype(np.float64)
    left = ref.gemm(ref.gemm(A, B), C)
    right = ref.gemm(A, ref.gemm(B, C))
    assert np.array_equal(left, right)
    assert np.array_equal(left, ref.chain(A, [B, C]))
    assert np.abs(left).max() < 2 ** 24           # also exact in fp32
    assert np.array_equal(ref.round_f32(left), left)


def test_workload_functions_reduce_to_gemm():
    rng = np.random.default_rng(2)
    A, B1, B2 = (rng.standard_normal((8, 8)) for _ in range(3))
    out = workloads.two_gemm({"A": A, "B1": B1, "B2": B2})
    assert np.array_equal(out["C2"], ref.gemm(ref.gemm(A, B1), B2))
    X, W1, W2 = rng.standard_normal((5, 4)), rng.standard_normal((4, 9)), rng.standard_normal((9, 4))
    y = workloads.mlp({"X": X, "W1": W1, "W2": W2})["Y"]
    assert ref.rel_frobenius(y, X @ W1 @ W2 + X) <= 1e-13
    # row sampling gives the same rows
    rows = [4, 0, 2]
    ys = workloads.mlp({"X": X, "W1": W1, "W2": W2}, rows=rows)["Y"]
    assert np.array_equal(ys, y[rows])
    dc = workloads.deep_chain({"C0": X, "B": [W1, W2, W1]})
    assert ref.rel_frobenius(dc["C"][3], X @ W1 @ W2 @ W1) <= 1e-13


def test_attention_batched_equals_loop_and_scale():
    rng = np.random.default_rng(4)
    Q, K, V = (rng.standard_normal((3, 10, 16)) for _ in range(3))
    out = workloads.attention({"Q": Q, "K": K, "V": V}, keep_s=True)
    for h in range(3):
        S = (Q[h] @ K[h].T) / 4.0               # 1/sqrt(16)
        assert ref.rel_frobenius(out["S"][h], S) <= 1e-13
        assert ref.rel_frobenius(out["O"][h], S @ V[h]) <= 1e-13


def test_grouped_query_map_equals_replication():
    rng = np.random.default_rng(6)
    t, hid, nq, nkv, ffn = 12, 16, 4, 2, 24
    dh = hid // nq
    inp = {"X": rng.standard_normal((t, hid)), "Wq": rng.standard_normal((hid, hid)),  # noqa
           "Wk": rng.standard_normal((hid, nkv * dh)), "Wv": rng.standard_normal((hid, nkv * dh)),
           "Wo": rng.standard_normal((hid, hid)), "Wg": rng.standard_normal((hid, ffn)),
           "Wu": rng.standard_normal((hid, ffn)), "Wd": rng.standard_normal((ffn, hid))}
    inp = {k: 0.3 * v for k, v in inp.items()}
    got = workloads.decoder_layer(inp, nq, nkv)
    # explicit head-wise replication of K and V (Alg. 2), then plain numpy
    X = inp["X"]
    Q, K, V = X @ inp["Wq"], X @ inp["Wk"], X @ inp["Wv"]
    Kr = np.repeat(K.reshape(t, nkv, dh), nq // nkv, axis=1)
    Vr = np.repeat(V.reshape(t, nkv, dh), nq // nkv, axis=1)
    O = np.empty((t, hid))
    for h in range(nq):
        S = Q[:, h * dh:(h + 1) * dh] @ Kr[:, h].T / np.sqrt(dh)
        O[:, h * dh:(h + 1) * dh] = S @ Vr[:, h]
    attn = O @ inp["Wo"]
    g, u = attn @ inp["Wg"], attn @ inp["Wu"]
    Y = (g / (1 + np.exp(-g)) * u) @ inp["Wd"]
    assert ref.rel_frobenius(got["O"], O) <= 1e-12
    assert ref.rel_frobenius(got["Y"], Y) <= 1e-12
    rows = [7, 1]
    sub = workloads.decoder_layer(inp, nq, nkv, rows=rows)
    assert np.allclose(sub["Y"], got["Y"][rows], rtol=0, atol=0)


def test_silu_mul_properties():
    x = np.array([0.0, 1.0, -1.0, 30.0, -30.0, 0.5])
    one = np.ones_like(x)
    s = ref.silu_mul(x, one)
    assert s[0] == 0.0
    assert abs(s[3] - 30.0) < 1e-11            # silu(x) -> x for large x
    assert abs(s[4]) < 1e-11
    # silu(x) - silu(-x) = x
    assert np.allclose(ref.silu_mul(x, one) - ref.silu_mul(-x, one), x, rtol=0, atol=1e-15 * 30)
    assert np.array_equal(ref.silu_mul(x, np.zeros_like(x)), np.zeros_like(x))
    # spot values from the definition x / (1 + e^-x)
    assert abs(s[1] - 1.0 / (1.0 + np.exp(-1.0))) < 1e-16
    assert abs(ref.silu_mul(np.array([2.0]), np.array([-3.0]))[0] + 3.0 * 2.0 / (1.0 + np.exp(-2.0))) < 1e-15
