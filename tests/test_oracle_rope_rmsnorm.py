"""Pins for the oracle's rotary embedding and RMS normalisation (section IV-A / contributions)."""
import numpy as np

from oracle import ref


def test_rope_hand_example_and_angles():
    # head_dim 4, base 100: frequencies 1 and 100^(-1/2) = 0.1
    th = ref.rope_angles([0, 1, 7], 4, base=100.0)
    assert np.allclose(th, [[0, 0], [1, 0.1], [7, 0.7]], rtol=1e-15, atol=0)
    # angles (pi/2, pi): (1,3) -> (-3, 1), (2,4) -> (-2, -4); second head rotates the same way
    ang = np.array([[np.pi / 2, np.pi]])
    x = np.array([[1.0, 2.0, 3.0, 4.0, 10.0, 20.0, 30.0, 40.0]])
    got = ref.rope(x, np.cos(ang), np.sin(ang), 4)
    assert np.allclose(got, [[-3, -2, 1, -4, -30, -20, 10, -40]], atol=1e-14)


def test_rope_is_a_rotation_with_the_relative_position_property():
    rng = np.random.default_rng(0)
    dh, T = 16, 12
    q, k = rng.standard_normal((T, 2 * dh)), rng.standard_normal((T, 2 * dh))
    pos = np.arange(T) + 5
    th = ref.rope_angles(pos, dh)
    rq, rk = ref.rope(q, np.cos(th), np.sin(th), dh), ref.rope(k, np.cos(th), np.sin(th), dh)
    half = dh // 2
    for h0 in (0, dh):
        a, b = q[:, h0:h0 + half], q[:, h0 + half:h0 + dh]
        # complex form: (a + ib) e^{i theta}
        z = (a + 1j * b) * np.exp(1j * th)
        assert np.allclose(rq[:, h0:h0 + half], z.real, rtol=1e-13, atol=1e-14)
        assert np.allclose(rq[:, h0 + half:h0 + dh], z.imag, rtol=1e-13, atol=1e-14)
    assert np.allclose((rq ** 2).sum(axis=1), (q ** 2).sum(axis=1), rtol=1e-13)      # norms kept
    # position 0 is the identity
    z0 = ref.rope_angles([0], dh)
    assert np.array_equal(ref.rope(q[:1], np.cos(z0), np.sin(z0), dh), q[:1])
    # <rope(q, m), rope(k, n)> depends on m - n only (per head)
    def at(x, p):
        t = ref.rope_angles([p], dh)
        return ref.rope(x, np.cos(t), np.sin(t), dh)
    for m, n in ((9, 4), (3, 11)):
        lhs = at(q[:1, :dh], m) @ at(k[:1, :dh], n).T
        rhs = at(q[:1, :dh], m - n + 20) @ at(k[:1, :dh], 20).T
        assert np.allclose(lhs, rhs, rtol=1e-12)


def test_rmsnorm_closed_forms():
    # 3-4-5: mean square 12.5
    got = ref.rmsnorm(np.array([[3.0, 4.0]]), np.array([2.0, 0.5]), 0.0)
    assert np.allclose(got, [[6.0 / np.sqrt(12.5), 2.0 / np.sqrt(12.5)]], rtol=1e-15)
    rng = np.random.default_rng(1)
    x = rng.standard_normal((5, 33))
    w = rng.standard_normal(33)
    y1 = ref.rmsnorm(x, np.ones(33), 0.0)
    assert np.allclose((y1 ** 2).mean(axis=1), 1.0, rtol=1e-13)                       # unit mean square
    assert np.allclose(ref.rmsnorm(7.5 * x, w, 0.0), ref.rmsnorm(x, w, 0.0), rtol=1e-13)  # scale invariant
    assert np.allclose(ref.rmsnorm(x, w, 0.0), y1 * w, rtol=1e-15)
    # eps enters under the root, added to the mean square: constant row c -> c / sqrt(c^2 + eps)
    c = ref.rmsnorm(np.full((1, 8), 2.0), np.ones(8), 5.0)
    assert np.allclose(c, 2.0 / 3.0, rtol=1e-15)
    assert np.array_equal(ref.rmsnorm(np.zeros((1, 4)), np.ones(4), 1e-6), np.zeros((1, 4)))


def test_llama_layer_row_sampling_equals_the_full_computation():
    from oracle import workloads
    from paper_2604_04599_amd import inputs
    inp, shape = inputs.make("llama_layer", t=24, hidden=64, n_q=4, n_kv=2, ffn=96)
    full = workloads.llama_layer(inp, 4, 2)
    rows = np.array([0, 5, 23])
    part = workloads.llama_layer(inp, 4, 2, rows=rows)
    for n in ("Q", "O", "A", "h2", "act", "Y"):
        assert np.allclose(part[n], full[n][rows], rtol=1e-12, atol=1e-14), n
    assert np.array_equal(part["K"], full["K"])
    # the layer is causal: changing a later token leaves earlier outputs alone
    inp2 = dict(inp)
    inp2["X"] = inp["X"].copy()
    inp2["X"][10:] += 1.0
    assert np.allclose(workloads.llama_layer(inp2, 4, 2)["Y"][:10], full["Y"][:10], rtol=1e-12, atol=1e-14)
