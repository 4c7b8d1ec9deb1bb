"""Pin of the oracle's whole-decoder-layer workload (Alg. 2 with its RoPE, causal mask and
softmax, between RMS-normalised residual blocks and the gated MLP) against a straight numpy
write-out of the layer that shares nothing with oracle/: matmul and einsum instead of the
oracle's GEMM, complex multiplication instead of its rotation, scipy's softmax over -inf
masked logits instead of its row softmax, explicit head-wise replication of K and V instead of
its index map.  A residual added to the wrong tensor, swapped norm weights, RoPE on V, a
missing scale or a mask off by one all fail here.
"""
import numpy as np
from scipy.special import softmax

from oracle import ref, workloads
from paper_2604_04599_amd import inputs


def _numpy_layer(inp, nq, nkv, eps, base):
    X = np.asarray(inp["X"], dtype=np.float64)
    W = {k: np.asarray(v, dtype=np.float64) for k, v in inp.items()}
    T, hid = X.shape
    dh = hid // nq
    rep = nq // nkv

    def rms(x, w):
        return x / np.sqrt((x * x).mean(axis=1, keepdims=True) + eps) * w[None, :]

    ang = np.outer(np.arange(T, dtype=np.float64), base ** (-2.0 * np.arange(dh // 2) / dh))

    def rot(M, heads):
        # a head's first half is the real part, its second half the imaginary part
        M = M.reshape(T, heads, 2, dh // 2)
        z = (M[:, :, 0, :] + 1j * M[:, :, 1, :]) * np.exp(1j * ang)[:, None, :]
        return np.stack([z.real, z.imag], axis=2).reshape(T, heads * dh)

    h1 = rms(X, W["norm1"])
    Q, K, V = rot(h1 @ W["Wq"], nq), rot(h1 @ W["Wk"], nkv), h1 @ W["Wv"]
    Kr = np.repeat(K.reshape(T, nkv, dh), rep, axis=1)        # head-wise replication (Alg. 2)
    Vr = np.repeat(V.reshape(T, nkv, dh), rep, axis=1)
    logits = np.einsum("thd,shd->hts", Q.reshape(T, nq, dh), Kr) / np.sqrt(dh)
    keep = np.tril(np.ones((T, T), dtype=bool))                # query t sees keys s <= t
    P = softmax(np.where(keep[None], logits, -np.inf), axis=-1)
    O = np.einsum("hts,shd->thd", P, Vr).reshape(T, hid)
    A = O @ W["Wo"] + X
    h2 = rms(A, W["norm2"])
    g, u = h2 @ W["Wg"], h2 @ W["Wu"]
    Y = (g / (1.0 + np.exp(-g)) * u) @ W["Wd"] + A
    return {"h1": h1, "Q": Q, "K": K, "V": V, "P": P, "O": O, "A": A, "h2": h2, "Y": Y}


def test_llama_layer_equals_a_plain_numpy_write_out():
    nq, nkv = 4, 2
    inp, shape = inputs.make("llama_layer", t=24, hidden=64, n_q=nq, n_kv=nkv, ffn=96)
    # weights of std 0.02 would leave the attention term tiny beside the residual: scale them up
    # so that every branch of the layer carries weight in Y
    inp = {k: (v * 6.0 if k.startswith("W") else v) for k, v in inp.items()}
    eps, base = 1.0 / shape["inv_eps"], float(shape["rope_base"])
    got = workloads.llama_layer(inp, nq, nkv, eps=eps, rope_base=base)
    want = _numpy_layer(inp, nq, nkv, eps, base)
    for name in ("h1", "Q", "K", "V", "O", "A", "h2", "Y"):
        assert ref.rel_frobenius(got[name], want[name]) <= 1e-12, name
    for h in range(nq):
        assert ref.rel_frobenius(got["P"][h], want["P"][h]) <= 1e-12, h
        assert np.all(np.triu(got["P"][h], 1) == 0.0)
    # the attention branch and both residuals matter at this scale: dropping any one of them
    # would move Y by far more than the tolerance
    assert ref.rel_frobenius(want["A"] - want["O"] @ np.asarray(inp["Wo"], dtype=np.float64), inp["X"]) <= 1e-12
    assert np.linalg.norm(want["O"] @ inp["Wo"]) > 0.05 * np.linalg.norm(want["A"])
    assert np.linalg.norm(want["Y"] - want["A"]) > 0.05 * np.linalg.norm(want["Y"])


def test_llama_layer_distinguishes_its_two_norm_weights_and_leaves_v_unrotated():
    nq, nkv = 4, 2
    inp, shape = inputs.make("llama_layer", t=16, hidden=64, n_q=nq, n_kv=nkv, ffn=64)
    inp = {k: (v * 6.0 if k.startswith("W") else v) for k, v in inp.items()}
    eps, base = 1.0 / shape["inv_eps"], float(shape["rope_base"])
    want = _numpy_layer(inp, nq, nkv, eps, base)
    swapped = dict(inp, norm1=inp["norm2"], norm2=inp["norm1"])
    got_swapped = workloads.llama_layer(swapped, nq, nkv, eps=eps, rope_base=base)
    assert ref.rel_frobenius(got_swapped["Y"], want["Y"]) > 1e-3       # the two weights are not interchangeable
    got = workloads.llama_layer(inp, nq, nkv, eps=eps, rope_base=base)
    h1 = want["h1"]
    assert ref.rel_frobenius(got["V"], h1 @ np.asarray(inp["Wv"], dtype=np.float64)) <= 1e-12   # V = h1 Wv, no rotation
    assert ref.rel_frobenius(got["K"], h1 @ np.asarray(inp["Wk"], dtype=np.float64)) > 1e-2     # K is rotated
