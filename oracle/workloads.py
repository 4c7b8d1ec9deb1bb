"""The benchmark workloads computed by the CPU oracle.  TEST INFRASTRUCTURE ONLY.

Each function takes the seeded input arrays (numpy, any float dtype; values are
used exactly) and evaluates the workload's GEMM chain on canonical row-major
fp64 arrays with oracle.ref.gemm (Eq. 1) stage by stage (Eq. 2).  The oracle
never computes in a packed layout: propagation changes where bytes live, not
their values.

`store` selects how an intermediate is rounded before the next stage reads it:
None keeps fp64 (the mathematical reference that acceptance uses), "f32" and
"bf16" mirror what a device stores and exist to explain error.

`rows` (index array) evaluates only those rows of every row-separable stage:
row r of each stage depends on row r of the chain input and on the full
weights (and, for attention, the full K and V, which are always computed whole).
"""
import numpy as np

from . import ref


def _st(x, store):
    if store is None:
        return x
    if store == "f32":
        return ref.round_f32(x)
    if store == "bf16":
        return ref.round_bf16(x)
    raise ValueError(store)


def _rows(x, rows):
    x = np.asarray(x, dtype=np.float64)
    return x if rows is None else x[np.asarray(rows)]


def two_gemm(inp, store=None, rows=None):
    """C1 = A*B1, C2 = C1*B2 (alpha 1, beta 0)."""
    c1 = _st(ref.gemm(_rows(inp["A"], rows), inp["B1"]), store)
    c2 = ref.gemm(c1, inp["B2"])
    return {"C1": c1, "C2": c2}


def mlp(inp, store=None, rows=None):
    """H = X*W1, Y = H*W2 + 1*X (the second GEMM has beta = 1 with C = X)."""
    x = _rows(inp["X"], rows)
    h = _st(ref.gemm(x, inp["W1"]), store)
    y = ref.gemm(h, inp["W2"], alpha=1.0, beta=1.0, C=x)
    return {"H": h, "Y": y}


def attention(inp, store=None, rows=None, heads=None, keep_s=False, softmax=False, causal=False):
    """Per head: S = (1/sqrt(d)) * Q_h * K_h^T, O = S * V_h.  With softmax=True the scale moves
    into the softmax, S = softmax((1/sqrt(d)) * Q_h K_h^T [causally masked]) (Alg. 2), and
    `rows` must then be None (a causal mask is positional).  Inputs Q, K, V: [heads, T, d]."""
    q, k, v = (np.asarray(inp[n], dtype=np.float64) for n in ("Q", "K", "V"))
    nh, _, d = q.shape
    alpha = 1.0 / np.sqrt(d)
    hs = range(nh) if heads is None else heads
    out = {"O": {}, "S": {}}
    for h in hs:
        if softmax:
            raw = _st(ref.gemm(q[h], k[h].T), store)
            s = _st(ref.softmax_rows(raw, scale=alpha, causal=causal), store)
        else:
            s = _st(ref.gemm(_rows(q[h], rows), k[h].T, alpha=alpha), store)
        out["O"][h] = ref.gemm(s, v[h])
        if keep_s:
            out["S"][h] = s
    return out


def deep_chain(inp, store=None, rows=None, depth=None):
    """C_{i+1} = C_i * B_i for i = 0..depth-1; returns every C_i (C[0] is the input)."""
    c = _rows(inp["C0"], rows)
    cs = [c]
    bs = inp["B"] if depth is None else inp["B"][:depth]
    for i, b in enumerate(bs):
        c = ref.gemm(c, b)
        if i + 1 < len(bs):
            c = _st(c, store)
        cs.append(c)
    return {"C": cs}


def decoder_layer(inp, n_q, n_kv, store=None, rows=None):
    """GEMM-only decoder-layer chain with grouped-query attention:
    Q,K,V projections; per q-head S = (1/sqrt(d)) Q_h K_g^T, O_h = S V_g with
    g = h // (n_q/n_kv) (a key/value head serves n_q/n_kv query heads, which
    equals replicating K and V head-wise as Alg. 2 does); output projection;
    gate and up projections; SiLU(gate)*up; down projection."""
    x = np.asarray(inp["X"], dtype=np.float64)
    xr = _rows(x, rows)
    d = inp["Wq"].shape[1] // n_q
    rep = n_q // n_kv
    alpha = 1.0 / np.sqrt(d)
    q = _st(ref.gemm(xr, inp["Wq"]), store)
    k = _st(ref.gemm(x, inp["Wk"]), store)
    v = _st(ref.gemm(x, inp["Wv"]), store)
    o = np.empty((xr.shape[0], n_q * d), dtype=np.float64)
    for h in range(n_q):
        g = h // rep
        kg = np.ascontiguousarray(k[:, g * d:(g + 1) * d].T)
        s = _st(ref.gemm(np.ascontiguousarray(q[:, h * d:(h + 1) * d]), kg, alpha=alpha), store)
        o[:, h * d:(h + 1) * d] = ref.gemm(s, np.ascontiguousarray(v[:, g * d:(g + 1) * d]))
    o = _st(o, store)
    attn = _st(ref.gemm(o, inp["Wo"]), store)
    gate = _st(ref.gemm(attn, inp["Wg"]), store)
    up = _st(ref.gemm(attn, inp["Wu"]), store)
    act = _st(ref.silu_mul(gate, up), store)
    y = ref.gemm(act, inp["Wd"])
    return {"Q": q, "K": k, "V": v, "O": o, "attn": attn, "gate": gate, "up": up,
            "act": act, "Y": y}



def llama_layer(inp, n_q, n_kv, eps=1e-5, rope_base=500000.0, store=None, rows=None):
    """A whole pre-norm decoder layer on the chain (Alg. 2 with its RoPE, causal mask and softmax,
    between RMSNorm-ed residual blocks, followed by the gated MLP):
        h1 = RMSNorm(X) ; Q, K, V = h1 Wq, h1 Wk, h1 Wv ; RoPE on Q and K (positions 0..T-1) ;
        per query head: P = softmax(causal((1/sqrt(d)) Q_h K_g^T)), O_h = P V_g ;
        A = O Wo + X ; h2 = RMSNorm(A) ; Y = (SiLU(h2 Wg) * (h2 Wu)) Wd + A.
    rows: compute only these token rows of everything downstream of K and V (which are always
    whole); a sampled row keeps its position for RoPE and for the causal mask."""
    x = np.asarray(inp["X"], dtype=np.float64)
    T = x.shape[0]
    pos = np.arange(T) if rows is None else np.asarray(rows)
    d = inp["Wq"].shape[1] // n_q
    rep = n_q // n_kv
    h1 = _st(ref.rmsnorm(x, inp["norm1"], eps), store)
    q = _st(ref.gemm(h1[pos], inp["Wq"]), store)
    k = _st(ref.gemm(h1, inp["Wk"]), store)
    v = _st(ref.gemm(h1, inp["Wv"]), store)
    th = ref.rope_angles(np.arange(T), d, rope_base)
    q = _st(ref.rope(q, np.cos(th[pos]), np.sin(th[pos]), d), store)
    k = _st(ref.rope(k, np.cos(th), np.sin(th), d), store)
    o = np.empty((len(pos), n_q * d), dtype=np.float64)
    P = {}
    for h in range(n_q):
        g = h // rep
        kg = np.ascontiguousarray(k[:, g * d:(g + 1) * d].T)
        s = _st(ref.gemm(np.ascontiguousarray(q[:, h * d:(h + 1) * d]), kg), store)
        if rows is None:
            p = ref.softmax_rows(s, scale=1.0 / np.sqrt(d), causal=True)
        else:
            p = np.zeros_like(s)
            for i, r in enumerate(pos):                  # row at position r sees keys 0..r
                p[i, :r + 1] = ref.softmax_rows(s[i:i + 1, :r + 1], scale=1.0 / np.sqrt(d))
        p = _st(p, store)
        P[h] = p
        o[:, h * d:(h + 1) * d] = ref.gemm(p, np.ascontiguousarray(v[:, g * d:(g + 1) * d]))
    o = _st(o, store)
    a = _st(ref.gemm(o, inp["Wo"], beta=1.0, C=x[pos]), store)
    h2 = _st(ref.rmsnorm(a, inp["norm2"], eps), store)
    gate = _st(ref.gemm(h2, inp["Wg"]), store)
    up = _st(ref.gemm(h2, inp["Wu"]), store)
    act = _st(ref.silu_mul(gate, up), store)
    y = ref.gemm(act, inp["Wd"], beta=1.0, C=a)
    return {"h1": h1, "Q": q, "K": k, "V": v, "P": P, "O": o, "A": a, "h2": h2, "act": act, "Y": y}
