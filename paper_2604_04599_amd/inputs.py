"""Seeded synthetic inputs and shape tables for the five chain workloads.

This module holds no arithmetic of the method: it only draws random matrices
with the shapes and value distributions the workloads name and counts GEMM
flops from shapes.  Both the GPU path and the CPU checker are fed from here so
that they see identical arrays.

Workloads (full sizes; every shape key can be overridden for small tests):
  two_gemm       A, B1, B2 [n x n] ~ U[-1,1]                               n=256
  mlp            X [m x d] ~ N(0,1); W1 [d x h] ~ N(0, std 1/sqrt(d));
                 W2 [h x d] ~ N(0, std 1/sqrt(h))                m=2048 d=1024 h=4096
  attention      Q, K, V [heads x t x dh] ~ N(0,1)              heads=32 t=2048 dh=64
  deep_chain     C0 [n x n] ~ U[-1,1]; B_i [n x n] ~ U[-1,1]/sqrt(n)   n=4096 depth=8
  decoder_layer  X [t x hidden] ~ N(0,1); weights ~ N(0, std 0.02); all values
                 rounded once to the nearest bf16-representable value (ties to
                 even)            t=4096 hidden=2048 n_q=32 n_kv=8 ffn=8192
Seeds are 1001..1005 in that order (numpy PCG64).

A sixth workload outside the benchmark set, `llama_layer` (seed 1006), is the decoder
layer with everything between its GEMMs present: the decoder_layer inputs plus the two
RMS-normalisation weight vectors norm1, norm2 [hidden] ~ N(1, std 0.1); the shape dict
also carries the integer RoPE base (500000) and 1/eps (100000).
"""
import numpy as np

WORKLOADS = ("two_gemm", "mlp", "attention", "deep_chain", "decoder_layer")

FULL_SHAPES = {
    "two_gemm": {"n": 256},
    "mlp": {"m": 2048, "d": 1024, "h": 4096},
    "attention": {"heads": 32, "t": 2048, "dh": 64},
    "deep_chain": {"n": 4096, "depth": 8},
    "decoder_layer": {"t": 4096, "hidden": 2048, "n_q": 32, "n_kv": 8, "ffn": 8192},
}

FULL_SHAPES["llama_layer"] = dict(FULL_SHAPES["decoder_layer"], rope_base=500000, inv_eps=100000)

SEEDS = {name: 1001 + i for i, name in enumerate(WORKLOADS)}
SEEDS["llama_layer"] = 1006

DTYPES = {"two_gemm": "f32", "mlp": "f32", "attention": "f32", "deep_chain": "f32",
          "decoder_layer": "bf16", "llama_layer": "bf16"}


def shape_of(name, **over):
    s = dict(FULL_SHAPES[name])
    for k, v in over.items():
        if k not in s:
            raise KeyError(f"{name} has no shape key {k!r}")
        s[k] = int(v)
    return s


def _rng(name, seed):
    return np.random.Generator(np.random.PCG64(SEEDS[name] if seed is None else seed))


def _uniform(rng, shape):
    return rng.uniform(-1.0, 1.0, size=shape).astype(np.float32)


def _normal(rng, shape, std=1.0):
    return (rng.standard_normal(size=shape, dtype=np.float32) * np.float32(std)).astype(np.float32)


def _bf16_representable(x):
    """Round each (finite) fp32 value to the nearest bf16-representable one, ties to even, on
    the bit pattern; the result is still float32 (its 16 low bits are zero)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32)


def make(name, seed=None, **over):
    """Return (inputs, shape): dict of float32 arrays and the shape dict used."""
    s = shape_of(name, **over)
    r = _rng(name, seed)
    if name == "two_gemm":
        n = s["n"]
        inp = {"A": _uniform(r, (n, n)), "B1": _uniform(r, (n, n)), "B2": _uniform(r, (n, n))}
    elif name == "mlp":
        m, d, h = s["m"], s["d"], s["h"]
        inp = {"X": _normal(r, (m, d)),
               "W1": _normal(r, (d, h), 1.0 / np.sqrt(d)),
               "W2": _normal(r, (h, d), 1.0 / np.sqrt(h))}
    elif name == "attention":
        hd, t, dh = s["heads"], s["t"], s["dh"]
        inp = {"Q": _normal(r, (hd, t, dh)), "K": _normal(r, (hd, t, dh)),
               "V": _normal(r, (hd, t, dh))}
    elif name == "deep_chain":
        n, depth = s["n"], s["depth"]
        inp = {"C0": _uniform(r, (n, n)),
               "B": [_uniform(r, (n, n)) / np.float32(np.sqrt(n)) for _ in range(depth)]}
    elif name in ("decoder_layer", "llama_layer"):
        t, hid, nq, nkv, ffn = s["t"], s["hidden"], s["n_q"], s["n_kv"], s["ffn"]
        if hid % nq or nq % nkv:
            raise ValueError("hidden must divide into n_q heads and n_q into n_kv groups")
        dh = hid // nq
        inp = {"X": _normal(r, (t, hid)),
               "Wq": _normal(r, (hid, hid), 0.02), "Wk": _normal(r, (hid, nkv * dh), 0.02),
               "Wv": _normal(r, (hid, nkv * dh), 0.02), "Wo": _normal(r, (hid, hid), 0.02),
               "Wg": _normal(r, (hid, ffn), 0.02), "Wu": _normal(r, (hid, ffn), 0.02),
               "Wd": _normal(r, (ffn, hid), 0.02)}
        inp = {k: _bf16_representable(v) for k, v in inp.items()}
        if name == "llama_layer":
            inp["norm1"] = (1.0 + _normal(r, (hid,), 0.1)).astype(np.float32)
            inp["norm2"] = (1.0 + _normal(r, (hid,), 0.1)).astype(np.float32)
    else:
        raise KeyError(name)
    return inp, s


def gemm_flops(name, s):
    """Sum of 2*m*n*k over the workload's GEMMs (scaling, residual adds and
    activations count as zero flops)."""
    if name == "two_gemm":
        return 2 * 2 * s["n"] ** 3
    if name == "mlp":
        return 2 * 2 * s["m"] * s["d"] * s["h"]
    if name == "attention":
        return s["heads"] * 2 * 2 * s["t"] * s["t"] * s["dh"]
    if name == "deep_chain":
        return s["depth"] * 2 * s["n"] ** 3
    if name in ("decoder_layer", "llama_layer"):
        t, hid, ffn = s["t"], s["hidden"], s["ffn"]
        dh = hid // s["n_q"]
        kvw = s["n_kv"] * dh
        return (2 * t * hid * (hid + 2 * kvw) + s["n_q"] * 4 * t * t * dh + 2 * t * hid * hid
                + 3 * 2 * t * hid * ffn)
    raise KeyError(name)
