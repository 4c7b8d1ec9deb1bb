"""GPU parity: a seeded random sweep of lpg_gemm_packed over shapes (biased towards the 32 / KB / tile
edges), dtypes, output roles and kinds, alpha / beta, fused epilogues, canonical inputs and output views
(none, on the grid, off the grid, ragged inside the parent).  Every case is compared with the oracle
(Eq. 1) and, when C is a view, the parent's bytes outside the view must not change."""
import numpy as np
import pytest

from oracle import ref
from paper_2604_04599_amd import api
from paper_2604_04599_amd.api import (LPG_BF16, LPG_COL_MAJOR, LPG_EPI_GATE_SILU, LPG_EPI_NONE, LPG_EPI_SILU, LPG_F32,
                                      LPG_PACKED_A, LPG_PACKED_B, LPG_ROW_MAJOR, desc)
from tests.gpu_util import ES, NP_RAW, bf16_raw_to_f64, dev_bytes, dev_empty, host, stream

pytestmark = pytest.mark.gpu

EDGES = [1, 2, 31, 32, 33, 63, 64, 65, 96, 127, 128, 129, 160, 255, 256, 257, 300]


def to_f64(raw, dtype):
    return raw.view(np.float32).astype(np.float64) if dtype == LPG_F32 else bf16_raw_to_f64(raw)


def to_raw(x64, dtype):
    f = np.ascontiguousarray(x64, dtype=np.float32)
    return f.view(np.uint32).copy() if dtype == LPG_F32 else ref.bf16_bits(f.view(np.uint32))


def draw_case(seed):
    rng = np.random.default_rng(50000 + seed)
    dim = lambda: int(rng.choice(EDGES)) if rng.random() < 0.7 else int(rng.integers(1, 400))
    c = {"in_dt": LPG_BF16 if rng.random() < 0.5 else LPG_F32, "m": dim(), "n": dim(), "k": dim()}
    c["out_dt"] = LPG_F32 if c["in_dt"] == LPG_F32 or rng.random() < 0.3 else LPG_BF16
    c["kind"] = int(rng.choice([LPG_PACKED_A, LPG_PACKED_B, LPG_PACKED_A, LPG_PACKED_B, LPG_ROW_MAJOR, LPG_COL_MAJOR]))
    c["alpha"] = float(rng.choice([1.0, 0.5, -1.25]))
    c["beta"] = float(rng.choice([0.0, 0.0, 1.0, -0.5]))
    c["epi"] = int(rng.choice([LPG_EPI_NONE, LPG_EPI_NONE, LPG_EPI_SILU, LPG_EPI_GATE_SILU]))
    c["view"] = str(rng.choice(["none", "none", "grid", "offgrid"])) if c["kind"] in (LPG_PACKED_A, LPG_PACKED_B) else "none"
    c["canon_a"] = bool(c["in_dt"] == LPG_F32 and c["k"] % 32 == 0 and rng.random() < 0.5)
    c["rng"] = rng
    return c


@pytest.mark.parametrize("streaming", [False, True])
@pytest.mark.parametrize("seed", range(96))
def test_random_gemm_case(seed, streaming, tune):
    c = draw_case(seed)
    if streaming:
        tune(api.LPG_TUNE_STREAM_STORES, 1)          # the epilogue's streaming-store form
    rng, in_dt, out_dt, kind = c["rng"], c["in_dt"], c["out_dt"], c["kind"]
    m, n, k, alpha, beta, epi = c["m"], c["n"], c["k"], c["alpha"], c["beta"], c["epi"]
    es_in, es = ES[in_dt], ES[out_dt]
    A = to_f64(to_raw(rng.standard_normal((m, k)), in_dt), in_dt)
    B = to_f64(to_raw(rng.standard_normal((k, n)) / np.sqrt(k), in_dt), in_dt)
    Bp = dev_bytes(ref.pack(to_raw(B, in_dt), False, es_in))
    bd = desc(LPG_PACKED_B, in_dt, k, n)
    if c["canon_a"]:
        ld = k + 4
        buf = np.full((m, ld), np.float32(9.0), dtype=np.float32)
        buf[:, :k] = A
        Ap, ad = dev_bytes(buf), desc(LPG_ROW_MAJOR, LPG_F32, m, k, ld=ld)
    else:
        Ap, ad = dev_bytes(ref.pack(to_raw(A, in_dt), True, es_in)), desc(LPG_PACKED_A, in_dt, m, k)
    packed = kind in (LPG_PACKED_A, LPG_PACKED_B)
    a_side = kind == LPG_PACKED_A
    kbo = ref.layout_consts(es)[2]
    # the parent C lives in, and the view's origin inside it
    if c["view"] == "none":
        prow, pcol, r0, c0 = m, n, 0, 0
    else:
        fg, kg = (32, kbo) if a_side else (kbo, 32)      # grid of (rows, cols)
        if c["view"] == "grid":
            r0, c0 = fg * int(rng.integers(0, 3)), kg * int(rng.integers(0, 3))
        else:
            r0, c0 = int(rng.integers(1, 70)), int(rng.integers(1, 70))
        prow, pcol = r0 + m + int(rng.integers(0, 40)), c0 + n + int(rng.integers(0, 40))
    before = to_raw(rng.standard_normal((prow, pcol)), out_dt)
    G = to_f64(to_raw(rng.uniform(-3, 3, (prow, pcol)), out_dt), out_dt)
    if packed:
        cbuf = dev_bytes(ref.pack(before, a_side, es))
        gbuf = dev_bytes(ref.pack(to_raw(G, out_dt), a_side, es))
        cd = desc(kind, out_dt, m, n, parent=(prow, pcol), origin=(r0, c0))
    else:
        rm = kind == LPG_ROW_MAJOR
        lay = (lambda x: np.ascontiguousarray(x)) if rm else (lambda x: np.ascontiguousarray(x.T))
        cbuf, gbuf = dev_bytes(lay(before)), dev_bytes(lay(to_raw(G, out_dt)))
        cd = desc(kind, out_dt, m, n)
    use_g = epi == LPG_EPI_GATE_SILU
    api.lpg_gemm_packed(alpha, Ap, ad, Bp, bd, beta, cbuf if beta != 0.0 else None, cbuf, cd, epi,
                        gbuf if use_g else None, stream())
    got_raw = host(cbuf, NP_RAW[out_dt])
    old = to_f64(before, out_dt)[r0:r0 + m, c0:c0 + n]
    want = ref.gemm(A, B, alpha=alpha, beta=beta, C=old if beta != 0.0 else None)
    if epi == LPG_EPI_SILU:
        want = ref.silu_mul(want, np.ones_like(want))
    elif use_g:
        want = ref.silu_mul(G[r0:r0 + m, c0:c0 + n], want)
    if packed:
        parent_now = ref.unpack(got_raw, prow, pcol, a_side, es)
        got_view = np.ascontiguousarray(parent_now[r0:r0 + m, c0:c0 + n])
        after = before.copy()
        after[r0:r0 + m, c0:c0 + n] = got_view
        full = ref.pack(after, a_side, es)       # neighbours and zero padding exactly as before
        assert np.array_equal(got_raw[:full.size], full), c
    else:
        arr = got_raw[:m * n].reshape((m, n) if kind == LPG_ROW_MAJOR else (n, m))
        got_view = np.ascontiguousarray(arr if kind == LPG_ROW_MAJOR else arr.T)
    tol = 1e-5 if (in_dt == LPG_F32 and out_dt == LPG_F32) else 1e-2
    err = ref.rel_frobenius(to_f64(got_view, out_dt), want)
    assert err <= tol, (err, {x: y for x, y in c.items() if x != "rng"})
