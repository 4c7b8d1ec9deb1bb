"""GPU parity: views whose ragged extent ends INSIDE a packed parent (a block of the parent is
shared between the view and its neighbours).

The rule the tests hold the library to: writing such a view is the same as updating that
rectangle of the parent's canonical matrix and packing the whole parent again, so the device
buffer after the call must equal the oracle's pack of the updated parent, bit for bit, in every
byte outside the rectangle as well (neighbouring elements and the parent's zero padding).
"""
import numpy as np
import pytest
import torch

from oracle import ref
from paper_2604_04599_amd import api
from paper_2604_04599_amd.api import (LPG_BF16, LPG_COL_MAJOR, LPG_EPI_NONE, LPG_EPI_SILU, LPG_F32, LPG_PACKED_A,
                                      LPG_PACKED_B, LPG_ROW_MAJOR, desc)
from tests.gpu_util import ES, NP_RAW, bf16_raw_to_f64, dev_bytes, dev_empty, host, stream

pytestmark = pytest.mark.gpu


def iota(rows, cols, dtype, salt=0):
    n = rows * cols
    return ((np.arange(n, dtype=np.int64) * 2654435761 + 12345 + salt) % (1 << (8 * ES[dtype]))).astype(
        NP_RAW[dtype]).reshape(rows, cols)


def kb(dtype):
    return ref.layout_consts(ES[dtype])[2]


def view_cases(dtype):
    """(parent rows, parent cols, row0, col0, rows, cols) in (free, contraction) terms are built by
    the caller; here: (PF, PK, f0, k0, F, K) with at least one ragged extent ending inside."""
    KB = kb(dtype)
    return [
        (100, 3 * KB + 7, 32, KB, 37, KB),            # free ragged inside, K whole blocks
        (100, 3 * KB + 7, 64, 0, 36, KB + 5),         # free at the parent's edge, K ragged inside
        (130, 3 * KB + 7, 32, KB, 41, KB + 9),        # both ragged inside
        (130, 2 * KB + 7, 96, KB, 20, KB + 7),        # free inside, K at the parent's edge
        (64, 2 * KB, 0, 0, 1, 1),                     # a single element
    ]


@pytest.mark.parametrize("dtype", [LPG_F32, LPG_BF16])
@pytest.mark.parametrize("kind", [LPG_PACKED_A, LPG_PACKED_B])
@pytest.mark.parametrize("src_kind", [LPG_ROW_MAJOR, LPG_COL_MAJOR])
@pytest.mark.parametrize("case", range(5))
def test_pack_into_an_inner_view_equals_repacking_the_parent(dtype, kind, src_kind, case):
    es = ES[dtype]
    PF, PK, f0, k0, F, K = view_cases(dtype)[case]
    a_side = kind == LPG_PACKED_A
    prow, pcol = (PF, PK) if a_side else (PK, PF)
    r0, c0 = (f0, k0) if a_side else (k0, f0)
    rows, cols = (F, K) if a_side else (K, F)
    before = iota(prow, pcol, dtype)
    piece = iota(rows, cols, dtype, salt=977)
    after = before.copy()
    after[r0:r0 + rows, c0:c0 + cols] = piece
    buf = dev_bytes(ref.pack(before, a_side, es))
    for odd in (0, 1):   # odd = 1 shifts the source off 16-byte alignment (scalar load path)
        if src_kind == LPG_ROW_MAJOR:
            canon = np.zeros(rows * (cols + 4) + 4, dtype=piece.dtype)
            canon[odd:odd + rows * (cols + 4)].reshape(rows, cols + 4)[:, :cols] = piece
            ld = cols + 4
        else:
            canon = np.zeros(cols * (rows + 4) + 4, dtype=piece.dtype)
            canon[odd:odd + cols * (rows + 4)].reshape(cols, rows + 4)[:, :rows] = piece.T
            ld = rows + 4
        src = dev_bytes(canon)[odd * es:]
        sd = desc(src_kind, dtype, rows, cols, ld=ld)
        dd = desc(kind, dtype, rows, cols, parent=(prow, pcol), origin=(r0, c0))
        api.lpg_pack(src, sd, buf, dd, stream())
        got = host(buf, NP_RAW[dtype])
        want = ref.pack(after, a_side, es)
        assert np.array_equal(got[:want.size], want)
        # and the view reads back alone
        back = dev_empty(rows * cols * es, fill=0x55)
        api.lpg_unpack(buf, dd, back, desc(LPG_ROW_MAJOR, dtype, rows, cols), stream())
        assert np.array_equal(host(back, NP_RAW[dtype], (rows, cols)), piece)


def to_f64(raw, dtype):
    return raw.view(np.float32).astype(np.float64) if dtype == LPG_F32 else bf16_raw_to_f64(raw)


def to_raw(x64, dtype):
    f = np.ascontiguousarray(x64, dtype=np.float32)
    return f.view(np.uint32).copy() if dtype == LPG_F32 else ref.bf16_bits(f.view(np.uint32))


GEMM_CASES = [
    # m, n, k, parent rows, parent cols, row0, col0 of the output view
    (37, 64, 96, 100, 199, 32, 64),     # rows ragged inside
    (64, 41, 96, 128, 199, 64, 64),     # cols ragged inside
    (45, 50, 130, 130, 203, 32, 128),   # both
    (70, 70, 64, 200, 200, 128, 64),    # several tiles, both ragged inside
]


@pytest.mark.parametrize("dtype", [LPG_F32, LPG_BF16])
@pytest.mark.parametrize("kind", [LPG_PACKED_A, LPG_PACKED_B])
@pytest.mark.parametrize("mode", ["plain", "beta", "silu"])
@pytest.mark.parametrize("case", range(len(GEMM_CASES)))
def test_gemm_into_an_inner_view_leaves_the_neighbours_alone(dtype, kind, mode, case):
    es = ES[dtype]
    m, n, k, prow, pcol, r0, c0 = GEMM_CASES[case]
    if kind == LPG_PACKED_B:     # origins are (contraction, free) multiples of (KB, 32) there
        r0, c0 = (r0 // kb(dtype)) * kb(dtype), (c0 // 32) * 32
    else:
        c0 = (c0 // kb(dtype)) * kb(dtype)
    rng = np.random.default_rng(1000 + case)
    A = to_f64(to_raw(rng.standard_normal((m, k)), dtype), dtype)
    B = to_f64(to_raw(rng.standard_normal((k, n)) / np.sqrt(k), dtype), dtype)
    before = to_raw(rng.standard_normal((prow, pcol)), dtype)
    a_side = kind == LPG_PACKED_A
    buf = dev_bytes(ref.pack(before, a_side, es))
    Ap = dev_bytes(ref.pack(to_raw(A, dtype), True, es))
    Bp = dev_bytes(ref.pack(to_raw(B, dtype), False, es))
    cd = desc(kind, dtype, m, n, parent=(prow, pcol), origin=(r0, c0))
    alpha, beta = (0.75, -0.5) if mode == "beta" else (1.0, 0.0)
    api.lpg_gemm_packed(alpha, Ap, desc(LPG_PACKED_A, dtype, m, k), Bp, desc(LPG_PACKED_B, dtype, k, n), beta,
                        buf if mode == "beta" else None, buf, cd,
                        LPG_EPI_SILU if mode == "silu" else LPG_EPI_NONE, None, stream())
    got = host(buf, NP_RAW[dtype])
    old = to_f64(before, dtype)[r0:r0 + m, c0:c0 + n]
    want = ref.gemm(A, B, alpha=alpha, beta=beta, C=old if mode == "beta" else None)
    if mode == "silu":
        want = ref.silu_mul(want, np.ones_like(want))
    # outside the view: the parent is bit for bit what it was (pack the parent with the view's
    # rectangle overwritten by what the device produced and compare whole buffers)
    after = before.copy()
    got_view = ref.unpack(got, prow, pcol, a_side, es)[r0:r0 + m, c0:c0 + n]
    after[r0:r0 + m, c0:c0 + n] = got_view
    full = ref.pack(after, a_side, es)
    assert np.array_equal(got[:full.size], full)
    # inside: the product, to the dtype's bar
    err = ref.rel_frobenius(to_f64(np.ascontiguousarray(got_view), dtype), want)
    assert err <= (1e-5 if dtype == LPG_F32 else 1e-2), err


@pytest.mark.parametrize("dtype", [LPG_F32, LPG_BF16])
def test_gemm_reads_an_inner_ragged_operand_without_touching_its_neighbours(dtype):
    """A = 37 rows out of the middle of a packed parent whose other rows hold NaN; B likewise a
    column range.  The rows and columns past the views only reach output elements that are
    never stored, so the result is finite and equals the oracle's."""
    es = ES[dtype]
    m, n, k = 37, 45, 2 * kb(dtype)
    rng = np.random.default_rng(5)
    A = to_f64(to_raw(rng.standard_normal((m, k)), dtype), dtype)
    B = to_f64(to_raw(rng.standard_normal((k, n)) / np.sqrt(k), dtype), dtype)
    nan = np.float32(np.nan)
    pa = np.full((128, k), nan, dtype=np.float32)
    pa[32:32 + m] = A
    pb = np.full((k, 160), nan, dtype=np.float32)
    pb[:, 64:64 + n] = B
    Ap = dev_bytes(ref.pack(to_raw(pa, dtype), True, es))
    Bp = dev_bytes(ref.pack(to_raw(pb, dtype), False, es))
    ad = desc(LPG_PACKED_A, dtype, m, k, parent=(128, k), origin=(32, 0))
    bd = desc(LPG_PACKED_B, dtype, k, n, parent=(k, 160), origin=(0, 64))
    for kind in (LPG_PACKED_A, LPG_PACKED_B, LPG_ROW_MAJOR):
        cd = desc(kind, dtype, m, n)
        nbytes = api.lpg_packed_bytes(cd) if kind != LPG_ROW_MAJOR else m * n * es
        out = dev_empty(nbytes, fill=0)
        api.lpg_gemm_packed(1.0, Ap, ad, Bp, bd, 0.0, None, out, cd, LPG_EPI_NONE, None, stream())
        raw = host(out, NP_RAW[dtype])
        if kind == LPG_ROW_MAJOR:
            got = raw[:m * n].reshape(m, n)
        else:
            want_pad = ref.pack(ref.unpack(raw, m, n, kind == LPG_PACKED_A, es), kind == LPG_PACKED_A, es)
            assert np.array_equal(raw[:want_pad.size], want_pad)      # padding is zeros, not NaN
            got = ref.unpack(raw, m, n, kind == LPG_PACKED_A, es)
        g = to_f64(np.ascontiguousarray(got), dtype)
        assert np.all(np.isfinite(g))
        assert ref.rel_frobenius(g, ref.gemm(A, B)) <= (1e-5 if dtype == LPG_F32 else 1e-2)


def test_appending_row_blocks_to_a_packed_cache_matches_packing_it_whole():
    """A growing left operand (a key cache: rows = tokens) filled by packs of 5, 37 and 22 rows
    at row offsets that are multiples of 32 only for the first of each group of 32."""
    dtype, es = LPG_BF16, 2
    cap, d = 128, 128
    full = iota(cap, d, dtype, salt=3)
    buf = dev_empty(api.lpg_packed_bytes(desc(LPG_PACKED_A, dtype, cap, d)), fill=0)
    have = np.zeros((cap, d), dtype=np.uint16)
    # appends must start on a 32-row boundary; each writes a ragged count of rows
    for r0, cnt in ((0, 5), (32, 37), (96, 22)):
        piece = full[r0:r0 + cnt]
        api.lpg_pack(dev_bytes(piece), desc(LPG_ROW_MAJOR, dtype, cnt, d), buf,
                     desc(LPG_PACKED_A, dtype, cnt, d, parent=(cap, d), origin=(r0, 0)), stream())
        have[r0:r0 + cnt] = piece
        want = ref.pack(have, True, es)
        assert np.array_equal(host(buf, np.uint16)[:want.size], want)


@pytest.mark.parametrize("dtype", [LPG_F32, LPG_BF16])
@pytest.mark.parametrize("mode", [api.LPG_CHAIN_PROPAGATED, api.LPG_CHAIN_CANONICAL])
def test_chain_appends_keys_to_a_cache_and_scores_against_the_filled_part(dtype, mode):
    """Two stages: K_new = X_new Wk written as 37 new rows of a 256-row packed key cache (rows
    64..100, the last block shared with rows that are still unset and hold NaN); then
    S = Q K[0:101]^T, which reads the filled part of the cache as a right operand whose free
    extent ends inside the parent."""
    es = ES[dtype]
    cap, d, dm, r0, cnt, tq = 256, 64, 128, 64, 37, 40
    rng = np.random.default_rng(11)
    rnd = lambda *s: to_f64(to_raw(rng.standard_normal(s), dtype), dtype)
    Xn, Wk, Q = rnd(cnt, dm), rnd(dm, d) / np.sqrt(dm), rnd(tq, d)
    cache = np.full((cap, d), np.nan)
    cache[:r0] = rnd(r0, d)
    buf = dev_bytes(ref.pack(to_raw(cache, dtype), True, es))
    T = r0 + cnt
    xd, wd, qd = desc(LPG_PACKED_A, dtype, cnt, dm), desc(LPG_PACKED_B, dtype, dm, d), desc(LPG_PACKED_A, dtype, tq, d)
    newd = desc(LPG_PACKED_A, dtype, cnt, d, parent=(cap, d), origin=(r0, 0))
    # the same bytes read as K^T: a right operand with free = tokens
    ktd = desc(LPG_PACKED_B, dtype, d, T, parent=(d, cap))
    sd = desc(LPG_PACKED_A, dtype, tq, T)
    S = dev_empty(api.lpg_packed_bytes(sd), fill=0)
    Xp, Wp, Qp = (dev_bytes(ref.pack(to_raw(a, dtype), side, es)) for a, side in ((Xn, True), (Wk, False), (Q, True)))
    stages = [api.stage_gemm(1.0, Xp, xd, Wp, wd, 0.0, None, buf, newd),
              api.stage_gemm(0.125, Qp, qd, buf, ktd, 0.0, None, S, sd)]
    nws = api.lpg_chain_workspace_bytes(stages, mode)
    ws = dev_empty(nws) if nws else None
    api.lpg_chain(stages, mode, ws, nws, stream())
    got_cache = to_f64(ref.unpack(host(buf, NP_RAW[dtype]), cap, d, True, es), dtype)
    assert np.array_equal(got_cache[:r0], cache[:r0]) and np.all(np.isnan(got_cache[T:]))
    tol = 1e-5 if dtype == LPG_F32 else 1e-2
    assert ref.rel_frobenius(got_cache[r0:T], ref.gemm(Xn, Wk)) <= tol
    got_s = to_f64(ref.unpack(host(S, NP_RAW[dtype]), tq, T, True, es), dtype)
    assert np.all(np.isfinite(got_s))
    assert ref.rel_frobenius(got_s, ref.gemm(Q, got_cache[:T].T, alpha=0.125)) <= tol
