"""GPU parity: written views whose ORIGIN is off the 32 / KB grid of the packed layout (the general
form of the store-stride / block-order parameters of section III-C): destination of lpg_pack,
source of lpg_unpack, C / C_in of lpg_gemm_packed.

Same rule as for ragged inner views: writing the view equals updating that rectangle of the
parent's canonical matrix and packing the whole parent again, so the device buffer must equal the
oracle's pack of the updated parent bit for bit, neighbours and padding included.
"""
import numpy as np
import pytest

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


def to_f64(raw, dtype):
    return raw.view(np.float32).astype(np.float64) if dtype == LPG_F32 else bf16_raw_to_f64(raw)


def to_raw(x64, dtype):
    f = np.ascontiguousarray(x64, dtype=np.float32)
    return f.view(np.uint32).copy() if dtype == LPG_F32 else ref.bf16_bits(f.view(np.uint32))


def view_cases(dtype):
    """(PF, PK, f0, k0, F, K) in (free, contraction) terms."""
    KB = kb(dtype)
    return [
        (100, 3 * KB + 7, 5, KB, 37, KB),               # free origin off the grid
        (100, 3 * KB + 7, 32, 3, 36, KB + 5),           # contraction origin off the grid
        (130, 3 * KB + 7, 33, KB + 1, 70, KB + 9),      # both, several blocks
        (130, 2 * KB + 7, 110, KB + 2, 20, KB + 5),     # ends at the parent's edge in both dimensions
        (64, 2 * KB, 31, KB - 1, 2, 2),                 # straddles a block corner
        (64, 2 * KB, 17, 9, 1, 1),                      # a single element
    ]


@pytest.mark.parametrize("dtype", [LPG_F32, LPG_BF16])
@pytest.mark.parametrize("kind", [LPG_PACKED_A, LPG_PACKED_B])
@pytest.mark.parametrize("src_kind", [LPG_ROW_MAJOR, LPG_COL_MAJOR])
@pytest.mark.parametrize("case", range(6))
def test_pack_into_an_offgrid_view_equals_repacking_the_parent(dtype, kind, src_kind, case):
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
    if src_kind == LPG_ROW_MAJOR:
        canon = np.zeros((rows, cols + 3), dtype=piece.dtype)
        canon[:, :cols] = piece
        ld = cols + 3
    else:
        canon = np.zeros((cols, rows + 3), dtype=piece.dtype)
        canon[:, :rows] = piece.T
        ld = rows + 3
    sd = desc(src_kind, dtype, rows, cols, ld=ld)
    dd = desc(kind, dtype, rows, cols, parent=(prow, pcol), origin=(r0, c0))
    api.lpg_pack(dev_bytes(canon), sd, buf, dd, stream())
    got = host(buf, NP_RAW[dtype])
    want = ref.pack(after, a_side, es)
    assert np.array_equal(got[:want.size], want)
    # the library's own index function agrees with the oracle's closed form on such a view
    for (r, c) in ((0, 0), (rows - 1, cols - 1), (rows // 2, cols // 3)):
        f, k = (r0 + r, c0 + c) if a_side else (c0 + c, r0 + r)
        assert api.lpg_layout_offset(dd, 0, r, c) == int(ref.packed_offset(f, k, PF, es))
    # the view reads back alone, into a poisoned buffer whose leading-dimension padding stays
    back = dev_empty(canon.nbytes, fill=0x55)
    api.lpg_unpack(buf, dd, back, sd, stream())
    b = host(back, NP_RAW[dtype])[:canon.size].reshape(canon.shape)
    poison = NP_RAW[dtype](0x5555 if es == 2 else 0x55555555)
    inner = b[:, :cols] if src_kind == LPG_ROW_MAJOR else b[:, :rows].T
    assert np.array_equal(inner, piece)
    assert np.all(b[:, (cols if src_kind == LPG_ROW_MAJOR else rows):] == poison)


def test_pack_converting_to_bf16_into_an_offgrid_view():
    rng = np.random.default_rng(3)
    PF, PK, f0, k0, F, K = 100, 200, 7, 70, 50, 90
    before = to_raw(rng.standard_normal((PF, PK)), LPG_BF16)
    piece = rng.standard_normal((F, K)).astype(np.float32)
    buf = dev_bytes(ref.pack(before, True, 2))
    api.lpg_pack(dev_bytes(piece), desc(LPG_ROW_MAJOR, LPG_F32, F, K), buf,
                 desc(LPG_PACKED_A, LPG_BF16, F, K, parent=(PF, PK), origin=(f0, k0)), stream())
    after = before.copy()
    after[f0:f0 + F, k0:k0 + K] = ref.bf16_bits(piece.view(np.uint32))
    want = ref.pack(after, True, 2)
    assert np.array_equal(host(buf, np.uint16)[:want.size], want)


GEMM_CASES = [
    # m, n, k, parent rows, parent cols, row0, col0 of the output view
    (37, 64, 96, 100, 199, 5, 64),      # row origin off the grid
    (64, 41, 96, 128, 199, 64, 3),      # column origin off the grid
    (45, 50, 130, 130, 203, 33, 129),   # both
    (70, 70, 64, 200, 200, 130, 130),   # several tiles, ends at the parent's edge
    (1, 64, 64, 64, 64, 17, 0),         # one row (a token appended to a cache)
    (64, 1, 64, 64, 64, 0, 17),         # one column
]


@pytest.mark.parametrize("dtype", [LPG_F32, LPG_BF16])
@pytest.mark.parametrize("kind", [LPG_PACKED_A, LPG_PACKED_B])
@pytest.mark.parametrize("mode", ["plain", "beta", "silu"])
@pytest.mark.parametrize("case", range(len(GEMM_CASES)))
def test_gemm_into_an_offgrid_view_leaves_the_neighbours_alone(dtype, kind, mode, case):
    es = ES[dtype]
    m, n, k, prow, pcol, r0, c0 = GEMM_CASES[case]
    rng = np.random.default_rng(2000 + case)
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
    after = before.copy()
    got_view = ref.unpack(got, prow, pcol, a_side, es)[r0:r0 + m, c0:c0 + n]
    after[r0:r0 + m, c0:c0 + n] = got_view
    full = ref.pack(after, a_side, es)
    assert np.array_equal(got[:full.size], full)
    err = ref.rel_frobenius(to_f64(np.ascontiguousarray(got_view), dtype), want)
    assert err <= (1e-5 if dtype == LPG_F32 else 1e-2), err
    # the same product written to an aligned buffer of its own: same bits when nothing is fused
    own = dev_empty(api.lpg_packed_bytes(desc(kind, dtype, m, n)), fill=0)
    own_in = None
    if mode == "beta":
        own_in = dev_bytes(ref.pack(np.ascontiguousarray(before[r0:r0 + m, c0:c0 + n]), a_side, es))
    api.lpg_gemm_packed(alpha, Ap, desc(LPG_PACKED_A, dtype, m, k), Bp, desc(LPG_PACKED_B, dtype, k, n), beta,
                        own_in, own, desc(kind, dtype, m, n),
                        LPG_EPI_SILU if mode == "silu" else LPG_EPI_NONE, None, stream())
    own_view = ref.unpack(host(own, NP_RAW[dtype]), m, n, a_side, es)
    if mode == "plain":
        assert np.array_equal(own_view, got_view)
    else:    # the element-wise epilogue may contract alpha*acc + beta*c differently: last-bit differences
        assert ref.rel_frobenius(to_f64(own_view, dtype), to_f64(np.ascontiguousarray(got_view), dtype)) <= (
            1e-6 if dtype == LPG_F32 else 4e-3)


@pytest.mark.parametrize("dtype", [LPG_F32, LPG_BF16])
def test_tokens_appended_one_by_one_fill_the_caches_like_one_product(dtype):
    """Decoding: every step projects one new token, k_t = x_t Wk and v_t = x_t Wv, and appends it
    to the packed caches the attention GEMMs read: K as a left-operand image (a new ROW, free
    index t) and V as a right-operand image (a new ROW of V = a new CONTRACTION index t).  After
    T steps both caches hold what one product over all T tokens writes."""
    es = ES[dtype]
    T, cap, d, dh = 45, 96, 64, 64
    rng = np.random.default_rng(77)
    X = to_f64(to_raw(rng.standard_normal((T, d)), dtype), dtype)
    Wk = to_f64(to_raw(rng.standard_normal((d, dh)) / np.sqrt(d), dtype), dtype)
    Wv = to_f64(to_raw(rng.standard_normal((d, dh)) / np.sqrt(d), dtype), dtype)
    Wkp = dev_bytes(ref.pack(to_raw(Wk, dtype), False, es))
    Wvp = dev_bytes(ref.pack(to_raw(Wv, dtype), False, es))
    kd_full = desc(LPG_PACKED_A, dtype, cap, dh)
    vd_full = desc(LPG_PACKED_B, dtype, cap, dh)
    kc = dev_empty(api.lpg_packed_bytes(kd_full), fill=0)
    vc = dev_empty(api.lpg_packed_bytes(vd_full), fill=0)
    for t in range(T):
        xt = dev_bytes(ref.pack(to_raw(X[t:t + 1], dtype), True, es))
        xd = desc(LPG_PACKED_A, dtype, 1, d)
        wd = desc(LPG_PACKED_B, dtype, d, dh)
        api.lpg_gemm_packed(1.0, xt, xd, Wkp, wd, 0.0, None, kc,
                            desc(LPG_PACKED_A, dtype, 1, dh, parent=(cap, dh), origin=(t, 0)), LPG_EPI_NONE, None, stream())
        api.lpg_gemm_packed(1.0, xt, xd, Wvp, wd, 0.0, None, vc,
                            desc(LPG_PACKED_B, dtype, 1, dh, parent=(cap, dh), origin=(t, 0)), LPG_EPI_NONE, None, stream())
    # one product over all tokens, written to aligned caches of the same capacity
    Xp = dev_bytes(ref.pack(to_raw(X, dtype), True, es))
    k1 = dev_empty(api.lpg_packed_bytes(kd_full), fill=0)
    v1 = dev_empty(api.lpg_packed_bytes(vd_full), fill=0)
    api.lpg_gemm_packed(1.0, Xp, desc(LPG_PACKED_A, dtype, T, d), Wkp, desc(LPG_PACKED_B, dtype, d, dh), 0.0, None, k1,
                        desc(LPG_PACKED_A, dtype, T, dh, parent=(cap, dh)), LPG_EPI_NONE, None, stream())
    api.lpg_gemm_packed(1.0, Xp, desc(LPG_PACKED_A, dtype, T, d), Wvp, desc(LPG_PACKED_B, dtype, d, dh), 0.0, None, v1,
                        desc(LPG_PACKED_B, dtype, T, dh, parent=(cap, dh)), LPG_EPI_NONE, None, stream())
    assert np.array_equal(host(kc, NP_RAW[dtype]), host(k1, NP_RAW[dtype]))
    assert np.array_equal(host(vc, NP_RAW[dtype]), host(v1, NP_RAW[dtype]))
    # and both equal the oracle's products
    gk = to_f64(ref.unpack(host(kc, NP_RAW[dtype]), cap, dh, True, es)[:T], dtype)
    gv = to_f64(ref.unpack(host(vc, NP_RAW[dtype]), cap, dh, False, es)[:T], dtype)
    tol = 1e-5 if dtype == LPG_F32 else 1e-2
    assert ref.rel_frobenius(gk, ref.gemm(X, Wk)) <= tol
    assert ref.rel_frobenius(gv, ref.gemm(X, Wv)) <= tol


@pytest.mark.parametrize("dtype", [LPG_F32, LPG_BF16])
@pytest.mark.parametrize("mode", [api.LPG_CHAIN_PROPAGATED, api.LPG_CHAIN_CANONICAL])
def test_chain_appends_keys_at_any_row_and_scores_against_the_filled_part(dtype, mode):
    """Two stages: K_new = X_new Wk written as rows 70..90 of a 256-row packed key cache whose other
    unset rows hold NaN; then S = Q K[0:91]^T reading the filled part as a right operand."""
    es = ES[dtype]
    cap, d, dm, r0, cnt, tq = 256, 64, 128, 70, 21, 40
    rng = np.random.default_rng(12)
    rnd = lambda *s: to_f64(to_raw(rng.standard_normal(s), dtype), dtype)
    Xn, Wk, Q = rnd(cnt, dm), rnd(dm, d) / np.sqrt(dm), rnd(tq, d)
    cache = np.full((cap, d), np.nan)
    cache[:r0] = rnd(r0, d)
    buf = dev_bytes(ref.pack(to_raw(cache, dtype), True, es))
    T = r0 + cnt
    xd, wd, qd = desc(LPG_PACKED_A, dtype, cnt, dm), desc(LPG_PACKED_B, dtype, dm, d), desc(LPG_PACKED_A, dtype, tq, d)
    newd = desc(LPG_PACKED_A, dtype, cnt, d, parent=(cap, d), origin=(r0, 0))
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
