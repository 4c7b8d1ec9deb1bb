"""GPU parity: lpg_gemm_packed and lpg_elementwise_packed against the oracle (Eq. 1)."""
import numpy as np
import pytest
import torch

from oracle import ref
from paper_2604_04599_amd import api
from paper_2604_04599_amd.api import (LPG_BF16, LPG_EPI_GATE_SILU, LPG_EPI_SILU, LPG_EW_ADD, LPG_EW_SCALE,
                                      LPG_EW_SILU_MUL, LPG_F32, LPG_PACKED_A, LPG_PACKED_B, LPG_ROW_MAJOR,
                                      desc)
from tests.gpu_util import ES, NP_RAW, dev_bytes, dev_empty, host, pack_dev, stream, unpack_dev

pytestmark = pytest.mark.gpu

F32_TOL = 1e-5      # relative Frobenius error per GEMM, fp32
BF16_TOL = 2e-2     # bf16 inputs


def bf16_exact(x):
    return (np.ascontiguousarray(x, dtype=np.float32).view(np.uint32) & np.uint32(0xFFFF0000)).view(np.float32)


def run_gemm(A, B, in_dt, out_dt, c_kind, alpha=1.0, beta=0.0, C=None, epi=0, E=None, poison_c=False):
    m, k = A.shape
    n = B.shape[1]
    ta, ad = pack_dev(A, LPG_PACKED_A, in_dt)
    tb, bd = pack_dev(B, LPG_PACKED_B, in_dt)
    cd = desc(c_kind, out_dt, m, n)
    tc = dev_empty(api.lpg_packed_bytes(cd), fill=0xFF)          # NaN patterns
    tcin = None
    if C is not None:
        tcin, _ = pack_dev(C, c_kind, out_dt)
    elif poison_c:
        tcin = dev_empty(api.lpg_packed_bytes(cd), fill=0xFF)
    te = pack_dev(E, c_kind, out_dt)[0] if E is not None else None
    api.lpg_gemm_packed(alpha, ta, ad, tb, bd, beta, tcin, tc, cd, epi, te, stream())
    raw = host(tc, NP_RAW[out_dt])[:api.lpg_packed_bytes(cd) // ES[out_dt]].copy()
    return unpack_dev(tc, cd), raw, cd


SHAPES = [(32, 32, 32), (64, 64, 64), (128, 128, 128), (256, 256, 256), (1, 1, 1), (33, 17, 65),
          (129, 257, 70), (160, 96, 200), (300, 40, 130), (40, 300, 33)]


@pytest.mark.parametrize("c_kind", [LPG_PACKED_A, LPG_PACKED_B])
@pytest.mark.parametrize("m,n,k", SHAPES)
def test_fp32_gemm_matches_oracle(c_kind, m, n, k):
    rng = np.random.default_rng(m * 7 + n * 3 + k)
    A = rng.uniform(-1, 1, (m, k)).astype(np.float32)
    B = rng.uniform(-1, 1, (k, n)).astype(np.float32)
    C = rng.uniform(-1, 1, (m, n)).astype(np.float32)
    got, raw, cd = run_gemm(A, B, LPG_F32, LPG_F32, c_kind, alpha=0.75, beta=-1.5, C=C)
    want = ref.gemm(A, B, alpha=0.75, beta=-1.5, C=C)
    assert ref.rel_frobenius(got, want) <= F32_TOL
    # the packed result, padding included, equals the packed oracle result where defined,
    # and padding is exactly zero
    wpk = ref.pack(got.astype(np.float32), c_kind == LPG_PACKED_A, 4)
    assert np.array_equal(raw, wpk)


@pytest.mark.parametrize("c_kind", [LPG_PACKED_A, LPG_PACKED_B])
def test_fp32_integer_inputs_are_bit_exact(c_kind):
    rng = np.random.default_rng(5)
    m, n, k = 150, 170, 260
    A = rng.integers(-2, 3, (m, k)).astype(np.float32)
    B = rng.integers(-2, 3, (k, n)).astype(np.float32)
    C = rng.integers(-4, 5, (m, n)).astype(np.float32)
    got, _, _ = run_gemm(A, B, LPG_F32, LPG_F32, c_kind, alpha=2.0, beta=-1.0, C=C)
    assert np.array_equal(got, ref.gemm(A, B, alpha=2.0, beta=-1.0, C=C))
    # identity and permutation
    P = np.eye(k, dtype=np.float32)[rng.permutation(k)][:, :n] if n <= k else None
    I = np.eye(k, dtype=np.float32)
    got, _, _ = run_gemm(A, I, LPG_F32, LPG_F32, c_kind)
    assert np.array_equal(got, A.astype(np.float64))
    if P is not None:
        got, _, _ = run_gemm(A, P, LPG_F32, LPG_F32, c_kind)
        assert np.array_equal(got, ref.gemm(A, P))


def test_beta_zero_never_reads_c_in_and_alpha_zero():
    rng = np.random.default_rng(8)
    A = rng.uniform(-1, 1, (70, 90)).astype(np.float32)
    B = rng.uniform(-1, 1, (90, 50)).astype(np.float32)
    got, _, _ = run_gemm(A, B, LPG_F32, LPG_F32, LPG_PACKED_A, alpha=1.0, beta=0.0, poison_c=True)
    assert np.isfinite(got).all()
    assert ref.rel_frobenius(got, ref.gemm(A, B)) <= F32_TOL
    C = rng.uniform(-1, 1, (70, 50)).astype(np.float32)
    got, _, _ = run_gemm(A, B, LPG_F32, LPG_F32, LPG_PACKED_B, alpha=0.0, beta=3.0, C=C)
    assert np.array_equal(got, (np.float32(3.0) * C).astype(np.float64))        # one fp32 rounding


def test_in_place_c():
    rng = np.random.default_rng(9)
    m, n, k = 100, 60, 40
    A = rng.uniform(-1, 1, (m, k)).astype(np.float32)
    B = rng.uniform(-1, 1, (k, n)).astype(np.float32)
    C = rng.uniform(-1, 1, (m, n)).astype(np.float32)
    ta, ad = pack_dev(A, LPG_PACKED_A, LPG_F32)
    tb, bd = pack_dev(B, LPG_PACKED_B, LPG_F32)
    tc, cd = pack_dev(C, LPG_PACKED_A, LPG_F32)
    api.lpg_gemm_packed(1.0, ta, ad, tb, bd, 1.0, tc, tc, cd, 0, None, stream())
    assert ref.rel_frobenius(unpack_dev(tc, cd), ref.gemm(A, B, 1.0, 1.0, C)) <= F32_TOL


@pytest.mark.parametrize("out_dt", [LPG_BF16, LPG_F32])
@pytest.mark.parametrize("c_kind", [LPG_PACKED_A, LPG_PACKED_B])
@pytest.mark.parametrize("m,n,k", [(64, 64, 64), (128, 128, 128), (33, 17, 65), (129, 257, 70), (96, 160, 200),
                                   (40, 300, 33)])
def test_bf16_gemm_matches_oracle(out_dt, c_kind, m, n, k):
    rng = np.random.default_rng(m + 3 * n + 5 * k)
    A = bf16_exact(rng.standard_normal((m, k)))
    B = bf16_exact(rng.standard_normal((k, n)))
    C = bf16_exact(rng.standard_normal((m, n)))
    got, raw, cd = run_gemm(A, B, LPG_BF16, out_dt, c_kind, alpha=0.5, beta=1.0, C=C)
    want = ref.gemm(A, B, alpha=0.5, beta=1.0, C=C)
    assert ref.rel_frobenius(got, want) <= (BF16_TOL if out_dt == LPG_BF16 else 1e-5)
    if out_dt == LPG_BF16:
        # every stored value is the bf16 nearest to a float32 within fp32 rounding of the truth:
        # at most one bf16 ulp from the rounded oracle value
        assert np.all(np.abs(got - ref.round_bf16(want)) <= np.abs(want) * 2.0 ** -7 + 1e-4)
    es = ES[out_dt]
    back = got.astype(np.float32).view(np.uint32)
    back = (back >> 16).astype(np.uint16) if es == 2 else back
    assert np.array_equal(raw, ref.pack(back, c_kind == LPG_PACKED_A, es))     # zero padding


def test_bf16_small_integers_are_bit_exact():
    rng = np.random.default_rng(12)
    m, n, k = 96, 130, 200
    A = rng.integers(-1, 2, (m, k)).astype(np.float32) * (rng.random((m, k)) < 0.3)
    B = rng.integers(-1, 2, (k, n)).astype(np.float32)
    want = ref.gemm(A, B)
    assert np.abs(want).max() <= 256
    for out_dt in (LPG_BF16, LPG_F32):
        got, _, _ = run_gemm(A, B, LPG_BF16, out_dt, LPG_PACKED_A)
        assert np.array_equal(got, want)


def test_epilogue_ops():
    rng = np.random.default_rng(13)
    m, n, k = 70, 100, 64
    A = rng.uniform(-1, 1, (m, k)).astype(np.float32)
    B = rng.uniform(-1, 1, (k, n)).astype(np.float32)
    G = rng.uniform(-3, 3, (m, n)).astype(np.float32)
    base = ref.gemm(A, B, alpha=2.0)
    got, _, _ = run_gemm(A, B, LPG_F32, LPG_F32, LPG_PACKED_A, alpha=2.0, epi=LPG_EPI_SILU)
    assert ref.rel_frobenius(got, ref.silu_mul(base, np.ones_like(base))) <= 1e-5
    got, _, _ = run_gemm(A, B, LPG_F32, LPG_F32, LPG_PACKED_B, alpha=2.0, epi=LPG_EPI_GATE_SILU, E=G)
    assert ref.rel_frobenius(got, ref.silu_mul(G, base)) <= 1e-5


def test_batched_heads_with_shared_kv_and_views():
    """S_h = a * Q_h K_g^T and O_h = S_h V_g with g = h // 2, Q/O as column views of a
    parent and K, V as views selected through batch_div (fp32, so K blocks are 32 wide)."""
    rng = np.random.default_rng(21)
    t, dh, nq, nkv = 100, 32, 4, 2
    Q = rng.standard_normal((t, nq * dh)).astype(np.float32)
    K = rng.standard_normal((t, nkv * dh)).astype(np.float32)
    V = rng.standard_normal((t, nkv * dh)).astype(np.float32)
    tq, qd = pack_dev(Q, LPG_PACKED_A, LPG_F32)
    tk, kd = pack_dev(K, LPG_PACKED_A, LPG_F32)        # = right-operand image of K^T
    tv, vd = pack_dev(V, LPG_PACKED_B, LPG_F32)
    q_view = desc(LPG_PACKED_A, LPG_F32, t, dh, parent=(t, nq * dh), batch=nq, batch_step=(0, dh))
    kt_view = desc(LPG_PACKED_B, LPG_F32, dh, t, parent=(nkv * dh, t), batch=nq, batch_div=2, batch_step=(dh, 0))
    v_view = desc(LPG_PACKED_B, LPG_F32, t, dh, parent=(t, nkv * dh), batch=nq, batch_div=2, batch_step=(0, dh))
    s_d = desc(LPG_PACKED_A, LPG_F32, t, t, batch=nq, batch_stride=ref.packed_elems(t, t, 4))
    o_view = desc(LPG_PACKED_A, LPG_F32, t, dh, parent=(t, nq * dh), batch=nq, batch_step=(0, dh))
    o_full = desc(LPG_PACKED_A, LPG_F32, t, nq * dh)
    ts = dev_empty(api.lpg_packed_bytes(s_d), fill=0xFF)
    to = dev_empty(api.lpg_packed_bytes(o_full), fill=0xFF)
    api.lpg_gemm_packed(0.25, tq, q_view, tk, kt_view, 0.0, None, ts, s_d, 0, None, stream())
    api.lpg_gemm_packed(1.0, ts, s_d, tv, v_view, 0.0, None, to, o_view, 0, None, stream())
    S = unpack_dev(ts, s_d)
    O = unpack_dev(to, o_full)
    for h in range(nq):
        g = h // 2
        s_ref = ref.gemm(Q[:, h * dh:(h + 1) * dh], K[:, g * dh:(g + 1) * dh].T.copy(), alpha=0.25)
        assert ref.rel_frobenius(S[h], s_ref) <= F32_TOL
        o_ref = ref.gemm(S[h], V[:, g * dh:(g + 1) * dh].copy())
        assert ref.rel_frobenius(O[:, h * dh:(h + 1) * dh], o_ref) <= F32_TOL


@pytest.mark.parametrize("dtype", [LPG_F32, LPG_BF16])
def test_elementwise_ops(dtype):
    rng = np.random.default_rng(31)
    rows, cols = 70, 130
    X = bf16_exact(rng.uniform(-4, 4, (rows, cols)))
    Y = bf16_exact(rng.uniform(-4, 4, (rows, cols)))
    tx, d = pack_dev(X, LPG_PACKED_A, dtype)
    ty, _ = pack_dev(Y, LPG_PACKED_A, dtype)
    tol = 1e-6 if dtype == LPG_F32 else 2.0 ** -8
    for op, s, want in ((LPG_EW_SCALE, 0.125, 0.125 * X.astype(np.float64)),
                        (LPG_EW_ADD, 2.0, X.astype(np.float64) + 2.0 * Y),
                        (LPG_EW_SILU_MUL, 0.0, ref.silu_mul(X, Y))):
        out = dev_empty(api.lpg_packed_bytes(d), fill=0xFF)
        api.lpg_elementwise_packed(op, tx, ty if op != LPG_EW_SCALE else None, s, out, d, stream())
        got = unpack_dev(out, d)
        assert np.all(np.abs(got - want) <= tol * np.abs(want) + 1e-30), op
        raw = host(out, NP_RAW[dtype])[:api.lpg_packed_bytes(d) // ES[dtype]]
        back = got.astype(np.float32).view(np.uint32)
        back = (back >> 16).astype(np.uint16) if dtype == LPG_BF16 else back
        assert np.array_equal(raw, ref.pack(back, True, ES[dtype]))            # padding stays zero


@pytest.mark.parametrize("cfg", range(8))
def test_every_tile_configuration(cfg, tune):
    """Each tile configuration of the GEMM kernel, forced through the LPG_TUNE_TILE hook, on shapes
    that span several tiles, a ragged tail and several tiles per persistent workgroup.  The
    first two shapes have at most 256 tiles (fp32 then runs its deeper staging ring), the
    third more than 256 tiles in every configuration up to 128 x 128, the fourth at most 256
    tiles and an even number of K blocks (fp32 then walks two K blocks per step)."""
    tune(api.LPG_TUNE_TILE, cfg)
    rng = np.random.default_rng(100 + cfg)
    for (m, n, k) in [(300, 520, 200), (70, 40, 33), (2100, 2100, 96), (200, 330, 256)]:
        A = rng.uniform(-1, 1, (m, k)).astype(np.float32)
        B = rng.uniform(-1, 1, (k, n)).astype(np.float32)
        C = rng.uniform(-1, 1, (m, n)).astype(np.float32)
        for c_kind in (LPG_PACKED_A, LPG_PACKED_B):
            got, raw, _ = run_gemm(A, B, LPG_F32, LPG_F32, c_kind, alpha=1.5, beta=0.5, C=C)
            assert ref.rel_frobenius(got, ref.gemm(A, B, 1.5, 0.5, C)) <= F32_TOL, (cfg, m, n, k)
            assert np.array_equal(raw, ref.pack(got.astype(np.float32), c_kind == LPG_PACKED_A, 4))
        Ab, Bb = bf16_exact(A), bf16_exact(B)
        got, _, _ = run_gemm(Ab, Bb, LPG_BF16, LPG_BF16, LPG_PACKED_A)
        assert ref.rel_frobenius(got, ref.gemm(Ab, Bb)) <= BF16_TOL, (cfg, m, n, k)
        got, _, _ = run_gemm(Ab, Bb, LPG_BF16, LPG_F32, LPG_PACKED_B)
        assert ref.rel_frobenius(got, ref.gemm(Ab, Bb)) <= 1e-5, (cfg, m, n, k)
    # integer inputs: exact, many tiles per workgroup (batched)
    A = rng.integers(-2, 3, (96, 64)).astype(np.float32)
    B = rng.integers(-2, 3, (64, 96)).astype(np.float32)
    got, _, _ = run_gemm(A, B, LPG_F32, LPG_F32, LPG_PACKED_A)
    assert np.array_equal(got, ref.gemm(A, B))


_LONG_K_CASES = {}


def _long_k_case(key):
    """Inputs and oracle results of the long-contraction cases, computed once per process."""
    if key not in _LONG_K_CASES:
        m, n, k = key
        rng = np.random.default_rng(m + 3 * n + 7 * k)
        A = rng.integers(-3, 4, (m, k)).astype(np.float32)     # small integers: every product and sum is exact in
        B = rng.integers(-3, 4, (k, n)).astype(np.float32)     # fp32 and in bf16 inputs with fp32 accumulation
        _LONG_K_CASES[key] = (A, B, ref.gemm(A, B))
    return _LONG_K_CASES[key]


@pytest.mark.parametrize("rings", [(0, 0), (1, 1)])
@pytest.mark.parametrize("cfg", range(8))
def test_long_contractions_in_every_ring_variant(cfg, rings, tune):
    """Contractions long enough that the copy cursor of every staging ring (up to four steps ahead) switches
    tile in the middle of a tile's step loop, in every tile configuration and with the whole-block / two-block
    step variants on and off: one shape of few tiles (the deeper rings of lone workgroups), one of more tiles
    than persistent workgroups (every workgroup walks several tiles, so the peeled tile-switch step runs with a
    live cursor), both ragged.  Integer inputs, so the result is exact in both dtypes and must equal the oracle
    bit for bit."""
    tune(api.LPG_TUNE_TILE, cfg)
    tune(api.LPG_TUNE_BF16_WHOLE_BLOCK_STEPS, rings[0])
    tune(api.LPG_TUNE_TWO_BLOCK_STEPS, rings[1])
    many = (4200, 4136, 330) if cfg in (4, 5, 6) else (2100, 2070, 330)
    for key in ((300, 520, 1100), many):
        A, B, want = _long_k_case(key)
        got, raw, _ = run_gemm(A, B, LPG_F32, LPG_F32, LPG_PACKED_A)
        assert np.array_equal(got, want), (cfg, rings, key, "f32")
        assert np.array_equal(raw, ref.pack(got.astype(np.float32), True, 4))
        got, _, _ = run_gemm(A, B, LPG_BF16, LPG_F32, LPG_PACKED_B)
        assert np.array_equal(got, want), (cfg, rings, key, "bf16 -> f32")
    A, B, want = _long_k_case((300, 520, 1100))
    got, _, _ = run_gemm(A, B, LPG_BF16, LPG_BF16, LPG_PACKED_A)
    assert np.array_equal(got, ref.round_bf16(want)), (cfg, rings, "bf16")


# ---- fused boundary kernels: canonical operands read / written by the GEMM itself

def _canon_dev(a, ld):
    rows, cols = a.shape
    buf = np.full((rows, ld), np.float32(777.0), dtype=np.float32)
    buf[:, :cols] = a
    return dev_bytes(buf), buf


@pytest.mark.parametrize("m,n,k", [(64, 64, 64), (130, 70, 96), (300, 520, 160), (33, 257, 32)])
@pytest.mark.parametrize("c_kind", [LPG_PACKED_A, LPG_PACKED_B])
def test_initial_kernel_reads_canonical_operands(m, n, k, c_kind):
    """A row-major and/or B column-major (both contiguous along k) fed straight to the GEMM:
    same bits as packing first."""
    rng = np.random.default_rng(m + n + k)
    A = rng.uniform(-1, 1, (m, k)).astype(np.float32)
    B = rng.uniform(-1, 1, (k, n)).astype(np.float32)
    want_bits, raw_ref, cd = run_gemm(A, B, LPG_F32, LPG_F32, c_kind, alpha=1.25)
    ta, _ = _canon_dev(A, k + 4)
    tbt, _ = _canon_dev(np.ascontiguousarray(B.T), k + 8)                 # B column-major, ld = k + 8
    a_can = desc(LPG_ROW_MAJOR, LPG_F32, m, k, ld=k + 4)
    b_can = desc(api.LPG_COL_MAJOR, LPG_F32, k, n, ld=k + 8)
    pa, pad = pack_dev(A, LPG_PACKED_A, LPG_F32)
    pb, pbd = pack_dev(B, LPG_PACKED_B, LPG_F32)
    for (xa, xad, xb, xbd) in ((ta, a_can, pb, pbd), (pa, pad, tbt, b_can), (ta, a_can, tbt, b_can)):
        tc = dev_empty(api.lpg_packed_bytes(cd), fill=0xFF)
        api.lpg_gemm_packed(1.25, xa, xad, xb, xbd, 0.0, None, tc, cd, 0, None, stream())
        raw = host(tc, np.uint32)[:raw_ref.size]
        assert np.array_equal(raw, raw_ref)
    assert ref.rel_frobenius(want_bits, ref.gemm(A, B, alpha=1.25)) <= F32_TOL


@pytest.mark.parametrize("m,n,k", [(64, 64, 64), (130, 70, 100), (300, 520, 33), (1, 1, 1)])
@pytest.mark.parametrize("c_kind", [LPG_ROW_MAJOR, api.LPG_COL_MAJOR])
@pytest.mark.parametrize("in_dt,out_dt", [(LPG_F32, LPG_F32), (LPG_BF16, LPG_F32), (LPG_BF16, LPG_BF16)])
def test_ending_kernel_writes_canonical_c(m, n, k, c_kind, in_dt, out_dt):
    """C written straight to row/column-major (with a leading dimension), beta*C_in read from
    the same canonical layout; elements outside the logical extent are never touched."""
    rng = np.random.default_rng(3 * m + n + k)
    A = bf16_exact(rng.uniform(-1, 1, (m, k)))
    B = bf16_exact(rng.uniform(-1, 1, (k, n)))
    C = bf16_exact(rng.uniform(-1, 1, (m, n)))
    rm = c_kind == LPG_ROW_MAJOR
    ld = (n if rm else m) + 5
    es = ES[out_dt]
    def to_canon(x):
        rows = x if rm else np.ascontiguousarray(x.T)
        buf = np.full((rows.shape[0], ld), 3.0, dtype=np.float32)
        buf[:, :rows.shape[1]] = rows
        if out_dt == LPG_BF16:
            return (buf.view(np.uint32) >> 16).astype(np.uint16)
        return buf
    cin = to_canon(C)
    t_cin = dev_bytes(cin)
    t_out = dev_bytes(to_canon(np.zeros((m, n), dtype=np.float32)))      # poison 3.0 everywhere outside
    ta, ad = pack_dev(A, LPG_PACKED_A, in_dt)
    tb, bd = pack_dev(B, LPG_PACKED_B, in_dt)
    cd = desc(c_kind, out_dt, m, n, ld=ld)
    api.lpg_gemm_packed(0.5, ta, ad, tb, bd, 2.0, t_cin, t_out, cd, 0, None, stream())
    got_raw = host(t_out, NP_RAW[out_dt])[:cin.size].reshape(cin.shape)
    got_f = got_raw.view(np.float32) if es == 4 else (got_raw.astype(np.uint32) << 16).view(np.float32)
    inner = got_f[:, :(n if rm else m)]
    got = (inner if rm else inner.T).astype(np.float64)
    want = ref.gemm(A, B, alpha=0.5, beta=2.0, C=C)
    assert ref.rel_frobenius(got, want) <= (BF16_TOL if out_dt == LPG_BF16 else 1e-5)
    assert np.all(got_f[:, (n if rm else m):] == 3.0)                      # ld padding untouched
    # identical bits to the packed result unpacked afterwards
    pk_kind = LPG_PACKED_A if not rm else LPG_PACKED_B
    got2, _, _ = run_gemm(A, B, in_dt, out_dt, pk_kind, alpha=0.5, beta=2.0, C=C)
    assert np.array_equal(got, got2)


def test_fused_boundaries_with_heads():
    """Initial + Ending in one call, batched over heads: S_h = Q_h K_h^T with Q, K row-major
    [heads, t, d] read directly and S written row-major."""
    rng = np.random.default_rng(77)
    nh, t, d = 3, 100, 64
    Q = rng.standard_normal((nh, t, d)).astype(np.float32)
    K = rng.standard_normal((nh, t, d)).astype(np.float32)
    qd = desc(LPG_ROW_MAJOR, LPG_F32, t, d, batch=nh, batch_stride=t * d)
    ktd = desc(api.LPG_COL_MAJOR, LPG_F32, d, t, batch=nh, batch_stride=t * d)      # K_h^T column-major = K_h row-major
    sd = desc(LPG_ROW_MAJOR, LPG_F32, t, t, batch=nh, batch_stride=t * t)
    ts = dev_empty(nh * t * t * 4, fill=0xFF)
    api.lpg_gemm_packed(0.125, dev_bytes(Q), qd, dev_bytes(K), ktd, 0.0, None, ts, sd, 0, None, stream())
    S = host(ts, np.float32, (nh, t, t)).astype(np.float64)
    for h in range(nh):
        assert ref.rel_frobenius(S[h], ref.gemm(Q[h], K[h].T.copy(), alpha=0.125)) <= F32_TOL
