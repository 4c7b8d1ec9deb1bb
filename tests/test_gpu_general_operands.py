"""GPU parity of the general Initial kernel (section III-A.1: the first kernel of a chain packs whatever
the caller has): lpg_gemm_packed with operands in every form the main kernel cannot copy verbatim -
canonical matrices of either order and either dtype (fp32 ones rounded to bf16 on the way when the
partner is bf16), any leading dimension and alignment, contractions of any length, views of packed
parents with any origin and extent - and shifted read views in the free dimension, which the main
kernel takes itself.  Every case is compared with the oracle (Eq. 1) and, bit for bit, with lpg_pack
of the same logical operands followed by the packed product."""
import numpy as np
import pytest

from oracle import ref
from paper_2604_04599_amd import api
from paper_2604_04599_amd.api import (LPG_BF16, LPG_COL_MAJOR, LPG_F32, LPG_PACKED_A, LPG_PACKED_B, LPG_ROW_MAJOR, desc)
from tests.gpu_util import ES, NP_RAW, bf16_raw_to_f64, dev_bytes, dev_empty, host, stream

pytestmark = pytest.mark.gpu

EDGES = [1, 2, 31, 32, 33, 63, 64, 65, 96, 127, 128, 129, 160, 255, 256, 257, 300]
NP_F = {LPG_F32: np.float32}


def f64(raw, dtype):
    return raw.view(np.float32).astype(np.float64) if dtype == LPG_F32 else bf16_raw_to_f64(raw)


def raw_of(x, dtype):
    f = np.ascontiguousarray(x, dtype=np.float32)
    return f.view(np.uint32).copy() if dtype == LPG_F32 else ref.bf16_bits(f.view(np.uint32))


def make_operand(rng, rows, cols, is_a, form, in_dt):
    """Returns (device buffer, descriptor, logical matrix as float64 after any rounding the product applies)."""
    kind = LPG_PACKED_A if is_a else LPG_PACKED_B
    es = ES[in_dt]
    kb = ref.layout_consts(es)[2]
    if form in ("packed", "view_f", "view_fk", "inner_k"):
        # a view [r0, r0+rows) x [c0, c0+cols) of a larger packed parent
        fdim_is_rows = is_a
        if form == "packed":
            r0 = c0 = 0
            prow, pcol = rows, cols
        else:
            f0 = int(rng.integers(1, 70)) if form in ("view_f", "view_fk") else 32 * int(rng.integers(0, 2))
            k0 = int(rng.integers(1, 70)) if form == "view_fk" else kb * int(rng.integers(0, 2))
            r0, c0 = (f0, k0) if is_a else (k0, f0)
            prow, pcol = r0 + rows + int(rng.integers(1, 40)), c0 + cols + int(rng.integers(1, 40))
        parent = f64(raw_of(rng.standard_normal((prow, pcol)), in_dt), in_dt)
        buf = dev_bytes(ref.pack(raw_of(parent, in_dt), fdim_is_rows, es))
        d = desc(kind, in_dt, rows, cols, parent=(prow, pcol), origin=(r0, c0))
        return buf, d, np.ascontiguousarray(parent[r0:r0 + rows, c0:c0 + cols])
    # canonical: row- or column-major, fp32 or bf16 elements, padded leading dimension, base off by a few elements
    src_dt = LPG_BF16 if form.endswith("_bf16") else LPG_F32
    order = LPG_ROW_MAJOR if form.startswith("row") else LPG_COL_MAJOR
    x = f64(raw_of(rng.standard_normal((rows, cols)), src_dt), src_dt)
    lead, other = (cols, rows) if order == LPG_ROW_MAJOR else (rows, cols)
    ld = lead + int(rng.integers(0, 6))
    shift = int(rng.integers(0, 4))
    stored = np.full(shift + other * ld, 7.0, dtype=np.float64)
    body = stored[shift:].reshape(other, ld)
    body[:, :lead] = x if order == LPG_ROW_MAJOR else x.T
    raw = raw_of(stored, src_dt)
    # the base must stay 16-byte aligned for the buffer; the shift is applied through the pointer
    buf = dev_bytes(raw)
    d = desc(order, src_dt, rows, cols, ld=ld)
    logical = f64(raw_of(x, in_dt), in_dt)             # an fp32 source feeding a bf16 product is rounded once
    return (buf, shift * ES[src_dt]), d, logical


A_FORMS = ["packed", "view_f", "view_fk", "inner_k", "row_f32", "col_f32", "row_bf16", "col_bf16"]


def draw(seed):
    rng = np.random.default_rng(90000 + seed)
    dim = lambda: int(rng.choice(EDGES)) if rng.random() < 0.6 else int(rng.integers(1, 400))
    c = {"m": dim(), "n": dim(), "k": dim(), "rng": rng}
    c["a_form"], c["b_form"] = A_FORMS[seed % 8], A_FORMS[(seed // 8 + seed) % 8]
    bf = c["a_form"].endswith("bf16") or c["b_form"].endswith("bf16")
    c["in_dt"] = LPG_BF16 if bf or rng.random() < 0.4 else LPG_F32
    if c["a_form"].endswith("f32") and c["b_form"].endswith("f32"):
        c["in_dt"] = LPG_F32                     # two fp32 canonical operands make an fp32 product
    c["out_dt"] = LPG_F32 if c["in_dt"] == LPG_F32 or rng.random() < 0.3 else LPG_BF16
    c["kind"] = int(rng.choice([LPG_PACKED_A, LPG_PACKED_B, LPG_ROW_MAJOR, LPG_COL_MAJOR]))
    c["alpha"], c["beta"] = float(rng.choice([1.0, -0.75])), float(rng.choice([0.0, 0.0, 1.0]))
    return c


def ptr_of(b):
    return b[0].data_ptr() + b[1] if isinstance(b, tuple) else b


@pytest.mark.parametrize("seed", range(96))
def test_general_operand_forms(seed):
    c = draw(seed)
    rng, m, n, k, in_dt, out_dt, kind = c["rng"], c["m"], c["n"], c["k"], c["in_dt"], c["out_dt"], c["kind"]
    es = ES[out_dt]
    abuf, ad, A = make_operand(rng, m, k, True, c["a_form"], in_dt)
    bbuf, bd, B = make_operand(rng, k, n, False, c["b_form"], in_dt)
    C = f64(raw_of(rng.standard_normal((m, n)), out_dt), out_dt)
    packed = kind in (LPG_PACKED_A, LPG_PACKED_B)
    a_side = kind == LPG_PACKED_A

    def c_buffer():
        if packed:
            return dev_bytes(ref.pack(raw_of(C, out_dt), a_side, es))
        return dev_bytes(raw_of(C if kind == LPG_ROW_MAJOR else C.T, out_dt))
    cd = desc(kind, out_dt, m, n)
    got_buf = c_buffer()
    api.lpg_gemm_packed(c["alpha"], ptr_of(abuf), ad, ptr_of(bbuf), bd, c["beta"], got_buf if c["beta"] else None, got_buf, cd, 0,
                        None, stream())
    got_raw = host(got_buf, NP_RAW[out_dt]).copy()
    # the same product on operands packed by lpg_pack's rule (here: the oracle's pack of the logical matrices)
    pa, pb = dev_bytes(ref.pack(raw_of(A, in_dt), True, ES[in_dt])), dev_bytes(ref.pack(raw_of(B, in_dt), False, ES[in_dt]))
    ref_buf = c_buffer()
    api.lpg_gemm_packed(c["alpha"], pa, desc(LPG_PACKED_A, in_dt, m, k), pb, desc(LPG_PACKED_B, in_dt, k, n), c["beta"],
                        ref_buf if c["beta"] else None, ref_buf, cd, 0, None, stream())
    assert np.array_equal(got_raw, host(ref_buf, NP_RAW[out_dt])), {x: y for x, y in c.items() if x != "rng"}
    if packed:
        got = f64(ref.unpack(got_raw, m, n, a_side, es), out_dt)
    else:
        arr = got_raw[:m * n].reshape((m, n) if kind == LPG_ROW_MAJOR else (n, m))
        got = f64(np.ascontiguousarray(arr if kind == LPG_ROW_MAJOR else arr.T), out_dt)
    want = ref.gemm(A, B, alpha=c["alpha"], beta=c["beta"], C=C if c["beta"] else None)
    tol = 1e-5 if (in_dt == LPG_F32 and out_dt == LPG_F32) else (1e-5 if out_dt == LPG_F32 else 1e-2)
    assert ref.rel_frobenius(got, want) <= tol, {x: y for x, y in c.items() if x != "rng"}


@pytest.mark.parametrize("dtype", [LPG_F32, LPG_BF16])
def test_row_major_weight_and_fp32_activations_of_a_bf16_layer(dtype):
    """The shapes the Initial kernel is for: X [m x k] row-major fp32 and a weight W [k x n] row-major (contiguous
    along n, not k), several tiles and K blocks, ragged everywhere; batched over slots with a shared weight."""
    rng = np.random.default_rng(11)
    nb, m, k, n = 3, 300, 200, 270
    X = f64(raw_of(rng.standard_normal((nb, m, k)), dtype), dtype)
    W = f64(raw_of(rng.standard_normal((k, n)) / np.sqrt(k), dtype), dtype)
    xd = desc(LPG_ROW_MAJOR, LPG_F32, m, k, batch=nb, batch_stride=m * k)
    wd = desc(LPG_ROW_MAJOR, LPG_F32, k, n, batch=nb, batch_div=nb)
    cd = desc(LPG_PACKED_A, dtype, m, n, batch=nb, batch_stride=ref.packed_elems(m, n, ES[dtype]))
    out = dev_empty(api.lpg_packed_bytes(cd), fill=0xFF)
    api.lpg_gemm_packed(1.0, dev_bytes(X.astype(np.float32)), xd, dev_bytes(W.astype(np.float32)), wd, 0.0, None, out, cd, 0, None, stream())
    raw = host(out, NP_RAW[dtype])
    per = ref.packed_elems(m, n, ES[dtype])
    for b in range(nb):
        got = f64(ref.unpack(raw[b * per:(b + 1) * per], m, n, True, ES[dtype]), dtype)
        assert ref.rel_frobenius(got, ref.gemm(X[b], W)) <= (1e-5 if dtype == LPG_F32 else 1e-2)


@pytest.mark.parametrize("dtype", [LPG_F32, LPG_BF16])
@pytest.mark.parametrize("shift", [(5, 0), (0, 16), (37, 24), (31, 0)])
def test_shifted_head_views_with_shared_key_value_slots(shift, dtype):
    """Batched read views whose origin is off the grid: query heads as column slices of a packed parent
    starting `shift[0]` tokens into it (free-dimension shift: main kernel, per-lane source addresses) and,
    for shift[1] != 0, `shift[1]` columns into a head (contraction-dimension shift: general kernel); keys
    shared by pairs of query heads through batch_div; block strides on the key parent."""
    rng = np.random.default_rng(sum(shift) + dtype)
    es = ES[dtype]
    kb = ref.layout_consts(es)[2]
    nh, t, dh, tk = 4, 70, kb, 150
    f0, k0 = shift
    dk = dh - k0                                           # contraction extent of the sliced heads
    Qp = f64(raw_of(rng.standard_normal((f0 + t + 9, nh * dh)), dtype), dtype)       # parent of Q: tokens x (heads*dh)
    Kp = f64(raw_of(rng.standard_normal((tk, (nh // 2) * dh)), dtype), dtype)        # parent of K: keys x (kv heads*dh)
    blk = 32 * kb
    ng, nk = (tk + 31) // 32, (nh // 2)
    gs, ks = (nk + 1) * blk, blk                           # groups outermost with room after each group
    qd = desc(LPG_PACKED_A, dtype, t, dk, parent=Qp.shape, origin=(f0, k0), batch=nh, batch_step=(0, dh))
    # K_g^T as the right operand: rows [g*dh + k0, g*dh + dh) of K^T, the same bytes as K's left-operand image
    ktd = desc(LPG_PACKED_B, dtype, dk, tk, parent=(Kp.shape[1], Kp.shape[0]), origin=(k0, 0), batch=nh, batch_div=2,
               batch_step=(dh, 0), group_stride=gs, kblock_stride=ks)
    sd = desc(LPG_PACKED_A, LPG_F32, t, tk, batch=nh, batch_stride=ref.packed_elems(t, tk, 4))
    qbuf = dev_bytes(ref.pack(raw_of(Qp, dtype), True, es))
    kbuf = dev_bytes(ref.pack(raw_of(Kp, dtype), True, es, group_stride=gs, kblock_stride=ks))
    out = dev_empty(api.lpg_packed_bytes(sd), fill=0xFF)
    api.lpg_gemm_packed(0.125, qbuf, qd, kbuf, ktd, 0.0, None, out, sd, 0, None, stream())
    raw = host(out, np.uint32)
    per = ref.packed_elems(t, tk, 4)
    for h in range(nh):
        g = h // 2
        q = Qp[f0:f0 + t, h * dh + k0:(h + 1) * dh]
        k = Kp[:, g * dh + k0:(g + 1) * dh]
        got = ref.unpack(raw[h * per:(h + 1) * per], t, tk, True, 4).view(np.float32).astype(np.float64)
        assert ref.rel_frobenius(got, ref.gemm(q, np.ascontiguousarray(k.T), alpha=0.125)) <= 1e-5, h


def test_a_chain_may_start_from_any_canonical_operands_and_match_the_packed_chain():
    """X (row-major fp32) times a row-major weight, then a packed weight, in a bf16 chain: the first
    stage is the general Initial kernel; propagated and canonical modes agree bit for bit, and both equal
    the chain that packs X and W1 first."""
    rng = np.random.default_rng(8)
    m, d, h = 200, 130, 96
    X = f64(raw_of(rng.standard_normal((m, d)), LPG_BF16), LPG_BF16)
    W1 = f64(raw_of(rng.standard_normal((d, h)) / np.sqrt(d), LPG_BF16), LPG_BF16)
    W2 = f64(raw_of(rng.standard_normal((h, d)) / np.sqrt(h), LPG_BF16), LPG_BF16)
    xs, w1s = dev_bytes(X.astype(np.float32)), dev_bytes(W1.astype(np.float32))
    pw2 = dev_bytes(ref.pack(raw_of(W2, LPG_BF16), False, 2))
    hd, yd = desc(LPG_PACKED_A, LPG_BF16, m, h), desc(LPG_PACKED_A, LPG_F32, m, d)
    ph, py = dev_empty(api.lpg_packed_bytes(hd), fill=0xFF), dev_empty(api.lpg_packed_bytes(yd), fill=0xFF)
    y = dev_empty(m * d * 4, fill=0xFF)
    rm_x, rm_w, rm_y = desc(LPG_ROW_MAJOR, LPG_F32, m, d), desc(LPG_ROW_MAJOR, LPG_F32, d, h), desc(LPG_ROW_MAJOR, LPG_F32, m, d)
    stages = [api.stage_gemm(1.0, xs, rm_x, w1s, rm_w, 0.0, None, ph, hd),
              api.stage_gemm(1.0, ph, hd, pw2, desc(LPG_PACKED_B, LPG_BF16, h, d), 0.0, None, py, yd),
              api.stage_unpack(py, yd, y, rm_y)]
    api.lpg_chain(stages, api.LPG_CHAIN_PROPAGATED, None, 0, stream())
    prop = host(y, np.float32, (m, d)).copy()
    Hq = ref.round_bf16(ref.gemm(X, W1))
    assert ref.rel_frobenius(prop, ref.gemm(Hq, W2)) <= 5e-3
    need = api.lpg_chain_workspace_bytes(stages, api.LPG_CHAIN_CANONICAL)
    ws = dev_empty(need)
    y.fill_(0xFF)
    api.lpg_chain(stages, api.LPG_CHAIN_CANONICAL, ws, need, stream())
    assert np.array_equal(host(y, np.uint32, (m, d)), prop.view(np.uint32))
    # the same chain entered through lpg_pack
    px, pw1 = dev_bytes(ref.pack(raw_of(X, LPG_BF16), True, 2)), dev_bytes(ref.pack(raw_of(W1, LPG_BF16), False, 2))
    y.fill_(0xFF)
    packed_stages = [api.stage_gemm(1.0, px, desc(LPG_PACKED_A, LPG_BF16, m, d), pw1, desc(LPG_PACKED_B, LPG_BF16, d, h), 0.0, None, ph, hd)] + stages[1:]
    api.lpg_chain(packed_stages, api.LPG_CHAIN_PROPAGATED, None, 0, stream())
    assert np.array_equal(host(y, np.uint32, (m, d)), prop.view(np.uint32))
