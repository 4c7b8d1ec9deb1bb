"""GPU parity of the "block order" and "store stride" parameters (section III-C): packed buffers whose
blocks lie in another order (groups outermost) or with room between them (group_stride / kblock_stride
of lpg_desc), through lpg_pack, lpg_unpack, lpg_gemm_packed and lpg_chain, against the oracle's pack
with the same strides (bit for bit: the room between blocks keeps what it held) and its GEMM."""
import numpy as np
import pytest
import torch

from oracle import ref
from paper_2604_04599_amd import api
from paper_2604_04599_amd.api import (LPG_BF16, LPG_COL_MAJOR, LPG_F32, LPG_PACKED_A, LPG_PACKED_B, LPG_ROW_MAJOR, desc)
from tests.gpu_util import ES, NP_RAW, bf16_raw_to_f64, dev_bytes, dev_empty, host, stream

pytestmark = pytest.mark.gpu


def strides_for(order, F, K, es):
    """(group_stride, kblock_stride) in elements for a parent of free extent F, contraction extent K."""
    kb = ref.layout_consts(es)[2]
    blk = 32 * kb
    ng, nk = (F + 31) // 32, (K + kb - 1) // kb
    return {"default": (0, 0), "groups_outer": (nk * blk, blk), "groups_outer_gaps": ((nk + 2) * blk, 0),
            "gaps": (2 * blk, (2 * ng + 3) * blk), "k_gaps": (0, (ng + 1) * blk)}[order]


ORDERS = ["groups_outer", "groups_outer_gaps", "gaps", "k_gaps"]


def iota(rows, cols, dtype):
    n = rows * cols
    return ((np.arange(n, dtype=np.int64) * 2654435761 + 99) % (1 << (8 * ES[dtype]))).astype(NP_RAW[dtype]).reshape(rows, cols)


@pytest.mark.parametrize("order", ORDERS)
@pytest.mark.parametrize("dtype", [LPG_F32, LPG_BF16])
@pytest.mark.parametrize("kind,src_kind", [(LPG_PACKED_A, LPG_ROW_MAJOR), (LPG_PACKED_B, LPG_ROW_MAJOR), (LPG_PACKED_A, LPG_COL_MAJOR)])
@pytest.mark.parametrize("rows,cols", [(70, 200), (33, 65), (257, 129)])
def test_pack_and_unpack_with_block_strides(rows, cols, kind, src_kind, dtype, order):
    es = ES[dtype]
    a_side = kind == LPG_PACKED_A
    F, K = (rows, cols) if a_side else (cols, rows)
    gs, ks = strides_for(order, F, K, es)
    a = iota(rows, cols, dtype)
    canon = a if src_kind == LPG_ROW_MAJOR else np.ascontiguousarray(a.T)
    sd = desc(src_kind, dtype, rows, cols)
    dd = desc(kind, dtype, rows, cols, group_stride=gs, kblock_stride=ks)
    nbytes = api.lpg_packed_bytes(dd)
    assert nbytes == ref.strided_elems(F, K, es, gs, ks) * es
    dst = dev_empty(nbytes, fill=0xEE)
    api.lpg_pack(dev_bytes(canon), sd, dst, dd, stream())
    got = host(dst, NP_RAW[dtype])[:nbytes // es]
    poison = np.full(nbytes // es, 0xEEEE if es == 2 else 0xEEEEEEEE, dtype=NP_RAW[dtype])
    want = ref.pack(a, a_side, es, out=poison, group_stride=gs, kblock_stride=ks)
    assert np.array_equal(got, want)                       # blocks where they belong, the room untouched
    back = dev_empty(canon.nbytes, fill=0x77)
    api.lpg_unpack(dst, dd, back, sd, stream())
    assert np.array_equal(host(back, NP_RAW[dtype])[:canon.size].reshape(canon.shape), canon)


def _f64(raw, dtype):
    return raw.view(np.float32).astype(np.float64) if dtype == LPG_F32 else bf16_raw_to_f64(raw)


def _raw(x, dtype):
    f = np.ascontiguousarray(x, dtype=np.float32)
    return f.view(np.uint32).copy() if dtype == LPG_F32 else ref.bf16_bits(f.view(np.uint32))


@pytest.mark.parametrize("c_kind", [LPG_PACKED_A, LPG_PACKED_B])
@pytest.mark.parametrize("in_dt,out_dt", [(LPG_F32, LPG_F32), (LPG_BF16, LPG_BF16), (LPG_BF16, LPG_F32)])
@pytest.mark.parametrize("orders", [("groups_outer", "gaps", "groups_outer_gaps"), ("gaps", "groups_outer", "k_gaps"),
                                    ("default", "k_gaps", "groups_outer")])
@pytest.mark.parametrize("m,n,k", [(300, 200, 130), (70, 520, 64), (33, 17, 65)])
def test_gemm_with_block_strides_on_every_operand(m, n, k, orders, in_dt, out_dt, c_kind):
    """A, B and C each under their own block order / store stride; beta reads C_in through C's strides."""
    rng = np.random.default_rng(m + n + k)
    es_in, es = ES[in_dt], ES[out_dt]
    A = _f64(_raw(rng.standard_normal((m, k)), in_dt), in_dt)
    B = _f64(_raw(rng.standard_normal((k, n)) / np.sqrt(k), in_dt), in_dt)
    C = _f64(_raw(rng.standard_normal((m, n)), out_dt), out_dt)
    ga, ka = strides_for(orders[0], m, k, es_in)
    gb, kb_ = strides_for(orders[1], n, k, es_in)
    a_side = c_kind == LPG_PACKED_A
    FC, KC = (m, n) if a_side else (n, m)
    gc, kc = strides_for(orders[2], FC, KC, es)
    ad = desc(LPG_PACKED_A, in_dt, m, k, group_stride=ga, kblock_stride=ka)
    bd = desc(LPG_PACKED_B, in_dt, k, n, group_stride=gb, kblock_stride=kb_)
    cd = desc(c_kind, out_dt, m, n, group_stride=gc, kblock_stride=kc)
    Ap = dev_bytes(ref.pack(_raw(A, in_dt), True, es_in, group_stride=ga, kblock_stride=ka))
    Bp = dev_bytes(ref.pack(_raw(B, in_dt), False, es_in, group_stride=gb, kblock_stride=kb_))
    room = np.full(api.lpg_packed_bytes(cd) // es, 0x5A5A if es == 2 else 0x5A5A5A5A, dtype=NP_RAW[out_dt])
    c_before = ref.pack(_raw(C, out_dt), a_side, es, out=room.copy(), group_stride=gc, kblock_stride=kc)
    Cp = dev_bytes(c_before)
    api.lpg_gemm_packed(0.5, Ap, ad, Bp, bd, -1.0, Cp, Cp, cd, 0, None, stream())
    got_raw = host(Cp, NP_RAW[out_dt])[:c_before.size]
    got = _f64(ref.unpack(got_raw, m, n, a_side, es, group_stride=gc, kblock_stride=kc), out_dt)
    want = ref.gemm(A, B, alpha=0.5, beta=-1.0, C=C)
    assert ref.rel_frobenius(got, want) <= (1e-5 if out_dt == LPG_F32 else 1e-2)
    # the whole buffer: the result packed under C's strides, zero padding inside blocks, the room as it was
    assert np.array_equal(got_raw, ref.pack(_raw(got, out_dt), a_side, es, out=room.copy(), group_stride=gc, kblock_stride=kc))


def test_a_chain_hands_a_strided_intermediate_from_gemm_to_gemm_in_both_modes():
    """X W1 W2 with the intermediate kept packed in groups-outermost order with room between groups; the
    canonical-layout control gives the same bits; a consumer that names other strides is refused."""
    rng = np.random.default_rng(5)
    m, d, h = 200, 96, 160
    X = rng.standard_normal((m, d)).astype(np.float32)
    W1 = (rng.standard_normal((d, h)) / np.sqrt(d)).astype(np.float32)
    W2 = (rng.standard_normal((h, d)) / np.sqrt(h)).astype(np.float32)
    gs, ks = strides_for("groups_outer_gaps", m, h, 4)
    xd, hd, yd = desc(LPG_PACKED_A, LPG_F32, m, d), desc(LPG_PACKED_A, LPG_F32, m, h, group_stride=gs, kblock_stride=ks), desc(LPG_PACKED_A, LPG_F32, m, d)
    w1d, w2d = desc(LPG_PACKED_B, LPG_F32, d, h), desc(LPG_PACKED_B, LPG_F32, h, d)
    xs, y = dev_bytes(X), dev_empty(m * d * 4, fill=0xFF)
    px, ph, py = (dev_empty(api.lpg_packed_bytes(dd), fill=0xFF) for dd in (xd, hd, yd))
    pw1 = dev_bytes(ref.pack(W1.view(np.uint32), False, 4))
    pw2 = dev_bytes(ref.pack(W2.view(np.uint32), False, 4))
    rm_x, rm_y = desc(LPG_ROW_MAJOR, LPG_F32, m, d), desc(LPG_ROW_MAJOR, LPG_F32, m, d)
    stages = [api.stage_pack(xs, rm_x, px, xd), api.stage_gemm(1.0, px, xd, pw1, w1d, 0.0, None, ph, hd),
              api.stage_gemm(1.0, ph, hd, pw2, w2d, 0.0, None, py, yd), api.stage_unpack(py, yd, y, rm_y)]
    api.lpg_chain(stages, api.LPG_CHAIN_PROPAGATED, None, 0, stream())
    prop = host(y, np.float32, (m, d)).copy()
    assert ref.rel_frobenius(prop, ref.gemm(ref.gemm(X, W1), W2)) <= 2e-5
    need = api.lpg_chain_workspace_bytes(stages, api.LPG_CHAIN_CANONICAL)
    ws = dev_empty(need)
    y.fill_(0xFF)
    api.lpg_chain(stages, api.LPG_CHAIN_CANONICAL, ws, need, stream())
    assert np.array_equal(host(y, np.uint32, (m, d)), prop.view(np.uint32))
    bad = list(stages)
    bad[2] = api.stage_gemm(1.0, ph, desc(LPG_PACKED_A, LPG_F32, m, h), pw2, w2d, 0.0, None, py, yd)
    with pytest.raises(api.LpgError) as e:
        api.lpg_chain(bad, api.LPG_CHAIN_PROPAGATED, None, 0, stream())
    assert e.value.code == api.LPG_ELAYOUT
    torch.cuda.synchronize()


def test_entry_points_that_need_the_default_order_say_so():
    d = desc(LPG_PACKED_A, LPG_F32, 64, 64, group_stride=2 * 1024, kblock_stride=8 * 1024)
    buf = dev_empty(api.lpg_packed_bytes(d), fill=0)
    for call in (lambda: api.lpg_elementwise_packed(api.LPG_EW_SCALE, buf, None, 1.0, buf, d, stream()),
                 lambda: api.lpg_softmax_packed(buf, buf, d, 1.0, False, stream())):
        with pytest.raises(api.LpgError) as e:
            call()
        assert e.value.code == api.LPG_EUNSUPPORTED
    torch.cuda.synchronize()
