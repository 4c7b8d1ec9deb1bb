"""GPU parity: lpg_pack / lpg_unpack against the oracle's loop-nest pack, bit for bit."""
import numpy as np
import pytest
import torch

from oracle import ref
from paper_2604_04599_amd import api
from paper_2604_04599_amd.api import (LPG_BF16, LPG_COL_MAJOR, LPG_F32, LPG_PACKED_A, LPG_PACKED_B,
                                      LPG_ROW_MAJOR, desc)
from tests.gpu_util import ES, NP_RAW, dev_bytes, dev_empty, host, stream

pytestmark = pytest.mark.gpu

SHAPES = [(1, 1), (32, 32), (33, 65), (70, 200), (256, 64), (5, 130), (257, 129)]


def iota(rows, cols, dtype):
    n = rows * cols
    return ((np.arange(n, dtype=np.int64) * 2654435761 + 12345) % (1 << (8 * ES[dtype]))).astype(
        NP_RAW[dtype]).reshape(rows, cols)


@pytest.mark.parametrize("dtype", [LPG_F32, LPG_BF16])
@pytest.mark.parametrize("kind", [LPG_PACKED_A, LPG_PACKED_B])
@pytest.mark.parametrize("src_kind", [LPG_ROW_MAJOR, LPG_COL_MAJOR])
@pytest.mark.parametrize("rows,cols", SHAPES)
def test_pack_is_bit_exact_and_round_trips(dtype, kind, src_kind, rows, cols):
    es = ES[dtype]
    a = iota(rows, cols, dtype)
    ld = (cols if src_kind == LPG_ROW_MAJOR else rows) + 3
    if src_kind == LPG_ROW_MAJOR:
        canon = np.zeros((rows, ld), dtype=a.dtype)
        canon[:, :cols] = a
    else:
        canon = np.zeros((cols, ld), dtype=a.dtype)
        canon[:, :rows] = a.T
    sd = desc(src_kind, dtype, rows, cols, ld=ld)
    dd = desc(kind, dtype, rows, cols)
    src = dev_bytes(canon)
    dst = dev_empty(api.lpg_packed_bytes(dd), fill=0xEE)
    api.lpg_pack(src, sd, dst, dd, stream())
    got = host(dst, NP_RAW[dtype])[:api.lpg_packed_bytes(dd) // es]
    want = ref.pack(a, kind == LPG_PACKED_A, es)
    assert got.size == want.size
    assert np.array_equal(got, want)
    # round trip into a poisoned canonical buffer: padding columns of ld stay untouched
    back = dev_empty(canon.nbytes, fill=0x77)
    api.lpg_unpack(dst, dd, back, sd, stream())
    b = host(back, NP_RAW[dtype])[:canon.size].reshape(canon.shape)
    poison = NP_RAW[dtype](0x7777 if es == 2 else 0x77777777)
    if src_kind == LPG_ROW_MAJOR:
        assert np.array_equal(b[:, :cols], a) and np.all(b[:, cols:] == poison)
    else:
        assert np.array_equal(b[:, :rows], a.T) and np.all(b[:, rows:] == poison)


def test_pack_converts_f32_to_bf16_like_the_oracle():
    rng = np.random.default_rng(17)
    rows, cols = 96, 160
    x = rng.standard_normal((rows, cols)).astype(np.float32)
    bits = x.view(np.uint32).copy()
    # plant ties, subnormals, huge values, signed zeros, infinities
    special = np.array([0x3F808000, 0x3F818000, 0x3F80FFFF, 0x00000001, 0x007FFFFF, 0x7F7FFFFF, 0x80000000,
                        0x7F800000, 0xFF800000, 0x3F800001, 0xBF808000, 0x00008000, 0x0000C000], dtype=np.uint32)
    bits.ravel()[:special.size] = special
    x = bits.view(np.float32)
    for kind in (LPG_PACKED_A, LPG_PACKED_B):
        dd = desc(kind, LPG_BF16, rows, cols)
        dst = dev_empty(api.lpg_packed_bytes(dd), fill=0xEE)
        api.lpg_pack(dev_bytes(x), desc(LPG_ROW_MAJOR, LPG_F32, rows, cols), dst, dd, stream())
        got = host(dst, np.uint16)[:api.lpg_packed_bytes(dd) // 2]
        want = ref.pack(ref.bf16_bits(bits), kind == LPG_PACKED_A, 2)
        assert np.array_equal(got, want)
        # bf16 -> f32 unpack is the exact widening
        out = dev_empty(rows * cols * 4)
        api.lpg_unpack(dst, dd, out, desc(LPG_ROW_MAJOR, LPG_F32, rows, cols), stream())
        wide = host(out, np.uint32, (rows, cols))
        assert np.array_equal(wide, ref.bf16_bits(bits).astype(np.uint32) << 16)
    # NaN stays NaN
    nan = np.array([[np.nan, 1.0]], dtype=np.float32)
    dd = desc(LPG_PACKED_A, LPG_BF16, 1, 2)
    dst = dev_empty(api.lpg_packed_bytes(dd))
    api.lpg_pack(dev_bytes(nan), desc(LPG_ROW_MAJOR, LPG_F32, 1, 2), dst, dd, stream())
    g = host(dst, np.uint16)
    assert (g[0] & 0x7F80) == 0x7F80 and (g[0] & 0x7F) != 0


@pytest.mark.parametrize("dtype", [LPG_F32, LPG_BF16])
def test_batched_views_pack_into_one_parent(dtype):
    """Head slices: batch b is the column block [b*KB, (b+1)*KB) of a packed parent."""
    es = ES[dtype]
    kb = ref.layout_consts(es)[2]
    nh, t = 3, 70
    whole = iota(t, nh * kb, dtype)
    heads = np.stack([whole[:, h * kb:(h + 1) * kb] for h in range(nh)])       # [nh, t, kb]
    sd = desc(LPG_ROW_MAJOR, dtype, t, kb, batch=nh, batch_stride=t * kb)
    dd = desc(LPG_PACKED_A, dtype, t, kb, parent=(t, nh * kb), batch=nh, batch_step=(0, kb))
    dst = dev_empty(api.lpg_packed_bytes(dd), fill=0xEE)
    api.lpg_pack(dev_bytes(heads), sd, dst, dd, stream())
    got = host(dst, NP_RAW[dtype])[:api.lpg_packed_bytes(dd) // es]
    assert np.array_equal(got, ref.pack(whole, True, es))
    # and unpack one strided view straight out of a row-major parent view
    out = dev_empty(whole.nbytes, fill=0)
    od = desc(LPG_ROW_MAJOR, dtype, t, kb, parent=(t, nh * kb), batch=nh, batch_step=(0, kb))
    api.lpg_unpack(dst, dd, out, od, stream())
    assert np.array_equal(host(out, NP_RAW[dtype], whole.shape), whole)
    # free-dimension views of a right operand (value heads): column block of [t x nh*32]
    wv = iota(t, nh * 32, dtype)
    dv = desc(LPG_PACKED_B, dtype, t, 32, parent=(t, nh * 32), batch=nh, batch_step=(0, 32))
    sv = desc(LPG_ROW_MAJOR, dtype, t, 32, parent=(t, nh * 32), batch=nh, batch_step=(0, 32))
    dst = dev_empty(api.lpg_packed_bytes(dv), fill=0xEE)
    api.lpg_pack(dev_bytes(wv), sv, dst, dv, stream())
    got = host(dst, NP_RAW[dtype])[:api.lpg_packed_bytes(dv) // es]
    assert np.array_equal(got, ref.pack(wv, False, es))


def test_empty_inputs_are_accepted():
    for rows, cols in ((0, 8), (8, 0)):
        sd = desc(LPG_ROW_MAJOR, LPG_F32, rows, cols)
        dd = desc(LPG_PACKED_A, LPG_F32, rows, cols)
        buf = dev_empty(64)
        assert api.lpg_pack(buf, sd, buf, dd, stream()) == 0
        assert api.lpg_unpack(buf, dd, buf, sd, stream()) == 0
    torch.cuda.synchronize()
