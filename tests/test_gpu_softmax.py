"""GPU parity of lpg_softmax_packed (scale, optional causal mask, row softmax on the packed
layout; Alg. 2) against the fp64 oracle, and of the attention chain that uses it.

Tolerance.  The kernel forms v = x * (scale*log2 e) in fp32 and evaluates 2^(v - max) with the
hardware exponential (about 1 ulp); rounding v costs |v| * 2^-24 relative in the result, and
|v - max| stays below ~40 for the inputs here, so one probability is off by at most a few
1e-6 relative; the fp32 row sum adds ~1e-6.  Acceptance: |got - want| <= 1e-5*want + 1e-12 per
element (fp32 out); bf16 out adds half an ulp of bf16, up to 2^-8 relative: 4e-3*want + 1e-12.
"""
import numpy as np
import pytest
import torch

from oracle import ref, workloads
from paper_2604_04599_amd import api, chains, inputs
from paper_2604_04599_amd.api import (LPG_BF16, LPG_CHAIN_CANONICAL, LPG_CHAIN_PROPAGATED, LPG_F32, LPG_PACKED_A,
                                      LPG_ROW_MAJOR, desc)
from gpu_util import ES, NP_RAW, bf16_raw_to_f64, dev_bytes, dev_empty, host, pack_dev, stream, unpack_dev

pytestmark = pytest.mark.gpu

REL = {LPG_F32: 1e-5, LPG_BF16: 4e-3}


def close(got, want, dtype):
    return np.all(np.abs(got - want) <= REL[dtype] * want + 1e-12)


# shapes chosen so that every kernel variant runs: rows kept in registers with 32, 16 or 8 rows
# per workgroup (fp32: cols <= 1024, 2048, 4096; bf16: twice that), and the streaming variant
SHAPES = [(1, 1), (33, 70), (70, 33), (100, 1000), (64, 1024), (70, 1500), (40, 3000), (33, 4200), (33, 8300)]


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("dtype", [LPG_F32, LPG_BF16])
@pytest.mark.parametrize("rows,cols", SHAPES)
def test_packed_softmax_matches_oracle(rows, cols, dtype, causal):
    rng = np.random.default_rng(rows * 10007 + cols)
    x = (rng.standard_normal((rows, cols)) * 3).astype(np.float32)
    px, d = pack_dev(x, LPG_PACKED_A, dtype)
    xin = unpack_dev(px, d)                                   # the values the kernel sees (bf16-rounded if bf16)
    out = dev_empty(api.lpg_packed_bytes(d), fill=0xA5)
    api.lpg_softmax_packed(px, out, d, 0.7, causal, stream())
    got = unpack_dev(out, d)
    want = ref.softmax_rows(xin, scale=0.7, causal=causal)
    assert close(got, want, dtype)
    if causal:
        shift = cols - rows
        i, j = np.indices((rows, cols))
        assert np.all(got[j > i + shift] == 0.0)              # masked positions are exactly zero
    # padding of the packed result is zero: no non-zero element outside the logical matrix
    raw = host(out, NP_RAW[dtype])
    assert np.count_nonzero(raw) == np.count_nonzero(got)
    # in place gives the same bytes
    api.lpg_softmax_packed(px, px, d, 0.7, causal, stream())
    assert np.array_equal(host(px, NP_RAW[dtype]), raw)


@pytest.mark.parametrize("dtype", [LPG_F32, LPG_BF16])
def test_packed_softmax_on_batched_views(dtype):
    """Three slots, each a 64 x KB-aligned view at a stepped origin inside one parent per slot."""
    kb = 32 if dtype == LPG_F32 else 64
    prow, pcol, rows, cols, nb = 160, 5 * kb, 64, 2 * kb, 3
    rng = np.random.default_rng(5)
    x = rng.standard_normal((nb, prow, pcol)).astype(np.float32)
    pe = ((prow + 31) // 32 * 32) * pcol
    whole = desc(LPG_PACKED_A, dtype, prow, pcol, batch=nb, batch_stride=pe)
    src = dev_bytes(x)
    px = dev_empty(api.lpg_packed_bytes(whole), fill=0)
    api.lpg_pack(src, desc(LPG_ROW_MAJOR, LPG_F32, prow, pcol, batch=nb, batch_stride=prow * pcol), px, whole, stream())
    before = unpack_dev(px, whole)
    view = desc(LPG_PACKED_A, dtype, rows, cols, parent=(prow, pcol), origin=(32, kb), batch=nb, batch_stride=pe,
                batch_step=(32, kb))
    api.lpg_softmax_packed(px, px, view, 1.0, True, stream())
    after = unpack_dev(px, whole)
    want = before.copy()
    for b in range(nb):
        r0, c0 = 32 + 32 * b, kb + kb * b
        want[b, r0:r0 + rows, c0:c0 + cols] = ref.softmax_rows(before[b, r0:r0 + rows, c0:c0 + cols], causal=True)
    outside = want == before
    assert np.array_equal(after[outside], before[outside])    # nothing outside the views is touched
    assert close(after[~outside], want[~outside], dtype)


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("dtype", [LPG_F32, LPG_BF16])
@pytest.mark.parametrize("rows,cols,ld", [(5, 7, 0), (33, 1000, 1003), (64, 4096, 0), (3, 9000, 9008)])
def test_row_major_softmax_matches_oracle(rows, cols, ld, dtype, causal):
    rng = np.random.default_rng(rows + cols)
    stride = ld or cols
    x = (rng.standard_normal((2, rows, stride)) * 2).astype(np.float32)
    if dtype == LPG_BF16:
        raw = ref.bf16_bits(x.view(np.uint32))
        xin = bf16_raw_to_f64(raw)
    else:
        raw = x.view(np.uint32)
        xin = x.astype(np.float64)
    d = desc(LPG_ROW_MAJOR, dtype, rows, cols, ld=ld, batch=2, batch_stride=rows * stride)
    src = dev_bytes(raw)
    out = dev_empty(raw.nbytes, fill=0xA5)
    api.lpg_softmax_packed(src, out, d, 1.3, causal, stream())
    got_raw = host(out, NP_RAW[dtype], raw.shape)
    got = bf16_raw_to_f64(got_raw) if dtype == LPG_BF16 else got_raw.view(np.float32).astype(np.float64)
    for b in range(2):
        want = ref.softmax_rows(xin[b, :, :cols], scale=1.3, causal=causal)
        assert close(got[b, :, :cols], want, dtype)
    fill = 0xA5A5 if dtype == LPG_BF16 else 0xA5A5A5A5
    assert np.all(got_raw[:, :, cols:] == fill)               # the gap between rows is left alone


def test_softmax_of_nothing_is_accepted():
    d = desc(LPG_PACKED_A, LPG_F32, 0, 64)
    buf = dev_empty(16)
    api.lpg_softmax_packed(buf, buf, d, 1.0, False, stream())
    d = desc(LPG_ROW_MAJOR, LPG_F32, 8, 0)
    api.lpg_softmax_packed(buf, buf, d, 1.0, False, stream())
    torch.cuda.synchronize()


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("fused", [False, True])
def test_attention_chain_with_softmax(causal, fused):
    inp, shape = inputs.make("attention", heads=3, t=160, dh=64)
    ch = chains.build("attention", inp, shape, fused=fused, softmax=True, causal=causal)
    ch.run(LPG_CHAIN_PROPAGATED)
    prop = ch.output("O").copy()
    p = ch.fetch("S")
    ch.outputs["O"].fill_(float("nan"))
    ch.run(LPG_CHAIN_CANONICAL)
    canon = ch.output("O").copy()
    want = workloads.attention(inp, softmax=True, causal=causal, keep_s=True)
    for h in range(shape["heads"]):
        assert close(p[h], want["S"][h], LPG_F32) or ref.rel_frobenius(p[h], want["S"][h]) <= 2e-5
        assert ref.rel_frobenius(prop[h], ref.gemm(p[h], inp["V"][h])) <= 1e-5      # stage-local
        assert ref.rel_frobenius(prop[h], want["O"][h]) <= 3e-5                      # end-to-end, three stages
        # the control runs the row-major softmax kernel: same values up to summation order
        assert ref.rel_frobenius(canon[h], want["O"][h]) <= 3e-5


@pytest.mark.parametrize("blocks", [2, 6])
def test_attention_chain_in_causal_row_blocks(blocks):
    """The three stages per block of query rows, on views that end at the causal diagonal: the
    oracle's O in both modes, the oracle's probabilities inside the blocks, and nothing written
    above the block diagonal."""
    inp, shape = inputs.make("attention", heads=3, t=192, dh=64)
    ch = chains.build("attention", inp, shape, softmax=True, causal=True, causal_blocks=blocks)
    ch.bufs["S"][0].view(torch.float32).fill_(-77.0)
    ch.run(LPG_CHAIN_PROPAGATED)
    prop = ch.output("O").copy()
    p = ch.fetch("S")
    ch.outputs["O"].fill_(float("nan"))
    ch.run(LPG_CHAIN_CANONICAL)
    canon = ch.output("O").copy()
    want = workloads.attention(inp, softmax=True, causal=True, keep_s=True)
    rb = shape["t"] // blocks
    for h in range(shape["heads"]):
        for i in range(blocks):
            r, kc = slice(i * rb, (i + 1) * rb), (i + 1) * rb
            assert ref.rel_frobenius(p[h][r, :kc], want["S"][h][r, :kc]) <= 2e-5
            assert np.all(p[h][r, kc:] == -77.0)
        assert ref.rel_frobenius(prop[h], want["O"][h]) <= 3e-5
        assert ref.rel_frobenius(canon[h], want["O"][h]) <= 3e-5


@pytest.mark.parametrize("blocks", [1, 4])
def test_attention_chain_with_softmax_full_size_sampled_heads(blocks):
    inp, shape = inputs.make("attention")
    ch = chains.build("attention", inp, shape, softmax=True, causal=True, causal_blocks=blocks)
    ch.run(LPG_CHAIN_PROPAGATED)
    prop = ch.output("O").copy()
    heads = [0, 17, 31]
    want = workloads.attention(inp, heads=heads, softmax=True, causal=True)
    for h in heads:
        assert ref.rel_frobenius(prop[h], want["O"][h]) <= 3e-5
