"""Pins for the oracle's packed layout P(X; F, K) and its pack/unpack.

The layout is this build's own (the paper fixes only a dimension order for its
CPU tiles, Eq. 3), so the pins are structural: hand-derived offsets, agreement of
a closed-form index with the loop-nest walk, bijectivity, zero padding, the
left/right-operand transpose equivalence, sub-views, round trips, and the two
register-image properties the MFMA kernels rely on.
"""
import numpy as np
import pytest

from oracle import ref

DT = {4: np.uint32, 2: np.uint16}


def iota(rows, cols, es, start=1):
    return (np.arange(rows * cols, dtype=np.int64) + start).astype(DT[es]).reshape(rows, cols)


def test_hand_derived_offsets_fp32():
    # F=64, K=64: Fp=64, KB=32, fragment = 32 f x 8 k = 256 elements, block = 1024
    PF = 64
    cases = {(0, 0): 0, (0, 1): 1, (0, 3): 3, (0, 4): 128, (0, 7): 131, (1, 0): 4, (31, 3): 127,
             (31, 7): 255, (0, 8): 256, (5, 13): 256 + 128 + 5 * 4 + 1, (0, 31): 3 * 256 + 128 + 3,
             (32, 0): 1024, (33, 9): 1024 + 256 + 4 + 1, (0, 32): 64 * 32, (63, 63): 64 * 64 - 1}
    for (f, k), want in cases.items():
        assert int(ref.packed_offset(f, k, PF, 4)) == want, (f, k)


def test_hand_derived_offsets_bf16():
    # F=64, K=128: KV=8, fragment = 32 f x 16 k = 512 elements, KB=64, block = 2048
    PF = 64
    cases = {(0, 0): 0, (0, 3): 3, (0, 4): 256, (0, 7): 259, (0, 8): 4, (0, 11): 7, (0, 12): 260,
             (0, 15): 263, (1, 0): 8, (31, 15): 511, (0, 16): 512, (0, 63): 3 * 512 + 263,
             (32, 0): 2048, (0, 64): 64 * 64, (63, 127): 64 * 128 - 1}
    for (f, k), want in cases.items():
        assert int(ref.packed_offset(f, k, PF, 2)) == want, (f, k)


@pytest.mark.parametrize("es", [4, 2])
@pytest.mark.parametrize("F,K", [(1, 1), (32, 32), (33, 65), (70, 200), (128, 64), (5, 130)])
def test_closed_form_equals_loop_nest_and_is_bijective(es, F, K):
    a = iota(F, K, es)
    packed = ref.pack(a, True, es)
    fp, kp = ref.padded_extents(F, K, es)
    assert packed.size == fp * kp
    ff, kk = np.meshgrid(np.arange(F), np.arange(K), indexing="ij")
    off = ref.packed_offset(ff, kk, F, es)
    assert np.array_equal(packed[off], a)                      # same place, two derivations
    # all padded positions: a permutation of 0..N-1
    ffp, kkp = np.meshgrid(np.arange(fp), np.arange(kp), indexing="ij")
    allo = ref.packed_offset(ffp, kkp, F, es).ravel()
    assert np.array_equal(np.sort(allo), np.arange(fp * kp))
    # padding is zero, logical elements are all there
    mask = np.ones(fp * kp, dtype=bool)
    mask[off.ravel()] = False
    assert not packed[mask].any()
    assert np.array_equal(np.sort(packed[~mask]), np.sort(a.ravel()))


@pytest.mark.parametrize("es", [4, 2])
def test_round_trip_and_transpose_equivalence(es):
    a = iota(45, 77, es)
    for free_is_rows in (True, False):
        p = ref.pack(a, free_is_rows, es)
        assert np.array_equal(ref.unpack(p, 45, 77, free_is_rows, es), a)
    # left-operand image of X == right-operand image of X^T, byte for byte
    pa = ref.pack(a, True, es)
    pbt = ref.pack(np.ascontiguousarray(a.T), False, es)
    assert np.array_equal(pa, pbt)


@pytest.mark.parametrize("es", [4, 2])
def test_sub_view_equals_slice_of_whole(es):
    kb = ref.layout_consts(es)[2]
    PF, PK = 96, 3 * kb
    whole = iota(PF, PK, es)
    packed_whole = ref.pack(whole, True, es)
    # build the same parent from four views
    buf = np.zeros_like(packed_whole)
    for f0, F in ((0, 32), (32, 64)):
        for k0, K in ((0, kb), (kb, 2 * kb)):
            ref.pack(whole[f0:f0 + F, k0:k0 + K], True, es, parent=(PF, PK), origin=(f0, k0), out=buf)
    assert np.array_equal(buf, packed_whole)
    got = ref.unpack(packed_whole, 64, kb, True, es, parent=(PF, PK), origin=(32, kb))
    assert np.array_equal(got, whole[32:96, kb:2 * kb])
    # a column block of the k range is one contiguous run of the parent
    fp = ref.padded_extents(PF, PK, es)[0]
    alone = ref.pack(whole[:, kb:2 * kb], True, es)
    assert np.array_equal(packed_whole[fp * kb:2 * fp * kb], alone)


@pytest.mark.parametrize("es", [4, 2])
def test_fragment_is_one_wave_load(es):
    """Lane l of a 64-lane wave reading 16 bytes at fragment_base + 16*l receives
    free index l%32 and the k values {8*(v/4) + 4*(l/32) + v%4}."""
    kv, kf, kb = ref.layout_consts(es)
    for c in range(4):
        for lane in range(64):
            for v in range(kv):
                f, k = lane % 32, kf * c + 8 * (v // 4) + 4 * (lane // 32) + v % 4
                assert int(ref.packed_offset(f, k, 32, es)) == c * 64 * kv + lane * kv + v


def test_accumulator_tile_is_already_packed_fp32():
    """A 32x32 accumulator tile held as: lane l, register r <-> (i = 8*(r/4) + 4*(l/32) + r%4,
    j = l%32).  Read as P(D; free=j, K=i), registers 4q..4q+3 of lane l are the 16
    contiguous bytes at fragment q, lane l."""
    for lane in range(64):
        for r in range(16):
            i, j = 8 * (r // 4) + 4 * (lane // 32) + r % 4, lane % 32
            assert int(ref.packed_offset(j, i, 32, 4)) == (r // 4) * 256 + lane * 4 + r % 4


def test_accumulator_tile_is_already_packed_bf16():
    """Same tile stored as bf16: registers 8p..8p+7 of lane l (converted) are the 16
    contiguous bytes at fragment p (p = 0, 1), lane l."""
    for lane in range(64):
        for r in range(16):
            i, j = 8 * (r // 4) + 4 * (lane // 32) + r % 4, lane % 32
            assert int(ref.packed_offset(j, i, 32, 2)) == (r // 8) * 512 + lane * 8 + r % 8


def test_ragged_view_padding_is_zero():
    a = iota(40, 50, 4)
    buf = np.full(ref.packed_elems(40, 50, 4), 0xFFFFFFFF, dtype=np.uint32)
    ref.pack(a, True, 4, out=buf)
    ff, kk = np.meshgrid(np.arange(40), np.arange(50), indexing="ij")
    off = ref.packed_offset(ff, kk, 40, 4).ravel()
    mask = np.ones(buf.size, dtype=bool)
    mask[off] = False
    assert not buf[mask].any()


@pytest.mark.parametrize("es", [4, 2])
def test_block_order_is_a_permutation_of_blocks_and_store_stride_leaves_room(es):
    """Section III-C's two parameters on the oracle's pack: with groups outermost the buffer is the
    default buffer with its block grid transposed (numpy reshape / transpose of whole 4 KiB blocks,
    nothing of the layout's inner order involved); with room between blocks every block sits at
    kb * ks + g * gs and the room keeps what it held; the closed form agrees; unpack inverts both."""
    kv, kf, kb = ref.layout_consts(es)
    dt = {4: np.uint32, 2: np.uint16}[es]
    F, K = 70, 2 * kb + 9                       # 3 groups, 3 K blocks
    ng, nk, blk = 3, 3, 32 * kb
    x = (np.arange(F * K, dtype=np.uint64) * 2654435761 % (1 << (8 * es))).astype(dt).reshape(F, K)
    base = ref.pack(x, True, es)
    assert base.size == ng * nk * blk
    # groups outermost
    got = ref.pack(x, True, es, group_stride=nk * blk, kblock_stride=blk)
    assert np.array_equal(got, base.reshape(nk, ng, blk).transpose(1, 0, 2).reshape(-1))
    assert np.array_equal(ref.unpack(got, F, K, True, es, group_stride=nk * blk, kblock_stride=blk), x)
    # room after every block and after every K block
    gs, ks = 2 * blk, 7 * blk
    poison = np.full(ref.strided_elems(F, K, es, gs, ks), 0xABCD, dtype=dt)
    got = ref.pack(x, True, es, out=poison.copy(), group_stride=gs, kblock_stride=ks)
    touched = np.zeros(got.size, dtype=bool)
    for kbi in range(nk):
        for g in range(ng):
            at = kbi * ks + g * gs
            assert np.array_equal(got[at:at + blk], base[(kbi * ng + g) * blk:(kbi * ng + g + 1) * blk])
            touched[at:at + blk] = True
    assert np.all(got[~touched] == 0xABCD)
    assert np.array_equal(ref.unpack(got, F, K, True, es, group_stride=gs, kblock_stride=ks), x)
    f, k = np.meshgrid(np.arange(F), np.arange(K), indexing="ij")
    assert np.array_equal(got[ref.packed_offset(f, k, F, es, gs, ks)], x)
    # a right operand under the same strides: the bytes of the transposed left operand
    assert np.array_equal(ref.pack(np.ascontiguousarray(x.T), False, es, out=poison.copy(), group_stride=gs, kblock_stride=ks), got)
