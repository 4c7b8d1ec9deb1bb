"""GPU parity: a seeded random sweep of lpg_pack / lpg_unpack over shapes (biased towards the 32 / KB
edges), dtypes (with the fp32 -> bf16 conversion), operand roles, canonical orders and leading
dimensions, batches in one or in separate parents, and destination views (none, on the grid, off the
grid).  The packed buffer must equal the oracle's pack of the updated parent, bit for bit."""
import numpy as np
import pytest

from oracle import ref
from paper_2604_04599_amd import api
from paper_2604_04599_amd.api import LPG_BF16, LPG_COL_MAJOR, LPG_F32, LPG_PACKED_A, LPG_PACKED_B, LPG_ROW_MAJOR, desc
from tests.gpu_util import ES, NP_RAW, dev_bytes, dev_empty, host, stream

pytestmark = pytest.mark.gpu

EDGES = [1, 2, 7, 31, 32, 33, 63, 64, 65, 96, 127, 128, 129, 200, 257]


def bits(rng, shape, dtype):
    """Random finite values as raw bit patterns of `dtype`."""
    x = rng.standard_normal(shape).astype(np.float32)
    return x.view(np.uint32).copy() if dtype == LPG_F32 else ref.bf16_bits(x.view(np.uint32))


@pytest.mark.parametrize("seed", range(80))
def test_random_pack_case(seed):
    rng = np.random.default_rng(70000 + seed)
    dim = lambda: int(rng.choice(EDGES)) if rng.random() < 0.7 else int(rng.integers(1, 300))
    p_dt = LPG_BF16 if rng.random() < 0.5 else LPG_F32
    c_dt = LPG_F32 if (p_dt == LPG_F32 or rng.random() < 0.4) else LPG_BF16     # f32 -> bf16 converts
    kind = LPG_PACKED_A if rng.random() < 0.5 else LPG_PACKED_B
    src_kind = LPG_ROW_MAJOR if rng.random() < 0.5 else LPG_COL_MAJOR
    rows, cols = dim(), dim()
    nb = int(rng.choice([1, 1, 2, 3]))
    view = str(rng.choice(["none", "grid", "offgrid"]))
    a_side = kind == LPG_PACKED_A
    es, ces = ES[p_dt], ES[c_dt]
    kbo = ref.layout_consts(es)[2]
    fg, kg = (32, kbo) if a_side else (kbo, 32)
    if view == "none":
        prow, pcol, r0, c0 = rows, cols, 0, 0
    else:
        if view == "grid":
            r0, c0 = fg * int(rng.integers(0, 3)), kg * int(rng.integers(0, 3))
        else:
            r0, c0 = int(rng.integers(1, 70)), int(rng.integers(1, 70))
        prow, pcol = r0 + rows + int(rng.integers(0, 40)), c0 + cols + int(rng.integers(0, 40))
    # canonical source: nb matrices, each with its own leading dimension padding
    rm = src_kind == LPG_ROW_MAJOR
    ld = (cols if rm else rows) + int(rng.integers(0, 6))
    outer = rows if rm else cols
    pieces = [bits(rng, (rows, cols), c_dt) for _ in range(nb)]
    canon = np.zeros((nb, outer, ld), dtype=NP_RAW[c_dt])
    for b in range(nb):
        src = pieces[b] if rm else pieces[b].T
        canon[b, :, :src.shape[1]] = src
    sd = desc(src_kind, c_dt, rows, cols, ld=ld, batch=nb, batch_stride=outer * ld if nb > 1 else 0)
    # packed destination: one parent per slot
    pelems = ref.packed_elems(prow if a_side else pcol, pcol if a_side else prow, es)
    befores = [bits(rng, (prow, pcol), p_dt) for _ in range(nb)]
    pbuf = np.concatenate([ref.pack(b_, a_side, es) for b_ in befores])
    dd = desc(kind, p_dt, rows, cols, parent=(prow, pcol), origin=(r0, c0), batch=nb,
              batch_stride=pelems if nb > 1 else 0)
    dst = dev_bytes(pbuf)
    api.lpg_pack(dev_bytes(canon), sd, dst, dd, stream())
    got = host(dst, NP_RAW[p_dt])
    want = []
    for b in range(nb):
        piece = pieces[b]
        if c_dt != p_dt:
            piece = ref.bf16_bits(piece)            # fp32 bits -> bf16 bits, round to nearest even
        after = befores[b].copy()
        after[r0:r0 + rows, c0:c0 + cols] = piece
        want.append(ref.pack(after, a_side, es))
    want = np.concatenate(want)
    assert np.array_equal(got[:want.size], want), (seed, view, kind, src_kind, rows, cols, nb)
    # and back: the views alone, into a poisoned canonical buffer of the packed dtype
    back_ld = (cols if rm else rows) + 2
    back = dev_empty(nb * outer * back_ld * es, fill=0x3C)
    bd = desc(src_kind, p_dt, rows, cols, ld=back_ld, batch=nb, batch_stride=outer * back_ld if nb > 1 else 0)
    api.lpg_unpack(dst, dd, back, bd, stream())
    barr = host(back, NP_RAW[p_dt])[:nb * outer * back_ld].reshape(nb, outer, back_ld)
    poison = NP_RAW[p_dt](0x3C3C if es == 2 else 0x3C3C3C3C)
    for b in range(nb):
        piece = pieces[b] if c_dt == p_dt else ref.bf16_bits(pieces[b])
        inner = barr[b][:, :(cols if rm else rows)]
        assert np.array_equal(inner if rm else inner.T, piece)
        assert np.all(barr[b][:, (cols if rm else rows):] == poison)
