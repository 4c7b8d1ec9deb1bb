"""CPU-only checks of the C-ABI library: it loads, exports every declared symbol,
its host index function equals the oracle's closed form, and descriptor errors are
caught on the host (no compute call is made here)."""
import ctypes
import os
import re
import subprocess

import numpy as np
import pytest

from oracle import ref
from paper_2604_04599_amd import api
from paper_2604_04599_amd.api import (LPG_BF16, LPG_COL_MAJOR, LPG_F32, LPG_PACKED_A, LPG_PACKED_B,
                                      LPG_ROW_MAJOR, desc)

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "lpg.h")).read()
    declared = set(re.findall(r"\b(lpg_[a-z0-9_]+)\s*\(", header))
    assert {"lpg_pack", "lpg_unpack", "lpg_gemm_packed", "lpg_elementwise_packed", "lpg_chain"} <= declared
    L = api.lib()
    for name in declared:
        assert hasattr(L, name), name
    assert set(api.EXPORTS) == declared
    assert "gfx950" in api.lpg_version()


def test_struct_layouts_match_header(tmp_path):
    """The ctypes mirrors against what a C compiler makes of include/lpg.h: sizes and the
    offset of every field."""
    # lpg_desc: 2 int32 + 7 int64 + 2 int32 + 5 int64
    assert ctypes.sizeof(api.lpg_desc) == 8 + 7 * 8 + 8 + 5 * 8
    fields = {"lpg_desc": [n for n, _ in api.lpg_desc._fields_], "lpg_stage": [n for n, _ in api.lpg_stage._fields_]}
    src = ['#include <stdio.h>', '#include <stddef.h>', '#include "lpg.h"', 'int main(void) {']
    for st, names in fields.items():
        src.append(f'printf("{st} %zu\\n", sizeof({st}));')
        for n in names:
            src.append(f'printf("{st}.{n} %zu\\n", offsetof({st}, {n}));')
    src += ['return 0; }']
    c = tmp_path / "layout.c"
    c.write_text("\n".join(src))
    exe = tmp_path / "layout"
    subprocess.run(["gcc", "-I", os.path.join(ROOT, "include"), str(c), "-o", str(exe)], check=True)
    got = dict(line.split() for line in subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.splitlines())
    for st, cls in (("lpg_desc", api.lpg_desc), ("lpg_stage", api.lpg_stage)):
        assert int(got[st]) == ctypes.sizeof(cls)
        for n in fields[st]:
            assert int(got[f"{st}.{n}"]) == getattr(cls, n).offset, (st, n)


@pytest.mark.parametrize("dtype,es", [(LPG_F32, 4), (LPG_BF16, 2)])
@pytest.mark.parametrize("rows,cols", [(1, 1), (33, 65), (70, 200), (128, 64)])
def test_layout_offset_matches_oracle_closed_form(dtype, es, rows, cols):
    da = desc(LPG_PACKED_A, dtype, rows, cols)
    db = desc(LPG_PACKED_B, dtype, rows, cols)
    fp, kp = ref.padded_extents(rows, cols, es)
    assert api.lpg_packed_bytes(da) == fp * kp * es
    fpb, kpb = ref.padded_extents(cols, rows, es)
    assert api.lpg_packed_bytes(db) == fpb * kpb * es
    rng = np.random.default_rng(1)
    for _ in range(200):
        r, c = int(rng.integers(rows)), int(rng.integers(cols))
        assert api.lpg_layout_offset(da, 0, r, c) == int(ref.packed_offset(r, c, rows, es))
        assert api.lpg_layout_offset(db, 0, r, c) == int(ref.packed_offset(c, r, cols, es))


def test_layout_offset_views_and_batches():
    es, kb = 2, 64
    parent = (96, 4 * kb)
    d = desc(LPG_PACKED_A, LPG_BF16, 96, kb, parent=parent, batch=4, batch_step=(0, kb))
    for b in range(4):
        for (r, c) in [(0, 0), (95, kb - 1), (40, 17)]:
            want = int(ref.packed_offset(r, b * kb + c, 96, es))
            assert api.lpg_layout_offset(d, b, r, c) == want
    # separate parents per slot, two matrices per slot
    one = ref.packed_elems(64, 64, 4)
    d2 = desc(LPG_PACKED_B, LPG_F32, 64, 64, batch=6, batch_div=2, batch_stride=one)
    assert api.lpg_layout_offset(d2, 5, 3, 7) == 2 * one + int(ref.packed_offset(7, 3, 64, 4))
    assert api.lpg_packed_bytes(d2) == 3 * one * 4
    # canonical
    rm = desc(LPG_ROW_MAJOR, LPG_F32, 10, 20, ld=32)
    cm = desc(LPG_COL_MAJOR, LPG_F32, 10, 20, ld=16)
    assert api.lpg_layout_offset(rm, 0, 3, 5) == 3 * 32 + 5
    assert api.lpg_layout_offset(cm, 0, 3, 5) == 3 + 5 * 16


def _err(fn, *a, **k):
    with pytest.raises(api.LpgError) as e:
        fn(*a, **k)
    return e.value.code


def test_descriptor_errors_are_caught_on_the_host():
    fake = 4096          # never dereferenced: every call below fails validation first
    pa = desc(LPG_PACKED_A, LPG_F32, 64, 64)
    pb = desc(LPG_PACKED_B, LPG_F32, 64, 64)
    rm = desc(LPG_ROW_MAJOR, LPG_F32, 64, 64)
    assert _err(api.lpg_pack, fake, pa, fake, pa) == api.LPG_ELAYOUT            # src must be canonical
    assert _err(api.lpg_pack, fake, rm, fake, rm) == api.LPG_ELAYOUT            # dst must be packed
    assert _err(api.lpg_pack, fake, desc(LPG_ROW_MAJOR, LPG_F32, 64, 32), fake, pa) == api.LPG_EINVAL
    assert _err(api.lpg_pack, fake, rm, fake + 4, pa) == api.LPG_EALIGN
    assert _err(api.lpg_pack, fake, desc(LPG_ROW_MAJOR, LPG_BF16, 64, 64), fake, pa) == api.LPG_EUNSUPPORTED
    assert _err(api.lpg_unpack, fake, desc(LPG_PACKED_A, LPG_F32, 64, 64), fake,
                desc(LPG_ROW_MAJOR, LPG_BF16, 64, 64)) == api.LPG_EUNSUPPORTED
    # GEMM: roles, inner dimension, dtype, beta without C, aliasing
    assert _err(api.lpg_gemm_packed, 1.0, fake, pb, fake, pb, 0.0, None, 2 * fake, pa) == api.LPG_ELAYOUT
    assert _err(api.lpg_gemm_packed, 1.0, fake, pa, fake, pa, 0.0, None, 2 * fake, pa) == api.LPG_ELAYOUT
    assert _err(api.lpg_gemm_packed, 1.0, fake, pa, fake, desc(LPG_PACKED_B, LPG_F32, 32, 64), 0.0, None,
                2 * fake, pa) == api.LPG_EINVAL
    assert _err(api.lpg_gemm_packed, 1.0, fake, pa, fake, pb, 0.0, None, 2 * fake,
                desc(LPG_PACKED_A, LPG_BF16, 64, 64)) == api.LPG_EUNSUPPORTED
    assert _err(api.lpg_gemm_packed, 1.0, fake, pa, fake, pb, 1.0, None, 2 * fake, pa) == api.LPG_EINVAL
    assert _err(api.lpg_gemm_packed, 1.0, fake, pa, 2 * fake, pb, 0.0, None, fake, pa) == api.LPG_EINVAL
    # views: the row, elementwise and attention entry points and stepped batches need origins on the
    # 32 / KB grid; a product takes any view of a packed parent as an input (checked below without a launch)
    bad = desc(LPG_PACKED_A, LPG_F32, 32, 64, parent=(64, 64), origin=(16, 0))
    assert _err(api.lpg_softmax_packed, fake, fake, bad, 1.0, False) == api.LPG_EALIGN
    assert _err(api.lpg_pack, fake, desc(LPG_ROW_MAJOR, LPG_F32, 32, 32, batch=2, batch_stride=1024), fake,
                desc(LPG_PACKED_A, LPG_F32, 32, 32, parent=(128, 64), origin=(8, 0), batch=2, batch_step=(40, 0))) == api.LPG_EALIGN
    inner_f = desc(LPG_PACKED_A, LPG_F32, 20, 32, parent=(64, 64), origin=(0, 0))
    assert _err(api.lpg_softmax_packed, fake, fake, inner_f, 1.0, False) == api.LPG_EALIGN
    assert _err(api.lpg_rmsnorm_packed, fake, fake, fake, inner_f, 1e-5) == api.LPG_EALIGN
    stepped = desc(LPG_PACKED_A, LPG_F32, 20, 32, parent=(64, 64), batch=2, batch_step=(32, 0))
    assert _err(api.lpg_pack, fake, desc(LPG_ROW_MAJOR, LPG_F32, 20, 32, batch=2, batch_stride=640), fake,
                stepped) == api.LPG_EALIGN
    bad = desc(LPG_PACKED_A, LPG_F32, 64, 64, parent=(64, 64), origin=(32, 0))
    assert _err(api.lpg_pack, fake, rm, fake, bad) == api.LPG_EINVAL
    assert "exceeds" in api.lpg_last_error()
    # elementwise: op range, sub-views
    assert _err(api.lpg_elementwise_packed, 9, fake, fake, 1.0, fake, pa) == api.LPG_EINVAL
    v = desc(LPG_PACKED_A, LPG_F32, 32, 32, parent=(64, 64))
    assert _err(api.lpg_elementwise_packed, api.LPG_EW_ADD, fake, fake, 1.0, fake, v) == api.LPG_EUNSUPPORTED
    # softmax: rows must be the free index, one slot per matrix, aligned packed buffers
    assert _err(api.lpg_softmax_packed, fake, fake, pb, 1.0, False) == api.LPG_EUNSUPPORTED
    assert _err(api.lpg_softmax_packed, fake, fake, desc(api.LPG_COL_MAJOR, LPG_F32, 64, 64), 1.0, False) == api.LPG_EUNSUPPORTED
    assert _err(api.lpg_softmax_packed, fake, fake, desc(LPG_PACKED_A, LPG_F32, 64, 64, batch=4, batch_div=2),
                1.0, False) == api.LPG_EUNSUPPORTED
    assert _err(api.lpg_softmax_packed, None, fake, pa, 1.0, False) == api.LPG_EINVAL
    assert _err(api.lpg_softmax_packed, fake, fake + 8, pa, 1.0, False) == api.LPG_EALIGN
    assert _err(api.lpg_softmax_packed, fake, fake, desc(LPG_PACKED_A, LPG_F32, 32, 32, parent=(64, 64), origin=(0, 16)),
                1.0, False) == api.LPG_EALIGN
    assert _err(api.lpg_softmax_packed, fake, fake, pa, 0.0, False) == api.LPG_EINVAL          # scale must be > 0
    assert _err(api.lpg_softmax_packed, fake, fake, pa, float("inf"), False) == api.LPG_EINVAL
    # RMS normalisation and RoPE share the softmax's descriptor rules and add their own
    assert _err(api.lpg_rmsnorm_packed, fake, None, fake, pa, 1e-5) == api.LPG_EINVAL           # no weight
    assert _err(api.lpg_rmsnorm_packed, fake, fake, fake, pa, -1.0) == api.LPG_EINVAL
    assert _err(api.lpg_rmsnorm_packed, fake, fake, fake, pb, 1e-5) == api.LPG_EUNSUPPORTED
    assert _err(api.lpg_rope_packed, fake, fake, pa, fake, fake, 48) == api.LPG_EINVAL          # 64 cols, head_dim 48
    assert _err(api.lpg_rope_packed, fake, fake, pa, fake, fake, 8) == api.LPG_EUNSUPPORTED     # halves < one fragment
    assert _err(api.lpg_rope_packed, fake, fake, desc(LPG_PACKED_A, LPG_BF16, 64, 64), fake, fake, 16) == api.LPG_EUNSUPPORTED
    assert _err(api.lpg_rope_packed, fake, fake, pa, fake + 4, fake, 16) == api.LPG_EALIGN
    assert _err(api.lpg_rope_packed, fake, fake, pa, None, fake, 16) == api.LPG_EINVAL
    assert _err(api.lpg_rope_packed, fake, fake, pa, fake, fake, 15) == api.LPG_EINVAL
    assert _err(api.lpg_rope_tables, fake, fake, 8, 7, 10000.0, 0) == api.LPG_EINVAL
    assert _err(api.lpg_rope_tables, fake, fake, 8, 8, -1.0, 0) == api.LPG_EINVAL
    assert _err(api.lpg_rope_tables, None, fake, 8, 8, 10000.0, 0) == api.LPG_EINVAL
    # a batch the pack kernel's grid cannot hold is reported, not narrowed
    many = 70000
    assert _err(api.lpg_pack, fake, desc(LPG_ROW_MAJOR, LPG_F32, 32, 32, batch=many, batch_stride=1024), fake,
                desc(LPG_PACKED_A, LPG_F32, 32, 32, batch=many, batch_stride=1024)) == api.LPG_EUNSUPPORTED
    # fused attention: roles, head_dim, shapes, dtype, aliasing
    qd, kd, vd = desc(LPG_PACKED_A, LPG_F32, 96, 64), desc(LPG_PACKED_A, LPG_F32, 80, 64), desc(LPG_PACKED_B, LPG_F32, 80, 64)
    od = desc(LPG_PACKED_A, LPG_F32, 96, 64)
    q, k, v, o = fake, 2 * fake, 3 * fake, 4 * fake
    assert _err(api.lpg_attention_packed, q, desc(LPG_PACKED_B, LPG_F32, 96, 64), k, kd, v, vd, o, od, 1.0) == api.LPG_ELAYOUT
    assert _err(api.lpg_attention_packed, q, desc(LPG_PACKED_A, LPG_F32, 96, 32), k, desc(LPG_PACKED_A, LPG_F32, 80, 32), v,
                desc(LPG_PACKED_B, LPG_F32, 80, 32), o, desc(LPG_PACKED_A, LPG_F32, 96, 32), 1.0) == api.LPG_EUNSUPPORTED
    assert _err(api.lpg_attention_packed, q, qd, k, kd, v, desc(LPG_PACKED_B, LPG_F32, 64, 64), o, od, 1.0) == api.LPG_EINVAL
    assert _err(api.lpg_attention_packed, q, qd, k, kd, v, desc(LPG_PACKED_A, LPG_F32, 80, 64), o, od, 1.0) == api.LPG_EINVAL
    assert _err(api.lpg_attention_packed, q, qd, k, desc(LPG_PACKED_A, LPG_BF16, 80, 64), v, vd, o, od, 1.0) == api.LPG_EUNSUPPORTED
    assert _err(api.lpg_attention_packed, q, qd, k, kd, v, vd, q, od, 1.0) == api.LPG_EINVAL
    assert _err(api.lpg_attention_packed, q, qd, k, kd, v, vd, o, od, -1.0) == api.LPG_EINVAL
    assert api.lib().lpg_attention_packed(q, ctypes.byref(qd), k, ctypes.byref(kd), v, ctypes.byref(vd), o,
                                          ctypes.byref(od), 1.0, 4, None) == api.LPG_EINVAL   # unknown flag bit
    assert _err(api.lpg_attention_packed, q, qd, k, kd, v, vd, o, desc(LPG_PACKED_A, LPG_F32, 96, 64, batch=2), 1.0) == api.LPG_EINVAL


def test_chain_link_check_and_workspace():
    fake = 1 << 20
    a_d = desc(LPG_PACKED_A, LPG_F32, 64, 64)
    b_d = desc(LPG_PACKED_B, LPG_F32, 64, 64)
    rm = desc(LPG_ROW_MAJOR, LPG_F32, 64, 64)
    x, w1, w2, c1, c2, y, src = (fake * i for i in range(1, 8))
    stages = [api.stage_pack(src, rm, x, a_d),
              api.stage_gemm(1.0, x, a_d, w1, b_d, 0.0, None, c1, a_d),
              api.stage_gemm(1.0, c1, a_d, w2, b_d, 0.0, None, c2, a_d),
              api.stage_unpack(c2, a_d, y, rm)]
    assert api.lpg_chain_workspace_bytes(stages, api.LPG_CHAIN_PROPAGATED) == 0
    # only C1 crosses a GEMM->GEMM boundary: one 64x64 fp32 row-major copy
    assert api.lpg_chain_workspace_bytes(stages, api.LPG_CHAIN_CANONICAL) == 64 * 64 * 4
    # a softmax between the GEMMs runs in place on that same copy: no extra workspace
    with_sm = stages[:2] + [api.stage_softmax(c1, c1, a_d, 0.5, True)] + stages[2:]
    assert api.lpg_chain_workspace_bytes(with_sm, api.LPG_CHAIN_CANONICAL) == 64 * 64 * 4
    with_sm[2] = api.stage_softmax(c1, c1, desc(LPG_PACKED_A, LPG_F32, 64, 64, parent=(128, 64)), 0.5, True)
    with pytest.raises(api.LpgError) as e:
        api.lpg_chain(with_sm, api.LPG_CHAIN_PROPAGATED)
    assert e.value.code == api.LPG_ELAYOUT
    # consumer reads C1 with another geometry -> layout error before any launch
    wrong = desc(LPG_PACKED_A, LPG_F32, 64, 64, parent=(128, 64))
    stages[2] = api.stage_gemm(1.0, c1, wrong, w2, b_d, 0.0, None, c2, desc(LPG_PACKED_A, LPG_F32, 64, 64))
    with pytest.raises(api.LpgError) as e:
        api.lpg_chain(stages, api.LPG_CHAIN_PROPAGATED)
    assert e.value.code == api.LPG_ELAYOUT
    # transposed reading of the same bytes is accepted by the link check (fails later only
    # because canonical mode gets no workspace here)
    stages[2] = api.stage_gemm(1.0, w2, a_d, c1, b_d, 0.0, None, c2, b_d)
    with pytest.raises(api.LpgError) as e:
        api.lpg_chain(stages, api.LPG_CHAIN_CANONICAL, None, 0)
    assert e.value.code == api.LPG_EWORKSPACE


def test_tune_hooks_round_trip_and_reject_unknown_keys():
    for key in range(8):
        assert api.lpg_tune_get(key) == api.LPG_TUNE_AUTO
    api.lpg_tune_set(api.LPG_TUNE_TILE, 3)
    assert api.lpg_tune_get(api.LPG_TUNE_TILE) == 3
    api.lpg_tune_set(api.LPG_TUNE_TILE, api.LPG_TUNE_AUTO)
    assert api.lpg_tune_get(api.LPG_TUNE_TILE) == api.LPG_TUNE_AUTO
    for bad in (-1, 8, 100):
        with pytest.raises(api.LpgError) as e:
            api.lpg_tune_set(bad, 1)
        assert e.value.code == api.LPG_EINVAL


def test_control_chain_of_odd_sizes_is_validated_before_launch():
    """GEMM -> SCALE -> GEMM on 33 x 35 fp32: the control runs the elementwise stage on a tight
    row-major copy whose size is not a multiple of 16 bytes.  The dry pass that sizes the workspace
    validates that stage as well (fake, never dereferenced addresses), and accepts it."""
    m, k, n = 33, 35, 35
    a_d, b_d, c_d = desc(LPG_PACKED_A, LPG_F32, m, k), desc(LPG_PACKED_B, LPG_F32, k, n), desc(LPG_PACKED_A, LPG_F32, m, n)
    A, B, C1, C2, C3 = (0x10000 * (i + 1) for i in range(5))
    stages = [api.stage_gemm(1.0, A, a_d, B, b_d, 0.0, None, C1, c_d),
              api.stage_elementwise(api.LPG_EW_SCALE, C1, None, 0.5, C2, c_d),
              api.stage_gemm(1.0, C2, c_d, B, b_d, 0.0, None, C3, c_d)]
    need = api.lpg_chain_workspace_bytes(stages, api.LPG_CHAIN_CANONICAL)
    assert need >= 2 * m * n * 4
    assert api.lpg_chain_workspace_bytes(stages, api.LPG_CHAIN_PROPAGATED) == 0
    # a stage the control could not run (misaligned x1) is reported by the same dry pass
    bad = list(stages)
    bad[1] = api.stage_elementwise(api.LPG_EW_ADD, C1, C2 + 4, 0.5, C2, c_d)
    with pytest.raises(api.LpgError):
        api.lpg_chain_workspace_bytes(bad, api.LPG_CHAIN_CANONICAL)


@pytest.mark.parametrize("dtype,es", [(LPG_F32, 4), (LPG_BF16, 2)])
def test_block_order_and_store_stride_in_the_host_index_function(dtype, es):
    """group_stride / kblock_stride (section III-C): sizes and offsets equal the oracle's closed form for
    groups-outermost order and for strides that leave room between blocks; overlapping or misaligned
    strides are refused."""
    kv, kf, kb = ref.layout_consts(es)
    rows, cols = 100, 3 * kb + 5                   # 4 groups, 4 K blocks
    blk = 32 * kb
    cases = [(4 * blk, blk),                       # groups outermost, K blocks back to back
             (4 * blk, 0),                         # the same, kblock_stride left to its default for that order
             (2 * blk, 9 * blk),                   # K blocks outermost with room after every block and every K block
             (0, 6 * blk)]                         # K blocks spread out, groups back to back
    rng = np.random.default_rng(2)
    for gs, ks in cases:
        d = desc(LPG_PACKED_A, dtype, rows, cols, group_stride=gs, kblock_stride=ks)
        assert api.lpg_packed_bytes(d) == ref.strided_elems(rows, cols, es, gs, ks) * es
        dt = desc(LPG_PACKED_B, dtype, cols, rows, group_stride=gs, kblock_stride=ks)      # the same bytes as a right operand
        for _ in range(100):
            r, c = int(rng.integers(rows)), int(rng.integers(cols))
            want = int(ref.packed_offset(r, c, rows, es, gs, ks))
            assert api.lpg_layout_offset(d, 0, r, c) == want
            assert api.lpg_layout_offset(dt, 0, c, r) == want
    for gs, ks in [(blk + 8, 0), (2 * blk, 3 * blk), (blk, 2 * blk)]:      # not whole blocks; blocks overlap (4 x 4 grid)
        with pytest.raises(api.LpgError) as e:
            api.lpg_layout_offset(desc(LPG_PACKED_A, dtype, rows, cols, group_stride=gs, kblock_stride=ks), 0, 0, 0)
        assert e.value.code == api.LPG_EINVAL
    assert api.lpg_packed_bytes(desc(LPG_PACKED_A, dtype, rows, cols, group_stride=blk + 8)) == 0


def _gemm_validates(a_d, b_d, c_d):
    """Host validation of one product without a launch: the dry pass that sizes the control chain's workspace."""
    A, B, C = 0x10000, 0x20000, 0x30000
    return api.lpg_chain_workspace_bytes([api.stage_gemm(1.0, A, a_d, B, b_d, 0.0, None, C, c_d)], api.LPG_CHAIN_CANONICAL)


def test_a_product_takes_any_operand_form():
    """What the Initial kernel accepts (section III-A.1: it packs whatever the caller has): packed views with any
    origin and extent, canonical matrices of either order and either dtype, contractions of any length."""
    pa, pb = desc(LPG_PACKED_A, LPG_F32, 64, 64), desc(LPG_PACKED_B, LPG_F32, 64, 64)
    shifted = desc(LPG_PACKED_A, LPG_F32, 32, 64, parent=(64, 64), origin=(16, 0))
    assert _gemm_validates(shifted, pb, desc(LPG_PACKED_A, LPG_F32, 32, 64)) == 0
    off_k = desc(LPG_PACKED_A, LPG_F32, 64, 40, parent=(64, 96), origin=(0, 8))
    assert _gemm_validates(off_k, desc(LPG_PACKED_B, LPG_F32, 40, 64), pa) == 0
    inner_k = desc(LPG_PACKED_A, LPG_F32, 64, 20, parent=(64, 64))
    assert _gemm_validates(inner_k, desc(LPG_PACKED_B, LPG_F32, 20, 64), pa) == 0
    for a_d, b_d in [(desc(LPG_COL_MAJOR, LPG_F32, 64, 50), desc(LPG_ROW_MAJOR, LPG_F32, 50, 64)),       # neither contiguous along k
                     (desc(LPG_ROW_MAJOR, LPG_BF16, 64, 50), desc(LPG_COL_MAJOR, LPG_F32, 50, 64)),     # bf16 beside fp32: a bf16 product
                     (desc(LPG_ROW_MAJOR, LPG_F32, 64, 50, ld=51), desc(LPG_PACKED_B, LPG_BF16, 50, 64))]:
        out_dt = LPG_BF16 if LPG_BF16 in (a_d.dtype, b_d.dtype) else LPG_F32
        assert _gemm_validates(a_d, b_d, desc(LPG_PACKED_A, out_dt, 64, 64)) == 0
    # still refused: a bf16 canonical operand beside an fp32 packed one; fp32 operands with a bf16 result
    with pytest.raises(api.LpgError):
        _gemm_validates(desc(LPG_ROW_MAJOR, LPG_BF16, 64, 64), pb, pa)
    with pytest.raises(api.LpgError):
        _gemm_validates(pa, pb, desc(LPG_PACKED_A, LPG_BF16, 64, 64))
