"""GPU parity on buffers past 2^32 bytes: every byte offset the kernels form (block strides, slot
strides, canonical leading dimensions) must be 64-bit.  The matrices are generated on the device;
the oracle supplies the packed position of sampled elements (closed form of the layout, section
III-B as re-laid for MFMA operands) and the fp64 values of sampled rows (Eq. 1, Alg. 2)."""
import numpy as np
import pytest
import torch

from oracle import ref
from paper_2604_04599_amd import api
from paper_2604_04599_amd.api import (LPG_BF16, LPG_F32, LPG_PACKED_A, LPG_PACKED_B, LPG_ROW_MAJOR, desc)
from tests.gpu_util import dev_empty, pack_dev, stream

pytestmark = pytest.mark.gpu

ROWS, COLS = 33001, 32801            # 4.33e9 bytes of fp32, ragged in both dimensions
ROW_SAMPLE = np.array([0, 1, 31, 32, 33, 9999, 16383, 16384, 16500, 32735, 32736, 32767, 32768, 32999, 33000])


def sample_positions(rows, cols, n, seed):
    """Random (row, col) pairs plus the corners and the elements whose canonical byte offset sits
    next to 2^31 and 2^32."""
    rng = np.random.default_rng(seed)
    r = rng.integers(0, rows, n)
    c = rng.integers(0, cols, n)
    extra = [(0, 0), (rows - 1, cols - 1), (rows - 1, 0), (0, cols - 1)]
    for edge in (1 << 29, 1 << 30):                    # element index of byte 2^31, 2^32 (fp32)
        for d in (-1, 0, 1):
            e = edge + d
            if e < rows * cols:
                extra.append((e // cols, e % cols))
    r = np.concatenate([r, [p[0] for p in extra]])
    c = np.concatenate([c, [p[1] for p in extra]])
    return r, c


def gather(flat, idx):
    return flat[torch.from_numpy(np.asarray(idx, dtype=np.int64)).cuda()].cpu().numpy()


def test_pack_and_unpack_past_4_gib():
    torch.manual_seed(5)
    x = torch.randn(ROWS, COLS, device="cuda")
    assert x.numel() * 4 > 1 << 32
    for kind in (LPG_PACKED_A, LPG_PACKED_B):
        a_side = kind == LPG_PACKED_A
        sd = desc(LPG_ROW_MAJOR, LPG_F32, ROWS, COLS)
        dd = desc(kind, LPG_F32, ROWS, COLS)
        nbytes = api.lpg_packed_bytes(dd)
        assert nbytes > 1 << 32
        p = dev_empty(nbytes, fill=0xA5)
        api.lpg_pack(x, sd, p, dd, stream())
        pi = p.view(torch.int32)
        r, c = sample_positions(ROWS, COLS, 200000, 11)
        f, k, pf = (r, c, ROWS) if a_side else (c, r, COLS)
        off = ref.packed_offset(f, k, pf, 4)
        want = gather(x.view(torch.int32).reshape(-1), r.astype(np.int64) * COLS + c)
        assert np.array_equal(gather(pi, off), want)
        # padding (free index past the extent, contraction index past the extent) is zero
        F, K = (ROWS, COLS) if a_side else (COLS, ROWS)
        fp, kp = ref.padded_extents(F, K, 4)
        rng = np.random.default_rng(12)
        pad_f = ref.packed_offset(rng.integers(F, fp, 5000), rng.integers(0, kp, 5000), pf, 4)
        pad_k = ref.packed_offset(rng.integers(0, fp, 5000), rng.integers(K, kp, 5000), pf, 4)
        assert not gather(pi, pad_f).any() and not gather(pi, pad_k).any()
        assert int(pad_f.max()) * 4 < nbytes and int(off.max()) * 4 < nbytes
        back = torch.full_like(x, 7.0)
        api.lpg_unpack(p, dd, back, sd, stream())
        assert torch.equal(back.view(torch.int32), x.view(torch.int32))
        del p, pi, back


@pytest.mark.parametrize("c_kind", [LPG_PACKED_A, LPG_PACKED_B, LPG_ROW_MAJOR])
def test_gemm_output_past_4_gib(c_kind):
    m, n, k = ROWS, COLS, 96
    rng = np.random.default_rng(21)
    A = rng.integers(-4, 5, (m, k)).astype(np.float32)      # small integers: every sum is exact
    B = rng.integers(-4, 5, (k, n)).astype(np.float32)
    ta, ad = pack_dev(A, LPG_PACKED_A, LPG_F32)
    tb, bd = pack_dev(B, LPG_PACKED_B, LPG_F32)
    cd = desc(c_kind, LPG_F32, m, n)
    nbytes = m * n * 4 if c_kind == LPG_ROW_MAJOR else api.lpg_packed_bytes(cd)
    assert nbytes > 1 << 32
    tc = dev_empty(nbytes, fill=0xFF)
    api.lpg_gemm_packed(1.0, ta, ad, tb, bd, 0.0, None, tc, cd, 0, None, stream())
    cf = tc.view(torch.float32)
    want = ref.gemm(A[ROW_SAMPLE], B)
    rr, cc = np.meshgrid(ROW_SAMPLE, np.arange(n), indexing="ij")
    if c_kind == LPG_ROW_MAJOR:
        off = rr.astype(np.int64) * n + cc
    elif c_kind == LPG_PACKED_A:
        off = ref.packed_offset(rr, cc, m, 4)
    else:
        off = ref.packed_offset(cc, rr, n, 4)
    got = gather(cf, off.reshape(-1)).reshape(want.shape).astype(np.float64)
    assert np.array_equal(got, want)
    col_sample = np.array([0, 31, 32, 16383, 16384, 32767, 32768, n - 1])
    want_c = ref.gemm(A, B[:, col_sample])
    rr, cc = np.meshgrid(np.arange(m), col_sample, indexing="ij")
    if c_kind == LPG_ROW_MAJOR:
        off = rr.astype(np.int64) * n + cc
    elif c_kind == LPG_PACKED_A:
        off = ref.packed_offset(rr, cc, m, 4)
    else:
        off = ref.packed_offset(cc, rr, n, 4)
    got_c = gather(cf, off.reshape(-1)).reshape(want_c.shape).astype(np.float64)
    assert np.array_equal(got_c, want_c)


def test_gemm_inputs_past_4_gib():
    """A canonical (Initial kernel) and packed left operand of 4.3 GB, fp32 and bf16."""
    m, k, n = ROWS, 32800, 64                                # a canonical operand needs k % 32 == 0
    assert m * k * 4 > 1 << 32
    torch.manual_seed(6)
    x = torch.randint(-3, 4, (m, k), device="cuda", dtype=torch.int32).float()
    rng = np.random.default_rng(22)
    B = rng.integers(-3, 4, (k, n)).astype(np.float32)
    a_rows = x[torch.from_numpy(ROW_SAMPLE).cuda()].cpu().numpy()
    want = ref.gemm(a_rows, B)                               # exact: |sum| < 2^24
    sd = desc(LPG_ROW_MAJOR, LPG_F32, m, k)
    cd = desc(LPG_PACKED_A, LPG_F32, m, n)
    off = ref.packed_offset(*np.meshgrid(ROW_SAMPLE, np.arange(n), indexing="ij"), m, 4).reshape(-1)
    tb, bd = pack_dev(B, LPG_PACKED_B, LPG_F32)
    # canonical A straight into the GEMM
    tc = dev_empty(api.lpg_packed_bytes(cd), fill=0xFF)
    api.lpg_gemm_packed(1.0, x, sd, tb, bd, 0.0, None, tc, cd, 0, None, stream())
    assert np.array_equal(gather(tc.view(torch.float32), off).reshape(want.shape), want)
    # packed A, fp32 and bf16 (the integers are exact in bf16)
    for dt in (LPG_F32, LPG_BF16):
        ad = desc(LPG_PACKED_A, dt, m, k)
        ta = dev_empty(api.lpg_packed_bytes(ad), fill=0xA5)
        api.lpg_pack(x, sd, ta, ad, stream())
        tbx, bdx = pack_dev(B, LPG_PACKED_B, dt)
        tc = dev_empty(api.lpg_packed_bytes(cd), fill=0xFF)
        api.lpg_gemm_packed(1.0, ta, ad, tbx, bdx, 0.0, None, tc, cd, 0, None, stream())
        assert np.array_equal(gather(tc.view(torch.float32), off).reshape(want.shape), want)
        del ta, tc


def test_batched_slots_past_4_gib():
    """Three heads whose output slots are 1.6 GB apart: the last slot starts past 2^31 bytes and
    ends past 2^32."""
    heads, m, n, k = 3, 20001, 19999, 32
    rng = np.random.default_rng(23)
    A = rng.integers(-4, 5, (heads, m, k)).astype(np.float32)
    B = rng.integers(-4, 5, (heads, k, n)).astype(np.float32)
    ea = ref.packed_elems(m, k, 4)
    eb = ref.packed_elems(n, k, 4)
    ec = ref.packed_elems(m, n, 4)
    assert heads * ec * 4 > 1 << 32
    ad = desc(LPG_PACKED_A, LPG_F32, m, k, batch=heads, batch_stride=ea)
    bd = desc(LPG_PACKED_B, LPG_F32, k, n, batch=heads, batch_stride=eb)
    cd = desc(LPG_PACKED_A, LPG_F32, m, n, batch=heads, batch_stride=ec)
    ta = torch.cat([pack_dev(A[h], LPG_PACKED_A, LPG_F32)[0][:ea * 4] for h in range(heads)])
    tb = torch.cat([pack_dev(B[h], LPG_PACKED_B, LPG_F32)[0][:eb * 4] for h in range(heads)])
    tc = dev_empty(heads * ec * 4, fill=0xFF)
    api.lpg_gemm_packed(1.0, ta, ad, tb, bd, 0.0, None, tc, cd, 0, None, stream())
    rows = np.array([0, 31, 32, 10000, m - 1])
    for h in range(heads):
        want = ref.gemm(A[h][rows], B[h])
        off = h * ec + ref.packed_offset(*np.meshgrid(rows, np.arange(n), indexing="ij"), m, 4).reshape(-1)
        assert np.array_equal(gather(tc.view(torch.float32), off).reshape(want.shape), want)


def test_softmax_past_4_gib():
    torch.manual_seed(7)
    x = torch.randn(ROWS, COLS, device="cuda") * 3
    sd = desc(LPG_ROW_MAJOR, LPG_F32, ROWS, COLS)
    dd = desc(LPG_PACKED_A, LPG_F32, ROWS, COLS)
    p = dev_empty(api.lpg_packed_bytes(dd), fill=0xA5)
    api.lpg_pack(x, sd, p, dd, stream())
    api.lpg_softmax_packed(p, p, dd, 0.5, True, stream())
    xin = x[torch.from_numpy(ROW_SAMPLE).cuda()].cpu().numpy().astype(np.float64)
    # causal with cols < rows: row i keeps columns j <= i + (cols - rows); rows with none are zero
    shift = COLS - ROWS
    got = gather(p.view(torch.float32),
                 ref.packed_offset(*np.meshgrid(ROW_SAMPLE, np.arange(COLS), indexing="ij"), ROWS, 4).reshape(-1))
    got = got.reshape(xin.shape).astype(np.float64)
    for i, r in enumerate(ROW_SAMPLE):
        keep = r + shift + 1
        if keep <= 0:
            assert not got[i].any()
            continue
        want = ref.softmax_rows(xin[i:i + 1, :keep], scale=0.5)[0]
        assert np.all(np.abs(got[i, :keep] - want) <= 1e-5 * want + 1e-12)
        assert not got[i, keep:].any()
