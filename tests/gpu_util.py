"""Helpers for the GPU parity tests: move arrays, call the C ABI, read results back."""
import numpy as np
import torch

from oracle import ref

from paper_2604_04599_amd import api
from paper_2604_04599_amd.api import LPG_BF16, LPG_F32, LPG_ROW_MAJOR, desc

NP_RAW = {LPG_F32: np.uint32, LPG_BF16: np.uint16}
ES = {LPG_F32: 4, LPG_BF16: 2}


def stream():
    return torch.cuda.current_stream().cuda_stream


def dev_bytes(a):
    """numpy array (any dtype) -> device uint8 tensor with the same bytes."""
    return torch.from_numpy(np.ascontiguousarray(a).view(np.uint8).reshape(-1).copy()).cuda()


def dev_empty(nbytes, fill=None):
    t = torch.empty(max(nbytes, 16), dtype=torch.uint8, device="cuda")
    if fill is not None:
        t.fill_(fill)
    return t


def host(t, np_dtype, shape=None):
    torch.cuda.synchronize()
    a = t.cpu().numpy().view(np_dtype)
    return a if shape is None else a[:int(np.prod(shape))].reshape(shape)


def bf16_raw_to_f64(u16):
    return (u16.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def pack_dev(a_f32, kind, dtype):
    """Pack a float32 numpy matrix on the device; returns (tensor, descriptor)."""
    rows, cols = a_f32.shape
    src = dev_bytes(a_f32.astype(np.float32))
    sd = desc(LPG_ROW_MAJOR, LPG_F32, rows, cols)
    dd = desc(kind, dtype, rows, cols)
    dst = dev_empty(api.lpg_packed_bytes(dd), fill=0xA5)
    api.lpg_pack(src, sd, dst, dd, stream())
    return dst, dd


def unpack_dev(t, d):
    """Unpack a whole packed buffer to float64 numpy (exact widening)."""
    nb = max(d.batch, 1)
    od = desc(LPG_ROW_MAJOR, LPG_F32, d.rows, d.cols, batch=nb,
              batch_stride=d.rows * d.cols if nb > 1 else 0)
    out = dev_empty(nb * d.rows * d.cols * 4)
    api.lpg_unpack(t, d, out, od, stream())
    shape = (nb, d.rows, d.cols) if nb > 1 else (d.rows, d.cols)
    return host(out, np.float32, shape).astype(np.float64)


def rms(x):
    return float(np.sqrt(np.mean(np.square(np.asarray(x, dtype=np.float64)))))


def assert_elements_f32(got, want, what):
    """Per element: fp32 accumulation of k <= 8192 terms stays within 1e-5 of the value plus 1e-4 of
    the matrix's typical magnitude (cancelling sums); one misplaced element is off by about that
    magnitude and fails."""
    bad = np.abs(got - want) > 1e-5 * np.abs(want) + 1e-4 * rms(want)
    assert not bad.any(), (what, int(bad.sum()), np.argwhere(bad)[:4].tolist())


def assert_elements_bf16(got, want, what):
    """Per element of a bf16-stored result: within one bf16 ulp (2^-7 relative) of the oracle value
    rounded to bf16, plus 2e-3 of the matrix's typical magnitude for sums that cancel."""
    bad = np.abs(got - ref.round_bf16(want)) > np.abs(want) * 2.0 ** -7 + 2e-3 * rms(want)
    assert not bad.any(), (what, int(bad.sum()), np.argwhere(bad)[:4].tolist())


def fetch_slot(ch, name, b):
    """Unpack matrix b of a batched packed buffer (whole parents at batch_stride) to float64."""
    t, d = ch.bufs[name]
    es = api.ELEM_SIZE[d.dtype]
    one = api.desc(d.kind, d.dtype, d.rows, d.cols)
    sub = t[b * d.batch_stride * es: b * d.batch_stride * es + api.lpg_packed_bytes(one)]
    out = torch.empty((d.rows, d.cols), dtype=torch.float32, device="cuda")
    api.lpg_unpack(sub, one, out, api.desc(api.LPG_ROW_MAJOR, api.LPG_F32, d.rows, d.cols),
                   torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    return out.cpu().numpy().astype(np.float64)


# Row (or column) samples of the full-size runs: `count` indices spread over all 256-blocks of the
# extent, walking through all eight 32-groups of a 256 x 256 tile and both halves of the 64 lanes.
def spread_rows(n, seed, count=32):
    i = np.arange(count)
    rows = ((i * (n // 256)) // count) * 256 + (i % 8) * 32 + (5 * i + seed) % 32
    assert len(set((rows % 256) // 32)) == 8 and len(set((rows % 32) // 16)) == 2 and rows.max() < n
    return np.unique(rows)
