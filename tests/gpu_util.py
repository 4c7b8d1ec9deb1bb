"""Helpers for the GPU parity tests: move arrays, call the C ABI, read results back."""
import numpy as np
import torch

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
