"""Python face of the CPU oracle.  TEST INFRASTRUCTURE ONLY.

Thin ctypes wrappers over oracle/lpg_oracle.c plus a closed-form index function
for the packed layout, written independently of the C loop nest so that the two
can be checked against each other.  Nothing here is imported by the product
package; only tests, the smoke check and the benchmark's CPU-baseline leg use it.

Conventions: matrices are numpy float64, C-contiguous, row-major.  Bit-pattern
functions take and return unsigned integer arrays.
"""
import ctypes
import os

import numpy as np

from . import build as _build

_lib = None


def lib():
    global _lib
    if _lib is None:
        path = _build.LIB
        if not os.path.exists(path):
            path = _build.build()
        L = ctypes.CDLL(path)
        i64, dbl, vp, i32 = ctypes.c_int64, ctypes.c_double, ctypes.c_void_p, ctypes.c_int
        L.orc_gemm.argtypes = [i64, i64, i64, dbl, vp, i64, vp, i64, dbl, vp, i64, vp, i64]
        L.orc_gemm.restype = None
        L.orc_round_f32.argtypes = [vp, i64]
        L.orc_round_bf16.argtypes = [vp, i64]
        L.orc_bf16_bits.argtypes = [ctypes.c_uint32]
        L.orc_bf16_bits.restype = ctypes.c_uint16
        L.orc_bf16_bits_array.argtypes = [vp, vp, i64]
        L.orc_silu_mul.argtypes = [vp, vp, vp, i64]
        L.orc_pack.argtypes = [vp, i64, i32, i32, vp, i64, i64, i64, i64, i64, i64]
        L.orc_unpack.argtypes = [vp, i64, i32, i32, vp, i64, i64, i64, i64, i64, i64]
        L.orc_pack_strided.argtypes = [vp, i64, i32, i32, vp, i64, i64, i64, i64, i64, i64, i64, i64]
        L.orc_unpack_strided.argtypes = [vp, i64, i32, i32, vp, i64, i64, i64, i64, i64, i64, i64, i64]
        L.orc_threads.restype = ctypes.c_int
        L.orc_softmax_rows.argtypes = [vp, vp, i64, i64, dbl, i32]
        _lib = L
    return _lib


def threads():
    """OpenMP threads the oracle GEMM uses."""
    return int(lib().orc_threads())


def _f64(x):
    return np.ascontiguousarray(x, dtype=np.float64)


# ------------------------------------------------------------------ GEMM (Eq. 1)

def gemm(A, B, alpha=1.0, beta=0.0, C=None):
    """alpha*A@B + beta*C on fp64 row-major arrays (Eq. 1).  beta == 0 never reads C."""
    A = _f64(A)
    B = _f64(B)
    m, k = A.shape
    k2, n = B.shape
    if k != k2:
        raise ValueError("inner dimensions differ")
    out = np.empty((m, n), dtype=np.float64)
    if beta != 0.0:
        if C is None:
            raise ValueError("beta != 0 needs C")
        C = _f64(C)
        if C.shape != (m, n):
            raise ValueError("C has the wrong shape")
        cptr, ldc_in = C.ctypes.data, n
    else:
        cptr, ldc_in = None, 0
    lib().orc_gemm(m, n, k, float(alpha), A.ctypes.data, k, B.ctypes.data, n,
                   float(beta), cptr, ldc_in, out.ctypes.data, n)
    return out


def chain(X, Bs, alphas=None):
    """Right-multiplication chain X*B_1*...*B_S (Eq. 2 with identity activations)."""
    C = _f64(X)
    for i, B in enumerate(Bs):
        C = gemm(C, B, alpha=1.0 if alphas is None else alphas[i])
    return C


# ------------------------------------------------------------- storage rounding

def round_f32(x):
    y = _f64(x).copy()
    lib().orc_round_f32(y.ctypes.data, y.size)
    return y


def round_bf16(x):
    y = _f64(x).copy()
    lib().orc_round_bf16(y.ctypes.data, y.size)
    return y


def bf16_bits(u32):
    """fp32 bit patterns (uint32 array) -> bf16 bit patterns (uint16), RNE."""
    u32 = np.ascontiguousarray(u32, dtype=np.uint32)
    out = np.empty(u32.shape, dtype=np.uint16)
    lib().orc_bf16_bits_array(u32.ctypes.data, out.ctypes.data, u32.size)
    return out


def silu_mul(g, u):
    g = _f64(g)
    u = _f64(u)
    out = np.empty_like(g)
    lib().orc_silu_mul(g.ctypes.data, u.ctypes.data, out.ctypes.data, g.size)
    return out


def softmax_rows(x, scale=1.0, causal=False):
    """softmax over each row of scale*x (2-D, fp64); causal keeps columns j <= i + cols - rows."""
    x = _f64(x)
    out = np.empty_like(x)
    lib().orc_softmax_rows(x.ctypes.data, out.ctypes.data, x.shape[0], x.shape[1], float(scale), int(bool(causal)))
    return out


def rope_angles(positions, head_dim, base=10000.0):
    """theta[t][i] = positions[t] * base**(-2i/head_dim), i < head_dim/2 (rotary position
    embedding; Alg. 2 applies it to Q and K before the score GEMM)."""
    i = np.arange(head_dim // 2, dtype=np.float64)
    return np.asarray(positions, dtype=np.float64)[:, None] * base ** (-2.0 * i / head_dim)[None, :]


def rope(x, cos, sin, head_dim):
    """Rotary embedding of every head of x [T, heads*head_dim] with tables cos, sin
    [T, head_dim/2]: element i of a head's first half pairs with element i of its second half,
    and the pair (a, b) of row t becomes (a cos - b sin, b cos + a sin) with the angle of
    (t, i).  Rows rotate independently (section IV-A)."""
    x = _f64(x)
    cos, sin = _f64(cos), _f64(sin)
    half = head_dim // 2
    out = np.empty_like(x)
    for h0 in range(0, x.shape[1], head_dim):
        a, b = x[:, h0:h0 + half], x[:, h0 + half:h0 + head_dim]
        out[:, h0:h0 + half] = a * cos - b * sin
        out[:, h0 + half:h0 + head_dim] = b * cos + a * sin
    return out


def rmsnorm(x, weight, eps):
    """Row-wise root-mean-square normalisation: y[t][j] = x[t][j] / sqrt(mean_j x[t][j]^2 + eps)
    * weight[j] (the RMSNorm of the contributions list; Llama's normalisation)."""
    x = _f64(x)
    w = _f64(weight)
    out = np.empty_like(x)
    for t in range(x.shape[0]):
        ms = 0.0
        for v in x[t]:
            ms += v * v
        ms /= x.shape[1]
        out[t] = x[t] / np.sqrt(ms + eps) * w
    return out


# ------------------------------------------------------------------ packed layout

def layout_consts(es):
    """(KV, KF, KB) for element size es in bytes."""
    kv = 16 // es
    return kv, 2 * kv, 8 * kv


def padded_extents(F, K, es):
    _, _, kb = layout_consts(es)
    return (F + 31) // 32 * 32, (K + kb - 1) // kb * kb


def packed_elems(F, K, es):
    fp, kp = padded_extents(F, K, es)
    return fp * kp


def block_strides(PF, es, group_stride=0, kblock_stride=0):
    """(group stride, K-block stride) in elements of a packed parent with free extent PF: the given
    ones ("block order" / "store stride", section III-C), or the defaults where 0: groups of a K
    block back to back, K blocks back to back."""
    _, _, kb = layout_consts(es)
    pfp = (PF + 31) // 32 * 32
    if not group_stride and not kblock_stride:
        return 32 * kb, pfp * kb
    return group_stride or 32 * kb, kblock_stride or 32 * kb


def strided_elems(PF, PK, es, group_stride=0, kblock_stride=0):
    """Elements a packed parent spans under the given block strides (room between blocks included)."""
    _, _, kb = layout_consts(es)
    fp, kp = padded_extents(PF, PK, es)
    gs, ks = block_strides(PF, es, group_stride, kblock_stride)
    return (fp // 32 - 1) * gs + (kp // kb - 1) * ks + 32 * kb


def packed_offset(f, k, PF, es, group_stride=0, kblock_stride=0):
    """Closed-form element offset of logical (f, k) inside a packed parent whose
    free extent is PF.  Derived from the nested-dimension order by summing
    index * stride for each dimension; works on numpy integer arrays."""
    kv, kf, kb = layout_consts(es)
    f = np.asarray(f, dtype=np.int64)
    k = np.asarray(k, dtype=np.int64)
    gs, ks = block_strides(PF, es, group_stride, kblock_stride)
    blk = (k // kb) * ks + (f // 32) * gs
    kin = k % kb
    c = kin // kf
    r = kin % kf              # position inside the fragment's k range
    h = (r // 4) % 2
    v = 4 * (r // 8) + r % 4
    return blk + c * (32 * kf) + h * (32 * kv) + (f % 32) * kv + v


def _raw(a, es):
    dt = {4: np.uint32, 2: np.uint16}[es]
    a = np.ascontiguousarray(a)
    if a.dtype.itemsize != es:
        raise ValueError("element size mismatch")
    return a.view(dt)


def pack(canon, free_is_rows, es, parent=None, origin=(0, 0), out=None, group_stride=0, kblock_stride=0):
    """Pack a 2-D canonical row-major array of raw elements.

    free_is_rows=True gives the left-operand layout P(X; rows, cols); False
    gives the right-operand layout P(X; cols, rows).  `parent` = (PF, PK)
    extents of the packed parent, `origin` = (f0, k0) of this view inside it.
    Returns (or fills `out`, a flat raw array of the parent's padded size).
    """
    a = _raw(canon, es)
    rows, cols = a.shape
    F, K = (rows, cols) if free_is_rows else (cols, rows)
    PF, PK = parent if parent is not None else (F, K)
    if out is None:
        out = np.zeros(strided_elems(PF, PK, es, group_stride, kblock_stride), dtype=a.dtype)
    lib().orc_pack_strided(a.ctypes.data, cols, 1 if free_is_rows else 0, es, out.ctypes.data,
                           PF, PK, origin[0], origin[1], F, K, group_stride, kblock_stride)
    return out


def unpack(packed, rows, cols, free_is_rows, es, parent=None, origin=(0, 0), group_stride=0, kblock_stride=0):
    """Inverse of pack(): returns a (rows, cols) raw array."""
    p = _raw(packed, es)
    F, K = (rows, cols) if free_is_rows else (cols, rows)
    PF, PK = parent if parent is not None else (F, K)
    out = np.zeros((rows, cols), dtype=p.dtype)
    lib().orc_unpack_strided(out.ctypes.data, cols, 1 if free_is_rows else 0, es, p.ctypes.data,
                             PF, PK, origin[0], origin[1], F, K, group_stride, kblock_stride)
    return out


# ------------------------------------------------------------------ error metric

def rel_frobenius(got, ref):
    """||got - ref||_F / ||ref||_F in fp64."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    den = np.linalg.norm(ref.ravel())
    num = np.linalg.norm((got - ref).ravel())
    return float(num / den) if den > 0 else float(num)
