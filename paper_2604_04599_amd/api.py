"""ctypes binding of the lpg C ABI (include/lpg.h): argument marshalling only.

Every function here has the name of the C entry point it calls and does no
arithmetic of its own.  Device buffers are anything with a `data_ptr()` (torch
tensors) or plain integer addresses.  There is no fallback: if the HIP library
is missing the first call raises.
"""
import ctypes
import os

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "liblpg.so")

# enums (mirrors of include/lpg.h)
LPG_OK, LPG_EINVAL, LPG_ELAYOUT, LPG_EUNSUPPORTED, LPG_EALIGN, LPG_EHIP, LPG_EWORKSPACE = 0, -1, -2, -3, -4, -5, -6
LPG_F32, LPG_BF16 = 0, 1
LPG_ROW_MAJOR, LPG_COL_MAJOR, LPG_PACKED_A, LPG_PACKED_B = 0, 1, 2, 3
LPG_EW_SCALE, LPG_EW_ADD, LPG_EW_SILU_MUL = 0, 1, 2
LPG_EPI_NONE, LPG_EPI_SILU, LPG_EPI_GATE_SILU = 0, 1, 2
LPG_STAGE_PACK, LPG_STAGE_GEMM, LPG_STAGE_ELEMENTWISE, LPG_STAGE_UNPACK, LPG_STAGE_SOFTMAX = 0, 1, 2, 3, 4
LPG_STAGE_RMSNORM, LPG_STAGE_ROPE, LPG_STAGE_ATTENTION = 5, 6, 7
LPG_CHAIN_PROPAGATED, LPG_CHAIN_CANONICAL = 0, 1
LPG_ATTN_CAUSAL, LPG_ATTN_NO_SOFTMAX = 1, 2
(LPG_TUNE_TILE, LPG_TUNE_BAND, LPG_TUNE_TWO_BLOCK_STEPS, LPG_TUNE_BF16_WHOLE_BLOCK_STEPS, LPG_TUNE_ROW_VARIANT,
 LPG_TUNE_ATTN_QUERY_GROUPS, LPG_TUNE_TRACE, LPG_TUNE_STREAM_STORES) = range(8)
LPG_TUNE_AUTO = -1
LPG_STATIC_SCRATCH_BYTES = 64 << 20

ELEM_SIZE = {LPG_F32: 4, LPG_BF16: 2}


class lpg_desc(ctypes.Structure):
    _fields_ = [
        ("kind", ctypes.c_int32), ("dtype", ctypes.c_int32),
        ("rows", ctypes.c_int64), ("cols", ctypes.c_int64), ("ld", ctypes.c_int64),
        ("parent_rows", ctypes.c_int64), ("parent_cols", ctypes.c_int64),
        ("row0", ctypes.c_int64), ("col0", ctypes.c_int64),
        ("batch", ctypes.c_int32), ("batch_div", ctypes.c_int32),
        ("batch_stride", ctypes.c_int64),
        ("batch_row_step", ctypes.c_int64), ("batch_col_step", ctypes.c_int64),
        ("group_stride", ctypes.c_int64), ("kblock_stride", ctypes.c_int64),
    ]

    def __repr__(self):
        return "lpg_desc(" + ", ".join(f"{n}={getattr(self, n)}" for n, _ in self._fields_) + ")"


class lpg_stage(ctypes.Structure):
    _fields_ = [
        ("type", ctypes.c_int32), ("op", ctypes.c_int32),
        ("alpha", ctypes.c_float), ("beta", ctypes.c_float), ("scalar", ctypes.c_float),
        ("reserved", ctypes.c_int32),
        ("in0", ctypes.c_void_p), ("in1", ctypes.c_void_p), ("in2", ctypes.c_void_p),
        ("epi_arg", ctypes.c_void_p), ("out", ctypes.c_void_p),
        ("in0_d", lpg_desc), ("in1_d", lpg_desc), ("out_d", lpg_desc), ("in2_d", lpg_desc),
    ]


class LpgError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"lpg error {code}: {msg}")
        self.code = code


_lib = None


def lib():
    """Load liblpg.so (built in-tree by build.py).  Raises if it is not there."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} not found: build it with `python -m paper_2604_04599_amd.build` "
                "(there is no CPU fallback)")
        L = ctypes.CDLL(LIB_PATH)
        vp, dp, sp = ctypes.c_void_p, ctypes.POINTER(lpg_desc), ctypes.POINTER(lpg_stage)
        L.lpg_packed_bytes.argtypes = [dp]
        L.lpg_packed_bytes.restype = ctypes.c_size_t
        L.lpg_layout_offset.argtypes = [dp, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64,
                                        ctypes.POINTER(ctypes.c_int64)]
        L.lpg_layout_offset.restype = ctypes.c_int
        L.lpg_pack.argtypes = [vp, dp, vp, dp, vp]
        L.lpg_pack.restype = ctypes.c_int
        L.lpg_unpack.argtypes = [vp, dp, vp, dp, vp]
        L.lpg_unpack.restype = ctypes.c_int
        L.lpg_gemm_packed.argtypes = [ctypes.c_float, vp, dp, vp, dp, ctypes.c_float, vp, vp, dp,
                                      ctypes.c_int, vp, vp]
        L.lpg_gemm_packed.restype = ctypes.c_int
        L.lpg_elementwise_packed.argtypes = [ctypes.c_int, vp, vp, ctypes.c_float, vp, dp, vp]
        L.lpg_elementwise_packed.restype = ctypes.c_int
        L.lpg_softmax_packed.argtypes = [vp, vp, dp, ctypes.c_float, ctypes.c_int, vp]
        L.lpg_softmax_packed.restype = ctypes.c_int
        L.lpg_attention_packed.argtypes = [vp, dp, vp, dp, vp, dp, vp, dp, ctypes.c_float, ctypes.c_int, vp]
        L.lpg_attention_packed.restype = ctypes.c_int
        L.lpg_rmsnorm_packed.argtypes = [vp, vp, vp, dp, ctypes.c_float, vp]
        L.lpg_rmsnorm_packed.restype = ctypes.c_int
        L.lpg_rope_tables.argtypes = [vp, vp, ctypes.c_int64, ctypes.c_int32, ctypes.c_double, ctypes.c_int64, vp]
        L.lpg_rope_tables.restype = ctypes.c_int
        L.lpg_rope_packed.argtypes = [vp, vp, dp, vp, vp, ctypes.c_int32, vp]
        L.lpg_rope_packed.restype = ctypes.c_int
        L.lpg_chain_workspace_bytes.argtypes = [sp, ctypes.c_int, ctypes.c_int]
        L.lpg_chain_workspace_bytes.restype = ctypes.c_size_t
        L.lpg_chain.argtypes = [sp, ctypes.c_int, ctypes.c_int, vp, ctypes.c_size_t, vp]
        L.lpg_chain.restype = ctypes.c_int
        L.lpg_chain_static.argtypes = [sp, ctypes.c_int, ctypes.c_int, vp]
        L.lpg_chain_static.restype = ctypes.c_int
        L.lpg_tune_set.argtypes = [ctypes.c_int, ctypes.c_int]
        L.lpg_tune_set.restype = ctypes.c_int
        L.lpg_tune_get.argtypes = [ctypes.c_int, ctypes.POINTER(ctypes.c_int)]
        L.lpg_tune_get.restype = ctypes.c_int
        L.lpg_last_error.restype = ctypes.c_char_p
        L.lpg_version.restype = ctypes.c_char_p
        _lib = L
    return _lib


EXPORTS = ("lpg_packed_bytes", "lpg_layout_offset", "lpg_pack", "lpg_unpack", "lpg_gemm_packed",
           "lpg_elementwise_packed", "lpg_softmax_packed", "lpg_attention_packed", "lpg_rmsnorm_packed", "lpg_rope_tables", "lpg_rope_packed",
           "lpg_chain_workspace_bytes", "lpg_chain", "lpg_chain_static", "lpg_tune_set", "lpg_tune_get", "lpg_last_error",
           "lpg_version")


def _ptr(x):
    if x is None:
        return None
    if isinstance(x, int):
        return x
    return x.data_ptr()


def _check(rc):
    if rc != LPG_OK:
        raise LpgError(rc, lpg_last_error())
    return rc


def desc(kind, dtype, rows, cols, ld=0, parent=None, origin=(0, 0), batch=1, batch_div=1,
         batch_stride=0, batch_step=(0, 0), group_stride=0, kblock_stride=0):
    """Convenience constructor for lpg_desc."""
    d = lpg_desc()
    d.kind, d.dtype, d.rows, d.cols, d.ld = kind, dtype, rows, cols, ld
    d.parent_rows, d.parent_cols = parent if parent is not None else (0, 0)
    d.row0, d.col0 = origin
    d.batch, d.batch_div, d.batch_stride = batch, batch_div, batch_stride
    d.batch_row_step, d.batch_col_step = batch_step
    d.group_stride, d.kblock_stride = group_stride, kblock_stride
    return d


def lpg_last_error():
    return lib().lpg_last_error().decode()


def lpg_version():
    return lib().lpg_version().decode()


def lpg_packed_bytes(d):
    return int(lib().lpg_packed_bytes(ctypes.byref(d)))


def lpg_layout_offset(d, b, row, col):
    off = ctypes.c_int64(0)
    _check(lib().lpg_layout_offset(ctypes.byref(d), b, row, col, ctypes.byref(off)))
    return off.value


def lpg_pack(src, src_d, dst, dst_d, stream=None):
    return _check(lib().lpg_pack(_ptr(src), ctypes.byref(src_d), _ptr(dst), ctypes.byref(dst_d), stream))


def lpg_unpack(src, src_d, dst, dst_d, stream=None):
    return _check(lib().lpg_unpack(_ptr(src), ctypes.byref(src_d), _ptr(dst), ctypes.byref(dst_d), stream))


def lpg_gemm_packed(alpha, A, a_d, B, b_d, beta, C_in, C_out, c_d, epilogue_op=LPG_EPI_NONE,
                    epi_arg=None, stream=None):
    return _check(lib().lpg_gemm_packed(alpha, _ptr(A), ctypes.byref(a_d), _ptr(B), ctypes.byref(b_d),
                                        beta, _ptr(C_in), _ptr(C_out), ctypes.byref(c_d),
                                        epilogue_op, _ptr(epi_arg), stream))


def lpg_elementwise_packed(op, x0, x1, s, out, d, stream=None):
    return _check(lib().lpg_elementwise_packed(op, _ptr(x0), _ptr(x1), s, _ptr(out), ctypes.byref(d), stream))


def lpg_softmax_packed(x, out, d, scale=1.0, causal=False, stream=None):
    return _check(lib().lpg_softmax_packed(_ptr(x), _ptr(out), ctypes.byref(d), scale, int(bool(causal)), stream))


def attention_flags(causal=False, softmax=True):
    return (LPG_ATTN_CAUSAL if causal else 0) | (0 if softmax else LPG_ATTN_NO_SOFTMAX)


def lpg_attention_packed(Q, q_d, K, k_d, V, v_d, O, o_d, scale, causal=False, stream=None, softmax=True):
    return _check(lib().lpg_attention_packed(_ptr(Q), ctypes.byref(q_d), _ptr(K), ctypes.byref(k_d), _ptr(V),
                                             ctypes.byref(v_d), _ptr(O), ctypes.byref(o_d), scale,
                                             attention_flags(causal, softmax), stream))


def lpg_rmsnorm_packed(x, weight, out, d, eps, stream=None):
    return _check(lib().lpg_rmsnorm_packed(_ptr(x), _ptr(weight), _ptr(out), ctypes.byref(d), eps, stream))


def lpg_rope_tables(cos_t, sin_t, rows, head_dim, base=10000.0, pos0=0, stream=None):
    return _check(lib().lpg_rope_tables(_ptr(cos_t), _ptr(sin_t), rows, head_dim, base, pos0, stream))


def lpg_rope_packed(x, out, d, cos_t, sin_t, head_dim, stream=None):
    return _check(lib().lpg_rope_packed(_ptr(x), _ptr(out), ctypes.byref(d), _ptr(cos_t), _ptr(sin_t), head_dim, stream))


def stage_array(stages):
    arr = (lpg_stage * len(stages))()
    for i, s in enumerate(stages):
        arr[i] = s
    return arr


def lpg_chain_workspace_bytes(stages, mode):
    arr = stages if isinstance(stages, ctypes.Array) else stage_array(stages)
    n = int(lib().lpg_chain_workspace_bytes(arr, len(arr), mode))
    if n == ctypes.c_size_t(-1).value:
        raise LpgError(LPG_EINVAL, lpg_last_error())
    return n


def lpg_chain(stages, mode=LPG_CHAIN_PROPAGATED, workspace=None, workspace_bytes=0, stream=None):
    arr = stages if isinstance(stages, ctypes.Array) else stage_array(stages)
    return _check(lib().lpg_chain(arr, len(arr), mode, _ptr(workspace), workspace_bytes, stream))


def lpg_chain_static(stages, mode=LPG_CHAIN_PROPAGATED, stream=None):
    arr = stages if isinstance(stages, ctypes.Array) else stage_array(stages)
    return _check(lib().lpg_chain_static(arr, len(arr), mode, stream))


def lpg_tune_set(key, value):
    return _check(lib().lpg_tune_set(key, value))


def lpg_tune_get(key):
    v = ctypes.c_int(0)
    _check(lib().lpg_tune_get(key, ctypes.byref(v)))
    return v.value


# stage constructors (pure marshalling)

def stage_pack(src, src_d, dst, dst_d):
    s = lpg_stage()
    s.type, s.in0, s.in0_d, s.out, s.out_d = LPG_STAGE_PACK, _ptr(src), src_d, _ptr(dst), dst_d
    return s


def stage_unpack(src, src_d, dst, dst_d):
    s = lpg_stage()
    s.type, s.in0, s.in0_d, s.out, s.out_d = LPG_STAGE_UNPACK, _ptr(src), src_d, _ptr(dst), dst_d
    return s


def stage_gemm(alpha, A, a_d, B, b_d, beta, C_in, C_out, c_d, epilogue_op=LPG_EPI_NONE, epi_arg=None):
    s = lpg_stage()
    s.type, s.op, s.alpha, s.beta = LPG_STAGE_GEMM, epilogue_op, alpha, beta
    s.in0, s.in0_d, s.in1, s.in1_d = _ptr(A), a_d, _ptr(B), b_d
    s.in2, s.epi_arg, s.out, s.out_d = _ptr(C_in), _ptr(epi_arg), _ptr(C_out), c_d
    return s


def stage_elementwise(op, x0, x1, scalar, out, d):
    s = lpg_stage()
    s.type, s.op, s.scalar = LPG_STAGE_ELEMENTWISE, op, scalar
    s.in0, s.in1, s.out, s.out_d = _ptr(x0), _ptr(x1), _ptr(out), d
    return s


def stage_softmax(x, out, d, scale=1.0, causal=False):
    s = lpg_stage()
    s.type, s.op, s.scalar = LPG_STAGE_SOFTMAX, int(bool(causal)), scale
    s.in0, s.out, s.out_d = _ptr(x), _ptr(out), d
    return s


def stage_rmsnorm(x, weight, out, d, eps):
    s = lpg_stage()
    s.type, s.scalar = LPG_STAGE_RMSNORM, eps
    s.in0, s.in1, s.out, s.out_d = _ptr(x), _ptr(weight), _ptr(out), d
    return s


def stage_rope(x, out, d, cos_t, sin_t, head_dim):
    s = lpg_stage()
    s.type, s.op = LPG_STAGE_ROPE, head_dim
    s.in0, s.in1, s.in2, s.out, s.out_d = _ptr(x), _ptr(cos_t), _ptr(sin_t), _ptr(out), d
    return s


def stage_attention(Q, q_d, K, k_d, V, v_d, O, o_d, scale, causal=False, softmax=True):
    s = lpg_stage()
    s.type, s.op, s.scalar = LPG_STAGE_ATTENTION, attention_flags(causal, softmax), scale
    s.in0, s.in0_d, s.in1, s.in1_d, s.in2, s.in2_d = _ptr(Q), q_d, _ptr(K), k_d, _ptr(V), v_d
    s.out, s.out_d = _ptr(O), o_d
    return s
