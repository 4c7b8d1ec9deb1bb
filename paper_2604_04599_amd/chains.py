"""The five benchmark workloads expressed as lpg chains (lists of lpg_stage).

Each builder has two forms.  The default packs the activations with lpg_pack at the
chain's entry and unpacks the result with lpg_unpack at its exit.  With fused=True the
first GEMM reads its canonical operand itself and the last GEMM writes the canonical
result itself (the Initial and Ending kernels), so those passes disappear where the
library supports it (fp32, k-contiguous inputs; any output).

This module only allocates device memory (torch), fills descriptors and stage
lists, and calls the C ABI through `api`; all computation happens in the HIP
library.  Weights are packed once when a chain is built (they are constants of
the model, as in the paper's Fig. 1, which leaves weight packing out); the timed
chain packs its activations at entry, runs its GEMMs with every intermediate
kept packed, and unpacks the result at exit.
"""
import numpy as np
import torch

from . import api
from .api import (LPG_BF16, LPG_CHAIN_CANONICAL, LPG_CHAIN_PROPAGATED, LPG_COL_MAJOR, LPG_EW_SILU_MUL,
                  LPG_F32, LPG_PACKED_A, LPG_PACKED_B, LPG_ROW_MAJOR, desc)

TORCH_DT = {LPG_F32: torch.float32, LPG_BF16: torch.bfloat16}


def _dev():
    if not torch.cuda.is_available():
        raise RuntimeError("lpg chains need a GPU (no CPU fallback)")
    return torch.device("cuda")


def _stream():
    return torch.cuda.current_stream().cuda_stream


def device_array(x):
    """numpy float32 array -> contiguous device tensor."""
    return torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(_dev())


def packed_buffer(d):
    """Uninitialised device buffer for a packed descriptor."""
    return torch.empty(api.lpg_packed_bytes(d), dtype=torch.uint8, device=_dev())


class Chain:
    """A built workload: stages, named buffers and their descriptors."""

    def __init__(self, name, shape, flops):
        self.name, self.shape, self.flops = name, shape, flops
        self.stages = []
        self.bufs = {}        # name -> (tensor, descriptor): packed intermediates and weights
        self.outputs = {}     # name -> canonical device tensor written by the exit unpack
        self.inputs = {}      # name -> canonical device tensor read by the entry pack
        self._arr = None
        self._ws = None
        self._ws_bytes = 0

    # -- building -------------------------------------------------------------------
    def new_packed(self, name, d):
        t = packed_buffer(d)
        self.bufs[name] = (t, d)
        return t

    def pack_weight(self, name, w, kind, dtype, transpose_src=False):
        """Pack a constant right now (outside the timed chain).  `w` is a numpy array
        [rows, cols]; transpose_src packs w^T, read through a column-major descriptor."""
        src = device_array(w)
        rows, cols = w.shape
        if transpose_src:
            sd = desc(LPG_COL_MAJOR, LPG_F32, cols, rows)
            dd = desc(kind, dtype, cols, rows)
        else:
            sd = desc(LPG_ROW_MAJOR, LPG_F32, rows, cols)
            dd = desc(kind, dtype, rows, cols)
        t = self.new_packed(name, dd)
        api.lpg_pack(src, sd, t, dd, _stream())
        torch.cuda.synchronize()
        return t, dd

    def add(self, stage):
        self.stages.append(stage)
        self._arr = None

    # -- running --------------------------------------------------------------------
    def stage_array(self):
        if self._arr is None:
            self._arr = api.stage_array(self.stages)
        return self._arr

    def workspace(self):
        need = api.lpg_chain_workspace_bytes(self.stage_array(), LPG_CHAIN_CANONICAL)
        if self._ws is None or self._ws_bytes < need:
            self._ws = torch.empty(max(need, 256), dtype=torch.uint8, device=_dev())
            self._ws_bytes = need
        return self._ws, need

    def run(self, mode=LPG_CHAIN_PROPAGATED):
        """Enqueue the whole chain on torch's current stream (asynchronous)."""
        if mode == LPG_CHAIN_CANONICAL:
            ws, need = self.workspace()
            api.lpg_chain(self.stage_array(), mode, ws, need, _stream())
        else:
            api.lpg_chain(self.stage_array(), mode, None, 0, _stream())

    def capture(self, mode=LPG_CHAIN_PROPAGATED):
        """Record the chain once into a HIP graph and return a callable that replays it on
        torch's current stream.  Every launch of lpg_chain is a plain kernel on the stream it
        is given and the call neither allocates nor synchronises, so stream capture sees the
        whole chain; for launch-bound chains (a few small GEMMs) a replay costs one graph
        launch instead of one launch per stage."""
        if mode == LPG_CHAIN_CANONICAL:
            self.workspace()                       # allocate before capture starts
        self.run(mode)                             # warm up outside the capture
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            self.run(mode)
        return graph.replay

    def fetch(self, name):
        """Unpack a named packed buffer to a numpy float32 array (for checks)."""
        t, d = self.bufs[name]
        nb = max(d.batch, 1)
        if d.parent_rows:
            raise ValueError("fetch works on whole buffers, not views")
        out = torch.empty((nb, d.rows, d.cols) if nb > 1 else (d.rows, d.cols), dtype=torch.float32,
                          device=_dev())
        od = desc(LPG_ROW_MAJOR, LPG_F32, d.rows, d.cols, batch=nb,
                  batch_stride=d.rows * d.cols if nb > 1 else 0)
        api.lpg_unpack(t, d, out, od, _stream())
        torch.cuda.synchronize()
        return out.cpu().numpy()

    def output(self, name):
        torch.cuda.synchronize()
        return self.outputs[name].cpu().numpy()


def _padded(n, m):
    return (n + m - 1) // m * m


def _packed_elems(dtype, free, k):
    kb = 32 if dtype == LPG_F32 else 64
    return _padded(free, 32) * _padded(k, kb)


# ------------------------------------------------------------------------------------

def build_two_gemm(inp, shape, fused=False):
    n = shape["n"]
    ch = Chain("two_gemm", shape, 2 * 2 * n ** 3)
    a = ch.inputs["A"] = device_array(inp["A"])
    _, b1d = ch.pack_weight("B1", inp["B1"], LPG_PACKED_B, LPG_F32)
    _, b2d = ch.pack_weight("B2", inp["B2"], LPG_PACKED_B, LPG_F32)
    ad = desc(LPG_PACKED_A, LPG_F32, n, n)
    pa = ch.new_packed("A", ad)
    c1 = ch.new_packed("C1", ad)
    c2 = ch.new_packed("C2", ad)
    out = ch.outputs["C2"] = torch.empty((n, n), dtype=torch.float32, device=_dev())
    rm = desc(LPG_ROW_MAJOR, LPG_F32, n, n)
    if fused:
        ch.add(api.stage_gemm(1.0, a, rm, ch.bufs["B1"][0], b1d, 0.0, None, c1, ad))
        ch.add(api.stage_gemm(1.0, c1, ad, ch.bufs["B2"][0], b2d, 0.0, None, out, rm))
        return ch
    ch.add(api.stage_pack(a, rm, pa, ad))
    ch.add(api.stage_gemm(1.0, pa, ad, ch.bufs["B1"][0], b1d, 0.0, None, c1, ad))
    ch.add(api.stage_gemm(1.0, c1, ad, ch.bufs["B2"][0], b2d, 0.0, None, c2, ad))
    ch.add(api.stage_unpack(c2, ad, out, rm))
    return ch


def build_mlp(inp, shape, fused=False):
    m, d, h = shape["m"], shape["d"], shape["h"]
    ch = Chain("mlp", shape, 2 * 2 * m * d * h)
    x = ch.inputs["X"] = device_array(inp["X"])
    _, w1d = ch.pack_weight("W1", inp["W1"], LPG_PACKED_B, LPG_F32)
    _, w2d = ch.pack_weight("W2", inp["W2"], LPG_PACKED_B, LPG_F32)
    xd = desc(LPG_PACKED_A, LPG_F32, m, d)
    hd = desc(LPG_PACKED_A, LPG_F32, m, h)
    px = ch.new_packed("X", xd)
    ph = ch.new_packed("H", hd)
    py = ch.new_packed("Y", xd)
    out = ch.outputs["Y"] = torch.empty((m, d), dtype=torch.float32, device=_dev())
    rm = desc(LPG_ROW_MAJOR, LPG_F32, m, d)
    if fused:
        # X is read twice, both times in row-major: as the first GEMM's left operand and as
        # the residual C_in of the second, whose C_out is row-major as well
        ch.add(api.stage_gemm(1.0, x, rm, ch.bufs["W1"][0], w1d, 0.0, None, ph, hd))
        ch.add(api.stage_gemm(1.0, ph, hd, ch.bufs["W2"][0], w2d, 1.0, x, out, rm))
        return ch
    ch.add(api.stage_pack(x, rm, px, xd))
    ch.add(api.stage_gemm(1.0, px, xd, ch.bufs["W1"][0], w1d, 0.0, None, ph, hd))
    # residual: Y = H*W2 + 1*X, with C_in = packed X (it has Y's layout) and a separate C_out
    ch.add(api.stage_gemm(1.0, ph, hd, ch.bufs["W2"][0], w2d, 1.0, px, py, xd))
    ch.add(api.stage_unpack(py, xd, out, rm))
    return ch


def build_attention(inp, shape, fused=False, softmax=False, causal=False, flash=False, causal_blocks=1):
    """softmax=False: O = (Q K^T / sqrt(dh)) V, the two chained GEMMs alone.  softmax=True: the
    scale moves into a softmax stage (optionally causally masked) that runs in place on the
    packed scores between the two GEMMs.  flash=True: one lpg_attention_packed stage replaces the
    two or three stages (with or without the softmax), and the scores are never stored.
    causal_blocks = n > 1 (with softmax and causal): the three stages run per block of t/n query
    rows on views that end at the last key those rows may see (build_llama_layer has the same)."""
    nh, t, dh = shape["heads"], shape["t"], shape["dh"]
    scale = 1.0 / float(np.sqrt(dh))
    alpha = 1.0 if softmax else scale
    ch = Chain("attention", shape, nh * 2 * 2 * t * t * dh)
    q = ch.inputs["Q"] = device_array(inp["Q"])
    k = ch.inputs["K"] = device_array(inp["K"])
    v = ch.inputs["V"] = device_array(inp["V"])
    pe = _packed_elems(LPG_F32, t, dh)
    rm = desc(LPG_ROW_MAJOR, LPG_F32, t, dh, batch=nh, batch_stride=t * dh)
    qd = desc(LPG_PACKED_A, LPG_F32, t, dh, batch=nh, batch_stride=pe)
    # K_h^T [dh x t] as a right operand; K_h stored row-major [t x dh] is K_h^T column-major
    ktd_src = desc(LPG_COL_MAJOR, LPG_F32, dh, t, batch=nh, batch_stride=t * dh)
    ktd = desc(LPG_PACKED_B, LPG_F32, dh, t, batch=nh, batch_stride=pe)
    vd = desc(LPG_PACKED_B, LPG_F32, t, dh, batch=nh, batch_stride=_packed_elems(LPG_F32, dh, t))
    sd = desc(LPG_PACKED_A, LPG_F32, t, t, batch=nh, batch_stride=_packed_elems(LPG_F32, t, t))
    od = desc(LPG_PACKED_A, LPG_F32, t, dh, batch=nh, batch_stride=pe)
    pq, pk, pv = ch.new_packed("Q", qd), ch.new_packed("Kt", ktd), ch.new_packed("V", vd)
    po = ch.new_packed("O", od)
    ps = None if flash else ch.new_packed("S", sd)
    out = ch.outputs["O"] = torch.empty((nh, t, dh), dtype=torch.float32, device=_dev())
    if fused:
        # Q_h and K_h^T are contiguous along the contraction index as they stand; V_h (a right
        # operand stored row-major) is not and is still packed
        ch.add(api.stage_pack(v, rm, pv, vd))
        ch.add(api.stage_gemm(alpha, q, rm, k, ktd_src, 0.0, None, ps, sd))
        if softmax:
            ch.add(api.stage_softmax(ps, ps, sd, scale, causal))
        ch.add(api.stage_gemm(1.0, ps, sd, pv, vd, 0.0, None, out, rm))
        return ch
    ch.add(api.stage_pack(q, rm, pq, qd))
    ch.add(api.stage_pack(k, ktd_src, pk, ktd))
    ch.add(api.stage_pack(v, rm, pv, vd))
    if flash:
        ch.add(api.stage_attention(pq, qd, pk, ktd, pv, vd, po, od, scale, causal, softmax=softmax))
        ch.add(api.stage_unpack(po, od, out, rm))
        return ch
    if causal_blocks > 1:
        rb = t // causal_blocks
        if not (softmax and causal) or t % causal_blocks or rb % 32:
            raise ValueError("causal_blocks needs the causal softmax stage and blocks of a multiple of 32 rows")
        for i in range(causal_blocks):
            r0, kc = i * rb, (i + 1) * rb              # query rows [r0, r0 + rb) see keys [0, kc)
            q_i = desc(LPG_PACKED_A, LPG_F32, rb, dh, parent=(t, dh), origin=(r0, 0), batch=nh, batch_stride=qd.batch_stride)
            kt_i = desc(LPG_PACKED_B, LPG_F32, dh, kc, parent=(dh, t), batch=nh, batch_stride=ktd.batch_stride)
            s_i = desc(LPG_PACKED_A, LPG_F32, rb, kc, parent=(t, t), origin=(r0, 0), batch=nh, batch_stride=sd.batch_stride)
            v_i = desc(LPG_PACKED_B, LPG_F32, kc, dh, parent=(t, dh), batch=nh, batch_stride=vd.batch_stride)
            o_i = desc(LPG_PACKED_A, LPG_F32, rb, dh, parent=(t, dh), origin=(r0, 0), batch=nh, batch_stride=od.batch_stride)
            ch.add(api.stage_gemm(alpha, pq, q_i, pk, kt_i, 0.0, None, ps, s_i))
            ch.add(api.stage_softmax(ps, ps, s_i, scale, True))
            ch.add(api.stage_gemm(1.0, ps, s_i, pv, v_i, 0.0, None, po, o_i))
        ch.add(api.stage_unpack(po, od, out, rm))
        return ch
    ch.add(api.stage_gemm(alpha, pq, qd, pk, ktd, 0.0, None, ps, sd))
    if softmax:
        ch.add(api.stage_softmax(ps, ps, sd, scale, causal))
    ch.add(api.stage_gemm(1.0, ps, sd, pv, vd, 0.0, None, po, od))
    ch.add(api.stage_unpack(po, od, out, rm))
    return ch


def build_deep_chain(inp, shape, fused=False):
    n, depth = shape["n"], shape["depth"]
    ch = Chain("deep_chain", shape, depth * 2 * n ** 3)
    c0 = ch.inputs["C0"] = device_array(inp["C0"])
    a_d = desc(LPG_PACKED_A, LPG_F32, n, n)
    b_d = desc(LPG_PACKED_B, LPG_F32, n, n)
    rm = desc(LPG_ROW_MAJOR, LPG_F32, n, n)
    for i in range(depth):
        ch.pack_weight(f"B{i}", inp["B"][i], LPG_PACKED_B, LPG_F32)
    out = ch.outputs["C"] = torch.empty((n, n), dtype=torch.float32, device=_dev())
    cm = desc(LPG_COL_MAJOR, LPG_F32, n, n)       # C^T column-major is C row-major
    cur, cur_a, cur_b = ch.new_packed("C0", a_d), a_d, b_d
    if fused:
        cur, cur_a, cur_b = c0, rm, cm              # C_0 (or C_0^T) read as it stands
    else:
        ch.add(api.stage_pack(c0, rm, cur, a_d))
    for i in range(depth):
        last = fused and i == depth - 1
        nxt = out if last else ch.new_packed(f"C{i + 1}", a_d)
        w = ch.bufs[f"B{i}"][0]
        if i % 2 == 0:
            # C_{i+1} = C_i * B_i : C_i consumed as a left operand
            ch.add(api.stage_gemm(1.0, cur, cur_a, w, b_d, 0.0, None, nxt, rm if last else a_d))
        else:
            # the same bytes read as the right operand C_i^T of C_{i+1}^T = B_i^T * C_i^T
            ch.add(api.stage_gemm(1.0, w, a_d, cur, cur_b, 0.0, None, nxt, cm if last else b_d))
        cur, cur_a, cur_b = nxt, a_d, b_d
    if not fused:
        ch.add(api.stage_unpack(cur, a_d, out, rm))
    return ch


def build_decoder_layer(inp, shape, fused=False, flash=False):
    t, hid, nq, nkv, ffn = shape["t"], shape["hidden"], shape["n_q"], shape["n_kv"], shape["ffn"]
    dh = hid // nq
    kvw = nkv * dh
    rep = nq // nkv
    if dh % 64:
        raise ValueError("bf16 head slices need head_dim to be a multiple of 64")
    flops = (2 * t * hid * (hid + 2 * kvw) + nq * 4 * t * t * dh + 2 * t * hid * hid + 3 * 2 * t * hid * ffn)
    ch = Chain("decoder_layer", shape, flops)
    B = LPG_BF16
    x = ch.inputs["X"] = device_array(inp["X"])
    for nm in ("Wq", "Wk", "Wv", "Wo", "Wg", "Wu", "Wd"):
        ch.pack_weight(nm, inp[nm], LPG_PACKED_B, B)
    wd = {nm: ch.bufs[nm][1] for nm in ("Wq", "Wk", "Wv", "Wo", "Wg", "Wu", "Wd")}
    wt = {nm: ch.bufs[nm][0] for nm in wd}
    xd = desc(LPG_PACKED_A, B, t, hid)
    qd = desc(LPG_PACKED_A, B, t, hid)
    kd = desc(LPG_PACKED_A, B, t, kvw)          # K written as a left-operand image ...
    vd = desc(LPG_PACKED_B, B, t, kvw)          # V written as a right operand
    px, pq, pk, pv = (ch.new_packed(n_, d_) for n_, d_ in (("X", xd), ("Q", qd), ("K", kd), ("V", vd)))
    sd = desc(LPG_PACKED_A, B, t, t, batch=nq, batch_stride=_packed_elems(B, t, t))
    ps = None if flash else ch.new_packed("S", sd)
    od_full = desc(LPG_PACKED_A, B, t, hid)
    po = ch.new_packed("O", od_full)
    ad = desc(LPG_PACKED_A, B, t, hid)
    pattn = ch.new_packed("attn", ad)
    gd = desc(LPG_PACKED_A, B, t, ffn)
    pg, pu, pact = ch.new_packed("gate", gd), ch.new_packed("up", gd), ch.new_packed("act", gd)
    yd = desc(LPG_PACKED_A, LPG_F32, t, hid)
    py = ch.new_packed("Y", yd)
    out = ch.outputs["Y"] = torch.empty((t, hid), dtype=torch.float32, device=_dev())
    rm_x = desc(LPG_ROW_MAJOR, LPG_F32, t, hid)

    ch.add(api.stage_pack(x, rm_x, px, xd))                                    # fp32 -> bf16 (exact here)
    ch.add(api.stage_gemm(1.0, px, xd, wt["Wq"], wd["Wq"], 0.0, None, pq, qd))
    ch.add(api.stage_gemm(1.0, px, xd, wt["Wk"], wd["Wk"], 0.0, None, pk, kd))
    ch.add(api.stage_gemm(1.0, px, xd, wt["Wv"], wd["Wv"], 0.0, None, pv, vd))
    # per query head h: S_h = (1/sqrt(dh)) Q_h K_g^T,  g = h // rep.
    q_view = desc(LPG_PACKED_A, B, t, dh, parent=(t, hid), batch=nq, batch_step=(0, dh))
    # ... and read here as the right operand K_g^T: rows [g*dh, (g+1)*dh) of K^T [kvw x t]
    kt_view = desc(LPG_PACKED_B, B, dh, t, parent=(kvw, t), batch=nq, batch_div=rep, batch_step=(dh, 0))
    v_view = desc(LPG_PACKED_B, B, t, dh, parent=(t, kvw), batch=nq, batch_div=rep, batch_step=(0, dh))
    o_view = desc(LPG_PACKED_A, B, t, dh, parent=(t, hid), batch=nq, batch_step=(0, dh))
    if flash:
        # the two attention GEMMs as one kernel, S_h kept in registers (no softmax in this workload)
        ch.add(api.stage_attention(pq, q_view, pk, kt_view, pv, v_view, po, o_view, 1.0 / float(np.sqrt(dh)),
                                   causal=False, softmax=False))
    else:
        ch.add(api.stage_gemm(1.0 / float(np.sqrt(dh)), pq, q_view, pk, kt_view, 0.0, None, ps, sd))
        ch.add(api.stage_gemm(1.0, ps, sd, pv, v_view, 0.0, None, po, o_view))
    ch.add(api.stage_gemm(1.0, po, od_full, wt["Wo"], wd["Wo"], 0.0, None, pattn, ad))
    ch.add(api.stage_gemm(1.0, pattn, ad, wt["Wg"], wd["Wg"], 0.0, None, pg, gd))
    if fused:
        # SiLU(gate) * up applied in the up projection's epilogue (no U buffer, no elementwise
        # pass), and the exit written row-major by the last GEMM.  The entry stays a pack: X is
        # converted fp32 -> bf16 there.
        ch.add(api.stage_gemm(1.0, pattn, ad, wt["Wu"], wd["Wu"], 0.0, None, pact, gd, api.LPG_EPI_GATE_SILU, pg))
        ch.add(api.stage_gemm(1.0, pact, gd, wt["Wd"], wd["Wd"], 0.0, None, out, desc(LPG_ROW_MAJOR, LPG_F32, t, hid)))
        return ch
    ch.add(api.stage_gemm(1.0, pattn, ad, wt["Wu"], wd["Wu"], 0.0, None, pu, gd))
    ch.add(api.stage_elementwise(LPG_EW_SILU_MUL, pg, pu, 0.0, pact, gd))
    ch.add(api.stage_gemm(1.0, pact, gd, wt["Wd"], wd["Wd"], 0.0, None, py, yd))
    ch.add(api.stage_unpack(py, yd, out, desc(LPG_ROW_MAJOR, LPG_F32, t, hid)))
    return ch


def build_linear_chain(x, weights, dtype=LPG_F32, fused=False):
    """X [m x k0] times weights[i] [k_i x k_{i+1}] in sequence (the DNN-style chains of section V:
    a few dependent GEMMs of unequal widths).  x and weights are numpy float32 arrays.  The result
    (fp32, row-major) is output "Y"; intermediates are buffers "C1", "C2", ..."""
    m = x.shape[0]
    widths = [x.shape[1]] + [w.shape[1] for w in weights]
    ch = Chain("linear_chain", {"m": m, "widths": widths}, sum(2 * m * a * b for a, b in zip(widths, widths[1:])))
    xs = ch.inputs["X"] = device_array(x)
    for i, w in enumerate(weights):
        ch.pack_weight(f"W{i}", w, LPG_PACKED_B, dtype)
    out = ch.outputs["Y"] = torch.empty((m, widths[-1]), dtype=torch.float32, device=_dev())
    rm_in = desc(LPG_ROW_MAJOR, LPG_F32, m, widths[0])
    rm_out = desc(LPG_ROW_MAJOR, LPG_F32, m, widths[-1])
    fuse_in = fused and dtype == LPG_F32 and widths[0] % 32 == 0
    cur, cur_d = xs, rm_in
    if not fuse_in:
        cur_d = desc(LPG_PACKED_A, dtype, m, widths[0])
        cur = ch.new_packed("C0", cur_d)
        ch.add(api.stage_pack(xs, rm_in, cur, cur_d))
    for i in range(len(weights)):
        last = i == len(weights) - 1
        if last and fused:
            nxt, nxt_d = out, rm_out
        else:
            nxt_d = desc(LPG_PACKED_A, LPG_F32 if last else dtype, m, widths[i + 1])
            nxt = ch.new_packed(f"C{i + 1}", nxt_d)
        ch.add(api.stage_gemm(1.0, cur, cur_d, ch.bufs[f"W{i}"][0], ch.bufs[f"W{i}"][1], 0.0, None, nxt, nxt_d))
        cur, cur_d = nxt, nxt_d
    if not fused:
        ch.add(api.stage_unpack(cur, cur_d, out, rm_out))
    return ch


def build_llama_layer(inp, shape, fused=False, flash=False, causal_blocks=1):
    """The decoder layer with every step between its GEMMs on the packed layout: RMSNorm, Q/K/V
    projections, RoPE on Q and K, causal softmax attention with grouped keys/values, output
    projection + residual, RMSNorm, gated MLP + residual.  bf16 intermediates, fp32 math.
    fused=True folds SiLU(gate)*up into the up projection's epilogue; flash=True runs the attention
    block as one lpg_attention_packed stage (no score matrix).  causal_blocks = n > 1 cuts the
    three attention stages into n blocks of t/n query rows, each a view of the same packed
    buffers that ends at the last key its rows may see: the blocks of S above the causal diagonal
    are then neither computed, nor normalised, nor multiplied (they only ever held zeros)."""
    t, hid, nq, nkv, ffn = shape["t"], shape["hidden"], shape["n_q"], shape["n_kv"], shape["ffn"]
    eps, base = 1.0 / shape["inv_eps"], float(shape["rope_base"])
    dh = hid // nq
    kvw = nkv * dh
    rep = nq // nkv
    if dh % 64:
        raise ValueError("bf16 head slices need head_dim to be a multiple of 64")
    flops = (2 * t * hid * (hid + 2 * kvw) + nq * 4 * t * t * dh + 2 * t * hid * hid + 3 * 2 * t * hid * ffn)
    ch = Chain("llama_layer", shape, flops)
    B = LPG_BF16
    x = ch.inputs["X"] = device_array(inp["X"])
    for nm in ("Wq", "Wk", "Wv", "Wo", "Wg", "Wu", "Wd"):
        ch.pack_weight(nm, inp[nm], LPG_PACKED_B, B)
    wd = {nm: ch.bufs[nm][1] for nm in ("Wq", "Wk", "Wv", "Wo", "Wg", "Wu", "Wd")}
    wt = {nm: ch.bufs[nm][0] for nm in wd}
    n1, n2 = device_array(inp["norm1"]), device_array(inp["norm2"])
    cos_t = torch.empty((t, dh // 2), dtype=torch.float32, device=_dev())
    sin_t = torch.empty_like(cos_t)
    api.lpg_rope_tables(cos_t, sin_t, t, dh, base, 0, _stream())          # constants of the model, like the weights
    torch.cuda.synchronize()
    ch.consts = (n1, n2, cos_t, sin_t)
    hd = desc(LPG_PACKED_A, B, t, hid)
    kd = desc(LPG_PACKED_A, B, t, kvw)          # K written as a left-operand image, read as K_g^T
    vd = desc(LPG_PACKED_B, B, t, kvw)
    gd = desc(LPG_PACKED_A, B, t, ffn)
    sd = desc(LPG_PACKED_A, B, t, t, batch=nq, batch_stride=_packed_elems(B, t, t))
    px, ph1, pq, po, pa, ph2, py = (ch.new_packed(n_, hd) for n_ in ("X", "h1", "Q", "O", "A", "h2", "Y"))
    pk, pv = ch.new_packed("K", kd), ch.new_packed("V", vd)
    ps = None if flash else ch.new_packed("S", sd)
    pg, pact = ch.new_packed("gate", gd), ch.new_packed("act", gd)
    out = ch.outputs["Y"] = torch.empty((t, hid), dtype=torch.float32, device=_dev())
    rm = desc(LPG_ROW_MAJOR, LPG_F32, t, hid)

    ch.add(api.stage_pack(x, rm, px, hd))
    ch.add(api.stage_rmsnorm(px, n1, ph1, hd, eps))
    ch.add(api.stage_gemm(1.0, ph1, hd, wt["Wq"], wd["Wq"], 0.0, None, pq, hd))
    ch.add(api.stage_gemm(1.0, ph1, hd, wt["Wk"], wd["Wk"], 0.0, None, pk, kd))
    ch.add(api.stage_gemm(1.0, ph1, hd, wt["Wv"], wd["Wv"], 0.0, None, pv, vd))
    ch.add(api.stage_rope(pq, pq, hd, cos_t, sin_t, dh))
    ch.add(api.stage_rope(pk, pk, kd, cos_t, sin_t, dh))
    q_view = desc(LPG_PACKED_A, B, t, dh, parent=(t, hid), batch=nq, batch_step=(0, dh))
    kt_view = desc(LPG_PACKED_B, B, dh, t, parent=(kvw, t), batch=nq, batch_div=rep, batch_step=(dh, 0))
    v_view = desc(LPG_PACKED_B, B, t, dh, parent=(t, kvw), batch=nq, batch_div=rep, batch_step=(0, dh))
    o_view = desc(LPG_PACKED_A, B, t, dh, parent=(t, hid), batch=nq, batch_step=(0, dh))
    if flash:
        ch.add(api.stage_attention(pq, q_view, pk, kt_view, pv, v_view, po, o_view, 1.0 / float(np.sqrt(dh)), True))
    elif causal_blocks > 1:
        rb = t // causal_blocks
        if t % causal_blocks or rb % 64:
            raise ValueError("causal_blocks must cut the rows into multiples of 64")
        selems = _packed_elems(B, t, t)
        for i in range(causal_blocks):
            r0, kc = i * rb, (i + 1) * rb              # query rows [r0, r0 + rb) see keys [0, kc)
            q_i = desc(LPG_PACKED_A, B, rb, dh, parent=(t, hid), origin=(r0, 0), batch=nq, batch_step=(0, dh))
            kt_i = desc(LPG_PACKED_B, B, dh, kc, parent=(kvw, t), batch=nq, batch_div=rep, batch_step=(dh, 0))
            s_i = desc(LPG_PACKED_A, B, rb, kc, parent=(t, t), origin=(r0, 0), batch=nq, batch_stride=selems)
            v_i = desc(LPG_PACKED_B, B, kc, dh, parent=(t, kvw), batch=nq, batch_div=rep, batch_step=(0, dh))
            o_i = desc(LPG_PACKED_A, B, rb, dh, parent=(t, hid), origin=(r0, 0), batch=nq, batch_step=(0, dh))
            ch.add(api.stage_gemm(1.0, pq, q_i, pk, kt_i, 0.0, None, ps, s_i))
            ch.add(api.stage_softmax(ps, ps, s_i, 1.0 / float(np.sqrt(dh)), True))
            ch.add(api.stage_gemm(1.0, ps, s_i, pv, v_i, 0.0, None, po, o_i))
    else:
        ch.add(api.stage_gemm(1.0, pq, q_view, pk, kt_view, 0.0, None, ps, sd))
        ch.add(api.stage_softmax(ps, ps, sd, 1.0 / float(np.sqrt(dh)), True))
        ch.add(api.stage_gemm(1.0, ps, sd, pv, v_view, 0.0, None, po, o_view))
    ch.add(api.stage_gemm(1.0, po, hd, wt["Wo"], wd["Wo"], 1.0, px, pa, hd))           # + residual X
    ch.add(api.stage_rmsnorm(pa, n2, ph2, hd, eps))
    ch.add(api.stage_gemm(1.0, ph2, hd, wt["Wg"], wd["Wg"], 0.0, None, pg, gd))
    if fused:
        ch.add(api.stage_gemm(1.0, ph2, hd, wt["Wu"], wd["Wu"], 0.0, None, pact, gd, api.LPG_EPI_GATE_SILU, pg))
    else:
        pu = ch.new_packed("up", gd)
        ch.add(api.stage_gemm(1.0, ph2, hd, wt["Wu"], wd["Wu"], 0.0, None, pu, gd))
        ch.add(api.stage_elementwise(LPG_EW_SILU_MUL, pg, pu, 0.0, pact, gd))
    ch.add(api.stage_gemm(1.0, pact, gd, wt["Wd"], wd["Wd"], 1.0, pa, py, hd))           # + residual A
    ch.add(api.stage_unpack(py, hd, out, rm))
    return ch


BUILDERS = {"llama_layer": build_llama_layer, "two_gemm": build_two_gemm, "mlp": build_mlp, "attention": build_attention,
            "deep_chain": build_deep_chain, "decoder_layer": build_decoder_layer}


def build(name, inp, shape, fused=False, **options):
    return BUILDERS[name](inp, shape, fused=fused, **options)
