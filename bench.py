#!/usr/bin/env python3
"""Benchmark of the layout-propagating GEMM chain on one MI355X.

A "step" is one pass of the whole hot path over one batch of synthetic input:
pack the activations, run every GEMM of the chain with intermediates kept packed,
unpack the result (weights are packed once, outside the timed region).  Inputs are
resident in HBM before timing starts.

Prints ONE JSON line.  `value` is the chained-GEMM throughput (GEMM flops only) of
the headline workload (the MLP-like fp32 chain); `workloads` carries the same
measurement for all five workloads, each with the canonical-layout control chain
timed beside it.  `roofline` is the fp32 MFMA GEMM kernel's own rate from HIP event
pairs around every one of its launches; `cpu_baseline` times the CPU oracle on a
bounded row sample of the same workload.
"""
import argparse
import json
import os
import statistics
import sys
import time

import numpy as np

PEAK_TFLOPS = {"f32": 157.3, "bf16": 2516.6}     # dense MFMA, MI355X (256 CU x 2.4 GHz)
# HBM bytes per fp32 GEMM launch of the headline chain, from profiles/hbm_traffic_mlp_chain.txt:
# FETCH_SIZE (x2.0 calibration) 64.3 and 136.3 MiB, WRITE_SIZE (x1.0) 32 and 8 MiB for the two
# launches of a step -> mean 120.3 MiB; the algorithmic bytes are 56 and 64 MiB.
GEMM_TRAFFIC_BYTES = 120.3 * 2 ** 20
GEMM_ALGORITHMIC_BYTES = 60.0 * 2 ** 20
HEADLINE = "mlp"


SETTLE_SECONDS = 0.05


def settle(ch, mode, seconds=None):
    """Set-up, before any warm-up or timed step: run the chain for ~50 ms once per chain and mode
    so that the device's clocks and the first-launch costs (code upload, LDS size attributes) are
    behind it.  Without it the first few milliseconds of a run measure the clock ramp: the same
    20 timed steps read 0.33 ms per step straight after start-up and 0.28 ms from then on."""
    import torch
    seconds = SETTLE_SECONDS if seconds is None else seconds
    done = ch.__dict__.setdefault("_settled_modes", set())
    if mode in done:
        return
    done.add(mode)
    t0 = time.perf_counter()
    while time.perf_counter() - t0 < seconds:
        for _ in range(4):
            ch.run(mode)
        torch.cuda.synchronize()


def time_chain(ch, mode, steps, warmup):
    import torch
    settle(ch, mode)
    for _ in range(warmup):
        ch.run(mode)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        ch.run(mode)
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / max(steps, 1)


def compare_modes(ch, steps, blocks=6):
    """Propagated and canonical chains timed in alternating blocks (so that clock and cache
    state drift hits both alike); returns the median per-step seconds of each mode."""
    import statistics
    from paper_2604_04599_amd import api
    per = max(1, steps // blocks)
    tp, tc = [], []
    for _ in range(blocks):
        tp.append(time_chain(ch, api.LPG_CHAIN_PROPAGATED, per, 1))
        tc.append(time_chain(ch, api.LPG_CHAIN_CANONICAL, per, 1))
    return statistics.median(tp), statistics.median(tc)


def time_gemm_launches(ch, steps):
    """Average duration of one GEMM kernel launch of the chain: every stage is issued
    through its own C-ABI call on torch's current stream, with an event pair around
    each GEMM launch.  Returns (seconds per GEMM launch, flops per GEMM launch)."""
    import torch
    from paper_2604_04599_amd import api
    st = torch.cuda.current_stream().cuda_stream
    pairs = []
    nflops = 0
    ngemm = 0
    for it in range(steps):
        for s in ch.stages:
            if s.type == api.LPG_STAGE_GEMM:
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                api.lpg_chain([s], api.LPG_CHAIN_PROPAGATED, None, 0, st)
                e1.record()
                pairs.append((e0, e1))
                if it == 0:
                    nb = max(s.out_d.batch, 1)
                    nflops += 2 * s.in0_d.rows * s.in0_d.cols * s.in1_d.cols * nb
                    ngemm += 1
            else:
                api.lpg_chain([s], api.LPG_CHAIN_PROPAGATED, None, 0, st)
    torch.cuda.synchronize()
    total_ms = sum(a.elapsed_time(b) for a, b in pairs)
    return total_ms * 1e-3 / len(pairs), nflops / ngemm


STAGE_NAMES = {0: "pack", 1: "gemm", 2: "elementwise", 3: "unpack", 4: "softmax", 5: "rmsnorm", 6: "rope", 7: "attention"}


def stage_breakdown(ch, steps):
    """Per stage of the chain (propagated mode, each stage issued through its own lpg_chain call
    with an event pair around it): median microseconds, and the rate it stands for: GEMM flops and
    algorithmic bytes ((m*k + k*n + m*n (+ m*n with beta)) * element size per matrix of the
    batch); other stages the bytes they read and write once."""
    import torch
    from paper_2604_04599_amd import api
    st = torch.cuda.current_stream().cuda_stream
    es = api.ELEM_SIZE
    pairs = [[] for _ in ch.stages]
    for _ in range(steps):
        for i, s in enumerate(ch.stages):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            api.lpg_chain([s], api.LPG_CHAIN_PROPAGATED, None, 0, st)
            e1.record()
            pairs[i].append((e0, e1))
    torch.cuda.synchronize()
    out = []
    for i, s in enumerate(ch.stages):
        us = statistics.median(a.elapsed_time(b) for a, b in pairs[i]) * 1e3
        o = s.out_d
        nb = max(o.batch, 1)
        row = {"stage": i, "kind": STAGE_NAMES[s.type], "us": round(us, 2)}
        if s.type == api.LPG_STAGE_GEMM:
            m, k, n = s.in0_d.rows, s.in0_d.cols, s.in1_d.cols
            nbytes = nb * ((m * k * es[s.in0_d.dtype]) // max(s.in0_d.batch_div, 1)
                           + (k * n * es[s.in1_d.dtype]) // max(s.in1_d.batch_div, 1)
                           + m * n * es[o.dtype] * (2 if s.beta != 0 else 1))
            row.update({"m": m, "n": n, "k": k, "batch": nb, "tflops": round(2.0 * m * n * k * nb / us / 1e6, 1)})
        elif s.type in (api.LPG_STAGE_PACK, api.LPG_STAGE_UNPACK):
            nbytes = nb * o.rows * o.cols * (es[s.in0_d.dtype] + es[o.dtype])
        elif s.type == api.LPG_STAGE_ELEMENTWISE:
            nbytes = nb * o.rows * o.cols * es[o.dtype] * (3 if s.in1 else 2)
        elif s.type == api.LPG_STAGE_SOFTMAX:
            r, c = o.rows, o.cols
            kept = r * c if not s.op else sum(min(c, max(0, j + c - r + 1)) for j in range(r))
            nbytes = nb * (kept + r * c) * es[o.dtype]
        elif s.type == api.LPG_STAGE_ATTENTION:
            tq, dh, tk = o.rows, o.cols, s.in2_d.rows
            pairs_kept = tq * tk if not (s.op & 1) else sum(min(tk, max(0, j + tk - tq + 1)) for j in range(tq))
            nbytes = nb * (2 * tq * dh + 2 * tk * dh // max(s.in1_d.batch_div, 1)) * es[o.dtype]
            row.update({"queries": tq, "keys": tk, "head_dim": dh, "batch": nb,
                        "tflops": round(4.0 * pairs_kept * dh * nb / us / 1e6, 1)})
        else:
            nbytes = nb * o.rows * o.cols * es[o.dtype] * 2
        row["hbm_gbps"] = round(nbytes / us / 1e3, 1)
        out.append(row)
    return out


def time_softmax_launches(ch, steps):
    """Average duration of the chain's softmax launch (event pair around each), with the bytes
    it has to move: the kept scores read once, the whole score matrix written once."""
    import torch
    from paper_2604_04599_amd import api
    st = torch.cuda.current_stream().cuda_stream
    pairs = []
    nbytes = 0
    for it in range(steps):
        for s in ch.stages:
            if s.type != api.LPG_STAGE_SOFTMAX:
                api.lpg_chain([s], api.LPG_CHAIN_PROPAGATED, None, 0, st)
                continue
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            api.lpg_chain([s], api.LPG_CHAIN_PROPAGATED, None, 0, st)
            e1.record()
            pairs.append((e0, e1))
            if it == 0:
                d = s.out_d
                r, c, nb = d.rows, d.cols, max(d.batch, 1)
                kept = r * c if not s.op else sum(min(c, max(0, i + c - r + 1)) for i in range(r))
                nbytes += (kept + r * c) * nb * api.ELEM_SIZE[d.dtype]
    torch.cuda.synchronize()
    t = sum(a.elapsed_time(b) for a, b in pairs) * 1e-3 / len(pairs)
    return t, nbytes


def measure(name, steps, warmup, shape_over=None, modes="both", options=None):
    from paper_2604_04599_amd import api, chains, inputs
    options = options or {}
    inp, shape = inputs.make(name, **(shape_over or {}))
    ch = chains.build(name, inp, shape, **options)
    flops = inputs.gemm_flops(name, shape)
    dt = inputs.DTYPES[name]
    res = {"dtype": dt, "shape": shape, "gemm_gflop": round(flops / 1e9, 3)}
    t_prop = t_canon = None
    if modes in ("both", "propagated"):
        t_prop = time_chain(ch, api.LPG_CHAIN_PROPAGATED, steps, warmup)
        tf = flops / t_prop / 1e12
        res.update({"ms_per_step": round(t_prop * 1e3, 4), "tflops": round(tf, 2),
                    "pct_mfma_peak": round(100 * tf / PEAK_TFLOPS[dt], 2)})
    if modes == "canonical":
        t_canon = time_chain(ch, api.LPG_CHAIN_CANONICAL, steps, warmup)
        res["canonical_ms_per_step"] = round(t_canon * 1e3, 4)
    if modes == "both":
        time_chain(ch, api.LPG_CHAIN_CANONICAL, 0, warmup)
        mp, mc = compare_modes(ch, max(steps, 12))
        res["canonical_ms_per_step"] = round(mc * 1e3, 4)
        res["propagated_ms_per_step_interleaved"] = round(mp * 1e3, 4)
        res["speedup_vs_canonical"] = round(mc / mp, 3)
        # the same chain with the entry pack / exit unpack fused into the first / last GEMM
        fch = chains.build(name, inp, shape, fused=True, **options)
        t_f = time_chain(fch, api.LPG_CHAIN_PROPAGATED, steps, warmup)
        res["fused_boundaries_ms_per_step"] = round(t_f * 1e3, 4)
        res["fused_boundaries_tflops"] = round(flops / t_f / 1e12, 2)
        del fch
        if name in ("llama_layer", "attention", "decoder_layer") and not options.get("flash"):
            # the attention block as one kernel that keeps the scores in registers
            ach = chains.build(name, inp, shape, flash=True, **options)
            t_a = time_chain(ach, api.LPG_CHAIN_PROPAGATED, steps, warmup)
            res["fused_attention_ms_per_step"] = round(t_a * 1e3, 4)
            res["fused_attention_tflops"] = round(flops / t_a / 1e12, 2)
            res["fused_attention_stages"] = stage_breakdown(ach, max(3, steps // 2))
            del ach
            if name != "attention":   # (the attention kernel itself takes packed operands only)
                # both: fused attention kernel, boundary pack / unpack and SiLU(gate)*up inside GEMMs
                bch = chains.build(name, inp, shape, fused=True, flash=True, **options)
                t_b = time_chain(bch, api.LPG_CHAIN_PROPAGATED, steps, warmup)
                res["fused_attention_and_boundaries_ms_per_step"] = round(t_b * 1e3, 4)
                res["fused_attention_and_boundaries_tflops"] = round(flops / t_b / 1e12, 2)
                del bch
        res["stages"] = stage_breakdown(ch, max(3, steps // 2))
        if name == "two_gemm":
            # launch-bound: the same chain replayed from a HIP graph
            replay = ch.capture(api.LPG_CHAIN_PROPAGATED)
            res["graph_replay_ms_per_step"] = round(_time_calls(replay, max(steps, 20)) * 1e3, 4)
    return res, ch, inp, shape


def cpu_baseline(inp, shape, budget_s=15.0):
    """The CPU oracle, as it stands, on the first R rows of the MLP-like chain."""
    from oracle import ref, workloads
    m = shape["m"]
    per_row = 2 * 2 * shape["d"] * shape["h"]
    probe = min(m, 256)
    t0 = time.perf_counter()
    workloads.mlp(inp, rows=np.arange(probe))
    dt = time.perf_counter() - t0
    rate = probe * per_row / dt
    rows = int(min(m, max(probe, budget_s * rate / per_row)))
    t0 = time.perf_counter()
    workloads.mlp(inp, rows=np.arange(rows))
    dt = time.perf_counter() - t0
    # when the whole sample takes well under the budget it is repeated, so that the figure rests on
    # about ten seconds of CPU work rather than on one short run
    reps = 1
    if dt < 5.0:
        extra = int(min(63, max(0, 10.0 / max(dt, 1e-3) - 1)))
        t0 = time.perf_counter()
        for _ in range(extra):
            workloads.mlp(inp, rows=np.arange(rows))
        dt += time.perf_counter() - t0
        reps += extra
    return {"value": round(reps * rows * per_row / dt / 1e12, 5), "unit": "TFLOP/s", "cores": ref.threads(),
            "kind": "oracle", "seconds": round(dt, 2),
            "sample": f"first {rows} of {m} rows of X through both GEMMs of the MLP-like chain "
                      f"(fp64 triple loop, OpenMP over rows), {reps} time(s)"}


SWEEP_GEMMS = [(n, n, n) for n in (256, 512, 1024, 2048, 4096, 8192)] + [
    (4096, 256, 4096), (4096, 4096, 256), (256, 4096, 4096), (16384, 1024, 1024), (1024, 16384, 1024),
    (1000, 1000, 1000), (4100, 2050, 1030)]
SWEEP_CHAINS = [(256, (512, 512, 512, 512)), (1024, (1024, 4096, 1024, 256)), (1024, (256, 1024, 4096, 1024)),
                (4096, (2048, 2048, 2048, 2048)), (4096, (1024, 4096, 1024, 4096)), (4096, (4096, 512, 4096, 512)),
                (8192, (1024, 1024, 1024, 1024)), (1000, (1000, 3000, 1000, 300))]


def _time_calls(fn, reps, min_seconds=0.03):
    """Seconds per call.  Small cases get more than `reps` calls: a measurement shorter than some
    tens of milliseconds sees the clocks of an idle device, not those of a loaded one."""
    import torch
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(2):
        fn()
    e1.record()
    torch.cuda.synchronize()
    per_call = max(e0.elapsed_time(e1) * 1e-3 / 2, 1e-6)
    reps = max(reps, min(2000, int(min_seconds / per_call)))
    for _ in range(reps // 2):
        fn()
    e0.record()
    for _ in range(reps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e-3 / reps


def sweep(reps):
    """Synthetic size sweep (the paper's single-GEMM and DNN-chain size lists are not available):
    (1) one GEMM M x K x N (fp32, then bf16 operands) with a pre-packed weight, as the Initial kernel (row-major A in,
    packed C out), the Intermediate kernel (packed in, packed out), the Ending kernel (packed in,
    row-major out) and as a BLAS-style call (pack A + GEMM + unpack C; the Initial kernel exists for fp32 only); (2) three-GEMM chains of
    unequal widths, propagated against the canonical control.  One JSON line per case."""
    import torch
    from paper_2604_04599_amd import api, chains
    from paper_2604_04599_amd.api import LPG_F32, LPG_PACKED_A, LPG_PACKED_B, LPG_ROW_MAJOR, desc
    st = torch.cuda.current_stream().cuda_stream
    rng = np.random.default_rng(2024)
    for dtype, tag in ((LPG_F32, "f32"), (api.LPG_BF16, "bf16")):
        for m, k, n in SWEEP_GEMMS:
            a = torch.from_numpy(rng.standard_normal((m, k), dtype=np.float32)).cuda()
            w = torch.from_numpy(rng.standard_normal((k, n), dtype=np.float32)).cuda()
            a_rm, w_rm, c_rm = (desc(LPG_ROW_MAJOR, LPG_F32, r, c) for r, c in ((m, k), (k, n), (m, n)))
            a_p, w_p, c_p = desc(LPG_PACKED_A, dtype, m, k), desc(LPG_PACKED_B, dtype, k, n), desc(LPG_PACKED_A, dtype, m, n)
            pa, pw, pc = (torch.empty(api.lpg_packed_bytes(d), dtype=torch.uint8, device="cuda") for d in (a_p, w_p, c_p))
            c = torch.empty((m, n), dtype=torch.float32, device="cuda")
            api.lpg_pack(a, a_rm, pa, a_p, st)
            api.lpg_pack(w, w_rm, pw, w_p, st)
            flops = 2.0 * m * k * n
            res = {"sweep": "gemm_" + tag, "m": m, "k": k, "n": n}
            if k % 32 == 0 and dtype == LPG_F32:
                res["initial_tflops"] = round(flops / _time_calls(
                    lambda: api.lpg_gemm_packed(1.0, a, a_rm, pw, w_p, 0.0, None, pc, c_p, stream=st), reps) / 1e12, 2)
            res["intermediate_tflops"] = round(flops / _time_calls(
                lambda: api.lpg_gemm_packed(1.0, pa, a_p, pw, w_p, 0.0, None, pc, c_p, stream=st), reps) / 1e12, 2)
            res["ending_tflops"] = round(flops / _time_calls(
                lambda: api.lpg_gemm_packed(1.0, pa, a_p, pw, w_p, 0.0, None, c, c_rm, stream=st), reps) / 1e12, 2)

            def blas_style():
                api.lpg_pack(a, a_rm, pa, a_p, st)
                api.lpg_gemm_packed(1.0, pa, a_p, pw, w_p, 0.0, None, pc, c_p, stream=st)
                api.lpg_unpack(pc, c_p, c, c_rm, st)
            res["pack_gemm_unpack_tflops"] = round(flops / _time_calls(blas_style, reps) / 1e12, 2)
            res["intermediate_vs_pack_gemm_unpack"] = round(res["intermediate_tflops"] / res["pack_gemm_unpack_tflops"], 3)
            print(json.dumps(res), flush=True)
            del a, w, pa, pw, pc, c
    for m, widths in SWEEP_CHAINS:
        x = rng.standard_normal((m, widths[0]), dtype=np.float32)
        ws = [rng.standard_normal((a, b), dtype=np.float32) / np.float32(np.sqrt(a)) for a, b in zip(widths, widths[1:])]
        ch = chains.build_linear_chain(x, ws)
        fch = chains.build_linear_chain(x, ws, fused=True)
        est = max(time_chain(ch, api.LPG_CHAIN_PROPAGATED, 3, 2), 1e-6)
        steps = max(6 * reps, min(6000, int(0.15 / est)))          # long enough for loaded clocks
        tp, tc = compare_modes(ch, steps)
        tf = time_chain(fch, api.LPG_CHAIN_PROPAGATED, max(reps, steps // 6), 2)
        print(json.dumps({"sweep": "chain3_f32", "m": m, "widths": list(widths),
                          "propagated_ms": round(tp * 1e3, 4), "canonical_ms": round(tc * 1e3, 4),
                          "fused_boundaries_ms": round(tf * 1e3, 4), "speedup_vs_canonical": round(tc / tp, 3),
                          "tflops": round(ch.flops / tp / 1e12, 2)}), flush=True)
        del ch, fch
        torch.cuda.empty_cache()


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workloads", default="all",
                    help="comma list of extra workloads to report beside the headline (the five configs' names, "
                         "attention_softmax, llama_layer), 'all' or 'none'")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--only", default=None,
                    help="profiling aid: time just this workload (a workload name, attention_softmax_causal, "
                         "llama_layer or llama_layer_fused_attention) and print its line")
    ap.add_argument("--mode", default="both", choices=["both", "propagated", "canonical"],
                    help="with --only: which chain mode(s) to run")
    ap.add_argument("--settle-ms", type=float, default=50.0,
                    help="set-up run of each chain before its warm-up steps, in milliseconds (0 for counter "
                         "collection runs, where every extra launch is paid for)")
    ap.add_argument("--sweep", action="store_true",
                    help="run the synthetic single-GEMM / three-GEMM-chain size sweep instead (--steps = "
                         "repetitions per case) and print one JSON line per case")
    ap.add_argument("--gemm", default=None, metavar="M,N,K,DTYPE",
                    help="profiling aid: run one packed-in, packed-out GEMM C[MxN] = A[MxK] B[KxN] (DTYPE f32 or "
                         "bf16) --steps times and print its rate")
    ap.add_argument("--gemm-data", default="zeros", choices=["zeros", "randn"],
                    help="with --gemm: operand values (the bf16 rate depends on them through the clock)")
    ap.add_argument("--gemm-seconds", type=float, default=0.0,
                    help="with --gemm: instead of --steps launches, run back to back for this long and sample "
                         "rocm-smi's shader clock every 0.3 s meanwhile")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="MIB",
                    help="profiling aid: run the elementwise SCALE kernel over a buffer of MIB MiB "
                         "(reads MIB, writes MIB per launch) --steps times, to scale HBM counters")
    ap.add_argument("--probe", action="store_true",
                    help="run the stand-alone main-loop probe (MFMA-only rates and the bf16 step rebuilt piece by "
                         "piece; csrc/probe_mainloop.hip) and print its lines")
    args = ap.parse_args()
    global SETTLE_SECONDS
    SETTLE_SECONDS = args.settle_ms * 1e-3
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    if args.probe:
        # a child process of its own: nothing here has touched the GPU yet
        import subprocess
        exe = os.path.join(os.path.dirname(os.path.abspath(__file__)), "paper_2604_04599_amd", "probe_mainloop")
        if not os.path.exists(exe):
            print("bench.py: probe not built (python -c 'import __graft_entry__ as g; g.build()')", file=sys.stderr)
            sys.exit(1)
        sys.exit(subprocess.run([exe]).returncode)

    import torch
    if not torch.cuda.is_available():
        print("bench.py: needs a GPU (the HIP library has no CPU fallback)", file=sys.stderr)
        sys.exit(1)
    torch.cuda.set_device(0)
    from paper_2604_04599_amd import inputs

    if args.sweep:
        sweep(max(args.steps, 5))
        return

    if args.gemm:
        from paper_2604_04599_amd import api
        m, n, k, dt = args.gemm.split(",")
        m, n, k = int(m), int(n), int(k)
        dtype = {"f32": api.LPG_F32, "bf16": api.LPG_BF16}[dt]
        a_p, w_p, c_p = (api.desc(kind, dtype, r, c) for kind, r, c in
                         ((api.LPG_PACKED_A, m, k), (api.LPG_PACKED_B, k, n), (api.LPG_PACKED_A, m, n)))
        pa, pw, pc = (torch.zeros(api.lpg_packed_bytes(d), dtype=torch.uint8, device="cuda") for d in (a_p, w_p, c_p))
        if args.gemm_data == "randn":   # a permutation of i.i.d. values is i.i.d.: fill the packed buffers directly
            tdt = torch.float32 if dt == "f32" else torch.bfloat16
            torch.manual_seed(7)
            pa.view(tdt).copy_(torch.randn(pa.numel() // pa.view(tdt).element_size(), device="cuda").to(tdt))
            pw.view(tdt).copy_((torch.randn(pw.numel() // pw.view(tdt).element_size(), device="cuda") / k ** 0.5).to(tdt))
        st = torch.cuda.current_stream().cuda_stream
        call = lambda: api.lpg_gemm_packed(1.0, pa, a_p, pw, w_p, 0.0, None, pc, c_p, stream=st)
        if args.gemm_seconds > 0:
            import re
            import subprocess
            import threading
            clocks, stop = [], threading.Event()

            def sample():
                while not stop.wait(0.3):
                    out = subprocess.run(["rocm-smi", "--showclocks"], capture_output=True, text=True).stdout
                    clocks.extend(int(x) for x in re.findall(r"sclk clock level: \d+: \((\d+)Mhz\)", out)[:1])
            for _ in range(20):
                call()
            torch.cuda.synchronize()
            th = threading.Thread(target=sample)
            th.start()
            t0, n_it = time.perf_counter(), 0
            while time.perf_counter() - t0 < args.gemm_seconds:
                for _ in range(50):
                    call()
                torch.cuda.synchronize()
                n_it += 50
            t = (time.perf_counter() - t0) / n_it
            stop.set()
            th.join()
            print(json.dumps({"gemm": args.gemm, "data": args.gemm_data, "us": round(t * 1e6, 2),
                              "tflops": round(2.0 * m * n * k / t / 1e12, 2), "sclk_mhz": clocks}))
            return
        t = _time_calls(call, args.steps)
        print(json.dumps({"gemm": args.gemm, "data": args.gemm_data, "us": round(t * 1e6, 2),
                          "tflops": round(2.0 * m * n * k / t / 1e12, 2)}))
        return

    if args.copy_calibration:
        from paper_2604_04599_amd import api
        n = args.copy_calibration << 20
        x = torch.zeros(n, dtype=torch.uint8, device="cuda")
        y = torch.empty_like(x)
        d = api.desc(api.LPG_ROW_MAJOR, api.LPG_F32, n // 4096, 1024)
        for _ in range(args.steps):
            api.lpg_elementwise_packed(api.LPG_EW_SCALE, x, None, 1.0, y, d, torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration_mib": args.copy_calibration, "launches": args.steps}))
        return

    if args.only:
        name, options = args.only, None
        if name == "attention_softmax_causal":
            name, options = "attention", {"softmax": True, "causal": True}
        elif name == "llama_layer_fused_attention":
            name, options = "llama_layer", {"flash": True}
        res, _, _, _ = measure(name, args.steps, args.warmup, modes=args.mode, options=options)
        print(json.dumps({"workload": args.only, **res}))
        return

    head, ch, inp, shape = measure(HEADLINE, args.steps, args.warmup)
    t_gemm, gemm_flops = time_gemm_launches(ch, args.steps)
    achieved = gemm_flops / t_gemm / 1e12
    roofline = {"bound": "mfma", "kernel": "gemm_kernel<F32,F32>", "achieved": round(achieved, 2),
                "peak": PEAK_TFLOPS["f32"], "unit": "TFLOP/s", "frac": round(achieved / PEAK_TFLOPS["f32"], 4),
                "avg_launch_us": round(t_gemm * 1e6, 2), "flops_per_launch": gemm_flops,
                "traffic": GEMM_TRAFFIC_BYTES, "algorithmic_bytes": GEMM_ALGORITHMIC_BYTES,
                "traffic_unit": "HBM bytes per launch (rocprofv3 FETCH_SIZE + WRITE_SIZE, calibrated)"}

    if args.workloads == "all":
        names = [w for w in inputs.WORKLOADS if w != HEADLINE]
    elif args.workloads == "none":
        names = []
    else:
        names = [w for w in args.workloads.split(",") if w in inputs.WORKLOADS and w != HEADLINE]
    per = {HEADLINE: head}
    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(inp, shape)
    del ch
    torch.cuda.empty_cache()
    for w in names:
        steps = args.steps if w != "deep_chain" else max(3, args.steps // 4)
        res, c2, _, _ = measure(w, steps, min(args.warmup, steps))
        per[w] = res
        del c2
        torch.cuda.empty_cache()

    if args.workloads == "all" or "attention_softmax" in args.workloads.split(","):
        # the attention chain with the scale + causal mask + softmax stage between its GEMMs,
        # run on the packed scores (propagated) or on their row-major copy (canonical control)
        res, c2, _, _ = measure("attention", args.steps, args.warmup, options={"softmax": True, "causal": True})
        t_sm, sm_bytes = time_softmax_launches(c2, args.steps)
        res["softmax_kernel"] = {"bound": "hbm", "achieved": round(sm_bytes / t_sm / 1e9, 1), "peak": 8000.0,
                                 "unit": "GB/s", "frac": round(sm_bytes / t_sm / 8e12, 4),
                                 "avg_launch_us": round(t_sm * 1e6, 2), "algorithmic_bytes": sm_bytes}
        per["attention_softmax_causal"] = res
        del c2
        torch.cuda.empty_cache()

    if args.workloads == "all" or "llama_layer" in args.workloads.split(","):
        # the decoder layer with RMSNorm, RoPE, causal softmax and both residuals between its GEMMs
        res, c2, _, _ = measure("llama_layer", args.steps, args.warmup)
        per["llama_layer"] = res
        del c2
        torch.cuda.empty_cache()

    out = {"metric": "chained_gemm_tflops", "value": head["tflops"], "unit": "TFLOP/s", "n_gpus": 1,
           "steps": args.steps, "warmup": args.warmup, "ms_per_step": head["ms_per_step"],
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32",
           "data": "synthetic",
           "config": {"workload": "MLP-like fp32 chain: X[2048x1024]*W1[1024x4096] -> H kept packed, "
                                  "then H*W2[4096x1024] + 1*X; pack X at entry, unpack Y at exit",
                      "shape": shape, "mode": "propagated"},
           "pct_mfma_peak": head["pct_mfma_peak"],
           "speedup_vs_canonical": head["speedup_vs_canonical"],
           "roofline": roofline, "cpu_baseline": cpu, "workloads": per,
           "context": "paper: 2.25x average over OpenBLAS for sequential GEMMs on a Xeon Gold 6252 "
                      "(AVX-512, 1 thread); other hardware, not a target"}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
