#!/usr/bin/env python3
"""Benchmark of the layout-propagating GEMM chain on one MI355X.

A "step" is one pass of the whole hot path over one batch of synthetic input:
pack the activations, run every GEMM of the chain with intermediates kept packed,
unpack the result (weights are packed once, outside the timed region).  Inputs are
resident in HBM before timing starts.

Prints ONE JSON line.  `value` is the chained-GEMM throughput (GEMM flops only) of
the headline workload, the deep fp32 chain of eight dependent 4096^3 GEMMs (the
largest fp32 configuration); `workloads` carries a compact record for all five
configurations, each with the canonical-layout control chain timed beside it, every
chain for at least half a second.  `roofline` is the fp32 MFMA GEMM kernel's own rate from
HIP event pairs around every one of its launches on the launch stream; `cpu_baseline`
times the CPU oracle on a bounded row sample of the same chain.  `--stages` adds the
per-stage lists.
"""
import argparse
import json
import os
import re
import statistics
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
PEAK_TFLOPS = {"f32": 157.3, "bf16": 2516.6}     # dense MFMA, MI355X (256 CU x 2.4 GHz)
HBM_PEAK_GBPS = 8000.0
# What MFMAs alone sustain on this part with bf16 operands that are not all zero: operands
# uniform in [-1, 1), kept in registers, no memory traffic, 1.76-1.83 PFLOP/s steady over seconds (the
# shader clock falls to 1.8-2.0 GHz under the power limit; on zeros the same loop runs at 2.49).
BF16_POWER_LIMITED_TFLOPS = 1830.0
HEADLINE = "deep_chain"
HEADLINE_TEXT = ("deep fp32 chain: 8 dependent GEMMs C_{i+1} = C_i*B_i, N=4096, alternating packed-A / packed-B "
                 "consumption; pack C_0 at entry, unpack C_8 at exit")
MIN_SECONDS = 0.5          # every chain and mode is timed for at least this long


SETTLE_SECONDS = 0.05


def settle(ch, mode, seconds=None):
    """Set-up, before any warm-up or timed step: run the chain for ~50 ms once per chain and mode
    so that the device's clocks and the first-launch costs (code upload, LDS size attributes) are
    behind it.  Without it the first few milliseconds of a run measure the clock ramp."""
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
    """Seconds per step over exactly `steps` steps, synchronised on both sides."""
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


def time_for(ch, mode, min_seconds=None, blocks=5):
    """Per-step seconds of one mode over at least `min_seconds` of back-to-back steps, in `blocks`
    blocks: returns (median of the blocks, mean over all steps, steps run)."""
    min_seconds = MIN_SECONDS if min_seconds is None else min_seconds
    est = max(time_chain(ch, mode, 3, 2), 1e-6)
    per = max(2, int(min_seconds / blocks / est) + 1)
    ts = [time_chain(ch, mode, per, 0) for _ in range(blocks)]
    return statistics.median(ts), sum(ts) / len(ts), per * blocks


def compare_modes(ch, min_seconds=None, blocks=5):
    """Propagated and canonical chains timed in alternating blocks (so that clock and cache
    state drift hits both alike), each mode for at least `min_seconds` in total; returns per mode
    (median of the blocks, mean over all steps, steps run)."""
    from paper_2604_04599_amd import api
    min_seconds = MIN_SECONDS if min_seconds is None else min_seconds
    out = {}
    pers = {}
    for mode in (api.LPG_CHAIN_PROPAGATED, api.LPG_CHAIN_CANONICAL):
        est = max(time_chain(ch, mode, 3, 2), 1e-6)
        pers[mode] = max(2, int(min_seconds / blocks / est) + 1)
        out[mode] = []
    for _ in range(blocks):
        for mode in pers:
            out[mode].append(time_chain(ch, mode, pers[mode], 0))
    return {m: (statistics.median(t), sum(t) / len(t), pers[m] * blocks) for m, t in out.items()}


def time_gemm_launches(ch, steps):
    """Average duration of one GEMM kernel launch of the chain: every stage is issued
    through its own C-ABI call on torch's current stream (the stream the kernels are launched
    on), with an event pair around each GEMM launch.  Returns (seconds per GEMM launch, flops
    per GEMM launch, algorithmic bytes per GEMM launch)."""
    import torch
    from paper_2604_04599_amd import api
    st = torch.cuda.current_stream().cuda_stream
    pairs = []
    nflops = nbytes = ngemm = 0
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
                    nbytes += stage_bytes(s)
                    ngemm += 1
            else:
                api.lpg_chain([s], api.LPG_CHAIN_PROPAGATED, None, 0, st)
    torch.cuda.synchronize()
    total_ms = sum(a.elapsed_time(b) for a, b in pairs)
    return total_ms * 1e-3 / len(pairs), nflops / ngemm, nbytes / ngemm


STAGE_NAMES = {0: "pack", 1: "gemm", 2: "elementwise", 3: "unpack", 4: "softmax", 5: "rmsnorm", 6: "rope", 7: "attention"}


def stage_bytes(s):
    """Algorithmic bytes of one stage: what it must read and write once.  GEMM:
    (m*k + k*n + m*n (+ m*n with beta)) * element size per matrix of the batch, shared operands
    counted once per sharing group; other stages the bytes they read and write once."""
    from paper_2604_04599_amd import api
    es = api.ELEM_SIZE
    o = s.out_d
    nb = max(o.batch, 1)
    if s.type == api.LPG_STAGE_GEMM:
        m, k, n = s.in0_d.rows, s.in0_d.cols, s.in1_d.cols
        return nb * ((m * k * es[s.in0_d.dtype]) // max(s.in0_d.batch_div, 1)
                     + (k * n * es[s.in1_d.dtype]) // max(s.in1_d.batch_div, 1)
                     + m * n * es[o.dtype] * (2 if s.beta != 0 else 1))
    if s.type in (api.LPG_STAGE_PACK, api.LPG_STAGE_UNPACK):
        return nb * o.rows * o.cols * (es[s.in0_d.dtype] + es[o.dtype])
    if s.type == api.LPG_STAGE_ELEMENTWISE:
        return nb * o.rows * o.cols * es[o.dtype] * (3 if s.in1 else 2)
    if s.type == api.LPG_STAGE_SOFTMAX:
        r, c = o.rows, o.cols
        kept = r * c if not s.op else sum(min(c, max(0, j + c - r + 1)) for j in range(r))
        return nb * (kept + r * c) * es[o.dtype]
    if s.type == api.LPG_STAGE_ATTENTION:
        tq, dh, tk = o.rows, o.cols, s.in2_d.rows
        return nb * (2 * tq * dh + 2 * tk * dh // max(s.in1_d.batch_div, 1)) * es[o.dtype]
    return nb * o.rows * o.cols * es[o.dtype] * 2


def stage_breakdown(ch, steps):
    """Per stage of the chain (propagated mode, each stage issued through its own lpg_chain call
    with an event pair around it): median microseconds, and the rate it stands for."""
    import torch
    from paper_2604_04599_amd import api
    st = torch.cuda.current_stream().cuda_stream
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
            row.update({"m": m, "n": n, "k": k, "batch": nb, "tflops": round(2.0 * m * n * k * nb / us / 1e6, 1)})
        elif s.type == api.LPG_STAGE_ATTENTION:
            tq, dh, tk = o.rows, o.cols, s.in2_d.rows
            pairs_kept = tq * tk if not (s.op & 1) else sum(min(tk, max(0, j + tk - tq + 1)) for j in range(tq))
            row.update({"queries": tq, "keys": tk, "head_dim": dh, "batch": nb,
                        "tflops": round(4.0 * pairs_kept * dh * nb / us / 1e6, 1)})
        row["hbm_gbps"] = round(stage_bytes(s) / us / 1e3, 1)
        out.append(row)
    return out


def score_gemm_rates(ch, stages):
    """The two GEMMs around the score matrix S of an attention-shaped chain are bound by HBM, not
    by MFMA: their achieved algorithmic bytes per second as a fraction of the HBM peak."""
    from paper_2604_04599_amd import api
    if "S" not in ch.bufs:
        return {}
    sp = ch.bufs["S"][0].data_ptr()
    out = {}
    for row, s in zip(stages, ch.stages):
        if s.type != api.LPG_STAGE_GEMM:
            continue
        if s.out == sp:
            out["s_write_gemm"] = {"us": row["us"], "gbps": row["hbm_gbps"], "hbm_frac": round(row["hbm_gbps"] / HBM_PEAK_GBPS, 3)}
        elif s.in0 == sp:
            out["s_read_gemm"] = {"us": row["us"], "gbps": row["hbm_gbps"], "hbm_frac": round(row["hbm_gbps"] / HBM_PEAK_GBPS, 3)}
    return out


def measure(name, shape_over=None, options=None, with_stages=False, extras=True):
    """One workload: propagated and canonical chains in alternating blocks (each at least
    MIN_SECONDS), the compact record of the bench line, and (with_stages) the per-stage lists."""
    import torch
    from paper_2604_04599_amd import api, chains, inputs
    options = options or {}
    inp, shape = inputs.make(name, **(shape_over or {}))
    ch = chains.build(name, inp, shape, **options)
    flops = inputs.gemm_flops(name, shape)
    dt = inputs.DTYPES[name]
    both = compare_modes(ch)
    (mp, ap, np_), (mc, ac, nc) = both[api.LPG_CHAIN_PROPAGATED], both[api.LPG_CHAIN_CANONICAL]
    tf = flops / mp / 1e12
    nbytes = sum(stage_bytes(s) for s in ch.stages)
    res = {"dtype": dt, "gemm_gflop": round(flops / 1e9, 2), "ms": round(mp * 1e3, 4),
           "tflops": round(tf, 2), "pct_mfma_peak": round(100 * tf / PEAK_TFLOPS[dt], 2),
           "canonical_ms": round(mc * 1e3, 4), "speedup_vs_canonical": round(mc / mp, 3),
           "hbm_frac": round(nbytes / mp / 1e9 / HBM_PEAK_GBPS, 3)}
    if dt == "bf16":
        res["pct_power_limited_peak"] = round(100 * tf / BF16_POWER_LIMITED_TFLOPS, 2)
    stages = stage_breakdown(ch, 20) if (with_stages or "S" in ch.bufs) else None
    if stages is not None:
        res.update(score_gemm_rates(ch, stages))
    if name == "decoder_layer" and stages is not None:
        # the MFMA-bound part of the layer: projections and MLP GEMMs (everything but the two score GEMMs)
        sp = ch.bufs["S"][0].data_ptr()
        us = fl = 0.0
        for row, s in zip(stages, ch.stages):
            if s.type == api.LPG_STAGE_GEMM and s.out != sp and s.in0 != sp:
                us += row["us"]
                fl += 2.0 * row["m"] * row["n"] * row["k"] * row["batch"]
        res["projection_and_mlp_gemms"] = {"us": round(us, 1), "tflops": round(fl / us / 1e6, 1),
                                           "pct_mfma_peak": round(100 * fl / us / 1e6 / PEAK_TFLOPS[dt], 2),
                                           "pct_power_limited_peak": round(100 * fl / us / 1e6 / BF16_POWER_LIMITED_TFLOPS, 2)}
    if with_stages:
        res["stages"] = stages
    if extras:
        # the same chain with the entry pack / exit unpack fused into the first / last GEMM
        fch = chains.build(name, inp, shape, fused=True, **options)
        res["fused_boundaries_ms"] = round(time_for(fch, api.LPG_CHAIN_PROPAGATED, 0.2)[0] * 1e3, 4)
        del fch
        if name in ("llama_layer", "attention", "decoder_layer") and not options.get("flash"):
            # the attention block as one kernel that keeps the scores in registers
            ach = chains.build(name, inp, shape, flash=True, **options)
            res["fused_attention_ms"] = round(time_for(ach, api.LPG_CHAIN_PROPAGATED, 0.2)[0] * 1e3, 4)
            del ach
        if (name == "llama_layer" and not options) or (name == "attention" and options.get("causal") and not options.get("flash")):
            # the three attention stages cut into four blocks of query rows that stop at the causal diagonal
            bch = chains.build(name, inp, shape, causal_blocks=4, **options)
            res["causal_row_blocks_ms"] = round(time_for(bch, api.LPG_CHAIN_PROPAGATED, 0.2)[0] * 1e3, 4)
            del bch
        if name == "two_gemm":
            # the launch-bound chain replayed from a HIP graph (one graph launch per step)
            replay = ch.capture()
            for _ in range(20):
                replay()
            torch.cuda.synchronize()
            reps = 2000
            t0 = time.perf_counter()
            for _ in range(reps):
                replay()
            torch.cuda.synchronize()
            res["graph_replay_ms_per_step"] = round((time.perf_counter() - t0) / reps * 1e3, 4)
        torch.cuda.empty_cache()
    return res, ch, inp, shape


def cpu_baseline(inp, shape, budget_s=15.0):
    """The CPU oracle, as it stands, on the first R rows of C_0 through all GEMMs of the deep
    chain (every stage is row-separable), extrapolated linearly in flops to the whole chain."""
    from oracle import ref, workloads
    n, depth = shape["n"], shape["depth"]
    per_row = depth * 2 * n * n
    probe = 128
    t0 = time.perf_counter()
    workloads.deep_chain(inp, rows=np.arange(probe))
    dt = time.perf_counter() - t0
    rate = probe * per_row / dt
    rows = int(min(n, max(probe, budget_s * rate / per_row)))
    t0 = time.perf_counter()
    workloads.deep_chain(inp, rows=np.arange(rows))
    dt = time.perf_counter() - t0
    tfl = rows * per_row / dt / 1e12
    return {"value": round(tfl, 5), "unit": "TFLOP/s", "cores": ref.threads(), "kind": "oracle", "seconds": round(dt, 2),
            "extrapolated_whole_chain_seconds": round(n * per_row / (tfl * 1e12), 1),
            "sample": f"first {rows} of {n} rows of C_0 through all {depth} GEMMs of the deep chain (fp64 triple "
                      f"loop, OpenMP over rows); the whole-chain time is extrapolated linearly in flops"}


def profile_traffic(kernel_tag):
    """L2-miss bytes per GEMM launch from the committed rocprofv3 counter summary of this
    workload (not measured in this run): the line 'SUMMARY <tag> ... bytes_per_launch=<n>'."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic_deep_chain.txt")
    try:
        for line in open(path):
            m = re.match(r"#?\s*SUMMARY\s+" + re.escape(kernel_tag) + r"\b.*bytes_per_launch=([0-9.eE+]+)", line)
            if m:
                return float(m.group(1)), os.path.relpath(path, ROOT)
    except OSError:
        pass
    return None, None


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
    packed C out; also with a row-major weight), the Intermediate kernel (packed in, packed out), the Ending kernel (packed in,
    row-major out) and as a BLAS-style call (pack A + GEMM + unpack C); (2) three-GEMM chains of
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
            # Initial kernel: row-major fp32 A read by the GEMM itself (fp32 with K a multiple of 32: copied
            # verbatim by the main kernel; otherwise, and for a bf16 product, gathered by the general kernel)
            res["initial_tflops"] = round(flops / _time_calls(
                lambda: api.lpg_gemm_packed(1.0, a, a_rm, pw, w_p, 0.0, None, pc, c_p, stream=st), reps) / 1e12, 2)
            # ... and with the weight row-major as well (contiguous along n): the general kernel for both
            res["initial_row_major_weight_tflops"] = round(flops / _time_calls(
                lambda: api.lpg_gemm_packed(1.0, a, a_rm, w, w_rm, 0.0, None, pc, c_p, stream=st), reps) / 1e12, 2)
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
        both = compare_modes(ch, 0.15)                               # long enough for loaded clocks
        tp, tc = both[api.LPG_CHAIN_PROPAGATED][0], both[api.LPG_CHAIN_CANONICAL][0]
        tf = time_for(fch, api.LPG_CHAIN_PROPAGATED, 0.05)[0]
        print(json.dumps({"sweep": "chain3_f32", "m": m, "widths": list(widths),
                          "propagated_ms": round(tp * 1e3, 4), "canonical_ms": round(tc * 1e3, 4),
                          "fused_boundaries_ms": round(tf * 1e3, 4), "speedup_vs_canonical": round(tc / tp, 3),
                          "tflops": round(ch.flops / tp / 1e12, 2)}), flush=True)
        del ch, fch
        torch.cuda.empty_cache()


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workloads", default="all",
                    help="comma list of workloads to report beside the headline (the five configs' names, "
                         "attention_softmax, llama_layer), 'all' or 'none'")
    ap.add_argument("--stages", action="store_true", help="add the per-stage lists to every workload's record")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--only", default=None,
                    help="profiling aid: run just this workload (a workload name, attention_softmax_causal, llama_layer_causal_row_blocks, "
                         "llama_layer or llama_layer_fused_attention) --steps times in --mode and print its line")
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
    ap.add_argument("--tune", default="", metavar="KEY=VALUE,...",
                    help="profiling aid: pin per-launch choices of the library (lpg_tune_set), e.g. tile=6,band=4")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="MIB",
                    help="profiling aid: run the elementwise SCALE kernel over a buffer of MIB MiB "
                         "(reads MIB, writes MIB per launch) --steps times, to scale HBM counters")
    args = ap.parse_args()
    global SETTLE_SECONDS
    SETTLE_SECONDS = args.settle_ms * 1e-3
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch
    if not torch.cuda.is_available():
        print("bench.py: needs a GPU (the HIP library has no CPU fallback)", file=sys.stderr)
        sys.exit(1)
    torch.cuda.set_device(0)
    from paper_2604_04599_amd import api, inputs
    if args.tune:
        keys = {"tile": api.LPG_TUNE_TILE, "band": api.LPG_TUNE_BAND, "two_block_steps": api.LPG_TUNE_TWO_BLOCK_STEPS,
                "bf16_whole_block_steps": api.LPG_TUNE_BF16_WHOLE_BLOCK_STEPS, "row_variant": api.LPG_TUNE_ROW_VARIANT,
                "attn_query_groups": api.LPG_TUNE_ATTN_QUERY_GROUPS, "trace": api.LPG_TUNE_TRACE}
        for kv in args.tune.split(","):
            key, val = kv.split("=")
            api.lpg_tune_set(keys[key], int(val))

    if args.sweep:
        sweep(max(args.steps, 5))
        return
    if args.gemm:
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
        from paper_2604_04599_amd import chains
        name, options = args.only, {}
        if name == "attention_softmax_causal":
            name, options = "attention", {"softmax": True, "causal": True}
        elif name == "llama_layer_fused_attention":
            name, options = "llama_layer", {"flash": True}
        elif name == "llama_layer_causal_row_blocks":
            name, options = "llama_layer", {"causal_blocks": 4}
        inp, shape = inputs.make(name)
        ch = chains.build(name, inp, shape, **options)
        res = {"workload": args.only, "steps": args.steps}
        flops = inputs.gemm_flops(name, shape)
        if options.get("causal_blocks"):
            # only the GEMM flops that are executed: n blocks of query rows do (n + 1) / 2n of the two attention GEMMs
            n = options["causal_blocks"]
            dh = shape["hidden"] // shape["n_q"]
            flops -= shape["n_q"] * 4.0 * shape["t"] * shape["t"] * dh * (1.0 - (n + 1) / (2.0 * n))
        if args.mode in ("both", "propagated"):
            t = time_chain(ch, api.LPG_CHAIN_PROPAGATED, args.steps, args.warmup)
            res.update({"ms_per_step": round(t * 1e3, 4), "tflops": round(flops / t / 1e12, 2)})
        if args.mode in ("both", "canonical"):
            t = time_chain(ch, api.LPG_CHAIN_CANONICAL, args.steps, args.warmup)
            res["canonical_ms_per_step"] = round(t * 1e3, 4)
        if args.stages:
            res["stages"] = stage_breakdown(ch, max(3, args.steps))
        print(json.dumps(res))
        return

    # ---- headline: exactly --steps steps of the deep chain after --warmup steps, synchronised on both sides
    from paper_2604_04599_amd import chains
    inp, shape = inputs.make(HEADLINE)
    ch = chains.build(HEADLINE, inp, shape)
    flops = inputs.gemm_flops(HEADLINE, shape)
    t_step = time_chain(ch, api.LPG_CHAIN_PROPAGATED, args.steps, args.warmup)
    value = flops / t_step / 1e12
    both = compare_modes(ch)
    (mp, apm, np_), (mc, ac, nc) = both[api.LPG_CHAIN_PROPAGATED], both[api.LPG_CHAIN_CANONICAL]
    t_gemm, gemm_flops, gemm_bytes = time_gemm_launches(ch, max(3, min(args.steps, 40)))
    achieved = gemm_flops / t_gemm / 1e12
    traffic, traffic_src = profile_traffic("gemm_kernel")
    roofline = {"bound": "mfma", "kernel": "gemm_kernel<F32,F32,256x256 tile, 8 waves> (every GEMM of the chain)",
                "achieved": round(achieved, 2), "peak": PEAK_TFLOPS["f32"], "unit": "TFLOP/s",
                "frac": round(achieved / PEAK_TFLOPS["f32"], 4), "avg_launch_us": round(t_gemm * 1e6, 2),
                "flops_per_launch": gemm_flops, "traffic": traffic, "algorithmic_bytes": gemm_bytes,
                "traffic_over_algorithmic": round(traffic / gemm_bytes, 2) if traffic else None,
                "traffic_unit": "L2-miss bytes per launch (rocprofv3 FETCH_SIZE + WRITE_SIZE, calibrated on a copy "
                                f"kernel), from {traffic_src}, not measured in this run" if traffic else None}
    head = {"dtype": "f32", "gemm_gflop": round(flops / 1e9, 2), "ms": round(mp * 1e3, 4),
            "steps_timed": np_, "tflops": round(flops / mp / 1e12, 2),
            "pct_mfma_peak": round(100 * flops / mp / 1e12 / PEAK_TFLOPS["f32"], 2),
            "canonical_ms": round(mc * 1e3, 4), "speedup_vs_canonical": round(mc / mp, 3),
            "hbm_frac": round(sum(stage_bytes(s) for s in ch.stages) / mp / 1e9 / HBM_PEAK_GBPS, 3)}
    if args.stages:
        head["stages"] = stage_breakdown(ch, 5)
    fch = chains.build(HEADLINE, inp, shape, fused=True)
    head["fused_boundaries_ms"] = round(time_for(fch, api.LPG_CHAIN_PROPAGATED, 0.2)[0] * 1e3, 4)
    del fch
    cpu = None if args.no_cpu_baseline else cpu_baseline(inp, shape)
    del ch, inp
    torch.cuda.empty_cache()

    per = {HEADLINE: head}
    wanted = args.workloads.split(",")
    if args.workloads == "all":
        names = [w for w in inputs.WORKLOADS if w != HEADLINE]
    elif args.workloads == "none":
        names = []
    else:
        names = [w for w in wanted if w in inputs.WORKLOADS and w != HEADLINE]
    for w in names:
        res, c2, _, _ = measure(w, with_stages=args.stages)
        per[w] = res
        del c2
        torch.cuda.empty_cache()
    if args.workloads == "all" or "attention_softmax" in wanted:
        # widening row: the attention chain with the scale + causal mask + softmax stage between its GEMMs
        res, c2, _, _ = measure("attention", options={"softmax": True, "causal": True}, with_stages=args.stages)
        per["attention_softmax_causal"] = res
        del c2
        torch.cuda.empty_cache()
    if args.workloads == "all" or "llama_layer" in wanted:
        # widening row: the decoder layer with RMSNorm, RoPE, causal softmax and both residuals between its GEMMs
        res, c2, _, _ = measure("llama_layer", with_stages=args.stages)
        per["llama_layer"] = res
        del c2
        torch.cuda.empty_cache()

    out = {"metric": "chained_gemm_tflops", "value": round(value, 2), "unit": "TFLOP/s", "n_gpus": 1,
           "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(t_step * 1e3, 4),
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32",
           "data": "synthetic",
           "config": {"workload": HEADLINE_TEXT, "shape": shape, "mode": "propagated"},
           "pct_mfma_peak": round(100 * value / PEAK_TFLOPS["f32"], 2),
           "speedup_vs_canonical": head["speedup_vs_canonical"],
           "roofline": roofline, "cpu_baseline": cpu, "workloads": per,
           "context": "paper: 2.25x average over OpenBLAS for sequential GEMMs on a Xeon Gold 6252 "
                      "(AVX-512, 1 thread); other hardware, not a target"}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
