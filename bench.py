#!/usr/bin/env python3
"""Benchmark of the fine-grained W4A8 integer-scale linear layer on one MI355X.

Default workload (N=1): the LLaMA-2-70B-shaped linears (qkv 8192->10240, o_proj 8192->8192, gate 8192->28672,
down 28672->8192; group-128 int4 weights in the kernel layout written offline by is_prepack_w4, int8 per-token
activations, alpha = 2^10) in decode (M = 1 and M = 32 token rows) and in prefill (M = 2048).  One step is one pass of the
whole hot path over that workload: for every M, every linear and every one of `--layers` layers (each with its own
weight buffers, so every decode GEMM streams cold weights from HBM as in a real decode step), the linear call on fp16
activations: the per-token activation quantiser and the integer-scale GEMM of Eq. (2) with its float epilogue (one
kernel for M = 1, quantiser + weight-streaming kernel for M = 32, quantising preparation pass + MFMA-bound tiled kernel
for M = 2048).  Inputs are synthetic (seeded) and resident in HBM before the timed region.  The launches of one
(M, linear) pair are recorded into a HIP graph and replayed; HIP events between the replays give each pair's average
duration inside the timed region.

Prints ONE JSON line.  `value` is the whole step's int8 tera-operations per second (the step's time is dominated by the
MFMA-bound prefill GEMMs, whose kernel is the `roofline` entry; the HBM-bound decode kernel has its own entry,
`roofline_hbm`).  Per shape the line carries the time of the step's call, of the integer-scale and of the float-scale
GEMM call alone (Eq. (1), built the same way) with their ratio, the time a plain streaming read of the same bytes
takes, and the roofline fractions; `alpha_sweep` shows the accuracy / overflow trade-off of the amplifier on one layer.

`--workload llama2_7b` (M in {1, 16, 64}) and `--workload llama3_8b` (M = 4096, Student-t activations) run the same
code on those shapes; `moe`, `w8a8` and `producers` measure the mixture-of-experts form, fine-grained W8A8 and the
fused activation producers; `gate_up` the gate_up GEMM with SiLU(gate) * up as its epilogue against the unfused sequence.
"""
from __future__ import annotations

import argparse
import json
import gc
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E
MFMA_I8_PEAK_TOPS = 5000.0     # dense int8 MFMA
GROUP = 128
ALPHA_LOG2 = 10
BATCHES = (1, 16, 64)


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--layers", type=int, default=None,
                    help="distinct weight copies per linear (default: 8 for llama2_70b, 32 for llama2_7b, 4 for llama3_8b)")
    ap.add_argument("--no-graph", action="store_true", help="launch eagerly instead of replaying HIP graphs")
    ap.add_argument("--no-floatscale", action="store_true", help="skip the float-scale comparison pass")
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip timing the CPU oracle")
    ap.add_argument("--no-traffic", action="store_true",
                    help="do not look up the measured HBM traffic in profiles/ (roofline.traffic = null); without this "
                         "flag a missing figure is an error")
    ap.add_argument("--workload", default="llama2_70b",
                    choices=("llama2_70b", "llama2_7b", "llama3_8b", "moe", "w8a8", "producers", "gate_up"))
    return ap.parse_args()


def measured_peaks(P, torch):
    """What this chip delivers, from the same run: a plain streaming read of 1 GiB out of HBM, and a register-only
    loop of int8 MFMAs, on constant operands and on operands that change from one MFMA to the next (the library's probe
    kernels, timed with events)."""
    dev = torch.device("cuda:0")
    buf = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
    buf.fill_(1)
    sink = torch.zeros(1, dtype=torch.int32, device=dev)

    def time_ms(fn, reps):
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    nbytes = P.is_probe_stream_read(buf, sink)
    ms_read = time_ms(lambda: P.is_probe_stream_read(buf, sink), 10)
    ops = P.is_probe_mfma_i8(2000, sink)
    ms_mfma = time_ms(lambda: P.is_probe_mfma_i8(2000, sink), 5)
    ops_r = P.is_probe_mfma_i8_random(2000, sink)
    ms_mfma_r = time_ms(lambda: P.is_probe_mfma_i8_random(2000, sink), 5)
    del buf
    return dict(hbm_read_gbs=round(nbytes / ms_read / 1e6, 1), mfma_i8_tops=round(ops / ms_mfma / 1e9, 1),
                mfma_i8_tops_random_operands=round(ops_r / ms_mfma_r / 1e9, 1),
                how="library probe kernels, same run: 1 GiB streaming read; register-only loop of independent "
                    "v_mfma_i32_16x16x64_i8, two waves per SIMD, on constant operands and on operands that change "
                    "from one MFMA to the next (the chip lowers its clock when the matrix pipe's inputs toggle)")


TRAFFIC_REQUIRED = True   # --no-traffic clears it


def measured_traffic(kernel, workload):
    """HBM bytes per launch of `kernel` as measured with rocprofv3 --pmc (FETCH_SIZE and WRITE_SIZE, scaled by what
    the same counters read for kernels of known size); the figures sit in the profile summary of this workload as lines
    `TRAFFIC <kernel name> <bytes per launch>`.  A missing file or line ends the run with an error (the figure would
    silently read null otherwise), unless --no-traffic says that none is wanted."""
    if not TRAFFIC_REQUIRED:
        return None
    path = os.path.join(ROOT, "profiles", f"bench_{workload}_pmc_traffic.txt")
    if os.path.exists(path):
        for ln in open(path):
            parts = ln.rstrip("\n").split("\t")
            if len(parts) == 3 and parts[0] == "TRAFFIC" and parts[1] == kernel:
                return float(parts[2])
    print(f"bench.py: no measured HBM traffic for kernel '{kernel}' in {path}: collect it (see the commands in "
          f"profiles/) or pass --no-traffic", file=sys.stderr)
    sys.exit(3)


class Segment:
    """A run of launches replayed as one unit, with the bookkeeping for its roofline figures."""

    def __init__(self, name, kernel, launches, alg_bytes, ops, fn, use_graph, torch):
        self.name, self.kernel, self.launches, self.alg_bytes, self.ops = name, kernel, launches, alg_bytes, ops
        self.fn = fn
        self.graph = None
        self.elapsed_ms = 0.0
        self.count = 0
        self.pending = []
        if use_graph:
            fn()                       # run once eagerly: every buffer is touched before capture
            torch.cuda.synchronize()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                fn()
            self.graph = g

    def run(self):
        if self.graph is not None:
            self.graph.replay()
        else:
            self.fn()


def main():
    global TRAFFIC_REQUIRED
    args = parse_args()
    # The interpreter's cyclic collector stays off for the whole run (reference counting frees everything here): a full
    # collection takes some 20 ms with this many live objects, it fell into the same place of the timed loop in every
    # run, and the GPU ran dry there (seen as one step of one segment 25 times longer than the others).
    gc.disable()
    TRAFFIC_REQUIRED = not args.no_traffic
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (one process, one MI355X); run with --gpus 1. "
              "Multi-GPU sharding is a design note, not a measured path.", file=sys.stderr)
        sys.exit(2)
    if args.workload in FAMILIES:
        return family_main(args)
    if args.layers is None:
        args.layers = 32
    if args.workload == "w8a8":
        return w8a8_main(args)
    if args.workload == "moe":
        return moe_main(args)
    if args.workload == "gate_up":
        return gate_up_main(args)
    return producers_main(args)



FAMILIES = {
    # workload -> configuration index of the input recipe, linears (name -> (K, N)), token-row counts, default layers
    "llama2_70b": dict(config=2, label="llama2-70b", skip=("up",), batches=(1, 32, 2048), layers=8),
    "llama2_7b": dict(config=1, label="llama2-7b", skip=(), batches=(1, 16, 64), layers=32),
    "llama3_8b": dict(config=3, label="llama3-8b", skip=(), batches=(4096,), layers=4),
}


def family_main(args):
    """The linear layers of one model family on the prepacked route: every (M, linear) pair is one segment of the step."""
    import numpy as np
    import torch

    import paper_2405_14597_amd as P
    import synth_inputs as S

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    P.load_library()
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    fam = FAMILIES[args.workload]
    cfg = fam["config"]
    table = {"llama2_70b": S.LLAMA2_70B, "llama2_7b": S.LLAMA2_7B, "llama3_8b": S.LLAMA3_8B}[args.workload]
    linears = [(n, kn) for n, kn in table.items() if n not in fam["skip"]]
    batches = fam["batches"]
    L = args.layers or fam["layers"]
    use_graph = not args.no_graph

    def grp(K):
        return GROUP

    # ---------------------------------------------------------------- data: one layer drawn on the host, quantised and
    # prepacked on the GPU by the library (the offline step), then copied into L distinct buffers (timing does not
    # depend on the values); both scale forms, for the float-scale twin
    weights = {}
    for idx, (name, (K, N)) in enumerate(linears):
        w = torch.from_numpy(S.make_weights(cfg, N, K, S.seed_for(cfg, idx, 1))).to(dev)
        qw = P.is_quantize_weights_int4_group(w, grp(K), ALPHA_LOG2, P.IS_SCALE_NORM)
        del w
        pi = P.is_prepack_w4(qw.qweight, qw.scale_i32, grp(K))
        pf = P.is_prepack_w4(qw.qweight, qw.scale_f32, grp(K))
        torch.cuda.synchronize()
        weights[name] = dict(
            canon=qw,
            pi=[pi] + [P.PackedWeights(pi.wpack.clone(), pi.spack.clone(), *pi[2:]) for _ in range(L - 1)],
            pf=[pf] + [P.PackedWeights(pf.wpack.clone(), pf.spack.clone(), *pf[2:]) for _ in range(L - 1)],
            c=[qw.chan_scale] + [qw.chan_scale.clone() for _ in range(L - 1)])
    acts = {}
    for M in batches:
        for idx, (name, (K, N)) in enumerate(linears):
            x = torch.from_numpy(S.make_activations(cfg, M, K, S.seed_for(cfg, idx, 2) + M)).to(dev)
            xq, sa = P.is_quantize_act_int8_token(x)
            acts[(M, name)] = dict(
                x=x, xq=xq, sa=sa, out=torch.empty((M, N), dtype=torch.float16, device=dev),
                # workspaces start zeroed: the K split's arrival counters live there and every call leaves them zero
                lws=torch.zeros(max(1, P.is_linear_prepacked_workspace_bytes(M, N, K, grp(K))), dtype=torch.uint8, device=dev),
                gws=torch.zeros(max(1, P.is_gemm_prepacked_workspace_bytes(M, N, K, grp(K))), dtype=torch.uint8, device=dev))
    torch.cuda.synchronize()

    def alg_bytes(M, N, K, fp16_in):
        b = S.algorithmic_bytes(M, N, K, grp(K))
        return b + M * K - 4 * M if fp16_in else b      # fp16 rows in instead of int8 codes and their scales

    # ---------------------------------------------------------------- segments
    def make_segments(kind):
        """kind: 'linear' (the step: fp16 in), 'gemm_is' / 'gemm_fs' (the GEMM calls alone: int8 codes in)."""
        segs = []
        for M in batches:
            for name, (K, N) in linears:
                a, w = acts[(M, name)], weights[name]
                if kind == "linear":
                    def fn(a=a, w=w):
                        for l in range(L):
                            P.is_linear_w4a8_intscale_prepacked(a["x"], w["pi"][l], w["c"][l], ALPHA_LOG2, out=a["out"],
                                                                workspace=a["lws"])
                    kernels = P.is_describe_prepacked(M, N, K, grp(K), True, True)
                elif kind == "gemm_is":
                    def fn(a=a, w=w):
                        for l in range(L):
                            P.is_gemm_w4a8_intscale_prepacked(a["xq"], a["sa"], w["pi"][l], w["c"][l], ALPHA_LOG2,
                                                              out=a["out"], workspace=a["gws"])
                    kernels = P.is_describe_prepacked(M, N, K, grp(K), True, False)
                elif kind == "gemm_is_prepared":
                    # the tiled kernel alone: the activations are prepared once (outside the replayed launches), the
                    # layers' GEMMs run on the prepared workspace
                    if len(P.is_describe_prepacked(M, N, K, grp(K), True, False)) < 2:
                        continue
                    P.is_prepare_activations_prepacked(a["xq"], a["gws"])

                    def fn(a=a, w=w):
                        for l in range(L):
                            P.is_gemm_w4a8_intscale_prepacked_prepared(a["sa"], w["pi"][l], w["c"][l], ALPHA_LOG2,
                                                                       a["gws"], out=a["out"])
                    kernels = P.is_describe_prepacked(M, N, K, grp(K), True, False)[-1:]
                else:
                    def fn(a=a, w=w):
                        for l in range(L):
                            P.is_gemm_w4a8_floatscale_prepacked(a["xq"], a["sa"], w["pf"][l], out=a["out"],
                                                                workspace=a["gws"])
                    kernels = P.is_describe_prepacked(M, N, K, grp(K), False, False)
                seg = Segment(f"{name}_M{M}", kernels[-1], L, L * alg_bytes(M, N, K, kind == "linear"),
                              L * S.algorithmic_ops(M, N, K), fn, use_graph, torch)
                seg.M, seg.K, seg.N, seg.kernels = M, K, N, kernels
                segs.append(seg)
        return segs

    def run_steps(segs, n, timed):
        for _ in range(n):
            ev = torch.cuda.Event(enable_timing=True)
            ev.record()
            for s in segs:
                s.run()
                nxt = torch.cuda.Event(enable_timing=True)
                nxt.record()
                if timed:
                    s.pending.append((ev, nxt))
                ev = nxt

    def timed_pass(segs, steps, warmup):
        run_steps(segs, warmup, False)
        torch.cuda.synchronize()
        gc.collect()
        t0 = time.perf_counter()
        run_steps(segs, steps, True)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        if os.environ.get("BENCH_TRACE_STEPS"):  # per step and segment, to stderr: where a one-off stall fell
            for s in segs:
                print(s.name, " ".join(f"{a.elapsed_time(b):.3f}" for a, b in s.pending), file=sys.stderr)
        for s in segs:
            s.elapsed_ms = sum(a.elapsed_time(b) for a, b in s.pending)
            s.count = len(s.pending) * s.launches
            s.pending = []
        return (t1 - t0) / steps

    def per_call_us(s):
        return 1e3 * s.elapsed_ms / max(s.count, 1)

    segs = make_segments("linear")
    sec_per_step = timed_pass(segs, args.steps, args.warmup)
    step_ops = sum(s.ops for s in segs)
    step_bytes = sum(s.alg_bytes for s in segs)

    # the GEMM calls alone, integer scale and its float-scale twin (one kernel per decode call, so the decode kernel's
    # own duration comes out of this pass; the tiled call is its preparation kernel + the tile kernel)
    n_cmp = max(3, args.steps // 2)
    g_is = make_segments("gemm_is")
    timed_pass(g_is, n_cmp, 2)
    g_fs = None
    if not args.no_floatscale:
        g_fs = make_segments("gemm_fs")
        timed_pass(g_fs, n_cmp, 2)
    # the tiled kernel by itself (its preparation kernel done once beforehand): the kernel's own launch duration
    g_tile = make_segments("gemm_is_prepared")
    if g_tile:
        timed_pass(g_tile, n_cmp, 2)
    tile_us = {s.name: per_call_us(s) for s in g_tile}

    # a plain streaming read of the same number of bytes as each decode GEMM (cold: a different buffer every launch)
    sink = torch.zeros(1, dtype=torch.int32, device=dev)
    probe_us = {}
    pool = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
    pool.fill_(1)
    for s in g_is:
        if s.M > 64:
            continue
        nb = (s.alg_bytes // s.launches) // 16 * 16
        slots = max(1, min(8, pool.numel() // nb))
        views = [pool[i * nb:(i + 1) * nb] for i in range(slots)]
        reps = 4 * slots
        for v in views:
            P.is_probe_stream_read(v, sink)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for r in range(reps):
            P.is_probe_stream_read(views[r % slots], sink)
        e1.record()
        torch.cuda.synchronize()
        probe_us[s.name] = 1e3 * e0.elapsed_time(e1) / reps
    del pool

    shapes = []
    for i, s in enumerate(segs):
        g = g_is[i]
        call_us, gemm_us = per_call_us(s), per_call_us(g)
        bytes_call = g.alg_bytes / g.launches
        ops_call = g.ops / g.launches
        row = dict(name=s.name, M=s.M, K=s.K, N=s.N, kernels=s.kernels, step_call_us=round(call_us, 3),
                   gemm_us=round(gemm_us, 3))
        if g_fs is not None:
            fs_us = per_call_us(g_fs[i])
            row["floatscale_gemm_us"] = round(fs_us, 3)
            row["floatscale_over_intscale"] = round(fs_us / gemm_us, 4)
        if s.M <= 64:
            row["gbs"] = round(bytes_call / gemm_us / 1e3, 1)
            row["hbm_frac"] = round(bytes_call / gemm_us / 1e3 / HBM_PEAK_GBS, 4)
            row["stream_read_same_bytes_us"] = round(probe_us[s.name], 3)
            row["gemm_over_stream_read"] = round(gemm_us / probe_us[s.name], 3)
        else:
            row["tops"] = round(ops_call / gemm_us / 1e6, 1)
            row["mfma_frac"] = round(ops_call / gemm_us / 1e6 / MFMA_I8_PEAK_TOPS, 4)
            if s.name in tile_us:  # the tiled kernel alone, on prepared activations
                row["tile_kernel_us"] = round(tile_us[s.name], 3)
                row["tile_kernel_mfma_frac"] = round(ops_call / tile_us[s.name] / 1e6 / MFMA_I8_PEAK_TOPS, 4)
        shapes.append(row)

    # ---------------------------------------------------------------- rooflines: per kernel instantiation, from the
    # GEMM-only pass; the dominant one by time inside the step is `roofline`
    by_kernel = {}
    for s in g_is:
        k = by_kernel.setdefault(s.kernel, dict(ms=0.0, launches=0, bytes=0.0, ops=0.0, tiled=s.M > 64, call_ms=0.0,
                                                alone=True))
        k["call_ms"] += s.elapsed_ms
        k["launches"] += s.count
        k["bytes"] += s.alg_bytes * (s.count / s.launches)
        k["ops"] += s.ops * (s.count / s.launches)
        if s.name in tile_us:  # the kernel's own duration: the pass on prepared activations (same launches, same weights)
            k["ms"] += tile_us[s.name] * s.count / 1e3
        else:
            k["ms"] += s.elapsed_ms
            k["alone"] = len(s.kernels) == 1
    peaks = measured_peaks(P, torch)
    profile = f"{args.workload}"

    def roof(name, k):
        us = 1e3 * k["ms"] / k["launches"]
        if k["tiled"]:
            ach = k["ops"] / k["launches"] / us / 1e6
            return dict(bound="mfma", kernel=name, achieved=round(ach, 1), peak=MFMA_I8_PEAK_TOPS, unit="TOP/s",
                        frac=round(ach / MFMA_I8_PEAK_TOPS, 4), traffic=measured_traffic(name, profile),
                        avg_launch_us=round(us, 3), alg_ops_per_launch=round(k["ops"] / k["launches"]),
                        frac_of_measured_peak=round(ach / peaks["mfma_i8_tops"], 4),
                        frac_of_measured_peak_random_operands=round(ach / peaks["mfma_i8_tops_random_operands"], 4),
                        gemm_call_us=round(1e3 * k["call_ms"] / k["launches"], 3),
                        frac_of_gemm_call=round(k["ops"] / k["launches"] / (1e3 * k["call_ms"] / k["launches"]) / 1e6
                                                / MFMA_I8_PEAK_TOPS, 4),
                        note="avg_launch_us = this kernel alone, timed with events around replayed launches of the "
                             "GEMM on prepared activations (is_prepare_activations_prepacked once, then "
                             "is_gemm_w4a8_intscale_prepacked_prepared per layer); gemm_call_us = the ordinary GEMM "
                             "call on int8 codes, i.e. with its activation preparation kernel" if k["alone"] else
                             "duration = the GEMM call on int8 codes: this kernel plus its activation preparation "
                             "kernel")
        ach = k["bytes"] / k["launches"] / us / 1e3
        return dict(bound="hbm", kernel=name, achieved=round(ach, 1), peak=HBM_PEAK_GBS, unit="GB/s",
                    frac=round(ach / HBM_PEAK_GBS, 4), traffic=measured_traffic(name, profile),
                    avg_launch_us=round(us, 3), alg_bytes_per_launch=round(k["bytes"] / k["launches"]),
                    frac_of_measured_peak=round(ach / peaks["hbm_read_gbs"], 4))

    ranked = sorted(by_kernel.items(), key=lambda kv: -kv[1]["ms"])
    roofline = roof(*ranked[0])
    other = [kv for kv in ranked if kv[1]["tiled"] != ranked[0][1]["tiled"]]
    roofline_other = roof(*other[0]) if other else None

    speedup = None
    if g_fs is not None:
        speedup = dict(
            all=round(sum(s.elapsed_ms for s in g_fs) / sum(s.elapsed_ms for s in g_is), 4),
            decode=None if not any(s.M <= 64 for s in g_is) else round(
                sum(s.elapsed_ms for s in g_fs if s.M <= 64) / sum(s.elapsed_ms for s in g_is if s.M <= 64), 4),
            prefill=None if not any(s.M > 64 for s in g_is) else round(
                sum(s.elapsed_ms for s in g_fs if s.M > 64) / sum(s.elapsed_ms for s in g_is if s.M > 64), 4))

    # ---------------------------------------------------------------- amplifier sweep on one layer (Sec. 4.1, Fig. 4):
    # integer-scale output against the float-scale output of the same quantised weights, and the worst-case bound
    sweep = None
    if not args.no_floatscale:
        name, (K, N) = linears[-1]
        M = min(batches[-1], 32) if batches[-1] > 64 else batches[-1]
        idx = len(linears) - 1
        w = torch.from_numpy(S.make_weights(cfg, N, K, S.seed_for(cfg, idx, 1))).to(dev)
        a = acts[(M if (M, name) in acts else batches[0], name)]
        sweep = []
        for al in (6, 8, 10, 12):
            qw = P.is_quantize_weights_int4_group(w, grp(K), al, P.IS_SCALE_NORM)
            ref = P.is_gemm_w4a8_floatscale(a["xq"], a["sa"], qw.qweight, qw.scale_f32, grp(K)).float()
            # (scale_f32 is the whole float group scale; scale_i32 its amplified, rounded quotient by chan_scale)
            got, _ = P.is_gemm_w4a8_intscale_prepacked(a["xq"], a["sa"], P.is_prepack_w4(qw.qweight, qw.scale_i32, grp(K)),
                                                       qw.chan_scale, al)
            bound = int(P.is_intscale_overflow_bound(qw.scale_i32, grp(K)).cpu()[0])
            err = (got.float() - ref).abs()
            sweep.append(dict(alpha_log2=al, mean_rel_err_vs_floatscale=float(err.mean() / ref.abs().mean()),
                              max_abs_err_over_mean_abs=float(err.max() / ref.abs().mean()),
                              worst_case_bound_log2=round(float(np.log2(max(1, bound))), 2)))
        sweep = dict(linear=name, M=a["xq"].shape[0], rows=sweep,
                     note="error of Eq. (2) against Eq. (1) on the same int4 weights; bound = max_n sum_g |IS| * G * 1024, "
                          "int32 cannot overflow iff its log2 is below 31")
        del w

    # ---------------------------------------------------------------- CPU oracle on a bounded sample of the same step
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import oracle as O
        cap = 2048         # token rows per call the oracle is timed on (its time is linear in M)
        t_cpu, cpu_ops = 0.0, 0
        ok_all, rel_all = True, 0.0
        for idx, (name, (K, N)) in enumerate(linears):
            hw = O.quantize_weights_int4_group(S.make_weights(cfg, N, K, S.seed_for(cfg, idx, 1)), grp(K), ALPHA_LOG2,
                                               O.SCALE_NORM)
            for M in batches:
                hx = S.make_activations(cfg, M, K, S.seed_for(cfg, idx, 2) + M)[:cap]
                t0 = time.perf_counter()
                xq, sa = O.quantize_act_int8_token(hx)
                ref = O.gemm_w4a8_intscale(xq, sa, hw.qweight, hw.scale_i32, hw.chan_scale, grp(K), ALPHA_LOG2)
                t_cpu += time.perf_counter() - t0
                cpu_ops += S.algorithmic_ops(hx.shape[0], N, K)
                # the oracle's result doubles as a live parity check of the step's call (first layer's weights)
                a, w = acts[(M, name)], weights[name]
                out, acc = P.is_linear_w4a8_intscale_prepacked(a["x"], w["pi"][0], w["c"][0], ALPHA_LOG2, want_acc=True,
                                                               workspace=a["lws"])
                torch.cuda.synchronize()
                rows = hx.shape[0]
                ok_all = ok_all and bool(np.array_equal(acc[:rows].cpu().numpy(), ref.acc))
                got = out[:rows].cpu().numpy().astype(np.float64)
                rel_all = max(rel_all, float(np.max(np.abs(got - ref.out) / np.maximum(np.abs(ref.out), 1e-3))))
                del out, acc, got, ref
            del hw
        cpu = dict(value=round(cpu_ops / t_cpu / 1e12, 5), unit="TOP/s", cores=O.num_threads(), kind="oracle",
                   sample=f"one layer of the step: {len(linears)} linears x M in {list(batches)} (quantiser + integer-scale "
                          f"GEMM), at most {cap} token rows per call, {t_cpu:.1f} s",
                   parity=dict(acc_bit_exact=ok_all, max_rel_err=rel_all))

    value = step_ops / sec_per_step / 1e12
    decode_bytes = sum(s.alg_bytes for s in segs if s.M <= 64)
    decode_ms = sum(s.elapsed_ms / (s.count / s.launches) for s in segs if s.M <= 64 and s.count)
    prefill_ops = sum(s.ops for s in segs if s.M > 64)
    prefill_ms = sum(s.elapsed_ms / (s.count / s.launches) for s in segs if s.M > 64 and s.count)
    line = {
        "metric": "W4A8 integer-scale GEMM TOPS + HBM GB/s (% roofline); speedup vs float-scale",
        "value": round(value, 1),
        "unit": "TOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(1e3 * sec_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "int8",
        "data": "synthetic",
        "config": {"workload": f"{fam['label']} linears ({', '.join(n for n, _ in linears)}), W4 group-{GROUP} x A8 "
                               f"per-token, alpha=2^{ALPHA_LOG2}, M in {list(batches)} (fp16 activations in, fp16 out), "
                               f"{L} layers of distinct weights per step",
                   "layout": "weights prepacked offline (is_prepack_w4)",
                   "launch": "hip-graph" if use_graph else "eager", "scale_mode": "norm"},
        "decode": None if not decode_ms else dict(
            gbs=round(decode_bytes / decode_ms / 1e6, 1), hbm_frac=round(decode_bytes / decode_ms / 1e6 / HBM_PEAK_GBS, 4),
            ms_per_step=round(decode_ms, 4), note="linear calls of the step with M <= 64, quantiser included"),
        "prefill": None if not prefill_ms else dict(
            tops=round(prefill_ops / prefill_ms / 1e9, 1),
            mfma_frac=round(prefill_ops / prefill_ms / 1e9 / MFMA_I8_PEAK_TOPS, 4), ms_per_step=round(prefill_ms, 4),
            note="linear calls of the step with M > 64, quantising preparation pass included"),
        "speedup_vs_floatscale": speedup,
        "roofline": roofline,
        "roofline_hbm" if roofline["bound"] == "mfma" else "roofline_mfma": roofline_other,
        "alpha_sweep": sweep,
        "measured_peaks": peaks,
        "cpu_baseline": cpu,
        "shapes": shapes,
    }
    print(json.dumps(line))


def w8a8_main(args):
    """Fine-grained W8A8 on the layer the paper's LLaMA-3 recipe uses it for: the LLaMA-3-8B down projection
    (14336 -> 4096), at M in {1, 16, 64} (weight stream, general kernel) and M = 4096 (tiled kernel).  One step =
    activation quantiser + integer-scale GEMM per M over `--layers` (default 8 here) distinct weight sets.  `value`
    is the algorithmic GB/s of the three small-M calls (HBM bound); the M = 4096 call is reported in `shapes` in TOP/s."""
    import numpy as np
    import torch

    import paper_2405_14597_amd as P
    import synth_inputs as S

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    P.load_library()
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    K, N = S.LLAMA3_8B["down"]
    L = args.layers if args.layers != 32 else 8
    MS = (1, 16, 64, 4096)
    w = torch.from_numpy(S.make_weights(3, N, K, S.seed_for(3, 2, 1))).to(dev)
    qw = P.is_quantize_weights_int8_group(w, GROUP, ALPHA_LOG2, P.IS_SCALE_NORM)
    del w
    q = qw.qweight.unsqueeze(0).repeat(L, 1, 1)  # L copies: 59 MB each, so that the weights come from HBM
    acts = {}
    for M in MS:
        x = torch.from_numpy(S.make_activations(3, M, K, S.seed_for(3, 2, 2) + M)).to(dev)
        acts[M] = dict(x=x, xq=torch.empty((M, K), dtype=torch.int8, device=dev),
                       sa=torch.empty((M,), dtype=torch.float32, device=dev),
                       out=torch.empty((M, N), dtype=torch.float16, device=dev),
                       ws=torch.empty(P.is_gemm_w8a8_workspace_bytes(M, N, K, GROUP), dtype=torch.uint8, device=dev))
    torch.cuda.synchronize()

    def gemm(M, l, int_scale):
        a = acts[M]
        if int_scale:
            P.is_gemm_w8a8_intscale(a["xq"], a["sa"], q[l], qw.scale_i32, qw.chan_scale, GROUP, ALPHA_LOG2, out=a["out"],
                                    workspace=a["ws"])
        else:
            P.is_gemm_w8a8_floatscale(a["xq"], a["sa"], q[l], qw.scale_f32, GROUP, out=a["out"], workspace=a["ws"])

    def run(int_scale, with_quant, steps, warmup):
        per = {M: 0.0 for M in MS}
        for it in range(warmup + steps):
            if it == warmup:
                torch.cuda.synchronize()
                t0 = time.perf_counter()
            for M in MS:
                a = acts[M]
                for l in range(L):
                    if with_quant:
                        P.is_quantize_act_int8_token(a["x"], a["xq"], a["sa"])
                    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    e0.record()
                    gemm(M, l, int_scale)
                    e1.record()
                    if it >= warmup:
                        a.setdefault("ev", []).append((e0, e1))
        torch.cuda.synchronize()
        sec = (time.perf_counter() - t0) / steps
        for M in MS:
            ev = acts[M].pop("ev")
            per[M] = 1e3 * sorted(x.elapsed_time(y) for x, y in ev)[len(ev) // 2]  # median: launches are eager
        return sec, per

    def alg_bytes(M):  # int8 weights, int32 scales, int8 activations, fp16 out, row/column scales
        return N * K + 4 * N * (K // GROUP) + M * K + 2 * M * N + 4 * M + 4 * N

    sec, per = run(True, True, args.steps, args.warmup)
    small = [M for M in MS if M <= 64]
    # value: the small-M calls only (quantiser + GEMM time measured per call below)
    small_us = sum(per[M] for M in small)
    value = sum(alg_bytes(M) for M in small) / small_us / 1e3
    shapes = [dict(name=f"w8a8_down_M{M}", us=round(per[M], 2), gbs=round(alg_bytes(M) / per[M] / 1e3, 1),
                   tops=round(2.0 * M * N * K / per[M] / 1e6, 1)) for M in MS]
    dom = max(small, key=lambda M: per[M])
    # the general kernel's int8 instance for this many token rows (as a rocprofv3 kernel trace names it)
    dom_kernel = "gemm_skinny_kernel<%d, 1, 2, true, true, true>" % (1 if dom <= 16 else 2 if dom <= 32 else 3 if dom <= 48 else 4)
    roofline = dict(bound="hbm", kernel=dom_kernel, achieved=round(alg_bytes(dom) / per[dom] / 1e3, 1),
                    peak=HBM_PEAK_GBS, unit="GB/s", frac=round(alg_bytes(dom) / per[dom] / 1e3 / HBM_PEAK_GBS, 4),
                    traffic=measured_traffic(dom_kernel, "w8a8"),
                    avg_launch_us=round(per[dom], 2), note=f"the M = {dom} call; M = 4096 (tiled kernel, MFMA bound): "
                    f"{2.0 * 4096 * N * K / per[4096] / 1e6:.0f} TOP/s = {2.0 * 4096 * N * K / per[4096] / 1e6 / MFMA_I8_PEAK_TOPS:.3f} of the int8 peak")
    peaks = measured_peaks(P, torch)
    roofline["frac_of_measured_peak"] = round(roofline["achieved"] / peaks["hbm_read_gbs"], 4)
    speedup = fs_detail = None
    if not args.no_floatscale:
        n = max(3, args.steps // 2)
        per_is = per
        _, per_fs = run(False, False, n, 2)
        fs_detail = {f"M{M}": round(per_fs[M] / per_is[M], 4) for M in MS}
        speedup = sum(per_fs.values()) / sum(per_is.values())
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import oracle as O
        M = 16
        hw = O.quantize_weights_int8_group(S.make_weights(3, N, K, S.seed_for(3, 2, 1)), GROUP, ALPHA_LOG2, O.SCALE_NORM)
        hx = S.make_activations(3, M, K, S.seed_for(3, 2, 2) + M)
        t0 = time.perf_counter()
        xq, sa = O.quantize_act_int8_token(hx)
        ref = O.gemm_w8a8_intscale(xq, sa, hw.qweight, hw.scale_i32, hw.chan_scale, GROUP, ALPHA_LOG2)
        dt = time.perf_counter() - t0
        a = acts[M]
        P.is_quantize_act_int8_token(a["x"], a["xq"], a["sa"])
        out, acc = P.is_gemm_w8a8_intscale(a["xq"], a["sa"], q[0], qw.scale_i32, qw.chan_scale, GROUP, ALPHA_LOG2,
                                           want_acc=True, workspace=a["ws"])
        torch.cuda.synchronize()
        got = out.cpu().numpy().astype(np.float64)
        cpu = dict(value=round(alg_bytes(M) / dt / 1e9, 3), unit="GB/s", cores=1, kind="oracle",
                   sample=f"the M = {M} call once (quantiser + integer-scale GEMM, numpy), {dt:.1f} s",
                   parity=dict(acc_bit_exact=bool(np.array_equal(acc.cpu().numpy(), ref.acc)),
                               weights_bit_exact=bool(np.array_equal(qw.qweight.cpu().numpy(), hw.qweight)),
                               max_rel_err=float(np.max(np.abs(got - ref.out) / np.maximum(np.abs(ref.out), 1e-3)))))
    line = {
        "metric": "W8A8 integer-scale GEMM TOPS + HBM GB/s (% roofline); speedup vs float-scale", "value": round(value, 1),
        "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(1e3 * sec, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "int8", "data": "synthetic",
        "config": {"workload": f"llama3-8b down projection ({K}->{N}) as fine-grained W8A8, group {GROUP}, alpha=2^{ALPHA_LOG2}, "
                               f"M in {list(MS)}, {L} distinct weight sets", "launch": "eager", "scale_mode": "norm"},
        "speedup_vs_floatscale": None if speedup is None else round(speedup, 4),
        "floatscale_over_intscale_by_shape": fs_detail, "roofline": roofline, "measured_peaks": peaks, "cpu_baseline": cpu,
        "shapes": shapes,
    }
    print(json.dumps(line))


def producers_main(args):
    """The activation quantiser folded into its producer, on LLaMA-3-8B shapes: RMSNorm + quantiser on [M, 4096]
    (in front of qkv and gate_up) and SiLU(gate) * up + quantiser on [M, 2 * 14336] (in front of down), at M = 4096
    (HBM bound; `value`) and M in {1, 16, 64} (latency bound; `shapes`).  Inputs rotate over enough buffers that each
    call reads from HBM.  One step = both calls at every M.  The library's plain quantiser on the same output shapes is
    timed beside them: the unfused chain costs at least that plus the producer's own pass."""
    import numpy as np
    import torch

    import paper_2405_14597_amd as P
    import synth_inputs as S

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    P.load_library()
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    K = S.LLAMA3_8B["qkv"][0]
    inter = S.LLAMA3_8B["down"][0]
    MS = (1, 16, 64, 4096)
    eps = 1e-5
    gamma = torch.from_numpy((1.0 + 0.1 * np.random.default_rng(1).standard_normal(K)).astype(np.float16)).to(dev)
    bufs = {}
    for M in MS:
        copies_x = max(2, min(16, (768 << 20) // (2 * M * K)))
        copies_g = max(2, min(16, (768 << 20) // (4 * M * inter)))
        x = torch.from_numpy(S.make_activations(3, M, K, S.seed_for(3, 0, 2) + M)).to(dev)
        g = torch.from_numpy(S.make_activations(3, M, 2 * inter, S.seed_for(3, 2, 3) + M)).to(dev)
        bufs[M] = dict(x=[x.clone() for _ in range(copies_x)], gu=[g.clone() for _ in range(copies_g)],
                       h=g[:, :inter].contiguous(),
                       xq=torch.empty((M, K), dtype=torch.int8, device=dev),
                       hq=torch.empty((M, inter), dtype=torch.int8, device=dev),
                       sa=torch.empty((M,), dtype=torch.float32, device=dev))
    torch.cuda.synchronize()

    def run(steps, warmup, fused=True):
        ev = {(M, k): [] for M in MS for k in ("norm", "silu")}
        for it in range(warmup + steps):
            if it == warmup:
                torch.cuda.synchronize()
                t0 = time.perf_counter()
            for M in MS:
                b = bufs[M]
                for k in ("norm", "silu"):
                    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    e0.record()
                    if k == "norm":
                        src = b["x"][it % len(b["x"])]
                        if fused:
                            P.is_rmsnorm_quantize_act_int8_token(src, gamma, eps, b["xq"], b["sa"])
                        else:
                            P.is_quantize_act_int8_token(src, b["xq"], b["sa"])
                    else:
                        if fused:
                            P.is_silu_mul_quantize_act_int8_token(b["gu"][it % len(b["gu"])], b["hq"], b["sa"])
                        else:
                            P.is_quantize_act_int8_token(b["h"], b["hq"], b["sa"])
                    e1.record()
                    if it >= warmup:
                        ev[(M, k)].append((e0, e1))
        torch.cuda.synchronize()
        sec = (time.perf_counter() - t0) / steps
        # medians: the launches are eager, a stall of the host between two of them would otherwise count
        return sec, {key: 1e3 * sorted(x.elapsed_time(y) for x, y in v)[len(v) // 2] for key, v in ev.items()}

    def alg_bytes(M, k):  # fp16 in, int8 out, one float per row (and gamma once)
        return 3 * M * K + 2 * K + 4 * M if k == "norm" else 5 * M * inter + 4 * M

    sec, per = run(args.steps, args.warmup)
    _, per_q = run(max(3, args.steps // 2), 2, fused=False)
    big = 4096
    value = sum(alg_bytes(big, k) for k in ("norm", "silu")) / (per[(big, "norm")] + per[(big, "silu")]) / 1e3
    shapes = [dict(name=f"{k}_quant_M{M}", us=round(per[(M, k)], 2), gbs=round(alg_bytes(M, k) / per[(M, k)] / 1e3, 1),
                   plain_quantiser_us=round(per_q[(M, k)], 2)) for M in MS for k in ("norm", "silu")]
    dom = max(("norm", "silu"), key=lambda k: per[(big, k)])
    ach = alg_bytes(big, dom) / per[(big, dom)] / 1e3
    kern = "silu_mul_quantize_resident_kernel<8, 256>" if dom == "silu" else "rmsnorm_quantize_resident_kernel<2, 256>"
    roofline = dict(bound="hbm", kernel=kern, achieved=round(ach, 1), peak=HBM_PEAK_GBS, unit="GB/s",
                    frac=round(ach / HBM_PEAK_GBS, 4), traffic=measured_traffic(kern, "producers"),
                    avg_launch_us=round(per[(big, dom)], 2))
    peaks = measured_peaks(P, torch)
    roofline["frac_of_measured_peak"] = round(ach / peaks["hbm_read_gbs"], 4)
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import oracle as O
        M = 1024
        hx = S.make_activations(3, M, K, S.seed_for(3, 0, 2) + M)
        hg = S.make_activations(3, M, 2 * inter, S.seed_for(3, 2, 3) + M)
        hgamma = gamma.cpu().numpy()
        t0 = time.perf_counter()
        rq, rs = O.rmsnorm_quantize_act_int8_token(hx, hgamma, eps)
        sq, ss = O.silu_mul_quantize_act_int8_token(hg)
        dt = time.perf_counter() - t0
        gq, gs = P.is_rmsnorm_quantize_act_int8_token(torch.from_numpy(hx).to(dev), gamma, eps)
        tq, ts = P.is_silu_mul_quantize_act_int8_token(torch.from_numpy(hg).to(dev))
        torch.cuda.synchronize()
        cpu = dict(value=round((alg_bytes(M, "norm") + alg_bytes(M, "silu")) / dt / 1e9, 3), unit="GB/s", cores=1,
                   kind="oracle", sample=f"both calls once at M = {M} (numpy), {dt:.1f} s",
                   parity=dict(norm_codes_bit_exact=bool(np.array_equal(gq.cpu().numpy(), rq)),
                               norm_scales_bit_exact=bool(np.array_equal(gs.cpu().numpy(), rs)),
                               silu_codes_bit_exact=bool(np.array_equal(tq.cpu().numpy(), sq)),
                               silu_scales_bit_exact=bool(np.array_equal(ts.cpu().numpy(), ss))))
    line = {
        "metric": "activation quantiser folded into its producer: HBM GB/s (% roofline)", "value": round(value, 1),
        "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(1e3 * sec, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"llama3-8b producers: RMSNorm+quant on [M,{K}], SiLU*up+quant on [M,2*{inter}], "
                               f"M in {list(MS)}; value = the M = {big} pair", "launch": "eager"},
        "roofline": roofline, "measured_peaks": peaks, "cpu_baseline": cpu, "shapes": shapes,
    }
    print(json.dumps(line))


def gate_up_main(args):
    """The front half of a gated feed-forward block, from the quantised input of gate_up to the quantised input of
    `down`, two ways on the prepacked route: (fused) the gate_up GEMM with SiLU(gate) * up as its epilogue, then the plain
    activation quantiser on [M, inter]; (unfused) the plain GEMM to [M, 2 inter], then SiLU * up folded into the
    quantiser.  LLaMA-3-8B (4096 -> 2 x 14336) at M = 4096 and LLaMA-2-70B (8192 -> 2 x 28672) at M = 2048 (tiled
    kernel: the epilogue is fused), and both at M = 32 (weight-streaming kernel: the [M, 2 inter] tensor goes through the
    workspace and a second kernel).  Each sequence is replayed as a HIP graph over `--layers` (default 2) weight copies.
    `value` = int8 operations of the fused sequences / their time."""
    import numpy as np
    import torch

    import paper_2405_14597_amd as P
    import synth_inputs as S

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    P.load_library()
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    L = args.layers if args.layers != 32 else 2
    cases = [("llama3-8b", 3, S.LLAMA3_8B["gate_up"][0], S.LLAMA3_8B["down"][0], (32, 4096)),
             ("llama2-70b", 2, S.LLAMA2_70B["gate"][0], S.LLAMA2_70B["gate"][1], (32, 2048))]
    segs, same = [], {}
    for label, cfg, K, inter, batches in cases:
        w = torch.from_numpy(S.make_weights(cfg, 2 * inter, K, S.seed_for(cfg, 2, 1))).to(dev)
        qw = P.is_quantize_weights_int4_group(w, GROUP, ALPHA_LOG2, P.IS_SCALE_NORM)
        del w
        plain = P.is_prepack_w4(qw.qweight, qw.scale_i32, GROUP)
        paired = P.is_prepack_w4_gate_up(qw.qweight, qw.scale_i32, qw.chan_scale, GROUP)
        torch.cuda.synchronize()
        plains = [plain] + [P.PackedWeights(plain.wpack.clone(), plain.spack.clone(), *plain[2:]) for _ in range(L - 1)]
        paireds = [paired] + [P.PackedGateUp(P.PackedWeights(paired.packed.wpack.clone(), paired.packed.spack.clone(),
                                                             *paired.packed[2:]), paired.chan_scale, inter)
                              for _ in range(L - 1)]
        for M in batches:
            x = torch.from_numpy(S.make_activations(cfg, M, K, S.seed_for(cfg, 2, 2) + M)).to(dev)
            xq, sa = P.is_quantize_act_int8_token(x)
            b = dict(xq=xq, sa=sa, gu=torch.empty((M, 2 * inter), dtype=torch.float16, device=dev),
                     h=torch.empty((M, inter), dtype=torch.float16, device=dev),
                     hq=torch.empty((M, inter), dtype=torch.int8, device=dev),
                     hs=torch.empty((M,), dtype=torch.float32, device=dev),
                     fws=torch.zeros(max(1, P.is_gemm_gate_up_silu_prepacked_workspace_bytes(M, inter, K, GROUP)),
                                     dtype=torch.uint8, device=dev),
                     gws=torch.zeros(max(1, P.is_gemm_prepacked_workspace_bytes(M, 2 * inter, K, GROUP)),
                                     dtype=torch.uint8, device=dev))

            def fused(b=b, paireds=paireds):
                for l in range(L):
                    P.is_gemm_w4a8_intscale_gate_up_silu_prepacked(b["xq"], b["sa"], paireds[l], ALPHA_LOG2, out=b["h"],
                                                                   workspace=b["fws"])
                    P.is_quantize_act_int8_token(b["h"], b["hq"], b["hs"])

            def unfused(b=b, plains=plains, c=qw.chan_scale):
                for l in range(L):
                    P.is_gemm_w4a8_intscale_prepacked(b["xq"], b["sa"], plains[l], c, ALPHA_LOG2, out=b["gu"],
                                                      workspace=b["gws"])
                    P.is_silu_mul_quantize_act_int8_token(b["gu"], b["hq"], b["hs"])

            # the two sequences give the same codes and token scales (both round the same fp16 products)
            fused()
            got = (b["hq"].clone(), b["hs"].clone())
            unfused()
            torch.cuda.synchronize()
            same[f"{label}_M{M}"] = bool(torch.equal(got[0], b["hq"]) and torch.equal(got[1], b["hs"]))
            for kind, fn in (("fused", fused), ("unfused", unfused)):
                seg = Segment(f"{label}_M{M}_{kind}", kind, L, 0, L * S.algorithmic_ops(M, 2 * inter, K), fn,
                              not args.no_graph, torch)
                seg.M, seg.K, seg.inter, seg.kind, seg.label = M, K, inter, kind, label
                segs.append(seg)
    torch.cuda.synchronize()

    def run_steps(n, timed):
        for _ in range(n):
            ev = torch.cuda.Event(enable_timing=True)
            ev.record()
            for s in segs:
                s.run()
                nxt = torch.cuda.Event(enable_timing=True)
                nxt.record()
                if timed:
                    s.pending.append((ev, nxt))
                ev = nxt

    run_steps(args.warmup, False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run_steps(args.steps, True)
    torch.cuda.synchronize()
    sec = (time.perf_counter() - t0) / args.steps
    us = {s.name: 1e3 * sum(a.elapsed_time(b) for a, b in s.pending) / (len(s.pending) * L) for s in segs}
    shapes = []
    for s in segs:
        if s.kind != "fused":
            continue
        other = s.name.replace("_fused", "_unfused")
        shapes.append(dict(name=f"{s.label}_M{s.M}", K=s.K, inter=s.inter, fused_us=round(us[s.name], 2),
                           unfused_us=round(us[other], 2), unfused_over_fused=round(us[other] / us[s.name], 3),
                           fused_tops=round(s.ops / L / us[s.name] / 1e6, 1)))
    fused = [s for s in segs if s.kind == "fused"]
    value = sum(s.ops / L for s in fused) / sum(us[s.name] for s in fused) / 1e6
    big = max(fused, key=lambda s: us[s.name])
    ach = big.ops / L / us[big.name] / 1e6
    roofline = dict(bound="mfma", kernel="gemm_tile_pk_kernel (SiLU * up epilogue) + quantiser", achieved=round(ach, 1),
                    peak=MFMA_I8_PEAK_TOPS, unit="TOP/s", frac=round(ach / MFMA_I8_PEAK_TOPS, 4), traffic=None,
                    avg_launch_us=round(us[big.name], 2), shape=big.name)
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import oracle as O
        rng = np.random.default_rng(11)
        M, inter, K = 1024, 14336, 4096
        xq = rng.integers(-128, 128, size=(M, K)).astype(np.int8)
        sa = (rng.random(M) * 0.02 + 0.001).astype(np.float32)
        q = O.pack_int4(rng.integers(-8, 8, size=(2 * inter, K)).astype(np.int8))
        IS = rng.integers(0, 1025, size=(2 * inter, K // GROUP)).astype(np.int32)
        c = (rng.random(2 * inter) * 0.01 + 0.001).astype(np.float32)
        t0 = time.perf_counter()
        r = O.gemm_w4a8_intscale(xq, sa, q, IS, c, GROUP, ALPHA_LOG2)
        h_ref = O.silu_mul_fp16(r.out.astype(np.float16))
        dt = time.perf_counter() - t0
        t = lambda a: torch.from_numpy(a).to(dev)
        gu = P.is_prepack_w4_gate_up(t(q), t(IS), t(c), GROUP)
        h, _ = P.is_gemm_w4a8_intscale_gate_up_silu_prepacked(t(xq), t(sa), gu, ALPHA_LOG2)
        got, want = h.cpu().numpy().astype(np.float64), h_ref.astype(np.float64)
        cpu = dict(value=round(2.0 * M * 2 * inter * K / dt / 1e12, 4), unit="TOP/s", cores=O.num_threads(), kind="oracle",
                   sample=f"GEMM of Eq. (2) (C, threaded) + SiLU * up (numpy) once at M = {M}, inter = {inter}, K = {K} "
                          f"(llama3-8b gate_up, a quarter of the rows), {dt:.1f} s",
                   parity=dict(within_1e_2=bool(np.all(np.abs(got - want) <= 1e-2 * np.abs(want) + 2.0 ** -24))))
    line = {
        "metric": "gate_up GEMM with SiLU(gate) * up epilogue + quantiser: int8 TOP/s (% roofline)",
        "value": round(value, 1), "unit": "TOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(1e3 * sec, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int8 x int4 -> int32", "data": "synthetic",
        "config": {"workload": "gated feed-forward front half (quantised x -> quantised input of down), fused epilogue "
                               "against GEMM + SiLU*up quantiser: llama3-8b M in {32, 4096}, llama2-70b M in {32, 2048}",
                   "launch": "eager" if args.no_graph else "HIP graph per sequence", "layers": L},
        "roofline": roofline, "cpu_baseline": cpu, "shapes": shapes, "fused_equals_unfused_bit_for_bit": same,
    }
    print(json.dumps(line))


def moe_main(args):
    """Mixtral-8x7B-shaped expert FFN as grouped GEMMs: 8 experts, 512 tokens, top-2 uniform router (1024 token rows,
    uneven per expert); w1 and w3 4096->14336, w2 14336->4096.  One step = quantiser + grouped integer-scale GEMM per
    linear on prepacked experts, over `--layers` (default 4 here) distinct sets of expert weights so that the weights come
    from HBM.  The canonical-layout grouped call is timed beside it (`canonical_us_by_shape`)."""
    import numpy as np
    import torch

    import paper_2405_14597_amd as P
    import synth_inputs as S

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    P.load_library()
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    E, TOKENS, TOPK = 8, 512, 2
    L = args.layers if args.layers != 32 else 4
    data = []
    for idx, (name, (K, N)) in enumerate(S.MIXTRAL_8X7B.items()):
        token, expert, offsets = S.moe_routing(TOKENS, E, TOPK, S.seed_for(4, idx, 3))
        x = torch.from_numpy(np.ascontiguousarray(S.make_activations(4, TOKENS, K, S.seed_for(4, idx, 2))[token])).to(dev)
        M = x.shape[0]
        qs = []
        for e in range(E):
            w = torch.from_numpy(S.make_weights(4, N, K, S.seed_for(4, idx, 1) + 7 * e)).to(dev)
            qs.append(P.is_quantize_weights_int4_group(w, GROUP, ALPHA_LOG2, P.IS_SCALE_NORM))
            del w
        stack = lambda f: torch.stack([f(q) for q in qs]).unsqueeze(0).repeat(L, *([1] * (f(qs[0]).dim() + 1)))
        data.append(dict(name=name, K=K, N=N, M=M, counts=np.diff(offsets).tolist(), off=torch.from_numpy(offsets).to(dev),
                         q=stack(lambda q: q.qweight), si=stack(lambda q: q.scale_i32), sf=stack(lambda q: q.scale_f32),
                         c=stack(lambda q: q.chan_scale), x=x,
                         xq=torch.empty((M, K), dtype=torch.int8, device=dev),
                         sa=torch.empty((M,), dtype=torch.float32, device=dev),
                         out=torch.empty((M, N), dtype=torch.float16, device=dev),
                         ws=torch.empty(P.is_gemm_grouped_workspace_bytes(E, M, N, K, GROUP), dtype=torch.uint8, device=dev),
                         pws=torch.empty(P.is_gemm_grouped_prepacked_workspace_bytes(E, M, N, K, GROUP), dtype=torch.uint8,
                                         device=dev)))
        d = data[-1]
        d["pi"] = [P.is_prepack_w4_experts(d["q"][l], d["si"][l], GROUP) for l in range(L)]
        d["pf"] = [P.is_prepack_w4_experts(d["q"][l], d["sf"][l], GROUP) for l in range(L)]
        del qs
    torch.cuda.synchronize()

    def quant(d):
        P.is_quantize_act_int8_token(d["x"], d["xq"], d["sa"])

    def gemm(d, l, int_scale, canonical=False):
        if not canonical:
            if int_scale:
                P.is_gemm_w4a8_intscale_grouped_prepacked(d["xq"], d["sa"], d["pi"][l], d["c"][l], d["off"], ALPHA_LOG2,
                                                          out=d["out"], workspace=d["pws"])
            else:
                P.is_gemm_w4a8_floatscale_grouped_prepacked(d["xq"], d["sa"], d["pf"][l], d["off"], out=d["out"],
                                                            workspace=d["pws"])
        elif int_scale:
            P.is_gemm_w4a8_intscale_grouped(d["xq"], d["sa"], d["q"][l], d["si"][l], d["c"][l], d["off"], GROUP, ALPHA_LOG2,
                                            out=d["out"], workspace=d["ws"])
        else:
            P.is_gemm_w4a8_floatscale_grouped(d["xq"], d["sa"], d["q"][l], d["sf"][l], d["off"], GROUP, out=d["out"],
                                              workspace=d["ws"])

    replays = {}

    def replay_of(d, int_scale, with_quant, canonical):
        """The L calls of one linear (one per set of expert weights) as one HIP graph (eager with --no-graph)."""
        key = (d["name"], int_scale, with_quant, canonical)
        if key not in replays:
            def calls():
                for l in range(L):
                    if with_quant:
                        quant(d)
                    gemm(d, l, int_scale, canonical)
            if args.no_graph:
                replays[key] = calls
            else:
                calls()                # every buffer is touched before capture
                torch.cuda.synchronize()
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g):
                    calls()
                replays[key] = g.replay
        return replays[key]

    def run(int_scale, with_quant, steps, warmup, canonical=False):
        per = {d["name"]: 0.0 for d in data}
        fns = [replay_of(d, int_scale, with_quant, canonical) for d in data]
        for it in range(warmup + steps):
            if it == warmup:
                torch.cuda.synchronize()
                t0 = time.perf_counter()
            for d, fn in zip(data, fns):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                fn()
                e1.record()
                if it >= warmup:
                    d.setdefault("marks", []).append((e0, e1))
        torch.cuda.synchronize()
        sec = (time.perf_counter() - t0) / steps
        for d in data:
            per[d["name"]] = sum(a.elapsed_time(b) for a, b in d.pop("marks")) / (steps * L)
        return sec, per

    sec_per_step, _ = run(True, True, args.steps, args.warmup)     # the step: quantiser + grouped GEMM per linear
    _, per = run(True, False, max(3, args.steps // 2), 2)          # the grouped GEMM calls alone (per-shape figures)

    def alg_bytes(d):  # every expert's weights and scales once, the routed rows once
        return E * (d["N"] * d["K"] // 2 + 4 * d["N"] * (d["K"] // GROUP) + 4 * d["N"]) + d["M"] * d["K"] + 2 * d["M"] * d["N"] + 4 * d["M"]

    step_bytes = L * sum(alg_bytes(d) + 3 * d["M"] * d["K"] + 4 * d["M"] for d in data)
    step_ops = L * sum(S.algorithmic_ops(d["M"], d["N"], d["K"]) for d in data)
    shapes = []
    for d in data:
        ms = per[d["name"]]
        t_hbm = alg_bytes(d) / (HBM_PEAK_GBS * 1e9)
        t_mfma = S.algorithmic_ops(d["M"], d["N"], d["K"]) / (MFMA_I8_PEAK_TOPS * 1e12)
        shapes.append(dict(name=f"grouped_{d['name']}", rows_per_expert=d["counts"], us=round(1e3 * ms, 2),
                           gbs=round(alg_bytes(d) / ms / 1e6, 1), tops=round(S.algorithmic_ops(d["M"], d["N"], d["K"]) / ms / 1e9, 1),
                           roofline_frac=round(max(t_hbm, t_mfma) / (ms * 1e-3), 4)))
    tot_ms = sum(per.values())
    achieved = sum(alg_bytes(d) for d in data) / tot_ms / 1e6
    kernel = P.is_describe_grouped_prepacked(E, data[0]["M"], data[0]["N"], data[0]["K"], GROUP, True)[-1]
    roofline = dict(bound="hbm", kernel=kernel, achieved=round(achieved, 1), peak=HBM_PEAK_GBS, unit="GB/s",
                    frac=round(achieved / HBM_PEAK_GBS, 4), traffic=measured_traffic(kernel, "moe"),
                    avg_launch_us=round(1e3 * tot_ms / len(data), 2),
                    note="per grouped call (tile kernel plus preparation kernels); near the ridge: per-shape "
                         "roofline_frac takes the larger of the HBM and the MFMA time")
    peaks = measured_peaks(P, torch)
    roofline["frac_of_measured_peak"] = round(achieved / peaks["hbm_read_gbs"], 4)
    speedup = fs_detail = canon = None
    if not args.no_floatscale:
        n = max(3, args.steps // 2)
        per_is = per
        _, per_fs = run(False, False, n, 2)
        speedup = sum(per_fs.values()) / sum(per_is.values())
        fs_detail = {k: round(per_fs[k] / per_is[k], 4) for k in per_is}
        _, per_canon = run(True, False, n, 2, canonical=True)
        canon = {k: round(1e3 * v, 2) for k, v in per_canon.items()}
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import oracle as O
        dt, cpu_bytes, ok_all, rel_all = 0.0, 0, True, 0.0
        for d in data:
            xq_h = None
            quant(d)
            torch.cuda.synchronize()
            x_h = d["x"].cpu().numpy()
            q_h, si_h, c_h, off_h = (d["q"][0].cpu().numpy(), d["si"][0].cpu().numpy(), d["c"][0].cpu().numpy(),
                                     d["off"].cpu().numpy())
            t0 = time.perf_counter()
            xq_h, sa_h = O.quantize_act_int8_token(x_h)
            acc_ref, out_ref = O.gemm_w4a8_intscale_grouped(xq_h, sa_h, q_h, si_h, c_h, off_h, GROUP, ALPHA_LOG2)
            dt += time.perf_counter() - t0
            cpu_bytes += alg_bytes(d) + 3 * d["M"] * d["K"] + 4 * d["M"]
            out, acc = P.is_gemm_w4a8_intscale_grouped_prepacked(d["xq"], d["sa"], d["pi"][0], d["c"][0], d["off"],
                                                                 ALPHA_LOG2, want_acc=True, workspace=d["pws"])
            torch.cuda.synchronize()
            ok_all = ok_all and bool(np.array_equal(acc.cpu().numpy(), acc_ref))
            got, want = out.cpu().numpy().astype(np.float64), out_ref.astype(np.float64)
            rel_all = max(rel_all, float(np.max(np.abs(got - want) / np.maximum(np.abs(want), 1e-3))))
        cpu = dict(value=round(cpu_bytes / dt / 1e9, 3), unit="GB/s", cores=O.num_threads(), kind="oracle",
                   sample=f"one of {L} weight sets, all three grouped linears (quantiser + integer-scale GEMM; the expert "
                          f"weights were quantised on the GPU, bit-identical to the oracle's), {dt:.1f} s",
                   parity=dict(acc_bit_exact=ok_all, max_rel_err=rel_all))
    value = step_bytes / sec_per_step / 1e9
    line = {
        "metric": "W4A8 integer-scale GEMM TOPS + HBM GB/s (% roofline); speedup vs float-scale",
        "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(1e3 * sec_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int8", "data": "synthetic",
        "config": {"workload": f"mixtral-8x7b expert FFN (w1, w3, w2) as grouped GEMMs over {E} experts, {TOKENS} tokens top-{TOPK} "
                               f"uniform router, W4 group-128 x A8 per-token, alpha=2^{ALPHA_LOG2}, {L} sets of expert weights",
                   "layout": "experts prepacked offline (is_prepack_w4)",
                   "launch": "eager" if args.no_graph else "hip-graph", "scale_mode": "norm"},
        "tops": round(step_ops / sec_per_step / 1e12, 3), "hbm_frac": round(value / HBM_PEAK_GBS, 4),
        "speedup_vs_floatscale": None if speedup is None else round(speedup, 4),
        "floatscale_over_intscale_by_shape": fs_detail, "canonical_us_by_shape": canon, "roofline": roofline, "measured_peaks": peaks,
        "cpu_baseline": cpu, "shapes": shapes,
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
