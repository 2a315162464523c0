#!/usr/bin/env python3
"""Benchmark of the MoQE hot path on one MI355X.

A step is one pass of the whole hot path over one batch: moqe_moe_layer, i.e. top-1
gating, histogram, scan, permutation, then FFN1 + bias + ReLU, FFN2 + bias and the
gate-weighted combine, on one MoE layer.  The default workload is the decode
configuration the metric is quoted on (c1: E=32 experts, d_model 1024, d_ff 4096, batch
of 24 tokens, int4 experts: three kernel launches per step); --workload selects the
other configurations (c3: 1536 tokens under Zipf load; c4_*: a layer of the 12-layer
int2 stack with the residual add, at 24 or 4096 tokens).
Consecutive steps use different layer copies (own weights, own router) so that the
packed weights of a step are not left in the 256 MB last-level cache by the previous
one: the weights really come from HBM.

Prints ONE JSON line: tokens/s (metric), ms per step, the roofline of the dominant
kernel (algorithmic bytes or flops per launch / measured kernel time, against the
8 TB/s HBM peak or the 2.5 PFLOP/s fp16 MFMA peak; for the HBM-bound workloads also
against a plain streaming read of the same number of bytes measured in the same run)
and the CPU oracle timed on the host's cores on a bounded sample of the same workload.
The decode workloads (c1, c2) time int4, int3 and int2 experts (`by_bits`).
"""

from __future__ import annotations

import argparse
import ctypes
import dataclasses
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_F16_PEAK_TFLOPS = 2500.0

# HBM traffic per launch of the dominant kernel measured with rocprofv3 --pmc (FETCH_SIZE and
# WRITE_SIZE runs of this script, each scaled by what the same counter reads for a 256 MiB
# device copy in the same run); from the profiles/*_hbm_traffic.txt summaries.  None where no
# counter run was made.  FFN1 of c1 (read + written; profiles/decode_c1_hbm_traffic.txt); for the
# many-token workloads the mean of the FFN1 and the FFN2 launch, as their time is reported
# (profiles/prefill_c3_int4.txt, profiles/prefill_c4_T4096_int2.txt):
MEASURED_TRAFFIC_BYTES = {("c1", 4): 39711835, ("c1", 3): 30099886, ("c1", 2): 20402059,
                          ("c3", 4): 84020000, ("c4_T4096_uniform", 2): 100735000}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=400)
    ap.add_argument("--warmup", type=int, default=40)
    ap.add_argument("--workload", default="c1",
                    choices=("c1", "c2", "c3", "c4_T24_uniform", "c4_T24_zipf", "c4_T4096_uniform", "c4_T4096_zipf",
                             "n2_e128", "n2_dense", "c1_T64", "c1_T64_zipf"))
    ap.add_argument("--bits", type=int, default=None, choices=(2, 3, 4, 8, 16),
                    help="bit width of the headline line (default: the workload's own)")
    ap.add_argument("--codec", default="linear", choices=("linear", "log"),
                    help="log: log-scale codes (App. A) instead of linear ones; needs --bits 2, 3 or 4")
    ap.add_argument("--copies", type=int, default=None, help="independent layer copies cycled through "
                    "(default 8; 12 for the c4 stack: its 12 layers)")
    ap.add_argument("--other-bits", action="store_true", help="also time the remaining widths (fp16, int8, and 4 / 3 / "
                    "2 bits where the workload does not time them anyway)")
    ap.add_argument("--only-bits", action="store_true", help="time the headline width alone")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-steps", type=int, default=None, help="oracle steps timed, the median is reported (default 5; 1 from 512 tokens on)")
    ap.add_argument("--no-graph", action="store_true", help="time eager launches only")
    ap.add_argument("--parts", action="store_true", help="also time each kernel of the step on its own")
    ap.add_argument("--decode", default="auto", choices=("auto", "general", "rows8", "rows4"),
                    help="which decode kernel serves batches of at most 64 tokens (moqe_set_decode_kernel)")
    ap.add_argument("--tiled", default="auto", choices=("auto", "streamed", "resident"),
                    help="which tiled kernel serves many-token segments (moqe_set_tiled_kernel); default: the library's choice")
    ap.add_argument("--tokens", type=int, default=None, metavar="T",
                    help="batch size in place of the workload's own (same layer, same routing recipe)")
    ap.add_argument("--prefill-policy", default=None, metavar="SEG,BATCH,PER_EXPERT",
                    help="thresholds of the path choice (moqe_set_prefill_policy) in place of the library's defaults")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="MiB",
                    help="also run three plain device-to-device copies of this size first: under "
                         "rocprofv3 --pmc they give the counter reading of a known amount of traffic")
    return ap.parse_args()


def algorithmic_bytes(seg_offsets, bits, d, f, T, residual):
    """Bytes the method must move for one layer-step, split per contraction.
    Per active expert: packed codes + fp16 scales + fp16 biases of the matrix;
    plus the fp16 activations entering and leaving the layer (x in FFN1, y in
    FFN2, the residual where the layer adds one).  The hidden activations h are
    not counted; the caller adds the router weights (2 d E)."""
    counts = np.diff(np.asarray(seg_offsets))
    active = int((counts > 0).sum())
    ffn1 = active * (d * f * bits // 8 + 2 * f + 2 * f) + 2 * T * d
    ffn2 = active * (d * f * bits // 8 + 2 * d + 2 * d) + 2 * T * d + (2 * T * d if residual else 0)
    return active, ffn1, ffn2


LOG_CODEC = False  # set from --codec: the 4-bit codes are log-scale ones


def wname(bits):
    """Weight format name of a bit width (16 = the unquantized baseline)."""
    if LOG_CODEC and bits in (2, 3, 4):
        return "log%d" % bits
    return "fp16" if bits == 16 else "int%d" % bits


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (--gpus must be 1)", file=sys.stderr)
        sys.exit(2)

    import torch

    from paper_2310_02410_amd import moqe, workloads as W
    from paper_2310_02410_amd import build as B

    if not os.path.exists(moqe.LIB_PATH):
        B.build_library()
    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)
    moqe.moqe_set_tiled_kernel({"auto": moqe.TILED_AUTO, "streamed": moqe.TILED_STREAMED, "resident": moqe.TILED_RESIDENT}[args.tiled])
    moqe.moqe_set_decode_kernel({"auto": moqe.DECODE_AUTO, "general": moqe.DECODE_GENERAL, "rows8": moqe.DECODE_ROWS8,
                                 "rows4": moqe.DECODE_ROWS4}[args.decode])
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()

    variants = dict(W.CONFIGS)
    variants.update({v.name: v for v in W.c4_variants()})
    variants.update(W.EXTRA)
    wl = variants[args.workload]
    if args.tokens is not None:
        if args.tokens < 1:
            print("bench.py: --tokens must be positive", file=sys.stderr)
            sys.exit(2)
        wl = dataclasses.replace(wl, name="%s_T%d" % (wl.name, args.tokens), T=args.tokens)
    if args.prefill_policy is not None:
        try:
            thresholds = [int(v) for v in args.prefill_policy.split(",")]
            if len(thresholds) != 3:
                raise ValueError
            moqe.moqe_set_prefill_policy(*thresholds)
        except ValueError:
            print("bench.py: --prefill-policy takes three integers >= 1, e.g. 5,65,16", file=sys.stderr)
            sys.exit(2)
    E, d, f, T = wl.E, wl.d, wl.f, wl.T
    residual = wl.layers > 1               # the stack adds the layer's output to its input
    compute_bound = T >= 512               # the tiled MFMA kernel dominates, not the weight stream
    global LOG_CODEC
    LOG_CODEC = args.codec == "log"
    bits0 = args.bits if args.bits is not None else wl.bits[0]
    if LOG_CODEC and bits0 not in (2, 3, 4):
        print("bench.py: --codec log needs --bits 2, 3 or 4", file=sys.stderr)
        sys.exit(2)
    # the metric is quoted at int4 / int3 / int2: the decode workloads time all three
    decode_set = [4, 3, 2] if (wl.name in ("c1", "c2") and not LOG_CODEC and not args.only_bits) else []
    bit_list = [bits0] + [b for b in decode_set if b != bits0]
    if args.other_bits:
        bit_list += [b for b in (16, 8, 4, 3, 2) if b not in bit_list]
    copies = args.copies if args.copies is not None else (12 if wl.layers > 1 else 8)
    steps, warmup = args.steps, args.warmup
    if compute_bound and steps == 400 and warmup == 40:
        steps, warmup = 100, 10            # defaults sized to keep the timed work near a minute at most
    cpu_steps = args.cpu_steps if args.cpu_steps is not None else (1 if compute_bound else 5)

    # ---- layer copies: generated on the host (seeded), quantized on the device ----
    t0 = time.time()
    layers = {b: [] for b in bit_list}
    layer0_host = None
    for i in range(copies):
        host = W.make_layer(wl, layer=i)
        if i == 0:
            layer0_host = host
        w1, w2 = dev(host["w1"]), dev(host["w2"])
        b1, b2, wg = dev(host["b1"]), dev(host["b2"]), dev(host["w_gate"])
        for b in bit_list:
            codec = moqe.CODEC_LOG if (LOG_CODEC and b in (2, 3, 4)) else moqe.CODEC_LINEAR
            layers[b].append(moqe.quantize_layer(w1, b1, w2, b2, b, wg, codec=codec))
        del w1, w2
        torch.cuda.synchronize()
        print(f"[bench] layer copy {i + 1}/{copies} ready ({time.time() - t0:.0f}s)", file=sys.stderr, flush=True)
    x_host = W.make_tokens(wl)
    x = dev(x_host)

    if args.copy_calibration > 0:
        src = torch.full((args.copy_calibration << 20,), 7, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    L = moqe.lib()
    route, _ = moqe.alloc_route(T, E, x.device)
    ws = moqe.alloc_workspace(moqe.moqe_layer_workspace_bytes(T, E, d, f), x.device)
    y = torch.empty_like(x)
    hbuf = torch.empty((T, f), dtype=torch.float16, device="cuda")

    def make_calls(qls):
        """ctypes calls with every argument marshalled once: the whole step and its parts."""
        structs = [ql.c_struct() for ql in qls]
        refs = [ctypes.byref(s) for s in structs]
        gates = [ql.w_gate.data_ptr() for ql in qls]
        xp, yp, hp = x.data_ptr(), y.data_ptr(), hbuf.data_ptr()
        rp = xp if residual else None
        ip, gp, sp, pp = (route.expert_idx.data_ptr(), route.gate.data_ptr(), route.seg_offsets.data_ptr(),
                          route.perm.data_ptr())
        wsp, wsn = ws.data_ptr(), ws.numel()
        n = len(qls)

        def check(st, what):
            if st:
                raise RuntimeError(f"{what} failed with status {st}")

        def step(i, stream):
            check(L.moqe_moe_layer(refs[i % n], gates[i % n], xp, T, ip, gp, sp, pp, rp, yp, wsp, wsn, stream),
                  "moqe_moe_layer")

        def ffn1(i, stream):
            check(L.moqe_expert_ffn1(refs[i % n], xp, T, sp, pp, hp, stream), "moqe_expert_ffn1")

        def ffn2(i, stream):
            check(L.moqe_expert_ffn2(refs[i % n], hp, T, gp, sp, pp, rp, yp, stream), "moqe_expert_ffn2")

        def router(i, stream):
            check(L.moqe_route(xp, gates[i % n], T, d, E, ip, gp, sp, pp, wsp, wsn, stream), "moqe_route")

        step.keep = (structs, refs)
        return step, ffn1, ffn2, router

    def time_steps(run, nsteps, nwarm):
        """(wall ms per step with a sync on both sides, HIP-event ms per step on the launch stream)"""
        for i in range(nwarm):
            run(i)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t = time.perf_counter()
        e0.record()
        for i in range(nsteps):
            run(nwarm + i)
        e1.record()
        torch.cuda.synchronize()
        return (time.perf_counter() - t) * 1e3 / nsteps, e0.elapsed_time(e1) / nsteps

    def time_graph(run, nsteps, nwarm):
        """The same calls captured once per layer copy into ONE graph (a pass over all copies),
        replayed: launch cost leaves the picture.  At least 10 replays, each timed by its own
        pair of events.  Returns (ms per step over all replays together, median and min over the
        replays of a replay's ms per step)."""
        side = torch.cuda.Stream()
        with torch.cuda.stream(side):
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=side):
                for k in range(copies):
                    run(k, torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        reps = max(10, nsteps // copies)
        for _ in range(max(2, nwarm // copies)):
            g.replay()
        torch.cuda.synchronize()
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(reps + 1)]
        ev[0].record()
        for i in range(reps):
            g.replay()
            ev[i + 1].record()
        torch.cuda.synchronize()
        each = np.array([ev[i].elapsed_time(ev[i + 1]) for i in range(reps)]) / copies
        return ev[0].elapsed_time(ev[reps]) / reps / copies, float(np.median(each)), float(each.min())

    # ---- the ceiling: a plain streaming read of as many bytes as the dominant kernel's launch
    # must read, on memory that is not cache resident (an arena twice the last-level cache,
    # walked launch by launch), in the decode kernels' launch shape ----
    arena = None
    sink = torch.zeros(64, dtype=torch.uint8, device="cuda")

    def time_stream_read(nbytes, nlaunch=200):
        nonlocal arena
        if arena is None:
            arena = torch.empty(768 << 20, dtype=torch.uint8, device="cuda").fill_(1)
        nbytes = max(1024, int(nbytes) // 1024 * 1024)
        stride = (nbytes + (2 << 20) - 1) // (2 << 20) * (2 << 20)
        slots = arena.numel() // stride
        stream = torch.cuda.current_stream().cuda_stream
        base, sp = arena.data_ptr(), sink.data_ptr()

        def go(i):
            st = L.moqe_stream_read(base + (i % slots) * stride, nbytes, sp, stream)
            if st:
                raise RuntimeError(f"moqe_stream_read failed with status {st}")
        _, ev = time_steps(go, nlaunch, 20)
        return ev * 1e3  # us per launch, back to back

    kbits = lambda b: 100 + b if (LOG_CODEC and b in (2, 3, 4)) else b  # the width the kernels are instantiated on
    results = {}
    for b in bit_list:
        qls = layers[b]
        step, ffn1, ffn2, router = make_calls(qls)
        stream = torch.cuda.current_stream().cuda_stream
        # realised routing of every layer copy -> algorithmic bytes of its step
        ab = []
        for k in range(len(qls)):
            step(k, stream)
            torch.cuda.synchronize()
            ab.append(algorithmic_bytes(route.seg_offsets.cpu().numpy(), b, d, f, T, residual))
        if moqe.workspace_error(ws):
            raise RuntimeError("a phase wait timed out: results invalid")
        # ---- the timed region: K whole steps ----
        eager_ms, eager_ev_ms = time_steps(lambda i: step(i, stream), steps, warmup)
        graph_ms, graph_med_ms, graph_min_ms = (None, None, None) if args.no_graph else time_graph(step, steps, warmup)
        # ---- the step's kernels on their own: the same launches through the per-step entry
        # points, K of them back to back between two HIP events on the launch stream.  The
        # dominant kernel is the expert contraction (FFN1 and FFN2 run the same kernel on
        # matrices of the same size).  Inside a step the same kernel runs a little longer,
        # because it starts on an idle chip instead of behind its predecessor's tail; the
        # committed profile summaries list both populations.
        parts = {}
        for name, fn in (("router", router), ("ffn1", ffn1), ("ffn2", ffn2)):
            _, ev = time_steps(lambda i: fn(i, stream), max(steps, 100), warmup)
            parts[name + "_back_to_back_us"] = ev * 1e3
        if moqe.workspace_error(ws):
            raise RuntimeError("a phase wait timed out: results invalid")

        layer_bytes = float(np.mean([a[1] + a[2] for a in ab])) + 2 * d * E
        ffn1_bytes = float(np.mean([a[1] for a in ab]))
        best_ms = min(eager_ms, graph_ms) if graph_ms is not None else eager_ms
        # what a step takes beyond its three kernels launched back to back on their own: inside a
        # step each kernel starts on an idle chip behind a different predecessor (the profile
        # summaries under profiles/ list the in-step durations kernel by kernel)
        parts["step_minus_parts_us"] = best_ms * 1e3 - sum(v for k, v in parts.items() if k.endswith("_back_to_back_us"))
        res = dict(ms_per_step=best_ms, eager_ms=eager_ms, graph_ms=graph_ms, graph_median_ms=graph_med_ms,
                   graph_min_ms=graph_min_ms, tokens_per_s=T / (best_ms * 1e-3),
                   active_experts=float(np.mean([a[0] for a in ab])), layer_bytes=layer_bytes, parts=parts,
                   step_gbs=layer_bytes / (best_ms * 1e-3) / 1e9, step_tflops=4.0 * T * d * f / (best_ms * 1e-3) / 1e12)
        # which kernels the two contractions launch at this size and width (the library's own answer)
        kb = kbits(b)
        paths = (moqe.moqe_contraction_path(b, T, E, d, f), moqe.moqe_contraction_path(b, T, E, f, d))
        tiled = all(p & (moqe.PATH_TILED_RESIDENT | moqe.PATH_TILED_STAGED) for p in paths)

        def kernels_of(p, mode):
            names = []
            if p & moqe.PATH_DECODE_SMALL:
                names.append("moe_decode_small_kernel<%d,*,%d,*>" % (kb, mode))
            if p & moqe.PATH_DECODE:
                names.append("moe_decode_kernel<%d,*,2>" % kb)
            if p & moqe.PATH_TILED_RESIDENT:
                names.append("moe_resident_kernel<%d,2,8,*,%d>" % (kb, mode))
            if p & moqe.PATH_TILED_STAGED:
                names.append("moe_prefill_kernel<%d,*>" % kb)
            return " + ".join(names)
        if compute_bound and tiled:
            # one launch of a tiled kernel per contraction, 2 T d f flops each
            kern_us = 0.5 * (parts["ffn1_back_to_back_us"] + parts["ffn2_back_to_back_us"])
            flops = 2.0 * T * d * f
            res.update(bound="mfma", kernel_us=kern_us, kernel_work=flops, achieved=flops / (kern_us * 1e-6) / 1e12,
                       peak=MFMA_F16_PEAK_TFLOPS, unit="TFLOP/s",
                       kernel="FFN1: %s; FFN2: %s (each launched back to back, the two averaged)"
                              % (kernels_of(paths[0], 0), kernels_of(paths[1], 1)))
        else:
            # below some hundred tokens the weight bytes set the time, whichever kernel reads them
            kern_us = parts["ffn1_back_to_back_us"]
            read_us = time_stream_read(ffn1_bytes)
            res.update(bound="hbm", kernel_us=kern_us, kernel_work=ffn1_bytes, ceiling_us=read_us,
                       ceiling_gbs=ffn1_bytes / (read_us * 1e-6) / 1e9,
                       achieved=ffn1_bytes / (kern_us * 1e-6) / 1e9, peak=HBM_PEAK_GBS, unit="GB/s",
                       kernel="%s (FFN1; FFN2 on a matrix of the same size: %s)"
                              % (kernels_of(paths[0], 0), kernels_of(paths[1], 1)))
        results[b] = res
        print(f"[bench] {wl.name} {wname(b)}: eager {eager_ms * 1e3:.1f} us/step (events {eager_ev_ms * 1e3:.1f}), graph "
              f"{(graph_ms or float('nan')) * 1e3:.1f} us/step; dominant kernel {res['kernel_us']:.1f} us = "
              f"{res['achieved']:.0f} {res['unit']}; parts {json.dumps(parts)}", file=sys.stderr, flush=True)

    # ---- CPU oracle on the host cores: bounded sample of the same workload ----
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import moqe_oracle as O
        ql0 = layers[bits0][0]
        c1, c2 = ql0.codes1.cpu().numpy(), ql0.codes2.cpu().numpy()
        s1, s2 = ql0.scales1.cpu().numpy(), ql0.scales2.cpu().numpy()
        cores = len(os.sched_getaffinity(0))

        class Lazy:
            """Unpacks and dequantizes an expert's matrix from its packed codes on access."""
            def __init__(self, codes, scales, K, N):
                self.codes, self.scales, self.K, self.N = codes, scales, K, N

            def __getitem__(self, e):
                if bits0 == 16:
                    return O.unpack_fp16(self.codes[e], self.K, self.N).astype(np.float64)
                if LOG_CODEC:
                    return O.dequantize_log(O.unpack(self.codes[e], bits0, self.K, self.N), self.scales[e], bits0)
                return O.dequantize(O.unpack(self.codes[e], bits0, self.K, self.N), self.scales[e])

        times = []
        for _ in range(cpu_steps):
            t = time.perf_counter()
            idx, gate, offs, perm = O.route(x_host, layer0_host["w_gate"])
            O.expert_ffn(x_host, idx, gate, Lazy(c1, s1, d, f), layer0_host["b1"], Lazy(c2, s2, f, d),
                         layer0_host["b2"], residual=x_host if residual else None)
            times.append(time.perf_counter() - t)
        med = float(np.median(times))
        cpu = dict(value=T / med, unit="tokens/s", cores=cores, kind="oracle",
                   sample=f"median of {cpu_steps} step(s) of route + expert FFN on layer copy 0 (T={T}, {wname(bits0)}, fp64, "
                          f"codes unpacked per call), {sum(times):.1f} s in all, fastest step {min(times):.2f} s")

    r = results[bits0]
    out = {
        "metric": "expert-FFN tokens/s (route + %s expert FFN, one MoE layer step)" % wname(bits0),
        "value": r["tokens_per_s"], "unit": "tokens/s", "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": r["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "%s weights x f16 activations, f32 accumulate" % wname(bits0), "data": "synthetic",
        "config": {"workload": "%s: E=%d d_model=%d d_ff=%d T=%d top-1 (%s load), %s experts%s, seed %d, "
                               "%d layer copies cycled" % (wl.name, E, d, f, T, wl.routing,
                                                           "unquantized fp16" if bits0 == 16 else
                                                           "%d-bit log-scale codes, per-channel absmax" % bits0 if LOG_CODEC else
                                                           "int%d per-channel RTN" % bits0,
                                                           ", fp16 residual add" if residual else "", wl.seed, copies),
                   "launch": "hip graph replay" if (r["graph_ms"] is not None and r["graph_ms"] <= r["eager_ms"]) else "eager",
                   "eager_ms_per_step": r["eager_ms"], "graph_ms_per_step": r["graph_ms"],
                   "graph_replay_ms_per_step_median": r["graph_median_ms"], "graph_replay_ms_per_step_min": r["graph_min_ms"],
                   "active_experts": r["active_experts"], "layer_algorithmic_bytes": r["layer_bytes"],
                   "step_gb_per_s": r["step_gbs"], "step_tflop_per_s": r["step_tflops"], "kernels_us": r["parts"]},
        "roofline": {"bound": r["bound"], "achieved": r["achieved"], "peak": r["peak"], "unit": r["unit"],
                     "frac": r["achieved"] / r["peak"], "traffic": MEASURED_TRAFFIC_BYTES.get((wl.name, bits0)),
                     "kernel": r["kernel"], "avg_kernel_us": r["kernel_us"],
                     **({"ceiling_gb_per_s": r["ceiling_gbs"], "frac_of_ceiling": r["achieved"] / r["ceiling_gbs"],
                         "ceiling": "plain streaming read of the same number of bytes (moqe_stream_read, back to back "
                                    "on memory that is not cache resident): %.2f us per launch" % r["ceiling_us"]}
                        if r["bound"] == "hbm" else {}),
                     ("algorithmic_flops_per_launch" if r["bound"] == "mfma" else "algorithmic_bytes_per_launch"):
                         r["kernel_work"]},
        "cpu_baseline": cpu,
    }
    if len(results) > 1:
        out["by_bits"] = {str(b): {"tokens_per_s": v["tokens_per_s"], "ms_per_step": v["ms_per_step"],
                                   "graph_replay_ms_per_step_median": v["graph_median_ms"],
                                   "graph_replay_ms_per_step_min": v["graph_min_ms"],
                                   "kernel_achieved": v["achieved"], "unit": v["unit"],
                                   "frac_of_peak": v["achieved"] / v["peak"], "avg_kernel_us": v["kernel_us"],
                                   **({"ceiling_gb_per_s": v["ceiling_gbs"], "frac_of_ceiling": v["achieved"] / v["ceiling_gbs"]}
                                      if v["bound"] == "hbm" else {}),
                                   "algorithmic_bytes_per_launch" if v["bound"] == "hbm" else "algorithmic_flops_per_launch":
                                       v["kernel_work"],
                                   "traffic": MEASURED_TRAFFIC_BYTES.get((wl.name, b)), "kernels_us": v["parts"]}
                          for b, v in results.items()}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
