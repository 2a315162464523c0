#!/usr/bin/env python3
"""Benchmark of the MoQE hot path on one MI355X.

A step is one pass of the whole hot path over one batch: moqe_route (top-1 gating,
histogram, scan, permutation) followed by moqe_expert_ffn (FFN1 + bias + ReLU,
FFN2 + bias, gate-weighted combine) on one MoE layer of the decode configuration
(E=32 experts, d_model 1024, d_ff 4096, batch of 24 tokens, int4 experts).
Consecutive steps use different layer copies (own weights, own router) so that the
packed weights of a step are not left in the 256 MB last-level cache by the
previous one: the weights really come from HBM.

Prints ONE JSON line: tokens/s (metric), ms per step, the roofline of the dominant
kernel (algorithmic bytes / measured kernel time, against the 8 TB/s HBM peak) and
the CPU oracle timed on the host's cores on a bounded sample of the same workload.
"""

from __future__ import annotations

import argparse
import ctypes
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0

# HBM traffic per launch of the dominant kernel measured with rocprofv3 --pmc
# (FETCH_SIZE and WRITE_SIZE runs, scaled by a copy kernel of known size); filled
# from the summaries under profiles/ once measured, per bit width, else None.
MEASURED_TRAFFIC_BYTES = {4: None, 3: None, 2: None}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=400)
    ap.add_argument("--warmup", type=int, default=40)
    ap.add_argument("--bits", type=int, default=4, choices=(2, 3, 4), help="bit width of the headline line")
    ap.add_argument("--copies", type=int, default=8, help="independent layer copies cycled through")
    ap.add_argument("--other-bits", action="store_true", help="also time the other two bit widths")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-steps", type=int, default=3)
    ap.add_argument("--no-graph", action="store_true", help="time eager launches only")
    return ap.parse_args()


def algorithmic_bytes(seg_offsets, bits, d, f, T):
    """Bytes the method must move for one layer-step, split per FFN launch.
    Per active expert: packed codes + fp16 scales + fp16 biases of the matrix;
    plus the fp16 activations entering and leaving the layer (x in FFN1, y in
    FFN2).  The hidden activations h are not counted."""
    counts = np.diff(np.asarray(seg_offsets))
    active = int((counts > 0).sum())
    ffn1 = active * (d * f * bits // 8 + 2 * f + 2 * f) + 2 * T * d
    ffn2 = active * (d * f * bits // 8 + 2 * d + 2 * d) + 2 * T * d
    return active, ffn1, ffn2


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
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()

    wl = W.CONFIGS["c1"]
    E, d, f, T = wl.E, wl.d, wl.f, wl.T
    bit_list = [args.bits] + ([b for b in (4, 3, 2) if b != args.bits] if args.other_bits else [])

    # ---- layer copies: generated on the host (seeded), quantized on the device ----
    t0 = time.time()
    layers = {b: [] for b in bit_list}
    layer0_host = None
    for i in range(args.copies):
        host = W.make_layer(wl, layer=i)
        if i == 0:
            layer0_host = host
        w1, w2 = dev(host["w1"]), dev(host["w2"])
        b1, b2, wg = dev(host["b1"]), dev(host["b2"]), dev(host["w_gate"])
        for b in bit_list:
            layers[b].append(moqe.quantize_layer(w1, b1, w2, b2, b, wg))
        del w1, w2
        torch.cuda.synchronize()
        print(f"[bench] layer copy {i + 1}/{args.copies} ready ({time.time() - t0:.0f}s)", file=sys.stderr, flush=True)
    x_host = W.make_tokens(wl)
    x = dev(x_host)

    L = moqe.lib()
    route, route_ws = moqe.alloc_route(T, E, x.device)
    ffn_ws = torch.empty(moqe.moqe_ffn_workspace_bytes(T, E, d, f), dtype=torch.uint8, device=x.device)
    y = torch.empty_like(x)

    def make_step(qls):
        structs = [ql.c_struct() for ql in qls]
        refs = [ctypes.byref(s) for s in structs]
        gates = [ql.w_gate.data_ptr() for ql in qls]
        xp, yp = x.data_ptr(), y.data_ptr()
        ip, gp, sp, pp = (route.expert_idx.data_ptr(), route.gate.data_ptr(), route.seg_offsets.data_ptr(),
                          route.perm.data_ptr())
        rws, rwsn, fws, fwsn = route_ws.data_ptr(), route_ws.numel(), ffn_ws.data_ptr(), ffn_ws.numel()

        def step(i, stream):
            k = i % len(qls)
            st = L.moqe_route(xp, gates[k], T, d, E, ip, gp, sp, pp, rws, rwsn, stream)
            st |= L.moqe_expert_ffn(refs[k], xp, T, ip, gp, sp, pp, None, yp, fws, fwsn, stream)
            if st:
                raise RuntimeError(f"moqe call failed with status {st}")

        def ffn_halves(i, stream, ev):
            k = i % len(qls)
            st = L.moqe_route(xp, gates[k], T, d, E, ip, gp, sp, pp, rws, rwsn, stream)
            ev[0].record()
            st |= L.moqe_expert_ffn1(refs[k], xp, T, sp, pp, fws, stream)
            ev[1].record()
            st |= L.moqe_expert_ffn2(refs[k], fws, T, gp, sp, pp, None, yp, stream)
            ev[2].record()
            if st:
                raise RuntimeError(f"moqe call failed with status {st}")

        step.keep = (structs, refs)
        return step, ffn_halves

    def time_steps(run, steps, warmup):
        for i in range(warmup):
            run(i)
        torch.cuda.synchronize()
        t = time.perf_counter()
        for i in range(steps):
            run(warmup + i)
        torch.cuda.synchronize()
        return (time.perf_counter() - t) * 1e3 / steps

    results = {}
    for b in bit_list:
        qls = layers[b]
        step, ffn_halves = make_step(qls)
        stream = torch.cuda.current_stream().cuda_stream
        eager_ms = time_steps(lambda i: step(i, stream), args.steps, args.warmup)

        graph_ms = None
        if not args.no_graph:
            side = torch.cuda.Stream()
            graphs = []
            with torch.cuda.stream(side):
                for k in range(len(qls)):
                    g = torch.cuda.CUDAGraph()
                    with torch.cuda.graph(g, stream=side):
                        step(k, torch.cuda.current_stream().cuda_stream)
                    graphs.append(g)
            torch.cuda.synchronize()
            graph_ms = time_steps(lambda i: graphs[i % len(graphs)].replay(), args.steps, args.warmup)

        # ---- per-kernel time of the dominant kernel (HIP events on the launch stream) ----
        n_ev = min(args.steps, 200)
        evs = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(n_ev)]
        segs = []
        for i in range(8):
            step(i, stream)
        torch.cuda.synchronize()
        for i in range(n_ev):
            ffn_halves(i, stream, evs[i])
            if i < len(qls):
                torch.cuda.synchronize()
                segs.append(route.seg_offsets.cpu().numpy().copy())
        torch.cuda.synchronize()
        t1 = np.array([e[0].elapsed_time(e[1]) for e in evs]) * 1e-3
        t2 = np.array([e[1].elapsed_time(e[2]) for e in evs]) * 1e-3
        ab = [algorithmic_bytes(s, b, d, f, T) for s in segs]
        by1 = np.array([ab[i % len(qls)][1] for i in range(n_ev)], dtype=np.float64)
        by2 = np.array([ab[i % len(qls)][2] for i in range(n_ev)], dtype=np.float64)
        launches = 2 * n_ev
        kern_s = float((t1.sum() + t2.sum()) / launches)
        kern_bytes = float((by1.sum() + by2.sum()) / launches)
        achieved = kern_bytes / kern_s / 1e9
        best_ms = min(eager_ms, graph_ms) if graph_ms is not None else eager_ms
        results[b] = dict(
            ms_per_step=best_ms, eager_ms=eager_ms, graph_ms=graph_ms, tokens_per_s=T / (best_ms * 1e-3),
            active_experts=float(np.mean([a[0] for a in ab])), layer_bytes=float(np.mean([a[1] + a[2] for a in ab])),
            kernel_us=kern_s * 1e6, kernel_bytes=kern_bytes, achieved_gbs=achieved,
            ffn1_us=float(t1.mean() * 1e6), ffn2_us=float(t2.mean() * 1e6),
            step_gbs=float(np.mean([a[1] + a[2] for a in ab])) / (best_ms * 1e-3) / 1e9)
        print(f"[bench] int{b}: eager {eager_ms * 1e3:.1f} us/step, graph "
              f"{(graph_ms or float('nan')) * 1e3:.1f} us/step, ffn kernels {t1.mean() * 1e6:.1f} + {t2.mean() * 1e6:.1f} us, "
              f"{achieved:.0f} GB/s", file=sys.stderr, flush=True)

    # ---- CPU oracle on the host cores: bounded sample of the same workload ----
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import moqe_oracle as O
        bits = args.bits
        ql0 = layers[bits][0]
        c1, c2 = ql0.codes1.cpu().numpy(), ql0.codes2.cpu().numpy()
        s1, s2 = ql0.scales1.cpu().numpy(), ql0.scales2.cpu().numpy()
        cores = len(os.sched_getaffinity(0))

        class Lazy:
            """Unpacks and dequantizes an expert's matrix from its packed codes on access."""
            def __init__(self, codes, scales, K, N):
                self.codes, self.scales, self.K, self.N = codes, scales, K, N

            def __getitem__(self, e):
                return O.dequantize(O.unpack(self.codes[e], bits, self.K, self.N), self.scales[e])

        t = time.perf_counter()
        for _ in range(args.cpu_steps):
            idx, gate, offs, perm = O.route(x_host, layer0_host["w_gate"])
            O.expert_ffn(x_host, idx, gate, Lazy(c1, s1, d, f), layer0_host["b1"], Lazy(c2, s2, f, d),
                         layer0_host["b2"])
        dt = time.perf_counter() - t
        cpu = dict(value=T * args.cpu_steps / dt, unit="tokens/s", cores=cores, kind="oracle",
                   sample=f"{args.cpu_steps} steps of route + expert FFN on layer copy 0 (T={T}, int{bits}, fp64, "
                          f"codes unpacked per call), {dt:.1f} s")

    r = results[args.bits]
    out = {
        "metric": "expert-FFN tokens/s (route + int%d expert FFN, one MoE layer step)" % args.bits,
        "value": r["tokens_per_s"], "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": r["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int%d weights x f16 activations, f32 accumulate" % args.bits, "data": "synthetic",
        "config": {"workload": "c1: E=32 d_model=1024 d_ff=4096 T=24 top-1, int%d per-channel RTN experts, seed 1, "
                               "%d layer copies cycled" % (args.bits, args.copies),
                   "launch": "hip graph replay" if (r["graph_ms"] is not None and r["graph_ms"] <= r["eager_ms"]) else "eager",
                   "eager_ms_per_step": r["eager_ms"], "graph_ms_per_step": r["graph_ms"],
                   "active_experts": r["active_experts"], "layer_algorithmic_bytes": r["layer_bytes"],
                   "step_gb_per_s": r["step_gbs"]},
        "roofline": {"bound": "hbm", "achieved": r["achieved_gbs"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": r["achieved_gbs"] / HBM_PEAK_GBS, "traffic": MEASURED_TRAFFIC_BYTES.get(args.bits),
                     "kernel": "ffn_decode_kernel<%d,32>" % args.bits, "avg_kernel_us": r["kernel_us"],
                     "algorithmic_bytes_per_launch": r["kernel_bytes"],
                     "ffn1_us": r["ffn1_us"], "ffn2_us": r["ffn2_us"]},
        "cpu_baseline": cpu,
    }
    if len(results) > 1:
        out["by_bits"] = {str(b): {"tokens_per_s": v["tokens_per_s"], "ms_per_step": v["ms_per_step"],
                                   "kernel_gb_per_s": v["achieved_gbs"], "frac_of_peak": v["achieved_gbs"] / HBM_PEAK_GBS,
                                   "avg_kernel_us": v["kernel_us"]} for b, v in results.items()}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
