#!/usr/bin/env python3
"""Benchmark of the semi-CRF forward-backward hot path on one MI355X.

A step is one whole pass (prefix sums -> forward/backward scans -> per-interval
marginals -> finalisation) of ``semicrf_fwd_bwd`` over one synthetic batch that
is already resident in HBM.  The default workload is the genomic configuration
(B=4, T=100 000, K=64, C=24), the one the metric's positions/s figure is quoted
on.  Prints ONE JSON line on stdout.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

FP64_VECTOR_PEAK_TFLOPS = 78.6   # MI355X published fp64 vector peak (256 CU x 64 FMA lanes x 2 x 2.4 GHz)


def cpu_baseline(name: str, sample_T: int):
    """The oracle as it stands, timed on the host cores on a bounded prefix-shaped sample."""
    import oracle
    from paper_2604_18780_amd import synth
    w = synth.make(name, T=sample_T)
    t0 = time.perf_counter()
    r = oracle.fwd_bwd(w.emis, w.lengths, w.trans, w.dur)
    dt = time.perf_counter() - t0
    return {
        "value": w.nominal_edges / dt,
        "unit": "edge evals/s",
        "cores": int(r.threads),
        "kind": "oracle",
        "sample": f"{name} workload with T cut to {sample_T} (B={w.B}, K={w.K}, C={w.C}); "
                  f"{w.nominal_edges:.3g} nominal edges in {dt:.1f} s; "
                  f"{w.positions / dt:.3g} positions/s",
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="genomic",
                    choices=["tiny", "nlp", "speech", "genomic", "longgen"])
    ap.add_argument("--ckpt-interval", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-T", type=int, default=0)
    ap.add_argument("--boundary-terms", action="store_true",
                    help="time semicrf_fwd_bwd_boundary with start/end projections, scalar boundaries and all "
                         "their outputs instead (whole-call time only; prints its own JSON line)")
    ap.add_argument("--viterbi", action="store_true",
                    help="time semicrf_viterbi (max-semiring decode + trace-back) instead; prints its own JSON line")
    ap.add_argument("--durtrans", action="store_true",
                    help="time semicrf_fwd_bwd_durtrans (one transition matrix per duration: K*C*C multiply-adds "
                         "per position and recurrence) instead; prints its own JSON line")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one 1 GiB device-to-device copy so that a rocprofv3 --pmc run of this "
                         "command holds a kernel of known traffic to scale FETCH_SIZE / WRITE_SIZE by")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build measures one GPU only (sequences shard across GPUs with a "
              "single small all-reduce of the parameter gradients; that path is not built)",
              file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2604_18780_amd import binding as sb
    from paper_2604_18780_amd import synth

    dev = "cuda:0"
    w = synth.make(args.workload)
    emis = torch.from_numpy(w.emis).to(dev)
    lengths = torch.from_numpy(w.lengths).to(dev)
    trans = torch.from_numpy(w.trans).to(dev)
    dur = torch.from_numpy(w.dur).to(dev)
    B, T, K, C = w.B, w.T, w.K, w.C
    ws_bytes = sb.semicrf_workspace_bytes(B, T, K, C, args.ckpt_interval, True)
    ws = sb.alloc_workspace(B, T, K, C, args.ckpt_interval, True, dev)
    out = (torch.empty(B, dtype=torch.float32, device=dev),
           torch.empty((B, T, C), dtype=torch.float32, device=dev),
           torch.empty((C, C), dtype=torch.float32, device=dev),
           torch.empty((K, C), dtype=torch.float32, device=dev),
           torch.empty((B, T, C), dtype=torch.float32, device=dev))
    if args.viterbi:
        nv = sb.semicrf_viterbi_workspace_bytes(B, T, K, C)
        raw = torch.empty(nv + 256, dtype=torch.uint8, device=dev)
        off = (-raw.data_ptr()) % 256
        vws = raw[off:off + nv]
        call = lambda: sb.semicrf_viterbi(emis, lengths, trans, dur, workspace=vws)
        for _ in range(args.warmup):
            o = call()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            o = call()
        torch.cuda.synchronize()
        ms = 1e3 * (time.perf_counter() - t0) / args.steps
        print(json.dumps({
            "metric": "semi-CRF Viterbi decode, edge evals/sec (B*T*K*C^2/s)",
            "value": w.nominal_edges / (ms * 1e-3), "unit": "edge evals/s",
            "positions_per_s": w.positions / (ms * 1e-3), "n_gpus": 1, "steps": args.steps,
            "warmup": args.warmup, "ms_per_step": ms, "higher_is_better": True, "scaling": "weak",
            "vs_baseline": None, "dtype": "f64", "data": "synthetic",
            "config": {"workload": f"{w.name}: B={B} T={T} K={K} C={C} (output tensors allocated inside the "
                                   f"timed calls)", "workspace_bytes": nv},
            "scans_accepted_chunk_parallel": int(sb.semicrf_scan_report(vws, B, T, K, C, 0, False)[0][:, 0].sum().item()),
            "scans_total": B,
            "score_mean": float(o[0].double().mean().item()), "segments": int(o[3].sum().item())}))
        return
    if args.durtrans:
        t3 = torch.from_numpy(synth.duration_transitions(w)).to(dev)
        dws = sb.alloc_durtrans_workspace(B, T, K, C, args.ckpt_interval, True, dev)
        call = lambda: sb.semicrf_fwd_bwd_durtrans(emis, lengths, t3, dur, None, args.ckpt_interval, workspace=dws)
        for _ in range(args.warmup):
            o = call()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            o = call()
        torch.cuda.synchronize()
        ms = 1e3 * (time.perf_counter() - t0) / args.steps
        dint = sb.semicrf_durtrans_ckpt_interval(B, T, K, C, args.ckpt_interval)
        acc, mis = sb.semicrf_scan_report(dws, B, T, K, C, dint, True)
        # forward recurrence, backward recurrence, marginals: 3 * K*C*C multiply-adds per position
        # (warm-up positions of the chunk-parallel scans are overhead and not counted)
        flop = 2.0 * 3.0 * K * C * C * w.positions
        print(json.dumps({
            "metric": "semi-CRF fwd+bwd with duration-dependent transitions, edge evals/sec (B*T*K*C^2/s)",
            "value": w.nominal_edges / (ms * 1e-3), "unit": "edge evals/s",
            "positions_per_s": w.positions / (ms * 1e-3), "n_gpus": 1, "steps": args.steps,
            "warmup": args.warmup, "ms_per_step": ms, "higher_is_better": True, "scaling": "weak",
            "vs_baseline": None, "dtype": "f64", "data": "synthetic",
            "config": {"workload": f"{w.name}: B={B} T={T} K={K} C={C}, trans3 [K,C,C] = trans + N(0, 0.1^2) "
                                   f"(output tensors allocated inside the timed calls)",
                       "ckpt_interval": dint, "workspace_bytes": int(dws.numel())},
            "roofline": {"bound": "alu", "achieved": flop / (ms * 1e-3) / 1e12, "peak": FP64_VECTOR_PEAK_TFLOPS,
                         "unit": "TFLOP/s", "frac": flop / (ms * 1e-3) / 1e12 / FP64_VECTOR_PEAK_TFLOPS,
                         "traffic": None, "flop_per_call": flop},
            "scans_accepted_chunk_parallel": int(acc.sum().item()), "scans_total": 2 * B,
            "logz_mean": float(o[0].double().mean().item())}))
        return
    if args.boundary_terms:
        ps, pe, pis, pie = (torch.from_numpy(a).to(dev) for a in synth.boundary_terms(w))
        call = lambda: sb.semicrf_fwd_bwd_boundary(emis, lengths, trans, dur, None, ps, pe, pis, pie,
                                                   args.ckpt_interval, workspace=ws)
        for _ in range(args.warmup):
            o = call()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            o = call()
        torch.cuda.synchronize()
        ms = 1e3 * (time.perf_counter() - t0) / args.steps
        print(json.dumps({
            "metric": "semi-CRF fwd+bwd with boundary projections, edge evals/sec (B*T*K*C^2/s)",
            "value": w.nominal_edges / (ms * 1e-3), "unit": "edge evals/s",
            "positions_per_s": w.positions / (ms * 1e-3), "n_gpus": 1, "steps": args.steps,
            "warmup": args.warmup, "ms_per_step": ms, "higher_is_better": True, "scaling": "weak",
            "vs_baseline": None, "dtype": "f64", "data": "synthetic",
            "config": {"workload": f"{w.name}: B={B} T={T} K={K} C={C} with proj_start, proj_end ~ N(0, 0.5^2), "
                                   f"pi_start, pi_end ~ N(0,1); all gradients and the boundary posterior "
                                   f"(output tensors allocated inside the timed calls)"},
            "logz_mean": float(o["logz"].double().mean().item())}))
        return
    events = [sb.StageEvents() for _ in range(args.steps)]

    if args.calibrate_copy:
        src = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        dst.copy_(src)          # 1 GiB read + 1 GiB written
        torch.cuda.synchronize()
        del src, dst
    for _ in range(args.warmup):
        sb.semicrf_fwd_bwd(emis, lengths, trans, dur, None, args.ckpt_interval, workspace=ws, out=out)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        sb.semicrf_fwd_bwd_profiled(emis, lengths, trans, dur, events[i], None, args.ckpt_interval,
                                    workspace=ws, out=out)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_step = 1e3 * dt / args.steps

    stage = [0.0, 0.0, 0.0, 0.0]
    for ev in events:
        for j, ms in enumerate(ev.stage_ms()):
            stage[j] += ms / args.steps
        ev.destroy()

    positions = w.positions
    edges = w.nominal_edges
    # fp64 flops per position (one multiply-add = 2 flop).  One "unit" is K*C (duration sum) +
    # C*C (transition product) multiply-adds.  The scan stage runs the forward and the backward
    # recurrence once each (2 units; its forward tasks also leave the rows that Algorithm 3 would
    # recompute per interval); the interval stage runs the backward recurrence again inside each
    # interval and accumulates the marginals (2 units).  Warm-up positions of the chunk-parallel
    # scans are overhead and are not counted.
    unit = 2.0 * (K * C + C * C) * positions
    # For K >= 128 the library takes the marginals from the rows both scans stored (position-local
    # products: 1 unit, no third recurrence), unless SEMICRF_MARGINALS forces a route; counting 1 unit
    # there can only understate the rate if the library fell back to the interval kernel.
    knob = os.environ.get("SEMICRF_MARGINALS", "")[:1]
    rows_route = knob == "r" or (K >= 128 and knob != "i")
    stage_flop = {"scans": 2 * unit, "intervals": (1 if rows_route else 2) * unit}
    kernels = {"scans": "k_spec (chunk-parallel forward + backward scans, one launch; stage time "
                        "includes its two small verification kernels)",
               "intervals": ("k_mg_dur + k_mg_te (marginals from the stored rows of both scans, two launches)"
                             if rows_route else
                             "k_interval_wave / k_interval (per-interval recompute + marginals, one launch)")}
    # HBM bytes per launch of the two big kernels at the genomic workload with the automatic
    # interval, from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs scaled by a 1 GiB copy
    # (profiles/hot_path_genomic_hbm_traffic_pmc.txt); unknown for other workloads.
    measured_traffic = {("genomic", "intervals"): 384.4e6, ("genomic", "scans"): 599.0e6 + 52.8e6}
    dom = "scans" if stage[1] >= stage[2] else "intervals"
    dom_s = (stage[1] if dom == "scans" else stage[2]) * 1e-3
    achieved = stage_flop[dom] / dom_s / 1e12
    whole = (stage_flop["scans"] + stage_flop["intervals"]) / (ms_step * 1e-3) / 1e12
    logz = out[0].double().cpu().numpy()
    acc, mis = sb.semicrf_scan_report(ws, B, T, K, C, args.ckpt_interval, True)
    torch.cuda.synchronize()

    rec = {
        "metric": "semi-CRF fwd+bwd edge evals/sec (B*T*K*C^2/s) + positions/sec at T=100k",
        "value": edges / (ms_step * 1e-3),
        "unit": "edge evals/s",
        "positions_per_s": positions / (ms_step * 1e-3),
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f64",
        "data": "synthetic",
        "config": {"workload": f"{w.name}: B={B} T={T} K={K} C={C}, fp32 emissions, "
                               f"sum of lengths {positions}",
                   "ckpt_interval": args.ckpt_interval, "workspace_bytes": ws_bytes,
                   "nominal_edges_per_step": edges},
        "stage_ms": {"prefix": stage[0], "scans": stage[1], "intervals": stage[2], "finalise": stage[3]},
        "roofline": {
            "bound": "alu",
            "kernel": kernels[dom],
            "achieved": achieved,
            "peak": FP64_VECTOR_PEAK_TFLOPS,
            "unit": "TFLOP/s",
            "frac": achieved / FP64_VECTOR_PEAK_TFLOPS,
            "traffic": measured_traffic.get((args.workload, dom)) if args.ckpt_interval == 0 else None,
            "flop_per_launch": stage_flop[dom],
            "launch_ms": dom_s * 1e3,
            "whole_path_achieved": whole,
            "whole_path_frac": whole / FP64_VECTOR_PEAK_TFLOPS,
        },
        "scans_accepted_chunk_parallel": int(acc.sum().item()),
        "scans_total": 2 * B,
        "scan_boundary_mismatch_max": float(mis.max().item()),
        "logz_mean": float(logz.mean()),
    }
    if not args.no_cpu_baseline:
        sample_T = args.cpu_sample_T or {"tiny": 512, "nlp": 256, "speech": 500,
                                         "genomic": 40000, "longgen": 16000}[args.workload]
        rec["cpu_baseline"] = cpu_baseline(args.workload, sample_T)
    print(json.dumps(rec))


if __name__ == "__main__":
    main()
