#!/usr/bin/env python3
"""Benchmark of the semi-CRF forward-backward hot path on one MI355X.

A step is one whole pass (prefix sums -> forward/backward scans -> per-interval
marginals -> finalisation) of ``semicrf_fwd_bwd`` over one synthetic batch that
is already resident in HBM.  The default workload is the genomic configuration
(B=4, T=100 000, K=64, C=24), the one the metric's positions/s figure is quoted
on.  Prints ONE JSON line on stdout: the headline keys for that workload, and
(unless ``--brief``) the other configurations, the forward-only pass, the other
entry points, the sensitivity of the chunk-parallel scans to the transition
model, and the oracle's rate on the host cores.
"""
from __future__ import annotations

import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

FP64_VECTOR_PEAK_TFLOPS = 78.6   # MI355X published fp64 vector peak (256 CU x 64 FMA lanes x 2 x 2.4 GHz)
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hot_path_genomic_hbm_traffic_pmc.txt")


def cpu_baseline(name: str, sample_T, threads: int):
    """The oracle as it stands, timed on the host cores; sample_T None = the whole workload."""
    import oracle
    from paper_2604_18780_amd import synth
    w = synth.make(name) if sample_T is None else synth.make(name, T=sample_T)
    t0 = time.perf_counter()
    r = oracle.fwd_bwd(w.emis, w.lengths, w.trans, w.dur, threads=threads)
    dt = time.perf_counter() - t0
    cut = "whole" if sample_T is None else f"T cut to {sample_T}"
    return {
        "value": w.nominal_edges / dt,
        "unit": "edge evals/s",
        "cores": int(r.threads),
        "kind": "oracle",
        "sample": f"{name} workload, {cut} (B={w.B}, T={w.T}, K={w.K}, C={w.C}); "
                  f"{w.nominal_edges:.3g} nominal edges in {dt:.1f} s; "
                  f"{w.positions / dt:.3g} positions/s",
        "seconds": dt,
    }


def exact_edges(w) -> float:
    """Edges the recurrence really visits: C^2 * sum_b sum_{t=1..L_b} min(t, K)
    (= C^2 * (K*L_b - K(K-1)/2) for L_b >= K)."""
    tot = 0
    for L in w.lengths.astype("int64").tolist():
        m = min(L, w.K)
        tot += m * (m + 1) // 2 + (L - m) * w.K
    return float(tot) * w.C * w.C


def read_traffic():
    """HBM bytes per launch of the two big kernels at the genomic workload, from the committed
    rocprofv3 --pmc summary (lines 'machine-readable: key=value ...'); None if the file has none."""
    out = {}
    try:
        for line in open(TRAFFIC_FILE):
            if "machine-readable:" not in line:
                continue
            kv = dict(m.groups() for m in re.finditer(r"(\w+)=(\S+)", line))
            if "stage" in kv and "bytes" in kv:
                out[kv["stage"]] = {"bytes": float(kv["bytes"]), "commit": kv.get("commit", "?")}
    except OSError:
        pass
    return out


class Problem:
    """One workload resident in HBM, with its workspace and output tensors."""

    def __init__(self, w, ckpt_interval, flags, dev="cuda:0"):
        import torch
        from paper_2604_18780_amd import binding as sb
        self.w, self.delta, self.flags, self.dev = w, ckpt_interval, flags, dev
        self.emis = torch.from_numpy(w.emis).to(dev)
        self.lengths = torch.from_numpy(w.lengths).to(dev)
        self.trans = torch.from_numpy(w.trans).to(dev)
        self.dur = torch.from_numpy(w.dur).to(dev)
        B, T, K, C = w.B, w.T, w.K, w.C
        self.kind = sb.grad_workspace_kind(flags)
        self.ws_bytes = sb.semicrf_workspace_bytes(B, T, K, C, ckpt_interval, self.kind)
        self.ws = sb.alloc_workspace(B, T, K, C, ckpt_interval, self.kind, dev)
        self.out = (torch.empty(B, dtype=torch.float32, device=dev),
                    torch.empty((B, T, C), dtype=torch.float32, device=dev),
                    torch.empty((C, C), dtype=torch.float32, device=dev),
                    torch.empty((K, C), dtype=torch.float32, device=dev),
                    torch.empty((B, T, C), dtype=torch.float32, device=dev))

    def set_transitions(self, trans):
        import torch
        self.trans = torch.from_numpy(trans).to(self.dev)

    def time_fwd_bwd(self, steps, warmup):
        """K timed steps after W warm-up steps; wall-clock ms per step and the stage times from HIP events."""
        import torch
        from paper_2604_18780_amd import binding as sb
        w = self.w
        events = [sb.StageEvents() for _ in range(steps)]
        for _ in range(warmup):
            sb.semicrf_fwd_bwd(self.emis, self.lengths, self.trans, self.dur, None, self.delta, self.flags,
                               workspace=self.ws, out=self.out)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            sb.semicrf_fwd_bwd_profiled(self.emis, self.lengths, self.trans, self.dur, events[i], None,
                                        self.delta, self.flags, workspace=self.ws, out=self.out)
        torch.cuda.synchronize()
        ms_step = 1e3 * (time.perf_counter() - t0) / steps
        stage = [0.0, 0.0, 0.0, 0.0]
        for ev in events:
            for j, ms in enumerate(ev.stage_ms()):
                stage[j] += ms / steps
            ev.destroy()
        acc, mis = sb.semicrf_scan_report(self.ws, w.B, w.T, w.K, w.C, self.delta, self.kind)
        torch.cuda.synchronize()
        return ms_step, stage, acc.cpu().numpy(), float(mis.max().item())

    def roofline(self, ms_step, stage):
        """The dominant stage against the fp64 vector peak.  One "unit" is K*C (duration sum) + C*C
        (transition product) multiply-adds per position.  The scan stage runs the forward and the backward
        recurrence once each (2 units; its forward tasks also leave the rows that Algorithm 3 would recompute
        per interval); the interval stage runs the backward recurrence again inside each interval and
        accumulates the marginals (2 units), or forms the marginals from the rows both scans stored (1 unit;
        the default wherever the plan has a row slot per interval for both scans).  Warm-up positions of the
        chunk-parallel scans are overhead, not counted."""
        from paper_2604_18780_amd import binding as sb
        w = self.w
        unit = 2.0 * (w.K * w.C + w.C * w.C) * w.positions
        # the plan of a default call holds the backward tasks' row slots exactly where that route is taken
        planned = (not (self.flags & sb.SEMICRF_LOW_MEMORY) and
                   sb.semicrf_workspace_bytes(w.B, w.T, w.K, w.C, self.delta, 1) >
                   sb.semicrf_workspace_bytes(w.B, w.T, w.K, w.C, self.delta, 2))
        rows_route = planned and not (self.flags & sb.SEMICRF_MARGINALS_INTERVAL)
        stage_flop = {"scans": 2 * unit, "intervals": (1 if rows_route else 2) * unit}
        kernels = {"scans": "k_spec (chunk-parallel forward + backward scans, one launch; stage time "
                            "includes its small verification kernels and the early exits of the retries)",
                   "intervals": (("k_mg_wave (marginals from the stored rows of both scans, one launch)" if w.K < 128 else
                                  "k_mg_dur + k_mg_te (marginals from the stored rows of both scans, two launches)")
                                 if rows_route else
                                 "k_interval_wave / k_interval (per-interval recompute + marginals, one launch)")}
        dom = "scans" if stage[1] >= stage[2] else "intervals"
        dom_s = (stage[1] if dom == "scans" else stage[2]) * 1e-3
        achieved = stage_flop[dom] / dom_s / 1e12
        whole = (stage_flop["scans"] + stage_flop["intervals"]) / (ms_step * 1e-3) / 1e12
        return dom, {
            "bound": "alu", "kernel": kernels[dom], "achieved": achieved, "peak": FP64_VECTOR_PEAK_TFLOPS,
            "unit": "TFLOP/s", "frac": achieved / FP64_VECTOR_PEAK_TFLOPS, "traffic": None,
            "flop_per_launch": stage_flop[dom], "launch_ms": dom_s * 1e3,
            "whole_path_achieved": whole, "whole_path_frac": whole / FP64_VECTOR_PEAK_TFLOPS,
        }


def time_call(call, steps, warmup):
    import torch
    for _ in range(warmup):
        o = call()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        o = call()
    torch.cuda.synchronize()
    return 1e3 * (time.perf_counter() - t0) / steps, o


def accepted_summary(acc):
    """How the (sequence, direction) scans were verified: first attempt / after repairs / long warm-up / sequential."""
    return {"first": int((acc == 1).sum()), "repaired": int((acc == 2).sum()),
            "long_warm_up": int((acc == 3).sum()), "sequential": int((acc == 0).sum())}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="genomic",
                    choices=["tiny", "nlp", "speech", "genomic", "longgen"])
    ap.add_argument("--ckpt-interval", type=int, default=0)
    ap.add_argument("--marginals", default="auto", choices=["auto", "rows", "interval"],
                    help="route of the marginals: from the stored rows of both scans, or the recurrence per interval")
    ap.add_argument("--matrix-scan", action="store_true", help="chunk-parallel scans on the matrix cores")
    ap.add_argument("--scan-waves", type=int, default=0, choices=[0, 1, 2],
                    help="waves per chunk-parallel scan task (0: the library's choice)")
    ap.add_argument("--extra-flags", type=lambda x: int(x, 0), default=0, help="further flag bits, as a number")
    ap.add_argument("--trans-scale", type=float, default=0.0,
                    help="standard deviation of the transition scores (the recipe's is 0.1)")
    ap.add_argument("--trans-band", type=int, default=-1,
                    help="forbid (score -1e4) transitions between labels further apart than this, cyclically")
    ap.add_argument("--brief", action="store_true", help="only the headline workload: no other configurations, "
                                                        "entry points, model variants")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-T", type=int, default=0,
                    help="cut T to this for the oracle's timing (default: the whole workload)")
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
    flags = sb.SEMICRF_CENTER
    flags |= {"auto": 0, "rows": sb.SEMICRF_MARGINALS_ROWS, "interval": sb.SEMICRF_MARGINALS_INTERVAL}[args.marginals]
    if args.matrix_scan:
        flags |= sb.SEMICRF_MATRIX_SCAN
    flags |= {0: 0, 1: sb.SEMICRF_ONE_WAVE_SCAN, 2: sb.SEMICRF_TWO_WAVE_SCAN}[args.scan_waves] | args.extra_flags
    w = synth.make(args.workload)
    if args.trans_scale > 0.0 or args.trans_band >= 0:
        w.trans = synth.reshape_transitions(w.trans, args.trans_scale or None,
                                            args.trans_band if args.trans_band >= 0 else None)
    B, T, K, C = w.B, w.T, w.K, w.C
    pb = Problem(w, args.ckpt_interval, flags, dev)
    emis, lengths, trans, dur, ws = pb.emis, pb.lengths, pb.trans, pb.dur, pb.ws

    def variant_line(metric, ms, extra):
        rec = {"metric": metric, "value": w.nominal_edges / (ms * 1e-3), "unit": "edge evals/s",
               "positions_per_s": w.positions / (ms * 1e-3), "n_gpus": 1, "steps": args.steps,
               "warmup": args.warmup, "ms_per_step": ms, "higher_is_better": True, "scaling": "weak",
               "vs_baseline": None, "dtype": "f64", "data": "synthetic"}
        rec.update(extra)
        print(json.dumps(rec))

    def viterbi_setup(p):
        nv = sb.semicrf_viterbi_workspace_bytes(p.w.B, p.w.T, p.w.K, p.w.C)
        raw = torch.empty(nv + 256, dtype=torch.uint8, device=dev)
        off = (-raw.data_ptr()) % 256
        vws = raw[off:off + nv]
        return nv, vws, (lambda: sb.semicrf_viterbi(p.emis, p.lengths, p.trans, p.dur, workspace=vws))

    def durtrans_setup(p):
        t3 = torch.from_numpy(synth.duration_transitions(p.w)).to(dev)
        dws = sb.alloc_durtrans_workspace(p.w.B, p.w.T, p.w.K, p.w.C, args.ckpt_interval, True, dev)
        return dws, (lambda: sb.semicrf_fwd_bwd_durtrans(p.emis, p.lengths, t3, p.dur, None, args.ckpt_interval,
                                                         workspace=dws))

    def boundary_setup(p):
        ps, pe, pis, pie = (torch.from_numpy(a).to(dev) for a in synth.boundary_terms(p.w))
        return lambda: sb.semicrf_fwd_bwd_boundary(p.emis, p.lengths, p.trans, p.dur, None, ps, pe, pis, pie,
                                                   args.ckpt_interval, workspace=p.ws)

    if args.viterbi:
        nv, vws, call = viterbi_setup(pb)
        ms, o = time_call(call, args.steps, args.warmup)
        variant_line("semi-CRF Viterbi decode, edge evals/sec (B*T*K*C^2/s)", ms, {
            "config": {"workload": f"{w.name}: B={B} T={T} K={K} C={C} (output tensors allocated inside the "
                                   f"timed calls)", "workspace_bytes": nv},
            "scans_accepted_chunk_parallel": int((sb.semicrf_scan_report(vws, B, T, K, C, 0, False)[0][:, 0] > 0).sum().item()),
            "scans_total": B,
            "score_mean": float(o[0].double().mean().item()), "segments": int(o[3].sum().item())})
        return
    if args.durtrans:
        dws, call = durtrans_setup(pb)
        ms, o = time_call(call, args.steps, args.warmup)
        dint = sb.semicrf_durtrans_ckpt_interval(B, T, K, C, args.ckpt_interval)
        acc, mis = sb.semicrf_scan_report(dws, B, T, K, C, dint, True)
        # forward recurrence, backward recurrence, marginals: 3 * K*C*C multiply-adds per position
        # (warm-up positions of the chunk-parallel scans are overhead and not counted)
        flop = 2.0 * 3.0 * K * C * C * w.positions
        variant_line("semi-CRF fwd+bwd with duration-dependent transitions, edge evals/sec (B*T*K*C^2/s)", ms, {
            "config": {"workload": f"{w.name}: B={B} T={T} K={K} C={C}, trans3 [K,C,C] = trans + N(0, 0.1^2) "
                                   f"(output tensors allocated inside the timed calls)",
                       "ckpt_interval": dint, "workspace_bytes": int(dws.numel())},
            "roofline": {"bound": "alu", "achieved": flop / (ms * 1e-3) / 1e12, "peak": FP64_VECTOR_PEAK_TFLOPS,
                         "unit": "TFLOP/s", "frac": flop / (ms * 1e-3) / 1e12 / FP64_VECTOR_PEAK_TFLOPS,
                         "traffic": None, "flop_per_call": flop},
            "scans_accepted_chunk_parallel": int((acc > 0).sum().item()), "scans_total": 2 * B,
            "logz_mean": float(o[0].double().mean().item())})
        return
    if args.boundary_terms:
        ms, o = time_call(boundary_setup(pb), args.steps, args.warmup)
        variant_line("semi-CRF fwd+bwd with boundary projections, edge evals/sec (B*T*K*C^2/s)", ms, {
            "config": {"workload": f"{w.name}: B={B} T={T} K={K} C={C} with proj_start, proj_end ~ N(0, 0.5^2), "
                                   f"pi_start, pi_end ~ N(0,1); all gradients and the boundary posterior "
                                   f"(output tensors allocated inside the timed calls)"},
            "logz_mean": float(o["logz"].double().mean().item())})
        return

    if args.calibrate_copy:
        src = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        dst.copy_(src)          # 1 GiB read + 1 GiB written
        torch.cuda.synchronize()
        del src, dst

    ms_step, stage, acc, mis = pb.time_fwd_bwd(args.steps, args.warmup)
    dom, roof = pb.roofline(ms_step, stage)
    plain = args.ckpt_interval == 0 and flags == sb.SEMICRF_CENTER and args.trans_scale == 0 and args.trans_band < 0
    traffic = read_traffic().get(dom) if (plain and args.workload == "genomic") else None
    if traffic:
        roof["traffic"] = traffic["bytes"]
        roof["traffic_source"] = f"profiles/{os.path.basename(TRAFFIC_FILE)} (taken at commit {traffic['commit']})"
    logz = pb.out[0].double().cpu().numpy()
    edges = w.nominal_edges
    positions = w.positions
    model = "" if plain else (f", transitions sd {args.trans_scale or 0.1}"
                              + (f", band {args.trans_band}" if args.trans_band >= 0 else ""))
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
                               f"sum of lengths {positions}{model}",
                   "ckpt_interval": sb.semicrf_ckpt_interval(B, T, K, C, args.ckpt_interval),
                   "workspace_bytes": pb.ws_bytes,
                   "nominal_edges_per_step": edges, "exact_edges_per_step": exact_edges(w)},
        "stage_ms": {"prefix": stage[0], "scans": stage[1], "intervals": stage[2], "finalise": stage[3]},
        "roofline": roof,
        "scans_accepted_chunk_parallel": int((acc > 0).sum()),
        "scans_total": 2 * B,
        "scans_accepted_by": accepted_summary(acc),
        "scan_boundary_mismatch_max": mis,
        "logz_mean": float(logz.mean()),
    }

    if not args.brief:
        few = max(3, min(args.steps, 5))
        # the forward pass alone (prefix sums + forward scan), same workload
        fws = sb.alloc_workspace(B, T, K, C, args.ckpt_interval, False, dev)
        lz = torch.empty(B, dtype=torch.float32, device=dev)
        ms, _ = time_call(lambda: sb.semicrf_logz_fwd(emis, lengths, trans, dur, args.ckpt_interval, flags,
                                                      workspace=fws, logz=lz), args.steps, args.warmup)
        rec["forward_only_ms"] = ms
        del fws
        # the other entry points on the same workload (their output tensors are allocated inside the timed calls)
        other = {}
        _, _, call = viterbi_setup(pb)
        other["viterbi"] = time_call(call, few, 2)[0]
        other["boundary_terms"] = time_call(boundary_setup(pb), few, 2)[0]
        dws, call = durtrans_setup(pb)
        other["durtrans"] = time_call(call, few, 2)[0]
        del dws, call
        rec["other_entry_points_ms"] = other
        # how the chunk-parallel scans take other transition models (same emissions, durations, lengths)
        sens = []
        for sd, band in ((1.0, None), (3.0, None), (0.1, 2), (3.0, 2)):
            pb.set_transitions(synth.reshape_transitions(w.trans, sd, band))
            m, st, a, e = pb.time_fwd_bwd(few, 2)
            sens.append({"trans_sd": sd, "band": band, "ms_per_step": m, "scans_ms": st[1],
                         "accepted_by": accepted_summary(a), "boundary_mismatch_max": e})
        pb.set_transitions(w.trans)
        rec["transition_model_sensitivity"] = sens
        # the low-memory plan on the same workload: milliseconds and bytes of both plans side by side
        pl = Problem(w, 0, sb.SEMICRF_CENTER | sb.SEMICRF_LOW_MEMORY, dev)
        m, st, a, e = pl.time_fwd_bwd(3, 1)
        rec["memory_plans"] = {
            "default": {"ms_per_step": ms_step, "workspace_bytes": pb.ws_bytes,
                        "forward_only_workspace_bytes": sb.semicrf_workspace_bytes(B, T, K, C, args.ckpt_interval, 0),
                        "ckpt_interval": sb.semicrf_ckpt_interval(B, T, K, C, args.ckpt_interval)},
            "low_memory": {"ms_per_step": m, "workspace_bytes": pl.ws_bytes,
                           "forward_only_workspace_bytes": sb.semicrf_workspace_bytes(B, T, K, C, 0, sb.PLAN_LOW_MEMORY),
                           "ckpt_interval": sb.semicrf_ckpt_interval_low_memory(B, T, K, C, 0),
                           "stage_ms": {"prefix": st[0], "scans": st[1], "intervals": st[2], "finalise": st[3]},
                           "accepted_by": accepted_summary(a)},
            "emission_bytes": B * T * C * 4}
        del pl
        # the two routes of the marginals on the same workload (the default takes the stored rows where planned)
        pi = Problem(w, args.ckpt_interval, sb.SEMICRF_CENTER | sb.SEMICRF_MARGINALS_INTERVAL, dev)
        m, st, a, e = pi.time_fwd_bwd(few, 2)
        rec["marginal_routes"] = {
            "default": {"ms_per_step": ms_step, "marginal_stage_ms": stage[2], "scans_ms": stage[1],
                        "workspace_bytes": pb.ws_bytes},
            "per_interval_recurrence": {"ms_per_step": m, "marginal_stage_ms": st[2], "scans_ms": st[1],
                                        "workspace_bytes": pi.ws_bytes}}
        del pi
        del pb, emis, lengths, trans, dur, ws
        torch.cuda.empty_cache()
        # the other configurations, each whole
        cfgs = {}
        for name in ("tiny", "nlp", "speech", "longgen"):
            if name == args.workload:
                continue
            wo = synth.make(name)
            po = Problem(wo, 0, sb.SEMICRF_CENTER, dev)
            m, st, a, e = po.time_fwd_bwd(few, 2)
            d, rf = po.roofline(m, st)
            cfgs[name] = {"shape": f"B={wo.B} T={wo.T} K={wo.K} C={wo.C}", "ms_per_step": m,
                          "edge_evals_per_s": wo.nominal_edges / (m * 1e-3),
                          "stage_ms": {"prefix": st[0], "scans": st[1], "intervals": st[2], "finalise": st[3]},
                          "roofline_frac": rf["frac"], "roofline_stage": d,
                          "whole_path_frac": rf["whole_path_frac"], "workspace_bytes": po.ws_bytes,
                          "accepted_by": accepted_summary(a)}
            del po, wo
            torch.cuda.empty_cache()
        rec["configs"] = cfgs

    if not args.no_cpu_baseline:
        # the whole workload with one thread per sequence (threads = min(B, cores)); and, for comparison, a cut
        # of it with every core, the spare ones splitting the label loop inside a position
        ncpu = os.cpu_count() or 1
        sample_T = args.cpu_sample_T or None
        if sample_T is None and args.workload in ("speech", "longgen"):
            sample_T = {"speech": 500, "longgen": 16000}[args.workload]
        rec["cpu_baseline"] = cpu_baseline(args.workload, sample_T, min(B, ncpu))
        if not args.brief:
            nested_T = {"tiny": 512, "nlp": 256, "speech": 500, "genomic": 20000, "longgen": 16000}[args.workload]
            rec["cpu_baseline_all_cores"] = cpu_baseline(args.workload, nested_T, 0)
    print(json.dumps(rec))


if __name__ == "__main__":
    main()
