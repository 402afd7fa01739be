#!/usr/bin/env python3
"""Writes the stored expected values for the full-size parity cases.

Calls ONLY the CPU oracle (``oracle/``) and the seeded input generators; nothing
here touches the GPU library.  For each named workload at its full size it runs
the fp64 oracle once and stores logZ, the accumulated gradients and the
per-position outputs at a fixed random sample of (sequence, position) rows:

    python tests/golden/make_golden.py speech genomic longgen

With ``--boundary`` after a name (``genomic --boundary``) the same is done with the seeded
boundary terms of ``synth.boundary_terms`` and the file is full_<name>_boundary.npz, which also
holds the gradients of those terms and the boundary posterior at the sampled rows.

With ``--viterbi`` the oracle's Viterbi decode is run instead and its best scores and segment
counts are stored in full_<name>_viterbi.npz.

With ``--durtrans`` the oracle runs with the seeded duration-dependent transitions of
``synth.duration_transitions`` (one matrix per duration) and the file is full_<name>_durtrans.npz
(grad_trans is then [K,C,C]).

Besides the random rows every file holds contiguous WINDOWS of rows (float32): around eight
boundaries of the checkpoint intervals (j*interval - K .. j*interval + K, where the chunk-parallel
scans hand over from one task to the next) and around four multiples of 32 that are no interval
boundary (where the scaling blocks of every length end).  The interval lengths are those the
library's planner reports for these shapes (INTERVALS below; the GPU tests check that they still
are, and fail if this file has to be run again).

Output: tests/golden/full_<name>.npz (float64 arrays, a few hundred KB each).
"""
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import oracle  # noqa: E402
from paper_2604_18780_amd import synth  # noqa: E402

NSAMPLE = 1024
# checkpoint interval of the default plan per workload (semicrf_ckpt_interval / semicrf_durtrans_ckpt_interval)
INTERVALS = {"speech": 64, "genomic": 392, "longgen": 784, "genomic--durtrans": 784}


def windows(w, interval):
    """(b, first token, length) of the stored windows: 8 interval boundaries +- K and 4 multiples of 32
    +- 8 that are no interval boundary, spread over the sequences and along them."""
    out = []
    seqs = [b for b in range(w.B) if int(w.lengths[b]) > 2 * interval]
    for i in range(8):
        b = seqs[i % len(seqs)]
        L = int(w.lengths[b])
        nint = (L + interval - 1) // interval
        j = 1 + (i * 7919 + 3 * b) % (nint - 1)                 # boundaries 1 .. nint-1
        lo = max(0, j * interval - w.K)
        hi = min(L, j * interval + w.K)
        out.append((b, lo, hi - lo))
    for i in range(4):
        b = seqs[(i + 1) % len(seqs)]
        L = int(w.lengths[b])
        m = 32 * (1 + (i * 104729 + 17) % (L // 32 - 1))
        while m % interval == 0:
            m += 32
        lo = max(0, m - 8)
        hi = min(L, m + 8)
        out.append((b, lo, hi - lo))
    return np.array(out, dtype=np.int64)


def window_values(a, win):
    """Rows of `a` [B,T,C] inside the windows, concatenated, as float32."""
    return np.concatenate([a[b, lo:lo + n] for b, lo, n in win], 0).astype(np.float32)


def sample_rows(w, seed=12345):
    """Fixed sample of valid (b, u) rows, always including the first and last token."""
    rng = np.random.default_rng(seed)
    rows = []
    for b in range(w.B):
        L = int(w.lengths[b])
        if L == 0:
            continue
        n = max(2, NSAMPLE // w.B)
        u = np.unique(np.concatenate([[0, L - 1], rng.integers(0, L, size=n)]))
        rows.append(np.stack([np.full_like(u, b), u], 1))
    return np.concatenate(rows, 0)


def main(args):
    names = [a for a in args if not a.startswith("--")]
    boundary = "--boundary" in args
    durtrans = "--durtrans" in args
    for name in names:
        w = synth.make(name)
        t0 = time.time()
        if "--viterbi" in args:   # best score and segment count of the Viterbi decode -> full_<name>_viterbi.npz
            score, labels, starts, nseg = oracle.viterbi(w.emis, w.lengths, w.trans, w.dur)
            dt = time.time() - t0
            out = os.path.join(os.path.dirname(os.path.abspath(__file__)), f"full_{name}_viterbi.npz")
            np.savez_compressed(out, score=score, nseg=nseg, oracle_seconds=np.array([dt]))
            print(f"{name}: oracle viterbi {dt:.1f}s -> {out}", flush=True)
            continue
        extra = {}
        if durtrans:
            r = oracle.fwd_bwd_durtrans(w.emis, w.lengths, synth.duration_transitions(w), w.dur)
        elif boundary:
            ps, pe, pis, pie = synth.boundary_terms(w)
            r = oracle.fwd_bwd(w.emis, w.lengths, w.trans, w.dur, proj_start=ps, proj_end=pe, pi_start=pis,
                               pi_end=pie)
        else:
            r = oracle.fwd_bwd(w.emis, w.lengths, w.trans, w.dur)
        dt = time.time() - t0
        rows = sample_rows(w)
        if boundary:
            extra = dict(grad_proj_start_rows=r.grad_proj_start[rows[:, 0], rows[:, 1]],
                         grad_proj_end_rows=r.grad_proj_end[rows[:, 0], rows[:, 1]],
                         bdy_post_rows=r.bdy_post[rows[:, 0], rows[:, 1]],
                         grad_pi_start=r.grad_pi_start, grad_pi_end=r.grad_pi_end,
                         bdy_post_total=np.array([r.bdy_post.sum()]))
        out = os.path.join(os.path.dirname(os.path.abspath(__file__)),
                           f"full_{name}{'_durtrans' if durtrans else ('_boundary' if boundary else '')}.npz")
        interval = INTERVALS[name + ("--durtrans" if durtrans else "")]
        win = windows(w, interval)
        extra.update(interval=np.array([interval]), windows=win, pos_marg_windows=window_values(r.pos_marg, win),
                     grad_emis_windows=window_values(r.grad_emis, win))
        np.savez_compressed(
            out, logz=r.logz, grad_trans=r.grad_trans, grad_dur=r.grad_dur, rows=rows,
            pos_marg_rows=r.pos_marg[rows[:, 0], rows[:, 1]],
            grad_emis_rows=r.grad_emis[rows[:, 0], rows[:, 1]],
            pos_marg_total=np.array([r.pos_marg.sum()]),
            oracle_seconds=np.array([dt]), oracle_threads=np.array([r.threads]), **extra)
        print(f"{name}: oracle {dt:.1f}s on {r.threads} threads -> {out}", flush=True)


if __name__ == "__main__":
    main(sys.argv[1:] or ["speech", "genomic", "longgen"])
