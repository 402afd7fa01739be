"""GPU parity of the lock-step scan on the matrix cores (flag SEMICRF_MATRIX_SCAN).

Same bar as the default path: relative 1e-5 on logZ, absolute 1e-4 on per-position gradients,
1e-4 * max(1, max|g|) on the accumulated ones, against the fp64 oracle; in addition every scan
must have been accepted chunk-parallel with a boundary mismatch at the rounding floor, and the
results must agree with the default kernels to the same tolerances.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2604_18780_amd import binding as sb
from paper_2604_18780_amd import synth

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
FLAGS = sb.SEMICRF_CENTER | sb.SEMICRF_MATRIX_SCAN


def _dev(w):
    emis = w.emis.copy()
    for b in range(w.B):
        emis[b, int(w.lengths[b]):] = np.nan      # padding must never be read
    return (torch.from_numpy(emis).to(DEV), torch.from_numpy(w.lengths).to(DEV),
            torch.from_numpy(w.trans).to(DEV), torch.from_numpy(w.dur).to(DEV))


def _check(w, delta, label):
    print(f"[case] matrix scan {label}: B={w.B} T={w.T} K={w.K} C={w.C} delta={delta} lengths={w.lengths.tolist()[:8]}",
          flush=True)
    emis, lengths, trans, dur = _dev(w)
    ws = sb.alloc_workspace(w.B, w.T, w.K, w.C, delta, True)
    logz, g_e, g_t, g_d, pm = sb.semicrf_fwd_bwd(emis, lengths, trans, dur, None, delta, FLAGS, workspace=ws)
    acc, mis = sb.semicrf_scan_report(ws, w.B, w.T, w.K, w.C, delta, True)
    logz_f = sb.semicrf_logz_fwd(emis, lengths, trans, dur, delta, FLAGS)
    ref = sb.semicrf_fwd_bwd(emis, lengths, trans, dur, None, delta, sb.SEMICRF_CENTER)
    torch.cuda.synchronize()
    nonempty = w.lengths > 0
    assert np.all(acc.cpu().numpy()[nonempty] == 1), acc
    assert np.all(mis.cpu().numpy()[nonempty] <= 1e-13), mis
    r = oracle.fwd_bwd(w.emis, w.lengths, w.trans, w.dur)
    lz = logz.double().cpu().numpy()
    assert np.all(np.abs(lz - r.logz) <= 1e-5 * np.maximum(1.0, np.abs(r.logz)))
    assert np.array_equal(lz, logz_f.double().cpu().numpy())
    assert np.abs(pm.double().cpu().numpy() - r.pos_marg).max() <= 1e-4
    assert np.abs(g_e.double().cpu().numpy() - r.grad_emis).max() <= 1e-4
    assert np.abs(g_t.double().cpu().numpy() - r.grad_trans).max() <= 1e-4 * max(1.0, np.abs(r.grad_trans).max())
    assert np.abs(g_d.double().cpu().numpy() - r.grad_dur).max() <= 1e-4 * max(1.0, np.abs(r.grad_dur).max())
    # against the default kernels
    assert torch.allclose(logz, ref[0], rtol=1e-6, atol=0)
    assert (pm - ref[4]).abs().max().item() <= 1e-5


@pytest.mark.parametrize("seed,B,T,K,C,delta", [
    (3, 2, 700, 33, 24, 64),      # window of two blocks
    (4, 3, 1500, 64, 24, 192),    # window of four blocks, the genomic sizes
    (5, 2, 900, 64, 17, 128),     # fewer labels than the layout holds
    (6, 4, 300, 16, 24, 32),      # window of one block
    (7, 3, 200, 5, 20, 32),       # K below one chunk of the window
    (8, 2, 500, 64, 24, 32),      # interval shorter than the window
])
def test_matrix_scan_ragged(seed, B, T, K, C, delta):
    w = synth.small_random(seed, B, T, K, C, ragged=True)
    _check(w, delta, f"seed {seed}")


def test_matrix_scan_empty_and_full_sequences():
    w = synth.small_random(11, 4, 400, 64, 24, ragged=True)
    w.lengths[0] = 0
    w.lengths[1] = w.T
    w.lengths[2] = 1
    _check(w, 64, "empty, full and one-token sequences")


def test_matrix_scan_genomic_shape_reduced():
    _check(synth.make("genomic", B=2, T=6000), 192, "genomic 2 x 6000")


def test_matrix_scan_large_scores_leave_short_blocks_to_the_default_kernel():
    # emissions of scale 12: scaling blocks shorter than 16 positions, which the matrix kernel does not take
    w = synth.small_random(12, 2, 300, 16, 24, ragged=True, scale=12.0)
    print("[case] matrix scan with short scaling blocks", flush=True)
    emis, lengths, trans, dur = _dev(w)
    logz, g_e, g_t, g_d, pm = sb.semicrf_fwd_bwd(emis, lengths, trans, dur, None, 32, FLAGS)
    torch.cuda.synchronize()
    r = oracle.fwd_bwd(w.emis, w.lengths, w.trans, w.dur)
    assert np.all(np.abs(logz.double().cpu().numpy() - r.logz) <= 1e-5 * np.maximum(1.0, np.abs(r.logz)))
    assert np.abs(pm.double().cpu().numpy() - r.pos_marg).max() <= 1e-4
