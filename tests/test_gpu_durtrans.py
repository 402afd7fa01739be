"""GPU parity of the duration-dependent transitions (trans3 [K,C,C]) against the fp64 CPU oracle.

Tolerances as for the main path: relative 1e-5 on logZ, absolute 1e-4 on the per-position
gradients, 1e-4 * max(1, max|g|) on the accumulated parameter gradients.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2604_18780_amd import binding as sb
from paper_2604_18780_amd import synth

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def trans3_of(w, seed, sd=0.3):
    """One matrix per duration: the workload's matrix plus duration-dependent noise."""
    return synth.duration_transitions(w, seed, sd)


def run(w, trans3, center=True, grad_logz=None, ckpt_interval=0, extra_flags=0):
    emis = w.emis.copy()
    for b in range(w.B):
        emis[b, int(w.lengths[b]):] = np.nan          # padding must never be read
    flags = (sb.SEMICRF_CENTER if center else 0) | extra_flags
    gl = None if grad_logz is None else torch.from_numpy(grad_logz.astype(np.float32)).to(DEV)
    args = (torch.from_numpy(emis).to(DEV), torch.from_numpy(w.lengths).to(DEV),
            torch.from_numpy(trans3).to(DEV), torch.from_numpy(w.dur).to(DEV))
    ws = sb.alloc_durtrans_workspace(w.B, w.T, w.K, w.C, ckpt_interval, True, DEV)
    out = sb.semicrf_fwd_bwd_durtrans(*args, gl, ckpt_interval, flags, workspace=ws)
    acc, mis = sb.semicrf_scan_report(ws, w.B, w.T, w.K, w.C,
                                      sb.semicrf_durtrans_ckpt_interval(w.B, w.T, w.K, w.C, ckpt_interval), True)
    lz_f = sb.semicrf_logz_fwd_durtrans(*args, ckpt_interval, flags)
    torch.cuda.synchronize()
    res = [None if o is None else o.double().cpu().numpy() for o in out]
    return res, lz_f.double().cpu().numpy(), acc.cpu().numpy(), mis.cpu().numpy()


def check(w, trans3, center=True, grad_logz=None, ckpt_interval=0, extra_flags=0, label="", expect_chunked=None):
    print(f"[case] {label or w.name} B={w.B} T={w.T} K={w.K} C={w.C} center={center} delta={ckpt_interval} "
          f"flags={extra_flags}", flush=True)
    (lz, g_e, g_t, g_d, pm), lz_f, acc, mis = run(w, trans3, center, grad_logz, ckpt_interval, extra_flags)
    r = oracle.fwd_bwd_durtrans(w.emis, w.lengths, trans3, w.dur, grad_logz=grad_logz, center=center)
    assert np.all(np.isfinite(lz))
    rel = np.abs(lz - r.logz) / np.maximum(1.0, np.abs(r.logz))
    assert rel.max() <= 1e-5, (rel.max(), lz, r.logz)
    relf = np.abs(lz_f - r.logz) / np.maximum(1.0, np.abs(r.logz))
    assert relf.max() <= 1e-5, (relf.max(), lz_f, r.logz)
    wmax = 1.0 if grad_logz is None else max(1.0, float(np.abs(grad_logz).max()))
    e_pm = np.abs(pm - r.pos_marg).max()
    e_ge = np.abs(g_e - r.grad_emis).max()
    e_t = np.abs(g_t - r.grad_trans).max()
    e_d = np.abs(g_d - r.grad_dur).max()
    print(f"       max err: logz rel {rel.max():.2e} pos_marg {e_pm:.2e} grad_emis {e_ge:.2e} "
          f"grad_trans3 {e_t:.2e} (max|g| {np.abs(r.grad_trans).max():.3g}) grad_dur {e_d:.2e} "
          f"(max|g| {np.abs(r.grad_dur).max():.3g}); scans accepted {int(acc.sum())} of {acc.size}, "
          f"largest mismatch {mis.max():.2e}", flush=True)
    assert e_pm <= 1e-4, e_pm
    assert e_ge <= 1e-4 * wmax, e_ge
    assert e_t <= 1e-4 * max(1.0, np.abs(r.grad_trans).max()), e_t
    assert e_d <= 1e-4 * max(1.0, np.abs(r.grad_dur).max()), e_d
    if expect_chunked is True:
        nonempty = w.lengths > 0
        assert acc[nonempty].all()
    if expect_chunked is False:
        assert not acc.any()
    return (lz, g_e, g_t, g_d, pm)


@pytest.mark.parametrize("seed,B,T,K,C", [
    (1, 3, 40, 5, 3), (2, 4, 300, 8, 6), (3, 2, 300, 33, 24), (4, 5, 130, 1, 7),
    (5, 3, 90, 2, 5), (6, 2, 50, 80, 4), (7, 6, 33, 7, 1), (8, 2, 257, 3, 17),
    (9, 1, 1, 1, 1), (10, 2, 150, 70, 8), (11, 2, 120, 4, 32),
])
def test_random_ragged_cases(seed, B, T, K, C):
    w = synth.small_random(seed, B, T, K, C, ragged=True)
    if seed == 2:
        w.lengths[0] = 0          # empty sequence
        w.lengths[1] = T          # full sequence
    rng = np.random.default_rng(seed)
    check(w, trans3_of(w, 100 + seed), grad_logz=rng.standard_normal(B))


def test_no_centering_and_large_emission_scale():
    w = synth.small_random(21, 2, 200, 6, 4, ragged=False, scale=8.0)
    check(w, trans3_of(w, 121), center=False)
    w = synth.small_random(22, 2, 120, 5, 3, ragged=False, scale=30.0)     # scaling blocks of one position
    check(w, trans3_of(w, 122))


def test_checkpoint_interval_invariance_and_sequential_scan():
    w = synth.small_random(31, 2, 210, 9, 5, ragged=True)
    w.lengths[:] = [210, 100]
    t3 = trans3_of(w, 131)
    ref = None
    for delta in [1, 3, 8, 10, 46, 210, 0]:
        cur = check(w, t3, ckpt_interval=delta, label=f"delta {delta}")
        if ref is None:
            ref = cur
        else:
            assert np.abs(cur[0] - ref[0]).max() <= 1e-6 * np.abs(ref[0]).max()
            for a, b in zip(cur[1:], ref[1:]):
                assert np.abs(a - b).max() <= 2e-6 * max(1.0, np.abs(b).max())
    seq = check(w, t3, ckpt_interval=10, extra_flags=sb.SEMICRF_SEQUENTIAL_SCAN, expect_chunked=False,
                label="sequential scans")
    for a, b in zip(seq, ref):
        assert np.abs(a - b).max() <= 2e-6 * max(1.0, np.abs(b).max())


def test_one_shared_matrix_reproduces_the_factorised_path():
    w = synth.small_random(41, 3, 180, 12, 6, ragged=True)
    t3 = np.broadcast_to(w.trans, (w.K, w.C, w.C)).astype(np.float32).copy()
    lz, g_e, g_t, g_d, pm = check(w, t3)
    dev = [torch.from_numpy(a).to(DEV) for a in (w.emis, w.lengths, w.trans, w.dur)]
    f = [o.double().cpu().numpy() for o in sb.semicrf_fwd_bwd(*dev)]
    torch.cuda.synchronize()
    assert np.abs(lz - f[0]).max() <= 1e-6 * np.abs(f[0]).max()
    assert np.abs(g_e - f[1]).max() <= 2e-6
    assert np.abs(g_t.sum(0) - f[2]).max() <= 2e-6 * max(1.0, np.abs(f[2]).max())
    assert np.abs(g_d - f[3]).max() <= 2e-6 * max(1.0, np.abs(f[3]).max())
    assert np.abs(pm - f[4]).max() <= 2e-6


def test_slow_mixing_input_falls_back_to_the_whole_sequence_scans():
    """Near-forbidden label changes: the recurrences forget their start too slowly for the
    warm-ups, the verification must reject the chunks and the whole-sequence scans must give
    the oracle's result."""
    B, T, K, C = 2, 600, 4, 3
    w = synth.small_random(51, B, T, K, C, ragged=False, scale=0.05)
    w.trans[:] = -14.0
    np.fill_diagonal(w.trans, 0.0)
    t3 = np.broadcast_to(w.trans, (K, C, C)).astype(np.float32).copy()
    check(w, t3, ckpt_interval=40, expect_chunked=False, label="slow mixing")


@pytest.mark.parametrize("name", ["nlp"])
def test_workload_shapes(name):
    w = synth.make(name)
    check(w, trans3_of(w, 7, sd=0.1), expect_chunked=True)


def test_reduced_genomic_and_longgen_shapes():
    for name, T in (("genomic", 3000), ("longgen", 4000)):
        w = synth.make(name)
        w2 = synth.small_random(61, 2, T, w.K, w.C, ragged=False)
        w2.dur[:] = w.dur
        check(w2, trans3_of(w2, 62, sd=0.1), label=f"{name} reduced", expect_chunked=True)


def test_unsupported_sizes_are_reported():
    with pytest.raises(sb.SemiCRFError) as e:
        sb.semicrf_durtrans_workspace_bytes(2, 100, 32, 64)          # 4096 label pairs
    assert e.value.status == -3
    with pytest.raises(sb.SemiCRFError) as e:
        sb.semicrf_durtrans_workspace_bytes(2, 100, 128, 32)         # 1024 pairs x 2 duration groups
    assert e.value.status == -3


def test_full_size_genomic_against_stored_oracle_values():
    """The genomic shape at full size, in the launch configuration bench.py --durtrans times,
    against oracle values stored by tests/golden/make_golden.py genomic --durtrans."""
    import os
    path = os.path.join(os.path.dirname(__file__), "golden", "full_genomic_durtrans.npz")
    if not os.path.exists(path):
        pytest.skip(f"{path} not generated")
    g = np.load(path)
    w = synth.make("genomic")
    t3 = synth.duration_transitions(w)
    print(f"[case] full genomic, duration-dependent transitions B={w.B} T={w.T} K={w.K} C={w.C}", flush=True)
    dev = [torch.from_numpy(a).to(DEV) for a in (w.emis, w.lengths, t3, w.dur)]
    logz, g_e, g_t, g_d, pm = sb.semicrf_fwd_bwd_durtrans(*dev)
    torch.cuda.synchronize()
    rel = np.abs(logz.double().cpu().numpy() - g["logz"]) / np.abs(g["logz"])
    rows = g["rows"]
    rb = torch.from_numpy(rows[:, 0]).to(DEV)
    ru = torch.from_numpy(rows[:, 1]).to(DEV)
    e_pm = np.abs(pm[rb, ru].double().cpu().numpy() - g["pos_marg_rows"]).max()
    e_ge = np.abs(g_e[rb, ru].double().cpu().numpy() - g["grad_emis_rows"]).max()
    e_t = np.abs(g_t.double().cpu().numpy() - g["grad_trans"]).max()
    e_d = np.abs(g_d.double().cpu().numpy() - g["grad_dur"]).max()
    print(f"       max err: logz rel {rel.max():.2e} pos_marg {e_pm:.2e} grad_emis {e_ge:.2e} "
          f"grad_trans3 {e_t:.2e} (max|g| {np.abs(g['grad_trans']).max():.3g}) "
          f"grad_dur {e_d:.2e} (max|g| {np.abs(g['grad_dur']).max():.3g})", flush=True)
    assert rel.max() <= 1e-5
    assert e_pm <= 1e-4 and e_ge <= 1e-4
    assert e_t <= 1e-4 * max(1.0, np.abs(g["grad_trans"]).max())
    assert e_d <= 1e-4 * max(1.0, np.abs(g["grad_dur"]).max())
    from golden_windows import check_windows
    check_windows(g, sb.semicrf_durtrans_ckpt_interval(w.B, w.T, w.K, w.C), pm, g_e)
    row_sum = pm.double().sum(-1)
    assert (row_sum - 1.0).abs().max().item() <= 1e-5              # every token of this workload is valid
    assert abs(g_t.double().sum().item() - g_d.double().sum().item()) <= 1e-5 * g_d.double().sum().item()
