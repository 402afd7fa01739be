"""GPU parity: the HIP path (through the C ABI) against the fp64 CPU oracle.

Tolerances (from the stated target): relative 1e-5 on logZ, absolute 1e-4 on
per-position gradients (grad_emis, pos_marg, all in [-1,1] up to the upstream
weight); the accumulated gradients grad_trans / grad_dur are sums of up to
sum_b L_b marginals, so they are held to 1e-4 * max(1, max|g|) and the raw
maximum error is printed.
"""
import os

import numpy as np
import pytest
import torch

import oracle
from paper_2604_18780_amd import binding as sb
from paper_2604_18780_amd import synth

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def to_dev(w, nan_pad=True):
    emis = w.emis.copy()
    if nan_pad:
        for b in range(w.B):
            emis[b, int(w.lengths[b]):] = np.nan      # padding must never be read
    return (torch.from_numpy(emis).to(DEV), torch.from_numpy(w.lengths).to(DEV),
            torch.from_numpy(w.trans).to(DEV), torch.from_numpy(w.dur).to(DEV))


def check_against_oracle(w, center=True, grad_logz=None, ckpt_interval=0, label="", extra_flags=0):
    """HIP path against the oracle.  Without a route in extra_flags the marginals are checked on both: the default
    one (stored rows of both scans where the plan has them) and the per-interval recurrence."""
    emis, lengths, trans, dur = to_dev(w)
    gl = None if grad_logz is None else torch.from_numpy(grad_logz.astype(np.float32)).to(DEV)
    r = oracle.fwd_bwd(w.emis, w.lengths, w.trans, w.dur, grad_logz=grad_logz, center=center)
    pinned = extra_flags & (sb.SEMICRF_MARGINALS_ROWS | sb.SEMICRF_MARGINALS_INTERVAL)
    for route in ([0] if pinned else [0, sb.SEMICRF_MARGINALS_INTERVAL]):
        flags = (sb.SEMICRF_CENTER if center else 0) | extra_flags | route
        print(f"[case] {label or w.name} B={w.B} T={w.T} K={w.K} C={w.C} center={center} "
              f"delta={ckpt_interval} flags={flags:#x}", flush=True)
        logz, g_e, g_t, g_d, pm = sb.semicrf_fwd_bwd(emis, lengths, trans, dur, gl, ckpt_interval, flags)
        logz_f = sb.semicrf_logz_fwd(emis, lengths, trans, dur, ckpt_interval, flags)
        torch.cuda.synchronize()
        lz = logz.double().cpu().numpy()
        assert np.all(np.isfinite(lz))
        rel = np.abs(lz - r.logz) / np.maximum(1.0, np.abs(r.logz))
        assert rel.max() <= 1e-5, (rel.max(), lz, r.logz)
        assert np.array_equal(lz, logz_f.double().cpu().numpy())       # forward-only entry agrees bit for bit
        e_pm = np.abs(pm.double().cpu().numpy() - r.pos_marg).max()
        e_ge = np.abs(g_e.double().cpu().numpy() - r.grad_emis).max()
        wmax = 1.0 if grad_logz is None else max(1.0, float(np.abs(grad_logz).max()))
        assert e_pm <= 1e-4, e_pm
        assert e_ge <= 1e-4 * wmax, e_ge
        e_t = np.abs(g_t.double().cpu().numpy() - r.grad_trans).max()
        e_d = np.abs(g_d.double().cpu().numpy() - r.grad_dur).max()
        print(f"       max err: logz rel {rel.max():.2e} pos_marg {e_pm:.2e} grad_emis {e_ge:.2e} "
              f"grad_trans {e_t:.2e} (max|g| {np.abs(r.grad_trans).max():.3g}) "
              f"grad_dur {e_d:.2e} (max|g| {np.abs(r.grad_dur).max():.3g})", flush=True)
        assert e_t <= 1e-4 * max(1.0, np.abs(r.grad_trans).max()), e_t
        assert e_d <= 1e-4 * max(1.0, np.abs(r.grad_dur).max()), e_d
    return r


def test_tiny_config_exact():
    check_against_oracle(synth.make("tiny"))


def test_tiny_config_no_centering():
    check_against_oracle(synth.make("tiny"), center=False)


@pytest.mark.parametrize("seed,B,T,K,C", [
    (1, 3, 40, 5, 3), (2, 4, 300, 8, 6), (3, 2, 700, 33, 24), (4, 5, 130, 1, 7),
    (5, 3, 90, 2, 5), (6, 2, 50, 80, 4), (7, 3, 257, 16, 64), (8, 6, 33, 7, 1),
    (9, 2, 513, 3, 17), (10, 1, 1, 1, 1),
])
def test_random_ragged_cases(seed, B, T, K, C):
    w = synth.small_random(seed, B, T, K, C, ragged=True)
    if seed == 2:
        w.lengths[0] = 0          # empty sequence
        w.lengths[1] = T          # full sequence
    rng = np.random.default_rng(seed)
    check_against_oracle(w, grad_logz=rng.standard_normal(B))


def test_large_emission_scale_changes_block_length():
    # emissions of scale 8 shorten the power-of-two scaling block
    check_against_oracle(synth.small_random(21, 2, 400, 12, 5, ragged=False, scale=8.0))
    check_against_oracle(synth.small_random(22, 2, 200, 6, 4, ragged=False, scale=30.0))


def test_checkpoint_interval_invariance():
    w = synth.small_random(31, 2, 210, 9, 5, ragged=True)
    w.lengths[:] = [210, 100]
    emis, lengths, trans, dur = to_dev(w)
    ref = None
    for delta in [1, 8, 9, 10, 15, 46, 210, 0]:
        out = sb.semicrf_fwd_bwd(emis, lengths, trans, dur, None, delta)
        torch.cuda.synchronize()
        cur = [o.double().cpu().numpy() for o in out]
        if ref is None:
            ref = cur
            check_against_oracle(w, ckpt_interval=delta)
        else:
            assert np.array_equal(cur[0], ref[0])                    # logZ does not depend on delta
            for a, b in zip(cur[1:], ref[1:]):
                assert np.abs(a - b).max() <= 2e-6


def test_padding_independence_and_determinism():
    w = synth.small_random(41, 3, 120, 10, 6, ragged=True)
    w.lengths[:] = [120, 77, 5]
    emis, lengths, trans, dur = to_dev(w)
    a = sb.semicrf_fwd_bwd(emis, lengths, trans, dur)
    b = sb.semicrf_fwd_bwd(emis, lengths, trans, dur)
    torch.cuda.synchronize()
    for x, y in zip(a, b):
        assert torch.equal(x, y)                                     # no atomics: bit-reproducible
    # sequence 1 alone, unpadded
    L = 77
    e1 = torch.from_numpy(w.emis[1:2, :L].copy()).to(DEV)
    l1 = torch.tensor([L], dtype=torch.int32, device=DEV)
    c = sb.semicrf_fwd_bwd(e1, l1, trans, dur, ckpt_interval=int(0))
    torch.cuda.synchronize()
    assert abs(float(c[0][0]) - float(a[0][1])) <= 1e-5 * abs(float(a[0][1]))
    assert (c[4][0] - a[4][1, :L]).abs().max().item() <= 2e-6
    assert torch.all(a[4][1, L:] == 0) and torch.all(a[1][1, L:] == 0)


def run_with_report(w, flags, ckpt_interval, warm_env=None):
    emis, lengths, trans, dur = to_dev(w)
    ws = sb.alloc_workspace(w.B, w.T, w.K, w.C, ckpt_interval, True, DEV)
    if warm_env is not None:
        flags |= sb.SEMICRF_WARMUP(warm_env)      # first warm-up length of the chunk-parallel scans
    out = sb.semicrf_fwd_bwd(emis, lengths, trans, dur, None, ckpt_interval, flags, workspace=ws)
    acc, mis = sb.semicrf_scan_report(ws, w.B, w.T, w.K, w.C, ckpt_interval, True)
    torch.cuda.synchronize()
    return [o.double().cpu().numpy() for o in out], acc.cpu().numpy(), mis.cpu().numpy()


def assert_outputs_match_oracle(out, r):
    assert np.abs(out[0] - r.logz).max() <= 1e-5 * max(1.0, np.abs(r.logz).max())
    assert np.abs(out[1] - r.grad_emis).max() <= 1e-4
    assert np.abs(out[4] - r.pos_marg).max() <= 1e-4
    assert np.abs(out[2] - r.grad_trans).max() <= 1e-4 * max(1.0, np.abs(r.grad_trans).max())
    assert np.abs(out[3] - r.grad_dur).max() <= 1e-4 * max(1.0, np.abs(r.grad_dur).max())


def test_chunk_parallel_and_sequential_scans_agree():
    """Default (chunk-parallel, verified) against SEMICRF_SEQUENTIAL_SCAN on a case with
    many chunks and a ragged batch; both against the oracle."""
    w = synth.small_random(71, 4, 1500, 12, 10, ragged=True)
    w.lengths[:] = [1500, 1499, 64, 3]
    r = oracle.fwd_bwd(w.emis, w.lengths, w.trans, w.dur)
    par, acc, mis = run_with_report(w, sb.SEMICRF_CENTER, 64)
    seq, acc_s, mis_s = run_with_report(w, sb.SEMICRF_CENTER | sb.SEMICRF_SEQUENTIAL_SCAN, 64)
    print(f"       boundary mismatch per (sequence, direction): {mis.ravel()}", flush=True)
    assert np.all(acc == 1) and np.all(mis >= 0) and np.all(mis <= 1e-10)
    assert np.all(acc_s == 0) and np.all(mis_s == -1)
    assert_outputs_match_oracle(par, r)
    assert_outputs_match_oracle(seq, r)
    assert np.abs(par[0] - seq[0]).max() <= 1e-6 * np.abs(seq[0]).max()
    for a, b in zip(par[1:], seq[1:]):
        assert np.abs(a - b).max() <= 2e-6 * max(1.0, np.abs(b).max())


def test_short_warm_up_is_rejected_then_longer_one_accepted():
    """First warm-up of K/2 positions cannot reproduce the ring state (it does not even fill
    the ring); the second attempt (four times as long) does.  Results as the oracle's."""
    w = synth.small_random(72, 2, 900, 16, 6, ragged=False)
    r = oracle.fwd_bwd(w.emis, w.lengths, w.trans, w.dur)
    out, acc, mis = run_with_report(w, sb.SEMICRF_CENTER, 48, warm_env=8)
    # every boundary disagrees at first, so restarting single intervals cannot settle it (attempt 2); the long
    # warm-up does (attempt 3)
    assert np.all(acc == 3) and np.all(mis <= 1e-10)
    assert_outputs_match_oracle(out, r)


@pytest.mark.parametrize("flat", [(590, 680), (600, 700)])
def test_disagreeing_boundaries_are_repaired_from_the_reached_state(flat):
    """A deterministic chain (segments of exactly two tokens, labels in a fixed cycle) is pinned by its
    emissions everywhere except on a flat stretch.  The interval boundary at 640, whose warm-up window of 32
    positions lies inside the flat stretch, cannot recover the phase, so its check fails in both directions.
    With the stretch 590..680 it is the only one; with 600..700 the forward window of the boundary at 704 holds
    just four informative positions, too few to bring the improbable entries to 1e-10, so two adjacent forward
    boundaries fail.  The repair attempts rerun just those intervals from the state their neighbour reached:
    accepted with code 2, results as the oracle's."""
    B, T, K, C = 2, 2000, 4, 4
    w = synth.small_random(74, B, T, K, C, ragged=False)
    label = (np.arange(T) // 2) % C
    w.emis[:] = 0.0
    w.emis[:, np.arange(T), label] = 8.0
    w.emis[:, flat[0]:flat[1], :] = 0.0              # nothing to pin the phase here
    w.trans[:] = -40.0
    for c in range(C):
        w.trans[c, (c + 1) % C] = 0.0                # fixed cycle
    w.dur[:] = -40.0
    w.dur[1, :] = 0.0                                # segments of exactly two tokens
    r = oracle.fwd_bwd(w.emis, w.lengths, w.trans, w.dur)
    out, acc, mis = run_with_report(w, sb.SEMICRF_CENTER, 64)
    print(f"       accepted {acc.ravel()} boundary mismatch {mis.ravel()}", flush=True)
    assert np.all(acc == 2) and np.all(mis <= 1e-10)
    assert_outputs_match_oracle(out, r)
    # the same input through the sequential scans
    seq, acc_s, _ = run_with_report(w, sb.SEMICRF_CENTER | sb.SEMICRF_SEQUENTIAL_SCAN, 64)
    assert np.all(acc_s == 0)
    for a, b in zip(out, seq):
        assert np.abs(a - b).max() <= 2e-6 * max(1.0, np.abs(b).max())


def test_slow_mixing_input_falls_back_to_the_sequential_scan():
    """A nearly deterministic two-label chain with weak emissions remembers its start for
    thousands of positions, so no warm-up of a few K reproduces the state: every boundary
    check must fail and the sequential scan must deliver the (oracle's) result."""
    rng = np.random.default_rng(73)
    B, T, K, C = 2, 2000, 2, 2
    w = synth.small_random(73, B, T, K, C, ragged=False)
    w.emis[:] = (0.05 * rng.standard_normal((B, T, C))).astype(np.float32)
    w.trans[:] = np.array([[0.0, -40.0], [-40.0, 0.0]], dtype=np.float32)
    w.dur[:] = 0.0
    r = oracle.fwd_bwd(w.emis, w.lengths, w.trans, w.dur)
    out, acc, mis = run_with_report(w, sb.SEMICRF_CENTER, 64)
    print(f"       boundary mismatch per (sequence, direction): {mis.ravel()}", flush=True)
    assert np.all(acc == 0) and np.all(mis > 1e-10)
    assert_outputs_match_oracle(out, r)


def test_sizes_beyond_the_one_wave_kernels_use_the_generic_kernels():
    """K too long for the register strips of the one-wave kernels (C=24: K > 128): the generic
    scan and interval kernels compute the result, sequentially."""
    w = synth.small_random(81, 2, 300, 200, 24, ragged=True)
    r = oracle.fwd_bwd(w.emis, w.lengths, w.trans, w.dur)
    out, acc, mis = run_with_report(w, sb.SEMICRF_CENTER, 0)
    assert np.all(acc == 0) and np.all(mis == -1)
    assert_outputs_match_oracle(out, r)


def test_more_than_64_labels_forward_only():
    """C > 64 is supported for logZ only (generic scan kernel); gradients are refused."""
    w = synth.small_random(82, 2, 120, 6, 100, ragged=True)
    emis, lengths, trans, dur = to_dev(w)
    lz = sb.semicrf_logz_fwd(emis, lengths, trans, dur).double().cpu().numpy()
    ref = oracle.logz(w.emis, w.lengths, w.trans, w.dur)
    assert np.abs(lz - ref).max() <= 1e-5 * np.abs(ref).max()
    with pytest.raises(sb.SemiCRFError) as ei:
        sb.semicrf_fwd_bwd(emis, lengths, trans, dur)
    assert ei.value.status == -3


def test_more_tasks_than_buffer_slots():
    """An explicit interval of 2 positions gives 2250 (sequence, interval) tasks, more than the
    1024 task buffers: the interval kernel then loops over tasks and recomputes its forward rows
    instead of taking them from the chunk-parallel scan."""
    w = synth.small_random(91, 3, 1500, 6, 5, ragged=True)
    w.lengths[:] = [1500, 1500, 1497]
    r = oracle.fwd_bwd(w.emis, w.lengths, w.trans, w.dur)
    out, acc, mis = run_with_report(w, sb.SEMICRF_CENTER, 2)
    assert np.all(acc == 1)
    assert_outputs_match_oracle(out, r)


def test_cum_scores_matches_oracle_prefix_sums():
    w = synth.small_random(51, 3, 700, 4, 9, ragged=True)
    w.lengths[:] = [700, 256, 0]
    emis, lengths, _, _ = to_dev(w)
    for center in (True, False):
        cum = sb.semicrf_cum_scores(emis, lengths, sb.SEMICRF_CENTER if center else 0)
        torch.cuda.synchronize()
        r = oracle.fwd_bwd(w.emis, w.lengths, w.trans, w.dur, center=center, tables=True)
        assert np.abs(cum.cpu().numpy() - r.S).max() <= 1e-9


def test_nlp_config():
    check_against_oracle(synth.make("nlp"))


def test_speech_config_reduced_batch():
    # the speech shape (K=32, C=64, lengths in [T/2, T]) on 6 sequences of T=600
    check_against_oracle(synth.make("speech", B=6, T=600))


def test_genomic_shape_reduced_length():
    check_against_oracle(synth.make("genomic", T=6000, B=2))


def test_longgen_shape_reduced_length():
    check_against_oracle(synth.make("longgen", T=3000))


def test_unsupported_and_invalid_arguments_are_rejected():
    w = synth.small_random(61, 1, 8, 2, 3, ragged=False)
    emis, lengths, trans, dur = to_dev(w, nan_pad=False)
    with pytest.raises(sb.SemiCRFError) as ei:
        sb.semicrf_fwd_bwd(emis, lengths, trans, dur, workspace=torch.empty(256, dtype=torch.uint8, device=DEV))
    assert ei.value.status == -2
    with pytest.raises(sb.SemiCRFError) as ei:
        sb.semicrf_logz_fwd(emis, lengths, trans, dur, ckpt_interval=-1)
    assert ei.value.status == -1


# --------------------------------------------------------------------------
# Full-size workloads, in the launch configuration bench.py times, against
# oracle values stored by tests/golden/make_golden.py (which calls only oracle/).
# --------------------------------------------------------------------------
import os

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


from golden_windows import check_windows  # noqa: E402


@pytest.mark.parametrize("name", ["speech", "genomic", "longgen"])
def test_full_size_workload_against_stored_oracle_values(name):
    path = os.path.join(GOLDEN, f"full_{name}.npz")
    if not os.path.exists(path):
        pytest.skip(f"{path} not generated")
    g = np.load(path)
    w = synth.make(name)
    emis, lengths, trans, dur = to_dev(w)
    print(f"[case] full {name} B={w.B} T={w.T} K={w.K} C={w.C}", flush=True)
    logz, g_e, g_t, g_d, pm = sb.semicrf_fwd_bwd(emis, lengths, trans, dur)
    torch.cuda.synchronize()
    lz = logz.double().cpu().numpy()
    rel = np.abs(lz - g["logz"]) / np.abs(g["logz"])
    assert rel.max() <= 1e-5, rel.max()
    rows = g["rows"]
    rb = torch.from_numpy(rows[:, 0]).to(DEV)
    ru = torch.from_numpy(rows[:, 1]).to(DEV)
    e_pm = np.abs(pm[rb, ru].double().cpu().numpy() - g["pos_marg_rows"]).max()
    e_ge = np.abs(g_e[rb, ru].double().cpu().numpy() - g["grad_emis_rows"]).max()
    e_t = np.abs(g_t.double().cpu().numpy() - g["grad_trans"]).max()
    e_d = np.abs(g_d.double().cpu().numpy() - g["grad_dur"]).max()
    print(f"       max err: logz rel {rel.max():.2e} pos_marg {e_pm:.2e} grad_emis {e_ge:.2e} "
          f"grad_trans {e_t:.2e} (max|g| {np.abs(g['grad_trans']).max():.3g}) "
          f"grad_dur {e_d:.2e} (max|g| {np.abs(g['grad_dur']).max():.3g})", flush=True)
    assert e_pm <= 1e-4 and e_ge <= 1e-4
    assert e_t <= 1e-4 * max(1.0, np.abs(g["grad_trans"]).max())
    assert e_d <= 1e-4 * max(1.0, np.abs(g["grad_dur"]).max())
    check_windows(g, sb.semicrf_ckpt_interval(w.B, w.T, w.K, w.C), pm, g_e)
    # properties over ALL rows: each valid token's label posterior sums to one,
    # padding carries no mass, total mass = number of valid tokens
    row_sum = pm.double().sum(-1)
    valid = torch.arange(w.T, device=DEV)[None, :] < lengths[:, None]
    assert (row_sum[valid] - 1.0).abs().max().item() <= 1e-5
    assert row_sum[~valid].abs().max().item() == 0.0 if (~valid).any() else True
    assert abs(pm.double().sum().item() - float(w.positions)) <= 1e-6 * w.positions
    assert pm.min().item() >= -1e-6 and pm.max().item() <= 1.0 + 1e-6
    # expected segment count from both accumulated gradients agrees
    assert abs(g_t.double().sum().item() - g_d.double().sum().item()) <= 1e-5 * g_d.double().sum().item()


# --------------------------------------------------------------------------
# Half-precision emissions (IEEE half, bfloat16): widened exactly on load
# --------------------------------------------------------------------------
@pytest.mark.parametrize("dtype", [torch.float16, torch.bfloat16])
def test_half_precision_emissions(dtype):
    w = synth.small_random(95, 3, 500, 10, 12, ragged=True)
    e_half = torch.from_numpy(w.emis).to(dtype)                 # round once, on the host
    w.emis = e_half.to(torch.float32).numpy().copy()            # the oracle sees exactly those values
    r = oracle.fwd_bwd(w.emis, w.lengths, w.trans, w.dur)
    _, lengths, trans, dur = to_dev(w)
    e_dev = e_half.to(DEV)
    for b in range(w.B):
        e_dev[b, int(w.lengths[b]):] = float("nan")
    out = sb.semicrf_fwd_bwd(e_dev, lengths, trans, dur)
    ref = sb.semicrf_fwd_bwd(e_dev.to(torch.float32), lengths, trans, dur)
    lz = sb.semicrf_logz_fwd(e_dev, lengths, trans, dur)
    cum = sb.semicrf_cum_scores(e_dev, lengths)
    torch.cuda.synchronize()
    assert_outputs_match_oracle([o.double().cpu().numpy() for o in out], r)
    for a, b_ in zip(out, ref):
        assert torch.equal(a, b_)                                # same values in, same bits out
    assert torch.equal(lz, out[0])
    rt = oracle.fwd_bwd(w.emis, w.lengths, w.trans, w.dur, tables=True)
    assert np.abs(cum.cpu().numpy() - rt.S).max() <= 1e-9
    # both storage flags at once are refused
    with pytest.raises(sb.SemiCRFError) as ei:
        lib = sb.load()
        rc = lib.semicrf_logz_fwd(e_dev.data_ptr(), None, trans.data_ptr(), dur.data_ptr(), w.B, w.T, w.K, w.C, 0,
                                  sb.SEMICRF_EMIS_F16 | sb.SEMICRF_EMIS_BF16, 4096, 1 << 30, lz.data_ptr(), None)
        sb._check(rc)
    assert ei.value.status == -1


# --------------------------------------------------------------------------
# Marginals from the stored rows of both scans (the route taken for K >= 128), forced on
# small shapes so that every case above also covers it
# --------------------------------------------------------------------------
@pytest.mark.parametrize("seed,B,T,K,C", [
    (1, 3, 40, 5, 3), (2, 4, 300, 8, 6), (3, 2, 700, 33, 24), (4, 5, 130, 1, 7),
    (6, 2, 50, 80, 4), (7, 3, 257, 16, 64), (8, 6, 33, 7, 1), (11, 2, 900, 130, 8),
])
def test_marginals_from_stored_rows(seed, B, T, K, C):
    ROWS = sb.SEMICRF_MARGINALS_ROWS
    w = synth.small_random(seed, B, T, K, C, ragged=True)
    if seed == 2:
        w.lengths[0] = 0
        w.lengths[1] = T
    rng = np.random.default_rng(seed)
    check_against_oracle(w, grad_logz=rng.standard_normal(B), label=f"stored rows, rand{seed}", extra_flags=ROWS)
    check_against_oracle(w, ckpt_interval=max(8, K // 2 + 3), label=f"stored rows, rand{seed}, short intervals",
                         extra_flags=ROWS)


@pytest.mark.parametrize("seed,B,T,K,C,delta,lengths,scale", [
    # two intervals of 320 cut into four parts of 80: lengths that end inside a part, on a part boundary, on the
    # interval boundary, one position into the second interval, and short of one block
    (81, 6, 600, 20, 5, 320, [600, 81, 160, 320, 321, 3], 1.0),
    # two label tiles on the matrix cores, parts of 88 >= K = 40; emissions of scale 6 shorten the scaling block,
    # so that part boundaries fall inside scaling blocks and the window fill crosses several of them
    (82, 2, 700, 40, 24, 352, [700, 439], 6.0),
    # 64 labels (one task per SIMD variant), parts of 64 >= K
    (83, 2, 300, 33, 64, 128, [300, 191], 1.0),
    # parts as short as the plan allows (K = 32 positions each) and a sequence that ends with position 0's block
    (84, 3, 256, 32, 8, 128, [256, 4, 97], 1.0),
])
def test_stored_row_marginals_in_parts(seed, B, T, K, C, delta, lengths, scale):
    """The one-wave stored-row kernel with every interval cut into parts (few tasks: the plan cuts into 2 or 4):
    upper parts start from the checkpoint, inner parts fill their window from the stored rows."""
    w = synth.small_random(seed, B, T, K, C, ragged=False, scale=scale)
    w.lengths[:] = lengths
    rng = np.random.default_rng(seed)
    check_against_oracle(w, grad_logz=rng.standard_normal(B), ckpt_interval=delta,
                         label=f"stored rows in parts, rand{seed}", extra_flags=sb.SEMICRF_MARGINALS_ROWS)
    # the per-part partial sums must give the same outputs as one partial sum per interval
    emis, lens, trans, dur = to_dev(w)
    a = sb.semicrf_fwd_bwd(emis, lens, trans, dur, None, delta, sb.SEMICRF_CENTER)
    b = sb.semicrf_fwd_bwd(emis, lens, trans, dur, None, delta, sb.SEMICRF_CENTER | sb.SEMICRF_MARGINALS_INTERVAL)
    torch.cuda.synchronize()
    for x, y in zip(a[1:], b[1:]):
        d = (x.double() - y.double()).abs().max().item()
        assert d <= 2e-5 * max(1.0, y.double().abs().max().item()), d


def test_marginals_from_stored_rows_large_scale_and_mixed_acceptance():
    ROWS, ITV = sb.SEMICRF_MARGINALS_ROWS, sb.SEMICRF_MARGINALS_INTERVAL
    # scaling blocks of a few positions
    check_against_oracle(synth.small_random(21, 2, 400, 12, 5, ragged=False, scale=8.0), label="stored rows, scale 8",
                         extra_flags=ROWS)
    # both routes agree with each other to rounding
    w = synth.small_random(96, 3, 600, 20, 6, ragged=True)
    dev = to_dev(w)
    rows = [o.double().cpu().numpy() for o in sb.semicrf_fwd_bwd(*dev, flags=sb.SEMICRF_CENTER | ROWS)]
    itv = [o.double().cpu().numpy() for o in sb.semicrf_fwd_bwd(*dev, flags=sb.SEMICRF_CENTER | ITV)]
    torch.cuda.synchronize()
    assert np.array_equal(rows[0], itv[0])
    for a, b in zip(rows[1:], itv[1:]):
        assert np.abs(a - b).max() <= 2e-6 * max(1.0, np.abs(b).max())
    # a slow-mixing input whose scans are rejected falls back to the interval kernels
    B, T, K, C = 2, 600, 4, 3
    w = synth.small_random(51, B, T, K, C, ragged=False, scale=0.05)
    w.trans[:] = -14.0
    np.fill_diagonal(w.trans, 0.0)
    check_against_oracle(w, ckpt_interval=40, label="stored rows requested, scans rejected", extra_flags=ROWS)


@pytest.mark.parametrize("seed,B,T,K,C,scale", [
    (31, 2, 1500, 160, 24, 1.0),   # three duration strips per label row of a wave
    (32, 1, 600, 128, 32, 1.0),    # K*C at the limit of the gradient kernels
    (35, 1, 2500, 1024, 4, 1.0),   # the longest durations they take
    (33, 2, 900, 130, 5, 30.0),    # scaling blocks of one or two positions: a frame per one or two positions
    (34, 3, 700, 200, 12, 8.0),
])
def test_long_durations_take_the_stored_rows_route_by_default(seed, B, T, K, C, scale):
    w = synth.small_random(seed, B, T, K, C, ragged=True, scale=scale)
    rng = np.random.default_rng(seed)
    check_against_oracle(w, grad_logz=rng.standard_normal(B), label=f"K >= 128, rand{seed}")


def test_longgen_shape_reduced_takes_the_stored_rows_route():
    w0 = synth.make("longgen")
    w = synth.small_random(97, 1, 6000, w0.K, w0.C, ragged=False)
    w.dur[:] = w0.dur
    check_against_oracle(w, label="longgen reduced (K = 512)")


@pytest.mark.parametrize("seed,B,T,K,C", [(81, 2, 3000, 8, 6), (82, 3, 1500, 40, 24), (83, 1, 5000, 130, 5),
                                          (84, 2, 90, 4, 3)])
def test_low_memory_plan_matches_oracle(seed, B, T, K, C):
    """SEMICRF_LOW_MEMORY: checkpoints every ceil(sqrt(T*K)) positions, eight row buffers per sequence, the
    forward rows of an interval recomputed from its checkpoint (Algorithm 3's body).  Same results."""
    w = synth.small_random(seed, B, T, K, C, ragged=True)
    w.lengths[0] = T
    delta = sb.semicrf_ckpt_interval_low_memory(B, T, K, C)
    assert delta == min(T, (int(np.ceil(np.sqrt(T * K))) + 7) // 8 * 8)
    check_against_oracle(w, label="low-memory plan", extra_flags=sb.SEMICRF_LOW_MEMORY,
                         grad_logz=np.random.default_rng(seed).standard_normal(B))
    # the workspace of the default plan has another layout: one that is too small for this call is refused
    emis, lengths, trans, dur = to_dev(w)
    small = sb.alloc_workspace(B, T, K, C, 0, sb.PLAN_LOW_MEMORY, DEV)      # forward-only size
    with pytest.raises(sb.SemiCRFError, match="-2"):
        sb.semicrf_fwd_bwd(emis, lengths, trans, dur, flags=sb.SEMICRF_CENTER | sb.SEMICRF_LOW_MEMORY, workspace=small)
    with pytest.raises(sb.SemiCRFError, match="-1"):
        sb.semicrf_fwd_bwd(emis, lengths, trans, dur,
                           flags=sb.SEMICRF_CENTER | sb.SEMICRF_LOW_MEMORY | sb.SEMICRF_MARGINALS_ROWS)


def test_low_memory_plan_more_tasks_than_row_buffers_genomic_shape():
    """Genomic shape cut to T = 20 000: 4 x 18 intervals of 1136 positions share 36 row buffers."""
    w = synth.make("genomic", T=20000)
    flags = sb.SEMICRF_CENTER | sb.SEMICRF_LOW_MEMORY
    kind = sb.grad_workspace_kind(flags)
    assert kind == 9
    emis, lengths, trans, dur = to_dev(w)
    ws = sb.alloc_workspace(w.B, w.T, w.K, w.C, 0, kind, DEV)
    out = sb.semicrf_fwd_bwd(emis, lengths, trans, dur, None, 0, flags, workspace=ws)
    acc, mis = sb.semicrf_scan_report(ws, w.B, w.T, w.K, w.C, 0, kind)
    ref = sb.semicrf_fwd_bwd(emis, lengths, trans, dur)
    torch.cuda.synchronize()
    assert np.all(acc.cpu().numpy() == 1) and float(mis.max()) <= 1e-10
    r = oracle.fwd_bwd(w.emis, w.lengths, w.trans, w.dur)
    assert_outputs_match_oracle([o.double().cpu().numpy() for o in out], r)
    for a, b in zip(out, ref):
        assert (a.double() - b.double()).abs().max().item() <= 2e-6 * max(1.0, b.double().abs().max().item())
    assert ws.numel() < 0.7 * sb.semicrf_workspace_bytes(w.B, w.T, w.K, w.C, 0, 1)


def test_sequence_report_range_flag_and_double_logz():
    """semicrf_seq_report: logZ in fp64 as the forward scan computed it, and the flag of sequences whose scores
    exceed the range the scaled recurrences are built for (300 nats per position)."""
    B, T, K, C = 3, 400, 6, 5
    w = synth.small_random(91, B, T, K, C, ragged=False)
    w.emis[1, 100, 2] = 5000.0            # one position that no scaling block can hold
    emis, lengths, trans, dur = to_dev(w)
    ws = sb.alloc_workspace(B, T, K, C, 0, 1, DEV)
    out = sb.semicrf_fwd_bwd(emis, lengths, trans, dur, workspace=ws)
    rng, lz64 = sb.semicrf_seq_report(ws, B, T, K, C, 0, 1)
    torch.cuda.synchronize()
    assert rng.cpu().numpy().tolist() == [0, 1, 0]
    r = oracle.fwd_bwd(w.emis, w.lengths, w.trans, w.dur)
    lz = lz64.cpu().numpy()
    for b in (0, 2):
        assert abs(lz[b] - r.logz[b]) <= 1e-9 * max(1.0, abs(r.logz[b]))
        assert np.float32(lz[b]) == out[0].cpu().numpy()[b]
    # forward-only calls leave the same fields
    fws = sb.alloc_workspace(B, T, K, C, 0, 0, DEV)
    sb.semicrf_logz_fwd(emis, lengths, trans, dur, workspace=fws)
    rng2, lz2 = sb.semicrf_seq_report(fws, B, T, K, C, 0, 0)
    torch.cuda.synchronize()
    assert rng2.cpu().numpy().tolist() == [0, 1, 0]
    assert np.array_equal(lz2.cpu().numpy()[[0, 2]], lz[[0, 2]])


@pytest.mark.parametrize("waves", ["one", "two"])
@pytest.mark.parametrize("seed,B,T,K,C,delta,scale", [
    (101, 3, 300, 8, 6, 0, 1.0), (102, 2, 700, 33, 24, 64, 1.0), (103, 3, 257, 16, 64, 32, 1.0), (104, 2, 513, 3, 17, 40, 8.0),
    (105, 2, 1500, 64, 24, 96, 8.0), (106, 2, 900, 130, 8, 0, 1.0), (107, 1, 1100, 512, 8, 0, 1.0), (108, 2, 50, 80, 4, 0, 30.0),
    (109, 4, 130, 1, 7, 16, 1.0), (110, 2, 600, 40, 32, 0, 1.0),
])
def test_scan_tasks_with_one_and_with_two_waves(waves, seed, B, T, K, C, delta, scale):
    """The chunk-parallel scan tasks in both forms (one wave; tip + helper) on shapes of every kernel variant:
    verified at the first attempt, results as the oracle's, and the two forms agree to rounding."""
    w = synth.small_random(seed, B, T, K, C, ragged=True, scale=scale)
    w.lengths[0] = T
    flag = sb.SEMICRF_ONE_WAVE_SCAN if waves == "one" else sb.SEMICRF_TWO_WAVE_SCAN
    out, acc, mis = run_with_report(w, sb.SEMICRF_CENTER | flag, delta)
    print(f"       accepted {acc.ravel()} boundary mismatch {mis.max():.1e}", flush=True)
    assert np.all(acc == 1) and np.all(mis <= 1e-10)
    r = oracle.fwd_bwd(w.emis, w.lengths, w.trans, w.dur)
    assert_outputs_match_oracle(out, r)
    other, _, _ = run_with_report(w, sb.SEMICRF_CENTER | (sb.SEMICRF_ONE_WAVE_SCAN | sb.SEMICRF_TWO_WAVE_SCAN) ^ flag, delta)
    for a, b_ in zip(out, other):
        assert np.abs(a - b_).max() <= 2e-6 * max(1.0, np.abs(b_).max())
    emis, lengths, trans, dur = to_dev(w)
    with pytest.raises(sb.SemiCRFError, match="-1"):
        sb.semicrf_logz_fwd(emis, lengths, trans, dur, flags=sb.SEMICRF_ONE_WAVE_SCAN | sb.SEMICRF_TWO_WAVE_SCAN)
