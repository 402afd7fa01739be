"""GPU parity of the boundary terms of Eq. 4 (start/end projections, scalar sequence
boundaries), their gradients and the boundary posterior, against the fp64 CPU oracle.

Tolerances as in test_gpu_parity.py: logZ relative 1e-5; per-position outputs (grad_emis,
pos_marg, grad_proj_start, grad_proj_end, bdy_post: probabilities times the upstream weight)
absolute 1e-4 * max(1, |w|); accumulated gradients 1e-4 * max(1, max|g|).
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2604_18780_amd import binding as sb
from paper_2604_18780_amd import synth

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def dev(a, dtype=np.float32):
    return None if a is None else torch.from_numpy(np.ascontiguousarray(a, dtype=dtype)).to(DEV)


def make_terms(seed, w, scale=0.5):
    rng = np.random.default_rng(seed)
    ps = (scale * rng.standard_normal((w.B, w.T, w.C))).astype(np.float32)
    pe = (scale * rng.standard_normal((w.B, w.T, w.C))).astype(np.float32)
    pis = rng.standard_normal(w.C).astype(np.float32)
    pie = rng.standard_normal(w.C).astype(np.float32)
    return ps, pe, pis, pie


def nan_pad(a, lengths):
    a = a.copy()
    for b in range(a.shape[0]):
        a[b, int(lengths[b]):] = np.nan       # rows beyond the sequence must never be read
    return a


def check(w, ps, pe, pis, pie, grad_logz=None, ckpt_interval=0, flags=sb.SEMICRF_CENTER, label=""):
    print(f"[case] {label} B={w.B} T={w.T} K={w.K} C={w.C} delta={ckpt_interval} flags={flags}", flush=True)
    emis = dev(nan_pad(w.emis, w.lengths))
    out = sb.semicrf_fwd_bwd_boundary(
        emis, dev(w.lengths, np.int32), dev(w.trans), dev(w.dur), dev(grad_logz),
        dev(None if ps is None else nan_pad(ps, w.lengths)), dev(None if pe is None else nan_pad(pe, w.lengths)),
        dev(pis), dev(pie), ckpt_interval, flags)
    lz_f = sb.semicrf_logz_fwd_boundary(emis, dev(w.lengths, np.int32), dev(w.trans), dev(w.dur),
                                        dev(None if ps is None else nan_pad(ps, w.lengths)),
                                        dev(None if pe is None else nan_pad(pe, w.lengths)), dev(pis), dev(pie),
                                        ckpt_interval, flags)
    torch.cuda.synchronize()
    o = {k: v.double().cpu().numpy() for k, v in out.items()}
    r = oracle.fwd_bwd(w.emis, w.lengths, w.trans, w.dur, grad_logz=grad_logz, proj_start=ps, proj_end=pe,
                       pi_start=pis, pi_end=pie, boundary=True, center=bool(flags & sb.SEMICRF_CENTER))
    wmax = 1.0 if grad_logz is None else max(1.0, float(np.abs(grad_logz).max()))
    assert np.all(np.isfinite(o["logz"]))
    assert np.abs(o["logz"] - r.logz).max() <= 1e-5 * max(1.0, np.abs(r.logz).max())
    assert np.array_equal(o["logz"], lz_f.double().cpu().numpy())
    errs = {}
    for name, ref in (("grad_emis", r.grad_emis), ("pos_marg", r.pos_marg), ("grad_proj_start", r.grad_proj_start),
                      ("grad_proj_end", r.grad_proj_end), ("bdy_post", r.bdy_post)):
        errs[name] = np.abs(o[name] - ref).max()
        assert errs[name] <= 1e-4 * wmax, (name, errs[name])
    for name, ref in (("grad_trans", r.grad_trans), ("grad_dur", r.grad_dur), ("grad_pi_start", r.grad_pi_start),
                      ("grad_pi_end", r.grad_pi_end)):
        errs[name] = np.abs(o[name] - ref).max()
        assert errs[name] <= 1e-4 * max(1.0, np.abs(ref).max()), (name, errs[name])
    print("       max err: " + " ".join(f"{k} {v:.1e}" for k, v in errs.items()), flush=True)
    return o, r


@pytest.mark.parametrize("seed,B,T,K,C", [
    (1, 3, 40, 5, 3), (2, 4, 300, 8, 6), (3, 2, 700, 33, 24), (4, 5, 130, 1, 7),
    (5, 3, 90, 2, 5), (6, 2, 50, 80, 4), (7, 3, 257, 16, 64), (8, 6, 33, 7, 1), (9, 1, 1, 1, 1),
])
def test_random_ragged_cases_with_all_boundary_terms(seed, B, T, K, C):
    w = synth.small_random(seed, B, T, K, C, ragged=True)
    if seed == 2:
        w.lengths[0] = 0
        w.lengths[1] = T
    rng = np.random.default_rng(seed)
    check(w, *make_terms(100 + seed, w), grad_logz=rng.standard_normal(B))


def test_each_term_alone_and_none():
    w = synth.small_random(21, 3, 260, 12, 10, ragged=True)
    ps, pe, pis, pie = make_terms(121, w)
    check(w, ps, None, None, None, label="start projections only")
    check(w, None, pe, None, None, label="end projections only")
    check(w, None, None, pis, pie, label="scalar boundaries only")
    o, _ = check(w, None, None, None, None, label="no boundary term")
    # with no term the plain entry point must give the same bits
    emis = dev(nan_pad(w.emis, w.lengths))
    plain = sb.semicrf_fwd_bwd(emis, dev(w.lengths, np.int32), dev(w.trans), dev(w.dur))
    torch.cuda.synchronize()
    for name, t in zip(("logz", "grad_emis", "grad_trans", "grad_dur", "pos_marg"), plain):
        assert np.array_equal(o[name], t.double().cpu().numpy()), name


@pytest.mark.parametrize("K,C,flags", [(130, 8, 0), (160, 5, 0), (12, 10, sb.SEMICRF_MARGINALS_ROWS)])
def test_boundary_inputs_without_boundary_outputs_where_the_stored_row_marginals_would_apply(K, C, flags):
    """Start / end projections as INPUTS only, at sizes where the marginals are otherwise formed from the stored
    rows of both scans (K >= 128, or on request): those kernels rebuild the emission sums from the stored
    (ES, 1/ES) pairs, which the projections change, so such calls must go through the interval kernel."""
    w = synth.small_random(61, 2, 900, K, C, ragged=True)
    w.lengths[0] = 900
    ps, pe, pis, pie = make_terms(62, w)
    flags |= sb.SEMICRF_CENTER
    emis, lengths = dev(nan_pad(w.emis, w.lengths)), dev(w.lengths, np.int32)
    o = sb.semicrf_fwd_bwd_boundary(emis, lengths, dev(w.trans), dev(w.dur), None, dev(nan_pad(ps, w.lengths)),
                                    dev(nan_pad(pe, w.lengths)), dev(pis), dev(pie), 0, flags, boundary_outputs=False)
    torch.cuda.synchronize()
    assert set(o) == {"logz", "grad_emis", "grad_trans", "grad_dur", "pos_marg"}
    r = oracle.fwd_bwd(w.emis, w.lengths, w.trans, w.dur, proj_start=ps, proj_end=pe, pi_start=pis, pi_end=pie,
                       boundary=True)
    g = {k: v.double().cpu().numpy() for k, v in o.items()}
    assert np.abs(g["logz"] - r.logz).max() <= 1e-5 * max(1.0, np.abs(r.logz).max())
    assert np.abs(g["pos_marg"] - r.pos_marg).max() <= 1e-4
    assert np.abs(g["grad_emis"] - r.grad_emis).max() <= 1e-4
    assert np.abs(g["grad_trans"] - r.grad_trans).max() <= 1e-4 * max(1.0, np.abs(r.grad_trans).max())
    assert np.abs(g["grad_dur"] - r.grad_dur).max() <= 1e-4 * max(1.0, np.abs(r.grad_dur).max())


def test_many_chunks_no_centering_and_sequential_fallback():
    w = synth.small_random(22, 2, 1500, 12, 10, ragged=True)
    w.lengths[:] = [1500, 1203]
    terms = make_terms(122, w)
    check(w, *terms, ckpt_interval=64, label="many chunks")
    check(w, *terms, ckpt_interval=64, flags=0, label="no centring")
    check(w, *terms, ckpt_interval=64, flags=sb.SEMICRF_CENTER | sb.SEMICRF_SEQUENTIAL_SCAN,
          label="sequential scans")


def test_generic_kernels_with_boundary_terms():
    w = synth.small_random(23, 2, 300, 200, 24, ragged=True)       # K beyond the one-wave kernels
    check(w, *make_terms(123, w), label="generic kernels")


def test_large_boundary_scores_shorten_the_scaling_block():
    w = synth.small_random(24, 2, 400, 12, 5, ragged=False)
    check(w, *make_terms(124, w, scale=10.0), label="large projections")


def test_workload_shapes_with_boundary_terms():
    w = synth.make("genomic", T=6000, B=2)
    check(w, *make_terms(125, w), label="genomic shape")
    w = synth.make("speech", B=4, T=600)
    check(w, *make_terms(126, w), label="speech shape")


def test_entropies_of_the_posteriors():
    w = synth.small_random(31, 4, 300, 9, 7, ragged=True)
    w.lengths[3] = 0
    ps, pe, pis, pie = make_terms(131, w)
    emis = dev(nan_pad(w.emis, w.lengths))
    out = sb.semicrf_fwd_bwd_boundary(emis, dev(w.lengths, np.int32), dev(w.trans), dev(w.dur), None,
                                      dev(nan_pad(ps, w.lengths)), dev(nan_pad(pe, w.lengths)), dev(pis), dev(pie))
    h_pos, h_bdy = sb.semicrf_entropies(out["pos_marg"], out["bdy_post"], dev(w.lengths, np.int32))
    torch.cuda.synchronize()
    r = oracle.fwd_bwd(w.emis, w.lengths, w.trans, w.dur, proj_start=ps, proj_end=pe, pi_start=pis, pi_end=pie)
    rp, rb = oracle.entropies(r.pos_marg, r.bdy_post, w.lengths)
    assert np.abs(h_pos.double().cpu().numpy() - rp).max() <= 1e-5 * max(1.0, np.abs(rp).max())
    assert np.abs(h_bdy.double().cpu().numpy() - rb).max() <= 1e-5 * max(1.0, np.abs(rb).max())
    # K = 1: ln L, whatever the parameters
    w1 = synth.small_random(32, 2, 200, 1, 5, ragged=True)
    o1 = sb.semicrf_fwd_bwd_boundary(dev(nan_pad(w1.emis, w1.lengths)), dev(w1.lengths, np.int32), dev(w1.trans),
                                     dev(w1.dur))
    _, hb = sb.semicrf_entropies(o1["pos_marg"], o1["bdy_post"], dev(w1.lengths, np.int32))
    assert np.abs(hb.double().cpu().numpy() - np.log(w1.lengths)).max() <= 1e-5


def test_full_size_genomic_with_boundary_terms_against_stored_oracle_values():
    """The genomic workload at full size with the seeded boundary terms of synth.boundary_terms,
    as `bench.py --boundary-terms` runs it, against oracle values stored by
    tests/golden/make_golden.py (which calls only oracle/): everything accumulated in full,
    per-position outputs at the sampled rows, and properties over all rows."""
    import os
    path = os.path.join(os.path.dirname(__file__), "golden", "full_genomic_boundary.npz")
    if not os.path.exists(path):
        pytest.skip(f"{path} not generated")
    g = np.load(path)
    w = synth.make("genomic")
    ps, pe, pis, pie = synth.boundary_terms(w)
    lengths = dev(w.lengths, np.int32)
    out = sb.semicrf_fwd_bwd_boundary(dev(w.emis), lengths, dev(w.trans), dev(w.dur), None,
                                      dev(ps), dev(pe), dev(pis), dev(pie))
    torch.cuda.synchronize()
    lz = out["logz"].double().cpu().numpy()
    assert (np.abs(lz - g["logz"]) / np.abs(g["logz"])).max() <= 1e-5
    rows = g["rows"]
    rb, ru = torch.from_numpy(rows[:, 0]).to(DEV), torch.from_numpy(rows[:, 1]).to(DEV)
    for name in ("pos_marg", "grad_emis", "grad_proj_start", "grad_proj_end", "bdy_post"):
        err = np.abs(out[name][rb, ru].double().cpu().numpy() - g[name + "_rows"]).max()
        print(f"       {name} max err at {len(rows)} sampled rows {err:.2e}", flush=True)
        assert err <= 1e-4, (name, err)
    for name in ("grad_trans", "grad_dur", "grad_pi_start", "grad_pi_end"):
        err = np.abs(out[name].double().cpu().numpy() - g[name]).max()
        assert err <= 1e-4 * max(1.0, np.abs(g[name]).max()), (name, err)
    from golden_windows import check_windows
    check_windows(g, sb.semicrf_ckpt_interval(w.B, w.T, w.K, w.C), out["pos_marg"], out["grad_emis"])
    # over all rows: one start and one end per segment; boundary mass = segments + sequences
    nseg = out["grad_dur"].double().sum().item()
    assert abs(out["grad_proj_start"].double().sum().item() - nseg) <= 1e-5 * nseg
    assert abs(out["grad_proj_end"].double().sum().item() - nseg) <= 1e-5 * nseg
    assert abs(out["bdy_post"].double().sum().item() - float(g["bdy_post_total"][0])) <= 1e-5 * nseg
    assert abs(out["bdy_post"].double().sum().item() - (nseg + w.B)) <= 1e-5 * nseg
    assert out["bdy_post"].min().item() >= 0.0 and out["bdy_post"].max().item() <= 1.0 + 1e-6
