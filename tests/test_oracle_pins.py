"""Pins of the fp64 CPU oracle against things other than itself (CPU only).

Each test fixes part of ``oracle/`` to something the paper or the mathematics
determines: a printed table, brute-force enumeration of every segmentation, the
textbook linear-chain CRF at K=1, the explicit two-term recurrence at K=2,
closed forms for all-zero potentials, central finite differences, marginal
invariants, the centring = effective-duration-prior identity (Eq. 5), shift
identities and padding independence.
"""
import itertools
import math
import os

import numpy as np
import pytest
from scipy.special import logsumexp

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def rand_case(seed, B, T, K, C, ragged=False, scale=1.0):
    rng = np.random.default_rng(seed)
    emis = scale * rng.standard_normal((B, T, C))
    trans = 0.7 * rng.standard_normal((C, C))
    dur = 0.7 * rng.standard_normal((K, C))
    lengths = rng.integers(1, T + 1, size=B).astype(np.int32) if ragged else np.full(B, T, np.int32)
    return emis, lengths, trans, dur


# --------------------------------------------------------------------------
# P1  baseline arithmetic of Eq. 1 against the printed toy table
# --------------------------------------------------------------------------
def test_baseline_matches_printed_toy_table():
    rows = []
    with open(os.path.join(GOLDEN, "toy_centering_table1.txt")) as fh:
        for line in fh:
            if line.startswith("#") or not line.strip():
                continue
            p = line.split()
            rows.append([float(x) for x in p[1:]])
    rows = np.array(rows)
    act, inact, prev, nu_print, pen_print, cen_print = rows.T
    T, C = 10000, 3
    counts = np.round(prev * T).astype(int)
    assert counts.sum() == T
    labels = np.repeat(np.arange(C), counts)
    np.random.default_rng(0).shuffle(labels)
    emis = np.tile(inact, (T, 1))
    emis[np.arange(T), labels] = act[labels]
    r = oracle.fwd_bwd(emis[None], None, np.zeros((C, C)), np.zeros((2, C)), tables=True)
    S = r.S[0]
    # Eq. 2: S[t] = sum_{u<t} f[u] - t*nu  =>  nu = (cumsum(f)[t-1] - S[t]) / t
    nu = (emis.cumsum(0)[-1] - S[T]) / T
    nu1 = (emis[0] - S[1])
    assert np.allclose(nu, nu1, atol=1e-9)
    assert np.all(np.abs(nu - nu_print) <= 0.005 + 1e-12), nu          # printed to 2 decimals
    assert np.all(np.abs(-100 * nu - pen_print) <= 0.5 + 1e-9)
    assert np.all(np.abs((act - nu) - cen_print) <= 0.005 + 1e-9)
    # S ends at zero when every position is valid (zero-mean walk)
    assert np.allclose(S[T], 0.0, atol=1e-7)
    # no centring: S is the raw prefix sum
    r0 = oracle.fwd_bwd(emis[None], None, np.zeros((C, C)), np.zeros((2, C)), center=False, tables=True)
    assert np.allclose(r0.S[0][1:], emis.cumsum(0), atol=1e-9)


# --------------------------------------------------------------------------
# P2  brute force over every segmentation (independent pure-Python code)
# --------------------------------------------------------------------------
def compositions(n, K):
    if n == 0:
        yield ()
        return
    for first in range(1, min(K, n) + 1):
        for rest in compositions(n - first, K):
            yield (first,) + rest


def brute_force(emis, L, trans, dur, center):
    """Z and expected statistics by explicit enumeration.  The first segment
    pays a transition from a virtual initial label c0 that ranges over all
    labels with weight 1 (alpha_0 = 0 for every label)."""
    T, C = emis.shape
    K = dur.shape[0]
    nu = emis[:L].mean(0) if (center and L > 0) else np.zeros(C)
    fbar = emis - nu
    Z = 0.0
    gTr = np.zeros((C, C))
    gD = np.zeros((K, C))
    pm = np.zeros((T, C))
    gS = np.zeros((T + 1, C))
    for comp in compositions(L, K):
        n = len(comp)
        for c0 in range(C):
            for labs in itertools.product(range(C), repeat=n):
                score = 0.0
                prev = c0
                s = 0
                for k, c in zip(comp, labs):
                    score += trans[prev, c] + dur[k - 1, c] + fbar[s:s + k, c].sum()
                    prev = c
                    s += k
                wgt = math.exp(score)
                Z += wgt
                prev = c0
                s = 0
                for k, c in zip(comp, labs):
                    gTr[prev, c] += wgt
                    gD[k - 1, c] += wgt
                    pm[s:s + k, c] += wgt
                    gS[s + k, c] += wgt
                    gS[s, c] -= wgt
                    prev = c
                    s += k
    return math.log(Z), gTr / Z, gD / Z, pm / Z, gS / Z


@pytest.mark.parametrize("T,K,C,center", [(5, 3, 2, True), (6, 4, 2, False), (4, 2, 3, True),
                                          (7, 7, 2, True), (5, 1, 3, True), (3, 5, 3, False)])
def test_brute_force_enumeration(T, K, C, center):
    emis, _, trans, dur = rand_case(100 + T * 10 + K, 1, T, K, C)
    r = oracle.fwd_bwd(emis, None, trans, dur, center=center, tables=True)
    lz, gTr, gD, pm, gS = brute_force(emis[0], T, trans, dur, center)
    assert abs(r.logz[0] - lz) < 1e-12 * max(1, abs(lz))
    assert np.allclose(r.grad_trans, gTr, atol=1e-10)
    assert np.allclose(r.grad_dur, gD, atol=1e-10)
    assert np.allclose(r.pos_marg[0], pm, atol=1e-10)
    assert np.allclose(r.gS[0], gS, atol=1e-10)
    # gradient w.r.t. raw emissions through the centring Jacobian
    gE = pm - (pm.mean(0) if center else 0.0)
    assert np.allclose(r.grad_emis[0], gE, atol=1e-10)


def test_brute_force_ragged_and_weighted():
    T, K, C = 6, 3, 2
    emis, _, trans, dur = rand_case(7, 3, T, K, C)
    lengths = np.array([6, 3, 1], np.int32)
    w = np.array([0.5, -2.0, 3.0])
    r = oracle.fwd_bwd(emis, lengths, trans, dur, grad_logz=w)
    gTr = np.zeros((C, C))
    gD = np.zeros((K, C))
    for b in range(3):
        L = int(lengths[b])
        lz, tr_b, d_b, pm, _ = brute_force(emis[b], L, trans, dur, True)
        assert abs(r.logz[b] - lz) < 1e-12
        assert np.allclose(r.pos_marg[b], pm, atol=1e-10)
        assert np.all(r.pos_marg[b, L:] == 0) and np.all(r.grad_emis[b, L:] == 0)
        gE = w[b] * (pm[:L] - pm[:L].mean(0))
        assert np.allclose(r.grad_emis[b, :L], gE, atol=1e-10)
        gTr += w[b] * tr_b
        gD += w[b] * d_b
    assert np.allclose(r.grad_trans, gTr, atol=1e-10)
    assert np.allclose(r.grad_dur, gD, atol=1e-10)


# --------------------------------------------------------------------------
# P3  K=1 is the textbook linear-chain CRF; K=2 is the explicit recurrence
# --------------------------------------------------------------------------
def test_k1_is_linear_chain_crf():
    T, C = 300, 5
    emis, _, trans, dur = rand_case(11, 2, T, 1, C)
    r = oracle.fwd_bwd(emis, None, trans, dur, center=True)
    for b in range(2):
        fbar = emis[b] - emis[b].mean(0)
        a = np.ones(C)
        log_scale = 0.0
        E = np.exp(trans)
        for t in range(T):
            a = (a @ E) * np.exp(fbar[t] + dur[0])
            s = a.sum()
            a /= s
            log_scale += math.log(s)
        assert abs(r.logz[b] - log_scale) < 1e-9
    # every boundary is certain at K=1: expected number of segments = T per sequence
    assert abs(r.grad_dur.sum() - 2 * T) < 1e-8


def test_k2_explicit_recurrence():
    T, C = 120, 4
    emis, _, trans, dur = rand_case(12, 1, T, 2, C)
    lz = oracle.logz(emis, None, trans, dur, center=False)[0]
    S = np.vstack([np.zeros(C), emis[0].cumsum(0)])
    a1 = np.zeros(C)               # alpha[t-1]
    a2 = np.full(C, -np.inf)       # alpha[t-2]
    for t in range(1, T + 1):
        s1 = S[t] - S[t - 1] + dur[0] + logsumexp(a1[:, None] + trans, axis=0)
        if t >= 2:
            s2 = S[t] - S[t - 2] + dur[1] + logsumexp(a2[:, None] + trans, axis=0)
            new = np.logaddexp(s1, s2)
        else:
            new = s1
        a2, a1 = a1, new
    assert abs(lz - logsumexp(a1)) < 1e-9


# --------------------------------------------------------------------------
# P4  closed forms for all-zero potentials
# --------------------------------------------------------------------------
@pytest.mark.parametrize("T,C", [(1, 3), (7, 2), (12, 5)])
def test_closed_forms_zero_potentials(T, C):
    z = np.zeros((1, T, C))
    # K >= T: A_t = C * sum_{s<t} A_s, A_0 = C  =>  logZ = 2 ln C + (T-1) ln(C+1)
    lz = oracle.logz(z, None, np.zeros((C, C)), np.zeros((T + 3, C)))[0]
    assert abs(lz - (2 * math.log(C) + (T - 1) * math.log(C + 1))) < 1e-10
    # K = 1: A_t = C * A_{t-1}  =>  logZ = (T+1) ln C
    lz1 = oracle.logz(z, None, np.zeros((C, C)), np.zeros((1, C)))[0]
    assert abs(lz1 - (T + 1) * math.log(C)) < 1e-10
    # general K by the integer recurrence
    K = 3
    A = [C]
    for t in range(1, T + 1):
        A.append(C * sum(A[max(0, t - K):t]))
    lzk = oracle.logz(z, None, np.zeros((C, C)), np.zeros((K, C)))[0]
    assert abs(lzk - math.log(A[T])) < 1e-10
    # empty sequence: logZ = ln C (alpha_0 = 0 for all labels)
    lz0 = oracle.logz(z, np.array([0], np.int32), np.zeros((C, C)), np.zeros((K, C)))[0]
    assert abs(lz0 - math.log(C)) < 1e-12


# --------------------------------------------------------------------------
# P5  central finite differences on every input element
# --------------------------------------------------------------------------
def test_finite_differences_all_inputs():
    B, T, K, C = 2, 9, 4, 3
    emis, _, trans, dur = rand_case(21, B, T, K, C)
    lengths = np.array([9, 6], np.int32)
    w = np.array([1.3, -0.7])
    r = oracle.fwd_bwd(emis, lengths, trans, dur, grad_logz=w, center=True)

    def loss(e, tr, d):
        return float((w * oracle.logz(e, lengths, tr, d, center=True)).sum())

    eps = 1e-6
    g = np.zeros_like(emis)
    for idx in np.ndindex(*emis.shape):
        ep, em = emis.copy(), emis.copy()
        ep[idx] += eps
        em[idx] -= eps
        g[idx] = (loss(ep, trans, dur) - loss(em, trans, dur)) / (2 * eps)
    assert np.allclose(r.grad_emis, g, atol=2e-8)
    g = np.zeros_like(trans)
    for idx in np.ndindex(*trans.shape):
        p, m = trans.copy(), trans.copy()
        p[idx] += eps
        m[idx] -= eps
        g[idx] = (loss(emis, p, dur) - loss(emis, m, dur)) / (2 * eps)
    assert np.allclose(r.grad_trans, g, atol=2e-8)
    g = np.zeros_like(dur)
    for idx in np.ndindex(*dur.shape):
        p, m = dur.copy(), dur.copy()
        p[idx] += eps
        m[idx] -= eps
        g[idx] = (loss(emis, trans, p) - loss(emis, trans, m)) / (2 * eps)
    assert np.allclose(r.grad_dur, g, atol=2e-8)


def test_finite_differences_paper_protocol_sizes():
    """The paper's own check: B=1, T=100, C=16, K=25 (sampled elements here)."""
    B, T, K, C = 1, 100, 25, 16
    emis, _, trans, dur = rand_case(22, B, T, K, C)
    r = oracle.fwd_bwd(emis, None, trans, dur, center=False)
    rng = np.random.default_rng(0)
    eps = 1e-5
    for _ in range(6):
        i, j = rng.integers(0, C, 2)
        p, m = trans.copy(), trans.copy()
        p[i, j] += eps
        m[i, j] -= eps
        fd = (oracle.logz(emis, None, p, dur, center=False)[0] - oracle.logz(emis, None, m, dur, center=False)[0]) / (2 * eps)
        assert abs(fd - r.grad_trans[i, j]) < 1e-6
        k, c = rng.integers(0, K), rng.integers(0, C)
        p, m = dur.copy(), dur.copy()
        p[k, c] += eps
        m[k, c] -= eps
        fd = (oracle.logz(emis, None, trans, p, center=False)[0] - oracle.logz(emis, None, trans, m, center=False)[0]) / (2 * eps)
        assert abs(fd - r.grad_dur[k, c]) < 1e-6
        u, c = rng.integers(0, T), rng.integers(0, C)
        p, m = emis.copy(), emis.copy()
        p[0, u, c] += eps
        m[0, u, c] -= eps
        fd = (oracle.logz(p, None, trans, dur, center=False)[0] - oracle.logz(m, None, trans, dur, center=False)[0]) / (2 * eps)
        assert abs(fd - r.pos_marg[0, u, c]) < 1e-6


# --------------------------------------------------------------------------
# P6  invariants of the marginals
# --------------------------------------------------------------------------
def test_marginal_invariants():
    B, T, K, C = 3, 200, 12, 6
    emis, lengths, trans, dur = rand_case(31, B, T, K, C, ragged=True)
    lengths[0] = T
    r = oracle.fwd_bwd(emis, lengths, trans, dur, tables=True)
    for b in range(B):
        L = int(lengths[b])
        pm = r.pos_marg[b]
        assert np.all(pm >= -1e-12) and np.all(pm <= 1 + 1e-12)
        assert np.allclose(pm[:L].sum(1), 1.0, atol=1e-10)
        assert np.all(pm[L:] == 0)
        assert abs(pm.sum() - L) < 1e-8
        gD, gTr = r.grad_dur_b[b], r.grad_trans_b[b]
        ks = np.arange(1, K + 1)[:, None]
        assert abs((ks * gD).sum() - L) < 1e-8                     # durations tile the sequence
        nseg = gD.sum()
        assert abs(gTr.sum() - nseg) < 1e-8                         # one transition per segment
        assert math.ceil(L / K) - 1e-9 <= nseg <= L + 1e-9
        gS = r.gS[b]
        assert np.allclose(gS[1:L].sum(1), 0.0, atol=1e-10)
        assert abs(gS[0].sum() + 1) < 1e-10 and abs(gS[L].sum() - 1) < 1e-10
        bdy = np.exp(r.alpha[b, :L + 1] + r.beta[b, :L + 1] - r.logz[b]).sum(1)
        assert np.all(bdy[1:] <= 1 + 1e-10) and abs(bdy[L] - 1) < 1e-10
        assert abs(bdy[1:L + 1].sum() - nseg) < 1e-8
        # beta at the origin carries the partition function (alpha_0 = 0)
        assert abs(logsumexp(r.beta[b, 0]) - r.logz[b]) < 1e-9
        # centred gradient sums to zero over valid positions for each label
        assert np.allclose(r.grad_emis[b, :L].sum(0), 0.0, atol=1e-9)


# --------------------------------------------------------------------------
# P7  centring == per-sequence effective duration prior (Eq. 5)
# --------------------------------------------------------------------------
def test_centering_equals_effective_duration_prior():
    B, T, K, C = 1, 40, 7, 4
    emis, _, trans, dur = rand_case(41, B, T, K, C)
    emis += np.array([2.0, -1.0, 0.3, 0.0])     # non-zero per-label means
    L = 33
    lengths = np.array([L], np.int32)
    nu = emis[0, :L].mean(0)
    dur_eff = dur - nu[None, :] * np.arange(1, K + 1)[:, None]
    a = oracle.fwd_bwd(emis, lengths, trans, dur, center=True)
    b = oracle.fwd_bwd(emis, lengths, trans, dur_eff, center=False)
    assert abs(a.logz[0] - b.logz[0]) < 1e-9
    assert np.allclose(a.pos_marg, b.pos_marg, atol=1e-10)
    assert np.allclose(a.grad_trans, b.grad_trans, atol=1e-10)
    assert np.allclose(a.grad_dur, b.grad_dur, atol=1e-10)
    # and centring is NOT path-invariant: it changes logZ
    c = oracle.fwd_bwd(emis, lengths, trans, dur, center=False)
    assert abs(a.logz[0] - c.logz[0]) > 1e-3


# --------------------------------------------------------------------------
# P8  shift identities
# --------------------------------------------------------------------------
def test_shift_identities():
    B, T, K, C = 1, 30, 5, 3
    emis, _, trans, dur = rand_case(51, B, T, K, C)
    shift = np.random.default_rng(3).standard_normal(T)
    e2 = emis + shift[None, :, None]
    # without centring a per-position scalar is path-invariant: logZ moves by its sum
    l0 = oracle.logz(emis, None, trans, dur, center=False)[0]
    l1 = oracle.logz(e2, None, trans, dur, center=False)[0]
    assert abs((l1 - l0) - shift.sum()) < 1e-9
    # with centring a constant per-label offset is removed exactly
    e3 = emis + np.array([5.0, -3.0, 0.5])[None, None, :]
    l2 = oracle.logz(emis, None, trans, dur, center=True)[0]
    l3 = oracle.logz(e3, None, trans, dur, center=True)[0]
    assert abs(l2 - l3) < 1e-9
    # marginals are untouched by the path-invariant shift
    a = oracle.fwd_bwd(emis, None, trans, dur, center=False)
    b = oracle.fwd_bwd(e2, None, trans, dur, center=False)
    assert np.allclose(a.pos_marg, b.pos_marg, atol=1e-10)


# --------------------------------------------------------------------------
# P10  padding independence
# --------------------------------------------------------------------------
def test_padding_independence():
    T, K, C = 25, 6, 3
    emis, _, trans, dur = rand_case(61, 1, T, K, C)
    L = 17
    alone = oracle.fwd_bwd(emis[:, :L], None, trans, dur)
    padded = emis.copy()
    padded[0, L:] = np.nan                       # must never be read
    other = np.random.default_rng(9).standard_normal((1, T, C))
    batch = np.concatenate([other, padded], 0)
    r = oracle.fwd_bwd(batch, np.array([T, L], np.int32), trans, dur, grad_logz=np.array([0.0, 1.0]))
    assert r.logz[1] == alone.logz[0]
    assert np.array_equal(r.pos_marg[1, :L], alone.pos_marg[0])
    assert np.all(r.pos_marg[1, L:] == 0)
    assert np.allclose(r.grad_trans, alone.grad_trans, atol=1e-12)
    assert np.allclose(r.grad_dur, alone.grad_dur, atol=1e-12)


# --------------------------------------------------------------------------
# transposition / index sensitivity: the pins above must be able to see a
# swapped transition matrix or a shifted duration row
# --------------------------------------------------------------------------
def test_pins_can_see_transposed_or_shifted_operands():
    T, K, C = 5, 3, 2
    emis, _, trans, dur = rand_case(150 + 3, 1, T, K, C)
    lz, *_ = brute_force(emis[0], T, trans, dur, True)
    assert abs(oracle.logz(emis, None, trans.T.copy(), dur)[0] - lz) > 1e-4
    assert abs(oracle.logz(emis, None, trans, np.roll(dur, 1, axis=0))[0] - lz) > 1e-4


def test_forward_only_entry_matches_full_entry():
    emis, lengths, trans, dur = rand_case(71, 3, 50, 9, 4, ragged=True)
    a = oracle.logz(emis, lengths, trans, dur)
    b = oracle.fwd_bwd(emis, lengths, trans, dur).logz
    assert np.array_equal(a, b)


# --------------------------------------------------------------------------
# P11  boundary terms of Eq. 4: start/end projections and scalar sequence boundaries
# --------------------------------------------------------------------------
def brute_force_boundary(emis, L, trans, dur, ps, pe, pis, pie, center):
    """Enumeration with the two boundary terms: a segment [s, s+k) with label c also pays
    ps[s,c] + pe[s+k-1,c]; the scalar boundaries are paid by the segment that starts at
    token 0 / ends at token L-1.  Returns logZ and the expected counts that are the gradients
    with respect to ps, pe, pis, pie, and the boundary posterior."""
    T, C = emis.shape
    K = dur.shape[0]
    nu = emis[:L].mean(0) if (center and L > 0) else np.zeros(C)
    fbar = emis - nu
    Z = 0.0
    gPs = np.zeros((T, C))
    gPe = np.zeros((T, C))
    gPis = np.zeros(C)
    gPie = np.zeros(C)
    pm = np.zeros((T, C))
    bdy = np.zeros(T + 1)
    for comp in compositions(L, K):
        n = len(comp)
        for c0 in range(C):
            for labs in itertools.product(range(C), repeat=n):
                score, prev, s = 0.0, c0, 0
                for k, c in zip(comp, labs):
                    score += trans[prev, c] + dur[k - 1, c] + fbar[s:s + k, c].sum() + ps[s, c] + pe[s + k - 1, c]
                    if s == 0:
                        score += pis[c]
                    if s + k == L:
                        score += pie[c]
                    prev, s = c, s + k
                wgt = math.exp(score)
                Z += wgt
                s = 0
                bdy[0] += wgt
                for k, c in zip(comp, labs):
                    gPs[s, c] += wgt
                    gPe[s + k - 1, c] += wgt
                    pm[s:s + k, c] += wgt
                    if s == 0:
                        gPis[c] += wgt
                    if s + k == L:
                        gPie[c] += wgt
                    s += k
                    bdy[s] += wgt
    return math.log(Z), gPs / Z, gPe / Z, gPis / Z, gPie / Z, pm / Z, bdy / Z


@pytest.mark.parametrize("T,K,C,center", [(5, 3, 2, True), (6, 4, 2, False), (4, 2, 3, True), (5, 1, 3, True)])
def test_brute_force_with_boundary_terms(T, K, C, center):
    rng = np.random.default_rng(500 + T * 10 + K)
    emis, _, trans, dur = rand_case(300 + T * 10 + K, 1, T, K, C)
    ps, pe = rng.standard_normal((1, T, C)), rng.standard_normal((1, T, C))
    pis, pie = rng.standard_normal(C), rng.standard_normal(C)
    r = oracle.fwd_bwd(emis, None, trans, dur, center=center, proj_start=ps, proj_end=pe, pi_start=pis, pi_end=pie)
    lz, gPs, gPe, gPis, gPie, pm, bdy = brute_force_boundary(emis[0], T, trans, dur, ps[0], pe[0], pis, pie, center)
    assert abs(r.logz[0] - lz) < 1e-12 * max(1, abs(lz))
    assert np.allclose(r.grad_proj_start[0], gPs, atol=1e-10)
    assert np.allclose(r.grad_proj_end[0], gPe, atol=1e-10)
    assert np.allclose(r.grad_pi_start, gPis, atol=1e-10)
    assert np.allclose(r.grad_pi_end, gPie, atol=1e-10)
    assert np.allclose(r.pos_marg[0], pm, atol=1e-10)
    assert np.allclose(r.bdy_post[0], bdy, atol=1e-10)
    # with all boundary terms zero the enumeration of P2 is recovered
    z = np.zeros((1, T, C))
    r0 = oracle.fwd_bwd(emis, None, trans, dur, center=center, proj_start=z, proj_end=z)
    r1 = oracle.fwd_bwd(emis, None, trans, dur, center=center)
    assert np.array_equal(r0.logz, r1.logz) and np.array_equal(r0.grad_dur, r1.grad_dur)


def test_boundary_terms_ragged_weighted_and_scalar_composition():
    """Ragged batch with upstream weights.  Scalar boundaries are the projections' rows of token 0
    and token L_b - 1 (composition rule of the boundary appendix): folding them into the
    projections by hand must give the same logZ, and their gradients are those rows summed."""
    rng = np.random.default_rng(77)
    B, T, K, C = 3, 9, 4, 3
    emis, _, trans, dur = rand_case(78, B, T, K, C)
    lengths = np.array([9, 6, 1], dtype=np.int32)
    w = np.array([1.0, -0.7, 2.5])
    ps, pe = rng.standard_normal((B, T, C)), rng.standard_normal((B, T, C))
    pis, pie = rng.standard_normal(C), rng.standard_normal(C)
    r = oracle.fwd_bwd(emis, lengths, trans, dur, grad_logz=w, proj_start=ps, proj_end=pe, pi_start=pis, pi_end=pie)
    ps2, pe2 = ps.copy(), pe.copy()
    for b in range(B):
        ps2[b, 0] += pis
        pe2[b, lengths[b] - 1] += pie
    r2 = oracle.fwd_bwd(emis, lengths, trans, dur, grad_logz=w, proj_start=ps2, proj_end=pe2)
    assert np.allclose(r.logz, r2.logz, rtol=0, atol=1e-12)
    assert np.allclose(r.grad_proj_start, r2.grad_proj_start, atol=1e-12)
    assert np.allclose(r.grad_pi_start, r.grad_proj_start[:, 0].sum(0), atol=1e-12)
    assert np.allclose(r.grad_pi_end, sum(r.grad_proj_end[b, lengths[b] - 1] for b in range(B)), atol=1e-12)
    # per sequence against the enumeration (weights scale the gradients)
    for b in range(B):
        L = int(lengths[b])
        lz, gPs, gPe, gPis, gPie, pm, bdy = brute_force_boundary(emis[b], L, trans, dur, ps[b], pe[b], pis, pie, True)
        assert abs(r.logz[b] - lz) < 1e-12 * max(1, abs(lz))
        assert np.allclose(r.grad_proj_start[b], w[b] * gPs, atol=1e-10)
        assert np.allclose(r.grad_proj_end[b], w[b] * gPe, atol=1e-10)
        assert np.allclose(r.bdy_post[b], bdy, atol=1e-10)
        assert np.all(r.grad_proj_start[b, L:] == 0) and np.all(r.grad_proj_end[b, L:] == 0)
    # every segment has one start and one end: both gradients sum to the expected number of segments
    for b in range(B):
        nseg = r.grad_dur_b[b].sum()
        assert abs(r.grad_proj_start[b].sum() - nseg) < 1e-10 and abs(r.grad_proj_end[b].sum() - nseg) < 1e-10


def test_k1_with_scalar_boundaries_is_the_chain_crf_with_start_and_end_scores():
    """K = 1 with scalar boundaries is the textbook linear-chain CRF with start and end
    scores: a_1 = (1 E) * exp(f_0 + dur + pi_start), ..., Z = sum_c a_T(c) exp(pi_end[c])
    (the transition from the free initial label is kept, as in the K=1 pin above)."""
    T, C = 200, 4
    rng = np.random.default_rng(13)
    emis, _, trans, dur = rand_case(14, 1, T, 1, C)
    pis, pie = rng.standard_normal(C), rng.standard_normal(C)
    lz = oracle.logz(emis, None, trans, dur, center=True, pi_start=pis, pi_end=pie)[0]
    fbar = emis[0] - emis[0].mean(0)
    a = np.ones(C)
    log_scale = 0.0
    E = np.exp(trans)
    for t in range(T):
        a = (a @ E) * np.exp(fbar[t] + dur[0] + (pis if t == 0 else 0.0) + (pie if t == T - 1 else 0.0))
        s = a.sum()
        a /= s
        log_scale += math.log(s)
    assert abs(lz - log_scale) < 1e-9


def test_finite_differences_boundary_terms():
    rng = np.random.default_rng(15)
    B, T, K, C = 2, 7, 3, 3
    emis, _, trans, dur = rand_case(16, B, T, K, C)
    lengths = np.array([7, 5], dtype=np.int32)
    w = np.array([0.8, -1.3])
    ps, pe = 0.5 * rng.standard_normal((B, T, C)), 0.5 * rng.standard_normal((B, T, C))
    pis, pie = rng.standard_normal(C), rng.standard_normal(C)
    r = oracle.fwd_bwd(emis, lengths, trans, dur, grad_logz=w, proj_start=ps, proj_end=pe, pi_start=pis, pi_end=pie)
    loss = lambda **kw: float(w @ oracle.logz(emis, lengths, trans, dur, **{**dict(proj_start=ps, proj_end=pe,
                                                                            pi_start=pis, pi_end=pie), **kw}))
    eps = 1e-6
    for name, arr, grad in (("proj_start", ps, r.grad_proj_start), ("proj_end", pe, r.grad_proj_end),
                            ("pi_start", pis, r.grad_pi_start), ("pi_end", pie, r.grad_pi_end)):
        for idx in np.ndindex(arr.shape):
            hi, lo = arr.copy(), arr.copy()
            hi[idx] += eps
            lo[idx] -= eps
            fd = (loss(**{name: hi}) - loss(**{name: lo})) / (2 * eps)
            assert abs(fd - grad[idx]) < 2e-7, (name, idx, fd, grad[idx])


def test_boundary_posterior_invariants():
    emis, lengths, trans, dur = rand_case(17, 3, 40, 6, 4, ragged=True)
    r = oracle.fwd_bwd(emis, lengths, trans, dur, boundary=True)
    for b in range(3):
        L = int(lengths[b])
        p = r.bdy_post[b]
        assert abs(p[0] - 1) < 1e-10 and abs(p[L] - 1) < 1e-10 and np.all(p[L + 1:] == 0)
        assert np.all(p[:L + 1] > 0) and np.all(p[:L + 1] <= 1 + 1e-12)
        # expected number of boundaries = expected number of segments + 1
        assert abs(p.sum() - (r.grad_dur_b[b].sum() + 1)) < 1e-9


def test_entropies_closed_forms():
    """K = 1: every token starts a segment, so the boundary entropy is ln L whatever the
    parameters (stated in the boundary-entropy paragraph).  All-zero potentials: the label
    posterior is uniform, so the position entropy is ln C; with K >= 1 and zero potentials the
    boundary posterior is the same at every interior position by symmetry only for K = 1, so
    the general case is checked against the definition written out on a tiny example."""
    emis, lengths, trans, dur = rand_case(18, 3, 30, 1, 4, ragged=True)
    r = oracle.fwd_bwd(emis, lengths, trans, dur, boundary=True)
    h_pos, h_bdy = oracle.entropies(r.pos_marg, r.bdy_post, lengths)
    assert np.allclose(h_bdy, np.log(lengths), atol=1e-12)
    z = oracle.fwd_bwd(np.zeros((1, 12, 5)), None, np.zeros((5, 5)), np.zeros((3, 5)), boundary=True)
    h_pos, h_bdy = oracle.entropies(z.pos_marg, z.bdy_post, None)
    assert abs(h_pos[0] - math.log(5)) < 1e-12
    # definition by hand on a 3-token example
    pm = np.array([[[0.5, 0.5], [1.0, 0.0], [0.25, 0.75]]])
    bd = np.array([[1.0, 0.5, 0.5, 1.0]])
    h_pos, h_bdy = oracle.entropies(pm, bd, None)
    hp = (math.log(2) + 0.0 - 0.25 * math.log(0.25) - 0.75 * math.log(0.75)) / 3
    ph = np.array([0.5, 0.25, 0.25])
    assert abs(h_pos[0] - hp) < 1e-12 and abs(h_bdy[0] + (ph * np.log(ph)).sum()) < 1e-12


# --------------------------------------------------------------------------
# P12  Viterbi decode (max semiring)
# --------------------------------------------------------------------------
def brute_force_best(emis, L, trans, dur, ps, pe, pis, pie, center):
    """Maximum over every segmentation and labelling, by enumeration (scores as in P11)."""
    T, C = emis.shape
    K = dur.shape[0]
    nu = emis[:L].mean(0) if (center and L > 0) else np.zeros(C)
    fbar = emis - nu
    best = -np.inf
    for comp in compositions(L, K):
        for c0 in range(C):
            for labs in itertools.product(range(C), repeat=len(comp)):
                score, prev, s = 0.0, c0, 0
                for k, c in zip(comp, labs):
                    score += trans[prev, c] + dur[k - 1, c] + fbar[s:s + k, c].sum() + ps[s, c] + pe[s + k - 1, c]
                    if s == 0:
                        score += pis[c]
                    if s + k == L:
                        score += pie[c]
                    prev, s = c, s + k
                best = max(best, score)
    return best


@pytest.mark.parametrize("T,K,C,center,bt", [(5, 3, 2, True, True), (6, 4, 2, False, False), (4, 2, 3, True, True),
                                             (7, 7, 2, True, False), (5, 1, 3, True, True)])
def test_viterbi_against_enumeration(T, K, C, center, bt):
    rng = np.random.default_rng(900 + T * 10 + K)
    emis, _, trans, dur = rand_case(700 + T * 10 + K, 1, T, K, C)
    z = np.zeros((1, T, C))
    ps, pe = (rng.standard_normal((1, T, C)), rng.standard_normal((1, T, C))) if bt else (z, z)
    pis, pie = (rng.standard_normal(C), rng.standard_normal(C)) if bt else (np.zeros(C), np.zeros(C))
    score, labels, starts, nseg = oracle.viterbi(emis, None, trans, dur, center=center, proj_start=ps, proj_end=pe,
                                                 pi_start=pis, pi_end=pie)
    best = brute_force_best(emis[0], T, trans, dur, ps[0], pe[0], pis, pie, center)
    assert abs(score[0] - best) < 1e-12 * max(1, abs(best))
    # the decoded path is a valid segmentation and achieves the reported score
    got = oracle.path_score(emis[0], T, trans, dur, labels[0], starts[0], center=center, proj_start=ps[0],
                            proj_end=pe[0], pi_start=pis, pi_end=pie)
    assert abs(got - score[0]) < 1e-10
    assert nseg[0] == starts[0].sum()


def test_viterbi_k1_is_the_textbook_chain_decoder():
    T, C = 150, 5
    emis, _, trans, dur = rand_case(19, 1, T, 1, C)
    score, labels, starts, nseg = oracle.viterbi(emis, None, trans, dur, center=True)
    fbar = emis[0] - emis[0].mean(0)
    v = np.zeros(C)
    back = np.zeros((T, C), dtype=int)
    for t in range(T):
        cand = v[:, None] + trans                      # [source, destination]
        back[t] = cand.argmax(0)
        v = cand.max(0) + fbar[t] + dur[0]
    assert abs(score[0] - v.max()) < 1e-9
    path = np.zeros(T, dtype=int)
    c = int(v.argmax())
    for t in range(T - 1, -1, -1):
        path[t] = c
        c = back[t, c]
    assert np.array_equal(labels[0], path) and np.all(starts[0] == 1) and nseg[0] == T


def test_viterbi_ragged_bounds_and_zero_temperature_limit():
    emis, lengths, trans, dur = rand_case(20, 3, 25, 5, 3, ragged=True)
    lengths[2] = 0
    score, labels, starts, nseg = oracle.viterbi(emis, lengths, trans, dur)
    lz = oracle.logz(emis, lengths, trans, dur)
    for b in range(3):
        L = int(lengths[b])
        assert np.all(labels[b, L:] == -1) and np.all(starts[b, L:] == 0)
        if L == 0:
            assert score[b] == 0.0 and nseg[b] == 0
            continue
        assert score[b] <= lz[b] + 1e-12                               # one path among those summed
        got = oracle.path_score(emis[b], L, trans, dur, labels[b], starts[b])
        assert abs(got - score[b]) < 1e-10
    # potentials scaled by a large factor: logZ / factor tends to the best score (centring is linear in emis)
    fac = 200.0
    lz_hot = oracle.logz(fac * emis, lengths, fac * trans, fac * dur)
    for b in range(2):
        assert abs(lz_hot[b] / fac - score[b]) < 0.2


# --------------------------------------------------------------------------
# P13  duration-dependent transitions trans[k-1,c',c] (the transition gradient with a
#      duration index of the gradient-workspace section)
# --------------------------------------------------------------------------
def brute_force_durtrans(emis, L, trans3, dur, center):
    """Explicit enumeration with one transition matrix per duration."""
    T, C = emis.shape
    K = dur.shape[0]
    nu = emis[:L].mean(0) if (center and L > 0) else np.zeros(C)
    fbar = emis - nu
    Z = 0.0
    gTr = np.zeros((K, C, C))
    gD = np.zeros((K, C))
    pm = np.zeros((T, C))
    for comp in compositions(L, K):
        n = len(comp)
        for c0 in range(C):
            for labs in itertools.product(range(C), repeat=n):
                score, prev, s = 0.0, c0, 0
                for k, c in zip(comp, labs):
                    score += trans3[k - 1, prev, c] + dur[k - 1, c] + fbar[s:s + k, c].sum()
                    prev = c
                    s += k
                wgt = math.exp(score)
                Z += wgt
                prev, s = c0, 0
                for k, c in zip(comp, labs):
                    gTr[k - 1, prev, c] += wgt
                    gD[k - 1, c] += wgt
                    pm[s:s + k, c] += wgt
                    prev = c
                    s += k
    return math.log(Z), gTr / Z, gD / Z, pm / Z


def rand_trans3(seed, K, C):
    return 0.7 * np.random.default_rng(seed).standard_normal((K, C, C))


@pytest.mark.parametrize("T,K,C,center", [(5, 3, 2, True), (6, 4, 2, False), (4, 2, 3, True),
                                          (6, 6, 2, True), (5, 1, 3, True), (3, 5, 2, False)])
def test_durtrans_brute_force_enumeration(T, K, C, center):
    emis, _, _, dur = rand_case(300 + T * 10 + K, 1, T, K, C)
    trans3 = rand_trans3(301 + T, K, C)
    r = oracle.fwd_bwd_durtrans(emis, None, trans3, dur, center=center)
    lz, gTr, gD, pm = brute_force_durtrans(emis[0], T, trans3, dur, center)
    assert abs(r.logz[0] - lz) < 1e-12 * max(1, abs(lz))
    assert np.allclose(r.grad_trans, gTr, atol=1e-10)
    assert np.allclose(r.grad_dur, gD, atol=1e-10)
    assert np.allclose(r.pos_marg[0], pm, atol=1e-10)
    gE = pm - (pm.mean(0) if center else 0.0)
    assert np.allclose(r.grad_emis[0], gE, atol=1e-10)
    assert abs(oracle.logz_durtrans(emis, None, trans3, dur, center=center)[0] - lz) < 1e-12 * max(1, abs(lz))


def test_durtrans_ragged_and_weighted():
    T, K, C = 6, 3, 2
    emis, _, _, dur = rand_case(17, 3, T, K, C)
    trans3 = rand_trans3(18, K, C)
    lengths = np.array([6, 3, 1], np.int32)
    w = np.array([0.5, -2.0, 3.0])
    r = oracle.fwd_bwd_durtrans(emis, lengths, trans3, dur, grad_logz=w)
    gTr = np.zeros((K, C, C))
    gD = np.zeros((K, C))
    for b in range(3):
        L = int(lengths[b])
        lz, tr_b, d_b, pm = brute_force_durtrans(emis[b], L, trans3, dur, True)
        assert abs(r.logz[b] - lz) < 1e-12
        assert np.allclose(r.pos_marg[b], pm, atol=1e-10)
        assert np.all(r.pos_marg[b, L:] == 0) and np.all(r.grad_emis[b, L:] == 0)
        assert np.allclose(r.grad_emis[b, :L], w[b] * (pm[:L] - pm[:L].mean(0)), atol=1e-10)
        gTr += w[b] * tr_b
        gD += w[b] * d_b
    assert np.allclose(r.grad_trans, gTr, atol=1e-10)
    assert np.allclose(r.grad_dur, gD, atol=1e-10)


def test_durtrans_reduces_to_one_shared_matrix_and_absorbs_the_duration_bias():
    B, T, K, C = 3, 11, 4, 3
    emis, lengths, trans, dur = rand_case(41, B, T, K, C, ragged=True)
    w = np.array([1.0, 0.3, -1.2])
    ref = oracle.fwd_bwd(emis, lengths, trans, dur, grad_logz=w)
    # the same matrix for every duration is the potential of Eq. 4
    r = oracle.fwd_bwd_durtrans(emis, lengths, np.broadcast_to(trans, (K, C, C)).copy(), dur, grad_logz=w)
    assert np.allclose(r.logz, ref.logz, rtol=1e-13)
    assert np.allclose(r.grad_trans.sum(0), ref.grad_trans, atol=1e-11)
    assert np.allclose(r.grad_dur, ref.grad_dur, atol=1e-11)
    assert np.allclose(r.pos_marg, ref.pos_marg, atol=1e-12)
    assert np.allclose(r.grad_emis, ref.grad_emis, atol=1e-12)
    # dur[k,c] and trans[k,c',c] enter the potential together: moving the bias into the
    # transitions changes nothing, and the bias gradient is the transition gradient summed
    # over the source label
    trans3 = rand_trans3(42, K, C)
    a = oracle.fwd_bwd_durtrans(emis, lengths, trans3, dur, grad_logz=w)
    b = oracle.fwd_bwd_durtrans(emis, lengths, trans3 + dur[:, None, :], np.zeros_like(dur), grad_logz=w)
    assert np.allclose(a.logz, b.logz, rtol=1e-13)
    assert np.allclose(a.grad_trans, b.grad_trans, atol=1e-11)
    assert np.allclose(a.grad_dur, a.grad_trans.sum(1), atol=1e-11)
    # every segment has exactly one (duration, source, destination):
    # with unit weights the transition gradient sums to the expected number of segments,
    # which is what the duration gradient sums to as well
    u = oracle.fwd_bwd_durtrans(emis, lengths, trans3, dur)
    assert abs(u.grad_trans.sum() - u.grad_dur.sum()) < 1e-10
    durw = (u.grad_dur * np.arange(1, K + 1)[:, None]).sum()
    assert abs(durw - lengths.sum()) < 1e-9          # durations tile the sequences


def test_durtrans_finite_differences():
    B, T, K, C = 2, 8, 3, 3
    emis, _, _, dur = rand_case(51, B, T, K, C)
    trans3 = rand_trans3(52, K, C)
    lengths = np.array([8, 5], np.int32)
    w = np.array([1.3, -0.7])
    r = oracle.fwd_bwd_durtrans(emis, lengths, trans3, dur, grad_logz=w)

    def loss(e, tr, d):
        return float((w * oracle.logz_durtrans(e, lengths, tr, d)).sum())

    eps = 1e-6
    for arr, grad, which in ((emis, r.grad_emis, 0), (trans3, r.grad_trans, 1), (dur, r.grad_dur, 2)):
        g = np.zeros_like(arr)
        for idx in np.ndindex(*arr.shape):
            p, m = arr.copy(), arr.copy()
            p[idx] += eps
            m[idx] -= eps
            args_p = [emis, trans3, dur]
            args_m = [emis, trans3, dur]
            args_p[which], args_m[which] = p, m
            g[idx] = (loss(*args_p) - loss(*args_m)) / (2 * eps)
        assert np.allclose(grad, g, atol=2e-8), which


def test_durtrans_pins_can_see_a_transposed_matrix_or_a_shifted_duration_index():
    T, K, C = 5, 3, 2
    emis, _, _, dur = rand_case(61, 1, T, K, C)
    trans3 = rand_trans3(62, K, C)
    lz, *_ = brute_force_durtrans(emis[0], T, trans3, dur, True)
    wrong_t = oracle.logz_durtrans(emis, None, trans3.transpose(0, 2, 1).copy(), dur)[0]
    wrong_k = oracle.logz_durtrans(emis, None, np.roll(trans3, 1, axis=0).copy(), dur)[0]
    assert abs(wrong_t - lz) > 1e-4 and abs(wrong_k - lz) > 1e-4
