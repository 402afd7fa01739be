"""fp64 CPU oracle of the semi-CRF forward-backward pass (TEST INFRASTRUCTURE).

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this package.  It compiles ``semicrf_oracle.c`` with
gcc (plain C, OpenMP) and calls it through ctypes; it imports nothing from the
GPU package and the GPU package imports nothing from here.

The C file's header states, passage by passage, which part of the paper each
step follows (Eq. 1-2 prefix sums, Eq. 4 edge potential, Algorithm 1 and
Algorithm 3 recurrences kept as full tables, the "Gradient Formulas" section).
Every function here is pinned by ``tests/test_oracle_pins.py`` (brute-force
enumeration, the K=1 linear-chain CRF, closed forms, finite differences,
marginal invariants, the centring/duration-prior identity of Eq. 5, the toy
baseline table; the boundary terms of Eq. 4 by enumeration with those terms, by
finite differences, by the K=1 chain with start/end scores and by the identity
between scalar boundaries and projections at the first/last token; the
duration-dependent transitions by enumeration, by the reduction to one shared
matrix, by finite differences and by the identity with the duration bias).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "semicrf_oracle.c")
_LIB = os.path.join(_HERE, "libsemicrf_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc; returns the path of the shared object."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True, cwd=_HERE)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        dp = ctypes.POINTER(ctypes.c_double)
        ip = ctypes.POINTER(ctypes.c_int32)
        lib.semicrf_oracle_fwd_bwd.restype = ctypes.c_int
        lib.semicrf_oracle_fwd_bwd.argtypes = [dp, ip, dp, dp, dp] + [ctypes.c_int] * 6 + [dp] * 11
        lib.semicrf_oracle_logz.restype = ctypes.c_int
        lib.semicrf_oracle_logz.argtypes = [dp, ip, dp, dp] + [ctypes.c_int] * 6 + [dp]
        lib.semicrf_oracle_fwd_bwd_boundary.restype = ctypes.c_int
        lib.semicrf_oracle_fwd_bwd_boundary.argtypes = ([dp, ip, dp, dp, dp] + [dp] * 4 + [ctypes.c_int] * 6
                                                        + [dp] * 16)
        lib.semicrf_oracle_fwd_bwd_durtrans.restype = ctypes.c_int
        lib.semicrf_oracle_fwd_bwd_durtrans.argtypes = [dp, ip, dp, dp, dp] + [ctypes.c_int] * 6 + [dp] * 5
        lib.semicrf_oracle_logz_durtrans.restype = ctypes.c_int
        lib.semicrf_oracle_logz_durtrans.argtypes = [dp, ip, dp, dp] + [ctypes.c_int] * 6 + [dp]
        lib.semicrf_oracle_viterbi.restype = ctypes.c_int
        lib.semicrf_oracle_viterbi.argtypes = [dp, ip, dp, dp] + [dp] * 4 + [ctypes.c_int] * 6 + [dp, ip, ip, ip]
        lib.semicrf_oracle_logz_boundary.restype = ctypes.c_int
        lib.semicrf_oracle_logz_boundary.argtypes = [dp, ip, dp, dp] + [dp] * 4 + [ctypes.c_int] * 6 + [dp]
        _lib = lib
    return _lib


def _dptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _as_f64(a):
    return np.ascontiguousarray(np.asarray(a), dtype=np.float64)


@dataclass
class OracleResult:
    logz: np.ndarray          # [B]
    grad_emis: np.ndarray     # [B,T,C]  d(sum_b w_b logZ_b)/d emis
    pos_marg: np.ndarray      # [B,T,C]  P(label of token u is c)
    grad_trans: np.ndarray    # [C,C]
    grad_dur: np.ndarray      # [K,C]
    grad_trans_b: np.ndarray  # [B,C,C]  per sequence (weighted by w_b)
    grad_dur_b: np.ndarray    # [B,K,C]
    threads: int
    S: np.ndarray | None = None      # [B,T+1,C] centred prefix sums
    alpha: np.ndarray | None = None  # [B,T+1,C]
    beta: np.ndarray | None = None   # [B,T+1,C]
    gS: np.ndarray | None = None     # [B,T+1,C] gradient w.r.t. the prefix sums
    grad_proj_start: np.ndarray | None = None  # [B,T,C] gradient w.r.t. the start projections
    grad_proj_end: np.ndarray | None = None    # [B,T,C] gradient w.r.t. the end projections
    grad_pi_start: np.ndarray | None = None    # [C] gradient w.r.t. the scalar start boundary
    grad_pi_end: np.ndarray | None = None      # [C] gradient w.r.t. the scalar end boundary
    bdy_post: np.ndarray | None = None         # [B,T+1] posterior of a segment boundary at position t


def fwd_bwd(emis, lengths, trans, dur, grad_logz=None, center=True, threads=0,
            tables=False, proj_start=None, proj_end=None, pi_start=None, pi_end=None,
            boundary=False) -> OracleResult:
    """Run the oracle.  emis [B,T,C], lengths [B] or None, trans [C,C]
    (source label first), dur [K,C] (row k-1), grad_logz [B] or None.
    proj_start / proj_end [B,T,C] and pi_start / pi_end [C] are the optional boundary
    terms of Eq. 4; with any of them (or boundary=True) the result also carries their
    gradients and the boundary posterior."""
    lib = _load()
    emis = _as_f64(emis)
    B, T, C = emis.shape
    trans = _as_f64(trans)
    dur = _as_f64(dur)
    K = dur.shape[0]
    assert trans.shape == (C, C) and dur.shape == (K, C)
    lp = None
    if lengths is not None:
        lengths = np.ascontiguousarray(np.asarray(lengths), dtype=np.int32)
        assert lengths.shape == (B,)
        lp = lengths.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))
    w = None if grad_logz is None else _as_f64(grad_logz)
    logz = np.zeros(B)
    gE = np.zeros((B, T, C))
    pm = np.zeros((B, T, C))
    gTr = np.zeros((C, C))
    gD = np.zeros((K, C))
    gTr_b = np.zeros((B, C, C))
    gD_b = np.zeros((B, K, C))
    S = np.zeros((B, T + 1, C)) if tables else None
    al = np.zeros((B, T + 1, C)) if tables else None
    be = np.zeros((B, T + 1, C)) if tables else None
    gS = np.zeros((B, T + 1, C)) if tables else None
    if boundary or any(x is not None for x in (proj_start, proj_end, pi_start, pi_end)):
        ps = None if proj_start is None else _as_f64(proj_start)
        pe = None if proj_end is None else _as_f64(proj_end)
        pis = None if pi_start is None else _as_f64(pi_start)
        pie = None if pi_end is None else _as_f64(pi_end)
        for a in (ps, pe):
            assert a is None or a.shape == (B, T, C)
        for a in (pis, pie):
            assert a is None or a.shape == (C,)
        gPs = np.zeros((B, T, C))
        gPe = np.zeros((B, T, C))
        gPis = np.zeros(C)
        gPie = np.zeros(C)
        bdy = np.zeros((B, T + 1))
        rc = lib.semicrf_oracle_fwd_bwd_boundary(
            _dptr(emis), lp, _dptr(trans), _dptr(dur), _dptr(w), _dptr(ps), _dptr(pe), _dptr(pis), _dptr(pie),
            B, T, K, C, int(bool(center)), int(threads),
            _dptr(logz), _dptr(gE), _dptr(pm), _dptr(gTr), _dptr(gD), _dptr(gTr_b), _dptr(gD_b),
            _dptr(S), _dptr(al), _dptr(be), _dptr(gS), _dptr(gPs), _dptr(gPe), _dptr(gPis), _dptr(gPie),
            _dptr(bdy))
        if rc < 0:
            raise ValueError("semicrf_oracle_fwd_bwd_boundary: bad arguments")
        return OracleResult(logz, gE, pm, gTr, gD, gTr_b, gD_b, rc, S, al, be, gS, gPs, gPe, gPis, gPie, bdy)
    rc = lib.semicrf_oracle_fwd_bwd(_dptr(emis), lp, _dptr(trans), _dptr(dur), _dptr(w),
                                    B, T, K, C, int(bool(center)), int(threads),
                                    _dptr(logz), _dptr(gE), _dptr(pm), _dptr(gTr), _dptr(gD),
                                    _dptr(gTr_b), _dptr(gD_b), _dptr(S), _dptr(al), _dptr(be), _dptr(gS))
    if rc < 0:
        raise ValueError("semicrf_oracle_fwd_bwd: bad arguments")
    return OracleResult(logz, gE, pm, gTr, gD, gTr_b, gD_b, rc, S, al, be, gS)


def logz(emis, lengths, trans, dur, center=True, threads=0, proj_start=None, proj_end=None,
         pi_start=None, pi_end=None) -> np.ndarray:
    """Forward pass only: logZ [B] (optional boundary terms as in fwd_bwd)."""
    lib = _load()
    emis = _as_f64(emis)
    B, T, C = emis.shape
    trans = _as_f64(trans)
    dur = _as_f64(dur)
    K = dur.shape[0]
    lp = None
    if lengths is not None:
        lengths = np.ascontiguousarray(np.asarray(lengths), dtype=np.int32)
        lp = lengths.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))
    out = np.zeros(B)
    if any(x is not None for x in (proj_start, proj_end, pi_start, pi_end)):
        ps = None if proj_start is None else _as_f64(proj_start)
        pe = None if proj_end is None else _as_f64(proj_end)
        pis = None if pi_start is None else _as_f64(pi_start)
        pie = None if pi_end is None else _as_f64(pi_end)
        rc = lib.semicrf_oracle_logz_boundary(_dptr(emis), lp, _dptr(trans), _dptr(dur), _dptr(ps), _dptr(pe),
                                              _dptr(pis), _dptr(pie), B, T, K, C, int(bool(center)),
                                              int(threads), _dptr(out))
    else:
        rc = lib.semicrf_oracle_logz(_dptr(emis), lp, _dptr(trans), _dptr(dur),
                                     B, T, K, C, int(bool(center)), int(threads), _dptr(out))
    if rc < 0:
        raise ValueError("semicrf_oracle_logz: bad arguments")
    return out


def entropies(pos_marg, bdy_post, lengths):
    """The two entropies of the paper's boundary-entropy paragraph, written out per sequence:
    h_pos = mean over the L tokens of the label entropy of pos_marg[u,:];
    h_bdy = Shannon entropy of bdy_post[0:L] normalised to sum 1 (a segment starts at token u
    iff a boundary falls at position u).  Plain loops over sequences, fp64."""
    pos_marg = _as_f64(pos_marg)
    bdy_post = _as_f64(bdy_post)
    B, T, C = pos_marg.shape
    h_pos = np.zeros(B)
    h_bdy = np.zeros(B)
    for b in range(B):
        L = T if lengths is None else int(lengths[b])
        if L < 1:
            continue
        pm = pos_marg[b, :L]
        safe = np.where(pm > 0, pm, 1.0)
        h_pos[b] = -(pm * np.log(safe)).sum() / L
        ph = bdy_post[b, :L] / bdy_post[b, :L].sum()
        safe = np.where(ph > 0, ph, 1.0)
        h_bdy[b] = -(ph * np.log(safe)).sum()
    return h_pos, h_bdy


def viterbi(emis, lengths, trans, dur, center=True, threads=0, proj_start=None, proj_end=None,
            pi_start=None, pi_end=None):
    """Best segmentation (max semiring).  Returns (score [B], labels [B,T] int32 with -1 beyond
    the sequence, starts [B,T] int32: 1 on the first token of every segment, nseg [B])."""
    lib = _load()
    emis = _as_f64(emis)
    B, T, C = emis.shape
    trans = _as_f64(trans)
    dur = _as_f64(dur)
    K = dur.shape[0]
    lp = None
    if lengths is not None:
        lengths = np.ascontiguousarray(np.asarray(lengths), dtype=np.int32)
        lp = lengths.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))
    opt = [None if a is None else _as_f64(a) for a in (proj_start, proj_end, pi_start, pi_end)]
    score = np.zeros(B)
    labels = np.zeros((B, T), dtype=np.int32)
    starts = np.zeros((B, T), dtype=np.int32)
    nseg = np.zeros(B, dtype=np.int32)
    i32 = lambda a: a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))
    rc = lib.semicrf_oracle_viterbi(_dptr(emis), lp, _dptr(trans), _dptr(dur), *[_dptr(a) for a in opt],
                                    B, T, K, C, int(bool(center)), int(threads), _dptr(score), i32(labels),
                                    i32(starts), i32(nseg))
    if rc < 0:
        raise ValueError("semicrf_oracle_viterbi: bad arguments")
    return score, labels, starts, nseg


def path_score(emis, L, trans, dur, labels, starts, center=True, proj_start=None, proj_end=None,
               pi_start=None, pi_end=None):
    """Score of ONE given segmentation of one sequence (emis [T,C], first L tokens), written out
    from the definition of the edge potential: the sum over its segments [s, s+k) with label c of
    the centred content, the duration bias, the transition from the previous segment's label (for
    the first segment: the best source label, since every initial label has score 0), and the
    boundary terms.  Independent of the dynamic programme; used to validate decoded paths."""
    emis = _as_f64(emis)
    T, C = emis.shape
    trans = _as_f64(trans)
    dur = _as_f64(dur)
    nu = emis[:L].mean(0) if (center and L > 0) else np.zeros(C)
    bounds = [u for u in range(L) if starts[u]] + [L]
    if L > 0:
        assert bounds[0] == 0, "the first token must start a segment"
    total = 0.0
    prev = None
    for s, e in zip(bounds[:-1], bounds[1:]):
        c = int(labels[s])
        k = e - s
        assert 1 <= k <= dur.shape[0] and all(int(labels[u]) == c for u in range(s, e))
        total += (emis[s:e, c] - nu[c]).sum() + dur[k - 1, c]
        total += trans[:, c].max() if prev is None else trans[prev, c]
        if proj_start is not None:
            total += proj_start[s, c]
        if proj_end is not None:
            total += proj_end[e - 1, c]
        if pi_start is not None and s == 0:
            total += pi_start[c]
        if pi_end is not None and e == L:
            total += pi_end[c]
        prev = c
    return total



def _lengths_ptr(lengths, B):
    if lengths is None:
        return None, None
    lengths = np.ascontiguousarray(np.asarray(lengths), dtype=np.int32)
    assert lengths.shape == (B,)
    return lengths, lengths.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))


def fwd_bwd_durtrans(emis, lengths, trans, dur, grad_logz=None, center=True, threads=0) -> OracleResult:
    """Duration-dependent transitions: trans [K,C,C] (row k-1, source label, destination label)
    replaces trans[c',c] in the potential.  grad_trans of the result is [K,C,C]."""
    lib = _load()
    emis = _as_f64(emis)
    B, T, C = emis.shape
    trans = _as_f64(trans)
    dur = _as_f64(dur)
    K = dur.shape[0]
    assert trans.shape == (K, C, C) and dur.shape == (K, C)
    keep, lp = _lengths_ptr(lengths, B)
    w = None if grad_logz is None else _as_f64(grad_logz)
    logz = np.zeros(B)
    gE = np.zeros((B, T, C))
    pm = np.zeros((B, T, C))
    gTr = np.zeros((K, C, C))
    gD = np.zeros((K, C))
    rc = lib.semicrf_oracle_fwd_bwd_durtrans(_dptr(emis), lp, _dptr(trans), _dptr(dur), _dptr(w), B, T, K, C,
                                             int(bool(center)), int(threads), _dptr(logz), _dptr(gE), _dptr(pm),
                                             _dptr(gTr), _dptr(gD))
    if rc < 0:
        raise ValueError("semicrf_oracle_fwd_bwd_durtrans: bad arguments")
    return OracleResult(logz, gE, pm, gTr, gD, None, None, rc)


def logz_durtrans(emis, lengths, trans, dur, center=True, threads=0) -> np.ndarray:
    """Forward only with trans [K,C,C]."""
    lib = _load()
    emis = _as_f64(emis)
    B, T, C = emis.shape
    trans = _as_f64(trans)
    dur = _as_f64(dur)
    K = dur.shape[0]
    assert trans.shape == (K, C, C) and dur.shape == (K, C)
    keep, lp = _lengths_ptr(lengths, B)
    logz = np.zeros(B)
    rc = lib.semicrf_oracle_logz_durtrans(_dptr(emis), lp, _dptr(trans), _dptr(dur), B, T, K, C,
                                          int(bool(center)), int(threads), _dptr(logz))
    if rc < 0:
        raise ValueError("semicrf_oracle_logz_durtrans: bad arguments")
    return logz
