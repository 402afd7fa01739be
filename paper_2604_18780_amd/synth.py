"""Seeded synthetic workloads shaped like the paper's (no method arithmetic here).

This module only draws random inputs; it holds none of the semi-CRF
computation, so both the CPU oracle's tests and the GPU path may use it.

Five named configurations (shapes from the workloads the paper describes:
NER-sized NLP batches, the TIMIT-like B=32 / C=64 / K~30 speech shape, the
genome-scale T=100 000 / C=24 validation shape and the large-K genomic regime):

  "tiny"     B=2  T=512     K=8   C=4   iid N(0,1) emissions, full lengths
  "nlp"      B=64 T=256     K=16  C=24  lengths U{128..256}, geometric segments (mean 6)
  "speech"   B=32 T=2000    K=32  C=64  lengths U{1000..2000}, geometric (mean 12), noise sd 1.5
  "genomic"  B=4  T=100000  K=64  C=24  geometric (mean 40), 10:1 label imbalance
  "longgen"  B=1  T=400000  K=512 C=8   log-normal lengths (median 150, capped at K), 20:1 imbalance

Recipe (fixed draw order: lengths, trans, dur, label path, noise):
  trans ~ N(0, 0.1^2) [C,C]; dur ~ N(0, 0.1^2) [K,C] ("speech": mean -0.01*k, k 1-based);
  label path: consecutive segments, label drawn from p and redrawn until it
  differs from the previous one, length from the stated distribution;
  emis[t,c] = 2.0 * [c == label(t)] + sd * N(0,1), float32.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np


@dataclass
class Workload:
    name: str
    emis: np.ndarray      # [B,T,C] float32
    lengths: np.ndarray   # [B] int32
    trans: np.ndarray     # [C,C] float32, source label first
    dur: np.ndarray       # [K,C] float32, row k-1
    B: int
    T: int
    K: int
    C: int

    @property
    def nominal_edges(self) -> float:
        """sum_b L_b * K * C^2 (the unit of the edge-evals/s metric)."""
        return float(self.lengths.astype(np.int64).sum()) * self.K * self.C * self.C

    @property
    def positions(self) -> int:
        return int(self.lengths.astype(np.int64).sum())


CONFIGS = {
    # name: B, T, K, C, (len_lo, len_hi) or None, seg model, seg param, imbalance, noise sd, dur slope, seed
    "tiny":    dict(B=2,  T=512,    K=8,   C=4,  lens=None,         seg=None,        segp=None,  imb=1.0,  sd=1.0, slope=0.0,   seed=0),
    "nlp":     dict(B=64, T=256,    K=16,  C=24, lens=(128, 256),   seg="geometric", segp=6.0,   imb=1.0,  sd=1.0, slope=0.0,   seed=2),
    "speech":  dict(B=32, T=2000,   K=32,  C=64, lens=(1000, 2000), seg="geometric", segp=12.0,  imb=1.0,  sd=1.5, slope=-0.01, seed=3),
    "genomic": dict(B=4,  T=100000, K=64,  C=24, lens=None,         seg="geometric", segp=40.0,  imb=10.0, sd=1.0, slope=0.0,   seed=4),
    "longgen": dict(B=1,  T=400000, K=512, C=8,  lens=None,         seg="lognormal", segp=150.0, imb=20.0, sd=1.0, slope=0.0,   seed=5),
}

ACTIVE_MEAN = 2.0
LOGNORMAL_SIGMA = 0.75


def _label_path(rng, T, C, K, seg, segp, imb):
    p = np.ones(C)
    p[0] = imb
    p = p / p.sum()
    labels = np.empty(T, dtype=np.int64)
    t = 0
    prev = -1
    while t < T:
        y = int(rng.choice(C, p=p))
        while y == prev and C > 1:
            y = int(rng.choice(C, p=p))
        if seg == "geometric":
            n = int(rng.geometric(1.0 / segp))
        else:  # log-normal with the stated median, capped at K
            n = int(np.ceil(rng.lognormal(np.log(segp), LOGNORMAL_SIGMA)))
            n = max(1, min(n, K))
        labels[t:t + n] = y
        t += n
        prev = y
    return labels


def make(name: str, T: int | None = None, B: int | None = None, seed: int | None = None,
         K: int | None = None, C: int | None = None) -> Workload:
    """Build a named workload; T/B/K/C override the shape (used for reduced
    parity cases and for the bounded CPU-baseline sample), seed the stream."""
    cfg = dict(CONFIGS[name])
    if T is not None:
        if cfg["lens"] is not None:
            lo, hi = cfg["lens"]
            cfg["lens"] = (max(1, int(round(lo * T / cfg["T"]))), T)
        cfg["T"] = T
    if B is not None:
        cfg["B"] = B
    if K is not None:
        cfg["K"] = K
    if C is not None:
        cfg["C"] = C
    if seed is not None:
        cfg["seed"] = seed
    B_, T_, K_, C_ = cfg["B"], cfg["T"], cfg["K"], cfg["C"]
    rng = np.random.default_rng(cfg["seed"])
    if cfg["lens"] is None:
        lengths = np.full(B_, T_, dtype=np.int32)
    else:
        lo, hi = cfg["lens"]
        lengths = rng.integers(lo, hi + 1, size=B_).astype(np.int32)
    trans = (0.1 * rng.standard_normal((C_, C_))).astype(np.float32)
    dur = 0.1 * rng.standard_normal((K_, C_))
    if cfg["slope"] != 0.0:
        dur = dur + cfg["slope"] * np.arange(1, K_ + 1)[:, None]
    dur = dur.astype(np.float32)
    emis = np.empty((B_, T_, C_), dtype=np.float32)
    for b in range(B_):
        if cfg["seg"] is None:
            mean = np.zeros((T_, C_), dtype=np.float32)
        else:
            labels = _label_path(rng, T_, C_, K_, cfg["seg"], cfg["segp"], cfg["imb"])
            mean = np.zeros((T_, C_), dtype=np.float32)
            mean[np.arange(T_), labels] = ACTIVE_MEAN
        noise = rng.standard_normal((T_, C_), dtype=np.float32)
        emis[b] = mean + np.float32(cfg["sd"]) * noise
    return Workload(name, emis, lengths, trans, dur, B_, T_, K_, C_)


def small_random(seed: int, B: int, T: int, K: int, C: int, ragged: bool = True,
                 scale: float = 1.0) -> Workload:
    """Unstructured random case for parity sweeps: N(0, scale^2) emissions,
    N(0, 0.3^2) transitions and duration bias, lengths uniform in [0, T] when
    ragged (so empty and full sequences both occur over a few seeds)."""
    rng = np.random.default_rng(seed)
    lengths = (rng.integers(0, T + 1, size=B) if ragged else np.full(B, T)).astype(np.int32)
    trans = (0.3 * rng.standard_normal((C, C))).astype(np.float32)
    dur = (0.3 * rng.standard_normal((K, C))).astype(np.float32)
    emis = (scale * rng.standard_normal((B, T, C))).astype(np.float32)
    return Workload(f"rand{seed}", emis, lengths, trans, dur, B, T, K, C)


def boundary_terms(w: Workload, seed: int = 12345, scale: float = 0.5):
    """Seeded stand-ins for the optional boundary terms of Eq. 4: start / end projections
    ~ N(0, scale^2) of shape [B,T,C] and scalar sequence boundaries ~ N(0, 1) of shape [C]
    (float32; draw order: proj_start, proj_end, pi_start, pi_end)."""
    rng = np.random.default_rng(seed)
    ps = (scale * rng.standard_normal((w.B, w.T, w.C))).astype(np.float32)
    pe = (scale * rng.standard_normal((w.B, w.T, w.C))).astype(np.float32)
    pis = rng.standard_normal(w.C).astype(np.float32)
    pie = rng.standard_normal(w.C).astype(np.float32)
    return ps, pe, pis, pie


def duration_transitions(w: Workload, seed: int = 777, sd: float = 0.1):
    """Seeded stand-in for duration-dependent transitions: one [C,C] matrix per duration, the
    workload's matrix plus N(0, sd^2) noise per (duration, source, destination); float32 [K,C,C]."""
    rng = np.random.default_rng(seed)
    return (w.trans[None] + sd * rng.standard_normal((w.K, w.C, w.C))).astype(np.float32)


def reshape_transitions(trans: np.ndarray, sd: float | None = None, band: int | None = None,
                        forbidden: float = -1.0e4) -> np.ndarray:
    """Other transition models on the same draw: scores rescaled from the recipe's N(0, 0.1^2) to
    N(0, sd^2), and / or every transition between labels further apart than `band` (cyclically)
    set to `forbidden` (an exact zero of exp(trans) in fp64).  A banded matrix mixes slowly: the case
    the chunk-parallel scans' verification is there for."""
    out = trans.astype(np.float64)
    if sd is not None:
        out = out * (sd / 0.1)
    if band is not None:
        C = out.shape[0]
        d = np.abs(np.arange(C)[:, None] - np.arange(C)[None, :])
        d = np.minimum(d, C - d)
        out = np.where(d <= band, out, forbidden)
    return out.astype(np.float32)
