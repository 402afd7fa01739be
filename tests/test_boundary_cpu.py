"""Host-side checks of the C-ABI library that need no GPU.

The shared library must load, export every symbol that ``include/semicrf.h``
declares, size its workspace sensibly and reject bad arguments before touching
the device.  No kernel is launched here.
"""
import ctypes
import math
import os
import re

import pytest

from paper_2604_18780_amd import binding as sb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "semicrf.h")


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(semicrf_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = ctypes.CDLL(sb.LIB_PATH)
    names = declared_functions()
    assert set(names) == set(sb.EXPORTS)
    for n in names:
        assert hasattr(lib, n), n


def test_version_and_strerror():
    assert sb.semicrf_version() >= 1
    assert sb.semicrf_strerror(0) == "ok"
    for code in (-1, -2, -3, -4):
        assert sb.semicrf_strerror(code) not in ("ok", "unknown status")
    assert sb.semicrf_strerror(-99) == "unknown status"


def test_workspace_bytes_rejects_bad_sizes():
    lib = sb.load()
    out = ctypes.c_size_t(0)
    for args in [(0, 8, 2, 3), (1, 0, 2, 3), (1, 8, 0, 3), (1, 8, 2, 0), (-1, 8, 2, 3)]:
        assert lib.semicrf_workspace_bytes(*args, 0, 1, ctypes.byref(out)) == -1
    assert lib.semicrf_workspace_bytes(1, 8, 2, 3, -5, 1, ctypes.byref(out)) == -1
    assert lib.semicrf_workspace_bytes(1, 8, 2, 3, 0, 1, None) == -1
    # label count beyond the kernels' limits
    assert lib.semicrf_workspace_bytes(1, 8, 2, 257, 0, 0, ctypes.byref(out)) == -3
    assert lib.semicrf_workspace_bytes(1, 8, 2, 65, 0, 1, ctypes.byref(out)) == -3
    assert lib.semicrf_workspace_bytes(1, 8, 2, 65, 0, 0, ctypes.byref(out)) == 0
    # K*C too large for the LDS ring
    assert lib.semicrf_workspace_bytes(1, 100000, 4096, 64, 0, 1, ctypes.byref(out)) == -3


def test_workspace_is_aligned_positive_and_monotone():
    prev = 0
    for T in (1000, 10000, 100000, 400000):
        n = sb.semicrf_workspace_bytes(4, T, 64, 24, 0, True)
        assert n % 256 == 0 and n > prev
        prev = n
    assert sb.semicrf_workspace_bytes(4, 1000, 64, 24, 0, False) < sb.semicrf_workspace_bytes(4, 1000, 64, 24, 0, True)


def test_working_memory_beyond_prefix_arrays_is_bounded_then_sublinear_in_T():
    """Checkpoints + per-interval recompute buffers (grad workspace - forward-only workspace).
    The automatic interval gives one task per SIMD, so up to T ~ 1024*sqrt(T*K)/B this part
    is two more O(T*C) arrays, the rows the forward and the backward scan tasks leave for the
    marginals (never more than 2.5x the prefix arrays); beyond that the interval is capped at
    sqrt(T*K), the rows go to a fixed number of slots and it must grow like sqrt(T).  A caller that
    asks for the per-interval recurrence (plan kind 2) has one such array (1.5x)."""
    B, K, C = 4, 64, 24
    extra = lambda T: (sb.semicrf_workspace_bytes(B, T, K, C, 0, True)
                       - sb.semicrf_workspace_bytes(B, T, K, C, 0, False))
    for T in (100000, 400000, 1600000):
        assert extra(T) < 2.5 * B * (T + 1) * C * 20
        assert (sb.semicrf_workspace_bytes(B, T, K, C, 0, 2)
                - sb.semicrf_workspace_bytes(B, T, K, C, 0, False)) < 1.5 * B * (T + 1) * C * 20
    # 16x longer sequences: sqrt growth is 4x (the number of rounds is an integer, hence the slack), linear 16x
    assert extra(204800000) / extra(12800000) < 6.0
    # long maximal durations (K >= 128): the same two row arrays while every task has a slot
    extra512 = lambda T: (sb.semicrf_workspace_bytes(2, T, 512, 8, 0, True)
                          - sb.semicrf_workspace_bytes(2, T, 512, 8, 0, False))
    for T in (400000, 1600000):
        assert extra512(T) < 2.5 * 2 * (T + 1) * 8 * 20
    # 4x longer: sqrt growth is 2x, linear 4x
    assert extra512(1000000000) / extra512(250000000) < 3.0
    # sequences beyond 2^30 positions are refused (positions are 32-bit in the kernels)
    with pytest.raises(Exception, match="-3"):
        sb.semicrf_workspace_bytes(1, (1 << 30) + 1, 4, 2, 0, True)
    # and it is of the order of what the paper's own per-interval layout (full K x C x C
    # gradient workspace per checkpoint) would need, without the K*C*C blow-up per interval
    T = 100000
    delta = math.ceil(math.sqrt(T * K))
    paper_ws = B * math.ceil(T / delta) * K * C * C * 8
    assert extra(T) < 40 * paper_ws


def test_working_memory_beyond_prefix_arrays_is_sublinear_in_T():
    """The low-memory plan (flag SEMICRF_LOW_MEMORY, workspace kinds 8 / 9): checkpoints every ceil(sqrt(T*K))
    positions and a fixed number of row buffers of one interval each per sequence.  The part of the workspace
    that is not the O(T*C) prefix arrays, measured as (gradient workspace - forward-only workspace), must grow
    like sqrt(T): at most 2.3x when T grows fourfold (it would quadruple if it were linear), from T = 100 000
    on, at the genomic and the long-duration shapes (the paper's "Complexity" section and memory table:
    O(KC) ring + O(sqrt(T/K) KC) checkpoints beyond the prefix sums)."""
    for (B, K, C) in ((4, 64, 24), (1, 512, 8)):
        extra = lambda T: (sb.semicrf_workspace_bytes(B, T, K, C, 0, 9) - sb.semicrf_workspace_bytes(B, T, K, C, 0, 8))
        e = [extra(T) for T in (100000, 400000, 1600000, 6400000)]
        for a, b in zip(e, e[1:]):
            assert 1.0 < b / a < 2.3, (B, K, C, e)
        # and it is small beside the emission array itself
        assert e[0] < 1.5 * B * 100000 * C * 4 * max(1.0, math.sqrt(K / 64.0))
        # the interval is the spacing of Algorithm 1
        for T in (100000, 400000):
            d = sb.semicrf_ckpt_interval_low_memory(B, T, K, C)
            assert d % 8 == 0 and math.ceil(math.sqrt(T * K)) <= d < math.ceil(math.sqrt(T * K)) + 8
    # the default plan needs more: it is the faster one, not the smaller one
    assert sb.semicrf_workspace_bytes(4, 100000, 64, 24, 0, 9) < 0.75 * sb.semicrf_workspace_bytes(4, 100000, 64, 24, 0, 1)
    # an explicit interval is taken as given, and kinds that do not exist are refused
    assert sb.semicrf_ckpt_interval_low_memory(4, 100000, 64, 24, 500) == 500
    for bad in (4, 7, 11, 16, -1):
        with pytest.raises(Exception, match="-1"):
            sb.semicrf_workspace_bytes(4, 1000, 8, 4, 0, bad)


def test_checkpoint_interval_choice():
    """Explicit intervals are clamped to T; the automatic one is a multiple of 8 (or T),
    at least max(8, K/2) and at most the sqrt(T*K) spacing of Algorithm 1 rounded up."""
    assert sb.semicrf_ckpt_interval(2, 100, 4, 3, 7) == 7
    assert sb.semicrf_ckpt_interval(2, 100, 4, 3, 1000) == 100
    for (B, T, K, C) in [(2, 512, 8, 4), (64, 256, 16, 24), (32, 2000, 32, 64), (4, 100000, 64, 24),
                         (1, 400000, 512, 8), (1, 3000, 512, 8), (1, 1, 1, 1), (4, 25600000, 64, 24)]:
        d = sb.semicrf_ckpt_interval(B, T, K, C)
        assert 1 <= d <= T
        assert d == T or d % 8 == 0
        if d < T:
            assert d >= max(8, K // 2)
            assert d <= math.ceil(math.sqrt(T * K)) + 7 or d <= max(8, K // 2) + 7
    # the genomic shape gets one task per SIMD
    d = sb.semicrf_ckpt_interval(4, 100000, 64, 24)
    assert 4 * math.ceil(100000 / d) == 1024


def test_memory_arithmetic_of_the_paper_example():
    """Section "Complexity": at T = 1e6, K = 200, C = 6 the edge tensor would be
    ~29 GB in float32, the prefix-sum array ~24 MB and the ring ~10 KB."""
    T, K, C = 10**6, 200, 6
    edge_bytes = T * K * C * C * 4
    prefix_bytes = (T + 1) * C * 4
    ring_bytes = K * C * 4 + 2 * K * C * 4          # K-slot forward ring + 2K-slot backward ring
    assert abs(edge_bytes / 1e9 - 28.8) < 0.1
    assert abs(prefix_bytes / 1e6 - 24.0) < 0.1
    assert 9e3 < ring_bytes < 15e3
    # this library: never anywhere near the edge tensor
    ws = sb.semicrf_workspace_bytes(1, T, K, C, 0, True)
    assert ws < edge_bytes / 50


def test_calls_reject_null_pointers_and_bad_workspace_before_any_launch():
    lib = sb.load()
    # every pointer null: invalid argument, checked on the host only
    rc = lib.semicrf_logz_fwd(None, None, None, None, 1, 8, 2, 3, 0, 1, None, 0, None, None)
    assert rc == -1
    rc = lib.semicrf_fwd_bwd(None, None, None, None, None, 1, 8, 2, 3, 0, 1, None, 0,
                             None, None, None, None, None, None)
    assert rc == -1
    rc = lib.semicrf_cum_scores(None, None, 1, 8, 3, 1, None, 0, None, None)
    assert rc == -1
    # non-null (fake, never dereferenced on the host) data pointers but no workspace
    fake = ctypes.c_void_p(4096)
    rc = lib.semicrf_logz_fwd(fake, None, fake, fake, 1, 8, 2, 3, 0, 1, None, 0, fake, None)
    assert rc == -2
    # misaligned workspace pointer
    rc = lib.semicrf_logz_fwd(fake, None, fake, fake, 1, 8, 2, 3, 0, 1, ctypes.c_void_p(4100), 1 << 30, fake, None)
    assert rc == -2
    # the entry points with the boundary terms of Eq. 4 check the same things
    rc = lib.semicrf_logz_fwd_boundary(None, None, None, None, None, None, None, None, 1, 8, 2, 3, 0, 1,
                                       None, 0, None, None)
    assert rc == -1
    rc = lib.semicrf_fwd_bwd_boundary(fake, None, fake, fake, None, None, None, None, None, 1, 8, 2, 3, 0, 1,
                                      None, 0, fake, fake, fake, fake, None, None, None, None, None, None, None)
    assert rc == -2
    # bad sizes win over everything else
    rc = lib.semicrf_logz_fwd(fake, None, fake, fake, 1, 8, 0, 3, 0, 1, fake, 1 << 30, fake, None)
    assert rc == -1


def test_viterbi_and_entropy_entries_check_their_arguments_on_the_host():
    lib = sb.load()
    out = ctypes.c_size_t(0)
    fake = ctypes.c_void_p(4096)
    assert lib.semicrf_viterbi_workspace_bytes(1, 8, 2, 3, None) == -1
    assert lib.semicrf_viterbi_workspace_bytes(0, 8, 2, 3, ctypes.byref(out)) == -1
    # label counts and windows beyond the one-wave decoder
    assert lib.semicrf_viterbi_workspace_bytes(1, 8, 2, 65, ctypes.byref(out)) == -3
    assert lib.semicrf_viterbi_workspace_bytes(1, 1000, 65, 64, ctypes.byref(out)) == -3
    assert lib.semicrf_viterbi_workspace_bytes(1, 1000, 512, 8, ctypes.byref(out)) == 0
    # O(T*C): the prefix arrays (20 B) plus a double pair, four ints and a byte per node
    n = sb.semicrf_viterbi_workspace_bytes(4, 100000, 64, 24)
    nodes = 4 * 100001 * 24
    assert n % 256 == 0 and nodes * (20 + 16 + 16 + 1) < n < nodes * 64
    rc = lib.semicrf_viterbi(None, None, None, None, None, None, None, None, 1, 8, 2, 3, 0, None, 0,
                             None, None, None, None, None)
    assert rc == -1
    rc = lib.semicrf_viterbi(fake, None, fake, fake, None, None, None, None, 1, 8, 2, 3, 0, None, 0,
                             fake, fake, fake, fake, None)
    assert rc == -2
    rc = lib.semicrf_viterbi(fake, None, fake, fake, None, None, None, None, 1, 8, 2, 3, 4 | 8, fake, 1 << 30,
                             fake, fake, fake, fake, None)
    assert rc == -1                                  # both storage types at once
    assert lib.semicrf_entropies(None, None, None, 1, 8, 3, None, None, None) == -1
    assert lib.semicrf_entropies(None, fake, None, 1, 8, 3, fake, None, None) == -1   # h_pos needs pos_marg
    assert lib.semicrf_entropies(fake, None, None, 1, 8, 3, None, fake, None) == -1   # h_bdy needs bdy_post
    assert lib.semicrf_entropies(fake, fake, None, 1, 0, 3, fake, fake, None) == -1


def test_duration_dependent_transition_entries_check_their_arguments_on_the_host():
    lib = sb.load()
    out = ctypes.c_size_t(0)
    iv = ctypes.c_int(0)
    fake = ctypes.c_void_p(4096)
    assert lib.semicrf_durtrans_workspace_bytes(1, 8, 2, 3, 0, 1, None) == -1
    assert lib.semicrf_durtrans_workspace_bytes(0, 8, 2, 3, 0, 1, ctypes.byref(out)) == -1
    assert lib.semicrf_durtrans_workspace_bytes(1, 8, 2, 3, -1, 1, ctypes.byref(out)) == -1
    # one label pair per thread: 33 labels and more do not fit a workgroup, nor 32 labels with K > 64
    assert lib.semicrf_durtrans_workspace_bytes(1, 100, 4, 33, 0, 1, ctypes.byref(out)) == -3
    assert lib.semicrf_durtrans_workspace_bytes(1, 100, 65, 32, 0, 1, ctypes.byref(out)) == -3
    assert lib.semicrf_durtrans_workspace_bytes(1, 100, 64, 32, 0, 1, ctypes.byref(out)) == 0
    # the gradient path needs the stored messages and the partial gradient tables on top
    assert (sb.semicrf_durtrans_workspace_bytes(4, 100000, 64, 24, 0, True)
            > sb.semicrf_durtrans_workspace_bytes(4, 100000, 64, 24, 0, False)
            > sb.semicrf_workspace_bytes(4, 100000, 64, 24, 0, False))
    # automatic interval: a multiple of 8 (or T), at least max(8, K/2); explicit ones are clamped to T
    for (B, T, K, C) in [(64, 256, 16, 24), (4, 100000, 64, 24), (1, 400000, 512, 8), (1, 1, 1, 1), (2, 50, 80, 4)]:
        d = sb.semicrf_durtrans_ckpt_interval(B, T, K, C)
        assert 1 <= d <= T and (d == T or (d % 8 == 0 and d >= max(8, K // 2)))
    assert sb.semicrf_durtrans_ckpt_interval(2, 100, 4, 3, 1000) == 100
    assert lib.semicrf_durtrans_ckpt_interval(2, 100, 4, 3, 0, None) == -1
    assert lib.semicrf_durtrans_ckpt_interval(2, 100, 4, 64, 0, ctypes.byref(iv)) == -3
    rc = lib.semicrf_logz_fwd_durtrans(None, None, None, None, 1, 8, 2, 3, 0, 1, None, 0, None, None)
    assert rc == -1
    rc = lib.semicrf_fwd_bwd_durtrans(fake, None, fake, fake, None, 1, 8, 2, 3, 0, 1, None, 0,
                                      fake, fake, fake, fake, None, None)
    assert rc == -2
    rc = lib.semicrf_fwd_bwd_durtrans(fake, None, fake, fake, None, 1, 8, 2, 3, 0, 1, fake, 1 << 30,
                                      fake, fake, None, fake, None, None)
    assert rc == -1                                  # grad_trans3 is required


def test_binding_requires_the_built_library(monkeypatch, tmp_path):
    import importlib
    mod = importlib.reload(sb)
    monkeypatch.setattr(mod, "LIB_PATH", str(tmp_path / "missing.so"))
    monkeypatch.setattr(mod, "_lib", None)
    with pytest.raises(FileNotFoundError):
        mod.load()
    importlib.reload(sb)


def test_bench_refuses_more_than_one_gpu():
    """One GPU only: `bench.py --gpus N` with N > 1 (or under a multi-rank launcher) exits with a
    message that says so, before anything touches a device."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode != 0 and "one GPU only" in r.stderr and r.stdout.strip() == ""
    env = dict(os.environ, WORLD_SIZE="2")
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py")], capture_output=True, text=True,
                       timeout=120, env=env)
    assert r.returncode != 0 and "one GPU only" in r.stderr
