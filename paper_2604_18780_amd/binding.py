"""Thin ctypes binding of ``libsemicrf.so`` (argument marshalling only).

Every function mirrors the C entry point of the same name in
``include/semicrf.h``: tensors are passed as device pointers, the work is
enqueued on torch's current HIP stream and nothing is computed here.  The
library must have been built (``python -m paper_2604_18780_amd.build``); a
missing library is an error, there is no fallback path.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsemicrf.so")
EXPORTS = ("semicrf_version", "semicrf_strerror", "semicrf_workspace_bytes",
           "semicrf_cum_scores", "semicrf_logz_fwd", "semicrf_fwd_bwd", "semicrf_fwd_bwd_profiled",
           "semicrf_scan_report", "semicrf_ckpt_interval", "semicrf_logz_fwd_boundary",
           "semicrf_fwd_bwd_boundary", "semicrf_entropies", "semicrf_viterbi_workspace_bytes",
           "semicrf_viterbi", "semicrf_durtrans_workspace_bytes", "semicrf_durtrans_ckpt_interval", "semicrf_logz_fwd_durtrans",
           "semicrf_fwd_bwd_durtrans", "semicrf_fwd_bwd_static", "semicrf_seq_report",
           "semicrf_ckpt_interval_low_memory")
SEMICRF_STATIC_WORKSPACE_BYTES = 64 << 20
SEMICRF_CENTER = 1
SEMICRF_SEQUENTIAL_SCAN = 2
SEMICRF_EMIS_F16 = 4
SEMICRF_EMIS_BF16 = 8
SEMICRF_MATRIX_SCAN = 16
SEMICRF_MARGINALS_ROWS = 32
SEMICRF_MARGINALS_INTERVAL = 64
SEMICRF_VITERBI_GLOBAL_TRACE = 128
SEMICRF_LOW_MEMORY = 256
SEMICRF_TWO_WAVE_SCAN = 512
SEMICRF_ONE_WAVE_SCAN = 1024
PLAN_LOW_MEMORY = 8   # added to want_grad for the workspace of SEMICRF_LOW_MEMORY calls


def SEMICRF_WARMUP(n: int) -> int:
    """flags bits 16..31: first warm-up length of the chunk-parallel scans."""
    return int(n) << 16


def grad_workspace_kind(flags: int) -> int:
    """The want_grad value of semicrf_workspace_bytes that fits a gradient call with these flags."""
    kind = 3 if flags & SEMICRF_MARGINALS_ROWS else (2 if flags & SEMICRF_MARGINALS_INTERVAL else 1)
    return kind | (PLAN_LOW_MEMORY if flags & SEMICRF_LOW_MEMORY else 0)


def fwd_workspace_kind(flags: int) -> int:
    """The want_grad value of semicrf_workspace_bytes that fits a forward-only call with these flags."""
    return PLAN_LOW_MEMORY if flags & SEMICRF_LOW_MEMORY else 0

_lib = None


class SemiCRFError(RuntimeError):
    def __init__(self, status: int, msg: str):
        super().__init__(f"semicrf status {status}: {msg}")
        self.status = status


def load():
    """Load the shared library (once) and declare the prototypes."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2604_18780_amd.build` "
            "(there is no CPU fallback)")
    lib = ctypes.CDLL(LIB_PATH)
    vp, ci, cu, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_uint, ctypes.c_size_t
    lib.semicrf_version.restype = ci
    lib.semicrf_version.argtypes = []
    lib.semicrf_strerror.restype = ctypes.c_char_p
    lib.semicrf_strerror.argtypes = [ci]
    lib.semicrf_workspace_bytes.restype = ci
    lib.semicrf_workspace_bytes.argtypes = [ci, ci, ci, ci, ci, ci, ctypes.POINTER(sz)]
    lib.semicrf_cum_scores.restype = ci
    lib.semicrf_cum_scores.argtypes = [vp, vp, ci, ci, ci, cu, vp, sz, vp, vp]
    lib.semicrf_logz_fwd.restype = ci
    lib.semicrf_logz_fwd.argtypes = [vp, vp, vp, vp, ci, ci, ci, ci, ci, cu, vp, sz, vp, vp]
    lib.semicrf_fwd_bwd.restype = ci
    lib.semicrf_fwd_bwd.argtypes = [vp, vp, vp, vp, vp, ci, ci, ci, ci, ci, cu, vp, sz,
                                    vp, vp, vp, vp, vp, vp]
    lib.semicrf_fwd_bwd_static.restype = ci
    lib.semicrf_fwd_bwd_static.argtypes = [vp, vp, vp, vp, vp, ci, ci, ci, ci, ci, cu, vp, vp, vp, vp, vp, vp]
    lib.semicrf_fwd_bwd_profiled.restype = ci
    lib.semicrf_fwd_bwd_profiled.argtypes = lib.semicrf_fwd_bwd.argtypes + [ctypes.POINTER(vp)]
    lib.semicrf_ckpt_interval.restype = ci
    lib.semicrf_ckpt_interval.argtypes = [ci, ci, ci, ci, ci, ctypes.POINTER(ci)]
    lib.semicrf_logz_fwd_boundary.restype = ci
    lib.semicrf_logz_fwd_boundary.argtypes = [vp] * 8 + [ci, ci, ci, ci, ci, cu, vp, sz, vp, vp]
    lib.semicrf_fwd_bwd_boundary.restype = ci
    lib.semicrf_fwd_bwd_boundary.argtypes = [vp] * 9 + [ci, ci, ci, ci, ci, cu, vp, sz] + [vp] * 11
    lib.semicrf_viterbi_workspace_bytes.restype = ci
    lib.semicrf_viterbi_workspace_bytes.argtypes = [ci, ci, ci, ci, ctypes.POINTER(sz)]
    lib.semicrf_viterbi.restype = ci
    lib.semicrf_viterbi.argtypes = [vp] * 8 + [ci, ci, ci, ci, cu, vp, sz] + [vp] * 5
    lib.semicrf_entropies.restype = ci
    lib.semicrf_entropies.argtypes = [vp, vp, vp, ci, ci, ci, vp, vp, vp]
    lib.semicrf_durtrans_workspace_bytes.restype = ci
    lib.semicrf_durtrans_workspace_bytes.argtypes = [ci, ci, ci, ci, ci, ci, ctypes.POINTER(sz)]
    lib.semicrf_durtrans_ckpt_interval.restype = ci
    lib.semicrf_durtrans_ckpt_interval.argtypes = [ci, ci, ci, ci, ci, ctypes.POINTER(ci)]
    lib.semicrf_logz_fwd_durtrans.restype = ci
    lib.semicrf_logz_fwd_durtrans.argtypes = lib.semicrf_logz_fwd.argtypes
    lib.semicrf_fwd_bwd_durtrans.restype = ci
    lib.semicrf_fwd_bwd_durtrans.argtypes = lib.semicrf_fwd_bwd.argtypes
    lib.semicrf_scan_report.restype = ci
    lib.semicrf_scan_report.argtypes = [vp, sz, ci, ci, ci, ci, ci, ci, vp, vp, vp]
    lib.semicrf_seq_report.restype = ci
    lib.semicrf_seq_report.argtypes = [vp, sz, ci, ci, ci, ci, ci, ci, vp, vp, vp]
    lib.semicrf_ckpt_interval_low_memory.restype = ci
    lib.semicrf_ckpt_interval_low_memory.argtypes = [ci, ci, ci, ci, ci, ctypes.POINTER(ci)]
    _lib = lib
    return lib


def _check(status: int):
    if status != 0:
        raise SemiCRFError(status, load().semicrf_strerror(status).decode())


def semicrf_version() -> int:
    return load().semicrf_version()


def semicrf_strerror(status: int) -> str:
    return load().semicrf_strerror(status).decode()


def semicrf_workspace_bytes(B, T, K, C, ckpt_interval=0, want_grad=True) -> int:
    out = ctypes.c_size_t(0)
    _check(load().semicrf_workspace_bytes(B, T, K, C, ckpt_interval, int(want_grad),
                                          ctypes.byref(out)))
    return out.value


def semicrf_ckpt_interval_low_memory(B, T, K, C, ckpt_interval=0) -> int:
    d = ctypes.c_int(0)
    _check(load().semicrf_ckpt_interval_low_memory(B, T, K, C, ckpt_interval, ctypes.byref(d)))
    return d.value


def semicrf_ckpt_interval(B, T, K, C, ckpt_interval=0) -> int:
    out = ctypes.c_int(0)
    _check(load().semicrf_ckpt_interval(B, T, K, C, ckpt_interval, ctypes.byref(out)))
    return out.value


def _ptr(t, dtype):
    if t is None:
        return None
    if not (t.is_cuda and t.is_contiguous() and t.dtype == dtype):
        raise ValueError(f"expected a contiguous {dtype} device tensor")
    return t.data_ptr()


def _emis(t, flags):
    """Pointer of the emission tensor and the flags with its storage type (float32, float16 or bfloat16)."""
    bits = {torch.float32: 0, torch.float16: SEMICRF_EMIS_F16, torch.bfloat16: SEMICRF_EMIS_BF16}
    if t.dtype not in bits:
        raise ValueError("emissions must be float32, float16 or bfloat16")
    return _ptr(t, t.dtype), (flags & ~(SEMICRF_EMIS_F16 | SEMICRF_EMIS_BF16)) | bits[t.dtype]


def _stream():
    return torch.cuda.current_stream().cuda_stream


def alloc_workspace(B, T, K, C, ckpt_interval=0, want_grad=True, device="cuda:0"):
    n = semicrf_workspace_bytes(B, T, K, C, ckpt_interval, want_grad)
    ws = torch.empty(n + 256, dtype=torch.uint8, device=device)
    off = (-ws.data_ptr()) % 256
    return ws[off:off + n]


def semicrf_cum_scores(emis, lengths, flags=SEMICRF_CENTER, workspace=None):
    B, T, C = emis.shape
    if workspace is None:
        workspace = alloc_workspace(B, T, 1, C, 0, False, emis.device)
    cum = torch.empty((B, T + 1, C), dtype=torch.float64, device=emis.device)
    ep, flags = _emis(emis, flags)
    _check(load().semicrf_cum_scores(ep, _ptr(lengths, torch.int32),
                                     B, T, C, flags, workspace.data_ptr(), workspace.numel(),
                                     cum.data_ptr(), _stream()))
    return cum


def semicrf_logz_fwd(emis, lengths, trans, dur, ckpt_interval=0, flags=SEMICRF_CENTER,
                     workspace=None, logz=None):
    B, T, C = emis.shape
    K = dur.shape[0]
    if workspace is None:
        workspace = alloc_workspace(B, T, K, C, ckpt_interval, fwd_workspace_kind(flags), emis.device)
    if logz is None:
        logz = torch.empty(B, dtype=torch.float32, device=emis.device)
    ep, flags = _emis(emis, flags)
    _check(load().semicrf_logz_fwd(ep, _ptr(lengths, torch.int32),
                                   _ptr(trans, torch.float32), _ptr(dur, torch.float32),
                                   B, T, K, C, ckpt_interval, flags,
                                   workspace.data_ptr(), workspace.numel(),
                                   _ptr(logz, torch.float32), _stream()))
    return logz


def semicrf_fwd_bwd(emis, lengths, trans, dur, grad_logz=None, ckpt_interval=0,
                    flags=SEMICRF_CENTER, workspace=None, want_pos_marg=True, out=None):
    """Returns (logz, grad_emis, grad_trans, grad_dur, pos_marg or None)."""
    B, T, C = emis.shape
    K = dur.shape[0]
    dev = emis.device
    if workspace is None:
        workspace = alloc_workspace(B, T, K, C, ckpt_interval, grad_workspace_kind(flags), dev)
    if out is None:
        logz = torch.empty(B, dtype=torch.float32, device=dev)
        g_e = torch.empty((B, T, C), dtype=torch.float32, device=dev)
        g_t = torch.empty((C, C), dtype=torch.float32, device=dev)
        g_d = torch.empty((K, C), dtype=torch.float32, device=dev)
        pm = torch.empty((B, T, C), dtype=torch.float32, device=dev) if want_pos_marg else None
    else:
        logz, g_e, g_t, g_d, pm = out
    ep, flags = _emis(emis, flags)
    _check(load().semicrf_fwd_bwd(ep, _ptr(lengths, torch.int32),
                                  _ptr(trans, torch.float32), _ptr(dur, torch.float32),
                                  _ptr(grad_logz, torch.float32), B, T, K, C, ckpt_interval, flags,
                                  workspace.data_ptr(), workspace.numel(),
                                  _ptr(logz, torch.float32), _ptr(g_e, torch.float32),
                                  _ptr(g_t, torch.float32), _ptr(g_d, torch.float32),
                                  _ptr(pm, torch.float32), _stream()))
    return logz, g_e, g_t, g_d, pm


def semicrf_fwd_bwd_static(emis, lengths, trans, dur, out, grad_logz=None, ckpt_interval=0,
                           flags=SEMICRF_CENTER):
    """semicrf_fwd_bwd on the library's static workspace.  `out` = (logz, grad_emis, grad_trans,
    grad_dur, pos_marg or None), preallocated by the caller: nothing is allocated here."""
    B, T, C = emis.shape
    K = dur.shape[0]
    logz, g_e, g_t, g_d, pm = out
    ep, flags = _emis(emis, flags)
    _check(load().semicrf_fwd_bwd_static(ep, _ptr(lengths, torch.int32), _ptr(trans, torch.float32),
                                         _ptr(dur, torch.float32), _ptr(grad_logz, torch.float32), B, T, K, C,
                                         ckpt_interval, flags, _ptr(logz, torch.float32),
                                         _ptr(g_e, torch.float32), _ptr(g_t, torch.float32),
                                         _ptr(g_d, torch.float32), _ptr(pm, torch.float32), _stream()))
    return out


def semicrf_logz_fwd_boundary(emis, lengths, trans, dur, proj_start=None, proj_end=None, pi_start=None,
                              pi_end=None, ckpt_interval=0, flags=SEMICRF_CENTER, workspace=None):
    B, T, C = emis.shape
    K = dur.shape[0]
    if workspace is None:
        workspace = alloc_workspace(B, T, K, C, ckpt_interval, fwd_workspace_kind(flags), emis.device)
    logz = torch.empty(B, dtype=torch.float32, device=emis.device)
    f32 = torch.float32
    ep, flags = _emis(emis, flags)
    _check(load().semicrf_logz_fwd_boundary(ep, _ptr(lengths, torch.int32), _ptr(trans, f32),
                                            _ptr(dur, f32), _ptr(proj_start, f32), _ptr(proj_end, f32),
                                            _ptr(pi_start, f32), _ptr(pi_end, f32), B, T, K, C, ckpt_interval,
                                            flags, workspace.data_ptr(), workspace.numel(), _ptr(logz, f32),
                                            _stream()))
    return logz


def semicrf_fwd_bwd_boundary(emis, lengths, trans, dur, grad_logz=None, proj_start=None, proj_end=None,
                             pi_start=None, pi_end=None, ckpt_interval=0, flags=SEMICRF_CENTER, workspace=None,
                             boundary_outputs=True):
    """Returns a dict with logz, grad_emis, grad_trans, grad_dur, pos_marg, grad_proj_start,
    grad_proj_end, grad_pi_start, grad_pi_end, bdy_post (the last five only with boundary_outputs:
    the C entry point takes NULL for each output that is not wanted)."""
    B, T, C = emis.shape
    K = dur.shape[0]
    dev = emis.device
    if workspace is None:
        workspace = alloc_workspace(B, T, K, C, ckpt_interval, grad_workspace_kind(flags), dev)
    f32 = torch.float32
    new = lambda *shape: torch.empty(shape, dtype=f32, device=dev)
    o = dict(logz=new(B), grad_emis=new(B, T, C), grad_trans=new(C, C), grad_dur=new(K, C), pos_marg=new(B, T, C),
             grad_proj_start=new(B, T, C), grad_proj_end=new(B, T, C), grad_pi_start=new(C), grad_pi_end=new(C),
             bdy_post=new(B, T + 1))
    if not boundary_outputs:
        for k in ("grad_proj_start", "grad_proj_end", "grad_pi_start", "grad_pi_end", "bdy_post"):
            o[k] = None
    ep, flags = _emis(emis, flags)
    _check(load().semicrf_fwd_bwd_boundary(ep, _ptr(lengths, torch.int32), _ptr(trans, f32),
                                           _ptr(dur, f32), _ptr(grad_logz, f32), _ptr(proj_start, f32),
                                           _ptr(proj_end, f32), _ptr(pi_start, f32), _ptr(pi_end, f32),
                                           B, T, K, C, ckpt_interval, flags, workspace.data_ptr(),
                                           workspace.numel(), *[_ptr(o[k], f32) for k in
                                                                ("logz", "grad_emis", "grad_trans", "grad_dur",
                                                                 "pos_marg", "grad_proj_start", "grad_proj_end",
                                                                 "grad_pi_start", "grad_pi_end", "bdy_post")],
                                           _stream()))
    return {k: v for k, v in o.items() if v is not None}


def semicrf_viterbi_workspace_bytes(B, T, K, C) -> int:
    out = ctypes.c_size_t(0)
    _check(load().semicrf_viterbi_workspace_bytes(B, T, K, C, ctypes.byref(out)))
    return out.value


def semicrf_viterbi(emis, lengths, trans, dur, proj_start=None, proj_end=None, pi_start=None, pi_end=None,
                    flags=SEMICRF_CENTER, workspace=None):
    """Returns (score [B] float32, labels [B,T] int32, starts [B,T] int32, nseg [B] int32)."""
    B, T, C = emis.shape
    K = dur.shape[0]
    dev = emis.device
    if workspace is None:
        n = semicrf_viterbi_workspace_bytes(B, T, K, C)
        ws = torch.empty(n + 256, dtype=torch.uint8, device=dev)
        off = (-ws.data_ptr()) % 256
        workspace = ws[off:off + n]
    f32 = torch.float32
    score = torch.empty(B, dtype=f32, device=dev)
    labels = torch.empty((B, T), dtype=torch.int32, device=dev)
    starts = torch.empty((B, T), dtype=torch.int32, device=dev)
    nseg = torch.empty(B, dtype=torch.int32, device=dev)
    ep, flags = _emis(emis, flags)
    _check(load().semicrf_viterbi(ep, _ptr(lengths, torch.int32), _ptr(trans, f32), _ptr(dur, f32),
                                  _ptr(proj_start, f32), _ptr(proj_end, f32), _ptr(pi_start, f32), _ptr(pi_end, f32),
                                  B, T, K, C, flags, workspace.data_ptr(), workspace.numel(), score.data_ptr(),
                                  labels.data_ptr(), starts.data_ptr(), nseg.data_ptr(), _stream()))
    return score, labels, starts, nseg


def semicrf_durtrans_workspace_bytes(B, T, K, C, ckpt_interval=0, want_grad=True) -> int:
    out = ctypes.c_size_t(0)
    _check(load().semicrf_durtrans_workspace_bytes(B, T, K, C, ckpt_interval, int(bool(want_grad)),
                                                   ctypes.byref(out)))
    return out.value


def semicrf_durtrans_ckpt_interval(B, T, K, C, ckpt_interval=0) -> int:
    out = ctypes.c_int(0)
    _check(load().semicrf_durtrans_ckpt_interval(B, T, K, C, ckpt_interval, ctypes.byref(out)))
    return out.value


def alloc_durtrans_workspace(B, T, K, C, ckpt_interval, want_grad, device):
    n = semicrf_durtrans_workspace_bytes(B, T, K, C, ckpt_interval, want_grad)
    ws = torch.empty(n + 256, dtype=torch.uint8, device=device)
    off = (-ws.data_ptr()) % 256
    return ws[off:off + n]


def semicrf_logz_fwd_durtrans(emis, lengths, trans3, dur, ckpt_interval=0, flags=SEMICRF_CENTER, workspace=None):
    """trans3 [K,C,C]: one transition matrix per duration.  Returns logz [B]."""
    B, T, C = emis.shape
    K = dur.shape[0]
    if workspace is None:
        workspace = alloc_durtrans_workspace(B, T, K, C, ckpt_interval, False, emis.device)
    logz = torch.empty(B, dtype=torch.float32, device=emis.device)
    ep, flags = _emis(emis, flags)
    _check(load().semicrf_logz_fwd_durtrans(ep, _ptr(lengths, torch.int32), _ptr(trans3, torch.float32),
                                            _ptr(dur, torch.float32), B, T, K, C, ckpt_interval, flags,
                                            workspace.data_ptr(), workspace.numel(), _ptr(logz, torch.float32),
                                            _stream()))
    return logz


def semicrf_fwd_bwd_durtrans(emis, lengths, trans3, dur, grad_logz=None, ckpt_interval=0,
                             flags=SEMICRF_CENTER, workspace=None, want_pos_marg=True):
    """trans3 [K,C,C].  Returns (logz, grad_emis, grad_trans3 [K,C,C], grad_dur, pos_marg or None)."""
    B, T, C = emis.shape
    K = dur.shape[0]
    dev = emis.device
    if workspace is None:
        workspace = alloc_durtrans_workspace(B, T, K, C, ckpt_interval, True, dev)
    f32 = torch.float32
    logz = torch.empty(B, dtype=f32, device=dev)
    g_e = torch.empty((B, T, C), dtype=f32, device=dev)
    g_t = torch.empty((K, C, C), dtype=f32, device=dev)
    g_d = torch.empty((K, C), dtype=f32, device=dev)
    pm = torch.empty((B, T, C), dtype=f32, device=dev) if want_pos_marg else None
    ep, flags = _emis(emis, flags)
    _check(load().semicrf_fwd_bwd_durtrans(ep, _ptr(lengths, torch.int32), _ptr(trans3, f32), _ptr(dur, f32),
                                           _ptr(grad_logz, f32), B, T, K, C, ckpt_interval, flags,
                                           workspace.data_ptr(), workspace.numel(), _ptr(logz, f32),
                                           _ptr(g_e, f32), _ptr(g_t, f32), _ptr(g_d, f32), _ptr(pm, f32),
                                           _stream()))
    return logz, g_e, g_t, g_d, pm


def semicrf_entropies(pos_marg, bdy_post, lengths):
    """Returns (h_pos [B], h_bdy [B]) from the outputs of semicrf_fwd_bwd_boundary."""
    B, T, C = pos_marg.shape
    h_pos = torch.empty(B, dtype=torch.float32, device=pos_marg.device)
    h_bdy = torch.empty(B, dtype=torch.float32, device=pos_marg.device)
    _check(load().semicrf_entropies(_ptr(pos_marg, torch.float32), _ptr(bdy_post, torch.float32),
                                    _ptr(lengths, torch.int32), B, T, C, h_pos.data_ptr(), h_bdy.data_ptr(),
                                    _stream()))
    return h_pos, h_bdy


def semicrf_scan_report(workspace, B, T, K, C, ckpt_interval=0, want_grad=True):
    """Returns (accepted [B,2] int32, mismatch [B,2] float64) of the last call on `workspace`."""
    acc = torch.empty((B, 2), dtype=torch.int32, device=workspace.device)
    mis = torch.empty((B, 2), dtype=torch.float64, device=workspace.device)
    _check(load().semicrf_scan_report(workspace.data_ptr(), workspace.numel(), B, T, K, C,
                                      ckpt_interval, int(want_grad), acc.data_ptr(),
                                      mis.data_ptr(), _stream()))
    return acc, mis


def semicrf_seq_report(workspace, B, T, K, C, ckpt_interval=0, want_grad=True):
    """Returns (range_exceeded [B] int32, logz64 [B] float64) of the last call on `workspace`."""
    rng = torch.empty(B, dtype=torch.int32, device=workspace.device)
    lz = torch.empty(B, dtype=torch.float64, device=workspace.device)
    _check(load().semicrf_seq_report(workspace.data_ptr(), workspace.numel(), B, T, K, C,
                                     ckpt_interval, int(want_grad), rng.data_ptr(), lz.data_ptr(), _stream()))
    return rng, lz


_hip = None


def _hiprt():
    """The HIP runtime, for the event handles the profiled entry point records."""
    global _hip
    if _hip is None:
        hip = ctypes.CDLL("libamdhip64.so")
        hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
        hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
        hip.hipEventDestroy.argtypes = [ctypes.c_void_p]
        _hip = hip
    return _hip


class StageEvents:
    """Five HIP events for one call of semicrf_fwd_bwd_profiled."""

    def __init__(self):
        hip = _hiprt()
        self.arr = (ctypes.c_void_p * 5)()
        for i in range(5):
            ev = ctypes.c_void_p()
            if hip.hipEventCreate(ctypes.byref(ev)) != 0:
                raise RuntimeError("hipEventCreate failed")
            self.arr[i] = ev

    def stage_ms(self):
        """Elapsed ms of the four stages; the stream must have been synchronised."""
        hip = _hiprt()
        out = []
        for i in range(4):
            ms = ctypes.c_float(0)
            if hip.hipEventElapsedTime(ctypes.byref(ms), self.arr[i], self.arr[i + 1]) != 0:
                raise RuntimeError("hipEventElapsedTime failed")
            out.append(ms.value)
        return out

    def destroy(self):
        hip = _hiprt()
        for i in range(5):
            hip.hipEventDestroy(self.arr[i])


def semicrf_fwd_bwd_profiled(emis, lengths, trans, dur, events, grad_logz=None, ckpt_interval=0,
                             flags=SEMICRF_CENTER, workspace=None, out=None):
    """semicrf_fwd_bwd that also records `events` (a StageEvents) on the stream."""
    B, T, C = emis.shape
    K = dur.shape[0]
    dev = emis.device
    if workspace is None:
        workspace = alloc_workspace(B, T, K, C, ckpt_interval, grad_workspace_kind(flags), dev)
    if out is None:
        out = (torch.empty(B, dtype=torch.float32, device=dev),
               torch.empty((B, T, C), dtype=torch.float32, device=dev),
               torch.empty((C, C), dtype=torch.float32, device=dev),
               torch.empty((K, C), dtype=torch.float32, device=dev),
               torch.empty((B, T, C), dtype=torch.float32, device=dev))
    logz, g_e, g_t, g_d, pm = out
    ep, flags = _emis(emis, flags)
    _check(load().semicrf_fwd_bwd_profiled(
        ep, _ptr(lengths, torch.int32), _ptr(trans, torch.float32),
        _ptr(dur, torch.float32), _ptr(grad_logz, torch.float32), B, T, K, C, ckpt_interval, flags,
        workspace.data_ptr(), workspace.numel(), _ptr(logz, torch.float32),
        _ptr(g_e, torch.float32), _ptr(g_t, torch.float32), _ptr(g_d, torch.float32),
        _ptr(pm, torch.float32), _stream(), events.arr))
    return out
