"""GPU test of the allocation-free entry point semicrf_fwd_bwd_static.

It must give what semicrf_fwd_bwd gives (same kernels, the workspace in the library's static
array instead of a caller buffer) on two calls in a row, the second with a smaller input, and
refuse sizes whose workspace does not fit the static array.  Collected last on purpose.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2604_18780_amd import binding as sb
from paper_2604_18780_amd import synth

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def _dev(w):
    return (torch.from_numpy(w.emis).to(DEV), torch.from_numpy(w.lengths).to(DEV),
            torch.from_numpy(w.trans).to(DEV), torch.from_numpy(w.dur).to(DEV))


def _outputs(w):
    f32 = torch.float32
    return (torch.full((w.B,), 7.0, dtype=f32, device=DEV), torch.full((w.B, w.T, w.C), 7.0, dtype=f32, device=DEV),
            torch.full((w.C, w.C), 7.0, dtype=f32, device=DEV), torch.full((w.K, w.C), 7.0, dtype=f32, device=DEV),
            torch.full((w.B, w.T, w.C), 7.0, dtype=f32, device=DEV))


def _compare(w, label):
    print(f"[case] static workspace: {label} B={w.B} T={w.T} K={w.K} C={w.C}", flush=True)
    emis, lengths, trans, dur = _dev(w)
    assert sb.semicrf_workspace_bytes(w.B, w.T, w.K, w.C, 0, True) <= sb.SEMICRF_STATIC_WORKSPACE_BYTES
    out = _outputs(w)
    sb.semicrf_fwd_bwd_static(emis, lengths, trans, dur, out)
    ref = sb.semicrf_fwd_bwd(emis, lengths, trans, dur)
    torch.cuda.synchronize()
    for name, a, b in zip(("logz", "grad_emis", "grad_trans", "grad_dur", "pos_marg"), out, ref):
        # same kernels on the same inputs: bit-equal, which is within every tolerance of the parity tests
        assert torch.equal(a, b), name
    r = oracle.fwd_bwd(w.emis, w.lengths, w.trans, w.dur)
    lz = out[0].double().cpu().numpy()
    assert np.all(np.abs(lz - r.logz) <= 1e-5 * np.maximum(1.0, np.abs(r.logz)))
    assert np.abs(out[4].double().cpu().numpy() - r.pos_marg).max() <= 1e-4
    assert np.abs(out[1].double().cpu().numpy() - r.grad_emis).max() <= 1e-4
    assert np.abs(out[2].double().cpu().numpy() - r.grad_trans).max() <= 1e-4 * max(1.0, np.abs(r.grad_trans).max())
    assert np.abs(out[3].double().cpu().numpy() - r.grad_dur).max() <= 1e-4 * max(1.0, np.abs(r.grad_dur).max())


def test_static_workspace_two_calls_second_smaller():
    _compare(synth.make("nlp", B=8, T=200), "first call")
    _compare(synth.small_random(21, 3, 90, 5, 7, ragged=True), "second call, smaller input")


def test_static_workspace_rejects_sizes_beyond_the_limit():
    B, T, K, C = 4, 100000, 64, 24
    assert sb.semicrf_workspace_bytes(B, T, K, C, 0, True) > sb.SEMICRF_STATIC_WORKSPACE_BYTES
    f32 = torch.float32
    # small stand-in tensors: the call must return before anything is read or launched
    emis = torch.zeros((1, 1, 1), dtype=f32, device=DEV)
    lib = sb.load()
    rc = lib.semicrf_fwd_bwd_static(emis.data_ptr(), None, emis.data_ptr(), emis.data_ptr(), None, B, T, K, C, 0,
                                    sb.SEMICRF_CENTER, emis.data_ptr(), emis.data_ptr(), emis.data_ptr(),
                                    emis.data_ptr(), None, None)
    assert rc == -2, rc
