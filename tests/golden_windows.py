"""Element-wise check of the stored windows of the full-size fixtures (tests/golden/make_golden.py)."""
import numpy as np
import torch

def check_windows(g, interval_now, pm, g_e):
    """The stored windows (rows around interval boundaries and scaling-block boundaries), element by element."""
    assert interval_now == int(g["interval"][0]), "the planner's interval changed: run tests/golden/make_golden.py again"
    win = g["windows"]
    on_boundary = sum(1 for b, lo, n in win if any((lo + i) % interval_now == 0 for i in range(1, n)))
    assert on_boundary >= 8 and len(win) >= 12
    pmw = torch.cat([pm[int(b), int(lo):int(lo + n)] for b, lo, n in win]).double().cpu().numpy()
    gew = torch.cat([g_e[int(b), int(lo):int(lo + n)] for b, lo, n in win]).double().cpu().numpy()
    e1 = np.abs(pmw - g["pos_marg_windows"]).max()
    e2 = np.abs(gew - g["grad_emis_windows"]).max()
    print(f"       {len(pmw)} rows in {len(win)} windows around interval / scaling-block boundaries: "
          f"pos_marg {e1:.2e} grad_emis {e2:.2e}", flush=True)
    assert e1 <= 1e-4 and e2 <= 1e-4
