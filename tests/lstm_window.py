"""Step-by-step gate for a recurrent run of several steps whose intermediate states cannot be read out.

A device run of n steps returns only (h_n, c_n).  Runs are bit-reproducible, so the run of n steps passes through
exactly the state the run of n-1 steps returned; the oracle therefore takes ONE step from the device's own state
after n-1 steps and the device's state after n steps has to lie within the one-step bound of it.  Every step of
the window is gated at the per-step tolerance, with no accumulation of bounds, and a step that consumed anything
but the previous step's state (a stale buffer, a partial sum of another step) fails at that step.

One-step bound (gate pre-activations z within tol*D of the oracle's, D = |W||[h;x]| + |b|; sigmoid is
1/4-Lipschitz, tanh 1-Lipschitz, |tanh| <= 1, sigmoid <= 1):
    |dc| <= tol*(D_f |c_prev| / 4 + D_i / 4 + D_g) + slack,    |dh| <= tol*D_o / 4 + |dc| + slack,
slack = 1e-5 for the device's fp32 exponentials."""
import numpy as np

from oracle import pivot_oracle as O


def one_step_bounds(D, c_prev, H, tol, slack=1e-5):
    Di, Df, Dg, Do = D[:, :H], D[:, H:2 * H], D[:, 2 * H:3 * H], D[:, 3 * H:]
    bc = tol * (Df * np.abs(c_prev) / 4 + Di / 4 + Dg) + slack
    bh = tol * Do / 4 + bc + slack
    return bh, bc


def chained_window_check(run, Wd, bias, xs, h0, c0, H, state_dtype, tol, n_max):
    """run(n) -> (h, c) as float arrays [batch][H]: the device's state after n steps from (h0, c0) on inputs
    xs[:n].  Returns the list of (n, worst |dh| / bound, worst |dc| / bound); raises AssertionError naming the
    first step that is out of bounds."""
    h_prev = np.asarray(h0, dtype=np.float32)
    c_prev = np.asarray(c0, dtype=np.float32)
    report = []
    for n in range(1, n_max + 1):
        h_dev, c_dev = run(n)
        h_fed = h_prev.astype(state_dtype)                       # what step n consumed: the stored state, rounded once
        z_ref, h_ref, c_ref, D = O.oracle_lstm_step(Wd, bias, h_fed, xs[n - 1], c_prev.astype(np.float64), H)
        bh, bc = one_step_bounds(D, c_prev.astype(np.float64), H, tol)
        rc = float(np.max(np.abs(c_dev - c_ref) / bc))
        rh = float(np.max(np.abs(h_dev - h_ref) / bh))
        report.append((n, rh, rc))
        assert rc <= 1.0, "step %d of the window: cell state off by %.3g of its one-step bound" % (n, rc)
        assert rh <= 1.0, "step %d of the window: hidden state off by %.3g of its one-step bound" % (n, rh)
        h_prev, c_prev = np.asarray(h_dev, dtype=np.float32), np.asarray(c_dev, dtype=np.float32)
    return report
