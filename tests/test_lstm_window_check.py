"""The step-by-step window gate used for the one-launch recurrent kernel, exercised on the CPU: a plain fp32
model of a device run passes it, the same model with a planted exchange mistake (a stale state or stale partial
sums from the buffer rotation) fails it at the step where the mistake first acts."""
import numpy as np
import pytest

from oracle import pivot_oracle as O
from paper_1712_01084_amd import workloads as WL

import lstm_window as LW


def _sig(v):
    return np.float32(1) / (np.float32(1) + np.exp(-v, dtype=np.float32))


def _model_run(Wd32, bias, xs, h0, c0, H, n, bug=None, nbuf=8):
    """n steps in fp32 with the fed-back state rounded to fp16 once per step.  bug = 'stale_state': from step
    nbuf on, rows 0..3 of the batch read the state of nbuf steps ago (a rotating buffer overwritten too late);
    bug = 'stale_partial': from step nbuf on, the first 16 gate rows reuse the sums of nbuf steps ago."""
    h = np.asarray(h0, dtype=np.float32).copy()
    c = np.asarray(c0, dtype=np.float32).copy()
    hist_h, hist_z = [], []
    for t in range(n):
        fed = h.astype(np.float16)
        if bug == "stale_state" and t >= nbuf:
            fed[:4] = hist_h[t - nbuf][:4]
        inp = np.concatenate([fed.astype(np.float32), xs[t].astype(np.float32)], axis=1)
        z = inp @ Wd32.T + bias[None, :].astype(np.float32)
        if bug == "stale_partial" and t >= nbuf:
            z[:, :16] = hist_z[t - nbuf][:, :16]
        hist_h.append(fed.copy())
        hist_z.append(z.copy())
        i, f, g, o = _sig(z[:, :H]), _sig(z[:, H:2 * H]), np.tanh(z[:, 2 * H:3 * H]), _sig(z[:, 3 * H:])
        c = f * c + i * g
        h = o * np.tanh(c)
    return h.astype(np.float64), c.astype(np.float64)


def _problem():
    lp = WL.config5(seed=9, batch=8, H=128, I=64, steps=14, frac=0.3)
    p = lp.fc
    Wd = O.dense_masked_natural(p.Wp, p.tile_mask, p.prow, p.pcol, p.bh, p.bw)
    h0 = (np.random.default_rng(1).standard_normal(lp.h0.shape) * 0.5).astype(np.float32)
    c0 = np.random.default_rng(2).standard_normal(lp.c0.shape).astype(np.float32)
    return lp, p, Wd, h0, c0


def test_faithful_model_passes_the_window_gate():
    lp, p, Wd, h0, c0 = _problem()
    Wd32 = Wd.astype(np.float32)
    rep = LW.chained_window_check(lambda n: _model_run(Wd32, p.bias, lp.xs, h0, c0, lp.H, n), Wd, p.bias, lp.xs, h0, c0,
                                  lp.H, np.float16, 2e-3, 14)
    assert len(rep) == 14 and max(r[1] for r in rep) < 0.1 and max(r[2] for r in rep) < 0.1


@pytest.mark.parametrize("bug", ["stale_state", "stale_partial"])
def test_planted_exchange_mistake_fails_the_window_gate_at_its_first_step(bug):
    lp, p, Wd, h0, c0 = _problem()
    Wd32 = Wd.astype(np.float32)
    with pytest.raises(AssertionError) as e:
        LW.chained_window_check(lambda n: _model_run(Wd32, p.bias, lp.xs, h0, c0, lp.H, n, bug=bug), Wd, p.bias, lp.xs,
                                h0, c0, lp.H, np.float16, 2e-3, 14)
    assert "step 9 of the window" in str(e.value)          # steps 1..8 are untouched; the ninth is the first stale one
    # a free run compared only at the end, at a loose absolute gate, would not have seen it
    h_bug, c_bug = _model_run(Wd32, p.bias, lp.xs, h0, c0, lp.H, 14, bug=bug)
    h_ok, c_ok = _model_run(Wd32, p.bias, lp.xs, h0, c0, lp.H, 14)
    print("end-state difference caused by %s: %.3g / %.3g" % (bug, np.abs(h_bug - h_ok).max(), np.abs(c_bug - c_ok).max()))
