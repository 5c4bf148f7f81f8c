"""Parity of layer chains (composed / eliminated boundary permutations) and of
the recurrent loop with the CPU oracle.  Needs a GPU."""
import numpy as np
import pytest
import torch

from oracle import pivot_oracle as O
from paper_1712_01084_amd import binding as B
from paper_1712_01084_amd import workloads as WL

import gpu_util as G
import lstm_window as LW

pytestmark = pytest.mark.gpu


def _layers(probs):
    return [dict(Wp=p.Wp, tile_mask=p.tile_mask, prow=p.prow, pcol=p.pcol, bias=p.bias, bh=p.bh, bw=p.bw, act=p.act)
            for p in probs]


def _run_chain(probs, flags=0, chunk_tiles=0, repeats=2, want_one_launch=None):
    plans = [G.dev_plan(p, chunk_tiles=chunk_tiles) for p in probs]
    mlp = B.pivot_mlp_plan(plans, flags)
    try:
        view = B.pivot_mlp_plan_host_view(mlp, [B.pivot_fc_plan_host_view(h) for h in plans])
        if want_one_launch is not None:
            assert view["one_launch"] == int(want_one_launch)
        x = probs[0].x
        batch = x.shape[0]
        xd = torch.from_numpy(x).cuda()
        keep = bool(flags & B.PIVOT_MLP_KEEP_FINAL_BLOCK_ORDER)
        last = probs[-1]
        ncols = last.nbr * last.bh if keep else last.M
        ws = G.workspace(B.pivot_mlp_workspace_bytes(mlp, batch))
        st = torch.cuda.current_stream().cuda_stream
        outs = []
        for _ in range(repeats):
            yd = torch.full((batch, ncols), float("nan"), dtype=torch.float32, device="cuda")
            B.pivot_mlp_run(mlp, xd.data_ptr(), probs[0].K, yd.data_ptr(), ncols, batch, ws.data_ptr(), ws.numel(), st)
            torch.cuda.synchronize()
            outs.append(yd.cpu().numpy())
        assert outs[0].tobytes() == outs[-1].tobytes()
        assert B.pivot_mlp_status(mlp, st) == 0
        y = outs[0].astype(np.float64)
        if keep:                                   # host relabels with prow of the last layer (Section 4.2.2)
            nat = np.empty((batch, last.M))
            nat[:, last.prow] = y[:, :last.M]
            y = nat
        return y
    finally:
        B.pivot_mlp_plan_destroy(mlp)
        for h in plans:
            B.pivot_fc_plan_destroy(h)


def _check_chain(probs, flags=0, chunk_tiles=0, want_one_launch=None, repeats=2):
    y = _run_chain(probs, flags=flags, chunk_tiles=chunk_tiles, want_one_launch=want_one_launch, repeats=repeats)
    bd = np.float16 if probs[0].wdtype == WL.F16 else None
    outs, scales, chain = O.oracle_mlp(_layers(probs), probs[0].x, boundary_dtype=bd, return_all=True)
    assert not np.isnan(y).any()
    # gate: a relative error of tol in EVERY layer, propagated to the output (chain scale S_L, see the oracle);
    # also reported against the last layer's own scale D_L = |W_L||h_{L-1}| + |b_L|, which an error made in an
    # earlier layer may legitimately exceed
    err = O.max_scaled_error(y, outs[-1], chain[-1])
    err_d = O.max_scaled_error(y, outs[-1], scales[-1])
    assert err <= G.TOL[probs[0].wdtype], err
    return err, err_d


@pytest.mark.parametrize("eliminated", [False, True])
@pytest.mark.parametrize("wdtype", [WL.F32, WL.F16])
@pytest.mark.parametrize("batch", [1, 3])
def test_small_chain(eliminated, wdtype, batch):
    probs = WL.config4(seed=5, batch=batch, dims=(200, 96, 128, 40), eliminated=eliminated, wdtype=wdtype)
    _check_chain(probs, chunk_tiles=2)
    _check_chain(probs, flags=B.PIVOT_MLP_KEEP_FINAL_BLOCK_ORDER)


def test_single_layer_chain_equals_fc_run():
    probs = WL.config4(seed=6, dims=(96, 72))
    _check_chain(probs)


def test_fp16_chain_batch16_uses_matrix_cores():
    probs = WL.config4(seed=7, batch=16, dims=(256, 128, 96), wdtype=WL.F16)
    _check_chain(probs, chunk_tiles=2)


@pytest.mark.parametrize("seed", [0, 1, 2])
@pytest.mark.parametrize("eliminated", [False, True])
def test_config4_full(eliminated, seed):
    probs = WL.config4(seed=seed, eliminated=eliminated)
    for flags, one in ((0, True), (B.PIVOT_MLP_LAUNCH_PER_LAYER, False)):
        err, err_d = _check_chain(probs, flags=flags, want_one_launch=one)
        print("config4 seed %d eliminated=%s %s: error / S_L %.3g, error / D_L %.3g"
              % (seed, eliminated, "one launch" if one else "launch per layer", err, err_d), flush=True)
        assert err_d <= 1e-5          # fp32: also within the tolerance on the last layer's own scale


@pytest.mark.parametrize("eliminated", [False, True])
@pytest.mark.parametrize("bh,bw,dims", [(32, 32, (300, 200, 136, 70)), (16, 16, (100, 90, 50)), (8, 64, (260, 72, 40, 24, 130)),
                                        (64, 16, (150, 190, 64)), (16, 32, (96, 64, 48)),
                                        (32, 32, (200, 256, 64, 256, 40)),     # workgroups 2-7 have no item in the narrow layer
                                        (32, 32, (64, 2048, 40)), (16, 16, (40, 1500, 1200, 30)),    # later layers whose wavefronts stage more than 64 elements
                                        (16, 16, (100, 32, 300)),              # most workgroups have no item in the first layer
                                        (16, 32, (64, 300, 40, 130))])         # ... none in the middle layer
@pytest.mark.parametrize("wdtype", [WL.F32, WL.F16])
def test_one_launch_chain_batch1(wdtype, eliminated, bh, bw, dims):
    # chains whose work items are whole block rows run at batch 1 in ONE launch: intermediates travel as
    # (value, launch tag) pairs.  Ragged M and K (padding rows are never stored, padding columns never waited
    # for), several tile shapes, 2 to 5 layers, both boundary variants, five launches in a row (a tag per launch)
    probs = WL.config4(seed=21 + bh, dims=dims, eliminated=eliminated, bh=bh, bw=bw, frac=0.4, wdtype=wdtype)
    _check_chain(probs, want_one_launch=True, repeats=5)
    _check_chain(probs, flags=B.PIVOT_MLP_KEEP_FINAL_BLOCK_ORDER, want_one_launch=True)
    y1 = _run_chain(probs, want_one_launch=True)
    y2 = _run_chain(probs, flags=B.PIVOT_MLP_LAUNCH_PER_LAYER, want_one_launch=False)
    bd = np.float16 if wdtype == WL.F16 else None
    outs, scales, chain = O.oracle_mlp(_layers(probs), probs[0].x, boundary_dtype=bd, return_all=True)
    assert O.max_scaled_error(y1, y2, chain[-1]) <= 2 * G.TOL[wdtype]


def test_one_launch_chain_long_first_input_copied_into_lds():
    # a first layer whose work items stream more than 48 KB copies x into LDS whole and gathers from there;
    # an x that is not 16-byte aligned takes the element gather instead, with the same result
    probs = WL.config4(seed=33, dims=(4096, 64, 48), frac=0.5)
    _check_chain(probs, want_one_launch=True, repeats=3)
    plans = [G.dev_plan(p) for p in probs]
    mlp = B.pivot_mlp_plan(plans, 0)
    try:
        st = torch.cuda.current_stream().cuda_stream
        ws = G.workspace(B.pivot_mlp_workspace_bytes(mlp, 1))
        outs = []
        for off in (0, 1):
            buf = torch.zeros(probs[0].K + 4, dtype=torch.float32, device="cuda")
            buf[off:off + probs[0].K] = torch.from_numpy(probs[0].x[0]).cuda()
            yd = torch.full((1, probs[-1].M), float("nan"), dtype=torch.float32, device="cuda")
            B.pivot_mlp_run(mlp, buf.data_ptr() + 4 * off, probs[0].K, yd.data_ptr(), probs[-1].M, 1, ws.data_ptr(), ws.numel(), st)
            torch.cuda.synchronize()
            outs.append(yd.cpu().numpy())
        assert B.pivot_mlp_status(mlp, st) == 0
        assert outs[0].tobytes() == outs[1].tobytes()      # same arithmetic in the same order
    finally:
        B.pivot_mlp_plan_destroy(mlp)
        for h in plans:
            B.pivot_fc_plan_destroy(h)


def test_one_launch_chain_in_a_replayed_graph():
    # the launch tag comes from a counter in device memory, so a captured launch gets a fresh tag on every
    # replay with no host work: several replays, eager work in between, every result equal to the eager one
    import bench_util as BU
    probs = WL.config4(seed=34, dims=(520, 256, 96, 40), frac=0.4)
    plans = [G.dev_plan(p) for p in probs]
    mlp = B.pivot_mlp_plan(plans, 0)
    try:
        xd = torch.from_numpy(probs[0].x).cuda()
        ws = G.workspace(B.pivot_mlp_workspace_bytes(mlp, 1))
        yd = torch.full((1, probs[-1].M), float("nan"), dtype=torch.float32, device="cuda")

        def enqueue(i, s):
            B.pivot_mlp_run(mlp, xd.data_ptr(), probs[0].K, yd.data_ptr(), probs[-1].M, 1, ws.data_ptr(), ws.numel(), s)

        st = torch.cuda.current_stream().cuda_stream
        enqueue(0, st)
        torch.cuda.synchronize()
        eager = yd.cpu().numpy().copy()
        g = BU.capture(enqueue, 3)
        for _ in range(4):
            yd.fill_(float("nan"))
            torch.cuda.synchronize()
            g.replay()
            torch.cuda.synchronize()
            assert yd.cpu().numpy().tobytes() == eager.tobytes()
            enqueue(0, st)                                  # an eager launch between replays
            torch.cuda.synchronize()
        assert B.pivot_mlp_status(mlp, st) == 0
        outs, scales, chain = O.oracle_mlp(_layers(probs), probs[0].x, return_all=True)
        assert O.max_scaled_error(eager.astype(np.float64), outs[-1], chain[-1]) <= G.TOL[WL.F32]
    finally:
        B.pivot_mlp_plan_destroy(mlp)
        for h in plans:
            B.pivot_fc_plan_destroy(h)


def test_one_launch_chain_degenerate_layers():
    # a middle layer without any kept tile (its outputs are relu(b), still tagged and waited for), an output
    # layer narrower than one tile, and a block row without tiles in the first layer
    probs = WL.config4(seed=35, dims=(200, 96, 130, 5), frac=0.4)
    probs[1].tile_mask[:] = 0
    probs[0].tile_mask[1, :] = 0
    _check_chain(probs, want_one_launch=True, repeats=3)
    _check_chain(probs, flags=B.PIVOT_MLP_LAUNCH_PER_LAYER, want_one_launch=False)


def test_one_launch_chain_falls_back():
    # split block rows and batch > 1 keep one launch per layer
    probs = WL.config4(seed=30, dims=(200, 96, 128), eliminated=False, frac=0.6)
    _check_chain(probs, chunk_tiles=1, want_one_launch=False)
    probs3 = WL.config4(seed=32, batch=3, dims=(200, 96, 128))
    _check_chain(probs3)                                  # one_launch plan, batch 3: per-layer launches
    wide = WL.config4(seed=36, dims=(64, 40000, 32), frac=0.5)
    _check_chain(wide, want_one_launch=False)             # 1250 block rows: more work items than the form takes


@pytest.mark.parametrize("wdtype", [WL.F32, WL.F16])
def test_chain_workspace_reused_across_batch_sizes(wdtype):
    # one workspace, cleared once, shared by runs of different batch sizes: ragged widths (padding columns in every
    # intermediate), split block rows in every layer, fp16 at batch 16 through the kernel that reads its inputs
    # straight from the block-order rows; each run is preceded by one of the same batch on NaN inputs
    probs = WL.config4(seed=41, batch=16, dims=(203, 100, 77, 40), wdtype=wdtype, bh=32, bw=32, frac=0.6)
    plans = [G.dev_plan(p, chunk_tiles=1) for p in probs]
    mlp = B.pivot_mlp_plan(plans, 0)
    try:
        batches = (16, 1, 5, 1, 9, 3)
        ws = G.workspace(max(B.pivot_mlp_workspace_bytes(mlp, b) for b in batches))
        st = torch.cuda.current_stream().cuda_stream
        bd = np.float16 if wdtype == WL.F16 else None
        for b in batches:
            x = np.ascontiguousarray(probs[0].x[:b])
            for poison in (True, False):
                xd = torch.from_numpy(np.full_like(x, np.nan) if poison else x).cuda()
                yd = torch.full((b, probs[-1].M), float("nan"), dtype=torch.float32, device="cuda")
                B.pivot_mlp_run(mlp, xd.data_ptr(), probs[0].K, yd.data_ptr(), probs[-1].M, b, ws.data_ptr(), ws.numel(), st)
                torch.cuda.synchronize()
            outs, scales, chain = O.oracle_mlp(_layers(probs), x, boundary_dtype=bd, return_all=True)
            y = yd.cpu().numpy().astype(np.float64)
            assert not np.isnan(y).any(), ("batch", b)
            assert O.max_scaled_error(y, outs[-1], chain[-1]) <= G.TOL[wdtype], ("batch", b)
    finally:
        B.pivot_mlp_plan_destroy(mlp)
        for h in plans:
            B.pivot_fc_plan_destroy(h)


def test_chain_padding_columns_of_a_directly_read_intermediate_are_cleared():
    # second layer: 3100 inputs (3104 with padding) in whole block rows of 97 tiles, batch 24: too long to stage
    # in LDS (and past the 16 rows of the form that copies x there), so the matrix-core kernel reads its B fragments
    # straight from the intermediate's rows, padding columns included; a first run on another batch size leaves
    # NaN where those columns are
    probs = WL.config4(seed=43, batch=24, dims=(64, 3100, 40), wdtype=WL.F16, bh=32, bw=32, frac=1.0)
    plans = [G.dev_plan(p, chunk_tiles=97) for p in probs]
    mlp = B.pivot_mlp_plan(plans, 0)
    try:
        assert B.pivot_fc_workspace_bytes(plans[1], 24) > 0      # whole rows: all of it is the block-order copy
        ws = G.workspace(max(B.pivot_mlp_workspace_bytes(mlp, b) for b in (64, 24)))
        st = torch.cuda.current_stream().cuda_stream
        for b, poison in ((64, True), (24, False)):
            x = np.full((b, 64), np.nan, dtype=np.float16) if poison else probs[0].x
            xd = torch.from_numpy(x).cuda()
            yd = torch.full((b, probs[-1].M), float("nan"), dtype=torch.float32, device="cuda")
            B.pivot_mlp_run(mlp, xd.data_ptr(), 64, yd.data_ptr(), probs[-1].M, b, ws.data_ptr(), ws.numel(), st)
            torch.cuda.synchronize()
        outs, scales, chain = O.oracle_mlp(_layers(probs), probs[0].x, boundary_dtype=np.float16, return_all=True)
        y = yd.cpu().numpy().astype(np.float64)
        assert not np.isnan(y).any()
        assert O.max_scaled_error(y, outs[-1], chain[-1]) <= G.TOL[WL.F16]
    finally:
        B.pivot_mlp_plan_destroy(mlp)
        for h in plans:
            B.pivot_fc_plan_destroy(h)


# ------------------------------------------------------------------------ LSTM

# max |dh|, |dc| of a free run against the oracle's trajectory: about ten times the largest value measured over all
# cases here (2.3e-5 on the small shapes, 4.8e-6 over the 256 steps of the full workload; see the printed lines);
# no bound follows from the per-step tolerance.  WINDOW_GATE: the same for the worst step of a window, as a
# fraction of the one-step bound at the 2e-3 tolerance (measured: at most 3.8e-3 of it)
FREE_RUN_GATE = 2e-4
WINDOW_GATE = 0.04


def _lstm_gpu(lp, plan, xs, h, c, want_z=True):
    steps, batch = xs.shape[0], xs.shape[1]
    H, I = lp.H, lp.I
    xsd = torch.from_numpy(np.ascontiguousarray(xs)).cuda()
    hd = torch.from_numpy(np.ascontiguousarray(h, dtype=np.float32)).cuda()
    cd = torch.from_numpy(np.ascontiguousarray(c, dtype=np.float32)).cuda()
    zd = torch.full((batch, 4 * H), float("nan"), dtype=torch.float32, device="cuda")
    ws = G.workspace(B.pivot_lstm_workspace_bytes(plan, H, I, steps, batch))
    st = torch.cuda.current_stream().cuda_stream
    B.pivot_lstm_run(plan, H, I, xsd.data_ptr(), hd.data_ptr(), cd.data_ptr(), zd.data_ptr() if want_z else None,
                     steps, batch, ws.data_ptr(), ws.numel(), st)
    assert B.pivot_lstm_status(plan, steps, batch, ws.data_ptr(), st) == 0      # also synchronises
    torch.cuda.synchronize()
    return hd.cpu().numpy().astype(np.float64), cd.cpu().numpy().astype(np.float64), zd.cpu().numpy().astype(np.float64)


def _check_lstm_steps(lp, record, tol, per_step=False, windows=(), window_len=12):
    # per_step=False: the library's choice (one launch for the whole sequence where the plan allows it);
    # per_step=True: one layer launch and one cell launch per step
    p = lp.fc
    Wd = O.dense_masked_natural(p.Wp, p.tile_mask, p.prow, p.pcol, p.bh, p.bw)
    sd = np.float16 if p.wdtype == WL.F16 else np.float32
    h_end, c_end, rec = O.oracle_lstm(Wd, p.bias, lp.xs, lp.h0, lp.c0, lp.H, state_dtype=sd,
                                      record=tuple(record) + tuple(windows))
    # (ONE_LAUNCH_ALWAYS: the single steps and the short windows below are to exercise the one-launch kernel too,
    # which the library otherwise takes from 4 steps on)
    plan = G.dev_plan(p, flags=B.PIVOT_PLAN_LSTM_LAUNCH_PER_STEP if per_step else B.PIVOT_PLAN_LSTM_ONE_LAUNCH_ALWAYS)
    try:
        H = lp.H
        for t in record:
            # one step from the oracle's state (both sides consume the same rounded values)
            h_fed = rec[t]["h_fed"].astype(np.float32)
            c_prev = rec[t]["c_prev"].astype(np.float32)
            z_ref, h_ref, c_ref, D = O.oracle_lstm_step(Wd, p.bias, h_fed.astype(sd), lp.xs[t], c_prev, H)
            h, c, z = _lstm_gpu(lp, plan, lp.xs[t:t + 1], h_fed, c_prev)
            assert O.max_scaled_error(z, z_ref, D) <= tol, ("z", t)
            bh, bc = LW.one_step_bounds(D, c_prev.astype(np.float64), H, tol)
            assert np.all(np.abs(c - c_ref) <= bc), ("c", t)
            assert np.all(np.abs(h - h_ref) <= bh), ("h", t)
        # windows of several steps inside ONE run, from the oracle's state at t0: every step gated at the one-step
        # bound against the oracle stepping from the device's own previous state (see lstm_window.py), and the
        # end of the window against the oracle's own trajectory from the same state
        for t0 in windows:
            n_max = min(window_len, lp.xs.shape[0] - t0)
            h0 = rec[t0]["h_fed"].astype(np.float32)
            c0 = rec[t0]["c_prev"].astype(np.float32)
            xs = lp.xs[t0:t0 + n_max]

            def run(n):
                h, c, _ = _lstm_gpu(lp, plan, xs[:n], h0, c0, want_z=False)
                return h, c
            rep = LW.chained_window_check(run, Wd, p.bias, xs, h0, c0, H, sd, tol, n_max)
            assert max(max(r[1], r[2]) for r in rep) <= WINDOW_GATE
            h_w, c_w, _ = O.oracle_lstm(Wd, p.bias, xs, h0, c0.astype(np.float64), H, state_dtype=sd)
            h, c = run(n_max)
            print("lstm window t0=%d, %d steps: worst step at %.3g / %.3g of the one-step bound; end of window vs "
                  "oracle trajectory |dh| %.3g |dc| %.3g" % (t0, n_max, max(r[1] for r in rep), max(r[2] for r in rep),
                                                             np.abs(h - h_w).max(), np.abs(c - c_w).max()), flush=True)
        # free-running trajectory against the oracle's: reported, and gated by the caller at a few times what
        # was measured (no bound follows from the per-step tolerance: the recurrence can amplify)
        h, c, _ = _lstm_gpu(lp, plan, lp.xs, lp.h0, lp.c0, want_z=False)
        h2, c2, _ = _lstm_gpu(lp, plan, lp.xs, lp.h0, lp.c0, want_z=False)
        assert np.array_equal(h, h2) and np.array_equal(c, c2)          # fixed summation order: bit-identical reruns
        dh, dc = float(np.abs(h - h_end).max()), float(np.abs(c - c_end).max())
        print("lstm free run %d steps: max|dh| = %.3g, max|dc| = %.3g" % (lp.xs.shape[0], dh, dc), flush=True)
        assert np.isfinite(h).all() and np.isfinite(c).all()
        return dh, dc
    finally:
        B.pivot_fc_plan_destroy(plan)


@pytest.mark.parametrize("per_step", [False, True])
@pytest.mark.parametrize("batch", [1, 2, 8])
def test_lstm_small(batch, per_step):
    lp = WL.config5(seed=3, batch=batch, H=64, I=32, steps=14, frac=0.5)
    lp.h0 = np.random.default_rng(1).standard_normal(lp.h0.shape).astype(np.float32) * 0.5
    lp.c0 = np.random.default_rng(2).standard_normal(lp.c0.shape).astype(np.float32)
    dh, dc = _check_lstm_steps(lp, record=(0, 1, 5), tol=2e-3, per_step=per_step, windows=(0, 2))
    assert dh < FREE_RUN_GATE and dc < FREE_RUN_GATE


@pytest.mark.parametrize("H,I,batch,frac", [(96, 40, 3, 0.3), (256, 128, 16, 0.2), (80, 8, 5, 1.0),
                                             (1024, 512, 8, 0.8),     # 10 tiles per wavefront: the 16-slot kernel
                                             (512, 256, 4, 0.5)])     # fewer workgroups than compute units
def test_lstm_one_launch_ragged_shapes(H, I, batch, frac):
    # K = H+I not a multiple of the tile width (padding columns), empty and split block rows, every tile kept
    lp = WL.config5(seed=5, batch=batch, H=H, I=I, steps=13, frac=frac)
    lp.h0 = np.random.default_rng(3).standard_normal(lp.h0.shape).astype(np.float32) * 0.5
    lp.c0 = np.random.default_rng(4).standard_normal(lp.c0.shape).astype(np.float32)
    dh, dc = _check_lstm_steps(lp, record=(0, 3, 8), tol=2e-3, windows=(0, 1))
    assert dh < FREE_RUN_GATE and dc < FREE_RUN_GATE


def test_lstm_short_sequences_take_the_launch_per_step_form():
    # fewer than 4 steps: the library runs a launch per step even where the one-launch form exists (same bits as
    # the plan that asks for launches per step); PIVOT_PLAN_LSTM_ONE_LAUNCH_ALWAYS keeps the one-launch kernel,
    # whose fixed summation order is another one (same values within the tolerance); from 4 steps on the default
    # is the one-launch form
    lp = WL.config5(seed=9, batch=8, H=256, I=128, steps=8, frac=0.25)
    res = {}
    for name, flags in (("default", 0), ("per_step", B.PIVOT_PLAN_LSTM_LAUNCH_PER_STEP), ("one_launch", B.PIVOT_PLAN_LSTM_ONE_LAUNCH_ALWAYS)):
        plan = G.dev_plan(lp.fc, flags=flags)
        try:
            res[name] = {n: _lstm_gpu(lp, plan, lp.xs[:n], lp.h0, lp.c0, want_z=True) for n in (1, 2, 3, 4)}
        finally:
            B.pivot_fc_plan_destroy(plan)
    for n in (1, 2, 3):
        for a, b in zip(res["default"][n], res["per_step"][n]):
            assert np.array_equal(a, b), n
        assert np.abs(res["default"][n][0] - res["one_launch"][n][0]).max() < 2e-3
    for a, b in zip(res["default"][4], res["one_launch"][4]):
        assert np.array_equal(a, b)


def test_lstm_one_launch_agrees_with_launch_per_step():
    lp = WL.config5(seed=7, batch=8, H=256, I=128, steps=20, frac=0.25)
    outs = []
    for flags in (0, B.PIVOT_PLAN_LSTM_LAUNCH_PER_STEP):
        plan = G.dev_plan(lp.fc, flags=flags)
        try:
            outs.append(_lstm_gpu(lp, plan, lp.xs, lp.h0, lp.c0, want_z=True))
        finally:
            B.pivot_fc_plan_destroy(plan)
    (h1, c1, z1), (h2, c2, z2) = outs
    # same inputs, same rounding points, different (fixed) summation orders
    assert np.abs(h1 - h2).max() < 2e-3 and np.abs(c1 - c2).max() < 4e-3 and np.abs(z1 - z2).max() < 2e-2


@pytest.mark.parametrize("seed", [0, 1, 2])
@pytest.mark.parametrize("per_step", [False, True])
def test_lstm_config5_full(per_step, seed):
    # single steps from the oracle's state, three 12-step windows inside one run (the one-launch form's step-to-step
    # exchange: marks, the rotation through eight partial buffers, the progress check from step 8 on), and the
    # 256-step free run
    lp = WL.config5(seed=seed)
    dh, dc = _check_lstm_steps(lp, record=(0, 1, 17, 255), tol=2e-3, per_step=per_step,
                               windows=(0, 100, 240) if seed == 0 or not per_step else (100,))
    assert dh < FREE_RUN_GATE and dc < FREE_RUN_GATE


def test_status_words_can_be_read_without_the_synchronising_calls():
    # the device address of each one-launch form's status word: copied back here with a plain hipMemcpy issued by
    # the test itself (a caller may equally read it from a kernel or an asynchronous copy behind the run)
    import ctypes
    hip = ctypes.CDLL("libamdhip64.so")
    hip.hipMemcpy.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int]

    def read_word(addr):
        w = ctypes.c_uint32(0xFFFFFFFF)
        assert hip.hipMemcpy(ctypes.byref(w), ctypes.c_void_p(addr), 4, 2) == 0      # device to host
        return w.value

    probs = WL.config4(seed=37, dims=(300, 200, 70), frac=0.4)
    plans = [G.dev_plan(p) for p in probs]
    st = torch.cuda.current_stream().cuda_stream
    for flags in (0, B.PIVOT_MLP_LAUNCH_PER_LAYER):
        mlp = B.pivot_mlp_plan(plans, flags)
        try:
            addr = B.pivot_mlp_status_word(mlp)
            assert (addr != 0) == (flags == 0)
            xd = torch.from_numpy(probs[0].x).cuda()
            yd = torch.empty((1, probs[-1].M), dtype=torch.float32, device="cuda")
            ws = G.workspace(B.pivot_mlp_workspace_bytes(mlp, 1))
            B.pivot_mlp_run(mlp, xd.data_ptr(), probs[0].K, yd.data_ptr(), probs[-1].M, 1, ws.data_ptr(), ws.numel(), st)
            torch.cuda.synchronize()
            if addr:
                assert read_word(addr) == 0
        finally:
            B.pivot_mlp_plan_destroy(mlp)
    for h in plans:
        B.pivot_fc_plan_destroy(h)
    lp = WL.config5(seed=8, batch=4, H=64, I=32, steps=8, frac=0.5)
    plan = G.dev_plan(lp.fc)
    try:
        xsd = torch.from_numpy(lp.xs).cuda()
        hd, cd = torch.from_numpy(lp.h0).cuda(), torch.from_numpy(lp.c0).cuda()
        ws = G.workspace(B.pivot_lstm_workspace_bytes(plan, lp.H, lp.I, 8, 4))
        B.pivot_lstm_run(plan, lp.H, lp.I, xsd.data_ptr(), hd.data_ptr(), cd.data_ptr(), None, 8, 4, ws.data_ptr(), ws.numel(), st)
        torch.cuda.synchronize()
        addr = B.pivot_lstm_status_word(plan, 8, 4, ws.data_ptr())
        assert ws.data_ptr() <= addr < ws.data_ptr() + ws.numel() and read_word(addr) == 0
        assert B.pivot_lstm_status(plan, 8, 4, ws.data_ptr(), st) == 0
    finally:
        B.pivot_fc_plan_destroy(plan)


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_random_chains_match_the_oracle(seed):
    # depth, widths, tile shape, weight type, batch, boundary variant, flags and chunking drawn together; whichever
    # form the library picks (one launch or one launch per layer) has to agree with the oracle
    rng = np.random.default_rng(seed)
    for it in range(12):
        depth = int(rng.integers(1, 6))
        bh = int(rng.choice([8, 16, 32, 64]))
        bw = int(rng.choice([8, 16, 32, 64]))
        dims = tuple(int(rng.integers(1, 500)) for _ in range(depth + 1))
        wdtype = WL.F32 if rng.random() < 0.5 else WL.F16
        batch = int(rng.choice([1, 1, 1, 2, 4, 9]))
        elim = bool(rng.random() < 0.5)
        flags = int(rng.choice([0, 0, B.PIVOT_MLP_KEEP_FINAL_BLOCK_ORDER, B.PIVOT_MLP_LAUNCH_PER_LAYER]))
        ct = int(rng.choice([0, 0, 1, 3]))
        frac = float(rng.choice([0.2, 0.5, 1.0]))
        print("chain dims %s tiles %dx%d %s batch %d eliminated=%s flags %d chunk_tiles %d kept %.1f"
              % (dims, bh, bw, wdtype, batch, elim, flags, ct, frac), flush=True)
        probs = WL.config4(seed=700 + 20 * seed + it, batch=batch, dims=dims, eliminated=elim, wdtype=wdtype,
                           bh=bh, bw=bw, frac=frac)
        _check_chain(probs, flags=flags, chunk_tiles=ct)
