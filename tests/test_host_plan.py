"""Host side of the C-ABI library, no GPU: the library loads, exports every
declared symbol, and its plan builder agrees bit-for-bit with the oracle's
independent builder; error paths return codes and leak nothing."""
import os
import re

import numpy as np
import pytest

from oracle import pivot_oracle as O
from paper_1712_01084_amd import binding as B
from paper_1712_01084_amd import workloads as WL

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

PLAN_ARRAYS = ("row_ptr", "col_idx", "vals", "bias_p", "invprow", "invpcol", "prow_pad", "pcol_pad",
               "chunks", "part_base", "xidx")


def _wd(p):
    return B.PIVOT_F32 if p.wdtype == WL.F32 else B.PIVOT_F16


def _host_plan(p, layout=B.PIVOT_BRC, chunk_tiles=3, natural=False, bias=True):
    W = O.unpivot_weights(p.Wp, p.prow, p.pcol) if natural else p.Wp
    return B.pivot_fc_plan(p.M, p.K, p.bh, p.bw, _wd(p), W,
                           B.PIVOT_W_NATURAL if natural else B.PIVOT_W_PIVOTED,
                           p.tile_mask, p.prow, p.pcol, p.bias if bias else None,
                           layout=layout, act=p.act, chunk_tiles=chunk_tiles, device=-1)


def test_library_exports_every_declared_symbol():
    lib = B.lib()
    assert B.pivot_version() == 100
    header = open(os.path.join(ROOT, "include", "pivot_fc.h")).read()
    declared = set(re.findall(r"\b(pivot_[a-z_]+)\s*\(", header))
    assert declared == set(B.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name


@pytest.mark.parametrize("layout", [B.PIVOT_BRC, B.PIVOT_BCR, B.PIVOT_CBR])
@pytest.mark.parametrize("natural", [False, True])
@pytest.mark.parametrize("shape", [(24, 32, 8, 8, WL.F32), (21, 30, 4, 8, WL.F16), (12, 9, 2, 3, WL.F32),
                                   (64, 96, 16, 32, WL.F16)])
def test_plan_matches_oracle_bit_for_bit(layout, natural, shape):
    M, K, bh, bw, wd = shape
    p = WL.gen_fc(M, K, bh, bw, 0.4, seed=21, wdtype=wd, act=WL.ACT_RELU)
    p.tile_mask[1, :] = 0                                   # an empty block row
    plan = _host_plan(p, layout=layout, natural=natural)
    try:
        v = B.pivot_fc_plan_host_view(plan)
    finally:
        B.pivot_fc_plan_destroy(plan)
    W = O.unpivot_weights(p.Wp, p.prow, p.pcol) if natural else p.Wp
    want = O.oracle_plan(W, not natural, p.tile_mask, p.prow, p.pcol, p.bias, M, K, bh, bw, layout, 3)
    assert (v["T"], v["M_pad"], v["K_pad"], v["chunk_tiles"]) == (want["T"], want["M_pad"], want["K_pad"], 3)
    for name in PLAN_ARRAYS:
        a, b = v[name], want[name]
        assert a.dtype == b.dtype and a.shape == b.shape, name
        assert a.tobytes() == b.tobytes(), name


def test_plan_of_workload_shapes_scaled_down():
    for p, ct in ((WL.config2(seed=1, M=256, K=1152), 5), (WL.config3(seed=1, M=256, K=512, frac=0.25), 4),
                  (WL.config5(seed=1, H=64, I=32, steps=1, batch=1, frac=0.5).fc, 2)):
        plan = _host_plan(p, chunk_tiles=ct)
        v = B.pivot_fc_plan_host_view(plan)
        B.pivot_fc_plan_destroy(plan)
        want = O.oracle_plan(p.Wp, True, p.tile_mask, p.prow, p.pcol, p.bias, p.M, p.K, p.bh, p.bw, O.LAYOUT_BRC, ct)
        for name in PLAN_ARRAYS:
            assert v[name].tobytes() == want[name].tobytes(), (p.name, name)


def _full_size_problems():
    yield WL.config1(seed=0)
    yield WL.config2(seed=0)
    for frac in WL.CONFIG3_FRACS:
        yield WL.config3(seed=0, frac=frac)
    yield WL.config5(seed=0, steps=1).fc


def test_plan_of_every_workload_at_full_size_is_bit_exact():
    # configs 1, 2, 3 (all five densities) and 5 at full size, with the schedule the library itself picks
    # (chunk_tiles = 0: the resolved chunk size is handed to the oracle's builder, which cuts and orders the
    # schedule on its own)
    for p in _full_size_problems():
        plan = _host_plan(p, chunk_tiles=0)
        v = B.pivot_fc_plan_host_view(plan)
        B.pivot_fc_plan_destroy(plan)
        want = O.oracle_plan(p.Wp, True, p.tile_mask, p.prow, p.pcol, p.bias, p.M, p.K, p.bh, p.bw, O.LAYOUT_BRC,
                             v["chunk_tiles"])
        assert (v["T"], v["M_pad"], v["K_pad"]) == (want["T"], want["M_pad"], want["K_pad"]), p.name
        for name in PLAN_ARRAYS:
            assert v[name].dtype == want[name].dtype and v[name].shape == want[name].shape, (p.name, name)
            assert v[name].tobytes() == want[name].tobytes(), (p.name, name)


@pytest.mark.parametrize("eliminated", [False, True])
def test_config4_chain_plan_at_full_size_is_bit_exact(eliminated):
    # the VGG-shaped chain: every layer's arrays and the composed boundary arrays q_l / dst_l (Section 4.2.1);
    # identity boundaries exactly when pcol_{l+1} == prow_l (Section 4.2.3)
    probs = WL.config4(seed=0, eliminated=eliminated)
    plans = [_host_plan(p, chunk_tiles=0) for p in probs]
    views = [B.pivot_fc_plan_host_view(h) for h in plans]
    mlp = B.pivot_mlp_plan(plans, 0)
    try:
        mv = B.pivot_mlp_plan_host_view(mlp, views)
    finally:
        B.pivot_mlp_plan_destroy(mlp)
        for h in plans:
            B.pivot_fc_plan_destroy(h)
    for p, v in zip(probs, views):
        want = O.oracle_plan(p.Wp, True, p.tile_mask, p.prow, p.pcol, p.bias, p.M, p.K, p.bh, p.bw, O.LAYOUT_BRC,
                             v["chunk_tiles"])
        for name in PLAN_ARRAYS:
            assert v[name].tobytes() == want[name].tobytes(), (p.name, name)
    qs, dsts = O.oracle_mlp_plan([p.prow for p in probs], [p.pcol for p in probs], [p.nbr * p.bh for p in probs])
    assert mv["identity"] == [int(eliminated)] * 2
    for l in range(2):
        assert mv["q"][l].tobytes() == qs[l].tobytes()
        assert mv["dst"][l].tobytes() == dsts[l].tobytes()


def test_null_bias_is_zero_and_default_chunking_is_valid():
    p = WL.gen_fc(64, 64, 8, 8, 0.5, seed=3)
    plan = _host_plan(p, chunk_tiles=0, bias=False)
    v = B.pivot_fc_plan_host_view(plan)
    B.pivot_fc_plan_destroy(plan)
    assert np.all(v["bias_p"] == 0) and v["chunk_tiles"] >= 1
    chunks, part_base = O.build_schedule(v["row_ptr"], v["chunk_tiles"])
    assert np.array_equal(chunks, v["chunks"]) and np.array_equal(part_base, v["part_base"])


def test_schedule_policy_on_the_workload_shapes():
    # the library's own choice of row slices, chunk size and wavefronts (chunk_tiles = row_slices = wg_waves = 0)
    # on the full workload shapes: about one work item per compute unit, block rows whole unless a work item
    # would stream 256 KB, slices below one wave-load only while a work item keeps 16 KB
    def policy(p):
        plan = _host_plan(p, chunk_tiles=0)
        v = B.pivot_fc_plan_host_view(plan)
        B.pivot_fc_plan_destroy(plan)
        return v["row_slices"], v["chunk_tiles"], v["wg_waves"], v["nchunks"]
    assert policy(WL.config2(seed=0)) == (2, 29, 8, 128)                       # 256 work items of 58 KB
    sl, ct, nw, nch = policy(WL.config1(seed=0))
    assert (sl, nw, nch) == (1, 4, 64)                                         # 11 KB halves would be too small
    for frac, want_sl, want_nw in ((0.05, 2, 4), (0.10, 4, 4), (0.25, 4, 8), (0.50, 4, 8)):
        sl, ct, nw, nch = policy(WL.config3(seed=0, frac=frac))
        assert (sl, nw, nch) == (want_sl, want_nw, 64), (frac, sl, ct, nw, nch) # whole block rows
    assert policy(WL.config3(seed=0, frac=1.0)) == (2, 128, 8, 128)            # 256 KB rows are cut in two
    assert policy(WL.paper_grid_case(8192, 0.03125, seed=0, wdtype=WL.F32, perms="random"))[2] == 4   # 32 KB items


def test_source_ordered_gather_lists():
    # the batch 3..16 kernel's gather lists: per piece of the schedule the same (source, staged position) pairs as
    # xidx, ordered by source with padding columns last, packed as source | position << 19; the block-order twin
    # reads column col_idx[t]*bw+c; plans the kernel cannot take (fp32, tiles off the MFMA shapes) carry none
    for p, ct in ((WL.config3(seed=2, M=256, K=500, frac=0.3), 3), (WL.config3(seed=3, M=128, K=512, frac=1.0), 0),
                  (WL.gen_fc(96, 200, 16, 32, 0.4, seed=5, wdtype=WL.F16), 2),
                  (WL.gen_fc(64, 64, 16, 32, 0.0, seed=5, wdtype=WL.F16), 0)):
        plan = _host_plan(p, chunk_tiles=ct)
        v = B.pivot_fc_plan_host_view(plan)
        B.pivot_fc_plan_destroy(plan)
        if v["T"] == 0:
            continue                                                   # nothing to list
        assert v["xsort"] is not None and v["xsort"].shape == v["xidx"].shape == v["xsort_blk"].shape, p.name
        bw, none = v["bw"], (1 << 19) - 1
        for br, tb, te, slot in v["chunks"]:
            for packed, blk in ((v["xsort"], False), (v["xsort_blk"], True)):
                ent = packed[tb * bw:te * bw].astype(np.int64) & 0xFFFFFFFF
                src, pos = ent & none, ent >> 19
                assert sorted(pos.tolist()) == list(range((te - tb) * bw)), (p.name, br)
                assert np.all(np.diff(src) >= 0), (p.name, br)                    # padding (all ones) sorts last
                want = (np.repeat(v["col_idx"][tb:te], bw) * bw + np.tile(np.arange(bw), te - tb)) if blk \
                    else v["xidx"][tb * bw:te * bw]
                want = np.where((want >= v["K"]) if blk else (want < 0), none, want)[pos]   # padding columns
                assert np.array_equal(src, want), (p.name, br, blk)
    for p in (WL.gen_fc(64, 64, 16, 32, 0.5, seed=1, wdtype=WL.F32), WL.gen_fc(64, 64, 8, 8, 0.5, seed=1, wdtype=WL.F16)):
        plan = _host_plan(p, chunk_tiles=0)
        v = B.pivot_fc_plan_host_view(plan)
        B.pivot_fc_plan_destroy(plan)
        assert v["xsort"] is None and v["xsort_blk"] is None


def test_error_paths_return_codes():
    p = WL.gen_fc(16, 16, 4, 4, 0.5, seed=4)
    args = dict(M=16, K=16, bh=4, bw=4, wdtype=B.PIVOT_F32, W=p.Wp, w_space=B.PIVOT_W_PIVOTED,
                tile_mask=p.tile_mask, prow=p.prow, pcol=p.pcol, bias=p.bias)

    def code(**kw):
        a = dict(args); a.update(kw)
        with pytest.raises(B.PivotError) as e:
            h = B.pivot_fc_plan(**a)
            B.pivot_fc_plan_destroy(h)
        assert B.pivot_last_error() != ""
        return e.value.code

    bad = p.prow.copy(); bad[0] = bad[1]
    assert code(prow=bad) == B.PIVOT_E_NOT_PERMUTATION
    oob = p.pcol.copy(); oob[3] = 16
    assert code(pcol=oob) == B.PIVOT_E_NOT_PERMUTATION
    neg = p.pcol.copy(); neg[3] = -1
    assert code(pcol=neg) == B.PIVOT_E_NOT_PERMUTATION
    assert code(W=None) == B.PIVOT_E_NULL
    assert code(tile_mask=None) == B.PIVOT_E_NULL
    assert code(M=0) == B.PIVOT_E_SHAPE
    assert code(bh=0) == B.PIVOT_E_SHAPE
    assert code(wdtype=7) == B.PIVOT_E_UNSUPPORTED
    assert code(layout=9) == B.PIVOT_E_UNSUPPORTED
    assert code(act=5) == B.PIVOT_E_UNSUPPORTED
    assert code(flags=16) == B.PIVOT_E_UNSUPPORTED
    assert code(chunk_tiles=-2) == B.PIVOT_E_SHAPE
    # shapes the device kernels do not cover are refused before any GPU call
    assert code(device=0) == B.PIVOT_E_UNSUPPORTED            # 4x4 tiles
    assert code(device=0, bh=8, bw=6, M=16, K=12, W=p.Wp[:, :12].copy(), pcol=np.arange(12, dtype=np.int32),
                tile_mask=np.ones((2, 2), np.uint8)) == B.PIVOT_E_UNSUPPORTED   # not a power of two
    B.pivot_fc_plan_destroy(None)                             # NULL-safe


def test_host_only_plan_cannot_run_and_workspace_sizes():
    p = WL.gen_fc(32, 32, 8, 8, 0.5, seed=5)
    plan = _host_plan(p, chunk_tiles=1)
    try:
        assert B.pivot_fc_workspace_bytes(plan, 1) > 0
        assert B.pivot_fc_workspace_bytes(plan, 0) == 0
        with pytest.raises(B.PivotError) as e:
            B.pivot_fc_run(plan, 16, 32, 16, 32, 1, 16, 1 << 20)
        assert e.value.code == B.PIVOT_E_NO_DEVICE
        # the recurrent entry points refuse a host-only plan too, and check their pointers first
        with pytest.raises(B.PivotError) as e:
            B.pivot_lstm_run(plan, 8, 24, 16, 16, 16, None, 2, 1, 16, 1 << 20)
        assert e.value.code == B.PIVOT_E_NO_DEVICE
        with pytest.raises(B.PivotError) as e:
            B.pivot_lstm_run(plan, 8, 24, None, 16, 16, None, 2, 1, 16, 1 << 20)
        assert e.value.code == B.PIVOT_E_NULL
        with pytest.raises(B.PivotError) as e:
            B.pivot_lstm_status(plan, 2, 1, 16)
        assert e.value.code == B.PIVOT_E_NO_DEVICE
        with pytest.raises(B.PivotError) as e:
            B.pivot_lstm_status(plan, 2, 1, None)
        assert e.value.code == B.PIVOT_E_NULL
    finally:
        B.pivot_fc_plan_destroy(plan)


def test_measurement_aids_check_their_arguments_without_a_device():
    with pytest.raises(B.PivotError) as e:
        B.pivot_stream_read_run(None, 4096, 16)
    assert e.value.code == B.PIVOT_E_NULL
    with pytest.raises(B.PivotError) as e:
        B.pivot_stream_read_run(4096, 100, 16)          # fewer than 1024 bytes
    assert e.value.code == B.PIVOT_E_SHAPE
    with pytest.raises(B.PivotError) as e:
        B.pivot_stream_read_run(4100, 4096, 16)         # not 16-byte aligned
    assert e.value.code == B.PIVOT_E_SHAPE
    with pytest.raises(B.PivotError) as e:
        B.pivot_dense_run(None, B.PIVOT_F32, 4, 4, 16, 4, None, 16, 4, 1, 0)
    assert e.value.code == B.PIVOT_E_NULL


@pytest.mark.parametrize("eliminated", [False, True])
def test_chain_plan_matches_oracle(eliminated):
    probs = WL.config4(seed=3, dims=(96, 64, 64, 40), eliminated=eliminated)
    plans = [_host_plan(p) for p in probs]
    views = [B.pivot_fc_plan_host_view(h) for h in plans]
    mlp = B.pivot_mlp_plan(plans, 0)
    try:
        mv = B.pivot_mlp_plan_host_view(mlp, views)
    finally:
        B.pivot_mlp_plan_destroy(mlp)
        for h in plans:
            B.pivot_fc_plan_destroy(h)
    qs, dsts = O.oracle_mlp_plan([p.prow for p in probs], [p.pcol for p in probs], [p.nbr * p.bh for p in probs])
    assert mv["L"] == 3 and mv["identity"] == [int(eliminated)] * 2
    for l in range(2):
        assert mv["q"][l].tobytes() == qs[l].tobytes()
        assert mv["dst"][l].tobytes() == dsts[l].tobytes()
        assert np.array_equal(mv["q"][l], np.arange(len(qs[l]))) == eliminated


def test_chain_plan_error_paths():
    a = WL.gen_fc(32, 48, 8, 8, 0.5, seed=6)
    b = WL.gen_fc(16, 40, 8, 8, 0.5, seed=7)              # takes 40 inputs, a produces 32
    pa, pb = _host_plan(a), _host_plan(b)
    try:
        with pytest.raises(B.PivotError) as e:
            B.pivot_mlp_plan([pa, pb], 0)
        assert e.value.code == B.PIVOT_E_SHAPE
        with pytest.raises(B.PivotError) as e:
            B.pivot_mlp_plan([pa], 64)
        assert e.value.code == B.PIVOT_E_UNSUPPORTED
        with pytest.raises(B.PivotError) as e:
            B.pivot_mlp_plan([], 0)
        assert e.value.code == B.PIVOT_E_SHAPE
    finally:
        B.pivot_fc_plan_destroy(pa)
        B.pivot_fc_plan_destroy(pb)
