"""Parity of the HIP path (through the C ABI) with the CPU oracle for single
layers.  Needs a GPU."""
import numpy as np
import pytest
import torch

from oracle import pivot_oracle as O
from paper_1712_01084_amd import binding as B
from paper_1712_01084_amd import workloads as WL

import gpu_util as G

pytestmark = pytest.mark.gpu

SHAPES = [(bh, bw) for bh in (8, 16, 32, 64) for bw in (8, 16, 32, 64)]


@pytest.mark.parametrize("wdtype", [WL.F32, WL.F16])
@pytest.mark.parametrize("bh,bw", SHAPES)
def test_every_tile_shape_ragged_small(bh, bw, wdtype):
    # several tiles per block row, ragged last block row and block column, an
    # empty block row, rows split over several work items
    M, K = 5 * bh - 3, 9 * bw - 5
    for batch, ct in ((1, 2), (3, 4)):
        p = WL.gen_fc(M, K, bh, bw, 0.6, seed=100 + bh + bw, wdtype=wdtype, batch=batch, act=WL.ACT_RELU)
        p.tile_mask[2, :] = 0
        G.check_fc(p, chunk_tiles=ct)


@pytest.mark.parametrize("wdtype", [WL.F32, WL.F16])
@pytest.mark.parametrize("bh,bw", SHAPES)
def test_every_tile_shape_with_gather_from_lds_copy(bh, bw, wdtype):
    # the same cases with the whole of x copied into LDS first (K is a multiple of 8 here, so the form applies)
    M, K = 5 * bh - 3, 9 * bw + 8
    for batch, ct in ((1, 2), (3, 4), (4, 9)):
        p = WL.gen_fc(M, K, bh, bw, 0.6, seed=200 + bh + bw, wdtype=wdtype, batch=batch, act=WL.ACT_RELU)
        p.tile_mask[2, :] = 0
        G.check_fc(p, chunk_tiles=ct, flags=B.PIVOT_PLAN_GATHER_FROM_LDS_COPY)


@pytest.mark.parametrize("wdtype,bh,bw", [(WL.F32, 32, 32), (WL.F32, 64, 16), (WL.F16, 64, 16), (WL.F16, 64, 64)])
@pytest.mark.parametrize("waves", [4, 8, 16])
@pytest.mark.parametrize("slices", [1, 2, 4, 8])
def test_row_slices_and_wave_counts(wdtype, bh, bw, waves, slices):
    for batch in (1, 4, 16):
        p = WL.gen_fc(3 * bh - 5, 12 * bw - 3, bh, bw, 0.7, seed=31, wdtype=wdtype, batch=batch, act=WL.ACT_RELU)
        p.tile_mask[1, :] = 0
        G.check_fc(p, chunk_tiles=5, wg_waves=waves, row_slices=slices)     # split rows
        G.check_fc(p, chunk_tiles=12, wg_waves=waves, row_slices=slices)    # whole rows


@pytest.mark.parametrize("layout", [B.PIVOT_BCR, B.PIVOT_CBR])
@pytest.mark.parametrize("wdtype", [WL.F32, WL.F16])
@pytest.mark.parametrize("bh,bw", SHAPES)
def test_column_major_layouts_every_tile_shape(bh, bw, wdtype, layout):
    M, K = 5 * bh - 3, 9 * bw - 5
    for batch, ct, waves in ((1, 2, 4), (3, 9, 8), (1, 4, 16)):
        p = WL.gen_fc(M, K, bh, bw, 0.6, seed=200 + bh + bw, wdtype=wdtype, batch=batch, act=WL.ACT_RELU)
        p.tile_mask[2, :] = 0
        G.check_fc(p, chunk_tiles=ct, wg_waves=waves, layout=layout)


@pytest.mark.parametrize("layout", [B.PIVOT_BCR, B.PIVOT_CBR])
def test_column_major_layouts_full_configs(layout):
    G.check_fc(WL.config1(seed=0), layout=layout)
    G.check_fc(WL.config2(seed=0), layout=layout)
    G.check_fc(WL.config3(seed=0, frac=0.25, batch=1), layout=layout)
    G.check_fc(WL.config3(seed=0, frac=0.1, batch=16), layout=layout)      # batch 16 through the vector kernel
    G.check_fc(WL.paper_grid_case(1024, 0.125, seed=1), layout=layout)


@pytest.mark.parametrize("batch", [1, 2, 3, 4, 5, 8])
def test_batches_fp32(batch):
    p = WL.gen_fc(200, 328, 16, 16, 0.5, seed=7, batch=batch, act=WL.ACT_NONE)
    G.check_fc(p, chunk_tiles=3)


@pytest.mark.parametrize("batch", [1, 2, 4, 7, 8, 16, 33, 64])
@pytest.mark.parametrize("bh,bw", [(64, 16), (16, 32), (32, 32), (16, 16)])
def test_batches_fp16_including_matrix_core_path(bh, bw, batch):
    p = WL.gen_fc(5 * bh - 1, 11 * bw - 2, bh, bw, 0.5, seed=8, wdtype=WL.F16, batch=batch, act=WL.ACT_RELU)
    p.tile_mask[1, :] = 0
    G.check_fc(p, chunk_tiles=3)


@pytest.mark.parametrize("batch", [3, 5, 6, 9, 13, 16])
@pytest.mark.parametrize("bh,bw", [(64, 16), (16, 32), (32, 64)])
def test_fp16_small_batches_matrix_cores_fed_from_lds(bh, bw, batch):
    # batch 3..16 with few staged elements: the tile is the MFMA A operand, the B fragments come from the
    # x-segments staged in LDS (4 or 8 rows per launch row; rows past the batch are zero and never stored); whole block
    # rows per work item, ragged M and K, one empty block row
    p = WL.gen_fc(3 * bh + 7, 6 * bw - 5, bh, bw, 0.6, seed=40 + batch, wdtype=WL.F16, batch=batch, act=WL.ACT_RELU)
    p.tile_mask[2, :] = 0
    G.check_fc(p)
    G.check_fc(p, wg_waves=8, row_slices=2)


@pytest.mark.parametrize("batch,frac", [(8, 0.3), (8, 1.0), (12, 0.6), (16, 0.3), (16, 0.1)])
def test_fp16_batches_gather_through_source_ordered_lists(batch, frac):
    # batch 5..16 with long work items: every thread takes several entries of the plan's source-ordered gather
    # list, in more than one round (2040 columns, 512 or 256 threads, 4 entries per round), with padding columns
    # at the end of the list (K is not a multiple of the tile width), whole and split block rows
    p = WL.gen_fc(4 * 64 + 9, 2040, 64, 16, frac, seed=70 + batch, wdtype=WL.F16, batch=batch, act=WL.ACT_RELU,
                  mask="full" if frac == 1.0 else "uniform")
    G.check_fc(p)
    G.check_fc(p, chunk_tiles=100, wg_waves=4, row_slices=2)
    p = WL.gen_fc(5 * 16 + 3, 1530, 16, 32, frac, seed=90 + batch, wdtype=WL.F16, batch=batch,
                  mask="full" if frac == 1.0 else "uniform")
    G.check_fc(p)


@pytest.mark.parametrize("batch", [3, 4, 8, 11, 16])
@pytest.mark.parametrize("bh,sl", [(64, 4), (32, 2), (64, 2)])
def test_fp16_16_column_tiles_in_16_row_slices_pair_their_tiles(bh, sl, batch):
    # tiles 16 columns wide cut into 16-row slices: one 16x16x32 MFMA step spans two consecutive tiles of the
    # block row; odd tile counts (the last pair's second half is zero weights against zeroed columns), block rows
    # of one tile, an empty block row, split block rows; (64, 2) keeps 32-row slices (the 32x32x16 form)
    p = WL.gen_fc(4 * bh - 5, 7 * 16 - 3, bh, 16, 1.0, seed=120 + batch, wdtype=WL.F16, batch=batch, mask="full",
                  act=WL.ACT_RELU)
    p.tile_mask[1, 1:] = 0                               # a block row of a single tile
    p.tile_mask[2, :] = 0                                # an empty one
    G.check_fc(p, row_slices=sl)
    G.check_fc(p, row_slices=sl, chunk_tiles=3, wg_waves=8)
    p = WL.gen_fc(3 * bh, 41 * 16, bh, 16, 0.5, seed=140 + batch, wdtype=WL.F16, batch=batch)
    G.check_fc(p, row_slices=sl)


@pytest.mark.parametrize("batch", [5, 8, 9, 12, 16])
@pytest.mark.parametrize("bh,bw,K", [(64, 16, 1024), (64, 16, 1000), (32, 32, 4096), (16, 64, 333), (64, 64, 2048)])
def test_fp16_batch_5_to_16_gathers_fragments_from_a_copy_of_x(bh, bw, K, batch):
    # batch 5..16: the rows of x are copied into LDS and every lane gathers the eight values of its B fragment
    # from there.  Rows that are whole aligned vectors are copied with 16-byte loads, anything else (K not a
    # multiple of 8, a row stride above K, an x that starts off a 16-byte boundary) element by element; rows past
    # the batch are never read from memory; whole and split block rows, every row-slice form, an empty block row
    # (batch 5..8 takes this form from a quarter of the columns per AVERAGE work item on, hence the denser mask)
    p = WL.gen_fc(3 * bh + 7, K, bh, bw, 0.3 if batch > 8 else 0.5, seed=300 + batch + bh, wdtype=WL.F16, batch=batch, act=WL.ACT_RELU)
    p.tile_mask[1, :] = 0
    plan = G.dev_plan(p)
    try:
        assert "fc_mfma_xrow_kernel" in B.pivot_fc_kernel_name(plan, batch)
        st = torch.cuda.current_stream().cuda_stream
        ws = G.workspace(B.pivot_fc_workspace_bytes(plan, batch))
        y_ref, D = G.oracle_of(p)
        for ldx, off in ((K, 0), (K + 8, 0), (K + 3, 0), (K, 1)):
            buf = torch.full((batch * ldx + 16,), float("nan"), dtype=torch.float16, device="cuda")
            xv = buf[off:off + batch * ldx].view(batch, ldx)
            xv[:, :K] = torch.from_numpy(p.x).cuda()
            yd = torch.full((batch, p.M), float("nan"), dtype=torch.float32, device="cuda")
            B.pivot_fc_run(plan, xv.data_ptr(), ldx, yd.data_ptr(), p.M, batch, ws.data_ptr(), ws.numel(), st)
            torch.cuda.synchronize()
            y = yd.cpu().numpy().astype(np.float64)
            assert not np.isnan(y).any(), (ldx, off)
            assert O.max_scaled_error(y, y_ref, D) <= G.TOL[p.wdtype], (ldx, off)
    finally:
        B.pivot_fc_plan_destroy(plan)
    G.check_fc(p, chunk_tiles=5, wg_waves=8, row_slices=2)
    G.check_fc(p, row_slices=4)


@pytest.mark.parametrize("batch", [1, 3, 8, 16])
@pytest.mark.parametrize("M,K,bh,bw,wdtype,frac", [(2048, 3072, 16, 32, WL.F16, 0.125), (1024, 4096, 32, 32, WL.F32, 0.125),
                                                     (4096, 2048, 64, 16, WL.F16, 0.125), (512, 4096, 8, 8, WL.F32, 0.2)])
def test_skewed_masks_cut_long_block_rows(M, K, bh, bw, wdtype, frac, batch):
    # per-row tile counts following a Zipf profile (the longest block row at least four times the average one):
    # the library cuts long rows into pieces of twice the average row (32..96 KB per work item), so these layers
    # run with hand-overs between the pieces of a row at every batch size and through every kernel family
    p = WL.gen_fc(M, K, bh, bw, frac, seed=400 + bh + batch, wdtype=wdtype, batch=batch, mask="zipf", act=WL.ACT_RELU)
    cnt = p.tile_mask.sum(axis=1)
    assert cnt.max() >= 4 * cnt.mean()
    plan = G.dev_plan(p)
    try:
        v = B.pivot_fc_plan_host_view(plan)
        es = 4 if wdtype == WL.F32 else 2
        piece = v["chunk_tiles"] * (bh // v["row_slices"]) * bw * es
        assert v["chunk_tiles"] < cnt.max() and 32 * 1024 <= piece <= 96 * 1024, (v["chunk_tiles"], piece)
    finally:
        B.pivot_fc_plan_destroy(plan)
    G.check_fc(p)


@pytest.mark.parametrize("batch", [16, 33, 64])
def test_fp16_long_rows_use_the_block_order_copy(batch):
    # work items too long for the LDS-fed form (8 batch rows of 4096 staged columns exceed its 48 KB; at batch 64
    # eight launch rows of 1232 columns exceed its column budget): x is copied to block order by one small kernel
    # and the matrix-core kernel reads its B fragments from the copy
    p = WL.gen_fc(2 * 64 - 3, 4096, 64, 16, 1.0, seed=160 + batch, wdtype=WL.F16, batch=batch, mask="full", act=WL.ACT_RELU)
    G.check_fc(p, chunk_tiles=256)
    if batch == 64:
        p = WL.gen_fc(3 * 64, 4096, 64, 16, 0.3, seed=170, wdtype=WL.F16, batch=batch, mask="balanced")
        G.check_fc(p)


def test_fp16_batches_beyond_the_gather_lists_range():
    # 2^19 input columns and more do not fit the packed list entries: the plan carries no lists and batch 3..16
    # falls back to the vector kernel (batch < 8) or to the block-order copy plus the matrix-core kernel
    p = WL.gen_fc(32, (1 << 19) + 40, 32, 16, 0.002, seed=77, wdtype=WL.F16, batch=9)
    plan = G.dev_plan(p)
    try:
        assert B.pivot_fc_plan_host_view(plan)["xsort"] is None
        for batch in (4, 9):
            y = G.run_fc(plan, p, x=p.x[:batch])
            y_ref, D = G.oracle_of(p, x=p.x[:batch])
            assert O.max_scaled_error(y, y_ref, D) <= G.TOL[p.wdtype], batch
    finally:
        B.pivot_fc_plan_destroy(plan)


def test_degenerate_masks_and_natural_weights():
    p = WL.gen_fc(64, 96, 16, 16, 0.5, seed=9, act=WL.ACT_RELU)
    p.tile_mask[:] = 0                                   # no tile kept: y = relu(b)
    G.check_fc(p)
    p = WL.gen_fc(64, 96, 16, 16, 1.0, seed=10, mask="full")
    G.check_fc(p, chunk_tiles=1)                         # every tile its own work item
    G.check_fc(p, chunk_tiles=6)                         # whole block rows
    p = WL.gen_fc(70, 100, 16, 32, 0.4, seed=11, wdtype=WL.F16, batch=2)
    G.check_fc(p, natural=True)


def test_identity_perms_full_mask_matches_dense_kernel():
    for wdtype in (WL.F32, WL.F16):
        p = WL.gen_fc(256, 512, 32, 32, 1.0, seed=12, mask="full", perms="identity", wdtype=wdtype, batch=4)
        G.check_fc(p)
        st = torch.cuda.current_stream().cuda_stream
        Wd = torch.from_numpy(p.Wp).cuda()
        xd = torch.from_numpy(p.x).cuda()
        bd = torch.from_numpy(p.bias).cuda()
        for batch in (1, 4):
            yd = torch.full((batch, p.M), float("nan"), dtype=torch.float32, device="cuda")
            B.pivot_dense_run(Wd.data_ptr(), G.wd(p), p.M, p.K, xd.data_ptr(), p.K, bd.data_ptr(), yd.data_ptr(),
                              p.M, batch, p.act, st)
            torch.cuda.synchronize()
            y_ref, D = G.oracle_of(p, x=p.x[:batch])
            assert O.max_scaled_error(yd.cpu().numpy(), y_ref, D) <= G.TOL[wdtype]


def test_fp16_subnormal_weights_are_kept():
    p = WL.gen_fc(128, 128, 64, 16, 0.5, seed=13, wdtype=WL.F16, batch=16)
    tiny = (np.random.default_rng(1).integers(1, 1024, size=p.Wp.shape).astype(np.uint16)).view(np.float16)
    p.Wp = tiny                                           # every weight a positive fp16 subnormal
    p.bias[:] = 0
    for batch in (1, 16):
        x = np.abs(p.x[:batch])
        y_ref, D = G.oracle_of(p, x=x)
        assert y_ref.max() > 0
        G.check_fc(p, chunk_tiles=2, x=x)


def test_strided_x_and_y():
    p = WL.gen_fc(96, 160, 32, 32, 0.5, seed=14, batch=3, act=WL.ACT_RELU)
    plan = G.dev_plan(p, chunk_tiles=2)
    try:
        ldx, ldy = p.K + 24, p.M + 8
        xd = torch.zeros((3, ldx), dtype=torch.float32, device="cuda")
        xd[:, :p.K] = torch.from_numpy(p.x).cuda()
        yd = torch.full((3, ldy), -7.0, dtype=torch.float32, device="cuda")
        ws = G.workspace(B.pivot_fc_workspace_bytes(plan, 3))
        B.pivot_fc_run(plan, xd.data_ptr(), ldx, yd.data_ptr(), ldy, 3, ws.data_ptr(), ws.numel(),
                       torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        y = yd.cpu().numpy()
        y_ref, D = G.oracle_of(p)
        assert O.max_scaled_error(y[:, :p.M], y_ref, D) <= 1e-5
        assert np.all(y[:, p.M:] == -7.0)                 # nothing written past M
    finally:
        B.pivot_fc_plan_destroy(plan)


def test_run_error_paths_on_device_plans():
    p = WL.gen_fc(64, 64, 16, 16, 0.5, seed=15)
    plan = G.dev_plan(p, chunk_tiles=1)
    try:
        xd = torch.zeros((1, 64), device="cuda")
        yd = torch.zeros((1, 64), device="cuda")
        for kw, code in ((dict(ws=0, nb=0), B.PIVOT_E_WORKSPACE), (dict(batch=0), B.PIVOT_E_SHAPE),
                         (dict(batch=65), B.PIVOT_E_SHAPE), (dict(ldx=8), B.PIVOT_E_SHAPE), (dict(x=0), B.PIVOT_E_NULL)):
            ws = G.workspace(B.pivot_fc_workspace_bytes(plan, 1))
            a = dict(x=xd.data_ptr(), ldx=64, y=yd.data_ptr(), ldy=64, batch=1, ws=ws.data_ptr(), nb=ws.numel())
            a.update(kw)
            with pytest.raises(B.PivotError) as e:
                B.pivot_fc_run(plan, a["x"], a["ldx"], a["y"], a["ldy"], a["batch"], a["ws"], a["nb"], None)
            assert e.value.code == code
    finally:
        B.pivot_fc_plan_destroy(plan)


@pytest.mark.parametrize("wdtype,bh,bw,batches", [(WL.F32, 32, 32, (1, 5, 1, 64, 3)), (WL.F16, 64, 16, (16, 1, 5, 8, 1, 33)),
                                                   (WL.F16, 16, 32, (8, 2, 16, 1))])
def test_one_workspace_reused_across_batch_sizes(wdtype, bh, bw, batches):
    # split block rows (arrival counters and partial sums in the workspace) and ragged M and K; the workspace is
    # cleared ONCE and then shared by runs of different batch sizes, each preceded by a run of the same batch on
    # NaN inputs, which leaves NaN in every partial sum and block-order copy the next run may find
    p = WL.gen_fc(3 * bh + 5, 203, bh, bw, 0.6, seed=51, wdtype=wdtype, batch=max(batches), act=WL.ACT_RELU)
    plan = G.dev_plan(p, chunk_tiles=2)
    try:
        ws = G.workspace(max(B.pivot_fc_workspace_bytes(plan, b) for b in batches))
        st = torch.cuda.current_stream().cuda_stream
        for b in batches:
            x = np.ascontiguousarray(p.x[:b])
            for poison in (True, False):
                xd = torch.from_numpy(np.full_like(x, np.nan) if poison else x).cuda()
                yd = torch.full((b, p.M), float("nan"), dtype=torch.float32, device="cuda")
                B.pivot_fc_run(plan, xd.data_ptr(), p.K, yd.data_ptr(), p.M, b, ws.data_ptr(), ws.numel(), st)
                torch.cuda.synchronize()
            y_ref, D = G.oracle_of(p, x=x)
            y = yd.cpu().numpy().astype(np.float64)
            assert not np.isnan(y).any(), ("batch", b)
            assert O.max_scaled_error(y, y_ref, D) <= G.TOL[wdtype], ("batch", b)
    finally:
        B.pivot_fc_plan_destroy(plan)


# ------------------------------------------------------------- full-size configurations

SEEDS = (0, 1, 2)


@pytest.mark.parametrize("seed", SEEDS)
def test_config1_full(seed):
    G.check_fc(WL.config1(seed=seed))


@pytest.mark.parametrize("seed", SEEDS)
def test_config2_full(seed):
    p = WL.config2(seed=seed)
    err = G.check_fc(p)
    print("config2 seed %d scaled error %.3g" % (seed, err))


@pytest.mark.parametrize("seed", SEEDS)
@pytest.mark.parametrize("frac", WL.CONFIG3_FRACS)
def test_config3_full(frac, seed):
    for batch in (1, 4, 16):
        G.check_fc(WL.config3(seed=seed, batch=batch, frac=frac))


def test_config5_gate_matrix_full_batch8():
    lp = WL.config5(seed=0, steps=1)
    p = lp.fc
    p.x = np.random.default_rng(3).standard_normal((8, p.K)).astype(np.float16)
    G.check_fc(p)


def test_stream_read_aid_sums_what_it_reads():
    # the read-only launch used as the measured ceiling: every byte is read exactly once
    rng = np.random.default_rng(0)
    for nkb in (1, 7, 2048, 14848):
        a = rng.integers(-8, 9, size=nkb * 256).astype(np.float32)      # small integers: the sum is exact in fp32
        buf = torch.from_numpy(a).cuda()
        out = torch.full((2048,), float("nan"), dtype=torch.float32, device="cuda")
        B.pivot_stream_read_run(buf.data_ptr(), nkb * 1024, out.data_ptr(), torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        assert float(out.cpu().numpy().astype(np.float64).sum()) == float(a.astype(np.float64).sum())
    with pytest.raises(B.PivotError):
        B.pivot_stream_read_run(buf.data_ptr(), 100, out.data_ptr(), None)


@pytest.mark.parametrize("wdtype,bh,bw,batch,K", [(WL.F32, 32, 32, 1, 320), (WL.F32, 16, 16, 3, 200), (WL.F16, 64, 16, 4, 264),
                                                 (WL.F16, 16, 32, 2, 96), (WL.F32, 8, 8, 1, 1024),
                                                 (WL.F16, 16, 32, 8, 96), (WL.F16, 32, 32, 13, 128)])
def test_gather_through_lds_copy_of_x_equals_gather_from_global(wdtype, bh, bw, batch, K):
    # the two forms of the column gather feed the same arithmetic in the same order: identical bits;
    # an x whose rows are not whole 16-byte vectors (or misaligned) silently takes the global form
    p = WL.gen_fc(4 * bh + 5, K, bh, bw, 0.4, seed=31, wdtype=wdtype, batch=batch, act=WL.ACT_RELU)
    outs = []
    for flags in (B.PIVOT_PLAN_GATHER_FROM_LDS_COPY, B.PIVOT_PLAN_GATHER_FROM_GLOBAL):
        plan = G.dev_plan(p, flags=flags)
        try:
            outs.append(G.run_fc(plan, p))
        finally:
            B.pivot_fc_plan_destroy(plan)
    assert outs[0].tobytes() == outs[1].tobytes()
    y_ref, D = G.oracle_of(p)
    assert O.max_scaled_error(outs[0], y_ref, D) <= G.TOL[p.wdtype]


@pytest.mark.parametrize("wdtype,K", [(WL.F32, 20000), (WL.F16, 40000), (WL.F32, 25088)])
def test_long_input_copied_into_lds_beyond_64_kb(wdtype, K):
    # an x of 80-100 KB: up to 16 vectors per thread, more than 64 KB of LDS per workgroup (allowed per kernel),
    # eight gather indices per thread up front; same bits as the element gather from global memory
    p = WL.gen_fc(96, K, 32, 32, 0.12, seed=41, wdtype=wdtype, act=WL.ACT_RELU)
    outs = []
    for flags in (B.PIVOT_PLAN_GATHER_FROM_LDS_COPY, B.PIVOT_PLAN_GATHER_FROM_GLOBAL):
        plan = G.dev_plan(p, flags=flags)
        try:
            outs.append(G.run_fc(plan, p))
        finally:
            B.pivot_fc_plan_destroy(plan)
    assert outs[0].tobytes() == outs[1].tobytes()
    y_ref, D = G.oracle_of(p)
    assert O.max_scaled_error(outs[0], y_ref, D) <= G.TOL[p.wdtype]
    G.check_fc(p)


def test_lds_copy_of_x_with_odd_row_length_and_offset_pointer():
    # K = 203 (not a multiple of 4) and an x that starts 4 bytes past a 16-byte boundary: the kernel must fall
    # back to the global gather on its own, with the same result
    p = WL.gen_fc(64, 203, 16, 16, 0.5, seed=33, batch=2, act=WL.ACT_NONE)
    plan = G.dev_plan(p, flags=B.PIVOT_PLAN_GATHER_FROM_LDS_COPY)
    try:
        G.check_fc(p)
        ld = 208
        xd = torch.zeros(2 * ld + 1, dtype=torch.float32, device="cuda")
        xv = xd[1:].view(2, ld)
        xv[:, :p.K] = torch.from_numpy(p.x).cuda()
        yd = torch.empty((2, p.M), dtype=torch.float32, device="cuda")
        ws = G.workspace(B.pivot_fc_workspace_bytes(plan, 2))
        B.pivot_fc_run(plan, xv.data_ptr(), ld, yd.data_ptr(), p.M, 2, ws.data_ptr(), ws.numel(),
                       torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        y_ref, D = G.oracle_of(p)
        assert O.max_scaled_error(yd.cpu().numpy(), y_ref, D) <= 1e-5
    finally:
        B.pivot_fc_plan_destroy(plan)
