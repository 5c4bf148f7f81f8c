"""pivot_fc_run_static (the entry point that brings its own scratch and allocates nothing) against pivot_fc_run:
same kernels, same arithmetic, so the outputs must agree bit for bit, and both with the oracle.  Needs a GPU."""
import numpy as np
import pytest
import torch

from oracle import pivot_oracle as O
from paper_1712_01084_amd import binding as B
from paper_1712_01084_amd import workloads as WL

import gpu_util as G

pytestmark = pytest.mark.gpu


def _both(p, x, chunk_tiles):
    plan = G.dev_plan(p, chunk_tiles=chunk_tiles)
    try:
        batch = x.shape[0]
        st = torch.cuda.current_stream().cuda_stream
        xd = torch.from_numpy(np.ascontiguousarray(x)).cuda()
        y_ws = torch.full((batch, p.M), float("nan"), dtype=torch.float32, device="cuda")
        y_st = torch.full((batch, p.M), float("nan"), dtype=torch.float32, device="cuda")
        ws = G.workspace(B.pivot_fc_workspace_bytes(plan, batch))
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated()
        B.pivot_fc_run_static(plan, xd.data_ptr(), p.K, y_st.data_ptr(), p.M, batch, st)
        assert torch.cuda.memory_allocated() == before
        B.pivot_fc_run(plan, xd.data_ptr(), p.K, y_ws.data_ptr(), p.M, batch, ws.data_ptr(), ws.numel(), st)
        torch.cuda.synchronize()
        a, b = y_st.cpu().numpy(), y_ws.cpu().numpy()
        assert not np.isnan(a).any()
        assert a.tobytes() == b.tobytes()
        y_ref, D = G.oracle_of(p, x=x)
        assert O.max_scaled_error(a.astype(np.float64), y_ref, D) <= G.TOL[p.wdtype]
    finally:
        B.pivot_fc_plan_destroy(plan)


def test_static_scratch_entry_point_two_calls_second_smaller():
    # split block rows (arrival counters + partial sums in the scratch), ragged M and K; the second call is a
    # smaller layer at a smaller batch, so it finds the first call's partial sums in the shared array
    big = WL.gen_fc(500, 1000, 32, 32, 0.5, seed=61, batch=5, act=WL.ACT_RELU)
    small = WL.gen_fc(77, 203, 16, 16, 0.6, seed=62, batch=2, act=WL.ACT_RELU)
    _both(big, big.x, chunk_tiles=3)
    _both(small, small.x, chunk_tiles=2)
    _both(big, big.x[:1], chunk_tiles=3)


def test_static_scratch_entry_point_matrix_core_forms():
    # fp16 at batch 16: staged in LDS (split rows); at batch 24 with whole rows of 97 tiles read from a block-order
    # copy of x that lives in the scratch; then a smaller batch of the first again
    a = WL.gen_fc(200, 520, 64, 16, 0.5, seed=63, wdtype=WL.F16, batch=16)
    b = WL.gen_fc(40, 3100, 32, 32, 1.0, seed=64, wdtype=WL.F16, batch=24, mask="full")
    _both(a, a.x, chunk_tiles=4)
    _both(b, b.x, chunk_tiles=97)
    _both(a, a.x[:3], chunk_tiles=4)


def test_static_scratch_entry_point_refuses_what_does_not_fit():
    # 2100 block rows cut into pieces: 2100 x 16 launch rows x 256 bytes of arrival counters = 8.6 MB, more than
    # the 4 MiB the built-in scratch keeps for them.  A host-side check: nothing is launched for the refused call.
    p = WL.gen_fc(8 * 2100, 64, 8, 8, 1.0, seed=65, mask="full", batch=1)
    plan = G.dev_plan(p, chunk_tiles=1)
    try:
        xd = torch.from_numpy(p.x).cuda()
        yd = torch.empty((1, p.M), dtype=torch.float32, device="cuda")
        with pytest.raises(B.PivotError) as e:
            B.pivot_fc_run_static(plan, xd.data_ptr(), p.K, yd.data_ptr(), p.M, 1, None)
        assert e.value.code == B.PIVOT_E_WORKSPACE and "use pivot_fc_run" in str(e.value)
        G.check_fc(p, chunk_tiles=1)                      # the same plan through a caller's workspace
    finally:
        B.pivot_fc_plan_destroy(plan)
