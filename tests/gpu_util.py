"""Helpers for the GPU parity tests: device memory through torch, everything
else through the C-ABI binding."""
import numpy as np
import torch

from oracle import pivot_oracle as O
from paper_1712_01084_amd import binding as B
from paper_1712_01084_amd import workloads as WL

TOL = {WL.F32: 1e-5, WL.F16: 2e-3}      # max |y - y_oracle| / (|W||x| + |b|)


def wd(p):
    return B.PIVOT_F32 if p.wdtype == WL.F32 else B.PIVOT_F16


def tdtype(p):
    return torch.float32 if p.wdtype == WL.F32 else torch.float16


def dev_plan(p, chunk_tiles=0, natural=False, wg_waves=0, row_slices=0, layout=B.PIVOT_BRC, flags=0):
    W = O.unpivot_weights(p.Wp, p.prow, p.pcol) if natural else p.Wp
    return B.pivot_fc_plan(p.M, p.K, p.bh, p.bw, wd(p), W,
                           B.PIVOT_W_NATURAL if natural else B.PIVOT_W_PIVOTED,
                           p.tile_mask, p.prow, p.pcol, p.bias, act=p.act, layout=layout,
                           chunk_tiles=chunk_tiles, device=0, wg_waves=wg_waves, row_slices=row_slices, flags=flags)


def workspace(nbytes):
    ws = torch.empty(max(nbytes, 256), dtype=torch.uint8, device="cuda")
    B.pivot_workspace_init(ws.data_ptr(), ws.numel(), torch.cuda.current_stream().cuda_stream)
    return ws


def run_fc(plan, p, x=None, repeats=1):
    """Runs the layer through pivot_fc_run; returns y as float64 numpy [batch][M]."""
    x = p.x if x is None else x
    batch = x.shape[0]
    xd = torch.from_numpy(np.ascontiguousarray(x)).cuda()
    ws = workspace(B.pivot_fc_workspace_bytes(plan, batch))
    st = torch.cuda.current_stream().cuda_stream
    outs = []
    for _ in range(repeats):
        yd = torch.full((batch, p.M), float("nan"), dtype=torch.float32, device="cuda")
        B.pivot_fc_run(plan, xd.data_ptr(), p.K, yd.data_ptr(), p.M, batch, ws.data_ptr(), ws.numel(), st)
        torch.cuda.synchronize()
        outs.append(yd.cpu().numpy())
    for o in outs[1:]:
        assert o.tobytes() == outs[0].tobytes(), "repeated runs differ in their bits"
    return outs[0].astype(np.float64)


def oracle_of(p, x=None):
    x = p.x if x is None else x
    return O.oracle_fc(p.Wp, p.tile_mask, p.prow, p.pcol, p.bias, x, p.bh, p.bw, p.act, return_scale=True)


def check_fc(p, chunk_tiles=0, natural=False, repeats=2, x=None, wg_waves=0, row_slices=0, layout=B.PIVOT_BRC, flags=0):
    plan = dev_plan(p, chunk_tiles=chunk_tiles, natural=natural, wg_waves=wg_waves, row_slices=row_slices, layout=layout,
                    flags=flags)
    try:
        y = run_fc(plan, p, x=x, repeats=repeats)
    finally:
        B.pivot_fc_plan_destroy(plan)
    y_ref, D = oracle_of(p, x=x)
    assert not np.isnan(y).any(), "some outputs were never written"
    err = O.max_scaled_error(y, y_ref, D)
    assert err <= TOL[p.wdtype], "%s: scaled error %.3g > %.3g" % (p.name, err, TOL[p.wdtype])
    return err
