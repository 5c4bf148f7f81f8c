"""The paper's experiment grid (Section 5: square block-diagonal matrices with
identical square blocks) through the HIP path, and the CSR comparator, against
the CPU oracle.  Needs a GPU."""
import numpy as np
import pytest
import scipy.sparse as sp
import torch

from oracle import pivot_oracle as O
from paper_1712_01084_amd import binding as B
from paper_1712_01084_amd import workloads as WL

import gpu_util as G

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("size,fill", [(64, 0.03125), (64, 0.25), (128, 0.0625), (256, 0.125), (512, 0.0625),
                                       (1024, 0.03125), (1024, 0.25), (2048, 0.125), (4096, 0.03125), (4096, 0.25)])
@pytest.mark.parametrize("wdtype", [WL.F32, WL.F16])
def test_paper_grid_case_parity(size, fill, wdtype):
    for perms in ("random", "identity"):
        p = WL.paper_grid_case(size, fill, seed=3, wdtype=wdtype, perms=perms, act=WL.ACT_RELU)
        G.check_fc(p)


@pytest.mark.parametrize("wdtype", [WL.F32, WL.F16])
@pytest.mark.parametrize("size,fill", [(64, 0.03125), (512, 0.0625), (2048, 0.25)])
def test_csr_comparator_matches_oracle(size, fill, wdtype):
    p = WL.paper_grid_case(size, fill, seed=4, wdtype=wdtype, act=WL.ACT_RELU)
    Wd = O.dense_masked_natural(p.Wp, p.tile_mask, p.prow, p.pcol, p.bh, p.bw)
    A = sp.csr_matrix(Wd.astype(np.float32))           # scipy has no fp16 CSR; the values are exact in fp32
    rp = torch.from_numpy(A.indptr.astype(np.int32)).cuda()
    ci = torch.from_numpy(A.indices.astype(np.int32)).cuda()
    va = torch.from_numpy(A.data.astype(p.Wp.dtype)).cuda()
    xd = torch.from_numpy(p.x[0].copy()).cuda()
    bd = torch.from_numpy(p.bias).cuda()
    yd = torch.full((p.M,), float("nan"), dtype=torch.float32, device="cuda")
    B.pivot_csr_run(rp.data_ptr(), ci.data_ptr(), va.data_ptr(), G.wd(p), p.M, A.nnz, xd.data_ptr(), bd.data_ptr(),
                    yd.data_ptr(), p.act, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    y_ref = O.fc_dense(Wd, p.x, p.bias, p.act)
    D = O.error_scale(Wd, p.x, p.bias)
    assert O.max_scaled_error(yd.cpu().numpy()[None, :], y_ref, D) <= G.TOL[wdtype]


def test_exchange_probe_runs_and_reports_bounded_waits():
    # the measurement aid for the one-launch forms: one trip between two workgroups, same XCD and other XCD.
    # Every wait in it is bounded, so it returns whatever the memory system does: the device-coherent series must
    # succeed (the one-launch kernels rely on exactly these accesses) with a trip of well under 20 us; the
    # workgroup-scope series may give up (-1); bad arguments are refused on the host.
    buf = torch.empty(B.PIVOT_PROBE_SCRATCH_BYTES + 256, dtype=torch.uint8, device="cuda")
    off = (-buf.data_ptr()) % 256
    st = torch.cuda.current_stream().cuda_stream
    rounds = 200
    B.pivot_exchange_probe_run(buf.data_ptr() + off, B.PIVOT_PROBE_SCRATCH_BYTES, rounds, st)
    torch.cuda.synchronize()
    out = buf[off:off + 64].cpu().numpy().view(np.int64)
    assert out[0] == 1
    assert out[4] > 0 and out[5] > 0 and out[4] != out[5]
    for k in (1, 3):
        us = out[k] / 100.0 / (2 * rounds)
        assert 0.05 < us < 20.0, (k, us)
    assert out[2] == -1 or out[2] > 0
    assert out[6] == -1 or out[6] > 0
    for kw in (dict(ptr=0), dict(nbytes=1024), dict(rounds=0), dict(ptr=buf.data_ptr() + off + 4)):
        with pytest.raises(B.PivotError):
            B.pivot_exchange_probe_run(kw.get("ptr", buf.data_ptr() + off), kw.get("nbytes", B.PIVOT_PROBE_SCRATCH_BYTES),
                                       kw.get("rounds", rounds), st)
