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
