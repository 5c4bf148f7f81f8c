"""Seeded random sweep of pivot_fc_run against the oracle: tile shapes, ragged
sizes, densities, batches, both weight types and every plan knob drawn
together, so that combinations no hand-written case names are still covered
(sub-wave-load row slices with several batch rows, forced gather forms on
split block rows, ...).  Needs a GPU."""
import numpy as np
import pytest

from paper_1712_01084_amd import binding as B
from paper_1712_01084_amd import workloads as WL

import gpu_util as G

pytestmark = pytest.mark.gpu


def _case(rng, it, big, skewed=False):
    wdtype = WL.F32 if rng.random() < 0.5 else WL.F16
    bh = int(rng.choice([8, 16, 32, 64]))
    bw = int(rng.choice([8, 16, 32, 64]))
    nbr = int(rng.integers(1, 40 if big else 9))
    nbc = int(rng.integers(1, 300 if big else 40))
    M = max(1, nbr * bh - int(rng.integers(0, bh)))
    K = max(1, nbc * bw - int(rng.integers(0, bw)))
    frac = float(rng.choice([0.1, 0.3, 0.6, 1.0]))
    batch = int(rng.choice([1, 2, 4, 5, 6, 7, 8, 9, 12, 16, 24, 33]) if skewed else rng.choice([1, 1, 1, 2, 3, 4, 5, 8, 9, 16, 17, 24, 33, 64]))
    kw = dict(chunk_tiles=int(rng.choice([0, 0, 1, 2, 5, 12])), wg_waves=int(rng.choice([0, 4, 8, 16])),
              row_slices=int(rng.choice([0, 1, 2, 4, 8])),
              flags=int(rng.choice([0, 0, B.PIVOT_PLAN_GATHER_FROM_GLOBAL, B.PIVOT_PLAN_GATHER_FROM_LDS_COPY])))
    mask = "full" if frac == 1.0 else str(rng.choice(["uniform", "balanced", "zipf", "zipf"] if skewed else ["uniform", "balanced"]))
    p = WL.gen_fc(M, K, bh, bw, frac, seed=5000 + it, wdtype=wdtype, batch=batch, act=int(rng.integers(0, 2)), mask=mask)
    if rng.random() < 0.3 and p.tile_mask.shape[0] > 1:
        p.tile_mask[int(rng.integers(0, p.tile_mask.shape[0])), :] = 0      # an empty block row
    return p, kw, "%s %dx%d tiles %dx%d kept %.1f %s batch %d %s" % (wdtype, M, K, bh, bw, frac, mask, batch, kw)


@pytest.mark.parametrize("seed,count,big", [(1, 60, False), (2, 60, False), (3, 40, True)])
def test_random_layers_match_the_oracle(seed, count, big):
    rng = np.random.default_rng(seed)
    for it in range(count):
        p, kw, desc = _case(rng, 100 * seed + it, big)
        print(desc, flush=True)
        G.check_fc(p, **kw)


@pytest.mark.parametrize("seed,count,big", [(4, 60, False), (5, 30, True)])
def test_random_layers_with_skewed_masks_match_the_oracle(seed, count, big):
    # the same sweep with Zipf-profile masks among the choices (long block rows are cut by the library's own
    # schedule) and the batch sizes between the kernel families' boundaries (5..8, 9..16, beyond)
    rng = np.random.default_rng(seed)
    for it in range(count):
        p, kw, desc = _case(rng, 100 * seed + it, big, skewed=True)
        print(desc, flush=True)
        G.check_fc(p, **kw)
