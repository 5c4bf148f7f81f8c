"""The seeded input generators: stated distributions, exact tile counts, and
the paper's experiment structure.  CPU only."""
import os

import numpy as np
import pytest

from paper_1712_01084_amd import workloads as WL

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rows(name):
    with open(os.path.join(GOLDEN, name)) as f:
        return [l.split() for l in f if l.strip() and not l.startswith("#")]


def test_paper_dimension_example_block_diagonal():
    (size, fill, nblk, edge), = _rows("paper_dimension_example.txt")
    p = WL.paper_grid_case(int(size), float(fill) / 100.0)
    assert (p.nbr, p.nbc, p.bh, p.bw) == (int(nblk), int(nblk), int(edge), int(edge))
    assert np.array_equal(p.tile_mask, np.eye(int(nblk), dtype=np.uint8))
    # no two blocks share rows or columns; kept coefficients = fill * size^2
    assert p.T * p.bh * p.bw == int(float(fill) / 100.0 * int(size) ** 2)
    assert p.meta["block_edge"] == int(edge) and p.meta["n_blocks"] == int(nblk)


def test_paper_grid_large_and_small_blocks():
    big = WL.paper_grid_case(1024, 0.25)                 # 4 blocks of 256x256 -> 64x64 tiles, 4x4 tiles per block
    assert (big.bh, big.bw, big.nbr) == (64, 64, 16) and big.T == 4 * 16
    assert np.all(big.tile_mask[:4, :4] == 1) and np.all(big.tile_mask[:4, 4:] == 0)
    assert big.T * 64 * 64 == 1024 * 1024 // 4
    small = WL.paper_grid_case(64, 0.03125)              # 32 blocks of 2x2 inside 8x8 tiles on the diagonal
    assert (small.bh, small.nbr, small.T) == (8, 8, 8)
    nz = small.Wp != 0
    r = np.arange(64)
    assert not np.any(nz & ((r[:, None] // 2) != (r[None, :] // 2)))      # nothing outside the 2x2 blocks
    assert int(nz.sum()) <= 32 * 4 and not nz[0, 2] and not nz[2, 0]
    for size in WL.PAPER_GRID_SIZES:
        for fill in WL.PAPER_GRID_FILLS:
            nblk = int(round(1 / fill))
            assert size % nblk == 0


def test_linear_speedup_is_reciprocal_fill():
    for fill, lin in _rows("table1_linear_speedup.txt"):
        p = WL.paper_grid_case(256, float(fill) / 100.0)
        assert p.M * p.K / (p.T * p.bh * p.bw) == float(lin)


def test_config1_counts_and_statistics():
    p = WL.config1(seed=0)
    assert (p.M, p.K, p.bh, p.bw, p.nbr, p.nbc) == (1024, 1024, 16, 16, 64, 64)
    assert p.T == 1024 and p.act == WL.ACT_RELU and p.Wp.dtype == np.float32
    assert sorted(p.prow.tolist()) == list(range(1024)) and sorted(p.pcol.tolist()) == list(range(1024))
    assert abs(float(p.Wp.std()) - 1024 ** -0.5) < 2e-4 and abs(float(p.Wp.mean())) < 2e-4
    assert abs(float(p.bias.std()) - 0.1) < 0.01
    assert abs(float(p.x.std()) - 1.0) < 0.1
    q = WL.config1(seed=0)
    assert np.array_equal(p.Wp, q.Wp) and np.array_equal(p.tile_mask, q.tile_mask)
    assert not np.array_equal(p.tile_mask, WL.config1(seed=1).tile_mask)
    assert p.algorithmic_bytes() == 1024 * 256 * 4 + 4 * 1024 + 4 * 65 + 1024 * 8 + 1024 * 8 + 4 * 1024


def test_config2_balanced_rows_small_scale():
    p = WL.config2(seed=0, M=256, K=9216)
    assert np.all(p.tile_mask.sum(axis=1) == 29) and p.nbc == 288
    assert np.all(p.x >= 0) and 0.3 < float((p.x == 0).mean()) < 0.7


def test_config3_fractions_and_dtype():
    for f, t in zip(WL.CONFIG3_FRACS, (819, 1638, 4096, 8192, 16384)):
        nbr, nbc = 64, 256
        rng = np.random.default_rng(0)
        m = WL.mask_full(nbr, nbc) if f >= 1 else WL.mask_uniform(rng, nbr, nbc, f)
        assert int(m.sum()) == t
    p = WL.config3(seed=0, batch=4, frac=0.25, M=256, K=256)
    assert p.Wp.dtype == np.float16 and p.x.dtype == np.float16 and p.x.shape == (4, 256)
    assert (p.bh, p.bw) == (64, 16)


def test_config4_shapes_and_elimination():
    ls = WL.config4(seed=0, dims=(256, 128, 128, 72))
    assert [(l.M, l.K) for l in ls] == [(128, 256), (128, 128), (72, 128)]
    assert [l.act for l in ls] == [WL.ACT_RELU, WL.ACT_RELU, WL.ACT_NONE]
    assert ls[2].nbr == 3 and ls[2].nbr * 32 > ls[2].M           # ragged last block row
    le = WL.config4(seed=0, dims=(256, 128, 128, 72), eliminated=True)
    assert np.array_equal(le[1].pcol, le[0].prow) and np.array_equal(le[2].pcol, le[1].prow)
    assert not np.array_equal(ls[1].pcol, ls[0].prow)
    assert WL.balanced_row_count(0.10, 784) == 78 and WL.balanced_row_count(0.10, 128) == 13
    assert WL.balanced_row_count(0.10, 288) == 29


def test_zipf_profile_full_size():
    prof = WL.zipf_profile(512, 96, 6144)
    assert int(prof.sum()) == 6144 and prof.max() == 96 and prof.min() >= 1
    assert np.all(np.diff(prof) <= 0)
    assert 10 <= int((prof == 96).sum()) <= 30
    lp = WL.config5(seed=0, H=64, I=32, steps=3, batch=2, frac=0.5)
    assert lp.fc.M == 256 and lp.fc.K == 96 and lp.xs.shape == (3, 2, 32)
    assert lp.fc.T == int(round(0.5 * lp.fc.nbr * lp.fc.nbc))
    assert np.all(lp.fc.tile_mask.sum(axis=1) >= 1)
