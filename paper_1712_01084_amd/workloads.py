"""Seeded synthetic inputs for pruned fully-connected layers in PBP form.

This module only *draws inputs* (tile masks, permutations, weights, biases,
activations).  It holds none of the method's arithmetic: no matrix product, no
packing, no permutation inversion or composition.  Both the CPU oracle's tests
and the HIP path's tests/bench take their inputs from here, so that the two
sides consume identical, already-rounded storage values.

Conventions (Section 4.1.4 of the paper, index-array form of a permutation):
an index array ``p`` acts as a gather, ``out[i] = in[p[i]]``.  ``prow`` and
``pcol`` pivot the natural-coordinate matrix into block space,
``W'[r][c] = W[prow[r]][pcol[c]]``; the tile mask lives in block space.

Draw order within one problem is fixed: mask, prow, pcol, W', bias, x.
The second parameter of every N(mean, v) in the workload list is a variance.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np

F32 = "f32"
F16 = "f16"

ACT_NONE = 0
ACT_RELU = 1


def storage_dtype(wdtype: str):
    return np.float32 if wdtype == F32 else np.float16


@dataclass
class FCProblem:
    """One pruned FC layer plus a batch of inputs, all in storage precision."""
    M: int
    K: int
    bh: int
    bw: int
    wdtype: str
    act: int
    tile_mask: np.ndarray      # uint8 [nbr][nbc], block (pivoted) space
    prow: np.ndarray           # int32 [M]
    pcol: np.ndarray           # int32 [K]
    Wp: np.ndarray             # storage dtype [M][K], block space (W')
    bias: np.ndarray           # float32 [M], natural output coordinates
    x: np.ndarray              # storage dtype [batch][K], natural coordinates
    name: str = ""
    meta: dict = field(default_factory=dict)

    @property
    def nbr(self) -> int:
        return -(-self.M // self.bh)

    @property
    def nbc(self) -> int:
        return -(-self.K // self.bw)

    @property
    def T(self) -> int:
        return int(self.tile_mask.sum())

    @property
    def batch(self) -> int:
        return int(self.x.shape[0])

    def algorithmic_bytes(self, batch: Optional[int] = None) -> int:
        """Bytes the method itself has to move for one layer application:
        kept tile values, block-sparse indices, x with its gather index,
        y with its scatter index, and the bias."""
        B = self.batch if batch is None else batch
        sw = 4 if self.wdtype == F32 else 2
        sx = sw
        T = self.T
        return (T * self.bh * self.bw * sw + 4 * T + 4 * (self.nbr + 1)
                + self.K * (4 + sx * B) + self.M * (4 + 4 * B) + 4 * self.M)

    def dense_bytes(self, batch: Optional[int] = None) -> int:
        B = self.batch if batch is None else batch
        sw = 4 if self.wdtype == F32 else 2
        return self.M * self.K * sw + self.K * sw * B + self.M * 4 * B + 4 * self.M


# ----------------------------------------------------------------------------
# tile masks
# ----------------------------------------------------------------------------

def mask_uniform(rng, nbr, nbc, frac):
    """Exactly round(frac*nbr*nbc) tiles, without replacement over the grid."""
    n = nbr * nbc
    t = int(round(frac * n))
    t = max(0, min(n, t))
    m = np.zeros(n, dtype=np.uint8)
    m[rng.choice(n, size=t, replace=False)] = 1
    return m.reshape(nbr, nbc)


def balanced_row_count(frac, nbc):
    return int(np.floor(frac * nbc + 0.5))


def mask_balanced(rng, nbr, nbc, frac):
    """The same number of tiles, floor(frac*nbc+0.5), in every block row."""
    per = max(0, min(nbc, balanced_row_count(frac, nbc)))
    m = np.zeros((nbr, nbc), dtype=np.uint8)
    for i in range(nbr):
        m[i, rng.choice(nbc, size=per, replace=False)] = 1
    return m


def zipf_profile(nbr, nbc, total, s=1.2):
    """Deterministic Zipf(s) profile of tiles per rank k=1..nbr.

    n_k = clip(floor(C*k^-s), 1, nbc) with C found by bisection so that the
    sum does not exceed ``total``; what is left is handed out one tile at a
    time in rank order, skipping full rows.
    """
    k = np.arange(1, nbr + 1, dtype=np.float64)
    w = k ** (-s)

    def counts(C):
        return np.clip(np.floor(C * w), 1, nbc).astype(np.int64)

    lo, hi = 0.0, float(nbc) * float(nbr) ** s + 1.0
    for _ in range(200):
        mid = 0.5 * (lo + hi)
        if counts(mid).sum() <= total:
            lo = mid
        else:
            hi = mid
    n = counts(lo)
    rem = int(total - n.sum())
    while rem > 0:
        progressed = False
        for i in range(nbr):
            if rem == 0:
                break
            if n[i] < nbc:
                n[i] += 1
                rem -= 1
                progressed = True
        if not progressed:
            break
    return n


def mask_zipf(rng, nbr, nbc, frac, s=1.2):
    total = int(round(frac * nbr * nbc))
    prof = zipf_profile(nbr, nbc, total, s)
    rows = rng.permutation(nbr)          # rank -> block row
    m = np.zeros((nbr, nbc), dtype=np.uint8)
    for rank in range(nbr):
        m[rows[rank], rng.choice(nbc, size=int(prof[rank]), replace=False)] = 1
    return m


def mask_full(nbr, nbc):
    return np.ones((nbr, nbc), dtype=np.uint8)


def mask_block_diagonal(nbr):
    """The paper's experiment structure (Section 5): identical square blocks
    on the diagonal, no two sharing rows or columns."""
    return np.eye(nbr, dtype=np.uint8)


# ----------------------------------------------------------------------------
# one layer
# ----------------------------------------------------------------------------

def _draw_normal(rng, shape, sigma, dtype):
    """N(0, sigma^2) drawn in float32 and rounded once to ``dtype``."""
    a = rng.standard_normal(size=shape, dtype=np.float32)
    a *= np.float32(sigma)
    return a.astype(dtype, copy=False)


def gen_fc(M, K, bh, bw, frac, seed, *, mask="uniform", wdtype=F32, batch=1,
           act=ACT_NONE, x_kind="normal", perms="random", name="",
           prow=None, pcol=None, rng=None, draw_x=True) -> FCProblem:
    rng = np.random.default_rng(seed) if rng is None else rng
    nbr, nbc = -(-M // bh), -(-K // bw)
    if isinstance(mask, np.ndarray):
        tm = np.ascontiguousarray(mask, dtype=np.uint8)
        assert tm.shape == (nbr, nbc)
    elif mask == "uniform":
        tm = mask_uniform(rng, nbr, nbc, frac)
    elif mask == "balanced":
        tm = mask_balanced(rng, nbr, nbc, frac)
    elif mask == "zipf":
        tm = mask_zipf(rng, nbr, nbc, frac)
    elif mask == "full":
        tm = mask_full(nbr, nbc)
    elif mask == "blockdiag":
        assert nbr == nbc
        tm = mask_block_diagonal(nbr)
    else:
        raise ValueError(mask)
    if prow is None:
        prow = (rng.permutation(M) if perms == "random" else np.arange(M))
    if pcol is None:
        pcol = (rng.permutation(K) if perms == "random" else np.arange(K))
    prow = np.ascontiguousarray(prow, dtype=np.int32)
    pcol = np.ascontiguousarray(pcol, dtype=np.int32)
    sd = storage_dtype(wdtype)
    Wp = _draw_normal(rng, (M, K), K ** -0.5, sd)
    bias = _draw_normal(rng, (M,), 0.1, np.float32)
    if draw_x:
        x = rng.standard_normal(size=(batch, K), dtype=np.float32)
        if x_kind == "relu_normal":
            np.maximum(x, 0, out=x)
        elif x_kind != "normal":
            raise ValueError(x_kind)
        x = x.astype(sd)
    else:
        x = np.zeros((batch, K), dtype=sd)
    return FCProblem(M, K, bh, bw, wdtype, act, tm, prow, pcol, Wp, bias, x,
                     name=name, meta=dict(seed=seed, frac=frac, mask=str(mask) if not isinstance(mask, np.ndarray) else "given"))


# ----------------------------------------------------------------------------
# the five workload configurations (full size unless scale < 1)
# ----------------------------------------------------------------------------

def config1(seed=0, batch=1):
    """1024x1024 fp32, 16x16 tiles, 25 % kept uniformly at random, ReLU."""
    return gen_fc(1024, 1024, 16, 16, 0.25, seed, mask="uniform", wdtype=F32,
                  batch=batch, act=ACT_RELU, name="cfg1_1024x1024_f32_t16x16_25")


def config2(seed=0, batch=1, M=4096, K=9216):
    """AlexNet-fc6 shape, fp32, 32x32 tiles, 10 % kept, balanced rows,
    x = ReLU(N(0,1)), ReLU output."""
    return gen_fc(M, K, 32, 32, 0.10, seed, mask="balanced", wdtype=F32,
                  batch=batch, act=ACT_RELU, x_kind="relu_normal",
                  name="cfg2_%dx%d_f32_t32x32_10bal" % (M, K))


CONFIG3_FRACS = (0.05, 0.10, 0.25, 0.50, 1.00)


def config3(seed=0, batch=1, frac=0.10, M=4096, K=4096):
    """4096x4096 fp16 weights, fp32 accumulate, 64x16 tiles, identity act."""
    return gen_fc(M, K, 64, 16, frac, seed,
                  mask=("full" if frac >= 1.0 else "uniform"), wdtype=F16,
                  batch=batch, act=ACT_NONE,
                  name="cfg3_%dx%d_f16_t64x16_%g_b%d" % (M, K, frac * 100, batch))


def config4(seed=0, batch=1, dims=(25088, 4096, 4096, 1000), eliminated=False,
            wdtype=F32, bh=32, bw=32, frac=0.10) -> List[FCProblem]:
    """VGG FC shapes, 32x32 tiles, 10 % kept per layer, balanced, ReLU between
    layers and identity on the logits.  ``eliminated`` makes every layer's
    column index array equal to the previous layer's row index array, the
    condition under which the composed boundary permutation is the identity
    (Section 4.2.3)."""
    rng = np.random.default_rng(seed)
    layers = []
    prev_prow = None
    L = len(dims) - 1
    for l in range(L):
        K, M = dims[l], dims[l + 1]
        pcol = prev_prow if (eliminated and prev_prow is not None) else None
        p = gen_fc(M, K, bh, bw, frac, seed, mask="balanced", wdtype=wdtype,
                   batch=batch, act=(ACT_RELU if l < L - 1 else ACT_NONE),
                   x_kind="relu_normal", pcol=pcol, rng=rng, draw_x=(l == 0),
                   name="cfg4_L%d_%dx%d" % (l + 1, M, K))
        prev_prow = p.prow
        layers.append(p)
    return layers


@dataclass
class LSTMProblem:
    fc: FCProblem              # gate matrix 4H x (H+I); fc.x unused
    H: int
    I: int
    xs: np.ndarray             # storage dtype [steps][batch][I]
    h0: np.ndarray             # float32 [batch][H]
    c0: np.ndarray             # float32 [batch][H]


def config5(seed=0, batch=8, H=2048, I=1024, steps=256, frac=0.125):
    """LSTM gate matrix 4H x (H+I), fp16 weights, 16x32 tiles, Zipf(1.2) row
    profile; gate order (i,f,g,o); input [h_{t-1}; x_t]; zero initial state."""
    rng = np.random.default_rng(seed)
    fc = gen_fc(4 * H, H + I, 16, 32, frac, seed, mask="zipf", wdtype=F16,
                batch=batch, act=ACT_NONE, rng=rng, draw_x=False,
                name="cfg5_lstm_H%d_I%d_f16_t16x32_zipf" % (H, I))
    xs = rng.standard_normal(size=(steps, batch, I), dtype=np.float32).astype(np.float16)
    h0 = np.zeros((batch, H), dtype=np.float32)
    c0 = np.zeros((batch, H), dtype=np.float32)
    return LSTMProblem(fc, H, I, xs, h0, c0)


def paper_grid_case(size, fill, seed=0, wdtype=F32, batch=1, perms="random", act=ACT_NONE):
    """The paper's experiment structure (Section 5): a square matrix with 1/fill
    identical square blocks of edge size*fill on the diagonal, no two sharing
    rows or columns (size 512 at 6.25 % is 16 blocks of 32x32).  Blocks larger
    than the largest device tile (64) are cut into 64x64 tiles; blocks smaller
    than the smallest (8) share an 8x8 tile on the diagonal, with zeros between
    them (the values outside the true blocks are zeroed here)."""
    nblk = int(round(1.0 / fill))
    edge = size // nblk
    assert edge * nblk == size and edge >= 1
    tile = min(max(edge, 8), 64)
    nbr = -(-size // tile)
    idx = np.arange(nbr)
    if edge >= tile:
        per = edge // tile
        mask = (idx[:, None] // per == idx[None, :] // per).astype(np.uint8)
    else:
        mask = np.eye(nbr, dtype=np.uint8)
    p = gen_fc(size, size, tile, tile, fill, seed, mask=mask, wdtype=wdtype, batch=batch, act=act, perms=perms,
               name="grid_%d_%g" % (size, fill * 100))
    if edge < tile:
        r = np.arange(size)
        p.Wp[(r[:, None] // edge) != (r[None, :] // edge)] = 0
    p.meta.update(block_edge=edge, n_blocks=nblk, fill=fill)
    return p


PAPER_GRID_SIZES = (64, 128, 256, 512, 1024, 2048, 4096)
PAPER_GRID_FILLS = (0.03125, 0.0625, 0.125, 0.25)
