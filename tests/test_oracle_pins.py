"""Pins for the CPU oracle: each test checks it against something fixed by the
paper or by mathematics, not against itself.  CPU only."""
import math
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import pivot_oracle as O
from paper_1712_01084_amd import workloads as WL

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _golden_rows(name):
    rows = []
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                rows.append(line.split())
    return rows


# ---------------------------------------------------------------- conventions

def test_index_array_paper_example():
    (target, source, *idx), = _golden_rows("index_array_example.txt")
    got = O.index_array_of(target, source)
    assert got.tolist() == [int(i) for i in idx]
    # and it acts as a gather: source[idx] spells target
    assert "".join(source[i] for i in got) == target


def test_gather_matrix_matches_index_form_and_is_orthogonal():
    rng = np.random.default_rng(1)
    p = rng.permutation(7)
    G = O.gather_matrix(p)
    v = rng.standard_normal(7)
    assert np.array_equal(G @ v, v[p])
    assert np.array_equal(G @ G.T, np.eye(7))
    inv = O.invert_permutation(p)
    assert np.array_equal(inv[p], np.arange(7))
    assert np.array_equal(O.gather_matrix(inv), G.T)


def test_is_permutation_rejects_bad_arrays():
    assert O.is_permutation(np.array([2, 0, 1]))
    assert not O.is_permutation(np.array([0, 0, 1]))
    assert not O.is_permutation(np.array([0, 1, 3]))
    assert not O.is_permutation(np.array([-1, 0, 1]))
    with pytest.raises(ValueError):
        O.invert_permutation(np.array([1, 1, 0]))


# ---------------------------------------------------- brute force, exact, tiny

def _brute_pbp(Wp, tile_mask, prow, pcol, bias, x, bh, bw, relu):
    """a_out = P_row (M_block (P_col a_in)) + b written out with explicit
    0/1 permutation matrices and pure-Python rational arithmetic.
    P_col gathers (Listing 1 line 4), P_row scatters (Listing 1 line 9)."""
    M, K = len(Wp), len(Wp[0])
    Mb = [[Fraction(Wp[r][c]) if tile_mask[r // bh][c // bw] else Fraction(0)
           for c in range(K)] for r in range(M)]
    Pc = [[1 if pcol[i] == j else 0 for j in range(K)] for i in range(K)]      # (Pc v)[i] = v[pcol[i]]
    Pr = [[1 if prow[r] == i else 0 for r in range(M)] for i in range(M)]      # (Pr v)[prow[r]] = v[r]
    ys = []
    for xv in x:
        xg = [sum(Pc[i][j] * Fraction(xv[j]) for j in range(K)) for i in range(K)]
        v = [sum(Mb[r][c] * xg[c] for c in range(K)) for r in range(M)]
        y = [sum(Pr[i][r] * v[r] for r in range(M)) + Fraction(bias[i]) for i in range(M)]
        if relu:
            y = [max(t, Fraction(0)) for t in y]
        ys.append(y)
    return ys


@pytest.mark.parametrize("M,K,bh,bw,seed", [(12, 9, 2, 3, 0), (8, 12, 4, 4, 1), (7, 10, 2, 3, 2), (6, 6, 3, 2, 3)])
@pytest.mark.parametrize("relu", [False, True])
def test_oracle_fc_equals_exact_brute_force(M, K, bh, bw, seed, relu):
    rng = np.random.default_rng(seed)
    nbr, nbc = -(-M // bh), -(-K // bw)
    tm = (rng.random((nbr, nbc)) < 0.5).astype(np.uint8)
    tm[0, :] = 0                      # one empty block row
    prow, pcol = rng.permutation(M), rng.permutation(K)
    Wp = rng.integers(-8, 9, size=(M, K)).astype(np.float64)
    bias = rng.integers(-4, 5, size=M).astype(np.float64)
    x = rng.integers(-5, 6, size=(2, K)).astype(np.float64)
    want = _brute_pbp(Wp.tolist(), tm.tolist(), prow.tolist(), pcol.tolist(), bias.tolist(),
                      x.tolist(), bh, bw, relu)
    got = O.oracle_fc(Wp, tm, prow, pcol, bias, x, bh, bw, O.ACT_RELU if relu else O.ACT_NONE)
    assert got.shape == (2, M)
    for n in range(2):
        for i in range(M):
            assert Fraction(got[n, i]) == want[n][i]      # integer data: float64 is exact


def test_oracle_fc_float_inputs_close_to_rational_result():
    rng = np.random.default_rng(5)
    M, K, bh, bw = 8, 9, 2, 3
    tm = (rng.random((4, 3)) < 0.6).astype(np.uint8)
    prow, pcol = rng.permutation(M), rng.permutation(K)
    Wp = rng.standard_normal((M, K)).astype(np.float32)
    bias = rng.standard_normal(M).astype(np.float32)
    x = rng.standard_normal((1, K)).astype(np.float32)
    want = _brute_pbp(Wp.tolist(), tm.tolist(), prow.tolist(), pcol.tolist(), bias.tolist(), x.tolist(), bh, bw, False)
    got, D = O.oracle_fc(Wp, tm, prow, pcol, bias, x, bh, bw, O.ACT_NONE, return_scale=True)
    for i in range(M):
        assert abs(Fraction(got[0, i]) - want[0][i]) <= Fraction(1, 10 ** 13) * max(1, Fraction(D[0, i]))


def test_planted_mistakes_are_caught_by_the_brute_force_pin():
    """Mutants of the natural-coordinate construction (swapped gather/scatter,
    mask applied in natural space, transposed operand) all disagree with the
    exact brute force on this input, so the pin would catch them."""
    rng = np.random.default_rng(11)
    M, K, bh, bw = 8, 8, 2, 2
    tm = (rng.random((4, 4)) < 0.5).astype(np.uint8)
    prow, pcol = rng.permutation(M), rng.permutation(K)
    Wp = rng.integers(-8, 9, size=(M, K)).astype(np.float64)
    bias = np.zeros(M)
    x = rng.integers(-5, 6, size=(1, K)).astype(np.float64)
    want = np.array([[float(v) for v in row] for row in
                     _brute_pbp(Wp.tolist(), tm.tolist(), prow.tolist(), pcol.tolist(), bias.tolist(), x.tolist(), bh, bw, False)])
    keep = O.expand_tile_mask(tm, bh, bw, M, K)
    Wm = np.where(keep, Wp, 0.0)
    good = np.empty((M, K)); good[np.ix_(prow, pcol)] = Wm
    assert np.array_equal(x @ good.T, want)
    def placed(rows, cols, src):
        A = np.zeros((M, K))
        A[np.ix_(rows, cols)] = src
        return A

    inv_r, inv_c = O.invert_permutation(prow), O.invert_permutation(pcol)
    mutants = {
        "gather_instead_of_scatter": Wm[np.ix_(prow, pcol)],
        "inverse_perms": placed(inv_r, inv_c, Wm),
        "mask_in_natural_space": np.where(keep, placed(prow, pcol, Wp), 0.0),
        "transposed": good.T,
        "swapped_perms": placed(pcol, prow, Wm),
        "row_perm_dropped": placed(np.arange(M), pcol, Wm),
        "col_perm_dropped": placed(prow, np.arange(K), Wm),
    }
    for name, Wbad in mutants.items():
        assert not np.array_equal(x @ Wbad.T, want), name


# ------------------------------------------------ reductions to library routines

def test_identity_perms_all_tiles_is_plain_matvec():
    rng = np.random.default_rng(2)
    M, K = 24, 40
    Wp = rng.standard_normal((M, K)).astype(np.float32)
    x = rng.standard_normal((3, K)).astype(np.float32)
    b = rng.standard_normal(M).astype(np.float32)
    y = O.oracle_fc(Wp, np.ones((3, 5), np.uint8), np.arange(M), np.arange(K), b, x, 8, 8, O.ACT_NONE)
    want = x.astype(np.float64) @ Wp.astype(np.float64).T + b.astype(np.float64)
    assert np.allclose(y, want, rtol=0, atol=1e-13)


def test_linearity_and_relu():
    p = WL.gen_fc(40, 56, 8, 8, 0.4, seed=3)
    args = (p.Wp, p.tile_mask, p.prow, p.pcol)
    x1 = p.x.astype(np.float64)
    x2 = np.random.default_rng(9).standard_normal(x1.shape)
    z = lambda xx, bb: O.oracle_fc(*args, bb, xx, p.bh, p.bw, O.ACT_NONE)
    zero = np.zeros(p.M)
    assert np.allclose(z(2 * x1 + 3 * x2, zero), 2 * z(x1, zero) + 3 * z(x2, zero), atol=1e-12)
    assert np.allclose(z(x1, p.bias) - z(x1, zero), p.bias.astype(np.float64)[None, :], atol=1e-14)
    yr = O.oracle_fc(*args, p.bias, x1, p.bh, p.bw, O.ACT_RELU)
    assert np.array_equal(yr, np.maximum(z(x1, p.bias), 0))


def test_ragged_rows_and_empty_block_row():
    M, K, bh, bw = 10, 8, 4, 4            # last block row has 2 valid rows
    rng = np.random.default_rng(4)
    tm = np.array([[1, 0], [0, 0], [1, 1]], dtype=np.uint8)
    prow, pcol = rng.permutation(M), rng.permutation(K)
    Wp = rng.standard_normal((M, K))
    b = rng.standard_normal(M)
    x = rng.standard_normal((1, K))
    y = O.oracle_fc(Wp, tm, prow, pcol, b, x, bh, bw, O.ACT_RELU)
    # block row 1 (block-space rows 4..7) is empty: its outputs are relu(b)
    for r in range(4, 8):
        assert y[0, prow[r]] == max(b[prow[r]], 0.0)
    # row 9 (block row 2, all tiles kept) is a full dot product
    r = 9
    assert math.isclose(y[0, prow[r]], max(0.0, float(Wp[r] @ x[0, pcol] + b[prow[r]])), rel_tol=1e-12)


def test_error_scale_brute_force():
    p = WL.gen_fc(12, 12, 4, 4, 0.5, seed=8, batch=2)
    Wd = O.dense_masked_natural(p.Wp, p.tile_mask, p.prow, p.pcol, 4, 4)
    D = O.error_scale(Wd, p.x, p.bias)
    for n in range(2):
        for i in range(12):
            s = sum(abs(Wd[i, j]) * abs(float(p.x[n, j])) for j in range(12)) + abs(float(p.bias[i]))
            assert math.isclose(D[n, i], s, rel_tol=1e-12, abs_tol=1e-300)
    assert O.max_scaled_error(np.ones((1, 2)), np.ones((1, 2)), np.zeros((1, 2))) == 0.0
    assert O.max_scaled_error(np.array([[1.0, 2.0]]), np.array([[1.0, 2.5]]), np.array([[0.0, 1.0]])) == 0.5
    assert O.max_scaled_error(np.array([[1.0]]), np.array([[2.0]]), np.array([[0.0]])) == np.inf


# ------------------------------------------------------ Observations 1 and 2

def test_observation1_pointwise_ops_and_softmax_commute_with_permutations():
    rng = np.random.default_rng(6)
    v = rng.standard_normal(33)
    p = rng.permutation(33)
    assert np.array_equal(np.maximum(v, 0)[p], np.maximum(v[p], 0))
    sm = lambda u: np.exp(u - u.max()) / np.exp(u - u.max()).sum()
    assert np.allclose(sm(v)[p], sm(v[p]), rtol=1e-15, atol=0)


def test_observation2_composition_and_boundary_array():
    rng = np.random.default_rng(7)
    n = 20
    prow_a, pcol_b = rng.permutation(n), rng.permutation(n)
    q = O.compose_boundary(prow_a, pcol_b)
    assert O.is_permutation(q)
    # meaning: producer leaves v_a in block order with h[prow_a[r]] = v_a[r]
    v_a = rng.standard_normal(n)
    h = np.empty(n); h[prow_a] = v_a
    assert np.array_equal(v_a[q], h[pcol_b])
    # as matrices: gather(pcol_b) @ scatter(prow_a) == gather(q)
    assert np.array_equal(O.gather_matrix(pcol_b) @ O.gather_matrix(prow_a).T, O.gather_matrix(q))
    # elimination condition (Section 4.2.3): identity iff pcol_b == prow_a
    assert np.array_equal(O.compose_boundary(prow_a, prow_a), np.arange(n))
    assert not np.array_equal(q, np.arange(n))


# ------------------------------------------------------------- chains of layers

def _block_space_chain(layers, x):
    """Independent of oracle_mlp: run the chain the way the fused device path
    does it, entirely in block space with composed boundary arrays, float64."""
    L0 = layers[0]
    xg = x.astype(np.float64)[:, L0["pcol"]]
    for li, L in enumerate(layers):
        M, K = L["Wp"].shape
        keep = O.expand_tile_mask(L["tile_mask"], L["bh"], L["bw"], M, K)
        Mb = np.where(keep, L["Wp"].astype(np.float64), 0.0)
        v = xg @ Mb.T + L["bias"].astype(np.float64)[L["prow"]][None, :]
        v = O.apply_act(v, L["act"])
        if li + 1 < len(layers):
            q = O.compose_boundary(L["prow"], layers[li + 1]["pcol"])
            xg = v[:, q]
        else:
            y = np.empty_like(v)
            y[:, L["prow"]] = v
    return y


def _as_layers(problems):
    return [dict(Wp=p.Wp, tile_mask=p.tile_mask, prow=p.prow, pcol=p.pcol, bias=p.bias,
                 bh=p.bh, bw=p.bw, act=p.act) for p in problems]


@pytest.mark.parametrize("eliminated", [False, True])
def test_fused_chain_equals_natural_coordinate_chain(eliminated):
    probs = WL.config4(seed=1, dims=(96, 64, 64, 40), eliminated=eliminated)
    layers = _as_layers(probs)
    x = probs[0].x
    y_nat = O.oracle_mlp(layers, x)
    y_blk = _block_space_chain(layers, x)
    assert np.allclose(y_nat, y_blk, rtol=1e-12, atol=1e-13)
    qs, dsts = O.oracle_mlp_plan([p.prow for p in probs], [p.pcol for p in probs],
                                 [p.nbr * p.bh for p in probs])
    for l, q in enumerate(qs):
        assert O.is_permutation(q)
        assert np.array_equal(q, np.arange(len(q))) == eliminated
        # producer-side scatter form is the inverse map
        d = dsts[l][:probs[l].M]
        assert np.array_equal(q[d], np.arange(probs[l].M))


def test_mlp_boundary_rounding_happens_once_between_layers():
    probs = WL.config4(seed=2, dims=(64, 32, 32), wdtype=WL.F16)
    layers = _as_layers(probs)
    outs, scales, chain = O.oracle_mlp(layers, probs[0].x, boundary_dtype=np.float16, return_all=True)
    assert np.array_equal(chain[0], scales[0]) and np.all(chain[1] >= scales[1])
    h1 = outs[0].astype(np.float16)
    want = O.oracle_fc(probs[1].Wp, probs[1].tile_mask, probs[1].prow, probs[1].pcol, probs[1].bias,
                       h1, 32, 32, probs[1].act)
    assert np.array_equal(outs[1], want)


def _chain_scale_loops(layers, x):
    """S_L of a chain written out with scalar loops: S_1 = D_1, S_l[i] = sum_j |W_l[i][j]| S_{l-1}[j] + D_l[i],
    D_l[i] = sum_j |W_l[i][j]| |h_{l-1}[j]| + |b_l[i]|, everything in natural coordinates from the definition of
    the masked matrix (tile of block-space (r,c) kept), no call into the oracle."""
    h = [float(v) for v in x]
    S = None
    for L in layers:
        Wp, tm, prow, pcol, b = L["Wp"], L["tile_mask"], L["prow"], L["pcol"], L["bias"]
        M, K, bh, bw = Wp.shape[0], Wp.shape[1], L["bh"], L["bw"]
        Wd = [[0.0] * K for _ in range(M)]
        for r in range(M):
            for c in range(K):
                if tm[r // bh][c // bw]:
                    Wd[int(prow[r])][int(pcol[c])] = float(Wp[r][c])
        z = [sum(Wd[i][j] * h[j] for j in range(K)) + float(b[i]) for i in range(M)]
        D = [sum(abs(Wd[i][j]) * abs(h[j]) for j in range(K)) + abs(float(b[i])) for i in range(M)]
        S = D if S is None else [sum(abs(Wd[i][j]) * S[j] for j in range(K)) + D[i] for i in range(M)]
        h = [max(v, 0.0) for v in z] if L["act"] == O.ACT_RELU else z
    return S, D, h


def test_chain_error_scale_against_scalar_loops():
    # the scale every chain parity gate divides by, recomputed with plain loops on a tiny three-layer chain
    probs = WL.config4(seed=11, dims=(14, 9, 11, 6), bh=2, bw=3, frac=0.5)
    layers = _as_layers(probs)
    outs, scales, chain = O.oracle_mlp(layers, probs[0].x, return_all=True)
    S, D, h = _chain_scale_loops(layers, probs[0].x[0])
    assert np.allclose(chain[-1][0], S, rtol=1e-12, atol=0)
    assert np.allclose(scales[-1][0], D, rtol=1e-12, atol=0)
    assert np.allclose(outs[-1][0], h, rtol=1e-12, atol=1e-15)
    # S_L >= D_L always, and strictly larger wherever an earlier layer feeds the output
    assert np.all(chain[-1] >= scales[-1]) and np.any(chain[-1] > scales[-1] * 1.01)
    # one layer: the chain scale is the layer scale
    o1, s1, c1 = O.oracle_mlp(layers[:1], probs[0].x, return_all=True)
    assert np.array_equal(c1[0], s1[0])


def _perturbed_chain(layers, x, eps, target):
    """The chain in float64 with every layer's pre-activation pushed by eps*D_l, signs chosen so that every push
    moves output `target` of the last layer upwards (the worst case a per-layer relative error eps allows, to
    first order).  Signs come from back-propagating through |.|-free products: sign of d out[target] / d z_l[i]."""
    Wds = [O.dense_masked_natural(L["Wp"], L["tile_mask"], L["prow"], L["pcol"], L["bh"], L["bw"]) for L in layers]
    hs, zs = [np.asarray(x, dtype=np.float64)], []
    for L, Wd in zip(layers, Wds):
        z = hs[-1] @ Wd.T + np.asarray(L["bias"], dtype=np.float64)
        zs.append(z)
        hs.append(np.maximum(z, 0) if L["act"] == O.ACT_RELU else z)
    g = np.zeros(Wds[-1].shape[0]); g[target] = 1.0
    signs = [None] * len(layers)
    for l in range(len(layers) - 1, -1, -1):
        if layers[l]["act"] == O.ACT_RELU:
            g = g * (zs[l][0] > 0)
        signs[l] = np.sign(g)
        g = g @ Wds[l]
    h = np.asarray(x, dtype=np.float64)
    for l, (L, Wd) in enumerate(zip(layers, Wds)):
        z = h @ Wd.T + np.asarray(L["bias"], dtype=np.float64)
        D = np.abs(h) @ np.abs(Wd).T + np.abs(np.asarray(L["bias"], dtype=np.float64))
        z = z + eps * signs[l] * D
        h = np.maximum(z, 0) if L["act"] == O.ACT_RELU else z
    return h


def test_chain_error_scale_bounds_a_per_layer_relative_error_and_the_layer_scale_does_not():
    # why chains are gated against eps*S_L: a relative error eps in EVERY layer (each within its own eps*D_l) can
    # move the last output by more than eps*D_L, but never (to first order) by more than eps*S_L
    probs = WL.config4(seed=12, dims=(48, 40, 32, 24), bh=4, bw=4, frac=0.5)
    layers = _as_layers(probs)
    outs, scales, chain = O.oracle_mlp(layers, probs[0].x, return_all=True)
    eps = 1e-7
    worst_S, worst_D = 0.0, 0.0
    for target in range(24):
        y = _perturbed_chain(layers, probs[0].x, eps, target)
        d = abs(y[0][target] - outs[-1][0][target])
        worst_S = max(worst_S, d / (eps * chain[-1][0][target]))
        worst_D = max(worst_D, d / (eps * scales[-1][0][target]))
    assert worst_S <= 1.0 + 1e-4            # never above eps*S_L (second-order terms are ~eps)
    assert worst_S > 0.2                    # and S_L is not loose: the worst case reaches a third of it (the rest
                                            # of S_L are paths through units the ReLU has switched off)
    assert worst_D > 1.05                   # eps*D_L alone IS exceeded by an error every layer is allowed to make


def test_gather_index_composed_with_the_tile_list():
    # xidx[t*bw + c] = pcol_pad[col_idx[t]*bw + c]: x index of column c of kept tile t, -1 in padding columns
    for M, K, bh, bw, seed in ((21, 30, 4, 8, 1), (12, 9, 2, 3, 2), (16, 16, 4, 4, 3)):
        p = WL.gen_fc(M, K, bh, bw, 0.5, seed=seed)
        plan = O.oracle_plan(p.Wp, True, p.tile_mask, p.prow, p.pcol, p.bias, M, K, bh, bw, O.LAYOUT_BRC, 2)
        T = plan["T"]
        assert plan["xidx"].shape == (T * bw,) and plan["xidx"].dtype == np.int32
        t = 0
        for i in range(p.nbr):
            for j in range(p.nbc):
                if not p.tile_mask[i][j]:
                    continue
                for c in range(bw):
                    col = j * bw + c                                  # block-space column
                    want = int(p.pcol[col]) if col < K else -1
                    assert plan["xidx"][t * bw + c] == want
                    assert plan["xidx"][t * bw + c] == plan["pcol_pad"][plan["col_idx"][t] * bw + c]
                t += 1
        assert t == T
        # and it is the gather Listing 1 does: x[xidx] spells the x-segments of the kept tiles in block order
        x = np.arange(K, dtype=np.float64) + 100.0
        xg = np.concatenate([x[p.pcol], np.zeros(p.nbc * bw - K)])
        seg = np.where(plan["xidx"] >= 0, x[np.maximum(plan["xidx"], 0)], 0.0)
        for t in range(T):
            j = plan["col_idx"][t]
            assert np.array_equal(seg[t * bw:(t + 1) * bw], xg[j * bw:(j + 1) * bw])


# -------------------------------------------------------------------- the plan

def test_value_offset_hand_computed_and_bijective():
    # tiles 2x3, T=4: hand-computed positions
    assert O.value_offset(O.LAYOUT_BRC, 1, 0, 1, 4, 2, 3) == 7
    assert O.value_offset(O.LAYOUT_BCR, 1, 0, 1, 4, 2, 3) == 8
    assert O.value_offset(O.LAYOUT_CBR, 1, 0, 1, 4, 2, 3) == 10
    for layout in (O.LAYOUT_BRC, O.LAYOUT_BCR, O.LAYOUT_CBR):
        seen = sorted(O.value_offset(layout, t, r, c, 4, 2, 3)
                      for t in range(4) for r in range(2) for c in range(3))
        assert seen == list(range(24))
    # fastest axis: BRC -> column, BCR and CBR -> row (Section 4.1.1)
    assert O.value_offset(O.LAYOUT_BRC, 2, 1, 2, 4, 2, 3) - O.value_offset(O.LAYOUT_BRC, 2, 1, 1, 4, 2, 3) == 1
    assert O.value_offset(O.LAYOUT_BCR, 2, 1, 2, 4, 2, 3) - O.value_offset(O.LAYOUT_BCR, 2, 0, 2, 4, 2, 3) == 1
    assert O.value_offset(O.LAYOUT_CBR, 2, 1, 2, 4, 2, 3) - O.value_offset(O.LAYOUT_CBR, 1, 1, 2, 4, 2, 3) == 2


@pytest.mark.parametrize("layout", [O.LAYOUT_BRC, O.LAYOUT_BCR, O.LAYOUT_CBR])
@pytest.mark.parametrize("pivoted", [True, False])
@pytest.mark.parametrize("M,K,bh,bw", [(24, 32, 8, 8), (21, 30, 4, 8)])
def test_plan_round_trip_is_bit_exact(layout, pivoted, M, K, bh, bw):
    p = WL.gen_fc(M, K, bh, bw, 0.45, seed=12, wdtype=WL.F16)
    W = p.Wp if pivoted else O.unpivot_weights(p.Wp, p.prow, p.pcol)
    plan = O.oracle_plan(W, pivoted, p.tile_mask, p.prow, p.pcol, p.bias, M, K, bh, bw, layout, 3)
    assert plan["row_ptr"][-1] == plan["T"] == p.T
    for i in range(p.nbr):
        cols = plan["col_idx"][plan["row_ptr"][i]:plan["row_ptr"][i + 1]]
        assert np.all(np.diff(cols) > 0)
        assert np.array_equal(np.nonzero(p.tile_mask[i])[0], cols)
    back = O.unpack_plan_to_dense(plan, M, K, bh, bw, layout)
    want = O.dense_masked_natural(p.Wp, p.tile_mask, p.prow, p.pcol, bh, bw)
    assert back.dtype == np.float16
    assert np.array_equal(back.astype(np.float64), want)           # values are copies: bit-for-bit
    assert np.array_equal(plan["bias_p"][:M], p.bias[p.prow])
    assert np.all(plan["bias_p"][M:] == 0)


def test_schedule_covers_every_tile_once_in_longest_first_order():
    row_ptr = np.array([0, 7, 7, 9, 20, 21], dtype=np.int32)
    chunks, part_base = O.build_schedule(row_ptr, 4)
    want_canonical = [(0, 0, 4), (0, 4, 7), (1, 7, 7), (2, 7, 9), (3, 9, 13), (3, 13, 17), (3, 17, 20), (4, 20, 21)]
    by_slot = sorted(chunks.tolist(), key=lambda c: c[3])
    assert [tuple(c[:3]) for c in by_slot] == want_canonical
    assert part_base.tolist() == [0, 2, 3, 4, 7, 8]
    lens = (chunks[:, 2] - chunks[:, 1]).tolist()
    assert lens == sorted(lens, reverse=True) and max(lens) <= 4
    # stable: equal lengths stay in (block row, tile_begin) order
    assert [tuple(c[:3]) for c in chunks.tolist()] == [
        (0, 0, 4), (3, 9, 13), (3, 13, 17), (0, 4, 7), (3, 17, 20), (2, 7, 9), (4, 20, 21), (1, 7, 7)]
    covered = np.zeros(21, dtype=int)
    for br, b, e, _ in chunks.tolist():
        assert row_ptr[br] <= b <= e <= row_ptr[br + 1]
        covered[b:e] += 1
    assert np.all(covered == 1)


# ------------------------------------------------------------------------ LSTM

def test_lstm_cell_against_scalar_loop():
    rng = np.random.default_rng(13)
    H, B = 5, 2
    z = rng.standard_normal((B, 4 * H))
    c0 = rng.standard_normal((B, H))
    h, c = O.lstm_cell(z, c0, H)
    sg = lambda t: 1.0 / (1.0 + math.exp(-t))
    for n in range(B):
        for j in range(H):
            i_, f_, g_, o_ = z[n, j], z[n, H + j], z[n, 2 * H + j], z[n, 3 * H + j]
            cc = sg(f_) * c0[n, j] + sg(i_) * math.tanh(g_)
            assert math.isclose(c[n, j], cc, rel_tol=1e-14, abs_tol=1e-300)
            assert math.isclose(h[n, j], sg(o_) * math.tanh(cc), rel_tol=1e-14, abs_tol=1e-300)


def test_lstm_zero_weights_closed_form():
    """With a zero gate matrix the gates are constants set by the bias and the
    cell state is a geometric series: c_t = a (1 - s^t)/(1 - s)."""
    H, I, B, steps = 4, 3, 2, 9
    Wd = np.zeros((4 * H, H + I))
    rng = np.random.default_rng(14)
    bias = rng.standard_normal(4 * H)
    xs = rng.standard_normal((steps, B, I)).astype(np.float16)
    h, c, _ = O.oracle_lstm(Wd, bias, xs, np.zeros((B, H)), np.zeros((B, H)), H)
    sg = lambda t: 1.0 / (1.0 + np.exp(-t))
    a = sg(bias[0:H]) * np.tanh(bias[2 * H:3 * H])
    s = sg(bias[H:2 * H])
    c_want = a * (1 - s ** steps) / (1 - s)
    assert np.allclose(c, c_want[None, :], rtol=1e-12)
    assert np.allclose(h, (sg(bias[3 * H:]) * np.tanh(c_want))[None, :], rtol=1e-12)


def test_lstm_step_uses_h_then_x_concatenation_and_rounded_state():
    H, I, B = 3, 2, 1
    rng = np.random.default_rng(15)
    Wd = rng.standard_normal((4 * H, H + I))
    bias = rng.standard_normal(4 * H)
    xs = rng.standard_normal((2, B, I)).astype(np.float16)
    h0 = rng.standard_normal((B, H)).astype(np.float32)
    c0 = rng.standard_normal((B, H)).astype(np.float32)
    _, _, rec = O.oracle_lstm(Wd, bias, xs, h0, c0, H, record=(0, 1))
    z0 = Wd[:, :H] @ h0.astype(np.float16).astype(np.float64)[0] + Wd[:, H:] @ xs[0, 0].astype(np.float64) + bias
    assert np.allclose(rec[0]["z"][0], z0, rtol=1e-13)
    assert np.array_equal(rec[1]["h_fed"], rec[0]["h"].astype(np.float16))
    assert np.array_equal(rec[1]["c_prev"], rec[0]["c"])
