"""Feed-back PBP permutation search (Section 3.2): pins of the oracle's
heuristic, then the host library against the oracle, index for index.  CPU only."""
import itertools
import os

import numpy as np
import pytest

from oracle import pivot_oracle as O
from paper_1712_01084_amd import binding as B

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rows(name):
    with open(os.path.join(GOLDEN, name)) as f:
        return [l.split() for l in f if l.strip() and not l.startswith("#")]


def _diag_mass(A, R, C, r1, c1):
    A = np.asarray(A, dtype=np.float64)
    return A[np.ix_(R[:r1], C[:c1])].sum() + A[np.ix_(R[r1:], C[c1:])].sum()


# ---- pins of the oracle ------------------------------------------------------

def test_fill_in_after_bisections_matches_the_papers_numbers():
    for lv, pct in _rows("feedback_fill_in.txt"):
        lv, pct = int(lv), float(pct)
        n = 64
        rr, cc = O.feedback_block_ranges(n, lv), O.feedback_block_ranges(n, lv)
        assert len(rr) == 2 ** lv
        kept = sum((re - rb) * (ce - cb) for (rb, re), (cb, ce) in zip(rr, cc))
        assert 100.0 * kept / (n * n) == pct
        # captured mass of an all-ones matrix is exactly that share
        ones = np.ones((n, n))
        ident = np.arange(n)
        assert O.feedback_captured_mass(ones, ident, ident, lv) == kept


def test_block_ranges_ragged_floor_first():
    assert O.feedback_block_ranges(7, 2) == [(0, 1), (1, 3), (3, 5), (5, 7)]
    assert O.feedback_block_ranges(3, 3) == [(0, 1), (1, 2), (2, 3)]


@pytest.mark.parametrize("seed", range(6))
def test_half_step_is_the_best_choice_for_its_side_by_brute_force(seed):
    rng = np.random.default_rng(seed)
    M, K = 6, 5
    A = rng.integers(0, 9, size=(M, K)).astype(np.float64)
    R = list(rng.permutation(M))
    C = list(rng.permutation(K))
    r1, c1 = M // 2, K // 2
    R2 = O.feedback_half_step(A, R, C, r1, c1, True)
    assert sorted(R2) == sorted(R)
    best = max(_diag_mass(A, list(S) + [r for r in R if r not in S], C, r1, c1)
               for S in itertools.combinations(R, r1))
    assert _diag_mass(A, R2, C, r1, c1) == best
    C2 = O.feedback_half_step(A, C, R2, c1, r1, False)
    best_c = max(_diag_mass(A, R2, list(S) + [c for c in C if c not in S], r1, c1)
                 for S in itertools.combinations(C, c1))
    assert _diag_mass(A, R2, C2, r1, c1) == best_c
    # both halves keep the relative order of the list they came from
    pos = {v: i for i, v in enumerate(R)}
    assert [pos[v] for v in R2[:r1]] == sorted(pos[v] for v in R2[:r1])
    assert [pos[v] for v in R2[r1:]] == sorted(pos[v] for v in R2[r1:])


@pytest.mark.parametrize("seed", range(6))
def test_search_ends_in_a_split_no_single_side_move_improves_and_never_loses_mass(seed):
    rng = np.random.default_rng(100 + seed)
    M, K = 6, 6
    A = rng.integers(0, 9, size=(M, K)).astype(np.float64)
    p0, c0 = rng.permutation(M), rng.permutation(K)
    prow, pcol = O.feedback_search(A, 1, p0, c0)
    assert O.is_permutation(prow, M) and O.is_permutation(pcol, K)
    R, C = list(prow), list(pcol)
    got = _diag_mass(A, R, C, 3, 3)
    assert got >= _diag_mass(A, list(p0), list(c0), 3, 3)
    assert got == O.feedback_captured_mass(A, prow, pcol, 1)
    for S in itertools.combinations(R, 3):
        assert _diag_mass(A, list(S) + [r for r in R if r not in S], C, 3, 3) <= got
    for S in itertools.combinations(C, 3):
        assert _diag_mass(A, R, list(S) + [c for c in C if c not in S], 3, 3) <= got
    # and it cannot beat the true optimum over all splits of both sides
    opt = max(_diag_mass(A, list(S) + [r for r in range(M) if r not in S],
                         list(Q) + [c for c in range(K) if c not in Q], 3, 3)
              for S in itertools.combinations(range(M), 3) for Q in itertools.combinations(range(K), 3))
    assert got <= opt


def _planted(rng, M, K, levels, noise):
    """|W| = 1 inside 2**levels hidden diagonal blocks, plus uniform noise in [0, noise) everywhere (it breaks
    the ties of an exactly balanced random start).  Returns (noisy, clean), hidden by the same permutations."""
    rr, cc = O.feedback_block_ranges(M, levels), O.feedback_block_ranges(K, levels)
    clean_p = np.zeros((M, K))
    for (rb, re), (cb, ce) in zip(rr, cc):
        clean_p[rb:re, cb:ce] = 1.0
    noisy_p = clean_p + noise * rng.random((M, K))
    hide_r, hide_c = rng.permutation(M), rng.permutation(K)
    noisy, clean = np.empty_like(noisy_p), np.empty_like(clean_p)
    noisy[np.ix_(hide_r, hide_c)] = noisy_p            # W[hide_r[r]][hide_c[c]] = W'[r][c]
    clean[np.ix_(hide_r, hide_c)] = clean_p
    return noisy.astype(np.float32), clean


@pytest.mark.parametrize("levels,M,K", [(1, 16, 24), (2, 32, 32), (3, 64, 48)])
def test_planted_block_structure_is_recovered_exactly(levels, M, K):
    rng = np.random.default_rng(7 + levels)
    W, clean = _planted(rng, M, K, levels, noise=0.05)
    prow, pcol = O.feedback_search(W, levels, rng.permutation(M), rng.permutation(K))
    # every planted one lands inside the diagonal blocks: nothing of the structure is deleted
    assert O.feedback_captured_mass(clean, prow, pcol, levels) == clean.sum()
    left = clean[np.ix_(prow, pcol)].copy()
    for (rb, re), (cb, ce) in zip(O.feedback_block_ranges(M, levels), O.feedback_block_ranges(K, levels)):
        left[rb:re, cb:ce] = 0
    assert not left.any()


def test_search_output_feeds_the_layer_oracle():
    # W' = W[prow][:, pcol] with a block-diagonal tile mask is what pivot_fc_plan takes: the layer oracle
    # applied to it equals the dense product with the off-diagonal blocks deleted.
    rng = np.random.default_rng(3)
    M = K = 16
    W = rng.standard_normal((M, K))
    prow, pcol = O.feedback_search(np.abs(W), 2, rng.permutation(M), rng.permutation(K))
    Wp = W[np.ix_(prow, pcol)]
    tile_mask = np.eye(4, dtype=np.uint8)
    x = rng.standard_normal((1, K))
    y = O.oracle_fc(Wp, tile_mask, prow, pcol, None, x, 4, 4, O.ACT_NONE)
    keep = np.zeros((M, K), dtype=bool)
    for b in range(4):
        keep[np.ix_(prow[4 * b:4 * b + 4], pcol[4 * b:4 * b + 4])] = True
    assert np.allclose(y, (np.where(keep, W, 0.0) @ x.T).T, rtol=0, atol=1e-12)


# ---- the host library against the oracle ---------------------------------------

@pytest.mark.parametrize("M,K,levels,seed", [(16, 16, 1, 0), (64, 48, 3, 1), (37, 53, 2, 2), (128, 256, 3, 3),
                                             (5, 3, 4, 4), (1, 1, 2, 5)])
def test_library_search_equals_oracle_index_for_index(M, K, levels, seed):
    rng = np.random.default_rng(seed)
    A = np.abs(rng.standard_normal((M, K))).astype(np.float32)
    p0, c0 = rng.permutation(M).astype(np.int32), rng.permutation(K).astype(np.int32)
    prow, pcol, mass = B.pivot_feedback_search(A, levels, p0, c0)
    orow, ocol = O.feedback_search(A, levels, p0, c0)
    assert np.array_equal(prow, orow) and np.array_equal(pcol, ocol)
    assert mass == pytest.approx(O.feedback_captured_mass(A, orow, ocol, levels), rel=1e-12)


def test_library_search_on_planted_structure_and_ties():
    rng = np.random.default_rng(11)
    W, clean = _planted(rng, 64, 64, 3, noise=0.05)
    p0, c0 = rng.permutation(64).astype(np.int32), rng.permutation(64).astype(np.int32)
    prow, pcol, mass = B.pivot_feedback_search(W, 3, p0, c0)
    orow, ocol = O.feedback_search(W, 3, p0, c0)
    assert np.array_equal(prow, orow) and np.array_equal(pcol, ocol)
    assert O.feedback_captured_mass(clean, prow, pcol, 3) == clean.sum()   # all planted ones are kept
    assert mass == pytest.approx(O.feedback_captured_mass(W, prow, pcol, 3), rel=1e-12)
    # all-equal magnitudes: every gain ties, nothing may move
    ones = np.ones((8, 8), dtype=np.float32)
    prow, pcol, _ = B.pivot_feedback_search(ones, 2, p0[:8].argsort().argsort().astype(np.int32),
                                            c0[:8].argsort().argsort().astype(np.int32))
    assert np.array_equal(prow, p0[:8].argsort().argsort()) and np.array_equal(pcol, c0[:8].argsort().argsort())


def test_library_search_error_paths():
    A = np.ones((4, 4), dtype=np.float32)
    ident = np.arange(4, dtype=np.int32)
    bad = np.array([0, 1, 1, 3], dtype=np.int32)
    with pytest.raises(B.PivotError) as e:
        B.pivot_feedback_search(A, 1, bad, ident)
    assert e.value.code == B.PIVOT_E_NOT_PERMUTATION
    with pytest.raises(B.PivotError) as e:
        B.pivot_feedback_search(A, -1, ident, ident)
    assert e.value.code == B.PIVOT_E_SHAPE
    with pytest.raises(B.PivotError) as e:
        B.pivot_feedback_search(A, 1, ident, ident, max_iter=0)
    assert e.value.code == B.PIVOT_E_SHAPE
