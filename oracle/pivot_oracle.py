"""CPU oracle for pruned fully-connected inference in PBP form.

TEST INFRASTRUCTURE ONLY.  Nothing on the product path may import this
package; it is used by the tests, by the smoke check and by the benchmark's
CPU-baseline leg.  It shares no code with the HIP path.

What it computes follows the paper directly.  A pruned FC layer is kept as
``M_sparse = P_row M_block P_col`` (Eq. 1) and applied as
``a_out = P_row (M_block (P_col a_in))`` (Eq. 2).  The method is an exact
re-association of a sparse matrix-vector product, not an approximation, so
the oracle is the plain definition: build the dense masked matrix in natural
coordinates and multiply in float64.

Index-array convention (Section 4.1.4): the index array of "cab" relative to
"abc" is [2,0,1], i.e. an index array ``p`` is a gather, ``out[i] = in[p[i]]``.
Listing 1 gathers the input through ``P_col`` and scatters the output through
``P_row``; therefore, with W' the block-space (pivoted) matrix,

    W'[r][c] = W[prow[r]][pcol[c]],      y[prow[r]] = v[r].

Parity status of every function here: pinned by tests/test_oracle_*.py
(exact rational brute force through explicit permutation matrices, the
paper's printed index-array example, reduction to a library matvec, closed
forms), except the free-running 256-step LSTM trajectory, which is
"parity unpinned" beyond the per-step check.  The feed-back permutation
search at the end of the file is a heuristic the paper only outlines; its
pins (tests/test_feedback_search.py) are brute force over all splits of tiny
matrices, exact recovery of a planted block structure and the paper's printed
fill-in factors.
"""
from __future__ import annotations

import numpy as np

ACT_NONE = 0
ACT_RELU = 1


# ----------------------------------------------------------------------------
# permutations as index arrays (Section 4.1.4, Observations 1 and 2)
# ----------------------------------------------------------------------------

def index_array_of(target, source):
    """Index array of ``target`` relative to ``source``: target[i] ==
    source[idx[i]].  Elements must be distinct."""
    pos = {}
    for j, s in enumerate(source):
        if s in pos:
            raise ValueError("source elements must be distinct")
        pos[s] = j
    return np.array([pos[t] for t in target], dtype=np.int64)


def is_permutation(p, n=None):
    p = np.asarray(p)
    n = p.shape[0] if n is None else n
    if p.ndim != 1 or p.shape[0] != n:
        return False
    if n == 0:
        return True
    if p.min() < 0 or p.max() >= n:
        return False
    return bool(np.array_equal(np.sort(p), np.arange(n)))


def invert_permutation(p):
    """inv[p[i]] = i."""
    p = np.asarray(p)
    if not is_permutation(p):
        raise ValueError("not a permutation")
    inv = np.empty(p.shape[0], dtype=np.int32)
    inv[p] = np.arange(p.shape[0], dtype=np.int32)
    return inv


def gather_matrix(p):
    """Dense 0/1 matrix G with (G v)[i] = v[p[i]]."""
    p = np.asarray(p)
    n = p.shape[0]
    G = np.zeros((n, n), dtype=np.float64)
    G[np.arange(n), p] = 1.0
    return G


def compose_boundary(prow_a, pcol_b):
    """Boundary index array between producer layer A and consumer layer B
    (Section 4.2.1).  Layer A leaves v_A in block order with
    h[prow_a[r]] = v_A[r]; layer B wants xg[c] = h[pcol_b[c]].  Hence
    xg[c] = v_A[q[c]] with q[c] = invprow_a[pcol_b[c]]."""
    inv = invert_permutation(prow_a)
    return inv[np.asarray(pcol_b)].astype(np.int32)


# ----------------------------------------------------------------------------
# the layer in natural coordinates (Eq. 1)
# ----------------------------------------------------------------------------

def expand_tile_mask(tile_mask, bh, bw, M, K):
    """Element mask in block space: keep'[r][c] = tile_mask[r//bh][c//bw]."""
    tm = np.asarray(tile_mask).astype(bool)
    return np.repeat(np.repeat(tm, bh, axis=0), bw, axis=1)[:M, :K]


def dense_masked_natural(Wp, tile_mask, prow, pcol, bh, bw):
    """M_sparse of Eq. 1 as a dense float64 matrix in natural coordinates:
    Wd[prow[r]][pcol[c]] = W'[r][c] where the tile of (r,c) is kept, else 0."""
    Wp = np.asarray(Wp)
    M, K = Wp.shape
    prow = np.asarray(prow)
    pcol = np.asarray(pcol)
    if not (is_permutation(prow, M) and is_permutation(pcol, K)):
        raise ValueError("prow/pcol must be permutations of range(M)/range(K)")
    keep = expand_tile_mask(tile_mask, bh, bw, M, K)
    Wm = np.where(keep, Wp.astype(np.float64), 0.0)
    Wd = np.empty((M, K), dtype=np.float64)
    Wd[np.ix_(prow, pcol)] = Wm
    return Wd


def unpivot_weights(Wp, prow, pcol):
    """Natural-coordinate weight matrix W with W[prow[r]][pcol[c]] = W'[r][c],
    in the storage dtype of W' (no masking)."""
    Wp = np.asarray(Wp)
    W = np.empty_like(Wp)
    W[np.ix_(np.asarray(prow), np.asarray(pcol))] = Wp
    return W


def apply_act(z, act):
    if act == ACT_NONE:
        return z
    if act == ACT_RELU:
        return np.maximum(z, 0.0)
    raise ValueError("unknown activation %r" % (act,))


def fc_dense(Wd, x, bias, act):
    """y[n][i] = act(sum_j Wd[i][j] x[n][j] + b[i]) in float64."""
    Wd = np.asarray(Wd, dtype=np.float64)
    x = np.asarray(x).astype(np.float64)
    if x.ndim == 1:
        x = x[None, :]
    b = np.zeros(Wd.shape[0]) if bias is None else np.asarray(bias).astype(np.float64)
    z = x @ Wd.T + b[None, :]
    return apply_act(z, act)


def error_scale(Wd, x, bias):
    """D[n][i] = sum_j |Wd[i][j]||x[n][j]| + |b[i]|: the magnitude against
    which the HIP path's error is normalised."""
    Wd = np.asarray(Wd, dtype=np.float64)
    x = np.abs(np.asarray(x).astype(np.float64))
    if x.ndim == 1:
        x = x[None, :]
    b = np.zeros(Wd.shape[0]) if bias is None else np.abs(np.asarray(bias).astype(np.float64))
    return x @ np.abs(Wd).T + b[None, :]


def oracle_fc(Wp, tile_mask, prow, pcol, bias, x, bh, bw, act, return_scale=False):
    """One pruned FC layer applied to a batch x[n][K]; returns y[n][M] float64
    in natural coordinates (and the error scale D if asked)."""
    Wd = dense_masked_natural(Wp, tile_mask, prow, pcol, bh, bw)
    y = fc_dense(Wd, x, bias, act)
    if return_scale:
        return y, error_scale(Wd, x, bias)
    return y


def max_scaled_error(y_test, y_ref, D):
    """max |y_test - y_ref| / D; entries with D == 0 have to match exactly."""
    y_test = np.asarray(y_test, dtype=np.float64)
    y_ref = np.asarray(y_ref, dtype=np.float64)
    diff = np.abs(y_test - y_ref)
    zero = D == 0
    if np.any(diff[zero] != 0):
        return np.inf
    if np.all(zero):
        return 0.0
    return float(np.max(diff[~zero] / D[~zero]))


# ----------------------------------------------------------------------------
# chains of layers (Section 4.2): natural coordinates only, no permutation
# logic in the forward path
# ----------------------------------------------------------------------------

def oracle_mlp(layers, x, boundary_dtype=None, return_all=False):
    """layers: list of dicts with keys Wp, tile_mask, prow, pcol, bias, bh, bw,
    act.  Each layer is applied in natural coordinates.  If ``boundary_dtype``
    is given the activation handed to the next layer is rounded to it once
    (the point where the HIP path stores a half-precision intermediate)."""
    h = np.asarray(x)
    outs, scales, chain = [], [], []
    S = None
    for li, L in enumerate(layers):
        Wd = dense_masked_natural(L["Wp"], L["tile_mask"], L["prow"], L["pcol"], L["bh"], L["bw"])
        y = fc_dense(Wd, h, L["bias"], L["act"])
        D = error_scale(Wd, h, L["bias"])
        # first-order bound on how an error of relative size eps in every layer
        # reaches this layer's output: eps * S with S_1 = D_1, S_l = |W_l| S_{l-1} + D_l
        S = D if S is None else S @ np.abs(Wd).T + D
        outs.append(y)
        scales.append(D)
        chain.append(S)
        h = y
        if boundary_dtype is not None and li + 1 < len(layers):
            h = y.astype(boundary_dtype)
    if return_all:
        return outs, scales, chain
    return outs[-1]


# ----------------------------------------------------------------------------
# LSTM cell around a pruned gate matrix (textbook cell; the paper only names
# recurrent nets as users of FC layers, Section 1)
# ----------------------------------------------------------------------------

def _sigmoid(z):
    return 1.0 / (1.0 + np.exp(-z))


def lstm_cell(z, c_prev, H):
    """Gate pre-activations z[n][4H] in order (i,f,g,o) -> (h, c) float64."""
    i = _sigmoid(z[:, 0 * H:1 * H])
    f = _sigmoid(z[:, 1 * H:2 * H])
    g = np.tanh(z[:, 2 * H:3 * H])
    o = _sigmoid(z[:, 3 * H:4 * H])
    c = f * c_prev + i * g
    h = o * np.tanh(c)
    return h, c


def oracle_lstm_step(Wd, bias, h_in, x_t, c_prev, H):
    """One step: z = Wd [h_in; x_t] + b, then the cell.  h_in and x_t are the
    storage-precision values the step consumes.  Returns (z, h, c, D)."""
    inp = np.concatenate([np.asarray(h_in).astype(np.float64),
                          np.asarray(x_t).astype(np.float64)], axis=1)
    z = fc_dense(Wd, inp, bias, ACT_NONE)
    D = error_scale(Wd, inp, bias)
    h, c = lstm_cell(z, np.asarray(c_prev, dtype=np.float64), H)
    return z, h, c, D


def oracle_lstm(Wd, bias, xs, h0, c0, H, state_dtype=np.float16, record=()):
    """Free-running recurrence.  The hidden state fed back into the gate
    matrix is rounded to ``state_dtype`` once per step (the HIP path stores it
    in that precision for the next step's input); the cell state stays
    float64.  Returns (h, c) after the last step and a dict of recorded
    (h_fed, c_prev, z, h, c) for the steps listed in ``record``."""
    h = np.asarray(h0, dtype=np.float64)
    c = np.asarray(c0, dtype=np.float64)
    rec = {}
    for t in range(xs.shape[0]):
        h_fed = h.astype(state_dtype)
        z, h_new, c_new, D = oracle_lstm_step(Wd, bias, h_fed, xs[t], c, H)
        if t in record:
            rec[t] = dict(h_fed=h_fed, c_prev=c.copy(), z=z, h=h_new, c=c_new, D=D)
        h, c = h_new, c_new
    return h, c, rec


# ----------------------------------------------------------------------------
# the canonical plan: an independent builder of the arrays the host-side
# "compiler" step has to produce (static, data independent: Eq. 1 discussion;
# layouts: Section 4.1.1; shared rows need a reduction: Section 4.1.5)
# ----------------------------------------------------------------------------

LAYOUT_BRC = 0   # block, row, column: row-major inside a tile
LAYOUT_BCR = 1   # block, column, row: column-major inside a tile
LAYOUT_CBR = 2   # column, block, row: one column position of all tiles together


def value_offset(layout, t, r, c, T, bh, bw):
    """Offset of element (r,c) of tile t; the rightmost named axis moves
    fastest (Section 4.1.1)."""
    if layout == LAYOUT_BRC:
        return (t * bh + r) * bw + c
    if layout == LAYOUT_BCR:
        return (t * bw + c) * bh + r
    if layout == LAYOUT_CBR:
        return (c * T + t) * bh + r
    raise ValueError(layout)


def build_schedule(row_ptr, chunk_tiles):
    """Cut every block row's tile list into consecutive chunks of at most
    ``chunk_tiles`` tiles (an empty block row gives one empty chunk, so that
    its bias still reaches the output).  ``slot`` numbers the chunks in
    (block row, tile_begin) order; ``part_base[i]`` is the first slot of block
    row i.  The chunks are then put in launch order: stable sort by
    descending length."""
    nbr = len(row_ptr) - 1
    chunks = []
    part_base = [0]
    for i in range(nbr):
        b, e = int(row_ptr[i]), int(row_ptr[i + 1])
        if b == e:
            chunks.append((i, b, e, len(chunks)))
        s = b
        while s < e:
            n = min(chunk_tiles, e - s)
            chunks.append((i, s, s + n, len(chunks)))
            s += n
        part_base.append(len(chunks))
    order = sorted(range(len(chunks)), key=lambda j: -(chunks[j][2] - chunks[j][1]))
    chunks = np.array([chunks[j] for j in order], dtype=np.int32).reshape(-1, 4)
    return chunks, np.array(part_base, dtype=np.int32)


def oracle_plan(W, w_space_pivoted, tile_mask, prow, pcol, bias, M, K, bh, bw,
                layout, chunk_tiles):
    """Canonical plan arrays.  ``W`` is M x K in storage dtype, either already
    pivoted (block space) or in natural coordinates."""
    W = np.asarray(W)
    prow = np.asarray(prow, dtype=np.int64)
    pcol = np.asarray(pcol, dtype=np.int64)
    nbr, nbc = -(-M // bh), -(-K // bw)
    Mp, Kp = nbr * bh, nbc * bw
    tm = np.asarray(tile_mask).reshape(nbr, nbc) != 0
    if w_space_pivoted:
        Wp = W
    else:
        Wp = W[np.ix_(prow, pcol)]
    Wpad = np.zeros((Mp, Kp), dtype=W.dtype)
    Wpad[:M, :K] = Wp
    row_ptr = np.zeros(nbr + 1, dtype=np.int32)
    col_idx = []
    for i in range(nbr):
        cols = np.nonzero(tm[i])[0]
        col_idx.extend(cols.tolist())
        row_ptr[i + 1] = len(col_idx)
    T = len(col_idx)
    col_idx = np.array(col_idx, dtype=np.int32)
    vals = np.zeros(T * bh * bw, dtype=W.dtype)
    t = 0
    for i in range(nbr):
        for j in col_idx[row_ptr[i]:row_ptr[i + 1]]:
            tile = Wpad[i * bh:(i + 1) * bh, j * bw:(j + 1) * bw]
            rr, cc = np.meshgrid(np.arange(bh), np.arange(bw), indexing="ij")
            vals[value_offset(layout, t, rr, cc, T, bh, bw)] = tile
            t += 1
    bias_p = np.zeros(Mp, dtype=np.float32)
    if bias is not None:
        bias_p[:M] = np.asarray(bias, dtype=np.float32)[prow]
    prow_pad = np.full(Mp, -1, dtype=np.int32)
    prow_pad[:M] = prow
    pcol_pad = np.full(Kp, -1, dtype=np.int32)
    pcol_pad[:K] = pcol
    # the column gather composed with the tile list: index into x of column c of tile t
    xidx = pcol_pad.reshape(nbc, bw)[col_idx].reshape(-1) if T else np.zeros(0, dtype=np.int32)
    chunks, part_base = build_schedule(row_ptr, chunk_tiles)
    return dict(xidx=np.ascontiguousarray(xidx, dtype=np.int32), row_ptr=row_ptr, col_idx=col_idx, vals=vals, bias_p=bias_p,
                invprow=invert_permutation(prow), invpcol=invert_permutation(pcol),
                prow_pad=prow_pad, pcol_pad=pcol_pad, chunks=chunks,
                part_base=part_base, T=T, M_pad=Mp, K_pad=Kp)


def unpack_plan_to_dense(plan, M, K, bh, bw, layout):
    """Inverse of the packing: dense natural-coordinate matrix rebuilt from
    the plan arrays alone (storage dtype)."""
    T = plan["T"]
    vals = plan["vals"]
    Wd = np.zeros((M, K), dtype=vals.dtype)
    prow_pad, pcol_pad = plan["prow_pad"], plan["pcol_pad"]
    nbr = len(plan["row_ptr"]) - 1
    for i in range(nbr):
        for t in range(plan["row_ptr"][i], plan["row_ptr"][i + 1]):
            j = plan["col_idx"][t]
            for r in range(bh):
                gr = prow_pad[i * bh + r]
                if gr < 0:
                    continue
                for c in range(bw):
                    gc = pcol_pad[j * bw + c]
                    if gc < 0:
                        continue
                    Wd[gr, gc] = vals[value_offset(layout, t, r, c, T, bh, bw)]
    return Wd


def oracle_mlp_plan(prows, pcols, Mpads):
    """Boundary arrays of a chain: for l = 0..L-2, q[l][c] = invprow_l[pcol_{l+1}[c]]
    (consumer-side gather form, Section 4.2.1) and its producer-side scatter
    form dst[l][r] = invpcol_{l+1}[prow_l[r]] (padding rows -> -1)."""
    qs, dsts = [], []
    for l in range(len(prows) - 1):
        q = compose_boundary(prows[l], pcols[l + 1])
        inv_next = invert_permutation(pcols[l + 1])
        dst = np.full(Mpads[l], -1, dtype=np.int32)
        dst[:len(prows[l])] = inv_next[np.asarray(prows[l])]
        qs.append(q)
        dsts.append(dst)
    return qs, dsts


# ----------------------------------------------------------------------------
# feed-back PBP pruning (Section 3.2): the producer of prow / pcol.
#
# The paper gives the objective and the search style, not a procedure: from the
# magnitudes of a trained dense layer, starting from random permutations, a
# greedy search picks P_row / P_col that maximise the magnitude inside the
# upper-left and lower-right sub-blocks; the off-diagonal sub-blocks are
# deleted (half the coefficients of the block); the same is repeated on every
# sub-block (three times for 12.5 % fill-in, twice for 25 %).
#
# Reading used here (a heuristic, so the steps are written out in order):
# a block is a list of rows R and a list of columns C in their current order,
# with halves R1|R2 and C1|C2 of sizes floor(n/2) and the rest.  One greedy
# half-step re-chooses R1 as the |R1| rows with the largest
# gain(r) = mass(r, C1) - mass(r, C2) (ties: earlier in the list first; both
# halves keep the list's relative order), which is the best R1 for the given
# column split; the next half-step does the same for the columns.  Half-steps
# alternate until neither changes anything (or max_iter rounds).  Sums are
# float64, added in list order.
# ----------------------------------------------------------------------------

def _best_half(gain, n1):
    """Positions chosen for the first half: the n1 largest gains, earlier
    position first among equals."""
    order = sorted(range(len(gain)), key=lambda i: (-gain[i], i))
    return set(order[:n1])


def _seq_sum(A):
    """Row sums added strictly left to right in float64."""
    if A.shape[1] == 0:
        return np.zeros(A.shape[0])
    return np.cumsum(A.astype(np.float64), axis=1)[:, -1]


def feedback_half_step(absW, own, other, n1, o1, rows_side):
    """One greedy half-step.  Returns the re-ordered list of ``own``."""
    own = list(own)
    other = list(other)
    A = absW[np.ix_(own, other)] if rows_side else absW[np.ix_(other, own)].T
    gain = _seq_sum(A[:, :o1]) - _seq_sum(A[:, o1:])
    first = _best_half(gain.tolist(), n1)
    return [own[i] for i in range(len(own)) if i in first] + [own[i] for i in range(len(own)) if i not in first]


def feedback_search(absW, levels, prow0, pcol0, max_iter=50):
    """Recursive greedy bisection.  Returns (prow, pcol): W'[r][c] =
    W[prow[r]][pcol[c]] keeps its mass in 2**levels diagonal blocks."""
    absW = np.asarray(absW)

    def bisect(R, C, lv):
        if lv == 0 or len(R) < 2 or len(C) < 2:
            return R, C
        r1, c1 = len(R) // 2, len(C) // 2
        for _ in range(max_iter):
            R2 = feedback_half_step(absW, R, C, r1, c1, True)
            C2 = feedback_half_step(absW, C, R2, c1, r1, False)
            moved = (R2 != R) or (C2 != C)
            R, C = R2, C2
            if not moved:
                break
        Ra, Ca = bisect(R[:r1], C[:c1], lv - 1)
        Rb, Cb = bisect(R[r1:], C[c1:], lv - 1)
        return Ra + Rb, Ca + Cb

    R, C = bisect([int(v) for v in prow0], [int(v) for v in pcol0], levels)
    return np.array(R, dtype=np.int32), np.array(C, dtype=np.int32)


def feedback_block_ranges(n, levels):
    """[begin, end) of the 2**levels diagonal blocks along one axis of length n
    (each range halved floor-first; a range shorter than 2 is not split)."""
    ranges = [(0, n)]
    for _ in range(levels):
        nxt = []
        for b, e in ranges:
            if e - b < 2:
                nxt.append((b, e))
            else:
                m = b + (e - b) // 2
                nxt += [(b, m), (m, e)]
        ranges = nxt
    return ranges


def feedback_captured_mass(absW, prow, pcol, levels):
    """Magnitude kept after deleting the off-diagonal sub-blocks at every level."""
    M, K = absW.shape
    Wp = np.asarray(absW, dtype=np.float64)[np.ix_(prow, pcol)]

    # a block that cannot be halved on one axis is not halved on the other either
    def rec(rb, re, cb, ce, lv):
        if lv == 0 or re - rb < 2 or ce - cb < 2:
            return float(Wp[rb:re, cb:ce].sum())
        rm, cm = rb + (re - rb) // 2, cb + (ce - cb) // 2
        return rec(rb, rm, cb, cm, lv - 1) + rec(rm, re, cm, ce, lv - 1)
    return rec(0, M, 0, K, levels)
