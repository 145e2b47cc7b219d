"""CPU oracle for the V:N:M sparse linear path (TEST INFRASTRUCTURE ONLY).

This module is the slow, plain definition the GPU library is checked against.
It is imported only by the tests, by the smoke check and by the benchmark's
``cpu_baseline`` leg.  It shares no code with the HIP path and must never be
imported by the product package.

Everything here follows the paper's own wording of the method:

* Section 3 ("Pruning of V:N:M sparsity"): the three pruning steps
  (importance score, column pruning per V x M block by column L1 norm,
  2:4 inside the four surviving columns of every row).
* Section 3, Eq. 1: the RIA importance score (importance_ria) as an
  alternative to |w|; prune() and compress() take any score matrix.
* Section 4.1 (Eq. 4-5, Appendix B): mask diversity and the two-phase (V, M)
  sifting (mask_diversity_log, select_vm).
* Section 4.2, Eq. 6: the layer evaluated on a channel-permuted weight
  (permute_weight, linear_fused_ref, fold_permutations); Eqs. 7-9: the search
  for the permutations (permutation_search and its parts).
* Section 4.3, Eq. 10: merging the low-rank LoRA matrices into the dense weight
  and refreshing the mask from the merged weight (lora_merge, refresh_mask).
* Section 3 ("Acceleration of V:N:M sparsity"): zero padding so that the
  input dimension is a multiple of M and the output dimension a multiple of V.
* Appendix A: the compressed triple -- the compact kept values (A_n), the four
  kept column indices of every block (A_i1), and for every kept value its
  position among the four surviving columns (A_i2).

Readings taken where the paper is silent (each is listed in the design notes):
ties are broken towards the lower index in both selection steps; the column
L1 norm is the exact sum; pruned entries of the masked matrix are +0.0; a kept
weight that happens to be zero still counts as kept (mask = 1 by position).

All floating point is fp64.  |fp16| values are multiples of 2**-24 below 2**16,
so a sum of V <= 8192 of them is exactly representable in fp64 whatever the
summation order; the column norms below are therefore exact.

Pins (tests/test_oracle_pins.py): pattern invariants, brute-force enumeration
on tiny blocks, optimality of the kept mass, the M = 4 (plain 2:4) and V = 1
(2-of-M per row) special cases, a hand-worked example, round trips, exact
integer column sums, for the scored path its reduction to ABS when the score
is |w|, brute force with random scores, and a hand-worked RIA example with
closed forms and invariances, and for the matmul a triple-loop dot product, one-hot
inputs and exactly representable small-integer products.  No function in this
file is "parity unpinned"; the paper itself prints no numeric example of a
pruned block (its figures are not part of the text), so the worked example is
derived by hand from the Section 3 definition.
"""

from __future__ import annotations

import numpy as np

N_KEPT = 2          # N is fixed to 2 (Section 4.1: N is identically 2)
COLS_KEPT = 4       # every block keeps exactly four columns (Section 3, step 3)


def padded_dims(out: int, inn: int, V: int, M: int):
    """Padded shape, block counts (Section 3, weight padding).

    Returns (out_pad, in_pad, R, B): rows padded to a multiple of V, columns to
    a multiple of M, R = row blocks, B = column blocks.
    """
    if V < 1 or M < COLS_KEPT or out < 1 or inn < 1:
        raise ValueError("need V >= 1, M >= 4, out >= 1, in >= 1")
    R = -(-out // V)
    B = -(-inn // M)
    return R * V, B * M, R, B


def _as_fp16_matrix(W) -> np.ndarray:
    W = np.asarray(W)
    if W.dtype != np.float16 or W.ndim != 2:
        raise TypeError("expected a 2-D float16 array")
    return W


def pad_weight(W: np.ndarray, V: int, M: int) -> np.ndarray:
    """Zero-extend W [out x in] to [out_pad x in_pad] (Section 3, padding)."""
    W = _as_fp16_matrix(W)
    out, inn = W.shape
    out_pad, in_pad, _, _ = padded_dims(out, inn, V, M)
    Wp = np.zeros((out_pad, in_pad), dtype=np.float16)
    Wp[:out, :inn] = W
    return Wp


def importance_abs(Wp: np.ndarray) -> np.ndarray:
    """Step 1 of Section 3 with the ABS criterion: score = |w|, in fp64."""
    return np.abs(Wp.astype(np.float64))


def importance_ria(W: np.ndarray, act: np.ndarray) -> np.ndarray:
    """Step 1 of Section 3 with the RIA criterion (Eq. 1), as fp32 scores [out x in]:

        RIA[i, j] = (|W[i,j]| / sum_i' |W[i',j]|  +  |W[i,j]| / sum_j' |W[i,j']|) * act[j]

    act[j] = (L2 norm of the activations of input channel j) ** a is an input (fp32 [in]); the
    equation's activation factor is taken per input channel j, as in the criterion it cites.
    The two sums are exact (integers, in units of 2**-24); every later operation is one IEEE
    fp64 operation -- convert, divide, divide, add, multiply -- followed by one rounding to
    fp32, so the scores are reproducible bit for bit.  A term whose sum is zero is zero.
    """
    W = _as_fp16_matrix(W)
    act = np.asarray(act)
    if act.dtype != np.float32 or act.shape != (W.shape[1],):
        raise TypeError("act: float32 vector of length in")
    units = np.rint(np.abs(W.astype(np.float64)) * 2.0 ** 24).astype(np.int64)     # exact
    col = units.sum(axis=0, dtype=np.int64)
    row = units.sum(axis=1, dtype=np.int64)
    a = units.astype(np.float64)
    with np.errstate(divide="ignore", invalid="ignore"):
        q_col = np.where(col[None, :] > 0, a / col.astype(np.float64)[None, :], 0.0)
        q_row = np.where(row[:, None] > 0, a / row.astype(np.float64)[:, None], 0.0)
    return ((q_col + q_row) * act.astype(np.float64)[None, :]).astype(np.float32)


def column_l1(S: np.ndarray, V: int, M: int) -> np.ndarray:
    """Step 2 of Section 3: L1 norm of every column of every V x M block.

    S is the padded score matrix; returns L [R, B, M] with
    L[r, b, c] = sum_v S[r*V + v, b*M + c].
    """
    out_pad, in_pad = S.shape
    R, B = out_pad // V, in_pad // M
    return S.reshape(R, V, B, M).sum(axis=1)


def column_l1_in_row_order(S: np.ndarray, V: int, M: int) -> np.ndarray:
    """Column L1 norms for a general score matrix: the same sums as column_l1, added in fp64
    one row after the other (v = 0, 1, ..., V-1).  Sums of arbitrary fp32 scores can depend on
    the order of addition in their last bit; fixing the order makes the selection unique."""
    out_pad, in_pad = S.shape
    R, B = out_pad // V, in_pad // M
    blk = S.reshape(R, V, B, M)
    L = np.zeros((R, B, M), dtype=np.float64)
    for v in range(V):
        L = L + blk[:, v, :, :]
    return L


def select_columns(L: np.ndarray) -> np.ndarray:
    """Step 2 of Section 3: keep the four columns of largest L1 norm.

    Sort key is (norm descending, index ascending); the survivors are stored in
    ascending index order (Appendix A: relative positions are preserved).
    Returns uint8 [R, B, 4].
    """
    order = np.argsort(-L, axis=-1, kind="stable")[..., :COLS_KEPT]
    return np.sort(order, axis=-1).astype(np.uint8)


def select_2_of_4(S: np.ndarray, colidx: np.ndarray, V: int, M: int) -> np.ndarray:
    """Step 3 of Section 3: per row, keep the two largest scores among the
    four surviving columns of the block; ties go to the lower position.

    Returns pos uint8 [out_pad, B, 2] with pos[..., 0] < pos[..., 1], each the
    position (0..3) of a kept value among the block's four surviving columns.
    """
    out_pad, in_pad = S.shape
    R, B = out_pad // V, in_pad // M
    blk = S.reshape(R, V, B, M)
    idx = np.broadcast_to(colidx[:, None, :, :].astype(np.intp), (R, V, B, COLS_KEPT))
    g = np.take_along_axis(blk, idx, axis=3)                     # [R, V, B, 4]
    rank = np.argsort(-g, axis=-1, kind="stable")[..., :N_KEPT]
    pos = np.sort(rank, axis=-1).astype(np.uint8)
    return pos.reshape(out_pad, B, N_KEPT)


def prune(W: np.ndarray, V: int, M: int, score: np.ndarray | None = None):
    """The pruning operator S_{V:N:M} of Section 3 with N = 2.

    W: fp16 [out x in].  score: optional [out x in] importance scores, finite
    and non-negative (default: ABS); they are padded with zeros like W, their
    column norms are added in row order (column_l1_in_row_order), and step 3
    compares the scores themselves.  Returns (colidx [R,B,4] u8,
    pos [out_pad,B,2] u8, mask [out x in] u8).
    """
    W = _as_fp16_matrix(W)
    out, inn = W.shape
    out_pad, in_pad, R, B = padded_dims(out, inn, V, M)
    if score is None:
        S = importance_abs(pad_weight(W, V, M))
        L = column_l1(S, V, M)
    else:
        S = np.zeros((out_pad, in_pad), dtype=np.float64)
        S[:out, :inn] = np.asarray(score, dtype=np.float64)
        L = column_l1_in_row_order(S, V, M)
    colidx = select_columns(L)
    pos = select_2_of_4(S, colidx, V, M)
    mask = mask_from_selection(colidx, pos, out, inn, V, M)
    return colidx, pos, mask


def kept_columns(colidx: np.ndarray, pos: np.ndarray, V: int, M: int) -> np.ndarray:
    """Absolute padded column of every kept value: int64 [out_pad, B, 2]."""
    out_pad, B, _ = pos.shape
    R = out_pad // V
    ci = np.repeat(colidx.astype(np.int64), V, axis=0)            # [out_pad, B, 4]
    inblock = np.take_along_axis(ci, pos.astype(np.intp), axis=2)  # [out_pad, B, 2]
    return inblock + (np.arange(B, dtype=np.int64) * M)[None, :, None]


def mask_from_selection(colidx, pos, out: int, inn: int, V: int, M: int) -> np.ndarray:
    """0-1 mask of Section 3 (W' = W (.) mask), reported on [out x in] only."""
    out_pad, in_pad, R, B = padded_dims(out, inn, V, M)
    cols = kept_columns(colidx, pos, V, M)
    mask = np.zeros((out_pad, in_pad), dtype=np.uint8)
    rows = np.arange(out_pad, dtype=np.int64)[:, None, None]
    mask[np.broadcast_to(rows, cols.shape), cols] = 1
    return np.ascontiguousarray(mask[:out, :inn])


def masked_dense(W: np.ndarray, mask: np.ndarray) -> np.ndarray:
    """W' of Section 3: kept entries are bit copies, pruned entries are +0.0."""
    W = _as_fp16_matrix(W)
    return np.where(mask.astype(bool), W, np.float16(0.0)).astype(np.float16)


def compress(W: np.ndarray, V: int, M: int, score: np.ndarray | None = None):
    """Prune and convert to the compressed triple of Appendix A.

    Returns (values, meta, colidx, mask):
      values fp16 [out_pad x 2B]  -- A_n: the two kept values of block b of a
                                     row sit at columns 2b, 2b+1 in ascending
                                     position order;
      meta   u8   [out_pad x ceil(B/2)] -- A_i2: nibble p0 | p1 << 2 per
                                     (row, block); byte j holds block 2j in its
                                     low nibble and block 2j+1 in its high one;
      colidx u8   [R x B x 4]     -- A_i1: in-block indices of the four kept
                                     columns, ascending;
      mask   u8   [out x in].
    """
    W = _as_fp16_matrix(W)
    out, inn = W.shape
    out_pad, in_pad, R, B = padded_dims(out, inn, V, M)
    colidx, pos, mask = prune(W, V, M, score)
    Wp = pad_weight(W, V, M)
    cols = kept_columns(colidx, pos, V, M)
    rows = np.broadcast_to(np.arange(out_pad, dtype=np.int64)[:, None, None], cols.shape)
    values = np.ascontiguousarray(Wp[rows, cols].reshape(out_pad, 2 * B))
    nib = (pos[..., 0] | (pos[..., 1] << 2)).astype(np.uint8)      # [out_pad, B]
    if B % 2:
        nib = np.concatenate([nib, np.zeros((out_pad, 1), np.uint8)], axis=1)
    meta = (nib[:, 0::2] | (nib[:, 1::2] << 4)).astype(np.uint8)
    return values, np.ascontiguousarray(meta), colidx, mask


def unpack_meta(meta: np.ndarray, B: int) -> np.ndarray:
    """Inverse of the nibble packing: pos u8 [out_pad, B, 2]."""
    out_pad = meta.shape[0]
    nib = np.empty((out_pad, 2 * meta.shape[1]), dtype=np.uint8)
    nib[:, 0::2] = meta & 0x0F
    nib[:, 1::2] = meta >> 4
    nib = nib[:, :B]
    return np.stack([nib & 3, (nib >> 2) & 3], axis=-1).astype(np.uint8)


def decompress(values, meta, colidx, out: int, inn: int, V: int, M: int) -> np.ndarray:
    """Scatter the compressed triple back to the dense fp16 W' [out x in]."""
    out_pad, in_pad, R, B = padded_dims(out, inn, V, M)
    pos = unpack_meta(np.asarray(meta), B)
    cols = kept_columns(np.asarray(colidx).reshape(R, B, COLS_KEPT), pos, V, M)
    rows = np.broadcast_to(np.arange(out_pad, dtype=np.int64)[:, None, None], cols.shape)
    Wd = np.zeros((out_pad, in_pad), dtype=np.float16)
    Wd[rows, cols] = np.asarray(values).reshape(out_pad, B, N_KEPT)
    return np.ascontiguousarray(Wd[:out, :inn])


def matmul_ref(X: np.ndarray, Wm: np.ndarray) -> np.ndarray:
    """Y = X . W'^T with fp64 products and fp64 accumulation.

    X fp16 [T x in], Wm fp16 [out x in] (the masked dense matrix).  A product
    of two fp16 numbers is exact in fp64.
    """
    return X.astype(np.float64) @ Wm.astype(np.float64).T


def spmm_ref(X, values, meta, colidx, out: int, inn: int, V: int, M: int) -> np.ndarray:
    """The sparse product written directly on the compressed triple:

      Y[t, o] = sum_b sum_{j in {0,1}} values[o, 2b+j] * X[t, b*M + colidx[o//V, b, pos_j(o, b)]]

    with X taken as 0 at padded columns.  fp64 throughout; returns [T x out].
    """
    X = np.asarray(X)
    T = X.shape[0]
    out_pad, in_pad, R, B = padded_dims(out, inn, V, M)
    pos = unpack_meta(np.asarray(meta), B)
    cols = kept_columns(np.asarray(colidx).reshape(R, B, COLS_KEPT), pos, V, M)
    Xp = np.zeros((T, in_pad), dtype=np.float64)
    Xp[:, :inn] = X.astype(np.float64)
    vals = np.asarray(values).astype(np.float64).reshape(out_pad, 2 * B)
    cols = cols.reshape(out_pad, 2 * B)
    Y = np.empty((T, out), dtype=np.float64)
    for o in range(out):
        Y[:, o] = Xp[:, cols[o]] @ vals[o]
    return Y


def max_normalised_error(Y, Y_ref) -> float:
    """max |Y - Y_ref| / max |Y_ref| -- the acceptance measure for the product."""
    Y_ref = np.asarray(Y_ref, dtype=np.float64)
    denom = float(np.max(np.abs(Y_ref))) if Y_ref.size else 0.0
    if denom == 0.0:
        return float(np.max(np.abs(np.asarray(Y, dtype=np.float64)))) if Y_ref.size else 0.0
    return float(np.max(np.abs(np.asarray(Y, dtype=np.float64) - Y_ref)) / denom)


# ---------------------------------------------------------------- permuted layer (Section 4.2, Eq. 6)

def permute_weight(W: np.ndarray, perm_out: np.ndarray, perm_in: np.ndarray) -> np.ndarray:
    """W_p = P_o W P_i of Eq. 6 in index form: row o of W_p is row perm_out[o] of W, column i of
    W_p is column perm_in[i] of W (P_o[o, perm_out[o]] = 1, P_i[perm_in[i], i] = 1)."""
    return np.ascontiguousarray(np.asarray(W)[np.asarray(perm_out)][:, np.asarray(perm_in)])


def linear_fused_ref(X, Wm_p, bias=None, perm_in=None, perm_out=None) -> np.ndarray:
    """The layer of Eq. 6 evaluated on the permuted (and pruned) weight, fp64:

      Y = P_o^T W_p P_i^T X  (+ bias),   i.e.   Y[t, perm_out[o]] = bias[o] + sum_i W_p[o, i] X[t, perm_in[i]].

    X fp16 [T x in] in the layer's own channel order, Wm_p [out x in] the masked weight in permuted
    order, bias [out] in the row order of Wm_p (the bias travels with its row); a missing
    permutation is the identity.  Returns Y [T x out] in the layer's own channel order.
    """
    X = np.asarray(X).astype(np.float64)
    Xp = X if perm_in is None else X[:, np.asarray(perm_in)]            # P_i^T X
    Yp = Xp @ np.asarray(Wm_p).astype(np.float64).T                     # W_p (P_i^T X)
    if bias is not None:
        Yp = Yp + np.asarray(bias).astype(np.float64)[None, :]
    if perm_out is None:
        return Yp
    Y = np.empty_like(Yp)
    Y[:, np.asarray(perm_out)] = Yp                                     # P_o^T (...)
    return Y


def fold_permutations(perm_out_prev: np.ndarray, perm_in_next: np.ndarray) -> np.ndarray:
    """Input permutation of the next layer when the previous layer leaves its output in permuted
    channel order (its P_o^T is not applied; Section 4.2: the permutations of adjacent layers can
    be merged).  The previous layer then delivers Z[:, o] = Y[:, perm_out_prev[o]], the next layer
    needs Y[:, perm_in_next[i]] = Z[:, inverse(perm_out_prev)[perm_in_next[i]]]."""
    po = np.asarray(perm_out_prev)
    inv = np.empty_like(po)
    inv[po] = np.arange(po.size, dtype=po.dtype)
    return inv[np.asarray(perm_in_next)]


# ---------------------------------------------------------------- permutation search (Section 4.2, Eqs. 7-9)
#
# The paper states the objective (Eq. 7: the retained importance after V:N:M pruning of the permuted
# matrix), the alternation (Eqs. 8-9, two iterations, both permutations start as the identity) and
# that each half-step is "approximately modelled" as a linear sum assignment problem solved by the
# Hungarian algorithm; it does not print the modelling.  The reading taken here: a half-step visits
# the in-block positions ("slots") one after the other; for slot q the channel at position q of
# every full block is lifted out, gain[b, k] is the retained importance of block k if the channel
# lifted from block b is put into its free position, and the assignment of lifted channels to
# blocks that maximises the total gain is applied.  The identity assignment reproduces the current
# state, so no step lowers the objective.  Importance scores are quantised once to non-negative
# integers (rint(score * scale), at most 2**32 - 1): all sums are then exact, whatever their order.
# Channels of a ragged last block stay where they are.

def quantise_scores(S: np.ndarray, scale: float) -> np.ndarray:
    """Integer scores used by the search: rint(S * scale) in fp64, clipped to [0, 2**32 - 1]; int64."""
    q = np.rint(np.asarray(S, dtype=np.float64) * float(scale))
    return np.clip(q, 0, 2.0 ** 32 - 1).astype(np.int64)


def retained_score(Sq: np.ndarray, V: int, M: int) -> int:
    """Objective of Eq. 7 for the matrix as it stands: sum of the scores that V:N:M pruning keeps
    when the scores themselves drive it (Section 3 steps 2-3, ties to the lower index)."""
    Sq = np.asarray(Sq, dtype=np.int64)
    _, _, mask = prune(np.zeros(Sq.shape, dtype=np.float16), V, M, score=Sq.astype(np.float64))
    return int(Sq[mask == 1].sum())


def permutation_objective(Sq, V: int, M: int, perm_out, perm_in) -> int:
    """Eq. 7 for given permutations: retained score of Sq[perm_out][:, perm_in]."""
    return retained_score(np.asarray(Sq)[np.asarray(perm_out)][:, np.asarray(perm_in)], V, M)


def perm_gain_in(Sp: np.ndarray, V: int, M: int, slot: int) -> np.ndarray:
    """Input half-step (Eq. 8), one slot: gain[b, k] = retained score of column block k (all rows)
    with its column at position `slot` replaced by the column at that position of block b.
    Sp is the matrix in its current permuted order; full blocks only.  int64 [B, B]."""
    Bf = Sp.shape[1] // M
    gain = np.zeros((Bf, Bf), dtype=np.int64)
    for k in range(Bf):
        for b in range(Bf):
            blk = Sp[:, k * M:(k + 1) * M].copy()
            blk[:, slot] = Sp[:, b * M + slot]
            gain[b, k] = retained_score(blk, V, M)
    return gain


def perm_gain_out(Sp: np.ndarray, V: int, M: int, slot: int) -> np.ndarray:
    """Output half-step (Eq. 9), one slot: gain[r, k] = retained score of row block k (all columns)
    with its row at position `slot` replaced by the row at that position of row block r.  [R, R]."""
    Rf = Sp.shape[0] // V
    gain = np.zeros((Rf, Rf), dtype=np.int64)
    for k in range(Rf):
        for r in range(Rf):
            blk = Sp[k * V:(k + 1) * V].copy()
            blk[slot] = Sp[r * V + slot]
            gain[r, k] = retained_score(blk, V, M)
    return gain


def lsa_max(gain: np.ndarray):
    """Linear sum assignment maximising sum_i gain[i, assign[i]] (library routine; the gains are
    integers below 2**53, exact in its fp64).  Returns (assign, total)."""
    from scipy.optimize import linear_sum_assignment
    rows, cols = linear_sum_assignment(np.asarray(gain, dtype=np.float64), maximize=True)
    assign = np.empty(len(rows), dtype=np.int64)
    assign[rows] = cols
    return assign, int(np.asarray(gain, dtype=np.int64)[rows, cols].sum())


def permutation_search(S: np.ndarray, V: int, M: int, scale: float, iterations: int = 2):
    """Alternating optimisation of Eqs. 8-9.  Returns (perm_out, perm_in, history): row o / column i
    of the permuted matrix is row perm_out[o] / column perm_in[i] of S; history[0] is the objective
    at the identity, then one entry after every half-step (input first)."""
    Sq = quantise_scores(S, scale)
    out, inn = Sq.shape
    po, pi = np.arange(out), np.arange(inn)
    hist = [permutation_objective(Sq, V, M, po, pi)]
    for _ in range(iterations):
        for slot in range(M):                                   # Eq. 8: P_i for fixed P_o
            assign, _ = lsa_max(perm_gain_in(Sq[po][:, pi], V, M, slot))
            new = pi.copy()
            for b, k in enumerate(assign):
                new[k * M + slot] = pi[b * M + slot]
            pi = new
        hist.append(permutation_objective(Sq, V, M, po, pi))
        for slot in range(V):                                   # Eq. 9: P_o for fixed P_i
            assign, _ = lsa_max(perm_gain_out(Sq[po][:, pi], V, M, slot))
            new = po.copy()
            for r, k in enumerate(assign):
                new[k * V + slot] = po[r * V + slot]
            po = new
        hist.append(permutation_objective(Sq, V, M, po, pi))
    return po, pi, hist


# ---------------------------------------------------------------- LoRA merge and mask refresh (Section 4.3, Eq. 10)

def lora_merge(W: np.ndarray, B: np.ndarray, A: np.ndarray, scale: float) -> np.ndarray:
    """W + scale * B A of Eq. 10 as the fp16 matrix the mask update prunes (Section 4.3, stage 2:
    the low-rank matrices are merged into the dense weight before scores are computed).

    W fp16 [out x in], B fp32 [out x r], A fp32 [r x in].  The paper fixes neither precision nor
    order; so that the refreshed mask is reproducible to the bit the merge is defined in fp32 with
    one rounding per operation and a fixed order:
        acc = 0;  for k = 0..r-1:  acc = acc + (B[o,k] * A[k,i]);  m = (scale * acc) + W[o,i]
    (every product and sum rounded to fp32, no fused multiply-add), then m rounded to fp16.
    """
    W = _as_fp16_matrix(W)
    B = np.asarray(B, dtype=np.float32)
    A = np.asarray(A, dtype=np.float32)
    acc = np.zeros(W.shape, dtype=np.float32)
    for k in range(B.shape[1]):
        acc = acc + B[:, k:k + 1] * A[k:k + 1, :]
    m = np.float32(scale) * acc + W.astype(np.float32)
    return m.astype(np.float16)


def refresh_mask(W, B, A, scale: float, V: int, M: int, act=None):
    """Mask update of the second LoRA stage (Section 4.3; Appendix on the LoRA details): merge, score
    (RIA if activation factors are given, else |w|), prune.  Returns (merged fp16, mask u8) with
    W' = merged (.) mask as in Eq. 10."""
    merged = lora_merge(W, B, A, scale)
    score = None if act is None else importance_ria(merged, act)
    _, _, mask = prune(merged, V, M, score=score)
    return merged, mask


# ---------------------------------------------------------------- V and M selection (Section 4.1)

def mask_diversity_log(V: int, M: int, N: int = N_KEPT) -> float:
    """ln K(V, M) of Eq. 5 / Appendix B: K = [C(M,4) * C(4,N)^V] ** (1 / (V*M)).

    The mask diversity of a layer [m x n] is K ** (m*n); for one network the order of the mask
    diversities of two (V, M) choices is the order of their K."""
    import math
    return (math.log(math.comb(M, COLS_KEPT)) + V * math.log(math.comb(COLS_KEPT, N))) / (V * M)


def select_vm(candidates, threshold: float):
    """Two-phase sifting of Section 4.1.  candidates: sequence of (V, M, speedup).  Returns the
    index of the selected candidate or -1.  Phase 1: among the candidates with speedup >=
    threshold keep, for every V, the smallest M.  Phase 2: largest K(V, M); ties (the paper is
    silent) go to the higher speedup, then the smaller V, then the earlier entry."""
    ok = [i for i, (_, _, s) in enumerate(candidates) if s >= threshold]
    kept = []
    for i in ok:
        V, M, _ = candidates[i]
        if all(not (candidates[j][0] == V and (candidates[j][1] < M or (candidates[j][1] == M and j < i)))
               for j in ok if j != i):
            kept.append(i)
    if not kept:
        return -1
    return min(kept, key=lambda i: (-mask_diversity_log(candidates[i][0], candidates[i][1]),
                                    -candidates[i][2], candidates[i][0], i))
