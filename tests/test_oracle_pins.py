"""Pins for the CPU oracle: everything here checks oracle/vnm_oracle.py against
something other than itself -- the pattern's invariants (Section 3), brute-force
enumeration on tiny blocks, special cases that reduce to textbook routines, a
hand-worked example, exact integer arithmetic and closed forms."""

import itertools
import json
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import vnm_oracle as orc
import synth_inputs as syn

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rand_w(rng, out, inn, kind):
    if kind == "normal":
        return (rng.standard_normal((out, inn)) * 0.02).astype(np.float16)
    if kind == "ints":        # many equal magnitudes and equal column sums
        return rng.integers(-2, 3, size=(out, inn)).astype(np.float16)
    if kind == "binary":
        return rng.integers(0, 2, size=(out, inn)).astype(np.float16)
    raise ValueError(kind)


# ---------------------------------------------------------------- invariants

@pytest.mark.parametrize("out,inn,V,M", [(128, 128, 64, 8), (64, 37, 16, 5), (96, 50, 32, 7),
                                         (40, 64, 16, 4), (33, 29, 16, 6), (256, 130, 128, 16)])
@pytest.mark.parametrize("kind", ["normal", "ints"])
def test_pattern_invariants(out, inn, V, M, kind):
    rng = np.random.default_rng(out * 131 + inn + V + M)
    W = _rand_w(rng, out, inn, kind)
    colidx, pos, mask = orc.prune(W, V, M)
    out_pad, in_pad, R, B = orc.padded_dims(out, inn, V, M)
    assert colidx.shape == (R, B, 4) and pos.shape == (out_pad, B, 2)
    # four distinct ascending in-block columns, two distinct ascending positions
    assert np.all(colidx[..., 1:] > colidx[..., :-1]) and colidx.max() < M
    assert np.all(pos[..., 0] < pos[..., 1]) and pos.max() < 4
    # mask over the padded matrix: every row of every block keeps exactly 2, inside 4 columns
    cols = orc.kept_columns(colidx, pos, V, M)
    full = np.zeros((out_pad, in_pad), np.uint8)
    full[np.arange(out_pad)[:, None, None], cols] = 1
    per_row_block = full.reshape(out_pad, B, M).sum(axis=2)
    assert np.all(per_row_block == 2)
    live_cols = (full.reshape(R, V, B, M).sum(axis=1) > 0).sum(axis=2)
    assert np.all(live_cols <= 4)
    # density closed form: 2 of every M
    assert full.sum() * M == out_pad * in_pad * 2
    assert np.array_equal(full[:out, :inn], mask)


# ------------------------------------------------------- brute force, tiny blocks

def _exact(x):
    return Fraction(float(x))


def _brute_block(Wb):
    """All C(M,4) column subsets and all 6 pairs, in exact rational arithmetic.
    Best = largest kept mass; among equals the lexicographically smallest tuple,
    which is what 'ties to the lower index' yields."""
    V, M = Wb.shape
    A = [[abs(_exact(Wb[v, c])) for c in range(M)] for v in range(V)]
    L = [sum(A[v][c] for v in range(V)) for c in range(M)]
    best = max(itertools.combinations(range(M), 4),
               key=lambda s: (sum(L[c] for c in s), tuple(-c for c in s)))
    rows = []
    for v in range(V):
        g = [A[v][c] for c in best]
        pair = max(itertools.combinations(range(4), 2),
                   key=lambda p: (g[p[0]] + g[p[1]], (-p[0], -p[1])))
        rows.append(pair)
    return best, rows


@pytest.mark.parametrize("V", [1, 2, 4])
@pytest.mark.parametrize("M", [4, 5, 6, 7, 8])
@pytest.mark.parametrize("kind", ["normal", "ints", "binary"])
def test_brute_force_tiny_blocks(V, M, kind):
    rng = np.random.default_rng(1000 * V + 10 * M + len(kind))
    R, B = 3, 4
    W = _rand_w(rng, R * V, B * M, kind)
    colidx, pos, _ = orc.prune(W, V, M)
    for r in range(R):
        for b in range(B):
            best, rows = _brute_block(W[r * V:(r + 1) * V, b * M:(b + 1) * M])
            assert tuple(int(c) for c in colidx[r, b]) == best
            for v in range(V):
                assert tuple(int(p) for p in pos[r * V + v, b]) == rows[v]


def test_kept_mass_is_optimal():
    rng = np.random.default_rng(7)
    V, M, R, B = 8, 7, 2, 5
    W = _rand_w(rng, R * V, B * M, "normal")
    colidx, pos, mask = orc.prune(W, V, M)
    A = np.abs(W.astype(np.float64))
    for r in range(R):
        for b in range(B):
            blk = A[r * V:(r + 1) * V, b * M:(b + 1) * M]
            L = blk.sum(axis=0)
            kept = L[colidx[r, b].astype(int)].sum()
            assert all(kept >= L[list(s)].sum() for s in itertools.combinations(range(M), 4))
            for v in range(V):
                g = blk[v, colidx[r, b].astype(int)]
                k2 = g[pos[r * V + v, b].astype(int)].sum()
                assert all(k2 >= g[list(p)].sum() for p in itertools.combinations(range(4), 2))


# ------------------------------------------------------------- special cases

def _textbook_2_4(W):
    """Plain 2:4 magnitude pruning of aligned groups of four, written as loops."""
    out, inn = W.shape
    mask = np.zeros((out, inn), np.uint8)
    for o in range(out):
        for g0 in range(0, inn, 4):
            grp = [abs(float(W[o, g0 + k])) for k in range(4)]
            order = sorted(range(4), key=lambda k: (-grp[k], k))
            for k in order[:2]:
                mask[o, g0 + k] = 1
    return mask


@pytest.mark.parametrize("V", [16, 32, 64])
def test_m4_reduces_to_plain_2_4(V):
    """M = 4 is plain 2:4 (abstract; caption of the selected-(V,M) table: '(X,4) means 2:4')."""
    rng = np.random.default_rng(V)
    W = _rand_w(rng, 64, 48, "ints" if V == 32 else "normal")
    colidx, pos, mask = orc.prune(W, V, 4)
    assert np.all(colidx == np.array([0, 1, 2, 3], np.uint8))
    assert np.array_equal(mask, _textbook_2_4(W))


@pytest.mark.parametrize("M", [5, 6, 8, 11])
def test_v1_reduces_to_top2_of_m(M):
    """With V = 1 the column norm is the weight's own magnitude, so keeping 4 of M
    and then 2 of 4 is the same as keeping the top 2 of each group of M."""
    rng = np.random.default_rng(M)
    W = _rand_w(rng, 12, 6 * M, "ints" if M == 6 else "normal")
    _, _, mask = orc.prune(W, 1, M)
    exp = np.zeros_like(mask)
    for o in range(W.shape[0]):
        for g0 in range(0, W.shape[1], M):
            grp = [abs(float(W[o, g0 + k])) for k in range(M)]
            for k in sorted(range(M), key=lambda k: (-grp[k], k))[:2]:
                exp[o, g0 + k] = 1
    assert np.array_equal(mask, exp)


def test_adversarial_ties():
    V, M = 4, 6
    # all-equal and all-zero matrices: first four columns, first two positions
    for W in (np.full((8, 12), 0.5, np.float16), np.zeros((8, 12), np.float16)):
        colidx, pos, mask = orc.prune(W, V, M)
        assert np.all(colidx == np.array([0, 1, 2, 3], np.uint8))
        assert np.all(pos == np.array([0, 1], np.uint8))
        assert np.array_equal(mask[:, :6], np.tile(np.array([1, 1, 0, 0, 0, 0], np.uint8), (8, 1)))
    # +w / -w pairs have equal magnitude: sign must not matter, -0.0 equals +0.0
    W = np.array([[1, -1, 1, -1, 1, -1]] * 4, np.float16)
    colidx, pos, _ = orc.prune(W, V, M)
    assert tuple(colidx[0, 0]) == (0, 1, 2, 3) and np.all(pos == np.array([0, 1], np.uint8))
    W = np.array([[-0.0, 0.0, -0.0, 0.0, 0.0, 3.0]] * 4, np.float16)
    colidx, pos, mask = orc.prune(W, V, M)
    assert tuple(colidx[0, 0]) == (0, 1, 2, 5)
    assert np.all(pos == np.array([0, 3], np.uint8))      # the 3.0, then the lowest-position zero
    # a single non-zero in the block, in the last column
    W = np.zeros((4, 6), np.float16); W[2, 5] = -1
    colidx, pos, mask = orc.prune(W, V, M)
    assert tuple(colidx[0, 0]) == (0, 1, 2, 5)
    assert tuple(pos[2, 0]) == (0, 3) and tuple(pos[0, 0]) == (0, 1)


def test_pad_columns_never_beat_real_columns():
    """in = 7 with M = 5: block 1 has real columns 5, 6 and three pad columns."""
    W = np.zeros((4, 7), np.float16)
    W[:, 6] = 1
    colidx, pos, mask = orc.prune(W, 4, 5)
    assert tuple(colidx[0, 1]) == (0, 1, 2, 3)           # real 0 (zero), real 1, pads 2, 3
    assert np.all(pos[:4, 1] == np.array([0, 1], np.uint8))
    assert mask.shape == (4, 7) and np.all(mask[:, 5:] == 1)


# ------------------------------------------------------------ worked example

def test_hand_worked_example():
    with open(os.path.join(GOLDEN, "worked_example_v2_m5.json")) as f:
        g = json.load(f)
    W = np.array(g["W"], np.float16)
    V, M, out, inn = g["V"], g["M"], g["out"], g["in"]
    values, meta, colidx, mask = orc.compress(W, V, M)
    _, pos, _ = orc.prune(W, V, M)
    assert colidx.tolist() == g["colidx"]
    assert pos.tolist() == g["pos"]
    assert mask.tolist() == g["mask"]
    assert values.astype(np.float64).tolist() == g["values"]
    assert meta.tolist() == g["meta"]
    Wm = orc.masked_dense(W, mask)
    assert Wm.astype(np.float64).tolist() == g["masked_dense"]
    assert orc.decompress(values, meta, colidx, out, inn, V, M).astype(np.float64).tolist() == g["masked_dense"]
    X = np.array(g["X"], np.float16)
    assert orc.matmul_ref(X, Wm).tolist() == g["Y"]
    assert orc.spmm_ref(X, values, meta, colidx, out, inn, V, M).tolist() == g["Y"]


# ---------------------------------------------------------------- round trips

@pytest.mark.parametrize("out,inn,V,M", [(128, 128, 64, 8), (70, 37, 16, 5), (96, 50, 32, 7), (64, 64, 32, 4)])
def test_round_trips(out, inn, V, M):
    rng = np.random.default_rng(out + inn)
    W = _rand_w(rng, out, inn, "normal")
    W[rng.random(W.shape) < 0.05] = np.float16(-0.0)        # kept -0.0 must stay -0.0
    values, meta, colidx, mask = orc.compress(W, V, M)
    Wm = orc.masked_dense(W, mask)
    Wd = orc.decompress(values, meta, colidx, out, inn, V, M)
    assert np.array_equal(Wd.view(np.uint16), Wm.view(np.uint16))          # bit for bit
    # pruned entries are +0.0
    assert np.all(Wm.view(np.uint16)[mask == 0] == 0)
    # compress(decompress(c)) reproduces the values and the mask (the selection of an
    # already-sparse matrix is itself unless zeros tie, so compare on the value level)
    v2, m2, c2, mask2 = orc.compress(Wd, V, M)
    Wd2 = orc.decompress(v2, m2, c2, out, inn, V, M)
    assert np.array_equal(Wd2.view(np.uint16) & 0x7FFF, Wd.view(np.uint16) & 0x7FFF)
    # shapes of the triple (Appendix A): positions mirror the values; 4 indices per block
    out_pad, in_pad, R, B = orc.padded_dims(out, inn, V, M)
    assert values.shape == (out_pad, 2 * B) and meta.shape == (out_pad, (B + 1) // 2)
    assert colidx.shape == (R, B, 4)
    assert np.array_equal(orc.unpack_meta(meta, B), orc.prune(W, V, M)[1])


# ------------------------------------------------- exact column sums (integers)

def _fp16_units(h):
    """|h| as an integer multiple of 2**-24, decoded from the bit pattern."""
    bits = int(np.float16(h).view(np.uint16)) & 0x7FFF
    e, m = bits >> 10, bits & 0x3FF
    return m if e == 0 else (1024 + m) << (e - 1)


def test_column_sums_are_exact():
    rng = np.random.default_rng(3)
    V, M = 128, 5
    W = (rng.standard_normal((V, 4 * M)) * np.array([1e-6, 0.02, 3.0, 500.0] * 5)).astype(np.float16)
    W[0, 0] = np.float16(6e-8)          # subnormal
    W[1, 1] = np.float16(65504.0)       # largest finite
    L = orc.column_l1(orc.importance_abs(W), V, M)
    for b in range(4):
        for c in range(M):
            exact = sum(_fp16_units(W[v, b * M + c]) for v in range(V))
            assert Fraction(float(L[0, b, c])) == Fraction(exact, 2 ** 24)
    # and the result does not depend on the order of the rows
    perm = rng.permutation(V)
    L2 = orc.column_l1(orc.importance_abs(W[perm]), V, M)
    assert np.array_equal(L, L2)


# ----------------------------------------------------------------- the product

def test_matmul_against_triple_loop_and_formula():
    rng = np.random.default_rng(11)
    out, inn, T, V, M = 32, 23, 5, 16, 5
    W = _rand_w(rng, out, inn, "normal")
    X = rng.standard_normal((T, inn)).astype(np.float16)
    values, meta, colidx, mask = orc.compress(W, V, M)
    Wm = orc.masked_dense(W, mask)
    Y = orc.matmul_ref(X, Wm)
    Ys = orc.spmm_ref(X, values, meta, colidx, out, inn, V, M)
    for t in range(T):
        for o in range(out):
            acc = Fraction(0)
            for i in range(inn):
                if mask[o, i]:
                    acc += Fraction(float(X[t, i])) * Fraction(float(W[o, i]))
            assert abs(Fraction(float(Y[t, o])) - acc) <= abs(acc) * Fraction(1, 10 ** 12) + Fraction(1, 10 ** 15)
            assert abs(Fraction(float(Ys[t, o])) - acc) <= abs(acc) * Fraction(1, 10 ** 12) + Fraction(1, 10 ** 15)


def test_matmul_one_hot_reads_back_masked_weights():
    rng = np.random.default_rng(12)
    out, inn, V, M = 32, 20, 16, 5
    W = _rand_w(rng, out, inn, "normal")
    values, meta, colidx, mask = orc.compress(W, V, M)
    X = np.eye(inn, dtype=np.float16)
    Wm = orc.masked_dense(W, mask)
    assert np.array_equal(orc.matmul_ref(X, Wm), Wm.astype(np.float64).T)
    assert np.array_equal(orc.spmm_ref(X, values, meta, colidx, out, inn, V, M), Wm.astype(np.float64).T)


def test_matmul_small_integers_exact():
    W, X = syn.small_integer_case(48, 35, 9, seed=5)
    V, M = 16, 7
    values, meta, colidx, mask = orc.compress(W, V, M)
    Wm = orc.masked_dense(W, mask)
    exp = (X.astype(np.int64) @ (W.astype(np.int64) * mask).T).astype(np.float64)
    assert np.array_equal(orc.matmul_ref(X, Wm), exp)
    assert np.array_equal(orc.spmm_ref(X, values, meta, colidx, out=48, inn=35, V=V, M=M), exp)


def test_error_measure():
    Y = np.array([[1.0, -4.0]]); Z = np.array([[1.5, -4.0]])
    assert orc.max_normalised_error(Z, Y) == 0.125
    assert orc.max_normalised_error(Y, Y) == 0.0


# ------------------------------------------------ density against Table 5

def test_density_matches_table5_param_counts():
    with open(os.path.join(GOLDEN, "table5_param_counts.json")) as f:
        g = json.load(f)
    for key in ("deit_small", "deit_base"):
        c = g[key]
        h, m, V, M = c["hidden"], c["mlp"], c["V"], c["M"]
        shapes = [(3 * h, h), (h, h), (m, h), (h, m)]
        dense = sum(o * i for o, i in shapes) * c["blocks"]
        kept = 0
        for o, i in shapes:
            out_pad, in_pad, R, B = orc.padded_dims(o, i, V, M)
            kept += out_pad * 2 * B                      # two values per row per block
        kept *= c["blocks"]
        rest = c["dense_M"] * 1e6 - dense                # embeddings, norms, head: left dense
        assert abs((kept + rest) / 1e6 - c["sparse_M"]) < 0.25
    # and the oracle's own mask has that density on one of these layers
    W, _ = syn.make_weight_and_input(384, 384, 1, seed=1001)
    _, _, mask = orc.prune(W, 64, 5)
    out_pad, in_pad, R, B = orc.padded_dims(384, 384, 64, 5)
    assert mask.sum() <= out_pad * 2 * B and mask.sum() >= out_pad * 2 * B - 384 * 2  # last block may keep pads


def test_config0_shapes():
    (layer,) = syn.config_single_gemm()
    W, X = syn.layer_tensors(layer)
    assert W.shape == (128, 128) and X.shape == (16, 128) and W.dtype == np.float16
    values, meta, colidx, mask = orc.compress(W, layer.V, layer.M)
    assert values.shape == (128, 32) and meta.shape == (128, 8) and colidx.shape == (2, 16, 4)
    assert mask.sum() == 128 * 128 // 4
    assert abs(float(W.astype(np.float64).std()) - 0.02) < 0.002


# ------------------------------------------------------- scored pruning and RIA (Section 3, Eq. 1)

@pytest.mark.parametrize("out,inn,V,M", [(128, 128, 64, 8), (64, 37, 16, 5), (96, 50, 32, 7), (40, 64, 8, 4)])
@pytest.mark.parametrize("kind", ["normal", "ints", "binary"])
def test_scored_prune_with_abs_scores_is_the_abs_prune(out, inn, V, M, kind):
    """|w| handed in as an fp32 score matrix must reproduce the ABS pruning exactly (the fp32
    copies are exact, and so are their column sums in any order)."""
    rng = np.random.default_rng(out + inn + V + M)
    W = _rand_w(rng, out, inn, kind)
    ref = orc.compress(W, V, M)
    got = orc.compress(W, V, M, score=np.abs(W).astype(np.float32))
    for a, b in zip(ref, got):
        assert np.array_equal(a.view(np.uint16) if a.dtype == np.float16 else a,
                              b.view(np.uint16) if b.dtype == np.float16 else b)


def _brute_block_scored(Sb):
    V, M = Sb.shape
    A = [[_exact(Sb[v, c]) for c in range(M)] for v in range(V)]
    L = [sum(A[v][c] for v in range(V)) for c in range(M)]
    best = max(itertools.combinations(range(M), 4),
               key=lambda s: (sum(L[c] for c in s), tuple(-c for c in s)))
    rows = []
    for v in range(V):
        g = [A[v][c] for c in best]
        rows.append(max(itertools.combinations(range(4), 2),
                        key=lambda p: (g[p[0]] + g[p[1]], (-p[0], -p[1]))))
    return best, rows


@pytest.mark.parametrize("V", [1, 2, 4])
@pytest.mark.parametrize("M", [4, 5, 7])
@pytest.mark.parametrize("kind", ["dyadic", "ints"])
def test_scored_brute_force_tiny_blocks(V, M, kind):
    """Scores unrelated to |w| (so that a mix-up of W and the score shows): enumeration of all
    column subsets and row pairs in exact arithmetic.  Scores are dyadic, their sums exact."""
    rng = np.random.default_rng(77 * V + M + len(kind))
    R, B = 3, 4
    W = _rand_w(rng, R * V, B * M, "normal")
    if kind == "dyadic":
        S = (rng.integers(0, 1 << 12, size=W.shape) / 256.0).astype(np.float32)
    else:
        S = rng.integers(0, 3, size=W.shape).astype(np.float32)
    colidx, pos, mask = orc.prune(W, V, M, score=S)
    for r in range(R):
        for b in range(B):
            best, rows = _brute_block_scored(S[r * V:(r + 1) * V, b * M:(b + 1) * M])
            assert tuple(int(c) for c in colidx[r, b]) == best
            for v in range(V):
                assert tuple(int(p) for p in pos[r * V + v, b]) == rows[v]
    values, meta, ci, _ = orc.compress(W, V, M, score=S)
    assert np.array_equal(orc.decompress(values, meta, ci, R * V, B * M, V, M).view(np.uint16),
                          orc.masked_dense(W, mask).view(np.uint16))


def test_scored_column_sums_are_added_in_row_order():
    """A column whose fp64 sum depends on the order of addition: 2^53 + 1 + 1 is 2^53 when the
    large term comes first (each 1 is rounded away) and 2^53 + 2 when it comes last."""
    V, M = 3, 4
    S = np.zeros((V, M), dtype=np.float64)
    S[:, 0] = [2.0 ** 53, 1.0, 1.0]
    S[:, 1] = [0.5, 0.0, 0.0]
    assert np.array_equal(S.astype(np.float32).astype(np.float64), S)      # all are fp32 values
    assert orc.column_l1_in_row_order(S, V, M)[0, 0, 0] == 2.0 ** 53
    assert orc.column_l1_in_row_order(S[::-1].copy(), V, M)[0, 0, 0] == 2.0 ** 53 + 2.0
    assert orc.column_l1_in_row_order(S, V, M)[0, 0, 1] == 0.5


def test_ria_hand_worked_example():
    with open(os.path.join(GOLDEN, "ria_example.json")) as f:
        g = json.load(f)
    W = np.array(g["W"], dtype=np.float16)
    act = np.array(g["act"], dtype=np.float32)
    S = orc.importance_ria(W, act)
    exp = np.array([[float(Fraction(x)) for x in row] for row in g["score_fractions"]], dtype=np.float64)
    assert S.dtype == np.float32 and S.shape == W.shape
    assert np.allclose(S.astype(np.float64), exp, rtol=2.0 ** -23, atol=0)


def test_ria_closed_forms_and_invariances():
    rng = np.random.default_rng(5)
    out, inn = 24, 40
    act = (rng.random(inn) + 0.5).astype(np.float32)
    # all magnitudes equal: every weight gets (1/out + 1/in) * act_j, whatever the signs
    W = (np.float16(0.375) * rng.choice([-1.0, 1.0], size=(out, inn))).astype(np.float16)
    S = orc.importance_ria(W, act)
    exp = ((1.0 / out + 1.0 / inn) * act.astype(np.float64)).astype(np.float32)
    assert np.allclose(S, np.broadcast_to(exp, S.shape), rtol=2.0 ** -22, atol=0)
    # rank one, W = u v^T with positive factors: (u_i / sum u + v_j / sum v) * act_j
    u = 2.0 ** rng.integers(-3, 3, size=out)
    v = 2.0 ** rng.integers(-3, 3, size=inn)
    W = np.outer(u, v).astype(np.float16)
    S = orc.importance_ria(W, act)
    exp = (u[:, None] / u.sum() + v[None, :] / v.sum()) * act.astype(np.float64)[None, :]
    assert np.allclose(S.astype(np.float64), exp, rtol=2.0 ** -22, atol=0)
    # scaling W by a power of two changes nothing, bit for bit; permutations permute the scores
    W = _rand_w(rng, out, inn, "normal")
    S = orc.importance_ria(W, act)
    assert np.array_equal(orc.importance_ria((W.astype(np.float32) * 4.0).astype(np.float16), act), S)
    pr, pc = rng.permutation(out), rng.permutation(inn)
    assert np.array_equal(orc.importance_ria(W[pr][:, pc], act[pc]), S[pr][:, pc])
    # the activation factor multiplies its input channel (column), nothing else
    act2 = act.copy(); act2[3] *= np.float32(2.0)
    S2 = orc.importance_ria(W, act2)
    assert np.array_equal(S2[:, 3], S[:, 3] * np.float32(2.0))
    assert np.array_equal(np.delete(S2, 3, axis=1), np.delete(S, 3, axis=1))


def test_ria_zero_rows_and_columns_give_zero_scores():
    rng = np.random.default_rng(6)
    W = _rand_w(rng, 16, 20, "normal")
    W[:, 4] = 0; W[7, :] = 0
    S = orc.importance_ria(W, np.ones(20, dtype=np.float32))
    assert np.all(np.isfinite(S)) and np.all(S[:, 4] == 0) and np.all(S[7, :] == 0) and np.all(S >= 0)
    colidx, pos, mask = orc.prune(W, 8, 5, score=S)
    assert mask.reshape(2, 8, 4, 5).sum(axis=3).max() == 2           # still 2 per row and block
