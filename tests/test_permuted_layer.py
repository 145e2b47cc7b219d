"""Pins for the oracle's permuted-layer functions (Section 4.2, Eq. 6) -- CPU only.

Eq. 6 is an identity between the layer on the original weight and the layer on the permuted weight
wrapped in the two transposed permutation matrices.  The pins evaluate that identity with explicit
0-1 permutation matrices and with the plain dense product of the ORIGINAL weight, neither of which
shares code with the oracle's index-based implementation: an inverted permutation, a permutation
applied on the wrong side, or a bias left in the wrong order fails them.
"""
import ctypes

import numpy as np
import pytest

from oracle import vnm_oracle as orc
import synth_inputs as syn


def _perm_matrices(po, pi):
    Po = np.zeros((po.size, po.size))
    Po[np.arange(po.size), po] = 1.0        # (P_o W)[o, :] = W[po[o], :]
    Pi = np.zeros((pi.size, pi.size))
    Pi[pi, np.arange(pi.size)] = 1.0        # (W P_i)[:, i] = W[:, pi[i]]
    return Po, Pi


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_permute_weight_is_po_w_pi(seed):
    rng = np.random.default_rng(seed)
    W = rng.standard_normal((12, 10))
    po, pi = rng.permutation(12), rng.permutation(10)
    Po, Pi = _perm_matrices(po, pi)
    assert np.array_equal(orc.permute_weight(W, po, pi), Po @ W @ Pi)


@pytest.mark.parametrize("seed,V,M", [(0, 4, 5), (1, 8, 6), (2, 16, 8)])
def test_eq6_with_explicit_matrices(seed, V, M):
    """Y = P_o^T W_p P_i^T X with the matrices written out (paper orientation: X is [in x T])."""
    rng = np.random.default_rng(seed)
    out, inn, T = 2 * V, 4 * M, 7
    W, X = syn.make_weight_and_input(out, inn, T, seed=seed)
    po, pi = rng.permutation(out), rng.permutation(inn)
    Wp = orc.permute_weight(W, po, pi)
    Wm_p = orc.masked_dense(Wp, orc.compress(Wp, V, M)[3])
    Po, Pi = _perm_matrices(po, pi)
    Y_paper = (Po.T @ Wm_p.astype(np.float64) @ Pi.T @ X.astype(np.float64).T).T
    Y = orc.linear_fused_ref(X, Wm_p, perm_in=pi, perm_out=po)
    assert np.allclose(Y, Y_paper, rtol=0, atol=1e-12 * np.abs(Y_paper).max())


@pytest.mark.parametrize("seed", [3, 4])
def test_lossless_case_equals_the_original_layer(seed):
    """If the permuted weight already has the pattern, pruning it changes nothing and the fused
    layer must equal the plain dense layer on the ORIGINAL weight and bias."""
    rng = np.random.default_rng(seed)
    V, M, out, inn, T = 8, 5, 24, 30, 9
    W0, X = syn.make_weight_and_input(out, inn, T, seed=seed)
    Wp_sparse = orc.masked_dense(W0, orc.compress(W0, V, M)[3])       # has the pattern
    po, pi = rng.permutation(out), rng.permutation(inn)
    W = np.zeros_like(Wp_sparse)
    W[np.ix_(po, pi)] = Wp_sparse                                      # W_p = P_o W P_i  <=>  W[po[o], pi[i]] = W_p[o, i]
    assert np.array_equal(orc.permute_weight(W, po, pi).view(np.uint16), Wp_sparse.view(np.uint16))
    bias = rng.standard_normal(out).astype(np.float16)                 # original channel order
    Y_dense = X.astype(np.float64) @ W.astype(np.float64).T + bias.astype(np.float64)[None, :]
    mask = orc.compress(orc.permute_weight(W, po, pi), V, M)[3]
    Wm_p = orc.masked_dense(orc.permute_weight(W, po, pi), mask)
    assert np.array_equal(Wm_p.view(np.uint16), Wp_sparse.view(np.uint16))
    Y = orc.linear_fused_ref(X, Wm_p, bias=bias[po], perm_in=pi, perm_out=po)
    assert np.allclose(Y, Y_dense, rtol=0, atol=1e-12 * np.abs(Y_dense).max())


def test_identity_and_missing_permutations():
    W, X = syn.make_weight_and_input(16, 20, 5, seed=9)
    Wm = orc.masked_dense(W, orc.compress(W, 8, 5)[3])
    Y0 = orc.matmul_ref(X, Wm)
    ident_o, ident_i = np.arange(16), np.arange(20)
    assert np.array_equal(orc.linear_fused_ref(X, Wm), Y0)
    assert np.array_equal(orc.linear_fused_ref(X, Wm, perm_in=ident_i, perm_out=ident_o), Y0)
    b = np.arange(16).astype(np.float16)
    assert np.array_equal(orc.linear_fused_ref(X, Wm, bias=b), Y0 + np.arange(16.0)[None, :])


def test_one_hot_inputs_read_back_permuted_columns():
    """Token t = unit vector of channel c: Y[t, po[o]] = W_p[o, i] with pi[i] = c."""
    rng = np.random.default_rng(5)
    out, inn = 8, 10
    Wp = rng.integers(-4, 5, size=(out, inn)).astype(np.float16)
    po, pi = rng.permutation(out), rng.permutation(inn)
    X = np.eye(inn, dtype=np.float16)
    Y = orc.linear_fused_ref(X, Wp, perm_in=pi, perm_out=po)
    for c in range(inn):
        i = int(np.where(pi == c)[0][0])
        for o in range(out):
            assert Y[c, po[o]] == float(Wp[o, i])


@pytest.mark.parametrize("seed", [0, 1])
def test_folding_two_layers(seed):
    """Two layers in a row: leaving the first layer's output in permuted order and folding its P_o
    into the second layer's input permutation gives the same result as un-permuting in between."""
    rng = np.random.default_rng(seed)
    d0, d1, d2, T = 10, 12, 8, 6
    W1p = rng.standard_normal((d1, d0)).astype(np.float16)
    W2p = rng.standard_normal((d2, d1)).astype(np.float16)
    X = rng.standard_normal((T, d0)).astype(np.float16)
    po1, pi1 = rng.permutation(d1), rng.permutation(d0)
    po2, pi2 = rng.permutation(d2), rng.permutation(d1)
    H = orc.linear_fused_ref(X, W1p, perm_in=pi1, perm_out=po1).astype(np.float16)
    Y_ref = orc.linear_fused_ref(H, W2p, perm_in=pi2, perm_out=po2)
    Hp = orc.linear_fused_ref(X, W1p, perm_in=pi1).astype(np.float16)          # permuted order kept
    Y = orc.linear_fused_ref(Hp, W2p, perm_in=orc.fold_permutations(po1, pi2), perm_out=po2)
    assert np.array_equal(Y, Y_ref)
    # choosing the next layer's input permutation equal to this layer's output permutation folds to the identity
    assert np.array_equal(orc.fold_permutations(po1, po1), np.arange(d1))


# ---------------------------------------------------------------- host entry point of the library

@pytest.fixture(scope="module")
def lib():
    import paper_2410_16135_amd as vnm
    return vnm.load_library()


def _fold(lib, po, pi):
    po = np.ascontiguousarray(po, dtype=np.int32)
    pi = np.ascontiguousarray(pi, dtype=np.int32)
    res = np.full(po.size, -7, dtype=np.int32)
    rc = lib.vnm_fold_permutations(po.ctypes.data_as(ctypes.c_void_p), pi.ctypes.data_as(ctypes.c_void_p),
                                   ctypes.c_int64(po.size), res.ctypes.data_as(ctypes.c_void_p))
    return rc, res


def test_library_fold_matches_oracle(lib):
    rng = np.random.default_rng(0)
    for n in (1, 2, 7, 64, 1000):
        po, pi = rng.permutation(n), rng.permutation(n)
        rc, res = _fold(lib, po, pi)
        assert rc == 0
        assert np.array_equal(res, orc.fold_permutations(po, pi))


def test_library_fold_rejects_non_permutations(lib):
    rc, _ = _fold(lib, [0, 1, 1], [0, 1, 2])
    assert rc == 2
    rc, _ = _fold(lib, [0, 1, 2], [0, 3, 2])
    assert rc == 2
    rc, _ = _fold(lib, [0, -1, 2], [0, 1, 2])
    assert rc == 2
    assert lib.vnm_fold_permutations(None, None, ctypes.c_int64(3), None) == 1
