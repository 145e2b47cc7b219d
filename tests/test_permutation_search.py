"""Pins for the oracle's permutation search (Section 4.2, Eqs. 7-9) and checks of the library's host
solver -- CPU only.

The paper prints no numbers for the search itself (its table on the number of iterations reports
accuracies of trained models), so the pins are identities that any correct implementation of the
stated objective must satisfy: the assignment solver against exhaustive enumeration, the gain
matrices against the objective evaluated on an actually permuted matrix, monotonicity, and a
planted case whose optimum is known.
"""
import ctypes
import itertools

import numpy as np
import pytest

from oracle import vnm_oracle as orc


def _scores(rng, out, inn):
    return (rng.random((out, inn)) ** 3).astype(np.float32)


@pytest.mark.parametrize("n", [1, 2, 3, 5, 6])
@pytest.mark.parametrize("seed", [0, 1, 2])
def test_assignment_against_enumeration(n, seed):
    rng = np.random.default_rng(seed)
    gain = rng.integers(0, 6 if seed else 1000, size=(n, n))            # seed 1, 2: many ties
    assign, total = orc.lsa_max(gain)
    best = max(sum(gain[i, p[i]] for i in range(n)) for p in itertools.permutations(range(n)))
    assert sorted(assign) == list(range(n))
    assert total == best == sum(gain[i, assign[i]] for i in range(n))


def test_quantisation():
    S = np.array([[0.0, 0.4999, 0.5001, 1.5, 2.5, 1e12, -3.0]], dtype=np.float32)
    q = orc.quantise_scores(S, 1.0)
    assert q.dtype == np.int64
    assert q.tolist() == [[0, 0, 1, 2, 2, 2 ** 32 - 1, 0]]               # rint: ties to even; clipped both ways


@pytest.mark.parametrize("out,inn,V,M", [(8, 20, 4, 5), (12, 18, 4, 6), (8, 17, 4, 4), (10, 20, 4, 5)])
def test_identity_assignment_reproduces_the_objective(out, inn, V, M):
    """Blocks are pruned independently, so the objective is the sum of the diagonal gains plus what
    the ragged tail keeps -- for every slot, in both half-steps."""
    rng = np.random.default_rng(out + inn)
    Sq = orc.quantise_scores(_scores(rng, out, inn), 1000.0)
    total = orc.retained_score(Sq, V, M)
    Bf, Rf = inn // M, out // V
    tail_cols = orc.retained_score(Sq[:, Bf * M:], V, M) if inn % M else 0
    tail_rows = orc.retained_score(Sq[Rf * V:], V, M) if out % V else 0
    for slot in range(M):
        assert np.trace(orc.perm_gain_in(Sq, V, M, slot)) + tail_cols == total
    for slot in range(V):
        assert np.trace(orc.perm_gain_out(Sq, V, M, slot)) + tail_rows == total


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_gains_predict_the_objective_after_a_swap(seed):
    """Swapping the slot channels of two blocks changes the objective by exactly
    gain[b,k] + gain[k,b] - gain[b,b] - gain[k,k]; the objective is evaluated on the really
    permuted matrix by the pruning oracle, not by the gain code."""
    rng = np.random.default_rng(seed)
    out, inn, V, M = 8, 20, 4, 5
    Sq = orc.quantise_scores(_scores(rng, out, inn), 1000.0)
    base = orc.retained_score(Sq, V, M)
    for slot in (0, 3):
        g = orc.perm_gain_in(Sq, V, M, slot)
        b, k = 0, 2
        pi = np.arange(inn)
        pi[[b * M + slot, k * M + slot]] = pi[[k * M + slot, b * M + slot]]
        assert orc.retained_score(Sq[:, pi], V, M) - base == g[b, k] + g[k, b] - g[b, b] - g[k, k]
    for slot in (1, 2):
        g = orc.perm_gain_out(Sq, V, M, slot)
        r, k = 1, 0
        po = np.arange(out)
        po[[r * V + slot, k * V + slot]] = po[[k * V + slot, r * V + slot]]
        assert orc.retained_score(Sq[po], V, M) - base == g[r, k] + g[k, r] - g[r, r] - g[k, k]


@pytest.mark.parametrize("out,inn,V,M", [(8, 20, 4, 5), (16, 24, 4, 6), (8, 16, 8, 4), (10, 22, 4, 5)])
def test_search_is_monotone_and_consistent(out, inn, V, M):
    rng = np.random.default_rng(out * inn)
    S = _scores(rng, out, inn)
    po, pi, hist = orc.permutation_search(S, V, M, scale=1000.0, iterations=2)
    assert len(hist) == 5
    assert all(b >= a for a, b in zip(hist, hist[1:]))
    assert sorted(po) == list(range(out)) and sorted(pi) == list(range(inn))
    Sq = orc.quantise_scores(S, 1000.0)
    assert orc.permutation_objective(Sq, V, M, po, pi) == hist[-1]
    # ragged tails stay in place
    assert list(po[(out // V) * V:]) == list(range((out // V) * V, out))
    assert list(pi[(inn // M) * M:]) == list(range((inn // M) * M, inn))


def test_planted_case_reaches_the_known_optimum():
    """Eight heavy columns sit in two blocks of eight (M = 8 keeps only 4 per block, so half of the
    heavy mass is lost); spreading them 4 + 4 + ... keeps everything heavy, which is optimal.  The
    input half-step must find an arrangement that keeps all heavy columns."""
    out, V, M, B = 8, 4, 8, 4
    S = np.full((out, B * M), 1.0, dtype=np.float32)
    S[:, 0:8] = 100.0                                   # block 0 holds all 8 heavy columns
    po, pi, hist = orc.permutation_search(S, V, M, scale=1.0, iterations=1)
    assert hist[0] == out * (2 * 100 + 3 * 2 * 1)       # block 0 keeps 2 heavy per row, the others 2 light
    assert hist[1] == out * (2 * 100 * 4)               # every block keeps 2 heavy values per row


# ---------------------------------------------------------------- the library's host solver

@pytest.fixture(scope="module")
def lib():
    import paper_2410_16135_amd as vnm
    return vnm.load_library()


def _lib_lsa(lib, gain):
    g = np.ascontiguousarray(gain, dtype=np.int64)
    n = g.shape[0]
    assign = np.full(n, -1, dtype=np.int32)
    total = ctypes.c_int64(0)
    rc = lib.vnm_lsa_max(g.ctypes.data_as(ctypes.c_void_p), n, assign.ctypes.data_as(ctypes.c_void_p),
                         ctypes.byref(total))
    return rc, assign, total.value


@pytest.mark.parametrize("n", [1, 2, 3, 6, 17, 64, 200])
@pytest.mark.parametrize("kind", ["random", "ties", "large"])
def test_library_assignment_matches_oracle_value(lib, n, kind):
    rng = np.random.default_rng(n)
    hi = {"random": 10 ** 6, "ties": 4, "large": 2 ** 45}[kind]
    gain = rng.integers(0, hi, size=(n, n))
    rc, assign, total = _lib_lsa(lib, gain)
    assert rc == 0
    assert sorted(assign) == list(range(n))
    assert total == sum(int(gain[i, assign[i]]) for i in range(n))
    assert total == orc.lsa_max(gain)[1]


def _lib_lsa_method(lib, gain, method):
    g = np.ascontiguousarray(gain, dtype=np.int64)
    n = g.shape[0]
    assign = np.full(n, -1, dtype=np.int32)
    total = ctypes.c_int64(0)
    rc = lib.vnm_lsa_max_method(g.ctypes.data_as(ctypes.c_void_p), n, method, assign.ctypes.data_as(ctypes.c_void_p),
                                ctypes.byref(total))
    return rc, assign, total.value


LSA_AUTO, LSA_HUNGARIAN, LSA_AUCTION, LSA_AUCTION_SCALAR = 0, 1, 2, 3


def _search_like_gain(n, seed):
    """A gain matrix with the structure the search produces: every row prefers the same few columns
    (block k gains max(0, x_i - t_k) summed over rows of the matrix), all values distinct or not."""
    rng = np.random.default_rng(seed)
    x = rng.integers(0, 2 ** 20, size=(n, 32))            # lifted channel i, 32 row blocks
    t = rng.integers(0, 2 ** 20, size=(n, 32))            # threshold of block k per row block
    base = rng.integers(2 ** 30, 2 ** 31, size=n)
    return base[None, :] + np.maximum(0, x[:, None, :] - t[None, :, :]).sum(axis=2)


@pytest.mark.parametrize("n", [1, 2, 3, 5, 17, 64, 200])
@pytest.mark.parametrize("kind", ["random", "ties", "large", "search"])
def test_auction_and_hungarian_agree_with_the_oracle(lib, n, kind):
    """Two independent exact methods of the library and the oracle's solver reach the same optimum;
    each returned assignment is a permutation that attains it."""
    rng = np.random.default_rng(100 + n)
    if kind == "search":
        gain = _search_like_gain(n, n)
    else:
        gain = rng.integers(0, {"random": 10 ** 6, "ties": 4, "large": 2 ** 45}[kind], size=(n, n))
    want = orc.lsa_max(gain)[1]
    got = {}
    for method in (LSA_HUNGARIAN, LSA_AUCTION, LSA_AUCTION_SCALAR, LSA_AUTO):
        rc, assign, total = _lib_lsa_method(lib, gain, method)
        assert rc == 0
        assert sorted(assign) == list(range(n))
        assert total == sum(int(gain[i, assign[i]]) for i in range(n)) == want
        got[method] = assign
    # the vector row scan and the scalar one make the same bids, so even among ties the same assignment
    assert np.array_equal(got[LSA_AUCTION], got[LSA_AUCTION_SCALAR])
    assert np.array_equal(got[LSA_AUCTION], got[LSA_AUTO])


def test_auction_brute_force_small(lib):
    """The auction against enumeration of all permutations, ties included."""
    import itertools
    rng = np.random.default_rng(5)
    for trial in range(40):
        n = int(rng.integers(2, 7))
        gain = rng.integers(0, 6 if trial % 2 else 1000, size=(n, n))
        best = max(sum(int(gain[i, p[i]]) for i in range(n)) for p in itertools.permutations(range(n)))
        rc, assign, total = _lib_lsa_method(lib, gain, LSA_AUCTION)
        assert rc == 0 and total == best and sorted(assign) == list(range(n))


def test_auction_gives_up_on_values_it_cannot_scale(lib):
    """Gains near 2^60 times n + 1 do not fit 62 bits: the auction alone refuses, the default falls
    back to the Hungarian method and is still exact."""
    rng = np.random.default_rng(9)
    gain = rng.integers(2 ** 59, 2 ** 60, size=(8, 8))
    assert _lib_lsa_method(lib, gain, LSA_AUCTION)[0] == 3          # VNM_ERR_UNSUPPORTED
    rc, assign, total = _lib_lsa_method(lib, gain, LSA_AUTO)
    assert rc == 0 and total == orc.lsa_max(gain)[1]
    assert _lib_lsa_method(lib, gain, 7)[0] == 3                    # unknown method


def test_library_assignment_errors(lib):
    assert lib.vnm_lsa_max(None, 3, None, None) == 1
    g = np.zeros((2, 2), dtype=np.int64)
    a = np.zeros(2, dtype=np.int32)
    t = ctypes.c_int64(0)
    assert lib.vnm_lsa_max(g.ctypes.data_as(ctypes.c_void_p), 0, a.ctypes.data_as(ctypes.c_void_p), ctypes.byref(t)) == 2
    g[0, 0] = -1
    assert lib.vnm_lsa_max(g.ctypes.data_as(ctypes.c_void_p), 2, a.ctypes.data_as(ctypes.c_void_p), ctypes.byref(t)) == 2
