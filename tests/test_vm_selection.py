"""V and M selection (Section 4.1): the oracle against the figures the paper prints, and the
library's host functions against the oracle.  No GPU is involved."""

import ctypes
import json
import math
import os

import numpy as np
import pytest

from oracle import vnm_oracle as orc

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


@pytest.fixture(scope="module")
def lib():
    path = os.path.join(ROOT, "paper_2410_16135_amd", "libvnm.so")
    if not os.path.exists(path):
        import __graft_entry__
        __graft_entry__.build()
    L = ctypes.CDLL(path)
    L.vnm_mask_diversity_log.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.POINTER(ctypes.c_double)]
    L.vnm_select_vm.argtypes = [ctypes.POINTER(ctypes.c_int), ctypes.POINTER(ctypes.c_int),
                                ctypes.POINTER(ctypes.c_double), ctypes.c_int, ctypes.c_double,
                                ctypes.POINTER(ctypes.c_int)]
    return L


@pytest.fixture(scope="module")
def golden():
    with open(os.path.join(GOLDEN, "vm_selection.json")) as f:
        return json.load(f)


def _lib_select(lib, cands, s):
    n = len(cands)
    V = (ctypes.c_int * n)(*[c[0] for c in cands])
    M = (ctypes.c_int * n)(*[c[1] for c in cands])
    sp = (ctypes.c_double * n)(*[c[2] for c in cands])
    sel = ctypes.c_int(-7)
    assert lib.vnm_select_vm(V, M, sp, n, s, ctypes.byref(sel)) == 0
    return sel.value


def test_simplified_md_matches_the_printed_table(golden):
    for V, M, printed in golden["simplified_md"]:
        assert abs(orc.mask_diversity_log(V, M) * golden["md_scale"] - printed) <= 1.0


def test_mask_diversity_is_the_count_of_configurations():
    """K ** (m n) is the number of (kept column set, kept pair per row) choices of a layer: check the
    closed form against direct counting on small layers."""
    for V, M, m, n in [(2, 5, 4, 10), (4, 6, 8, 6), (1, 4, 3, 8)]:
        per_block = math.comb(M, 4) * math.comb(4, 2) ** V
        count = per_block ** ((m // V) * (n // M))
        assert math.isclose(orc.mask_diversity_log(V, M) * m * n, math.log(count), rel_tol=1e-12)


def test_k_decreases_with_m_and_with_v():
    for V in (16, 32, 64, 128):
        ks = [orc.mask_diversity_log(V, M) for M in range(5, 33)]
        assert all(a > b for a, b in zip(ks, ks[1:]))
    for M in (5, 8, 16):
        ks = [orc.mask_diversity_log(V, M) for V in (16, 32, 64, 128)]
        assert all(a > b for a, b in zip(ks, ks[1:]))
    assert len({round(orc.mask_diversity_log(V, 4), 15) for V in (16, 32, 64, 128)}) == 1   # 2:4: V has no say


def test_selection_reproduces_the_printed_example(golden):
    cands = [tuple(c) for c in golden["bs1_candidates"]]
    for s, want in zip(golden["bs1_thresholds"], golden["bs1_selected"]):
        i = orc.select_vm(cands, s)
        assert list(cands[i][:2]) == want, (s, cands[i])
    assert orc.select_vm(cands, 2.5) == -1


def test_selection_phases():
    # phase 1: the smallest M of a V wins even when a larger M of the same V is faster
    assert orc.select_vm([(64, 8, 3.0), (64, 6, 2.0)], 1.5) == 1
    # phase 2: across V the larger K wins: (32, 6) beats (128, 5)?  ln K decides, not M alone
    c = [(128, 5, 2.0), (32, 6, 2.0)]
    want = 0 if orc.mask_diversity_log(128, 5) > orc.mask_diversity_log(32, 6) else 1
    assert orc.select_vm(c, 1.0) == want
    # ties in K (plain 2:4 entries): higher speedup, then smaller V, then earlier entry
    assert orc.select_vm([(64, 4, 1.2), (128, 4, 1.3)], 1.0) == 1
    assert orc.select_vm([(128, 4, 1.2), (64, 4, 1.2)], 1.0) == 1
    assert orc.select_vm([(64, 4, 1.2), (64, 4, 1.2)], 1.0) == 0


def test_library_matches_oracle(lib):
    rng = np.random.default_rng(11)
    k = ctypes.c_double()
    for V in (1, 16, 32, 64, 128):
        for M in (4, 5, 7, 16, 64, 255):
            assert lib.vnm_mask_diversity_log(V, 2, M, ctypes.byref(k)) == 0
            assert math.isclose(k.value, orc.mask_diversity_log(V, M), rel_tol=1e-14)
    for trial in range(200):
        n = int(rng.integers(0, 12))
        cands = [(int(rng.choice([16, 32, 64, 128])), int(rng.integers(4, 17)),
                  float(np.round(rng.random() * 2.0 + 0.8, 1))) for _ in range(n)]
        s = float(np.round(rng.random() * 2.0 + 0.8, 1))
        assert _lib_select(lib, cands, s) == orc.select_vm(cands, s), (cands, s)


def test_library_argument_errors(lib):
    k = ctypes.c_double()
    sel = ctypes.c_int()
    assert lib.vnm_mask_diversity_log(64, 2, 5, None) == 1
    assert lib.vnm_mask_diversity_log(64, 3, 5, ctypes.byref(k)) == 3
    assert lib.vnm_mask_diversity_log(64, 2, 3, ctypes.byref(k)) == 3
    assert lib.vnm_select_vm(None, None, None, 0, 1.0, ctypes.byref(sel)) == 0 and sel.value == -1
    assert lib.vnm_select_vm(None, None, None, 2, 1.0, ctypes.byref(sel)) == 1
    V = (ctypes.c_int * 1)(64); M = (ctypes.c_int * 1)(3); sp = (ctypes.c_double * 1)(2.0)
    assert lib.vnm_select_vm(V, M, sp, 1, 1.0, ctypes.byref(sel)) == 3
    assert lib.vnm_select_vm(V, M, sp, -1, 1.0, ctypes.byref(sel)) == 2
