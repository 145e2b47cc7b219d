"""Pins for the oracle's LoRA merge / mask refresh (Section 4.3, Eq. 10) -- CPU only.

The merge is a rank-r update in a fixed fp32 order; the pins check it against exact integer
arithmetic where every intermediate is representable, against an fp64 evaluation within the rounding
bound of that order, and against closed forms; the refreshed mask against Eq. 10's structure."""
import numpy as np
import pytest

from oracle import vnm_oracle as orc
import synth_inputs as syn


def test_zero_adapter_and_zero_scale_leave_w_unchanged():
    W, _ = syn.make_weight_and_input(24, 40, 1, seed=0)
    A = np.random.default_rng(0).standard_normal((4, 40)).astype(np.float32)
    assert np.array_equal(orc.lora_merge(W, np.zeros((24, 4), np.float32), A, 2.0).view(np.uint16), W.view(np.uint16))
    B = np.random.default_rng(1).standard_normal((24, 4)).astype(np.float32)
    assert np.array_equal(orc.lora_merge(W, B, A, 0.0).view(np.uint16), W.view(np.uint16))
    assert np.array_equal(orc.lora_merge(W, np.zeros((24, 0), np.float32), np.zeros((0, 40), np.float32), 2.0).view(np.uint16),
                          W.view(np.uint16))


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_small_integers_are_exact(seed):
    """Integer-valued operands: every product and partial sum is an integer below 2^11, exact in
    fp32 and in fp16, so the merge must equal W + s B A computed in integer arithmetic."""
    rng = np.random.default_rng(seed)
    W = rng.integers(-20, 21, size=(16, 24)).astype(np.float16)
    B = rng.integers(-3, 4, size=(16, 5)).astype(np.float32)
    A = rng.integers(-3, 4, size=(5, 24)).astype(np.float32)
    want = W.astype(np.int64) + 2 * (B.astype(np.int64) @ A.astype(np.int64))
    assert np.array_equal(orc.lora_merge(W, B, A, 2.0).astype(np.int64), want)


@pytest.mark.parametrize("r", [1, 16, 64])
def test_within_the_rounding_bound_of_an_fp64_evaluation(r):
    rng = np.random.default_rng(r)
    W, _ = syn.make_weight_and_input(32, 48, 1, seed=r)
    B = (rng.standard_normal((32, r)) * 0.05).astype(np.float32)
    A = (rng.standard_normal((r, 48)) * 0.05).astype(np.float32)
    exact = W.astype(np.float64) + 2.0 * (B.astype(np.float64) @ A.astype(np.float64))
    got = orc.lora_merge(W, B, A, 2.0).astype(np.float64)
    # fp32 chain: (r + 2) roundings of relative 2^-24 on magnitudes bounded by sum |b a|; then one fp16 rounding
    bound = (r + 2) * 2.0 ** -24 * (np.abs(W).astype(np.float64) + 2.0 * (np.abs(B).astype(np.float64) @ np.abs(A).astype(np.float64)))
    half_ulp16 = np.maximum(np.abs(exact), 2.0 ** -14) * 2.0 ** -11
    assert np.all(np.abs(got - exact) <= bound + half_ulp16 * 1.0001)


def test_rank_one_closed_form():
    """B = column of ones, A = row a, W = 0, scale 1: every row of the result is fp16(a)."""
    a = (np.arange(40, dtype=np.float32) - 20) / 7
    got = orc.lora_merge(np.zeros((8, 40), np.float16), np.ones((8, 1), np.float32), a[None, :], 1.0)
    assert np.array_equal(got.view(np.uint16), np.tile(a.astype(np.float16), (8, 1)).view(np.uint16))


@pytest.mark.parametrize("with_act", [False, True])
def test_refreshed_mask_has_the_pattern_and_eq10_holds(with_act):
    rng = np.random.default_rng(3)
    out, inn, V, M, r = 32, 40, 8, 5, 4
    W, _ = syn.make_weight_and_input(out, inn, 1, seed=3)
    B = (rng.standard_normal((out, r)) * 0.1).astype(np.float32)
    A = (rng.standard_normal((r, inn)) * 0.1).astype(np.float32)
    act = (0.5 + rng.random(inn)).astype(np.float32) if with_act else None
    merged, mask = orc.refresh_mask(W, B, A, 2.0, V, M, act)
    assert mask.sum() == out * inn * 2 // M
    blk = mask.reshape(out // V, V, inn // M, M)
    assert np.all((blk.sum(axis=1) > 0).sum(axis=-1) <= 4)          # at most 4 columns per block carry kept weights
    assert np.all(blk.sum(axis=-1) == 2)                            # 2 per row and block
    # Eq. 10: W' = (W + BA) (.) M, and the mask really is the pruning of the merged matrix
    score = None if act is None else orc.importance_ria(merged, act)
    values, meta, colidx, mask2 = orc.compress(merged, V, M, score=score)
    assert np.array_equal(mask, mask2)
    Wp = orc.decompress(values, meta, colidx, out, inn, V, M)
    assert np.array_equal(Wp.view(np.uint16), orc.masked_dense(merged, mask).view(np.uint16))
    # the adapter changes the mask (otherwise the test would not see a merge that was skipped)
    assert not np.array_equal(mask, orc.refresh_mask(W, np.zeros_like(B), A, 2.0, V, M, act)[1])
