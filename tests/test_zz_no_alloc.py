"""vnm_spmm_noalloc (the entry point for callers that cannot allocate) against vnm_spmm through the C
ABI: same kernels, the workspace replaced by the scratch array inside the library.  Two calls in a
row on the same GPU, the second with a smaller input, so that whatever the first call left in the
shared array is still there when the second one runs."""

import numpy as np
import pytest
import torch

import paper_2410_16135_amd as vnm
import synth_inputs as syn
from oracle import vnm_oracle as orc

pytestmark = pytest.mark.gpu
TOL = 1e-2
DEV = "cuda:0"


def _dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def _pair(out, inn, V, M, T, seed, y_dtype):
    W, X = syn.make_weight_and_input(out, inn, T, seed=seed)
    Wd, Xd = _dev(W), _dev(X)
    c = vnm.vnm_prune_compress(Wd, V, M, want_mask=True)
    Y_ref = vnm.vnm_spmm(Xd, c, out_dtype=y_dtype)
    Y = torch.full((T, out), float("nan"), dtype=y_dtype, device=DEV)
    before = torch.cuda.memory_allocated()
    vnm.vnm_spmm_noalloc(Xd, c, Y)
    assert torch.cuda.memory_allocated() == before                 # torch's allocator was not asked for anything
    torch.cuda.synchronize()
    Wm = orc.masked_dense(W, c.mask.cpu().numpy())
    oracle = orc.matmul_ref(X, Wm)
    got, ref = Y.cpu().numpy(), Y_ref.cpu().numpy()
    assert np.isfinite(got).all()
    assert orc.max_normalised_error(got, oracle) <= TOL
    # against the existing entry point: both within the tolerance of the oracle and of each other (the
    # built-in scratch may leave less room for split-K partials than a full workspace, which changes
    # the order of the fp32 additions, not the result beyond rounding)
    assert orc.max_normalised_error(got.astype(np.float64), ref.astype(np.float64)) <= TOL
    return got, ref


@pytest.mark.parametrize("y_dtype", [torch.float16, torch.float32])
def test_noalloc_matches_vnm_spmm_two_calls_in_a_row(y_dtype):
    # staged path with K split over workgroups (300 tokens), then a smaller input on the same array
    _pair(256, 640, 64, 5, 300, seed=11, y_dtype=y_dtype)
    _pair(128, 320, 64, 5, 40, seed=12, y_dtype=y_dtype)
    # few tokens (single kernel; the array serves as split-K scratch only), then larger again
    _pair(192, 2048, 32, 8, 16, seed=13, y_dtype=y_dtype)
    _pair(256, 640, 128, 6, 1000, seed=14, y_dtype=y_dtype)


def test_noalloc_token_groups_of_the_few_token_kernel():
    # 33 to 256 tokens served by the few-token kernel in token groups (no staging; the array holds split-K
    # partial products at most), unsplit and with K split, then a smaller input
    _pair(2048, 2048, 64, 5, 100, seed=17, y_dtype=torch.float16)
    _pair(1024, 11008, 64, 5, 24, seed=18, y_dtype=torch.float32)
    _pair(512, 2048, 32, 6, 7, seed=19, y_dtype=torch.float16)


def test_noalloc_bit_equal_where_the_split_is_the_same():
    # above 2048 tokens nothing is split: the two entry points run the same kernels on the same data
    got, ref = _pair(128, 256, 64, 8, 2500, seed=15, y_dtype=torch.float16)
    assert np.array_equal(got.view(np.uint16), ref.view(np.uint16))


def test_noalloc_rejects_what_does_not_fit():
    W, X = syn.make_weight_and_input(64, 4096, 4200, seed=16)          # staged activations of about 45 MB
    c = vnm.vnm_prune_compress(_dev(W), 64, 5)
    Xd = _dev(X)
    Y = torch.empty((4200, 64), dtype=torch.float16, device=DEV)
    with pytest.raises(vnm.VnmError) as e:
        vnm.vnm_spmm_noalloc(Xd, c, Y)
    assert e.value.status == 5 and "built-in scratch" in str(e.value)
    # the generic kernel needs no scratch and still runs
    vnm.vnm_spmm_noalloc(Xd[:64], c, Y[:64], path=vnm.PATH_GENERIC)
    torch.cuda.synchronize()
