"""GPU parity of the single-kernel product that turns its slice of X around into LDS itself (no
staging pass): whole K range in LDS (short K, any token count) and K streaming through LDS in chunks
(few output channels, many tokens), through vnm_spmm / vnm_spmm_fused, against the CPU oracle."""

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


def _choice(T, c):
    return vnm.vnm_spmm_kernel_choice(T, c, vnm.vnm_spmm_workspace_bytes(T, c))


ROW_MODE = [
    # out, in, T, V, M: more than 256 tokens and a K range that fits LDS (8 M rows of 184 bytes per K step)
    (384, 384, 1000, 64, 5), (1152, 384, 700, 64, 5), (200, 768, 333, 64, 8), (130, 256, 257, 32, 6),
    (520, 400, 4100, 128, 7), (64, 640, 300, 64, 16), (1000, 96, 520, 32, 4),
]
CHUNKED = [
    # out, in, T, V, M: at most 1024 output channels, at least 8192 tokens, a K range beyond LDS, M <= 8:
    # one or two held row blocks per wave, ragged last chunk, ragged token tile, both table layouts
    (384, 1536, 8200, 64, 5), (768, 3072, 8193, 64, 8), (1000, 2048, 9000, 32, 6), (200, 4096, 8300, 128, 7),
    (520, 1000, 8256, 64, 4),
]
SHORT_T = [
    # 33 to 256 tokens with short K: still the whole-K form (several row parts fill the chip)
    (4096, 640, 64, 64, 5), (11008, 384, 192, 64, 8), (64, 64, 40, 64, 4), (8320, 512, 77, 128, 6),
]


@pytest.mark.parametrize("out,inn,T,V,M", ROW_MODE + CHUNKED + SHORT_T)
@pytest.mark.parametrize("ydt", [torch.float16, torch.float32])
def test_resident_kernel_matches_oracle(out, inn, T, V, M, ydt):
    rng = np.random.default_rng(out + 3 * inn + 7 * T + V + M)
    W = (rng.standard_normal((out, inn)) * 0.02).astype(np.float16)
    X = rng.standard_normal((T, inn)).astype(np.float16)
    c = vnm.vnm_prune_compress(_dev(W), V, M, want_mask=True)
    assert _choice(T, c) == vnm.KERNEL_RESIDENT
    Y = vnm.vnm_spmm(_dev(X), c, out_dtype=ydt, path=vnm.PATH_SMFMAC)
    torch.cuda.synchronize()
    Y_ref = orc.matmul_ref(X, orc.masked_dense(W, c.mask.cpu().numpy()))
    assert Y.shape == (T, out)
    assert orc.max_normalised_error(Y.float().cpu().numpy(), Y_ref) <= TOL


@pytest.mark.parametrize("out,inn,T,V,M", [(384, 384, 300, 64, 5), (130, 256, 600, 32, 6), (384, 1536, 8200, 64, 5),
                                         (1000, 2048, 8200, 32, 6), (4096, 640, 64, 64, 5), (192, 512, 200, 128, 8)])
def test_resident_kernel_small_integers_exact(out, inn, T, V, M):
    """Integer-valued operands: every partial sum is exact, so the result equals the oracle exactly
    whatever the split of K over waves and workgroups -- a zero-tolerance check of the indexing."""
    W, X = syn.small_integer_case(out, inn, T, seed=out + T, lo=-2, hi=2)
    c = vnm.vnm_prune_compress(_dev(W), V, M, want_mask=True)
    assert _choice(T, c) == vnm.KERNEL_RESIDENT
    Y = vnm.vnm_spmm(_dev(X), c, out_dtype=torch.float32, path=vnm.PATH_SMFMAC)
    torch.cuda.synchronize()
    Y_ref = orc.matmul_ref(X, orc.masked_dense(W, c.mask.cpu().numpy()))
    assert np.array_equal(Y.cpu().numpy().astype(np.float64), Y_ref)


def test_resident_kernel_strided_unaligned_and_fused():
    """Leading dimensions above the widths, a Y that rules out vector stores, pad columns behind X
    that hold NaN, and the fused epilogue (bias, output permutation) in both forms."""
    rng = np.random.default_rng(6)
    for (out, inn, T, V, M) in [(200, 384, 300, 64, 5), (200, 2048, 8200, 64, 5)]:
        W = (rng.standard_normal((out, inn)) * 0.02).astype(np.float16)
        Xfull = np.full((T, inn + 24), np.nan, dtype=np.float16)
        Xfull[:, :inn] = rng.standard_normal((T, inn)).astype(np.float16)
        c = vnm.vnm_prune_compress(_dev(W), V, M, want_mask=True)
        Wm = orc.masked_dense(W, c.mask.cpu().numpy())
        Xd = _dev(Xfull)[:, :inn]
        Ybig = torch.zeros((T, out + 3), dtype=torch.float16, device=DEV)
        vnm.vnm_spmm(Xd, c, Y=Ybig[:, 1:out + 1], path=vnm.PATH_SMFMAC)
        torch.cuda.synchronize()
        Y_ref = orc.matmul_ref(Xfull[:, :inn], Wm)
        assert orc.max_normalised_error(Ybig[:, 1:out + 1].float().cpu().numpy(), Y_ref) <= TOL
        assert torch.all(Ybig[:, 0] == 0) and torch.all(Ybig[:, out + 1:] == 0)       # nothing written outside Y
        bias = rng.standard_normal(out).astype(np.float16)
        po = rng.permutation(out).astype(np.int32)
        Yf = vnm.vnm_spmm_fused(Xd, c, bias=_dev(bias), perm_out=_dev(po), out_dtype=torch.float32)
        torch.cuda.synchronize()
        ref = orc.linear_fused_ref(Xfull[:, :inn], Wm, bias, None, po)
        assert orc.max_normalised_error(Yf.cpu().numpy(), ref) <= TOL
