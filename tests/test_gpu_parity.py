"""GPU parity: every call of the hot path through the C ABI against the CPU oracle, element by
element.  Masks, column indices, positions and kept values must be bit-exact; the product must stay
within 1e-2 of the fp64 oracle, normalised by max |Y_ref| (fp16 operands, fp32 accumulation)."""

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


def _check_compressed(c, W, V, M, with_mask=True):
    values, meta, colidx, mask = orc.compress(W, V, M)
    assert np.array_equal(c.colidx.cpu().numpy(), colidx.reshape(-1)), "colidx"
    assert np.array_equal(c.meta.cpu().numpy(), meta.reshape(-1)), "meta"
    assert np.array_equal(c.values.cpu().numpy().view(np.uint16), values.reshape(-1).view(np.uint16)), "values"
    if with_mask:
        assert np.array_equal(c.mask.cpu().numpy(), mask), "mask"
    return values, meta, colidx, mask


def _rand_w(rng, out, inn, kind):
    if kind == "normal":
        return (rng.standard_normal((out, inn)) * 0.02).astype(np.float16)
    if kind == "ints":
        return rng.integers(-2, 3, size=(out, inn)).astype(np.float16)
    if kind == "wide":           # subnormals up to large values, signed zeros
        W = (rng.standard_normal((out, inn)) * 10.0 ** rng.integers(-7, 4, size=(out, inn))).astype(np.float16)
        W[rng.random(W.shape) < 0.05] = np.float16(-0.0)
        return W
    raise ValueError(kind)


PRUNE_CASES = [
    # out, in, V, M
    (128, 128, 64, 8), (64, 40, 16, 5), (200, 333, 32, 5), (130, 77, 64, 7), (256, 96, 128, 6),
    (96, 64, 32, 4), (64, 512, 64, 16), (48, 200, 16, 33), (100, 1030, 32, 5), (64, 510, 64, 255),
]


@pytest.mark.parametrize("out,inn,V,M", PRUNE_CASES)
@pytest.mark.parametrize("kind", ["normal", "ints", "wide"])
def test_prune_compress_bit_exact(out, inn, V, M, kind):
    rng = np.random.default_rng(out * 7 + inn * 3 + V + M)
    W = _rand_w(rng, out, inn, kind)
    c = vnm.vnm_prune_compress(_dev(W), V, M, want_mask=True)
    torch.cuda.synchronize()
    values, meta, colidx, mask = _check_compressed(c, W, V, M)
    # decompress(compress(W)) is the masked dense matrix, bit for bit
    Wd = vnm.vnm_decompress(c).cpu().numpy()
    assert np.array_equal(Wd.view(np.uint16), orc.masked_dense(W, mask).view(np.uint16))


def test_prune_compress_strided_input_and_degenerate_blocks():
    rng = np.random.default_rng(5)
    big = _rand_w(rng, 96, 160, "normal")
    big[:, 10:30] = 0                       # all-zero blocks
    big[32:64, :] = np.float16(0.25)        # all-equal rows
    Wt = _dev(big)[:, :100]                 # leading dimension 160, width 100
    W = big[:, :100].copy()
    c = vnm.vnm_prune_compress(Wt, 32, 5, want_mask=True)
    torch.cuda.synchronize()
    _check_compressed(c, W, 32, 5)


@pytest.mark.parametrize("ldw", [(1 << 23) - 8, 1 << 23])
def test_prune_compress_at_the_row_pitch_limit_of_the_fast_kernel(ldw):
    """The one-pass pruning kernel keeps a thread's byte offset inside its workgroup's rows in 32 bits with the
    row pitch as a 24-bit factor: a pitch just below 2^23 elements still takes it, 2^23 takes the general
    kernels; both give the oracle's bits.  (130 rows: a full 128-row block and a ragged one.)"""
    rng = np.random.default_rng(ldw % 1000)
    out, inn, V, M = 130, 320, 128, 5
    W = _rand_w(rng, out, inn, "normal")
    buf = torch.zeros((out - 1) * ldw + inn, dtype=torch.float16, device="cuda:0")
    Wt = buf.as_strided((out, inn), (ldw, 1))
    Wt.copy_(torch.from_numpy(W))
    c = vnm.vnm_prune_compress(Wt, V, M, want_mask=True)
    torch.cuda.synchronize()
    values, meta, colidx, mask = _check_compressed(c, W, V, M)
    Wd = vnm.vnm_decompress(c).cpu().numpy()
    assert np.array_equal(Wd.view(np.uint16), orc.masked_dense(W, mask).view(np.uint16))


SPMM_CASES = [
    # out, in, T, V, M
    (128, 128, 16, 64, 8), (128, 128, 1, 64, 8), (192, 160, 130, 64, 5), (96, 200, 300, 32, 5),
    (256, 264, 77, 128, 6), (130, 96, 200, 64, 7), (64, 640, 257, 64, 16), (160, 128, 64, 32, 4),
    (100, 72, 50, 32, 9), (384, 384, 520, 64, 5),
]


@pytest.mark.parametrize("out,inn,T,V,M", SPMM_CASES)
@pytest.mark.parametrize("path", [vnm.PATH_GENERIC, vnm.PATH_SMFMAC])
@pytest.mark.parametrize("ydt", [torch.float16, torch.float32])
def test_spmm_matches_oracle(out, inn, T, V, M, path, ydt):
    rng = np.random.default_rng(out + inn + T + V + M)
    W = _rand_w(rng, out, inn, "normal")
    X = rng.standard_normal((T, inn)).astype(np.float16)
    c = vnm.vnm_prune_compress(_dev(W), V, M, want_mask=True)
    Y = vnm.vnm_spmm(_dev(X), c, out_dtype=ydt, path=path)
    torch.cuda.synchronize()
    values, meta, colidx, mask = _check_compressed(c, W, V, M)
    Y_ref = orc.matmul_ref(X, orc.masked_dense(W, mask))
    assert Y.shape == (T, out)
    assert orc.max_normalised_error(Y.float().cpu().numpy(), Y_ref) <= TOL


@pytest.mark.parametrize("path", [vnm.PATH_GENERIC, vnm.PATH_SMFMAC])
@pytest.mark.parametrize("out,inn,T,V,M", [(128, 160, 70, 64, 5), (256, 128, 33, 128, 8), (96, 120, 129, 32, 6)])
def test_spmm_small_integers_exact(out, inn, T, V, M, path):
    """Integer-valued operands: every product and partial sum is exact in fp32, so the result must
    equal the oracle exactly -- a zero-tolerance check of the indexing."""
    W, X = syn.small_integer_case(out, inn, T, seed=out + T)
    c = vnm.vnm_prune_compress(_dev(W), V, M, want_mask=True)
    Y = vnm.vnm_spmm(_dev(X), c, out_dtype=torch.float32, path=path)
    torch.cuda.synchronize()
    _, _, _, mask = _check_compressed(c, W, V, M)
    Y_ref = orc.matmul_ref(X, orc.masked_dense(W, mask))
    assert np.array_equal(Y.cpu().numpy().astype(np.float64), Y_ref)


def test_spmm_one_hot_reads_back_masked_weights():
    rng = np.random.default_rng(3)
    out, inn, V, M = 128, 120, 64, 5
    W = _rand_w(rng, out, inn, "normal")
    X = np.eye(inn, dtype=np.float16)
    c = vnm.vnm_prune_compress(_dev(W), V, M, want_mask=True)
    Y = vnm.vnm_spmm(_dev(X), c, out_dtype=torch.float16, path=vnm.PATH_SMFMAC)
    torch.cuda.synchronize()
    _, _, _, mask = _check_compressed(c, W, V, M)
    Wm = orc.masked_dense(W, mask)
    assert np.array_equal(Y.cpu().numpy().T.view(np.uint16) & 0x7FFF, Wm.view(np.uint16) & 0x7FFF)


def test_spmm_edge_cases():
    rng = np.random.default_rng(9)
    out, inn, V, M = 128, 128, 64, 8
    W = _rand_w(rng, out, inn, "normal")
    c = vnm.vnm_prune_compress(_dev(W), V, M)
    # T == 0: no-op
    Y = vnm.vnm_spmm(torch.empty((0, inn), dtype=torch.float16, device=DEV), c)
    assert Y.shape == (0, out)
    # in not a multiple of 8: AUTO must fall back to the generic kernel; forcing smfmac is refused
    W2 = _rand_w(rng, 64, 100, "normal"); X2 = rng.standard_normal((40, 100)).astype(np.float16)
    c2 = vnm.vnm_prune_compress(_dev(W2), 32, 5, want_mask=True)
    Y2 = vnm.vnm_spmm(_dev(X2), c2, out_dtype=torch.float32)
    torch.cuda.synchronize()
    Y_ref = orc.matmul_ref(X2, orc.masked_dense(W2, c2.mask.cpu().numpy()))
    assert orc.max_normalised_error(Y2.cpu().numpy(), Y_ref) <= TOL
    with pytest.raises(vnm.VnmError):
        vnm.vnm_spmm(_dev(X2), c2, path=vnm.PATH_SMFMAC)
    # strided X and Y (leading dimensions above the widths)
    Xbig = _dev(rng.standard_normal((50, 256)).astype(np.float16))
    Xv = Xbig[:, :inn]
    Ybig = torch.zeros((50, 200), dtype=torch.float16, device=DEV)
    vnm.vnm_spmm(Xv, c, Y=Ybig[:, :out], path=vnm.PATH_SMFMAC)
    torch.cuda.synchronize()
    values, meta, colidx, mask = orc.compress(W, V, M)
    Y_ref = orc.matmul_ref(Xv.cpu().numpy(), orc.masked_dense(W, mask))
    assert orc.max_normalised_error(Ybig[:, :out].float().cpu().numpy(), Y_ref) <= TOL
    assert torch.all(Ybig[:, out:] == 0)                         # nothing written outside Y
    # pack from a stored canonical triple gives the same product
    c3 = vnm.Compressed(c.values, c.meta, c.colidx, None, out, inn, V, M)
    vnm.vnm_pack(c3)
    Y3 = vnm.vnm_spmm(Xv, c3, path=vnm.PATH_SMFMAC)
    torch.cuda.synchronize()
    assert torch.equal(Y3, Ybig[:, :out])


def test_stage_once_multiply_many():
    """vnm_stage_x + vnm_spmm_staged equal vnm_spmm (bit for bit where vnm_spmm runs the same two
    kernels), and one staging serves several layers that share their input (as q/k/v or gate/up do)."""
    rng = np.random.default_rng(21)
    inn, T, V, M = 320, 300, 64, 5
    X = rng.standard_normal((T, inn)).astype(np.float16)
    Xd = _dev(X)
    staged = vnm.vnm_stage_x(Xd, M)
    for out in (128, 192):
        W = _rand_w(rng, out, inn, "normal")
        c = vnm.vnm_prune_compress(_dev(W), V, M, want_mask=True)
        Y1 = vnm.vnm_spmm_staged(staged, T, c, out_dtype=torch.float32)
        Y2 = vnm.vnm_spmm(Xd, c, out_dtype=torch.float32, path=vnm.PATH_SMFMAC)
        torch.cuda.synchronize()
        if vnm.vnm_spmm_kernel_choice(T, c, vnm.vnm_spmm_workspace_bytes(T, c)) == vnm.KERNEL_STAGED:
            assert torch.equal(Y1, Y2)                       # the same two kernels
        else:                                                # vnm_spmm took the single-kernel path: same values up to rounding
            assert orc.max_normalised_error(Y2.cpu().numpy(), Y1.cpu().numpy().astype(np.float64)) <= 1e-5
        Y_ref = orc.matmul_ref(X, orc.masked_dense(W, c.mask.cpu().numpy()))
        assert orc.max_normalised_error(Y1.cpu().numpy(), Y_ref) <= TOL


SPLITK_CASES = [
    # out, in, T, V, M: few tokens, enough K steps (in / 8M) for the product to be split along K
    (1024, 4096, 16, 64, 5), (960, 2048, 1, 64, 8), (512, 3000, 40, 128, 6), (640, 5120, 130, 64, 16),
    (1000, 4104, 7, 64, 5),
    # more than 256 tokens on matrices with few row groups: split while the grid would leave most CUs idle
    (1024, 4096, 300, 64, 5), (2048, 8192, 700, 64, 8), (4096, 8000, 1000, 64, 5),
]


@pytest.mark.parametrize("out,inn,T,V,M", SPLITK_CASES)
@pytest.mark.parametrize("ydt", [torch.float16, torch.float32])
def test_spmm_few_tokens_split_k(out, inn, T, V, M, ydt):
    """Few tokens: K is split over workgroups and the fp32 partial products are summed by a second
    kernel.  Checked against the oracle, and -- with integer-valued operands, where every order of
    summation is exact -- bit for bit against the same call without scratch (no split)."""
    rng = np.random.default_rng(out + inn + T)
    W = _rand_w(rng, out, inn, "normal")
    X = rng.standard_normal((T, inn)).astype(np.float16)
    c = vnm.vnm_prune_compress(_dev(W), V, M, want_mask=True)
    assert vnm.vnm_spmm_scratch_bytes(T, out) > 0
    Y = vnm.vnm_spmm(_dev(X), c, out_dtype=ydt, path=vnm.PATH_SMFMAC)
    torch.cuda.synchronize()
    Y_ref = orc.matmul_ref(X, orc.masked_dense(W, c.mask.cpu().numpy()))
    assert orc.max_normalised_error(Y.float().cpu().numpy(), Y_ref) <= TOL
    Wi, Xi = syn.small_integer_case(out, inn, T, seed=T + M, lo=-2, hi=2)
    ci = vnm.vnm_prune_compress(_dev(Wi), V, M, want_mask=True)
    staged = vnm.vnm_stage_x(_dev(Xi), M)
    Ya = vnm.vnm_spmm_staged(staged, T, ci, out_dtype=torch.float32)                      # default scratch: split
    none = torch.empty(0, dtype=torch.uint8, device=DEV)
    Yb = vnm.vnm_spmm_staged(staged, T, ci, out_dtype=torch.float32, scratch=none)        # no scratch: one pass
    torch.cuda.synchronize()
    assert torch.equal(Ya, Yb)
    Yi_ref = orc.matmul_ref(Xi, orc.masked_dense(Wi, ci.mask.cpu().numpy()))
    assert np.array_equal(Ya.cpu().numpy().astype(np.float64), Yi_ref)


RESIDENT_X_CASES = [
    # out, in, T, V, M: at most 16 tokens and at least 32 K steps (in / 8M) per workgroup -- the few-token kernel
    # that keeps the workgroup's slice of X in LDS: unsplit (more than 128 row blocks), with two column tables
    # (V = 32), with 128-row blocks, and with K split over 4 and over 16 workgroups
    (8256, 2048, 16, 64, 5), (8256, 2080, 9, 32, 6), (8320, 4104, 13, 128, 8), (4096, 11008, 16, 64, 5),
    (640, 20480, 1, 64, 5),
    # at most 128 row blocks, K unsplit: one workgroup per 32-row tile -- one column table, two tables (V = 32),
    # 128-row blocks, and V = 32 with an odd number of 32-row blocks (the last 64-row block has one real tile)
    (4096, 4096, 16, 64, 5), (4096, 2080, 9, 32, 6), (2048, 4104, 13, 128, 8), (2080, 2048, 7, 32, 5),
    # 17 to 32 tokens on at most 64 row blocks: the same kernel, two groups of 16 tokens per row block (a full and
    # a ragged second group, two column tables, 128-row blocks, and K split over workgroups as well)
    (4096, 4096, 32, 64, 5), (4096, 2080, 17, 32, 6), (2048, 4104, 25, 128, 8), (2080, 2048, 31, 32, 5),
    (1024, 11008, 20, 64, 5),
    # 33 to 64 tokens while (row blocks x groups of 16 tokens) still fit the compute units at once
    (4096, 4096, 33, 64, 5), (4096, 4096, 64, 64, 5), (2080, 2048, 50, 32, 5), (2048, 4104, 64, 128, 8), (5000, 2048, 40, 64, 8),
    # two row blocks per workgroup: more row blocks than fit one by one (even and odd count, two column tables),
    # a slice of X that needs K split (4096 x 11008), and three token groups
    (11008, 2048, 20, 64, 5), (8384, 2048, 32, 64, 5), (8352, 2080, 25, 32, 6), (4096, 11008, 32, 64, 5), (6000, 2048, 48, 64, 5),
    # up to 128 tokens (eight groups) on at most 64 row blocks
    (4096, 4096, 128, 64, 5), (4096, 4096, 100, 64, 5), (2080, 2048, 77, 32, 5), (1000, 4104, 128, 128, 8),
    # groups of 32 tokens per workgroup where groups of 16 would not fit the compute units: four row blocks per
    # workgroup with K split in two (192 and 256 tokens on 64 row blocks; 64 tokens on 172 row blocks; two column
    # tables), two row blocks unsplit, and many groups of 16 on very few row blocks
    (4096, 4096, 192, 64, 5), (4096, 4096, 256, 64, 5), (11008, 4096, 64, 64, 5), (4160, 4096, 200, 32, 6),
    (4096, 2048, 200, 64, 5), (1024, 2048, 250, 64, 5),
]


@pytest.mark.parametrize("out,inn,T,V,M", RESIDENT_X_CASES)
@pytest.mark.parametrize("ydt", [torch.float16, torch.float32])
def test_spmm_up_to_16_tokens_x_resident_in_lds(out, inn, T, V, M, ydt):
    """The few-token kernel with X resident in LDS and a ring of weight operands in flight (up to 16 tokens per
    workgroup, up to 32 per call), against the oracle; with integer-valued operands bit for bit against the
    general kernel."""
    rng = np.random.default_rng(out + inn + T)
    W = _rand_w(rng, out, inn, "normal")
    X = rng.standard_normal((T, inn)).astype(np.float16)
    c = vnm.vnm_prune_compress(_dev(W), V, M, want_mask=True)
    Y = vnm.vnm_spmm(_dev(X), c, out_dtype=ydt, path=vnm.PATH_SMFMAC)
    torch.cuda.synchronize()
    Y_ref = orc.matmul_ref(X, orc.masked_dense(W, c.mask.cpu().numpy()))
    assert orc.max_normalised_error(Y.float().cpu().numpy(), Y_ref) <= TOL
    Wi, Xi = syn.small_integer_case(out, inn, T, seed=T + M, lo=-2, hi=2)
    ci = vnm.vnm_prune_compress(_dev(Wi), V, M, want_mask=True)
    Ya = vnm.vnm_spmm(_dev(Xi), ci, out_dtype=torch.float32, path=vnm.PATH_SMFMAC)
    Yb = vnm.vnm_spmm(_dev(Xi), ci, out_dtype=torch.float32, path=vnm.PATH_GENERIC)
    torch.cuda.synchronize()
    assert torch.equal(Ya, Yb)
    Yi_ref = orc.matmul_ref(Xi, orc.masked_dense(Wi, ci.mask.cpu().numpy()))
    assert np.array_equal(Ya.cpu().numpy().astype(np.float64), Yi_ref)


VECTOR_ALU_CASES = [
    # out, in, T, V, M: one to four tokens -- the product on the vector ALUs (no matrix instructions): every token
    # count, one and two column tables (V = 32), 128-row blocks, M from 4 to 16, `in` ragged against M, `out`
    # ragged against the 32-row tile, a single K step, fewer K steps than waves, more K steps than one ring of
    # weights per wave (two rounds of loads), rows of X longer than one 16-byte piece per thread
    (4096, 4096, 1, 64, 5), (4096, 4096, 2, 64, 5), (4096, 4096, 3, 64, 5), (4096, 4096, 4, 64, 5),
    (2080, 2048, 3, 32, 5), (1000, 4104, 4, 128, 8), (70, 40, 1, 64, 5), (33, 8, 2, 32, 4), (640, 20480, 1, 64, 5),
    (1024, 11008, 4, 64, 5), (300, 16384, 2, 32, 16), (257, 2048, 4, 64, 7), (96, 1280, 3, 64, 16),
    # more 32-row tiles than compute units (workgroups of 8 waves; with three tokens the matrix-core kernel
    # takes over); a long K on few tiles at one token
    (8320, 1288, 2, 64, 5), (8320, 1288, 3, 64, 5), (11008, 4096, 1, 64, 5), (512, 11008, 1, 128, 5),
]


@pytest.mark.parametrize("out,inn,T,V,M", VECTOR_ALU_CASES)
@pytest.mark.parametrize("ydt", [torch.float16, torch.float32])
def test_spmm_up_to_4_tokens_on_the_vector_alus(out, inn, T, V, M, ydt):
    """The kernel for one to four tokens (the packed weight streamed through the vector ALUs), against the
    oracle; with integer-valued operands exact, and bit for bit equal to the general kernel."""
    rng = np.random.default_rng(out + inn + T)
    W = _rand_w(rng, out, inn, "normal")
    X = rng.standard_normal((T, inn)).astype(np.float16)
    c = vnm.vnm_prune_compress(_dev(W), V, M, want_mask=True)
    Y = vnm.vnm_spmm(_dev(X), c, out_dtype=ydt, path=vnm.PATH_SMFMAC)
    torch.cuda.synchronize()
    Y_ref = orc.matmul_ref(X, orc.masked_dense(W, c.mask.cpu().numpy()))
    assert orc.max_normalised_error(Y.float().cpu().numpy(), Y_ref) <= TOL
    Wi, Xi = syn.small_integer_case(out, inn, T, seed=T + M, lo=-2, hi=2)
    ci = vnm.vnm_prune_compress(_dev(Wi), V, M, want_mask=True)
    Ya = vnm.vnm_spmm(_dev(Xi), ci, out_dtype=torch.float32, path=vnm.PATH_SMFMAC)
    Yb = vnm.vnm_spmm(_dev(Xi), ci, out_dtype=torch.float32, path=vnm.PATH_GENERIC)
    torch.cuda.synchronize()
    assert torch.equal(Ya, Yb)
    Yi_ref = orc.matmul_ref(Xi, orc.masked_dense(Wi, ci.mask.cpu().numpy()))
    assert np.array_equal(Ya.cpu().numpy().astype(np.float64), Yi_ref)


def test_spmm_up_to_4_tokens_ignores_what_lies_behind_x():
    """Rows of X beyond T and the columns between `in` and the row pitch hold NaN: none of it may reach Y."""
    out, inn, T, V, M = 320, 1288, 3, 64, 5
    rng = np.random.default_rng(5)
    W = _rand_w(rng, out, inn, "normal")
    X = rng.standard_normal((T, inn)).astype(np.float16)
    big = torch.full((T + 5, inn + 24), float("nan"), dtype=torch.float16, device=DEV)
    big[:T, :inn] = _dev(X)
    c = vnm.vnm_prune_compress(_dev(W), V, M, want_mask=True)
    Y = vnm.vnm_spmm(big[:T, :inn], c, out_dtype=torch.float32, path=vnm.PATH_SMFMAC)
    torch.cuda.synchronize()
    Y_ref = orc.matmul_ref(X, orc.masked_dense(W, c.mask.cpu().numpy()))
    assert orc.max_normalised_error(Y.cpu().numpy(), Y_ref) <= TOL


def test_spmm_bound_call_equals_the_plain_call():
    """vnm_spmm_bind marshals the arguments once; the call it returns must do what vnm_spmm does (few tokens, the
    single-kernel path for short K, and the staged path), also when called repeatedly."""
    for (out, inn, T, V, M) in [(1024, 2048, 1, 64, 5), (1024, 2048, 16, 64, 5), (384, 384, 200, 64, 5), (512, 4096, 300, 64, 5)]:
        rng = np.random.default_rng(out + T)
        W = _rand_w(rng, out, inn, "normal")
        X = _dev(rng.standard_normal((T, inn)).astype(np.float16))
        c = vnm.vnm_prune_compress(_dev(W), V, M)
        ws = torch.empty(max(vnm.vnm_spmm_workspace_bytes(T, c), 256), dtype=torch.uint8, device=DEV)
        Y_ref = vnm.vnm_spmm(X, c, workspace=ws)
        Y = torch.zeros_like(Y_ref)
        call = vnm.vnm_spmm_bind(X, c, Y, ws)
        for _ in range(3):
            Y.zero_()
            assert call() is Y
            torch.cuda.synchronize()
            assert torch.equal(Y, Y_ref)


def _random_few_token_cases(n, seed):
    rng = np.random.default_rng(seed)
    cases = []
    for _ in range(n):
        V = int(rng.choice([32, 64, 128])); M = int(rng.choice([4, 5, 6, 7, 8, 11, 16]))
        S = int(rng.choice([32, 33, 57, 103, 129, 140, 276]))
        inn = S * 8 * M - 8 * int(rng.integers(0, M))
        budget = 6_000_000 // inn
        out = int(rng.integers(1, budget + 1)) if rng.random() < 0.7 else int(min(budget, rng.integers(129, 140) * 64))
        cases.append((max(out, 1), inn, int(rng.integers(1, 17)), V, M))
    return cases


@pytest.mark.parametrize("out,inn,T,V,M", _random_few_token_cases(16, 2024))
def test_random_few_token_shapes(out, inn, T, V, M):
    """Seeded random shapes with at most 16 tokens and at least 32 K steps (ragged `in`, one to many
    row blocks, all block heights): integer-valued operands, so the product is exact in any order."""
    Wi, Xi = syn.small_integer_case(out, inn, T, seed=out + inn + T, lo=-2, hi=2)
    c = vnm.vnm_prune_compress(_dev(Wi), V, M, want_mask=True)
    Y_ref = orc.matmul_ref(Xi, orc.masked_dense(Wi, c.mask.cpu().numpy()))
    for ydt in (torch.float32, torch.float16):
        Y = vnm.vnm_spmm(_dev(Xi), c, out_dtype=ydt, path=vnm.PATH_SMFMAC)
        torch.cuda.synchronize()
        if ydt == torch.float32:
            assert np.array_equal(Y.cpu().numpy().astype(np.float64), Y_ref)
        else:
            assert orc.max_normalised_error(Y.float().cpu().numpy(), Y_ref) <= TOL


def test_spmm_pad_columns_are_never_read():
    """in = 72 at M = 5 pads to 75: the pad columns must count as zero even when the memory right
    after each X row holds NaN."""
    rng = np.random.default_rng(4)
    out, inn, T, V, M = 64, 72, 40, 32, 5
    W = _rand_w(rng, out, inn, "normal")
    Xfull = np.full((T, 80), np.nan, dtype=np.float16)
    Xfull[:, :inn] = rng.standard_normal((T, inn)).astype(np.float16)
    c = vnm.vnm_prune_compress(_dev(W), V, M, want_mask=True)
    Xd = _dev(Xfull)[:, :inn]
    for path in (vnm.PATH_GENERIC, vnm.PATH_SMFMAC):
        Y = vnm.vnm_spmm(Xd, c, out_dtype=torch.float32, path=path)
        torch.cuda.synchronize()
        Y_ref = orc.matmul_ref(Xfull[:, :inn], orc.masked_dense(W, c.mask.cpu().numpy()))
        assert orc.max_normalised_error(Y.cpu().numpy(), Y_ref) <= TOL


def test_config0_single_gemm():
    (layer,) = syn.config_single_gemm()
    W, X = syn.layer_tensors(layer)
    c = vnm.vnm_prune_compress(_dev(W), layer.V, layer.M, want_mask=True)
    Y = vnm.vnm_spmm(_dev(X), c, out_dtype=torch.float32)
    torch.cuda.synchronize()
    _, _, _, mask = _check_compressed(c, W, layer.V, layer.M)
    assert orc.max_normalised_error(Y.cpu().numpy(), orc.matmul_ref(X, orc.masked_dense(W, mask))) <= TOL


@pytest.mark.parametrize("cfg", ["deit_small", "deit_base"])
def test_deit_shaped_layers_full(cfg):
    layers = syn.config_deit_small() if cfg == "deit_small" else syn.config_deit_base()
    for layer in layers:
        W, X = syn.layer_tensors(layer)
        c = vnm.vnm_prune_compress(_dev(W), layer.V, layer.M, want_mask=True)
        Y = vnm.vnm_spmm(_dev(X), c, path=vnm.PATH_SMFMAC)
        Wd = vnm.vnm_decompress(c)
        torch.cuda.synchronize()
        _, _, _, mask = _check_compressed(c, W, layer.V, layer.M)
        Wm = orc.masked_dense(W, mask)
        # (small matrices: pruning and decompression run with spans of one or two K steps here)
        assert np.array_equal(Wd.cpu().numpy().view(np.uint16), Wm.view(np.uint16)), layer.name
        Y_ref = orc.matmul_ref(X, Wm)
        err = orc.max_normalised_error(Y.float().cpu().numpy(), Y_ref)
        assert err <= TOL, (layer.name, err)


@pytest.mark.parametrize("which", [0, 4, 6])
def test_llama_shaped_layers_sampled_tokens(which):
    """Full-size Llama-2-7B-shaped layers in the benchmark's launch configuration (T = 4096);
    the oracle product is computed for 256 sampled tokens over all output channels."""
    layer = syn.config_llama2_7b()[which]
    W, X = syn.layer_tensors(layer)
    c = vnm.vnm_prune_compress(_dev(W), layer.V, layer.M, want_mask=True)
    Y = vnm.vnm_spmm(_dev(X), c, path=vnm.PATH_SMFMAC)
    Wd = vnm.vnm_decompress(c)
    torch.cuda.synchronize()
    _, _, _, mask = _check_compressed(c, W, layer.V, layer.M)
    Wm = orc.masked_dense(W, mask)
    assert np.array_equal(Wd.cpu().numpy().view(np.uint16), Wm.view(np.uint16))
    rng = np.random.default_rng(99)
    tok = np.sort(rng.choice(layer.tokens, size=256, replace=False))
    tok[0], tok[-1] = 0, layer.tokens - 1
    Y_ref = orc.matmul_ref(X[tok], Wm)
    err = orc.max_normalised_error(Y[torch.from_numpy(tok).to(DEV)].float().cpu().numpy(), Y_ref)
    assert err <= TOL, err


SWEEP_POINTS = [
    # (layer index in the sweep's two shapes: 0 = 11008 x 4096, 1 = 4096 x 11008), V, M, tokens
    (0, 128, 16, 4096), (1, 32, 8, 4096), (0, 64, 7, 16), (1, 128, 5, 16), (1, 64, 4, 1),
]


@pytest.mark.parametrize("shape,V,M,T", SWEEP_POINTS)
def test_sweep_points_full_size(shape, V, M, T):
    """Points of the V x M x tokens sweep at full layer size: 128-row patterns (stored as 64-row
    blocks in the matrix-core copy), 32-row patterns, and the few-token kernel with and without
    split K.  Compression is checked bit for bit, the product on up to 128 sampled tokens."""
    name = ("gate", "down")[shape]
    layer = next(L for L in syn.config_sweep() if L.name == f"{name}_V{V}_M{M}_T{max(T, 16)}")
    W, X = syn.layer_tensors(layer, tokens=T)
    c = vnm.vnm_prune_compress(_dev(W), V, M, want_mask=True)
    Y = vnm.vnm_spmm(_dev(X), c, path=vnm.PATH_SMFMAC)
    torch.cuda.synchronize()
    _, _, _, mask = _check_compressed(c, W, V, M)
    Wm = orc.masked_dense(W, mask)
    rng = np.random.default_rng(7)
    tok = np.sort(rng.choice(T, size=min(T, 128), replace=False))
    tok[0], tok[-1] = 0, T - 1
    Y_ref = orc.matmul_ref(X[tok], Wm)
    err = orc.max_normalised_error(Y[torch.from_numpy(tok).to(DEV)].float().cpu().numpy(), Y_ref)
    assert err <= TOL, err


# ------------------------------------------------------- scored pruning and RIA (Section 3, Eq. 1)

def _check_compressed_scored(c, W, S, V, M):
    values, meta, colidx, mask = orc.compress(W, V, M, score=S)
    assert np.array_equal(c.colidx.cpu().numpy(), colidx.reshape(-1)), "colidx"
    assert np.array_equal(c.meta.cpu().numpy(), meta.reshape(-1)), "meta"
    assert np.array_equal(c.values.cpu().numpy().view(np.uint16), values.reshape(-1).view(np.uint16)), "values"
    assert np.array_equal(c.mask.cpu().numpy(), mask), "mask"
    return mask


@pytest.mark.parametrize("out,inn", [(128, 128), (70, 333), (200, 77), (1, 8), (257, 1030)])
@pytest.mark.parametrize("kind", ["normal", "wide", "ints"])
def test_ria_scores_bit_exact(out, inn, kind):
    rng = np.random.default_rng(out * 3 + inn)
    W = _rand_w(rng, out, inn, kind)
    if kind == "ints":
        W[:, inn // 2] = 0          # a zero column and a zero row: their terms count as zero
        W[out // 2, :] = 0
    act = (rng.random(inn) * 4.0 + 0.01).astype(np.float32)
    S = vnm.vnm_ria_scores(_dev(W), _dev(act))
    torch.cuda.synchronize()
    S_ref = orc.importance_ria(W, act)
    assert np.array_equal(S.cpu().numpy().view(np.uint32), S_ref.view(np.uint32))


@pytest.mark.parametrize("out,inn,V,M", [(128, 128, 64, 8), (64, 40, 16, 5), (200, 333, 32, 5), (130, 77, 64, 7),
                                         (256, 96, 128, 6), (48, 200, 16, 33)])
@pytest.mark.parametrize("score", ["ria", "foreign", "ties", "order"])
def test_prune_compress_scored_bit_exact(out, inn, V, M, score):
    rng = np.random.default_rng(out + inn * 5 + V + M)
    W = _rand_w(rng, out, inn, "normal")
    if score == "ria":
        S = orc.importance_ria(W, (rng.random(inn) * 2.0 + 0.1).astype(np.float32))
    elif score == "foreign":     # unrelated to |w|: a mix-up of W and S cannot pass
        S = rng.random((out, inn)).astype(np.float32)
    elif score == "ties":
        S = rng.integers(0, 3, size=(out, inn)).astype(np.float32)
    else:                        # column sums that depend on the order of addition
        S = (rng.random((out, inn)) * 10.0 ** rng.integers(-3, 12, size=(out, inn))).astype(np.float32)
    c = vnm.vnm_prune_compress_scored(_dev(W), _dev(S), V, M, want_mask=True)
    torch.cuda.synchronize()
    mask = _check_compressed_scored(c, W, S, V, M)
    Wd = vnm.vnm_decompress(c).cpu().numpy()
    assert np.array_equal(Wd.view(np.uint16), orc.masked_dense(W, mask).view(np.uint16))
    if c.packed is not None and inn % 8 == 0:
        X = rng.standard_normal((33, inn)).astype(np.float16)
        Y = vnm.vnm_spmm(_dev(X), c, out_dtype=torch.float32, path=vnm.PATH_SMFMAC)
        Y_ref = orc.matmul_ref(X, orc.masked_dense(W, mask))
        assert orc.max_normalised_error(Y.cpu().numpy(), Y_ref) <= TOL


def test_scored_path_strided_and_abs_equivalence():
    """Row strides larger than the width, and |w| as the score reproduces vnm_prune_compress."""
    rng = np.random.default_rng(8)
    out, inn, V, M = 96, 120, 32, 5
    Wbig = _dev(_rand_w(rng, out, inn + 24, "normal"))
    Sbig = torch.rand((out, inn + 40), device=DEV, dtype=torch.float32)
    Wv, Sv = Wbig[:, :inn], Sbig[:, :inn]
    c = vnm.vnm_prune_compress_scored(Wv, Sv, V, M, want_mask=True)
    torch.cuda.synchronize()
    _check_compressed_scored(c, Wv.cpu().numpy(), Sv.cpu().numpy(), V, M)
    Wn = Wv.cpu().numpy()
    c_abs = vnm.vnm_prune_compress(Wv, V, M, want_mask=True)
    c_s = vnm.vnm_prune_compress_scored(Wv, Wv.abs().float(), V, M, want_mask=True)
    torch.cuda.synchronize()
    for a, b in ((c_abs.values, c_s.values), (c_abs.meta, c_s.meta), (c_abs.colidx, c_s.colidx), (c_abs.mask, c_s.mask)):
        assert torch.equal(a.view(torch.uint8), b.view(torch.uint8))
    _check_compressed(c_abs, Wn, V, M)


def test_ria_prune_llama_shaped_layer_full_size():
    layer = syn.config_llama2_7b()[0]
    W, X = syn.layer_tensors(layer, tokens=64)
    act = np.sqrt((X.astype(np.float64) ** 2).sum(axis=0)).astype(np.float32) ** np.float32(0.5)
    S = vnm.vnm_ria_scores(_dev(W), _dev(act))
    c = vnm.vnm_prune_compress_scored(_dev(W), S, layer.V, layer.M, want_mask=True)
    torch.cuda.synchronize()
    S_ref = orc.importance_ria(W, act)
    assert np.array_equal(S.cpu().numpy().view(np.uint32), S_ref.view(np.uint32))
    _check_compressed_scored(c, W, S_ref, layer.V, layer.M)


@pytest.mark.parametrize("name", ["gate", "down"])
def test_ria_scores_of_the_wide_and_tall_layers_are_exact_and_repeatable(name):
    """11008 x 4096 and 4096 x 11008: more workgroups than compute units in every kernel of the score
    path.  The scores equal the oracle's bit for bit on every call (three calls on the same inputs)."""
    layer = [l for l in syn.config_llama2_7b() if l.name == name][0]
    W, X = syn.layer_tensors(layer, tokens=64)
    act = np.sqrt((X.astype(np.float64) ** 2).sum(axis=0)).astype(np.float32) ** np.float32(0.5)
    S_ref = orc.importance_ria(W, act).view(np.uint32)
    Wd, ad = _dev(W), _dev(act)
    for _ in range(3):
        S = vnm.vnm_ria_scores(Wd, ad)
        torch.cuda.synchronize()
        assert np.array_equal(S.cpu().numpy().view(np.uint32), S_ref)


@pytest.mark.parametrize("out,inn,V,M", [(96, 160, 32, 5), (160, 256, 32, 8), (200, 128, 64, 6), (130, 320, 128, 7),
                                         (32, 64, 32, 4)])
def test_pack_from_triple_equals_fused_copy(out, inn, V, M):
    """vnm_pack on the canonical triple builds the same matrix-core copy as the fused pruning kernel
    (byte for byte, up to the trailing slack that no one writes), for 32-row patterns -- two row
    blocks per 64-row packed block, also with an odd number of them --, 64 and 128; and the product
    from either copy, many-token and few-token kernel, matches the oracle."""
    rng = np.random.default_rng(out + inn + V)
    W = _rand_w(rng, out, inn, "normal")
    c = vnm.vnm_prune_compress(_dev(W), V, M, want_mask=True)
    c2 = vnm.Compressed(c.values, c.meta, c.colidx, None, out, inn, V, M, c.mask)
    vnm.vnm_pack(c2)
    torch.cuda.synchronize()
    # sections of the copy (each starts on a 256-byte boundary; the gaps and the slack are unwritten)
    up = lambda x: (x + 255) // 256 * 256
    Rp, S = (-(-out // V) * V + 63) // 64, -(-(-(-inn // M)) // 8)
    sizes = [Rp * S * 2048, Rp * S * 256, Rp * S * 32 * (2 if V == 32 else 1)]
    off = 0
    for nbytes in sizes:
        assert torch.equal(c.packed[off:off + nbytes], c2.packed[off:off + nbytes])
        off += up(nbytes)
    assert off + 8192 == c.packed.numel()
    Wm = orc.masked_dense(W, c.mask.cpu().numpy())
    for T in (7, 150):
        X = rng.standard_normal((T, inn)).astype(np.float16)
        Y = vnm.vnm_spmm(_dev(X), c2, out_dtype=torch.float32, path=vnm.PATH_SMFMAC)
        torch.cuda.synchronize()
        assert orc.max_normalised_error(Y.cpu().numpy(), orc.matmul_ref(X, Wm)) <= TOL


def _random_cases(n, seed):
    rng = np.random.default_rng(seed)
    cases = []
    for _ in range(n):
        V = int(rng.choice([16, 32, 64, 128]))
        M = int(rng.choice([4, 5, 6, 7, 8, 9, 12, 16, 19]))
        out = int(rng.integers(1, 5) * V + rng.integers(-V + 1, 1)) if rng.random() < 0.5 else int(rng.integers(1, 400))
        inn = int(rng.integers(1, 60)) * 8 if rng.random() < 0.7 else int(rng.integers(4, 500))
        T = int(rng.choice([1, 2, 15, 16, 17, 31, 32, 33, 64, 127, 128, 129, 200, 257, 300]))
        cases.append((max(out, 1), inn, T, V, M))
    return cases


@pytest.mark.parametrize("out,inn,T,V,M", _random_cases(48, 2024))
def test_random_shapes_whole_path(out, inn, T, V, M):
    """Seeded random shapes through the whole path with the default dispatch (whatever kernel the
    library picks: fused or general pruning, few-token, split-K, staged matrix-core or generic
    product), ragged in every dimension, token counts around every internal boundary."""
    rng = np.random.default_rng(out * 131 + inn * 17 + T + V + M)
    W = _rand_w(rng, out, inn, "normal" if (out + inn) % 3 else "ints")
    X = rng.standard_normal((T, inn)).astype(np.float16)
    c = vnm.vnm_prune_compress(_dev(W), V, M, want_mask=True)
    Y = vnm.vnm_spmm(_dev(X), c, out_dtype=torch.float32)
    Yh = vnm.vnm_spmm(_dev(X), c, out_dtype=torch.float16)
    Wd = vnm.vnm_decompress(c)
    torch.cuda.synchronize()
    _, _, _, mask = _check_compressed(c, W, V, M)
    Wm = orc.masked_dense(W, mask)
    assert np.array_equal(Wd.cpu().numpy().view(np.uint16), Wm.view(np.uint16))
    Y_ref = orc.matmul_ref(X, Wm)
    assert orc.max_normalised_error(Y.cpu().numpy(), Y_ref) <= TOL
    assert orc.max_normalised_error(Yh.float().cpu().numpy(), Y_ref) <= TOL


# ---------------------------------------------------------------- sizes beyond single-launch grid limits

@pytest.mark.parametrize("path", [vnm.PATH_GENERIC, vnm.PATH_SMFMAC])
def test_more_tokens_than_one_grid_dimension(path):
    """T = 70 001 (above the 65 535 limit of a grid's y dimension, ragged last token tile) on the
    single-GEMM layer; every output checked."""
    (layer,) = syn.config_single_gemm()
    W, _ = syn.layer_tensors(layer)
    rng = np.random.default_rng(70001)
    X = rng.standard_normal((70001, layer.inn), dtype=np.float32).astype(np.float16)
    c = vnm.vnm_prune_compress(_dev(W), layer.V, layer.M, want_mask=True)
    Y = vnm.vnm_spmm(_dev(X), c, path=path)
    torch.cuda.synchronize()
    Y_ref = orc.matmul_ref(X, orc.masked_dense(W, orc.compress(W, layer.V, layer.M)[3]))
    assert orc.max_normalised_error(Y.cpu().numpy(), Y_ref) <= TOL


@pytest.mark.parametrize("V,M,inn", [(64, 5, 40), (16, 5, 35), (128, 8, 64)])
def test_more_rows_than_one_grid_dimension(V, M, inn):
    """out = 66 048 rows (1 032 ... 4 128 row blocks; the row-wise kernels cross the 65 535 limit)."""
    out = 66048
    rng = np.random.default_rng(V * M)
    W = _rand_w(rng, out, inn, "normal")
    c = vnm.vnm_prune_compress(_dev(W), V, M, want_mask=True)
    torch.cuda.synchronize()
    values, meta, colidx, mask = _check_compressed(c, W, V, M)
    Wd = vnm.vnm_decompress(c).cpu().numpy()
    assert np.array_equal(Wd.view(np.uint16), orc.masked_dense(W, mask).view(np.uint16))
    X = rng.integers(-2, 3, size=(40, inn)).astype(np.float16)
    Wi = rng.integers(-2, 3, size=(out, inn)).astype(np.float16)
    ci = vnm.vnm_prune_compress(_dev(Wi), V, M, want_mask=True)
    Y = vnm.vnm_spmm(_dev(X), ci, out_dtype=torch.float32)
    torch.cuda.synchronize()
    Y_ref = orc.matmul_ref(X, orc.masked_dense(Wi, orc.compress(Wi, V, M)[3]))
    assert np.array_equal(Y.cpu().numpy().astype(np.float64), Y_ref)
