"""GPU parity of vnm_spmm_fused (bias and the channel permutations of Section 4.2, Eq. 6) against the
CPU oracle, on every kernel the call can take: the generic one, the single-kernel path for up to 32
tokens, the staged matrix-core path, and its split-K variant.  Tolerance as for vnm_spmm."""

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


def _layer(out, inn, T, V, M, seed):
    """A channel-permuted layer: original W, permutations, the compressed permuted weight."""
    rng = np.random.default_rng(seed)
    W, X = syn.make_weight_and_input(out, inn, T, seed=seed)
    po = rng.permutation(out).astype(np.int32)
    pi = rng.permutation(inn).astype(np.int32)
    bias = (rng.standard_normal(out) * 0.5).astype(np.float16)     # row order of the permuted weight
    Wp = orc.permute_weight(W, po, pi)
    c = vnm.vnm_prune_compress(_dev(Wp), V, M, want_mask=True)
    Wm_p = orc.masked_dense(Wp, orc.compress(Wp, V, M)[3])
    return X, Wm_p, bias, pi, po, c


FUSED_CASES = [
    # out, in, T, V, M        (T <= 32: single kernel; 33..256 on few row blocks: split K; else staged)
    (128, 128, 16, 64, 8), (192, 160, 7, 64, 5), (96, 200, 32, 32, 5), (256, 264, 20, 128, 6),
    (192, 160, 130, 64, 5), (96, 200, 300, 32, 5), (256, 264, 77, 128, 6), (130, 96, 200, 64, 7),
    (64, 640, 257, 64, 16), (384, 384, 520, 64, 5), (512, 2048, 100, 64, 5), (1024, 1280, 40, 64, 8),
    (130, 96, 300, 64, 7), (2048, 512, 24, 64, 5),
    # at most 16 tokens, X resident in LDS: epilogue in the kernel (unsplit) and in the reduction (split K)
    (8256, 1320, 12, 64, 5), (4096, 5600, 16, 64, 5), (1024, 2048, 24, 64, 5), (512, 5600, 29, 64, 5), (1024, 2048, 47, 64, 5), (8384, 1320, 30, 64, 5), (1024, 2048, 90, 64, 5), (4096, 2048, 200, 64, 5), (4096, 4096, 192, 64, 5),
    # one to four tokens, the product on the vector ALUs: 16 waves per tile, 8 waves (more tiles than compute
    # units), two column tables
    (1024, 1280, 1, 64, 5), (8320, 1320, 2, 64, 5), (352, 2048, 4, 32, 8),
]
WHICH = [("bias",), ("perm_in",), ("perm_out",), ("bias", "perm_in", "perm_out")]


@pytest.mark.parametrize("out,inn,T,V,M", FUSED_CASES)
@pytest.mark.parametrize("which", WHICH, ids=["bias", "pin", "pout", "all"])
@pytest.mark.parametrize("path", [vnm.PATH_GENERIC, vnm.PATH_SMFMAC])
@pytest.mark.parametrize("ydt", [torch.float16, torch.float32])
def test_fused_matches_oracle(out, inn, T, V, M, which, path, ydt):
    X, Wm_p, bias, pi, po, c = _layer(out, inn, T, V, M, seed=out + inn + T + V + M)
    kw = {"bias": _dev(bias) if "bias" in which else None,
          "perm_in": _dev(pi) if "perm_in" in which else None,
          "perm_out": _dev(po) if "perm_out" in which else None}
    Y = vnm.vnm_spmm_fused(_dev(X), c, out_dtype=ydt, path=path, **kw)
    torch.cuda.synchronize()
    Y_ref = orc.linear_fused_ref(X, Wm_p, bias=bias if "bias" in which else None,
                                 perm_in=pi if "perm_in" in which else None,
                                 perm_out=po if "perm_out" in which else None)
    err = orc.max_normalised_error(Y.cpu().numpy(), Y_ref)
    assert err <= TOL, err


@pytest.mark.parametrize("path", [vnm.PATH_GENERIC, vnm.PATH_SMFMAC])
@pytest.mark.parametrize("out,inn,T,V,M", [(128, 160, 70, 64, 5), (256, 128, 33, 128, 8), (96, 120, 129, 32, 6),
                                           (128, 160, 9, 64, 5), (512, 2048, 100, 64, 5)])
def test_fused_small_integers_exact(out, inn, T, V, M, path):
    """Integer-valued operands and bias: every partial sum is exact, so the fp32 result equals the
    oracle's to the bit -- a zero-tolerance check of all three index mappings."""
    rng = np.random.default_rng(out + T)
    Wp = rng.integers(-2, 3, size=(out, inn)).astype(np.float16)
    X = rng.integers(-3, 4, size=(T, inn)).astype(np.float16)
    bias = rng.integers(-8, 9, size=out).astype(np.float16)
    po, pi = rng.permutation(out).astype(np.int32), rng.permutation(inn).astype(np.int32)
    c = vnm.vnm_prune_compress(_dev(Wp), V, M, want_mask=True)
    Wm_p = orc.masked_dense(Wp, orc.compress(Wp, V, M)[3])
    Y = vnm.vnm_spmm_fused(_dev(X), c, bias=_dev(bias), perm_in=_dev(pi), perm_out=_dev(po),
                           out_dtype=torch.float32, path=path)
    torch.cuda.synchronize()
    assert np.array_equal(Y.cpu().numpy().astype(np.float64), orc.linear_fused_ref(X, Wm_p, bias, pi, po))


@pytest.mark.parametrize("T", [12, 200])
def test_lossless_permuted_layer_equals_dense_layer(T):
    """Eq. 6 end to end: if the permuted weight already has the pattern, the fused call on the
    compressed permuted weight reproduces the dense layer on the ORIGINAL weight and bias."""
    rng = np.random.default_rng(T)
    out, inn, V, M = 256, 320, 64, 5
    W0, X = syn.make_weight_and_input(out, inn, T, seed=T)
    Wp_sparse = orc.masked_dense(W0, orc.compress(W0, V, M)[3])
    po, pi = rng.permutation(out).astype(np.int32), rng.permutation(inn).astype(np.int32)
    W = np.zeros_like(Wp_sparse)
    W[np.ix_(po, pi)] = Wp_sparse
    bias = rng.standard_normal(out).astype(np.float16)                 # original channel order
    Y_dense = X.astype(np.float64) @ W.astype(np.float64).T + bias.astype(np.float64)[None, :]
    c = vnm.vnm_prune_compress(_dev(orc.permute_weight(W, po, pi)), V, M)
    Y = vnm.vnm_spmm_fused(_dev(X), c, bias=_dev(bias[po]), perm_in=_dev(pi), perm_out=_dev(po))
    torch.cuda.synchronize()
    assert orc.max_normalised_error(Y.cpu().numpy(), Y_dense) <= TOL


def test_two_layers_with_folded_permutation():
    """First layer leaves its output in the row order of its weight; its P_o is folded into the
    second layer's input permutation on the host.  Same result as un-permuting in between."""
    rng = np.random.default_rng(11)
    d0, d1, d2, T, V, M = 160, 256, 128, 150, 64, 5
    X = rng.integers(-2, 3, size=(T, d0)).astype(np.float16)
    W1p = rng.integers(-1, 2, size=(d1, d0)).astype(np.float16)
    W2p = rng.integers(-1, 2, size=(d2, d1)).astype(np.float16)
    po1, pi1 = rng.permutation(d1).astype(np.int32), rng.permutation(d0).astype(np.int32)
    po2, pi2 = rng.permutation(d2).astype(np.int32), rng.permutation(d1).astype(np.int32)
    c1 = vnm.vnm_prune_compress(_dev(W1p), V, M)
    c2 = vnm.vnm_prune_compress(_dev(W2p), V, M)
    H = vnm.vnm_spmm_fused(_dev(X), c1, perm_in=_dev(pi1), perm_out=_dev(po1))
    Y_a = vnm.vnm_spmm_fused(H, c2, perm_in=_dev(pi2), perm_out=_dev(po2), out_dtype=torch.float32)
    Hp = vnm.vnm_spmm_fused(_dev(X), c1, perm_in=_dev(pi1))
    folded = vnm.vnm_fold_permutations(po1, pi2)
    assert np.array_equal(folded, orc.fold_permutations(po1, pi2))
    Y_b = vnm.vnm_spmm_fused(Hp, c2, perm_in=_dev(folded), perm_out=_dev(po2), out_dtype=torch.float32)
    torch.cuda.synchronize()
    assert torch.equal(Y_a, Y_b)
    # and against the oracle (small integers: the intermediate fp16 rounding is exact)
    Wm1 = orc.masked_dense(W1p, orc.compress(W1p, V, M)[3])
    Wm2 = orc.masked_dense(W2p, orc.compress(W2p, V, M)[3])
    H_ref = orc.linear_fused_ref(X, Wm1, perm_in=pi1, perm_out=po1)
    assert np.abs(H_ref).max() < 2048
    Y_ref = orc.linear_fused_ref(H_ref.astype(np.float16), Wm2, perm_in=pi2, perm_out=po2)
    assert np.array_equal(Y_a.cpu().numpy().astype(np.float64), Y_ref)


@pytest.mark.parametrize("path", [vnm.PATH_GENERIC, vnm.PATH_SMFMAC])
@pytest.mark.parametrize("T", [8, 140])
def test_out_of_range_entries_are_ignored(path, T):
    """An entry outside the range is not an error the host can see (device arrays): such an input
    channel reads as zero and such an output channel is not stored."""
    rng = np.random.default_rng(3)
    out, inn, V, M = 128, 160, 64, 5
    Wp = rng.integers(-2, 3, size=(out, inn)).astype(np.float16)
    X = rng.integers(-3, 4, size=(T, inn)).astype(np.float16)
    pi = rng.permutation(inn).astype(np.int32)
    po = rng.permutation(out).astype(np.int32)
    bad_in, bad_out = [3, 77, 159], [0, 64, 127]
    pi_bad, po_bad = pi.copy(), po.copy()
    pi_bad[bad_in] = [-1, inn, 2 ** 31 - 1]
    po_bad[bad_out] = [-5, out, 2 ** 30]
    c = vnm.vnm_prune_compress(_dev(Wp), V, M)
    Wm_p = orc.masked_dense(Wp, orc.compress(Wp, V, M)[3])
    Y = torch.full((T, out), -77.0, dtype=torch.float32, device=DEV)
    vnm.vnm_spmm_fused(_dev(X), c, perm_in=_dev(pi_bad), perm_out=_dev(po_bad), Y=Y, path=path)
    torch.cuda.synchronize()
    Wz = Wm_p.copy()
    Wz[:, bad_in] = 0                                    # those weight columns meet a zero input
    Y_ref = orc.linear_fused_ref(X, Wz, perm_in=pi, perm_out=po)
    mapped = np.setdiff1d(np.arange(out), po[bad_out])   # columns nothing maps to are unspecified
    assert np.array_equal(Y.cpu().numpy().astype(np.float64)[:, mapped], Y_ref[:, mapped])


@pytest.mark.parametrize("T", [40, 300])
def test_perm_in_without_room_for_a_permuted_copy(T):
    """With only the workspace vnm_spmm asks for, the staging pass gathers the permuted columns
    itself; same result."""
    X, Wm_p, bias, pi, po, c = _layer(256, 320, T, 64, 5, seed=T)
    nb = vnm.vnm_spmm_workspace_bytes(T, c)
    ws = torch.empty(nb, dtype=torch.uint8, device=DEV)
    Y = vnm.vnm_spmm_fused(_dev(X), c, perm_in=_dev(pi), workspace=ws, path=vnm.PATH_SMFMAC, out_dtype=torch.float32)
    torch.cuda.synchronize()
    assert orc.max_normalised_error(Y.cpu().numpy(), orc.linear_fused_ref(X, Wm_p, perm_in=pi)) <= TOL


@pytest.mark.parametrize("T", [5, 70])
def test_rows_of_x_too_long_for_the_permuting_pass(T):
    """in * 2 bytes beyond the LDS budget of the row-permuting pass: the gathering staging pass
    serves every T (for few tokens too)."""
    out, inn, V, M = 64, 73760, 64, 5
    rng = np.random.default_rng(T)
    Wp = rng.integers(-2, 3, size=(out, inn)).astype(np.float16)
    X = rng.integers(-2, 3, size=(T, inn)).astype(np.float16)
    pi = rng.permutation(inn).astype(np.int32)
    c = vnm.vnm_prune_compress(_dev(Wp), V, M)
    Wm_p = orc.masked_dense(Wp, orc.compress(Wp, V, M)[3])
    Y = vnm.vnm_spmm_fused(_dev(X), c, perm_in=_dev(pi), path=vnm.PATH_SMFMAC, out_dtype=torch.float32)
    torch.cuda.synchronize()
    assert np.array_equal(Y.cpu().numpy().astype(np.float64), orc.linear_fused_ref(X, Wm_p, perm_in=pi))


def test_rows_of_y_too_long_for_the_permuting_pass():
    """out * 4 bytes beyond that budget: the product kernel scatters the permuted outputs itself."""
    out, inn, T, V, M = 36928, 40, 300, 64, 5
    rng = np.random.default_rng(8)
    Wp = rng.integers(-2, 3, size=(out, inn)).astype(np.float16)
    X = rng.integers(-2, 3, size=(T, inn)).astype(np.float16)
    bias = rng.integers(-8, 9, size=out).astype(np.float16)
    po = rng.permutation(out).astype(np.int32)
    c = vnm.vnm_prune_compress(_dev(Wp), V, M)
    Wm_p = orc.masked_dense(Wp, orc.compress(Wp, V, M)[3])
    for ydt in (torch.float32, torch.float16):            # fp16 rows fit (in-place pass), fp32 rows do not
        Y = vnm.vnm_spmm_fused(_dev(X), c, bias=_dev(bias), perm_out=_dev(po), path=vnm.PATH_SMFMAC, out_dtype=ydt)
        torch.cuda.synchronize()
        assert np.array_equal(Y.cpu().numpy().astype(np.float64), orc.linear_fused_ref(X, Wm_p, bias=bias, perm_out=po))


def test_fused_argument_errors():
    X, Wm_p, bias, pi, po, c = _layer(128, 128, 40, 64, 8, seed=1)
    lib = vnm.load_library()
    Xd, Y = _dev(X), torch.empty((40, 128), dtype=torch.float16, device=DEV)
    pid = _dev(pi)

    def call(perm_in_ptr, ws_ptr, ws_bytes, T=40):
        return lib.vnm_spmm_fused(Xd.data_ptr(), T, 128, c.values.data_ptr(), c.meta.data_ptr(), c.colidx.data_ptr(),
                                  c.packed.data_ptr(), 128, 128, 64, 2, 8, None, perm_in_ptr, None, Y.data_ptr(), 128,
                                  0, vnm.PATH_AUTO, ws_ptr, ws_bytes, None)
    assert call(pid.data_ptr() + 4, None, 0) == 4                    # perm_in not 16-byte aligned
    assert call(pid.data_ptr(), None, 0) == 5                        # staged path without workspace
    assert call(pid.data_ptr(), None, 0, T=8) == 5                   # few tokens + perm_in: workspace needed too
    assert call(None, None, 0, T=8) == 0                             # few tokens, no perm_in: none needed
    torch.cuda.synchronize()


def test_llama_shaped_layer_fused_sampled_tokens():
    """Full-size layer in the launch configuration the benchmark times; sampled outputs."""
    layer = syn.config_llama2_7b()[0]
    W, X = syn.layer_tensors(layer)
    rng = np.random.default_rng(77)
    po = rng.permutation(layer.out).astype(np.int32)
    pi = rng.permutation(layer.inn).astype(np.int32)
    bias = (rng.standard_normal(layer.out) * 0.5).astype(np.float16)
    c = vnm.vnm_prune_compress(_dev(W), layer.V, layer.M, want_mask=True)
    Y = vnm.vnm_spmm_fused(_dev(X), c, bias=_dev(bias), perm_in=_dev(pi), perm_out=_dev(po))
    torch.cuda.synchronize()
    Wm = orc.masked_dense(W, c.mask.cpu().numpy())
    toks = np.sort(rng.choice(X.shape[0], size=64, replace=False))
    Y_ref = orc.linear_fused_ref(X[toks], Wm, bias=bias, perm_in=pi, perm_out=po)
    assert orc.max_normalised_error(Y.cpu().numpy()[toks], Y_ref) <= TOL


@pytest.mark.parametrize("T", [16, 200])
def test_calls_replay_from_a_hip_graph(T):
    """The product calls are plain kernel launches on the caller's stream (no allocation, no memset
    node, no host synchronisation), so a captured graph of them replays correctly: three replays on
    fresh inputs, each checked against an eager call, with eager work in between."""
    X, Wm_p, bias, pi, po, c = _layer(256, 320, T, 64, 5, seed=40 + T)
    Xd = _dev(X)
    bd, pid, pod = _dev(bias), _dev(pi), _dev(po)
    lib = vnm.load_library()
    import ctypes
    nb = ctypes.c_int64(0)
    assert lib.vnm_spmm_fused_workspace_bytes(T, 256, 320, 64, 2, 5, 1, ctypes.byref(nb)) == 0
    ws = torch.empty(nb.value, dtype=torch.uint8, device=DEV)
    Y_plain = torch.empty((T, 256), dtype=torch.float16, device=DEV)
    Y_fused = torch.empty((T, 256), dtype=torch.float16, device=DEV)

    def work():
        vnm.vnm_spmm(Xd, c, Y=Y_plain, workspace=ws)
        vnm.vnm_spmm_fused(Xd, c, bias=bd, perm_in=pid, perm_out=pod, Y=Y_fused, workspace=ws)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        work()                                   # warm-up outside the capture (one-off attribute calls)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        work()
    rng = np.random.default_rng(T)
    for rep in range(3):
        Xn = rng.standard_normal(X.shape).astype(np.float16)
        Xd.copy_(_dev(Xn))
        graph.replay()
        torch.cuda.synchronize()
        got_plain, got_fused = Y_plain.clone(), Y_fused.clone()
        work()                                   # eager, same buffers
        torch.cuda.synchronize()
        assert torch.equal(got_plain, Y_plain) and torch.equal(got_fused, Y_fused), rep
        assert orc.max_normalised_error(got_plain.cpu().numpy(), orc.matmul_ref(Xn, Wm_p)) <= TOL
        assert orc.max_normalised_error(got_fused.cpu().numpy(), orc.linear_fused_ref(Xn, Wm_p, bias, pi, po)) <= TOL
