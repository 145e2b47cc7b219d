"""Every device result that decides or carries data must be the same bits on every call.  The three
layer shapes of the Llama-shaped block (4096 x 4096, 11008 x 4096, 4096 x 11008) are each run several
times through the entry points of the path and its extensions, in the launch shapes the benchmark
uses, and compared with the first call byte for byte.  Shapes with more workgroups than compute
units are the point: a kernel can pass every small parity case and still lose updates there."""

import numpy as np
import pytest
import torch

import paper_2410_16135_amd as vnm
import synth_inputs as syn

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _same(a, b):
    return torch.equal(a.view(torch.uint8).reshape(-1), b.view(torch.uint8).reshape(-1))


def _packed_sections(c):
    """The written parts of the matrix-core copy: three sections, each starting on a 256-byte boundary;
    the gaps and the 8 KiB of trailing slack are never written."""
    up = lambda x: (x + 255) // 256 * 256
    Rp, S = (-(-c.out // c.V) * c.V + 63) // 64, -(-(-(-c.inn // c.M)) // 8)
    parts, off = [], 0
    for nbytes in (Rp * S * 2048, Rp * S * 256, Rp * S * 32 * (2 if c.V == 32 else 1)):
        parts.append(c.packed[off:off + nbytes].clone())
        off += up(nbytes)
    assert off + 8192 == c.packed.numel()
    return torch.cat(parts)


def _layer(name, tokens):
    layer = [l for l in syn.config_llama2_7b() if l.name == name][0]
    W, X = syn.layer_tensors(layer, tokens=tokens)
    return layer, torch.from_numpy(W).to(DEV), torch.from_numpy(X).to(DEV)


@pytest.mark.parametrize("tokens", [512, 4096])           # K split over workgroups + reduction; the benchmark's launch
@pytest.mark.parametrize("name", ["q", "gate", "down"])
def test_prune_spmm_decompress_repeat_bit_for_bit(name, tokens):
    layer, Wd, Xd = _layer(name, tokens)
    first = None
    for _ in range(3):
        c = vnm.vnm_prune_compress(Wd, layer.V, layer.M)
        Y = vnm.vnm_spmm(Xd, c)
        Y16 = vnm.vnm_spmm(Xd[:16].contiguous(), c)
        Wp = vnm.vnm_decompress(c)
        torch.cuda.synchronize()
        got = (c.values.clone(), c.meta.clone(), c.colidx.clone(), _packed_sections(c), Y, Y16, Wp)
        if first is None:
            first = got
        else:
            for a, b in zip(first, got):
                assert _same(a, b)


@pytest.mark.parametrize("name", ["q", "gate", "down"])
def test_few_token_products_repeat_bit_for_bit(name):
    """One to 256 tokens at the full layer sizes: the vector-ALU kernel, the resident-X kernel alone, in token
    groups, with several row blocks per workgroup and with K split -- every call must return the same bits (the
    sums through LDS and the split-K reduction run in a fixed order; wave-private LDS strips are written and read
    back without a barrier)."""
    layer, Wd, Xd = _layer(name, 256)
    c = vnm.vnm_prune_compress(Wd, layer.V, layer.M)
    for T in (1, 2, 4, 7, 16, 24, 32, 48, 64, 100, 192, 256):
        X = Xd[:T].contiguous()
        first = vnm.vnm_spmm(X, c)
        for _ in range(4):
            again = vnm.vnm_spmm(X, c)
            torch.cuda.synchronize()
            assert _same(first, again), T


@pytest.mark.parametrize("name", ["q", "gate", "down"])
def test_scores_search_kernels_and_merge_repeat_bit_for_bit(name):
    layer, Wd, Xd = _layer(name, 64)
    act = Xd.float().pow(2).sum(dim=0).sqrt().pow(0.5).contiguous()
    g = torch.Generator(device="cpu").manual_seed(3)
    B = (torch.randn(layer.out, 8, generator=g) * 0.01).to(DEV)
    A = (torch.randn(8, layer.inn, generator=g) * 0.01).to(DEV)
    first = None
    for _ in range(3):
        S = vnm.vnm_ria_scores(Wd, act)
        scale = float(2 ** 30) / float(S.max().item())
        cs = vnm.vnm_prune_compress_scored(Wd, S, layer.V, layer.M)
        obj = vnm.vnm_retained_score(S, layer.V, layer.M, scale)
        g_in = vnm.vnm_permutation_gain(S, layer.V, layer.M, scale, 0, 1)
        g_out = vnm.vnm_permutation_gain(S, layer.V, layer.M, scale, 1, 2)
        Wm = vnm.vnm_lora_merge(Wd, B, A, 2.0)
        torch.cuda.synchronize()
        got = (S, cs.values.clone(), cs.meta.clone(), cs.colidx.clone(), Wm)
        host = (obj, g_in, g_out)
        if first is None:
            first = (got, host)
        else:
            for a, b in zip(first[0], got):
                assert _same(a, b)
            assert first[1][0] == host[0]
            assert np.array_equal(first[1][1], host[1]) and np.array_equal(first[1][2], host[2])
