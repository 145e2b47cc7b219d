"""GPU parity of vnm_lora_merge and the mask refresh (Section 4.3, Eq. 10): bit-exact against the
oracle's fixed-order fp32 merge, and the refreshed mask / compressed triple bit-exact as well."""

import numpy as np
import pytest
import torch

import paper_2410_16135_amd as vnm
import synth_inputs as syn
from oracle import vnm_oracle as orc

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def _adapter(rng, out, inn, r, amp=0.05):
    return (rng.standard_normal((out, r)) * amp).astype(np.float32), (rng.standard_normal((r, inn)) * amp).astype(np.float32)


@pytest.mark.parametrize("out,inn,r", [(128, 128, 16), (70, 333, 4), (200, 77, 64), (1, 8, 1), (257, 1030, 16), (64, 40, 0)])
def test_merge_bit_exact(out, inn, r):
    rng = np.random.default_rng(out + inn + r)
    W, _ = syn.make_weight_and_input(out, inn, 1, seed=out + r)
    B, A = _adapter(rng, out, inn, r)
    got = vnm.vnm_lora_merge(_dev(W), _dev(B), _dev(A), 2.0).cpu().numpy()
    assert np.array_equal(got.view(np.uint16), orc.lora_merge(W, B, A, 2.0).view(np.uint16))


def test_merge_strided_and_in_place():
    rng = np.random.default_rng(9)
    big = _dev(syn.make_weight_and_input(96, 160, 1, seed=9)[0])
    Wt = big[:, :100]                                   # leading dimension 160, width 100
    W = Wt.cpu().numpy().copy()
    B, A = _adapter(rng, 96, 100, 8)
    want = orc.lora_merge(W, B, A, 1.5)
    vnm.vnm_lora_merge(Wt, _dev(B), _dev(A), 1.5, W_merged=Wt)      # in place
    torch.cuda.synchronize()
    assert np.array_equal(Wt.cpu().numpy().view(np.uint16), want.view(np.uint16))


@pytest.mark.parametrize("with_act", [False, True])
@pytest.mark.parametrize("out,inn,V,M", [(128, 160, 64, 5), (96, 200, 32, 8), (200, 77, 16, 7)])
def test_refreshed_mask_bit_exact(out, inn, V, M, with_act):
    rng = np.random.default_rng(out + M)
    W, _ = syn.make_weight_and_input(out, inn, 1, seed=M)
    B, A = _adapter(rng, out, inn, 16, amp=0.1)
    act = (0.5 + rng.random(inn)).astype(np.float32) if with_act else None
    c = vnm.vnm_refresh_mask(_dev(W), _dev(B), _dev(A), 2.0, V, M, act=None if act is None else _dev(act))
    torch.cuda.synchronize()
    merged, mask = orc.refresh_mask(W, B, A, 2.0, V, M, act)
    assert np.array_equal(c.mask.cpu().numpy(), mask)
    score = None if act is None else orc.importance_ria(merged, act)
    values, meta, colidx, _ = orc.compress(merged, V, M, score=score)
    assert np.array_equal(c.values.cpu().numpy().view(np.uint16), values.reshape(-1).view(np.uint16))
    assert np.array_equal(c.meta.cpu().numpy(), meta.reshape(-1))
    assert np.array_equal(c.colidx.cpu().numpy(), colidx.reshape(-1))
    # Eq. 10: the decompressed weight is (W + BA) (.) M
    assert np.array_equal(vnm.vnm_decompress(c).cpu().numpy().view(np.uint16),
                          orc.masked_dense(merged, mask).view(np.uint16))


def test_merge_llama_shaped_layer_full_size():
    layer = syn.config_llama2_7b()[0]
    W, _ = syn.layer_tensors(layer, tokens=1)
    rng = np.random.default_rng(16)
    B, A = _adapter(rng, layer.out, layer.inn, 16, amp=0.02)
    got = vnm.vnm_lora_merge(_dev(W), _dev(B), _dev(A), 2.0).cpu().numpy()
    assert np.array_equal(got.view(np.uint16), orc.lora_merge(W, B, A, 2.0).view(np.uint16))


def test_merge_argument_errors():
    lib = vnm.load_library()
    W = torch.zeros((8, 16), dtype=torch.float16, device=DEV)
    B = torch.zeros((8, 4), dtype=torch.float32, device=DEV)
    A = torch.zeros((4, 16), dtype=torch.float32, device=DEV)
    call = lambda **k: lib.vnm_lora_merge(k.get("W", W.data_ptr()), 8, 16, k.get("ldw", 16), B.data_ptr(), k.get("ldb", 4),
                                          A.data_ptr(), 16, k.get("r", 4), 2.0, W.data_ptr(), 16, None)
    assert call() == 0
    assert call(W=None) == 1 and call(ldw=8) == 2 and call(ldb=2) == 2 and call(r=-1) == 2
    torch.cuda.synchronize()
