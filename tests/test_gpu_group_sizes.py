"""Group sizes 64 and 256 (Section 5.4.1 of the paper varies the group size; Section 4.2 for the
arithmetic): the front ends and the group GEMM against the oracle, which takes any group size.
Codes, scales and per-group integer sums bit-identical; Y bit-identical too (the plain kernel
adds the groups in one ascending chain, as the oracle does)."""
import numpy as np
import pytest
import torch

import oracle
import paper_2310_19102_amd as atom
from _gpu_util import assert_quant_equal, dev, npy

pytestmark = pytest.mark.gpu


def _inputs(M, K, N, seed, norm=True):
    g = torch.Generator().manual_seed(seed)
    sigma = torch.exp(1.5 * torch.randn(K, generator=g))
    x = (torch.randn((M, K), generator=g) * sigma).to(torch.float16)
    w = (0.02 * torch.randn((N, K), generator=g)).to(torch.float16)
    gamma = (1 + 0.1 * torch.randn(K, generator=g)).to(torch.float16) if norm else None
    idx = torch.argsort(sigma, stable=True).to(torch.int32)
    return x, w, gamma, idx


@pytest.mark.parametrize("gs,M,K,N,O,norm", [
    (64, 1, 256, 8, 64, True),          # three INT4 groups and one INT8 group of 64
    (64, 33, 1024, 200, 128, True),     # two INT8 groups, ragged M and N
    (64, 70, 4096, 130, 128, False),    # the Llama-7B hidden size: 64 groups
    (64, 5, 11008, 40, 128, True),      # 172 groups
    (256, 3, 512, 40, 256, False),      # one INT4 and one INT8 group of 256
    (256, 65, 4096, 72, 256, True),     # 16 groups
    (256, 130, 2048, 257, 512, True),   # two INT8 groups, three row tiles
    (256, 9, 11008, 24, 256, False),    # 43 groups: the sweep of the front end ends ragged
])
def test_group_size_front_end_and_gemm(gs, M, K, N, O, norm):
    print(f"[case] group size {gs}: M={M} K={K} N={N} O={O} norm={norm}", flush=True)
    x, w, gamma, idx = _inputs(M, K, N, gs + M + K, norm)
    eps = 1e-5
    ga = atom.atom_quantize_act(dev(x), dev(gamma), eps, dev(idx), gs, O, 0.9)
    gw = atom.atom_quantize_weight(dev(w), dev(idx), gs, O, 0.85)
    torch.cuda.synchronize()
    ra = oracle.quantize_act(x.numpy(), None if gamma is None else gamma.numpy(), eps, idx.numpy(), gs, O, 0.9)
    rw = oracle.quantize_weight(w.numpy(), idx.numpy(), gs, O, 0.85)
    assert ga[2].shape == (M, K // gs)
    assert_quant_equal(ga, ra, "act")
    assert_quant_equal(gw, rw, "weight")
    ref = oracle.w4a4_gemm(*ra, *rw, gs, want_partials=True)
    part = torch.empty((M, N, K // gs), dtype=torch.int32, device="cuda")
    y = atom.atom_w4a4_gemm(*ga, *gw, gs, partials=part)
    y1 = atom.atom_w4a4_gemm(*ga, *gw, gs)
    torch.cuda.synchronize()
    assert np.array_equal(npy(part), ref["partials"]), "int32 partials differ"
    assert np.array_equal(npy(y).view(np.uint16), ref["y"].view(np.uint16)), "Y differs from the oracle's"
    assert torch.equal(y, y1)


@pytest.mark.parametrize("gs", [64, 256])
def test_group_size_other_front_ends(gs):
    """Residual add, SwiGLU, no index and 3-bit codes at the other group sizes."""
    M, K, O = 12, 2048, 256
    x, _, gamma, idx = _inputs(M, K, 8, 5 * gs)
    g = torch.Generator().manual_seed(gs)
    res = (0.7 * torch.randn((M, K), generator=g)).to(torch.float16)
    h, q4, q8, sc = atom.atom_add_quantize_act(dev(x), dev(res), dev(gamma), 1e-5, dev(idx), gs, O, 0.9)
    torch.cuda.synchronize()
    ref = oracle.add_quantize_act(x.numpy(), res.numpy(), gamma.numpy(), 1e-5, idx.numpy(), gs, O, 0.9)
    assert np.array_equal(npy(h).view(np.uint16), ref[0].view(np.uint16))
    assert_quant_equal((q4, q8, sc), ref[1:], "add")
    got = atom.atom_swiglu_quantize_act(dev(x), dev(res), dev(idx), gs, O, 0.9)
    assert_quant_equal(got, oracle.swiglu_quantize_act(x.numpy(), res.numpy(), idx.numpy(), gs, O, 0.9), "swiglu")
    got = atom.atom_quantize_act(dev(x), dev(gamma), 1e-5, None, gs, O, 0.9)
    ident = np.arange(K, dtype=np.int32)
    assert_quant_equal(got, oracle.quantize_act(x.numpy(), gamma.numpy(), 1e-5, ident, gs, O, 0.9), "no index")
    got = atom.atom_quantize_act(dev(x), dev(gamma), 1e-5, dev(idx), gs, O, 0.9, bits=3)
    assert_quant_equal(got, oracle.quantize_act(x.numpy(), gamma.numpy(), 1e-5, idx.numpy(), gs, O, 0.9, 3), "3 bits")


def test_group_size_limits():
    x, w, gamma, idx = _inputs(4, 512, 16, 1)
    with pytest.raises(atom.AtomError) as e:
        atom.atom_quantize_act(dev(x), None, 0.0, dev(idx), 32, 128, 0.9)
    assert e.value.status == 3                              # only 64, 128, 256
    with pytest.raises(atom.AtomError) as e:
        atom.atom_quantize_act(dev(x), None, 0.0, dev(idx), 256, 128, 0.9)
    assert e.value.status == 2                              # O must be a multiple of the group size
    qw = atom.atom_quantize_weight(dev(w), dev(idx), 64, 128, 0.85)
    with pytest.raises(atom.AtomError) as e:
        atom.atom_pack_weight(*qw, 64)
    assert e.value.status == 3                              # the packed path is built around groups of 128
    with pytest.raises(atom.AtomError) as e:
        atom.atom_decode_linear(dev(x), None, 0.0, dev(idx), *qw, 64)
    assert e.value.status == 3
