"""GPU parity for the W3A3 configuration (normal channels at 3 bits, Section 5.2 of the paper):
the front ends and the weight path with bits = 3 against the CPU oracle, bit for bit, and the
unchanged GEMM on the 3-bit codes (int32 partials bit-exact, fp16 outputs within 1e-3)."""
import numpy as np
import pytest
import torch

import oracle
import paper_2310_19102_amd as atom
from _gpu_util import Y_TOL, assert_quant_equal, dev, npy, y_rel_err

pytestmark = pytest.mark.gpu


def _inputs(M, K, N, seed, norm):
    g = torch.Generator().manual_seed(seed)
    sigma = torch.exp(1.5 * torch.randn(K, generator=g))
    x = (torch.randn((M, K), generator=g) * sigma).to(torch.float16)
    w = (0.02 * torch.randn((N, K), generator=g)).to(torch.float16)
    gamma = (1 + 0.1 * torch.randn(K, generator=g)).to(torch.float16) if norm else None
    idx = torch.argsort(sigma, stable=True).to(torch.int32)
    return x, w, gamma, idx


@pytest.mark.parametrize("M,K,N,O,norm", [
    (1, 512, 64, 128, True),         # single token, decode GEMM
    (33, 1024, 200, 256, True),      # ragged M and N, two INT8 groups
    (70, 1408, 130, 128, False),     # 11 groups, big-tile GEMM
    (9, 20480, 24, 128, True),       # K > 16384: 1024 threads per row in the front end
])
def test_w3a3_linear(M, K, N, O, norm):
    x, w, gamma, idx = _inputs(M, K, N, 31 * M + K, norm)
    eps = 1e-6 if norm else 0.0
    print(f"[case] W3A3 linear M={M} K={K} N={N} O={O} norm={norm}", flush=True)
    ra = oracle.quantize_act(x.numpy(), None if gamma is None else gamma.numpy(), eps, idx.numpy(), 128, O,
                             0.9, bits=3)
    rw = oracle.quantize_weight(w.numpy(), idx.numpy(), 128, O, 0.85, bits=3)
    ga = atom.atom_quantize_act(dev(x), dev(gamma), eps, dev(idx), 128, O, 0.9, bits=3)
    gw = atom.atom_quantize_weight(dev(w), dev(idx), 128, O, 0.85, bits=3)
    torch.cuda.synchronize()
    assert_quant_equal(ga, ra, "W3 act")
    assert_quant_equal(gw, rw, "W3 weight")
    # the codes are 3-bit: [-4, 3] in every nibble of the normal block
    q4 = npy(ga[0])
    lo, hi = (q4 & 0xF).astype(np.int16), (q4 >> 4).astype(np.int16)
    for c in (lo, hi):
        c = np.where(c >= 8, c - 16, c)
        assert c.min() >= -4 and c.max() <= 3
    G = K // 128
    ref = oracle.w4a4_gemm(*ra, *rw, 128, want_partials=True)
    part = torch.empty((M, N, G), dtype=torch.int32, device="cuda")
    y = atom.atom_w4a4_gemm(*ga, *gw, 128, partials=part)
    y2 = atom.atom_w4a4_gemm(*ga, *gw, 128)
    torch.cuda.synchronize()
    assert np.array_equal(npy(part), ref["partials"]), "int32 partials differ"
    assert y_rel_err(npy(y), ref["y"]) <= Y_TOL
    assert y_rel_err(npy(y2), ref["y"]) <= Y_TOL


def test_w3a3_fused_front_ends_and_ties():
    """Residual add and SwiGLU in front at 3 bits; rows built so that quotients fall on and next to
    rounding ties of the 3-bit grid."""
    M, K, O = 12, 1024, 128
    x, _, gamma, idx = _inputs(M, K, 8, 77, True)
    g = torch.Generator().manual_seed(78)
    res = (torch.randn((M, K), generator=g) * 0.5).to(torch.float16)
    # every quotient a multiple of 1/2: amax = 3.5 steps of 1.0 -> s = 2 * 3.5 / 7 = 1
    x[0] = ((torch.arange(K) % 15 - 7).to(torch.float16) * 0.5)
    res[0] = 0
    print("[case] W3A3 fused front ends", flush=True)
    want = oracle.add_quantize_act(x.numpy(), res.numpy(), None, 0.0, idx.numpy(), 128, O, 1.0, bits=3)
    h, *q = atom.atom_add_quantize_act(dev(x), dev(res), None, 0.0, dev(idx), 128, O, 1.0, bits=3)
    torch.cuda.synchronize()
    assert np.array_equal(npy(h).view(np.uint16), want[0].view(np.uint16))
    assert_quant_equal(tuple(q), want[1:], "W3 add+quantize")
    want = oracle.add_quantize_act(x.numpy(), res.numpy(), gamma.numpy(), 1e-6, idx.numpy(), 128, O, 0.9, bits=3)
    h, *q = atom.atom_add_quantize_act(dev(x), dev(res), dev(gamma), 1e-6, dev(idx), 128, O, 0.9, bits=3)
    torch.cuda.synchronize()
    assert_quant_equal(tuple(q), want[1:], "W3 add+norm+quantize")
    up = (torch.randn((M, K), generator=g)).to(torch.float16)
    want = oracle.swiglu_quantize_act(x.numpy(), up.numpy(), idx.numpy(), 128, O, 0.9, bits=3)
    got = atom.atom_swiglu_quantize_act(dev(x), dev(up), dev(idx), 128, O, 0.9, bits=3)
    torch.cuda.synchronize()
    assert_quant_equal(got, want, "W3 swiglu+quantize")


def test_w3a3_unsupported_widths():
    x, _, _, idx = _inputs(2, 256, 8, 5, False)
    for bits in (2, 5):
        with pytest.raises(atom.AtomError) as e:
            atom.atom_quantize_act(dev(x), None, 0.0, dev(idx), 128, 128, 0.9, bits=bits)
        assert e.value.status == 3
