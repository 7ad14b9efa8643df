"""The front ends that write the packed GEMM's tiled activations directly: byte for byte what the
canonical front end followed by atom_pack_act produces (which the other tests hold against the
oracle), on every variant (RMSNorm or not, index or not, residual add, SwiGLU, 3-bit codes), row
counts that end inside a unit of 64, and every thread / register-set configuration of the kernel;
and the GEMM on it gives the oracle's Y."""
import numpy as np
import pytest
import torch

import oracle
import paper_2310_19102_amd as atom
from _gpu_util import dev, npy

pytestmark = pytest.mark.gpu


def _inputs(M, K, seed, norm=True):
    g = torch.Generator().manual_seed(seed)
    sigma = torch.exp(1.5 * torch.randn(K, generator=g))
    x = (torch.randn((M, K), generator=g) * sigma).to(torch.float16)
    gamma = (1 + 0.1 * torch.randn(K, generator=g)).to(torch.float16) if norm else None
    idx = torch.argsort(sigma, stable=True).to(torch.int32)
    return x, gamma, idx


def _same(a, b, what):
    assert a.numel() == b.numel(), what
    if not torch.equal(a, b):
        bad = (a != b).nonzero().flatten()
        raise AssertionError(f"{what}: {bad.numel()} bytes differ, first at {int(bad[0])}")


@pytest.mark.parametrize("M,K,O,norm,index", [
    (1, 512, 128, True, True),          # a single row: 63 pad rows of zeros
    (64, 1024, 128, True, True),        # exactly one unit
    (70, 1408, 128, True, True),        # 11 groups, a second unit with 6 rows
    (33, 4096, 256, False, True),       # two INT8 groups
    (130, 4096, 128, True, False),      # no index
    (200, 4096, 128, False, False),     # no index, no norm: the variant without any barrier of its own
    (9, 8192, 128, True, True),         # 512 threads per row
    (5, 11008, 128, False, True),       # ragged last sweep
    (4, 12416, 128, True, True),
    (3, 20480, 128, True, True),        # 1024 threads per row
    (66, 28672, 128, False, True),      # the Llama-70B intermediate size
    (2, 32768, 128, False, False),      # the largest K fits without an index
])
def test_packed_front_end_is_front_end_then_retile(M, K, O, norm, index):
    print(f"[case] packed front end M={M} K={K} O={O} norm={norm} index={index}", flush=True)
    x, gamma, idx = _inputs(M, K, M + K, norm)
    i = dev(idx) if index else None
    qa = atom.atom_quantize_act(dev(x), dev(gamma), 1e-5, i, 128, O, 0.9)
    want = atom.atom_pack_act(*qa)
    got = torch.full_like(want, 0xA5)
    atom.atom_quantize_act_packed(dev(x), dev(gamma), 1e-5, i, 128, O, 0.9, out=got)
    torch.cuda.synchronize()
    _same(got, want, "packed activations")


def test_packed_front_end_variants_and_gemm():
    M, K, N, O = 150, 2048, 200, 128
    x, gamma, idx = _inputs(M, K, 3)
    g = torch.Generator().manual_seed(9)
    res = (0.7 * torch.randn((M, K), generator=g)).to(torch.float16)
    w = (0.02 * torch.randn((N, K), generator=g)).to(torch.float16)
    # residual add
    h, q4, q8, sc = atom.atom_add_quantize_act(dev(x), dev(res), dev(gamma), 1e-5, dev(idx))
    h2, pk = atom.atom_add_quantize_act_packed(dev(x), dev(res), dev(gamma), 1e-5, dev(idx))
    torch.cuda.synchronize()
    assert torch.equal(h, h2)
    _same(pk, atom.atom_pack_act(q4, q8, sc), "add")
    # SwiGLU, with and without index
    for i in (dev(idx), None):
        q = atom.atom_swiglu_quantize_act(dev(x), dev(res), i)
        _same(atom.atom_swiglu_quantize_act_packed(dev(x), dev(res), i), atom.atom_pack_act(*q), "swiglu")
    # 3-bit codes
    q = atom.atom_quantize_act(dev(x), dev(gamma), 1e-5, dev(idx), bits=3)
    _same(atom.atom_quantize_act_packed(dev(x), dev(gamma), 1e-5, dev(idx), bits=3), atom.atom_pack_act(*q), "3 bits")
    # the GEMM on the directly packed activations: the oracle's Y bit for bit
    qw = atom.atom_quantize_weight(dev(w), dev(idx))
    apk = atom.atom_quantize_act_packed(dev(x), dev(gamma), 1e-5, dev(idx))
    y = atom.atom_w4a4_gemm_prepacked(apk, M, atom.atom_pack_weight(*qw), N, K)
    torch.cuda.synchronize()
    ra = oracle.quantize_act(x.numpy(), gamma.numpy(), 1e-5, idx.numpy(), 128, O, 0.9)
    rw = oracle.quantize_weight(w.numpy(), idx.numpy(), 128, O, 0.85)
    ref = oracle.w4a4_gemm(*ra, *rw, 128)
    assert np.array_equal(npy(y).view(np.uint16), ref["y"].view(np.uint16))


def test_packed_front_end_limits():
    x, gamma, idx = _inputs(4, 32768, 1)
    with pytest.raises(atom.AtomError) as e:
        atom.atom_quantize_act_packed(dev(x), dev(gamma), 1e-5, dev(idx))
    assert e.value.status == 3                       # 4 K + K / 2 + the packed row: beyond the LDS
    x, gamma, idx = _inputs(4, 512, 2)
    with pytest.raises(atom.AtomError) as e:
        atom.atom_quantize_act_packed(dev(x), None, 0.0, dev(idx), clip=1e-9)
    assert e.value.status == 3
    small = torch.empty(100, dtype=torch.uint8, device="cuda")
    with pytest.raises(atom.AtomError) as e:
        atom.atom_quantize_act_packed(dev(x), None, 0.0, dev(idx), out=small)
    assert e.value.status in (4, 5)                  # too small (or, by luck of the allocator, misaligned)
