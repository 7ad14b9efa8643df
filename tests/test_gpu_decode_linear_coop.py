"""The one-launch decode linear whose front end runs once (atom_decode_linear_coop: the first M
workgroups quantise the rows while the others already stream their weights) against the CPU
oracle and the two-launch path: codes and scales bit-identical to the oracle's (Sections 4.1 and
4.2 of the paper), Y bit-identical to atom_quantize_act + atom_w4a4_gemm (the same kernel routine)
and within 1e-3 of the oracle.  The calls share their code arrays and their counters, and the
inputs change from call to call: codes left over from the call before, or a workgroup that did not
wait, would show as a wrong Y."""
import numpy as np
import pytest
import torch

import oracle
import paper_2310_19102_amd as atom
from paper_2310_19102_amd import synth
from _gpu_util import (Y_TOL, assert_quant_equal, dev, gpu_quantize_weight, npy, ref_quantize_act,
                       ref_quantize_weight, y_rel_err)

pytestmark = pytest.mark.gpu


def _rand_linear(M, K, N, seed, norm=True):
    g = torch.Generator().manual_seed(seed)
    sigma = torch.exp(1.5 * torch.randn(K, generator=g))
    x = (torch.randn((M, K), generator=g) * sigma).to(torch.float16)
    w = (0.02 * torch.randn((N, K), generator=g)).to(torch.float16)
    gamma = (1 + 0.1 * torch.randn(K, generator=g)).to(torch.float16) if norm else None
    idx = torch.argsort(sigma, stable=True).to(torch.int32)
    return synth.Linear("rand", x, w, gamma, idx, n_outlier=128)


@pytest.mark.parametrize("M,K,N,norm,index", [
    (1, 4096, 4096, True, True),       # Llama-7B attention projection, one token
    (8, 4096, 11008, True, True),      # gate or up projection: 688 consumers
    (16, 4096, 200, False, True),      # the largest M, ragged N, no norm
    (8, 11008, 4096, False, True),     # down projection: 86 groups (a last block of two), three register sets
    (5, 8192, 130, True, True),        # two register sets in the front end
    (16, 12288, 32, True, True),       # the largest K
    (3, 1024, 16, True, True),         # eight groups: one consumer, most wavefronts without a group
    (4, 4096, 22016, True, False),     # no index; 1376 consumers: more than are resident at one time
    (9, 11008, 4096, False, False),
])
def test_coop_decode_linear(M, K, N, norm, index):
    print(f"[case] cooperative decode linear M={M} K={K} N={N} norm={norm} index={index}", flush=True)
    lin = _rand_linear(M, K, N, seed=M * 31 + K + N, norm=norm)
    gw = gpu_quantize_weight(lin)
    rw = ref_quantize_weight(lin)
    idx = dev(lin.idx) if index else None
    idx_ref = lin.idx.numpy() if index else np.arange(K, dtype=np.int32)
    sync = atom.atom_decode_linear_coop_sync()
    codes = None
    xs = [lin.x, (0.5 * lin.x.flip(0)).to(torch.float16), lin.x.roll(1, 1).contiguous()]
    for it in range(6):
        x = xs[it % 3]
        y, codes = atom.atom_decode_linear_coop(dev(x), dev(lin.gamma), lin.eps, idx, *gw, sync, lin.group_size,
                                                lin.clip_act, codes=codes)
        qa = atom.atom_quantize_act(dev(x), dev(lin.gamma), lin.eps, idx, lin.group_size, 128, lin.clip_act)
        y2 = atom.atom_w4a4_gemm(*qa, *gw, lin.group_size)
        torch.cuda.synchronize()
        assert not npy(sync).any(), f"call {it}: counters {np.nonzero(npy(sync))}"
        for got, want in zip(codes, qa):
            assert torch.equal(got, want), f"call {it}: codes differ from atom_quantize_act"
        assert torch.equal(y, y2), f"call {it}: Y differs from the two-launch path"
        if it < 2:
            ra = oracle.quantize_act(x.numpy(), None if lin.gamma is None else lin.gamma.numpy(), lin.eps, idx_ref,
                                     lin.group_size, 128, lin.clip_act)
            assert_quant_equal(codes, ra, "codes of the producers")
            ref = oracle.w4a4_gemm(*ra, *rw, lin.group_size)
            assert y_rel_err(npy(y), ref["y"]) <= Y_TOL


def test_coop_decode_linear_in_a_graph():
    """Captured once, replayed with new inputs: the counters are left zero by every launch."""
    M, K, N = 8, 4096, 4096
    lin = _rand_linear(M, K, N, seed=77)
    gw = gpu_quantize_weight(lin)
    x, gamma, idx = dev(lin.x).clone(), dev(lin.gamma), dev(lin.idx)
    sync = atom.atom_decode_linear_coop_sync()
    y = torch.empty((M, N), dtype=torch.float16, device="cuda")
    _, codes = atom.atom_decode_linear_coop(x, gamma, lin.eps, idx, *gw, sync, out=y)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        for _ in range(3):      # three launches back to back on the same arrays
            atom.atom_decode_linear_coop(x, gamma, lin.eps, idx, *gw, sync, out=y, codes=codes)
    for r in range(4):
        x.copy_(dev((lin.x * (1.0 + 0.25 * r)).to(torch.float16)))
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        qa = atom.atom_quantize_act(x, gamma, lin.eps, idx)
        y2 = atom.atom_w4a4_gemm(*qa, *gw)
        torch.cuda.synchronize()
        assert torch.equal(y, y2), f"replay {r}"
        assert not npy(sync).any()


def test_coop_decode_linear_limits():
    lin = _rand_linear(4, 1408, 32, seed=8)              # 11 groups: odd
    gw = gpu_quantize_weight(lin)
    sync = atom.atom_decode_linear_coop_sync()
    with pytest.raises(atom.AtomError) as e:
        atom.atom_decode_linear_coop(dev(lin.x), dev(lin.gamma), lin.eps, dev(lin.idx), *gw, sync)
    assert e.value.status == 3
    lin = _rand_linear(17, 1024, 32, seed=9)             # too many rows
    gw = gpu_quantize_weight(lin)
    with pytest.raises(atom.AtomError) as e:
        atom.atom_decode_linear_coop(dev(lin.x), dev(lin.gamma), lin.eps, dev(lin.idx), *gw, sync)
    assert e.value.status == 3
    # no rows: nothing runs
    y, _ = atom.atom_decode_linear_coop(dev(lin.x)[:0], dev(lin.gamma), lin.eps, dev(lin.idx), *gw, sync)
    assert y.shape == (0, 32)
    torch.cuda.synchronize()
    assert not npy(sync).any()


def test_coop_decode_linear_strided_and_w3a3():
    """Row strides on x and Y; 3-bit normal codes (Section 5.4.1's W3A3 variant)."""
    lin = _rand_linear(6, 2048, 72, seed=77)
    xs = torch.zeros((6, 2048 + 64), dtype=torch.float16, device="cuda")
    xs[:, :2048] = dev(lin.x)
    ys = torch.full((6, 100), 7.0, dtype=torch.float16, device="cuda")
    sync = atom.atom_decode_linear_coop_sync()
    for bits in (4, 3):
        gw = atom.atom_quantize_weight(dev(lin.w), dev(lin.idx), 128, 128, lin.clip_weight, bits=bits)
        y, codes = atom.atom_decode_linear_coop(xs[:, :2048], dev(lin.gamma), lin.eps, dev(lin.idx), *gw, sync, 128,
                                                lin.clip_act, out=ys[:, :72], bits=bits)
        torch.cuda.synchronize()
        ra = oracle.quantize_act(lin.x.numpy(), lin.gamma.numpy(), lin.eps, lin.idx.numpy(), 128, 128,
                                 lin.clip_act, bits)
        assert_quant_equal(codes, ra, f"codes, {bits} bits")
        rw = oracle.quantize_weight(lin.w.numpy(), lin.idx.numpy(), 128, 128, lin.clip_weight, bits)
        ref = oracle.w4a4_gemm(*ra, *rw, 128)
        assert y_rel_err(npy(ys[:, :72]), ref["y"]) <= Y_TOL
        assert (ys[:, 72:] == 7.0).all(), "columns beyond N were written"
        assert not npy(sync).any()


def test_coop_decode_linear_random_shapes():
    """Seeded random problems (M 1..16, even group counts 8..30, ragged N, with and without norm and
    index) on one set of counters: Y of the one launch equals Y of the two launches bit for bit."""
    rng = np.random.default_rng(77)
    sync = atom.atom_decode_linear_coop_sync()
    for case in range(24):
        M = int(rng.integers(1, 17))
        G = int(rng.choice([8, 10, 12, 14, 16, 18, 22, 26, 30]))
        K = 128 * G
        N = int(rng.integers(1, 3000))
        norm, index = bool(rng.integers(0, 2)), bool(rng.integers(0, 2))
        print(f"[case] random cooperative decode linear {case}: M={M} K={K} N={N} norm={norm} index={index}", flush=True)
        lin = _rand_linear(M, K, N, seed=3000 + case, norm=norm)
        gw = gpu_quantize_weight(lin)
        idx = dev(lin.idx) if index else None
        y, codes = atom.atom_decode_linear_coop(dev(lin.x), dev(lin.gamma), lin.eps, idx, *gw, sync, lin.group_size,
                                                lin.clip_act)
        qa = atom.atom_quantize_act(dev(lin.x), dev(lin.gamma), lin.eps, idx, lin.group_size, 128, lin.clip_act)
        y2 = atom.atom_w4a4_gemm(*qa, *gw, lin.group_size)
        torch.cuda.synchronize()
        for got, want in zip(codes, qa):
            assert torch.equal(got, want), f"case {case}: codes"
        assert torch.equal(y, y2), f"case {case}: Y"
        assert not npy(sync).any(), f"case {case}: counters"
