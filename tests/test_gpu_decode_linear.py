"""The one-launch decode linear (front end in the prologue of the weight-streaming GEMM) against
the CPU oracle: activation codes and scales bit-identical (Sections 4.1 and 4.2 of the paper), Y
within 1e-3 of the oracle's group GEMM on those codes, and bit-identical to the two-launch path
(atom_quantize_act, atom_w4a4_gemm), whose sum over groups is the same tree at these shapes."""
import numpy as np
import pytest
import torch

import oracle
import paper_2310_19102_amd as atom
from paper_2310_19102_amd import synth
from _gpu_util import (Y_TOL, assert_quant_equal, dev, gpu_quantize_weight, npy, ref_quantize_act,
                       ref_quantize_weight, y_rel_err)

pytestmark = pytest.mark.gpu


def _rand_linear(M, K, N, O, seed, norm=True):
    g = torch.Generator().manual_seed(seed)
    sigma = torch.exp(1.5 * torch.randn(K, generator=g))
    x = (torch.randn((M, K), generator=g) * sigma).to(torch.float16)
    w = (0.02 * torch.randn((N, K), generator=g)).to(torch.float16)
    gamma = (1 + 0.1 * torch.randn(K, generator=g)).to(torch.float16) if norm else None
    idx = torch.argsort(sigma, stable=True).to(torch.int32)
    return synth.Linear("rand", x, w, gamma, idx, n_outlier=O)


@pytest.mark.parametrize("M,K,N,O,norm,same_tree", [
    (1, 4096, 4096, 128, True, True),      # Llama-7B attention projection, one token
    (8, 4096, 11008, 128, True, True),     # Llama-7B gate or up projection
    (16, 4096, 200, 128, False, True),     # the largest M, ragged N, no norm
    (8, 11008, 4096, 128, False, True),    # Llama-7B down projection: 86 groups, runs of 8 and 12 groups
    (5, 8192, 130, 128, True, True),       # two register sets in the front end, one batch of eight groups
    (3, 1408, 40, 128, True, False),       # 11 groups (odd): runs of single groups
    (7, 768, 24, 256, True, True),         # two INT8 groups
    (2, 256, 16, 128, False, False),       # one INT4 + one INT8 group: most wavefronts have no group
    (16, 12288, 32, 128, True, True),      # the largest K
])
def test_decode_linear_matches_oracle_and_two_launch_path(M, K, N, O, norm, same_tree):
    print(f"[case] decode linear M={M} K={K} N={N} O={O} norm={norm}", flush=True)
    lin = _rand_linear(M, K, N, O, seed=M * 31 + K + N, norm=norm)
    gw = gpu_quantize_weight(lin)
    rw = ref_quantize_weight(lin)
    assert_quant_equal(gw, rw, "weight")
    y, codes = atom.atom_decode_linear(dev(lin.x), dev(lin.gamma), lin.eps, dev(lin.idx), *gw,
                                       lin.group_size, lin.clip_act, debug=True)
    torch.cuda.synchronize()
    ra = ref_quantize_act(lin)
    assert_quant_equal(codes, ra, "activation codes computed in the prologue")
    ref = oracle.w4a4_gemm(*ra, *rw, lin.group_size)
    err = y_rel_err(npy(y), ref["y"])
    assert err <= Y_TOL, f"Y rel err {err}"
    # without the debug outputs: the same Y
    y1 = atom.atom_decode_linear(dev(lin.x), dev(lin.gamma), lin.eps, dev(lin.idx), *gw, lin.group_size, lin.clip_act)
    assert torch.equal(y, y1)
    # the two-launch path
    qa = atom.atom_quantize_act(dev(lin.x), dev(lin.gamma), lin.eps, dev(lin.idx), lin.group_size, O, lin.clip_act)
    y2 = atom.atom_w4a4_gemm(*qa, *gw, lin.group_size)
    torch.cuda.synchronize()
    if same_tree:
        assert torch.equal(y, y2), "one launch and two launches differ"
    else:
        assert y_rel_err(npy(y), npy(y2)) <= Y_TOL


def test_decode_linear_strided_and_w3a3():
    """Row strides on x and Y; 3-bit normal codes (Section 5.4.1's W3A3 variant)."""
    lin = _rand_linear(6, 2048, 72, 128, seed=77)
    xs = torch.zeros((6, 2048 + 64), dtype=torch.float16, device="cuda")
    xs[:, :2048] = dev(lin.x)
    ys = torch.full((6, 100), 7.0, dtype=torch.float16, device="cuda")
    for bits in (4, 3):
        gw = atom.atom_quantize_weight(dev(lin.w), dev(lin.idx), 128, 128, lin.clip_weight, bits=bits)
        y, codes = atom.atom_decode_linear(xs[:, :2048], dev(lin.gamma), lin.eps, dev(lin.idx), *gw, 128,
                                           lin.clip_act, out=ys[:, :72], debug=True, bits=bits)
        torch.cuda.synchronize()
        ra = oracle.quantize_act(lin.x.numpy(), lin.gamma.numpy(), lin.eps, lin.idx.numpy(), 128, 128,
                                 lin.clip_act, bits)
        assert_quant_equal(codes, ra, f"codes, {bits} bits")
        rw = oracle.quantize_weight(lin.w.numpy(), lin.idx.numpy(), 128, 128, lin.clip_weight, bits)
        ref = oracle.w4a4_gemm(*ra, *rw, 128)
        assert y_rel_err(npy(ys[:, :72]), ref["y"]) <= Y_TOL
        assert (ys[:, 72:] == 7.0).all(), "columns beyond N were written"


def test_decode_linear_limits():
    lin = _rand_linear(2, 512, 16, 128, seed=3)
    gw = gpu_quantize_weight(lin)
    x17 = torch.zeros((17, 512), dtype=torch.float16, device="cuda")
    with pytest.raises(atom.AtomError) as e:
        atom.atom_decode_linear(x17, None, 0.0, dev(lin.idx), *gw)
    assert e.value.status == 3                       # M > 16: unsupported
    with pytest.raises(atom.AtomError) as e:
        atom.atom_decode_linear(dev(lin.x), None, 0.0, dev(lin.idx), *gw, clip=1e-9)
    assert e.value.status == 3                       # clip below 2^-20
    assert atom.atom_decode_linear_lds_bytes(16, 12288, 128, True) <= 160 * 1024
    y = atom.atom_decode_linear(torch.zeros((0, 512), dtype=torch.float16, device="cuda"), None, 0.0,
                                dev(lin.idx), *gw)
    assert y.shape == (0, 16)


@pytest.mark.parametrize("M,K,N,O,norm", [
    (1, 4096, 4096, 128, False),     # one wavefront per row
    (8, 4096, 256, 128, True),       # the same with RMSNorm: the wavefront's own sum of squares
    (16, 4096, 48, 128, True),       # two rows per wavefront
    (8, 11008, 4096, 128, False),    # Llama-7B down projection behind a permuted gate/up: 22 vectors per lane, ragged
    (5, 8192, 130, 128, True),       # RMSNorm over a long row: the workgroup-wide routine without its gather
    (16, 12288, 32, 128, True),
    (3, 1408, 40, 128, False),
    (7, 768, 24, 256, True),         # two INT8 groups
])
def test_decode_linear_without_index(M, K, N, O, norm):
    """No reorder index: x already is in reordered order.  Codes as the oracle's with the identity index."""
    print(f"[case] decode linear, no index, M={M} K={K} N={N} O={O} norm={norm}", flush=True)
    lin = _rand_linear(M, K, N, O, seed=M * 17 + K + N, norm=norm)
    ident = np.arange(K, dtype=np.int32)
    gw = atom.atom_quantize_weight(dev(lin.w), None, lin.group_size, O, lin.clip_weight)
    rw = oracle.quantize_weight(lin.w.numpy(), ident, lin.group_size, O, lin.clip_weight)
    assert_quant_equal(gw, rw, "weight")
    y, codes = atom.atom_decode_linear(dev(lin.x), dev(lin.gamma), lin.eps, None, *gw, lin.group_size, lin.clip_act,
                                       debug=True)
    torch.cuda.synchronize()
    ra = oracle.quantize_act(lin.x.numpy(), None if lin.gamma is None else lin.gamma.numpy(), lin.eps, ident,
                             lin.group_size, O, lin.clip_act)
    assert_quant_equal(codes, ra, "activation codes computed in the prologue")
    ref = oracle.w4a4_gemm(*ra, *rw, lin.group_size)
    assert y_rel_err(npy(y), ref["y"]) <= Y_TOL
    qa = atom.atom_quantize_act(dev(lin.x), dev(lin.gamma), lin.eps, None, lin.group_size, O, lin.clip_act)
    y2 = atom.atom_w4a4_gemm(*qa, *gw, lin.group_size)
    torch.cuda.synchronize()
    assert y_rel_err(npy(y), npy(y2)) <= Y_TOL


@pytest.mark.parametrize("M,K,N", [(1, 4096, 4096), (8, 4096, 11008), (16, 4096, 200), (32, 4096, 4096),
                                   (64, 4096, 1030), (8, 11264, 4090), (3, 1024, 16),
                                   # K/128 = 4 j + 2: the last block is one INT4 group and the INT8 group
                                   (8, 11008, 4096), (1, 11008, 100), (13, 1280, 48), (32, 11008, 520), (50, 1792, 64),
                                   # the fused gate/up projection of the benchmark's decode sweep: two rounds of workgroups
                                   (8, 4096, 22016),
                                   # more than 32 rows and more blocks of 16 channels than CUs: two channel blocks per
                                   # workgroup; an odd number of blocks, a ragged last block, both kinds of last batch
                                   (64, 1024, 4112), (40, 1280, 4200), (33, 4096, 11008),
                                   # 65 to 256 rows: blocks of 64 rows, the last one ragged or not
                                   (65, 1024, 520), (100, 4096, 4096), (128, 1280, 4200), (128, 1792, 48),
                                   (200, 1024, 520), (256, 4096, 4096)])
def test_decode_gemm_on_tiled_weights_is_bit_identical(M, K, N):
    """Weight codes re-tiled into whole 128-byte lines per load: same arithmetic, same tree, same Y
    as the canonical decode-sized GEMM, which the other tests hold against the oracle; ragged N
    (rows past N are zeros in the tiled arrays)."""
    print(f"[case] tiled decode weights M={M} K={K} N={N}", flush=True)
    lin = _rand_linear(M, K, N, 128, seed=M + K + N, norm=False)
    gw = gpu_quantize_weight(lin)
    qa = atom.atom_quantize_act(dev(lin.x), None, 0.0, dev(lin.idx), 128, 128, lin.clip_act)
    t4, t8 = atom.atom_tile_weight_decode(gw[0], gw[1])
    y = atom.atom_w4a4_gemm(*qa, *gw)
    yt = atom.atom_w4a4_gemm_decode_tiled(*qa, t4, t8, gw[2])
    torch.cuda.synchronize()
    assert torch.equal(y, yt)
    ra = ref_quantize_act(lin)
    ref = oracle.w4a4_gemm(*ra, *ref_quantize_weight(lin), 128)
    assert y_rel_err(npy(yt), ref["y"]) <= Y_TOL


def test_decode_tiled_limits():
    lin = _rand_linear(4, 768, 32, 256, seed=8)          # two INT8 groups: not taken
    gw = gpu_quantize_weight(lin)
    qa = atom.atom_quantize_act(dev(lin.x), dev(lin.gamma), lin.eps, dev(lin.idx), 128, 256, lin.clip_act)
    t4, t8 = atom.atom_tile_weight_decode(gw[0], gw[1])
    with pytest.raises(atom.AtomError) as e:
        atom.atom_w4a4_gemm_decode_tiled(*qa, t4, t8, gw[2])
    assert e.value.status == 3


def test_decode_gemm_random_shapes():
    """Seeded random decode-sized problems (M 1..64, even group counts 8..30, ragged N): canonical and
    tiled weights give the same bits wherever both run the decode kernels, and Y is the oracle's within
    the bar."""
    rng = np.random.default_rng(2024)
    for case in range(24):
        M = int(rng.integers(1, 65))
        G = int(rng.choice([8, 10, 12, 14, 16, 18, 22, 26, 30]))
        K = 128 * G
        N = int(rng.integers(1, 700))
        print(f"[case] random decode GEMM {case}: M={M} K={K} N={N}", flush=True)
        lin = _rand_linear(M, K, N, 128, seed=1000 + case, norm=False)
        gw = gpu_quantize_weight(lin)
        qa = atom.atom_quantize_act(dev(lin.x), None, 0.0, dev(lin.idx), 128, 128, lin.clip_act)
        t4, t8 = atom.atom_tile_weight_decode(gw[0], gw[1])
        y = atom.atom_w4a4_gemm(*qa, *gw)
        yt = atom.atom_w4a4_gemm_decode_tiled(*qa, t4, t8, gw[2])
        torch.cuda.synchronize()
        assert torch.equal(y, yt), f"case {case}: tiled and canonical weights differ"
        ref = oracle.w4a4_gemm(*ref_quantize_act(lin), *ref_quantize_weight(lin), 128)
        assert y_rel_err(npy(yt), ref["y"]) <= Y_TOL, f"case {case}"


def test_decode_gemm_random_shapes_up_to_256_rows():
    """The same for 65 to 256 rows (blocks of 64 rows along the grid's second dimension) and up to
    4200 output channels (one or two channel blocks per workgroup)."""
    rng = np.random.default_rng(2025)
    for case in range(8):
        M = int(rng.integers(65, 257))
        G = int(rng.choice([8, 10, 14, 16, 22]))
        K = 128 * G
        N = int(rng.integers(1, 4200))
        print(f"[case] random decode GEMM, many rows {case}: M={M} K={K} N={N}", flush=True)
        lin = _rand_linear(M, K, N, 128, seed=3000 + case, norm=False)
        gw = gpu_quantize_weight(lin)
        qa = atom.atom_quantize_act(dev(lin.x), None, 0.0, dev(lin.idx), 128, 128, lin.clip_act)
        t4, t8 = atom.atom_tile_weight_decode(gw[0], gw[1])
        y = atom.atom_w4a4_gemm(*qa, *gw)
        yt = atom.atom_w4a4_gemm_decode_tiled(*qa, t4, t8, gw[2])
        torch.cuda.synchronize()
        ref = oracle.w4a4_gemm(*ref_quantize_act(lin), *ref_quantize_weight(lin), 128)
        assert y_rel_err(npy(yt), ref["y"]) <= Y_TOL, f"case {case}"
        assert y_rel_err(npy(y), ref["y"]) <= Y_TOL, f"case {case} (canonical weights)"

