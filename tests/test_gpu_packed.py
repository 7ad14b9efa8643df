"""GPU parity of the GEMM on packed (tiled, FP6-carried) weights: atom_pack_weight +
atom_w4a4_gemm_packed against the CPU oracle.  The INT4 codes are re-encoded, not re-quantised, so
the per-group integer sums must equal the oracle's bit for bit, and since the kernel adds the
groups in the oracle's order (one ascending chain of fused multiply-adds) so must Y."""
import numpy as np
import pytest
import torch

import oracle
import paper_2310_19102_amd as atom
from paper_2310_19102_amd import synth
from _gpu_util import (Y_TOL, dev, gpu_quantize_act, gpu_quantize_weight, npy, ref_quantize_act,
                       ref_quantize_weight, y_rel_err)
from test_gpu_parity import _rand_linear

pytestmark = pytest.mark.gpu


def _check_packed(lin, what, partials=True):
    print(f"[case] packed {what}: M={lin.M} K={lin.K} N={lin.N} O={lin.n_outlier}", flush=True)
    ga, gw = gpu_quantize_act(lin), gpu_quantize_weight(lin)
    ra, rw = ref_quantize_act(lin), ref_quantize_weight(lin)
    wp = atom.atom_pack_weight(*gw, lin.group_size)
    ref = oracle.w4a4_gemm(*ra, *rw, lin.group_size, want_partials=partials)
    y = atom.atom_w4a4_gemm_packed(*ga, wp, lin.N, lin.group_size)
    torch.cuda.synchronize()
    err = y_rel_err(npy(y), ref["y"])
    assert err <= Y_TOL, f"{what}: Y rel err {err}"
    assert np.array_equal(npy(y).view(np.uint16), ref["y"].view(np.uint16)), f"{what}: Y not bit-identical"
    if partials:
        G = lin.K // lin.group_size
        part = torch.empty((lin.M, lin.N, G), dtype=torch.int32, device="cuda")
        y2 = atom.atom_w4a4_gemm_packed(*ga, wp, lin.N, lin.group_size, partials=part)
        torch.cuda.synchronize()
        assert np.array_equal(npy(part), ref["partials"]), f"{what}: int32 partials differ"
        assert np.array_equal(npy(y2).view(np.uint16), ref["y"].view(np.uint16))


@pytest.mark.parametrize("M,K,N,O,norm", [
    (300, 512, 200, 128, True),     # three INT4 groups: fewer than the LDS stages; ragged M and N
    (257, 256, 129, 128, False),    # one INT4 group; a second row tile with one valid row
    (130, 640, 136, 256, False),    # two INT8 groups
    (1024, 1024, 384, 128, True),   # whole tiles, seven INT4 groups
    (100, 384, 130, 128, True),     # 65..128 rows: the 128-row tile
    (40, 384, 70, 128, False),      # at most 64 rows: the 64-row tile
    (1, 256, 8, 128, True),         # a single row and eight columns
    (640, 4096, 520, 128, True),    # the Llama-7B K: 31 INT4 groups through the stage ring
    (2300, 1280, 1100, 128, False), # nine row tiles (two bands of the tile order), nine column tiles
    (2100, 1024, 14600, 128, False),# 1035 tiles of 256 rows: workgroups that walk several tiles; a last row tile with
                                    # one unit, a last column tile with one unit and 8 columns, seven INT4 groups
    (4096, 1408, 8192, 128, True),  # the same with whole tiles and ten INT4 groups
])
def test_packed_gemm(M, K, N, O, norm):
    # (the dump of the integer sums of the two largest cases would take a gigabyte; their sums are
    # checked through Y, which must be bit-identical)
    _check_packed(_rand_linear(M, K, N, O, seed=7 * M + N, norm=norm), f"M{M}", partials=M * N < (1 << 24))


def test_packed_gemm_extreme_codes():
    """Every INT4 code -8 (the one value whose square reaches the largest group sum, 8192) and
    mixed +7 / -8 rows; INT8 codes at -128 and 127."""
    M, K, N, O = 96, 512, 80, 128
    g = torch.Generator().manual_seed(5)
    K4, G = K - O, K // 128
    a4 = torch.full((M, K4 // 2), 0x88, dtype=torch.uint8)
    w4 = torch.full((N, K4 // 2), 0x88, dtype=torch.uint8)
    a4[1::2] = torch.randint(0, 2, (M // 2, K4 // 2), generator=g).to(torch.uint8) * 0x0F + 0x78   # 0x78 or 0x87
    w4[1::3] = 0x77
    a8 = torch.where(torch.rand((M, O), generator=g) < 0.5, -128, 127).to(torch.int8)
    w8 = torch.where(torch.rand((N, O), generator=g) < 0.5, -128, 127).to(torch.int8)
    asc = torch.full((M, G), 2.0 ** -6, dtype=torch.float16)
    wsc = torch.full((N, G), 2.0 ** -7, dtype=torch.float16)
    ref = oracle.w4a4_gemm(a4.numpy(), a8.numpy(), asc.numpy(), w4.numpy(), w8.numpy(), wsc.numpy(), 128, want_partials=True)
    wp = atom.atom_pack_weight(dev(w4), dev(w8), dev(wsc))
    part = torch.empty((M, N, G), dtype=torch.int32, device="cuda")
    y = atom.atom_w4a4_gemm_packed(dev(a4), dev(a8), dev(asc), wp, N, partials=part)
    y1 = atom.atom_w4a4_gemm_packed(dev(a4), dev(a8), dev(asc), wp, N)
    torch.cuda.synchronize()
    assert ref["partials"][..., :3].max() == 8 * 8 * 128          # the largest INT4 group sum there is
    assert np.array_equal(npy(part), ref["partials"])
    assert np.array_equal(npy(y).view(np.uint16), ref["y"].view(np.uint16))
    assert np.array_equal(npy(y1).view(np.uint16), ref["y"].view(np.uint16))


def test_packed_gemm_w3a3():
    lin = _rand_linear(200, 640, 150, 128, seed=33)
    ga = atom.atom_quantize_act(dev(lin.x), dev(lin.gamma), lin.eps, dev(lin.idx), 128, 128, lin.clip_act, bits=3)
    gw = atom.atom_quantize_weight(dev(lin.w), dev(lin.idx), 128, 128, lin.clip_weight, bits=3)
    ra = oracle.quantize_act(lin.x.numpy(), lin.gamma.numpy(), lin.eps, lin.idx.numpy(), 128, 128, lin.clip_act, bits=3)
    rw = oracle.quantize_weight(lin.w.numpy(), lin.idx.numpy(), 128, 128, lin.clip_weight, bits=3)
    ref = oracle.w4a4_gemm(*ra, *rw, 128)
    y = atom.atom_w4a4_gemm_packed(*ga, atom.atom_pack_weight(*gw), lin.N)
    torch.cuda.synchronize()
    assert np.array_equal(npy(y).view(np.uint16), ref["y"].view(np.uint16))


def test_packed_gemm_strided_output_and_errors():
    lin = _rand_linear(70, 256, 40, 128, seed=3)
    ga, gw = gpu_quantize_act(lin), gpu_quantize_weight(lin)
    wp = atom.atom_pack_weight(*gw)
    ref = oracle.w4a4_gemm(*ref_quantize_act(lin), *ref_quantize_weight(lin), 128)
    big = torch.full((70, 100), 7.0, dtype=torch.float16, device="cuda")
    atom.atom_w4a4_gemm_packed(*ga, wp, lin.N, out=big[:, 8:48])
    torch.cuda.synchronize()
    assert np.array_equal(npy(big[:, 8:48]).view(np.uint16), ref["y"].view(np.uint16))
    assert (npy(big[:, :8]) == 7).all() and (npy(big[:, 48:]) == 7).all()      # nothing written outside
    small = torch.empty(256, dtype=torch.uint8, device="cuda")
    with pytest.raises(atom.AtomError) as e:                                   # packed buffer too small
        atom.atom_pack_weight(*gw, out=small)
    assert e.value.status == 5


def test_packed_gemm_many_tiles_strided_and_unaligned_output():
    """1032 tiles of 256 rows (workgroups that walk several tiles) with an output whose rows are
    not 16-byte aligned: every wavefront takes the conditional store path, tile after tile.  Same bits
    as the contiguous output, nothing written outside."""
    lin = _rand_linear(2048, 1024, 16500, 128, seed=11, norm=False)
    print(f"[case] packed, many tiles, strided output: M={lin.M} K={lin.K} N={lin.N}", flush=True)
    ga, gw = gpu_quantize_act(lin), gpu_quantize_weight(lin)
    wp = atom.atom_pack_weight(*gw)
    y = atom.atom_w4a4_gemm_packed(*ga, wp, lin.N)
    big = torch.full((lin.M, lin.N + 13), 7.0, dtype=torch.float16, device="cuda")
    atom.atom_w4a4_gemm_packed(*ga, wp, lin.N, out=big[:, 5:5 + lin.N])
    torch.cuda.synchronize()
    assert torch.equal(big[:, 5:5 + lin.N], y)
    assert bool((big[:, :5] == 7).all()) and bool((big[:, 5 + lin.N:] == 7).all())
    rows = np.array([0, 255, 256, 1000, 2047])
    ref = oracle.w4a4_gemm(*ref_quantize_act(lin, rows=torch.from_numpy(rows)), *ref_quantize_weight(lin), 128)
    assert np.array_equal(npy(y)[rows].view(np.uint16), ref["y"].view(np.uint16))


def test_packed_gemm_many_tiles_random_shapes():
    """Seeded random problems of 1024 and more tiles of 256 rows (one workgroup per CU walks them): Y
    must be the bits of the instantiation that also dumps the integer sums, which runs one
    workgroup per tile and is held against the oracle by the tests above.  Random codes and
    scales; ragged M and N, odd unit counts, seven to eleven INT4 groups."""
    rng = np.random.default_rng(77)
    g = torch.Generator(device="cuda").manual_seed(77)
    for case in range(6):
        G = int(rng.integers(8, 13))
        K, O = 128 * G, 128
        mt = int(rng.integers(5, 12))                                   # row tiles of 256
        M = 256 * mt - int(rng.integers(0, 256))
        nt = -(-1024 // mt) + int(rng.integers(0, 40))                  # column tiles of 128
        N = 128 * nt - int(rng.integers(0, 128))
        print(f"[case] packed, many tiles, random {case}: M={M} K={K} N={N}", flush=True)
        a = (torch.randint(0, 256, (M, (K - O) // 2), dtype=torch.uint8, device="cuda", generator=g),
             torch.randint(-128, 128, (M, O), dtype=torch.int8, device="cuda", generator=g),
             (torch.rand((M, G), device="cuda", generator=g) * 0.01 + 0.001).half())
        w = (torch.randint(0, 256, (N, (K - O) // 2), dtype=torch.uint8, device="cuda", generator=g),
             torch.randint(-128, 128, (N, O), dtype=torch.int8, device="cuda", generator=g),
             (torch.rand((N, G), device="cuda", generator=g) * 0.01 + 0.001).half())
        wp = atom.atom_pack_weight(*w)
        y = atom.atom_w4a4_gemm_packed(*a, wp, N)
        part = torch.empty((M, N, G), dtype=torch.int32, device="cuda")
        y2 = atom.atom_w4a4_gemm_packed(*a, wp, N, partials=part)
        torch.cuda.synchronize()
        assert torch.equal(y, y2), f"case {case}"
        del part, y, y2, wp, a, w
        torch.cuda.empty_cache()


@pytest.mark.parametrize("which", [0, 1])
def test_packed_config4(which):
    """Full-size Llama-7B MLP launches; sampled rows against the oracle, bit for bit."""
    lin = synth.make(4, which)
    print(f"[case] packed config4[{which}]: M={lin.M} K={lin.K} N={lin.N}", flush=True)
    ga, gw = gpu_quantize_act(lin), gpu_quantize_weight(lin)
    rw = ref_quantize_weight(lin)
    y = atom.atom_w4a4_gemm_packed(*ga, atom.atom_pack_weight(*gw), lin.N)
    torch.cuda.synchronize()
    # one row of every 32-row sub-tile of the first and of the last 256-row tile, plus random rows
    rng = np.random.default_rng(4 + which)
    rows = np.unique(np.concatenate([np.arange(0, 256, 32) + rng.integers(0, 32, 8),
                                     lin.M - 256 + np.arange(0, 256, 32) + rng.integers(0, 32, 8),
                                     rng.integers(0, lin.M, 8)]))
    ra = ref_quantize_act(lin, rows=torch.from_numpy(rows))
    ref = oracle.w4a4_gemm(*ra, *rw, lin.group_size)
    assert np.array_equal(npy(y)[rows].view(np.uint16), ref["y"].view(np.uint16))
