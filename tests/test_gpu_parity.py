"""GPU parity: the HIP library (through the C ABI) against the CPU oracle on the
same seeded inputs.  Codes, scales and per-group int32 partials must be
bit-identical; fp16 outputs within 1e-3 max relative error."""
import numpy as np
import pytest
import torch

import oracle
import paper_2310_19102_amd as atom
from paper_2310_19102_amd import synth
from _gpu_util import (Y_TOL, assert_quant_equal, dev, gpu_quantize_act, gpu_quantize_weight, npy,
                       ref_quantize_act, ref_quantize_weight, y_rel_err)

pytestmark = pytest.mark.gpu


def _rand_linear(M, K, N, O, seed, norm=True):
    g = torch.Generator().manual_seed(seed)
    sigma = torch.exp(1.5 * torch.randn(K, generator=g))
    x = (torch.randn((M, K), generator=g) * sigma).to(torch.float16)
    w = (0.02 * torch.randn((N, K), generator=g)).to(torch.float16)
    gamma = (1 + 0.1 * torch.randn(K, generator=g)).to(torch.float16) if norm else None
    idx = torch.argsort(sigma, stable=True).to(torch.int32)
    return synth.Linear("rand", x, w, gamma, idx, n_outlier=O)


def _check_linear(lin, what, full_partials=True):
    print(f"[case] {what}: M={lin.M} K={lin.K} N={lin.N} O={lin.n_outlier} "
          f"norm={lin.gamma is not None}", flush=True)
    ga = gpu_quantize_act(lin)
    ra = ref_quantize_act(lin)
    assert_quant_equal(ga, ra, what + " act")
    gw = gpu_quantize_weight(lin)
    rw = ref_quantize_weight(lin)
    assert_quant_equal(gw, rw, what + " weight")
    G = lin.K // lin.group_size
    ref = oracle.w4a4_gemm(*ra, *rw, lin.group_size, want_partials=full_partials)
    # plain call
    y = atom.atom_w4a4_gemm(*ga, *gw, lin.group_size)
    torch.cuda.synchronize()
    err = y_rel_err(npy(y), ref["y"])
    assert err <= Y_TOL, f"{what}: Y rel err {err}"
    if full_partials:
        part = torch.empty((lin.M, lin.N, G), dtype=torch.int32, device="cuda")
        y2 = atom.atom_w4a4_gemm(*ga, *gw, lin.group_size, partials=part)
        torch.cuda.synchronize()
        assert np.array_equal(npy(part), ref["partials"]), f"{what}: int32 partials differ"
        assert y_rel_err(npy(y2), ref["y"]) <= Y_TOL
    return err


def test_config1_tiny():
    _check_linear(synth.make(1), "config1")


@pytest.mark.parametrize("M,K,N,O,norm", [
    (1, 512, 64, 128, True),       # single token
    (3, 256, 40, 128, False),      # one INT4 + one INT8 group, ragged N
    (33, 1024, 200, 256, True),    # two INT8 groups, ragged M and N
    (70, 1408, 130, 128, True),    # K/128 = 11: ragged last 4-group sweep of the front end
    (130, 768, 257, 128, False),   # spans two 128-row tiles with a 2-row tail
    (257, 512, 129, 384, True),    # O > K4
    (8, 1408, 100, 128, True),     # decode kernel: 11 groups over 8 K-slices, ragged N
    (17, 896, 48, 256, False),     # decode kernel, two row blocks, two INT8 groups
    (40, 640, 33, 128, True),      # decode kernel, four row blocks; fewer groups than slices
    (64, 2304, 16, 128, True),     # decode kernel at its largest M, several load batches
    (65, 384, 72, 128, True),      # smallest M of the big-tile kernel
    (70, 256, 130, 128, False),    # two wavefront sets, three K-steps: one set gets a single step
    (200, 1152, 300, 256, True),   # two wavefront sets, two INT8 groups, odd/even split of the steps
    (1200, 256, 3000, 128, False), # 128x128 tiles, one set, minimal K (one INT4 + one INT8 group)
    (5, 12416, 24, 128, True),     # front end with eight register sets of gather offsets (K > 12288)
    (520, 28672, 24, 128, True),   # front end on 1024 threads per row (K > 16384), several rows per workgroup
    (8, 11008, 40, 128, False),    # decode kernel at the Llama-7B down projection: 86 groups = 21.5 blocks of four
    (16, 5120, 48, 128, True),     # 40 groups (Llama-13B): five blocks over eight wavefronts, three of them idle
    (40, 2560, 32, 128, True),     # four row blocks, 20 groups
    (24, 768, 20, 256, True),      # two INT8 groups: the general slots with the blocked runs (6 groups, 2 blocks)
    (100, 256, 200, 128, True),    # 64 x 64 tiles, four wavefront sets and two groups: two sets stay empty
    (130, 640, 136, 256, False),   # four sets on five groups (1, 1, 1, 2), two of them INT8, ragged tile edges
    (320, 1024, 3500, 128, True),  # 275 tiles of 64 x 64: two wavefront sets per workgroup
    (260, 512, 4200, 256, False),  # two sets, four groups: set 0 the INT4 pair, set 1 the INT8 pair
    (5000, 256, 24, 128, True),    # tall and narrow: 79 row tiles of one partial 64 x 32 column tile
    (48, 384, 4200, 128, False),   # 33..64 rows, just over 4096 output channels: 64 x 32 tiles, ragged in M and N
    (48, 384, 8200, 128, False),   # 33..64 rows and many output channels: the big-tile kernel on one partial row tile
    (200, 4096, 300, 128, True),   # six tiles of the big-tile kernel at the Llama-7B K (33 K-steps, two wavefront sets)
    (300, 2048, 1000, 256, False), # 24 tiles, 18 K-steps, two INT8 groups, ragged edges
])
def test_ragged_shapes(M, K, N, O, norm):
    _check_linear(_rand_linear(M, K, N, O, seed=M * 1000 + N, norm=norm), f"ragged M{M}")


def test_degenerate_values():
    """Zero rows (scale 0 -> codes 0), a row of fp16 max, subnormal rows."""
    lin = _rand_linear(8, 512, 64, 128, seed=5, norm=False)
    lin.x[0] = 0
    lin.x[1] = 65504.0
    lin.x[2] = torch.tensor(6e-8, dtype=torch.float16)
    lin.x[3, ::2] = 0
    lin.w[0] = 0
    _check_linear(lin, "degenerate")
    lin2 = _rand_linear(4, 512, 64, 128, seed=6, norm=True)
    lin2.x[1] = 65504.0           # sum of squares 2.2e12: fine in fp32
    lin2.x[2] = torch.tensor(6e-8, dtype=torch.float16)
    _check_linear(lin2, "degenerate-norm")


def test_front_end_plain_and_fast_kernels_agree():
    """The front end has a fast kernel (shared reciprocal refinement for the division) and a
    plain one (compiler-generated IEEE division) that takes over for clip < 2^-20; both must give the oracle's codes and scales, whose division is the C
    compiler's.  Values chosen so that quotients land on and next to rounding ties."""
    lin = _rand_linear(6, 1024, 32, 128, seed=11, norm=False)
    # rows of exact multiples of half a quantisation step: every quotient is a tie or an integer
    step = torch.tensor(0.75, dtype=torch.float16)
    lin.x[0] = (torch.arange(1024) % 31 - 15).to(torch.float16) * step * 0.5
    lin.x[1] = lin.x[0] * torch.tensor(1.0009765625, dtype=torch.float16)   # one fp16 ulp off
    for clip in (0.9, 1.0, 2.0 ** -20, 5e-7, 1e-9):
        lin.clip_act = clip
        ga = gpu_quantize_act(lin)
        assert_quant_equal(ga, ref_quantize_act(lin), f"clip {clip}")


@pytest.mark.parametrize("M,K,O,norm,clip", [
    (7, 512, 128, True, 0.9),        # one register set of gather offsets
    (33, 4096, 128, True, 0.9),      # the Llama-7B hidden size
    (9, 11008, 128, False, 0.9),     # 512 threads per row
    (3000, 512, 256, True, 1.0),     # several rows per workgroup: the next row is prefetched
    (4, 20480, 128, True, 0.9),      # K > 16384: 1024 threads per row, three register sets
    (530, 28672, 128, True, 0.9),    # the Llama-70B intermediate size, four sets, rows prefetched
    (5, 1024, 128, False, 1e-8),     # clip below 2^-20: the plain kernel
])
def test_add_quantize_act(M, K, O, norm, clip):
    """Residual add fused in front of the front end: the fp16 sum, the codes and the scales
    are bit-exact against the oracle; in place on either input gives the same."""
    g = torch.Generator().manual_seed(M * 7 + K)
    sigma = torch.exp(1.5 * torch.randn(K, generator=g))
    x = (torch.randn((M, K), generator=g) * sigma).to(torch.float16)
    res = (torch.randn((M, K), generator=g) * sigma * 0.7).to(torch.float16)
    res[0, :16] = -x[0, :16]                                  # exact cancellation
    gamma = (1 + 0.1 * torch.randn(K, generator=g)).to(torch.float16) if norm else None
    idx = torch.argsort(sigma, stable=True).to(torch.int32)
    eps = 1e-6 if norm else 0.0
    print(f"[case] add+quantize M={M} K={K} O={O} norm={norm} clip={clip}", flush=True)
    want = oracle.add_quantize_act(x.numpy(), res.numpy(), None if gamma is None else gamma.numpy(),
                                   eps, idx.numpy(), 128, O, clip)
    xd, rd = dev(x), dev(res)
    h, q4, q8, sc = atom.atom_add_quantize_act(xd, rd, dev(gamma), eps, dev(idx), 128, O, clip)
    torch.cuda.synchronize()
    assert np.array_equal(npy(h).view(np.uint16), want[0].view(np.uint16)), "sum differs"
    assert_quant_equal((q4, q8, sc), want[1:], "add+quantize")
    assert np.array_equal(npy(xd).view(np.uint16), x.numpy().view(np.uint16)), "input was modified"
    # in place on the residual (the usual use), then on x
    for target in ("residual", "x"):
        xd, rd = dev(x), dev(res)
        t = rd if target == "residual" else xd
        h2, q4, q8, sc = atom.atom_add_quantize_act(xd, rd, dev(gamma), eps, dev(idx), 128, O, clip,
                                                    sum_out=t)
        torch.cuda.synchronize()
        assert h2.data_ptr() == t.data_ptr()
        assert np.array_equal(npy(t).view(np.uint16), want[0].view(np.uint16)), f"in place on {target}"
        assert_quant_equal((q4, q8, sc), want[1:], f"in place on {target}")


def test_add_quantize_act_strided_and_errors():
    K = 512
    g = torch.Generator().manual_seed(3)
    x = torch.randn((6, K), generator=g).to(torch.float16)
    res = torch.randn((6, K), generator=g).to(torch.float16)
    idx = torch.randperm(K, generator=g).to(torch.int32)
    want = oracle.add_quantize_act(x.numpy(), res.numpy(), None, 0.0, idx.numpy(), 128, 128, 0.9)
    bx = torch.zeros((6, 2 * K), dtype=torch.float16); bx[:, :K] = x
    br = torch.zeros((6, 3 * K), dtype=torch.float16); br[:, K:2 * K] = res
    bo = torch.zeros((6, 2 * K), dtype=torch.float16).cuda()
    h, q4, q8, sc = atom.atom_add_quantize_act(bx.cuda()[:, :K], br.cuda()[:, K:2 * K], None, 0.0,
                                               dev(idx), sum_out=bo[:, K:])
    torch.cuda.synchronize()
    assert np.array_equal(npy(bo[:, K:]).view(np.uint16), want[0].view(np.uint16))
    assert not npy(bo[:, :K]).any()                              # nothing written outside
    assert_quant_equal((q4, q8, sc), want[1:], "strided add")
    # empty call, and a residual row stride that breaks the 16-byte alignment
    e = atom.atom_add_quantize_act(dev(x[:0]), dev(res[:0]), None, 0.0, dev(idx))
    assert e[0].shape[0] == 0 and e[1].shape[0] == 0
    odd = torch.zeros((6, K + 4), dtype=torch.float16).cuda()[:, :K]
    with pytest.raises(atom.AtomError) as err:
        atom.atom_add_quantize_act(dev(x), odd, None, 0.0, dev(idx))
    assert err.value.status == 4


@pytest.mark.parametrize("M,K,O,clip", [
    (7, 512, 128, 0.9),
    (33, 11008, 128, 0.9),           # the Llama-7B intermediate size, 512 threads per row
    (3000, 256, 128, 1.0),           # several rows per workgroup
    (4, 20480, 256, 0.9),            # K > 16384: 1024 threads per row, three register sets
    (530, 28672, 128, 0.9),          # the Llama-70B intermediate size, four sets, rows prefetched
    (5, 1024, 128, 1e-8),            # clip below 2^-20: the plain kernel
])
def test_swiglu_quantize_act(M, K, O, clip):
    """silu(gate)*up fused in front of the front end; gate and up are the two halves of one
    [M, 2K] matrix, as the fused gate/up projection leaves them.  Codes and scales are
    bit-exact against the oracle, whose exp is the same fixed sequence of IEEE operations."""
    g = torch.Generator().manual_seed(M * 13 + K)
    sigma = torch.exp(1.0 * torch.randn(K, generator=g))
    gu = torch.empty((M, 2 * K), dtype=torch.float16)
    gu[:, :K] = (3.0 * torch.randn((M, K), generator=g)).to(torch.float16)
    gu[:, K:] = (torch.randn((M, K), generator=g) * sigma).to(torch.float16)
    # gates that exercise the clamp, sigma == 1, zero, and the largest fp16 values
    gu[0, :8] = torch.tensor([-65504.0, -100.0, -87.5, -20.0, 0.0, 20.0, 100.0, 65504.0]).to(torch.float16)
    gu[0, K:K + 8] = torch.tensor([1.0, -2.0, 3.0, 0.5, 7.0, 1.0, -0.25, 0.001]).to(torch.float16)
    idx = torch.argsort(sigma, stable=True).to(torch.int32)
    print(f"[case] swiglu+quantize M={M} K={K} O={O} clip={clip}", flush=True)
    want = oracle.swiglu_quantize_act(gu[:, :K].numpy(), gu[:, K:].numpy(), idx.numpy(), 128, O, clip)
    gud = gu.cuda()
    got = atom.atom_swiglu_quantize_act(gud[:, :K], gud[:, K:], dev(idx), 128, O, clip)
    torch.cuda.synchronize()
    assert_quant_equal(got, want, "swiglu+quantize")
    assert np.array_equal(npy(gud).view(np.uint16), gu.numpy().view(np.uint16)), "inputs were modified"


def test_swiglu_quantize_act_errors():
    K = 512
    gate = torch.zeros((4, K), dtype=torch.float16).cuda()
    idx = torch.arange(K, dtype=torch.int32).cuda()
    e = atom.atom_swiglu_quantize_act(gate[:0], gate[:0], idx)
    assert e[0].shape[0] == 0
    odd = torch.zeros((4, K + 4), dtype=torch.float16).cuda()[:, :K]      # row stride not a multiple of 8
    with pytest.raises(atom.AtomError) as err:
        atom.atom_swiglu_quantize_act(gate, odd, idx)
    assert err.value.status == 4
    with pytest.raises(ValueError):
        atom.atom_swiglu_quantize_act(gate, gate[:, :256], idx)


def test_strided_input_rows():
    lin = _rand_linear(16, 512, 64, 128, seed=7)
    big = torch.zeros((16, 1024), dtype=torch.float16)
    big[:, :512] = lin.x
    xs = big.cuda()[:, :512]              # ldx = 1024
    q = atom.atom_quantize_act(xs, dev(lin.gamma), lin.eps, dev(lin.idx), 128, 128, lin.clip_act)
    torch.cuda.synchronize()
    assert_quant_equal(q, ref_quantize_act(lin), "strided")


def test_empty_and_error_paths():
    lin = _rand_linear(4, 512, 64, 128, seed=8)
    q = atom.atom_quantize_act(dev(lin.x[:0]), dev(lin.gamma), lin.eps, dev(lin.idx))
    assert q[0].shape[0] == 0
    with pytest.raises(atom.AtomError) as e:
        atom.atom_quantize_act(dev(lin.x[:, :500].contiguous()), None, 0.0, dev(lin.idx[:500]))
    assert e.value.status == 2          # K % 128 != 0
    with pytest.raises(atom.AtomError) as e:
        atom.atom_quantize_act(dev(lin.x), None, 0.0, dev(lin.idx), group_size=32)
    assert e.value.status == 3


def test_run_twice_is_deterministic():
    lin = synth.make(2, 0, M=64)
    ga = gpu_quantize_act(lin)
    gw = gpu_quantize_weight(lin)
    y1 = atom.atom_w4a4_gemm(*ga, *gw)
    y2 = atom.atom_w4a4_gemm(*ga, *gw)
    torch.cuda.synchronize()
    assert torch.equal(y1, y2)


@pytest.mark.parametrize("K", [1024, 768, 1280])        # 8 groups (whole blocks of four), 6 and 10 (a half block last)
@pytest.mark.parametrize("shift", [1, 2, 4])            # scale arrays 2, 4 and 8 bytes off a 16-byte boundary
def test_decode_gemm_scale_alignment(K, shift):
    """The decode kernel picks its scale loads (8-byte, 4-byte, 2-byte) by the alignment of the
    scale arrays and by the group count: every choice gives the same result."""
    lin = _rand_linear(24, K, 72, 128, seed=60 + K + shift)
    print(f"[case] scale alignment: K={K} shift={shift}", flush=True)
    ga = gpu_quantize_act(lin)
    gw = gpu_quantize_weight(lin)
    y0 = atom.atom_w4a4_gemm(*ga, *gw)

    def moved(sc):
        buf = torch.zeros(sc.numel() + 8, dtype=sc.dtype, device=sc.device)
        off = (-(buf.data_ptr() // 2) % 8 + shift) % 8  # elements to the wanted misalignment
        v = buf[off:off + sc.numel()].view(sc.shape)
        v.copy_(sc)
        assert v.data_ptr() % 16 == 2 * shift
        return v
    y1 = atom.atom_w4a4_gemm(ga[0], ga[1], moved(ga[2]), gw[0], gw[1], moved(gw[2]))
    torch.cuda.synchronize()
    ref = oracle.w4a4_gemm(*ref_quantize_act(lin), *ref_quantize_weight(lin), lin.group_size, want_partials=False)
    assert y_rel_err(npy(y0), ref["y"]) <= Y_TOL
    assert y_rel_err(npy(y1), ref["y"]) <= Y_TOL


@pytest.mark.parametrize("M,N,norm", [(3, 40, True), (70, 24, False)])
def test_maximum_k(M, N, norm):
    """K = 32768, the largest the library takes (256 groups): front end with the whole fp32
    row staged, decode kernel (M = 3) and few-tile kernel (M = 70) on the longest chains."""
    _check_linear(_rand_linear(M, 32768, N, 128, seed=91 + M, norm=norm), f"K=32768 M={M}")
    lin = _rand_linear(2, 32768 + 128, 8, 128, seed=5, norm=False)
    with pytest.raises(atom.AtomError) as e:
        atom.atom_quantize_act(dev(lin.x), None, 0.0, dev(lin.idx))
    assert e.value.status == 3          # K above the limit: unsupported, nothing launched


@pytest.mark.parametrize("which", [0, 1])
def test_config2_llama7b_attention(which):
    _check_linear(synth.make(2, which), f"config2[{which}]", full_partials=(which == 0))


@pytest.mark.parametrize("which", range(8))
def test_config3_decode(which):
    _check_linear(synth.make(3, which), f"config3[{which}]", full_partials=True)


def _check_sampled(lin, what, n_rows=48):
    """Full-size launch on the GPU; the oracle runs the front end in full and
    the GEMM on a seeded sample of rows."""
    print(f"[case] {what}: M={lin.M} K={lin.K} N={lin.N}", flush=True)
    ga = gpu_quantize_act(lin)
    assert_quant_equal(ga, ref_quantize_act(lin), what + " act")
    gw = gpu_quantize_weight(lin)
    rw = ref_quantize_weight(lin)
    assert_quant_equal(gw, rw, what + " weight")
    y = atom.atom_w4a4_gemm(*ga, *gw, lin.group_size)
    torch.cuda.synchronize()
    rng = np.random.default_rng(lin.M + lin.N)
    rows = np.unique(np.concatenate([[0, lin.M - 1], rng.integers(0, lin.M, n_rows)]))
    ra = ref_quantize_act(lin, rows=torch.from_numpy(rows))
    G = lin.K // lin.group_size
    ncols = min(lin.N, 2048)               # partial dumps on a column band keep the oracle quick
    c0 = int(rng.integers(0, lin.N - ncols + 1))
    ref = oracle.w4a4_gemm(*ra, *rw, lin.group_size)
    err = y_rel_err(npy(y)[rows], ref["y"])
    assert err <= Y_TOL, f"{what}: sampled rows rel err {err}"
    # partials through a sub-problem call: the sampled rows against a band of W
    sub_a = tuple(t[torch.from_numpy(rows).cuda()].contiguous() for t in ga)
    sub_w = tuple(t[c0:c0 + ncols].contiguous() for t in gw)
    part = torch.empty((len(rows), ncols, G), dtype=torch.int32, device="cuda")
    atom.atom_w4a4_gemm(*sub_a, *sub_w, lin.group_size, partials=part)
    torch.cuda.synchronize()
    refp = oracle.w4a4_gemm(*ra, *(t[c0:c0 + ncols] for t in rw), lin.group_size,
                            want_partials=True)
    assert np.array_equal(npy(part), refp["partials"]), f"{what}: partials differ"


@pytest.mark.parametrize("which", [0, 1])
def test_config4_llama7b_mlp(which):
    _check_sampled(synth.make(4, which), f"config4[{which}]")


@pytest.mark.parametrize("which", [0, 1, 2])
def test_config5_llama70b(which):
    _check_sampled(synth.make(5, which), f"config5[{which}]", n_rows=16)
