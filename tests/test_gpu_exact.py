"""Bit-exact checks that reach the kernels production calls run (no debug instantiation).

Two constructions on synthetic codes and scales, at the shapes that select every instantiation of
the group GEMM (Section 4.2, steps 1-3) and at the full benchmark sizes:

* one active group: a_scale is 1 in group g and 0 elsewhere, w_scale is 1, so
  Y[m, n] = fp16(P[m, n, g]); one launch per group.  |P| < 2048 is exact in fp16, so any wrong code,
  dropped byte or misplaced channel in group g of the production kernel shows as a wrong integer
  (larger sums are compared after the same fp16 rounding);
* power-of-two scales: every product and every partial sum of the fp32 accumulation is exact
  whatever the order of the additions (split-K trees included), so Y must equal the oracle's Y bit
  for bit.
The oracle computes the sampled rows and column bands; the GPU runs the whole problem."""
import numpy as np
import pytest
import torch

import oracle
import paper_2310_19102_amd as atom
from _gpu_util import npy

pytestmark = pytest.mark.gpu


def _codes(rows, K, O, rng, small8):
    q4 = rng.integers(0, 256, (rows, (K - O) // 2), dtype=np.uint8)
    lo, hi = (-8, 8) if small8 else (-128, 128)
    q8 = rng.integers(lo, hi, (rows, O), dtype=np.int64).astype(np.int8)
    return q4, q8


def _sample(M, N, rng):
    """Rows: one in every 32-row sub-tile of the first and of the last 256 rows, plus random ones.
    Columns: the first and the last 128 and a random aligned block of 128."""
    def pick(n, count):
        first = [min(n - 1, 32 * i + int(rng.integers(0, 32))) for i in range(8)]
        last = [max(0, n - 256 + 32 * i + int(rng.integers(0, 32))) for i in range(8)]
        return np.unique(np.concatenate([first, last, [0, n - 1], rng.integers(0, n, count)]))
    rows = pick(M, 6)
    blk = int(rng.integers(0, max(1, N // 128))) * 128
    cols = np.unique(np.concatenate([np.arange(0, min(128, N)), np.arange(max(0, N - 128), N),
                                     np.arange(blk, min(blk + 128, N))]))
    return rows, cols


class _Problem:
    def __init__(self, M, K, N, O, seed, small8=True):
        rng = np.random.default_rng(seed)
        self.M, self.K, self.N, self.O, self.G = M, K, N, O, K // 128
        self.a4, self.a8 = _codes(M, K, O, rng, small8)
        self.w4, self.w8 = _codes(N, K, O, rng, small8)
        self.rows, self.cols = _sample(M, N, rng)
        self.rng = rng
        self.dev = [torch.from_numpy(t).cuda() for t in (self.a4, self.a8, self.w4, self.w8)]

    def oracle(self, asc, wsc, partials=False):
        r, c = self.rows, self.cols
        return oracle.w4a4_gemm(self.a4[r], self.a8[r], asc[r], self.w4[c], self.w8[c], wsc[c], 128,
                                want_partials=partials)


def _run(pr, asc, wsc, packed=None, out=None):
    a4, a8, w4, w8 = pr.dev
    if packed is not None:
        return atom.atom_w4a4_gemm_packed(a4, a8, asc, packed[0], pr.N, out=out, workspace=packed[1])
    return atom.atom_w4a4_gemm(a4, a8, asc, w4, w8, wsc, out=out)


# M, K, N, O, what the dispatcher picks
SHAPES = [
    (8, 4096, 4096, 128, "decode, staged rows <2 staging instructions>, whole blocks of four groups"),
    (8, 11008, 4096, 128, "decode, staged rows: 86 groups (two left over)"),
    (32, 4096, 4096, 128, "decode <2 row blocks, 1 channel block>"),
    (32, 11008, 4096, 128, "decode <2 row blocks, 1 channel block>: 86 groups"),
    (64, 4096, 4096, 128, "decode <4 row blocks, 1 channel block>"),
    (64, 11008, 4096, 128, "decode <4 row blocks, 1 channel block>: 86 groups"),
    (64, 4096, 11008, 128, "decode <4 row blocks, 2 channel blocks>"),
    (48, 1792, 4112, 128, "decode <4 row blocks, 2 channel blocks>: 14 groups, an odd number of channel blocks"),
    (8, 768, 64, 256, "decode <1, vector scales> with two INT8 groups"),
    (8, 1408, 64, 128, "decode <1, 2-byte scale loads>: 11 groups"),
    (24, 1408, 64, 128, "decode <2, 2-byte scale loads>"),
    (24, 768, 64, 256, "decode <2, vector scales>, two INT8 groups"),
    (48, 768, 64, 256, "decode <4>, two INT8 groups"),
    (128, 4096, 4096, 128, "decode <4 row blocks, 2 channel blocks>, two blocks of 64 rows"),
    (96, 11008, 4096, 128, "decode, two blocks of 64 rows, the second of 32; 86 groups"),
    (192, 4096, 2048, 128, "few tiles <64, 32, four wavefront sets>"),
    (256, 4096, 4096, 128, "decode <4 row blocks, 2 channel blocks>, four blocks of 64 rows"),
    (256, 11008, 4096, 128, "decode, four blocks of 64 rows, 86 groups"),
    (320, 4096, 3072, 128, "few tiles <64, 64, four sets>"),
    (320, 11008, 3072, 128, "few tiles <64, 64, four sets>, 86 groups"),
    (256, 4096, 8192, 128, "few tiles <64, 64, two sets>"),
    (1024, 4096, 22016, 128, "big <256, 128, one set>: Llama-7B gate/up"),
    (1024, 11008, 4096, 128, "big <128, 128, two sets>: Llama-7B down"),
    (1024, 4096, 8192, 128, "big <128, 128, one set>"),
    (4096, 8192, 10240, 128, "big <256, 128>: Llama-70B QKV"),
    (4096, 28672, 8192, 128, "big <256, 128>: Llama-70B down, 224 groups"),
]
PACKED_SHAPES = [s for s in SHAPES if s[0] >= 128] + [(4096, 8192, 57344, 128, "Llama-70B gate/up")]


def _one_group(pr, packed):
    a4, a8, w4, w8 = pr.dev
    ones_w = np.ones((pr.N, pr.G), np.float16)
    part = pr.oracle(np.ones((pr.M, pr.G), np.float16), ones_w, partials=True)["partials"]
    wsc = torch.from_numpy(ones_w).cuda()
    pk = None
    if packed:
        ws = torch.empty(atom.atom_w4a4_gemm_packed_workspace_bytes(pr.M, pr.N, pr.K), dtype=torch.uint8, device="cuda")
        pk = (atom.atom_pack_weight(w4, w8, wsc), ws)
    asc = torch.zeros((pr.M, pr.G), dtype=torch.float16, device="cuda")
    y = torch.empty((pr.M, pr.N), dtype=torch.float16, device="cuda")
    r = torch.from_numpy(pr.rows).cuda()
    c = torch.from_numpy(pr.cols).cuda()
    g4 = (pr.K - pr.O) // 128
    exact = 0
    for g in range(pr.G):
        # INT8 groups (full-range codes, |P| up to 2^21) are scaled by 2^-6 to stay inside fp16
        s = 1.0 if g < g4 else 2.0 ** -6
        asc.zero_()
        asc[:, g] = s
        _run(pr, asc, wsc, pk, out=y)
        got = npy(y[r][:, c])
        want = (part[:, :, g].astype(np.float32) * np.float32(s)).astype(np.float16)   # exact below 2048
        assert np.array_equal(got.view(np.uint16), want.view(np.uint16)), f"group {g}: partial sums differ"
        if g < g4:
            exact += int((np.abs(part[:, :, g]) < 2048).sum())
    assert exact > 0.98 * part[:, :, :g4].size, "almost every sampled INT4 partial must be pinned to the integer"


@pytest.mark.parametrize("M,K,N,O,what", SHAPES)
def test_production_kernels_one_group_at_a_time(M, K, N, O, what):
    print(f"[case] one active group, {what}: M={M} K={K} N={N} O={O}", flush=True)
    _one_group(_Problem(M, K, N, O, seed=M + K + N, small8=False), packed=False)


@pytest.mark.parametrize("M,K,N,O,what", PACKED_SHAPES)
def test_packed_kernel_one_group_at_a_time(M, K, N, O, what):
    print(f"[case] one active group, packed weights, {what}: M={M} K={K} N={N}", flush=True)
    _one_group(_Problem(M, K, N, O, seed=M + K + N + 1, small8=False), packed=True)


def _pow2(pr, packed):
    """Scales 2^e.  INT4 groups: activations e in {0, 1}, weights e in {-8, -7}: a term is a
    multiple of 2^-8 of magnitude at most 8192 * 2 * 2^-7 = 128.  INT8 groups (full-range codes,
    |P| <= 2^21): 1 and 2^-8, a multiple of 2^-8 of at most 8192 per group.  With at most 223 + 1
    groups every partial sum, in any order, is a multiple of 2^-8 below 2^16: exact in fp32."""
    rng = pr.rng
    assert pr.G <= 224 and pr.O == 128 or pr.G <= 16
    asc = (2.0 ** rng.integers(0, 2, (pr.M, pr.G))).astype(np.float16)
    wsc = (2.0 ** rng.integers(-8, -6, (pr.N, pr.G))).astype(np.float16)
    g4 = (pr.K - pr.O) // 128
    asc[:, g4:] = 1.0
    wsc[:, g4:] = 2.0 ** -8
    want = pr.oracle(asc, wsc)["y"]
    a4, a8, w4, w8 = pr.dev
    ad, wd = torch.from_numpy(asc).cuda(), torch.from_numpy(wsc).cuda()
    pk = None
    if packed:
        ws = torch.empty(atom.atom_w4a4_gemm_packed_workspace_bytes(pr.M, pr.N, pr.K), dtype=torch.uint8, device="cuda")
        pk = (atom.atom_pack_weight(w4, w8, wd), ws)
    y = _run(pr, ad, wd, pk)
    torch.cuda.synchronize()
    r, c = torch.from_numpy(pr.rows).cuda(), torch.from_numpy(pr.cols).cuda()
    got = npy(y[r][:, c])
    assert np.isfinite(want.astype(np.float32)).all()
    assert np.array_equal(got.view(np.uint16), want.view(np.uint16)), "Y differs from the oracle's"


@pytest.mark.parametrize("M,K,N,O,what", SHAPES)
def test_production_kernels_power_of_two_scales(M, K, N, O, what):
    print(f"[case] power-of-two scales, {what}: M={M} K={K} N={N} O={O}", flush=True)
    _pow2(_Problem(M, K, N, O, seed=7 * M + K + N, small8=False), packed=False)


@pytest.mark.parametrize("M,K,N,O,what", PACKED_SHAPES)
def test_packed_kernel_power_of_two_scales(M, K, N, O, what):
    print(f"[case] power-of-two scales, packed weights, {what}: M={M} K={K} N={N}", flush=True)
    _pow2(_Problem(M, K, N, O, seed=7 * M + K + N + 1, small8=False), packed=True)


def test_one_group_check_sees_a_single_wrong_code():
    """The mistake is planted on the CPU side: one INT4 code of one sampled row is changed by one
    in the oracle's copy of the activations.  The check of that group must then fail, and the
    checks of the other groups must still pass."""
    pr = _Problem(256, 1024, 512, 128, seed=99, small8=False)
    row, byte = int(pr.rows[3]), 64 * 5 + 17                  # group 5, channel 34 of the group
    pr.a4[row, byte] ^= 0x01                                   # low nibble: the code changes by one
    part = pr.oracle(np.ones((pr.M, pr.G), np.float16), np.ones((pr.N, pr.G), np.float16), partials=True)["partials"]
    a4, a8, w4, w8 = pr.dev                                    # uploaded before the change
    wsc = torch.ones((pr.N, pr.G), dtype=torch.float16, device="cuda")
    r, c = torch.from_numpy(pr.rows).cuda(), torch.from_numpy(pr.cols).cuda()
    bad = []
    for g in range(pr.G - 1):
        asc = torch.zeros((pr.M, pr.G), dtype=torch.float16, device="cuda")
        asc[:, g] = 1
        got = npy(atom.atom_w4a4_gemm(a4, a8, asc, w4, w8, wsc)[r][:, c])
        want = part[:, :, g].astype(np.float32).astype(np.float16)
        if not np.array_equal(got.view(np.uint16), want.view(np.uint16)):
            bad.append(g)
            assert (got != want).any(axis=1).nonzero()[0].tolist() == [3], "only the changed row differs"
    assert bad == [5]


@pytest.mark.parametrize("M,K,N,packed", [(8, 4096, 4096, False), (8, 1024, 64, False), (40, 1024, 64, False),
                                          (200, 1024, 256, False), (2048, 1024, 2048, False),
                                          (200, 1024, 256, True), (1024, 4096, 4096, True)])
def test_subnormal_scales_are_not_flushed(M, K, N, packed):
    """Activation scales that are fp16 subnormals (2^-16, 2^-17: tiny activations) against weight
    scales of 2^6, 2^7: every term is a multiple of 2^-11 below 2^11, every sum exact in fp32 in any
    order, so Y equals the oracle's bit for bit, unless a kernel reads a subnormal scale as zero."""
    print(f"[case] subnormal activation scales M={M} K={K} N={N} packed={packed}", flush=True)
    pr = _Problem(M, K, N, 128, seed=M + K + N + 5, small8=True)
    asc = (2.0 ** pr.rng.integers(-17, -15, (pr.M, pr.G))).astype(np.float16)
    wsc = (2.0 ** pr.rng.integers(6, 8, (pr.N, pr.G))).astype(np.float16)
    assert (asc > 0).all() and (asc < 2.0 ** -14).all()
    want = pr.oracle(asc, wsc)["y"]
    assert (want != 0).mean() > 0.9
    ad, wd = torch.from_numpy(asc).cuda(), torch.from_numpy(wsc).cuda()
    pk = None
    if packed:
        ws = torch.empty(atom.atom_w4a4_gemm_packed_workspace_bytes(pr.M, pr.N, pr.K), dtype=torch.uint8, device="cuda")
        pk = (atom.atom_pack_weight(pr.dev[2], pr.dev[3], wd), ws)
    y = _run(pr, ad, wd, pk)
    torch.cuda.synchronize()
    got = npy(y[torch.from_numpy(pr.rows).cuda()][:, torch.from_numpy(pr.cols).cuda()])
    assert np.array_equal(got.view(np.uint16), want.view(np.uint16)), "Y differs from the oracle's"
