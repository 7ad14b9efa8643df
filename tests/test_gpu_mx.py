"""GPU parity of the MX variant (FP4 E2M1 / FP8 E4M3 codes, E8M0 scale per 32 channels): the
front end's codes and scale bytes bit-identical to the CPU oracle; the scaled-MFMA GEMM against
the oracle's exact sum.

Tolerance of the GEMM.  The FP4 steps come out of the matrix core exactly (their products are
small multiples of 1/4).  The 64 FP8 products of one instruction are summed in a window that
ends about 13 bits below the largest of them (measured on gfx950: the error beyond the final
fp16 rounding stays under 2^-12.5 of the largest |a| times the largest |w| among the outlier
channels of the row and column).  So an element may be off by the library's usual bar, 1e-3 of
max(|ref|, 1% of the largest |ref|), plus 2^-11 of that outlier product bound."""
import numpy as np
import pytest
import torch

import oracle
import paper_2310_19102_amd as atom
from paper_2310_19102_amd import synth

pytestmark = pytest.mark.gpu

Y_TOL = 1e-3


def _npy(t):
    return t.detach().cpu().numpy()


def _row_major(g):
    """The library's step-major arrays ([step][row][64 bytes], scales [slab][row][4]) as the
    oracle's row-major ones: a pure permutation of bytes."""
    q4, q8, e8 = (_npy(t) for t in g)
    rows = q4.shape[1]
    return (q4.transpose(1, 0, 2).reshape(rows, -1), q8.transpose(1, 0, 2).reshape(rows, -1),
            e8.transpose(1, 0, 2).reshape(rows, -1))


def _equal(g, r, what):
    for name, a, b in zip(("q4", "q8", "e8"), _row_major(g) if g[0].ndim == 3 else g, r):
        a = _npy(a) if hasattr(a, "detach") else a
        assert a.shape == b.shape, f"{what}: {name} shape"
        if not np.array_equal(a, b):
            bad = np.argwhere(a != b)
            raise AssertionError(f"{what}: {name} differs at {len(bad)} places, first {bad[0]}: "
                                 f"gpu {a[tuple(bad[0])]} oracle {b[tuple(bad[0])]}")


_E4M3 = None


def _outlier_amax(q8, e8):
    """Largest dequantised |outlier| per row: FP8 codes [rows, O], scale bytes [rows, K/32]."""
    global _E4M3
    if _E4M3 is None:
        _E4M3 = np.array([abs(oracle.e4m3_to_f32(c)) if c & 0x7F != 0x7F else 0.0 for c in range(256)])
    O = q8.shape[1]
    sc = np.repeat(np.exp2(e8[:, -(O // 32):].astype(np.float64) - 127.0), 32, axis=1)
    return (_E4M3[q8] * sc).max(axis=1)


def _rel_err(y, ref, ra, rw):
    """Largest |y - ref| in units of the allowed error of its element."""
    y, ref = y.astype(np.float64), ref.astype(np.float64)
    floor = 1e-2 * max(np.abs(ref).max(), 1e-30)
    allowed = Y_TOL * np.maximum(np.abs(ref), floor) + \
        2.0 ** -11 * _outlier_amax(ra[1], ra[2])[:, None] * _outlier_amax(rw[1], rw[2])[None, :]
    return float((np.abs(y - ref) / allowed).max())


def _rand_linear(M, K, N, O, seed, norm=True):
    g = torch.Generator().manual_seed(seed)
    sigma = torch.exp(1.5 * torch.randn(K, generator=g))
    x = (torch.randn((M, K), generator=g) * sigma).to(torch.float16)
    w = (0.02 * torch.randn((N, K), generator=g)).to(torch.float16)
    gamma = (1 + 0.1 * torch.randn(K, generator=g)).to(torch.float16) if norm else None
    idx = torch.argsort(sigma, stable=True).to(torch.int32)
    return synth.Linear("rand", x, w, gamma, idx, n_outlier=O)


def _check(lin, what, clip_a=0.9, clip_w=0.85):
    print(f"[case] mx {what}: M={lin.M} K={lin.K} N={lin.N} O={lin.n_outlier} norm={lin.gamma is not None}",
          flush=True)
    idx = lin.idx.cuda()
    ga = atom.atom_mx_quantize_act(lin.x.cuda(), None if lin.gamma is None else lin.gamma.cuda(), lin.eps,
                                   idx, lin.n_outlier, clip_a)
    gw = atom.atom_mx_quantize_weight(lin.w.cuda(), idx, lin.n_outlier, clip_w)
    torch.cuda.synchronize()
    ra = oracle.mx_quantize_act(lin.x.numpy(), None if lin.gamma is None else lin.gamma.numpy(), lin.eps,
                                lin.idx.numpy(), lin.n_outlier, clip_a)
    rw = oracle.mx_quantize_weight(lin.w.numpy(), lin.idx.numpy(), lin.n_outlier, clip_w)
    _equal(ga, ra, what + " act")
    _equal(gw, rw, what + " weight")
    y = atom.atom_mx_gemm(*ga, *gw)
    torch.cuda.synchronize()
    ref = oracle.mx_gemm(*ra, *rw)
    err = _rel_err(_npy(y), ref, ra, rw)
    assert err <= 1.0, f"{what}: Y error {err} x the allowed"


@pytest.mark.parametrize("M,K,N,O,norm", [
    (1, 256, 8, 128, True),          # one FP4 step, two FP8 steps, a single row
    (16, 512, 64, 128, True),
    (33, 1024, 200, 256, False),     # four FP8 steps, ragged M and N
    (257, 384, 300, 128, True),      # two row tiles and two column tiles, ragged both ways
    (300, 1536, 513, 128, True),     # twelve steps; N just past two tiles
    (70, 640, 100, 384, False),      # more outlier than normal steps
])
def test_mx_small(M, K, N, O, norm):
    _check(_rand_linear(M, K, N, O, 100 + M, norm), f"{M}x{K}x{N}")


def test_mx_clip_one_and_special_rows():
    lin = _rand_linear(40, 512, 48, 128, 7)
    lin.x[3] = 0                                       # all-zero row: scale bytes 0, codes 0
    lin.x[4, :] = 6.0                                  # constant row
    lin.x[5, ::2] *= -1
    lin.x[6] = lin.x[6] * 0 + torch.tensor(6e-8).half()   # fp16's smallest subnormal everywhere
    lin.x[7, 5] = 65504.0                              # fp16's largest value
    _check(lin, "special", clip_a=1.0, clip_w=1.0)
    lin.gamma = None
    _check(lin, "special, no norm", clip_a=1.0, clip_w=1.0)


def test_mx_front_end_every_tie_and_saturation():
    """Rows built from every midpoint between neighbouring FP4 and FP8 magnitudes and from
    values around the saturation points, at several block scales."""
    K, O = 512, 128
    e2m1 = np.array([0, .5, 1, 1.5, 2, 3, 4, 6])
    mids4 = (e2m1[:-1] + e2m1[1:]) / 2
    vals4 = np.concatenate([e2m1, mids4, mids4 * (1 + 2.0 ** -10), mids4 * (1 - 2.0 ** -10), [6.5, 7, 7.9]])
    tab8 = np.array([oracle.e4m3_to_f32(c) for c in range(0x7F)])
    mids8 = (tab8[:-1] + tab8[1:]) / 2
    vals8 = np.concatenate([tab8, mids8, [449, 460, 464, 480, 500]])
    rows = []
    rng = np.random.default_rng(0)
    for sc in (1.0, 2.0 ** -6, 2.0 ** 5):
        for rep in range(6):
            r = np.zeros(K)
            r[:K - O] = rng.choice(vals4, K - O) * rng.choice([-1, 1], K - O) * sc
            r[K - O:] = rng.choice(vals8, O) * rng.choice([-1, 1], O) * sc * 2.0 ** -4
            # pin each block's exponent with one full-scale element
            r[0:K - O:32] = 4.0 * sc
            r[K - O::32] = 256.0 * sc * 2.0 ** -4
            rows.append(r)
    x = torch.tensor(np.stack(rows), dtype=torch.float16)
    idx = torch.arange(K, dtype=torch.int32)
    g = atom.atom_mx_quantize_act(x.cuda(), None, 0.0, idx.cuda(), O, 1.0)
    torch.cuda.synchronize()
    _equal(g, oracle.mx_quantize_act(x.numpy(), None, 0.0, idx.numpy(), O, 1.0), "ties")


def test_mx_config1_and_config2():
    lin = synth.make(1)
    _check(lin, "config1")
    lin = synth.make(2, 0)
    _check(lin, "config2 attn_proj")


def test_mx_full_size_sampled():
    """Llama-7B MLP gate/up at M = 1024 (the shape the bench times): front ends bit-exact on all
    rows of the activations and a sample of the weight rows, the GEMM checked by the oracle on a
    sample of rows and columns."""
    lin = synth.make(4, 0)
    idx = lin.idx.cuda()
    ga = atom.atom_mx_quantize_act(lin.x.cuda(), lin.gamma.cuda(), lin.eps, idx, lin.n_outlier, 0.9)
    gw = atom.atom_mx_quantize_weight(lin.w.cuda(), idx, lin.n_outlier, 0.85)
    y = _npy(atom.atom_mx_gemm(*ga, *gw))
    rng = np.random.default_rng(1)
    rows = np.sort(rng.choice(lin.M, 48, replace=False))
    cols = np.sort(np.concatenate([rng.choice(lin.N, 120, replace=False), [0, lin.N - 1]]))
    ra = oracle.mx_quantize_act(lin.x.numpy()[rows], lin.gamma.numpy(), lin.eps, lin.idx.numpy(), lin.n_outlier, 0.9)
    rw = oracle.mx_quantize_weight(lin.w.numpy()[cols], lin.idx.numpy(), lin.n_outlier, 0.85)
    _equal(tuple(t[rows] for t in _row_major(ga)), ra, "act rows")
    _equal(tuple(t[cols] for t in _row_major(gw)), rw, "weight rows")
    ref = oracle.mx_gemm(*ra, *rw)
    err = _rel_err(y[np.ix_(rows, cols)], ref, ra, rw)
    assert err <= 1.0, f"sampled Y error {err} x the allowed"


def test_mx_errors():
    x = torch.zeros((4, 256), dtype=torch.float16, device="cuda")
    idx = torch.arange(256, dtype=torch.int32, device="cuda")
    with pytest.raises(atom.AtomError) as e:                  # O must be a multiple of 128
        atom.atom_mx_quantize_act(x, None, 0.0, idx, 64, 1.0)
    assert e.value.status == 2
    with pytest.raises(atom.AtomError) as e:                  # no outliers: not built
        atom.atom_mx_quantize_act(x, None, 0.0, idx, 0, 1.0)
    assert e.value.status == 3
    q = atom.atom_mx_quantize_act(x, None, 0.0, idx, 128, 1.0)
    y = atom.atom_mx_gemm(*q, *q)
    torch.cuda.synchronize()
    assert not _npy(y).any()
    empty = atom.atom_mx_quantize_act(x[:0], None, 0.0, idx, 128, 1.0)
    assert atom.atom_mx_gemm(*empty, *q).shape == (0, 4)
    with pytest.raises(ValueError):                           # row-major arrays are not accepted
        atom.atom_mx_gemm(q[0].reshape(4, -1), q[1].reshape(4, -1), q[2].reshape(4, -1), *q)
