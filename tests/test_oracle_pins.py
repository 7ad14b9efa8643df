"""Pins for the CPU oracle: everything here checks ``oracle/`` against
something other than itself -- numpy's IEEE conversions, exact rational
arithmetic, hand-worked cases (tests/golden), closed forms, invariants of
symmetric group quantisation (Section 2 of the paper), an fp64
dequantise-then-matmul brute force (Section 4.2) and torch's RMSNorm.

No GPU is needed and the HIP library is never touched.
"""
import json
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

import oracle


# ----------------------------------------------------------------- helpers --

def rne_int(fr: Fraction) -> int:
    """Round a rational to the nearest integer, ties to even."""
    fl = fr.numerator // fr.denominator
    rem = fr - fl
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and fl % 2 == 1):
        fl += 1
    return fl


def round_binary(fr: Fraction, p: int, emin: int) -> Fraction:
    """Round a rational to a binary float with p significand bits and minimum
    normal exponent emin (gradual underflow), ties to even.  No overflow."""
    if fr == 0:
        return Fraction(0)
    sign = -1 if fr < 0 else 1
    a = abs(fr)
    e = a.numerator.bit_length() - a.denominator.bit_length()
    if Fraction(2) ** e > a:
        e -= 1
    assert Fraction(2) ** e <= a < Fraction(2) ** (e + 1)
    quantum = Fraction(2) ** (max(e, emin) - (p - 1))
    return sign * rne_int(a / quantum) * quantum


def rf32(fr):
    return round_binary(fr, 24, -126)


def rf16(fr):
    out = round_binary(fr, 11, -14)
    return min(out, Fraction(65504))     # scales saturate instead of overflowing


def exact_group_quant(y_vals, clip, bits):
    """Symmetric quantisation of one group (Section 2) in exact rationals with
    explicit fp32 / fp16 roundings.  y_vals: python floats holding fp16/fp32
    values exactly.  Returns (scale Fraction, codes list)."""
    ys = [Fraction(float(v)) for v in y_vals]
    amax = max(abs(v) for v in ys)
    c = Fraction(float(np.float32(clip)))
    s32 = rf32(rf32(rf32(2 * amax) * c) / ((1 << bits) - 1))
    s = rf16(s32)
    qmin, qmax = -(1 << (bits - 1)), (1 << (bits - 1)) - 1
    codes = []
    for v in ys:
        if s == 0:
            codes.append(0)
        else:
            codes.append(max(qmin, min(qmax, rne_int(rf32(v / s)))))
    return s, codes


def np_unpack(q4, q8):
    """Independent numpy unpack of the code layout: [rows, K] int64 in
    reordered channel order (even column = low nibble)."""
    lo = (q4 & 0xF).astype(np.int64)
    hi = (q4 >> 4).astype(np.int64)
    lo = np.where(lo >= 8, lo - 16, lo)
    hi = np.where(hi >= 8, hi - 16, hi)
    c4 = np.stack([lo, hi], axis=-1).reshape(q4.shape[0], -1)
    return np.concatenate([c4, q8.astype(np.int64)], axis=1)


def quant_one_group(y_fp16, bits, clip):
    """Run the oracle on a single group of the given bit-width.  The oracle
    needs at least one INT4 group, so an INT8 group is appended after a dummy
    INT4 group of zeros, and vice versa nothing is needed for INT4."""
    y = np.asarray(y_fp16, np.float16)
    n = y.shape[0]
    Gs = n + (n % 2)
    ypad = np.zeros(Gs, np.float16)
    ypad[:n] = y
    if bits in (3, 4):
        x = ypad[None, :]
        idx = np.arange(Gs, dtype=np.int32)
        q4, q8, sc = oracle.quantize_act(x, None, 0.0, idx, group_size=Gs, n_outlier=0, clip=clip, bits=bits)
        codes = np_unpack(q4, q8)[0, :n]
    else:
        x = np.concatenate([np.zeros(Gs, np.float16), ypad])[None, :]
        idx = np.arange(2 * Gs, dtype=np.int32)
        q4, q8, sc = oracle.quantize_act(x, None, 0.0, idx, group_size=Gs, n_outlier=Gs, clip=clip)
        assert not q4.any() and sc[0, 0] == 0
        codes = q8[0, :n].astype(np.int64)
    return float(sc[0, -1]), codes, q4


@pytest.fixture(scope="module")
def worked(golden_dir):
    with open(os.path.join(golden_dir, "worked_examples.json")) as f:
        return json.load(f)


# ------------------------------------------------------------ fp16 <-> fp32 --

def test_f16_to_f32_all_patterns_match_numpy():
    bits = np.arange(65536, dtype=np.uint16)
    ref = bits.view(np.float16).astype(np.float32)
    for h in range(65536):
        v = np.float32(oracle.f16_to_f32(h))
        if np.isnan(ref[h]):
            assert np.isnan(v)
        else:
            assert v.tobytes() == ref[h].tobytes(), h


def test_f32_to_f16_matches_numpy_rne():
    rng = np.random.default_rng(1)
    vals = (rng.standard_normal(30000) * np.exp(rng.uniform(-22, 11, 30000))).astype(np.float32)
    # exact ties, subnormal edges, overflow edge
    edge = np.array([0.0, -0.0, 2.0 ** -25, 2.0 ** -25 * 1.0000001, 2.0 ** -24, 3 * 2.0 ** -25,
                     65504.0, 65519.9, 65520.0, 1e9, -1e9, 1.00048828125, 1.0009765625 + 2.0 ** -11,
                     2.0 ** -14, 2.0 ** -14 - 2.0 ** -25, 6.1e-5, np.inf, -np.inf], np.float32)
    with np.errstate(over="ignore"):
        for v in np.concatenate([vals, edge]):
            assert oracle.f32_to_f16(v) == int(np.float32(v).astype(np.float16).view(np.uint16)), v


# ------------------------------------------------------- hand-worked cases --

def test_worked_quantize_examples(worked):
    for ex in worked["quantize"]:
        s, codes, q4 = quant_one_group(ex["y"], ex["bits"], ex["clip"])
        assert s == ex["scale"], ex["name"]
        assert codes.tolist() == ex["codes"], ex["name"]
        if "packed_hex" in ex:
            assert q4.tobytes().hex() == ex["packed_hex"]
        # and the exact-rational derivation agrees with the hand arithmetic
        y16 = np.asarray(ex["y"], np.float16)
        s_x, codes_x = exact_group_quant(y16, ex["clip"], ex["bits"])
        assert float(s_x) == ex["scale"] and codes_x == ex["codes"], ex["name"]


def test_worked_sumsq_tree(worked):
    for ex in worked["sumsq"]:
        K = ex["K"]
        x = np.full(K, ex["fill"], np.float16)
        x[ex["zero_every_8th_from"]::8] = 0
        for k in ex["extra_zero"]:
            x[k] = 0
        for k in ex["extra_one"]:
            x[k] = 1
        for k, v in ex["set"].items():
            x[int(k)] = v
        assert float(oracle.sumsq(x)) == ex["S"], ex["name"]


def test_worked_rmsnorm(worked):
    for ex in worked["rmsnorm"]:
        y = oracle.rmsnorm_row(np.asarray(ex["x"], np.float16),
                               np.asarray(ex["gamma"], np.float16), ex["eps"])
        assert y.tolist() == [float(np.float32(v)) for v in ex["y"]]


def test_worked_gemm(worked):
    for ex in worked["gemm"]:
        Gs, O = ex["group_size"], ex["n_outlier"]
        a, w = ex["a_codes"], ex["w_codes"]
        K4 = len(a) - O

        def pack(c):
            q4 = np.array([[(c[2 * b] & 0xF) | ((c[2 * b + 1] & 0xF) << 4) for b in range(K4 // 2)]],
                          np.uint8)
            return q4, np.array([c[K4:]], np.int8)
        a4, a8 = pack(a)
        w4, w8 = pack(w)
        out = oracle.w4a4_gemm(a4, a8, np.array([ex["a_scale"]], np.float16),
                               w4, w8, np.array([ex["w_scale"]], np.float16),
                               group_size=Gs, want_partials=True, want_acc=True)
        assert out["partials"][0, 0].tolist() == ex["partials"]
        assert float(out["acc"][0, 0]) == ex["acc"]
        assert float(out["y"][0, 0]) == ex["y"]


# ------------------------------------------------------------ closed forms --

def test_effective_bits_closed_form(golden_dir):
    """Storage per row equals the paper's 4.25 effective bits at K=4096."""
    kv = {}
    with open(os.path.join(golden_dir, "effective_bits.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                k, v = line.split()
                kv[k] = float(v)
    K, Gs, O = int(kv["K"]), int(kv["group_size"]), int(kv["n_outlier"])
    x = np.random.default_rng(0).standard_normal((2, K)).astype(np.float16)
    q4, q8, sc = oracle.quantize_act(x, None, 0.0, np.arange(K, dtype=np.int32), Gs, O, 0.9)
    row_bytes = q4[0].nbytes + q8[0].nbytes + sc[0].nbytes
    assert row_bytes == 2176
    assert row_bytes * 8 / K == kv["effective_bits"]


def test_sumsq_exact_cases_and_fp64_bound():
    assert float(oracle.sumsq(np.ones(4096, np.float16))) == 4096.0
    x = np.zeros(512, np.float16)
    x[137] = -3.0
    assert float(oracle.sumsq(x)) == 9.0
    rng = np.random.default_rng(2)
    xi = rng.integers(-15, 16, 2048).astype(np.float16)       # every partial sum exact
    assert float(oracle.sumsq(xi)) == float((xi.astype(np.float64) ** 2).sum())
    for K in (8, 24, 512, 4096, 11008, 1000):
        x = (rng.standard_normal(K) * np.exp(rng.standard_normal(K))).astype(np.float16)
        exact = float((x.astype(np.float64) ** 2).sum())
        got = float(oracle.sumsq(x))
        # depth of the tree: 3 levels in a vector, K/512 sequential adds, 6 folds
        depth = 3 + (K + 511) // 512 + 6
        assert abs(got - exact) <= depth * 2.0 ** -24 * exact


def test_rmsnorm_against_torch_fp64():
    rng = np.random.default_rng(3)
    for K in (512, 4096, 11008):
        x = (rng.standard_normal(K) * np.exp(1.5 * rng.standard_normal(K))).astype(np.float16)
        g = (1 + 0.1 * rng.standard_normal(K)).astype(np.float16)
        eps = 1e-6
        y = oracle.rmsnorm_row(x, g, eps)
        ref = torch.nn.functional.rms_norm(torch.from_numpy(x.astype(np.float64)), (K,),
                                           torch.from_numpy(g.astype(np.float64)), eps).numpy()
        err = np.abs(y.astype(np.float64) - ref)
        assert np.all(err <= 4 * 2.0 ** -23 * np.abs(ref) + 1e-30)
        # gamma is applied in ORIGINAL channel order: a wrong index would show here
        assert np.argmax(np.abs(y)) == np.argmax(np.abs(ref))


def test_rmsnorm_scale_invariance_eps0():
    """With eps = 0, scaling x by a power of two changes nothing after the norm."""
    rng = np.random.default_rng(4)
    K = 1024
    x = rng.standard_normal(K).astype(np.float16)
    g = (1 + 0.1 * rng.standard_normal(K)).astype(np.float16)
    idx = rng.permutation(K).astype(np.int32)
    a = oracle.quantize_act(x[None], g, 0.0, idx, 128, 128, 0.9)
    b = oracle.quantize_act((x * np.float16(8))[None], g, 0.0, idx, 128, 128, 0.9)
    for u, v in zip(a, b):
        assert np.array_equal(u, v)


# ------------------------------------------- exact-rational brute force ----

@pytest.mark.parametrize("bits,clip", [(4, 1.0), (4, 0.9), (4, 0.85), (8, 1.0), (8, 0.9), (8, 0.85),
                                       (3, 1.0), (3, 0.9), (3, 0.85)])
def test_group_quant_matches_exact_rationals(bits, clip):
    rng = np.random.default_rng(10 * bits + int(clip * 100))
    for trial in range(40):
        n = int(rng.choice([2, 4, 6, 16]))
        scale = np.exp(rng.uniform(-12, 8))
        y = (rng.standard_normal(n) * scale).astype(np.float16)
        if trial % 7 == 0:
            y[:] = 0                                       # zero group: scale 0, codes 0
        if trial % 11 == 3:
            y = (y * 0 + np.float16(6e-8) * rng.integers(-2, 3, n)).astype(np.float16)  # subnormals
        s, codes, _ = quant_one_group(y, bits, clip)
        s_x, codes_x = exact_group_quant(y, clip, bits)
        assert s == float(s_x), (y, s, float(s_x))
        assert codes.tolist() == codes_x, (y, codes, codes_x)


def test_scale_saturates_at_fp16_max():
    y = np.array([65504.0, -65504.0, 30000.0, 1.0], np.float16)
    s, codes, _ = quant_one_group(y, 4, 8.0)               # s32 = 2*65504*8/15 > 65504
    assert s == 65504.0
    assert codes.tolist() == [1, -1, 0, 0]


def test_quantize_with_gamma_matches_exact_rationals():
    """Norm output (fp32, never rounded to fp16) feeds the quantiser."""
    rng = np.random.default_rng(5)
    K, Gs, O = 64, 16, 16
    x = (rng.standard_normal((3, K)) * np.exp(rng.standard_normal(K))).astype(np.float16)
    g = (1 + 0.1 * rng.standard_normal(K)).astype(np.float16)
    idx = rng.permutation(K).astype(np.int32)
    q4, q8, sc = oracle.quantize_act(x, g, 1e-6, idx, Gs, O, 0.9)
    codes = np_unpack(q4, q8)
    for m in range(3):
        y = oracle.rmsnorm_row(x[m], g, 1e-6)
        yr = y[idx]
        for gi in range(K // Gs):
            bits = 4 if gi < (K - O) // Gs else 8
            s_x, c_x = exact_group_quant(yr[gi * Gs:(gi + 1) * Gs], 0.9, bits)
            assert float(sc[m, gi]) == float(s_x)
            assert codes[m, gi * Gs:(gi + 1) * Gs].tolist() == c_x


# ----------------------------------------------------------- invariants ----

def _heavy(rng, M, K):
    sig = np.exp(1.5 * rng.standard_normal(K))
    return (rng.standard_normal((M, K)) * sig).astype(np.float16), np.argsort(sig, kind="stable").astype(np.int32)


@pytest.mark.parametrize("clip", [1.0, 0.9])
def test_code_ranges_and_dequant_error(clip):
    rng = np.random.default_rng(6)
    M, K, Gs, O = 8, 1024, 128, 128
    x, idx = _heavy(rng, M, K)
    q4, q8, sc = oracle.quantize_act(x, None, 0.0, idx, Gs, O, clip)
    codes = np_unpack(q4, q8)
    G4 = (K - O) // Gs
    yr = x[:, idx].astype(np.float64)
    s = np.repeat(sc.astype(np.float64), Gs, axis=1)
    qmax = np.repeat(np.where(np.arange(K // Gs) < G4, 7, 127), Gs)[None, :]
    qmin = -qmax - 1
    assert np.all(codes >= qmin) and np.all(codes <= qmax)
    ratio = yr / s
    sat_hi = codes == qmax
    sat_lo = codes == qmin
    inside = ~(sat_hi | sat_lo)
    # unsaturated: nearest code, so |y - q*s| <= s/2 (fp32 division slack 2^-20)
    assert np.all(np.abs(yr - codes * s)[inside] <= 0.5 * s[inside] * (1 + 2.0 ** -20))
    # saturated codes are never further from y than a free rounding would allow on the inner side
    assert np.all(ratio[sat_hi] >= qmax.repeat(M, 0)[sat_hi] - 0.5 - 1e-6)
    assert np.all(ratio[sat_lo] <= qmin.repeat(M, 0)[sat_lo] + 0.5 + 1e-6)
    # each group reaches (clip <= 1) the largest magnitude code on its amax element
    mag = np.abs(codes).reshape(M, K // Gs, Gs).max(axis=2)
    need = np.where(np.arange(K // Gs) < G4, 7, 127)[None, :]
    assert np.all(mag >= need)
    # textbook reading: scale = 2*amax*c/(2^n-1) within fp16 rounding
    amax = np.abs(yr).reshape(M, K // Gs, Gs).max(axis=2)
    denom = np.where(np.arange(K // Gs) < G4, 15.0, 255.0)[None, :]
    want = 2 * amax * clip / denom
    assert np.all(np.abs(sc.astype(np.float64) - want) <= want * 2.0 ** -11 + 1e-12)


def test_power_of_two_row_scaling_and_in_group_permutation():
    rng = np.random.default_rng(7)
    M, K, Gs, O = 4, 512, 128, 128
    x, idx = _heavy(rng, M, K)
    x = (x / 16).astype(np.float16)
    base = oracle.quantize_act(x, None, 0.0, idx, Gs, O, 0.9)
    up = oracle.quantize_act((x * np.float16(4)).astype(np.float16), None, 0.0, idx, Gs, O, 0.9)
    assert np.array_equal(base[0], up[0]) and np.array_equal(base[1], up[1])
    assert np.array_equal(base[2].astype(np.float32) * 4, up[2].astype(np.float32))
    # permuting the index inside each group permutes codes, keeps scales
    idx2 = idx.copy().reshape(K // Gs, Gs)
    perms = [rng.permutation(Gs) for _ in range(K // Gs)]
    idx2 = np.stack([row[p] for row, p in zip(idx2, perms)]).reshape(-1).astype(np.int32)
    per = oracle.quantize_act(x, None, 0.0, idx2, Gs, O, 0.9)
    assert np.array_equal(base[2], per[2])
    c0 = np_unpack(base[0], base[1]).reshape(M, K // Gs, Gs)
    c1 = np_unpack(per[0], per[1]).reshape(M, K // Gs, Gs)
    for g, p in enumerate(perms):
        assert np.array_equal(c0[:, g, :][:, p], c1[:, g, :])


def test_identity_index_no_norm_is_plain_absmax_rtn():
    """With the identity index and no norm the front end is ordinary
    per-group absmax round-to-nearest; compare with an fp64 computation away
    from rounding boundaries."""
    rng = np.random.default_rng(8)
    M, K, Gs, O = 4, 512, 128, 128
    x = rng.standard_normal((M, K)).astype(np.float16)
    q4, q8, sc = oracle.quantize_act(x, None, 0.0, np.arange(K, dtype=np.int32), Gs, O, 1.0)
    codes = np_unpack(q4, q8)
    s = np.repeat(sc.astype(np.float64), Gs, axis=1)
    t = x.astype(np.float64) / s
    qmax = np.repeat(np.where(np.arange(K // Gs) < (K - O) // Gs, 7, 127), Gs)[None, :]
    want = np.clip(np.rint(t), -qmax - 1, qmax)
    away = np.abs(t - np.floor(t) - 0.5) > 1e-4
    assert np.array_equal(codes[away], want[away].astype(np.int64))


def test_weight_path_equals_front_end_without_norm():
    rng = np.random.default_rng(9)
    w = (0.02 * rng.standard_normal((8, 512))).astype(np.float16)
    idx = rng.permutation(512).astype(np.int32)
    a = oracle.quantize_weight(w, idx, 128, 128, 0.85)
    b = oracle.quantize_act(w, None, 0.0, idx, 128, 128, 0.85)
    for u, v in zip(a, b):
        assert np.array_equal(u, v)


# -------------------------------------------------------- GEMM brute force --

@pytest.mark.parametrize("M,N,K,Gs,O", [(3, 5, 16, 2, 4), (4, 3, 32, 4, 8), (5, 7, 512, 128, 128),
                                        (2, 4, 768, 128, 256), (5, 7, 512, 64, 128), (3, 4, 1024, 256, 256)])
def test_gemm_against_fp64_dequant_matmul(M, N, K, Gs, O):
    rng = np.random.default_rng(M * 100 + N)
    x, idx = _heavy(rng, M, K)
    w = (0.02 * rng.standard_normal((N, K))).astype(np.float16)
    g = (1 + 0.1 * rng.standard_normal(K)).astype(np.float16)
    a4, a8, asc = oracle.quantize_act(x, g, 1e-6, idx, Gs, O, 0.9)
    w4, w8, wsc = oracle.quantize_weight(w, idx, Gs, O, 0.85)
    out = oracle.w4a4_gemm(a4, a8, asc, w4, w8, wsc, Gs, want_partials=True, want_acc=True)
    ca, cw = np_unpack(a4, a8), np_unpack(w4, w8)
    G = K // Gs
    # exact integer partials, independent triple loop
    P = np.einsum("mgk,ngk->mng", ca.reshape(M, G, Gs), cw.reshape(N, G, Gs))
    assert np.array_equal(out["partials"].astype(np.int64), P)
    # fp64 dequantise-then-matmul over all of K at once
    A = ca * np.repeat(asc.astype(np.float64), Gs, axis=1)
    W = cw * np.repeat(wsc.astype(np.float64), Gs, axis=1)
    Y64 = A @ W.T
    terms = np.abs(P * (asc.astype(np.float64)[:, None, :] * wsc.astype(np.float64)[None, :, :])).sum(axis=2)
    assert np.all(np.abs(out["acc"].astype(np.float64) - Y64) <= G * 2.0 ** -23 * terms + 1e-30)
    assert np.array_equal(out["y"], out["acc"].astype(np.float16))


def test_gemm_extreme_codes_do_not_overflow():
    """All codes at -8 / -128: the largest partials the format allows."""
    K, Gs, O = 256, 128, 128
    a4 = np.full((1, 64), 0x88, np.uint8)
    a8 = np.full((1, 128), -128, np.int8)
    sc = np.ones((1, 2), np.float16)
    out = oracle.w4a4_gemm(a4, a8, sc, a4, a8, sc, Gs, want_partials=True, want_acc=True)
    assert out["partials"][0, 0].tolist() == [64 * 128, 128 * 128 * 128]
    assert float(out["acc"][0, 0]) == 64 * 128 + 2.0 ** 21


# ------------------------------------- the method as a whole (Section 4.1) --

def test_reorder_leaves_the_product_unchanged_and_outliers_matter():
    """Reordering A and W by the same index does not change A W^T; keeping the
    outlier channels in INT8 is what makes W4A4 accurate (Section 4.1)."""
    rng = np.random.default_rng(11)
    M, N, K, Gs, O = 16, 32, 1024, 128, 128
    x, idx = _heavy(rng, M, K)
    w = (0.02 * rng.standard_normal((N, K))).astype(np.float16)
    A, W = x.astype(np.float64), w.astype(np.float64)
    dense = A @ W.T
    assert np.allclose(A[:, idx] @ W[:, idx].T, dense, rtol=1e-12, atol=1e-12)

    def run(index):
        a = oracle.quantize_act(x, None, 0.0, index, Gs, O, 0.9)
        b = oracle.quantize_weight(w, index, Gs, O, 0.85)
        y = oracle.w4a4_gemm(*a, *b, Gs)["y"].astype(np.float64)
        return np.linalg.norm(y - dense) / np.linalg.norm(dense)
    good = run(idx)                       # largest channels last -> INT8
    bad = run(idx[::-1].copy())           # smallest channels in INT8 instead
    assert good < 0.2
    assert bad > 1.5 * good


# ---------------------------------------------------------------- residual add in front


def test_add_is_the_correctly_rounded_fp16_sum():
    """h = fp16(x + res): the oracle forms the sum in fp32 and rounds once; the pin forms it
    in fp64, where the sum of two fp16 values is always exact, and rounds that once with
    numpy's double -> half conversion.  Includes pairs more than 2^13 apart (fp32 sum
    inexact), exact ties, cancellation, subnormals and overflow to infinity."""
    rng = np.random.default_rng(7)
    a = rng.standard_normal(4096).astype(np.float16) * np.float16(3.0)
    b = np.clip(rng.standard_normal(4096) * np.exp(4.0 * rng.standard_normal(4096)), -6e4, 6e4).astype(np.float16)
    special_a = np.array([2048, 2048, 1, 65504, 65504, -65504, 6e-8, 6e-8, 1024, 0.1, 4096, 4096],
                         dtype=np.float16)
    special_b = np.array([1, 3, 2.0 ** -11, 16, 32, 65504, 6e-8, -6e-8, 0.5, -0.1, 2.0 ** -14, 2],
                         dtype=np.float16)
    a = np.concatenate([a, special_a, np.zeros(4, np.float16)])[:4096 + 16]
    b = np.concatenate([b, special_b, np.zeros(4, np.float16)])[:4096 + 16]
    K = 128 * ((a.size + 127) // 128)                     # whole groups; the rest stays zero
    x = np.zeros((1, K), np.float16)
    r = np.zeros((1, K), np.float16)
    x[0, :a.size], r[0, :b.size] = a, b
    idx = np.arange(K, dtype=np.int32)
    with np.errstate(over="ignore"):
        want = (x.astype(np.float64) + r.astype(np.float64)).astype(np.float16)
    # keep the quantiser's inputs finite: the sum itself is what is pinned here
    finite = np.isfinite(want)
    x[~finite] = 0
    r[~finite] = 0
    want[~finite] = 0
    h, q4, q8, sc = oracle.add_quantize_act(x, r, None, 0.0, idx, 128, 128, 1.0)
    assert np.array_equal(h.view(np.uint16), want.view(np.uint16))
    # the one overflowing pair, on its own: 65504 + 32 rounds to infinity in fp16
    assert oracle.f32_to_f16(np.float32(65504.0) + np.float32(32.0)) == 0x7C00


def test_add_quantize_is_quantize_of_the_sum():
    """The fused entry point equals the plain front end applied to the rounded sum (whose own
    pins are above), with and without RMSNorm, and the sum is returned."""
    rng = np.random.default_rng(8)
    M, K = 5, 512
    x = (rng.standard_normal((M, K)) * np.exp(rng.standard_normal(K))).astype(np.float16)
    r = (rng.standard_normal((M, K)) * 0.5).astype(np.float16)
    gamma = (1 + 0.1 * rng.standard_normal(K)).astype(np.float16)
    idx = rng.permutation(K).astype(np.int32)
    hsum = (x.astype(np.float64) + r.astype(np.float64)).astype(np.float16)
    for g, eps in ((gamma, 1e-6), (None, 0.0)):
        h, q4, q8, sc = oracle.add_quantize_act(x, r, g, eps, idx, 128, 128, 0.9)
        w4, w8, wsc = oracle.quantize_act(hsum, g, eps, idx, 128, 128, 0.9)
        assert np.array_equal(h.view(np.uint16), hsum.view(np.uint16))
        assert np.array_equal(q4, w4) and np.array_equal(q8, w8)
        assert np.array_equal(sc.view(np.uint16), wsc.view(np.uint16))
    # a planted mistake (sum rounded to fp16 only after the norm, i.e. norm on the fp32 sum)
    # must be visible: x + r has fp16 rounding error in most elements
    assert np.any(hsum.astype(np.float32) != x.astype(np.float32) + r.astype(np.float32))


# ---------------------------------------------------------------- SwiGLU in front


def test_expf_against_float64():
    """The oracle's exp is a fixed sequence of IEEE operations; the pin is the libm exp in
    float64.  A dropped polynomial term (1e-4 and worse), a wrong ln2 split or a wrong sign
    in the range reduction all exceed the bound by orders of magnitude."""
    import math
    xs = np.concatenate([np.linspace(-87, 87, 20001), np.linspace(-0.4, 0.4, 2001),
                         np.array([0.0, 1.0, -1.0, 0.34657359, -0.34657359, 86.999, -86.999])])
    worst = 0.0
    for x in xs.astype(np.float32):
        got = oracle.expf(x)
        ref = math.exp(float(x))
        worst = max(worst, abs(got - ref) / ref)
    assert worst < 1.0e-7, worst                   # under one fp32 ulp; the degree-7 term alone is 1.2e-7
    assert oracle.expf(0.0) == 1.0
    assert oracle.expf(-1000.0) == oracle.expf(-87.0)      # clamped, still a normal number
    assert oracle.expf(1000.0) == oracle.expf(87.0)
    assert oracle.expf(-87.0) > 1.1754944e-38


def test_silu_mul_against_float64_for_every_fp16_gate():
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    g = bits.view(np.float16)
    g = g[np.isfinite(g)]
    u = np.full(g.shape, 1.5, np.float16)
    got = oracle.silu_mul(g, u).astype(np.float64)
    g64 = g.astype(np.float64)
    with np.errstate(over="ignore"):
        ref = g64 / (1.0 + np.exp(-g64)) * 1.5
    # gates below -87 are clamped in the exp: silu there is below 1e-35 in magnitude either way
    main = g64 > -87.0
    err = np.abs(got[main] - ref[main])
    assert np.all(err <= 6e-7 * np.abs(ref[main]) + 1e-40), (err / (np.abs(ref[main]) + 1e-300)).max()
    assert np.all(np.abs(got[~main]) < 1e-32)
    # closed forms: silu(0) = 0; sigma rounds to 1 for large gates, so y = g*u exactly
    assert oracle.silu_mul(np.array([0.0], np.float16), np.array([3.0], np.float16))[0] == 0.0
    big = np.array([20.0, 100.0, 1000.0], np.float16)
    assert np.array_equal(oracle.silu_mul(big, np.array([2.0, 0.5, -4.0], np.float16)),
                          np.array([40.0, 50.0, -4000.0], np.float32))
    # the order of the two multiplies is part of the contract: (g*sigma)*u, not g*(sigma*u)
    gg, uu = np.array([1.2373046875], np.float16), np.array([0.337158203125], np.float16)
    sig = np.float32(1.0) / (np.float32(1.0) + np.float32(oracle.expf(-np.float32(gg[0]))))
    assert oracle.silu_mul(gg, uu)[0] == (np.float32(gg[0]) * sig) * np.float32(uu[0])


def test_swiglu_quantize_reduces_to_the_plain_front_end():
    """Where sigma(g) rounds to exactly 1 and g*u is exact in fp16, silu(g)*u is an fp16
    number and the fused entry point must equal the (pinned) plain front end on it; a
    second case checks codes and scales on general values by re-deriving them from the
    fp32 rows with exact rationals."""
    from fractions import Fraction
    rng = np.random.default_rng(11)
    M, K = 4, 256
    g = rng.integers(20, 60, size=(M, K)).astype(np.float16)            # sigma == 1
    u = rng.choice(np.array([0.5, 1.0, 2.0, -1.0, -0.25], np.float16), size=(M, K))
    idx = rng.permutation(K).astype(np.int32)
    y16 = (g.astype(np.float32) * u.astype(np.float32)).astype(np.float16)
    assert np.array_equal(y16.astype(np.float32), oracle.silu_mul(g, u))
    got = oracle.swiglu_quantize_act(g, u, idx, 128, 128, 0.9)
    want = oracle.quantize_act(y16, None, 0.0, idx, 128, 128, 0.9)
    for a, b in zip(got, want):
        assert np.array_equal(a.view(np.uint8), b.view(np.uint8))
    # general values: one row, exact-rational scale and codes from the oracle's own fp32 y
    g = (rng.standard_normal((1, K)) * 3).astype(np.float16)
    u = (rng.standard_normal((1, K)) * 2).astype(np.float16)
    idx = np.arange(K, dtype=np.int32)
    q4, q8, sc = oracle.swiglu_quantize_act(g, u, idx, 128, 128, 1.0)
    y = oracle.silu_mul(g, u)[0]
    amax = max(abs(float(v)) for v in y[:128])
    s32 = np.float32(np.float32(np.float32(2.0) * np.float32(amax)) * np.float32(1.0)) / np.float32(15.0)
    assert sc[0, 0] == np.float16(s32)
    s = Fraction(float(sc[0, 0]))
    for j in range(0, 128, 7):
        qf = np.float32(np.float32(y[j]) / np.float32(sc[0, 0]))            # IEEE fp32 division
        t = Fraction(float(qf))
        fl = t.numerator // t.denominator
        frac = t - fl
        q = fl + (1 if frac > Fraction(1, 2) or (frac == Fraction(1, 2) and fl % 2) else 0)
        q = max(-8, min(7, q))
        nib = (int(q4[0, j // 2]) >> (4 * (j % 2))) & 0xF
        assert (nib - 16 if nib >= 8 else nib) == q, (j, q, nib)
    assert s > 0


# ------------------------------------------------------------ W3A3 -------

def test_three_bit_codes_ranges_fused_variants_and_gemm():
    """The W3A3 configuration (Section 5.2): normal channels at n = 3.  Codes stay in [-4, 3]
    and reach both ends; the outlier block is untouched by the width; the fused front ends
    and the weight path take the width the same way; and the unchanged GEMM on 3-bit codes
    equals the float64 product of the dequantised operands."""
    rng = np.random.default_rng(33)
    M, N, K, Gs, O = 5, 6, 64, 16, 16
    x = (rng.standard_normal((M, K)) * np.exp(rng.uniform(-1, 1, (1, K)))).astype(np.float16)
    w = (rng.standard_normal((N, K)) * 0.05).astype(np.float16)
    idx = rng.permutation(K).astype(np.int32)
    a3 = oracle.quantize_act(x, None, 0.0, idx, Gs, O, 1.0, bits=3)
    a4 = oracle.quantize_act(x, None, 0.0, idx, Gs, O, 1.0, bits=4)
    c3 = np_unpack(a3[0], a3[1])
    assert c3[:, :K - O].min() == -4 and c3[:, :K - O].max() == 3
    assert np.array_equal(a3[1], a4[1])                                  # INT8 block: same codes
    assert np.array_equal(a3[2][:, (K - O) // Gs:], a4[2][:, (K - O) // Gs:])    # and same scales
    # scale ratio of a normal group: (2 amax c / 7) / (2 amax c / 15) = 15 / 7 up to fp16 rounding
    r = a3[2][:, :(K - O) // Gs].astype(np.float64) / a4[2][:, :(K - O) // Gs].astype(np.float64)
    assert np.all(np.abs(r - 15.0 / 7.0) < 15.0 / 7.0 * 2.0 ** -9)
    # weight path and fused variants
    w3 = oracle.quantize_weight(w, idx, Gs, O, 0.85, bits=3)
    w3b = oracle.quantize_act(w, None, 0.0, idx, Gs, O, 0.85, bits=3)
    assert all(np.array_equal(u, v) for u, v in zip(w3, w3b))
    res = (rng.standard_normal((M, K)) * 0.5).astype(np.float16)
    gamma = (1.0 + 0.1 * rng.standard_normal(K)).astype(np.float16)
    h, *q = oracle.add_quantize_act(x, res, gamma, 1e-5, idx, Gs, O, 0.9, bits=3)
    q_ref = oracle.quantize_act(h, gamma, 1e-5, idx, Gs, O, 0.9, bits=3)
    assert all(np.array_equal(u, v) for u, v in zip(q, q_ref))
    # silu(32) = 32 to fp32 rounding and 32 x is an fp16 number: SwiGLU in front reduces to the
    # plain front end on 32 x
    big = np.full((M, K), 32.0, np.float16)
    assert np.array_equal(oracle.silu_mul(big, x), np.float32(32.0) * x.astype(np.float32))
    sg = oracle.swiglu_quantize_act(big, x, idx, Gs, O, 0.9, bits=3)
    sref = oracle.quantize_act((np.float32(32.0) * x.astype(np.float32)).astype(np.float16), None, 0.0, idx,
                               Gs, O, 0.9, bits=3)
    assert all(np.array_equal(u, v) for u, v in zip(sg, sref))
    # GEMM on 3-bit operands against float64
    y16 = oracle.w4a4_gemm(*a3, *w3, group_size=Gs)["y"]
    ca, cw = np_unpack(a3[0], a3[1]).astype(np.float64), np_unpack(w3[0], w3[1]).astype(np.float64)
    sa = np.repeat(a3[2].astype(np.float64), Gs, axis=1)
    sw = np.repeat(w3[2].astype(np.float64), Gs, axis=1)
    ref = (ca * sa) @ (cw * sw).T
    assert np.allclose(y16.astype(np.float64), ref, rtol=2e-3, atol=1e-6)
