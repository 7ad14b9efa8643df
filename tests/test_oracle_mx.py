"""Pins of the oracle's MX (microscaling) variant (CPU only): FP4 E2M1 normal channels, FP8
E4M3 outliers, one E8M0 scale per block of 32.  The paper (Section 5.2, FP4 paragraph)
evaluates its recipe in FP4 and names the MX formats; the formats themselves are fixed by the
specification it cites.  Pinned against a hand-worked example, torch's float8_e4m3fn, exact
rationals, closed forms, invariants and a float64 numpy matmul."""
import json
import math
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

import oracle

GOLD = os.path.join(os.path.dirname(__file__), "golden", "mx_worked_example.json")
E2M1 = [Fraction(0), Fraction(1, 2), Fraction(1), Fraction(3, 2), Fraction(2), Fraction(3), Fraction(4), Fraction(6)]


def _unpack4(q):
    lo, hi = (q & 0xF).astype(np.int32), (q >> 4).astype(np.int32)
    return np.stack([lo, hi], axis=-1).reshape(q.shape[:-1] + (2 * q.shape[-1],))


def _e4m3_table():
    codes = torch.arange(256, dtype=torch.int32).to(torch.uint8)
    return codes.view(torch.float8_e4m3fn).to(torch.float32).numpy()


def _decode(q4, q8, e8):
    """float64 [rows, K] from the three arrays, with a table typed here and torch's FP8."""
    fp4 = np.array([float(v) for v in E2M1] + [-float(v) for v in E2M1])
    a4 = fp4[_unpack4(q4)]
    a8 = _e4m3_table().astype(np.float64)[q8]
    a = np.concatenate([a4, a8], axis=1)
    return a * np.repeat(np.exp2(e8.astype(np.float64) - 127.0), 32, axis=1)


def test_worked_example():
    g = json.load(open(GOLD))
    x = np.array([g["x"]], np.float16)
    idx = np.arange(g["K"], dtype=np.int32)
    q4, q8, e8 = oracle.mx_quantize_act(x, None, 0.0, idx, g["n_outlier"], g["clip"])
    assert e8[0].tolist() == g["scale_bytes"]
    assert _unpack4(q4)[0].tolist() == g["fp4_codes"]
    assert q8[0].tolist() == g["fp8_codes"]


def test_e4m3_decode_is_torch_float8_e4m3fn():
    ref = _e4m3_table()
    for c in range(256):
        v = oracle.e4m3_to_f32(c)
        if np.isnan(ref[c]):
            assert math.isnan(v) and c in (0x7F, 0xFF)
        else:
            assert v == ref[c] and math.copysign(1, v) == math.copysign(1, ref[c])


def test_e4m3_encode_against_torch_cast_and_saturation():
    rng = np.random.default_rng(0)
    v = np.concatenate([rng.standard_normal(4000) * np.exp2(rng.integers(-12, 9, 4000)),
                        rng.uniform(-448, 448, 2000)]).astype(np.float32)
    v = v[np.abs(v) <= 448]
    ref = torch.from_numpy(v).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    got = np.array([oracle.f32_to_e4m3(x) for x in v], np.uint8)
    same_value = _e4m3_table()[got] == _e4m3_table()[ref]          # -0 and +0 compare equal
    assert same_value.all()
    # every midpoint between neighbours goes to the even code; beyond 448 saturates
    tab = _e4m3_table()
    for c in range(0x7E):
        mid = (Fraction(float(tab[c])) + Fraction(float(tab[c + 1]))) / 2
        assert oracle.f32_to_e4m3(float(mid)) == (c if c % 2 == 0 else c + 1)
        assert oracle.f32_to_e4m3(-float(mid)) == 0x80 | (c if c % 2 == 0 else c + 1)
    for big in (448.0, 449.0, 464.0, 480.0, 1e6, 3e38):
        assert oracle.f32_to_e4m3(big) == 0x7E and oracle.f32_to_e4m3(-big) == 0xFE


def test_e2m1_encode_exact_rationals():
    """Nearest of the eight magnitudes by exact arithmetic, ties to the even code."""
    rng = np.random.default_rng(1)
    vals = list(rng.uniform(-7, 7, 3000).astype(np.float32)) + [k / 8 for k in range(-64, 65)]
    for v in vals:
        fr = abs(Fraction(float(np.float32(v))))
        best = min(range(8), key=lambda c: (abs(fr - E2M1[c]), c % 2))
        want = best | (8 if math.copysign(1, float(v)) < 0 else 0)
        assert oracle.f32_to_e2m1(v) == want, v
    assert [oracle.e2m1_to_f32(c) for c in range(8)] == [float(x) for x in E2M1]
    assert [oracle.e2m1_to_f32(c + 8) for c in range(1, 8)] == [-float(x) for x in E2M1[1:]]


def test_scale_byte_closed_form():
    for emax in (2, 8):
        for e in range(-140, 128):
            for f in (1.0, 1.0000001, 1.5, 1.9999999):
                a = np.float32(f) * np.float32(2.0) ** np.float32(e) if e > -127 else np.float32(f * 2.0 ** e)
                if not np.isfinite(a) or a == 0:
                    continue
                fl = math.floor(math.log2(Fraction(float(a))))
                want = min(max(fl - emax, -127), 127) + 127
                assert oracle.mx_scale_byte(a, emax) == want, (a, emax)
        assert oracle.mx_scale_byte(0.0, emax) == 0


def _rand_rows(rows, K, seed):
    rng = np.random.default_rng(seed)
    sigma = np.exp(1.5 * rng.standard_normal(K))
    x = (rng.standard_normal((rows, K)) * sigma).astype(np.float16)
    idx = np.argsort(sigma, kind="stable").astype(np.int32)
    return x, idx


@pytest.mark.parametrize("clip", [1.0, 0.9])
def test_quantise_rederived_with_exact_rationals(clip):
    x, idx = _rand_rows(6, 256, 2)
    O = 64
    q4, q8, e8 = oracle.mx_quantize_act(x, None, 0.0, idx, O, clip)
    codes4 = _unpack4(q4)
    tab8 = [Fraction(float(v)) for v in _e4m3_table()[:0x7F]]
    for r in range(x.shape[0]):
        y = x[r].astype(np.float32)[idx]
        for b in range(256 // 32):
            blk = y[32 * b:32 * b + 32]
            a = np.float32(np.abs(blk).max()) * np.float32(clip)
            fp4 = 32 * b < 256 - O
            emax = 2 if fp4 else 8
            E = min(max(math.floor(math.log2(Fraction(float(a)))) - emax, -127), 127) if a > 0 else -127
            assert int(e8[r, b]) == E + 127
            for t in range(0, 32, 3):
                v = Fraction(float(blk[t])) / (Fraction(2) ** E)
                table = E2M1 if fp4 else tab8
                best = min(range(len(table)), key=lambda c: (abs(abs(v) - table[c]), c % 2))
                got = int(codes4[r, 32 * b + t]) if fp4 else int(q8[r, 32 * b + t - (256 - O)])
                mag = got & (7 if fp4 else 0x7F)
                assert mag == best
                if v != 0:
                    assert bool(got & (8 if fp4 else 0x80)) == (v < 0)


def test_invariants():
    x, idx = _rand_rows(16, 512, 3)
    q = oracle.mx_quantize_act(x, None, 0.0, idx, 128, 1.0)
    # scaling the row by a power of two moves the scale bytes and leaves the codes alone
    q2 = oracle.mx_quantize_act((x.astype(np.float32) * 4).astype(np.float16), None, 0.0, idx, 128, 1.0)
    assert np.array_equal(q[0], q2[0]) and np.array_equal(q[1], q2[1])
    assert np.array_equal(q[2].astype(int) + 2, q2[2].astype(int))
    # with clip 1 the largest element of a block lands in the top binade [4, 8) resp. [256, 512);
    # below the largest magnitude (6 resp. 448) the error is at most half the local spacing,
    # above it the element saturates
    y = x.astype(np.float64)[:, idx]
    deq = _decode(*q)
    scale = np.repeat(np.exp2(q[2].astype(np.float64) - 127), 32, axis=1)
    v = np.abs(y) / scale
    K4 = 512 - 128
    v4 = v[:, :K4]
    half4 = np.where(v4 < 2, 0.25, np.where(v4 < 4, 0.5, np.where(v4 <= 6, 1.0, v4 - 6)))
    assert (v4 < 8).all() and (np.abs(y - deq)[:, :K4] <= half4 * scale[:, :K4] * (1 + 1e-12)).all()
    v8 = v[:, K4:]
    bound8 = np.where(v8 <= 448, np.maximum(v8 / 16, 2.0 ** -10), v8 - 448)
    assert (v8 < 512).all() and (np.abs(y - deq)[:, K4:] <= bound8 * scale[:, K4:] * (1 + 1e-12)).all()
    top4 = np.abs(_unpack4(q[0]) & 7).reshape(16, -1, 32).max(axis=2)
    assert (top4 >= 6).all()                        # amax / 2^E is in [4, 8): code 6 or 7
    # permuting channels inside one block permutes its codes and leaves its scale alone
    perm = idx.copy()
    perm[:32] = perm[:32][::-1]
    qp = oracle.mx_quantize_act(x, None, 0.0, perm, 128, 1.0)
    assert np.array_equal(qp[2], q[2])
    assert np.array_equal(_unpack4(qp[0])[:, :32], _unpack4(q[0])[:, :32][:, ::-1])
    assert np.array_equal(_unpack4(qp[0])[:, 32:], _unpack4(q[0])[:, 32:])
    # an all-zero block
    z = np.zeros((1, 64), np.float16)
    qz = oracle.mx_quantize_act(z, None, 0.0, np.arange(64, dtype=np.int32), 32, 1.0)
    assert not qz[0].any() and not qz[1].any() and not qz[2].any()


def test_norm_front_end_is_rmsnorm_then_quantise():
    """With gamma the rows are RMS-normalised first (fp32, the pinned oracle routine), and the
    result matches quantising an fp16-exact pre-normalised row."""
    K = 128
    x = np.zeros((1, K), np.float16)
    x[0, :] = 2.0
    x[0, ::2] = -2.0                                  # mean square 4 -> r = 0.5 -> y = +-1 * gamma
    gamma = (np.arange(K) % 8 + 1).astype(np.float16) / 2
    idx = np.arange(K, dtype=np.int32)
    a = oracle.mx_quantize_act(x, gamma, 0.0, idx, 32, 1.0)
    y = (np.where(np.arange(K) % 2 == 0, -1.0, 1.0) * gamma.astype(np.float64)).astype(np.float16)[None]
    b = oracle.mx_quantize_act(y, None, 0.0, idx, 32, 1.0)
    for u, v in zip(a, b):
        assert np.array_equal(u, v)


def test_gemm_is_float64_matmul_of_the_dequantised_operands():
    x, idx = _rand_rows(9, 384, 4)
    rng = np.random.default_rng(5)
    w = (0.02 * rng.standard_normal((13, 384))).astype(np.float16)
    qa = oracle.mx_quantize_act(x, None, 0.0, idx, 128, 0.9)
    qw = oracle.mx_quantize_weight(w, idx, 128, 0.85)
    y = oracle.mx_gemm(*qa, *qw).astype(np.float64)
    ref = _decode(*qa) @ _decode(*qw).T
    assert np.abs(y - ref).max() <= np.abs(ref).max() * 2.0 ** -10
    assert (np.abs(y - ref) <= np.abs(ref) * 2.0 ** -10 + 1e-12).all()
    # and it tracks the unquantised product about as well as 4 bits can
    full = x.astype(np.float64)[:, idx] @ w.astype(np.float64)[:, idx].T
    assert np.abs(y - full).max() < 0.25 * np.abs(full).max()
