"""Pins of the oracle's INT4 KV-cache functions (CPU only).

Section 2 of the paper gives the asymmetric quantisation equations, Section 4.4 applies them
to the KV cache per attention head, Section 4.5 fuses the dequantisation into the decode
attention operator.  The oracle is pinned against a hand-worked example, an exact-rational
re-derivation, invariants, and an independent float64 numpy attention."""
import json
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle

GOLD = os.path.join(os.path.dirname(__file__), "golden", "kv_worked_example.json")


def _unpack(q):
    lo, hi = (q & 0xF).astype(np.int32), (q >> 4).astype(np.int32)
    return np.stack([lo, hi], axis=-1).reshape(q.shape[:-1] + (2 * q.shape[-1],))


def _rne(fr: Fraction) -> int:
    fl = fr.numerator // fr.denominator
    rem = fr - fl
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and fl % 2):
        return fl + 1
    return fl


def test_worked_example():
    g = json.load(open(GOLD))
    x = np.array([g["x"]], np.float16)
    q, s, z = oracle.kv_quantize(x, 1.0)
    assert float(s[0]) == g["scale"]
    assert int(z[0]) == g["zero"]
    assert q[0].tolist() == g["bytes"]
    assert _unpack(q)[0].tolist() == g["codes"]
    assert oracle.kv_dequant(q, s, z)[0].tolist() == g["dequant"]


@pytest.mark.parametrize("clip", [1.0, 0.9])
def test_exact_rational_rederivation(clip):
    """Scale, zero point and codes re-derived with numpy fp32 scalars for the IEEE steps and
    exact rationals for every rounding decision."""
    rng = np.random.default_rng(3)
    x = (rng.standard_normal((40, 128)) * np.exp(rng.standard_normal((40, 1))) + rng.standard_normal((40, 1))
         ).astype(np.float16)
    q, s, z = oracle.kv_quantize(x, clip)
    codes = _unpack(q)
    for r in range(x.shape[0]):
        row = x[r].astype(np.float32)
        s32 = np.float32(np.float32(row.max() - row.min()) * np.float32(clip)) / np.float32(15.0)
        assert s[r] == np.float16(s32)
        sf = np.float32(s[r])
        zz = _rne(Fraction(float(np.float32(-row.min()) / sf)))
        assert int(z[r]) == zz
        for d in range(0, 128, 5):
            t = _rne(Fraction(float(np.float32(row[d]) / sf))) + zz
            assert codes[r, d] == max(0, min(15, t)), (r, d)


def test_invariants_and_degenerate_rows():
    rng = np.random.default_rng(4)
    x = (rng.standard_normal((64, 128)) * 2 + 0.3).astype(np.float16)
    q, s, z = oracle.kv_quantize(x, 1.0)
    codes = _unpack(q)
    assert codes.min() >= 0 and codes.max() <= 15
    xh = oracle.kv_dequant(q, s, z).astype(np.float64)
    sf = s.astype(np.float64)[:, None]
    # at clip 1 the minimum maps to code 0 exactly (round is odd) and nothing is clamped by
    # more than one step at the top; the reconstruction error is at most half a step (+ the
    # clamped top code: one step)
    assert np.all(codes[np.arange(64), x.argmin(axis=1)] == 0)
    assert np.all(codes[np.arange(64), x.argmax(axis=1)] >= 14)
    err = np.abs(xh - x.astype(np.float64))
    assert np.all(err <= sf * (1.0 + 1e-3))
    assert np.mean(err <= sf * 0.5 * (1.0 + 1e-3)) > 0.97
    # constant row: zero scale, zero point 0, codes 0
    c = np.full((1, 128), 1.25, np.float16)
    q, s, z = oracle.kv_quantize(c, 1.0)
    assert s[0] == 0 and z[0] == 0 and not q.any()
    # all-negative row far from zero: the zero point is large, codes still span 0..15
    n = (-50 + rng.standard_normal((1, 128))).astype(np.float16)
    q, s, z = oracle.kv_quantize(n, 1.0)
    assert z[0] > 100 and _unpack(q).min() == 0 and _unpack(q).max() >= 14
    assert np.abs(oracle.kv_dequant(q, s, z) - n.astype(np.float32)).max() <= float(s[0]) * 1.001
    # dequantisation is (code - z) * s in fp32
    q, s, z = oracle.kv_quantize(x[:3], 0.9)
    want = (_unpack(q) - z.astype(np.int32)[:, None]).astype(np.float32) * s.astype(np.float32)[:, None]
    assert np.array_equal(oracle.kv_dequant(q, s, z), want)


def _numpy_attention(q, kq, ks, kz, vq, vs, vz, seq_len, sm_scale):
    B, H, D = q.shape
    Hkv = kq.shape[1]
    K = oracle.kv_dequant(kq, ks, kz).astype(np.float64)
    V = oracle.kv_dequant(vq, vs, vz).astype(np.float64)
    out = np.zeros((B, H, D))
    for b in range(B):
        T = int(seq_len[b])
        for h in range(H):
            kv = h // (H // Hkv)
            if T == 0:
                continue
            sc = (K[b, kv, :T] @ q[b, h].astype(np.float64)) * sm_scale
            p = np.exp(sc - sc.max())
            out[b, h] = (p / p.sum()) @ V[b, kv, :T]
    return out


def _random_cache(rng, B, Hkv, Tmax, D):
    k = (rng.standard_normal((B, Hkv, Tmax, D)) * 1.5).astype(np.float16)
    v = (rng.standard_normal((B, Hkv, Tmax, D)) + 0.2).astype(np.float16)
    return oracle.kv_quantize(k, 1.0) + oracle.kv_quantize(v, 1.0)


def test_attention_against_numpy_float64():
    rng = np.random.default_rng(5)
    B, H, Hkv, Tmax, D = 3, 8, 2, 70, 128
    cache = _random_cache(rng, B, Hkv, Tmax, D)
    q = rng.standard_normal((B, H, D)).astype(np.float16)
    seq_len = np.array([70, 33, 0], np.int32)
    # garbage beyond seq_len must not matter
    cache[0][1, :, 33:] = 0xFF
    cache[1][1, :, 33:] = np.float16(1000.0)
    out = oracle.decode_attention_kv4(q, *cache[:3], *cache[3:], seq_len, 1.0 / np.sqrt(D))
    ref = _numpy_attention(q, *cache[:3], *cache[3:], seq_len, 1.0 / np.sqrt(D))
    assert not out[2].any()
    err = np.abs(out.astype(np.float64) - ref)
    assert err.max() <= 2.0 ** -11 * np.abs(ref).max() + 1e-7          # one fp16 rounding
    # grouped query heads 0..3 read cache head 0, 4..7 cache head 1
    q2 = np.repeat(q[:, :1], H, axis=1)
    out2 = oracle.decode_attention_kv4(q2, *cache[:3], *cache[3:], seq_len, 0.1)
    assert np.array_equal(out2[:, 0], out2[:, 3]) and np.array_equal(out2[:, 4], out2[:, 7])
    assert not np.array_equal(out2[0, 0], out2[0, 4])


def test_attention_special_cases():
    rng = np.random.default_rng(6)
    B, H, Tmax, D = 2, 2, 9, 64
    kq, ks, kz, vq, vs, vz = _random_cache(rng, B, H, Tmax, D)
    q = rng.standard_normal((B, H, D)).astype(np.float16)
    V = oracle.kv_dequant(vq, vs, vz)
    # one token: the output is that token's dequantised value row
    out = oracle.decode_attention_kv4(q, kq, ks, kz, vq, vs, vz, np.array([1, 1], np.int32), 0.3)
    assert np.array_equal(out, V[:, :, 0].astype(np.float16))
    # zero softmax scale: plain mean over the tokens
    out = oracle.decode_attention_kv4(q, kq, ks, kz, vq, vs, vz, np.array([9, 4], np.int32), 0.0)
    want = np.stack([V[0, :, :9].astype(np.float64).mean(axis=1), V[1, :, :4].astype(np.float64).mean(axis=1)])
    assert np.abs(out.astype(np.float64) - want).max() <= 2.0 ** -11 * np.abs(want).max() + 1e-7
    # the order of the tokens does not matter
    perm = rng.permutation(9)
    out_a = oracle.decode_attention_kv4(q, kq, ks, kz, vq, vs, vz, np.array([9, 9], np.int32), 0.2)
    out_b = oracle.decode_attention_kv4(q, kq[:, :, perm], ks[:, :, perm], kz[:, :, perm], vq[:, :, perm],
                                        vs[:, :, perm], vz[:, :, perm], np.array([9, 9], np.int32), 0.2)
    assert np.abs(out_a.astype(np.float64) - out_b.astype(np.float64)).max() <= 2.0 ** -10 * np.abs(out_a).max()
    # a sharply peaked score picks one token: q aligned with one key, large scale
    k0 = oracle.kv_dequant(kq, ks, kz)[0, 0, 5]
    qq = np.zeros((B, H, D), np.float16)
    qq[0, 0] = k0.astype(np.float16)
    out = oracle.decode_attention_kv4(qq, kq, ks, kz, vq, vs, vz, np.array([9, 9], np.int32), 50.0)
    assert np.array_equal(out[0, 0], V[0, 0, 5].astype(np.float16))
