"""CPU oracle for the Atom W4A4 hot path -- TEST INFRASTRUCTURE ONLY.

A plain single-threaded C implementation (``atom_ref.c``) with a numpy/ctypes
wrapper.  Only the tests, the smoke check and the benchmark's CPU-baseline leg
may import this package; the product (``paper_2310_19102_amd``) never does, and
this package never imports the product.

fp16 tensors are numpy ``float16`` arrays; codes are ``uint8`` (two INT4 per
byte, even column in the low nibble) and ``int8``.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "atom_ref.c")
_LIB = os.path.join(_HERE, "libatom_ref.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile ``atom_ref.c`` with gcc into ``libatom_ref.so`` next to it."""
    stale = (not os.path.exists(_LIB)
             or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
             or os.path.getmtime(_LIB) < os.path.getmtime(os.path.join(_HERE, "atom_ref.h")))
    if force or stale:
        cmd = ["gcc", "-O2", "-ftree-vectorize", "-ffp-contract=off", "-fno-fast-math",
               "-std=c11", "-Wall", "-Wextra", "-shared", "-fPIC", _SRC, "-o", _LIB, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is not None:
        return _lib
    build()
    L = ctypes.CDLL(_LIB)
    vp, i64, i32, f32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32, ctypes.c_float
    L.atom_ref_f16_to_f32.restype = f32
    L.atom_ref_f16_to_f32.argtypes = [ctypes.c_uint16]
    L.atom_ref_f32_to_f16.restype = ctypes.c_uint16
    L.atom_ref_f32_to_f16.argtypes = [f32]
    L.atom_ref_sumsq.restype = f32
    L.atom_ref_sumsq.argtypes = [vp, i32]
    L.atom_ref_rmsnorm_row.restype = None
    L.atom_ref_rmsnorm_row.argtypes = [vp, vp, f32, i32, vp]
    L.atom_ref_quantize_act.restype = ctypes.c_int
    L.atom_ref_quantize_act.argtypes = [vp, i64, i64, vp, f32, vp, i32, i32, i32, f32, vp, vp, vp]
    L.atom_ref_add_quantize_act.restype = ctypes.c_int
    L.atom_ref_add_quantize_act.argtypes = [vp, vp, i64, i64, i64, vp, i64, vp, f32, vp, i32, i32,
                                            i32, f32, vp, vp, vp]
    L.atom_ref_expf.restype = f32
    L.atom_ref_expf.argtypes = [f32]
    L.atom_ref_silu_mul.restype = f32
    L.atom_ref_silu_mul.argtypes = [ctypes.c_uint16, ctypes.c_uint16]
    L.atom_ref_swiglu_quantize_act.restype = ctypes.c_int
    L.atom_ref_swiglu_quantize_act.argtypes = [vp, vp, i64, i64, i64, vp, i32, i32, i32, f32, vp, vp, vp]
    L.atom_ref_kv_quantize.restype = ctypes.c_int
    L.atom_ref_kv_quantize.argtypes = [vp, i64, i64, i32, f32, vp, vp, vp]
    L.atom_ref_kv_dequant.restype = f32
    L.atom_ref_kv_dequant.argtypes = [ctypes.c_uint8, ctypes.c_uint16, ctypes.c_int16]
    L.atom_ref_decode_attention_kv4.restype = ctypes.c_int
    L.atom_ref_decode_attention_kv4.argtypes = [vp, i32, i32, i32, i32, i32, vp, vp, vp, vp, vp, vp,
                                                vp, f32, vp]
    u8 = ctypes.c_uint8
    L.atom_ref_e2m1_to_f32.restype = f32
    L.atom_ref_e2m1_to_f32.argtypes = [u8]
    L.atom_ref_e4m3_to_f32.restype = f32
    L.atom_ref_e4m3_to_f32.argtypes = [u8]
    L.atom_ref_f32_to_e2m1.restype = u8
    L.atom_ref_f32_to_e2m1.argtypes = [f32]
    L.atom_ref_f32_to_e4m3.restype = u8
    L.atom_ref_f32_to_e4m3.argtypes = [f32]
    L.atom_ref_mx_scale_byte.restype = u8
    L.atom_ref_mx_scale_byte.argtypes = [f32, ctypes.c_int]
    L.atom_ref_mx_quantize_act.restype = ctypes.c_int
    L.atom_ref_mx_quantize_act.argtypes = [vp, i64, i64, vp, f32, vp, i32, i32, f32, vp, vp, vp]
    L.atom_ref_mx_gemm.restype = ctypes.c_int
    L.atom_ref_mx_gemm.argtypes = [vp, vp, vp, i64, vp, vp, vp, i64, i32, i32, vp, i64]
    L.atom_ref_calibrate_reorder.restype = ctypes.c_int
    L.atom_ref_calibrate_reorder.argtypes = [vp, i64, i64, i32, vp, vp]
    L.atom_ref_quantize_weight.restype = ctypes.c_int
    L.atom_ref_quantize_weight.argtypes = [vp, i64, i64, vp, i32, i32, i32, f32, vp, vp, vp]
    L.atom_ref_quantize_act_n.restype = ctypes.c_int
    L.atom_ref_quantize_act_n.argtypes = [vp, i64, i64, vp, f32, vp, i32, i32, i32, i32, f32, vp, vp, vp]
    L.atom_ref_add_quantize_act_n.restype = ctypes.c_int
    L.atom_ref_add_quantize_act_n.argtypes = [vp, vp, i64, i64, i64, vp, i64, vp, f32, vp, i32, i32,
                                              i32, i32, f32, vp, vp, vp]
    L.atom_ref_swiglu_quantize_act_n.restype = ctypes.c_int
    L.atom_ref_swiglu_quantize_act_n.argtypes = [vp, vp, i64, i64, i64, vp, i32, i32, i32, i32, f32, vp, vp, vp]
    L.atom_ref_w4a4_gemm.restype = ctypes.c_int
    L.atom_ref_w4a4_gemm.argtypes = [vp, vp, vp, i64, vp, vp, vp, i64, i32, i32, i32,
                                     vp, i64, vp, vp]
    _lib = L
    return L


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _c(a, dtype):
    a = np.ascontiguousarray(a)
    if a.dtype != dtype:
        raise TypeError(f"expected {dtype}, got {a.dtype}")
    return a


def f16_to_f32(bits: int) -> float:
    return float(_load().atom_ref_f16_to_f32(int(bits) & 0xFFFF))


def f32_to_f16(value) -> int:
    return int(_load().atom_ref_f32_to_f16(np.float32(value)))


def sumsq(x_row: np.ndarray) -> np.float32:
    x = _c(x_row, np.float16)
    return np.float32(_load().atom_ref_sumsq(_p(x), x.shape[0]))


def rmsnorm_row(x_row: np.ndarray, gamma, eps: float) -> np.ndarray:
    x = _c(x_row, np.float16)
    g = None if gamma is None else _c(gamma, np.float16)
    y = np.empty(x.shape[0], np.float32)
    _load().atom_ref_rmsnorm_row(_p(x), _p(g), eps, x.shape[0], _p(y))
    return y


def quantize_act(x, gamma, eps, idx, group_size=128, n_outlier=128, clip=0.9, bits=4):
    """Returns (q4 uint8 [M,K4/2], q8 int8 [M,O], scale float16 [M,G]).  ``bits``: width of
    the normal channels, 4 or 3 (codes of either width sit sign-extended in nibbles)."""
    x = _c(x, np.float16)
    M, K = x.shape
    g = None if gamma is None else _c(gamma, np.float16)
    idx = _c(idx, np.int32)
    K4, G = K - n_outlier, K // group_size
    q4 = np.zeros((M, K4 // 2), np.uint8)
    q8 = np.zeros((M, n_outlier), np.int8)
    sc = np.zeros((M, G), np.float16)
    rc = _load().atom_ref_quantize_act_n(_p(x), M, K, _p(g), eps, _p(idx), K, group_size,
                                         n_outlier, bits, clip, _p(q4), _p(q8), _p(sc))
    if rc != 0:
        raise ValueError("atom_ref_quantize_act: bad shapes")
    return q4, q8, sc


def add_quantize_act(x, res, gamma, eps, idx, group_size=128, n_outlier=128, clip=0.9, bits=4):
    """Residual add fused in front of the front end.
    Returns (sum float16 [M,K], q4, q8, scale)."""
    x, res = _c(x, np.float16), _c(res, np.float16)
    M, K = x.shape
    g = None if gamma is None else _c(gamma, np.float16)
    idx = _c(idx, np.int32)
    K4, G = K - n_outlier, K // group_size
    h = np.zeros((M, K), np.float16)
    q4 = np.zeros((M, K4 // 2), np.uint8)
    q8 = np.zeros((M, n_outlier), np.int8)
    sc = np.zeros((M, G), np.float16)
    rc = _load().atom_ref_add_quantize_act_n(_p(x), _p(res), M, K, K, _p(h), K, _p(g), eps,
                                             _p(idx), K, group_size, n_outlier, bits, clip, _p(q4),
                                             _p(q8), _p(sc))
    if rc != 0:
        raise ValueError("atom_ref_add_quantize_act: bad shapes")
    return h, q4, q8, sc


def expf(x) -> float:
    return float(_load().atom_ref_expf(float(np.float32(x))))


def silu_mul(gate, up):
    """(g * sigma(g)) * u in fp32 for fp16 arrays of equal shape; float32 array."""
    g, u = _c(gate, np.float16), _c(up, np.float16)
    L = _load()
    out = np.empty(g.shape, np.float32)
    gb, ub = g.view(np.uint16).ravel(), u.view(np.uint16).ravel()
    flat = out.ravel()
    for i in range(gb.size):
        flat[i] = L.atom_ref_silu_mul(int(gb[i]), int(ub[i]))
    return out


def swiglu_quantize_act(gate, up, idx, group_size=128, n_outlier=128, clip=0.9, bits=4):
    """silu(gate)*up fused in front of reorder + group quantisation.
    Returns (q4, q8, scale)."""
    g, u = _c(gate, np.float16), _c(up, np.float16)
    M, K = g.shape
    idx = _c(idx, np.int32)
    K4, G = K - n_outlier, K // group_size
    q4 = np.zeros((M, K4 // 2), np.uint8)
    q8 = np.zeros((M, n_outlier), np.int8)
    sc = np.zeros((M, G), np.float16)
    rc = _load().atom_ref_swiglu_quantize_act_n(_p(g), _p(u), M, K, K, _p(idx), K, group_size,
                                                n_outlier, bits, clip, _p(q4), _p(q8), _p(sc))
    if rc != 0:
        raise ValueError("atom_ref_swiglu_quantize_act: bad shapes")
    return q4, q8, sc


def quantize_weight(w, idx, group_size=128, n_outlier=128, clip=0.85, bits=4):
    """Returns (q4 uint8 [N,K4/2], q8 int8 [N,O], scale float16 [N,G])."""
    if bits != 4:
        return quantize_act(w, None, 0.0, idx, group_size, n_outlier, clip, bits)
    w = _c(w, np.float16)
    N, K = w.shape
    idx = _c(idx, np.int32)
    K4, G = K - n_outlier, K // group_size
    q4 = np.zeros((N, K4 // 2), np.uint8)
    q8 = np.zeros((N, n_outlier), np.int8)
    sc = np.zeros((N, G), np.float16)
    rc = _load().atom_ref_quantize_weight(_p(w), N, K, _p(idx), K, group_size, n_outlier,
                                          clip, _p(q4), _p(q8), _p(sc))
    if rc != 0:
        raise ValueError("atom_ref_quantize_weight: bad shapes")
    return q4, q8, sc


def w4a4_gemm(a_q4, a_q8, a_scale, w_q4, w_q8, w_scale, group_size=128,
              want_partials=False, want_acc=False):
    """Returns dict with 'y' float16 [M,N] and optionally 'partials' int32
    [M,N,G] and 'acc' float32 [M,N]."""
    a_q4, w_q4 = _c(a_q4, np.uint8), _c(w_q4, np.uint8)
    a_q8, w_q8 = _c(a_q8, np.int8), _c(w_q8, np.int8)
    a_scale, w_scale = _c(a_scale, np.float16), _c(w_scale, np.float16)
    M, N, O = a_q8.shape[0], w_q8.shape[0], a_q8.shape[1]
    K = a_q4.shape[1] * 2 + O
    G = K // group_size
    y = np.zeros((M, N), np.float16)
    part = np.zeros((M, N, G), np.int32) if want_partials else None
    acc = np.zeros((M, N), np.float32) if want_acc else None
    rc = _load().atom_ref_w4a4_gemm(_p(a_q4), _p(a_q8), _p(a_scale), M, _p(w_q4), _p(w_q8),
                                    _p(w_scale), N, K, group_size, O, _p(y), N, _p(part), _p(acc))
    if rc != 0:
        raise ValueError("atom_ref_w4a4_gemm: bad shapes")
    out = {"y": y}
    if want_partials:
        out["partials"] = part
    if want_acc:
        out["acc"] = acc
    return out


def kv_quantize(x, clip=1.0):
    """Asymmetric INT4 quantisation of rows of head_dim values: x float16 [..., D].
    Returns (codes uint8 [..., D/2], scale float16 [...], zero int16 [...])."""
    x = _c(x, np.float16)
    D = x.shape[-1]
    lead = x.shape[:-1]
    x2 = x.reshape(-1, D)
    R = x2.shape[0]
    q = np.zeros((R, D // 2), np.uint8)
    sc = np.zeros(R, np.float16)
    z = np.zeros(R, np.int16)
    rc = _load().atom_ref_kv_quantize(_p(x2), R, D, D, clip, _p(q), _p(sc), _p(z))
    if rc != 0:
        raise ValueError("atom_ref_kv_quantize: bad shapes")
    return q.reshape(lead + (D // 2,)), sc.reshape(lead), z.reshape(lead)


def kv_dequant(q, scale, zero):
    """float32 [..., D] from codes [..., D/2], scale [...], zero [...]."""
    q = _c(q, np.uint8)
    lo = (q & 0xF).astype(np.int32)
    hi = (q >> 4).astype(np.int32)
    codes = np.stack([lo, hi], axis=-1).reshape(q.shape[:-1] + (2 * q.shape[-1],))
    zz = np.asarray(zero, np.int32)[..., None]
    return (codes - zz).astype(np.float32) * np.asarray(scale, np.float16).astype(np.float32)[..., None]


def decode_attention_kv4(q, kq, ks, kz, vq, vs, vz, seq_len, sm_scale):
    """q float16 [B,H,D]; caches [B,Hkv,Tmax,...]; seq_len int32 [B].  Returns float16 [B,H,D]."""
    q = _c(q, np.float16)
    B, H, D = q.shape
    kq, vq = _c(kq, np.uint8), _c(vq, np.uint8)
    ks, vs = _c(ks, np.float16), _c(vs, np.float16)
    kz, vz = _c(kz, np.int16), _c(vz, np.int16)
    Hkv, Tmax = kq.shape[1], kq.shape[2]
    seq_len = _c(seq_len, np.int32)
    out = np.zeros((B, H, D), np.float16)
    rc = _load().atom_ref_decode_attention_kv4(_p(q), B, H, Hkv, D, Tmax, _p(seq_len), _p(kq),
                                               _p(ks), _p(kz), _p(vq), _p(vs), _p(vz), sm_scale,
                                               _p(out))
    if rc != 0:
        raise ValueError("atom_ref_decode_attention_kv4: bad shapes")
    return out


# ---- MX (microscaling) variant: FP4 E2M1 normal channels, FP8 E4M3 outliers, E8M0 scale per 32

def e2m1_to_f32(code):
    return float(_load().atom_ref_e2m1_to_f32(int(code)))


def e4m3_to_f32(code):
    return float(_load().atom_ref_e4m3_to_f32(int(code)))


def f32_to_e2m1(v):
    return int(_load().atom_ref_f32_to_e2m1(float(np.float32(v))))


def f32_to_e4m3(v):
    return int(_load().atom_ref_f32_to_e4m3(float(np.float32(v))))


def mx_scale_byte(clipped_amax, emax):
    return int(_load().atom_ref_mx_scale_byte(float(np.float32(clipped_amax)), int(emax)))


def mx_quantize_act(x, gamma, eps, idx, n_outlier=128, clip=1.0):
    """x float16 [M, K]; gamma float16 [K] or None (no norm).  Returns
    (q4 uint8 [M, K4/2], q8 uint8 [M, O], e8 uint8 [M, K/32])."""
    x = _c(x, np.float16)
    idx = _c(idx, np.int32)
    M, K = x.shape
    O = int(n_outlier)
    q4 = np.zeros((M, (K - O) // 2), np.uint8)
    q8 = np.zeros((M, O), np.uint8)
    e8 = np.zeros((M, K // 32), np.uint8)
    g = None if gamma is None else _c(gamma, np.float16)
    rc = _load().atom_ref_mx_quantize_act(_p(x), M, K, None if g is None else _p(g), eps, _p(idx), K, O,
                                          clip, _p(q4), _p(q8), _p(e8))
    if rc != 0:
        raise ValueError("atom_ref_mx_quantize_act: bad shapes")
    return q4, q8, e8


def mx_quantize_weight(w, idx, n_outlier=128, clip=1.0):
    return mx_quantize_act(w, None, 0.0, idx, n_outlier, clip)


def mx_gemm(a_q4, a_q8, a_e8, w_q4, w_q8, w_e8):
    """Y float16 [M, N] from the two MX-quantised operands."""
    a_q4, a_q8, a_e8 = _c(a_q4, np.uint8), _c(a_q8, np.uint8), _c(a_e8, np.uint8)
    w_q4, w_q8, w_e8 = _c(w_q4, np.uint8), _c(w_q8, np.uint8), _c(w_e8, np.uint8)
    M, O = a_q8.shape
    N = w_q8.shape[0]
    K = 2 * a_q4.shape[1] + O
    y = np.zeros((M, N), np.float16)
    rc = _load().atom_ref_mx_gemm(_p(a_q4), _p(a_q8), _p(a_e8), M, _p(w_q4), _p(w_q8), _p(w_e8), N, K, O,
                                  _p(y), N)
    if rc != 0:
        raise ValueError("atom_ref_mx_gemm: bad shapes")
    return y


def calibrate_reorder(x):
    """Per-channel square sums (float64 [K]) of calibration activations x float16 [T, K] and the
    reorder index (int32 [K], ascending by (square sum, channel), outliers last)."""
    x = _c(x, np.float16)
    T, K = x.shape
    stat = np.zeros(K, np.float64)
    idx = np.zeros(K, np.int32)
    rc = _load().atom_ref_calibrate_reorder(_p(x), T, K, K, _p(stat), _p(idx))
    if rc != 0:
        raise ValueError("atom_ref_calibrate_reorder: bad shapes")
    return stat, idx
