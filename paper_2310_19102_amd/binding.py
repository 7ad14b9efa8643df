"""ctypes binding of ``libatom.so``: argument marshalling only.

torch is used for device memory and the current HIP stream; no arithmetic of
the method happens in Python.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libatom.so")
_lib = None

EXPORTS = (
    "atom_quantize_act",
    "atom_add_quantize_act",
    "atom_swiglu_quantize_act",
    "atom_quantize_weight",
    "atom_w4a4_gemm",
    "atom_w4a4_gemm_workspace_bytes",
    "atom_tile_weight_decode_bytes",
    "atom_tile_weight_decode",
    "atom_w4a4_gemm_decode_tiled",
    "atom_permute_rows",
    "atom_decode_linear",
    "atom_decode_linear_coop",
    "atom_decode_linear_coop_sync_bytes",
    "atom_decode_linear_lds_bytes",
    "atom_pack_weight_bytes",
    "atom_pack_weight",
    "atom_w4a4_gemm_packed_workspace_bytes",
    "atom_w4a4_gemm_packed",
    "atom_pack_act",
    "atom_quantize_act_packed",
    "atom_add_quantize_act_packed",
    "atom_swiglu_quantize_act_packed",
    "atom_w4a4_gemm_prepacked",
    "atom_mx_quantize_act",
    "atom_mx_quantize_weight",
    "atom_mx_gemm",
    "atom_calibrate_reorder",
    "atom_calibrate_reorder_workspace_bytes",
    "atom_kv_quantize",
    "atom_kv_quantize_pair",
    "atom_decode_attention_kv4",
    "atom_decode_attention_kv4_workspace_bytes",
    "atom_decode_attention_kv4_static",
    "atom_static_scratch_bytes",
    "atom_mfma_rate_probe",
    "atom_check_reorder_idx",
    "atom_status_string",
)


class AtomError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {atom_status_string(status)} (status {status})")


class _Desc(ctypes.Structure):
    _fields_ = [("K", ctypes.c_int32), ("group_size", ctypes.c_int32), ("n_outlier", ctypes.c_int32),
                ("bits_normal", ctypes.c_int32), ("bits_outlier", ctypes.c_int32)]


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Load ``libatom.so`` built in-tree.  Raises if it is missing: there is
    no fallback path."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError(
            f"{_LIB_PATH} not found: build it with `python -m paper_2310_19102_amd.build` "
            "(hipcc, gfx950).  This package has no CPU or PyTorch fallback.")
    L = ctypes.CDLL(_LIB_PATH)
    vp, i64, f32, sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_float, ctypes.c_size_t
    i32 = ctypes.c_int32
    dp = ctypes.POINTER(_Desc)
    L.atom_quantize_act.restype = ctypes.c_int
    L.atom_quantize_act.argtypes = [vp, i64, i64, vp, f32, vp, dp, f32, vp, vp, vp, vp]
    L.atom_add_quantize_act.restype = ctypes.c_int
    L.atom_add_quantize_act.argtypes = [vp, vp, i64, i64, i64, vp, i64, vp, f32, vp, dp, f32, vp, vp, vp, vp]
    L.atom_swiglu_quantize_act.restype = ctypes.c_int
    L.atom_swiglu_quantize_act.argtypes = [vp, vp, i64, i64, i64, vp, dp, f32, vp, vp, vp, vp]
    L.atom_quantize_weight.restype = ctypes.c_int
    L.atom_quantize_weight.argtypes = [vp, i64, i64, vp, dp, f32, vp, vp, vp, vp]
    L.atom_w4a4_gemm.restype = ctypes.c_int
    L.atom_w4a4_gemm.argtypes = [vp, vp, vp, i64, vp, vp, vp, i64, dp, vp, i64, vp, vp, sz, vp]
    L.atom_w4a4_gemm_workspace_bytes.restype = sz
    L.atom_w4a4_gemm_workspace_bytes.argtypes = [i64, i64, dp]
    L.atom_tile_weight_decode_bytes.restype = sz
    L.atom_tile_weight_decode_bytes.argtypes = [i64, dp, i32]
    L.atom_tile_weight_decode.restype = ctypes.c_int
    L.atom_tile_weight_decode.argtypes = [vp, vp, i64, dp, vp, sz, vp, sz, vp]
    L.atom_w4a4_gemm_decode_tiled.restype = ctypes.c_int
    L.atom_w4a4_gemm_decode_tiled.argtypes = [vp, vp, vp, i64, vp, vp, vp, i64, dp, vp, i64, vp]
    L.atom_permute_rows.restype = ctypes.c_int
    L.atom_permute_rows.argtypes = [vp, i64, i64, i64, vp, i64, vp, i64, vp]
    L.atom_decode_linear.restype = ctypes.c_int
    L.atom_decode_linear.argtypes = [vp, i64, i64, vp, f32, vp, dp, f32, vp, vp, vp, i64, vp, i64, vp, vp, vp, vp]
    L.atom_decode_linear_coop_sync_bytes.restype = sz
    L.atom_decode_linear_coop_sync_bytes.argtypes = []
    L.atom_decode_linear_coop.restype = ctypes.c_int
    L.atom_decode_linear_coop.argtypes = [vp, i64, i64, vp, f32, vp, dp, f32, vp, vp, vp, i64, vp, i64, vp, vp, vp, vp, vp]
    L.atom_decode_linear_lds_bytes.restype = sz
    L.atom_decode_linear_lds_bytes.argtypes = [i64, dp, i32, i32]
    L.atom_pack_weight_bytes.restype = sz
    L.atom_pack_weight_bytes.argtypes = [i64, dp]
    L.atom_pack_weight.restype = ctypes.c_int
    L.atom_pack_weight.argtypes = [vp, vp, vp, i64, dp, vp, sz, vp]
    L.atom_w4a4_gemm_packed_workspace_bytes.restype = sz
    L.atom_w4a4_gemm_packed_workspace_bytes.argtypes = [i64, i64, dp]
    L.atom_w4a4_gemm_packed.restype = ctypes.c_int
    L.atom_w4a4_gemm_packed.argtypes = [vp, vp, vp, i64, vp, i64, dp, vp, i64, vp, vp, sz, vp]
    L.atom_pack_act.restype = ctypes.c_int
    L.atom_pack_act.argtypes = [vp, vp, vp, i64, dp, vp, sz, vp]
    L.atom_quantize_act_packed.restype = ctypes.c_int
    L.atom_quantize_act_packed.argtypes = [vp, i64, i64, vp, f32, vp, dp, f32, vp, sz, vp]
    L.atom_add_quantize_act_packed.restype = ctypes.c_int
    L.atom_add_quantize_act_packed.argtypes = [vp, vp, i64, i64, i64, vp, i64, vp, f32, vp, dp, f32, vp, sz, vp]
    L.atom_swiglu_quantize_act_packed.restype = ctypes.c_int
    L.atom_swiglu_quantize_act_packed.argtypes = [vp, vp, i64, i64, i64, vp, dp, f32, vp, sz, vp]
    L.atom_w4a4_gemm_prepacked.restype = ctypes.c_int
    L.atom_w4a4_gemm_prepacked.argtypes = [vp, i64, vp, i64, dp, vp, i64, vp, vp]
    i32 = ctypes.c_int32
    L.atom_mx_quantize_act.restype = ctypes.c_int
    L.atom_mx_quantize_act.argtypes = [vp, i64, i64, vp, f32, vp, dp, f32, vp, vp, vp, vp]
    L.atom_mx_quantize_weight.restype = ctypes.c_int
    L.atom_mx_quantize_weight.argtypes = [vp, i64, i64, vp, dp, f32, vp, vp, vp, vp]
    L.atom_mx_gemm.restype = ctypes.c_int
    L.atom_mx_gemm.argtypes = [vp, vp, vp, i64, vp, vp, vp, i64, dp, vp, i64, vp]
    L.atom_calibrate_reorder.restype = ctypes.c_int
    L.atom_calibrate_reorder.argtypes = [vp, i64, i64, i32, vp, sz, vp, vp]
    L.atom_calibrate_reorder_workspace_bytes.restype = sz
    L.atom_calibrate_reorder_workspace_bytes.argtypes = [i64, i32]
    L.atom_kv_quantize.restype = ctypes.c_int
    L.atom_kv_quantize.argtypes = [vp, i64, i64, i32, f32, vp, i32, i64, vp, vp, vp, vp]
    L.atom_kv_quantize_pair.restype = ctypes.c_int
    L.atom_kv_quantize_pair.argtypes = [vp, vp, i64, i64, i32, f32, vp, i32, i64, vp, vp, vp, vp, vp, vp, vp]
    L.atom_decode_attention_kv4.restype = ctypes.c_int
    L.atom_decode_attention_kv4.argtypes = [vp, i32, i32, i32, i32, i64, vp, vp, vp, vp, vp, vp, vp,
                                            f32, vp, vp, sz, vp]
    L.atom_decode_attention_kv4_workspace_bytes.restype = sz
    L.atom_decode_attention_kv4_workspace_bytes.argtypes = [i32, i32, i32, i32, i64]
    L.atom_decode_attention_kv4_static.restype = ctypes.c_int
    L.atom_decode_attention_kv4_static.argtypes = [vp, i32, i32, i32, i32, i64, vp, vp, vp, vp, vp, vp, vp,
                                                   f32, vp, vp]
    L.atom_static_scratch_bytes.restype = sz
    L.atom_static_scratch_bytes.argtypes = []
    L.atom_mfma_rate_probe.restype = ctypes.c_double
    L.atom_mfma_rate_probe.argtypes = [i32, i32, vp, vp, ctypes.POINTER(ctypes.c_int)]
    L.atom_check_reorder_idx.restype = ctypes.c_int
    L.atom_check_reorder_idx.argtypes = [vp, ctypes.c_int32]
    L.atom_status_string.restype = ctypes.c_char_p
    L.atom_status_string.argtypes = [ctypes.c_int]
    _lib = L
    return L


def _desc(K: int, group_size: int, n_outlier: int, bits: int = 4) -> _Desc:
    return _Desc(K, group_size, n_outlier, bits, 8)


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dev(t: torch.Tensor, dtype, name: str):
    if not t.is_cuda:
        raise ValueError(f"{name} must be a device tensor")
    if t.dtype != dtype:
        raise TypeError(f"{name}: expected {dtype}, got {t.dtype}")
    return t


def atom_mfma_rate_probe(kind: int, iters: int, scratch: torch.Tensor) -> float:
    """Launch the MFMA-only loop (0: INT8 32x32x32, 1: FP6 32x32x64) on the current stream; returns
    the operations of the launch."""
    st = ctypes.c_int(0)
    ops = load_library().atom_mfma_rate_probe(kind, iters, _ptr(scratch), _stream(), ctypes.byref(st))
    if st.value != 0:
        raise AtomError(st.value, "atom_mfma_rate_probe")
    return float(ops)


def atom_status_string(status: int) -> str:
    return load_library().atom_status_string(int(status)).decode()


def atom_check_reorder_idx(idx: torch.Tensor) -> int:
    """Host check that ``idx`` (CPU int32 tensor) is a permutation. Returns the status."""
    idx = idx.detach().cpu().contiguous()
    if idx.dtype != torch.int32:
        raise TypeError("idx must be int32")
    return int(load_library().atom_check_reorder_idx(ctypes.c_void_p(idx.data_ptr()), idx.numel()))


def _quant_outputs(rows: int, K: int, group_size: int, n_outlier: int, device):
    q4 = torch.empty((rows, (K - n_outlier) // 2), dtype=torch.uint8, device=device)
    q8 = torch.empty((rows, n_outlier), dtype=torch.int8, device=device)
    sc = torch.empty((rows, K // group_size), dtype=torch.float16, device=device)
    return q4, q8, sc


def atom_quantize_act(x: torch.Tensor, gamma: Optional[torch.Tensor], eps: float,
                      reorder_idx: Optional[torch.Tensor], group_size: int = 128, n_outlier: int = 128,
                      clip: float = 0.9, out: Optional[Tuple[torch.Tensor, ...]] = None, bits: int = 4):
    """Fused RMSNorm -> reorder -> dynamic group quantisation of ``x`` [M, K]
    (fp16, last dim contiguous).  Returns ``(q4, q8, scale)`` device tensors.  ``bits``: width
    of the normal channels, 4 or 3 (same layouts: one code per nibble)."""
    L = load_library()
    _dev(x, torch.float16, "x")
    if reorder_idx is not None:        # None: x already is in reordered order
        _dev(reorder_idx, torch.int32, "reorder_idx")
    if gamma is not None:
        _dev(gamma, torch.float16, "gamma")
    if x.dim() != 2 or x.stride(1) != 1:
        raise ValueError("x must be [M, K] with a contiguous last dimension")
    M, K = x.shape
    q4, q8, sc = out if out is not None else _quant_outputs(M, K, group_size, n_outlier, x.device)
    d = _desc(K, group_size, n_outlier, bits)
    st = L.atom_quantize_act(_ptr(x), M, x.stride(0) if M > 1 else max(K, x.stride(0)), _ptr(gamma),
                             eps, _ptr(reorder_idx), ctypes.byref(d), clip, _ptr(q4), _ptr(q8),
                             _ptr(sc), _stream())
    if st != 0:
        raise AtomError(st, "atom_quantize_act")
    return q4, q8, sc


def atom_tile_weight_decode(w_q4: torch.Tensor, w_q8: torch.Tensor, group_size: int = 128):
    """Re-tile canonical weight codes for ``atom_w4a4_gemm_decode_tiled`` (once, offline).  Returns
    ``(w_q4_tiled, w_q8_tiled)`` as flat uint8 / int8 device tensors."""
    L = load_library()
    _dev(w_q4, torch.uint8, "w_q4")
    _dev(w_q8, torch.int8, "w_q8")
    N, O = w_q8.shape
    K = 2 * w_q4.shape[1] + O
    d = _desc(K, group_size, O, 4)
    b4 = int(L.atom_tile_weight_decode_bytes(N, ctypes.byref(d), 0))
    b8 = int(L.atom_tile_weight_decode_bytes(N, ctypes.byref(d), 1))
    t4 = torch.empty(b4, dtype=torch.uint8, device=w_q4.device)
    t8 = torch.empty(b8, dtype=torch.int8, device=w_q4.device)
    st = L.atom_tile_weight_decode(_ptr(w_q4), _ptr(w_q8), N, ctypes.byref(d), _ptr(t4), b4, _ptr(t8), b8, _stream())
    if st != 0:
        raise AtomError(st, "atom_tile_weight_decode")
    return t4, t8


def atom_w4a4_gemm_decode_tiled(a_q4, a_q8, a_scale, w_q4_tiled, w_q8_tiled, w_scale, group_size: int = 128,
                                out: Optional[torch.Tensor] = None):
    """Decode-sized group GEMM (M <= 256) on re-tiled weight codes; ``w_scale`` [N, G] canonical."""
    L = load_library()
    M, O = a_q8.shape
    N, G = w_scale.shape
    K = G * group_size
    y = out if out is not None else torch.empty((M, N), dtype=torch.float16, device=a_q4.device)
    d = _desc(K, group_size, O, 4)
    st = L.atom_w4a4_gemm_decode_tiled(_ptr(a_q4), _ptr(a_q8), _ptr(a_scale), M, _ptr(w_q4_tiled), _ptr(w_q8_tiled),
                                       _ptr(w_scale), N, ctypes.byref(d), _ptr(y),
                                       y.stride(0) if M > 1 else max(N, y.stride(0)), _stream())
    if st != 0:
        raise AtomError(st, "atom_w4a4_gemm_decode_tiled")
    return y


def atom_permute_rows(mat: torch.Tensor, row_idx: torch.Tensor, out: Optional[torch.Tensor] = None):
    """``out[r, :] = mat[row_idx[r], :]`` for an fp16 matrix (or a vector, taken as one column): the
    offline step that lets the operator producing an activation emit it in reordered order."""
    L = load_library()
    _dev(mat, torch.float16, "mat")
    _dev(row_idx, torch.int32, "row_idx")
    m2 = mat if mat.dim() == 2 else mat.reshape(-1, 1)
    if m2.stride(1) != 1 and m2.shape[1] != 1:
        raise ValueError("mat must have a contiguous last dimension")
    R, C = row_idx.numel(), m2.shape[1]
    o = out if out is not None else torch.empty((R, C), dtype=torch.float16, device=mat.device)
    o2 = o if o.dim() == 2 else o.reshape(-1, 1)
    st = L.atom_permute_rows(_ptr(m2), m2.shape[0], C, max(C, m2.stride(0)), _ptr(row_idx), R, _ptr(o2),
                             max(C, o2.stride(0)), _stream())
    if st != 0:
        raise AtomError(st, "atom_permute_rows")
    return o if mat.dim() == 2 else o.reshape(-1)


def atom_decode_linear(x: torch.Tensor, gamma: Optional[torch.Tensor], eps: float,
                       reorder_idx: Optional[torch.Tensor], w_q4: torch.Tensor, w_q8: torch.Tensor,
                       w_scale: torch.Tensor, group_size: int = 128, clip: float = 0.9,
                       out: Optional[torch.Tensor] = None, debug: bool = False, bits: int = 4):
    """One launch for ``Y = linear(x)`` at M <= 16 rows: front end (RMSNorm when ``gamma`` is given,
    reorder, group quantisation) and weight-streaming group GEMM.  Returns ``Y`` [M, N] fp16, or
    ``(Y, (q4, q8, scale))`` with ``debug`` (the activation codes the kernel computed)."""
    L = load_library()
    _dev(x, torch.float16, "x")
    if reorder_idx is not None:        # None: x already is in reordered order
        _dev(reorder_idx, torch.int32, "reorder_idx")
    if gamma is not None:
        _dev(gamma, torch.float16, "gamma")
    _dev(w_q4, torch.uint8, "w_q4")
    _dev(w_q8, torch.int8, "w_q8")
    _dev(w_scale, torch.float16, "w_scale")
    if x.dim() != 2 or x.stride(1) != 1:
        raise ValueError("x must be [M, K] with a contiguous last dimension")
    M, K = x.shape
    N, O = w_q8.shape
    y = out if out is not None else torch.empty((M, N), dtype=torch.float16, device=x.device)
    dbg = _quant_outputs(M, K, group_size, O, x.device) if debug else (None, None, None)
    d = _desc(K, group_size, O, bits)
    st = L.atom_decode_linear(_ptr(x), M, x.stride(0) if M > 1 else max(K, x.stride(0)), _ptr(gamma), eps,
                              _ptr(reorder_idx), ctypes.byref(d), clip, _ptr(w_q4), _ptr(w_q8), _ptr(w_scale), N,
                              _ptr(y), y.stride(0) if M > 1 else max(N, y.stride(0)), _ptr(dbg[0]), _ptr(dbg[1]),
                              _ptr(dbg[2]), _stream())
    if st != 0:
        raise AtomError(st, "atom_decode_linear")
    return (y, dbg) if debug else y


def atom_decode_linear_coop_sync(device="cuda") -> torch.Tensor:
    """The zeroed counters atom_decode_linear_coop works with (one per stream of calls)."""
    n = int(load_library().atom_decode_linear_coop_sync_bytes())
    return torch.zeros(n // 4, dtype=torch.int32, device=device)


def atom_decode_linear_coop(x: torch.Tensor, gamma: Optional[torch.Tensor], eps: float,
                            reorder_idx: Optional[torch.Tensor], w_q4: torch.Tensor, w_q8: torch.Tensor,
                            w_scale: torch.Tensor, sync_words: torch.Tensor, group_size: int = 128,
                            clip: float = 0.9, out: Optional[torch.Tensor] = None,
                            codes: Optional[Tuple[torch.Tensor, ...]] = None, bits: int = 4):
    """One launch for ``Y = linear(x)`` at M <= 16 rows with the front end done once: the first M
    workgroups quantise the rows, the others stream the weights meanwhile.  ``sync_words``:
    ``atom_decode_linear_coop_sync()`` (int32 zeros on the device), zero before the first call, left
    zero by every call (word 1 set = a wait ran out).  Returns ``(Y, (q4, q8, scale))``: the codes are outputs as in atom_quantize_act."""
    L = load_library()
    _dev(x, torch.float16, "x")
    if reorder_idx is not None:        # None: x already is in reordered order
        _dev(reorder_idx, torch.int32, "reorder_idx")
    if gamma is not None:
        _dev(gamma, torch.float16, "gamma")
    _dev(w_q4, torch.uint8, "w_q4")
    _dev(w_q8, torch.int8, "w_q8")
    _dev(w_scale, torch.float16, "w_scale")
    _dev(sync_words, torch.int32, "sync_words")
    if 4 * sync_words.numel() < int(L.atom_decode_linear_coop_sync_bytes()) or not sync_words.is_contiguous():
        raise ValueError("sync_words is too small: take atom_decode_linear_coop_sync()")
    if x.dim() != 2 or x.stride(1) != 1:
        raise ValueError("x must be [M, K] with a contiguous last dimension")
    M, K = x.shape
    N, O = w_q8.shape
    y = out if out is not None else torch.empty((M, N), dtype=torch.float16, device=x.device)
    q = codes if codes is not None else _quant_outputs(M, K, group_size, O, x.device)
    d = _desc(K, group_size, O, bits)
    st = L.atom_decode_linear_coop(_ptr(x), M, x.stride(0) if M > 1 else max(K, x.stride(0)), _ptr(gamma), eps,
                                   _ptr(reorder_idx), ctypes.byref(d), clip, _ptr(w_q4), _ptr(w_q8), _ptr(w_scale),
                                   N, _ptr(y), y.stride(0) if M > 1 else max(N, y.stride(0)), _ptr(q[0]), _ptr(q[1]),
                                   _ptr(q[2]), _ptr(sync_words), _stream())
    if st != 0:
        raise AtomError(st, "atom_decode_linear_coop")
    return y, q


def atom_decode_linear_lds_bytes(M: int, K: int, n_outlier: int = 128, norm: bool = True, group_size: int = 128,
                                 index: bool = True) -> int:
    d = _desc(K, group_size, n_outlier, 4)
    return int(load_library().atom_decode_linear_lds_bytes(M, ctypes.byref(d), 1 if norm else 0, 1 if index else 0))


def atom_add_quantize_act(x: torch.Tensor, residual: torch.Tensor, gamma: Optional[torch.Tensor],
                          eps: float, reorder_idx: Optional[torch.Tensor], group_size: int = 128,
                          n_outlier: int = 128, clip: float = 0.9,
                          sum_out: Optional[torch.Tensor] = None,
                          out: Optional[Tuple[torch.Tensor, ...]] = None, bits: int = 4):
    """``h = fp16(x + residual)`` followed by the front end on ``h``.  ``sum_out`` may be
    ``x`` or ``residual`` (in place) or a separate [M, K] tensor; a new one by default.
    Returns ``(h, q4, q8, scale)``."""
    L = load_library()
    _dev(x, torch.float16, "x")
    _dev(residual, torch.float16, "residual")
    if reorder_idx is not None:        # None: x already is in reordered order
        _dev(reorder_idx, torch.int32, "reorder_idx")
    if gamma is not None:
        _dev(gamma, torch.float16, "gamma")
    if x.dim() != 2 or x.stride(1) != 1 or residual.shape != x.shape or residual.stride(1) != 1:
        raise ValueError("x and residual must be [M, K] with a contiguous last dimension")
    M, K = x.shape
    if sum_out is None:
        sum_out = torch.empty((M, K), dtype=torch.float16, device=x.device)
    _dev(sum_out, torch.float16, "sum_out")
    if sum_out.shape != x.shape or sum_out.stride(1) != 1:
        raise ValueError("sum_out must be [M, K] with a contiguous last dimension")
    d = _desc(K, group_size, n_outlier, bits)
    q4, q8, sc = out if out is not None else _quant_outputs(M, K, group_size, n_outlier, x.device)
    ld = lambda t: t.stride(0) if M > 1 else max(K, t.stride(0))
    st = L.atom_add_quantize_act(_ptr(x), _ptr(residual), M, ld(x), ld(residual), _ptr(sum_out),
                                 ld(sum_out), _ptr(gamma), eps, _ptr(reorder_idx), ctypes.byref(d),
                                 clip, _ptr(q4), _ptr(q8), _ptr(sc), _stream())
    if st != 0:
        raise AtomError(st, "atom_add_quantize_act")
    return sum_out, q4, q8, sc


def atom_swiglu_quantize_act(gate: torch.Tensor, up: torch.Tensor, reorder_idx: Optional[torch.Tensor],
                             group_size: int = 128, n_outlier: int = 128, clip: float = 0.9,
                             out: Optional[Tuple[torch.Tensor, ...]] = None, bits: int = 4):
    """``silu(gate) * up`` (fp32, never stored) followed by reorder and group quantisation.
    ``gate`` and ``up`` are [M, K] fp16 with a contiguous last dimension, e.g. the two halves
    of the fused gate/up projection's output.  Returns ``(q4, q8, scale)``."""
    L = load_library()
    _dev(gate, torch.float16, "gate")
    _dev(up, torch.float16, "up")
    if reorder_idx is not None:        # None: x already is in reordered order
        _dev(reorder_idx, torch.int32, "reorder_idx")
    if gate.dim() != 2 or gate.stride(1) != 1 or up.shape != gate.shape or up.stride(1) != 1:
        raise ValueError("gate and up must be [M, K] with a contiguous last dimension")
    M, K = gate.shape
    q4, q8, sc = out if out is not None else _quant_outputs(M, K, group_size, n_outlier, gate.device)
    d = _desc(K, group_size, n_outlier, bits)
    ld = lambda t: t.stride(0) if M > 1 else max(K, t.stride(0))
    st = L.atom_swiglu_quantize_act(_ptr(gate), _ptr(up), M, ld(gate), ld(up), _ptr(reorder_idx),
                                    ctypes.byref(d), clip, _ptr(q4), _ptr(q8), _ptr(sc), _stream())
    if st != 0:
        raise AtomError(st, "atom_swiglu_quantize_act")
    return q4, q8, sc


def atom_quantize_weight(w: torch.Tensor, reorder_idx: Optional[torch.Tensor], group_size: int = 128,
                         n_outlier: int = 128, clip: float = 0.85,
                         out: Optional[Tuple[torch.Tensor, ...]] = None, bits: int = 4):
    """One-time reorder + group quantisation of ``w`` [N, K] fp16."""
    L = load_library()
    _dev(w, torch.float16, "w")
    if reorder_idx is not None:        # None: x already is in reordered order
        _dev(reorder_idx, torch.int32, "reorder_idx")
    if w.dim() != 2 or w.stride(1) != 1:
        raise ValueError("w must be [N, K] with a contiguous last dimension")
    N, K = w.shape
    q4, q8, sc = out if out is not None else _quant_outputs(N, K, group_size, n_outlier, w.device)
    d = _desc(K, group_size, n_outlier, bits)
    st = L.atom_quantize_weight(_ptr(w), N, w.stride(0) if N > 1 else max(K, w.stride(0)),
                                _ptr(reorder_idx), ctypes.byref(d), clip, _ptr(q4), _ptr(q8),
                                _ptr(sc), _stream())
    if st != 0:
        raise AtomError(st, "atom_quantize_weight")
    return q4, q8, sc


def atom_w4a4_gemm_workspace_bytes(M: int, N: int, K: int, group_size: int = 128,
                                   n_outlier: int = 128) -> int:
    d = _desc(K, group_size, n_outlier)
    return int(load_library().atom_w4a4_gemm_workspace_bytes(M, N, ctypes.byref(d)))


def atom_w4a4_gemm(a_q4, a_q8, a_scale, w_q4, w_q8, w_scale, group_size: int = 128,
                   out: Optional[torch.Tensor] = None, partials: Optional[torch.Tensor] = None,
                   workspace: Optional[torch.Tensor] = None):
    """Y[M, N] fp16 = group-dequantised product of quantised activations and
    weights.  ``partials`` (int32 [M, N, G]) also receives every per-group
    integer sum."""
    L = load_library()
    for t, dt, nm in ((a_q4, torch.uint8, "a_q4"), (a_q8, torch.int8, "a_q8"),
                      (a_scale, torch.float16, "a_scale"), (w_q4, torch.uint8, "w_q4"),
                      (w_q8, torch.int8, "w_q8"), (w_scale, torch.float16, "w_scale")):
        _dev(t, dt, nm)
        if not t.is_contiguous():
            raise ValueError(f"{nm} must be contiguous")
    M, O = a_q8.shape
    N = w_q8.shape[0]
    K = a_q4.shape[1] * 2 + O
    if w_q4.shape[1] != a_q4.shape[1] or w_q8.shape[1] != O:
        raise ValueError("activation and weight code shapes disagree")
    if out is None:
        out = torch.empty((M, N), dtype=torch.float16, device=a_q4.device)
    _dev(out, torch.float16, "out")
    if partials is not None:
        _dev(partials, torch.int32, "partials")
        if tuple(partials.shape) != (M, N, K // group_size) or not partials.is_contiguous():
            raise ValueError("partials must be contiguous int32 [M, N, G]")
    d = _desc(K, group_size, n_outlier=O)
    need = int(L.atom_w4a4_gemm_workspace_bytes(M, N, ctypes.byref(d)))
    if need and (workspace is None or workspace.numel() * workspace.element_size() < need):
        workspace = torch.empty(need, dtype=torch.uint8, device=a_q4.device)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    st = L.atom_w4a4_gemm(_ptr(a_q4), _ptr(a_q8), _ptr(a_scale), M, _ptr(w_q4), _ptr(w_q8),
                          _ptr(w_scale), N, ctypes.byref(d), _ptr(out),
                          out.stride(0) if M > 1 else max(N, out.stride(0)),
                          _ptr(partials), _ptr(workspace), ws_bytes, _stream())
    if st != 0:
        raise AtomError(st, "atom_w4a4_gemm")
    return out


def atom_pack_weight(w_q4, w_q8, w_scale, group_size: int = 128, out: Optional[torch.Tensor] = None):
    """Canonical weight codes and scales -> the opaque tiled layout of ``atom_w4a4_gemm_packed``
    (a uint8 device tensor)."""
    L = load_library()
    for t, dt, nm in ((w_q4, torch.uint8, "w_q4"), (w_q8, torch.int8, "w_q8"), (w_scale, torch.float16, "w_scale")):
        _dev(t, dt, nm)
        if not t.is_contiguous():
            raise ValueError(f"{nm} must be contiguous")
    N, O = w_q8.shape
    K = w_q4.shape[1] * 2 + O
    d = _desc(K, group_size, n_outlier=O)
    need = int(L.atom_pack_weight_bytes(N, ctypes.byref(d)))
    if out is None:
        out = torch.empty(max(need, 1), dtype=torch.uint8, device=w_q4.device)
    _dev(out, torch.uint8, "out")
    st = L.atom_pack_weight(_ptr(w_q4), _ptr(w_q8), _ptr(w_scale), N, ctypes.byref(d), _ptr(out),
                            out.numel(), _stream())
    if st != 0:
        raise AtomError(st, "atom_pack_weight")
    return out


def atom_pack_act(a_q4, a_q8, a_scale, group_size: int = 128, out: Optional[torch.Tensor] = None):
    """Canonical activation codes and scales -> the tiled layout (``atom_w4a4_gemm_prepacked``)."""
    L = load_library()
    for t, dt, nm in ((a_q4, torch.uint8, "a_q4"), (a_q8, torch.int8, "a_q8"), (a_scale, torch.float16, "a_scale")):
        _dev(t, dt, nm)
        if not t.is_contiguous():
            raise ValueError(f"{nm} must be contiguous")
    M, O = a_q8.shape
    K = a_q4.shape[1] * 2 + O
    d = _desc(K, group_size, n_outlier=O)
    need = int(L.atom_pack_weight_bytes(M, ctypes.byref(d)))
    if out is None:
        out = torch.empty(max(need, 1), dtype=torch.uint8, device=a_q4.device)
    _dev(out, torch.uint8, "out")
    st = L.atom_pack_act(_ptr(a_q4), _ptr(a_q8), _ptr(a_scale), M, ctypes.byref(d), _ptr(out), out.numel(), _stream())
    if st != 0:
        raise AtomError(st, "atom_pack_act")
    return out


def _packed_out(L, M, d, out, device):
    need = int(L.atom_pack_weight_bytes(M, ctypes.byref(d)))
    if out is None:
        out = torch.empty(max(need, 1), dtype=torch.uint8, device=device)
    _dev(out, torch.uint8, "out")
    return out


def atom_quantize_act_packed(x: torch.Tensor, gamma: Optional[torch.Tensor], eps: float,
                             reorder_idx: Optional[torch.Tensor], group_size: int = 128, n_outlier: int = 128,
                             clip: float = 0.9, out: Optional[torch.Tensor] = None, bits: int = 4):
    """``atom_quantize_act`` writing the tiled activations of ``atom_w4a4_gemm_prepacked`` directly
    (the bytes ``atom_pack_act`` would make of its result)."""
    L = load_library()
    _dev(x, torch.float16, "x")
    if x.dim() != 2 or x.stride(1) != 1:
        raise ValueError("x must be [M, K] with a contiguous last dimension")
    M, K = x.shape
    d = _desc(K, group_size, n_outlier, bits)
    out = _packed_out(L, M, d, out, x.device)
    st = L.atom_quantize_act_packed(_ptr(x), M, x.stride(0) if M > 1 else max(K, x.stride(0)), _ptr(gamma), eps,
                                    _ptr(reorder_idx), ctypes.byref(d), clip, _ptr(out), out.numel(), _stream())
    if st != 0:
        raise AtomError(st, "atom_quantize_act_packed")
    return out


def atom_add_quantize_act_packed(x: torch.Tensor, residual: torch.Tensor, gamma: Optional[torch.Tensor], eps: float,
                                 reorder_idx: Optional[torch.Tensor], group_size: int = 128, n_outlier: int = 128,
                                 clip: float = 0.9, sum_out: Optional[torch.Tensor] = None,
                                 out: Optional[torch.Tensor] = None, bits: int = 4):
    """``atom_add_quantize_act`` writing the tiled activations directly.  Returns ``(h, a_packed)``."""
    L = load_library()
    _dev(x, torch.float16, "x")
    _dev(residual, torch.float16, "residual")
    M, K = x.shape
    h = sum_out if sum_out is not None else torch.empty((M, K), dtype=torch.float16, device=x.device)
    d = _desc(K, group_size, n_outlier, bits)
    out = _packed_out(L, M, d, out, x.device)
    ld = lambda t: t.stride(0) if M > 1 else max(K, t.stride(0))
    st = L.atom_add_quantize_act_packed(_ptr(x), _ptr(residual), M, ld(x), ld(residual), _ptr(h), ld(h), _ptr(gamma),
                                        eps, _ptr(reorder_idx), ctypes.byref(d), clip, _ptr(out), out.numel(), _stream())
    if st != 0:
        raise AtomError(st, "atom_add_quantize_act_packed")
    return h, out


def atom_swiglu_quantize_act_packed(gate: torch.Tensor, up: torch.Tensor, reorder_idx: Optional[torch.Tensor],
                                    group_size: int = 128, n_outlier: int = 128, clip: float = 0.9,
                                    out: Optional[torch.Tensor] = None, bits: int = 4):
    """``atom_swiglu_quantize_act`` writing the tiled activations directly."""
    L = load_library()
    _dev(gate, torch.float16, "gate")
    _dev(up, torch.float16, "up")
    M, K = gate.shape
    d = _desc(K, group_size, n_outlier, bits)
    out = _packed_out(L, M, d, out, gate.device)
    ld = lambda t: t.stride(0) if M > 1 else max(K, t.stride(0))
    st = L.atom_swiglu_quantize_act_packed(_ptr(gate), _ptr(up), M, ld(gate), ld(up), _ptr(reorder_idx),
                                           ctypes.byref(d), clip, _ptr(out), out.numel(), _stream())
    if st != 0:
        raise AtomError(st, "atom_swiglu_quantize_act_packed")
    return out


def atom_w4a4_gemm_prepacked(a_packed, M: int, w_packed, N: int, K: int, group_size: int = 128,
                             n_outlier: int = 128, out: Optional[torch.Tensor] = None,
                             partials: Optional[torch.Tensor] = None):
    """The GEMM on two tiled operands (``atom_pack_act`` / ``atom_pack_weight``)."""
    L = load_library()
    _dev(a_packed, torch.uint8, "a_packed")
    _dev(w_packed, torch.uint8, "w_packed")
    d = _desc(K, group_size, n_outlier)
    if (a_packed.numel() < int(L.atom_pack_weight_bytes(M, ctypes.byref(d))) or
            w_packed.numel() < int(L.atom_pack_weight_bytes(N, ctypes.byref(d)))):
        raise ValueError("a packed operand is smaller than atom_pack_weight_bytes of its rows")
    if out is None:
        out = torch.empty((M, N), dtype=torch.float16, device=a_packed.device)
    _dev(out, torch.float16, "out")
    if partials is not None:
        _dev(partials, torch.int32, "partials")
        if tuple(partials.shape) != (M, N, K // group_size) or not partials.is_contiguous():
            raise ValueError("partials must be contiguous int32 [M, N, G]")
    st = L.atom_w4a4_gemm_prepacked(_ptr(a_packed), M, _ptr(w_packed), N, ctypes.byref(d), _ptr(out),
                                    out.stride(0) if M > 1 else max(N, out.stride(0)), _ptr(partials), _stream())
    if st != 0:
        raise AtomError(st, "atom_w4a4_gemm_prepacked")
    return out


def atom_w4a4_gemm_packed_workspace_bytes(M: int, N: int, K: int, group_size: int = 128,
                                          n_outlier: int = 128) -> int:
    d = _desc(K, group_size, n_outlier)
    return int(load_library().atom_w4a4_gemm_packed_workspace_bytes(M, N, ctypes.byref(d)))


def atom_w4a4_gemm_packed(a_q4, a_q8, a_scale, w_packed, N: int, group_size: int = 128,
                          out: Optional[torch.Tensor] = None, partials: Optional[torch.Tensor] = None,
                          workspace: Optional[torch.Tensor] = None):
    """``atom_w4a4_gemm`` against weights packed by ``atom_pack_weight``."""
    L = load_library()
    for t, dt, nm in ((a_q4, torch.uint8, "a_q4"), (a_q8, torch.int8, "a_q8"),
                      (a_scale, torch.float16, "a_scale"), (w_packed, torch.uint8, "w_packed")):
        _dev(t, dt, nm)
        if not t.is_contiguous():
            raise ValueError(f"{nm} must be contiguous")
    M, O = a_q8.shape
    K = a_q4.shape[1] * 2 + O
    d = _desc(K, group_size, n_outlier=O)
    if w_packed.numel() < int(L.atom_pack_weight_bytes(N, ctypes.byref(d))):
        raise ValueError("w_packed is smaller than atom_pack_weight_bytes(N)")
    if out is None:
        out = torch.empty((M, N), dtype=torch.float16, device=a_q4.device)
    _dev(out, torch.float16, "out")
    if partials is not None:
        _dev(partials, torch.int32, "partials")
        if tuple(partials.shape) != (M, N, K // group_size) or not partials.is_contiguous():
            raise ValueError("partials must be contiguous int32 [M, N, G]")
    need = int(L.atom_w4a4_gemm_packed_workspace_bytes(M, N, ctypes.byref(d)))
    if workspace is None or workspace.numel() * workspace.element_size() < need:
        workspace = torch.empty(max(need, 1), dtype=torch.uint8, device=a_q4.device)
    st = L.atom_w4a4_gemm_packed(_ptr(a_q4), _ptr(a_q8), _ptr(a_scale), M, _ptr(w_packed), N,
                                 ctypes.byref(d), _ptr(out), out.stride(0) if M > 1 else max(N, out.stride(0)),
                                 _ptr(partials), _ptr(workspace), workspace.numel() * workspace.element_size(),
                                 _stream())
    if st != 0:
        raise AtomError(st, "atom_w4a4_gemm_packed")
    return out


def atom_decode_attention_kv4_workspace_bytes(B: int, H: int, Hkv: int, D: int, Tmax: int) -> int:
    return int(load_library().atom_decode_attention_kv4_workspace_bytes(B, H, Hkv, D, Tmax))


def atom_kv_quantize(x: torch.Tensor, clip: float = 1.0,
                     cache: Optional[Tuple[torch.Tensor, ...]] = None,
                     pos: Optional[torch.Tensor] = None):
    """Asymmetric INT4 quantisation of K or V rows, one scale and zero point per head.

    Without ``cache``: ``x`` is [..., D] fp16 (any leading shape, contiguous); returns
    new ``(codes [..., D/2] uint8, scale [...] fp16, zero [...] int16)``.
    With ``cache = (codes [B, Hkv, Tmax, D/2], scale [B, Hkv, Tmax], zero [B, Hkv, Tmax])``
    and ``pos`` (device int32 [B]): ``x`` is [B, Hkv, D], the new token of every sequence,
    written in place at position ``pos[b]``; returns ``cache``."""
    L = load_library()
    _dev(x, torch.float16, "x")
    if x.dim() < 1 or not x.is_contiguous():
        raise ValueError("x must be contiguous [..., D]")
    D = x.shape[-1]
    R = x.numel() // D if D else 0
    if cache is None:
        if pos is not None:
            raise ValueError("pos needs a cache to append to")
        lead = tuple(x.shape[:-1])
        codes = torch.empty(lead + (D // 2,), dtype=torch.uint8, device=x.device)
        scale = torch.empty(lead, dtype=torch.float16, device=x.device)
        zero = torch.empty(lead, dtype=torch.int16, device=x.device)
        st = L.atom_kv_quantize(_ptr(x), R, D, D, clip, None, 0, 0, _ptr(codes), _ptr(scale),
                                _ptr(zero), _stream())
    else:
        codes, scale, zero = cache
        _dev(codes, torch.uint8, "cache codes")
        _dev(scale, torch.float16, "cache scale")
        _dev(zero, torch.int16, "cache zero")
        if pos is None:
            raise ValueError("appending to a cache needs pos")
        _dev(pos, torch.int32, "pos")
        if x.dim() != 3 or codes.dim() != 4 or not (codes.is_contiguous() and scale.is_contiguous()
                                                    and zero.is_contiguous()):
            raise ValueError("x must be [B, Hkv, D] and the cache contiguous [B, Hkv, Tmax, ...]")
        B, Hkv, Tmax = codes.shape[:3]
        if (tuple(x.shape) != (B, Hkv, D) or codes.shape[3] * 2 != D or tuple(scale.shape) != (B, Hkv, Tmax)
                or tuple(zero.shape) != (B, Hkv, Tmax) or tuple(pos.shape) != (B,)
                or not pos.is_contiguous()):
            raise ValueError("cache, x and pos shapes disagree")
        st = L.atom_kv_quantize(_ptr(x), R, D, D, clip, _ptr(pos), Hkv, Tmax, _ptr(codes),
                                _ptr(scale), _ptr(zero), _stream())
    if st != 0:
        raise AtomError(st, "atom_kv_quantize")
    return codes, scale, zero


def atom_kv_quantize_pair(k: torch.Tensor, v: torch.Tensor, k_cache: Tuple[torch.Tensor, ...],
                          v_cache: Tuple[torch.Tensor, ...], pos: torch.Tensor, clip: float = 1.0):
    """The new K and V rows of every sequence ([B, Hkv, D] fp16 each) appended in place to
    their caches at position ``pos[b]`` in one launch; the same results as two
    ``atom_kv_quantize`` calls.  Returns ``(k_cache, v_cache)``."""
    L = load_library()
    _dev(pos, torch.int32, "pos")
    for x, cache, nm in ((k, k_cache, "k"), (v, v_cache, "v")):
        _dev(x, torch.float16, nm)
        codes, scale, zero = cache
        _dev(codes, torch.uint8, nm + " cache codes")
        _dev(scale, torch.float16, nm + " cache scale")
        _dev(zero, torch.int16, nm + " cache zero")
        if x.dim() != 3 or codes.dim() != 4 or not (x.is_contiguous() and codes.is_contiguous()
                                                    and scale.is_contiguous() and zero.is_contiguous()):
            raise ValueError(nm + " must be contiguous [B, Hkv, D] and its cache contiguous [B, Hkv, Tmax, ...]")
    B, Hkv, Tmax = k_cache[0].shape[:3]
    D = k.shape[-1]
    for x, (codes, scale, zero) in ((k, k_cache), (v, v_cache)):
        if (tuple(x.shape) != (B, Hkv, D) or tuple(codes.shape) != (B, Hkv, Tmax, D // 2)
                or tuple(scale.shape) != (B, Hkv, Tmax) or tuple(zero.shape) != (B, Hkv, Tmax)):
            raise ValueError("cache and row shapes disagree")
    if tuple(pos.shape) != (B,) or not pos.is_contiguous():
        raise ValueError("pos must be contiguous int32 [B]")
    st = L.atom_kv_quantize_pair(_ptr(k), _ptr(v), B * Hkv, D, D, clip, _ptr(pos), Hkv, Tmax,
                                 _ptr(k_cache[0]), _ptr(k_cache[1]), _ptr(k_cache[2]),
                                 _ptr(v_cache[0]), _ptr(v_cache[1]), _ptr(v_cache[2]), _stream())
    if st != 0:
        raise AtomError(st, "atom_kv_quantize_pair")
    return k_cache, v_cache


def _attention_args(q, k_cache, v_cache, seq_len, out):
    _dev(q, torch.float16, "q")
    _dev(seq_len, torch.int32, "seq_len")
    if q.dim() != 3 or not q.is_contiguous():
        raise ValueError("q must be contiguous [B, H, D]")
    B, H, D = q.shape
    kq, ks, kz = k_cache
    vq, vs, vz = v_cache
    for t, dt, nm in ((kq, torch.uint8, "k codes"), (vq, torch.uint8, "v codes"),
                      (ks, torch.float16, "k scale"), (vs, torch.float16, "v scale"),
                      (kz, torch.int16, "k zero"), (vz, torch.int16, "v zero")):
        _dev(t, dt, nm)
        if not t.is_contiguous():
            raise ValueError(f"{nm} must be contiguous")
    if kq.dim() != 4 or kq.shape[0] != B or kq.shape[3] * 2 != D:
        raise ValueError("k codes must be [B, Hkv, Tmax, D/2]")
    Hkv, Tmax = kq.shape[1], kq.shape[2]
    if (vq.shape != kq.shape or tuple(ks.shape) != (B, Hkv, Tmax) or ks.shape != vs.shape
            or kz.shape != ks.shape or vz.shape != ks.shape or tuple(seq_len.shape) != (B,)
            or not seq_len.is_contiguous()):
        raise ValueError("cache and seq_len shapes disagree")
    if out is None:
        out = torch.empty((B, H, D), dtype=torch.float16, device=q.device)
    _dev(out, torch.float16, "out")
    if tuple(out.shape) != (B, H, D) or not out.is_contiguous():
        raise ValueError("out must be contiguous [B, H, D]")
    return B, H, Hkv, D, Tmax, out


def atom_decode_attention_kv4(q: torch.Tensor, k_cache: Tuple[torch.Tensor, ...],
                              v_cache: Tuple[torch.Tensor, ...], seq_len: torch.Tensor,
                              sm_scale: float, out: Optional[torch.Tensor] = None,
                              workspace: Optional[torch.Tensor] = None):
    """Attention of one query token per sequence over the INT4 cache.  ``q`` [B, H, D] fp16;
    each cache is ``(codes [B, Hkv, Tmax, D/2] uint8, scale [B, Hkv, Tmax] fp16,
    zero [B, Hkv, Tmax] int16)``; ``seq_len`` device int32 [B].  Returns [B, H, D] fp16."""
    L = load_library()
    B, H, Hkv, D, Tmax, out = _attention_args(q, k_cache, v_cache, seq_len, out)
    kq, ks, kz = k_cache
    vq, vs, vz = v_cache
    need = int(L.atom_decode_attention_kv4_workspace_bytes(B, H, Hkv, D, Tmax))
    if need and (workspace is None or workspace.numel() * workspace.element_size() < need):
        workspace = torch.empty(need, dtype=torch.uint8, device=q.device)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    st = L.atom_decode_attention_kv4(_ptr(q), B, H, Hkv, D, Tmax, _ptr(seq_len), _ptr(kq), _ptr(ks),
                                     _ptr(kz), _ptr(vq), _ptr(vs), _ptr(vz), sm_scale, _ptr(out),
                                     _ptr(workspace), ws_bytes, _stream())
    if st != 0:
        raise AtomError(st, "atom_decode_attention_kv4")
    return out


def atom_static_scratch_bytes() -> int:
    return int(load_library().atom_static_scratch_bytes())


def atom_decode_attention_kv4_static(q: torch.Tensor, k_cache: Tuple[torch.Tensor, ...],
                                     v_cache: Tuple[torch.Tensor, ...], seq_len: torch.Tensor,
                                     sm_scale: float, out: torch.Tensor):
    """``atom_decode_attention_kv4`` through the entry point that allocates nothing: ``out`` is the
    caller's, the partials of a split launch live in the library's own per-GPU scratch array."""
    L = load_library()
    if out is None:
        raise ValueError("out must be given: this call allocates nothing")
    B, H, Hkv, D, Tmax, out = _attention_args(q, k_cache, v_cache, seq_len, out)
    kq, ks, kz = k_cache
    vq, vs, vz = v_cache
    st = L.atom_decode_attention_kv4_static(_ptr(q), B, H, Hkv, D, Tmax, _ptr(seq_len), _ptr(kq), _ptr(ks),
                                            _ptr(kz), _ptr(vq), _ptr(vs), _ptr(vz), sm_scale, _ptr(out),
                                            _stream())
    if st != 0:
        raise AtomError(st, "atom_decode_attention_kv4_static")
    return out


def _mx_outputs(rows: int, K: int, n_outlier: int, device):
    # step-major: [K step][row][64 bytes], scales [128-channel slab][row][4 bytes]
    q4 = torch.empty(((K - n_outlier) // 128, rows, 64), dtype=torch.uint8, device=device)
    q8 = torch.empty((n_outlier // 64, rows, 64), dtype=torch.uint8, device=device)
    e8 = torch.empty((K // 128, rows, 4), dtype=torch.uint8, device=device)
    return q4, q8, e8


def atom_mx_quantize_act(x: torch.Tensor, gamma: Optional[torch.Tensor], eps: float,
                         reorder_idx: torch.Tensor, n_outlier: int = 128, clip: float = 1.0,
                         out: Optional[Tuple[torch.Tensor, ...]] = None):
    """MX variant of the front end: RMSNorm -> reorder -> FP4 E2M1 (normal channels) / FP8 E4M3
    (outliers) with one E8M0 scale byte per 32 channels.  Returns ``(q4, q8, e8)``."""
    L = load_library()
    _dev(x, torch.float16, "x")
    _dev(reorder_idx, torch.int32, "reorder_idx")
    if gamma is not None:
        _dev(gamma, torch.float16, "gamma")
    if x.dim() != 2 or x.stride(1) != 1:
        raise ValueError("x must be [M, K] with a contiguous last dimension")
    M, K = x.shape
    q4, q8, e8 = out if out is not None else _mx_outputs(M, K, n_outlier, x.device)
    d = _Desc(K, 32, n_outlier, 4, 8)
    st = L.atom_mx_quantize_act(_ptr(x), M, x.stride(0) if M > 1 else max(K, x.stride(0)), _ptr(gamma),
                                eps, _ptr(reorder_idx), ctypes.byref(d), clip, _ptr(q4), _ptr(q8),
                                _ptr(e8), _stream())
    if st != 0:
        raise AtomError(st, "atom_mx_quantize_act")
    return q4, q8, e8


def atom_mx_quantize_weight(w: torch.Tensor, reorder_idx: torch.Tensor, n_outlier: int = 128,
                            clip: float = 1.0, out: Optional[Tuple[torch.Tensor, ...]] = None):
    """One-time reorder + MX quantisation of ``w`` [N, K] fp16."""
    L = load_library()
    _dev(w, torch.float16, "w")
    _dev(reorder_idx, torch.int32, "reorder_idx")
    if w.dim() != 2 or w.stride(1) != 1:
        raise ValueError("w must be [N, K] with a contiguous last dimension")
    N, K = w.shape
    q4, q8, e8 = out if out is not None else _mx_outputs(N, K, n_outlier, w.device)
    d = _Desc(K, 32, n_outlier, 4, 8)
    st = L.atom_mx_quantize_weight(_ptr(w), N, w.stride(0) if N > 1 else max(K, w.stride(0)),
                                   _ptr(reorder_idx), ctypes.byref(d), clip, _ptr(q4), _ptr(q8),
                                   _ptr(e8), _stream())
    if st != 0:
        raise AtomError(st, "atom_mx_quantize_weight")
    return q4, q8, e8


def atom_mx_gemm(a_q4, a_q8, a_e8, w_q4, w_q8, w_e8, out: Optional[torch.Tensor] = None):
    """Y[M, N] fp16 from the two MX-quantised operands; the block scales are applied by the
    scaled MFMA instruction itself."""
    L = load_library()
    for t, nm in ((a_q4, "a_q4"), (a_q8, "a_q8"), (a_e8, "a_e8"), (w_q4, "w_q4"), (w_q8, "w_q8"),
                  (w_e8, "w_e8")):
        _dev(t, torch.uint8, nm)
        if not t.is_contiguous():
            raise ValueError(f"{nm} must be contiguous")
    if a_q4.dim() != 3 or a_q8.dim() != 3 or w_q4.dim() != 3 or w_q8.dim() != 3:
        raise ValueError("operands must be the step-major arrays atom_mx_quantize_* produce")
    M, N = a_q8.shape[1], w_q8.shape[1]
    O = a_q8.shape[0] * 64
    K = a_q4.shape[0] * 128 + O
    if (w_q4.shape[0] != a_q4.shape[0] or w_q8.shape[0] != a_q8.shape[0] or a_q4.shape[1] != M
            or w_q4.shape[1] != N or tuple(a_e8.shape) != (K // 128, M, 4) or tuple(w_e8.shape) != (K // 128, N, 4)):
        raise ValueError("activation and weight code shapes disagree")
    if out is None:
        out = torch.empty((M, N), dtype=torch.float16, device=a_q4.device)
    _dev(out, torch.float16, "out")
    d = _Desc(K, 32, O, 4, 8)
    st = L.atom_mx_gemm(_ptr(a_q4), _ptr(a_q8), _ptr(a_e8), M, _ptr(w_q4), _ptr(w_q8), _ptr(w_e8), N,
                        ctypes.byref(d), _ptr(out), out.stride(0) if M > 1 else max(N, out.stride(0)),
                        _stream())
    if st != 0:
        raise AtomError(st, "atom_mx_gemm")
    return out


def atom_calibrate_reorder(x: torch.Tensor):
    """Reorder index from calibration activations ``x`` [T, K] fp16: the channels in ascending
    order of their square sums (double), the outliers last.  Returns ``(idx int32 [K],
    stat float64 [K])`` device tensors."""
    L = load_library()
    _dev(x, torch.float16, "x")
    if x.dim() != 2 or x.stride(1) != 1:
        raise ValueError("x must be [T, K] with a contiguous last dimension")
    T, K = x.shape
    need = int(L.atom_calibrate_reorder_workspace_bytes(T, K))
    ws = torch.empty(max(need, 8) // 8, dtype=torch.float64, device=x.device)
    idx = torch.empty(K, dtype=torch.int32, device=x.device)
    st = L.atom_calibrate_reorder(_ptr(x), T, x.stride(0) if T > 1 else max(K, x.stride(0)), K, _ptr(ws),
                                  ws.numel() * 8, _ptr(idx), _stream())
    if st != 0:
        raise AtomError(st, "atom_calibrate_reorder")
    return idx, ws[-K:]
