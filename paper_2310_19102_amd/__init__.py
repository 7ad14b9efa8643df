"""MI355X-native hot path of Atom's W4A4 quantisation (arxiv 2310.19102).

The product is ``libatom.so`` (hand-written HIP kernels for gfx950 behind the C
ABI declared in ``include/atom.h``).  This package is a thin binding with the
same entry-point names: it marshals torch device tensors into plain pointers and
sizes; every step of the path runs in the library's kernels.  There is no CPU
or PyTorch fallback: loading fails loudly when the library has not been built.
"""
from .binding import (  # noqa: F401
    AtomError,
    atom_check_reorder_idx,
    atom_quantize_act,
    atom_add_quantize_act,
    atom_swiglu_quantize_act,
    atom_quantize_weight,
    atom_mx_quantize_act,
    atom_mx_quantize_weight,
    atom_mx_gemm,
    atom_calibrate_reorder,
    atom_kv_quantize,
    atom_kv_quantize_pair,
    atom_decode_attention_kv4,
    atom_decode_attention_kv4_workspace_bytes,
    atom_decode_attention_kv4_static,
    atom_static_scratch_bytes,
    atom_status_string,
    atom_mfma_rate_probe,
    atom_w4a4_gemm,
    atom_w4a4_gemm_workspace_bytes,
    atom_decode_linear,
    atom_decode_linear_coop,
    atom_decode_linear_coop_sync,
    atom_permute_rows,
    atom_tile_weight_decode,
    atom_w4a4_gemm_decode_tiled,
    atom_decode_linear_lds_bytes,
    atom_pack_weight,
    atom_pack_act,
    atom_quantize_act_packed,
    atom_add_quantize_act_packed,
    atom_swiglu_quantize_act_packed,
    atom_w4a4_gemm_prepacked,
    atom_w4a4_gemm_packed,
    atom_w4a4_gemm_packed_workspace_bytes,
    library_path,
    load_library,
)
