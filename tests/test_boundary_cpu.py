"""Host-side checks of the C ABI that need no GPU: the library loads, exports
every symbol the header declares, and its host-only entry points behave."""
import ctypes
import os
import re

import numpy as np
import pytest
import torch

import paper_2310_19102_amd as atom
from paper_2310_19102_amd import binding, synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "atom.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(atom_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = atom.load_library()
    names = _declared_symbols()
    assert set(names) == set(binding.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None


def test_status_strings():
    seen = {atom.atom_status_string(s) for s in range(7)}
    assert len(seen) == 7 and "ok" in seen
    assert atom.atom_status_string(99) == "unknown status"


def test_check_reorder_idx():
    assert atom.atom_check_reorder_idx(torch.arange(512, dtype=torch.int32)) == 0
    bad = torch.arange(512, dtype=torch.int32)
    bad[7] = 8
    assert atom.atom_check_reorder_idx(bad) == 2
    bad[7] = 512
    assert atom.atom_check_reorder_idx(bad) == 2
    bad[7] = -1
    assert atom.atom_check_reorder_idx(bad) == 2


def test_host_side_argument_validation_needs_no_gpu():
    """Failures are decided on the host before any launch, so they can be
    exercised here with fake (never dereferenced) device pointers."""
    lib = atom.load_library()
    D = binding._Desc
    p = ctypes.c_void_p(0x1000)
    ok = D(4096, 128, 128, 4, 8)
    q = lib.atom_quantize_act
    assert q(None, 4, 4096, None, 0.0, p, ctypes.byref(ok), 0.9, p, p, p, None) == 1
    assert q(p, 4, 4000, None, 0.0, p, ctypes.byref(ok), 0.9, p, p, p, None) == 2
    assert q(p, -1, 4096, None, 0.0, p, ctypes.byref(ok), 0.9, p, p, p, None) == 2
    assert q(p, 0, 4096, None, 0.0, p, ctypes.byref(ok), 0.9, p, p, p, None) == 0
    assert q(ctypes.c_void_p(0x1002), 4, 4096, None, 0.0, p, ctypes.byref(ok), 0.9, p, p, p, None) == 4
    assert q(p, 4, 4100, None, 0.0, p, ctypes.byref(ok), 0.9, p, p, p, None) == 4
    for desc, want in ((D(4096, 32, 128, 4, 8), 3), (D(4096, 512, 512, 4, 8), 3), (D(4096, 128, 128, 5, 8), 3), (D(4096, 128, 128, 2, 8), 3), (D(4096, 128, 128, 3, 4), 3),
                       (D(4100, 128, 128, 4, 8), 2), (D(4096, 128, 100, 4, 8), 2),
                       (D(128, 128, 128, 4, 8), 2), (D(65536, 128, 128, 4, 8), 3),
                       (D(4096, 128, 0, 4, 8), 3)):
        assert q(p, 4, 65536, None, 0.0, p, ctypes.byref(desc), 0.9, p, p, p, None) == want
    g = lib.atom_w4a4_gemm
    assert g(p, p, p, 4, p, p, p, 8, ctypes.byref(ok), p, 4, None, None, 0, None) == 2   # ldy < N
    assert g(p, p, p, 4, p, None, p, 8, ctypes.byref(ok), p, 8, None, None, 0, None) == 1
    assert g(p, p, p, 0, p, p, p, 8, ctypes.byref(ok), p, 8, None, None, 0, None) == 0
    assert g(p, p, p, 4, p, p, p, 8, None, p, 8, None, None, 0, None) == 1
    assert lib.atom_w4a4_gemm_workspace_bytes(0, 8, ctypes.byref(ok)) == 0


def test_synthetic_inputs_are_seeded_and_shaped():
    a, b = synth.make(1), synth.make(1)
    assert torch.equal(a.x, b.x) and torch.equal(a.w, b.w) and torch.equal(a.idx, b.idx)
    assert a.x.shape == (16, 512) and a.w.shape == (512, 512) and a.x.dtype == torch.float16
    assert atom.atom_check_reorder_idx(a.idx) == 0
    lin = synth.make(3, 1)
    assert (lin.M, lin.K, lin.N) == (8, 4096, 4096)
    assert atom.atom_check_reorder_idx(lin.idx) == 0
    # the last 128 reordered channels carry the largest magnitudes
    mag = lin.x.float().abs().mean(0)[lin.idx.long()]
    assert mag[-128:].min() > mag[:-128].median()
    assert torch.isfinite(lin.x.float()).all()


def test_host_side_validation_of_the_kv_cache_and_mx_entry_points():
    """Same contract for the entry points of the INT4 KV cache and of the MX variant."""
    lib = atom.load_library()
    D = binding._Desc
    p = ctypes.c_void_p(0x1000)
    kvq = lib.atom_kv_quantize
    assert kvq(None, 4, 128, 128, 1.0, None, 0, 0, p, p, p, None) == 1
    assert kvq(p, 4, 128, 96, 1.0, None, 0, 0, p, p, p, None) == 3              # head dimension not built
    assert kvq(p, 4, 128, 7, 1.0, None, 0, 0, p, p, p, None) == 2
    assert kvq(p, 4, 64, 128, 1.0, None, 0, 0, p, p, p, None) == 2              # ldx < D
    assert kvq(p, 5, 128, 128, 1.0, p, 4, 16, p, p, p, None) == 2               # rows not a multiple of rows_per_seq
    assert kvq(p, 4, 128, 128, 1.0, p, 4, 0, p, p, p, None) == 2                # Tmax
    assert kvq(p, 0, 128, 128, 1.0, None, 0, 0, p, p, p, None) == 0
    assert kvq(ctypes.c_void_p(0x1002), 4, 128, 128, 1.0, None, 0, 0, p, p, p, None) == 4
    kvp = lib.atom_kv_quantize_pair
    assert kvp(p, None, 4, 128, 128, 1.0, p, 4, 16, p, p, p, p, p, p, None) == 1   # no V rows
    assert kvp(p, p, 4, 128, 128, 1.0, p, 4, 16, p, p, p, p, p, None, None) == 1   # no V zero points
    assert kvp(p, p, 4, 128, 96, 1.0, p, 4, 16, p, p, p, p, p, p, None) == 3
    assert kvp(p, p, 5, 128, 128, 1.0, p, 4, 16, p, p, p, p, p, p, None) == 2
    assert kvp(p, ctypes.c_void_p(0x1002), 4, 128, 128, 1.0, p, 4, 16, p, p, p, p, p, p, None) == 4
    assert kvp(p, p, 0, 128, 128, 1.0, p, 4, 16, p, p, p, p, p, p, None) == 0
    att = lib.atom_decode_attention_kv4
    base = [p, 2, 8, 4, 128, 64, p, p, p, p, p, p, p, 1.0, p]
    assert att(*base[:2], 6, *base[3:], None, 0, None) == 2                     # H % Hkv
    assert att(*base[:4], 64, *base[5:], None, 0, None) == 3                    # head dimension
    assert att(*base[:6], None, *base[7:], None, 0, None) == 1                  # seq_len
    assert att(p, 0, *base[2:], None, 0, None) == 0
    assert att(*base[:5], (1 << 25) + 1, *base[6:], None, 0, None) == 3         # 32-bit byte offsets inside a cache head
    assert lib.atom_decode_attention_kv4_workspace_bytes(64, 32, 32, 128, 1024) == 0
    need = lib.atom_decode_attention_kv4_workspace_bytes(1, 2, 2, 128, 8192)
    assert need > 0 and need % (130 * 4) == 0
    assert att(p, 1, 2, 2, 128, 8192, p, p, p, p, p, p, p, 1.0, p, None, 0, None) == 5   # workspace missing
    assert lib.atom_decode_attention_kv4_workspace_bytes(1, 2, 2, 64, 8192) == 0
    assert lib.atom_decode_attention_kv4_workspace_bytes(1, 6, 4, 128, 8192) == 0            # H % Hkv
    # grouped-query launches are sized by B * Hkv workgroups: more splits than the per-head shape
    gq = lib.atom_decode_attention_kv4_workspace_bytes(16, 64, 8, 128, 4096)
    assert gq > 0 and gq % (16 * 64 * 130 * 4) == 0

    mq = lib.atom_mx_quantize_act
    ok = D(4096, 32, 128, 4, 8)
    assert mq(None, 4, 4096, None, 0.0, p, ctypes.byref(ok), 1.0, p, p, p, None) == 1
    assert mq(p, 0, 4096, None, 0.0, p, ctypes.byref(ok), 1.0, p, p, p, None) == 0
    for desc, want in ((D(4096, 128, 128, 4, 8), 3), (D(4096, 32, 64, 4, 8), 2), (D(4096, 32, 0, 4, 8), 3),
                       (D(4000, 32, 128, 4, 8), 2), (D(4096, 32, 128, 4, 4), 3)):
        assert mq(p, 4, 65536, None, 0.0, p, ctypes.byref(desc), 1.0, p, p, p, None) == want
    mg = lib.atom_mx_gemm
    assert mg(p, p, p, 4, p, p, p, 8, ctypes.byref(ok), p, 4, None) == 2         # ldy < N
    assert mg(p, p, None, 4, p, p, p, 8, ctypes.byref(ok), p, 8, None) == 1
    assert mg(p, p, p, 0, p, p, p, 8, ctypes.byref(ok), p, 8, None) == 0
    assert mg(p, p, ctypes.c_void_p(0x1002), 4, p, p, p, 8, ctypes.byref(ok), p, 8, None) == 4


def test_kv_inputs_are_seeded():
    a, b = synth.kv_case(2, 4, 2, 128, 33, case_id=1), synth.kv_case(2, 4, 2, 128, 33, case_id=1)
    assert torch.equal(a.k, b.k) and torch.equal(a.v, b.v) and torch.equal(a.q, b.q)
    assert torch.equal(a.seq_len, b.seq_len) and int(a.seq_len.max()) <= 33 and int(a.seq_len.min()) >= 1
    assert a.k.shape == (2, 2, 33, 128) and a.q.shape == (2, 4, 128) and a.k.dtype == torch.float16


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "ONE GPU" in (r.stderr + r.stdout)


def test_gemm_refuses_shapes_beyond_its_32_bit_offsets():
    """The tiled kernels index the code and scale arrays with 32-bit offsets: shapes whose arrays
    reach 4 GiB are refused on the host, before any launch (fake pointers, never dereferenced)."""
    lib = atom.load_library()
    D = binding._Desc
    p = ctypes.c_void_p(0x1000)
    g = lib.atom_w4a4_gemm
    d = D(32768, 128, 128, 4, 8)
    rows = (1 << 32) // ((32768 - 128) // 2) + 1                     # rows * K4 / 2 >= 2^32
    assert g(p, p, p, rows, p, p, p, 128, ctypes.byref(d), p, 128, None, None, 0, None) == 3
    assert g(p, p, p, 128, p, p, p, rows, ctypes.byref(d), p, rows, None, None, 0, None) == 3
    d = D(256, 128, 128, 4, 8)                                        # tiny K: the tile count overflows first
    big = 1 << 24
    assert g(p, p, p, big, p, p, p, big, ctypes.byref(d), p, big, None, None, 0, None) == 3


def test_packed_gemm_argument_validation():
    lib = atom.load_library()
    D = binding._Desc
    p = ctypes.c_void_p(0x1000)
    ok = D(4096, 128, 128, 4, 8)
    nbytes = lib.atom_pack_weight_bytes(4096, ctypes.byref(ok))
    assert nbytes == 64 * (31 * 6656 + 8704)                         # 64 units of 64 rows, 31 INT4 images and one INT8 image each
    assert lib.atom_pack_weight_bytes(4097, ctypes.byref(ok)) == 65 * (31 * 6656 + 8704)
    assert lib.atom_pack_weight_bytes(0, ctypes.byref(ok)) == 0
    assert lib.atom_pack_weight_bytes(4096, ctypes.byref(D(4096, 64, 128, 4, 8))) == 0
    pk = lib.atom_pack_weight
    assert pk(None, p, p, 4096, ctypes.byref(ok), p, nbytes, None) == 1
    assert pk(p, p, p, 4096, ctypes.byref(ok), p, nbytes - 1, None) == 5
    assert pk(p, p, p, 4096, ctypes.byref(ok), ctypes.c_void_p(0x1010), nbytes, None) == 4
    assert pk(p, p, p, -1, ctypes.byref(ok), p, nbytes, None) == 2
    assert pk(p, p, p, 0, ctypes.byref(ok), p, 0, None) == 0
    assert pk(p, p, p, 65536 * 64, ctypes.byref(ok), p, 1 << 62, None) == 3
    g = lib.atom_w4a4_gemm_packed
    need = lib.atom_w4a4_gemm_packed_workspace_bytes(256, 4096, ctypes.byref(ok))
    assert need == 4 * (31 * 6656 + 8704)
    assert g(p, p, p, 256, p, 4096, ctypes.byref(ok), p, 4096, None, None, 0, None) == 5
    assert g(p, p, p, 256, p, 4096, ctypes.byref(ok), p, 4096, None, p, need - 1, None) == 5
    assert g(p, p, p, 256, p, 4096, ctypes.byref(ok), p, 4000, None, p, need, None) == 2
    assert g(p, p, p, 256, None, 4096, ctypes.byref(ok), p, 4096, None, p, need, None) == 1
    assert g(p, p, p, 0, p, 4096, ctypes.byref(ok), p, 4096, None, p, need, None) == 0
    assert g(p, p, p, 256, p, 4096, ctypes.byref(ok), p, 4096, None, ctypes.c_void_p(0x1010), need, None) == 4


def test_static_scratch_entry_point_validation():
    lib = atom.load_library()
    p = ctypes.c_void_p(0x1000)
    st = lib.atom_decode_attention_kv4_static
    f = ctypes.c_float(1.0)
    assert lib.atom_static_scratch_bytes() == 4 << 20
    assert st(p, 0, 32, 32, 128, 64, p, p, p, p, p, p, p, f, p, None) == 0           # B == 0
    assert st(p, 1, 32, 5, 128, 64, p, p, p, p, p, p, p, f, p, None) == 2            # H % Hkv
    assert st(p, 1, 32, 32, 64, 64, p, p, p, p, p, p, p, f, p, None) == 3            # D
    assert st(p, 1, 1024, 64, 128, 1 << 20, p, p, p, p, p, p, p, f, p, None) == 5    # partials beyond the array


def test_cooperative_decode_linear_argument_validation():
    """atom_decode_linear_coop decides every refusal on the host (fake pointers, never dereferenced)."""
    lib = atom.load_library()
    D = binding._Desc
    p = ctypes.c_void_p(0x1000)
    ok = D(4096, 128, 128, 4, 8)
    assert lib.atom_decode_linear_coop_sync_bytes() == 4 * (64 + 32 * 32)
    f = lib.atom_decode_linear_coop

    def call(x=p, M=8, ldx=4096, d=ok, clip=0.9, N=4096, ldy=4096, codes=p, scales=p, sync=p, w_scale=p):
        return f(x, M, ldx, p, ctypes.c_float(1e-5), p, ctypes.byref(d), ctypes.c_float(clip), p, p, w_scale, N, p, ldy,
                 codes, codes, scales, sync, None)

    assert call(M=0) == 0                                        # nothing to do
    assert call(N=0) == 0
    assert call(M=-1) == 2 and call(ldx=4095) == 2 and call(ldy=4095) == 2
    assert call(x=None) == 1 and call(sync=None) == 1 and call(codes=None) == 1
    assert call(codes=ctypes.c_void_p(0x1040)) == 4              # the code arrays own whole 128-byte lines
    assert call(sync=ctypes.c_void_p(0x1040)) == 4
    assert call(w_scale=ctypes.c_void_p(0x1004)) == 4
    assert call(M=17) == 3                                       # more rows than producers
    assert call(clip=1e-8) == 3
    assert call(d=D(1408, 128, 128, 4, 8), ldx=1408) == 3        # 11 groups: odd
    assert call(d=D(768, 128, 128, 4, 8), ldx=768) == 3          # six groups: fewer than wavefronts
    assert call(d=D(4096, 128, 256, 4, 8)) == 3                  # two INT8 groups
    assert call(d=D(16384, 128, 128, 4, 8), ldx=16384) == 3      # K beyond the front end of one workgroup
    assert call(d=D(4096, 64, 128, 4, 8)) == 3                   # group size
