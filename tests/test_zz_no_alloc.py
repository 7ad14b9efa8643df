"""The entry point that allocates nothing (atom_decode_attention_kv4_static: the partials of a
split launch live in the library's own per-GPU scratch array) against the entry point that takes a
workspace: the same kernels, so the same bits.  Two calls in a row, the second on a smaller input,
so that stale contents of the shared scratch from the first call would show."""
import numpy as np
import pytest
import torch

import paper_2310_19102_amd as atom
from paper_2310_19102_amd import synth

pytestmark = pytest.mark.gpu


def _caches(kv):
    k = atom.atom_kv_quantize(kv.k.cuda(), 1.0)
    v = atom.atom_kv_quantize(kv.v.cuda(), 1.0)
    return k, v


def _both(kv):
    k, v = _caches(kv)
    q, sl = kv.q.cuda(), kv.seq_len.cuda()
    B, H, D = q.shape
    Hkv, Tmax = k[0].shape[1], k[0].shape[2]
    need = atom.atom_decode_attention_kv4_workspace_bytes(B, H, Hkv, D, Tmax)
    assert 0 < need <= atom.atom_static_scratch_bytes(), "the case must use the scratch and fit it"
    want = atom.atom_decode_attention_kv4(q, k, v, sl, kv.sm_scale)
    got = torch.full_like(want, float("nan"))
    torch.cuda.synchronize()
    # the number of device allocations made so far (a count of events: tensors of earlier tests
    # that the garbage collector frees in the meantime do not change it)
    before = torch.cuda.memory_stats().get("allocation.all.allocated", 0)
    atom.atom_decode_attention_kv4_static(q, k, v, sl, kv.sm_scale, out=got)
    torch.cuda.synchronize()
    assert torch.cuda.memory_stats().get("allocation.all.allocated", 0) == before, "the call allocated device memory"
    return got.cpu().numpy(), want.cpu().numpy()


def test_static_scratch_two_calls_second_smaller():
    # per-head kernel, 16 wavefronts, two splits; then grouped-query, four splits; then a smaller
    # per-head case on four wavefronts, two splits
    cases = [synth.kv_case(2, 4, 4, 128, 2048, case_id=11),
             synth.kv_case(1, 8, 2, 128, 1024, case_id=12),
             synth.kv_case(1, 4, 4, 128, 512, case_id=13)]
    for i, kv in enumerate(cases):
        print(f"[case] no-alloc attention call {i}: B={kv.q.shape[0]} H={kv.q.shape[1]} T={kv.k.shape[2]}", flush=True)
        got, want = _both(kv)
        assert np.array_equal(got.view(np.uint16), want.view(np.uint16)), f"call {i} differs"


def test_static_scratch_rejects_oversized():
    """Sizes whose partials exceed the array are refused on the host, before any launch."""
    st = atom.load_library().atom_decode_attention_kv4_static
    B, H, Hkv, T = 1, 1024, 64, 1 << 20            # 16 query heads per cache head, many splits
    need = atom.atom_decode_attention_kv4_workspace_bytes(B, H, Hkv, 128, T)
    assert need > atom.atom_static_scratch_bytes()
    import ctypes
    one = ctypes.c_void_p(256)                      # never dereferenced: the size check comes first
    rc = st(one, B, H, Hkv, 128, T, one, one, one, one, one, one, one, ctypes.c_float(1.0), one, None)
    assert rc == 5
