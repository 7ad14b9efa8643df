"""GPU parity of the offline calibration: square sums and reorder index bit-identical to the
CPU oracle (both sum exactly, in integers of 2^-48, so no order of additions is shared)."""
import numpy as np
import pytest
import torch

import oracle
import paper_2310_19102_amd as atom
from paper_2310_19102_amd import synth

pytestmark = pytest.mark.gpu


def _check(x, what):
    print(f"[case] calibrate {what}: T={x.shape[0]} K={x.shape[1]}", flush=True)
    idx, stat = atom.atom_calibrate_reorder(x.cuda())
    torch.cuda.synchronize()
    rs, ri = oracle.calibrate_reorder(x.numpy())
    assert np.array_equal(stat.cpu().numpy().view(np.uint64), rs.view(np.uint64)), f"{what}: square sums differ"
    assert np.array_equal(idx.cpu().numpy(), ri), f"{what}: index differs"
    assert atom.atom_check_reorder_idx(idx.cpu()) == 0
    return idx


@pytest.mark.parametrize("T,K", [(1, 8), (255, 100), (256, 256), (257, 300), (1000, 512), (3000, 4096)])
def test_calibrate(T, K):
    g = torch.Generator().manual_seed(T + K)
    sigma = torch.exp(1.5 * torch.randn(K, generator=g))
    x = (torch.randn((T, K), generator=g) * sigma).to(torch.float16)
    _check(x, "random")


def test_calibrate_ties_zero_rows_and_stride():
    g = torch.Generator().manual_seed(3)
    x = torch.randint(-4, 5, (600, 64), generator=g).to(torch.float16)
    x[:, 9] = x[:, 40]                                  # equal channels keep their order
    x[:, 3] = 0
    idx = _check(x, "ties").cpu().tolist()
    assert idx[0] == 3 and idx.index(9) + 1 == idx.index(40)
    _check(torch.zeros((0, 16), dtype=torch.float16), "no rows")
    wide = torch.randn((300, 96), generator=g).to(torch.float16)
    view = wide[:, :64]                                 # row stride 96
    i1, s1 = atom.atom_calibrate_reorder(view.cuda()[:, :64])
    rs, ri = oracle.calibrate_reorder(np.ascontiguousarray(view.numpy()))
    assert np.array_equal(i1.cpu().numpy(), ri) and np.array_equal(s1.cpu().numpy(), rs)


def test_calibrated_index_feeds_the_front_end():
    """The index computed from a layer's own activations puts its heavy channels last, and the
    front end takes it as it is."""
    lin = synth.make(2, 0)
    idx, _ = atom.atom_calibrate_reorder(lin.x.cuda())
    ri = oracle.calibrate_reorder(lin.x.numpy())[1]
    assert np.array_equal(idx.cpu().numpy(), ri)
    assert set(ri[-128:].tolist()) == set(lin.idx.numpy()[-128:].tolist()) or \
        len(set(ri[-128:].tolist()) & set(lin.idx.numpy()[-128:].tolist())) >= 120
    q = atom.atom_quantize_act(lin.x.cuda(), lin.gamma.cuda(), lin.eps, idx)
    r = oracle.quantize_act(lin.x.numpy(), lin.gamma.numpy(), lin.eps, ri, 128, 128, 0.9)
    for a, b in zip(q, r):
        assert np.array_equal(a.cpu().numpy().view(np.uint8), b.view(np.uint8))


def test_calibrate_errors():
    x = torch.zeros((4, 16), dtype=torch.float16, device="cuda")
    L = atom.load_library()
    import ctypes
    P = lambda t: ctypes.c_void_p(t.data_ptr())
    idx = torch.empty(16, dtype=torch.int32, device="cuda")
    ws = torch.empty(128, dtype=torch.float64, device="cuda")
    assert L.atom_calibrate_reorder(P(x), 4, 8, 16, P(ws), 1024, P(idx), None) == 2     # ldx < K
    assert L.atom_calibrate_reorder(P(x), 4, 16, 16, P(ws), 16, P(idx), None) == 5      # workspace too small
    assert L.atom_calibrate_reorder(P(x), 4, 16, 16, None, 0, P(idx), None) == 1
    assert L.atom_calibrate_reorder(P(x), 4, 16, 40000, P(ws), 1024, P(idx), None) == 2  # ldx < K
    assert L.atom_calibrate_reorder_workspace_bytes(4, 16) == 2 * 16 * 16 + 16 * 8


def test_calibrate_wide_range_and_special_values():
    """Channels mixing the largest and the smallest fp16 magnitudes (sums beyond 2^64 units next to
    subnormal squares), Inf and NaN: still bit-identical, and independent of the order of the rows."""
    g = torch.Generator().manual_seed(17)
    x = (torch.randn((777, 40), generator=g) * 3).to(torch.float16)
    x[::3, 0] = 65504.0
    x[1::3, 0] = 6e-8
    x[:, 1] = 6e-8
    x[5, 2] = float("inf")
    x[6, 3] = float("nan")
    x[:, 4] = -65504.0
    i0 = _check(x, "wide range")
    perm = torch.randperm(777, generator=g)
    i1, s1 = atom.atom_calibrate_reorder(x[perm].cuda())
    s0 = atom.atom_calibrate_reorder(x.cuda())[1]
    assert torch.equal(i0, i1) and torch.equal(s0.view(torch.int64), s1.view(torch.int64))
