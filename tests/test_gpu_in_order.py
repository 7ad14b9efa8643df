"""The front end without a reorder index (Section 4.1 of the paper: the reorder fused into the operator
that produces the activation, which then arrives in reordered channel order).  A NULL index must give what
the identity index gives (oracle: index 0..K-1), on every entry point; and a producer whose weight rows
were permuted offline (atom_permute_rows) must lead to the codes of the gathering front end bit for bit."""
import numpy as np
import pytest
import torch

import oracle
import paper_2310_19102_amd as atom
from _gpu_util import assert_quant_equal, dev, npy

pytestmark = pytest.mark.gpu


def _inputs(M, K, seed, norm):
    g = torch.Generator().manual_seed(seed)
    sigma = torch.exp(1.5 * torch.randn(K, generator=g))
    x = (torch.randn((M, K), generator=g) * sigma).to(torch.float16)
    gamma = (1 + 0.1 * torch.randn(K, generator=g)).to(torch.float16) if norm else None
    idx = torch.argsort(sigma, stable=True).to(torch.int32)
    return x, gamma, idx


@pytest.mark.parametrize("M,K,O,norm,clip", [
    (7, 512, 128, True, 0.9),        # one register set
    (33, 4096, 128, True, 0.9),      # the Llama-7B hidden size
    (9, 11008, 128, False, 0.9),     # 512 threads per row, three sets, ragged last sweep
    (3000, 512, 256, True, 1.0),     # several rows per workgroup
    (5, 1408, 128, True, 0.9),       # 11 groups
    (6, 8192, 128, True, 0.9),
    (4, 12416, 128, True, 0.9),      # four sets on 512 threads
    (4, 20480, 128, True, 0.9),      # 1024 threads per row
    (530, 28672, 128, False, 0.9),   # the Llama-70B intermediate size
    (3, 32768, 128, True, 0.9),      # the largest K
    (5, 1024, 128, True, 1e-8),      # clip below 2^-20: the plain kernel, which takes no index as the identity
])
def test_front_end_without_index_is_the_identity_index(M, K, O, norm, clip):
    print(f"[case] no index M={M} K={K} O={O} norm={norm} clip={clip}", flush=True)
    x, gamma, _ = _inputs(M, K, M + K, norm)
    eps = 1e-5
    ident = np.arange(K, dtype=np.int32)
    got = atom.atom_quantize_act(dev(x), dev(gamma), eps, None, 128, O, clip)
    torch.cuda.synchronize()
    want = oracle.quantize_act(x.numpy(), None if gamma is None else gamma.numpy(), eps, ident, 128, O, clip)
    assert_quant_equal(got, want, "no index")
    # and what the library itself gives for an explicit identity index
    got2 = atom.atom_quantize_act(dev(x), dev(gamma), eps, torch.from_numpy(ident).cuda(), 128, O, clip)
    assert_quant_equal(got2, want, "identity index")


@pytest.mark.parametrize("M,K", [(9, 1024), (40, 11008), (3, 20480)])
def test_add_and_swiglu_front_ends_without_index(M, K):
    g = torch.Generator().manual_seed(K + M)
    x, gamma, _ = _inputs(M, K, 5 * M + K, True)
    res = (0.7 * torch.randn((M, K), generator=g)).to(torch.float16)
    ident = np.arange(K, dtype=np.int32)
    h, q4, q8, sc = atom.atom_add_quantize_act(dev(x), dev(res), dev(gamma), 1e-5, None, 128, 128, 0.9)
    torch.cuda.synchronize()
    ref = oracle.add_quantize_act(x.numpy(), res.numpy(), gamma.numpy(), 1e-5, ident, 128, 128, 0.9)
    assert np.array_equal(npy(h).view(np.uint16), ref[0].view(np.uint16))
    assert_quant_equal((q4, q8, sc), ref[1:], "add, no index")
    gate = (3.0 * torch.randn((M, K), generator=g)).to(torch.float16)
    up = torch.randn((M, K), generator=g).to(torch.float16)
    got = atom.atom_swiglu_quantize_act(dev(gate), dev(up), None, 128, 128, 0.9)
    torch.cuda.synchronize()
    assert_quant_equal(got, oracle.swiglu_quantize_act(gate.numpy(), up.numpy(), ident, 128, 128, 0.9), "swiglu, no index")


def test_permuted_producer_gives_the_gathered_codes():
    """gate/up weight rows permuted offline with the down projection's index: the GEMM output columns
    arrive permuted, exactly, and silu(gate) * up quantised without an index has the codes and scales
    of the gathering front end on the unpermuted output."""
    M, Kin, Kmid = 24, 512, 1408
    g = torch.Generator().manual_seed(12)
    x, gamma, idx_in = _inputs(M, Kin, 3, True)
    w_gu = (0.05 * torch.randn((2 * Kmid, Kin), generator=g)).to(torch.float16)
    sigma = torch.exp(1.0 * torch.randn(Kmid, generator=g))
    idx_mid = torch.argsort(sigma, stable=True).to(torch.int32)
    # offline: rows of gate and of up permuted by the down projection's index
    rows = torch.cat([idx_mid, idx_mid + Kmid]).to(torch.int32)
    w_perm = atom.atom_permute_rows(dev(w_gu), dev(rows))
    torch.cuda.synchronize()
    assert torch.equal(w_perm.cpu(), w_gu[rows.long()])
    qa = atom.atom_quantize_act(dev(x), dev(gamma), 1e-5, dev(idx_in))
    y = atom.atom_w4a4_gemm(*qa, *atom.atom_quantize_weight(dev(w_gu), dev(idx_in)))
    yp = atom.atom_w4a4_gemm(*qa, *atom.atom_quantize_weight(w_perm, dev(idx_in)))
    torch.cuda.synchronize()
    assert torch.equal(yp, y[:, dev(rows).long()]), "permuted weight rows = permuted output columns"
    gathered = atom.atom_swiglu_quantize_act(y[:, :Kmid], y[:, Kmid:], dev(idx_mid))
    in_order = atom.atom_swiglu_quantize_act(yp[:, :Kmid], yp[:, Kmid:], None)
    torch.cuda.synchronize()
    for a, b in zip(gathered, in_order):
        assert torch.equal(a, b)
    # gamma as a one-column matrix
    gp = atom.atom_permute_rows(dev(gamma), dev(idx_in))
    assert torch.equal(gp.cpu(), gamma[idx_in.long()])
    # without a norm the plain front end agrees as well
    xs = x[:, idx_in.long()].contiguous()
    a = atom.atom_quantize_act(dev(x), None, 0.0, dev(idx_in))
    b = atom.atom_quantize_act(dev(xs), None, 0.0, None)
    for u, v in zip(a, b):
        assert torch.equal(u, v)


def test_permute_rows_errors():
    m = torch.zeros((4, 8), dtype=torch.float16, device="cuda")
    i = torch.zeros(4, dtype=torch.int32, device="cuda")
    with pytest.raises(atom.AtomError) as e:
        atom.atom_permute_rows(m, i, out=m)
    assert e.value.status == 3                        # in place: unsupported
    far = torch.tensor([0, 3, 99, -5], dtype=torch.int32, device="cuda")
    out = atom.atom_permute_rows(torch.arange(32, dtype=torch.float16, device="cuda").reshape(4, 8), far)
    assert out[2, 0] == 24 and out[3, 0] == 0          # indices outside the matrix are clamped into it
