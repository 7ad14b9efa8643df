"""Guard bands around every output of the hot path: the kernels write their outputs and nothing
else.  Each output lives inside a larger allocation filled with a byte pattern (a band in front, a
band behind, and the padding columns of strided rows); shapes are ragged on purpose (rows and
columns that end inside a tile).  After the call every byte outside the output must still hold the
pattern.  Results themselves are checked by the parity tests."""
import numpy as np
import pytest
import torch

import paper_2310_19102_amd as atom

pytestmark = pytest.mark.gpu

PAT = 0xA5
BAND = 4096          # bytes in front of and behind each output


class Guarded:
    """A [rows, cols] view (row stride ld elements) inside a pattern-filled byte buffer."""

    def __init__(self, rows, cols, dtype, ld=None):
        self.rows, self.cols, self.ld = rows, cols, ld or cols
        self.item = torch.empty(0, dtype=dtype).element_size()
        self.nbytes = max(rows * self.ld, 1) * self.item
        self.raw = torch.full((BAND + self.nbytes + BAND,), PAT, dtype=torch.uint8, device="cuda")
        body = self.raw[BAND:BAND + self.nbytes].view(dtype)
        self.view = body[:rows * self.ld].view(rows, self.ld)[:, :cols] if rows else body[:0].view(0, cols)

    def check(self, what):
        raw = self.raw.cpu().numpy()
        assert (raw[:BAND] == PAT).all(), f"{what}: bytes in front of the output were written"
        assert (raw[BAND + self.nbytes:] == PAT).all(), f"{what}: bytes behind the output were written"
        if self.ld > self.cols and self.rows:
            body = raw[BAND:BAND + self.nbytes].reshape(self.rows, self.ld * self.item)
            assert (body[:, self.cols * self.item:] == PAT).all(), f"{what}: padding columns were written"
        written = self.view.contiguous().view(torch.uint8).cpu().numpy()
        assert written.size == 0 or (written != PAT).any(), f"{what}: the output itself was never written"


def _inputs(M, K, N, O, seed):
    g = torch.Generator().manual_seed(seed)
    sigma = torch.exp(1.5 * torch.randn(K, generator=g))
    x = (torch.randn((M, K), generator=g) * sigma).to(torch.float16).cuda()
    w = (0.02 * torch.randn((N, K), generator=g)).to(torch.float16).cuda()
    gamma = (1 + 0.1 * torch.randn(K, generator=g)).to(torch.float16).cuda()
    idx = torch.argsort(sigma, stable=True).to(torch.int32).cuda()
    return x, w, gamma, idx


def _quant_guards(rows, K, O):
    return (Guarded(rows, (K - O) // 2, torch.uint8), Guarded(rows, O, torch.int8), Guarded(rows, K // 128, torch.float16))


@pytest.mark.parametrize("M,K,O", [(1, 512, 128), (7, 1408, 128), (33, 4096, 256), (3, 11008, 128), (5, 20480, 128),
                                   (2, 32768, 128)])
def test_front_end_outputs(M, K, O):
    x, _, gamma, idx = _inputs(M, K, 8, O, M + K)
    res = (0.5 * x).clone()
    for name, call in (
        ("quantize_act", lambda out: atom.atom_quantize_act(x, gamma, 1e-5, idx, 128, O, 0.9, out=out)),
        ("quantize_act, no index", lambda out: atom.atom_quantize_act(x, gamma, 1e-5, None, 128, O, 0.9, out=out)),
        ("quantize_act, plain kernel", lambda out: atom.atom_quantize_act(x, None, 0.0, idx, 128, O, 1e-8, out=out)),
        ("swiglu", lambda out: atom.atom_swiglu_quantize_act(x, res, idx, 128, O, 0.9, out=out)),
        ("quantize_weight", lambda out: atom.atom_quantize_weight(x, idx, 128, O, 0.85, out=out)),
    ):
        g = _quant_guards(M, K, O)
        call(tuple(t.view for t in g))
        torch.cuda.synchronize()
        for t, part in zip(g, ("q4", "q8", "scale")):
            t.check(f"{name} M={M} K={K}: {part}")
    g = _quant_guards(M, K, O)
    hs = Guarded(M, K, torch.float16, ld=K + 24)
    atom.atom_add_quantize_act(x, res, gamma, 1e-5, idx, 128, O, 0.9, sum_out=hs.view, out=tuple(t.view for t in g))
    torch.cuda.synchronize()
    hs.check("add: sum")
    for t, part in zip(g, ("q4", "q8", "scale")):
        t.check(f"add M={M} K={K}: {part}")


# shapes that end inside a tile of every GEMM kernel: decode (16-column blocks, row blocks of 16),
# few tiles (64 x 32 / 64 x 64), big tiles (128 / 256 rows x 128 columns), packed (64-row units)
GEMM_SHAPES = [(1, 512, 17), (8, 1408, 100), (17, 896, 48), (40, 640, 33), (64, 2304, 16), (65, 384, 72),
               (70, 256, 130), (200, 1152, 300), (129, 512, 257), (300, 1024, 1000), (1030, 512, 2050)]


@pytest.mark.parametrize("M,K,N", GEMM_SHAPES)
def test_gemm_outputs(M, K, N):
    x, w, gamma, idx = _inputs(M, K, N, 128, M + N)
    qa = atom.atom_quantize_act(x, gamma, 1e-5, idx)
    qw = atom.atom_quantize_weight(w, idx)
    y = Guarded(M, N, torch.float16, ld=N + 40)
    atom.atom_w4a4_gemm(*qa, *qw, out=y.view)
    torch.cuda.synchronize()
    y.check(f"gemm {M}x{K}x{N}")
    y = Guarded(M, N, torch.float16)
    part = Guarded(M * N, K // 128, torch.int32)
    atom.atom_w4a4_gemm(*qa, *qw, out=y.view, partials=part.view.view(M, N, K // 128))
    torch.cuda.synchronize()
    y.check(f"gemm with partials {M}x{K}x{N}")
    part.check(f"partials {M}x{K}x{N}")
    # packed weights: the packed arrays and Y
    nbytes = atom.atom_pack_weight(*qw).numel()
    wp = Guarded(1, nbytes, torch.uint8)
    atom.atom_pack_weight(*qw, out=wp.view.view(-1))
    ws = Guarded(1, atom.atom_w4a4_gemm_packed_workspace_bytes(M, N, K), torch.uint8)
    y = Guarded(M, N, torch.float16, ld=N + 8)
    atom.atom_w4a4_gemm_packed(*qa, wp.view.view(-1), N, out=y.view, workspace=ws.view.view(-1))
    torch.cuda.synchronize()
    wp.check(f"packed weights N={N} K={K}")
    ws.check(f"re-tiled activations M={M} K={K}")
    y.check(f"packed gemm {M}x{K}x{N}")


@pytest.mark.parametrize("M,K,N", [(1, 1024, 17), (5, 4096, 100), (16, 2048, 33)])
def test_decode_paths_outputs(M, K, N):
    x, w, gamma, idx = _inputs(M, K, N, 128, M + N + 1)
    qa = atom.atom_quantize_act(x, gamma, 1e-5, idx)
    qw = atom.atom_quantize_weight(w, idx)
    y = Guarded(M, N, torch.float16, ld=N + 24)
    atom.atom_decode_linear(x, gamma, 1e-5, idx, *qw, out=y.view)
    torch.cuda.synchronize()
    y.check(f"decode linear {M}x{K}x{N}")
    t4 = Guarded(1, (N + 15) // 16 * 16 * (K - 128) // 2, torch.uint8)
    t8 = Guarded(1, (N + 15) // 16 * 16 * 128, torch.int8)
    L = atom.load_library()
    import ctypes
    from paper_2310_19102_amd.binding import _desc, _ptr, _stream
    d = _desc(K, 128, 128, 4)
    assert L.atom_tile_weight_decode(_ptr(qw[0]), _ptr(qw[1]), N, ctypes.byref(d), _ptr(t4.view), t4.view.numel(),
                                     _ptr(t8.view), t8.view.numel(), _stream()) == 0
    y = Guarded(M, N, torch.float16, ld=N + 24)
    atom.atom_w4a4_gemm_decode_tiled(*qa, t4.view.view(-1), t8.view.view(-1), qw[2], out=y.view)
    torch.cuda.synchronize()
    t4.check("tiled INT4 weights")
    t8.check("tiled INT8 weights")
    y.check(f"tiled decode gemm {M}x{K}x{N}")
