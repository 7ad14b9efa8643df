"""The hot path under HIP graph capture and from two host threads.

A captured chain (front end -> activation re-tiling -> packed GEMM, and the one-launch decode linear)
is replayed several times with new inputs written into the same buffers and eager work in between;
every replay must give what the eager calls give on the same inputs, bit for bit (the entry points
allocate nothing and keep no state, so capture needs no special path).  Two host threads that make
their first calls of different kernel variants at the same time, each on its own stream, must both
get the right results (the one-time kernel attribute set-up is kept in atomics)."""
import threading

import numpy as np
import pytest
import torch

import paper_2310_19102_amd as atom

pytestmark = pytest.mark.gpu


def _inputs(M, K, N, seed):
    g = torch.Generator().manual_seed(seed)
    sigma = torch.exp(1.5 * torch.randn(K, generator=g))
    x = (torch.randn((M, K), generator=g) * sigma).to(torch.float16).cuda()
    w = (0.02 * torch.randn((N, K), generator=g)).to(torch.float16).cuda()
    gamma = (1 + 0.1 * torch.randn(K, generator=g)).to(torch.float16).cuda()
    idx = torch.argsort(sigma, stable=True).to(torch.int32).cuda()
    return x, w, gamma, idx


def test_graph_replays_match_eager():
    M, K, N = 200, 1024, 384
    x, w, gamma, idx = _inputs(M, K, N, 1)
    qw = atom.atom_quantize_weight(w, idx)
    wp = atom.atom_pack_weight(*qw)
    xs = torch.empty_like(x)                         # the graph's input buffer
    qa = atom.atom_quantize_act(x, gamma, 1e-5, idx)
    apk = torch.empty(atom.atom_w4a4_gemm_packed_workspace_bytes(M, N, K), dtype=torch.uint8, device="cuda")
    y = torch.empty((M, N), dtype=torch.float16, device="cuda")
    yd = torch.empty((8, N), dtype=torch.float16, device="cuda")

    def chain():
        atom.atom_quantize_act(xs, gamma, 1e-5, idx, out=qa)
        atom.atom_pack_act(*qa, out=apk)
        atom.atom_w4a4_gemm_prepacked(apk, M, wp, N, K, out=y)
        atom.atom_decode_linear(xs[:8], gamma, 1e-5, idx, *qw, out=yd)

    xs.copy_(x)
    chain()                                          # first calls outside the capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        chain()
    for rep in range(4):
        xn = (x * (0.5 + rep)).roll(rep, dims=0).contiguous()
        # eager reference on separate buffers, between the replays
        ra = atom.atom_quantize_act(xn, gamma, 1e-5, idx)
        want = atom.atom_w4a4_gemm_packed(*ra, wp, N)
        want_d = atom.atom_decode_linear(xn[:8].contiguous(), gamma, 1e-5, idx, *qw)
        torch.cuda.synchronize()
        xs.copy_(xn)
        y.fill_(float("nan"))
        yd.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(y, want), f"replay {rep}: packed GEMM differs from the eager result"
        assert torch.equal(yd, want_d), f"replay {rep}: decode linear differs from the eager result"


def test_two_host_threads_first_calls():
    shapes = [(300, 2048, 512), (1100, 512, 1300)]          # different kernel variants (tile heights, front ends)
    data = [_inputs(M, K, N, 10 + i) for i, (M, K, N) in enumerate(shapes)]
    results, errors = [None, None], []
    start = threading.Barrier(2)

    def work(i):
        try:
            x, w, gamma, idx = data[i]
            with torch.cuda.stream(torch.cuda.Stream()):
                start.wait()
                qa = atom.atom_quantize_act(x, gamma, 1e-5, idx)
                qw = atom.atom_quantize_weight(w, idx)
                y = atom.atom_w4a4_gemm_packed(*qa, atom.atom_pack_weight(*qw), w.shape[0])
                y2 = atom.atom_w4a4_gemm(*qa, *qw)
                torch.cuda.current_stream().synchronize()
            results[i] = (y, y2)
        except Exception as e:                                   # noqa: BLE001
            errors.append(e)

    threads = [threading.Thread(target=work, args=(i,)) for i in range(2)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not errors, errors
    torch.cuda.synchronize()
    for i, (x, w, gamma, idx) in enumerate(data):
        qa = atom.atom_quantize_act(x, gamma, 1e-5, idx)
        qw = atom.atom_quantize_weight(w, idx)
        y = atom.atom_w4a4_gemm_packed(*qa, atom.atom_pack_weight(*qw), w.shape[0])
        y2 = atom.atom_w4a4_gemm(*qa, *qw)
        torch.cuda.synchronize()
        assert torch.equal(results[i][0], y) and torch.equal(results[i][1], y2), f"thread {i}"
