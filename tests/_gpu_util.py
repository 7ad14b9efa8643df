"""Helpers shared by the GPU parity tests: run the HIP library through its
Python binding (which calls the C ABI) and the CPU oracle on the same seeded
inputs, and compare."""
import numpy as np
import torch

import oracle
import paper_2310_19102_amd as atom

Y_TOL = 1e-3   # max relative error on the fp16 outputs (floor: 1% of max|Yref|)


def dev(t):
    return t.cuda() if t is not None else None


def npy(t):
    return t.detach().cpu().numpy()


def y_rel_err(y, yref):
    y = y.astype(np.float64)
    yref = yref.astype(np.float64)
    if yref.size == 0:
        return 0.0
    floor = 1e-2 * np.abs(yref).max()
    return float((np.abs(y - yref) / np.maximum(np.abs(yref), max(floor, 1e-30))).max())


def gpu_quantize_act(lin, rows=None):
    x = lin.x if rows is None else lin.x[rows]
    q = atom.atom_quantize_act(dev(x.contiguous()), dev(lin.gamma), lin.eps, dev(lin.idx),
                               lin.group_size, lin.n_outlier, lin.clip_act)
    torch.cuda.synchronize()
    return q


def gpu_quantize_weight(lin):
    q = atom.atom_quantize_weight(dev(lin.w), dev(lin.idx), lin.group_size, lin.n_outlier,
                                  lin.clip_weight)
    torch.cuda.synchronize()
    return q


def ref_quantize_act(lin, rows=None):
    x = lin.x if rows is None else lin.x[rows]
    g = None if lin.gamma is None else lin.gamma.numpy()
    return oracle.quantize_act(x.numpy(), g, lin.eps, lin.idx.numpy(), lin.group_size,
                               lin.n_outlier, lin.clip_act)


def ref_quantize_weight(lin):
    return oracle.quantize_weight(lin.w.numpy(), lin.idx.numpy(), lin.group_size, lin.n_outlier,
                                  lin.clip_weight)


def assert_quant_equal(gpu, ref, what):
    names = ("q4", "q8", "scale")
    for name, g, r in zip(names, gpu, ref):
        g = npy(g)
        if name == "scale":
            g, r = g.view(np.uint16), r.view(np.uint16)
        if not np.array_equal(g, r):
            bad = np.argwhere(g != r)
            raise AssertionError(f"{what}: {name} differs at {len(bad)} places, first {bad[0]}: "
                                 f"gpu {g[tuple(bad[0])]} ref {r[tuple(bad[0])]}")
