"""Seeded synthetic inputs shaped like the paper's Llama workloads.

This module holds no quantisation arithmetic: it only draws the fp16
activations, weights, RMSNorm gains and the channel reorder index that both the
HIP library and the CPU oracle are fed, byte for byte.  The paper evaluates its
kernels on Llama-7B-shaped linears (Section 5.3.1) with real activations whose
few outlier channels are orders of magnitude larger than the rest (Section 4.1);
here heavy-tailed per-channel magnitudes stand in for those activations and a
synthetic per-channel statistic stands in for the calibration that picks the
128 outlier channels (Section 5.1).

Everything is generated on the CPU with ``torch.Generator`` so the same seed
gives the same bytes on every machine.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Optional

import torch

BASE_SEED = 20231019
GROUP_SIZE = 128
N_OUTLIER = 128
CLIP_ACT = 0.9     # Section 5.1: grid-searched clip factor for activations
CLIP_WEIGHT = 0.85  # Section 5.1: clip factor for weights
EPS = 1e-6


def _gen(config: int, tensor_id: int) -> torch.Generator:
    g = torch.Generator(device="cpu")
    g.manual_seed(BASE_SEED + 1000 * config + tensor_id)
    return g


@dataclass
class Linear:
    """One quantised linear layer's inputs (all CPU tensors)."""
    name: str
    x: torch.Tensor                 # [M, K] fp16 activations
    w: torch.Tensor                 # [N, K] fp16 weights (nn.Linear layout)
    gamma: Optional[torch.Tensor]   # [K] fp16 RMSNorm gain, or None (no norm)
    idx: torch.Tensor               # [K] int32 reorder index, outliers last
    eps: float = EPS
    clip_act: float = CLIP_ACT
    clip_weight: float = CLIP_WEIGHT
    group_size: int = GROUP_SIZE
    n_outlier: int = N_OUTLIER

    @property
    def M(self): return self.x.shape[0]

    @property
    def K(self): return self.x.shape[1]

    @property
    def N(self): return self.w.shape[0]


def gamma_vector(K: int, config: int, tensor_id: int) -> torch.Tensor:
    return (1.0 + 0.1 * torch.randn(K, generator=_gen(config, tensor_id))).to(torch.float16)


def weight_matrix(N: int, K: int, std: float, config: int, tensor_id: int) -> torch.Tensor:
    # drawn in row chunks so a 57344 x 8192 matrix never needs a 1.9 GB fp32 temporary
    g = _gen(config, tensor_id)
    out = torch.empty((N, K), dtype=torch.float16)
    step = 4096
    for r in range(0, N, step):
        rows = min(step, N - r)
        out[r:r + rows] = (std * torch.randn((rows, K), generator=g)).to(torch.float16)
    return out


def tiny_linear(config: int = 1, M: int = 16, K: int = 512, N: int = 512) -> Linear:
    """Config 1: N(0,1) activations with 128 random channels scaled x20."""
    x = torch.randn((M, K), generator=_gen(config, 0))
    perm = torch.randperm(K, generator=_gen(config, 1))
    outl = torch.sort(perm[:N_OUTLIER]).values
    x[:, outl] *= 20.0
    mask = torch.ones(K, dtype=torch.bool)
    mask[outl] = False
    normal = torch.nonzero(mask).flatten()
    idx = torch.cat([normal, outl]).to(torch.int32)
    w = weight_matrix(N, K, 0.02, config, 2)
    gamma = gamma_vector(K, config, 3)
    return Linear("tiny", x.to(torch.float16), w, gamma, idx)


def heavy_tailed_activations(M: int, K: int, config: int, tensor_id: int):
    """x[m,k] = z * sigma_k with lognormal(sigma=1.5) channel magnitudes.
    Returns (x fp16, idx int32) where idx is the stable ascending argsort of
    sigma, so the 128 largest-magnitude channels come last."""
    xi = torch.randn(K, generator=_gen(config, tensor_id))
    sigma = torch.exp(1.5 * xi)
    g = _gen(config, tensor_id + 50)
    x = torch.empty((M, K), dtype=torch.float16)
    step = 512
    for r in range(0, M, step):
        rows = min(step, M - r)
        x[r:r + rows] = (torch.randn((rows, K), generator=g) * sigma).to(torch.float16)
    idx = torch.argsort(sigma, stable=True).to(torch.int32)
    return x, idx


def llama_linear(name: str, M: int, K: int, N: int, config: int, tensor_base: int = 0,
                 norm: bool = True, w_std: float = 0.02) -> Linear:
    x, idx = heavy_tailed_activations(M, K, config, tensor_base + 0)
    w = weight_matrix(N, K, w_std, config, tensor_base + 2)
    gamma = gamma_vector(K, config, tensor_base + 3) if norm else None
    return Linear(name, x, w, gamma, idx)


# The five benchmark configurations, by the numbering used in the tests and in
# bench.py.  Each entry: (name, M, K, N, norm, w_std).
CONFIG_SHAPES = {
    1: [("tiny", 16, 512, 512, True, 0.02)],
    2: [("attn_proj", 256, 4096, 4096, True, 0.02),
        ("fused_qkv", 256, 4096, 12288, True, 0.02)],
    3: [(f"decode_m{m}_n{n}", m, 4096, n, True, 0.02)
        for n in (4096, 11008) for m in (1, 8, 32, 64)],
    4: [("mlp_gate_up", 1024, 4096, 22016, True, 0.02),
        ("mlp_down", 1024, 11008, 4096, False, 0.02)],
    5: [("l70_qkv", 4096, 8192, 10240, True, 0.01),
        ("l70_gate_up", 4096, 8192, 57344, True, 0.01),
        ("l70_down", 4096, 28672, 8192, False, 0.01)],
}


def make(config: int, which: int = 0, M: Optional[int] = None) -> Linear:
    """Build linear number ``which`` of benchmark configuration ``config``.
    ``M`` overrides the row count (a row-subset problem with the same
    weights, reorder index and gain: activations of a smaller M are NOT a
    prefix of the larger one)."""
    name, m, K, N, norm, std = CONFIG_SHAPES[config][which]
    if M is not None:
        m = M
    if config == 1:
        return tiny_linear(config, m, K, N)
    return llama_linear(name, m, K, N, config, tensor_base=10 * which, norm=norm, w_std=std)


@dataclass
class KVCase:
    """Inputs of one decode-attention step over a KV cache (all CPU tensors)."""
    q: torch.Tensor         # [B, H, D] fp16 query of the new token
    k: torch.Tensor         # [B, Hkv, Tmax, D] fp16 keys
    v: torch.Tensor         # [B, Hkv, Tmax, D] fp16 values
    seq_len: torch.Tensor   # [B] int32, tokens in the cache per sequence
    sm_scale: float


def kv_case(B: int, H: int, Hkv: int, D: int, Tmax: int, seq_lens=None, case_id: int = 0) -> KVCase:
    """Keys with per-channel offsets and magnitudes (a few channels of a head are
    consistently larger, which is what an asymmetric per-head range has to absorb; Section
    4.4), values close to Gaussian, a unit-variance query.  ``seq_lens`` defaults to a
    ragged mix between Tmax/4 and Tmax."""
    cfg = 900 + case_id
    mu = torch.randn((1, Hkv, 1, D), generator=_gen(cfg, 0))
    sigma = torch.exp(0.5 * torch.randn((1, Hkv, 1, D), generator=_gen(cfg, 1)))
    k = (torch.randn((B, Hkv, Tmax, D), generator=_gen(cfg, 2)) * sigma + mu).to(torch.float16)
    v = (0.5 * torch.randn((B, Hkv, Tmax, D), generator=_gen(cfg, 3))).to(torch.float16)
    q = torch.randn((B, H, D), generator=_gen(cfg, 4)).to(torch.float16)
    if seq_lens is None:
        lo = max(1, Tmax // 4)
        seq_lens = torch.randint(lo, Tmax + 1, (B,), generator=_gen(cfg, 5)) if Tmax > 0 else torch.zeros(B)
    seq_len = torch.as_tensor(seq_lens, dtype=torch.int32)
    return KVCase(q, k, v, seq_len, 1.0 / float(D) ** 0.5)
