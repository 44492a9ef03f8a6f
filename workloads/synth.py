"""Seeded synthetic inputs for the MoE verify layer: shapes, value distributions and skew of
the five benchmark configurations.  Shared by the tests, the smoke check and the benchmark;
used to feed BOTH the HIP library and the CPU oracle the same numbers.

Nothing of the method is computed here: only random tensors, their rounding to the run
dtype, and token-id patterns.  The paper's workloads (NLLB-MoE on WMT-14, Mixtral-8x7B and
Llama-4-Scout on CNN-DailyMail; Table I) are not available offline; these inputs stand in
for them with the layer shapes of Table I and a skewed router for the "hotness" the paper
describes in Sec. 3.2.
"""
from __future__ import annotations

import dataclasses
import math

import numpy as np
import torch


@dataclasses.dataclass(frozen=True)
class MoEConfig:
    name: str
    dtype: str            # "f32" | "bf16"
    d_model: int
    d_ff: int
    E: int
    k: int
    B: int
    gamma: int
    x_std: float          # activations ~ N(0, x_std^2)
    w_std: float          # expert weights ~ N(0, w_std^2)
    router_std: float     # router weights ~ N(0, router_std^2)
    zipf: float = 0.0     # > 0: per-expert logit bias  -zipf * ln(rank)
    renorm: bool = True
    vocab: int = 32000
    n_layers: int = 1
    match_prob: float = -1.0   # >= 0: target repeats the draft with this probability per position

    @property
    def T(self) -> int:
        return self.B * (self.gamma + 1)

    @property
    def P(self) -> int:
        return self.T * self.k

    @property
    def torch_dtype(self):
        return torch.float32 if self.dtype == "f32" else torch.bfloat16

    def flops(self) -> float:
        """Algorithmic flops of one layer: experts 6*P*d*f plus router 2*T*d*E."""
        return 6.0 * self.P * self.d_model * self.d_ff + 2.0 * self.T * self.d_model * self.E


CONFIGS = {
    1: MoEConfig("cfg1-tiny-f32", "f32", 256, 512, 8, 2, 4, 3,
                 x_std=0.02, w_std=0.02, router_std=0.1, vocab=1000),
    2: MoEConfig("cfg2-mixtral-layer", "bf16", 4096, 14336, 8, 2, 16, 4,
                 x_std=1.0 / math.sqrt(4096), w_std=0.02, router_std=0.02),
    3: MoEConfig("cfg3-fine-grained-zipf", "bf16", 2048, 1408, 64, 6, 64, 4,
                 x_std=1.0 / math.sqrt(2048), w_std=0.02, router_std=1.0, zipf=1.1),
    4: MoEConfig("cfg4-large-batch-verify", "bf16", 4096, 14336, 8, 2, 256, 7,
                 x_std=1.0 / math.sqrt(4096), w_std=0.02, router_std=0.02),
    5: MoEConfig("cfg5-32-layer-stack", "bf16", 4096, 14336, 8, 2, 32, 4,
                 x_std=1.0 / math.sqrt(4096), w_std=0.02, router_std=0.02,
                 n_layers=32, match_prob=0.7),
    # Llama-4-Scout-shaped block (Table I: 16 experts, top-1 routing, skewness 0.59; 218 GB over
    # 48 layers -> d = 5120, f = 8192).  Zipf exponent 0.53 with unit logit noise puts 59 % of
    # the tokens on the 4 hottest experts.
    6: MoEConfig("cfg6-scout-top1", "bf16", 5120, 8192, 16, 1, 256, 7,
                 x_std=1.0 / math.sqrt(5120), w_std=0.02, router_std=1.0, zipf=0.53),
}


def _gen(device, seed):
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def _normal(shape, std, dtype, device, seed, chunk_rows=None):
    """N(0, std^2) drawn in fp32 and rounded once (to nearest even) to `dtype`."""
    g = _gen(device, seed)
    if chunk_rows is None or len(shape) < 2:
        return (torch.randn(shape, generator=g, device=device, dtype=torch.float32) * std).to(dtype)
    out = torch.empty(shape, device=device, dtype=dtype)
    flat = out.view(-1, shape[-1])
    for r0 in range(0, flat.shape[0], chunk_rows):
        r1 = min(flat.shape[0], r0 + chunk_rows)
        flat[r0:r1] = (torch.randn((r1 - r0, shape[-1]), generator=g, device=device,
                                   dtype=torch.float32) * std).to(dtype)
    return out


def make_layer(cfg: MoEConfig, device="cpu", seed=0, layer=0, T=None):
    """Tensors of one MoE layer in the run dtype, on `device`.

    Keys: x [T,d], w_router [E,d], bias [E] fp32 or None, w_gate/w_up [E,f,d], w_down [E,d,f].
    Tensor i of layer l uses seed  1000*seed + 10*l + i.
    """
    dt = cfg.torch_dtype
    T = cfg.T if T is None else T
    base = 1000 * int(seed) + 10 * int(layer)
    big = 65536
    out = {
        "x": _normal((T, cfg.d_model), cfg.x_std, dt, device, base + 0),
        "w_router": _normal((cfg.E, cfg.d_model), cfg.router_std, dt, device, base + 1),
        "w_gate": _normal((cfg.E, cfg.d_ff, cfg.d_model), cfg.w_std, dt, device, base + 2, big),
        "w_up": _normal((cfg.E, cfg.d_ff, cfg.d_model), cfg.w_std, dt, device, base + 3, big),
        "w_down": _normal((cfg.E, cfg.d_model, cfg.d_ff), cfg.w_std, dt, device, base + 4, big),
        "bias": None,
    }
    if cfg.zipf > 0:
        g = _gen("cpu", base + 5)
        rank = torch.randperm(cfg.E, generator=g).to(torch.float32) + 1.0
        out["bias"] = (-cfg.zipf * torch.log(rank)).to(torch.float32).to(device)
    return out


def make_stack(cfg: MoEConfig, device="cpu", seed=0, n_layers=None):
    """Per-layer tensors of the multi-layer configuration (gain = 1 + small noise, bf16/f32)."""
    n_layers = cfg.n_layers if n_layers is None else n_layers
    layers = []
    for l in range(n_layers):
        L = make_layer(cfg, device, seed, layer=l + 1, T=1)
        del L["x"]
        g = _gen("cpu", 1000 * int(seed) + 10 * (l + 1) + 6)
        L["gain"] = (1.0 + 0.05 * torch.randn(cfg.d_model, generator=g)).to(cfg.torch_dtype).to(device)
        layers.append(L)
    x = _normal((cfg.T, cfg.d_model), 1.0, cfg.torch_dtype, device, 1000 * int(seed) + 7)
    return x, layers


def make_tokens(cfg: MoEConfig, seed=0, B=None, gamma=None):
    """Draft ids [B,gamma] and target ids [B,gamma+1], int32, on the CPU.

    match_prob < 0: both uniform in [0, vocab).  Otherwise target[b,i] repeats draft[b,i]
    with probability match_prob independently per position and is a different id else;
    target[b,gamma] is uniform.
    """
    B = cfg.B if B is None else B
    gamma = cfg.gamma if gamma is None else gamma
    rng = np.random.default_rng(7919 * int(seed) + 13)
    draft = rng.integers(0, cfg.vocab, size=(B, gamma), dtype=np.int64)
    target = rng.integers(0, cfg.vocab, size=(B, gamma + 1), dtype=np.int64)
    if cfg.match_prob >= 0:
        keep = rng.random(size=(B, gamma)) < cfg.match_prob
        other = (draft + 1 + rng.integers(0, cfg.vocab - 1, size=(B, gamma))) % cfg.vocab
        target[:, :gamma] = np.where(keep, draft, other)
    return (torch.from_numpy(draft.astype(np.int32)), torch.from_numpy(target.astype(np.int32)))


def forced_accept_cases(gamma, vocab=1000):
    """One sequence per possible first-mismatch position 0..gamma (gamma = all match)."""
    draft = np.arange(gamma, dtype=np.int32)[None, :].repeat(gamma + 1, axis=0) % vocab
    target = np.concatenate([draft, np.full((gamma + 1, 1), vocab - 1, np.int32)], axis=1)
    for b in range(gamma):
        target[b, b] = (target[b, b] + 1) % vocab      # first mismatch at position b
        target[b, b + 1:gamma] = draft[b, b + 1:]        # later positions match again
    return torch.from_numpy(draft.copy()), torch.from_numpy(target.astype(np.int32))


def to_f64(t: torch.Tensor) -> np.ndarray:
    """Exact widening of an fp32/bf16 tensor to a numpy fp64 array on the host."""
    return t.detach().to("cpu").to(torch.float64).numpy()
