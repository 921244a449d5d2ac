"""Seeded synthetic inputs shaped like the paper's workloads.

Holds data generation only (no entropy, budget, scoring or selection
arithmetic), so both the HIP path's tests and the CPU oracle's tests can draw
the same bits from it.

Recipe (stands in for Llama/Qwen key/value activations on long prompts, which
need weights and datasets that are not available): for every (layer, batch,
KV head) a rank r is drawn uniformly from the config's range, then
    K = s_l * (U V^T + 0.1 E),  U [N,r], V [D,r] ~ N(0,1)/sqrt(r), E ~ N(0,1)
with s_l a per-layer scale, values V_cache ~ N(0,1), and the observation-window
queries of each of the G query heads sharing a KV head built the same way with
the same V:  Q = U' V^T + 0.1 E'.  Tokens generated after the prompt (decode
steps) get keys and queries from the same V with fresh coefficients and noise.
Everything is generated in fp32 with torch's
generator for the chosen device (seed = seed0 + linear (layer,batch,head) index,
so a single head can be regenerated alone), then rounded once to the config's
dtype; every consumer reads those rounded bits.
"""
from __future__ import annotations

import dataclasses
import math

import torch


@dataclasses.dataclass(frozen=True)
class Config:
    name: str
    dtype: str          # "f32" | "bf16"
    L: int              # layers
    B: int              # batch
    H: int              # KV heads
    G: int              # query heads per KV head
    N: int              # sequence length
    D: int              # head_dim
    w: int              # observation window
    pool: int           # max-pool kernel
    k_trunc: int        # eigenvalue truncation rank
    avg_budget: int     # mean tokens kept per head
    rank_lo: int
    rank_hi: int
    layer_scale: bool   # per-layer key scale ~ U[0.5, 2]
    M: int = 8          # head groups

    @property
    def torch_dtype(self):
        return torch.float32 if self.dtype == "f32" else torch.bfloat16

    @property
    def step(self) -> int:
        """Budget step between consecutive head groups: avg_budget // 6 rounded
        down to even, so that n_max - (M-1)*step stays above the window."""
        s = self.avg_budget // 6
        return s - (s % 2)

    @property
    def n_max(self) -> int:
        """Largest group budget such that the M budgets average avg_budget."""
        return self.avg_budget + ((self.M - 1) * self.step) // 2

    @property
    def cap(self) -> int:
        return min(self.n_max, self.N)


CONFIGS = {
    0: Config("single-layer-fp32-1k", "f32", 1, 1, 8, 4, 1024, 128, 32, 7, 32, 128, 4, 64, False),
    1: Config("llama3-8b-8k", "bf16", 32, 1, 8, 4, 8192, 128, 32, 7, 32, 512, 4, 96, True),
    2: Config("llama3-8b-32k", "bf16", 32, 1, 8, 4, 32768, 128, 32, 7, 32, 1024, 4, 96, True),
    3: Config("llama3-8b-128k", "bf16", 32, 1, 8, 4, 131072, 128, 64, 7, 32, 2048, 4, 96, True),
    4: Config("llama3-70b-16k-b8", "bf16", 80, 8, 8, 8, 16384, 128, 32, 7, 32, 768, 4, 128, False),
}


def tiny_config(**kw) -> Config:
    """A small config for unit tests; any field can be overridden."""
    base = dict(name="tiny", dtype="f32", L=1, B=1, H=2, G=2, N=96, D=128, w=8, pool=7,
                k_trunc=32, avg_budget=24, rank_lo=2, rank_hi=16, layer_scale=False, M=2)
    base.update(kw)
    return Config(**base)


def layer_scales(cfg: Config, seed0: int) -> torch.Tensor:
    if not cfg.layer_scale:
        return torch.ones(cfg.L, dtype=torch.float32)
    g = torch.Generator(device="cpu").manual_seed(seed0 + 0x5CA1E)
    return 0.5 + 1.5 * torch.rand(cfg.L, generator=g, dtype=torch.float32)


def head_rank(cfg: Config, seed0: int, l: int, b: int, h: int) -> int:
    g = torch.Generator(device="cpu").manual_seed(seed0 + 7919 * (((l * cfg.B) + b) * cfg.H + h) + 13)
    return int(torch.randint(cfg.rank_lo, cfg.rank_hi + 1, (1,), generator=g).item())


def gen_head(cfg: Config, seed0: int, l: int, b: int, h: int, device="cpu", scale: float = 1.0):
    """One (layer, batch, KV head): returns K [N,D], V [N,D], Qwin [G,w,D] in the
    config's dtype on ``device``."""
    r = head_rank(cfg, seed0, l, b, h)
    g = torch.Generator(device=device).manual_seed(seed0 + (((l * cfg.B) + b) * cfg.H + h))
    f32 = dict(generator=g, device=device, dtype=torch.float32)
    inv = 1.0 / math.sqrt(r)
    U = torch.randn(cfg.N, r, **f32) * inv
    Vf = torch.randn(cfg.D, r, **f32) * inv
    E = torch.randn(cfg.N, cfg.D, **f32)
    K = scale * (U @ Vf.T + 0.1 * E)
    del U, E
    Vc = torch.randn(cfg.N, cfg.D, **f32)
    Uq = torch.randn(cfg.G, cfg.w, r, **f32) * inv
    Eq = torch.randn(cfg.G, cfg.w, cfg.D, **f32)
    Q = Uq @ Vf.T + 0.1 * Eq
    dt = cfg.torch_dtype
    return K.to(dt), Vc.to(dt), Q.to(dt)


def gen_decode_tokens(cfg: Config, seed0: int, l: int, b: int, h: int, T: int, device="cpu", scale: float = 1.0):
    """T generated tokens that follow gen_head's prompt for the same (layer, batch, KV
    head): keys k [T,D], values v [T,D] and queries q [T,G,D] drawn from the same factor
    matrix V as the prompt (re-drawn here from the head's seed), with their own noise."""
    r = head_rank(cfg, seed0, l, b, h)
    head = ((l * cfg.B) + b) * cfg.H + h
    g = torch.Generator(device=device).manual_seed(seed0 + head)
    f32 = dict(generator=g, device=device, dtype=torch.float32)
    inv = 1.0 / math.sqrt(r)
    torch.randn(cfg.N, r, **f32)                       # the prompt's U: drawn to reach V's place in the stream
    Vf = torch.randn(cfg.D, r, **f32) * inv
    g2 = torch.Generator(device=device).manual_seed(seed0 + 0xDEC0DE + 31 * head)
    f32 = dict(generator=g2, device=device, dtype=torch.float32)
    k = scale * ((torch.randn(T, r, **f32) * inv) @ Vf.T + 0.1 * torch.randn(T, cfg.D, **f32))
    v = torch.randn(T, cfg.D, **f32)
    q = (torch.randn(T, cfg.G, r, **f32) * inv) @ Vf.T + 0.1 * torch.randn(T, cfg.G, cfg.D, **f32)
    dt = cfg.torch_dtype
    return k.to(dt), v.to(dt), q.to(dt)


def gen_layers(cfg: Config, seed0: int, layers, device="cpu"):
    """K, V [len(layers), B, H, N, D] and Qwin [len(layers), B, H*G, w, D] for the
    listed layer indices."""
    layers = list(layers)
    dt = cfg.torch_dtype
    nl = len(layers)
    K = torch.empty(nl, cfg.B, cfg.H, cfg.N, cfg.D, dtype=dt, device=device)
    V = torch.empty_like(K)
    Q = torch.empty(nl, cfg.B, cfg.H * cfg.G, cfg.w, cfg.D, dtype=dt, device=device)
    scales = layer_scales(cfg, seed0)
    for i, l in enumerate(layers):
        for b in range(cfg.B):
            for h in range(cfg.H):
                k, v, q = gen_head(cfg, seed0, l, b, h, device=device, scale=float(scales[l]))
                K[i, b, h] = k
                V[i, b, h] = v
                Q[i, b, h * cfg.G:(h + 1) * cfg.G] = q
    return K, V, Q


def gen_all(cfg: Config, seed0: int, device="cpu"):
    return gen_layers(cfg, seed0, range(cfg.L), device=device)
