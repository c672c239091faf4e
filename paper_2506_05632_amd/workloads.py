"""Seeded synthetic inputs shaped like the paper's workloads.

This module only draws inputs (logits, log-weights); it holds none of the
sampler's arithmetic and is the one module that both the tests' CPU side and
the GPU side use.  Tensors are generated with torch on the requested device
from a fixed per-config seed, so a given (config, device type) always yields
the same bits; tests copy the rows they check to the host and feed the same
bits to both implementations.

The five configurations stand in for the paper's measured workloads (LLM
next-token distributions over vocabularies of 32 000 / 128 256 / 152 064
entries with K = 4..16 drafts, Section 4.3 and Appendix D.1; the Gaussian
source with N = 2^15 prior samples and up to four decoders, Section 5 and
Appendix D.2).  No dataset or model output is reproduced: logits follow a
Zipf-like rank profile with Gaussian noise.
"""
import math
from dataclasses import dataclass, field
from typing import Optional

import torch

SAMPLER_SEED_BASE = 0x5EED0000
INPUT_SEED_BASE = 1000


@dataclass
class Workload:
    name: str
    cfg: int
    B: int
    K: int
    V: int
    dtype: torch.dtype
    kind: str                      # "logits" or "logw"
    draft: torch.Tensor            # [B,V] (one proposal per row) or [B,K,V]
    target: torch.Tensor           # [B,V]
    temp_target: float = 1.0
    temp_draft: float = 1.0
    seed: int = 0
    row_offset: int = 0
    shared_draft: bool = True
    extra: dict = field(default_factory=dict)

    @property
    def elems(self) -> int:
        return self.B * self.K * self.V


SHAPES = {
    1: dict(B=64, V=1024, K=4),
    2: dict(B=256, V=32000, K=4),
    3: dict(B=1024, V=128256, K=8),
    4: dict(B=512, V=152064, K=16),
    5: dict(B=4096, V=65536, K=4),
}


def _gen(device, cfg):
    g = torch.Generator(device=device)
    g.manual_seed(INPUT_SEED_BASE + cfg)
    return g


def _zipf_logits(B, V, noise_sigma, g, device):
    """-1.1 ln(rank) + N(0, sigma^2), ranks a fresh random permutation of 1..V per row."""
    out = torch.empty(B, V, dtype=torch.float32, device=device)
    step = max(1, min(B, (1 << 25) // V))
    for b0 in range(0, B, step):
        n = min(step, B - b0)
        ranks = torch.rand(n, V, generator=g, device=device).argsort(dim=1).argsort(dim=1) + 1
        out[b0:b0 + n] = -1.1 * torch.log(ranks.to(torch.float32))
        out[b0:b0 + n] += noise_sigma * torch.randn(n, V, generator=g, device=device)
    return out


def make(cfg: int, device="cpu", rows: Optional[int] = None) -> Workload:
    """Build configuration `cfg` (1..5); `rows` overrides B (tests on the CPU use fewer rows)."""
    shp = SHAPES[cfg]
    B = rows if rows is not None else shp["B"]
    V, K = shp["V"], shp["K"]
    device = torch.device(device)
    g = _gen(device, cfg)
    seed = SAMPLER_SEED_BASE + cfg
    randn = lambda *s: torch.randn(*s, generator=g, device=device)

    if cfg == 1:
        tq = 2.0 * randn(B, V)
        td = tq + randn(B, V)
        return Workload("tiny", 1, B, K, V, torch.float32, "logits", td, tq, 1.0, 1.0, seed)
    if cfg == 2:
        tq = _zipf_logits(B, V, 0.5, g, device)
        td = tq + randn(B, V)
        return Workload("specdec_v32000_k4_bf16", 2, B, K, V, torch.bfloat16, "logits",
                        td.to(torch.bfloat16), tq.to(torch.bfloat16), 1.0, 1.0, seed)
    if cfg == 3:
        tq = _zipf_logits(B, V, 0.5, g, device)
        td = tq + 0.5 * randn(B, V)
        return Workload("largevocab_v128256_k8_f32", 3, B, K, V, torch.float32, "logits",
                        td, tq, 0.7, 0.7, seed)
    if cfg == 4:
        tq = _zipf_logits(B, V, 0.5, g, device)
        sigma = 0.3 + 1.2 * torch.rand(K, generator=g, device=device)
        td = torch.empty(B, K, V, dtype=torch.bfloat16, device=device)
        for k in range(K):
            td[:, k, :] = (tq + sigma[k] * randn(B, V)).to(torch.bfloat16)
        return Workload("distinct_v152064_k16_bf16", 4, B, K, V, torch.bfloat16, "logits",
                        td, tq.to(torch.bfloat16), 1.0, 1.0, seed, shared_draft=False,
                        extra={"sigma": sigma})
    if cfg == 5:
        # Gaussian source in standardised form: W | A = x ~ N(rho x, 1 - rho^2), W ~ N(0, 1),
        # side information y = x + N(0, s^2)  =>  W | y ~ N(rho y / (1 + s^2), 1 - rho^2 / (1 + s^2)).
        rho, s2 = 0.9, 0.25
        x = randn(B)
        u = randn(B, V)
        y = x[:, None] + math.sqrt(s2) * randn(B, K)

        def log_ratio(u_, mean, var):
            # log N(u; mean, var) - log N(u; 0, 1)
            return -0.5 * math.log(var) - 0.5 * (u_ - mean) ** 2 / var + 0.5 * u_ ** 2

        enc = log_ratio(u, rho * x[:, None], 1.0 - rho * rho)
        dec = torch.empty(B, K, V, dtype=torch.float32, device=device)
        var_d = 1.0 - rho * rho / (1.0 + s2)
        for l in range(K):
            dec[:, l, :] = log_ratio(u, rho * y[:, l:l + 1] / (1.0 + s2), var_d)
        return Workload("is_n65536_l4_f32", 5, B, K, V, torch.float32, "logw", dec, enc,
                        1.0, 1.0, seed, shared_draft=False,
                        extra={"x": x, "y": y, "u": u})
    raise ValueError(f"unknown config {cfg}")
