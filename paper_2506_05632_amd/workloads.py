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


def _zipf_logits(B, V, noise_sigma, g, device, alpha=1.1):
    """-alpha ln(rank) + N(0, sigma^2), ranks a fresh random permutation of 1..V per row."""
    out = torch.empty(B, V, dtype=torch.float32, device=device)
    step = max(1, min(B, (1 << 25) // V))
    for b0 in range(0, B, step):
        n = min(step, B - b0)
        ranks = torch.rand(n, V, generator=g, device=device).argsort(dim=1).argsort(dim=1) + 1
        out[b0:b0 + n] = -alpha * torch.log(ranks.to(torch.float32))
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
        # (in the paper's parametrisation W / rho = A + eta: var of W/rho given A is (1 - rho^2) / rho^2)
        return Workload("is_n65536_l4_f32", 5, B, K, V, torch.float32, "logw", dec, enc,
                        1.0, 1.0, seed, shared_draft=False,
                        extra={"x": x, "y": y, "u": u, "rho": rho, "var_t_given_a": s2,
                               "var_w_given_a": (1.0 - rho * rho) / (rho * rho)})
    raise ValueError(f"unknown config {cfg}")


@dataclass
class VerifyWorkload:
    name: str
    S: int
    L: int
    K: int
    V: int
    dtype: torch.dtype
    kind: str
    target: torch.Tensor           # [S, L+1, K, V]
    tokens: torch.Tensor           # [S, L, K] int32
    temp_target: float = 1.0
    seed: int = 0
    row_offset: int = 0

    @property
    def elems(self) -> int:
        return self.S * (self.L + 1) * self.K * self.V


VERIFY_SHAPES = {
    # name: S sequences, L draft tokens, K drafts, V vocabulary
    "tiny": dict(S=24, L=3, K=4, V=1000, dtype=torch.float32, temp=1.0),
    "small_bf16": dict(S=12, L=4, K=6, V=32000, dtype=torch.bfloat16, temp=1.0),
    "largevocab": dict(S=128, L=7, K=8, V=128256, dtype=torch.float32, temp=0.7),
}


def make_verify(name: str, device="cpu", sequences: Optional[int] = None) -> VerifyWorkload:
    """Inputs of Algorithm 2's verification loop, shaped like a batched target-model pass over
    K drafts of L tokens (Section 4.2): target[s, j, k, :] are Zipf-like logits (rank exponent
    1.8: a peaked next-token law, so that blocks of several tokens occur); drafts of one
    sequence whose first j tokens coincide see the same row at position j (the target model is
    conditioned on the same prefix), so all K rows coincide at j = 0.  Draft tokens are the
    row's most likely token with probability 0.85 and a uniform token otherwise, so that some
    drafts stay viable for several positions.  The draw uses no sampler arithmetic."""
    shp = VERIFY_SHAPES[name]
    S = sequences if sequences is not None else shp["S"]
    L, K, V = shp["L"], shp["K"], shp["V"]
    device = torch.device(device)
    g = torch.Generator(device=device)
    g.manual_seed(INPUT_SEED_BASE + 100 + sorted(VERIFY_SHAPES).index(name))
    target = torch.empty(S, L + 1, K, V, dtype=shp["dtype"], device=device)
    for j in range(L + 1):
        for k in range(K):
            target[:, j, k, :] = _zipf_logits(S, V, 0.5, g, device, alpha=1.8).to(shp["dtype"])
    tokens = torch.empty(S, L, K, dtype=torch.int32, device=device)
    same_prefix = torch.ones(S, K, K, dtype=torch.bool, device=device)  # [s, k, k']: prefixes equal so far
    first = torch.arange(K, device=device)
    for j in range(L + 1):
        # the first draft with the same prefix supplies the row
        cand = torch.where(same_prefix, first.view(1, 1, K), K)
        src = cand.min(dim=2).values                                    # [S, K], src <= k
        for k in range(1, K):
            rows = torch.nonzero(src[:, k] != k).flatten()
            if rows.numel():
                target[rows, j, k, :] = target[rows, j, src[rows, k], :]
        if j == L:
            break
        top = target[:, j].float().argmax(dim=2).to(torch.int32)        # [S, K]
        rnd = torch.randint(0, V, (S, K), generator=g, device=device, dtype=torch.int32)
        pick = torch.rand(S, K, generator=g, device=device) < 0.85
        # drafts that share a prefix and a coin keep sharing; others diverge
        tokens[:, j] = torch.where(pick, top, rnd)
        same_prefix &= tokens[:, j].view(S, K, 1) == tokens[:, j].view(S, 1, K)
    return VerifyWorkload(f"verify_{name}_s{S}_l{L}_k{K}_v{V}", S, L, K, V, shp["dtype"], "logits",
                          target, tokens, shp["temp"], SAMPLER_SEED_BASE + 64, 0)


@dataclass
class TopmWorkload:
    name: str
    B: int
    K: int
    M: int
    V: int
    dtype: torch.dtype
    draft_ids: torch.Tensor        # [B,M] int32 (one list per row) or [B,K,M]
    draft_val: torch.Tensor
    target_ids: torch.Tensor       # [B,M] int32
    target_val: torch.Tensor
    temp_target: float = 1.0
    temp_draft: float = 1.0
    seed: int = 0

    @property
    def elems(self) -> int:
        return self.B * self.K * self.M


TOPM_SHAPES = {
    # the paper's deployment setting keeps the 50 most likely tokens of each model (Appendix D.1)
    "top50": dict(B=1024, V=128256, K=8, M=50, dtype=torch.float32, distinct=False),
    "top50_distinct_bf16": dict(B=256, V=32000, K=4, M=50, dtype=torch.bfloat16, distinct=True),
    "top256": dict(B=64, V=32000, K=5, M=256, dtype=torch.float32, distinct=True),
}


def make_topm(name: str, device="cpu", rows: Optional[int] = None) -> TopmWorkload:
    """Candidate lists: the M largest logits of Zipf-like target and draft rows (draft = target +
    N(0, 0.5^2) per entry), with their token ids, in descending order of the logit."""
    shp = TOPM_SHAPES[name]
    B = rows if rows is not None else shp["B"]
    V, K, M = shp["V"], shp["K"], shp["M"]
    device = torch.device(device)
    g = torch.Generator(device=device)
    g.manual_seed(INPUT_SEED_BASE + 200 + sorted(TOPM_SHAPES).index(name))
    tq = _zipf_logits(B, V, 0.5, g, device)
    t_val, t_ids = tq.topk(M, dim=1)
    if shp["distinct"]:
        d_val = torch.empty(B, K, M, dtype=torch.float32, device=device)
        d_ids = torch.empty(B, K, M, dtype=torch.int64, device=device)
        for k in range(K):
            td = tq + 0.5 * torch.randn(B, V, generator=g, device=device)
            d_val[:, k], d_ids[:, k] = td.topk(M, dim=1)
    else:
        td = tq + 0.5 * torch.randn(B, V, generator=g, device=device)
        d_val, d_ids = td.topk(M, dim=1)
    dt = shp["dtype"]
    return TopmWorkload(f"topm_{name}_b{B}_k{K}_m{M}", B, K, M, V, dt,
                        d_ids.to(torch.int32).contiguous(), d_val.to(dt).contiguous(),
                        t_ids.to(torch.int32).contiguous(), t_val.to(dt).contiguous(),
                        1.0, 1.0, SAMPLER_SEED_BASE + 80)


@dataclass
class GaussianSource:
    """Inputs of the compression scheme on the synthetic Gaussian source (Section 5.3, Appendix D.2)."""
    name: str
    B: int                         # trials
    K: int                         # decoders
    N: int                         # prior samples
    l_max: int
    var_w_given_a: float
    var_t_given_a: float
    a: torch.Tensor                # [B] source samples A ~ N(0, 1)
    t: torch.Tensor                # [B,K] side information T_k = A + N(0, var_t_given_a)
    u: torch.Tensor                # [B,N] candidates U_i ~ p_W = N(0, 1 + var_w_given_a)
    bins: torch.Tensor             # [B,N] uint8, uniform on 0..l_max-1
    logw_enc: torch.Tensor         # [B,N]   ln p_{W|A}(U_i|a) - ln p_W(U_i)
    logw_dec: torch.Tensor         # [B,K,N] ln p_{W|T}(U_i|t_k) - ln p_W(U_i)
    seed: int = 0


def make_gaussian_source(trials: int, K: int, l_max: int, var_w_given_a: float, device="cpu", *,
                         N: int = 1 << 15, var_t_given_a: float = 0.5, input_seed: int = 0) -> GaussianSource:
    """The synthetic Gaussian source of Appendix D.2 with the appendix's own parametrisation:
    W = A + eta, T_k = A + zeta_k; p_{W|T}(.|t) = N(t / var T, var W - 1 / var T).  Only inputs are
    drawn and the log-weights formed (the importance weights of Appendix C are the caller's); the
    selection, the decoders' outputs and the distortion are the library's."""
    device = torch.device(device)
    g = torch.Generator(device=device)
    g.manual_seed(INPUT_SEED_BASE + 300 + input_seed)
    s_e, s_z = float(var_w_given_a), float(var_t_given_a)
    var_w, var_t = 1.0 + s_e, 1.0 + s_z
    var_wt = var_w - 1.0 / var_t
    a = torch.randn(trials, generator=g, device=device)
    t = a[:, None] + math.sqrt(s_z) * torch.randn(trials, K, generator=g, device=device)
    u = math.sqrt(var_w) * torch.randn(trials, N, generator=g, device=device)
    bins = torch.randint(0, l_max, (trials, N), generator=g, device=device, dtype=torch.uint8)

    def log_ratio(mean, var):
        # ln N(u; mean, var) - ln N(u; 0, var_w), in fp64, rounded once to fp32
        u64 = u.double()
        return (-0.5 * math.log(var / var_w) - 0.5 * (u64 - mean) ** 2 / var + 0.5 * u64 ** 2 / var_w).float()

    enc = log_ratio(a.double()[:, None], s_e)
    dec = torch.empty(trials, K, N, dtype=torch.float32, device=device)
    for k in range(K):
        dec[:, k] = log_ratio(t.double()[:, k:k + 1] / var_t, var_wt)
    return GaussianSource(f"gaussian_source_k{K}_lmax{l_max}_n{N}", trials, K, N, l_max, s_e, s_z,
                          a, t, u, bins, enc, dec, SAMPLER_SEED_BASE + 96)
