"""Seeded synthetic inputs shaped like the paper's workloads.

This module draws random numbers and lays them out; it contains none of the
method's arithmetic (no norms, projections, softmax, salience, selection).
Both the HIP path and the CPU checker are handed the tensors made here.

Shapes follow Sec. 5.1 / App. C of the paper: a LLaMA-2-7B-shaped backbone,
256 image tokens (16x16 patches) + 256 point tokens per view, language tokens
last.  Real observations are replaced by Gaussian hidden states with a
per-modality mean offset; the heavy tail of real attention maps is imitated by
a log-normal additive bias on the scoring logits of a random 10% of the visual
tokens.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, List, Optional, Tuple

import torch


@dataclass(frozen=True)
class Workload:
    name: str
    L: int            # decoder layers
    D: int            # hidden size
    H: int            # heads
    dh: int           # head dim
    F: int            # MLP width
    n2: int           # 2D (image) tokens
    n3: int           # 3D (point) tokens
    nt: int           # language tokens
    keep_permille: int
    B: int
    p: int            # layers run on the full sequence before pruning
    seed: int
    offsets: bool     # per-modality mean offset on the hidden states
    heavy_tail: bool  # log-normal scoring-logit bias on 10% of visual tokens
    steps: int = 1    # consecutive action-iteration timesteps
    beta_mass: bool = False  # per-sample 2D:3D mass drawn from Beta(2,2)
    rms_eps: float = 1e-5
    rope_base: float = 10000.0

    @property
    def n_vis(self) -> int:
        return self.n2 + self.n3

    @property
    def S(self) -> int:
        return self.n2 + self.n3 + self.nt

    @property
    def k_total(self) -> int:
        # round-half-up(keep * n_vis), in integers
        return (self.keep_permille * self.n_vis + 500) // 1000

    @property
    def S_kept(self) -> int:
        return self.k_total + self.nt


_7B = dict(D=4096, H=32, dh=128, F=11008)

WORKLOADS: Dict[str, Workload] = {
    "tiny": Workload("tiny", L=1, D=256, H=4, dh=64, F=1024, n2=64, n3=64,
                     nt=16, keep_permille=500, B=1, p=0, seed=0,
                     offsets=False, heavy_tail=False),
    "single_view": Workload("single_view", L=4, **_7B, n2=256, n3=256, nt=32,
                            keep_permille=400, B=1, p=2, seed=1,
                            offsets=True, heavy_tail=True),
    "multi_view": Workload("multi_view", L=32, **_7B, n2=768, n3=1024, nt=48,
                           keep_permille=300, B=8, p=2, seed=2,
                           offsets=True, heavy_tail=True),
    "action_iter": Workload("action_iter", L=4, **_7B, n2=256, n3=256, nt=32,
                            keep_permille=400, B=4, p=2, seed=3,
                            offsets=True, heavy_tail=True, steps=16),
    "ratio_sweep": Workload("ratio_sweep", L=32, **_7B, n2=512, n3=2048, nt=64,
                            keep_permille=500, B=16, p=2, seed=4,
                            offsets=True, heavy_tail=True, beta_mass=True),
}
RATIO_SWEEP_PERMILLE = (1000, 700, 500, 300, 150)


def with_keep(w: Workload, keep_permille: int) -> Workload:
    return replace(w, keep_permille=keep_permille)


def _gen(seed: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def layer_weights(w: Workload, layer: int, device="cpu") -> Dict[str, torch.Tensor]:
    """bf16 weights of one decoder layer, ~N(0, 0.02); RMSNorm gains
    1 + N(0, 0.02).  Matrices are [out_features, in_features]."""
    g = _gen(w.seed * 1000003 + 7919 * (layer + 1), device)

    def mat(o, i):
        return (torch.randn(o, i, generator=g, device=device, dtype=torch.float32)
                * 0.02).to(torch.bfloat16)

    def gain(n):
        return (1.0 + 0.02 * torch.randn(n, generator=g, device=device,
                                         dtype=torch.float32)).to(torch.bfloat16)

    return dict(wq=mat(w.D, w.D), wk=mat(w.D, w.D), wv=mat(w.D, w.D),
                wo=mat(w.D, w.D), w_gate=mat(w.F, w.D), w_up=mat(w.F, w.D),
                w_down=mat(w.D, w.F), g_attn=gain(w.D), g_mlp=gain(w.D))


def modal_offsets(w: Workload, device="cpu") -> torch.Tensor:
    """Per-modality mean vectors [2, D] fp32 ~ N(0, 0.5^2) (zeros if unused)."""
    if not w.offsets:
        return torch.zeros(2, w.D, dtype=torch.float32, device=device)
    g = _gen(w.seed * 5 + 3, "cpu")
    return (0.5 * torch.randn(2, w.D, generator=g, dtype=torch.float32)).to(device)


def hidden_states(w: Workload, device="cpu", B: Optional[int] = None
                  ) -> Tuple[torch.Tensor, torch.Tensor]:
    """x [B,S,D] bf16 ~ N(0,1) (+ per-modality offset), pos [B,S] int32 = 0..S-1."""
    B = w.B if B is None else B
    g = _gen(w.seed * 7 + 11, device)
    x = torch.randn(B, w.S, w.D, generator=g, device=device, dtype=torch.float32)
    mu = modal_offsets(w, device)
    x[:, :w.n2] += mu[0]
    x[:, w.n2:w.n_vis] += mu[1]
    pos = torch.arange(w.S, dtype=torch.int32, device=device).repeat(B, 1)
    return x.to(torch.bfloat16), pos.contiguous()


def scoring_bias(w: Workload, device="cpu", B: Optional[int] = None,
                 step: int = 0) -> Optional[torch.Tensor]:
    """Additive bias on the scoring logits, [B,S] fp32, or None.

    exp(z), z ~ N(0,1), on a random 10% of the visual tokens; with
    ``beta_mass`` every 2D key additionally gets log(rho/(1-rho)) with
    rho ~ Beta(2,2) per sample, which moves attention mass between modalities.
    """
    if not (w.heavy_tail or w.beta_mass):
        return None
    B = w.B if B is None else B
    g = _gen(w.seed * 13 + 101 + 977 * step, "cpu")
    bias = torch.zeros(B, w.S, dtype=torch.float32)
    n_hot = w.n_vis // 10
    for b in range(B):
        if w.heavy_tail:
            hot = torch.randperm(w.n_vis, generator=g)[:n_hot]
            bias[b, hot] = torch.exp(torch.randn(n_hot, generator=g))
        if w.beta_mass:
            # Beta(2,2) from two seeded Gamma(2) draws built out of uniforms
            u = torch.rand(4, generator=g).clamp_min(1e-12)
            ga = -(torch.log(u[0]) + torch.log(u[1]))
            gb = -(torch.log(u[2]) + torch.log(u[3]))
            rho = (ga / (ga + gb)).clamp(0.02, 0.98)
            bias[b, :w.n2] += torch.log(rho / (1 - rho))
    return bias.to(device)


def synthetic_salience(w: Workload, device="cpu", B: Optional[int] = None,
                       levels: int = 0) -> torch.Tensor:
    """Stand-alone salience-like scores [B, n_vis] fp32 for the selection
    benchmarks and tie tests: log-normal(sigma=1) per token; ``levels`` > 0
    quantises them to that many distinct values to force ties."""
    B = w.B if B is None else B
    g = _gen(w.seed * 17 + 5, device)
    s = torch.exp(torch.randn(B, w.n_vis, generator=g, device=device,
                              dtype=torch.float32))
    if levels > 0:
        q = torch.clamp((s * levels / 4.0).floor(), 0, levels - 1)
        s = (q + 1.0) / levels
    return s.contiguous()


def synthetic_probs(w: Workload, device="cpu", B: Optional[int] = None
                    ) -> torch.Tensor:
    """Row-stochastic stand-in for the language-query attention [B,H,nt,S]
    fp32 (rows sum to 1, causal support), for the salience-kernel tests."""
    B = w.B if B is None else B
    g = _gen(w.seed * 19 + 3, device)
    e = torch.rand(B, w.H, w.nt, w.S, generator=g, device=device,
                   dtype=torch.float32) ** 4
    q = torch.arange(w.nt, device=device)[:, None] + w.n_vis
    j = torch.arange(w.S, device=device)[None, :]
    e = e * (j <= q)
    return (e / e.sum(-1, keepdim=True)).contiguous()


def next_timestep(w: Workload, x_prev: torch.Tensor, step: int) -> torch.Tensor:
    """Action-iteration drift: previous visual tokens + N(0, 0.05), then 10%
    of the visual tokens resampled fresh; language tokens unchanged."""
    device = x_prev.device
    g = _gen(w.seed * 23 + 31 * step + 1, device)
    B = x_prev.shape[0]
    x = x_prev.to(torch.float32).clone()
    x[:, :w.n_vis] += 0.05 * torch.randn(B, w.n_vis, w.D, generator=g,
                                         device=device, dtype=torch.float32)
    gc = _gen(w.seed * 29 + 37 * step + 2, "cpu")
    n_new = w.n_vis // 10
    mu = modal_offsets(w, device)
    for b in range(B):
        idx = torch.randperm(w.n_vis, generator=gc)[:n_new].to(device)
        fresh = torch.randn(n_new, w.D, generator=g, device=device,
                            dtype=torch.float32)
        x[b, idx] = fresh + mu[(idx >= w.n2).long()]
    return x.to(torch.bfloat16)


def _beta(a: int, b: int, shape, g: torch.Generator) -> torch.Tensor:
    """Beta(a, b) for integer a, b from sums of seeded exponentials."""
    ea = -torch.log(torch.rand(a, *shape, generator=g).clamp_min(1e-12)).sum(0)
    eb = -torch.log(torch.rand(b, *shape, generator=g).clamp_min(1e-12)).sum(0)
    return ea / (ea + eb)


def uniform_draws(w: Workload, device="cpu", B: Optional[int] = None,
                  step: int = 0) -> torch.Tensor:
    """The random numbers the background rule of the mask generation consumes:
    one uniform in [0, 1) per patch, [B, n2] fp32."""
    B = w.B if B is None else B
    g = _gen(w.seed * 41 + 613 * step + 7, "cpu")
    return torch.rand(B, w.n2, generator=g, dtype=torch.float32).to(device)


def weaken_3d(w: Workload, x: torch.Tensor) -> torch.Tensor:
    """Scale every 3D token by a per-patch log-normal factor (median 0.12,
    sigma 0.6), so that the 3D share of a patch's feature norm spreads around
    the ~10 % the paper's Table 1 shows instead of the 50 % of i.i.d. tokens."""
    g = _gen(w.seed * 43 + 19, "cpu")
    f = 0.12 * torch.exp(0.6 * torch.randn(x.shape[0], w.n3, 1, generator=g))
    y = x.to(torch.float32).clone()
    y[:, w.n2:w.n_vis] *= f.to(x.device)
    return y.to(torch.bfloat16)


def synthetic_indicators(w: Workload, device="cpu", B: Optional[int] = None,
                         n_patch: Optional[int] = None, seed: int = 0) -> torch.Tensor:
    """Stand-alone smoothed indicators [4, B, P] fp32 in the order
    (M2D^S1, M3D^S1, M2D^S2, M3D^S2) for the mask-kernel tests: 3D feature
    share ~ Beta(2,12) (mean 0.14), 2D attention share ~ Beta(4,3), orthogonal
    3D share = (1 - 2D share) * Beta(1,4)."""
    B = w.B if B is None else B
    P = w.n2 if n_patch is None else n_patch
    g = _gen(w.seed * 47 + 23 + 131 * seed, "cpu")
    m3_s1 = _beta(2, 12, (B, P), g)
    m2_s2 = _beta(4, 3, (B, P), g)
    m3_s2 = (1 - m2_s2) * _beta(1, 4, (B, P), g)
    return torch.stack([1 - m3_s1, m3_s1, m2_s2, m3_s2]).to(torch.float32).contiguous().to(device)
