"""Seeded synthetic inputs for one GPU's share of an MoE layer's training step.

This module only draws random tensors and shapes them like the paper's
workloads (model shapes of Table 1; skewed expert load as described in the
"Straggler Effects" paragraph of the background section).  It contains none of
the method's arithmetic: no gating, no permutation, no FFN.  Both the CPU
oracle's tests and the HIP path's tests/bench take their inputs from here, so
the two sides always see byte-identical arrays.

Routing inputs (logits), tokens X and the upstream gradient dY are always drawn
on the host, so the realised per-expert loads are the same on every machine.
Expert weights are drawn on the device they will live on (22.6 GB at the
DeepSeek-V3 shape); a CPU consumer receives a copy of those same bytes.
"""
from __future__ import annotations

import dataclasses
import math
from typing import Dict, Optional

import torch


@dataclasses.dataclass(frozen=True)
class MoEConfig:
    """Shape of one MoE layer and the recipe of its synthetic routing."""

    name: str
    T: int                 # tokens on this GPU
    d: int                 # hidden size
    E: int                 # routed experts
    k: int                 # experts per token
    d_ff: int              # routed expert width
    n_shared: int = 0      # always-on shared experts
    d_ff_shared: int = 0
    dtype: str = "bf16"    # "f32" or "bf16": X, weights, activations, Y, dW
    gate: str = "softmax"  # "softmax" or "sigmoid"
    renorm: bool = True    # weights normalised over the selected k
    routing: str = "zipf"  # "zipf" (bias log p_e) or "stress" (forced hot/zero experts)
    zipf_s: float = 0.0    # Zipf exponent; 0 = uniform load
    hot_frac: float = 0.30  # stress: share of tokens that select the hot expert
    n_zero: int = 10        # stress: experts that receive nothing
    seed: int = 0
    aux_alpha: float = 0.0  # weight of the auxiliary load-balancing loss (0: not computed)
    ffn: str = "swiglu"     # expert body: "swiglu" (Wg, Wu, Wd) or "gelu" (two matrices Wg = W^A, Wd = W^B)

    @property
    def A(self) -> int:
        return self.T * self.k

    @property
    def torch_dtype(self) -> torch.dtype:
        return torch.float32 if self.dtype == "f32" else torch.bfloat16

    def flops(self) -> Dict[str, float]:
        """Algorithmic FLOPs over real rows only: per row 6·d·F forward and 12·d·F backward with three
        matrices per expert, 4·d·F and 8·d·F with two."""
        routed = self.A * self.d * self.d_ff
        shared = self.n_shared * self.T * self.d * self.d_ff_shared
        m = 3.0 if self.ffn == "swiglu" else 2.0   # matrices per expert
        return {
            "fwd": 2.0 * m * (routed + shared),
            "bwd": 4.0 * m * (routed + shared),
            "total": 6.0 * m * (routed + shared),
            "routed_total": 6.0 * m * routed,
            "shared_total": 6.0 * m * shared,
        }


# every model of the paper's evaluation trains with an auxiliary load-balancing loss of this weight
AUX_ALPHA = 0.001

# The five layers BASELINE names.  Shapes d, d_ff, top-k follow Table 1 of the paper.
CONFIGS: Dict[str, MoEConfig] = {
    "tiny": MoEConfig("tiny", T=256, d=128, E=8, k=2, d_ff=256, dtype="f32", zipf_s=0.0, aux_alpha=AUX_ALPHA),
    "qwen": MoEConfig("qwen", T=4096, d=2048, E=60, k=4, d_ff=1408, n_shared=4,
                      d_ff_shared=1408, zipf_s=1.0, aux_alpha=AUX_ALPHA),
    "phi": MoEConfig("phi", T=8192, d=4096, E=16, k=2, d_ff=6400, zipf_s=0.8, aux_alpha=AUX_ALPHA),
    "dsv3": MoEConfig("dsv3", T=8192, d=7168, E=256, k=8, d_ff=2048, n_shared=1,
                      d_ff_shared=2048, gate="sigmoid", zipf_s=1.2, aux_alpha=AUX_ALPHA),
    "stress": MoEConfig("stress", T=16384, d=2048, E=60, k=4, d_ff=1408, routing="stress",
                        zipf_s=1.5, aux_alpha=AUX_ALPHA),
}

# The paper's synthetic models (Table 1): GPT-3 sparsified, two matrices per expert, d_ffn = 4 d_model,
# top-2, 2 experts per GPU on 32 GPUs = 64 experts; T = four sequences of 2048 tokens on this GPU.
# The load skew is not given for them: the exponent of the Qwen-shaped workload is reused.
CONFIGS.update({
    "gpt-s": MoEConfig("gpt-s", T=8192, d=768, E=64, k=2, d_ff=3072, ffn="gelu", zipf_s=1.0, aux_alpha=AUX_ALPHA),
    "gpt-l": MoEConfig("gpt-l", T=8192, d=1536, E=64, k=2, d_ff=6144, ffn="gelu", zipf_s=1.0, aux_alpha=AUX_ALPHA),
})

# The paper's top-k sweep (sensitivity study of Section 5.4: Qwen1.5-MoE with k = 2 ... 5); k = 4 is "qwen" itself.
CONFIGS.update({"qwen-k%d" % k: dataclasses.replace(CONFIGS["qwen"], name="qwen-k%d" % k, k=k) for k in (2, 3, 5)})

WEIGHT_STD = 0.02
TOKEN_STD = 0.02
GRAD_STD = 0.02

# one independent random stream per tensor
_STREAM = {"logits": 1, "order": 2, "hot_tokens": 3, "X": 4, "dY": 5,
           "Wg": 10, "Wu": 11, "Wd": 12, "Wsg": 13, "Wsu": 14, "Wsd": 15}


def _gen(cfg: MoEConfig, what: str, device: str = "cpu") -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed((cfg.seed << 20) + 7919 * _STREAM[what] + 1)
    return g


def scaled(cfg: MoEConfig, **kw) -> MoEConfig:
    """A copy of cfg with some fields replaced (reduced sizes for CPU-checkable cases)."""
    return dataclasses.replace(cfg, **kw)


def expert_order(cfg: MoEConfig) -> torch.Tensor:
    """Seeded random ordering of experts: order[r] is the expert of popularity rank r (0 = most)."""
    return torch.randperm(cfg.E, generator=_gen(cfg, "order"))


def zipf_log_p(n: int, s: float) -> torch.Tensor:
    """log p_r for ranks r = 1..n with p_r proportional to r^-s."""
    r = torch.arange(1, n + 1, dtype=torch.float64)
    lp = -s * torch.log(r)
    return lp - torch.logsumexp(lp, 0)


def make_logits(cfg: MoEConfig) -> torch.Tensor:
    """Router logits [T, E] fp32 on the host: N(0,1) noise plus a per-expert popularity bias."""
    z = torch.randn(cfg.T, cfg.E, generator=_gen(cfg, "logits"), dtype=torch.float32)
    order = expert_order(cfg)
    if cfg.routing == "zipf":
        bias = torch.empty(cfg.E, dtype=torch.float64)
        bias[order] = zipf_log_p(cfg.E, cfg.zipf_s)
        return (z + bias.to(torch.float32)).contiguous()
    if cfg.routing != "stress":
        raise ValueError(f"unknown routing recipe {cfg.routing!r}")
    # stress: order[0] is the hot expert, order[1:1+n_zero] receive nothing,
    # the rest carry a Zipf(s) bias over their own ranks.
    hot = int(order[0])
    zero = order[1:1 + cfg.n_zero]
    rest = order[1 + cfg.n_zero:]
    if rest.numel() < cfg.k:
        raise ValueError("stress routing needs at least k experts outside the hot/zero sets")
    bias = torch.zeros(cfg.E, dtype=torch.float64)
    bias[rest] = zipf_log_p(rest.numel(), cfg.zipf_s)
    logits = z + bias.to(torch.float32)
    logits[:, zero] = -1.0e4
    n_hot = int(round(cfg.hot_frac * cfg.T))
    chosen = torch.randperm(cfg.T, generator=_gen(cfg, "hot_tokens"))[:n_hot]
    logits[:, hot] = -1.0e4
    # k other experts would all have to draw N(0,1)+log p above this for the hot expert to be
    # left out; the tests assert the realised count
    logits[chosen, hot] = 4.0
    return logits.contiguous()


def stress_sets(cfg: MoEConfig):
    """(hot expert, zero-load experts, number of tokens that select the hot expert)."""
    order = expert_order(cfg)
    return int(order[0]), [int(e) for e in order[1:1 + cfg.n_zero]], int(round(cfg.hot_frac * cfg.T))


def _normal(shape, std, gen, device, dtype) -> torch.Tensor:
    x = torch.randn(*shape, generator=gen, device=device, dtype=torch.float32)
    x.mul_(std)
    return x.to(dtype)


def make_tokens(cfg: MoEConfig, std: float = TOKEN_STD) -> torch.Tensor:
    """X [T, d] in the config dtype, on the host."""
    return _normal((cfg.T, cfg.d), std, _gen(cfg, "X"), "cpu", cfg.torch_dtype)


def make_grad_out(cfg: MoEConfig, std: float = GRAD_STD) -> torch.Tensor:
    """Upstream gradient dY [T, d] in the config dtype, on the host."""
    return _normal((cfg.T, cfg.d), std, _gen(cfg, "dY"), "cpu", cfg.torch_dtype)


def make_weights(cfg: MoEConfig, device: str = "cpu", std: Optional[float] = None) -> Dict[str, torch.Tensor]:
    """Expert weights in the config dtype on `device`.

    Wg, Wu: [E, d, d_ff];  Wd: [E, d_ff, d];  shared experts (if any)
    Wsg, Wsu: [S, d, d_ff_shared];  Wsd: [S, d_ff_shared, d].  Row-major.
    Drawn expert by expert so the fp32 staging buffer stays one expert large.
    """
    std = WEIGHT_STD if std is None else std
    dev_type = torch.device(device).type
    out: Dict[str, torch.Tensor] = {}

    def fill(name: str, n: int, rows: int, cols: int):
        w = torch.empty(n, rows, cols, device=device, dtype=cfg.torch_dtype)
        g = _gen(cfg, name, dev_type)
        for e in range(n):
            w[e].copy_(_normal((rows, cols), std, g, device, cfg.torch_dtype))
        out[name] = w

    gated = cfg.ffn == "swiglu"
    fill("Wg", cfg.E, cfg.d, cfg.d_ff)
    if gated:
        fill("Wu", cfg.E, cfg.d, cfg.d_ff)
    fill("Wd", cfg.E, cfg.d_ff, cfg.d)
    if cfg.n_shared:
        fill("Wsg", cfg.n_shared, cfg.d, cfg.d_ff_shared)
        if gated:
            fill("Wsu", cfg.n_shared, cfg.d, cfg.d_ff_shared)
        fill("Wsd", cfg.n_shared, cfg.d_ff_shared, cfg.d)
    return out


def unit_scale_stds(cfg: MoEConfig):
    """(token std, weight std) that make the expert pre-activations O(1).

    At the paper-like N(0, 0.02^2) scale SiLU works in its near-linear range; parity
    cases also run at this scale so that the nonlinearity and its derivative matter.
    """
    return 1.0, 1.0 / math.sqrt(cfg.d)
