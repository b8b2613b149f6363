"""Seeded synthetic inputs for the VATP hot path (shared by tests, bench and smoke).

This module only draws random tensors with the shapes and structure of the paper's
workload; it contains none of the method's arithmetic (no softmax, no scores, no
selection).  Both the CPU oracle and the HIP path receive the tensors produced here,
already rounded to the storage dtype, so that they start from identical values.

Structure reproduced (paper, Fig. 1 and its discussion in the Observations section):
a few leading "attention sink" tokens that attract a large share of the attention while
their value vectors are close to zero, and value-vector l1 norms that vary strongly
from token to token everywhere else.  Shapes follow the 7B model the paper measures
(32 layers, 32 heads, head dimension 128; Inference Efficiency paragraph).

Recipe, per (batch, head) unit, with g* ~ N(0,1) i.i.d.:
  * queries       q_j = gQ_j + 4 u          (u: one random unit vector per head unit,
                                             shared by prompt and decode queries)
  * sink keys     k_s = (8 sqrt(d) / <qbar,qbar>) qbar, s < n_sinks, qbar = mean prompt
                  query, so the mean scaled logit of a sink key is +8
  * sink values   v_s = 0.01 gV_s
  * other values  v_i = gV_i * exp(sigma z_i), z_i ~ N(0,1)   (lognormal row scale)
  * other keys    k_i = gK_i
With grouped queries (q_per_kv = g > 1: g query heads per K/V head) every query head has its
own u, and qbar of a sink key is the mean over its group's query heads.
Everything is drawn in fp32 on the requested device from a torch.Generator seeded with
(seed, layer), then rounded once (round-to-nearest-even) to the storage dtype.
"""
from __future__ import annotations

import dataclasses
import math
from typing import Dict, List, Optional

import torch


@dataclasses.dataclass(frozen=True)
class VatpConfig:
    name: str
    batch: int
    layers: int
    n_heads: int
    head_dim: int
    prompt_len: int            # fixed prompt length (ignored when ragged is set)
    dtype: str                 # "fp32" | "bf16"
    n_sinks: int
    sigma: float
    budget_pct: int            # B = floor(L * pct / 100)
    recent: int                # R
    decode_steps: int          # T
    ragged: Optional[tuple] = None   # (lo, hi) inclusive prompt-length range
    q_per_kv: int = 1                # query heads per K/V head (n_heads counts K/V heads); > 1: grouped queries

    @property
    def n_sink_keep(self) -> int:
        """F, the forced-keep prefix: the number of sink tokens of the config."""
        return self.n_sinks

    def torch_dtype(self) -> torch.dtype:
        return torch.float32 if self.dtype == "fp32" else torch.bfloat16

    def prompt_lens(self, seed: int) -> List[int]:
        if self.ragged is None:
            return [self.prompt_len] * self.batch
        lo, hi = self.ragged
        g = torch.Generator(device="cpu")
        g.manual_seed(1_000_003 * seed + 17)
        u = torch.rand(self.batch, generator=g, dtype=torch.float64)
        return [int(lo + math.floor(float(x) * (hi - lo + 1))) for x in u]

    def budgets(self, lens: List[int]) -> List[int]:
        return [(L * self.budget_pct) // 100 for L in lens]


# The five workloads named by the baseline description.
CONFIGS: Dict[str, VatpConfig] = {
    "tiny": VatpConfig("tiny", 1, 1, 4, 64, 256, "fp32", 2, 0.5, 50, 16, 32),
    "llama7b_layer": VatpConfig("llama7b_layer", 1, 1, 32, 128, 4096, "bf16", 2, 0.5, 50, 64, 128),
    "llama7b_stack": VatpConfig("llama7b_stack", 8, 32, 32, 128, 4096, "bf16", 2, 0.5, 20, 64, 256),
    "long32k": VatpConfig("long32k", 1, 1, 32, 128, 32768, "bf16", 4, 1.0, 10, 128, 64),
    "ragged16": VatpConfig("ragged16", 16, 1, 32, 128, 0, "bf16", 2, 0.5, 30, 64, 128,
                           ragged=(1024, 8192)),
}


def scaled(cfg: VatpConfig, **kw) -> VatpConfig:
    """A copy of cfg with some fields replaced (used for reduced-size parity cases)."""
    return dataclasses.replace(cfg, **kw)


@dataclasses.dataclass
class VatpInputs:
    cfg: VatpConfig
    lens: List[int]            # prompt length per sequence
    budgets: List[int]         # B per sequence
    cap: int                   # rows allocated per (b, h) in Q/K/V
    Q: torch.Tensor            # [b, H * q_per_kv, cap, d]   prompt queries (rows >= len are zero)
    K: torch.Tensor            # [b, H, cap, d]
    V: torch.Tensor            # [b, H, cap, d]
    qd: torch.Tensor           # [T, b, H * q_per_kv, d]     decode-step queries
    kd: torch.Tensor           # [T, b, H, d]
    vd: torch.Tensor           # [T, b, H, d]


def make_inputs(cfg: VatpConfig, seed: int = 0, layer: int = 0,
                device: str | torch.device = "cpu", cap: Optional[int] = None) -> VatpInputs:
    """Draw one layer's worth of Q/K/V (prompt + decode rows) for `cfg`."""
    device = torch.device(device)
    g = torch.Generator(device=device)
    g.manual_seed(7_919 * seed + 104_729 * layer + 1)
    b, H, d, T = cfg.batch, cfg.n_heads, cfg.head_dim, cfg.decode_steps
    lens = cfg.prompt_lens(seed)
    Lmax = max(lens)
    cap = Lmax if cap is None else cap
    assert cap >= Lmax
    dt = cfg.torch_dtype()

    def randn(*shape):
        return torch.randn(*shape, generator=g, device=device, dtype=torch.float32)

    Hq = H * cfg.q_per_kv             # query heads: head h * q_per_kv + r attends to K/V head h
    u = randn(b, Hq, 1, d)
    u = u / u.norm(dim=-1, keepdim=True)

    Q = randn(b, Hq, cap, d)
    Q.add_(4.0 * u)
    qd = randn(T, b, Hq, d)
    qd.add_(4.0 * u.squeeze(2).unsqueeze(0))
    K = randn(b, H, cap, d)
    kd = randn(T, b, H, d)
    V = randn(b, H, cap, d)
    vscale = torch.exp(cfg.sigma * randn(b, H, cap, 1))
    vscale[:, :, :cfg.n_sinks, :] = 0.01
    V.mul_(vscale)
    vd = randn(T, b, H, d)
    vd.mul_(torch.exp(cfg.sigma * randn(T, b, H, 1)))

    lens_t = torch.tensor(lens, device=device).view(b, 1, 1, 1)
    row = torch.arange(cap, device=device).view(1, 1, cap, 1)
    valid = row < lens_t
    Q.mul_(valid)
    K.mul_(valid)
    V.mul_(valid)

    ns = cfg.n_sinks
    if ns > 0:
        qbar = Q.sum(dim=2, keepdim=True) / lens_t.to(torch.float32)        # [b,Hq,1,d]
        if cfg.q_per_kv > 1:                                                 # a sink key serves its whole group
            qbar = qbar.view(b, H, cfg.q_per_kv, 1, d).mean(dim=2)
        sink = (8.0 * math.sqrt(d)) * qbar / (qbar * qbar).sum(dim=-1, keepdim=True)
        K[:, :, :ns, :] = sink

    return VatpInputs(cfg, lens, cfg.budgets(lens), cap,
                      Q.to(dt), K.to(dt), V.to(dt), qd.to(dt), kd.to(dt), vd.to(dt))


def buffer_digests(inp: VatpInputs) -> Dict[str, str]:
    """SHA-256 of every generated buffer (the bytes of the storage dtype, as the oracle and the HIP path receive
    them), so that a run can state exactly which inputs it was measured or checked on."""
    import hashlib
    out = {}
    for name in ("Q", "K", "V", "qd", "kd", "vd"):
        t = getattr(inp, name).detach().contiguous().cpu()
        out[name] = hashlib.sha256(t.view(torch.uint8).numpy().tobytes()).hexdigest()
    return out
