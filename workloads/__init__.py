"""Seeded synthetic inputs for the MoE-layer hot path.

This module only draws random tensors and lays them out; it holds none of the layer's
arithmetic, so both the CPU oracle's tests and the GPU library's callers can take their inputs
from it without sharing any code of the method.

The paper serves Qwen1.5-MoE-2.7B (60 routed + 4 shared experts per layer, Sec. 5 "Model
Selection") on BIG-Bench prompts from six concurrent tenants (Sec. 4.2).  Neither the weights nor
the prompts are available here, so random tensors with the layer's shapes stand in for them, and
router biases stand in for tenants that favour different expert subsets (Sec. 3).

Every tensor is drawn on the CPU from ``torch.Generator`` so the bytes are the same on every
machine; callers move them to the GPU.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional, Tuple

import torch


@dataclass(frozen=True)
class Shape:
    T: int           # tokens
    H: int           # hidden size
    E: int           # routed experts
    K: int           # experts per token
    I: int           # routed-expert intermediate size
    Is: int          # shared-expert intermediate size (0: none)
    renorm: bool     # divide the K gate weights by their sum

    @property
    def P(self) -> int:
        return self.T * self.K


QWEN = dict(H=2048, E=60, K=4, I=1408, Is=5632, renorm=False)


@dataclass
class Workload:
    name: str
    shape: Shape
    x: torch.Tensor                          # [T,H]
    Wr: torch.Tensor                         # [E,H]
    Wg: torch.Tensor                         # [E,I,H]
    Wu: torch.Tensor                         # [E,I,H]
    Wd: torch.Tensor                         # [E,H,I]
    bias: Optional[torch.Tensor] = None      # [E] fp32, or [n_tenants,E]
    Wsg: Optional[torch.Tensor] = None       # [Is,H]
    Wsu: Optional[torch.Tensor] = None       # [Is,H]
    Wsd: Optional[torch.Tensor] = None       # [H,Is]
    wgate: Optional[torch.Tensor] = None     # [H]
    tenant_rows: Optional[List[Tuple[int, int]]] = None   # token ranges per tenant
    meta: Dict[str, object] = field(default_factory=dict)

    def tensors(self) -> Dict[str, Optional[torch.Tensor]]:
        return dict(x=self.x, Wr=self.Wr, Wg=self.Wg, Wu=self.Wu, Wd=self.Wd, bias=self.bias,
                    Wsg=self.Wsg, Wsu=self.Wsu, Wsd=self.Wsd, wgate=self.wgate)

    def to_bf16(self) -> "Workload":
        """Same workload with every tensor except the fp32 router bias rounded once to bf16."""
        kw = {k: (v if v is None or k == "bias" else v.to(torch.bfloat16))
              for k, v in self.tensors().items()}
        return Workload(name=self.name, shape=self.shape, tenant_rows=self.tenant_rows,
                        meta=dict(self.meta), **kw)

    def to(self, device) -> "Workload":
        kw = {k: (None if v is None else v.to(device)) for k, v in self.tensors().items()}
        return Workload(name=self.name, shape=self.shape, tenant_rows=self.tenant_rows,
                        meta=dict(self.meta), **kw)

    def f32_numpy(self) -> Dict[str, object]:
        """Every tensor widened exactly to float32 numpy (what the oracle takes)."""
        return {k: (None if v is None else v.detach().cpu().float().numpy())
                for k, v in self.tensors().items()}


def _randn(g: torch.Generator, shape, std: float, dtype: torch.dtype) -> torch.Tensor:
    # drawn in fp32 one leading slice at a time so a 60-expert tensor never needs a 2 GB temporary
    dev = g.device
    if len(shape) == 3:
        out = torch.empty(shape, dtype=dtype, device=dev)
        for e in range(shape[0]):
            out[e] = (torch.randn(shape[1:], generator=g, dtype=torch.float32, device=dev) * std).to(dtype)
        return out
    return (torch.randn(shape, generator=g, dtype=torch.float32, device=dev) * std).to(dtype)


def layer_weights(H: int, E: int, I: int, Is: int, seed: int, std_expert: float, std_router: float,
                  dtype: torch.dtype, device: str = "cpu") -> Dict[str, Optional[torch.Tensor]]:
    """Random weights of one MoE layer.  Draw order is fixed: Wr, Wg, Wu, Wd, then the shared
    expert (Wsg, Wsu, Wsd, wgate) when Is > 0.  device="cpu" (default) gives the same bytes on every
    machine; a GPU device draws there (for the 26 GB stack, whose bytes no test depends on)."""
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    w: Dict[str, Optional[torch.Tensor]] = {}
    w["Wr"] = _randn(g, (E, H), std_router, dtype)
    w["Wg"] = _randn(g, (E, I, H), std_expert, dtype)
    w["Wu"] = _randn(g, (E, I, H), std_expert, dtype)
    w["Wd"] = _randn(g, (E, H, I), std_expert, dtype)
    if Is > 0:
        w["Wsg"] = _randn(g, (Is, H), std_expert, dtype)
        w["Wsu"] = _randn(g, (Is, H), std_expert, dtype)
        w["Wsd"] = _randn(g, (H, Is), std_expert, dtype)
        w["wgate"] = _randn(g, (H,), std_router, dtype)
    else:
        w["Wsg"] = w["Wsu"] = w["Wsd"] = w["wgate"] = None
    return w


def tokens(T: int, H: int, seed: int, dtype: torch.dtype) -> torch.Tensor:
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)
    return _randn(g, (T, H), 1.0, dtype)


def zipf_bias(E: int, seed: int, s: float = 1.1, span: float = 2.0) -> torch.Tensor:
    """Per-expert router bias with a Zipf(s) profile over a seeded random ranking, mapped
    linearly so the top-ranked expert gets +span and the tail approaches -span."""
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)
    rank = torch.randperm(E, generator=g).to(torch.float64) + 1.0     # rank of expert e, 1..E
    z = rank.pow(-s)
    b = -span + 2.0 * span * (z - z.min()) / (z.max() - z.min())
    return b.to(torch.float32)


def tenant_bias(n_tenants: int, E: int, seed: int) -> torch.Tensor:
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)
    return torch.randn((n_tenants, E), generator=g, dtype=torch.float32)


# ------------------------------------------------------------------------------ the configs

def tiny(seed: int = 0, T: int = 16, H: int = 64, E: int = 8, K: int = 2, I: int = 128, Is: int = 0,
         renorm: bool = False, with_bias: bool = False) -> Workload:
    """Tiny fp32 layer: T 16, H 64, 8 experts top-2, intermediate 128, no shared expert;
    activations N(0,1), expert weights N(0,0.05), router weights N(0,0.1)."""
    shp = Shape(T=T, H=H, E=E, K=K, I=I, Is=Is, renorm=renorm)
    w = layer_weights(H, E, I, Is, seed, 0.05, 0.1, torch.float32)
    x = tokens(T, H, seed + 7919, torch.float32)
    bias = None
    if with_bias:
        g = torch.Generator(device="cpu")
        g.manual_seed(seed + 104729)
        bias = torch.randn((E,), generator=g, dtype=torch.float32) * 0.1
    return Workload(name="tiny", shape=shp, x=x, bias=bias, **w)


def qwen_layer(T: int, seed: int, bias: Optional[torch.Tensor] = None, name: str = "qwen",
               weights: Optional[Dict[str, Optional[torch.Tensor]]] = None, **over) -> Workload:
    """One Qwen1.5-MoE-2.7B-shaped layer in bf16: hidden 2048, 60 experts top-4 without
    renormalisation, expert intermediate 1408, shared intermediate 5632 with a sigmoid gate;
    weights N(0,0.02), activations N(0,1).  ``over`` shrinks dimensions for quick tests."""
    d = dict(QWEN)
    d.update(over)
    shp = Shape(T=T, **d)
    if weights is None:
        weights = layer_weights(shp.H, shp.E, shp.I, shp.Is, seed, 0.02, 0.02, torch.bfloat16)
    x = tokens(T, shp.H, seed + 7919, torch.bfloat16)
    return Workload(name=name, shape=shp, x=x, bias=bias, **weights)


def decode(seed: int = 1, T: int = 128, **over) -> Workload:
    """Decode batch: one token per request, T = 128, no router bias."""
    return qwen_layer(T, seed, None, "decode", **over)


def prefill(seed: int = 2, T: int = 4096, **over) -> Workload:
    """Prefill batch, T = 4096, with routing skewed by a Zipf(1.1) router bias scaled to
    +-2 logits, so a few experts receive most of the tokens."""
    E = over.get("E", QWEN["E"])
    wl = qwen_layer(T, seed, zipf_bias(E, seed + 15485863), "prefill", **over)
    return wl


def tenants(seed: int = 3, n_tenants: int = 4, T_per: int = 512, **over) -> Workload:
    """Multi-tenant batch: n_tenants x T_per tokens concatenated, each tenant with its own
    N(0,1) router bias per expert (bias is [n_tenants, E]; tenant_rows gives the token ranges)."""
    E = over.get("E", QWEN["E"])
    wl = qwen_layer(n_tenants * T_per, seed, tenant_bias(n_tenants, E, seed + 15485863), "tenants",
                    **over)
    wl.tenant_rows = [(i * T_per, (i + 1) * T_per) for i in range(n_tenants)]
    return wl


def stack_layer_weights(layer: int, device: str = "cpu", **over) -> Dict[str, Optional[torch.Tensor]]:
    """Weights of layer ``layer`` of the 24-layer stack (seed 1000 + layer)."""
    d = dict(QWEN)
    d.update(over)
    d.pop("K", None)
    d.pop("renorm", None)
    return layer_weights(d["H"], d["E"], d["I"], d["Is"], 1000 + layer, 0.02, 0.02, torch.bfloat16, device)


def partition(E: int, g: int) -> List[Tuple[int, int]]:
    """Expert blocks of g consecutive experts (the last may be shorter)."""
    return [(lo, min(lo + g, E)) for lo in range(0, E, g)]
