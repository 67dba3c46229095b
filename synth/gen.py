"""Seeded generators for weights and per-worker gradients of the measured configurations.

Values are drawn with torch's generator on the device the caller names (CPU for the
host-only tests, the GPU for the large configurations); whoever needs the same inputs
elsewhere copies the bytes.  Recipes:

  config 1  one 1024x1024 tensor, weights N(0, 1/1024), grads N(0, 1e-3^2), global s=0.8, W=4
  config 2  ResNet-18 shapes, He-normal conv/fc weights, norm gamma=1, beta=0, bias=0,
            grads N(0, sigma_l^2) with sigma_l = 1e-3*sqrt(576/fan_in_l) (1e-3 for 1-D
            tensors), every tensor its own prune scope at s=0.9, W=8
  config 3  BERT-base shapes, matrices/embeddings N(0, 0.02^2), gamma=1, beta=bias=0,
            grads 1e-4 * t3/sqrt(3) (Student-t, 3 degrees of freedom, unit variance
            scaling), global s=0.7, W=8
  config 4  GPT-2-medium shapes, same weight recipe, grads N(0, 1e-4^2) rounded once to
            bf16 (nearest even), global s=0.9, W=16
  config 5  1.3B decoder shapes, same weight recipe, fp32 grads N(0, 1e-4^2), every
            tensor its own scope, s taken from (0.5, 0.8, 0.95) by step, W=8
  configs 6-8  the paper's own evaluation models with a 100-way classifier (Sec. IV-A: VGG19,
            ResNet152, ViT-Base-16 on CIFAR-100), at its default pruning ratio 0.5 and its 8 workers
            (Sec. IV-C), fp32: the two convolutional nets with config 2's recipe, the transformer
            with config 5's; every tensor its own prune scope
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Dict, List, Optional

import torch

from .shapes import TensorSpec, _decoder, config_shapes, flat_size, seg_offsets

CONFIGS: Dict[int, dict] = {
    1: dict(name="single-1024x1024", scope="global", sparsity=(0.8,), workers=4, dtype="f32"),
    2: dict(name="resnet18-shaped", scope="per-layer", sparsity=(0.9,), workers=8, dtype="f32"),
    3: dict(name="bert-base-shaped", scope="global", sparsity=(0.7,), workers=8, dtype="f32"),
    4: dict(name="gpt2-medium-shaped", scope="global", sparsity=(0.9,), workers=16, dtype="bf16"),
    5: dict(name="decoder-1.3b-shaped", scope="per-layer", sparsity=(0.5, 0.8, 0.95), workers=8, dtype="f32"),
    6: dict(name="vgg19-cifar100-shaped", scope="per-layer", sparsity=(0.5,), workers=8, dtype="f32"),
    7: dict(name="resnet152-cifar100-shaped", scope="per-layer", sparsity=(0.5,), workers=8, dtype="f32"),
    8: dict(name="vit-base-16-cifar100-shaped", scope="per-layer", sparsity=(0.5,), workers=8, dtype="f32"),
}

CONV_NETS = (2, 6, 7)   # He-normal weights, fan-in scaled gradients

SEED_BASE = 0x5AC70000


def config_seed(config_id: int) -> int:
    return SEED_BASE + 256 * config_id


@dataclass
class Workload:
    config_id: int
    name: str
    specs: List[TensorSpec]
    n: int
    scope: str                      # "global" | "per-layer"
    scope_offsets: List[int]        # prune-scope boundaries in the flat set
    sparsity_schedule: tuple        # one value, or the per-step cycle of config 5
    workers: int
    dtype: str                      # "f32" | "bf16" gradient payload
    weights: torch.Tensor           # fp32, flat, on `device`
    grads: List[torch.Tensor] = field(default_factory=list)   # W flat tensors

    def sparsity_at(self, step: int = 0) -> List[float]:
        s = self.sparsity_schedule[step % len(self.sparsity_schedule)]
        return [s] * (len(self.scope_offsets) - 1)


def _reduced_specs(config_id: int) -> List[TensorSpec]:
    """Same tensor kinds and order, fewer layers and smaller odd-sized dimensions."""
    if config_id in (1, 2, 6, 7, 8):
        return config_shapes(config_id)
    if config_id == 3:
        from .shapes import _linear, _ln  # local: builds a 2-layer BERT-like list
        h, f = 96, 384
        t = [TensorSpec("emb.word", (1531, h), "embed", h), TensorSpec("emb.pos", (64, h), "embed", h),
             TensorSpec("emb.type", (2, h), "embed", h)]
        _ln(t, "emb.ln", h)
        for i in range(2):
            p = f"layer{i}"
            for proj in ("q", "k", "v", "o"):
                _linear(t, f"{p}.attn.{proj}", h, h)
            _ln(t, p + ".attn.ln", h)
            _linear(t, p + ".ffn.in", f, h)
            _linear(t, p + ".ffn.out", h, f)
            _ln(t, p + ".ffn.ln", h)
        _linear(t, "pooler", h, h)
        return t
    if config_id == 4:
        return _decoder(128, 512, 2, 2053, 64)
    if config_id == 5:
        return _decoder(160, 640, 2, 1021, 96)
    raise ValueError(config_id)


def _fill_weights(flat: torch.Tensor, specs: List[TensorSpec], config_id: int, gen: torch.Generator) -> None:
    off = 0
    if config_id == 1:
        flat.normal_(0.0, 1.0 / 32.0, generator=gen)
        return
    if config_id not in CONV_NETS:
        flat.normal_(0.0, 0.02, generator=gen)
    for s in specs:
        view = flat[off:off + s.numel]
        if s.kind == "gamma":
            view.fill_(1.0)
        elif s.kind in ("beta", "bias"):
            view.zero_()
        elif config_id in CONV_NETS:
            view.normal_(0.0, math.sqrt(2.0 / s.fan_in), generator=gen)
        off += s.numel


def _student_t3(n: int, device, gen: torch.Generator, chunk: int = 1 << 26) -> torch.Tensor:
    out = torch.empty(n, dtype=torch.float32, device=device)
    for a in range(0, n, chunk):
        b = min(n, a + chunk)
        z = torch.randn(4, b - a, dtype=torch.float32, device=device, generator=gen)
        chi = (z[1] * z[1] + z[2] * z[2] + z[3] * z[3]) / 3.0
        out[a:b] = z[0] * torch.rsqrt(chi)
    return out


def _make_grad(specs: List[TensorSpec], n: int, config_id: int, dtype: str, device, gen: torch.Generator) -> torch.Tensor:
    if config_id == 3:
        g = _student_t3(n, device, gen)
        g.mul_(1e-4 / math.sqrt(3.0))
    else:
        g = torch.empty(n, dtype=torch.float32, device=device)
        if config_id == 1:
            g.normal_(0.0, 1e-3, generator=gen)
        elif config_id in CONV_NETS:
            off = 0
            for s in specs:
                sigma = 1e-3 * math.sqrt(576.0 / s.fan_in) if s.fan_in else 1e-3
                g[off:off + s.numel].normal_(0.0, sigma, generator=gen)
                off += s.numel
        else:
            g.normal_(0.0, 1e-4, generator=gen)
    if dtype == "bf16":
        g = g.to(torch.bfloat16)   # round to nearest even, once
    return g


def make_workload(config_id: int, device="cpu", reduced: bool = False, workers: Optional[int] = None,
                  with_grads: bool = True) -> Workload:
    cfg = CONFIGS[config_id]
    specs = _reduced_specs(config_id) if reduced else config_shapes(config_id)
    n = flat_size(specs)
    dev = torch.device(device)
    seed = config_seed(config_id)
    gen = torch.Generator(device=dev)
    gen.manual_seed(seed)
    weights = torch.empty(n, dtype=torch.float32, device=dev)
    _fill_weights(weights, specs, config_id, gen)
    scope_offsets = seg_offsets(specs) if cfg["scope"] == "per-layer" else [0, n]
    W = workers if workers is not None else cfg["workers"]
    wl = Workload(config_id, cfg["name"] + ("-reduced" if reduced else ""), specs, n, cfg["scope"],
                  scope_offsets, tuple(cfg["sparsity"]), W, cfg["dtype"], weights)
    if with_grads:
        for w in range(W):
            g = torch.Generator(device=dev)
            g.manual_seed(seed + 1 + w)
            wl.grads.append(_make_grad(specs, n, config_id, cfg["dtype"], dev, g))
    return wl
