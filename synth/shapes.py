"""Tensor lists of the measured configurations, in flat (concatenation) order.

A gradient bucket reaches the communication hook as one flat 1-D tensor (Sec. I, Mask
Tracker paragraph of Sec. III-B); here the flat set is the row-major concatenation of the
listed tensors with no padding.  The vision model is one of the paper's own workloads
(Sec. IV-A); the language-model shapes stand in for its "vision and language models".
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Tuple


@dataclass(frozen=True)
class TensorSpec:
    name: str
    shape: Tuple[int, ...]
    kind: str      # "matrix" | "conv" | "embed" | "gamma" | "beta" | "bias"
    fan_in: int    # inputs feeding one output unit (0 for 1-D tensors)

    @property
    def numel(self) -> int:
        n = 1
        for d in self.shape:
            n *= d
        return n


def _single() -> List[TensorSpec]:
    return [TensorSpec("w", (1024, 1024), "matrix", 1024)]


def _resnet18() -> List[TensorSpec]:
    t: List[TensorSpec] = []

    def conv(name, cout, cin, k):
        t.append(TensorSpec(name, (cout, cin, k, k), "conv", cin * k * k))

    def bn(name, c):
        t.append(TensorSpec(name + ".gamma", (c,), "gamma", 0))
        t.append(TensorSpec(name + ".beta", (c,), "beta", 0))

    conv("conv1", 64, 3, 7)
    bn("bn1", 64)
    cin = 64
    for stage, cout in enumerate((64, 128, 256, 512), start=1):
        for block in range(2):
            p = f"layer{stage}.{block}"
            conv(p + ".conv1", cout, cin if block == 0 else cout, 3)
            bn(p + ".bn1", cout)
            conv(p + ".conv2", cout, cout, 3)
            bn(p + ".bn2", cout)
            if block == 0 and cin != cout:
                conv(p + ".down", cout, cin, 1)
                bn(p + ".down_bn", cout)
        cin = cout
    t.append(TensorSpec("fc.weight", (1000, 512), "matrix", 512))
    t.append(TensorSpec("fc.bias", (1000,), "bias", 0))
    return t


def _ln(t, name, h):
    t.append(TensorSpec(name + ".gamma", (h,), "gamma", 0))
    t.append(TensorSpec(name + ".beta", (h,), "beta", 0))


def _linear(t, name, dout, din):
    t.append(TensorSpec(name + ".weight", (dout, din), "matrix", din))
    t.append(TensorSpec(name + ".bias", (dout,), "bias", 0))


def _bert_base() -> List[TensorSpec]:
    h, f, layers = 768, 3072, 12
    t: List[TensorSpec] = [
        TensorSpec("emb.word", (30522, h), "embed", h),
        TensorSpec("emb.pos", (512, h), "embed", h),
        TensorSpec("emb.type", (2, h), "embed", h),
    ]
    _ln(t, "emb.ln", h)
    for i in range(layers):
        p = f"layer{i}"
        for proj in ("q", "k", "v", "o"):
            _linear(t, f"{p}.attn.{proj}", h, h)
        _ln(t, p + ".attn.ln", h)
        _linear(t, p + ".ffn.in", f, h)
        _linear(t, p + ".ffn.out", h, f)
        _ln(t, p + ".ffn.ln", h)
    _linear(t, "pooler", h, h)
    return t


def _decoder(h: int, f: int, layers: int, vocab: int, positions: int) -> List[TensorSpec]:
    t: List[TensorSpec] = [
        TensorSpec("wte", (vocab, h), "embed", h),
        TensorSpec("wpe", (positions, h), "embed", h),
    ]
    for i in range(layers):
        p = f"h{i}"
        _ln(t, p + ".ln1", h)
        _linear(t, p + ".attn.qkv", 3 * h, h)
        _linear(t, p + ".attn.proj", h, h)
        _ln(t, p + ".ln2", h)
        _linear(t, p + ".mlp.fc", f, h)
        _linear(t, p + ".mlp.fc2", h, f)
    _ln(t, "ln_f", h)
    return t


# ---- the paper's own evaluation models (Sec. IV-A: VGG19, ResNet152, ViT-Base-16 on CIFAR-100) ----
# Layer dimensions are those of the published architectures with a `classes`-way classifier; with
# classes = 1000 the element counts are the well-known 143,667,240 / 60,192,808 / 86,567,656.

def _vgg19(classes: int) -> List[TensorSpec]:
    t: List[TensorSpec] = []
    cin = 3
    for i, cout in enumerate((64, 64, 128, 128, 256, 256, 256, 256, 512, 512, 512, 512, 512, 512, 512, 512)):
        t.append(TensorSpec(f"features.{i}.weight", (cout, cin, 3, 3), "conv", cin * 9))
        t.append(TensorSpec(f"features.{i}.bias", (cout,), "bias", 0))
        cin = cout
    _linear(t, "classifier.0", 4096, 512 * 7 * 7)
    _linear(t, "classifier.3", 4096, 4096)
    _linear(t, "classifier.6", classes, 4096)
    return t


def _resnet152(classes: int) -> List[TensorSpec]:
    t: List[TensorSpec] = []

    def conv(name, cout, cin, k):
        t.append(TensorSpec(name, (cout, cin, k, k), "conv", cin * k * k))

    def bn(name, c):
        t.append(TensorSpec(name + ".gamma", (c,), "gamma", 0))
        t.append(TensorSpec(name + ".beta", (c,), "beta", 0))

    conv("conv1", 64, 3, 7)
    bn("bn1", 64)
    cin = 64
    for stage, (width, blocks) in enumerate(((64, 3), (128, 8), (256, 36), (512, 3)), start=1):
        for b in range(blocks):
            p = f"layer{stage}.{b}"
            conv(p + ".conv1", width, cin, 1)
            bn(p + ".bn1", width)
            conv(p + ".conv2", width, width, 3)
            bn(p + ".bn2", width)
            conv(p + ".conv3", 4 * width, width, 1)
            bn(p + ".bn3", 4 * width)
            if b == 0:
                conv(p + ".down", 4 * width, cin, 1)
                bn(p + ".down_bn", 4 * width)
            cin = 4 * width
    _linear(t, "fc", classes, 2048)
    return t


def _vit_base_16(classes: int) -> List[TensorSpec]:
    h, f, layers, patches = 768, 3072, 12, 196
    t: List[TensorSpec] = [
        TensorSpec("class_token", (1, 1, h), "embed", h),
        TensorSpec("conv_proj.weight", (h, 3, 16, 16), "conv", 3 * 256),
        TensorSpec("conv_proj.bias", (h,), "bias", 0),
        TensorSpec("pos_embedding", (1, patches + 1, h), "embed", h),
    ]
    for i in range(layers):
        p = f"encoder.{i}"
        _ln(t, p + ".ln_1", h)
        _linear(t, p + ".attn.in_proj", 3 * h, h)
        _linear(t, p + ".attn.out_proj", h, h)
        _ln(t, p + ".ln_2", h)
        _linear(t, p + ".mlp.0", f, h)
        _linear(t, p + ".mlp.3", h, f)
    _ln(t, "encoder.ln", h)
    _linear(t, "head", classes, h)
    return t


def config_shapes(config_id: int) -> List[TensorSpec]:
    if config_id == 1:
        return _single()
    if config_id == 2:
        return _resnet18()
    if config_id == 3:
        return _bert_base()
    if config_id == 4:
        return _decoder(1024, 4096, 24, 50257, 1024)
    if config_id == 5:
        return _decoder(2048, 8192, 24, 50257, 2048)
    if config_id == 6:
        return _vgg19(100)
    if config_id == 7:
        return _resnet152(100)
    if config_id == 8:
        return _vit_base_16(100)
    raise ValueError(f"unknown config {config_id}")


def flat_size(specs: List[TensorSpec]) -> int:
    return sum(s.numel for s in specs)


def seg_offsets(specs: List[TensorSpec]) -> List[int]:
    off = [0]
    for s in specs:
        off.append(off[-1] + s.numel)
    return off
