"""Parameter-shape lists of the public architectures the benchmark configurations name.

Only shapes are used: the synthetic gradient sets take their tensor sizes and
per-tensor fan-in from these lists.  No weights, datasets or model code are
involved.  Each function returns tensors in forward (topological) order as
``Tensor(name, shape, fan_in)``; the DDP-style bucketiser then walks the list
in reverse (paper §3.3: buckets follow the reversed topological order).

fan_in rule (input recipe of the synthetic workloads): conv = in_channels *
kernel area, linear = in_features, embedding = embedding dim, 1-D tensors
(biases, norm scales/shifts) = 1.
"""
from __future__ import annotations

from dataclasses import dataclass
from math import prod
from typing import List, Tuple


@dataclass(frozen=True)
class Tensor:
    name: str
    shape: Tuple[int, ...]
    fan_in: int

    @property
    def numel(self) -> int:
        return prod(self.shape)


def _conv(name, cout, cin, k):
    return Tensor(name, (cout, cin, k, k), cin * k * k)


def _vec(name, n):
    return Tensor(name, (n,), 1)


def _linear(prefix, out_f, in_f, bias=True):
    ts = [Tensor(prefix + ".weight", (out_f, in_f), in_f)]
    if bias:
        ts.append(_vec(prefix + ".bias", out_f))
    return ts


def _norm(prefix, n):
    return [_vec(prefix + ".weight", n), _vec(prefix + ".bias", n)]


def resnet50() -> List[Tensor]:
    """ResNet-50 (bottleneck blocks 3-4-6-3, 1000 classes): 161 tensors."""
    ts: List[Tensor] = [_conv("conv1.weight", 64, 3, 7)] + _norm("bn1", 64)
    inplanes = 64
    for li, (planes, blocks) in enumerate([(64, 3), (128, 4), (256, 6), (512, 3)], 1):
        for b in range(blocks):
            p = f"layer{li}.{b}"
            ts.append(_conv(p + ".conv1.weight", planes, inplanes, 1))
            ts += _norm(p + ".bn1", planes)
            ts.append(_conv(p + ".conv2.weight", planes, planes, 3))
            ts += _norm(p + ".bn2", planes)
            ts.append(_conv(p + ".conv3.weight", planes * 4, planes, 1))
            ts += _norm(p + ".bn3", planes * 4)
            if b == 0:
                ts.append(_conv(p + ".downsample.0.weight", planes * 4, inplanes, 1))
                ts += _norm(p + ".downsample.1", planes * 4)
            inplanes = planes * 4
    ts += _linear("fc", 1000, 2048)
    return ts


def resnet50_bn_channels() -> List[int]:
    """Channel count of each of ResNet-50's 53 BatchNorm layers, forward order."""
    return [t.shape[0] for t in resnet50()
            if t.name.endswith(".weight") and len(t.shape) == 1]


def bert_base() -> List[Tensor]:
    """BERT-base encoder with pooler (vocab 30522, 12 layers, d=768): 199 tensors."""
    d, ff = 768, 3072
    ts: List[Tensor] = [
        Tensor("embeddings.word", (30522, d), d),
        Tensor("embeddings.position", (512, d), d),
        Tensor("embeddings.token_type", (2, d), d),
    ] + _norm("embeddings.ln", d)
    for i in range(12):
        p = f"layer{i}"
        for nm in ("q", "k", "v", "attn_out"):
            ts += _linear(f"{p}.{nm}", d, d)
        ts += _norm(f"{p}.attn_ln", d)
        ts += _linear(f"{p}.ffn_in", ff, d)
        ts += _linear(f"{p}.ffn_out", d, ff)
        ts += _norm(f"{p}.ffn_ln", d)
    ts += _linear("pooler", d, d)
    return ts


def gpt2_medium() -> List[Tensor]:
    """GPT-2-medium (vocab 50257, ctx 1024, 24 layers, d=1024): 292 tensors.

    Projection weights are stored (in_features, out_features)."""
    d = 1024
    ts: List[Tensor] = [Tensor("wte", (50257, d), d), Tensor("wpe", (1024, d), d)]
    for i in range(24):
        p = f"h{i}"
        ts += _norm(p + ".ln_1", d)
        ts += [Tensor(p + ".attn.c_attn.weight", (d, 3 * d), d), _vec(p + ".attn.c_attn.bias", 3 * d)]
        ts += [Tensor(p + ".attn.c_proj.weight", (d, d), d), _vec(p + ".attn.c_proj.bias", d)]
        ts += _norm(p + ".ln_2", d)
        ts += [Tensor(p + ".mlp.c_fc.weight", (d, 4 * d), d), _vec(p + ".mlp.c_fc.bias", 4 * d)]
        ts += [Tensor(p + ".mlp.c_proj.weight", (4 * d, d), 4 * d), _vec(p + ".mlp.c_proj.bias", d)]
    ts += _norm("ln_f", d)
    return ts


def flat(n: int) -> List[Tensor]:
    """One flat tensor of n elements with fan_in 1 (the smallest configuration)."""
    return [Tensor("flat", (n,), 1)]
