"""Seeded synthetic workloads: shapes and value distributions only.

This module draws the fp32 tensors (weights, activations) that both the HIP
path and the CPU checker consume.  It holds none of the method's arithmetic:
no quantisation, no expansion, no contraction.  Every tensor comes from a
counter-based generator (numpy Philox) keyed by ``BASE_SEED + 1000*config +
tensor_id``, so the same call returns the same bytes on every machine with
this numpy.

The five workloads stand in for the networks the paper evaluates (ImageNet
ConvNets, BERT on GLUE, LLM layers with outlier channels): only layer shapes
and value distributions are taken; no dataset item or trained weight is used.
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import Dict, Optional, Tuple

import numpy as np

BASE_SEED = 231115806


def _rng(config: int, tensor_id: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(BASE_SEED + 1000 * config + tensor_id))


def normal(config: int, tensor_id: int, shape, std: float = 1.0) -> np.ndarray:
    """fp32 N(0, std^2)."""
    a = _rng(config, tensor_id).standard_normal(size=shape, dtype=np.float32)
    if std != 1.0:
        a *= np.float32(std)
    return a


def student_t(config: int, tensor_id: int, shape, df: float, scale: float) -> np.ndarray:
    """fp32 Student-t(df) * scale (heavy-tailed weights)."""
    a = _rng(config, tensor_id).standard_t(df, size=shape)
    return (a * scale).astype(np.float32)


def pick_indices(config: int, tensor_id: int, n: int, frac: float) -> np.ndarray:
    """A fixed, seeded set of round(frac*n) (at least 1 if frac>0) distinct indices."""
    if frac <= 0.0:
        return np.zeros(0, dtype=np.int64)
    cnt = max(1, int(round(frac * n)))
    return np.sort(_rng(config, tensor_id).choice(n, size=cnt, replace=False))


@dataclass(frozen=True)
class LayerSpec:
    """One expanded layer: quantisation hyper-parameters (the paper's b, K, gamma)."""
    out_features: int
    in_features: int
    bits: int            # 8, 4 or 2 (ternary)
    K: int               # expansion order
    gamma: float         # fraction of channel groups KEPT at orders k>=2
    group: int           # output channels per group


@dataclass(frozen=True)
class Workload:
    name: str
    config: int                      # 1..5, index into the benchmark's config list
    kind: str                        # "linear" | "conv2d" | "mlp_gelu" | "mlp_gated" | "chain"
    layers: Tuple[LayerSpec, ...]
    tokens: int                      # T (conv: N*H_out*W_out)
    split: Tuple[int, ...]           # ensemble grouping [K_1..K_M]
    conv: Optional[Dict[str, int]] = None   # N,C,H,W,kh,kw,stride,pad
    w_dist: Dict[str, float] = field(default_factory=dict)
    x_dist: Dict[str, float] = field(default_factory=dict)
    # kind "chain": per layer (activation "none" | "relu" | "gelu", skip_from, skip_pre_act);
    # skip_from = -1 none, j = the tensor that entered layer j (0 = the network input)
    chain: Optional[Tuple[Tuple[str, int, bool], ...]] = None


C1 = Workload(
    name="c1_linear_256_w8a8_k2", config=1, kind="linear",
    layers=(LayerSpec(256, 256, 8, 2, 1.0, 16),), tokens=16, split=(2,),
    w_dist=dict(kind=0, std=0.02), x_dist=dict(kind=0))
C2 = Workload(
    name="c2_conv3x3_256_w4a8_k3", config=2, kind="conv2d",
    layers=(LayerSpec(256, 256 * 9, 4, 3, 0.5, 16),), tokens=32 * 14 * 14, split=(2, 1),
    conv=dict(N=32, C=256, H=14, W=14, kh=3, kw=3, stride=1, pad=1),
    w_dist=dict(kind=0, std=float(np.sqrt(2.0 / 2304.0))), x_dist=dict(kind=1))
C3 = Workload(
    name="c3_bert_mlp_w4a8_k3", config=3, kind="mlp_gelu",
    layers=(LayerSpec(3072, 768, 4, 3, 0.5, 32), LayerSpec(768, 3072, 4, 3, 0.5, 32)),
    tokens=4096, split=(3,),
    w_dist=dict(kind=1, df=4.0, scale=0.02),
    x_dist=dict(kind=0, outlier_frac=0.02, outlier_mul=10.0))
C4 = Workload(
    name="c4_llm7b_linear_ternary_k4", config=4, kind="linear",
    layers=(LayerSpec(11008, 4096, 2, 4, 0.25, 64),), tokens=4096, split=(4,),
    w_dist=dict(kind=1, df=3.0, scale=0.015, outlier_frac=0.01, outlier_mul=8.0),
    x_dist=dict(kind=0, outlier_frac=0.005, outlier_mul=20.0))
C5 = Workload(
    name="c5_llm7b_gated_mlp_w4a8_k4", config=5, kind="mlp_gated",
    layers=(LayerSpec(2 * 11008, 4096, 4, 4, 0.5, 64), LayerSpec(4096, 11008, 4, 4, 0.5, 64)),
    tokens=4096, split=(2, 2),
    w_dist=dict(kind=1, df=3.0, scale=0.015, outlier_frac=0.01, outlier_mul=8.0),
    x_dist=dict(kind=0, outlier_frac=0.005, outlier_mul=20.0))

WORKLOADS = {w.config: w for w in (C1, C2, C3, C4, C5)}


def residual_stack(width: int, blocks: int, out_features: int, bits: int, K: int, gamma: float, group: int,
                   tokens: int, split, name: str = "chain_residual_stack") -> Workload:
    """A synthetic residual network as a chain of fully-connected layers, standing in for the
    residual ConvNet of the paper's run-time table: a stem layer, `blocks` residual blocks of two
    layers each (a1 = ReLU(W1 a), a2 = ReLU(W2 a1 + a)), and a linear head.  He-scaled normal
    weights keep the activations of the stack O(1)."""
    layers = [LayerSpec(width, width, bits, K, gamma, group)]
    chain = [("relu", -1, True)]
    for b in range(blocks):
        first = len(layers)                       # the block's input is the tensor entering this layer
        layers += [LayerSpec(width, width, bits, K, gamma, group)] * 2
        chain += [("relu", -1, True), ("relu", first, True)]
    layers.append(LayerSpec(out_features, width, bits, K, gamma, group))
    chain.append(("none", -1, True))
    return Workload(name=name, config=6, kind="chain", layers=tuple(layers), tokens=tokens, split=tuple(split),
                    w_dist=dict(kind=0, std=float(np.sqrt(2.0 / width))), x_dist=dict(kind=0), chain=tuple(chain))


# ResNet-like stack for the ensemble run-time comparison: ternary, K = 8, half the groups kept
CHAIN = residual_stack(2048, 3, 1024, 2, 8, 0.5, 64, 4096, (4, 4))


def decode_stack(layers: int = 8, tokens: int = 16) -> Workload:
    """A decode-time stack of layers of config 4's shape and distributions (11008 x 4096 and back,
    ternary, K = 4, a quarter of the groups kept), ReLU between them: what a resident decode step
    streams layer after layer.  Two fp32 weights (one per shape) serve all layers; every layer still has
    its own expansion, so its codes are streamed from memory of their own."""
    up = LayerSpec(11008, 4096, 2, 4, 0.25, 64)
    down = LayerSpec(4096, 11008, 2, 4, 0.25, 64)
    specs = tuple(up if l % 2 == 0 else down for l in range(layers))
    chain = tuple(("relu", -1, True) if l < layers - 1 else ("none", -1, True) for l in range(layers))
    return Workload(name="decode_stack_%d_layers_c4_shape" % layers, config=4, kind="chain", layers=specs, tokens=tokens,
                    split=(4,), w_dist=C4.w_dist, x_dist=C4.x_dist, chain=chain)


DECODE_STACK = decode_stack()


def with_tokens(w: Workload, tokens: int) -> Workload:
    """Same layer, another token count (conv workloads keep their geometry)."""
    if w.kind == "conv2d":
        raise ValueError("conv workloads derive tokens from their geometry")
    return replace(w, tokens=int(tokens))


def scaled(w: Workload, out_div: int = 1, in_div: int = 1, tokens: Optional[int] = None) -> Workload:
    """A reduced copy (same distributions and hyper-parameters, smaller shapes) that the
    CPU checker finishes in seconds.  Divisors must keep out % group == 0."""
    if w.kind == "conv2d":
        c = dict(w.conv)
        c["C"] //= in_div
        l0 = w.layers[0]
        layers = (replace(l0, out_features=l0.out_features // out_div,
                          in_features=c["C"] * c["kh"] * c["kw"]),)
        if tokens is not None:
            c["N"] = max(1, tokens // (c["H"] * c["W"]))
        t = c["N"] * c["H"] * c["W"]
        return replace(w, layers=layers, conv=c, tokens=t, name=w.name + "_small")
    if w.kind == "linear":
        l0 = w.layers[0]
        layers = (replace(l0, out_features=l0.out_features // out_div,
                          in_features=l0.in_features // in_div),)
    else:
        l0, l1 = w.layers
        hid = l1.in_features // out_div
        mult = 2 if w.kind == "mlp_gated" else 1
        layers = (replace(l0, out_features=mult * hid, in_features=l0.in_features // in_div),
                  replace(l1, out_features=l1.out_features // in_div, in_features=hid))
    for l in layers:
        if l.out_features % l.group:
            raise ValueError("scaled shape breaks out % group == 0")
    return replace(w, layers=layers, tokens=w.tokens if tokens is None else int(tokens),
                   name=w.name + "_small")


def make_weight(w: Workload, layer: int) -> np.ndarray:
    """fp32 weight [out, in] (conv: [out, C*kh*kw], rows are flattened [C, kh, kw])."""
    spec = w.layers[layer]
    shape = (spec.out_features, spec.in_features)
    d = w.w_dist
    tid = 10 + layer
    if d["kind"] == 0:
        W = normal(w.config, tid, shape, d["std"])
    else:
        W = student_t(w.config, tid, shape, d["df"], d["scale"])
    if d.get("outlier_frac", 0.0) > 0.0:
        rows = pick_indices(w.config, 20 + layer, shape[0], d["outlier_frac"])
        W[rows, :] *= np.float32(d["outlier_mul"])
    return np.ascontiguousarray(W)


def make_input(w: Workload) -> np.ndarray:
    """fp32 input: [T, in] for linear/MLP workloads, NCHW for conv."""
    d = w.x_dist
    if w.kind == "conv2d":
        c = w.conv
        x = normal(w.config, 1, (c["N"], c["C"], c["H"], c["W"]))
        np.maximum(x, 0.0, out=x)          # post-ReLU feature map
        return x
    I = w.layers[0].in_features
    x = normal(w.config, 1, (w.tokens, I))
    if d.get("outlier_frac", 0.0) > 0.0:
        cols = pick_indices(w.config, 2, I, d["outlier_frac"])
        x[:, cols] *= np.float32(d["outlier_mul"])
    return np.ascontiguousarray(x)


def make_bias(w: Workload, layer: int) -> np.ndarray:
    """Optional fp32 bias [out] ~ N(0, 0.1^2); the benchmark configs run without one."""
    return normal(w.config, 30 + layer, (w.layers[layer].out_features,), 0.1)
