"""Seeded synthetic multi-tenant workloads.

This module only draws numbers and describes shapes: tenant models (layer lists,
weights, biases), the arrival-ordered tenant id of every request and the request
inputs.  It contains none of the inference arithmetic, and it is the one module
both the reference evaluator's tests and the GPU library's tests may import, so
that both see identical bytes.

The paper (section 3.2) measures on off-the-shelf networks from a public model zoo
and on resnet18; neither is available offline, so these generic tenant mixes stand
in for them.  The five named mixes:

  c1  4 tenants, MLP 256-512-512-10, ReLU, fp32; 64 requests, tenant uniform;
      x ~ N(0,1)
  c2  64 tenants, MLP 784-1024-1024-10, ReLU, bf16; 4096 requests, tenant
      popularity Zipf(s=1.1); x ~ U(0,1)
  c3  256 tenants, MLP 1024-{512,1024,2048}^(D-1)-100 with D uniform in 2..6 linear
      layers and every hidden width drawn independently, ReLU, bf16; 16384 requests,
      Zipf(s=1.2); x ~ N(0,1)
  c4  32 tenants, CNN on 32x32x3 (NHWC): conv3x3 3-32 s1, 32-64 s2, 64-128 s2, ReLU
      each, global average pool, FC 128-10, bf16; 2048 requests uniform; x ~ N(0,1)
  c5  8 tenants, MLP 4096-4096-4096-4096-1000, GELU, bf16; 32768 requests uniform;
      x ~ N(0,1)
and, for the wider layer catalogue, r18: 4 tenants with resnet18-shaped models (the paper's
running example, section 1.1) on 224x224x3 inputs, bf16, 64 requests uniform.

Readings: weights ~ N(0, 1/fan_in) and biases ~ N(0, 0.01) where the second argument
is a variance (std fan_in^-1/2 and 0.1; fan_in = K for FC, 9*C_in for conv), for all
five mixes; "n-layer" counts linear layers; no activation after the last layer; Zipf
is p_k ~ k^-s on ranks 1..T with a seeded rank->tenant permutation; requests are
i.i.d. draws kept in arrival order.  For bf16 mixes the generator rounds weights and
inputs to bfloat16 once (library conversion), so every consumer starts from the same
representable values; biases stay fp32.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional

import numpy as np
import torch

FC, CONV, GAP, MAXPOOL, ADD = 0, 1, 2, 3, 4
ACT_NONE, ACT_RELU, ACT_GELU = 0, 1, 2

BASE_SEED = 190106887


@dataclass
class LayerSpec:
    kind: int
    act: int = ACT_NONE
    in_features: int = 0      # FC: K      CONV: C_in   GAP: C
    out_features: int = 0     # FC: N      CONV: C_out  GAP: C
    in_h: int = 0
    in_w: int = 0
    stride: int = 1
    ksize: int = 3            # CONV, MAXPOOL: window k x k
    pad: int = 1              # CONV, MAXPOOL
    src: int = 0              # j + 1: reads the output of layer j; 0: the previous layer
    src2: int = 0             # ADD: the second operand, same convention

    def out_hw(self):
        if self.kind == ADD:
            return (self.in_h, self.in_w)
        if self.kind not in (CONV, MAXPOOL):
            return (1, 1)
        return ((self.in_h + 2 * self.pad - self.ksize) // self.stride + 1,
                (self.in_w + 2 * self.pad - self.ksize) // self.stride + 1)

    def in_len(self) -> int:
        return self.in_features if self.kind == FC else self.in_h * self.in_w * self.in_features

    def out_len(self) -> int:
        if self.kind == FC:
            return self.out_features
        if self.kind == GAP:
            return self.in_features
        oh, ow = self.out_hw()
        return oh * ow * (self.out_features if self.kind == CONV else self.in_features)


@dataclass
class TenantModel:
    layers: List[LayerSpec]
    weights: List[Optional[np.ndarray]]   # float32 arrays holding representable values
    biases: List[Optional[np.ndarray]]    # float32
    # batch normalisation behind convolution l, to be folded into it at registration:
    # bn[l] = (gamma, beta, mean, var), float32 [C_out] each, or None; absent: no layer has one
    bn: Optional[List[Optional[tuple]]] = None
    bn_eps: float = 1e-5

    @property
    def in_len(self) -> int:
        return self.layers[0].in_len()

    @property
    def n_classes(self) -> int:
        return self.layers[-1].out_len()

    def n_params(self) -> int:
        return sum(0 if w is None else w.size for w in self.weights)


@dataclass
class Workload:
    name: str
    dtype: str                              # "f32" or "bf16"
    tenants: Dict[int, TenantModel]
    tenant_ids: np.ndarray                  # int32 [R], arrival order
    inputs: np.ndarray                      # float32 [R, in_len], representable values
    meta: dict = field(default_factory=dict)

    @property
    def n_requests(self) -> int:
        return int(self.tenant_ids.size)

    def counts(self) -> Dict[int, int]:
        ids, c = np.unique(self.tenant_ids, return_counts=True)
        return {int(i): int(n) for i, n in zip(ids, c)}


# ---- number formats (repacking only) ---------------------------------------
def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """float32 -> nearest bfloat16 (library conversion), returned widened to float32."""
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32))
    return t.to(torch.bfloat16).to(torch.float32).numpy()


def bf16_bits(a: np.ndarray) -> np.ndarray:
    """Bit pattern (uint16) of float32 values that are already bfloat16-representable."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    assert not np.any(u & 0xFFFF), "values are not bfloat16-representable"
    return (u >> 16).astype(np.uint16)


def bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


# ---- draws --------------------------------------------------------------------
def _rng(*key) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([BASE_SEED, *key])))


def _normal(rng, shape, std, dtype) -> np.ndarray:
    a = rng.standard_normal(shape, dtype=np.float32) * np.float32(std)
    return round_to_bf16(a) if dtype == "bf16" else a


def make_model(layers: List[LayerSpec], dtype: str, *key) -> TenantModel:
    weights, biases = [], []
    for li, l in enumerate(layers):
        rng = _rng(*key, li)
        if l.kind == FC:
            w = _normal(rng, (l.out_features, l.in_features), l.in_features ** -0.5, dtype)
        elif l.kind == CONV:
            k = l.ksize
            w = _normal(rng, (l.out_features, l.in_features, k, k), (k * k * l.in_features) ** -0.5, dtype)
        else:
            weights.append(None); biases.append(None)
            continue
        b = rng.standard_normal(l.out_features, dtype=np.float32) * np.float32(0.1)
        weights.append(w); biases.append(b.astype(np.float32))
    return TenantModel(layers, weights, biases)


def with_batchnorm(model: TenantModel, *key) -> TenantModel:
    """Give every convolution of the model a batch normalisation (gamma ~ U(0.5, 1.5), beta ~ N(0, 0.01),
    running mean ~ N(0, 0.01), running variance ~ U(0.5, 1.5)), to be folded in at registration."""
    bn = []
    for li, l in enumerate(model.layers):
        if l.kind != CONV:
            bn.append(None)
            continue
        rng = _rng(*key, li, 7005)
        c = l.out_features
        bn.append(((0.5 + rng.random(c, dtype=np.float32)), rng.standard_normal(c, dtype=np.float32) * np.float32(0.1),
                   rng.standard_normal(c, dtype=np.float32) * np.float32(0.1), (0.5 + rng.random(c, dtype=np.float32))))
    model.bn = bn
    return model


def mlp_layers(dims: List[int], act: int) -> List[LayerSpec]:
    n = len(dims) - 1
    return [LayerSpec(FC, act if i < n - 1 else ACT_NONE, dims[i], dims[i + 1]) for i in range(n)]


def cnn_layers(hw: int = 32, chans=(3, 32, 64, 128), strides=(1, 2, 2), classes: int = 10) -> List[LayerSpec]:
    layers, h = [], hw
    for i, s in enumerate(strides):
        l = LayerSpec(CONV, ACT_RELU, chans[i], chans[i + 1], h, h, s)
        layers.append(l)
        h = l.out_hw()[0]
    layers.append(LayerSpec(GAP, ACT_NONE, chans[-1], chans[-1], h, h))
    layers.append(LayerSpec(FC, ACT_NONE, chans[-1], classes))
    return layers


def resnet18_layers(hw: int = 32, chans: int = 3, widths=(64, 128, 256, 512), classes: int = 1000,
                    stem_kernel: int = 7) -> List[LayerSpec]:
    """The layer graph of an 18-layer residual network (the paper's running example, section 1.1) as a
    layer list with skip sources: 7x7 stride-2 stem, 3x3 stride-2 max-pool, four stages of two basic blocks
    (3x3 convolution, ReLU, 3x3 convolution, plus the block's input, ReLU; the first block of stages 2-4
    halves the image and takes its input through a 1x1 stride-2 convolution), global average pool, FC.
    Every convolution is followed by a batch normalisation, which `with_batchnorm` supplies and
    registration folds in.  The shape only: image size, widths and class count are free."""
    L: List[LayerSpec] = []
    stem = LayerSpec(CONV, ACT_RELU, chans, widths[0], hw, hw, 2, ksize=stem_kernel, pad=(stem_kernel - 1) // 2)
    L.append(stem)
    h = stem.out_hw()[0]
    pool = LayerSpec(MAXPOOL, ACT_NONE, widths[0], widths[0], h, h, 2, ksize=3, pad=1)
    L.append(pool)
    h = pool.out_hw()[0]
    c_in = widths[0]
    for stage, c in enumerate(widths):
        for block in range(2):
            stride = 2 if (stage > 0 and block == 0) else 1
            x_idx = len(L)                                     # src code of the block's input: the output of layer len(L) - 1
            conv1 = LayerSpec(CONV, ACT_RELU, c_in, c, h, h, stride, ksize=3, pad=1)
            L.append(conv1)
            h2 = conv1.out_hw()[0]
            L.append(LayerSpec(CONV, ACT_NONE, c, c, h2, h2, 1, ksize=3, pad=1))
            main_idx = len(L)                                  # src code of the main branch's output
            if stride != 1 or c_in != c:
                L.append(LayerSpec(CONV, ACT_NONE, c_in, c, h, h, stride, ksize=1, pad=0, src=x_idx))
                L.append(LayerSpec(ADD, ACT_RELU, c, c, h2, h2, src=main_idx, src2=len(L)))
            else:
                L.append(LayerSpec(ADD, ACT_RELU, c, c, h2, h2, src2=x_idx))
            c_in, h = c, h2
    L.append(LayerSpec(GAP, ACT_NONE, c_in, c_in, h, h))
    L.append(LayerSpec(FC, ACT_NONE, c_in, classes))
    return L


def uniform_ids(n_tenants: int, n_requests: int, *key) -> np.ndarray:
    return _rng(*key, 7001).integers(0, n_tenants, size=n_requests).astype(np.int32)


def zipf_ids(n_tenants: int, n_requests: int, s: float, *key) -> np.ndarray:
    rng = _rng(*key, 7002)
    p = np.arange(1, n_tenants + 1, dtype=np.float64) ** (-s)
    p /= p.sum()
    rank_to_tenant = rng.permutation(n_tenants)
    ranks = rng.choice(n_tenants, size=n_requests, p=p)
    return rank_to_tenant[ranks].astype(np.int32)


def _inputs(kind: str, shape, dtype: str, *key) -> np.ndarray:
    rng = _rng(*key, 7003)
    if kind == "normal":
        x = rng.standard_normal(shape, dtype=np.float32)
    else:
        x = rng.random(shape, dtype=np.float32)
    return round_to_bf16(x) if dtype == "bf16" else x


# ---- the five mixes (sizes can be overridden to get reduced test cases) -----
def c1(n_tenants=4, n_requests=64, dims=(256, 512, 512, 10), seed=1) -> Workload:
    tenants = {t: make_model(mlp_layers(list(dims), ACT_RELU), "f32", seed, t) for t in range(n_tenants)}
    return Workload("c1", "f32", tenants, uniform_ids(n_tenants, n_requests, seed),
                    _inputs("normal", (n_requests, dims[0]), "f32", seed))


def c2(n_tenants=64, n_requests=4096, dims=(784, 1024, 1024, 10), s=1.1, seed=2) -> Workload:
    tenants = {t: make_model(mlp_layers(list(dims), ACT_RELU), "bf16", seed, t) for t in range(n_tenants)}
    return Workload("c2", "bf16", tenants, zipf_ids(n_tenants, n_requests, s, seed),
                    _inputs("uniform", (n_requests, dims[0]), "bf16", seed))


def c3(n_tenants=256, n_requests=16384, in_dim=1024, widths=(512, 1024, 2048), classes=100,
       depth_lo=2, depth_hi=6, s=1.2, seed=3) -> Workload:
    rng = _rng(seed, 7004)
    tenants = {}
    for t in range(n_tenants):
        depth = int(rng.integers(depth_lo, depth_hi + 1))
        hidden = [int(widths[i]) for i in rng.integers(0, len(widths), size=depth - 1)]
        tenants[t] = make_model(mlp_layers([in_dim, *hidden, classes], ACT_RELU), "bf16", seed, t)
    return Workload("c3", "bf16", tenants, zipf_ids(n_tenants, n_requests, s, seed),
                    _inputs("normal", (n_requests, in_dim), "bf16", seed))


def c4(n_tenants=32, n_requests=2048, hw=32, chans=(3, 32, 64, 128), strides=(1, 2, 2), classes=10,
       seed=4) -> Workload:
    tenants = {t: make_model(cnn_layers(hw, chans, strides, classes), "bf16", seed, t)
               for t in range(n_tenants)}
    return Workload("c4", "bf16", tenants, uniform_ids(n_tenants, n_requests, seed),
                    _inputs("normal", (n_requests, hw * hw * chans[0]), "bf16", seed))


def c5(n_tenants=8, n_requests=32768, dims=(4096, 4096, 4096, 4096, 1000), seed=5) -> Workload:
    tenants = {t: make_model(mlp_layers(list(dims), ACT_GELU), "bf16", seed, t) for t in range(n_tenants)}
    return Workload("c5", "bf16", tenants, uniform_ids(n_tenants, n_requests, seed),
                    _inputs("normal", (n_requests, dims[0]), "bf16", seed))


def resnet(n_tenants=4, n_requests=64, hw=32, widths=(64, 128, 256, 512), classes=1000, dtype="bf16", seed=6) -> Workload:
    """Tenants with resnet18-shaped models (synthetic weights; the trained ones are not available
    offline), batch normalisation behind every convolution, requests uniform over tenants."""
    tenants = {t: with_batchnorm(make_model(resnet18_layers(hw, 3, widths, classes), dtype, seed, t), seed, t)
               for t in range(n_tenants)}
    return Workload("resnet18-shaped", dtype, tenants, uniform_ids(n_tenants, n_requests, seed),
                    _inputs("normal", (n_requests, hw * hw * 3), dtype, seed))


def r18(n_tenants=4, n_requests=64, seed=6) -> Workload:
    """The paper's running example as a multi-tenant mix: resnet18-shaped models (224x224x3 images, 64..512
    channels, 1000 classes, ~1.8 GFLOP per request) of several tenants, each with weights of its own."""
    w = resnet(n_tenants, n_requests, 224, (64, 128, 256, 512), 1000, "bf16", seed)
    w.name = "r18"
    return w


CONFIGS = {"r18": r18, "c1": c1, "c2": c2, "c3": c3, "c4": c4, "c5": c5}


# ---- algorithmic cost of a run (exact flops are known a priori: section 3.2) -
def algorithmic_cost(w: Workload) -> dict:
    """Flops (2*M*K*N with true dims; conv counts all 9 taps) and bytes under the model:
    inputs read once, every hidden activation written once and read once, every ACTIVE
    tenant's weights and biases read once, logits/probs/labels written once."""
    es = 4 if w.dtype == "f32" else 2
    flops = 0
    wbytes = abytes = obytes = 0
    for t, m_t in w.counts().items():
        model = w.tenants[t]
        for li, l in enumerate(model.layers):
            if l.kind == FC:
                flops += 2 * m_t * l.in_features * l.out_features
            elif l.kind == CONV:
                oh, ow = l.out_hw()
                flops += 2 * m_t * oh * ow * l.ksize * l.ksize * l.in_features * l.out_features
            if model.weights[li] is not None:
                wbytes += model.weights[li].size * es + model.biases[li].size * 4
            if li == 0:
                abytes += m_t * l.in_len() * es
            if li < len(model.layers) - 1:
                abytes += 2 * m_t * l.out_len() * es
            else:
                obytes += m_t * (2 * l.out_len() * 4 + 4)
    return {"flops": int(flops), "weight_bytes": int(wbytes), "act_bytes": int(abytes),
            "out_bytes": int(obytes), "bytes": int(wbytes + abytes + obytes)}
