"""Python face of the fp64 reference evaluator in ``mt_oracle.c``.

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by the smoke check and by the
benchmark's CPU-baseline leg.  The product package never imports it, and this
module never imports the product package.

A model is described the way the paper's primer (section 1.1) describes a DNN:
an ordered list of layers plus, per layer, the stored tensor of learned values.
``forward`` evaluates requests one by one, each through its own model, layer by
layer; ``run_batch`` does so for a mixed-tenant batch and returns predictions
in submission order (section 3: tenants upload a DNN, then send requests).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "mt_oracle.c")
_LIB = os.path.join(_HERE, "libmt_oracle.so")

FC, CONV, GAP, MAXPOOL, ADD = 0, 1, 2, 3, 4
ACT_NONE, ACT_RELU, ACT_GELU = 0, 1, 2


class _CLayer(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("kind", "act", "in_features", "out_features", "in_h", "in_w", "stride", "ksize", "pad", "src", "src2")]


def build(force: bool = False) -> str:
    """Compile the C source with gcc (plain -O2, no fast-math) and return the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-pthread",
                               "-fno-fast-math", "-ffp-contract=off", "-o", _LIB, _SRC, "-lm"])
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        L = ctypes.CDLL(build())
        dp = ctypes.POINTER(ctypes.c_double)
        dpp = ctypes.POINTER(dp)
        lp = ctypes.POINTER(_CLayer)
        ip = ctypes.POINTER(ctypes.c_int32)
        L.orc_round_bf16.restype = ctypes.c_double
        L.orc_round_bf16.argtypes = [ctypes.c_double]
        L.orc_act.restype = ctypes.c_double
        L.orc_act.argtypes = [ctypes.c_double, ctypes.c_int]
        L.orc_layer_out_len.restype = ctypes.c_int
        L.orc_layer_out_len.argtypes = [lp]
        L.orc_layer_in_len.restype = ctypes.c_int
        L.orc_layer_in_len.argtypes = [lp]
        for name in ("orc_fc", "orc_conv", "orc_conv_via_im2col"):
            f = getattr(L, name)
            f.restype = ctypes.c_uint64
            f.argtypes = [lp, dp, dp, dp, dp]
        L.orc_gap.restype = None
        L.orc_gap.argtypes = [lp, dp, dp]
        L.orc_maxpool.restype = None
        L.orc_maxpool.argtypes = [lp, dp, dp]
        L.orc_add.restype = None
        L.orc_add.argtypes = [lp, dp, dp, dp]
        L.orc_fold_bn.restype = None
        L.orc_fold_bn.argtypes = [dp, dp, ctypes.c_int, ctypes.c_int, dp, dp, dp, dp, ctypes.c_double, ctypes.c_int]
        L.orc_head.restype = None
        L.orc_head.argtypes = [dp, ctypes.c_int, dp, ip]
        L.orc_forward_one.restype = ctypes.c_uint64
        L.orc_forward_one.argtypes = [lp, ctypes.c_int, dpp, dpp, ctypes.c_int, dp, dp, dp, ip, dp]
        L.orc_forward_rows.restype = ctypes.c_uint64
        L.orc_forward_rows.argtypes = [lp, ctypes.c_int, dpp, dpp, ctypes.c_int, dp, ctypes.c_int,
                                       ctypes.c_int, dp, dp, ip]
        _lib = L
    return _lib


def _dp(a: Optional[np.ndarray]):
    if a is None:
        return ctypes.POINTER(ctypes.c_double)()
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


@dataclass
class Layer:
    kind: int
    act: int = ACT_NONE
    in_features: int = 0
    out_features: int = 0
    in_h: int = 0
    in_w: int = 0
    stride: int = 1
    ksize: int = 3            # CONV / MAXPOOL window (k x k)
    pad: int = 1              # CONV / MAXPOOL padding
    src: int = 0              # j + 1: this layer reads the output of layer j; 0: the previous layer
    src2: int = 0             # ADD: the second operand, same convention

    def c(self) -> _CLayer:
        return _CLayer(self.kind, self.act, self.in_features, self.out_features,
                       self.in_h, self.in_w, self.stride, self.ksize, self.pad, self.src, self.src2)

    def out_hw(self):
        return ((self.in_h + 2 * self.pad - self.ksize) // self.stride + 1,
                (self.in_w + 2 * self.pad - self.ksize) // self.stride + 1)

    def in_len(self) -> int:
        return int(lib().orc_layer_in_len(ctypes.byref(self.c())))

    def out_len(self) -> int:
        return int(lib().orc_layer_out_len(ctypes.byref(self.c())))


@dataclass
class Model:
    """layers[l] with weights[l] (FC: [N,K]; CONV: [Co,Ci,k,k]; GAP, MAXPOOL, ADD: None) and biases[l]."""
    layers: List[Layer]
    weights: List[Optional[np.ndarray]]
    biases: List[Optional[np.ndarray]]
    round_bf16: bool = False
    _w64: list = field(default_factory=list, repr=False)
    _b64: list = field(default_factory=list, repr=False)

    def _prep(self):
        if not self._w64:
            self._w64 = [None if w is None else np.ascontiguousarray(w, dtype=np.float64)
                         for w in self.weights]
            self._b64 = [None if b is None else np.ascontiguousarray(b, dtype=np.float64)
                         for b in self.biases]
        n = len(self.layers)
        larr = (_CLayer * n)(*[l.c() for l in self.layers])
        dp = ctypes.POINTER(ctypes.c_double)
        warr = (dp * n)(*[_dp(w) for w in self._w64])
        barr = (dp * n)(*[_dp(b) for b in self._b64])
        return larr, warr, barr

    @property
    def in_len(self) -> int:
        return self.layers[0].in_len()

    @property
    def n_classes(self) -> int:
        return self.layers[-1].out_len()

    def macs_per_request(self) -> int:
        """Closed-form multiply-accumulate count of one request (the paper, section 3.2: the
        exact number of flops of each layer is known a priori).  Padding taps of a
        convolution are not counted, matching what the loop nest really multiplies."""
        total = 0
        for l in self.layers:
            if l.kind == FC:
                total += l.in_features * l.out_features
            elif l.kind == CONV:
                s = l.stride
                oh, ow = l.out_hw()
                taps_h = sum(1 for o in range(oh) for k in range(l.ksize) if 0 <= o * s + k - l.pad < l.in_h)
                taps_w = sum(1 for o in range(ow) for k in range(l.ksize) if 0 <= o * s + k - l.pad < l.in_w)
                total += taps_h * taps_w * l.in_features * l.out_features
        return total


def round_bf16(x) -> np.ndarray:
    f = lib().orc_round_bf16
    return np.vectorize(lambda v: f(float(v)), otypes=[np.float64])(np.asarray(x, dtype=np.float64))


def act(x, kind: int) -> np.ndarray:
    f = lib().orc_act
    return np.vectorize(lambda v: f(float(v), kind), otypes=[np.float64])(np.asarray(x, dtype=np.float64))


def fc(layer: Layer, W, b, h) -> np.ndarray:
    W = np.ascontiguousarray(W, dtype=np.float64)
    b = None if b is None else np.ascontiguousarray(b, dtype=np.float64)
    h = np.ascontiguousarray(h, dtype=np.float64)
    z = np.empty(layer.out_features, dtype=np.float64)
    lib().orc_fc(ctypes.byref(layer.c()), _dp(W), _dp(b), _dp(h), _dp(z))
    return z


def conv(layer: Layer, W, b, h, via_im2col: bool = False) -> np.ndarray:
    W = np.ascontiguousarray(W, dtype=np.float64)
    b = None if b is None else np.ascontiguousarray(b, dtype=np.float64)
    h = np.ascontiguousarray(h, dtype=np.float64)
    z = np.empty(layer.out_len(), dtype=np.float64)
    fn = lib().orc_conv_via_im2col if via_im2col else lib().orc_conv
    fn(ctypes.byref(layer.c()), _dp(W), _dp(b), _dp(h), _dp(z))
    oh, ow = layer.out_hw()
    return z.reshape(oh, ow, layer.out_features)


def maxpool(layer: Layer, h) -> np.ndarray:
    h = np.ascontiguousarray(h, dtype=np.float64)
    z = np.empty(layer.out_len(), dtype=np.float64)
    lib().orc_maxpool(ctypes.byref(layer.c()), _dp(h), _dp(z))
    oh, ow = layer.out_hw()
    return z.reshape(oh, ow, layer.in_features)


def add(layer: Layer, a, b) -> np.ndarray:
    a = np.ascontiguousarray(a, dtype=np.float64)
    b = np.ascontiguousarray(b, dtype=np.float64)
    z = np.empty(layer.out_len(), dtype=np.float64)
    lib().orc_add(ctypes.byref(layer.c()), _dp(a), _dp(b), _dp(z))
    return z.reshape(layer.in_h, layer.in_w, layer.in_features)


def fold_bn(W, b, gamma, beta, mean, var, eps: float, to_bf16: bool):
    """Filters [Co, ...] and bias [Co] of a convolution with the batch normalisation behind it folded in
    (fp64 arithmetic, filters rounded once to bfloat16 or fp32, bias to fp32).  Returns new arrays."""
    W2 = np.array(W, dtype=np.float64, order="C", copy=True)
    Co = W2.shape[0]
    b2 = np.zeros(Co) if b is None else np.array(b, dtype=np.float64, copy=True)
    g, be, mu, va = (np.ascontiguousarray(v, dtype=np.float64) for v in (gamma, beta, mean, var))
    lib().orc_fold_bn(_dp(W2), _dp(b2), Co, int(W2.size // Co), _dp(g), _dp(be), _dp(mu), _dp(va), float(eps), int(to_bf16))
    return W2, b2


def gap(layer: Layer, h) -> np.ndarray:
    h = np.ascontiguousarray(h, dtype=np.float64)
    z = np.empty(layer.in_features, dtype=np.float64)
    lib().orc_gap(ctypes.byref(layer.c()), _dp(h), _dp(z))
    return z


def head(logits):
    logits = np.ascontiguousarray(logits, dtype=np.float64)
    probs = np.empty_like(logits)
    label = ctypes.c_int32(0)
    lib().orc_head(_dp(logits), logits.size, _dp(probs), ctypes.byref(label))
    return probs, int(label.value)


def forward_one(model: Model, x, want_hidden: bool = False):
    """One request.  Returns (logits, probs, label, macs[, hidden])."""
    larr, warr, barr = model._prep()
    x = np.ascontiguousarray(x, dtype=np.float64).reshape(-1)
    assert x.size == model.in_len
    C = model.n_classes
    logits = np.empty(C); probs = np.empty(C); label = ctypes.c_int32(0)
    hidden = None
    if want_hidden:
        hidden = np.zeros(sum(l.out_len() for l in model.layers[:-1]), dtype=np.float64)
    macs = lib().orc_forward_one(larr, len(model.layers), warr, barr, int(model.round_bf16),
                                 _dp(x), _dp(logits), _dp(probs), ctypes.byref(label), _dp(hidden))
    out = (logits, probs, int(label.value), int(macs))
    return out + (hidden,) if want_hidden else out


def forward(model: Model, X, threads: int = 1):
    """Rows of X through one model.  Returns (logits [M,C], probs [M,C], labels [M], macs)."""
    larr, warr, barr = model._prep()
    X = np.ascontiguousarray(X, dtype=np.float64).reshape(-1, model.in_len)
    M, C = X.shape[0], model.n_classes
    logits = np.empty((M, C)); probs = np.empty((M, C)); labels = np.empty(M, dtype=np.int32)
    macs = lib().orc_forward_rows(larr, len(model.layers), warr, barr, int(model.round_bf16),
                                  _dp(X), M, threads, _dp(logits), _dp(probs),
                                  labels.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)))
    return logits, probs, labels, int(macs)


def run_batch(models: Dict[int, Model], tenant_ids: Sequence[int], inputs, threads: int = 1):
    """Mixed-tenant batch in submission order.

    ``inputs`` is [R, in_len] (all models must share in_len) or a list of per-request
    vectors.  Returns (logits [R,Cmax], probs [R,Cmax], labels [R], n_classes [R], macs); columns
    past a request's class count are zero.
    """
    tenant_ids = np.asarray(tenant_ids, dtype=np.int64)
    R = tenant_ids.size
    cmax = max((m.n_classes for m in models.values()), default=1)
    logits = np.zeros((R, cmax)); probs = np.zeros((R, cmax))
    labels = np.full(R, -1, dtype=np.int32); ncls = np.zeros(R, dtype=np.int32)
    macs = 0
    for t in np.unique(tenant_ids):
        m = models[int(t)]
        idx = np.nonzero(tenant_ids == t)[0]
        if isinstance(inputs, np.ndarray):
            X = inputs[idx][:, :m.in_len]
        else:
            X = np.stack([np.asarray(inputs[i], dtype=np.float64).reshape(-1) for i in idx])
        lg, pr, lb, mc = forward(m, X, threads)
        logits[idx, :m.n_classes] = lg
        probs[idx, :m.n_classes] = pr
        labels[idx] = lb
        ncls[idx] = m.n_classes
        macs += mc
    return logits, probs, labels, ncls, macs


def models_from_workload(w) -> Dict[int, Model]:
    """Oracle models for a ``workloads.Workload`` (duck-typed: nothing is imported from it)."""
    out = {}
    for t, tm in w.tenants.items():
        layers = [Layer(l.kind, l.act, l.in_features, l.out_features, l.in_h, l.in_w, l.stride,
                        getattr(l, "ksize", 3), getattr(l, "pad", 1), getattr(l, "src", 0), getattr(l, "src2", 0))
                  for l in tm.layers]
        weights, biases = list(tm.weights), list(tm.biases)
        for i, bn in enumerate(getattr(tm, "bn", None) or []):
            if bn is not None:              # (gamma, beta, mean, var) behind convolution i: fold it
                weights[i], biases[i] = fold_bn(weights[i], biases[i], *bn, getattr(tm, "bn_eps", 1e-5), w.dtype == "bf16")
        out[int(t)] = Model(layers, weights, biases, round_bf16=(w.dtype == "bf16"))
    return out
