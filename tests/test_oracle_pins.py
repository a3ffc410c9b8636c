"""Pins for the fp64 reference evaluator: closed forms, invariants, library special
cases and hand arithmetic, chosen so that a dropped term, a wrong index or a
transposed operand anywhere in it fails at least one of them.  CPU only."""
import math

import numpy as np
import pytest
import scipy.signal
import scipy.special
import torch

import oracle
from oracle import ACT_GELU, ACT_NONE, ACT_RELU, CONV, FC, GAP, Layer, Model

rng = np.random.default_rng(12345)


def mlp(dims, act, weights=None, biases=None, bf16=False):
    L = [Layer(FC, act if i < len(dims) - 2 else ACT_NONE, dims[i], dims[i + 1]) for i in range(len(dims) - 1)]
    if weights is None:
        weights = [rng.standard_normal((dims[i + 1], dims[i])) / math.sqrt(dims[i]) for i in range(len(dims) - 1)]
    if biases is None:
        biases = [0.1 * rng.standard_normal(dims[i + 1]) for i in range(len(dims) - 1)]
    return Model(L, weights, biases, round_bf16=bf16)


# ---- bf16 rounding -----------------------------------------------------------
def test_bf16_roundtrip_all_patterns():
    bits = np.arange(65536, dtype=np.uint32)
    vals = (bits << 16).astype(np.uint32).view(np.float32)
    finite = np.isfinite(vals)
    r = oracle.round_bf16(vals[finite].astype(np.float64))
    assert np.array_equal(r, vals[finite].astype(np.float64))


def test_bf16_ties_to_even():
    assert oracle.round_bf16(1 + 2.0 ** -8) == 1.0                 # halfway, even is below
    assert oracle.round_bf16(1 + 3 * 2.0 ** -8) == 1 + 2.0 ** -6   # halfway, even is above
    assert oracle.round_bf16(1 + 2.0 ** -8 + 2.0 ** -30) == 1 + 2.0 ** -7
    assert oracle.round_bf16(-(1 + 2.0 ** -8)) == -1.0
    assert oracle.round_bf16(2.0 ** -133 * 1.5) == 2.0 ** -132      # subnormal spacing 2^-133, tie -> even
    assert oracle.round_bf16(2.0 ** -134) == 0.0                    # half of the smallest subnormal -> even (0)
    assert np.isinf(oracle.round_bf16(3.4e38))
    assert oracle.round_bf16(0.0) == 0.0


def test_bf16_matches_library_conversion():
    x = np.concatenate([rng.standard_normal(20000).astype(np.float32) * 10.0 ** rng.integers(-20, 20, 20000),
                        rng.standard_normal(2000).astype(np.float32) * np.float32(1e-39)]).astype(np.float32)
    lib = torch.from_numpy(x).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(oracle.round_bf16(x.astype(np.float64)), lib)


# ---- activations -------------------------------------------------------------
def test_gelu_identities():
    x = np.linspace(-6, 6, 241)
    g = oracle.act(x, ACT_GELU)
    assert oracle.act(0.0, ACT_GELU) == 0.0
    assert np.allclose(g - oracle.act(-x, ACT_GELU), x, atol=1e-14)
    assert abs(float(oracle.act(12.0, ACT_GELU)) - 12.0) < 1e-14
    assert np.allclose(g, x * scipy.special.ndtr(x), atol=1e-14)   # x * Phi(x), library normal CDF
    assert math.isclose(float(oracle.act(1.0, ACT_GELU)), 0.8413447460685429, rel_tol=1e-14)


def test_relu_and_none():
    x = np.array([-2.0, -0.0, 0.0, 3.5])
    assert np.array_equal(oracle.act(x, ACT_RELU), np.array([0.0, 0.0, 0.0, 3.5]))
    assert np.array_equal(oracle.act(x, ACT_NONE), x)


# ---- fully-connected ----------------------------------------------------------
def test_fc_identity_and_orientation():
    K = 7
    x = rng.standard_normal(K)
    m = mlp([K, K, K], ACT_NONE, [np.eye(K), np.eye(K)], [np.zeros(K), np.zeros(K)])
    lg, _, _, _ = oracle.forward_one(m, x)
    assert np.array_equal(lg, x)
    m = mlp([K, K, K], ACT_RELU, [np.eye(K), np.eye(K)], [np.zeros(K), np.zeros(K)])
    lg, _, _, _ = oracle.forward_one(m, x)
    assert np.array_equal(lg, np.maximum(x, 0))
    # W is [N][K]: a single 1 at W[n=2][k=5] moves x[5] to z[2] (a transposed read would move x[2] to z[5])
    W = np.zeros((4, 6)); W[2, 5] = 1.0
    z = oracle.fc(Layer(FC, ACT_NONE, 6, 4), W, None, np.arange(6.0))
    assert np.array_equal(z, np.array([0, 0, 5.0, 0]))


def test_fc_matches_library_matmul():
    K, N = 37, 23
    W = rng.standard_normal((N, K)); b = rng.standard_normal(N); x = rng.standard_normal(K)
    z = oracle.fc(Layer(FC, ACT_NONE, K, N), W, b, x)
    assert np.allclose(z, W @ x + b, rtol=0, atol=1e-12)


def test_relu_of_known_affine_map():
    a = np.array([2.0, -1.0, 0.5, 3.0]); b = np.array([-1.0, 0.25, -2.0, 0.0])
    x = np.array([1.0, 2.0, 3.0, -4.0])
    m = mlp([4, 4, 4], ACT_RELU, [np.diag(a), np.eye(4)], [b, np.zeros(4)])
    lg, _, _, _ = oracle.forward_one(m, x)
    assert np.array_equal(lg, np.maximum(a * x + b, 0.0))           # bias is added before the activation
    assert np.array_equal(lg, np.array([1.0, 0.0, 0.0, 0.0]))


def test_zero_weights_give_bias_and_uniform_probs():
    m = mlp([5, 6, 4], ACT_RELU, [np.zeros((6, 5)), np.zeros((4, 6))], [np.zeros(6), np.array([0.1, 0.7, -0.3, 0.7])])
    lg, pr, lb, _ = oracle.forward_one(m, rng.standard_normal(5))
    assert np.array_equal(lg, np.array([0.1, 0.7, -0.3, 0.7]))
    assert lb == 1                                                   # lowest index among equal maxima
    m.biases = [np.zeros(6), np.zeros(4)]; m._w64 = []
    lg, pr, lb, _ = oracle.forward_one(m, rng.standard_normal(5))
    assert np.array_equal(pr, np.full(4, 0.25)) and lb == 0


def test_linearity():
    m = mlp([9, 11, 6], ACT_NONE, biases=[np.zeros(11), np.zeros(6)])
    x, y = rng.standard_normal(9), rng.standard_normal(9)
    f = lambda v: oracle.forward_one(m, v)[0]
    assert np.allclose(f(2.5 * x - 0.75 * y), 2.5 * f(x) - 0.75 * f(y), rtol=0, atol=1e-12)


def test_hand_computed_two_tenant_three_neuron_nets():
    # tenant 0: 2 -> 3 (ReLU) -> 2
    W1 = np.array([[1.0, -1.0], [0.5, 0.5], [-2.0, 1.0]]); b1 = np.array([0.0, -1.0, 0.5])
    W2 = np.array([[1.0, 2.0, -1.0], [0.0, -1.0, 1.0]]); b2 = np.array([0.25, -0.5])
    t0 = Model([Layer(FC, ACT_RELU, 2, 3), Layer(FC, ACT_NONE, 3, 2)], [W1, W2], [b1, b2])
    # tenant 1: 2 -> 3 (no activation) -> 3
    V1 = np.array([[2.0, 0.0], [0.0, -1.0], [1.0, 1.0]]); c1 = np.array([1.0, 1.0, -1.0])
    V2 = np.array([[1.0, 0.0, 0.0], [0.0, 1.0, 0.0], [1.0, 1.0, 1.0]]); c2 = np.array([0.0, 0.0, 0.5])
    t1 = Model([Layer(FC, ACT_NONE, 2, 3), Layer(FC, ACT_NONE, 3, 3)], [V1, V2], [c1, c2])
    xa, xb = np.array([3.0, 1.0]), np.array([-1.0, 2.0])
    # by hand, tenant 0 on xa: z1 = [2, 1, -4.5] -> h = [2, 1, 0] -> logits = [4.25, -1.5]
    # by hand, tenant 0 on xb: z1 = [-3, -0.5, 4.5] -> h = [0, 0, 4.5] -> logits = [-4.25, 4.0]
    # by hand, tenant 1 on xa: h = [7, 0, 3] -> logits = [7, 0, 10.5]
    # by hand, tenant 1 on xb: h = [-1, -1, 0] -> logits = [-1, -1, -1.5]
    lg, pr, lb, nc, macs = oracle.run_batch({0: t0, 1: t1}, [1, 0, 0, 1], np.stack([xa, xa, xb, xb]))
    assert np.array_equal(lg, np.array([[7, 0, 10.5], [4.25, -1.5, 0], [-4.25, 4.0, 0], [-1, -1, -1.5]]))
    assert list(lb) == [2, 0, 1, 0] and list(nc) == [3, 2, 2, 3]
    e = np.exp(np.array([4.25, -1.5]) - 4.25)
    assert np.allclose(pr[1, :2], e / e.sum(), atol=1e-15) and pr[1, 2] == 0
    assert macs == 2 * (6 + 6) + 2 * (6 + 9)


def test_permutation_invariance_and_batch_independence():
    models = {t: mlp([8, 12, 5], ACT_RELU) for t in range(3)}
    ids = rng.integers(0, 3, 20); X = rng.standard_normal((20, 8))
    lg, pr, lb, _, _ = oracle.run_batch(models, ids, X)
    p = rng.permutation(20)
    lg2, pr2, lb2, _, _ = oracle.run_batch(models, ids[p], X[p])
    assert np.array_equal(lg2, lg[p]) and np.array_equal(pr2, pr[p]) and np.array_equal(lb2, lb[p])
    relabel = {0: 2, 1: 0, 2: 1}
    lg3, _, lb3, _, _ = oracle.run_batch({relabel[t]: m for t, m in models.items()},
                                         np.array([relabel[int(t)] for t in ids]), X)
    assert np.array_equal(lg3, lg) and np.array_equal(lb3, lb)
    for i in (0, 7, 19):                                            # stateless: alone == in the batch
        one = oracle.forward_one(models[int(ids[i])], X[i])
        assert np.array_equal(one[0], lg[i]) and one[2] == lb[i]
    lgt, _, _, _ = oracle.forward(models[0], X, threads=4)          # threading changes nothing
    lgs, _, _, _ = oracle.forward(models[0], X, threads=1)
    assert np.array_equal(lgt, lgs)


def test_layer_prefix_and_rounding_points():
    m = mlp([16, 24, 20, 6], ACT_RELU, bf16=True)
    x = rng.standard_normal(16)
    lg, _, _, _, hid = oracle.forward_one(m, x, want_hidden=True)
    xq = oracle.round_bf16(x)
    h1 = oracle.round_bf16(np.maximum(m.weights[0] @ xq + m.biases[0], 0))
    h2 = oracle.round_bf16(np.maximum(m.weights[1] @ h1 + m.biases[1], 0))
    assert np.allclose(hid[:24], h1, atol=1e-12) and np.allclose(hid[24:], h2, atol=1e-12)
    assert np.allclose(lg, m.weights[2] @ h2 + m.biases[2], atol=1e-12)
    # hidden activations are representable in bf16; logits are not rounded
    assert np.array_equal(oracle.round_bf16(hid), hid)
    assert not np.array_equal(oracle.round_bf16(lg), lg)
    prefix = Model(m.layers[:2], m.weights[:2], m.biases[:2], round_bf16=True)
    prefix.layers[-1] = Layer(FC, ACT_NONE, 24, 20)
    lgp, _, _, _ = oracle.forward_one(prefix, x)
    assert np.allclose(oracle.round_bf16(np.maximum(lgp, 0)), hid[24:], atol=0)


def test_mac_counter_equals_closed_form():
    m = mlp([13, 17, 19, 5], ACT_RELU)
    _, _, _, macs = oracle.forward(m, rng.standard_normal((7, 13)))
    assert macs == 7 * (13 * 17 + 17 * 19 + 19 * 5) == 7 * m.macs_per_request()
    cnn = Model([Layer(CONV, ACT_RELU, 2, 3, 5, 4, 2), Layer(GAP, ACT_NONE, 3, 3, 3, 2), Layer(FC, ACT_NONE, 3, 2)],
                [rng.standard_normal((3, 2, 3, 3)), None, rng.standard_normal((2, 3))],
                [rng.standard_normal(3), None, rng.standard_normal(2)])
    _, _, _, macs = oracle.forward_one(cnn, rng.standard_normal(5 * 4 * 2))
    assert macs == cnn.macs_per_request()


# ---- head ------------------------------------------------------------------------
def test_softmax_properties():
    z = rng.standard_normal(11) * 5
    p, lb = oracle.head(z)
    assert abs(p.sum() - 1) < 1e-15 and np.all(p >= 0) and lb == int(np.argmax(z))
    p2, lb2 = oracle.head(z + 123.0)
    assert np.allclose(p, p2, atol=1e-13) and lb == lb2
    assert np.allclose(p, scipy.special.softmax(z), atol=1e-15)
    p3, _ = oracle.head(np.array([1000.0, 0.0]))                    # stable: no overflow
    assert p3[0] == 1.0 and p3[1] == 0.0


# ---- convolution -----------------------------------------------------------------
def test_conv_delta_kernel():
    C, H, W = 3, 6, 5
    x = rng.standard_normal((H, W, C))
    Wd = np.zeros((C, C, 3, 3))
    for c in range(C):
        Wd[c, c, 1, 1] = 1.0
    assert np.array_equal(oracle.conv(Layer(CONV, ACT_NONE, C, C, H, W, 1), Wd, None, x), x)
    y2 = oracle.conv(Layer(CONV, ACT_NONE, C, C, H, W, 2), Wd, None, x)
    assert np.array_equal(y2, x[::2, ::2])
    # off-centre tap: kernel[kh=0,kw=2] reads the pixel one row up and one column right
    Ws = np.zeros((1, 1, 3, 3)); Ws[0, 0, 0, 2] = 1.0
    img = np.arange(12.0).reshape(3, 4, 1)
    y = oracle.conv(Layer(CONV, ACT_NONE, 1, 1, 3, 4, 1), Ws, None, img)[..., 0]
    exp = np.zeros((3, 4)); exp[1:, :3] = img[:2, 1:, 0]
    assert np.array_equal(y, exp)


def test_conv_all_ones_counts_padding():
    Ci, Co, H, W = 4, 2, 5, 6
    y = oracle.conv(Layer(CONV, ACT_NONE, Ci, Co, H, W, 1), np.ones((Co, Ci, 3, 3)), None, np.ones((H, W, Ci)))
    assert np.all(y[1:-1, 1:-1] == 9 * Ci)
    assert np.all(y[0, 1:-1] == 6 * Ci) and np.all(y[1:-1, 0] == 6 * Ci)
    assert y[0, 0, 0] == 4 * Ci and y[-1, -1, 1] == 4 * Ci


@pytest.mark.parametrize("stride", [1, 2])
def test_conv_matches_library_correlation_and_im2col(stride):
    Ci, Co, H, W = 3, 4, 9, 8
    x = rng.standard_normal((H, W, Ci)); Wt = rng.standard_normal((Co, Ci, 3, 3)); b = rng.standard_normal(Co)
    L = Layer(CONV, ACT_NONE, Ci, Co, H, W, stride)
    y = oracle.conv(L, Wt, b, x)
    ref = np.zeros((H, W, Co))
    for co in range(Co):
        for ci in range(Ci):
            ref[..., co] += scipy.signal.correlate2d(x[..., ci], Wt[co, ci], mode="same", boundary="fill")
        ref[..., co] += b[co]
    assert np.allclose(y, ref[::stride, ::stride], atol=1e-12)
    assert y.shape == ((H + 2 - 3) // stride + 1, (W + 2 - 3) // stride + 1, Co)
    y2 = oracle.conv(L, Wt, b, x, via_im2col=True)
    assert np.allclose(y, y2, atol=1e-12)


def test_gap_closed_forms():
    C, H, W = 5, 4, 3
    L = Layer(GAP, ACT_NONE, C, C, H, W)
    assert np.array_equal(oracle.gap(L, np.full((H, W, C), 2.5)), np.full(C, 2.5))
    x = rng.standard_normal((H, W, C))
    assert np.allclose(oracle.gap(L, x), x.mean(axis=(0, 1)), atol=1e-15)
    Wf = rng.standard_normal((3, C)); bf = rng.standard_normal(3)
    m = Model([L, Layer(FC, ACT_NONE, C, 3)], [None, Wf], [None, bf])
    lg, _, _, _ = oracle.forward_one(m, x)
    assert np.allclose(lg, (Wf / (H * W)) @ x.sum(axis=(0, 1)) + bf, atol=1e-13)


def test_cnn_end_to_end_against_composition():
    layers = [Layer(CONV, ACT_RELU, 3, 4, 8, 8, 1), Layer(CONV, ACT_RELU, 4, 6, 8, 8, 2),
              Layer(GAP, ACT_NONE, 6, 6, 4, 4), Layer(FC, ACT_NONE, 6, 3)]
    ws = [rng.standard_normal((4, 3, 3, 3)) / 5, rng.standard_normal((6, 4, 3, 3)) / 6, None, rng.standard_normal((3, 6))]
    bs = [rng.standard_normal(4) / 10, rng.standard_normal(6) / 10, None, rng.standard_normal(3) / 10]
    m = Model(layers, ws, bs, round_bf16=True)
    x = rng.standard_normal(8 * 8 * 3)
    lg, pr, lb, _ = oracle.forward_one(m, x)
    q = oracle.round_bf16
    h = q(x).reshape(8, 8, 3)
    h = q(np.maximum(oracle.conv(layers[0], ws[0], bs[0], h), 0))
    h = q(np.maximum(oracle.conv(layers[1], ws[1], bs[1], h), 0))
    h = q(h.mean(axis=(0, 1)))
    assert np.allclose(lg, ws[3] @ h + bs[3], atol=1e-12)
