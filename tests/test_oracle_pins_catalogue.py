"""Pins for the wider layer catalogue of the fp64 reference evaluator (paper section 1.1: DNNs are
built from a few dozen layer types; section 3.1: the system supports a pre-defined set of them):
k x k convolutions (1x1, 7x7), max-pooling, residual additions with skip sources, and batch
normalisation folded into the convolution before it.  Closed forms, library routines, hand numbers and
compositions from single layers, chosen so that a wrong offset, a dropped tap, a swapped operand or a
wrong sign fails at least one of them.  CPU only."""
import numpy as np
import pytest
import scipy.ndimage
import scipy.signal

import oracle
from oracle import ACT_NONE, ACT_RELU, ADD, CONV, FC, GAP, MAXPOOL, Layer, Model

rng = np.random.default_rng(2468)


def conv_layer(ci, co, h, w, k, s, act=ACT_NONE, src=0):
    return Layer(CONV, act, ci, co, h, w, s, ksize=k, pad=(k - 1) // 2, src=src)


# ---- k x k convolution --------------------------------------------------------------------------
def test_conv1x1_is_a_matrix_product_per_pixel():
    L = conv_layer(5, 7, 6, 4, 1, 1)
    W, b, x = rng.standard_normal((7, 5, 1, 1)), rng.standard_normal(7), rng.standard_normal((6, 4, 5))
    z = oracle.conv(L, W, b, x)
    assert z.shape == (6, 4, 7)
    assert np.allclose(z, x @ W[:, :, 0, 0].T + b, atol=1e-13)
    z2 = oracle.conv(conv_layer(5, 7, 6, 4, 1, 2), W, b, x)        # stride 2: every other pixel, starting at (0, 0)
    assert z2.shape == (3, 2, 7) and np.allclose(z2, z[::2, ::2], atol=1e-13)


@pytest.mark.parametrize("k,s,h,w", [(7, 1, 9, 11), (7, 2, 12, 10), (7, 2, 7, 7), (3, 2, 9, 8), (1, 2, 5, 5)])
def test_conv_matches_library_correlation(k, s, h, w):
    ci, co = 3, 4
    L = conv_layer(ci, co, h, w, k, s)
    W, b, x = rng.standard_normal((co, ci, k, k)), rng.standard_normal(co), rng.standard_normal((h, w, ci))
    z = oracle.conv(L, W, b, x)
    p = (k - 1) // 2
    xp = np.pad(x, ((p, p), (p, p), (0, 0)))                        # zero padding, then a 'valid' correlation
    for c in range(co):
        full = sum(scipy.signal.correlate2d(xp[:, :, i], W[c, i], mode="valid") for i in range(ci)) + b[c]
        assert np.allclose(z[:, :, c], full[::s, ::s], atol=1e-12)
    assert np.allclose(oracle.conv(L, W, b, x, via_im2col=True), z, atol=1e-12)     # the second, independent loop nest


def test_conv7x7_delta_taps_and_all_ones_counts():
    h = w = 10
    x = rng.standard_normal((h, w, 2))
    W = np.zeros((2, 2, 7, 7)); W[0, 0, 3, 3] = W[1, 1, 3, 3] = 1.0                  # centre tap: identity
    assert np.array_equal(oracle.conv(conv_layer(2, 2, h, w, 7, 1), W, None, x), x)
    assert np.array_equal(oracle.conv(conv_layer(2, 2, h, w, 7, 2), W, None, x), x[::2, ::2])
    W = np.zeros((1, 2, 7, 7)); W[0, 1, 0, 6] = 1.0                                  # tap (kh 0, kw 6): input 3 up, 3 right
    z = oracle.conv(conv_layer(2, 1, h, w, 7, 1), W, None, x)[:, :, 0]
    want = np.zeros((h, w)); want[3:, :w - 3] = x[:h - 3, 3:, 1]
    assert np.array_equal(z, want)
    ones = oracle.conv(conv_layer(3, 1, h, w, 7, 1), np.ones((1, 3, 7, 7)), None, np.ones((h, w, 3)))[:, :, 0]
    assert ones[0, 0] == 16 * 3 and ones[0, 5] == 28 * 3 and ones[5, 5] == 49 * 3 and ones[9, 9] == 16 * 3 and ones[1, 2] == 5 * 6 * 3
    # the multiply-accumulate counter counts exactly the taps inside the image
    m = Model([conv_layer(3, 1, h, w, 7, 1, ACT_RELU), Layer(GAP, ACT_NONE, 1, 1, h, w), Layer(FC, ACT_NONE, 1, 2)],
              [np.ones((1, 3, 7, 7)), None, np.ones((2, 1))], [None, None, None])
    assert oracle.forward_one(m, np.ones(h * w * 3))[3] == int(ones.sum()) + 2 == m.macs_per_request()


# ---- max-pooling ---------------------------------------------------------------------------------
def test_maxpool_hand_numbers_and_padding_never_wins():
    x = np.array([[1, 5, 2, 0], [3, 4, 9, 1], [7, 0, 2, 2], [1, 8, 3, 6]], dtype=np.float64).reshape(4, 4, 1)
    L = Layer(MAXPOOL, ACT_NONE, 1, 1, 4, 4, 2, ksize=2, pad=0)
    assert np.array_equal(oracle.maxpool(L, x)[:, :, 0], [[5, 9], [8, 6]])
    L = Layer(MAXPOOL, ACT_NONE, 1, 1, 4, 4, 2, ksize=3, pad=1)               # windows centred on (0,0), (0,2), (2,0), (2,2)
    assert np.array_equal(oracle.maxpool(L, x)[:, :, 0], [[5, 9], [8, 9]])
    neg = np.full((5, 7, 2), -5.0)
    z = oracle.maxpool(Layer(MAXPOOL, ACT_NONE, 2, 2, 5, 7, 2, ksize=3, pad=1), neg)
    assert z.shape == (3, 4, 2) and np.all(z == -5.0)                        # zero (or any) padding would have won
    ramp = np.arange(6 * 6, dtype=np.float64).reshape(6, 6, 1)
    z = oracle.maxpool(Layer(MAXPOOL, ACT_NONE, 1, 1, 6, 6, 2, ksize=3, pad=1), ramp)[:, :, 0]
    assert np.array_equal(z, [[7, 9, 11], [19, 21, 23], [31, 33, 35]])        # bottom-right tap of every window


@pytest.mark.parametrize("k,s,p,h,w", [(3, 2, 1, 9, 12), (3, 1, 1, 5, 5), (2, 2, 0, 8, 6), (3, 2, 0, 7, 9)])
def test_maxpool_matches_library_maximum_filter(k, s, p, h, w):
    c = 3
    x = rng.standard_normal((h, w, c))
    L = Layer(MAXPOOL, ACT_NONE, c, c, h, w, s, ksize=k, pad=p)
    z = oracle.maxpool(L, x)
    oh, ow = (h + 2 * p - k) // s + 1, (w + 2 * p - k) // s + 1
    assert z.shape == (oh, ow, c)
    xp = np.pad(x, ((p, p + k), (p, p + k), (0, 0)), constant_values=-np.inf)
    # library filter with its window anchored at the top-left corner (origin shifts the centred window)
    full = scipy.ndimage.maximum_filter(xp, size=(k, k, 1), mode="constant", cval=-np.inf, origin=(-(k // 2), -(k // 2), 0))
    assert np.array_equal(z, full[:oh * s:s, :ow * s:s])


# ---- residual addition and skip sources ----------------------------------------------------------
def test_add_is_elementwise_and_takes_the_named_sources():
    L = Layer(ADD, ACT_RELU, 2, 2, 1, 2)
    assert np.array_equal(oracle.add(L, [1.0, -2.0, 3.0, 0.5], [0.5, 1.0, -4.0, 0.25]).reshape(-1), [1.5, -1.0, -1.0, 0.75])   # the sum; act is the model's
    h = w = 6
    ci, c = 3, 4
    layers = [conv_layer(ci, c, h, w, 3, 1, ACT_RELU),                 # 0: A
              conv_layer(c, c, h, w, 3, 1, ACT_RELU),                  # 1: B = conv(A)
              conv_layer(c, c, h, w, 3, 1, ACT_NONE),                  # 2: C = conv(B)
              Layer(ADD, ACT_RELU, c, c, h, w, src2=1),                # 3: relu(C + A): second operand is the output of layer 0
              conv_layer(c, c, h, w, 1, 2, ACT_NONE, src=2),           # 4: D = conv1x1 s2 of B (reads layer 1, not layer 3)
              conv_layer(c, c, h, w, 3, 2, ACT_NONE, src=4),           # 5: E = conv3x3 s2 of layer 3's output
              Layer(ADD, ACT_RELU, c, c, 3, 3, src2=5),                # 6: relu(E + D)
              Layer(GAP, ACT_NONE, c, c, 3, 3), Layer(FC, ACT_NONE, c, 5)]
    Ws = [rng.standard_normal((c, ci if i == 0 else c, k, k)) * 0.3 for i, k in ((0, 3), (1, 3), (2, 3))] + [None] + \
         [rng.standard_normal((c, c, 1, 1)), rng.standard_normal((c, c, 3, 3)) * 0.3, None, None, rng.standard_normal((5, c))]
    bs = [None if W is None else rng.standard_normal(W.shape[0]) * 0.1 for W in Ws]
    x = rng.standard_normal((h, w, ci))
    for bf16 in (False, True):
        q = oracle.round_bf16 if bf16 else (lambda v: v)
        m = Model(layers, Ws, bs, round_bf16=bf16)
        logits, _, _, _, hidden = oracle.forward_one(m, x.reshape(-1), want_hidden=True)
        relu = lambda v: np.maximum(v, 0.0)
        xq = q(x)
        A = q(relu(oracle.conv(layers[0], Ws[0], bs[0], xq)))
        B = q(relu(oracle.conv(layers[1], Ws[1], bs[1], A)))
        C = q(oracle.conv(layers[2], Ws[2], bs[2], B))
        S = q(relu(C + A))
        D = q(oracle.conv(layers[4], Ws[4], bs[4], B))
        E = q(oracle.conv(layers[5], Ws[5], bs[5], S))
        T = q(relu(E + D))
        pooled = q(T.mean(axis=(0, 1)))
        want = Ws[8] @ pooled + bs[8]
        assert np.allclose(logits, want, rtol=0, atol=1e-12)
        assert np.array_equal(hidden[:A.size], A.reshape(-1))           # layer-prefix check: the first hidden output
        # swapping the operands of either addition or reading the wrong source changes the answer
        wrong = [Layer(**{**l.__dict__}) for l in layers]
        wrong[4] = conv_layer(c, c, h, w, 1, 2, ACT_NONE, src=0)        # would read layer 3's output instead of layer 1's
        assert not np.allclose(oracle.forward_one(Model(wrong, Ws, bs, round_bf16=bf16), x.reshape(-1))[0], want, atol=1e-6)


def test_a_block_with_zero_branch_passes_its_input_through():
    # residual block: y = relu(conv2(relu(conv1(x))) + x); with conv2 = 0 the block is relu(x)
    h = w = 5
    c = 3
    layers = [conv_layer(c, c, h, w, 3, 1, ACT_RELU), conv_layer(c, c, h, w, 3, 1, ACT_RELU), conv_layer(c, c, h, w, 3, 1, ACT_NONE),
              Layer(ADD, ACT_RELU, c, c, h, w, src2=1), Layer(GAP, ACT_NONE, c, c, h, w), Layer(FC, ACT_NONE, c, c)]
    W0 = np.zeros((c, c, 3, 3)); W0[np.arange(c), np.arange(c), 1, 1] = 1.0        # layer 0: identity, so its output is relu(x)
    Ws = [W0, rng.standard_normal((c, c, 3, 3)), np.zeros((c, c, 3, 3)), None, None, np.eye(c)]
    x = rng.standard_normal((h, w, c))
    logits = oracle.forward_one(Model(layers, Ws, [None] * 6), x.reshape(-1))[0]
    assert np.allclose(logits, np.maximum(x, 0).mean(axis=(0, 1)), atol=1e-13)


# ---- batch normalisation folded into a convolution -----------------------------------------------
def test_folded_batchnorm_equals_the_unfolded_definition():
    co, ci, k, h, w = 5, 3, 3, 6, 7
    W, b = rng.standard_normal((co, ci, k, k)), rng.standard_normal(co)
    gamma, beta = rng.uniform(0.5, 2.0, co), rng.standard_normal(co)
    mean, var, eps = rng.standard_normal(co), rng.uniform(0.2, 3.0, co), 1e-5
    x = rng.standard_normal((h, w, ci))
    L = conv_layer(ci, co, h, w, k, 1)
    unfolded = gamma * (oracle.conv(L, W, b, x) - mean) / np.sqrt(var + eps) + beta       # batch normalisation as defined
    Wf, bf = oracle.fold_bn(W, b, gamma, beta, mean, var, eps, to_bf16=False)
    folded = oracle.conv(L, Wf, bf, x)
    assert np.allclose(folded, unfolded, rtol=0, atol=5e-6)                              # fp32 rounding of W' and b' only
    assert np.array_equal(Wf, Wf.astype(np.float32).astype(np.float64)) and np.array_equal(bf, bf.astype(np.float32).astype(np.float64))
    # bf16 models: the folded filters are bfloat16 values within half a unit in the last place of W * s
    Wq, bq = oracle.fold_bn(W, b, gamma, beta, mean, var, eps, to_bf16=True)
    assert np.array_equal(Wq, oracle.round_bf16(Wq)) and np.array_equal(bq, bf)
    exact = W * (gamma / np.sqrt(var + eps))[:, None, None, None]
    assert np.all(np.abs(Wq - exact) <= np.abs(exact) * 2.0 ** -8)
    assert np.allclose(oracle.conv(L, Wq, bq, x), unfolded, rtol=0, atol=0.15)             # same function up to weight rounding


def test_fold_special_values():
    W, b = rng.standard_normal((3, 2, 1, 1)), np.array([0.5, -1.0, 2.0])
    one, zero = np.ones(3), np.zeros(3)
    # gamma = 2, var + eps = 4 (eps = 0): scale 1 exactly, b' = b - mean + beta
    Wf, bf = oracle.fold_bn(W.astype(np.float32), b, 2 * one, np.array([1.0, 2.0, 3.0]), np.array([0.5, 0.5, 0.5]), 4 * one, 0.0, False)
    assert np.array_equal(Wf, W.astype(np.float32).astype(np.float64)) and np.array_equal(bf, [1.0, 0.5, 4.5])
    # gamma = 0: the convolution vanishes, the output is beta
    Wf, bf = oracle.fold_bn(W, b, zero, np.array([0.25, 0.5, 0.75]), one, one, 1e-5, True)
    assert np.all(Wf == 0) and np.array_equal(bf, [0.25, 0.5, 0.75])
    # without a bias the convolution's bias is zero
    Wf, bf = oracle.fold_bn(W, None, one, zero, np.array([1.0, 2.0, 3.0]), one, 0.0, False)
    assert np.array_equal(bf, [-1.0, -2.0, -3.0])
