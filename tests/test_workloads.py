"""The seeded generators: determinism, shapes and the stated distributions.  CPU only."""
import numpy as np

import workloads as wl


def test_deterministic_and_representable():
    a = wl.c2(n_tenants=6, n_requests=200, dims=(40, 64, 10))
    b = wl.c2(n_tenants=6, n_requests=200, dims=(40, 64, 10))
    assert np.array_equal(a.tenant_ids, b.tenant_ids) and np.array_equal(a.inputs, b.inputs)
    for t in a.tenants:
        for wa, wb in zip(a.tenants[t].weights, b.tenants[t].weights):
            assert np.array_equal(wa, wb)
        assert np.array_equal(wl.bits_to_f32(wl.bf16_bits(a.tenants[t].weights[0])), a.tenants[t].weights[0])
    assert a.inputs.min() >= 0 and a.inputs.max() <= 1


def test_weight_scale_is_variance_one_over_fan_in():
    w = wl.c1(n_tenants=1, n_requests=4)
    W = w.tenants[0].weights[1]
    assert W.shape == (512, 512)
    assert abs(W.std() * np.sqrt(512) - 1) < 0.02
    assert abs(w.tenants[0].biases[1].std() - 0.1) < 0.02


def test_zipf_is_skewed_and_normalised():
    ids = wl.zipf_ids(64, 4096, 1.1, 2)
    counts = np.sort(np.bincount(ids, minlength=64))[::-1]
    p = np.arange(1, 65) ** -1.1
    p /= p.sum()
    assert abs(counts[0] / 4096 - p[0]) < 0.03
    assert counts[0] > 20 * max(1, counts[-1])
    assert counts.sum() == 4096


def test_c3_depth_and_width_ranges():
    w = wl.c3(n_tenants=40, n_requests=100, in_dim=32, widths=(16, 32, 64), classes=7)
    depths = {len(m.layers) for m in w.tenants.values()}
    assert depths <= {2, 3, 4, 5, 6} and len(depths) >= 4
    for m in w.tenants.values():
        assert m.layers[0].in_features == 32 and m.n_classes == 7
        assert all(l.out_features in (16, 32, 64) for l in m.layers[:-1])
        assert m.layers[-1].act == wl.ACT_NONE


def test_cnn_geometry_and_cost():
    w = wl.c4(n_tenants=2, n_requests=6)
    m = w.tenants[0]
    assert [l.out_len() for l in m.layers] == [32 * 32 * 32, 16 * 16 * 64, 8 * 8 * 128, 128, 10]
    assert m.n_params() == 27 * 32 + 288 * 64 + 576 * 128 + 1280
    cost = wl.algorithmic_cost(w)
    per_img = 2 * (1024 * 27 * 32 + 256 * 288 * 64 + 64 * 576 * 128 + 1280)
    assert cost["flops"] == 6 * per_img


def test_c2_cost_matches_closed_form():
    w = wl.c2(n_tenants=3, n_requests=50, dims=(20, 30, 5))
    cost = wl.algorithmic_cost(w)
    assert cost["flops"] == 50 * 2 * (20 * 30 + 30 * 5)
    active = len(w.counts())
    assert cost["weight_bytes"] == active * ((20 * 30 + 30 * 5) * 2 + 35 * 4)


def test_resnet18_shaped_layer_graph():
    """17 convolutions of 3x3 and the 7x7 stem, 3 projections of 1x1, one max-pool, 8 residual
    additions, pooling, FC; every layer's input shape is the output shape of the layer it names."""
    L = wl.resnet18_layers(64, 3, (64, 128, 256, 512), 1000)
    kinds = [l.kind for l in L]
    assert kinds.count(wl.CONV) == 20 and kinds.count(wl.ADD) == 8 and kinds.count(wl.MAXPOOL) == 1 and kinds[-2:] == [wl.GAP, wl.FC]
    assert sorted((l.ksize for l in L if l.kind == wl.CONV), reverse=True)[:4] == [7, 3, 3, 3] and sum(1 for l in L if l.kind == wl.CONV and l.ksize == 1) == 3
    def out_shape(j):            # (h, w, c) of the output of layer j
        l = L[j]
        h, w = l.out_hw()
        return (h, w, l.out_features if l.kind == wl.CONV else l.in_features)
    for i, l in enumerate(L):
        if i == 0 or l.kind == wl.FC:
            continue
        src = l.src - 1 if l.src else i - 1
        assert src < i and out_shape(src) == (l.in_h, l.in_w, l.in_features), i
        if l.kind == wl.ADD:
            assert 0 < l.src2 <= i and out_shape(l.src2 - 1) == (l.in_h, l.in_w, l.in_features), i
    assert out_shape(len(L) - 3) == (2, 2, 512)           # 64 -> 32 (stem) -> 16 (pool) -> 16, 8, 4, 2
    w = wl.resnet(n_tenants=2, n_requests=5, hw=32, widths=(8, 16, 24, 32), classes=7)
    assert all(b is not None for l, b in zip(w.tenants[0].layers, w.tenants[0].bn) if l.kind == wl.CONV)
    assert w.tenants[0].weights[0].shape == (8, 3, 7, 7) and w.inputs.shape == (5, 32 * 32 * 3)
