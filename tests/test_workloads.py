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
