"""Why a single row is held to a looser bar than a tensor (see gpu_common.py): with bf16 hidden
activations one hidden value that lies on a rounding boundary decides the row.  The case below came up
in a sweep of random fleets: a five-layer linear MLP whose first layer has 33 outputs, one of which is
3e-8 (relative) away from the midpoint of two bfloat16 values for this request.  Accumulated in fp32,
in any order, that value can land on either side; taking the other side moves the three logits by 7e-3
of their norm (the per-row bar is 1e-2 for that reason), with every other operation exact.  The test pins both facts on the
CPU, from the seeded generators alone: the distance to the boundary and the size of the effect."""
import numpy as np
import torch

import workloads as wl
from test_gpu_random_fleets import random_model


def bf16(v):
    return torch.from_numpy(np.asarray(v, dtype=np.float32)).to(torch.bfloat16).to(torch.float64).numpy()


def test_one_rounding_flip_moves_a_narrow_net_by_more_than_the_row_tolerance():
    # the fleet of seed 214, drawn exactly as tests/test_gpu_random_fleets.py draws it; accepted row 146
    seed, tenant = 214, 1
    rng = np.random.default_rng(seed)
    n_tenants = int(rng.integers(3, 12))
    kinds = [str(rng.choice(["mlp", "cnn"])) for _ in range(n_tenants)]
    tenants = {t: random_model(rng, kinds[t], 192, "bf16", (seed, t)) for t in range(n_tenants)}
    R = int(rng.integers(40, 700))
    share = rng.random(n_tenants) ** 3 + 1e-3
    ids = rng.choice(n_tenants, size=R, p=share / share.sum())
    x = bf16(rng.standard_normal((R, 192)).astype(np.float32))
    rejected = rng.choice(R, size=3, replace=False)
    row = np.setdiff1d(np.arange(R), rejected)[146]
    m = tenants[tenant]
    assert ids[row] == tenant and [l.out_features for l in m.layers] == [33, 72, 136, 200, 3]
    assert all(l.act == wl.ACT_NONE for l in m.layers)

    def logits(flip_unit=None):
        h = x[row]
        for li, (W, b) in enumerate(zip(m.weights, m.biases)):
            z = W.astype(np.float64) @ h + b.astype(np.float64)
            if li == len(m.weights) - 1:
                return z
            h = bf16(z)
            if li == 0 and flip_unit is not None:       # the other neighbour of z on the bfloat16 grid
                j = flip_unit
                ulp = 2.0 ** (np.floor(np.log2(abs(z[j]))) - 7)
                lo = np.floor(abs(z[j]) / ulp) * ulp
                h[j] = np.sign(z[j]) * (lo + ulp if abs(abs(h[j]) - lo) < 1e-12 else lo)

    # distance of every first-layer value to the midpoint of its two bfloat16 neighbours, in ulps
    z = m.weights[0].astype(np.float64) @ x[row] + m.biases[0].astype(np.float64)
    ulp = 2.0 ** (np.floor(np.log2(np.abs(z))) - 7)
    dist = np.abs(np.abs(z) / ulp - np.floor(np.abs(z) / ulp) - 0.5)
    j = int(np.argmin(dist))
    assert j == 32 and dist[j] < 1e-5                   # 1e-5 ulp is 4e-8 relative: below fp32 accumulation noise
    assert np.sort(dist)[1] > 1e-3                      # and it is the only such value in the layer
    exact, other = logits(), logits(flip_unit=j)
    rel = np.linalg.norm(other - exact) / np.linalg.norm(exact)
    assert 5e-3 < rel < 1e-2, rel


def test_exactly_rounded_fp32_accumulation_already_shows_the_two_kinds_of_rows():
    """The bar of tests/gpu_common.py rests on this: with bf16 hidden activations even an fp32 path whose
    every dot product is *exactly rounded* (computed in fp64, rounded once) differs from the fp64 oracle in
    two ways only: most rows agree to ~1e-7, and a row in which one hidden value crossed a bfloat16
    rounding boundary is off by 1e-4 .. 3e-3.  So no fp32-accumulating kernel can hold single rows to 1e-3,
    while a tensor of many rows stays within it.  Here: 400 requests of a 24-tenant mix drawn like c3
    (depths 2..6, widths 512/1024/2048), every model evaluated request by request."""
    import oracle
    w = wl.c3(n_tenants=24, n_requests=400, seed=3)
    models = oracle.models_from_workload(w)
    lg = oracle.run_batch(models, w.tenant_ids, w.inputs.astype(np.float64), threads=8)[0]

    def fp32_path(model, x):
        h = x.astype(np.float32)
        for li, (W, b) in enumerate(zip(model.weights, model.biases)):
            z = (W.astype(np.float64) @ h.astype(np.float64)).astype(np.float32)     # exactly rounded fp32 dot products
            z = (z + b).astype(np.float32)
            if li == len(model.weights) - 1:
                return z.astype(np.float64)
            h = bf16(np.maximum(z, 0)).astype(np.float32)

    g = np.stack([fp32_path(w.tenants[int(t)], x) for t, x in zip(w.tenant_ids, w.inputs)])
    err = np.linalg.norm(g - lg[:, :100], axis=1) / np.linalg.norm(lg[:, :100], axis=1)
    assert np.mean(err < 1e-6) >= 0.95                  # flip-free rows: fp32 rounding of the logits only
    assert np.sum(err > 1e-3) >= 2 and err.max() < 5e-3 # rows with a flip: beyond 1e-3, far inside the 1e-2 row bar
    assert np.mean((err >= 1e-6) & (err <= 1e-5)) == 0  # nothing in between the two kinds
    assert np.linalg.norm(g - lg[:, :100]) / np.linalg.norm(lg[:, :100]) < 1e-3     # the run's tensor holds the bar


def test_a_deep_narrow_net_turns_one_flip_into_more_than_the_tensor_bar():
    """The resnet18-shaped tenants at reduced widths (20 convolutions, the last ones on 1x1 images of 128
    channels): evaluated layer by layer with every layer's result *exactly rounded to fp32* before the
    activation and the bfloat16 rounding, 39 of 40 requests agree with the fp64 oracle to ~1e-8 and one
    is 6.6e-3 off, which alone puts the 40-row tensor at 1.26e-3.  The GPU path gives the same row and
    the same value; deep bf16 nets are therefore compared at the wider bar of tests/gpu_common.py."""
    import oracle
    w = wl.resnet(n_tenants=3, n_requests=40, hw=32, widths=(16, 32, 64, 128), classes=10)
    models = oracle.models_from_workload(w)
    lg = oracle.run_batch(models, w.tenant_ids, w.inputs.astype(np.float64), threads=8)[0]

    def fp32_path(m, x):
        outs = [bf16(x)]
        for l, L in enumerate(m.layers):
            src = outs[L.src if L.src > 0 else l]
            if L.kind == oracle.CONV:
                z = oracle.conv(L, m.weights[l], m.biases[l], src).reshape(-1)
            elif L.kind == oracle.FC:
                z = oracle.fc(L, m.weights[l], m.biases[l], src)
            elif L.kind == oracle.MAXPOOL:
                z = oracle.maxpool(L, src).reshape(-1)
            elif L.kind == oracle.ADD:
                z = oracle.add(L, src, outs[L.src2 if L.src2 > 0 else l]).reshape(-1)
            else:
                z = oracle.gap(L, src)
            z = z.astype(np.float32).astype(np.float64)
            if l == len(m.layers) - 1:
                return z
            outs.append(bf16(np.maximum(z, 0) if L.act == oracle.ACT_RELU else z))

    g = np.stack([fp32_path(models[int(t)], x) for t, x in zip(w.tenant_ids, w.inputs.astype(np.float64))])
    err = np.linalg.norm(g - lg, axis=1) / np.linalg.norm(lg, axis=1)
    assert np.sum(err > 1e-5) == 1 and 5e-3 < err.max() < 8e-3 and np.median(err) < 1e-6
    assert np.linalg.norm(g - lg) / np.linalg.norm(lg) > 1e-3
