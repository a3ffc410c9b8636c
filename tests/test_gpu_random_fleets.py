"""Randomised fleets: tenants with MLPs and CNNs of random depth, width and image size share one
context; requests arrive in random order, split over random submissions, with a few unknown
ids.  Every answer is compared with the oracle, and a second run of the same batch in another
submission pattern must give the same bits."""
import numpy as np
import pytest
import torch

import paper_1901_06887_amd as mt
import workloads as wl
from gpu_common import compare, make_context, oracle_rows
from paper_1901_06887_amd import torch_io

pytestmark = pytest.mark.gpu


def random_model(rng, kind, in_len_mlp, dtype, key):
    if kind == "mlp":
        depth = int(rng.integers(1, 6))
        dims = [in_len_mlp] + [int(rng.choice([24, 33, 64, 72, 100, 136, 200, 264])) for _ in range(depth - 1)] + [int(rng.choice([3, 10, 32, 33, 70]))]
        act = int(rng.choice([wl.ACT_RELU, wl.ACT_GELU, wl.ACT_NONE]))
        return wl.make_model(wl.mlp_layers(dims, act), dtype, *key)
    n_conv = int(rng.integers(1, 4))
    chans = [3] + [int(rng.choice([8, 16, 24, 40, 64])) for _ in range(n_conv)]
    strides = [int(rng.choice([1, 2])) for _ in range(n_conv)]
    return wl.make_model(wl.cnn_layers(8, chans, strides, int(rng.choice([4, 10, 40]))), dtype, *key)


@pytest.mark.parametrize("seed,dtype", [(101, "bf16"), (102, "bf16"), (103, "bf16"), (104, "f32")])
def test_random_fleet(seed, dtype):
    rng = np.random.default_rng(seed)
    n_tenants = int(rng.integers(3, 12))
    in_len = 8 * 8 * 3                                     # MLPs take the same 192 values the CNNs take as an 8x8x3 image
    kinds = [str(rng.choice(["mlp", "cnn"])) for _ in range(n_tenants)]
    tenants = {t: random_model(rng, kinds[t], in_len, dtype, (seed, t)) for t in range(n_tenants)}
    R = int(rng.integers(40, 700))
    weights = rng.random(n_tenants) ** 3 + 1e-3            # skewed traffic, some tenants nearly idle
    ids = rng.choice(n_tenants, size=R, p=weights / weights.sum()).astype(np.int32)
    x = rng.standard_normal((R, in_len)).astype(np.float32)
    if dtype == "bf16":
        x = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    w = wl.Workload("fleet %d" % seed, dtype, tenants, ids, x)
    ctx = make_context(w, max_tenants=n_tenants + 2)
    d_x = torch_io.to_device(x, dtype)
    bad = ids.copy()
    bad_rows = rng.choice(R, size=3, replace=False)
    bad[bad_rows] = [n_tenants, n_tenants + 5, -2]           # registered range without a model, out of range, negative
    d_ids = torch.from_numpy(bad).cuda()

    def run(cuts):
        out = torch_io.alloc_outputs(R, ctx.cfg.max_classes)
        for a, b in zip(cuts[:-1], cuts[1:]):
            assert ctx.submit_batch(d_ids.data_ptr() + 4 * int(a), d_x.data_ptr() + int(a) * in_len * d_x.element_size(), int(b - a), in_len) == a
        ctx.debug_poison()
        n = ctx.run(torch.cuda.current_stream().cuda_stream, out.labels.data_ptr(), out.probs.data_ptr(), out.logits.data_ptr(),
                    out.n_classes.data_ptr(), R, ctx.cfg.max_classes)
        torch.cuda.synchronize()
        assert n == R
        return (out.logits.cpu().numpy().astype(np.float64), out.probs.cpu().numpy().astype(np.float64),
                out.labels.cpu().numpy(), out.n_classes.cpu().numpy())

    one = run([0, R])
    cuts = np.unique(np.concatenate([[0, R], rng.integers(1, R, size=int(rng.integers(1, 6)))]))
    many = run(list(cuts))
    assert np.array_equal(one[0], many[0]) and np.array_equal(one[2], many[2])
    good = np.setdiff1d(np.arange(R), bad_rows)
    assert np.all(one[2][bad_rows] == -1) and np.all(one[3][bad_rows] == 0) and np.all(one[0][bad_rows] == 0)
    sub = wl.Workload(w.name, dtype, tenants, ids[good], x[good])
    worst = compare(sub, tuple(a[good] for a in one), oracle_rows(sub), what=w.name)
    print("%s: %d tenants (%s), %d rows, worst rel fro %.2e" % (w.name, n_tenants, "".join(k[0] for k in kinds), R, worst), flush=True)
    ctx.close()
