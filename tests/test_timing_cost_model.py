"""Tests that assert on measured time; the file name sorts them behind every parity test, so that a
slow machine cannot keep those from running.

Cost prediction on the GPU (paper section 3.2: the cost of inference is known a
priori; section 1.3: users should pay for the work done).  The per-tenant counters the batcher
keeps must equal the submitted rows exactly; the run-time estimate, computed from the registered
descriptors before anything is enqueued, must be close to the measured device time of the run."""
import time

import numpy as np
import pytest
import torch

import paper_1901_06887_amd as mt
import workloads as wl
from paper_1901_06887_amd import torch_io

pytestmark = pytest.mark.gpu

# The estimate is a per-kernel model with constants fitted on one MI355X; machines of the pool
# differ by several percent and the model's own error is up to ~15 % per kernel.
REL_TOL = 0.20          # the five mixes the constants were fitted on
REL_TOL_OTHER = 0.30    # mixes the fit has not seen


def other_mixes():
    c2 = wl.c2()
    uniform = wl.Workload("c2-uniform", c2.dtype, c2.tenants, np.random.default_rng(9).permutation(np.arange(4096, dtype=np.int32) % 64), c2.inputs)
    return {"c2-uniform": lambda: uniform, "c3-other-seed": lambda: wl.c3(seed=11), "c3-half-batch": lambda: wl.c3(n_requests=8192),
            "c4-half-batch": lambda: wl.c4(n_requests=1024), "c5-half-batch": lambda: wl.c5(n_requests=16384),
            "c5-six-tenants": lambda: wl.c5(n_tenants=6, n_requests=24576)}


@pytest.mark.parametrize("name", ["c1", "c2", "c3", "c4", "c5", "c2-uniform", "c3-other-seed", "c3-half-batch", "c4-half-batch",
                                  "c5-half-batch", "c5-six-tenants"])
def test_estimated_run_time_matches_the_measured_one(name):
    w = wl.CONFIGS[name]() if name in wl.CONFIGS else other_mixes()[name]()
    ctx = mt.context_for(w.tenants, w.dtype, w.n_requests)
    mt.register_tenants(ctx, w.tenants)
    est = ctx.estimate_run(np.bincount(w.tenant_ids, minlength=ctx.cfg.max_tenants))
    d_ids, d_x = torch.from_numpy(w.tenant_ids).cuda(), torch_io.to_device(w.inputs, w.dtype)
    out = torch_io.alloc_outputs(w.n_requests, ctx.cfg.max_classes)
    for _ in range(5):
        mt.serve(ctx, d_ids, d_x, out=out)
    torch.cuda.synchronize()
    assert est["launches"] == ctx.stats()["last_run_launches"]
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(20)]
    for e0, e1 in ev:
        e0.record()
        mt.serve(ctx, d_ids, d_x, out=out)
        e1.record()
    torch.cuda.synchronize()
    measured = float(np.median([e0.elapsed_time(e1) for e0, e1 in ev]))
    ratio = est["device_ms"] / measured
    print("%s: estimated %.4f ms, measured %.4f ms, ratio %.2f" % (name, est["device_ms"], measured, ratio), flush=True)
    assert abs(ratio - 1.0) <= (REL_TOL if name in wl.CONFIGS else REL_TOL_OTHER)
    ctx.close()


def test_admitted_runs_keep_the_latency_budget():
    # more requests are waiting than a run of the target latency can serve: admit a fair share of
    # every tenant's backlog, run it, and find the measured device time within the budget
    w = wl.c3()
    ctx = mt.context_for(w.tenants, w.dtype, w.n_requests)
    mt.register_tenants(ctx, w.tenants)
    pending = np.bincount(w.tenant_ids, minlength=ctx.cfg.max_tenants)
    d_x = torch_io.to_device(w.inputs, w.dtype)
    order = np.argsort(w.tenant_ids, kind="stable")
    start = np.concatenate([[0], np.cumsum(pending)])
    for budget in (0.47, 0.52):      # (any request of a tenant costs a pass over its weights: ~0.45 ms for one request each)
        admitted, est = ctx.admit(pending, budget)
        admitted = np.array(admitted)
        assert 0 < admitted.sum() < w.n_requests and admitted.max() < pending.max()
        rows = np.sort(np.concatenate([order[start[t]:start[t] + admitted[t]] for t in range(len(pending))]))   # arrival order
        d_ids = torch.from_numpy(np.ascontiguousarray(w.tenant_ids[rows])).cuda()
        x = d_x[torch.from_numpy(rows).cuda()].contiguous()
        out = torch_io.alloc_outputs(len(rows), ctx.cfg.max_classes)
        for _ in range(3):
            mt.serve(ctx, d_ids, x, out=out)
        torch.cuda.synchronize()
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(15)]
        for e0, e1 in ev:
            e0.record(); mt.serve(ctx, d_ids, x, out=out); e1.record()
        torch.cuda.synchronize()
        measured = float(np.median([e0.elapsed_time(e1) for e0, e1 in ev]))
        print("budget %.2f ms: level %d, %d of %d requests admitted, predicted %.3f ms, measured %.3f ms" % (
            budget, admitted.max(), admitted.sum(), w.n_requests, est["device_ms"], measured), flush=True)
        assert measured <= budget * (1 + REL_TOL_OTHER)      # partial mixes: the estimate reads 10-12 % low on these
    ctx.close()


def test_upload_time_follows_the_footprint():
    # section 3.3: transfer latency is predictable because a model's footprint is fixed
    w = wl.c5(n_tenants=3, n_requests=64, dims=(4096, 4096, 4096, 1000))        # ~75 MB per model
    acc_bytes = None
    ctx = mt.context_for(w.tenants, w.dtype, w.n_requests, arena_bytes=int(1.2 * 76e6), cache=True)
    mt.register_tenants(ctx, w.tenants)
    s = torch.cuda.current_stream().cuda_stream
    times = []
    for t in (0, 1, 2, 0, 1, 2):
        assert ctx.tenant_account(t)["resident"] == 0
        acc_bytes = ctx.tenant_account(t)["arena_bytes"]
        counts = [0, 0, 0]; counts[t] = 10
        predicted = ctx.estimate_run(counts)["upload_ms"]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        ctx.prefetch([t], s)
        torch.cuda.synchronize()
        times.append((time.perf_counter() - t0) * 1e3)
    measured = float(np.median(times))
    print("upload of %.1f MB: measured %.3f ms (%.1f GB/s), predicted %.3f ms" % (acc_bytes / 1e6, measured, acc_bytes / measured / 1e6, predicted), flush=True)
    assert abs(predicted / measured - 1.0) <= 0.35
    ctx.close()


@pytest.mark.parametrize("name", ["c2", "c3", "c4", "c5"])
def test_run_time_is_predictable(name):
    """Paper section 3.2: inference time is predictable, the 99th percentile within 15 % of the mean.
    Device time of a run between two events, 100 runs of the same batch back to back."""
    w = wl.CONFIGS[name]()
    ctx = mt.context_for(w.tenants, w.dtype, w.n_requests)
    mt.register_tenants(ctx, w.tenants)
    d_ids, d_x = torch.from_numpy(w.tenant_ids).cuda(), torch_io.to_device(w.inputs, w.dtype)
    out = torch_io.alloc_outputs(w.n_requests, ctx.cfg.max_classes)
    for _ in range(10):
        mt.serve(ctx, d_ids, d_x, out=out)
    torch.cuda.synchronize()
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(100)]
    for e0, e1 in ev:
        e0.record(); mt.serve(ctx, d_ids, d_x, out=out); e1.record()
    torch.cuda.synchronize()
    ms = np.array([e0.elapsed_time(e1) for e0, e1 in ev])
    ratio = float(np.percentile(ms, 99) / ms.mean())
    print("%s: mean %.4f ms, p99 %.4f ms, p99/mean %.3f, max/mean %.3f" % (name, ms.mean(), np.percentile(ms, 99), ratio, ms.max() / ms.mean()), flush=True)
    assert ratio <= 1.15
    ctx.close()
