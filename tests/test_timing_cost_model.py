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
BREAK_EVEN_TOL = 0.15   # hit ratio at which upload and execution take equally long: predicted against measured


def other_mixes():
    c2 = wl.c2()
    uniform = wl.Workload("c2-uniform", c2.dtype, c2.tenants, np.random.default_rng(9).permutation(np.arange(4096, dtype=np.int32) % 64), c2.inputs)
    return {"c2-uniform": lambda: uniform, "c3-other-seed": lambda: wl.c3(seed=11), "c3-half-batch": lambda: wl.c3(n_requests=8192),
            "c4-half-batch": lambda: wl.c4(n_requests=1024), "c5-half-batch": lambda: wl.c5(n_requests=16384),
            "c5-six-tenants": lambda: wl.c5(n_tenants=6, n_requests=24576),
            "r18": wl.r18, "r18-one-request": lambda: wl.resnet(n_tenants=2, n_requests=1, hw=224), "r18-256-requests": lambda: wl.r18(n_requests=256)}


@pytest.mark.parametrize("name", ["c1", "c2", "c3", "c4", "c5", "c2-uniform", "c3-other-seed", "c3-half-batch", "c4-half-batch",
                                  "c5-half-batch", "c5-six-tenants", "r18", "r18-one-request", "r18-256-requests"])
def test_estimated_run_time_matches_the_measured_one(name):
    w = other_mixes()[name]() if name in other_mixes() else wl.CONFIGS[name]()
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
    assert abs(ratio - 1.0) <= (REL_TOL if name in wl.CONFIGS and name != "r18" else REL_TOL_OTHER)
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


def test_cache_hit_ratio_from_which_the_host_link_is_no_longer_the_bottleneck():
    """Paper section 3.3: copying the ~78 MB of a resnet18 takes ~7 ms over a 12 GB/s link, executing it at batch 1
    ~1 ms (section 1.3: 1031 inferences/s), so the link is the bottleneck unless 85 % or more of the requests find
    their model resident.  The reasoning in closed form: every request costs t_exec on the GPU and a miss costs t_copy
    on the link, so the GPU is the bottleneck when (1 - h) t_copy <= t_exec, i.e. from h = 1 - t_exec / t_copy on.
    The paper's numbers give 0.86.  The same form is evaluated here for a resnet18-shaped model at batch 1, once from
    the library's prediction alone (footprint -> upload time, layer descriptions -> run time) and once from measured
    times; both follow from fixed quantities, so the two break-even ratios must agree: on this machine's link (a
    23 MB model crosses it as fast as one request runs, so there the link never is the bottleneck) and on one of the
    paper's 12 GB/s."""
    assert 0.85 <= 1.0 - (1e3 / 1031.0) / 7.0 <= 0.87
    w = wl.resnet(n_tenants=2, n_requests=2, hw=224)
    fp = mt.model_footprint(torch_io.specs_of(w.tenants[0].layers), mt.binding.MT_BF16)["arena_bytes"]
    ctx = mt.context_for(w.tenants, w.dtype, 4, arena_bytes=int(1.3 * fp), cache=True)           # room for one of the two models
    mt.register_tenants(ctx, w.tenants)
    s = torch.cuda.current_stream().cuda_stream
    x = torch_io.to_device(w.inputs[:1], w.dtype)
    out = torch_io.alloc_outputs(1, ctx.cfg.max_classes)
    copy_ms, exec_ms, pred = [], [], None
    for t in (0, 1, 0, 1, 0, 1):
        assert ctx.tenant_account(t)["resident"] == 0
        counts = [0, 0]; counts[t] = 1
        pred = ctx.estimate_run(counts)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        ctx.prefetch([t], s)
        torch.cuda.synchronize()
        copy_ms.append((time.perf_counter() - t0) * 1e3)
        ids = torch.full((1,), t, dtype=torch.int32, device="cuda")
        for _ in range(3):
            mt.serve(ctx, ids, x, out=out)
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(10)]
        for e0, e1 in ev:
            e0.record()
            mt.serve(ctx, ids, x, out=out)
            e1.record()
        torch.cuda.synchronize()
        exec_ms.append(float(np.median([e0.elapsed_time(e1) for e0, e1 in ev])))
    t_copy, t_exec = float(np.median(copy_ms)), float(np.median(exec_ms))
    assert abs(pred["upload_ms"] / t_copy - 1.0) <= 0.35 and abs(pred["device_ms"] / t_exec - 1.0) <= REL_TOL_OTHER
    # the break-even ratio on this machine's link, and on a link of the paper's 12 GB/s (the copy time follows from the footprint)
    paper_link_ms = fp / 12e9 * 1e3
    h = lambda run_ms, copy: max(0.0, 1.0 - run_ms / copy)
    print("resnet18-shaped model, %.1f MB: copy %.3f ms measured / %.3f predicted (%.0f GB/s), batch-1 run %.3f ms measured / %.3f predicted; "
          "the link is the bottleneck below a hit ratio of %.2f (measured) / %.2f (predicted) here, %.2f / %.2f over a 12 GB/s link; "
          "the paper's V100 and link: 0.86" % (fp / 1e6, t_copy, pred["upload_ms"], fp / t_copy / 1e6, t_exec, pred["device_ms"],
                                               h(t_exec, t_copy), h(pred["device_ms"], pred["upload_ms"]), h(t_exec, paper_link_ms), h(pred["device_ms"], paper_link_ms)), flush=True)
    assert abs(h(t_exec, t_copy) - h(pred["device_ms"], pred["upload_ms"])) <= BREAK_EVEN_TOL
    assert abs(h(t_exec, paper_link_ms) - h(pred["device_ms"], paper_link_ms)) <= BREAK_EVEN_TOL
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
