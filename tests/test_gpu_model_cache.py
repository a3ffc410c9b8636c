"""The device arena as a cache of the registered models (paper section 3.3): a worker holds more
models than fit the device, evicts the least recently used ones and reloads them on demand; the
cost of a miss follows from the model's fixed footprint.  Answers must not depend on where in the
arena a model lands or how often it was evicted, and must match the oracle."""
import numpy as np
import pytest
import torch

import paper_1901_06887_amd as mt
import workloads as wl
from gpu_common import compare, oracle_rows
from paper_1901_06887_amd import torch_io

pytestmark = pytest.mark.gpu


def served(ctx, w, rows, stream=None):
    ids = torch.from_numpy(np.ascontiguousarray(w.tenant_ids[rows])).cuda()
    x = torch_io.to_device(w.inputs[rows], w.dtype)
    out = mt.serve(ctx, ids, x, stream=stream)
    torch.cuda.synchronize()
    return (out.logits.cpu().numpy().astype(np.float64), out.probs.cpu().numpy().astype(np.float64),
            out.labels.cpu().numpy(), out.n_classes.cpu().numpy())


def test_more_models_than_the_arena_holds():
    w = wl.c2(n_tenants=12, n_requests=900, dims=(200, 320, 272, 10), s=0.6, seed=61)
    one_model = 320 * 256 * 2 + 320 * 320 * 2 + 64 * 320 * 2 + 3 * 2048      # padded layouts, roughly
    ctx = mt.context_for(w.tenants, w.dtype, w.n_requests, arena_bytes=5 * one_model, cache=True)
    mt.register_tenants(ctx, w.tenants)
    st = ctx.cache_stats()
    assert 3 <= st["resident_models"] < 12 and st["evictions"] == 12 - st["resident_models"]
    cap = st["resident_models"]
    groups = [list(range(0, cap)), list(range(cap, min(12, 2 * cap))), list(range(12 - cap, 12)), list(range(0, cap))]
    first = {}
    for gi, g in enumerate(groups):
        rows = np.flatnonzero(np.isin(w.tenant_ids, g))
        ctx.prefetch(g, torch.cuda.current_stream().cuda_stream)
        gpu = served(ctx, w, rows)
        sub = wl.Workload("cache group %d" % gi, w.dtype, w.tenants, w.tenant_ids[rows], w.inputs[rows])
        compare(sub, gpu, oracle_rows(sub), what=sub.name)
        key = tuple(g)
        if key in first:                                   # same tenants again, after being evicted in between: same bits
            assert np.array_equal(first[key][0], gpu[0]) and np.array_equal(first[key][2], gpu[2])
        first[key] = gpu
    assert ctx.cache_stats()["evictions"] > 12 - cap and ctx.cache_stats()["resident_models"] == cap

    # rows of a model that is registered but not resident are answered like rows without a model
    away = [t for t in range(12) if not ctx.tenant_account(t)["resident"]]
    rows = np.flatnonzero(np.isin(w.tenant_ids, away[:1] + groups[-1][:1]))
    lg, pr, lb, nc = served(ctx, w, rows)
    miss = w.tenant_ids[rows] == away[0]
    assert miss.any() and np.all(lb[miss] == -1) and np.all(nc[miss] == 0) and np.all(lb[~miss] >= 0)

    # per-tenant submissions name their tenant on the host: mt_run brings the model in by itself
    t = away[0]
    rows = np.flatnonzero(w.tenant_ids == t)
    x = torch_io.to_device(w.inputs[rows], w.dtype)
    out = torch_io.alloc_outputs(len(rows), ctx.cfg.max_classes)
    ctx.submit(t, x.data_ptr(), len(rows))
    ctx.run(torch.cuda.current_stream().cuda_stream, out.labels.data_ptr(), out.probs.data_ptr(), out.logits.data_ptr(),
            out.n_classes.data_ptr(), len(rows), ctx.cfg.max_classes)
    torch.cuda.synchronize()
    sub = wl.Workload("auto prefetch", w.dtype, w.tenants, w.tenant_ids[rows], w.inputs[rows])
    compare(sub, (out.logits.cpu().numpy().astype(np.float64), out.probs.cpu().numpy().astype(np.float64),
                  out.labels.cpu().numpy(), out.n_classes.cpu().numpy()), oracle_rows(sub), what="auto prefetch")
    assert ctx.tenant_account(t)["resident"] == 1
    ctx.close()


def test_prefetch_overlaps_a_run_and_later_runs_wait_for_it():
    # residency changes are enqueued on one stream while runs go on another: the upload queues up
    # behind the run in flight, and the next run (on the other stream) waits for the upload
    w = wl.c2(n_tenants=8, n_requests=600, dims=(200, 320, 272, 10), s=0.3, seed=62)
    one_model = 320 * 256 * 2 + 320 * 320 * 2 + 64 * 320 * 2 + 3 * 2048
    ctx = mt.context_for(w.tenants, w.dtype, w.n_requests, arena_bytes=5 * one_model, cache=True, run_slots=2)
    mt.register_tenants(ctx, w.tenants)
    ref = mt.context_for(w.tenants, w.dtype, w.n_requests)      # everything resident: the answers to match
    mt.register_tenants(ref, w.tenants)
    run_stream, copy_stream = torch.cuda.Stream(), torch.cuda.Stream()
    torch.cuda.synchronize()
    a, b = [0, 1, 2, 3], [4, 5, 6, 7]
    for g in (a, b, a, b):
        rows = np.flatnonzero(np.isin(w.tenant_ids, g))
        ids = torch.from_numpy(np.ascontiguousarray(w.tenant_ids[rows])).cuda()
        x = torch_io.to_device(w.inputs[rows], w.dtype)
        torch.cuda.synchronize()
        ctx.prefetch(g, copy_stream.cuda_stream)                 # evicts part of the other group behind its run
        out = mt.serve(ctx, ids, x, stream=run_stream)           # no host wait in between
        want = mt.serve(ref, ids, x)
        torch.cuda.synchronize()
        assert torch.equal(out.logits, want.logits) and torch.equal(out.labels, want.labels), g
    ctx.close(); ref.close()


def test_a_model_placed_twice_before_its_first_upload_ran():
    """Host far ahead of the GPU: prefetch A, run, prefetch the others (which evicts A), run, prefetch A
    again (another arena offset), run, with no host synchronisation in between.  The table rows of the
    first upload of A must be the ones taken when it was enqueued, not what the host holds by the time
    the copy executes; every run must answer like a context that holds everything."""
    w = wl.c2(n_tenants=6, n_requests=500, dims=(200, 320, 272, 10), s=0.2, seed=63)
    one_model = 320 * 256 * 2 + 320 * 320 * 2 + 64 * 320 * 2 + 3 * 2048
    ctx = mt.context_for(w.tenants, w.dtype, w.n_requests, arena_bytes=int(3.3 * one_model), cache=True, run_slots=2)
    mt.register_tenants(ctx, w.tenants)
    ref = mt.context_for(w.tenants, w.dtype, w.n_requests)
    mt.register_tenants(ref, w.tenants)
    stream = torch.cuda.Stream()
    busy = torch.zeros(1 << 30, dtype=torch.uint8, device="cuda")       # keeps the stream behind the host
    groups = ([0, 1], [2, 3, 4], [0, 5], [1, 2, 3], [0, 4])
    batches = []
    for g in groups:
        rows = np.flatnonzero(np.isin(w.tenant_ids, g))
        batches.append((torch.from_numpy(np.ascontiguousarray(w.tenant_ids[rows])).cuda(), torch_io.to_device(w.inputs[rows], w.dtype)))
    torch.cuda.synchronize()
    outs = []
    with torch.cuda.stream(stream):
        for _ in range(10):
            busy.add_(1)                                               # milliseconds of queued work before the first prefetch executes
        for g, (ids, x) in zip(groups, batches):
            ctx.prefetch(g, stream.cuda_stream)
            outs.append(mt.serve(ctx, ids, x, stream=stream))
    assert ctx.cache_stats()["evictions"] >= 4
    torch.cuda.synchronize()
    for g, (ids, x), out in zip(groups, batches, outs):
        want = mt.serve(ref, ids, x)
        torch.cuda.synchronize()
        assert torch.equal(out.labels, want.labels) and torch.equal(out.logits, want.logits), g
        assert int((out.labels < 0).sum()) == 0
    ctx.close(); ref.close()
