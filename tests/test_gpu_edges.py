"""GPU edge cases of the hot path: empty runs, tenants without traffic, rejected ids, the
per-tenant submit call, determinism, statelessness (a request's answer does not depend on
what shares its batch; paper section 1.1), full-capacity runs and reuse of a context."""
import numpy as np
import pytest
import torch

import paper_1901_06887_amd as mt
import workloads as wl
from gpu_common import compare, gpu_run, make_context, oracle_rows
from paper_1901_06887_amd import torch_io

pytestmark = pytest.mark.gpu


def small():
    return wl.c2(n_tenants=6, n_requests=300, dims=(100, 192, 136, 10))


def test_empty_run_serves_nothing():
    w = small()
    ctx = make_context(w)
    out = torch_io.alloc_outputs(4, ctx.cfg.max_classes)
    n = ctx.run(torch.cuda.current_stream().cuda_stream, out.labels.data_ptr(), out.probs.data_ptr(),
                out.logits.data_ptr(), out.n_classes.data_ptr(), 4, ctx.cfg.max_classes)
    assert n == 0 and ctx.stats()["last_run_rows"] == 0
    ctx.close()


def test_tenants_without_traffic_and_single_rows():
    w = small()
    ids = np.where(w.tenant_ids == 3, 1, w.tenant_ids).astype(np.int32)    # tenant 3 gets nothing
    ids[:] = np.where(ids == 5, 0, ids)
    ids[17] = 5                                                             # tenant 5 gets exactly one row
    w.tenant_ids = ids
    ctx = make_context(w)
    gpu = gpu_run(ctx, w, poison=True)
    counts = ctx.last_counts()
    assert counts[3] == 0 and counts[5] == 1
    compare(w, gpu, oracle_rows(w), what="sparse-traffic")
    ctx.close()


def test_unknown_tenant_ids_are_rejected_on_device():
    w = small()
    ctx = make_context(w, max_tenants=10)          # ids 6..9 exist but have no model
    ids = w.tenant_ids.copy()
    bad = np.array([0, 5, 77, 150, 299])
    ids[bad] = [7, -1, 10, 1 << 20, 9]
    lg, pr, lb, nc = gpu_run(ctx, w, ids=ids, poison=True)
    assert np.all(lb[bad] == -1) and np.all(nc[bad] == 0)
    assert np.all(lg[bad] == 0) and np.all(pr[bad] == 0)
    good = np.setdiff1d(np.arange(w.n_requests), bad)
    w2 = wl.Workload(w.name, w.dtype, w.tenants, ids[good], w.inputs[good])
    compare(w2, (lg[good], pr[good], lb[good], nc[good]), oracle_rows(w2), what="rejected-ids")
    assert ctx.last_counts().sum() == len(good)
    ctx.close()


def test_per_tenant_submit_matches_batch_submit():
    w = small()
    ctx = make_context(w)
    ref = gpu_run(ctx, w)
    d_x = torch_io.to_device(w.inputs, w.dtype)
    # arrival order is kept: every maximal run of one tenant becomes one mt_submit call
    ids = w.tenant_ids
    starts = np.flatnonzero(np.r_[True, ids[1:] != ids[:-1]])
    ends = np.r_[starts[1:], len(ids)]
    es = d_x.element_size()
    for s, e in zip(starts, ends):
        first = ctx.submit(int(ids[s]), d_x.data_ptr() + int(s) * d_x.shape[1] * es, int(e - s))
        assert first == s
    out = torch_io.alloc_outputs(w.n_requests, ctx.cfg.max_classes)
    n = ctx.run(torch.cuda.current_stream().cuda_stream, out.labels.data_ptr(), out.probs.data_ptr(),
                out.logits.data_ptr(), out.n_classes.data_ptr(), w.n_requests, ctx.cfg.max_classes)
    torch.cuda.synchronize()
    assert n == w.n_requests
    assert np.array_equal(out.logits.cpu().numpy().astype(np.float64), ref[0])
    assert np.array_equal(out.labels.cpu().numpy(), ref[2])
    ctx.close()


def test_runs_are_bit_reproducible_and_context_is_reusable():
    w = wl.c3(n_tenants=10, n_requests=700, in_dim=128, widths=(64, 128, 256), classes=100)
    ctx = make_context(w)
    a = gpu_run(ctx, w)
    b = gpu_run(ctx, w, poison=True)
    for x, y in zip(a, b):
        assert np.array_equal(x, y)
    # a different, smaller batch on the same context, then the first one again
    half = w.n_requests // 3
    w2 = wl.Workload(w.name, w.dtype, w.tenants, w.tenant_ids[:half][::-1].copy(), w.inputs[:half][::-1].copy())
    compare(w2, gpu_run(ctx, w2), oracle_rows(w2), what="second-batch")
    c = gpu_run(ctx, w)
    assert np.array_equal(a[0], c[0]) and np.array_equal(a[2], c[2])
    ctx.close()


def test_answers_do_not_depend_on_the_batch():
    w = small()
    ctx = make_context(w)
    full = gpu_run(ctx, w)
    for i in (0, 123, 299):
        one = gpu_run(ctx, w, ids=w.tenant_ids[i:i + 1], inputs=w.inputs[i:i + 1])
        assert np.array_equal(one[0][0], full[0][i]) and one[2][0] == full[2][i]
    # arrival order shuffled: same per-request answers
    p = np.random.default_rng(3).permutation(w.n_requests)
    sh = gpu_run(ctx, w, ids=w.tenant_ids[p], inputs=w.inputs[p])
    assert np.array_equal(sh[0], full[0][p]) and np.array_equal(sh[2], full[2][p])
    ctx.close()


def test_full_capacity_and_capacity_errors():
    w = small()
    ctx = make_context(w, max_requests=w.n_requests)          # exactly full
    gpu = gpu_run(ctx, w)
    compare(w, gpu, oracle_rows(w), what="full-capacity")
    d_ids = torch.from_numpy(w.tenant_ids).cuda()
    d_x = torch_io.to_device(w.inputs, w.dtype)
    ctx.submit_batch(d_ids.data_ptr(), d_x.data_ptr(), w.n_requests, d_x.shape[1])
    with pytest.raises(mt.MtError) as e:
        ctx.submit_batch(d_ids.data_ptr(), d_x.data_ptr(), 1, d_x.shape[1])
    assert e.value.status == 6
    out = torch_io.alloc_outputs(10, ctx.cfg.max_classes)
    with pytest.raises(mt.MtError) as e:                       # outputs too small: nothing is launched
        ctx.run(0, out.labels.data_ptr(), out.probs.data_ptr(), out.logits.data_ptr(), out.n_classes.data_ptr(),
                10, ctx.cfg.max_classes)
    assert e.value.status == 1
    ctx.close()


def test_unregister_then_serve_remaining_tenants():
    w = small()
    ctx = make_context(w)
    ctx.unregister_model(2)
    lg, pr, lb, nc = gpu_run(ctx, w)
    gone = w.tenant_ids == 2
    assert np.all(lb[gone] == -1)
    keep = ~gone
    w2 = wl.Workload(w.name, w.dtype, {t: m for t, m in w.tenants.items() if t != 2}, w.tenant_ids[keep], w.inputs[keep])
    compare(w2, (lg[keep], pr[keep], lb[keep], nc[keep]), oracle_rows(w2), what="after-unregister")
    ctx.close()


def test_staged_and_separate_head_paths_match_the_fused_ones(monkeypatch):
    """The FC kernel may gather layer-0 inputs and finish <=32-class rows itself; the staged
    gather pass and the separate head kernel must give the same answers."""
    w = wl.c2(n_tenants=5, n_requests=260, dims=(96, 160, 128, 10))     # 96 bf16 = 12 chunks: fused gather applies
    ctx = make_context(w)
    fused = gpu_run(ctx, w, poison=True)
    ctx.close()
    compare(w, fused, oracle_rows(w), what="fused")
    monkeypatch.setenv("MT_NO_FUSED_GATHER", "1")
    monkeypatch.setenv("MT_NO_FUSED_HEAD", "1")
    ctx = make_context(w)
    plain = gpu_run(ctx, w, poison=True)
    assert ctx.stats()["last_run_launches"] == 6                          # batcher, gather, 3 layers, head
    ctx.close()
    assert np.array_equal(fused[0], plain[0]) and np.array_equal(fused[2], plain[2])
    assert np.allclose(fused[1], plain[1], rtol=1e-6, atol=1e-7)


def test_mixed_class_counts_use_both_head_paths():
    a = wl.c2(n_tenants=3, n_requests=150, dims=(64, 128, 10), seed=11)
    b = wl.c2(n_tenants=3, n_requests=150, dims=(64, 128, 70), seed=12)
    tenants = {0: a.tenants[0], 1: b.tenants[0], 2: a.tenants[1], 3: b.tenants[2]}
    ids = np.random.default_rng(5).integers(0, 4, 150).astype(np.int32)
    w = wl.Workload("mixed", "bf16", tenants, ids, a.inputs)
    ctx = make_context(w)
    gpu = gpu_run(ctx, w, poison=True)
    compare(w, gpu, oracle_rows(w), what="mixed-classes")
    ctx.close()


def test_more_than_1024_tenants():
    # two tenants per batcher thread (the wide instantiation of the segmentation kernel), most with
    # one or two rows, some with none
    w = wl.c2(n_tenants=1500, n_requests=2600, dims=(24, 40, 6), s=0.3)
    assert len(w.counts()) < 1500
    ctx = make_context(w)
    gpu = gpu_run(ctx, w, poison=True)
    counts = ctx.last_counts()
    assert np.array_equal(counts, np.bincount(w.tenant_ids, minlength=len(counts)))
    compare(w, gpu, oracle_rows(w), what="1500-tenants")
    ctx.close()


def test_deepest_model_and_head_boundaries():
    # eight layers, and class counts on both sides of the fused-head boundary (32 | 33)
    deep = wl.c2(n_tenants=2, n_requests=90, dims=(40, 72, 64, 96, 64, 136, 64, 48, 32), seed=31)   # 8 FC layers, 32 classes
    wide = wl.c2(n_tenants=2, n_requests=90, dims=(40, 80, 33), seed=32)                              # 33 classes
    tenants = {0: deep.tenants[0], 1: wide.tenants[0], 2: deep.tenants[1], 3: wide.tenants[1]}
    assert len(tenants[0].layers) == 8                  # one whole group of layer indices of the segmentation kernel
    ids = np.random.default_rng(6).integers(0, 4, 90).astype(np.int32)
    w = wl.Workload("deep+boundary", "bf16", tenants, ids, deep.inputs)
    ctx = make_context(w)
    gpu = gpu_run(ctx, w, poison=True)
    compare(w, gpu, oracle_rows(w), what="deep+boundary")
    ctx.close()


def test_large_batch_in_several_submissions():
    # >= 8192 rows: the rows are ranked by a kernel of its own, spread over the chip, from one
    # submission and from a mix of batch and per-tenant submissions; a few ids are unknown
    base = wl.c2(n_tenants=6, n_requests=9100, dims=(64, 96, 10), seed=41)
    ids = base.tenant_ids.copy()
    ids[3000:3500] = 2                                   # will be one per-tenant submission
    w = wl.Workload("large-mixed", base.dtype, base.tenants, ids, base.inputs)
    ctx = make_context(w)
    ref = gpu_run(ctx, w, poison=True)
    compare(w, ref, oracle_rows(w), what="large, one submission")

    d_x = torch_io.to_device(w.inputs, w.dtype)
    d_ids = torch.from_numpy(ids).cuda()
    es, K = d_x.element_size(), d_x.shape[1]
    assert ctx.submit_batch(d_ids.data_ptr(), d_x.data_ptr(), 3000, K) == 0
    assert ctx.submit(2, d_x.data_ptr() + 3000 * K * es, 500) == 3000
    assert ctx.submit_batch(d_ids.data_ptr() + 3500 * 4, d_x.data_ptr() + 3500 * K * es, 9100 - 3500, K) == 3500
    out = torch_io.alloc_outputs(w.n_requests, ctx.cfg.max_classes)
    n = ctx.run(torch.cuda.current_stream().cuda_stream, out.labels.data_ptr(), out.probs.data_ptr(),
                out.logits.data_ptr(), out.n_classes.data_ptr(), w.n_requests, ctx.cfg.max_classes)
    torch.cuda.synchronize()
    assert n == w.n_requests
    assert np.array_equal(out.logits.cpu().numpy().astype(np.float64), ref[0])
    assert np.array_equal(out.labels.cpu().numpy(), ref[2])

    bad = ids.copy()
    bad[[5, 4100, 9099]] = [77, -3, 6]
    lg, pr, lb, nc = gpu_run(ctx, w, ids=bad)
    rej = np.isin(np.arange(len(ids)), [5, 4100, 9099])
    assert np.all(lb[rej] == -1) and np.all(nc[rej] == 0) and np.all(lg[rej] == 0)
    assert np.array_equal(lg[~rej], ref[0][~rej]) and np.array_equal(lb[~rej], ref[2][~rej])
    ctx.close()


def test_two_runs_in_flight_on_two_streams():
    # run_slots = 2: consecutive runs alternate between two sets of device scratch and may overlap on
    # different streams; every run still gives exactly the answers of a run on its own
    wa = wl.c2(n_tenants=6, n_requests=700, dims=(100, 192, 136, 10), seed=51)
    wb = wl.Workload("other batch", wa.dtype, wa.tenants, wl.c2(n_tenants=6, n_requests=450, dims=(100, 192, 136, 10), seed=52).tenant_ids,
                     wl.c2(n_tenants=6, n_requests=450, dims=(100, 192, 136, 10), seed=52).inputs)
    single = make_context(wa)
    ref_a, ref_b = gpu_run(single, wa), gpu_run(single, wb)
    single.close()
    compare(wa, ref_a, oracle_rows(wa), what="batch a"); compare(wb, ref_b, oracle_rows(wb), what="batch b")

    ctx = mt.context_for(wa.tenants, wa.dtype, 700, run_slots=2)
    mt.register_tenants(ctx, wa.tenants)
    dev = [(torch.from_numpy(w.tenant_ids).cuda(), torch_io.to_device(w.inputs, w.dtype)) for w in (wa, wb)]
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    torch.cuda.synchronize()
    outs = []
    for i in range(6):                                   # a, b, a, b, ... without waiting in between
        ids, x = dev[i % 2]
        outs.append(mt.serve(ctx, ids, x, stream=streams[i % 2]))
    # a third stream takes a slot that another stream used last: it has to wait for that run
    outs.append(mt.serve(ctx, *dev[0], stream=torch.cuda.Stream()))
    torch.cuda.synchronize()
    for i, o in enumerate(outs):
        ref = ref_a if i % 2 == 0 else ref_b
        assert np.array_equal(o.logits.cpu().numpy().astype(np.float64), ref[0]), i
        assert np.array_equal(o.labels.cpu().numpy(), ref[2]), i
    assert ctx.last_counts().sum() == 700
    ctx.close()


@pytest.mark.parametrize("dtype_mix", ["f32", "bf16"])
def test_small_runs_agree_with_the_oracle_in_both_tile_shapes(monkeypatch, dtype_mix):
    """A run whose layer launches would be a few dozen tiles takes FC tiles of one column block with K
    split over the waves; the ordinary shape stays available through MT_NO_AUTO_SPLIT_K.  Both must give
    the oracle's answers, for wide hidden layers (several column blocks), a fused head and more than 32
    classes (separate head)."""
    if dtype_mix == "f32":
        w = wl.c1(n_tenants=3, n_requests=70, dims=(96, 256, 160, 10), seed=61)
    else:
        a = wl.c2(n_tenants=2, n_requests=90, dims=(104, 256, 192, 10), seed=62)
        b = wl.c2(n_tenants=2, n_requests=90, dims=(104, 320, 40), seed=63)                  # 40 classes: not fused
        tenants = {0: a.tenants[0], 1: a.tenants[1], 2: b.tenants[0], 3: b.tenants[1]}
        ids = np.concatenate([a.tenant_ids[:45], b.tenant_ids[:45] + 2]).astype(np.int32)
        w = wl.Workload("two-shapes", "bf16", tenants, ids, np.concatenate([a.inputs[:45], b.inputs[:45]]))
    ref = oracle_rows(w)
    results = []
    for env in ({"MT_NO_AUTO_SPLIT_K": "1"}, {}):
        monkeypatch.delenv("MT_NO_AUTO_SPLIT_K", raising=False)
        for k, v in env.items():
            monkeypatch.setenv(k, v)
        ctx = make_context(w)
        gpu = gpu_run(ctx, w, poison=True)
        compare(w, gpu, ref, what="small-run %s %s" % (dtype_mix, "ordinary" if env else "k-split"))
        results.append(gpu)
        ctx.close()
    # the two shapes add the same products in different orders: close, not necessarily equal
    np.testing.assert_allclose(results[0][0], results[1][0], rtol=5e-2, atol=5e-2)


def test_tiny_run_among_many_registered_models():
    """The tile shape of a run follows the tenants that can have rows (at most one per request), not the
    number of registered models: 150 models, 40 requests to three of them."""
    w = wl.c2(n_tenants=150, n_requests=40, dims=(64, 256, 10), s=0.3, seed=71)
    w.tenant_ids = np.array([7, 93, 149], dtype=np.int32)[np.arange(40) % 3]
    ctx = make_context(w)
    gpu = gpu_run(ctx, w, poison=True)
    counts = ctx.last_counts()
    assert counts.sum() == 40 and counts[7] == 14 and counts[93] == 13 and counts[149] == 13
    compare(w, gpu, oracle_rows(w), what="tiny run, many models")
    ctx.close()


def test_served_requests_are_counted_per_tenant():
    w = wl.c2(n_tenants=6, n_requests=300, dims=(100, 192, 136, 10))
    ctx = mt.context_for(w.tenants, w.dtype, w.n_requests, max_tenants=8, run_slots=2)
    mt.register_tenants(ctx, w.tenants)
    d_x = torch_io.to_device(w.inputs, w.dtype)
    ids = w.tenant_ids.copy()
    ids[[3, 77]] = [7, -1]                                  # two rejected rows: served for nobody
    only_some = np.where(ids == 4, 2, ids)                  # second mix: tenant 4 has no traffic
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    torch.cuda.synchronize()
    for i, v in enumerate((ids, only_some, ids)):
        mt.serve(ctx, torch.from_numpy(v.astype(np.int32)).cuda(), d_x, stream=streams[i % 2])
    torch.cuda.synchronize()
    for t in range(6):
        acc = ctx.tenant_account(t)
        expect = 2 * int((ids == t).sum()) + int((only_some == t).sum())
        assert acc["requests"] == expect, t
        assert acc["runs"] == (2 if t == 4 else 3), t
    ctx.close()


def test_heads_of_33_to_128_classes_are_finished_by_the_fc_tile(monkeypatch):
    """Class counts around every boundary of the fused head (one column block: 32 | 33; one tile of
    four: 64 | 65, 96 | 97, 128 | 129), several row tiles per tenant and ragged ones: the tile's own
    softmax/argmax must give the oracle's answers and exactly the logits of the separate head kernel.
    With at most 128 classes everywhere no head kernel runs at all."""
    monkeypatch.setenv("MT_NO_AUTO_SPLIT_K", "1")                 # the ordinary tile shape also for this small run
    for name, classes in (("no head launch", (33, 64, 65, 96, 97, 100, 128, 10)), ("head for the widest only", (40, 128, 129, 300, 32))):
        tenants, parts = {}, []
        for t, c in enumerate(classes):
            m = wl.c2(n_tenants=1, n_requests=1, dims=(72, 160, c), seed=90 + t)
            tenants[t] = m.tenants[0]
        rng = np.random.default_rng(17)
        ids = rng.choice(len(classes), size=900, p=np.array([8, 1, 3, 1, 5, 2, 1, 1][:len(classes)]) / sum([8, 1, 3, 1, 5, 2, 1, 1][:len(classes)])).astype(np.int32)
        x = wl.round_to_bf16(rng.standard_normal((900, 72)).astype(np.float32))
        w = wl.Workload(name, "bf16", tenants, ids, x)
        ref = oracle_rows(w)
        ctx = make_context(w)
        fused = gpu_run(ctx, w, poison=True)
        n_fused = ctx.stats()["last_run_launches"]
        compare(w, fused, ref, what=name)
        ctx.close()
        monkeypatch.setenv("MT_NO_FUSED_HEAD", "1")
        ctx = make_context(w)
        plain = gpu_run(ctx, w, poison=True)
        n_plain = ctx.stats()["last_run_launches"]
        ctx.close()
        monkeypatch.delenv("MT_NO_FUSED_HEAD")
        assert n_plain - n_fused == (1 if max(classes) <= 128 else 0), name
        assert np.array_equal(fused[0], plain[0]) and np.array_equal(fused[2], plain[2]) and np.array_equal(fused[3], plain[3])
        assert np.allclose(fused[1], plain[1], rtol=1e-6, atol=1e-7)


@pytest.mark.parametrize("static", [False, True])
def test_a_run_captured_in_a_graph_replays_to_the_same_answers(static):
    """Callers with launch-bound loops capture a run in a HIP graph: the run makes no call that a capturing stream
    refuses (mt_run_static, which allocates nothing, clears with kernels), and every replay gives the bits of the
    eager run, with eager runs and synchronisations of the same context between the replays."""
    w = wl.resnet(n_tenants=2, n_requests=6, hw=16, widths=(16, 32, 64, 128), classes=10, seed=301) if not static else wl.c1(n_tenants=5, n_requests=300, seed=302)
    ctx = make_context(w)
    ids = torch.from_numpy(w.tenant_ids).cuda()
    x = torch_io.to_device(w.inputs, w.dtype)
    eager = torch_io.alloc_outputs(w.n_requests, ctx.cfg.max_classes)
    replayed = torch_io.alloc_outputs(w.n_requests, ctx.cfg.max_classes)
    mt.serve(ctx, ids, x, out=eager, static=static)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.graph(g, stream=s):
        mt.serve(ctx, ids, x, out=replayed, stream=s, static=static)
    torch.cuda.synchronize()
    for _ in range(4):
        replayed.logits.zero_(); replayed.probs.zero_(); replayed.labels.fill_(-7)
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(replayed.logits, eager.logits) and torch.equal(replayed.labels, eager.labels) and torch.equal(replayed.probs, eager.probs)
        half = mt.serve(ctx, ids[: w.n_requests // 2].contiguous(), x[: w.n_requests // 2].contiguous(), static=static)    # eager work of another size in between
        torch.cuda.synchronize()
        assert torch.equal(half.labels, eager.labels[: w.n_requests // 2])
    assert np.array_equal(eager.labels.cpu().numpy(), oracle_rows(w)[2])
    ctx.close()
