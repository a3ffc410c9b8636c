"""mt_run_static, the entry point that allocates nothing: the same run as mt_run with its scratch in
the library's static device array.  Checked against mt_run, bit for bit, through the C ABI: two calls
in a row, the second with a smaller batch (the array keeps what the first one left), then a CNN mix, residual networks,
a run on another stream, and a run that does not fit the array (refused, nothing enqueued, mt_run
still serves it)."""
import numpy as np
import pytest
import torch

import paper_1901_06887_amd as mt
import workloads as wl
from paper_1901_06887_amd import binding as B
from paper_1901_06887_amd import torch_io

pytestmark = pytest.mark.gpu


def both_ways(ctx, w, rows, stream=None):
    ids = torch.from_numpy(np.ascontiguousarray(w.tenant_ids[rows])).cuda()
    x = torch_io.to_device(w.inputs[rows], w.dtype)
    got = mt.serve(ctx, ids, x, stream=stream, static=True)
    torch.cuda.synchronize()
    counts = ctx.last_counts()
    want = mt.serve(ctx, ids, x)
    torch.cuda.synchronize()
    assert np.array_equal(counts, np.bincount(w.tenant_ids[rows], minlength=len(counts)))
    assert np.array_equal(counts, ctx.last_counts())
    for a, b in ((got.labels, want.labels), (got.n_classes, want.n_classes), (got.logits, want.logits), (got.probs, want.probs)):
        assert torch.equal(a, b)
    assert int((got.labels < 0).sum()) == 0
    return got


def test_static_run_matches_mt_run_on_two_calls_in_a_row_the_second_smaller():
    w = wl.c2(n_tenants=6, n_requests=700, dims=(200, 320, 272, 10), seed=81)
    ctx = mt.context_for(w.tenants, w.dtype, w.n_requests, max_tenants=8)
    mt.register_tenants(ctx, w.tenants)
    both_ways(ctx, w, np.arange(700))
    # smaller batch, fewer tenants with traffic: stale descriptors of the first run must not show
    rows = np.flatnonzero(np.isin(w.tenant_ids, [1, 4]))[:150]
    assert 0 < len(rows) <= 150
    both_ways(ctx, w, rows)
    both_ways(ctx, w, np.arange(0, 700, 2), stream=torch.cuda.Stream())      # another stream: ordered behind the last static run
    ctx.close()


def test_static_run_serves_a_cnn_mix_and_a_second_context():
    w = wl.c4(n_tenants=3, n_requests=40, hw=16, seed=82)
    ctx = mt.context_for(w.tenants, w.dtype, w.n_requests)
    mt.register_tenants(ctx, w.tenants)
    both_ways(ctx, w, np.arange(40))
    w2 = wl.c1(n_tenants=3, n_requests=50, dims=(64, 96, 10), seed=83)       # fp32, another context, same device array
    ctx2 = mt.context_for(w2.tenants, w2.dtype, w2.n_requests)
    mt.register_tenants(ctx2, w2.tenants)
    both_ways(ctx2, w2, np.arange(50))
    both_ways(ctx, w, np.arange(7))
    w3 = wl.resnet(n_tenants=2, n_requests=12, hw=32, widths=(16, 32, 64, 128), classes=10, seed=85)   # skip connections: three activation buffers in the array
    ctx3 = mt.context_for(w3.tenants, w3.dtype, w3.n_requests)
    mt.register_tenants(ctx3, w3.tenants)
    both_ways(ctx3, w3, np.arange(12))
    both_ways(ctx3, w3, np.arange(5))
    ctx.close(); ctx2.close(); ctx3.close()


def test_static_run_refuses_what_does_not_fit_and_keeps_the_pending_rows():
    w = wl.c5(n_tenants=2, n_requests=3000, dims=(4096, 512, 10), seed=84)    # two activation buffers of ~25 MB each
    ctx = mt.context_for(w.tenants, w.dtype, w.n_requests)
    mt.register_tenants(ctx, w.tenants)
    ids = torch.from_numpy(w.tenant_ids).cuda()
    x = torch_io.to_device(w.inputs, w.dtype)
    out = torch_io.alloc_outputs(w.n_requests, ctx.cfg.max_classes)
    s = torch.cuda.current_stream().cuda_stream
    ctx.submit_batch(ids.data_ptr(), x.data_ptr(), w.n_requests, x.shape[1])
    with pytest.raises(B.MtError) as e:
        ctx.run_static(s, out.labels.data_ptr(), out.probs.data_ptr(), out.logits.data_ptr(), out.n_classes.data_ptr(), w.n_requests, ctx.cfg.max_classes)
    assert e.value.status == 1 and "static array" in str(e.value)
    n = ctx.run(s, out.labels.data_ptr(), out.probs.data_ptr(), out.logits.data_ptr(), out.n_classes.data_ptr(), w.n_requests, ctx.cfg.max_classes)
    assert n == w.n_requests                                                 # the refused call left the submission in place
    torch.cuda.synchronize()
    small = mt.serve(ctx, ids[:200].contiguous(), x[:200].contiguous(), static=True)     # 200 rows of the same context fit
    want = mt.serve(ctx, ids[:200].contiguous(), x[:200].contiguous())
    torch.cuda.synchronize()
    assert torch.equal(small.labels, want.labels) and torch.equal(small.logits, want.logits)
    assert torch.equal(small.labels, out.labels[:200])                       # (and the labels of the same rows in the big run)
    ctx.close()
