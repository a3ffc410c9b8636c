"""Host logic of the C ABI that needs no GPU: the library loads, exports every declared
symbol, and a host-only context validates models, accounts for arena space and returns
error codes (never aborts).  No compute call is made here."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_1901_06887_amd as mt
from paper_1901_06887_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def host_ctx(dtype=B.MT_BF16, arena=1 << 22, max_width=4096, max_classes=100, max_requests=1024, max_tenants=16, run_slots=1):
    return B.Context(max_tenants, max_requests, max_width, max_classes, arena, dtype, device=-1, run_slots=run_slots)


def fc(k, n, act=B.MT_ACT_NONE):
    return B.layer_spec(B.MT_FC, act, k, n)


def zeros_for(specs, dtype=B.MT_BF16):
    ws, bs = [], []
    for s in specs:
        if s.kind == B.MT_FC:
            ws.append(np.zeros((s.out_features, s.in_features), dtype=np.uint16 if dtype == B.MT_BF16 else np.float32))
            bs.append(np.zeros(s.out_features, dtype=np.float32))
        elif s.kind == B.MT_CONV2D:
            ws.append(np.zeros((s.out_features, s.in_features, 3, 3), dtype=np.uint16 if dtype == B.MT_BF16 else np.float32))
            bs.append(np.zeros(s.out_features, dtype=np.float32))
        else:
            ws.append(None); bs.append(None)
    return ws, bs


def test_every_declared_symbol_is_exported():
    header = "".join(open(os.path.join(ROOT, "include", h)).read() for h in sorted(os.listdir(os.path.join(ROOT, "include"))) if h.endswith(".h"))
    names = set(re.findall(r"\b(mt_[a-z_]+)\s*\(", header))
    assert {"mt_debug_copy", "mt_get_profile", "mt_model_footprint_get"} <= names      # both headers were read
    assert {"mt_create", "mt_destroy", "mt_register_model", "mt_submit", "mt_submit_batch", "mt_run"} <= names
    lib = B.load_library()
    for n in names:
        assert hasattr(lib, n), n
    assert "gfx950" in mt.version()


def test_struct_layouts_match_header_sizes():
    assert ctypes.sizeof(B.mt_layer_spec) == 48
    assert ctypes.sizeof(B.mt_config) == 40
    assert ctypes.sizeof(B.mt_outputs) == 40


def test_create_rejects_bad_config():
    for kw in (dict(max_tenants=0), dict(max_requests=0), dict(max_width=0), dict(max_classes=0), dict(arena=0),
               dict(max_tenants=5000), dict(dtype=7), dict(run_slots=5)):
        with pytest.raises(B.MtError) as e:
            host_ctx(**kw)
        assert e.value.status == 1


def test_register_validates_the_closed_layer_set():
    c = host_ctx()
    good = [fc(64, 128, B.MT_ACT_RELU), fc(128, 10)]
    c.register_model(0, good, *zeros_for(good))
    cases = [
        ([fc(64, 128, B.MT_ACT_RELU), fc(100, 10)], 5),                         # dims do not chain
        ([B.layer_spec(9, 0, 64, 10)], 5),                                       # unknown kind
        ([fc(64, 10, 7)], 5),                                                    # unknown activation
        ([fc(64, 10, B.MT_ACT_RELU)], 5),                                        # activation on the logits layer
        ([fc(64, 128)] * 0, 5),                                                  # empty
        ([fc(64, 64, B.MT_ACT_RELU)] * B.MT_MAX_LAYERS + [fc(64, 10)], 5),       # too deep
        ([fc(64, 500)], 5),                                                      # more classes than max_classes
        ([fc(8192, 10)], 5),                                                     # wider than max_width
        ([B.layer_spec(B.MT_CONV2D, B.MT_ACT_RELU, 3, 8, 8, 8, 3), fc(8 * 9, 10)], 5),   # stride 3
        ([B.layer_spec(B.MT_CONV2D, B.MT_ACT_RELU, 3, 6, 8, 8, 1), fc(6 * 64, 10)], 5),  # C_out not multiple of 8
    ]
    for specs, status in cases:
        with pytest.raises(B.MtError) as e:
            ws, bs = zeros_for(specs)
            c.register_model(1, specs, ws, bs)
        assert e.value.status == status, (specs, str(e.value))
    assert c.stats()["n_tenants"] == 1
    with pytest.raises(B.MtError) as e:
        c.register_model(0, good, *zeros_for(good))
    assert e.value.status == 4                                                   # MT_EEXIST
    with pytest.raises(B.MtError) as e:
        c.register_model(99, good, *zeros_for(good))
    assert e.value.status == 1


def test_cnn_chain_is_accepted():
    c = host_ctx(max_width=32 * 32 * 32, arena=1 << 22)
    specs = [B.layer_spec(B.MT_CONV2D, B.MT_ACT_RELU, 3, 32, 32, 32, 1),
             B.layer_spec(B.MT_CONV2D, B.MT_ACT_RELU, 32, 64, 32, 32, 2),
             B.layer_spec(B.MT_CONV2D, B.MT_ACT_RELU, 64, 128, 16, 16, 2),
             B.layer_spec(B.MT_GAP, B.MT_ACT_NONE, 128, 128, 8, 8),
             fc(128, 10)]
    c.register_model(3, specs, *zeros_for(specs))
    # packed sizes: K padded to 64 elements per row (conv1: 9*8=72 -> 128), the logits layer's
    # rows padded to 32, 256-byte aligned slices
    exp = sum((n * k * 2 + 255) // 256 * 256 + (n * 4 + 255) // 256 * 256
              for n, k in ((32, 128), (64, 320), (128, 576), (32, 128)))     # conv rows are padded to 32 too (32, 64, 128 already are)
    assert c.stats()["arena_used"] == exp


def test_arena_accounting_exhaustion_and_reuse():
    c = host_ctx(arena=310_000)
    specs = [fc(64, 512, B.MT_ACT_RELU), fc(512, 10)]            # logits rows are stored padded to 32
    per = 512 * 64 * 2 + 512 * 4 + 32 * 512 * 2 + 256
    for t in range(3):
        c.register_model(t, specs, *zeros_for(specs))
    assert c.stats()["arena_used"] == 3 * per
    with pytest.raises(B.MtError) as e:
        c.register_model(3, specs, *zeros_for(specs))
    assert e.value.status == 2                                   # MT_ENOMEM, nothing leaked
    assert c.stats()["arena_used"] == 3 * per and c.stats()["n_tenants"] == 3
    c.unregister_model(1)
    assert c.stats()["arena_used"] == 2 * per
    c.register_model(3, specs, *zeros_for(specs))                # the freed slice is reused
    assert c.stats()["arena_used"] == 3 * per
    for t in (0, 2, 3):
        c.unregister_model(t)
    assert c.stats()["arena_used"] == 0
    with pytest.raises(B.MtError) as e:
        c.unregister_model(0)
    assert e.value.status == 3


def test_submit_errors_and_host_only_run():
    c = host_ctx(max_requests=8)
    specs = [fc(64, 10)]
    c.register_model(2, specs, *zeros_for(specs))
    with pytest.raises(B.MtError) as e:
        c.submit(5, 0x1000, 1)
    assert e.value.status == 3                                   # unknown tenant
    with pytest.raises(B.MtError) as e:
        c.submit(2, 0, 1)
    assert e.value.status == 1                                   # null inputs
    assert c.submit(2, 0x1000, 5) == 0
    assert c.submit(2, 0x9000, 3) == 5
    with pytest.raises(B.MtError) as e:
        c.submit(2, 0x1000, 1)
    assert e.value.status == 6                                   # MT_EFULL
    with pytest.raises(B.MtError) as e:
        c.unregister_model(2)
    assert e.value.status == 7                                   # pending requests
    with pytest.raises(B.MtError) as e:
        c.run(0, 0x1000, 0, 0, 0, 8, 10)
    assert e.value.status == 7                                   # host-only context cannot run


def test_bf16_weights_must_be_representable():
    c = host_ctx()
    specs = [fc(64, 10)]
    with pytest.raises(ValueError):
        c.register_model(0, specs, [np.full((10, 64), 0.1, dtype=np.float32)], [None])


def test_request_cost_and_run_estimate_follow_the_model_description():
    # section 3.2: the cost of a request is known from the model description alone.  The library's
    # figures must equal the closed forms the workload module computes from the layer shapes.
    import paper_1901_06887_amd as mt
    import workloads as wl
    for w in (wl.c2(n_tenants=5, n_requests=300, dims=(100, 192, 136, 10)), wl.c4(n_tenants=3, n_requests=20, hw=8, chans=(3, 16, 24, 40), classes=5)):
        ctx = mt.context_for(w.tenants, w.dtype, w.n_requests, device=-1)
        mt.register_tenants(ctx, w.tenants)
        counts = np.bincount(w.tenant_ids, minlength=ctx.cfg.max_tenants)
        est = ctx.estimate_run(counts)
        cost = wl.algorithmic_cost(w)
        assert est["rows"] == w.n_requests and est["flops"] == cost["flops"] and est["hbm_bytes"] == cost["bytes"]
        assert est["launches"] >= 1 + len(next(iter(w.tenants.values())).layers) - (w.name == "c4") and est["device_ms"] > 0
        one = wl.Workload("one", w.dtype, w.tenants, w.tenant_ids[:1], w.inputs[:1])
        c1 = wl.algorithmic_cost(one)
        acc = ctx.tenant_account(int(w.tenant_ids[0]))
        assert acc["flops_per_request"] == c1["flops"] and acc["weight_bytes"] == c1["weight_bytes"]
        assert acc["io_bytes_per_request"] == c1["act_bytes"] + c1["out_bytes"] and acc["requests"] == 0
        # more work never costs less; an empty run costs nothing
        assert ctx.estimate_run(counts * 2 // 3)["device_ms"] <= est["device_ms"]
        assert ctx.estimate_run(counts * 0)["device_ms"] == 0
        with pytest.raises(B.MtError) as e:
            ctx.estimate_run(counts * 50)
        assert e.value.status == 1
        ctx.unregister_model(0)
        with pytest.raises(B.MtError) as e:
            ctx.estimate_run(counts + 1)
        assert e.value.status == 3
        with pytest.raises(B.MtError) as e:
            ctx.tenant_account(0)
        assert e.value.status == 3
        ctx.close()


def test_model_cache_bookkeeping_on_the_host():
    # cache mode: a full arena evicts the least recently used models instead of failing; models named
    # in one prefetch never give way to one another; a model larger than the arena can never be held
    specs = [fc(256, 256, B.MT_ACT_RELU), fc(256, 10)]            # 256*256*2 + 1 KiB bias + 64*256*2... about 160 KiB each
    c = B.Context(8, 64, 1024, 16, 3 * 170 * 1024, B.MT_BF16, device=-1, cache=True)
    for t in range(5):
        c.register_model(t, specs, *zeros_for(specs))
    resident = [c.tenant_account(t)["resident"] for t in range(5)]
    assert resident == [0, 0, 1, 1, 1] and c.cache_stats()["evictions"] == 2 and c.cache_stats()["resident_models"] == 3
    c.prefetch([0, 3])                                           # 0 comes back; the oldest other model (2) gives way
    assert [c.tenant_account(t)["resident"] for t in range(5)] == [1, 0, 0, 1, 1]
    c.prefetch([3, 0])                                           # nothing to do
    assert c.cache_stats()["evictions"] == 3
    with pytest.raises(B.MtError) as e:
        c.prefetch([0, 1, 2, 3])                                 # four models do not fit together
    assert e.value.status == 2
    with pytest.raises(B.MtError) as e:
        c.prefetch([6])
    assert e.value.status == 3
    big = [fc(1024, 1024, B.MT_ACT_RELU), fc(1024, 10)]
    with pytest.raises(B.MtError) as e:
        c.register_model(7, big, *zeros_for(big))
    assert e.value.status == 2
    # (a prefetch that fails may already have brought in the models named first)
    res = [c.tenant_account(t)["resident"] for t in range(5)]
    assert sum(res) == 3
    est = c.estimate_run([1, 1, 1, 1, 1, 0, 0, 0])               # a run over all five: two have to be brought in first
    assert est["upload_bytes"] == 2 * c.tenant_account(1)["arena_bytes"] and est["upload_ms"] > 0
    counts = [0] * 8
    counts[res.index(1)] = 3
    assert c.estimate_run(counts)["upload_bytes"] == 0 and c.estimate_run(counts)["upload_ms"] == 0
    c.unregister_model(1)                                        # not resident: only its host image goes
    c.unregister_model(0)
    assert c.cache_stats()["resident_models"] == sum(c.tenant_account(t)["resident"] for t in (2, 3, 4))
    c.close()
    # outside cache mode a full arena is an error, as before, and prefetch only checks its arguments
    c = B.Context(8, 64, 1024, 16, 3 * 170 * 1024, B.MT_BF16, device=-1)
    for t in range(3):
        c.register_model(t, specs, *zeros_for(specs))
    with pytest.raises(B.MtError) as e:
        c.register_model(3, specs, *zeros_for(specs))
    assert e.value.status == 2
    c.prefetch([0, 1, 2])
    c.close()


def test_admission_is_max_min_fair_within_the_budget():
    import paper_1901_06887_amd as mt
    import workloads as wl
    w = wl.c3(n_tenants=40, n_requests=6000, in_dim=256, widths=(128, 256), classes=20, seed=4)
    ctx = mt.context_for(w.tenants, w.dtype, 4000, device=-1)          # fewer rows per run than are waiting
    mt.register_tenants(ctx, w.tenants)
    pending = np.bincount(w.tenant_ids, minlength=ctx.cfg.max_tenants)
    everything = ctx.estimate_run(np.minimum(pending, 50))["device_ms"]
    last_level = -1
    for budget in (everything * 0.3, everything * 0.6, everything * 5):
        admitted, est = ctx.admit(pending, budget)
        admitted = np.array(admitted)
        level = admitted.max()
        assert np.array_equal(admitted, np.minimum(pending, level))             # a water level: nobody is passed over
        assert admitted.sum() <= 4000 and est["rows"] == admitted.sum()
        assert est["device_ms"] + est["upload_ms"] <= budget
        assert level >= last_level                                              # a larger budget never admits less
        last_level = level
        if level < pending.max():                                                # one more per tenant would not fit
            more = np.minimum(pending, level + 1)
            assert more.sum() > 4000 or ctx.estimate_run(more)["device_ms"] > budget
    admitted, est = ctx.admit(pending, 1e-4)                                     # nothing fits 0.1 us
    assert sum(admitted) == 0 and est["device_ms"] == 0
    with pytest.raises(B.MtError) as e:
        ctx.admit(pending, 0.0)
    assert e.value.status == 1
    ctx.close()


def test_footprint_of_a_model_is_what_registration_takes():
    """mt_model_footprint_get needs no context: its arena bytes are what mt_register_model takes from
    the arena, its width and class count the smallest limits a context must have."""
    mlp = [fc(784, 1024, B.MT_ACT_RELU), fc(1024, 100, B.MT_ACT_GELU), fc(100, 10)]
    cnn = [B.layer_spec(B.MT_CONV2D, B.MT_ACT_RELU, 3, 32, 16, 16, 1), B.layer_spec(B.MT_CONV2D, B.MT_ACT_RELU, 32, 64, 16, 16, 2),
           B.layer_spec(B.MT_GAP, 0, 64, 64, 8, 8), fc(64, 7)]
    for dtype in (B.MT_BF16, B.MT_F32):
        for specs in (mlp, cnn):
            f = B.model_footprint(specs, dtype)
            c = host_ctx(dtype=dtype, arena=1 << 24, max_width=f["min_width"], max_classes=f["n_classes"])
            c.register_model(3, specs, *zeros_for(specs, dtype))
            assert c.stats()["arena_used"] == f["arena_bytes"]
            assert c.tenant_account(3)["arena_bytes"] == f["arena_bytes"]
            c.close()
            if f["min_width"] > 64:
                c = host_ctx(dtype=dtype, arena=1 << 24, max_width=f["min_width"] - 64, max_classes=f["n_classes"])
                with pytest.raises(B.MtError):
                    c.register_model(3, specs, *zeros_for(specs, dtype))
                c.close()
    assert B.model_footprint(mlp, B.MT_BF16)["in_len"] == 784 and B.model_footprint(cnn, B.MT_BF16)["in_len"] == 16 * 16 * 3
    es = 2
    assert B.model_footprint(mlp, B.MT_BF16)["arena_bytes"] == sum(
        (n * k * es + 255) // 256 * 256 + (n * 4 + 255) // 256 * 256 for n, k in ((1024, 832), (128, 1024), (32, 128)))
    with pytest.raises(B.MtError) as e:
        B.model_footprint([fc(64, 10, B.MT_ACT_RELU)], B.MT_BF16)       # activation on the logits layer
    assert e.value.status == 5


def test_wider_catalogue_is_validated():
    """Window sizes, skip sources and shapes of the wider layer set (paper section 3.1: a pre-defined set of
    supported layer types): what is outside it is refused with MT_EUNSUPPORTED and allocates nothing."""
    c = host_ctx(max_width=1 << 16)
    conv = lambda ci, co, hw, k, s=1, act=B.MT_ACT_RELU, src=0: B.layer_spec(B.MT_CONV2D, act, ci, co, hw, hw, s, ksize=k, pad=(k - 1) // 2, src=src)
    pool = lambda ch, hw, k=3, s=2, p=1: B.layer_spec(B.MT_MAXPOOL, 0, ch, ch, hw, hw, s, ksize=k, pad=p)
    add = lambda ch, hw, src2, src=0, act=B.MT_ACT_RELU: B.layer_spec(B.MT_ADD, act, ch, ch, hw, hw, src=src, src2=src2)
    gap = lambda ch, hw: B.layer_spec(B.MT_GAP, 0, ch, ch, hw, hw)
    block = [conv(3, 16, 16, 7, 2), pool(16, 8), conv(16, 16, 4, 3), conv(16, 16, 4, 3, act=0), add(16, 4, src2=2),
             conv(16, 32, 4, 3, 2), conv(32, 32, 2, 3, act=0), conv(16, 32, 4, 1, 2, act=0, src=5), add(32, 2, src=7, src2=8), gap(32, 2), fc(32, 5)]
    def zeros(specs):
        ws, bs = [], []
        for sp in specs:
            if sp.kind == B.MT_FC:
                ws.append(np.zeros((sp.out_features, sp.in_features), dtype=np.uint16)); bs.append(np.zeros(sp.out_features, dtype=np.float32))
            elif sp.kind == B.MT_CONV2D:
                ws.append(np.zeros((sp.out_features, sp.in_features, sp.kh, sp.kw), dtype=np.uint16)); bs.append(np.zeros(sp.out_features, dtype=np.float32))
            else:
                ws.append(None); bs.append(None)
        return ws, bs
    c.register_model(0, block, *zeros(block))
    used = c.stats()["arena_used"]
    assert used == B.model_footprint(block, B.MT_BF16)["arena_bytes"] > 0
    def bad(i, spec):
        m = list(block); m[i] = spec
        return m
    cases = [bad(0, conv(3, 16, 16, 5, 2)),                       # 5x5 window
             bad(0, B.layer_spec(B.MT_CONV2D, 1, 3, 16, 16, 16, 2, ksize=7, pad=1)),   # pad that is not (k - 1) / 2
             bad(1, pool(16, 8, k=4)), bad(1, pool(16, 8, k=2, p=2)),                 # window / padding outside the set
             bad(4, add(16, 4, src2=0)),                         # an addition without a second source
             bad(4, add(16, 4, src2=1)),                         # second source of another shape (the stem's 8x8 image)
             bad(4, add(16, 4, src2=6)),                         # a source that comes later
             bad(7, conv(16, 32, 4, 1, 2, act=0, src=7)),        # projection reading a 2x2x32 image as 4x4x16
             bad(2, B.layer_spec(B.MT_CONV2D, 1, 16, 16, 4, 4, 1, src2=1)),           # only additions take a second source
             bad(10, gap(32, 2)),                                # the last layer must be FC
             [conv(3, 16, 8, 3), fc(8 * 8 * 16, 5)],             # FC straight after an image
             [conv(3, 16, 8, 3), gap(16, 8), add(16, 1, src2=1), fc(16, 5)]]           # adding a vector
    for specs in cases:
        with pytest.raises(B.MtError) as e:
            c.register_model(1, specs, *zeros(specs))
        assert e.value.status == 5, [s.kind for s in specs]
        with pytest.raises(B.MtError):
            B.model_footprint(specs, B.MT_BF16)
    assert c.stats()["arena_used"] == used and c.stats()["n_tenants"] == 1
    # five values alive at once: more than the four activation buffers of a run
    wide = [conv(3, 8, 8, 3), conv(8, 8, 8, 3), conv(8, 8, 8, 3, src=1), conv(8, 8, 8, 3, src=1), conv(8, 8, 8, 3, src=1),
            add(8, 8, src=2, src2=3), add(8, 8, src2=4), add(8, 8, src2=5), add(8, 8, src2=1), gap(8, 8), fc(8, 3)]
    with pytest.raises(B.MtError) as e:
        c.register_model(1, wide, *zeros(wide))
    assert e.value.status == 5 and "alive" in str(e.value)
    # batch normalisation can only follow a convolution, and needs a positive variance
    bn = [None] * len(block)
    bn[1] = (np.ones(16), np.zeros(16), np.zeros(16), np.ones(16))
    with pytest.raises(B.MtError) as e:
        c.register_model(1, block, *zeros(block), bn=bn)
    assert e.value.status == 5
    bn = [None] * len(block)
    bn[0] = (np.ones(16), np.zeros(16), np.zeros(16), -np.ones(16))
    with pytest.raises(B.MtError) as e:
        c.register_model(1, block, *zeros(block), bn=bn)
    assert e.value.status == 1
    c.close()


def test_additions_are_planned_into_the_convolution_in_front_of_them(monkeypatch):
    """Host planning only: an addition whose operand is the output of the convolution right before it, read by nothing
    else, costs no launch (the run estimate counts launches as mt_run enqueues them); one whose convolution output has a
    second reader, or that follows a pooling layer, keeps its launch; MT_NO_FUSED_ADD=1 keeps them all."""
    import workloads as wl
    conv = lambda ci, co, hw, k=3, s=1, act=wl.ACT_RELU, src=0: wl.LayerSpec(wl.CONV, act, ci, co, hw, hw, s, ksize=k, pad=(k - 1) // 2, src=src)
    add = lambda ch, hw, src2, src=0, act=wl.ACT_RELU: wl.LayerSpec(wl.ADD, act, ch, ch, hw, hw, src=src, src2=src2)
    pool = lambda ch, hw: wl.LayerSpec(wl.MAXPOOL, wl.ACT_NONE, ch, ch, hw, hw, 1, ksize=3, pad=1)
    tail = lambda ch, hw: [wl.LayerSpec(wl.GAP, wl.ACT_NONE, ch, ch, hw, hw), wl.LayerSpec(wl.FC, wl.ACT_NONE, ch, 4)]
    c = 16
    taken = [conv(3, c, 8), conv(c, c, 8), conv(c, c, 8, act=wl.ACT_NONE), add(c, 8, src2=1)] + tail(c, 8)                 # 1 addition, taken over
    swapped = [conv(3, c, 8), conv(c, c, 8), conv(c, c, 8, act=wl.ACT_NONE), add(c, 8, src=1, src2=3)] + tail(c, 8)       # the same with the operands swapped
    shared = [conv(3, c, 8), conv(c, c, 8, act=wl.ACT_NONE), add(c, 8, src2=1), add(c, 8, src=2, src2=3)] + tail(c, 8)     # the convolution's output has two readers
    pooled = [conv(3, c, 8), conv(c, c, 8), pool(c, 8), add(c, 8, src2=1)] + tail(c, 8)                                   # the addition follows a pooling layer
    def launches(layers):
        w = wl.Workload("m", "bf16", {0: wl.make_model(layers, "bf16", 5, 0)}, np.zeros(3, dtype=np.int32), np.zeros((3, 8 * 8 * 3), dtype=np.float32))
        ctx = mt.context_for(w.tenants, w.dtype, 3, device=-1)
        mt.register_tenants(ctx, w.tenants)
        n = ctx.estimate_run(np.array([3], dtype=np.uint32))["launches"]
        ctx.close()
        return n
    monkeypatch.setenv("MT_NO_FUSED_ADD", "1")
    plain = {k: launches(v) for k, v in (("taken", taken), ("swapped", swapped), ("shared", shared), ("pooled", pooled))}
    monkeypatch.delenv("MT_NO_FUSED_ADD")
    fused = {k: launches(v) for k, v in (("taken", taken), ("swapped", swapped), ("shared", shared), ("pooled", pooled))}
    assert fused["taken"] == plain["taken"] - 1 and fused["swapped"] == plain["swapped"] - 1
    assert fused["shared"] == plain["shared"] and fused["pooled"] == plain["pooled"]


def test_which_rows_and_layers_the_compute_bound_kernels_take():
    """The two pure functions that let a benchmark attribute flops and launches: a tenant-layer takes big tiles
    from 2048 rows and 192 (padded) outputs on, a last row tile of at most 128 rows is left to the streaming kernel,
    and the tiles are walked by one workgroup per compute unit when the fan-in, padded to 64, is at least 256."""
    assert mt.debug_big_tile_rows(2047, 4096) == 0 and mt.debug_big_tile_rows(4096, 160) == 0
    assert mt.debug_big_tile_rows(2048, 192) == 2048 and mt.debug_big_tile_rows(2048, 161) == 2048
    assert mt.debug_big_tile_rows(4096 + 128, 4096) == 4096 and mt.debug_big_tile_rows(4096 + 129, 4096) == 4096 + 129
    assert [mt.debug_big_tile_walk(k) for k in (64, 192, 193, 256, 4096)] == [False, False, True, True, True]


def test_row_tiling_of_convolution_layers():
    """3x3 convolutions at stride 1 are cut into tiles of whole output rows whose input rows (the tile's rows, one above,
    one below, a pixel left and right, 16 bytes of padding per pixel) fit 96 KiB of LDS: as many rows as fit 128 pixels,
    fewer when the frame would not fit; images of at most 64 pixels share a tile, 2, 4 or 8 of them.  Everything else
    (stride 2, other windows, rows wider than a tile) is left to the gathering kernels."""
    t = mt.debug_conv_row_tiling
    frame = lambda rows, images, w, cin, es=2: images * (rows + 2) * (w + 2) * (cin * es + 16)
    assert t(56, 56, 64) == {"rows_per_tile": 2, "images_per_tile": 1, "tiles_per_image": 28, "frame_bytes": frame(2, 1, 56, 64)}
    assert t(28, 28, 128) == {"rows_per_tile": 4, "images_per_tile": 1, "tiles_per_image": 7, "frame_bytes": frame(4, 1, 28, 128)}
    assert t(14, 14, 256) == {"rows_per_tile": 9, "images_per_tile": 1, "tiles_per_image": 2, "frame_bytes": frame(9, 1, 14, 256)}
    assert t(7, 7, 512) == {"rows_per_tile": 7, "images_per_tile": 1, "tiles_per_image": 1, "frame_bytes": frame(7, 1, 7, 512)}   # two images would take 168 KiB
    assert t(7, 7, 64) == {"rows_per_tile": 7, "images_per_tile": 2, "tiles_per_image": 1, "frame_bytes": frame(7, 2, 7, 64)}
    assert t(4, 4, 32)["images_per_tile"] == 8 and t(6, 6, 32)["images_per_tile"] == 2 and t(8, 8, 16)["images_per_tile"] == 2
    assert t(32, 32, 3) == {"rows_per_tile": 4, "images_per_tile": 1, "tiles_per_image": 8, "frame_bytes": 6 * 34 * 16}        # a padded 3-channel pixel is one 16-byte chunk
    assert t(12, 12, 24) is None and t(12, 12, 24, elem_size=4)["rows_per_tile"] == 10     # channels in whole k steps: 16 bf16, 8 fp32 elements
    assert t(14, 14, 512)["rows_per_tile"] == 3 and t(14, 14, 512)["frame_bytes"] == frame(3, 1, 14, 512) <= 96 * 1024           # rows given up until the frame fits
    assert t(14, 14, 1024) is None                                                                                             # not even one row does
    assert t(56, 56, 64, stride=2) is None and t(56, 56, 64, ksize=1) is None and t(224, 224, 3, ksize=7, stride=2) is None
    assert t(8, 200, 16) is None                                                                                               # a row is wider than a tile
