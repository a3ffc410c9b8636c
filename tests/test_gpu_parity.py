"""GPU parity: the HIP path behind the C ABI against the fp64 oracle, element by element on
the same seeded inputs.  Reduced cases span several workgroup tiles and ragged tails; the
full-size cases run in the launch configuration the benchmark times and are checked on
rows the oracle evaluates one by one (all rows where that takes seconds)."""
import numpy as np
import pytest
import torch

import workloads as wl
from gpu_common import compare, gpu_run, make_context, oracle_rows, sample_rows

pytestmark = pytest.mark.gpu


def run_and_compare(w, what, poison=True, min_clean_frac=None):
    ctx = make_context(w)
    gpu = gpu_run(ctx, w, poison=poison)
    counts = ctx.last_counts()
    exp = np.bincount(w.tenant_ids, minlength=len(counts))
    assert np.array_equal(counts, exp), what
    worst = compare(w, gpu, oracle_rows(w), what=what, min_clean_frac=min_clean_frac)
    print("%s: worst per-tensor rel fro %.2e, flip-free rows %.3f" % (what, worst, compare.last_clean_frac), flush=True)
    ctx.close()


# ---- reduced cases (seconds on the oracle, several tiles, ragged tails) --------------------
def test_c1_full_fp32():
    run_and_compare(wl.c1(), "c1")


def test_c1_fp32_is_tight():
    w = wl.c1()
    ctx = make_context(w)
    lg, pr, lb, _ = gpu_run(ctx, w)
    o = oracle_rows(w)
    assert np.linalg.norm(lg[:, :10] - o[0]) / np.linalg.norm(o[0]) < 2e-6   # true fp32 arithmetic, not bf16
    ctx.close()


def test_c2_reduced_skewed_batches():
    run_and_compare(wl.c2(n_tenants=12, n_requests=900, dims=(784, 320, 272, 10)), "c2-reduced")


def test_c3_reduced_heterogeneous_depths():
    w = wl.c3(n_tenants=24, n_requests=1200, in_dim=200, widths=(96, 160, 288), classes=100)
    assert len({len(m.layers) for m in w.tenants.values()}) >= 4
    run_and_compare(w, "c3-reduced")


def test_c4_reduced_cnn():
    run_and_compare(wl.c4(n_tenants=3, n_requests=24), "c4-reduced")


def test_c4_small_images_stride_and_ragged_tiles():
    run_and_compare(wl.c4(n_tenants=2, n_requests=7, hw=8, chans=(3, 16, 24, 40), classes=5), "c4-small")


def test_c5_reduced_gelu_wide_head():
    run_and_compare(wl.c5(n_tenants=2, n_requests=520, dims=(512, 384, 512, 256, 1000)), "c5-reduced")


# A layer index gets big tiles only when its qualifying tenants make enough of them to fill
# the chip; the reduced cases lower that bar to one tile so that they reach the big kernel.
@pytest.fixture
def big_tiles_always(monkeypatch):
    monkeypatch.setenv("MT_BIG_MIN_TILES", "1")


def test_big_tile_path_reduced(big_tiles_always):
    # >= 2048 rows per tenant: the compute-bound 256x256 tiles, with ragged row and column tiles,
    # a hidden GELU epilogue and a wide (200-class) logits epilogue
    w = wl.c5(n_tenants=3, n_requests=8400, dims=(192, 320, 448, 200))
    assert min(w.counts().values()) >= 2048
    run_and_compare(w, "c5-big-reduced")


def test_big_tenants_leave_a_short_remainder_to_the_streaming_kernel(big_tiles_always):
    # rows past the last full 256-row tile: 40 and 128 (streamed), 129 (a ragged big tile), 0
    counts = [2048 + 40, 2304 + 128, 2048 + 129, 2304]
    base = wl.c5(n_tenants=4, n_requests=sum(counts), dims=(192, 320, 448, 200), seed=15)
    ids = np.random.default_rng(15).permutation(np.repeat(np.arange(4), counts)).astype(np.int32)
    w = wl.Workload("big+remainder", base.dtype, base.tenants, ids, base.inputs)
    assert [w.counts()[t] for t in range(4)] == counts
    run_and_compare(w, "big+remainder")


def test_big_tiles_of_tenants_with_different_layer_shapes(big_tiles_always):
    # four tenants, each with >= 2048 rows, whose layers at the same index differ in fan-in, width and activation:
    # the workgroups that walk the big tiles pass from a tile of one reduction length to a tile of another (10, 14,
    # 16, 20 stages of the operand ring), from GELU to ReLU, from a full column tile to a ragged one; the third
    # tenant's second layer (K = 192) keeps the whole layer index on the one-tile-per-workgroup kernel
    dims = [(320, 512, 384, 100), (320, 448, 640, 50), (320, 320, 192, 40), (320, 640, 256, 200)]
    acts = [wl.ACT_GELU, wl.ACT_RELU, wl.ACT_GELU, wl.ACT_RELU]
    tenants = {t: wl.make_model(wl.mlp_layers(list(d), a), "bf16", 33, t) for t, (d, a) in enumerate(zip(dims, acts))}
    counts = [2048 + 300, 2304, 2048 + 64, 2560 + 129]
    ids = np.random.default_rng(33).permutation(np.repeat(np.arange(4), counts)).astype(np.int32)
    x = wl.round_to_bf16(np.random.default_rng(34).standard_normal((sum(counts), 320)).astype(np.float32))
    run_and_compare(wl.Workload("big-mixed-shapes", "bf16", tenants, ids, x), "big-mixed-shapes")


def test_big_and_streaming_tenants_in_one_run(big_tiles_always):
    w = wl.c2(n_tenants=5, n_requests=8300, dims=(128, 320, 256, 40), s=2.2)    # one tenant dominates
    c = w.counts()
    assert max(c.values()) >= 2048 and min(c.values()) < 256
    run_and_compare(w, "big+streaming")


def test_few_big_tiles_fall_back_to_the_streaming_kernel():
    # same mix at the default bar: the dominant tenant's few big tiles go to the streaming
    # kernel instead, and the answers still match
    w = wl.c2(n_tenants=5, n_requests=8300, dims=(128, 320, 256, 40), s=2.2)
    run_and_compare(w, "big-fallback")


def test_fp32_big_tiles(big_tiles_always):
    w = wl.c1(n_tenants=2, n_requests=8200, dims=(64, 256, 10))
    assert min(w.counts().values()) >= 2048
    run_and_compare(w, "fp32-big")


def test_big_tiles_long_reductions(big_tiles_always):
    # K = 2048 (64 stages of the operand ring per tile, walked by one workgroup per CU): 9 row tiles with a
    # ragged last one (5 row blocks), 9 full ones beside a streamed remainder, 16; a ragged second column
    # tile (320 outputs), a logits epilogue (200 classes, 7 column blocks), and a short layer in between (K = 320)
    counts = [2048 + 129, 2304 + 128, 4096 + 4]
    base = wl.c5(n_tenants=3, n_requests=sum(counts), dims=(2048, 320, 2048, 200), seed=31)
    ids = np.random.default_rng(31).permutation(np.repeat(np.arange(3), counts)).astype(np.int32)
    w = wl.Workload("long-k", base.dtype, base.tenants, ids, base.inputs)
    ctx = make_context(w)
    gpu = gpu_run(ctx, w, poison=True)
    got = ctx.last_counts()
    assert [int(got[t]) for t in range(3)] == counts
    rows = sample_rows(w, got, n_random=400)
    worst = compare(w, tuple(a[rows] for a in gpu), oracle_rows(w, rows), rows=rows, what="long-k")
    print("long-k: %d rows checked, worst rel fro %.2e, flip-free rows %.3f" % (len(rows), worst, compare.last_clean_frac), flush=True)
    lg, pr, lb, nc = gpu
    assert np.all(np.isfinite(lg)) and np.array_equal(lb, np.argmax(lg, axis=1))
    ctx.close()


@pytest.mark.parametrize("walk", ["1", "0"])
def test_fp32_big_tiles_long_reductions(big_tiles_always, monkeypatch, walk):
    # both ways of handing out big tiles: walked by one workgroup per CU, and a workgroup per tile
    monkeypatch.setenv("MT_BIG_WALK", walk)
    w = wl.c1(n_tenants=2, n_requests=4400, dims=(2048, 256, 10))
    assert min(w.counts().values()) >= 2048
    run_and_compare(w, "fp32-long-k")


def test_fp32_cnn_and_gelu():
    w = wl.c4(n_tenants=2, n_requests=6, hw=8, chans=(3, 8, 16, 16), classes=4)
    w.dtype = "f32"
    run_and_compare(w, "cnn-fp32")


def test_cnn_wide_layers_three_channel_blocks():
    # 72 and 96 output channels: convolution tiles of 3 channel blocks (the 4-wide kernel with an
    # idle wave), ragged pixel tiles, stride 1 and 2
    run_and_compare(wl.c4(n_tenants=2, n_requests=9, hw=12, chans=(3, 72, 96, 40), strides=(1, 2, 1), classes=7), "cnn-wide")


def test_cnn_fp32_wide_layers():
    w = wl.c4(n_tenants=2, n_requests=5, hw=8, chans=(3, 64, 128, 16), strides=(2, 1, 2), classes=4)
    w.dtype = "f32"
    run_and_compare(w, "cnn-fp32-wide")


def test_cnn_tenants_of_different_widths_share_a_launch():
    # same layer indices, different channel counts: the launch is sized for the widest tenant and
    # the narrow tenant's tiles leave waves idle
    a = wl.c4(n_tenants=2, n_requests=10, hw=8, chans=(3, 16, 32, 24), classes=6, seed=21)
    b = wl.c4(n_tenants=2, n_requests=10, hw=8, chans=(3, 64, 128, 64), classes=6, seed=22)
    tenants = {0: a.tenants[0], 1: b.tenants[0], 2: b.tenants[1]}
    ids = np.random.default_rng(9).integers(0, 3, 10).astype(np.int32)
    run_and_compare(wl.Workload("cnn-mixed", "bf16", tenants, ids, a.inputs), "cnn-mixed-widths")


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_convolutions_with_the_input_resident_in_lds(monkeypatch, dtype):
    """Layers whose 128-pixel tiles are whole output rows of one image (16x16 outputs: 8 rows of it) or
    whole small images (8x8 outputs: two of them) keep the tile's input rows in LDS instead of gathering
    every tap: stride 1 and 2, two and four channel blocks, a ragged last tile (5 images of 64 pixels),
    tenants with frames of different size in one launch.  The answers must match the oracle, and the
    gathering kernels' answers when that kernel is switched off."""
    cases = [wl.c4(n_tenants=2, n_requests=5, hw=8, chans=(3, 16, 64, 128), strides=(1, 1, 1), classes=6, seed=31),
             wl.c4(n_tenants=2, n_requests=3, hw=32, chans=(3, 32, 64, 40), strides=(1, 2, 1), classes=5, seed=32),
             wl.c4(n_tenants=1, n_requests=4, hw=16, chans=(3, 32, 128, 72), strides=(1, 1, 2), classes=4, seed=33),
             wl.c4(n_tenants=2, n_requests=7, hw=15, chans=(3, 32, 64, 64), strides=(2, 1, 1), classes=5, seed=36)]   # 15x15 inputs, 8x8 outputs
    a = wl.c4(n_tenants=1, n_requests=6, hw=8, chans=(3, 16, 64, 64), strides=(1, 1, 1), classes=4, seed=34)
    b = wl.c4(n_tenants=1, n_requests=6, hw=8, chans=(3, 32, 128, 64), strides=(1, 1, 1), classes=4, seed=35)
    cases.append(wl.Workload("two frames", "bf16", {0: a.tenants[0], 1: b.tenants[0]},
                             np.array([0, 1, 1, 0, 1, 0], dtype=np.int32), a.inputs))
    for w in cases:
        w.dtype = dtype
        ref = oracle_rows(w)
        got = []
        for off in ("0", "1"):
            monkeypatch.setenv("MT_NO_CONV_IMG", off)
            ctx = make_context(w)
            gpu = gpu_run(ctx, w, poison=True)
            compare(w, gpu, ref, what="%s %s conv_img %s" % (w.name, dtype, "off" if off == "1" else "on"))
            got.append(gpu)
            ctx.close()
        np.testing.assert_allclose(got[0][0], got[1][0], rtol=1e-2, atol=1e-2)     # same products, possibly another order


def test_more_than_1024_classes():
    # the head kernel holds rows of up to 1024 logits in registers; wider rows take its loop
    run_and_compare(wl.c2(n_tenants=3, n_requests=70, dims=(64, 96, 1100)), "wide-head")


def rect_cnn(h, w, chans, strides, classes):
    layers, hh, ww = [], h, w
    for i, st in enumerate(strides):
        l = wl.LayerSpec(wl.CONV, wl.ACT_RELU, chans[i], chans[i + 1], hh, ww, st)
        layers.append(l)
        hh, ww = l.out_hw()
    layers.append(wl.LayerSpec(wl.GAP, wl.ACT_NONE, chans[-1], chans[-1], hh, ww))
    layers.append(wl.LayerSpec(wl.FC, wl.ACT_NONE, chans[-1], classes))
    return layers


def cnn_workload(name, layer_lists, n_requests, dtype="bf16", seed=71):
    tenants = {t: wl.make_model(l, dtype, seed, t) for t, l in enumerate(layer_lists)}
    in_len = layer_lists[0][0].in_len()
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((n_requests, in_len)).astype(np.float32)
    if dtype == "bf16":
        import torch
        x = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    ids = rng.integers(0, len(layer_lists), n_requests).astype(np.int32)
    return wl.Workload(name, dtype, tenants, ids, x)


def test_pooling_done_by_the_last_convolution(monkeypatch):
    # 64-channel-multiple convolutions whose images have 64 (8x8) or 32 (8x4) output pixels pool by
    # themselves when every model of the fleet allows it; the separate pooling kernel must agree
    square = rect_cnn(16, 16, (3, 16, 64, 128), (1, 1, 2), 7)          # 8x8 final map, two channel groups of 64.. 128 channels
    narrow = rect_cnn(16, 8, (3, 16, 64, 64), (1, 1, 2), 7)            # 8x4 final map: one pixel block per image
    for name, lists in (("pool-8x8", [square, square]), ("pool-8x4", [narrow, narrow, narrow])):
        w = cnn_workload(name, lists, 37)
        ctx = make_context(w)
        assert ctx.stats()["last_run_launches"] == 0
        fused = gpu_run(ctx, w, poison=True)
        n_fused = ctx.stats()["last_run_launches"]
        compare(w, fused, oracle_rows(w), what=name)
        ctx.close()
        monkeypatch.setenv("MT_NO_FUSED_POOL", "1")
        ctx = make_context(w)
        apart = gpu_run(ctx, w, poison=True)
        assert ctx.stats()["last_run_launches"] == n_fused + 1          # the pooling launch
        monkeypatch.delenv("MT_NO_FUSED_POOL")
        compare(w, apart, oracle_rows(w), what=name + " (separate pooling)")
        assert np.array_equal(fused[2], apart[2]) and np.allclose(fused[0], apart[0], rtol=0, atol=2e-2)
        ctx.close()
    # a fleet in which one model cannot (40 channels): nobody does, and the answers still match
    odd = rect_cnn(16, 16, (3, 16, 24, 40), (1, 1, 2), 7)
    w = cnn_workload("pool-mixed", [square, odd], 29)
    run_and_compare(w, "pool-mixed")


# ---- full-size configurations ---------------------------------------------------------------
def test_c2_full():
    run_and_compare(wl.c2(), "c2", min_clean_frac=0.9)


def test_c2_full_three_runs_in_flight():
    # the configuration the benchmark times: three runs in flight, each on a stream of its own
    import torch
    import paper_1901_06887_amd as mt
    from paper_1901_06887_amd import torch_io
    w = wl.c2()
    ctx = mt.context_for(w.tenants, w.dtype, w.n_requests, run_slots=3)
    mt.register_tenants(ctx, w.tenants)
    d_ids, d_x = torch.from_numpy(w.tenant_ids).cuda(), torch_io.to_device(w.inputs, w.dtype)
    streams = [torch.cuda.Stream() for _ in range(3)]
    ctx.debug_poison()
    torch.cuda.synchronize()
    outs = [mt.serve(ctx, d_ids, d_x, stream=streams[i % 3]) for i in range(6)]
    torch.cuda.synchronize()
    orc = oracle_rows(w)
    for i, o in enumerate(outs):
        gpu = (o.logits.cpu().numpy().astype(np.float64), o.probs.cpu().numpy().astype(np.float64),
               o.labels.cpu().numpy(), o.n_classes.cpu().numpy())
        compare(w, gpu, orc, what="c2, run %d of 6 in flight" % i)
    ctx.close()


def test_c3_full_all_rows():
    w = wl.c3()
    ctx = make_context(w)
    gpu = gpu_run(ctx, w, poison=True)
    counts = ctx.last_counts()
    assert np.array_equal(counts, np.bincount(w.tenant_ids, minlength=len(counts)))
    # most of this mix's tenants have fewer than 16 rows: the pooled small-tenant checks of compare() carry it
    assert int(np.sum((counts > 0) & (counts < 16))) >= 100
    worst = compare(w, gpu, oracle_rows(w), what="c3", min_clean_frac=0.85)
    print("c3: all %d rows checked, worst per-tensor rel fro %.2e, flip-free rows %.3f" % (w.n_requests, worst, compare.last_clean_frac), flush=True)
    ctx.close()


def test_c4_full_all_rows():
    w = wl.c4()
    ctx = make_context(w)
    gpu = gpu_run(ctx, w, poison=True)
    worst = compare(w, gpu, oracle_rows(w), what="c4", min_clean_frac=0.85)
    print("c4: all %d rows checked, worst per-tensor rel fro %.2e, flip-free rows %.3f" % (w.n_requests, worst, compare.last_clean_frac), flush=True)
    ctx.close()


def test_c5_full_quarter_of_the_rows_and_every_tile_edge():
    w = wl.c5()
    ctx = make_context(w)
    gpu = gpu_run(ctx, w, poison=True)
    counts = ctx.last_counts()
    assert np.array_equal(counts, np.bincount(w.tenant_ids, minlength=len(counts)))
    # every tenant's segment edges and the rows around every 32-row boundary (all tile edges of the
    # 256-row tiles and of the streaming tiles that serve the remainders), plus a random quarter of the
    # batch: ~10 thousand rows of ~54 M fp64 multiply-accumulates each
    rows = sample_rows(w, counts, n_random=w.n_requests // 4)
    assert len(rows) >= w.n_requests // 4
    worst = compare(w, tuple(a[rows] for a in gpu), oracle_rows(w, rows), rows=rows, what="c5")
    print("c5: %d rows checked, worst rel fro %.2e, flip-free rows %.3f" % (len(rows), worst, compare.last_clean_frac), flush=True)
    # properties that hold at any size, on all rows
    lg, pr, lb, nc = gpu
    assert np.all(nc == 1000) and np.all(np.isfinite(lg))
    assert np.allclose(pr.sum(axis=1), 1.0, atol=1e-5)
    assert np.array_equal(lb, np.argmax(lg, axis=1))
    ctx.close()
