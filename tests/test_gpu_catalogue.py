"""GPU parity of the wider layer catalogue (paper section 1.1: DNNs are built from a few dozen layer
types, the running example is an 18-layer residual network; section 3.1: a pre-defined set of supported
layers): 1x1 / 3x3 / 7x7 convolutions, max-pooling, residual additions with skip sources, batch
normalisation folded at registration, and resnet18-shaped tenants, against the fp64 oracle through the C ABI."""
import numpy as np
import pytest

import workloads as wl
from gpu_common import compare, gpu_run, make_context, oracle_rows

pytestmark = pytest.mark.gpu


def conv(ci, co, hw, k, s=1, act=wl.ACT_RELU, src=0):
    h, w = hw if isinstance(hw, tuple) else (hw, hw)
    return wl.LayerSpec(wl.CONV, act, ci, co, h, w, s, ksize=k, pad=(k - 1) // 2, src=src)


def pool(ch, hw, k=3, s=2, p=1):
    h, w = hw if isinstance(hw, tuple) else (hw, hw)
    return wl.LayerSpec(wl.MAXPOOL, wl.ACT_NONE, ch, ch, h, w, s, ksize=k, pad=p)


def add(ch, hw, src2, src=0, act=wl.ACT_RELU):
    h, w = hw if isinstance(hw, tuple) else (hw, hw)
    return wl.LayerSpec(wl.ADD, act, ch, ch, h, w, src=src, src2=src2)


def tail(ch, hw, classes):
    h, w = hw if isinstance(hw, tuple) else (hw, hw)
    return [wl.LayerSpec(wl.GAP, wl.ACT_NONE, ch, ch, h, w), wl.LayerSpec(wl.FC, wl.ACT_NONE, ch, classes)]


def fleet(name, layer_lists, n_requests, dtype="bf16", seed=201, bn=False):
    tenants = {}
    for t, layers in enumerate(layer_lists):
        m = wl.make_model(layers, dtype, seed, t)
        tenants[t] = wl.with_batchnorm(m, seed, t) if bn else m
    in_len = layer_lists[0][0].in_len()
    assert all(l[0].in_len() == in_len for l in layer_lists)
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((n_requests, in_len)).astype(np.float32)
    if dtype == "bf16":
        x = wl.round_to_bf16(x)
    ids = rng.integers(0, len(layer_lists), n_requests).astype(np.int32)
    return wl.Workload(name, dtype, tenants, ids, x)


def run_and_compare(w, what, deep=False, tight=None):
    ctx = make_context(w)
    gpu = gpu_run(ctx, w, poison=True)
    counts = ctx.last_counts()
    assert np.array_equal(counts, np.bincount(w.tenant_ids, minlength=len(counts))), what
    ref = oracle_rows(w)
    worst = compare(w, gpu, ref, what=what, deep=deep)
    if tight is not None:                  # fp32 models: every row to rounding noise
        C = ref[0].shape[1]
        row_err = np.linalg.norm(gpu[0][:, :C] - ref[0], axis=1) / np.linalg.norm(ref[0], axis=1)
        assert row_err.max() <= tight, "%s: a row is off by %.3e" % (what, row_err.max())
    print("%s: worst per-tensor rel fro %.2e, flip-free rows %.3f" % (what, worst, compare.last_clean_frac), flush=True)
    ctx.close()
    return gpu


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_convolution_windows_1x1_3x3_7x7(dtype):
    """Every window of the set at stride 1 and 2, odd and even images, narrow (one channel block), wide
    (two to four) and ragged (72, 136) channel counts, tenants of different shapes in one launch."""
    nets = [
        [conv(3, 16, 12, 7, 2), conv(16, 24, 6, 1), conv(24, 40, 6, 3, 2)] + tail(40, 3, 5),              # 7x7 stem, 1x1, 3x3
        [conv(3, 64, 12, 7, 1), conv(64, 128, 12, 1, 2), conv(128, 72, 6, 7, 1)] + tail(72, 6, 5),        # wide 1x1 and 7x7 (quad gathers)
        [conv(3, 8, 12, 1, 1), conv(8, 136, 12, 3, 2), conv(136, 32, 6, 1, 1)] + tail(32, 6, 5),          # 1x1 on the padded 3-channel input, 8 channels wide
        [conv(3, 32, 12, 3, 1), conv(32, 32, 12, 7, 2), conv(32, 64, 6, 1, 2)] + tail(64, 3, 5),
    ]
    run_and_compare(fleet("windows", nets, 23, dtype), "conv windows %s" % dtype)
    odd = [[conv(3, 16, (9, 11), 7, 2), conv(16, 16, (5, 6), 1, 2), conv(16, 48, (3, 3), 3, 1)] + tail(48, 3, 4),
           [conv(3, 40, (9, 11), 1, 2), conv(40, 16, (5, 6), 7, 1), conv(16, 16, (5, 6), 3, 2)] + tail(16, 3, 4)]
    run_and_compare(fleet("odd images", odd, 17, dtype, seed=202), "conv windows, odd images %s" % dtype)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_max_pooling(dtype):
    nets = [
        [conv(3, 16, 12, 3, 1), pool(16, 12, 3, 2, 1), conv(16, 32, 6, 3, 1), pool(32, 6, 2, 2, 0)] + tail(32, 3, 6),
        [conv(3, 8, 12, 3, 1, act=wl.ACT_NONE), pool(8, 12, 3, 1, 1), pool(8, 12, 2, 2, 0), pool(8, 6, 3, 2, 0)] + tail(8, 2, 6),   # negative values, pad 0 and 1
        [conv(3, 72, 12, 7, 2, act=wl.ACT_NONE), pool(72, 6, 2, 1, 1), conv(72, 16, 7, 1, 1)] + tail(16, 7, 6),                     # 2x2 window with padding: 7x7 out
    ]
    run_and_compare(fleet("max-pool", nets, 19, dtype, seed=203), "max-pool %s" % dtype)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_residual_blocks_with_identity_and_projection_skips(dtype):
    c = 16
    identity = [conv(3, c, 8, 3), conv(c, c, 8, 3), conv(c, c, 8, 3, act=wl.ACT_NONE), add(c, 8, src2=1)] + tail(c, 8, 4)
    projected = [conv(3, c, 8, 3), conv(c, 2 * c, 8, 3, 2), conv(2 * c, 2 * c, 4, 3, act=wl.ACT_NONE),
                 conv(c, 2 * c, 8, 1, 2, act=wl.ACT_NONE, src=1), add(2 * c, 4, src=3, src2=4)] + tail(2 * c, 4, 4)
    two_blocks = [conv(3, c, 8, 7, 1), pool(c, 8, 3, 2, 1),
                  conv(c, c, 4, 3), conv(c, c, 4, 3, act=wl.ACT_NONE), add(c, 4, src2=2),
                  conv(c, c, 4, 3), conv(c, c, 4, 3, act=wl.ACT_NONE), add(c, 4, src2=5, act=wl.ACT_GELU)] + tail(c, 4, 4)
    plain = [conv(3, c, 8, 3), conv(c, c, 8, 3, 2), conv(c, 64, 4, 3, 2)] + tail(64, 2, 4)           # a chain next to them: pools by itself or not, as the fleet allows
    mlp = wl.mlp_layers([8 * 8 * 3, 96, 64, 4], wl.ACT_RELU)                                            # and an MLP on the same rows
    run_and_compare(fleet("residual", [identity, projected, two_blocks, plain, mlp], 41, dtype, seed=204), "residual blocks %s" % dtype)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_large_images_share_a_row_among_workgroups(dtype):
    """Images of more than 2048 pixels: several workgroups share one packed row in the image gather (three-channel
    rows with an even and with an odd pixel count, and eight-channel rows, which take the generic path), in the
    max-pool (window over a 53 x 61 image: the slices end inside an image row) and in the residual addition."""
    c = 16
    three = [conv(3, c, (53, 61), 3, 1), pool(c, (53, 61), 3, 2, 1), conv(c, c, (27, 31), 3, act=wl.ACT_NONE), add(c, (27, 31), src2=2)] + tail(c, (27, 31), 5)
    wide = [conv(3, 8, (53, 61), 1, 1, act=wl.ACT_NONE), pool(8, (53, 61), 2, 1, 0), conv(8, 24, (52, 60), 3, 2),
            conv(24, 24, (26, 30), 3, act=wl.ACT_NONE), add(24, (26, 30), src2=3, act=wl.ACT_NONE)] + tail(24, (26, 30), 5)
    run_and_compare(fleet("large three-channel images", [three, wide], 7, dtype, seed=206), "large images, 3 channels, %s" % dtype)
    eight = [conv(8, c, (48, 50), 3, 2), pool(c, (24, 25), 3, 1, 1), conv(c, c, (24, 25), 3, act=wl.ACT_NONE), add(c, (24, 25), src2=2)] + tail(c, (24, 25), 5)
    run_and_compare(fleet("large eight-channel images", [eight, eight], 5, dtype, seed=207), "large images, 8 channels, %s" % dtype)
    even = [conv(3, c, (54, 60), 3, 2), conv(c, c, (27, 30), 3)] + tail(c, (27, 30), 5)
    run_and_compare(fleet("large three-channel images, pixel pairs", [even], 4, dtype, seed=208), "large images, even pixel count, %s" % dtype)


def test_additions_done_by_the_convolution_in_front_of_them(monkeypatch):
    """A convolution whose output feeds only the residual addition behind it adds the other operand itself
    (either operand order, identity and projected skips, an activation on the convolution as well, ragged
    channel counts); an addition whose first operand has another reader, or follows a pooling layer, stays a
    launch of its own.  With the takeover switched off the outputs are the same to the bit, and the run
    has more launches."""
    c = 24
    swapped = [conv(3, c, 8, 3), conv(c, c, 8, 3), conv(c, c, 8, 3, act=wl.ACT_GELU), add(c, 8, src=1, src2=3, act=wl.ACT_NONE)] + tail(c, 8, 4)       # the convolution's output as second operand, activations on both
    projected = [conv(3, 16, 8, 3), conv(16, 72, 8, 3, 2), conv(72, 72, 4, 3, act=wl.ACT_NONE),
                 conv(16, 72, 8, 1, 2, act=wl.ACT_NONE, src=1), add(72, 4, src=3, src2=4)] + tail(72, 4, 4)               # the 1x1 projection takes the sum; 72 channels: a ragged block
    shared = [conv(3, c, 8, 3), conv(c, c, 8, 3, act=wl.ACT_NONE), add(c, 8, src2=1), add(c, 8, src=2, src2=3)] + tail(c, 8, 4)      # the convolution's output is read twice: not taken over
    pooled = [conv(3, c, 8, 3), conv(c, c, 8, 3), pool(c, 8, 3, 1, 1), add(c, 8, src2=1)] + tail(c, 8, 4)                   # behind a pooling layer
    for dtype in ("bf16", "f32"):
        w = fleet("additions", [swapped, projected, shared, pooled], 37, dtype, seed=209)
        counts = np.bincount(w.tenant_ids, minlength=4).astype(np.uint32)
        monkeypatch.delenv("MT_NO_FUSED_ADD", raising=False)
        ctx = make_context(w)
        fused_launches = ctx.estimate_run(counts)["launches"]
        ctx.close()
        fused = run_and_compare(w, "additions taken over, %s" % dtype)
        monkeypatch.setenv("MT_NO_FUSED_ADD", "1")
        ctx = make_context(w)
        plain_launches = ctx.estimate_run(counts)["launches"]
        plain = gpu_run(ctx, w, poison=True)
        ctx.close()
        monkeypatch.delenv("MT_NO_FUSED_ADD")
        assert np.array_equal(fused[0], plain[0]) and np.array_equal(fused[2], plain[2]), dtype
        assert fused_launches < plain_launches, (fused_launches, plain_launches)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_tiles_of_whole_output_rows(dtype):
    """3x3 layers at stride 1 whose tiles are whole output rows with the input rows in LDS, on shapes that fill a
    tile badly: 14-pixel rows (9 rows per tile, an image's second tile has 5), 10x6 images (two per tile, an odd
    number of requests per tenant), 20-pixel rows of 10 (6 + 4), a residual addition taken over by such a layer;
    and layer indices at which one tenant's layer is row-tiled and another's is not (a 1x1 window, stride 2), so
    that the launch falls back to the gathering kernels, whose lists count the row-tiled tenant's tiles generously."""
    nets = [
        [conv(3, 16, 14, 3), conv(16, 32, 14, 3), conv(32, 32, 14, 3), conv(32, 64, 14, 3, 2)] + tail(64, 7, 6),
        [conv(3, 32, 14, 3), conv(32, 32, 14, 3, act=wl.ACT_NONE), conv(32, 32, 14, 1), conv(32, 48, 14, 3)] + tail(48, 14, 6),
        [conv(3, 16, 14, 3), conv(16, 16, 14, 3, act=wl.ACT_NONE), add(16, 14, src2=1), conv(16, 32, 14, 3)] + tail(32, 14, 6),
    ]
    run_and_compare(fleet("row tiles, 14x14", nets, 23, dtype, seed=231), "row tiles 14x14", tight=2e-5 if dtype == "f32" else None)
    small = [
        [conv(3, 16, (10, 6), 3), conv(16, 32, (10, 6), 3), conv(32, 32, (10, 6), 3)] + tail(32, (10, 6), 5),
        [conv(3, 32, (10, 6), 3), conv(32, 64, (10, 6), 3), conv(64, 16, (10, 6), 3)] + tail(16, (10, 6), 5),
    ]
    run_and_compare(fleet("row tiles, two images per tile", small, 31, dtype, seed=232), "row tiles 10x6", tight=2e-5 if dtype == "f32" else None)
    wide = [[conv(3, 16, (10, 20), 3), conv(16, 128, (10, 20), 3), conv(128, 32, (10, 20), 3)] + tail(32, (10, 20), 5)] * 2
    run_and_compare(fleet("row tiles, 20-pixel rows", wide, 9, dtype, seed=233), "row tiles 10x20", tight=2e-5 if dtype == "f32" else None)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_long_reductions_in_launches_of_few_tiles(dtype):
    """Deep layers of small batches: at most one tile per CU and K >= 1024, the shape that gets loader waves, here
    with the pooling done by the convolution (8x8 and 4x8 images of 128 and 192 channels in front of the global
    average), with a residual addition taken over by it, and with tenants of unequal widths in one launch."""
    pooled = [conv(3, 32, 16, 3), conv(32, 128, 16, 3, 2), conv(128, 128, 8, 3)] + tail(128, 8, 7)
    wide = [conv(3, 32, 16, 3), conv(32, 128, 16, 3, 2), conv(128, 192, 8, 3)] + tail(192, 8, 7)
    rect = [conv(3, 32, (8, 16), 3), conv(32, 128, (8, 16), 3, 2), conv(128, 128, (4, 8), 3)] + tail(128, (4, 8), 7)
    run_and_compare(fleet("long K, pooled", [pooled, wide], 21, dtype, seed=210), "long K, few tiles, pooled, %s" % dtype)
    run_and_compare(fleet("long K, pooled, 4x8", [rect, rect], 9, dtype, seed=212), "long K, few tiles, pooled 4x8 images, %s" % dtype)
    block = [conv(3, 32, 16, 3), conv(32, 128, 16, 3, 2), conv(128, 128, 8, 3), conv(128, 128, 8, 3, act=wl.ACT_NONE), add(128, 8, src2=2),
             conv(128, 256, 8, 3, 2), conv(256, 256, 4, 3, act=wl.ACT_NONE), conv(128, 256, 8, 1, 2, act=wl.ACT_NONE, src=5), add(256, 4, src=7, src2=8)] + tail(256, 4, 7)
    run_and_compare(fleet("long K, residual", [block, block], 5, dtype, seed=211), "long K, few tiles, residual, %s" % dtype, deep=(dtype == "bf16"))


def test_folded_batch_normalisation():
    nets = [[conv(3, 16, 8, 3), conv(16, 32, 8, 1, 2), conv(32, 32, 4, 3, act=wl.ACT_NONE), conv(16, 32, 8, 1, 2, act=wl.ACT_NONE, src=1),
             add(32, 4, src=3, src2=4)] + tail(32, 4, 6)] * 3
    for dtype in ("bf16", "f32"):
        w = fleet("bn", nets, 29, dtype, seed=205, bn=True)
        got = run_and_compare(w, "folded batch-norm %s" % dtype)
        # the normalisation matters: the same filters without it give other answers
        for m in w.tenants.values():
            m.bn = None
        ctx = make_context(w)
        plain = gpu_run(ctx, w)
        ctx.close()
        assert np.abs(plain[0] - got[0]).max() > 1e-2


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_resnet18_shaped_tenants(dtype):
    """The 18-layer residual network's layer graph (31 layer indices, three live activations, batch
    normalisation behind every convolution) at reduced widths on 32x32 images, three tenants; then at full
    widths (64..512 channels, 1000 classes) on 64x64 images, next to a plain CNN tenant and an MLP tenant in
    the same run.  In fp32 every row must agree to rounding noise; in bf16 the deep-net bar applies."""
    deep, tight = (True, None) if dtype == "bf16" else (False, 5e-6)
    run_and_compare(wl.resnet(n_tenants=3, n_requests=200, hw=32, widths=(16, 32, 64, 128), classes=10, dtype=dtype), "resnet18-shaped, reduced, " + dtype,
                    deep=deep, tight=tight)
    full = wl.resnet(n_tenants=2, n_requests=9, hw=64, widths=(64, 128, 256, 512), classes=1000, dtype=dtype, seed=7)
    cnn = wl.make_model(wl.cnn_layers(64, (3, 32, 64, 128), (2, 2, 2), 10), dtype, 7, 50)
    mlp = wl.make_model(wl.mlp_layers([64 * 64 * 3, 256, 100], wl.ACT_GELU), dtype, 7, 51)
    tenants = dict(full.tenants); tenants[2] = cnn; tenants[3] = mlp
    ids = np.array([0, 2, 1, 3, 0, 1, 2, 3, 0, 1, 1, 2], dtype=np.int32)
    x = np.random.default_rng(8).standard_normal((12, 64 * 64 * 3)).astype(np.float32)
    if dtype == "bf16":
        x = wl.round_to_bf16(x)
    run_and_compare(wl.Workload("resnet18-shaped + cnn + mlp", dtype, tenants, ids, x), "resnet18-shaped, full widths, mixed fleet, " + dtype,
                    deep=deep, tight=tight)


def test_models_deeper_than_one_group_of_layer_indices():
    """The segmentation kernel builds the tile lists eight layer indices at a time: MLPs of 11 and 20
    layers next to a two-layer one, several row tiles each."""
    dims = lambda n: [96] + [64 + 32 * (i % 3) for i in range(n - 1)] + [7]
    nets = [wl.mlp_layers(dims(11), wl.ACT_RELU), wl.mlp_layers(dims(20), wl.ACT_GELU), wl.mlp_layers([96, 128, 7], wl.ACT_RELU)]
    run_and_compare(fleet("deep mlps", nets, 700, "bf16", seed=206), "deep MLPs")
    run_and_compare(fleet("deep mlps", nets, 90, "f32", seed=207), "deep MLPs, small run")


def test_r18_as_the_benchmark_runs_it():
    """Four resnet18-shaped tenants on 224x224 images, 64 requests: the configuration bench.py times."""
    run_and_compare(wl.r18(), "r18", deep=True)
