#!/usr/bin/env python3
"""Throughput of the multi-tenant hot path on one MI355X.

One step = one pass of the whole path over one synthetic batch: mt_submit_batch + mt_run
(tenant segmentation, gather, every grouped layer launch, softmax/argmax head), inputs and
models already resident in device memory.  Prints one JSON line.

With no --config the headline is the largest mix (c5: 8 tenants x 4096 requests, compute
bound) and `per_config` carries the same measurements for c1..c4 and for r18 (four tenants with
resnet18-shaped models, the wider layer catalogue); with --config X only that mix is measured
(the form the rocprofv3 summaries under profiles/ are made with).

  value        inferences/sec over the K timed steps, one run at a time: the K steps are
               enqueued on one stream, each run after the other, and timed by the wall clock
               between two device synchronisations; ms_per_step is that time / K
  device_ms    per-step device time between two events around the run over at least 100
               steps (median, mean, p99/mean, inferences/sec at the median), and the same
               with the caches flushed before every step (`cold`): a batch whose weights fit
               the last-level cache is otherwise partly served from it on repeated runs
  roofline     the dominant grouped kernel against HBM bandwidth (weight-streaming mixes) or
               the bf16 MFMA peak (c5): algorithmic bytes or flops per launch / its average
               launch duration, measured with HIP events on the run's stream in a separate
               pass over the same K steps (event brackets cost microseconds per kernel, so
               they stay out of the timed steps).  `traffic` is the HBM bytes per launch of
               that kernel from stored hardware-counter runs (`traffic_source` names the
               file under profiles/), null when there is none for this mix or the device
               code has changed since they were taken.  For the MFMA-bound mix
               `sustained_mfma_tflops` is what a loop of nothing but MFMAs on random bf16
               operands reaches on this very GPU in the same process (the chip lowers its
               clock under MFMA load, so the published peak is not attainable).
  interleaved  the same K steps with three runs in flight on three streams (batch
               interleaving); a secondary figure, never the headline
  cpu_baseline the fp64 oracle timed on the host cores on a bounded sample of the same batch
"""
import argparse
import hashlib
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0
FP32_MATRIX_PEAK_TFLOPS = 157.3

KERNEL_SOURCES = ("csrc/mt_device.h", "csrc/batcher.hip", "csrc/fc_stream.hip", "csrc/fc_big.hip", "csrc/conv.hip",
                  "csrc/small.hip", "csrc/mt_internal.h")


def kernel_source_sha256() -> str:
    """Fingerprint of the device code: counters taken before a change to it no longer apply.
    Comments and white space are left out, so that editing a comment does not void a measurement."""
    h = hashlib.sha256()
    for rel in KERNEL_SOURCES:
        with open(os.path.join(ROOT, "paper_1901_06887_amd", rel), "r") as f:
            text = f.read()
        text = re.sub(r"/\*.*?\*/", " ", text, flags=re.S)     # block comments
        text = re.sub(r"//[^\n]*", " ", text)                  # line comments (the sources hold no string with //)
        h.update(" ".join(text.split()).encode())
    return h.hexdigest()


def read_stored_traffic(path: str):
    """`traffic_bytes_per_launch` of a stored counter summary, or None when there is none or the
    device code has changed since it was taken."""
    try:
        text = open(path).read()
    except OSError:
        return None
    sha = re.search(r"^kernel_source_sha256: ([0-9a-f]{64})$", text, re.M)
    val = re.search(r"^traffic_bytes_per_launch: (\d+)$", text, re.M)
    if not sha or not val or sha.group(1) != kernel_source_sha256():
        return None
    return float(val.group(1))


def gemm_launch_costs(w, es, rows_of=None, pooled_by_conv=False):
    """Algorithmic flops and bytes of the grouped GEMM launch of every layer index: each active
    tenant's weights and bias read once, its input rows read once, its output rows written once
    (hidden: element type; logits: fp32).  `rows_of(rows, layer)`: the rows of a tenant-layer
    that the kernel in question serves (default: all of them)."""
    import workloads as wl
    flops, bytes_ = {}, {}
    for t, rows_t in w.counts().items():
        model = w.tenants[t]
        n = len(model.layers)
        for l, L in enumerate(model.layers):
            if L.kind not in (wl.FC, wl.CONV):
                continue
            m_t = rows_t if rows_of is None else rows_of(rows_t, L)
            if m_t == 0:
                continue
            if L.kind == wl.FC:
                f = 2 * m_t * L.in_features * L.out_features
            else:
                oh, ow = L.out_hw()
                f = 2 * m_t * oh * ow * L.ksize * L.ksize * L.in_features * L.out_features
            b = model.weights[l].size * es + model.biases[l].size * 4
            b += m_t * L.in_len() * es
            if pooled_by_conv and l + 1 < n and model.layers[l + 1].kind == wl.GAP:
                b += m_t * L.out_features * es          # the launch writes the pooled activation, not the image
            else:
                b += m_t * L.out_len() * (4 if l == n - 1 else es)
            flops[l] = flops.get(l, 0) + f
            bytes_[l] = bytes_.get(l, 0) + b
    return flops, bytes_


def cpu_baseline(w, seconds):
    """The oracle as it stands on the host cores, on an arrival-ordered prefix of the batch
    worth about `seconds` of its time (arrival order is an i.i.d. draw of the tenant mix, so a
    prefix is a seeded random sample of it and its rate stands for the whole batch)."""
    import numpy as np
    import oracle
    threads = min(16, os.cpu_count() or 1)
    models = oracle.models_from_workload(w)
    R = w.n_requests
    macs_per_row = np.array([models[int(t)].macs_per_request() for t in w.tenant_ids], dtype=np.float64)
    budget = seconds * 1.5e9 * threads                    # ~1.5 GMAC/s per thread
    n_sample = int(min(R, max(threads, np.searchsorted(np.cumsum(macs_per_row), budget))))
    x64 = w.inputs[:n_sample].astype(np.float64)
    reps, t0 = 0, time.perf_counter()
    while True:                       # a batch the oracle finishes in under a second is repeated for a stable figure
        oracle.run_batch(models, w.tenant_ids[:n_sample], x64, threads=threads)
        reps += 1
        cdt = time.perf_counter() - t0
        if cdt >= 0.6 * seconds or reps >= 200:
            break
    per_tenant = np.bincount(w.tenant_ids[:n_sample], minlength=len(w.tenants))
    return {"value": n_sample * reps / cdt, "unit": "inferences/sec", "cores": threads, "kind": "oracle",
            "sample": "first %d of %d requests of %s in arrival order (%d..%d per tenant with traffic), %d pass(es), "
                      "fp64 loop nests, %.1f s; the rate of the sample stands for the batch" % (
                          n_sample, R, w.name, int(per_tenant[per_tenant > 0].min()), int(per_tenant.max()), reps, cdt)}


def measure(name, steps, warmup, interleave, cpu_seconds, calibrate_copy_mib=0):
    """Everything bench.py reports for one mix."""
    import numpy as np
    import torch

    import paper_1901_06887_amd as mt
    import workloads as wl
    from paper_1901_06887_amd import torch_io

    t_setup = time.perf_counter()
    w = wl.CONFIGS[name]()
    es = 4 if w.dtype == "f32" else 2
    R = w.n_requests
    ctx = mt.context_for(w.tenants, w.dtype, R, run_slots=max(1, min(interleave, 4)))
    mt.register_tenants(ctx, w.tenants)
    d_ids = torch.from_numpy(w.tenant_ids).cuda()
    d_x = torch_io.to_device(w.inputs, w.dtype)
    out = torch_io.alloc_outputs(R, ctx.cfg.max_classes)
    stream = torch.cuda.current_stream()
    setup_s = time.perf_counter() - t_setup

    def step():
        mt.serve(ctx, d_ids, d_x, out=out, stream=stream)

    if calibrate_copy_mib:
        nb = calibrate_copy_mib << 20
        a_buf, b_buf = torch.zeros(nb, dtype=torch.uint8, device="cuda"), torch.empty(nb, dtype=torch.uint8, device="cuda")
        for _ in range(4):
            mt.debug_copy(b_buf.data_ptr(), a_buf.data_ptr(), nb, stream.cuda_stream)
        torch.cuda.synchronize()
        del a_buf, b_buf

    # ---- the timed steps: one run at a time on one stream ----
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    host_dt = time.perf_counter() - t0          # the host's share: mt_submit_batch + mt_run through the binding, K times
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / steps * 1e3
    value = R * steps / dt

    # ---- per-step device time (two events around each step), warm and with caches flushed between steps ----
    def device_times(n, flush=None):
        for _ in range(3):                      # the first bracketed steps after another pass are not part of the statistic
            if flush is not None:
                flush.add_(1)
            step()
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n)]
        for e0, e1 in ev:
            if flush is not None:
                flush.add_(1)
            e0.record(stream)
            step()
            e1.record(stream)
        torch.cuda.synchronize()
        return np.array([e0.elapsed_time(e1) for e0, e1 in ev])
    warm = device_times(max(100, steps))
    n_cold = 30
    flush = torch.zeros(1 << 30, dtype=torch.uint8, device="cuda")       # 4x the last-level cache
    cold = device_times(n_cold, flush)
    del flush
    device_ms = {"steps": int(warm.size), "median": float(np.median(warm)), "mean": float(warm.mean()),
                 "p99_over_mean": float(np.percentile(warm, 99) / warm.mean()), "max_over_mean": float(warm.max() / warm.mean()),
                 "inferences_per_sec_at_median": float(R / (np.median(warm) * 1e-3)),
                 "cold_median": float(np.median(cold)), "cold_steps": n_cold,
                 "cold_inferences_per_sec": float(R / (np.median(cold) * 1e-3))}

    # ---- the same steps with several runs in flight (batch interleaving): a secondary figure ----
    interleaved = None
    if interleave > 1:
        n_il = min(interleave, 4)
        streams = [torch.cuda.Stream() for _ in range(n_il)]
        outs = [torch_io.alloc_outputs(R, ctx.cfg.max_classes) for _ in range(n_il)]
        torch.cuda.synchronize()
        for i in range(max(warmup, n_il)):
            mt.serve(ctx, d_ids, d_x, out=outs[i % n_il], stream=streams[i % n_il])
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            mt.serve(ctx, d_ids, d_x, out=outs[i % n_il], stream=streams[i % n_il])
        torch.cuda.synchronize()
        dt_il = time.perf_counter() - t0
        same = all(torch.equal(o.labels, out.labels) and torch.equal(o.logits, out.logits) for o in outs)
        interleaved = {"streams": n_il, "value": R * steps / dt_il, "unit": "inferences/sec",
                       "ms_per_step": dt_il / steps * 1e3, "same_answers_as_single_stream": bool(same)}
        del outs, streams
        if not same:
            raise SystemExit("runs in flight together gave other answers than runs one at a time")

    # what a pair of events reads with nothing between them: every per-kernel bracket below
    # carries that much on top of the kernel's own duration
    for _ in range(3):
        step()
    pairs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(32)]
    for e0, e1 in pairs:
        step()                                     # same queue state as in the profiled pass: work ahead of the bracket
        e0.record(stream)
        e1.record(stream)
    torch.cuda.synchronize()
    bracket_ms = float(np.median([e0.elapsed_time(e1) for e0, e1 in pairs]))

    # ---- second pass over the same steps with per-kernel HIP events on the run's stream ----
    ctx.set_profiling(True)
    prof = []
    for _ in range(steps):
        step()
        prof.append(ctx.get_profile())
    ctx.set_profiling(False)
    n_slots = mt.MT_MAX_LAYERS
    fc_ms = [float(np.mean([p["fc_ms"][l] + p["fc_big_ms"][l] for p in prof])) for l in range(n_slots)]
    big_ms = [float(np.mean([p["fc_big_ms"][l] for p in prof])) for l in range(n_slots)]
    conv_ms = [float(np.mean([p["conv_ms"][l] for p in prof])) for l in range(n_slots)]
    # a mix with pooling layers but no pooling launch: the convolutions before them pooled on the way out
    has_pool = any(L.kind == wl.GAP for m in w.tenants.values() for L in m.layers)
    pool_ms = sum(float(np.mean([p["gap_ms"][l] for p in prof])) for l in range(n_slots))
    flops, bytes_ = gemm_launch_costs(w, es, pooled_by_conv=has_pool and pool_ms == 0.0)
    # the dominant kernel: the grouped FC kernel, or the grouped conv kernel for the CNN mix
    dom_ms, dom_name = (fc_ms, "fc_kernel") if sum(fc_ms) >= sum(conv_ms) else (conv_ms, "conv_kernel")
    if dom_ms is fc_ms and sum(big_ms) > 0.5 * sum(fc_ms):
        walked = os.environ.get("MT_BIG_WALK", "1") != "0" and all(
            mt.debug_big_tile_walk(L.in_features) for m in w.tenants.values() for L in m.layers if L.kind == wl.FC)
        dom_ms, dom_name = big_ms, ("fc_big_walk_kernel" if walked else "fc_big_kernel")
        # the big-tile kernel is credited only with the rows it serves (a short remainder of a
        # tenant's rows goes to the streaming kernel)
        flops, bytes_ = gemm_launch_costs(w, es, lambda rows, L: mt.debug_big_tile_rows(rows, L.out_features) if L.kind == wl.FC else 0)
    other_ms = fc_ms if dom_ms is conv_ms else conv_ms
    launches = [l for l in range(n_slots) if dom_ms[l] > 0 and other_ms[l] == 0 and l in bytes_]
    # The bracket of a launch (two events on the run's stream) is what is reported: it reads within
    # 2-4 % of the kernel-trace duration of the same launches.  What two events with nothing between
    # them read behind a run is reported next to it; it is ~0.6 us under rocprofv3 and 3-5 us in a
    # plain run, so subtracting it would make the plain-run figure disagree with the trace.
    avg_dur_s = sum(dom_ms[l] for l in launches) / len(launches) * 1e-3
    avg_bytes = sum(bytes_[l] for l in launches) / len(launches)
    avg_flops = sum(flops[l] for l in launches) / len(launches)
    cost = wl.algorithmic_cost(w)
    intensity = avg_flops / avg_bytes
    if w.dtype == "bf16" and intensity > MFMA_BF16_PEAK_TFLOPS * 1e12 / (HBM_PEAK_GBS * 1e9):
        achieved = avg_flops / avg_dur_s / 1e12
        roofline = {"bound": "mfma", "achieved": achieved, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                    "frac": achieved / MFMA_BF16_PEAK_TFLOPS, "traffic": None}
        sustained = mt.debug_mfma_rate(stream.cuda_stream)
        roofline["sustained_mfma_tflops"] = sustained
        roofline["frac_of_sustained"] = achieved / sustained if sustained else None
    else:
        achieved = avg_bytes / avg_dur_s / 1e9
        roofline = {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": achieved / HBM_PEAK_GBS, "traffic": None}
    traffic_rel = os.path.join("profiles", "%s_%s_hbm_traffic.md" % (dom_name, w.name))
    roofline["traffic"] = read_stored_traffic(os.path.join(ROOT, traffic_rel))
    roofline["traffic_source"] = ("stored: " + traffic_rel) if roofline["traffic"] is not None else None
    # (the convolution launches of a step run conv_img_kernel, conv_lds_kernel or conv_kernel, by layer shape)
    roofline.update({"kernel": "%s<%s>" % ("conv_*kernel" if dom_name == "conv_kernel" else dom_name, "bf16" if es == 2 else "float"),
                     "launches_per_step": len(launches),
                     "avg_launch_us": avg_dur_s * 1e6, "empty_bracket_us": bracket_ms * 1e3,
                     "algorithmic_bytes_per_launch": avg_bytes, "algorithmic_flops_per_launch": avg_flops})
    kernels_us = {"batcher": float(np.mean([p["batcher_ms"] for p in prof])) * 1e3,
                  "gather": float(np.mean([p["gather_ms"] for p in prof])) * 1e3,
                  "fc_by_layer": [g * 1e3 for g in fc_ms if g > 0],
                  "fc_big_by_layer": [g * 1e3 for g in big_ms if g > 0],
                  "conv_by_layer": [g * 1e3 for g in conv_ms if g > 0],
                  "gap": float(np.sum([np.mean([p["gap_ms"][l] for p in prof]) for l in range(n_slots)])) * 1e3,
                  "image_ops_by_layer": [g * 1e3 for g in (float(np.mean([p["ops_ms"][l] for p in prof])) for l in range(n_slots)) if g > 0],
                  "head": float(np.mean([p["head_ms"] for p in prof])) * 1e3,
                  "device_total": float(np.mean([p["total_ms"] for p in prof])) * 1e3}
    ctx.close()
    del d_ids, d_x, out
    torch.cuda.empty_cache()

    cpu = cpu_baseline(w, cpu_seconds) if cpu_seconds > 0 else None

    def fracs(ms):
        return {"hbm": cost["bytes"] / (ms * 1e-3) / (HBM_PEAK_GBS * 1e9), "mfma": cost["flops"] / (ms * 1e-3) / (MFMA_BF16_PEAK_TFLOPS * 1e12)}
    whole = {"ms_per_step": fracs(ms_per_step), "device_median": fracs(device_ms["median"]), "device_cold_median": fracs(device_ms["cold_median"])}
    return {"workload": w.name, "value": value, "unit": "inferences/sec", "steps": steps, "warmup": warmup, "ms_per_step": ms_per_step,
            "dtype": "f32" if es == 4 else "bf16",
            "config": {"workload": w.name, "tenants": len(w.tenants), "requests_per_step": R, "active_tenants": len(w.counts()),
                       "runs_in_flight": 1, "algorithmic_flops_per_step": cost["flops"], "algorithmic_bytes_per_step": cost["bytes"],
                       "whole_path_frac_of_peak": whole, "setup_seconds": setup_s},
            "host_enqueue_us_per_step": host_dt / steps * 1e6,
            "roofline": roofline, "device_ms": device_ms, "kernels_us": kernels_us, "interleaved": interleaved, "cpu_baseline": cpu}


# steps / warm-up / oracle seconds of the mixes reported next to the headline
SIDE = {"c1": (200, 20, 3.0), "c2": (200, 20, 4.0), "c3": (100, 10, 5.0), "c4": (100, 10, 4.0), "r18": (50, 5, 3.0)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", default=None, choices=["c1", "c2", "c3", "c4", "c5", "r18"],
                    help="measure this mix only (default: c5 as the headline, c1..c4 and r18 in per_config)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--interleave", type=int, default=3,
                    help="runs in flight in the secondary interleaved pass, each on a stream of its own (1: pass left out)")
    ap.add_argument("--cpu-seconds", type=float, default=10.0, help="target oracle time of the headline's CPU baseline sample")
    ap.add_argument("--calibrate-copy-mib", type=int, default=0,
                    help="first run the library's plain copy kernel over this many MiB (byte-counter yardstick)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this program runs on one GPU only (no sharding, no collectives); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch

    import paper_1901_06887_amd as mt

    mt.load_library()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    head_name = args.config or "c5"
    head = measure(head_name, args.steps, args.warmup, args.interleave, 0.0 if args.no_cpu_baseline else args.cpu_seconds,
                   args.calibrate_copy_mib)
    per_config = None
    if args.config is None:
        per_config = {}
        for name, (k, wu, cs) in SIDE.items():
            per_config[name] = measure(name, k, wu, args.interleave, 0.0 if args.no_cpu_baseline else cs)
    line = {"metric": "inferences/sec across tenants at 1 GPU", "value": head["value"], "unit": "inferences/sec",
            "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": head["ms_per_step"],
            "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
            "dtype": head["dtype"], "data": "synthetic", "config": head["config"],
            "roofline": head["roofline"], "cpu_baseline": head["cpu_baseline"], "device_ms": head["device_ms"],
            "kernels_us": head["kernels_us"], "host_enqueue_us_per_step": head["host_enqueue_us_per_step"],
            "interleaved": head["interleaved"], "per_config": per_config}
    print(json.dumps(line))


if __name__ == "__main__":
    main()
