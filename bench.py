#!/usr/bin/env python3
"""Throughput of the multi-tenant hot path on one MI355X.

One step = one pass of the whole path over one synthetic batch: mt_submit_batch + mt_run
(tenant segmentation, gather, every grouped layer launch, softmax/argmax head), inputs and
models already resident in device memory.  Prints one JSON line.

  value       inferences/sec over the K timed steps (wall clock between device syncs), with
              `config.runs_in_flight` runs in flight, each a whole step on a stream and output
              buffers of its own; `one_run_at_a_time` is the same K steps on one stream
  roofline    the grouped GEMM kernel against HBM bandwidth (weight-streaming mixes) or the
              bf16 MFMA peak (c5), from its average launch duration measured with HIP events
              on the run's stream in a second pass over the same K steps (event brackets cost
              microseconds per kernel, so they stay out of the throughput pass), one run at a
              time; the bracket of a launch reads within 2 % of its kernel-trace duration
              `traffic` is the HBM bytes per launch of that kernel from stored hardware-counter
              runs (profiles/), null when there is none for this workload or the device code
              has changed since they were taken
  one_run_at_a_time  also carries host_enqueue_us_per_step: wall time of the K submit + run calls
              before the final wait (an upper bound of the host's cost per step: a full queue blocks)
  device_ms   per-step device time between two events around the run (median, p99/mean), and
              the same with the caches flushed between steps (`cold`): a batch whose weights
              fit the last-level cache is otherwise partly served from it on repeated runs
  cpu_baseline the fp64 oracle timed on the host cores on a bounded sample of the same batch
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0
FP32_MATRIX_PEAK_TFLOPS = 157.3


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
            if L.kind == wl.GAP:
                continue
            m_t = rows_t if rows_of is None else rows_of(rows_t, L)
            if m_t == 0:
                continue
            if L.kind == wl.FC:
                f = 2 * m_t * L.in_features * L.out_features
            else:
                oh, ow = L.out_hw()
                f = 2 * m_t * oh * ow * 9 * L.in_features * L.out_features
            b = model.weights[l].size * es + model.biases[l].size * 4
            b += m_t * L.in_len() * es
            if pooled_by_conv and l + 1 < n and model.layers[l + 1].kind == wl.GAP:
                b += m_t * L.out_features * es          # the launch writes the pooled activation, not the image
            else:
                b += m_t * L.out_len() * (4 if l == n - 1 else es)
            flops[l] = flops.get(l, 0) + f
            bytes_[l] = bytes_.get(l, 0) + b
    return flops, bytes_


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", default="c2", choices=["c1", "c2", "c3", "c4", "c5"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--interleave", type=int, default=3,
                    help="runs in flight during the timed steps, each on a stream of its own (1: one run at a time); "
                         "the one-at-a-time figure is always reported too")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="target oracle time of the CPU baseline sample")
    ap.add_argument("--calibrate-copy-mib", type=int, default=0,
                    help="first run the library's plain copy kernel over this many MiB (byte-counter yardstick)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this program runs on one GPU only (no sharding, no collectives); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_1901_06887_amd as mt
    import workloads as wl
    from paper_1901_06887_amd import torch_io

    mt.load_library()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    w = wl.CONFIGS[args.config]()
    es = 4 if w.dtype == "f32" else 2
    R = w.n_requests
    ctx = mt.context_for(w.tenants, w.dtype, R, run_slots=max(1, min(args.interleave, 4)))
    mt.register_tenants(ctx, w.tenants)
    d_ids = torch.from_numpy(w.tenant_ids).cuda()
    d_x = torch_io.to_device(w.inputs, w.dtype)
    out = torch_io.alloc_outputs(R, ctx.cfg.max_classes)
    stream = torch.cuda.current_stream()

    def step():
        mt.serve(ctx, d_ids, d_x, out=out, stream=stream)

    if args.calibrate_copy_mib:
        nb = args.calibrate_copy_mib << 20
        a_buf, b_buf = torch.zeros(nb, dtype=torch.uint8, device="cuda"), torch.empty(nb, dtype=torch.uint8, device="cuda")
        for _ in range(4):
            mt.debug_copy(b_buf.data_ptr(), a_buf.data_ptr(), nb, stream.cuda_stream)
        torch.cuda.synchronize()
        del a_buf, b_buf

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    host_dt = time.perf_counter() - t0          # the host's share: mt_submit_batch + mt_run through the binding, K times
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3
    value = R * args.steps / dt

    # the same steps with several runs in flight, each on a stream and an output buffer of its own
    # (batch interleaving, footnote of paper section 1.3); reported next to the headline value
    interleaved = None
    if args.interleave > 1:
        n_il = min(args.interleave, 4)
        streams = [torch.cuda.Stream() for _ in range(n_il)]
        outs = [torch_io.alloc_outputs(R, ctx.cfg.max_classes) for _ in range(n_il)]
        torch.cuda.synchronize()
        for i in range(max(args.warmup, n_il)):
            mt.serve(ctx, d_ids, d_x, out=outs[i % n_il], stream=streams[i % n_il])
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            mt.serve(ctx, d_ids, d_x, out=outs[i % n_il], stream=streams[i % n_il])
        torch.cuda.synchronize()
        dt_il = time.perf_counter() - t0
        same = all(torch.equal(o.labels, out.labels) and torch.equal(o.logits, out.logits) for o in outs)
        interleaved = {"streams": n_il, "value": R * args.steps / dt_il, "unit": "inferences/sec",
                       "ms_per_step": dt_il / args.steps * 1e3, "same_answers_as_single_stream": bool(same)}
        del outs
        if not same:
            raise SystemExit("runs in flight together gave other answers than runs one at a time")

    # per-step device time (two events around each step), warm and with caches flushed between steps
    def device_times(n, flush=None):
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n)]
        for e0, e1 in ev:
            if flush is not None:
                flush.add_(1)
            e0.record(stream)
            step()
            e1.record(stream)
        torch.cuda.synchronize()
        return np.array([e0.elapsed_time(e1) for e0, e1 in ev])
    warm = device_times(args.steps)
    n_cold = max(5, min(args.steps, 30))
    flush = torch.zeros(1 << 30, dtype=torch.uint8, device="cuda")       # 4x the last-level cache
    cold = device_times(n_cold, flush)
    del flush
    device_ms = {"median": float(np.median(warm)), "mean": float(warm.mean()), "p99_over_mean": float(np.percentile(warm, 99) / warm.mean()),
                 "cold_median": float(np.median(cold)), "cold_steps": n_cold,
                 "cold_inferences_per_sec": float(R / (np.median(cold) * 1e-3))}

    # what a pair of events reads with nothing between them: every per-kernel bracket below
    # carries that much on top of the kernel's own duration
    pairs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(64)]
    for e0, e1 in pairs:
        step()                                     # same queue state as in the profiled pass: work ahead of the bracket
        e0.record(stream)
        e1.record(stream)
    torch.cuda.synchronize()
    bracket_ms = float(np.median([e0.elapsed_time(e1) for e0, e1 in pairs]))

    # second pass over the same steps with per-kernel HIP events on the run's stream
    ctx.set_profiling(True)
    prof = []
    for _ in range(args.steps):
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
        dom_ms, dom_name = big_ms, "fc_big_kernel"
        # the big-tile kernel is credited only with the rows it serves (a short remainder of a
        # tenant's rows goes to the streaming kernel)
        flops, bytes_ = gemm_launch_costs(w, es, lambda rows, L: mt.debug_big_tile_rows(rows, L.out_features) if L.kind == wl.FC else 0)
    other_ms = fc_ms if dom_ms is conv_ms else conv_ms
    launches = [l for l in range(n_slots) if dom_ms[l] > 0 and other_ms[l] == 0 and l in bytes_]
    # The bracket of a launch (two events on the run's stream) is what is reported: it reads within
    # 2 % of the kernel-trace duration of the same launches.  What two events with nothing between
    # them read behind a run is reported next to it; it is ~0.6 us under rocprofv3 and 3-5 us in a
    # plain run, so subtracting it would make the plain-run figure disagree with the trace.
    raw_dur_s = sum(dom_ms[l] for l in launches) / len(launches) * 1e-3
    avg_dur_s = raw_dur_s
    avg_bytes = sum(bytes_[l] for l in launches) / len(launches)
    avg_flops = sum(flops[l] for l in launches) / len(launches)
    cost = wl.algorithmic_cost(w)
    intensity = avg_flops / avg_bytes
    if w.dtype == "bf16" and intensity > MFMA_BF16_PEAK_TFLOPS * 1e12 / (HBM_PEAK_GBS * 1e9):
        achieved = avg_flops / avg_dur_s / 1e12
        roofline = {"bound": "mfma", "achieved": achieved, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                    "frac": achieved / MFMA_BF16_PEAK_TFLOPS, "traffic": None}
    else:
        achieved = avg_bytes / avg_dur_s / 1e9
        roofline = {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": achieved / HBM_PEAK_GBS, "traffic": None}
    from paper_1901_06887_amd import profile_summary
    traffic_file = os.path.join(ROOT, "profiles", "%s_%s_hbm_traffic.md" % (dom_name, w.name))
    roofline["traffic"] = profile_summary.read_traffic(traffic_file)
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
                  "head": float(np.mean([p["head_ms"] for p in prof])) * 1e3,
                  "device_total": float(np.mean([p["total_ms"] for p in prof])) * 1e3}

    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        threads = min(16, os.cpu_count() or 1)
        models = oracle.models_from_workload(w)
        macs_per_row = np.array([models[int(t)].macs_per_request() for t in w.tenant_ids], dtype=np.float64)
        # bounded sample: arrival-ordered prefix of the batch worth ~cpu_seconds at ~1.5 GMAC/s per thread
        budget = args.cpu_seconds * 1.5e9 * threads
        n_sample = int(min(R, max(threads, np.searchsorted(np.cumsum(macs_per_row), budget))))
        x64 = w.inputs[:n_sample].astype(np.float64)
        reps, t0 = 0, time.perf_counter()
        while True:                       # a batch the oracle finishes in under a second is repeated for a stable figure
            oracle.run_batch(models, w.tenant_ids[:n_sample], x64, threads=threads)
            reps += 1
            cdt = time.perf_counter() - t0
            if cdt >= min(10.0, args.cpu_seconds) or reps >= 200:
                break
        cpu = {"value": n_sample * reps / cdt, "unit": "inferences/sec", "cores": threads, "kind": "oracle",
               "sample": "first %d of %d requests of %s in arrival order, %d pass(es), fp64 loop nests, %.1f s" % (
                   n_sample, R, w.name, reps, cdt)}

    # headline: throughput of the timed steps with `interleave` runs in flight (every step is a whole
    # mt_run over the whole batch; nothing is shared between steps but the registered weights);
    # `one_run_at_a_time` is the same number of steps enqueued on one stream, each after the other
    one_at_a_time = {"value": value, "unit": "inferences/sec", "ms_per_step": ms_per_step,
                     "host_enqueue_us_per_step": host_dt / args.steps * 1e6}
    if interleaved is not None:
        value, ms_per_step = interleaved["value"], interleaved["ms_per_step"]
    line = {"metric": "inferences/sec across tenants at 1 GPU", "value": value, "unit": "inferences/sec",
            "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
            "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
            "dtype": "f32" if es == 4 else "bf16", "data": "synthetic",
            "config": {"workload": w.name, "tenants": len(w.tenants), "requests_per_step": R,
                       "active_tenants": len(w.counts()), "runs_in_flight": interleaved["streams"] if interleaved else 1,
                       "algorithmic_flops_per_step": cost["flops"],
                       "algorithmic_bytes_per_step": cost["bytes"],
                       "whole_path_hbm_frac": cost["bytes"] / (ms_per_step * 1e-3) / (HBM_PEAK_GBS * 1e9),
                       "whole_path_mfma_frac": cost["flops"] / (ms_per_step * 1e-3) / (MFMA_BF16_PEAK_TFLOPS * 1e12)},
            "roofline": roofline, "device_ms": device_ms, "kernels_us": kernels_us, "one_run_at_a_time": one_at_a_time,
            "cpu_baseline": cpu}
    print(json.dumps(line))
    ctx.close()


if __name__ == "__main__":
    main()
