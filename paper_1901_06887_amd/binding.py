"""ctypes binding of ``libmt.so`` (the C ABI in ``include/mt.h``).

Argument marshalling only: every step of the inference path runs in the library's HIP
kernels.  PyTorch appears here only as the owner of device buffers and streams.  If the
shared library has not been built, importing a context raises; there is no fallback.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmt.so")

MT_OK = 0
MT_STATIC_SCRATCH_BYTES = 16 << 20
STATUS_NAMES = {0: "MT_OK", 1: "MT_EINVAL", 2: "MT_ENOMEM", 3: "MT_ENOTFOUND", 4: "MT_EEXIST",
                5: "MT_EUNSUPPORTED", 6: "MT_EFULL", 7: "MT_ESTATE", 8: "MT_EDEVICE"}
MT_FC, MT_CONV2D, MT_GAP, MT_MAXPOOL, MT_ADD = 0, 1, 2, 3, 4
MT_ACT_NONE, MT_ACT_RELU, MT_ACT_GELU = 0, 1, 2
MT_F32, MT_BF16 = 0, 1
MT_MAX_LAYERS = 48


class MtError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__("%s: %s" % (STATUS_NAMES.get(status, status), text))
        self.status = status


class mt_layer_spec(ctypes.Structure):
    _fields_ = [(n, ctypes.c_uint32) for n in
                ("kind", "act", "in_features", "out_features", "in_h", "in_w", "kh", "kw", "stride", "pad", "src", "src2")]


class mt_config(ctypes.Structure):
    _fields_ = [("max_tenants", ctypes.c_uint32), ("max_requests", ctypes.c_uint32),
                ("max_width", ctypes.c_uint32), ("max_classes", ctypes.c_uint32),
                ("arena_bytes", ctypes.c_uint64), ("dtype", ctypes.c_uint32), ("device", ctypes.c_int32),
                ("run_slots", ctypes.c_uint32), ("cache", ctypes.c_uint32)]


class mt_tenant_account(ctypes.Structure):
    _fields_ = [("requests", ctypes.c_uint64), ("runs", ctypes.c_uint64), ("flops_per_request", ctypes.c_uint64),
                ("weight_bytes", ctypes.c_uint64), ("io_bytes_per_request", ctypes.c_uint64),
                ("resident", ctypes.c_uint64), ("arena_bytes", ctypes.c_uint64)]


class mt_cache_stats(ctypes.Structure):
    _fields_ = [("resident_models", ctypes.c_uint32), ("uploads", ctypes.c_uint64), ("upload_bytes", ctypes.c_uint64),
                ("evictions", ctypes.c_uint64)]


class mt_run_estimate(ctypes.Structure):
    _fields_ = [("flops", ctypes.c_double), ("hbm_bytes", ctypes.c_double), ("device_ms", ctypes.c_double),
                ("rows", ctypes.c_uint32), ("launches", ctypes.c_uint32),
                ("upload_bytes", ctypes.c_double), ("upload_ms", ctypes.c_double)]


class mt_model_footprint(ctypes.Structure):
    _fields_ = [("arena_bytes", ctypes.c_uint64), ("min_width", ctypes.c_uint32), ("n_classes", ctypes.c_uint32),
                ("in_len", ctypes.c_uint32), ("reserved", ctypes.c_uint32)]


class mt_outputs(ctypes.Structure):
    _fields_ = [("labels", ctypes.c_void_p), ("probs", ctypes.c_void_p), ("logits", ctypes.c_void_p),
                ("n_classes", ctypes.c_void_p), ("capacity", ctypes.c_uint32), ("row_stride", ctypes.c_uint32)]


class mt_stats(ctypes.Structure):
    _fields_ = [("n_tenants", ctypes.c_uint32), ("arena_used", ctypes.c_uint64), ("arena_bytes", ctypes.c_uint64),
                ("last_run_rows", ctypes.c_uint32), ("last_run_launches", ctypes.c_uint32)]


class mt_profile(ctypes.Structure):
    _fields_ = [("batcher_ms", ctypes.c_float), ("gather_ms", ctypes.c_float), ("head_ms", ctypes.c_float),
                ("fc_ms", ctypes.c_float * MT_MAX_LAYERS), ("fc_big_ms", ctypes.c_float * MT_MAX_LAYERS), ("conv_ms", ctypes.c_float * MT_MAX_LAYERS),
                ("gap_ms", ctypes.c_float * MT_MAX_LAYERS), ("ops_ms", ctypes.c_float * MT_MAX_LAYERS),
                ("total_ms", ctypes.c_float)]


_lib = None


def load_library() -> ctypes.CDLL:
    """Load libmt.so; raises if it has not been built (no fallback path exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError("%s is missing: build it with `python -m paper_1901_06887_amd.build`" % LIB_PATH)
    L = ctypes.CDLL(LIB_PATH)
    vp, u32 = ctypes.c_void_p, ctypes.c_uint32
    L.mt_create.argtypes = [ctypes.POINTER(vp), ctypes.POINTER(mt_config)]
    L.mt_destroy.argtypes = [vp]
    L.mt_register_model.argtypes = [vp, u32, ctypes.POINTER(mt_layer_spec), u32, ctypes.POINTER(vp), ctypes.POINTER(vp)]
    L.mt_register_model_bn.argtypes = [vp, u32, ctypes.POINTER(mt_layer_spec), u32, ctypes.POINTER(vp), ctypes.POINTER(vp),
                                       ctypes.POINTER(vp), ctypes.c_float]
    L.mt_unregister_model.argtypes = [vp, u32]
    L.mt_submit.argtypes = [vp, u32, vp, u32, ctypes.POINTER(u32)]
    L.mt_submit_batch.argtypes = [vp, vp, vp, u32, u32, ctypes.POINTER(u32)]
    L.mt_run.argtypes = [vp, vp, ctypes.POINTER(mt_outputs), ctypes.POINTER(u32)]
    L.mt_run_static.argtypes = [vp, vp, ctypes.POINTER(mt_outputs), ctypes.POINTER(u32)]
    L.mt_last_counts.argtypes = [vp, ctypes.POINTER(u32)]
    L.mt_get_stats.argtypes = [vp, ctypes.POINTER(mt_stats)]
    L.mt_tenant_account_get.argtypes = [vp, u32, ctypes.POINTER(mt_tenant_account)]
    L.mt_estimate_run.argtypes = [vp, ctypes.POINTER(u32), ctypes.POINTER(mt_run_estimate)]
    L.mt_admit.argtypes = [vp, ctypes.POINTER(u32), ctypes.c_double, ctypes.POINTER(u32), ctypes.POINTER(mt_run_estimate)]
    L.mt_prefetch.argtypes = [vp, ctypes.POINTER(u32), u32, vp]
    L.mt_cache_stats_get.argtypes = [vp, ctypes.POINTER(mt_cache_stats)]
    L.mt_model_footprint_get.argtypes = [ctypes.POINTER(mt_layer_spec), u32, u32, ctypes.POINTER(mt_model_footprint)]
    L.mt_debug_mfma_rate.argtypes = [vp, ctypes.POINTER(ctypes.c_double)]
    L.mt_debug_poison.argtypes = [vp]
    L.mt_debug_copy.argtypes = [vp, vp, ctypes.c_uint64, vp]
    L.mt_debug_big_tile_rows.argtypes = [u32, u32]
    L.mt_debug_big_tile_rows.restype = u32
    L.mt_debug_big_tile_walk.argtypes = [u32]
    L.mt_debug_big_tile_walk.restype = u32
    L.mt_debug_conv_row_tiling.argtypes = [u32, u32, u32, u32, u32, u32, ctypes.POINTER(u32), ctypes.POINTER(u32), ctypes.POINTER(u32), ctypes.POINTER(ctypes.c_uint64)]
    L.mt_debug_conv_row_tiling.restype = ctypes.c_int
    L.mt_set_profiling.argtypes = [vp, ctypes.c_int]
    L.mt_get_profile.argtypes = [vp, ctypes.POINTER(mt_profile)]
    L.mt_last_error.argtypes = [vp]
    L.mt_last_error.restype = ctypes.c_char_p
    L.mt_version.restype = ctypes.c_char_p
    for name in ("mt_create", "mt_destroy", "mt_register_model", "mt_register_model_bn", "mt_unregister_model", "mt_submit",
                 "mt_submit_batch", "mt_run", "mt_run_static", "mt_last_counts", "mt_get_stats", "mt_tenant_account_get", "mt_estimate_run", "mt_prefetch", "mt_cache_stats_get", "mt_admit", "mt_debug_poison", "mt_debug_copy",
                 "mt_set_profiling", "mt_get_profile", "mt_model_footprint_get", "mt_debug_mfma_rate"):
        getattr(L, name).restype = ctypes.c_int
    _lib = L
    return L


def layer_spec(kind, act=MT_ACT_NONE, in_features=0, out_features=0, in_h=0, in_w=0, stride=1, ksize=3, pad=1,
               src=0, src2=0) -> mt_layer_spec:
    window = kind in (MT_CONV2D, MT_MAXPOOL)
    return mt_layer_spec(kind, act, in_features, out_features, in_h, in_w, ksize if window else 0, ksize if window else 0,
                         stride if window else 0, pad if window else 0, src, src2)


def _host_array(a, dtype_code: int) -> np.ndarray:
    """Contiguous host array in the context's element type (bf16 as uint16 bit patterns)."""
    a = np.asarray(a)
    if dtype_code == MT_BF16:
        if a.dtype != np.uint16:
            a32 = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
            if np.any(a32 & 0xFFFF):
                raise ValueError("weights of a bf16 context must be bfloat16-representable or uint16 bit patterns")
            a = (a32 >> 16).astype(np.uint16)
        return np.ascontiguousarray(a)
    return np.ascontiguousarray(a, dtype=np.float32)


class Context:
    """One worker context (mt_ctx).  Methods mirror the C entry points one to one."""

    def __init__(self, max_tenants: int, max_requests: int, max_width: int, max_classes: int,
                 arena_bytes: int, dtype: int, device: int = 0, run_slots: int = 1, cache: bool = False):
        self._lib = load_library()
        self.dtype = dtype
        self.cfg = mt_config(max_tenants, max_requests, max_width, max_classes, arena_bytes, dtype, device, run_slots, int(cache))
        self._h = ctypes.c_void_p()
        st = self._lib.mt_create(ctypes.byref(self._h), ctypes.byref(self.cfg))
        if st != MT_OK:
            raise MtError(st, "mt_create failed")

    def _check(self, st: int):
        if st != MT_OK:
            raise MtError(st, self._lib.mt_last_error(self._h).decode())

    def close(self):
        if self._h:
            self._lib.mt_destroy(self._h)
            self._h = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- mt_register_model ---------------------------------------------------------------
    def register_model(self, tenant: int, specs: Sequence[mt_layer_spec], weights, biases, bn=None, bn_eps: float = 1e-5):
        """mt_register_model, or mt_register_model_bn when `bn` (per layer: None or (gamma, beta, mean, var)) is given."""
        n = len(specs)
        arr = (mt_layer_spec * n)(*specs)
        keep = []
        wp = (ctypes.c_void_p * n)()
        bp = (ctypes.c_void_p * n)()
        np_ = (ctypes.c_void_p * n)()
        for i in range(n):
            if weights[i] is not None:
                w = _host_array(weights[i], self.dtype); keep.append(w); wp[i] = w.ctypes.data
            if biases is not None and biases[i] is not None:
                b = np.ascontiguousarray(biases[i], dtype=np.float32); keep.append(b); bp[i] = b.ctypes.data
            if bn is not None and bn[i] is not None:
                q = np.ascontiguousarray(np.stack([np.asarray(v, dtype=np.float32) for v in bn[i]])); keep.append(q); np_[i] = q.ctypes.data
        if bn is None:
            self._check(self._lib.mt_register_model(self._h, tenant, arr, n, wp, bp))
        else:
            self._check(self._lib.mt_register_model_bn(self._h, tenant, arr, n, wp, bp, np_, float(bn_eps)))

    def unregister_model(self, tenant: int):
        self._check(self._lib.mt_unregister_model(self._h, tenant))

    # -- mt_submit / mt_submit_batch (device pointers) -------------------------------------
    def submit(self, tenant: int, inputs_ptr: int, n_rows: int) -> int:
        first = ctypes.c_uint32(0)
        self._check(self._lib.mt_submit(self._h, tenant, ctypes.c_void_p(inputs_ptr), n_rows, ctypes.byref(first)))
        return first.value

    def submit_batch(self, tenant_ids_ptr: int, inputs_ptr: int, n_rows: int, row_stride: int) -> int:
        first = ctypes.c_uint32(0)
        self._check(self._lib.mt_submit_batch(self._h, ctypes.c_void_p(tenant_ids_ptr), ctypes.c_void_p(inputs_ptr),
                                              n_rows, row_stride, ctypes.byref(first)))
        return first.value

    # -- mt_run ------------------------------------------------------------------------------
    def run(self, stream_ptr: int, labels_ptr: int, probs_ptr: int, logits_ptr: int, n_classes_ptr: int,
            capacity: int, row_stride: int) -> int:
        out = mt_outputs(labels_ptr or None, probs_ptr or None, logits_ptr or None, n_classes_ptr or None,
                         capacity, row_stride)
        n = ctypes.c_uint32(0)
        self._check(self._lib.mt_run(self._h, ctypes.c_void_p(stream_ptr or None), ctypes.byref(out), ctypes.byref(n)))
        return n.value

    def run_static(self, stream_ptr: int, labels_ptr: int, probs_ptr: int, logits_ptr: int, n_classes_ptr: int,
                   capacity: int, row_stride: int) -> int:
        """mt_run_static: the same run with its scratch in the library's static device array (allocates nothing)."""
        out = mt_outputs(labels_ptr or None, probs_ptr or None, logits_ptr or None, n_classes_ptr or None,
                         capacity, row_stride)
        n = ctypes.c_uint32(0)
        self._check(self._lib.mt_run_static(self._h, ctypes.c_void_p(stream_ptr or None), ctypes.byref(out), ctypes.byref(n)))
        return n.value

    def last_counts(self) -> np.ndarray:
        counts = np.zeros(self.cfg.max_tenants, dtype=np.uint32)
        self._check(self._lib.mt_last_counts(self._h, counts.ctypes.data_as(ctypes.POINTER(ctypes.c_uint32))))
        return counts

    def set_profiling(self, enable: bool):
        self._check(self._lib.mt_set_profiling(self._h, int(enable)))

    def get_profile(self) -> dict:
        p = mt_profile()
        self._check(self._lib.mt_get_profile(self._h, ctypes.byref(p)))
        return {"batcher_ms": p.batcher_ms, "gather_ms": p.gather_ms, "head_ms": p.head_ms,
                "fc_ms": list(p.fc_ms), "fc_big_ms": list(p.fc_big_ms), "conv_ms": list(p.conv_ms), "gap_ms": list(p.gap_ms), "ops_ms": list(p.ops_ms), "total_ms": p.total_ms}

    def debug_poison(self):
        self._check(self._lib.mt_debug_poison(self._h))

    def tenant_account(self, tenant: int) -> dict:
        a = mt_tenant_account()
        self._check(self._lib.mt_tenant_account_get(self._h, tenant, ctypes.byref(a)))
        return {k: int(getattr(a, k)) for k, _ in mt_tenant_account._fields_}

    def estimate_run(self, counts) -> dict:
        arr = (ctypes.c_uint32 * self.cfg.max_tenants)(*[int(x) for x in counts])
        e = mt_run_estimate()
        self._check(self._lib.mt_estimate_run(self._h, arr, ctypes.byref(e)))
        return {k: getattr(e, k) for k, _ in mt_run_estimate._fields_}

    def admit(self, pending, budget_ms: float):
        """(admitted counts, estimate of the admitted run) for a device-time budget."""
        T = self.cfg.max_tenants
        arr = (ctypes.c_uint32 * T)(*[int(x) for x in pending])
        out = (ctypes.c_uint32 * T)()
        e = mt_run_estimate()
        self._check(self._lib.mt_admit(self._h, arr, float(budget_ms), out, ctypes.byref(e)))
        return [int(x) for x in out], {k: getattr(e, k) for k, _ in mt_run_estimate._fields_}

    def prefetch(self, tenants, stream_ptr: int = 0) -> None:
        arr = (ctypes.c_uint32 * max(1, len(tenants)))(*[int(t) for t in tenants])
        self._check(self._lib.mt_prefetch(self._h, arr, len(tenants), ctypes.c_void_p(stream_ptr or None)))

    def cache_stats(self) -> dict:
        st = mt_cache_stats()
        self._check(self._lib.mt_cache_stats_get(self._h, ctypes.byref(st)))
        return {k: int(getattr(st, k)) for k, _ in mt_cache_stats._fields_}

    def stats(self) -> dict:
        s = mt_stats()
        self._check(self._lib.mt_get_stats(self._h, ctypes.byref(s)))
        return {k: getattr(s, k) for k, _ in mt_stats._fields_}


def model_footprint(specs: Sequence[mt_layer_spec], dtype: int) -> dict:
    """mt_model_footprint_get: arena bytes, smallest max_width / max_classes, input length of a model."""
    n = len(specs)
    f = mt_model_footprint()
    st = load_library().mt_model_footprint_get((mt_layer_spec * n)(*specs), n, dtype, ctypes.byref(f))
    if st != MT_OK:
        raise MtError(st, "mt_model_footprint_get failed")
    return {"arena_bytes": int(f.arena_bytes), "min_width": int(f.min_width), "n_classes": int(f.n_classes), "in_len": int(f.in_len)}


def debug_mfma_rate(stream: int = 0) -> float:
    """TFLOP/s that a loop of nothing but bf16 matrix instructions sustains on the current device."""
    v = ctypes.c_double(0.0)
    st = load_library().mt_debug_mfma_rate(ctypes.c_void_p(stream or None), ctypes.byref(v))
    if st != MT_OK:
        raise MtError(st, "mt_debug_mfma_rate failed")
    return v.value


def debug_copy(dst: int, src: int, nbytes: int, stream: int = 0) -> None:
    """Plain device copy kernel of a known size (a yardstick for byte counters)."""
    st = load_library().mt_debug_copy(dst, src, nbytes, stream)
    if st != 0:
        raise MtError(st, "mt_debug_copy failed")


def debug_big_tile_rows(rows: int, out_features: int) -> int:
    """Rows of a tenant's FC layer that the compute-bound kernel serves when a run uses it (0: none)."""
    return int(load_library().mt_debug_big_tile_rows(rows, out_features))


def debug_big_tile_walk(in_features: int) -> bool:
    """Whether the big tiles of a layer index with this shortest fan-in are walked by one workgroup per compute unit."""
    return bool(load_library().mt_debug_big_tile_walk(in_features))


def debug_conv_row_tiling(in_h: int, in_w: int, in_channels: int, ksize: int = 3, stride: int = 1, elem_size: int = 2):
    """How a convolution layer is tiled: None (runs of 128 pixels, gathered), or a dict with the output rows per tile,
    the whole images per tile, the tiles per image and the bytes of LDS that a tile's input rows take."""
    n_oh, ni, tpi, frame = ctypes.c_uint32(), ctypes.c_uint32(), ctypes.c_uint32(), ctypes.c_uint64()
    if not load_library().mt_debug_conv_row_tiling(in_h, in_w, in_channels, ksize, stride, elem_size,
                                                   ctypes.byref(n_oh), ctypes.byref(ni), ctypes.byref(tpi), ctypes.byref(frame)):
        return None
    return {"rows_per_tile": n_oh.value, "images_per_tile": ni.value, "tiles_per_image": tpi.value, "frame_bytes": frame.value}


def version() -> str:
    return load_library().mt_version().decode()
