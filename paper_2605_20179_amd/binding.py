"""ctypes binding of libtide's C ABI (include/tide.h): argument marshalling only.

Every step of the path runs inside the library's HIP kernels; torch is used to
own device memory and to supply the stream.  There is no CPU fallback: if the
shared library is missing the import of this module raises."""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libtide.so")

TIDE_OK, TIDE_E_INVAL, TIDE_E_RANGE, TIDE_E_STATE, TIDE_E_HIP, TIDE_E_NOMEM = 0, -1, -2, -3, -4, -5
TIDE_GATING_SOFTMAX, TIDE_GATING_SIGMOID = 0, 1
TIDE_BIAS_NONE, TIDE_BIAS_LOGIT, TIDE_BIAS_SELECT = 0, 1, 2
TIDE_RESIDENT_BF16, TIDE_RESIDENT_P12 = 0, 1

EXPORTS = [
    "tide_create", "tide_destroy", "tide_last_error", "tide_expert_blob_bytes", "tide_pack_expert",
    "tide_register_experts", "tide_set_shared", "tide_set_resident", "tide_moe_step", "tide_moe_step_routed",
    "tide_interval_stats", "tide_refresh", "tide_wait_refresh", "tide_get_table", "tide_read_slot",
    "tide_refresh_copy_ms", "tide_profile", "tide_profile_read", "tide_counters", "tide_moe_apply_misses",
    "tide_step_histogram", "tide_routing_stability", "tide_interval_costs", "tide_optimal_interval", "tide_fit_drift", "tide_scale_counts", "tide_refresh_deferred", "tide_commit",
    "tide_host_experts", "tide_moe_apply_misses_host", "tide_host_miss_ms", "tide_host_expert", "tide_host_link_share", "tide_host_misses",
    "tide_compressed_blob_bytes", "tide_compress_expert", "tide_decompress_expert", "tide_register_compressed",
    "tide_refresh_async", "tide_refresh_result",
    "tide_moe_step_noalloc", "tide_noalloc_scratch_bytes", "tide_set_counts", "tide_read_work_items",
    "tide_refresh_engine", "tide_queue_refresh_wait", "tide_hbm_stream_probe", "tide_moe_stack_step",
]
KERNEL_NAMES = ["router_logits", "topk_gate", "dispatch", "gate_up_swiglu", "down", "combine", "gate_up_swiglu_big", "down_big"]


class tide_config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("d", "n_experts", "top_k", "d_ff", "n_shared", "n_layers", "capacity",
                                          "max_tokens", "gating", "bias_mode", "resident_format")]


class tide_miss(C.Structure):
    _fields_ = [("token", C.c_int32), ("expert", C.c_int32), ("weight", C.c_float)]


class tide_copy(C.Structure):
    _fields_ = [("expert", C.c_int32), ("slot", C.c_int32), ("host_offset", C.c_uint64), ("bytes", C.c_uint64)]


MISS_DTYPE = np.dtype([("token", np.int32), ("expert", np.int32), ("weight", np.float32)])


class TideError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__("libtide error %d: %s" % (code, text))
        self.code = code


def _load() -> C.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError("libtide.so is not built (%s); run `python -m paper_2605_20179_amd.build`. "
                          "There is no fallback path." % LIB_PATH)
    lib = C.CDLL(LIB_PATH)
    vp, i32p, f32p = C.c_void_p, C.POINTER(C.c_int32), C.POINTER(C.c_float)
    cfgp = C.POINTER(tide_config)
    lib.tide_create.argtypes = [cfgp, C.POINTER(vp)]
    lib.tide_destroy.argtypes = [vp]
    lib.tide_last_error.argtypes = [vp]
    lib.tide_last_error.restype = C.c_char_p
    lib.tide_expert_blob_bytes.argtypes = [cfgp]
    lib.tide_expert_blob_bytes.restype = C.c_uint64
    lib.tide_pack_expert.argtypes = [cfgp, vp, vp, vp, vp]
    lib.tide_compressed_blob_bytes.argtypes = [cfgp]
    lib.tide_compressed_blob_bytes.restype = C.c_uint64
    lib.tide_compress_expert.argtypes = [cfgp, vp, vp]
    lib.tide_decompress_expert.argtypes = [cfgp, vp, vp]
    lib.tide_register_compressed.argtypes = [vp, C.c_int, vp, C.c_uint64]
    lib.tide_register_experts.argtypes = [vp, C.c_int, vp, C.c_uint64]
    lib.tide_set_shared.argtypes = [vp, C.c_int, vp]
    lib.tide_set_resident.argtypes = [vp, C.c_int, vp, C.c_int]
    lib.tide_moe_step.argtypes = [vp, C.c_int, vp, C.c_int, vp, vp, vp, vp, C.c_int, vp, vp, vp, vp]
    lib.tide_moe_step_routed.argtypes = [vp, C.c_int, vp, C.c_int, vp, vp, vp, vp, C.c_int, vp, vp]
    lib.tide_moe_step_noalloc.argtypes = lib.tide_moe_step.argtypes
    lib.tide_moe_stack_step.argtypes = [vp, C.c_int, C.c_int, vp, C.c_int, vp, vp, vp, vp, C.c_int, vp, vp]
    lib.tide_noalloc_scratch_bytes.argtypes = []
    lib.tide_noalloc_scratch_bytes.restype = C.c_uint64
    lib.tide_moe_apply_misses.argtypes = [vp, C.c_int, vp, C.c_int, vp, C.c_int, vp, vp, vp]
    lib.tide_moe_apply_misses_host.argtypes = lib.tide_moe_apply_misses.argtypes
    lib.tide_host_experts.argtypes = [vp, C.c_int]
    lib.tide_host_miss_ms.argtypes = [vp, vp]
    lib.tide_host_link_share.argtypes = [vp, C.c_int]
    lib.tide_host_expert.argtypes = [cfgp, vp, vp, C.c_int, vp]
    lib.tide_host_misses.argtypes = [cfgp, vp, C.c_uint64, vp, C.c_int, vp, C.c_int, C.c_int, vp]
    lib.tide_interval_stats.argtypes = [vp, C.c_int, vp, C.c_int, vp]
    lib.tide_set_counts.argtypes = [vp, C.c_int, vp, vp]
    lib.tide_read_work_items.argtypes = [vp, vp, C.c_int, C.POINTER(C.c_int), vp, C.c_int, C.POINTER(C.c_int), vp]
    lib.tide_refresh.argtypes = [vp, C.c_int, vp, C.c_int, C.c_int, vp, vp, C.POINTER(C.c_int), vp]
    lib.tide_refresh_deferred.argtypes = lib.tide_refresh.argtypes
    lib.tide_refresh_async.argtypes = [vp, C.c_int, vp, C.c_int, C.c_int, vp]
    lib.tide_refresh_result.argtypes = [vp, C.c_int, vp, vp, C.POINTER(C.c_int)]
    lib.tide_commit.argtypes = [vp, C.c_int, vp]
    lib.tide_wait_refresh.argtypes = [vp, C.c_int]
    lib.tide_queue_refresh_wait.argtypes = [vp, C.c_int, vp]
    lib.tide_refresh_engine.argtypes = [vp, C.c_int]
    lib.tide_get_table.argtypes = [vp, C.c_int, vp, vp]
    lib.tide_read_slot.argtypes = [vp, C.c_int, C.c_int, vp]
    lib.tide_refresh_copy_ms.argtypes = [vp, C.c_int, C.POINTER(C.c_float)]
    lib.tide_profile.argtypes = [vp, C.c_int]
    lib.tide_profile_read.argtypes = [vp, vp, vp]
    lib.tide_counters.argtypes = [vp, vp, C.c_int, vp]
    lib.tide_hbm_stream_probe.argtypes = [vp, C.c_int, C.c_int, C.POINTER(C.c_double), C.POINTER(C.c_uint64)]
    lib.tide_step_histogram.argtypes = [vp, vp, C.c_int, vp]
    lib.tide_routing_stability.argtypes = [vp, vp, C.c_int, C.c_int, C.c_int, vp, vp, vp, vp]
    lib.tide_interval_costs.argtypes = [C.c_int, C.c_int, C.c_double, C.c_double, C.c_double, vp, vp, vp]
    lib.tide_scale_counts.argtypes = [vp, C.c_int, C.c_int, C.c_int, vp]
    lib.tide_fit_drift.argtypes = [C.c_double, C.c_int, C.c_int, C.c_int, C.POINTER(C.c_double)]
    lib.tide_optimal_interval.argtypes = [C.c_int, C.c_int, C.c_double, C.c_double, C.c_double, vp, C.POINTER(C.c_int),
                                          C.POINTER(C.c_double)]
    for name in EXPORTS:
        if name not in ("tide_last_error", "tide_expert_blob_bytes", "tide_compressed_blob_bytes", "tide_noalloc_scratch_bytes"):
            getattr(lib, name).restype = C.c_int
    return lib


lib = _load()


def make_config(d, n_experts, top_k, d_ff, n_shared, n_layers, capacity, max_tokens, gating, bias_mode,
                resident_format=0) -> tide_config:
    return tide_config(d, n_experts, top_k, d_ff, n_shared, n_layers, capacity, max_tokens, gating, bias_mode, resident_format)


def _check(rc: int, ctx) -> None:
    if rc != TIDE_OK:
        raise TideError(rc, lib.tide_last_error(ctx).decode())


def _ptr(t) -> Optional[int]:
    """Address of a torch tensor, numpy array or None."""
    if t is None:
        return None
    if isinstance(t, np.ndarray):
        assert t.flags["C_CONTIGUOUS"]
        return t.ctypes.data
    assert t.is_contiguous()
    return t.data_ptr()


def _stream_ptr(stream) -> Optional[int]:
    if stream is None:
        return None
    return int(stream.cuda_stream) if hasattr(stream, "cuda_stream") else int(stream)


def tide_expert_blob_bytes(cfg: tide_config) -> int:
    return int(lib.tide_expert_blob_bytes(C.byref(cfg)))


def tide_pack_expert(cfg: tide_config, wg: np.ndarray, wu: np.ndarray, wd: np.ndarray, blob) -> None:
    """wg/wu [d_ff,d], wd [d,d_ff] uint16 (bf16 bits) host arrays -> packed blob (host uint8 buffer)."""
    assert wg.dtype == np.uint16 and wg.shape == (cfg.d_ff, cfg.d) and wu.shape == wg.shape
    assert wd.dtype == np.uint16 and wd.shape == (cfg.d, cfg.d_ff)
    _check(lib.tide_pack_expert(C.byref(cfg), _ptr(np.ascontiguousarray(wg)), _ptr(np.ascontiguousarray(wu)),
                                _ptr(np.ascontiguousarray(wd)), _ptr(blob)), None)


def tide_compressed_blob_bytes(cfg: tide_config) -> int:
    return int(lib.tide_compressed_blob_bytes(C.byref(cfg)))


def tide_compress_expert(cfg: tide_config, blob, comp) -> None:
    """packed blob (host uint8 buffer) -> its 12-bit form (host uint8 buffer of tide_compressed_blob_bytes)."""
    _check(lib.tide_compress_expert(C.byref(cfg), _ptr(blob), _ptr(comp)), None)


def tide_decompress_expert(cfg: tide_config, comp, blob) -> None:
    """12-bit form (host uint8 buffer) -> the packed blob (host uint8 buffer of tide_expert_blob_bytes)."""
    _check(lib.tide_decompress_expert(C.byref(cfg), _ptr(comp), _ptr(blob)), None)


def tide_register_compressed(ctx, layer: int, comp_blobs, comp_stride: int) -> None:
    _check(lib.tide_register_compressed(ctx, layer, _ptr(comp_blobs), comp_stride), ctx)


def tide_create(cfg: tide_config) -> int:
    h = C.c_void_p()
    rc = lib.tide_create(C.byref(cfg), C.byref(h))
    _check(rc, None)
    return h.value


def tide_destroy(ctx: int) -> None:
    lib.tide_destroy(ctx)


def tide_register_experts(ctx, layer: int, host_blobs, blob_stride: int) -> None:
    _check(lib.tide_register_experts(ctx, layer, _ptr(host_blobs), blob_stride), ctx)


def tide_set_shared(ctx, layer: int, blob_host) -> None:
    _check(lib.tide_set_shared(ctx, layer, _ptr(blob_host)), ctx)


def tide_set_resident(ctx, layer: int, experts: Sequence[int]) -> None:
    a = np.ascontiguousarray(np.asarray(experts, dtype=np.int32))
    _check(lib.tide_set_resident(ctx, layer, _ptr(a), len(a)), ctx)


def tide_moe_step(ctx, layer: int, hidden, n_tokens: int, router_w, router_bias, out, miss, miss_cap: int, n_miss,
                  topk_idx=None, topk_w=None, stream=None) -> None:
    _check(lib.tide_moe_step(ctx, layer, _ptr(hidden), n_tokens, _ptr(router_w), _ptr(router_bias), _ptr(out),
                             _ptr(miss), miss_cap, _ptr(n_miss), _ptr(topk_idx), _ptr(topk_w), _stream_ptr(stream)), ctx)


def tide_moe_step_noalloc(ctx, layer: int, hidden, n_tokens: int, router_w, router_bias, out, miss, miss_cap: int, n_miss,
                          topk_idx=None, topk_w=None, stream=None) -> None:
    _check(lib.tide_moe_step_noalloc(ctx, layer, _ptr(hidden), n_tokens, _ptr(router_w), _ptr(router_bias), _ptr(out),
                                     _ptr(miss), miss_cap, _ptr(n_miss), _ptr(topk_idx), _ptr(topk_w), _stream_ptr(stream)), ctx)


def _ptr_array(items):
    """Host array of device (or host) addresses, one per item (None -> NULL)."""
    return (C.c_void_p * len(items))(*[_ptr(t) for t in items])


def tide_moe_stack_step(ctx, first_layer: int, hidden, n_tokens: int, router_w, router_bias, out, miss, miss_cap: int,
                        n_miss, stream=None) -> None:
    """hidden / router_w / router_bias / out / miss / n_miss: one entry per layer (router_bias may be None)."""
    n = len(hidden)
    assert len(router_w) == len(out) == len(n_miss) == n and (miss is None or len(miss) == n)
    bias = None if router_bias is None or all(b is None for b in router_bias) else _ptr_array(router_bias)
    _check(lib.tide_moe_stack_step(ctx, first_layer, n, _ptr_array(hidden), n_tokens, _ptr_array(router_w), bias, _ptr_array(out),
                                   None if miss is None else _ptr_array(miss), miss_cap, _ptr_array(n_miss), _stream_ptr(stream)), ctx)


def tide_noalloc_scratch_bytes() -> int:
    return int(lib.tide_noalloc_scratch_bytes())


def tide_moe_step_routed(ctx, layer: int, hidden, n_tokens: int, topk_idx, topk_w, out, miss, miss_cap: int, n_miss,
                         stream=None) -> None:
    _check(lib.tide_moe_step_routed(ctx, layer, _ptr(hidden), n_tokens, _ptr(topk_idx), _ptr(topk_w), _ptr(out),
                                    _ptr(miss), miss_cap, _ptr(n_miss), _stream_ptr(stream)), ctx)


def tide_moe_apply_misses(ctx, layer: int, hidden, n_tokens: int, miss, miss_cap: int, n_miss, out, stream=None) -> None:
    _check(lib.tide_moe_apply_misses(ctx, layer, _ptr(hidden), n_tokens, _ptr(miss), miss_cap, _ptr(n_miss), _ptr(out),
                                     _stream_ptr(stream)), ctx)


def tide_host_experts(ctx, n_threads: int) -> None:
    _check(lib.tide_host_experts(ctx, n_threads), ctx)


def tide_moe_apply_misses_host(ctx, layer: int, hidden, n_tokens: int, miss, miss_cap: int, n_miss, out, stream=None) -> None:
    _check(lib.tide_moe_apply_misses_host(ctx, layer, _ptr(hidden), n_tokens, _ptr(miss), miss_cap, _ptr(n_miss),
                                          _ptr(out), _stream_ptr(stream)), ctx)


def tide_host_link_share(ctx, percent: int) -> None:
    _check(lib.tide_host_link_share(ctx, percent), ctx)


def tide_host_miss_ms(ctx):
    """(ms waiting for the list, ms of host experts, ms of the whole call) of the last host miss pass."""
    ms = np.zeros(3, dtype=np.float32)
    _check(lib.tide_host_miss_ms(ctx, _ptr(ms)), ctx)
    return float(ms[0]), float(ms[1]), float(ms[2])


def tide_host_misses(cfg: tide_config, blobs: np.ndarray, x_bits: np.ndarray, miss: np.ndarray, n_threads: int,
                     out: np.ndarray) -> None:
    """out[token] += weight * e_expert(x_token) for every entry of miss (MISS_DTYPE), on n_threads host threads.
    blobs: uint8 [E, blob_bytes] packed blobs (host)."""
    x = np.ascontiguousarray(x_bits, dtype=np.uint16)
    m = np.ascontiguousarray(miss, dtype=MISS_DTYPE)
    assert blobs.dtype == np.uint8 and blobs.ndim == 2 and blobs.flags["C_CONTIGUOUS"]
    assert out.dtype == np.float32 and out.shape == (x.shape[0], cfg.d) and out.flags["C_CONTIGUOUS"]
    _check(lib.tide_host_misses(C.byref(cfg), _ptr(blobs), blobs.shape[1], _ptr(x), x.shape[0], m.ctypes.data if m.size else None,
                                m.size, n_threads, _ptr(out)), None)


def tide_host_expert(cfg: tide_config, blob, x_bits: np.ndarray) -> np.ndarray:
    """e(x) of m token states (uint16 bf16 bits [m, d]) through one packed blob, on the calling host thread."""
    x = np.ascontiguousarray(x_bits, dtype=np.uint16)
    assert x.ndim == 2 and x.shape[1] == cfg.d
    y = np.zeros((x.shape[0], cfg.d), dtype=np.float32)
    _check(lib.tide_host_expert(C.byref(cfg), _ptr(blob), _ptr(x), x.shape[0], _ptr(y)), None)
    return y


def tide_interval_stats(ctx, layer: int, n_experts: int, reset: bool, stream=None) -> np.ndarray:
    counts = np.zeros(n_experts, dtype=np.int32)
    _check(lib.tide_interval_stats(ctx, layer, _ptr(counts), int(reset), _stream_ptr(stream)), ctx)
    return counts


def tide_set_counts(ctx, layer: int, counts: np.ndarray, stream=None) -> None:
    a = np.ascontiguousarray(np.asarray(counts, dtype=np.int32))
    _check(lib.tide_set_counts(ctx, layer, _ptr(a), _stream_ptr(stream)), ctx)


WORK_ITEM_DTYPE = np.dtype([("slot", np.int32), ("row0", np.int32), ("nrows", np.int32), ("kind", np.int32)])


def tide_read_work_items(ctx, max_items: int, max_rows: int, stream=None):
    """(work items of the last step as a WORK_ITEM_DTYPE array, row_token[rows])."""
    items = np.zeros(max(max_items, 1), dtype=WORK_ITEM_DTYPE)
    rows = np.zeros(max(max_rows, 1), dtype=np.int32)
    n_items, n_rows = C.c_int(0), C.c_int(0)
    _check(lib.tide_read_work_items(ctx, items.ctypes.data, max_items, C.byref(n_items), rows.ctypes.data, max_rows,
                                    C.byref(n_rows), _stream_ptr(stream)), ctx)
    assert n_items.value <= max_items and n_rows.value <= max_rows, "work-item snapshot truncated"
    return items[:n_items.value].copy(), rows[:n_rows.value].copy()


def tide_refresh(ctx, layer: int, ctx_capacity: int, capacity: int, counts: Optional[np.ndarray] = None,
                 reset_counts: bool = True, stream=None, deferred: bool = False):
    """Returns (expert_in_slot[ctx_capacity] int32, plan = list of (expert, slot, host_offset, bytes)).
    deferred: tide_refresh_deferred (the placement takes effect at tide_commit)."""
    resident = np.full(ctx_capacity, -1, dtype=np.int32)
    plan = (tide_copy * max(ctx_capacity, 1))()
    n = C.c_int(0)
    cnt = None if counts is None else np.ascontiguousarray(np.asarray(counts, dtype=np.int32))
    fn = lib.tide_refresh_deferred if deferred else lib.tide_refresh
    _check(fn(ctx, layer, _ptr(cnt), capacity, int(reset_counts), _ptr(resident),
              C.cast(plan, C.c_void_p), C.byref(n), _stream_ptr(stream)), ctx)
    return resident, [(plan[i].expert, plan[i].slot, plan[i].host_offset, plan[i].bytes) for i in range(n.value)]


def tide_refresh_async(ctx, layer: int, capacity: int, counts: Optional[np.ndarray] = None, reset_counts: bool = True,
                       stream=None) -> None:
    cnt = None if counts is None else np.ascontiguousarray(np.asarray(counts, dtype=np.int32))
    _check(lib.tide_refresh_async(ctx, layer, _ptr(cnt), capacity, int(reset_counts), _stream_ptr(stream)), ctx)


def tide_refresh_result(ctx, layer: int, ctx_capacity: int):
    """(expert_in_slot, plan) of the layer's last refresh, as tide_refresh returns them."""
    resident = np.full(ctx_capacity, -1, dtype=np.int32)
    plan = (tide_copy * max(ctx_capacity, 1))()
    n = C.c_int(0)
    _check(lib.tide_refresh_result(ctx, layer, _ptr(resident), C.cast(plan, C.c_void_p), C.byref(n)), ctx)
    return resident, [(plan[i].expert, plan[i].slot, plan[i].host_offset, plan[i].bytes) for i in range(n.value)]


def tide_wait_refresh(ctx, layer: int) -> None:
    _check(lib.tide_wait_refresh(ctx, layer), ctx)


TIDE_COPY_KERNEL, TIDE_COPY_DMA = 0, 1


def tide_refresh_engine(ctx, engine: int) -> None:
    _check(lib.tide_refresh_engine(ctx, engine), ctx)


def tide_queue_refresh_wait(ctx, layer: int, stream=None) -> None:
    _check(lib.tide_queue_refresh_wait(ctx, layer, _stream_ptr(stream)), ctx)


def tide_refresh_copy_ms(ctx, layer: int) -> float:
    ms = C.c_float(0)
    _check(lib.tide_refresh_copy_ms(ctx, layer, C.byref(ms)), ctx)
    return float(ms.value)


def tide_get_table(ctx, layer: int, n_experts: int, stream=None) -> np.ndarray:
    t = np.zeros(n_experts, dtype=np.int32)
    _check(lib.tide_get_table(ctx, layer, _ptr(t), _stream_ptr(stream)), ctx)
    return t


def tide_read_slot(ctx, layer: int, slot: int, blob_bytes: int) -> np.ndarray:
    b = np.zeros(blob_bytes, dtype=np.uint8)
    _check(lib.tide_read_slot(ctx, layer, slot, _ptr(b)), ctx)
    return b


def tide_profile(ctx, enable) -> None:
    """False/0 off, True/1 every kernel of a step, 2 the expert GEMM kernels only, 3 gate/up and the kernel before it."""
    _check(lib.tide_profile(ctx, int(enable)), ctx)


def tide_profile_read(ctx):
    """Returns {kernel name: (summed ms, launches)} since the last read."""
    ms = np.zeros(len(KERNEL_NAMES), dtype=np.float64)
    n = np.zeros(len(KERNEL_NAMES), dtype=np.int64)
    _check(lib.tide_profile_read(ctx, _ptr(ms), _ptr(n)), ctx)
    return {name: (float(ms[i]), int(n[i])) for i, name in enumerate(KERNEL_NAMES)}


def tide_counters(ctx, reset: bool = False, stream=None):
    """Returns dict(steps, active_slots, rows, misses): running totals kept by the step kernels."""
    out = np.zeros(4, dtype=np.int64)
    _check(lib.tide_counters(ctx, _ptr(out), int(reset), _stream_ptr(stream)), ctx)
    return dict(steps=int(out[0]), active_slots=int(out[1]), rows=int(out[2]), misses=int(out[3]))


def tide_hbm_stream_probe(ctx, layer: int = 0, repeats: int = 8):
    """(GB/s, bytes per launch) of a read-only pass over the layer's cache slots in the GEMMs' weight-stream shape."""
    rate, nbytes = C.c_double(0.0), C.c_uint64(0)
    _check(lib.tide_hbm_stream_probe(ctx, layer, repeats, C.byref(rate), C.byref(nbytes)), ctx)
    return rate.value, nbytes.value


def tide_step_histogram(ctx, n_experts: int, stream=None) -> np.ndarray:
    """The last step's activation vector (tokens per expert) as a host array."""
    out = np.zeros(n_experts, dtype=np.int32)
    _check(lib.tide_step_histogram(ctx, _ptr(out), n_experts, _stream_ptr(stream)), ctx)
    return out


def tide_routing_stability(ctx, counts_dev, n_steps: int, n_experts: int, budget: int, sim_dev, unique_dev, drift_dev,
                           stream=None) -> None:
    _check(lib.tide_routing_stability(ctx, _ptr(counts_dev), n_steps, n_experts, budget, _ptr(sim_dev), _ptr(unique_dev),
                                      _ptr(drift_dev), _stream_ptr(stream)), ctx)


def tide_interval_costs(budget: int, n_steps: int, d: float, c_io: float, c_cpu: float, f):
    """(lat_io[tau-1], lat_cpu[tau-1]) for tau = 1..n_steps-1."""
    f = np.ascontiguousarray(f, dtype=np.float64)
    assert n_steps < 2 or f.size == n_steps - 1
    io, cpu = np.zeros(n_steps - 1), np.zeros(n_steps - 1)
    _check(lib.tide_interval_costs(budget, n_steps, d, c_io, c_cpu, _ptr(f), _ptr(io), _ptr(cpu)), None)
    return io, cpu


def tide_optimal_interval(budget: int, n_steps: int, d: float, c_io: float, c_cpu: float, f):
    """(tau, total cost) minimising lat_io + lat_cpu over tau = 1..n_steps-1."""
    f = np.ascontiguousarray(f, dtype=np.float64)
    assert n_steps < 2 or f.size == n_steps - 1
    tau, cost = C.c_int(0), C.c_double(0.0)
    _check(lib.tide_optimal_interval(budget, n_steps, d, c_io, c_cpu, _ptr(f), C.byref(tau), C.byref(cost)), None)
    return tau.value, cost.value


def tide_fit_drift(migrations: float, budget: int, n_steps: int, tau: int) -> float:
    d = C.c_double(0.0)
    _check(lib.tide_fit_drift(migrations, budget, n_steps, tau, C.byref(d)), None)
    return d.value


def tide_scale_counts(ctx, layer: int, num: int, den: int, stream=None) -> None:
    _check(lib.tide_scale_counts(ctx, layer, num, den, _stream_ptr(stream)), ctx)


def tide_commit(ctx, layer: int, stream=None) -> None:
    _check(lib.tide_commit(ctx, layer, _stream_ptr(stream)), ctx)
