"""ctypes binding of libcoe.so: argument marshalling only, same names as the C ABI in include/coe.h.

Every step of the hot path runs inside the library's HIP kernels.  There is no fallback: importing this module
without a built library raises, and creating a context without a GPU fails with COE_EDEVICE.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libcoe.so")

COE_OK, COE_DONE = 0, 1
COE_EINVAL, COE_ENOMEM, COE_ESTATE, COE_EGRAPH, COE_EDEVICE, COE_ERANGE, COE_EIO = -1, -2, -3, -4, -5, -6, -7
K_REGROUP_INDEX, K_REGROUP_GATHER, K_CONV_MFMA, K_CONV_DIRECT, K_POOL, K_HEAD, K_SWITCH, K_CONV_STEM = range(8)
KERNEL_CLASS_NAMES = ["regroup_index", "regroup_gather", "conv_mfma", "conv_direct", "pool", "head", "switch", "conv_stem", "attention", "token_ops", "conv_slab", "switch_wait"]

EXPORTS = [
    "coe_create", "coe_destroy", "coe_last_error", "coe_register_arch", "coe_arch_blob_bytes", "coe_register_expert",
    "coe_set_dependency_graph", "coe_submit", "coe_step", "coe_sync", "coe_collect", "coe_reset_requests",
    "coe_debug_last_regroup", "coe_debug_switch_log", "coe_debug_resident", "coe_debug_forward", "coe_debug_layer_output", "coe_debug_regroup", "coe_debug_conv",
    "coe_profile_read", "coe_profile_issued", "coe_validate_graph", "coe_policy_create", "coe_policy_destroy", "coe_policy_init_fill",
    "coe_policy_stage", "coe_policy_resident", "coe_policy_set_eviction", "coe_policy_set_in_use_depth", "coe_set_arranging", "coe_arrange_defer", "coe_set_latency_model", "coe_assign_executors", "coe_debug_last_assignment",
    "coe_regroup_static", "coe_debug_last_chunks", "coe_set_host_tier", "coe_debug_host_log", "coe_profiler_memory_scores", "coe_profiler_expert_budget", "coe_profiler_executable_batch", "coe_profiler_usage_probabilities",
    "coe_profiler_fit_latency", "coe_profiler_max_batch", "coe_profiler_arranging_window", "coe_profiler_window_step",
]


class coe_layer(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("op", "src", "dst", "res", "k", "r", "s", "stride", "pad", "act", "aux0", "aux1")]


class coe_arch_desc(C.Structure):
    _fields_ = [("dtype", C.c_int32), ("in_h", C.c_int32), ("in_w", C.c_int32), ("in_c", C.c_int32),
                ("n_classes", C.c_int32), ("n_layers", C.c_int32), ("layers", C.POINTER(coe_layer))]


class coe_config(C.Structure):
    _fields_ = [("device", C.c_int32), ("max_requests", C.c_int32), ("max_batch", C.c_int32), ("max_stages", C.c_int32),
                ("cache_cap_experts", C.c_int32), ("profile", C.c_int32), ("cache_cap_bytes", C.c_int64),
                ("compute_stream", C.c_void_p), ("copy_stream", C.c_void_p), ("group_small", C.c_int32), ("eviction", C.c_int32), ("prefetch_depth", C.c_int32), ("executors", C.c_int32)]


class coe_step_stats(C.Structure):
    _fields_ = [("n_pending", C.c_int32), ("n_groups", C.c_int32), ("n_chunks", C.c_int32), ("n_hits", C.c_int32),
                ("n_misses", C.c_int32), ("n_evictions", C.c_int32), ("bytes_switched", C.c_int64),
                ("host_plan_us", C.c_double), ("n_grouped", C.c_int32), ("n_group_sets", C.c_int32),
                ("n_deferred_groups", C.c_int32), ("n_deferred_requests", C.c_int32), ("n_executors_used", C.c_int32),
                ("n_device_allocs", C.c_int32), ("n_host_misses", C.c_int32), ("bytes_read", C.c_int64),
                ("read_us", C.c_double)]


class coe_window_state(C.Structure):
    _fields_ = [("status", C.c_int32), ("n_next", C.c_int32), ("window_low", C.c_double), ("window_high", C.c_double),
                ("n_low", C.c_int32), ("n_high", C.c_int32), ("linear_error", C.c_double)]


COE_WINDOW_MEASURE, COE_WINDOW_SHORTFALL, COE_WINDOW_END = 0, 1, 2


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2503_02354_amd.build` "
                          "(there is no CPU fallback)")
    L = C.CDLL(LIB_PATH)
    vp, i32, i64 = C.c_void_p, C.c_int32, C.c_int64
    L.coe_create.argtypes = [C.POINTER(coe_config), C.POINTER(vp)]
    L.coe_destroy.argtypes = [vp]; L.coe_destroy.restype = None
    L.coe_last_error.argtypes = [vp]; L.coe_last_error.restype = C.c_char_p
    L.coe_register_arch.argtypes = [vp, C.POINTER(coe_arch_desc), C.POINTER(i32)]
    L.coe_arch_blob_bytes.argtypes = [vp, i32]; L.coe_arch_blob_bytes.restype = i64
    L.coe_register_expert.argtypes = [vp, i32, i32, vp, C.c_size_t, C.c_float]
    L.coe_set_dependency_graph.argtypes = [vp, i32, vp, vp]
    L.coe_submit.argtypes = [vp, i32, vp, C.c_int, vp, C.POINTER(i64)]
    L.coe_step.argtypes = [vp, C.POINTER(coe_step_stats)]
    L.coe_sync.argtypes = [vp]
    L.coe_collect.argtypes = [vp, i32, vp, vp, vp, C.POINTER(i32)]
    L.coe_reset_requests.argtypes = [vp]
    L.coe_debug_last_regroup.argtypes = [vp, C.POINTER(i32), C.POINTER(i32), vp, vp, vp, vp, i32]
    L.coe_debug_switch_log.argtypes = [vp, i32, vp, C.POINTER(i32)]
    L.coe_debug_resident.argtypes = [vp, vp]
    L.coe_set_host_tier.argtypes = [vp, i32, C.c_char_p]
    L.coe_debug_host_log.argtypes = [vp, i32, vp, C.POINTER(i32)]
    L.coe_debug_forward.argtypes = [vp, i32, i32, vp, vp]
    L.coe_debug_layer_output.argtypes = [vp, i32, i32, vp, i32, vp, C.c_size_t]
    L.coe_debug_regroup.argtypes = [vp, i32, vp, i32, vp, vp, vp, vp]
    L.coe_debug_conv.argtypes = [vp, i32, vp, vp, vp, vp, vp] + [i32] * 11 + [C.POINTER(i32)]
    L.coe_profile_read.argtypes = [vp, i32, C.POINTER(i64), C.POINTER(C.c_double), C.POINTER(C.c_double)]
    L.coe_profile_issued.argtypes = [vp, i32, C.POINTER(i64)]
    L.coe_validate_graph.argtypes = [i32, vp, vp, vp]
    L.coe_policy_create.argtypes = [i32, vp, vp, vp, vp, i32, i64]; L.coe_policy_create.restype = vp
    L.coe_policy_destroy.argtypes = [vp]; L.coe_policy_destroy.restype = None
    L.coe_policy_init_fill.argtypes = [vp, vp]
    L.coe_policy_stage.argtypes = [vp, vp, vp, C.POINTER(i32), vp, i32]
    L.coe_policy_resident.argtypes = [vp, vp]
    L.coe_policy_set_eviction.argtypes = [vp, i32]
    L.coe_policy_set_in_use_depth.argtypes = [vp, i32]
    L.coe_set_arranging.argtypes = [vp, i32, i32, i32, i32]
    L.coe_set_latency_model.argtypes = [vp, i32, C.c_int64, C.c_int64, C.c_int64]
    L.coe_assign_executors.argtypes = [i32, vp, i32, vp]
    L.coe_debug_last_assignment.argtypes = [vp, i32, vp, vp, vp, C.POINTER(i32)]
    L.coe_arrange_defer.argtypes = [i32, vp, vp, vp, vp, vp, vp, vp]
    L.coe_debug_last_chunks.argtypes = [vp, i32, vp, C.POINTER(i32)]
    L.coe_profiler_fit_latency.argtypes = [i32, vp, vp, C.POINTER(C.c_double), C.POINTER(C.c_double)]
    L.coe_profiler_max_batch.argtypes = [i32, vp, vp, C.c_double, C.POINTER(i32)]
    L.coe_profiler_arranging_window.argtypes = [C.c_double, C.c_double, C.c_double, C.c_double, C.POINTER(i32), C.POINTER(i32)]
    L.coe_profiler_memory_scores.argtypes = [i32, vp, vp, C.POINTER(i64)]
    L.coe_profiler_expert_budget.argtypes = [i64, i64, i64, i32, i64, C.POINTER(i64), C.POINTER(C.c_double)]
    L.coe_profiler_executable_batch.argtypes = [i64, i64, i32, C.POINTER(i32)]
    L.coe_profiler_usage_probabilities.argtypes = [i32, i32, vp, i32, vp]
    L.coe_profiler_window_step.argtypes = [i32, C.c_double, C.c_double, i32, i32, vp, C.POINTER(coe_window_state)]
    L.coe_regroup_static.argtypes = [i32, vp, i32, vp, vp, vp, vp, vp]
    return L


lib = _load()


class CoEError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"coe error {code}: {msg}")
        self.code = code


def _ptr(a):
    if a is None:
        return None
    if isinstance(a, np.ndarray):
        return a.ctypes.data_as(C.c_void_p)
    return C.c_void_p(int(a))


def coe_regroup_static(n: int, cur: int, n_experts: int, cnt: int, off: int, perm: int, inv: int, stream: int = 0) -> None:
    """Regroup on device arrays (integer device addresses) without any allocation; enqueued on `stream`."""
    rc = lib.coe_regroup_static(n, _ptr(cur or None), n_experts, _ptr(cnt or None), _ptr(off or None), _ptr(perm or None),
                                _ptr(inv or None), C.c_void_p(stream or None))
    if rc < 0:
        raise CoEError(rc, lib.coe_last_error(None).decode())


def coe_profiler_fit_latency(batch, latency_us) -> Tuple[float, float]:
    b = np.ascontiguousarray(batch, np.int32); t = np.ascontiguousarray(latency_us, np.float64)
    assert b.shape == t.shape and b.ndim == 1
    k, c = C.c_double(0), C.c_double(0)
    rc = lib.coe_profiler_fit_latency(b.shape[0], _ptr(b), _ptr(t), C.byref(k), C.byref(c))
    if rc < 0:
        raise CoEError(rc, "coe_profiler_fit_latency")
    return k.value, c.value


def coe_profiler_max_batch(batch, latency_us, tol: float = 0.05) -> int:
    b = np.ascontiguousarray(batch, np.int32); t = np.ascontiguousarray(latency_us, np.float64)
    assert b.shape == t.shape and b.ndim == 1
    out = C.c_int32(0)
    rc = lib.coe_profiler_max_batch(b.shape[0], _ptr(b), _ptr(t), tol, C.byref(out))
    if rc < 0:
        raise CoEError(rc, "coe_profiler_max_batch")
    return out.value


def coe_profiler_arranging_window(k_us: float, b_us: float, load_us: float, efficiency: float) -> Tuple[int, int]:
    a, b = C.c_int32(0), C.c_int32(0)
    rc = lib.coe_profiler_arranging_window(k_us, b_us, load_us, efficiency, C.byref(a), C.byref(b))
    if rc < 0:
        raise CoEError(rc, "coe_profiler_arranging_window")
    return a.value, b.value


def coe_profiler_memory_scores(nbytes) -> Tuple[np.ndarray, int]:
    b = np.ascontiguousarray(nbytes, np.int64)
    score = np.zeros(b.shape[0], np.float64)
    unit = C.c_int64(0)
    rc = lib.coe_profiler_memory_scores(b.shape[0], _ptr(b) if b.shape[0] else None, _ptr(score) if b.shape[0] else None, C.byref(unit))
    if rc < 0:
        raise CoEError(rc, "coe_profiler_memory_scores")
    return score, unit.value


def coe_profiler_expert_budget(total_bytes: int, reserve_bytes: int, bytes_per_request: int, max_batch: int, unit_bytes: int) -> Tuple[int, float]:
    left, scores = C.c_int64(0), C.c_double(0.0)
    rc = lib.coe_profiler_expert_budget(total_bytes, reserve_bytes, bytes_per_request, max_batch, unit_bytes, C.byref(left), C.byref(scores))
    if rc < 0:
        raise CoEError(rc, "coe_profiler_expert_budget")
    return left.value, scores.value


def coe_profiler_usage_probabilities(path, n_experts: int) -> np.ndarray:
    p = np.ascontiguousarray(path, np.int32)
    assert p.ndim == 2
    prob = np.zeros(max(n_experts, 1), np.float32)
    rc = lib.coe_profiler_usage_probabilities(p.shape[0], p.shape[1], _ptr(p) if p.size else None, n_experts, _ptr(prob))
    if rc < 0:
        raise CoEError(rc, "coe_profiler_usage_probabilities")
    return prob[:n_experts]


def coe_profiler_executable_batch(free_bytes: int, bytes_per_request: int, profiled_max_batch: int) -> int:
    out = C.c_int32(0)
    rc = lib.coe_profiler_executable_batch(free_bytes, bytes_per_request, profiled_max_batch, C.byref(out))
    if rc < 0:
        raise CoEError(rc, "coe_profiler_executable_batch")
    return out.value


def coe_profiler_window_step(n_experts_total: int, initial_window: float, error_margin: float, fit_points: int, throughput) -> coe_window_state:
    t = np.ascontiguousarray(throughput, np.float64)
    st = coe_window_state()
    rc = lib.coe_profiler_window_step(n_experts_total, initial_window, error_margin, fit_points, t.shape[0],
                                      _ptr(t) if t.shape[0] else None, C.byref(st))
    if rc < 0:
        raise CoEError(rc, "coe_profiler_window_step")
    return st


# ---- host-only functions --------------------------------------------------------------------------------------
def coe_arrange_defer(count, age, resident, min_group_resident, min_group_missing, max_wait_steps) -> np.ndarray:
    """The arranging window's rule (host only): which queued groups stay queued in this step."""
    a = [np.ascontiguousarray(v, np.int32) for v in (count, age, min_group_resident, min_group_missing, max_wait_steps)]
    res = np.ascontiguousarray(np.asarray(resident, dtype=np.uint8))
    n = a[0].shape[0]
    assert all(v.shape == (n,) for v in a) and res.shape == (n,)
    out = np.zeros(n, np.uint8)
    rc = lib.coe_arrange_defer(n, _ptr(a[0]), _ptr(a[1]), _ptr(res), _ptr(a[2]), _ptr(a[3]), _ptr(a[4]), _ptr(out))
    if rc < 0:
        raise CoEError(rc, "coe_arrange_defer")
    return out.astype(bool)


def coe_assign_executors(cost_ns, n_executors: int) -> np.ndarray:
    """The executor assignment rule (host only): which executor every unit goes to, in order."""
    cost = np.ascontiguousarray(cost_ns, np.int64)
    out = np.zeros(cost.shape[0], np.int32)
    rc = lib.coe_assign_executors(cost.shape[0], _ptr(cost), n_executors, _ptr(out))
    if rc < 0:
        raise CoEError(rc, "coe_assign_executors")
    return out


def coe_validate_graph(n_experts: int, succ_off, succ, n_classes=None) -> int:
    so = np.ascontiguousarray(succ_off, np.int32); su = np.ascontiguousarray(succ, np.int32)
    nc = None if n_classes is None else np.ascontiguousarray(n_classes, np.int32)
    return int(lib.coe_validate_graph(n_experts, _ptr(so), _ptr(su) if su.size else None, _ptr(nc)))


class Policy:
    """coe_policy_* : the library's cache policy without a device."""

    def __init__(self, nbytes, prob, succ_off, succ, cap_experts=0, cap_bytes=0, eviction=0, in_use_depth=0):
        self.E = len(nbytes)
        b = np.ascontiguousarray(nbytes, np.int64); p = np.ascontiguousarray(prob, np.float32)
        so = np.ascontiguousarray(succ_off, np.int32); su = np.ascontiguousarray(succ, np.int32)
        if su.size == 0:
            su = np.zeros(1, np.int32)
        self._h = lib.coe_policy_create(self.E, _ptr(b), _ptr(p), _ptr(so), _ptr(su), cap_experts, cap_bytes)
        if not self._h:
            raise CoEError(COE_EINVAL, "coe_policy_create failed")
        rc = lib.coe_policy_set_eviction(self._h, eviction) or lib.coe_policy_set_in_use_depth(self._h, in_use_depth)
        if rc:
            raise CoEError(rc, "coe_policy_set_eviction / coe_policy_set_in_use_depth")

    def __del__(self):
        if getattr(self, "_h", None):
            lib.coe_policy_destroy(self._h); self._h = None

    def init_fill(self) -> List[int]:
        out = np.zeros(self.E, np.int32)
        n = lib.coe_policy_init_fill(self._h, _ptr(out))
        return [int(v) for v in out[:n]]

    def stage(self, has_group):
        hg = np.ascontiguousarray(np.asarray(has_group, dtype=np.uint8))
        order = np.zeros(self.E, np.int32); n_order = C.c_int32(0)
        cap = 4 * self.E * self.E + 16
        log = np.zeros(cap, np.int32)
        nl = lib.coe_policy_stage(self._h, _ptr(hg), _ptr(order), C.byref(n_order), _ptr(log), cap)
        if nl == COE_ENOMEM:
            raise MemoryError("expert does not fit")
        if nl < 0:
            raise CoEError(nl, "coe_policy_stage")
        return [int(v) for v in order[:n_order.value]], parse_switch_log(log[:nl])

    def resident(self) -> np.ndarray:
        out = np.zeros(self.E, np.uint8)
        lib.coe_policy_resident(self._h, _ptr(out))
        return out.astype(bool)


def parse_switch_log(log) -> List[Tuple[int, List[int]]]:
    sw = []; i = 0
    while i < len(log):
        e, nv = int(log[i]), int(log[i + 1])
        sw.append((e, [int(v) for v in log[i + 2:i + 2 + nv]])); i += 2 + nv
    return sw


# ---- device context -----------------------------------------------------------------------------------------------
class Context:
    """One coe_ctx.  Methods are the C entry points with numpy / raw-pointer marshalling."""

    def __init__(self, max_requests: int, max_stages: int = 2, max_batch: int = 0, cache_cap_experts: int = 0,
                 cache_cap_bytes: int = 0, device: int = 0, profile: bool = False, compute_stream: int = 0,
                 copy_stream: int = 0, group_small: int = 0, eviction: int = 0, prefetch_depth: int = 0, executors: int = 0):
        cfg = coe_config(device, max_requests, max_batch, max_stages, cache_cap_experts, int(profile), cache_cap_bytes,
                         compute_stream or None, copy_stream or None, group_small, eviction, prefetch_depth, executors)
        h = C.c_void_p()
        rc = lib.coe_create(C.byref(cfg), C.byref(h))
        if rc != COE_OK:
            raise CoEError(rc, "coe_create failed (no usable GPU?)" if rc == COE_EDEVICE else "coe_create failed")
        self._h = h
        self.max_stages = max_stages
        self.max_classes = 0
        self._arch_classes: List[int] = []
        self._in_bytes = 0
        self.n_experts = 0

    def close(self):
        if getattr(self, "_h", None):
            lib.coe_destroy(self._h); self._h = None

    def __del__(self):
        self.close()

    def _chk(self, rc: int) -> int:
        if rc < 0:
            raise CoEError(rc, lib.coe_last_error(self._h).decode())
        return rc

    def coe_register_arch(self, arch) -> int:
        layers = np.ascontiguousarray(arch.layers, np.int32)
        d = coe_arch_desc(arch.dtype, arch.in_h, arch.in_w, arch.in_c, arch.n_classes, layers.shape[0],
                          layers.ctypes.data_as(C.POINTER(coe_layer)))
        aid = C.c_int32(-1)
        self._chk(lib.coe_register_arch(self._h, C.byref(d), C.byref(aid)))
        self.max_classes = max(self.max_classes, arch.n_classes)
        self._arch_classes.append(arch.n_classes)
        self._in_bytes = arch.in_h * arch.in_w * arch.in_c * (2 if arch.dtype == 1 else 4)
        return aid.value

    def coe_arch_blob_bytes(self, arch_id: int) -> int:
        return int(self._chk(lib.coe_arch_blob_bytes(self._h, arch_id)))

    def coe_register_expert(self, expert_id: int, arch_id: int, blob: np.ndarray, usage_prob: float):
        blob = np.ascontiguousarray(blob, np.uint8)
        self._chk(lib.coe_register_expert(self._h, expert_id, arch_id, _ptr(blob), blob.nbytes, usage_prob))
        self._expert_arch = getattr(self, "_expert_arch", {})
        self._expert_arch[expert_id] = arch_id

    def coe_set_dependency_graph(self, succ_off, succ):
        so = np.ascontiguousarray(succ_off, np.int32); su = np.ascontiguousarray(succ, np.int32)
        if su.size == 0:
            su = np.zeros(1, np.int32)
        self.n_experts = len(so) - 1
        self._chk(lib.coe_set_dependency_graph(self._h, self.n_experts, _ptr(so), _ptr(su)))

    def coe_submit(self, n: int, inputs, on_device: bool, first_expert: Optional[np.ndarray] = None) -> int:
        """inputs: numpy array (host) or an integer device address."""
        fe = None if first_expert is None else np.ascontiguousarray(first_expert, np.int32)
        if isinstance(inputs, np.ndarray):
            inputs = np.ascontiguousarray(inputs)
            assert not on_device and (self._in_bytes == 0 or inputs.nbytes == n * self._in_bytes)
        rid = C.c_int64(-1)
        self._chk(lib.coe_submit(self._h, n, _ptr(inputs), 1 if on_device else 0, _ptr(fe), C.byref(rid)))
        return rid.value

    def coe_step(self) -> Tuple[int, coe_step_stats]:
        st = coe_step_stats()
        rc = self._chk(lib.coe_step(self._h, C.byref(st)))
        return rc, st

    def coe_sync(self):
        self._chk(lib.coe_sync(self._h))

    def coe_set_arranging(self, arch_id: int, min_group_resident: int, min_group_missing: int, max_wait_steps: int):
        self._chk(lib.coe_set_arranging(self._h, arch_id, min_group_resident, min_group_missing, max_wait_steps))

    def coe_set_latency_model(self, arch_id: int, k_ns: int, b_ns: int, load_ns: int):
        self._chk(lib.coe_set_latency_model(self._h, arch_id, int(k_ns), int(b_ns), int(load_ns)))

    def coe_debug_last_assignment(self, cap: int = 4096):
        fe = np.zeros(cap, np.int32); cost = np.zeros(cap, np.int64); ex = np.zeros(cap, np.int32); n = C.c_int32(0)
        self._chk(lib.coe_debug_last_assignment(self._h, cap, _ptr(fe), _ptr(cost), _ptr(ex), C.byref(n)))
        m = min(n.value, cap)
        return fe[:m], cost[:m], ex[:m]

    def coe_debug_last_chunks(self, cap: int = 65536) -> np.ndarray:
        """[n][3] int32: {expert, first row in the regrouped order, requests} of every batch of the last step."""
        out = np.zeros((cap, 3), np.int32); n = C.c_int32(0)
        self._chk(lib.coe_debug_last_chunks(self._h, cap, _ptr(out), C.byref(n)))
        return out[:min(n.value, cap)]

    def coe_collect(self, cap: int):
        ids = np.zeros(cap, np.int64); logits = np.zeros((cap, max(self.max_classes, 1)), np.float32)
        path = np.full((cap, self.max_stages), -1, np.int32); n = C.c_int32(0)
        self._chk(lib.coe_collect(self._h, cap, _ptr(ids), _ptr(logits), _ptr(path), C.byref(n)))
        return ids[:n.value], logits[:n.value], path[:n.value]

    def coe_reset_requests(self):
        self._chk(lib.coe_reset_requests(self._h))

    def coe_debug_last_regroup(self, max_requests: int):
        npend, nlive = C.c_int32(0), C.c_int32(0)
        E = self.n_experts
        cnt = np.zeros(E, np.int32); off = np.zeros(E + 1, np.int32)
        perm = np.full(max_requests, -1, np.int32); inv = np.full(max_requests, -1, np.int32)
        self._chk(lib.coe_debug_last_regroup(self._h, C.byref(npend), C.byref(nlive), _ptr(cnt), _ptr(off), _ptr(perm), _ptr(inv),
                                             max_requests))
        return dict(n_pending=npend.value, n_live=nlive.value, cnt=cnt, off=off, perm=perm[:npend.value], inv=inv[:nlive.value])

    def coe_debug_switch_log(self):
        n = C.c_int32(0)
        self._chk(lib.coe_debug_switch_log(self._h, 0, None, C.byref(n)))
        log = np.zeros(max(n.value, 1), np.int32)
        self._chk(lib.coe_debug_switch_log(self._h, n.value, _ptr(log), C.byref(n)))
        return parse_switch_log(log[:n.value])

    def coe_set_host_tier(self, host_cap_experts: int, backing_path: str):
        self._chk(lib.coe_set_host_tier(self._h, host_cap_experts, os.fsencode(backing_path)))

    def coe_debug_host_log(self):
        n = C.c_int32(0)
        self._chk(lib.coe_debug_host_log(self._h, 0, None, C.byref(n)))
        log = np.zeros(max(n.value, 1), np.int32)
        self._chk(lib.coe_debug_host_log(self._h, n.value, _ptr(log), C.byref(n)))
        return parse_switch_log(log[:n.value])

    def coe_debug_resident(self) -> np.ndarray:
        out = np.zeros(max(self.n_experts, 1), np.uint8)
        self._chk(lib.coe_debug_resident(self._h, _ptr(out)))
        return out[:self.n_experts].astype(bool)

    def coe_debug_forward(self, expert_id: int, n: int, device_inputs: int) -> np.ndarray:
        ncls = self._arch_classes[self._expert_arch[expert_id]]
        out = np.zeros((n, ncls), np.float32)
        self._chk(lib.coe_debug_forward(self._h, expert_id, n, C.c_void_p(int(device_inputs)), _ptr(out)))
        return out

    def coe_debug_layer_output(self, expert_id: int, n: int, device_inputs: int, layer: int, shape, dtype) -> np.ndarray:
        """Output tensor of one layer, shape (n, p, q, k), dtype np.uint16 (bf16 bits) or np.float32."""
        out = np.zeros(shape, dtype)
        self._chk(lib.coe_debug_layer_output(self._h, expert_id, n, C.c_void_p(int(device_inputs)), layer, _ptr(out), out.nbytes))
        return out

    def coe_debug_regroup(self, cur: np.ndarray, n_experts: int):
        cur = np.ascontiguousarray(cur, np.int32); n = cur.shape[0]
        cnt = np.zeros(n_experts, np.int32); off = np.zeros(n_experts + 1, np.int32)
        perm = np.full(max(n, 1), -1, np.int32); inv = np.full(max(n, 1), -1, np.int32)
        m = self._chk(lib.coe_debug_regroup(self._h, n, _ptr(cur), n_experts, _ptr(cnt), _ptr(off), _ptr(perm), _ptr(inv)))
        return dict(n_pending=m, cnt=cnt, off=off, perm=perm[:m], inv=inv[:n])

    def coe_debug_conv(self, dtype: int, x: np.ndarray, w: np.ndarray, bias: np.ndarray, res: Optional[np.ndarray], stride: int,
                       pad: int, act: int, repeat: int = 1):
        """x [n][h][w][c], w [k][r][s][c] (uint16 bf16 bits or float32), bias float32 -> (y, kernel class)."""
        x = np.ascontiguousarray(x); w = np.ascontiguousarray(w); bias = np.ascontiguousarray(bias, np.float32)
        n, h, wd, c = x.shape; k, r, s, c2 = w.shape
        assert c2 == c and x.dtype == w.dtype
        p = (h + 2 * pad - r) // stride + 1; q = (wd + 2 * pad - s) // stride + 1
        y = np.zeros((n, p, q, k), x.dtype)
        if res is not None:
            res = np.ascontiguousarray(res); assert res.shape == y.shape and res.dtype == x.dtype
        cls = C.c_int32(-1)
        self._chk(lib.coe_debug_conv(self._h, dtype, _ptr(x), _ptr(w), _ptr(bias), _ptr(res), _ptr(y), n, h, wd, c, k, r, s, stride,
                                     pad, act, repeat, C.byref(cls)))
        return y, cls.value

    def coe_profile_read(self, kernel_class: int):
        n = C.c_int64(0); ms = C.c_double(0); work = C.c_double(0)
        self._chk(lib.coe_profile_read(self._h, kernel_class, C.byref(n), C.byref(ms), C.byref(work)))
        return n.value, ms.value, work.value

    def coe_profile_issued(self, kernel_class: int) -> int:
        n = C.c_int64(0)
        self._chk(lib.coe_profile_issued(self._h, kernel_class, C.byref(n)))
        return n.value


def setup_workload(ctx: Context, wl, blobs: Optional[Sequence[np.ndarray]] = None):
    """Register a workload's architectures, experts and graph on a context (marshalling helper)."""
    ids = [ctx.coe_register_arch(a) for a in wl.archs]
    for e in range(wl.graph.n_experts):
        blob = wl.blob(e) if blobs is None else blobs[e]
        ctx.coe_register_expert(e, ids[wl.expert_arch[e]], blob, float(wl.usage_prob[e]))
    ctx.coe_set_dependency_graph(wl.graph.succ_off, wl.graph.succ)
