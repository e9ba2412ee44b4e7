"""ctypes front end of the CPU oracle (oracle/coe_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests, by the smoke check and by the benchmark's CPU-baseline leg.
The product path never imports this module, and this module never imports the HIP library or its binding.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "coe_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
LAYER_WORDS = 12


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (OpenMP over requests).  AVX2 only, so the binary runs on any recent x86-64."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O3", "-mavx2", "-mfma", "-ffp-contract=off", "-fopenmp", "-fPIC", "-shared", "-std=c11",
               "-Wall", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


class _Arch(C.Structure):
    _fields_ = [("dtype", C.c_int32), ("in_h", C.c_int32), ("in_w", C.c_int32), ("in_c", C.c_int32),
                ("n_classes", C.c_int32), ("n_layers", C.c_int32), ("layers", C.POINTER(C.c_int32))]


def lib():
    global _lib
    if _lib is None:
        build()
        L = C.CDLL(_LIB)
        L.orc_bf16_round.restype = C.c_float
        L.orc_bf16_round.argtypes = [C.c_float]
        L.orc_cache_new.restype = C.c_void_p
        L.orc_cache_free.argtypes = [C.c_void_p]
        L.orc_cache_set_rule.argtypes = [C.c_void_p, C.c_int]
        L.orc_cache_set_in_use.argtypes = [C.c_void_p, C.c_int]
        L.orc_cache_init_fill.argtypes = [C.c_void_p, C.c_void_p]
        L.orc_cache_resident.argtypes = [C.c_void_p, C.c_void_p]
        L.orc_cache_stage.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.POINTER(C.c_int), C.c_void_p, C.c_int]
        _lib = L
    return _lib


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def bf16_round(x) -> np.ndarray:
    L = lib()
    x = np.asarray(x, dtype=np.float32)
    return np.array([L.orc_bf16_round(C.c_float(float(v))) for v in x.ravel()], dtype=np.float32).reshape(x.shape)


def conv2d(x, w, bias, res=None, stride=1, pad=0, act=0, dtype=0) -> np.ndarray:
    """x [H][W][C], w [K][R][S][C], bias [K], res [P][Q][K] or None -> y [P][Q][K] (fp32 values in storage precision)."""
    x = np.ascontiguousarray(x, np.float32); w = np.ascontiguousarray(w, np.float32)
    bias = np.ascontiguousarray(bias, np.float32)
    H, W_, Cc = x.shape; K, R, S, C2 = w.shape
    assert C2 == Cc
    P = (H + 2 * pad - R) // stride + 1; Q = (W_ + 2 * pad - S) // stride + 1
    y = np.empty((P, Q, K), np.float32)
    if res is not None:
        res = np.ascontiguousarray(res, np.float32); assert res.shape == y.shape
    lib().orc_conv2d(_p(x), H, W_, Cc, _p(w), _p(bias), _p(res), K, R, S, stride, pad, act, dtype, _p(y))
    return y


def maxpool(x, r=3, stride=2, pad=1) -> np.ndarray:
    x = np.ascontiguousarray(x, np.float32)
    H, W_, Cc = x.shape
    P = (H + 2 * pad - r) // stride + 1; Q = (W_ + 2 * pad - r) // stride + 1
    y = np.empty((P, Q, Cc), np.float32)
    lib().orc_maxpool(_p(x), H, W_, Cc, r, r, stride, pad, _p(y))
    return y


def gap_fc(x, w, b) -> np.ndarray:
    x = np.ascontiguousarray(x, np.float32); w = np.ascontiguousarray(w, np.float32); b = np.ascontiguousarray(b, np.float32)
    H, W_, Cc = x.shape
    out = np.empty(w.shape[0], np.float32)
    lib().orc_gap_fc(_p(x), H, W_, Cc, _p(w), _p(b), w.shape[0], _p(out))
    return out


def tokens(x, cls, pos, dtype=0) -> np.ndarray:
    x = np.ascontiguousarray(x, np.float32); cls = np.ascontiguousarray(cls, np.float32); pos = np.ascontiguousarray(pos, np.float32)
    T0, Cc = x.shape
    y = np.empty((T0 + 1, Cc), np.float32)
    lib().orc_tokens(_p(x), T0, Cc, _p(cls), _p(pos), dtype, _p(y))
    return y


def layernorm(x, gamma, beta, dtype=0) -> np.ndarray:
    x = np.ascontiguousarray(x, np.float32); gamma = np.ascontiguousarray(gamma, np.float32); beta = np.ascontiguousarray(beta, np.float32)
    T, Cc = x.shape
    y = np.empty((T, Cc), np.float32)
    lib().orc_layernorm(_p(x), T, Cc, _p(gamma), _p(beta), dtype, _p(y))
    return y


def attention(qkv, heads, dtype=0) -> np.ndarray:
    qkv = np.ascontiguousarray(qkv, np.float32)
    T, D3 = qkv.shape
    y = np.empty((T, D3 // 3), np.float32)
    lib().orc_attention(_p(qkv), T, D3 // 3, heads, dtype, _p(y))
    return y


def concat(a, b) -> np.ndarray:
    a = np.ascontiguousarray(a, np.float32); b = np.ascontiguousarray(b, np.float32)
    H, W_, Ca = a.shape; Cb = b.shape[2]
    assert b.shape[:2] == (H, W_)
    y = np.empty((H, W_, Ca + Cb), np.float32)
    lib().orc_concat(_p(a), _p(b), H * W_, Ca, Cb, _p(y))
    return y


def upsample2(x) -> np.ndarray:
    x = np.ascontiguousarray(x, np.float32)
    H, W_, Cc = x.shape
    y = np.empty((2 * H, 2 * W_, Cc), np.float32)
    lib().orc_upsample2(_p(x), H, W_, Cc, _p(y))
    return y


def det_head(maps, anchors: int, ncls: int) -> np.ndarray:
    """maps: list of [H][W][anchors * (5 + ncls)] arrays -> [ncls] best detection score per class."""
    ms = [np.ascontiguousarray(m, np.float32) for m in maps]
    ptrs = (C.c_void_p * len(ms))(*[m.ctypes.data for m in ms])
    hw = (C.c_int * len(ms))(*[m.shape[0] * m.shape[1] for m in ms])
    out = np.empty(ncls, np.float32)
    lib().orc_det_head(ptrs, hw, len(ms), anchors, ncls, _p(out))
    return out


def forward(arch, blob: np.ndarray, x: np.ndarray) -> np.ndarray:
    """One request through one expert.  arch: object with dtype/in_h/in_w/in_c/n_classes/layers; returns fp32 logits."""
    layers = np.ascontiguousarray(arch.layers, np.int32)
    blob = np.ascontiguousarray(blob, np.uint8)
    x = np.ascontiguousarray(x)
    out = np.zeros(arch.n_classes, np.float32)
    rc = lib().orc_forward(arch.dtype, arch.in_h, arch.in_w, arch.in_c, layers.shape[0], _p(layers), _p(blob), _p(x), _p(out))
    if rc:
        raise RuntimeError(f"orc_forward failed: {rc}")
    return out


def forward_layer(arch, blob: np.ndarray, x: np.ndarray, layer: int) -> np.ndarray:
    """Output tensor [h][w][c] of layer `layer` (not a head) of one request's forward, fp32 values in storage precision."""
    layers = np.ascontiguousarray(arch.layers, np.int32)
    blob = np.ascontiguousarray(blob, np.uint8)
    x = np.ascontiguousarray(x)
    cap = 1 << 24
    out = np.zeros(cap, np.float32)
    shape = np.zeros(3, np.int32)
    L = lib()
    L.orc_forward_layer.argtypes = [C.c_int] * 5 + [C.c_void_p] * 3 + [C.c_int, C.c_void_p, C.c_int64, C.c_void_p]
    rc = L.orc_forward_layer(arch.dtype, arch.in_h, arch.in_w, arch.in_c, layers.shape[0], _p(layers), _p(blob), _p(x), layer,
                             _p(out), cap, _p(shape))
    if rc:
        raise RuntimeError(f"orc_forward_layer failed: {rc}")
    h, w, c = (int(v) for v in shape)
    return out[:h * w * c].reshape(h, w, c).copy()


def run_chain(archs: Sequence, expert_arch: Sequence[int], blobs: Sequence[np.ndarray], succ_off, succ, inputs: np.ndarray,
              first_expert: Optional[np.ndarray], max_stages: int, max_classes: int, threads: int = 0):
    """Every request through its whole chain.  Returns dict(logits, path, all_logits, margin)."""
    L = lib()
    n_req = inputs.shape[0]
    layer_arrays = [np.ascontiguousarray(a.layers, np.int32) for a in archs]
    arr = (_Arch * len(archs))()
    for i, a in enumerate(archs):
        arr[i] = _Arch(a.dtype, a.in_h, a.in_w, a.in_c, a.n_classes, layer_arrays[i].shape[0],
                       layer_arrays[i].ctypes.data_as(C.POINTER(C.c_int32)))
    blobs = [np.ascontiguousarray(b, np.uint8) for b in blobs]
    bp = (C.c_void_p * len(blobs))(*[b.ctypes.data for b in blobs])
    ea = np.ascontiguousarray(expert_arch, np.int32)
    so = np.ascontiguousarray(succ_off, np.int32); su = np.ascontiguousarray(succ, np.int32)
    if su.size == 0:
        su = np.zeros(1, np.int32)
    inputs = np.ascontiguousarray(inputs)
    fe = None if first_expert is None else np.ascontiguousarray(first_expert, np.int32)
    logits = np.zeros((n_req, max_classes), np.float32)
    path = np.full((n_req, max_stages), -1, np.int32)
    all_logits = np.zeros((n_req, max_stages, max_classes), np.float32)
    margin = np.full((n_req, max_stages), -1, np.float32)
    rc = L.orc_run_chain(len(archs), arr, len(blobs), _p(ea), bp, _p(so), _p(su), n_req, _p(inputs), _p(fe),
                         max_stages, max_classes, _p(logits), _p(path), _p(all_logits), _p(margin), threads)
    if rc:
        raise RuntimeError(f"orc_run_chain failed: {rc}")
    return dict(logits=logits, path=path, all_logits=all_logits, margin=margin)


def threads() -> int:
    return int(lib().orc_threads())


def regroup(cur: np.ndarray, n_experts: int):
    cur = np.ascontiguousarray(cur, np.int32)
    n = cur.shape[0]
    cnt = np.zeros(n_experts, np.int32); off = np.zeros(n_experts + 1, np.int32)
    perm = np.full(max(n, 1), -1, np.int32); inv = np.full(max(n, 1), -1, np.int32)
    m = lib().orc_regroup(_p(cur), n, n_experts, _p(cnt), _p(off), _p(perm), _p(inv))
    return dict(n_pending=m, cnt=cnt, off=off, perm=perm[:m], inv=inv[:n])


def split(off: np.ndarray, order: Sequence[int], max_batch: int) -> np.ndarray:
    off = np.ascontiguousarray(off, np.int32); order = np.ascontiguousarray(order, np.int32)
    cap = int(off[-1]) + len(order) + 1
    chunks = np.zeros((cap, 3), np.int32)
    n = lib().orc_split(_p(off), len(order), _p(order), max_batch, _p(chunks), cap)
    assert n >= 0
    return chunks[:n]


class CacheSim:
    """Replay of the expert-cache policy: initial fill, then one call per stage."""

    def __init__(self, nbytes: Sequence[int], prob: Sequence[float], succ_off, succ, cap_experts: int = 0, cap_bytes: int = 0,
                 rule: int = 0, in_use: int = 0):
        self.E = len(nbytes)
        self._bytes = np.ascontiguousarray(nbytes, np.int64); self._prob = np.ascontiguousarray(prob, np.float32)
        self._so = np.ascontiguousarray(succ_off, np.int32); self._su = np.ascontiguousarray(succ, np.int32)
        if self._su.size == 0:
            self._su = np.zeros(1, np.int32)
        L = lib()
        L.orc_cache_new.argtypes = [C.c_int, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_int64]
        self._h = L.orc_cache_new(self.E, _p(self._bytes), _p(self._prob), _p(self._so), _p(self._su), cap_experts, cap_bytes)
        if L.orc_cache_set_rule(self._h, rule):          # 0 two-stage, 1 least recently used, 2 first in first out
            raise ValueError("unknown replacement rule")
        if L.orc_cache_set_in_use(self._h, in_use):      # experts of this many preceding groups are busy during a load
            raise ValueError("negative depth")

    def __del__(self):
        if getattr(self, "_h", None):
            lib().orc_cache_free(self._h); self._h = None

    def init_fill(self) -> List[int]:
        out = np.zeros(self.E, np.int32)
        n = lib().orc_cache_init_fill(self._h, _p(out))
        return [int(v) for v in out[:n]]

    def resident(self) -> np.ndarray:
        out = np.zeros(self.E, np.uint8)
        lib().orc_cache_resident(self._h, _p(out))
        return out.astype(bool)

    def stage(self, has_group: Sequence[bool]):
        """Returns (order, switches) with switches = [(expert, [victims...]), ...]; raises MemoryError if it cannot fit."""
        hg = np.ascontiguousarray(np.asarray(has_group, dtype=np.uint8))
        order = np.zeros(self.E, np.int32); n_order = C.c_int(0)
        cap = 4 * self.E * self.E + 16
        log = np.zeros(cap, np.int32)
        nl = lib().orc_cache_stage(self._h, _p(hg), _p(order), C.byref(n_order), _p(log), cap)
        if nl < 0:
            raise MemoryError("expert does not fit")
        sw = []; i = 0
        while i < nl:
            e, nv = int(log[i]), int(log[i + 1])
            sw.append((e, [int(v) for v in log[i + 2:i + 2 + nv]])); i += 2 + nv
        return [int(v) for v in order[:n_order.value]], sw


class TieredCacheSim:
    """Replay of two cache levels (Section 1: experts are offloaded to CPU memory or SSD; Section 5.1: CPU memory as a cache in
    front of the SSD).  The reading: the lower level is a cache of the same kind whose requests are the upper level's loads,
    one at a time in the order they are issued; each level applies the replacement rule to its own residency; the lower
    level's initial fill (Section 4.1, descending usage probability) precedes the upper one's."""

    def __init__(self, nbytes, prob, succ_off, succ, cap_device: int, cap_host: int, rule: int = 0, in_use: int = 0):
        self.E = len(nbytes)
        self.dev = CacheSim(nbytes, prob, succ_off, succ, cap_experts=cap_device, rule=rule, in_use=in_use)
        self.host = CacheSim(nbytes, prob, succ_off, succ, cap_experts=cap_host, rule=rule)

    def _serve(self, e: int):
        need = np.zeros(self.E, np.uint8)
        need[e] = 1
        return self.host.stage(need)[1]

    def init_fill(self):
        """Returns (experts loaded to the device, reads of the lower level as [(expert, victims)])."""
        reads = [(e, []) for e in self.host.init_fill()]
        loaded = self.dev.init_fill()
        for e in loaded:
            reads += self._serve(e)
        return loaded, reads

    def stage(self, has_group):
        """Returns (order, device switches, reads of the lower level)."""
        order, sw = self.dev.stage(has_group)
        reads = []
        for e, _ in sw:
            reads += self._serve(e)
        return order, sw, reads
