"""Seeded synthetic CoE workloads: architecture descriptors, expert weight blobs,
dependency graphs and request images.

This package is pure data generation and belongs to neither the HIP library nor
the CPU oracle; both are fed from it and it imports neither.  It holds no
convolution, routing, regroup or cache arithmetic: it only describes expert
architectures as flat layer lists, draws random numbers from counter-based
Philox streams and lays tensors out in the canonical weight-blob format that
both sides consume.  Head-bias calibration files written by the oracle-side
script live next to it in calib/ and are read by both sides as inputs.

CoE structure follows the paper's Section 2.1: a routing rule picks a first
expert, an expert's output either selects the next expert or is the final
result, and several upstream experts may share one downstream expert.  The
paper's own experts (ResNet101 / YOLOv5 on a private circuit-board dataset) are
not available, so every workload here is a synthetic stand-in of the same
structure.

Canonical formats
-----------------
Layer descriptor: 12 int32 words
    [op, src, dst, res, k, r, s, stride, pad, act, aux0, aux1]
    op   1 = CONV      y = act(conv(x) + bias (+ res))         NHWC, weights [K][R][S][C]
         2 = MAXPOOL   r x s window, stride, pad (padding never wins the max)
         3 = HEAD      global average pool over H*W, then FC to k logits
         4 = TOKENS    prepend a class token to the H*W tokens and add a
                       position embedding; weights cls[C], pos[(H*W+1)][C]
         5 = LAYERNORM over channels; weights gamma[C], beta[C] (fp32), eps 1e-6
         6 = ATTENTION src holds [T][3*D] (q | k | v), aux0 = heads; softmax(q k^T / sqrt(dh)) v
         7 = HEAD_CLS  layer norm of token 0 then FC to k logits
         8 = CONCAT    dst = [src | res] along channels (same height and width)
         9 = UPSAMPLE  nearest neighbour, factor 2
        10 = HEAD_DET  src (and res, if >= 0) are detection maps with aux0 anchors x (5 + k) channels per position:
                       logits[c] = max over maps, positions, anchors of sigmoid(objectness) * sigmoid(class c); no weights
    src/dst/res are activation buffer ids (0 = the request's input, res -1 = none)
    act  0 none, 1 ReLU, 2 GELU (erf form), 3 SiLU
Architecture header: dtype (0 fp32, 1 bf16), in_h, in_w, in_c, n_classes.
Weight blob: tensors in layer order, every tensor at a 256-byte aligned offset.
    CONV   W[K][R][S][C] in the arch dtype, then bias[K] fp32
    HEAD   W[k][F] in the arch dtype, then bias[k] fp32
    TOKENS cls[C] dtype, pos[T][C] dtype
    LAYERNORM gamma[C] fp32, beta[C] fp32
    HEAD_CLS gamma[C] fp32, beta[C] fp32, W[k][C] dtype, bias[k] fp32
"""
from __future__ import annotations

import dataclasses
import json
import math
import os
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

OP_CONV, OP_MAXPOOL, OP_HEAD, OP_TOKENS, OP_LAYERNORM, OP_ATTENTION, OP_HEAD_CLS = 1, 2, 3, 4, 5, 6, 7
OP_CONCAT, OP_UPSAMPLE, OP_HEAD_DET = 8, 9, 10
ACT_NONE, ACT_RELU, ACT_GELU, ACT_SILU = 0, 1, 2, 3
DT_F32, DT_BF16 = 0, 1
LAYER_WORDS = 12
BLOB_ALIGN = 256


# ----------------------------------------------------------------------------
# bf16 quantisation of generated data (input generation only)
# ----------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bfloat16 (ties to even); returns uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = u + np.uint32(0x7FFF) + lsb
    return (r >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


# ----------------------------------------------------------------------------
# counter-based random streams
# ----------------------------------------------------------------------------
_KIND_WEIGHT, _KIND_INPUT, _KIND_MISC = 1, 2, 3


def _stream(seed: int, kind: int, a: int, b: int = 0) -> np.random.Generator:
    """Philox-4x64 stream keyed by (seed, kind, a, b); streams are independent of each other."""
    k1 = ((kind & 0xFF) << 56) | ((a & 0xFFFFFFF) << 28) | (b & 0xFFFFFFF)
    return np.random.Generator(np.random.Philox(key=np.array([seed & (2**64 - 1), k1], dtype=np.uint64)))


# ----------------------------------------------------------------------------
# architecture descriptors
# ----------------------------------------------------------------------------
@dataclasses.dataclass
class Arch:
    name: str
    dtype: int
    in_h: int
    in_w: int
    in_c: int
    n_classes: int
    layers: np.ndarray  # [n_layers][12] int32
    # per layer: multiplier applied to the He-normal std of that layer's weights
    gains: List[float]

    @property
    def n_layers(self) -> int:
        return int(self.layers.shape[0])

    @property
    def elem_bytes(self) -> int:
        return 2 if self.dtype == DT_BF16 else 4

    @property
    def input_elems(self) -> int:
        return self.in_h * self.in_w * self.in_c


class _Prog:
    """Tiny builder that tracks activation shapes per buffer and allocates scratch buffers."""

    def __init__(self, h: int, w: int, c: int, n_scratch: int = 4):
        self.shape: Dict[int, Tuple[int, int, int]] = {0: (h, w, c)}
        self.layers: List[List[int]] = []
        self.gains: List[float] = []
        self.n_scratch = n_scratch

    def free_buf(self, busy: Sequence[int]) -> int:
        for b in range(1, self.n_scratch + 1):
            if b not in busy:
                return b
        raise RuntimeError("out of scratch buffers")

    def conv(self, src, dst, k, r, stride, pad, act, res=-1, gain=1.0):
        h, w, c = self.shape[src]
        p = (h + 2 * pad - r) // stride + 1
        q = (w + 2 * pad - r) // stride + 1
        self.shape[dst] = (p, q, k)
        self.layers.append([OP_CONV, src, dst, res, k, r, r, stride, pad, act, 0, 0])
        self.gains.append(gain)

    def maxpool(self, src, dst, r, stride, pad):
        h, w, c = self.shape[src]
        p = (h + 2 * pad - r) // stride + 1
        q = (w + 2 * pad - r) // stride + 1
        self.shape[dst] = (p, q, c)
        self.layers.append([OP_MAXPOOL, src, dst, -1, c, r, r, stride, pad, 0, 0, 0])
        self.gains.append(1.0)

    def head(self, src, n_classes):
        self.layers.append([OP_HEAD, src, -1, -1, n_classes, 0, 0, 0, 0, 0, 0, 0])
        self.gains.append(1.0)

    def concat(self, a, b, dst):
        ha, wa, ca = self.shape[a]
        hb, wb, cb = self.shape[b]
        assert (ha, wa) == (hb, wb)
        self.shape[dst] = (ha, wa, ca + cb)
        self.layers.append([OP_CONCAT, a, dst, b, ca + cb, 0, 0, 0, 0, 0, 0, 0])
        self.gains.append(1.0)

    def upsample(self, src, dst):
        h, w, c = self.shape[src]
        self.shape[dst] = (2 * h, 2 * w, c)
        self.layers.append([OP_UPSAMPLE, src, dst, -1, c, 0, 0, 0, 0, 0, 0, 0])
        self.gains.append(1.0)

    def det_head(self, a, b, n_classes, anchors):
        self.layers.append([OP_HEAD_DET, a, -1, b, n_classes, 0, 0, 0, 0, 0, anchors, 0])
        self.gains.append(1.0)

    def raw(self, words, gain=1.0):
        self.layers.append(list(words))
        self.gains.append(gain)


def tiny_cnn(n_classes: int = 4, hw: int = 64, dtype: int = DT_F32) -> Arch:
    """conv3x3(3->16)-ReLU-conv3x3(16->32)-ReLU-conv3x3(32->64)-ReLU-GAP-FC(64->n_classes), pad 1 stride 1."""
    p = _Prog(hw, hw, 3)
    p.conv(0, 1, 16, 3, 1, 1, ACT_RELU)
    p.conv(1, 2, 32, 3, 1, 1, ACT_RELU)
    p.conv(2, 1, 64, 3, 1, 1, ACT_RELU)
    p.head(1, n_classes)
    return Arch("tiny_cnn", dtype, hw, hw, 3, n_classes, np.array(p.layers, dtype=np.int32), p.gains)


RES_BRANCH_GAIN = 0.5  # std multiplier on the last conv of every residual branch


def resnet18(n_classes: int, hw: int = 224, dtype: int = DT_BF16, width: int = 64) -> Arch:
    """ResNet-18-shaped expert: 7x7/2 stem, 3x3/2 max pool, four stages of two basic blocks, GAP, FC.

    Batch norm is folded: every conv is weights + per-channel fp32 bias."""
    p = _Prog(hw, hw, 3)
    p.conv(0, 1, width, 7, 2, 3, ACT_RELU)
    p.maxpool(1, 2, 3, 2, 1)
    x = 2
    for stage, ch in enumerate([width, 2 * width, 4 * width, 8 * width]):
        for blk in range(2):
            stride = 2 if (stage > 0 and blk == 0) else 1
            t = p.free_buf([x])
            p.conv(x, t, ch, 3, stride, 1, ACT_RELU)
            if stride != 1 or p.shape[x][2] != ch:
                sc = p.free_buf([x, t])
                p.conv(x, sc, ch, 1, stride, 0, ACT_NONE)
            else:
                sc = x
            y = p.free_buf([x, t, sc])
            p.conv(t, y, ch, 3, 1, 1, ACT_RELU, res=sc, gain=RES_BRANCH_GAIN)
            x = y
    p.head(x, n_classes)
    return Arch("resnet18", dtype, hw, hw, 3, n_classes, np.array(p.layers, dtype=np.int32), p.gains)


def resnet50(n_classes: int, hw: int = 224, dtype: int = DT_BF16, width: int = 64) -> Arch:
    """ResNet-50-shaped expert: bottleneck blocks [3,4,6,3], stride on the 3x3 conv of a downsampling block."""
    p = _Prog(hw, hw, 3)
    p.conv(0, 1, width, 7, 2, 3, ACT_RELU)
    p.maxpool(1, 2, 3, 2, 1)
    x = 2
    for stage, (mid, nblk) in enumerate(zip([width, 2 * width, 4 * width, 8 * width], [3, 4, 6, 3])):
        for blk in range(nblk):
            stride = 2 if (stage > 0 and blk == 0) else 1
            out = 4 * mid
            a = p.free_buf([x])
            p.conv(x, a, mid, 1, 1, 0, ACT_RELU)
            b = p.free_buf([x, a])
            p.conv(a, b, mid, 3, stride, 1, ACT_RELU)
            if stride != 1 or p.shape[x][2] != out:
                sc = p.free_buf([x, b])
                p.conv(x, sc, out, 1, stride, 0, ACT_NONE)
            else:
                sc = x
            y = p.free_buf([x, b, sc])
            p.conv(b, y, out, 1, 1, 0, ACT_RELU, res=sc, gain=RES_BRANCH_GAIN)
            x = y
    p.head(x, n_classes)
    return Arch("resnet50", dtype, hw, hw, 3, n_classes, np.array(p.layers, dtype=np.int32), p.gains)


def vit(n_classes: int, hw: int = 224, patch: int = 16, dim: int = 768, depth: int = 12, heads: int = 12,
        mlp: int = 3072, dtype: int = DT_BF16) -> Arch:
    """ViT-shaped expert: patch embedding, class token + learned positions, pre-LN blocks, LN + FC on the class token.

    Token tensors are stored as images of height T, width 1, so every linear layer is a 1x1 CONV op."""
    p = _Prog(hw, hw, 3, n_scratch=5)
    p.conv(0, 1, dim, patch, patch, 0, ACT_NONE)                    # [hw/patch][hw/patch][dim]
    gh = hw // patch
    t = gh * gh + 1
    p.raw([OP_TOKENS, 1, 2, -1, dim, 0, 0, 0, 0, 0, 0, 0])          # [t][1][dim]
    p.shape[2] = (t, 1, dim)
    x = 2
    for _ in range(depth):
        n1 = p.free_buf([x])
        p.raw([OP_LAYERNORM, x, n1, -1, dim, 0, 0, 0, 0, 0, 0, 0]); p.shape[n1] = (t, 1, dim)
        qkv = p.free_buf([x, n1])
        p.conv(n1, qkv, 3 * dim, 1, 1, 0, ACT_NONE)
        at = p.free_buf([x, qkv])
        p.raw([OP_ATTENTION, qkv, at, -1, dim, 0, 0, 0, 0, 0, heads, 0]); p.shape[at] = (t, 1, dim)
        x2 = p.free_buf([x, at])
        p.conv(at, x2, dim, 1, 1, 0, ACT_NONE, res=x)
        n2 = p.free_buf([x2])
        p.raw([OP_LAYERNORM, x2, n2, -1, dim, 0, 0, 0, 0, 0, 0, 0]); p.shape[n2] = (t, 1, dim)
        h = p.free_buf([x2, n2])
        p.conv(n2, h, mlp, 1, 1, 0, ACT_GELU)
        x3 = p.free_buf([x2, h])
        p.conv(h, x3, dim, 1, 1, 0, ACT_NONE, res=x2)
        x = x3
    p.raw([OP_HEAD_CLS, x, -1, -1, n_classes, 0, 0, 0, 0, 0, 0, 0])
    return Arch("vit", dtype, hw, hw, 3, n_classes, np.array(p.layers, dtype=np.int32), p.gains)


def detector(n_classes: int = 27, hw: int = 224, width: int = 64, anchors: int = 3, dtype: int = DT_BF16) -> Arch:
    """Detector-shaped expert in the style of the one-stage detectors the paper uses downstream of its classifiers (Section
    5.1): strided conv stem, cross-stage blocks (two 1x1 branches, a residual bottleneck on one, concatenation, 1x1 fusion),
    a pooling pyramid (three chained 5x5 max pools, concatenated), a top-down neck (upsample + concatenate with the
    finer map), 1x1 detection outputs on two scales with `anchors` x (5 + n_classes) channels, SiLU activations.  The
    expert's logits are its best detection score per class (HEAD_DET).  anchors * (5 + n_classes) must be a multiple of 32."""
    assert (anchors * (5 + n_classes)) % 32 == 0
    S = ACT_SILU
    p = _Prog(hw, hw, 3, n_scratch=7)

    def csp(x, c, keep=()):
        """cross-stage block on buffer x with c channels; returns the output buffer (x is free afterwards)"""
        a = p.free_buf([x, *keep]); p.conv(x, a, c // 2, 1, 1, 0, S)
        b = p.free_buf([x, a, *keep]); p.conv(x, b, c // 2, 1, 1, 0, S)
        t = p.free_buf([a, b, *keep]); p.conv(a, t, c // 2, 1, 1, 0, S)
        a2 = p.free_buf([a, b, t, *keep]); p.conv(t, a2, c // 2, 3, 1, 1, S, res=a, gain=RES_BRANCH_GAIN)
        cat = p.free_buf([a2, b, *keep]); p.concat(a2, b, cat)
        y = p.free_buf([cat, *keep]); p.conv(cat, y, c, 1, 1, 0, S)
        return y

    p.conv(0, 1, width, 6, 2, 2, S)                                   # hw/2
    p.conv(1, 2, 2 * width, 3, 2, 1, S)                               # hw/4
    x = csp(2, 2 * width)
    d = p.free_buf([x]); p.conv(x, d, 4 * width, 3, 2, 1, S)          # hw/8
    p4 = csp(d, 4 * width)                                            # kept for the neck
    d = p.free_buf([p4]); p.conv(p4, d, 8 * width, 3, 2, 1, S)        # hw/16
    x = csp(d, 8 * width, keep=(p4,))
    # pooling pyramid
    q = p.free_buf([x, p4]); p.conv(x, q, 4 * width, 1, 1, 0, S)
    m1 = p.free_buf([q, p4]); p.maxpool(q, m1, 5, 1, 2)
    c1 = p.free_buf([q, m1, p4]); p.concat(q, m1, c1)
    m2 = p.free_buf([m1, c1, p4]); p.maxpool(m1, m2, 5, 1, 2)
    c2 = p.free_buf([c1, m2, p4]); p.concat(c1, m2, c2)
    m3 = p.free_buf([m2, c2, p4]); p.maxpool(m2, m3, 5, 1, 2)
    c3 = p.free_buf([c2, m3, p4]); p.concat(c2, m3, c3)               # 16 * width channels
    p5 = p.free_buf([c3, p4]); p.conv(c3, p5, 8 * width, 1, 1, 0, S)
    # neck: coarse map reduced, upsampled, concatenated with the finer one
    r = p.free_buf([p5, p4]); p.conv(p5, r, 4 * width, 1, 1, 0, S)
    u = p.free_buf([r, p5, p4]); p.upsample(r, u)
    cat = p.free_buf([u, p5, p4]); p.concat(u, p4, cat)               # 8 * width channels at hw/8
    f = p.free_buf([cat, p5]); p.conv(cat, f, 4 * width, 1, 1, 0, S)
    g = p.free_buf([f, p5]); p.conv(f, g, 4 * width, 3, 1, 1, S)
    det_c = anchors * (5 + n_classes)
    d4 = p.free_buf([g, p5]); p.conv(g, d4, det_c, 1, 1, 0, ACT_NONE)
    d5 = p.free_buf([d4, p5]); p.conv(p5, d5, det_c, 1, 1, 0, ACT_NONE)
    p.det_head(d4, d5, n_classes, anchors)
    return Arch("detector", dtype, hw, hw, 3, n_classes, np.array(p.layers, dtype=np.int32), p.gains)


# ----------------------------------------------------------------------------
# shape walk and blob layout
# ----------------------------------------------------------------------------
@dataclasses.dataclass
class TensorSpec:
    layer: int
    name: str
    shape: Tuple[int, ...]
    is_param_dtype: bool   # True: stored in the arch dtype; False: stored as fp32
    offset: int
    nbytes: int


def _align(x: int, a: int = BLOB_ALIGN) -> int:
    return (x + a - 1) // a * a


def walk(arch: Arch):
    """Per layer: (src_shape, dst_shape) as (h, w, c); heads have dst_shape None."""
    shp: Dict[int, Tuple[int, int, int]] = {0: (arch.in_h, arch.in_w, arch.in_c)}
    out = []
    for L in arch.layers:
        op, src, dst, res, k, r, s, stride, pad = [int(v) for v in L[:9]]
        h, w, c = shp[src]
        if op in (OP_CONV, OP_MAXPOOL):
            d = ((h + 2 * pad - r) // stride + 1, (w + 2 * pad - s) // stride + 1, k)
        elif op == OP_TOKENS:
            d = (h * w + 1, 1, c)
        elif op == OP_LAYERNORM:
            d = (h, w, c)
        elif op == OP_ATTENTION:
            d = (h, w, c // 3)
        elif op == OP_CONCAT:
            d = (h, w, c + shp[res][2])
        elif op == OP_UPSAMPLE:
            d = (2 * h, 2 * w, c)
        else:
            d = None
        if d is not None:
            shp[dst] = d
        out.append(((h, w, c), d))
    return out


def blob_layout(arch: Arch) -> Tuple[List[TensorSpec], int]:
    specs: List[TensorSpec] = []
    off = 0
    eb = arch.elem_bytes

    def add(layer, name, shape, param_dtype):
        nonlocal off
        off = _align(off)
        nb = int(np.prod(shape)) * (eb if param_dtype else 4)
        specs.append(TensorSpec(layer, name, tuple(int(v) for v in shape), param_dtype, off, nb))
        off += nb

    for i, (L, (sshape, dshape)) in enumerate(zip(arch.layers, walk(arch))):
        op, k, r, s = int(L[0]), int(L[4]), int(L[5]), int(L[6])
        h, w, c = sshape
        if op == OP_CONV:
            add(i, "w", (k, r, s, c), True)
            add(i, "b", (k,), False)
        elif op == OP_HEAD:
            add(i, "w", (k, c), True)
            add(i, "b", (k,), False)
        elif op == OP_TOKENS:
            add(i, "cls", (c,), True)
            add(i, "pos", (h * w + 1, c), True)
        elif op == OP_LAYERNORM:
            add(i, "gamma", (c,), False)
            add(i, "beta", (c,), False)
        elif op == OP_HEAD_CLS:
            add(i, "gamma", (c,), False)
            add(i, "beta", (c,), False)
            add(i, "w", (k, c), True)
            add(i, "b", (k,), False)
    return specs, _align(off)


# ----------------------------------------------------------------------------
# expert weights
# ----------------------------------------------------------------------------
BIAS_STD = 0.05


def make_expert_blob(arch: Arch, seed: int, expert_id: int, head_bias: Optional[np.ndarray] = None) -> np.ndarray:
    """He-normal weights (std sqrt(2/fan_in) x the layer's gain), biases N(0, BIAS_STD^2), packed into a blob.

    head_bias, when given, replaces the head's bias (calibrated routing offsets).  Returns uint8[nbytes]."""
    specs, nbytes = blob_layout(arch)
    blob = np.zeros(nbytes, dtype=np.uint8)
    for t_idx, sp in enumerate(specs):
        g = _stream(seed, _KIND_WEIGHT, expert_id, t_idx)
        n = int(np.prod(sp.shape))
        op = int(arch.layers[sp.layer][0])
        if sp.name == "w":
            fan_in = n // sp.shape[0]
            if op == OP_CONV:
                act = int(arch.layers[sp.layer][9])
                std = math.sqrt((2.0 if act in (ACT_RELU, ACT_SILU) or int(arch.layers[sp.layer][3]) >= 0 else 1.0) / fan_in)
                if arch.name == "vit":
                    std = math.sqrt(1.0 / fan_in)
                std *= arch.gains[sp.layer]
            else:
                std = math.sqrt(1.0 / fan_in)
            v = g.standard_normal(n, dtype=np.float32) * np.float32(std)
        elif sp.name == "b":
            v = g.standard_normal(n, dtype=np.float32) * np.float32(BIAS_STD)
            if op in (OP_HEAD, OP_HEAD_CLS) and head_bias is not None:
                v = np.asarray(head_bias, dtype=np.float32).reshape(n).copy()
        elif sp.name == "gamma":
            v = (1.0 + 0.1 * g.standard_normal(n, dtype=np.float32)).astype(np.float32)
        elif sp.name == "beta":
            v = (0.1 * g.standard_normal(n, dtype=np.float32)).astype(np.float32)
        elif sp.name in ("cls", "pos"):
            v = (0.5 * g.standard_normal(n, dtype=np.float32)).astype(np.float32)
        else:
            raise AssertionError(sp.name)
        if sp.is_param_dtype and arch.dtype == DT_BF16:
            blob[sp.offset:sp.offset + sp.nbytes] = f32_to_bf16_bits(v).view(np.uint8)
        else:
            blob[sp.offset:sp.offset + sp.nbytes] = v.astype(np.float32).view(np.uint8)
    return blob


def blob_tensor(arch: Arch, blob: np.ndarray, layer: int, name: str) -> np.ndarray:
    """Decode one tensor of a blob to float32 (test helper)."""
    specs, _ = blob_layout(arch)
    for sp in specs:
        if sp.layer == layer and sp.name == name:
            raw = blob[sp.offset:sp.offset + sp.nbytes]
            if sp.is_param_dtype and arch.dtype == DT_BF16:
                return bf16_bits_to_f32(raw.view(np.uint16)).reshape(sp.shape)
            return raw.view(np.float32).reshape(sp.shape).copy()
    raise KeyError((layer, name))


# ----------------------------------------------------------------------------
# request inputs
# ----------------------------------------------------------------------------
STRUCT_GRID = 2           # a structured image's coarse pattern has STRUCT_GRID x STRUCT_GRID cells per channel
STRUCT_NOISE_STD = 0.5    # and pixel noise of this standard deviation on top


def make_inputs(arch: Arch, seed: int, request_ids: Sequence[int], subseeds: Optional[Sequence[int]] = None,
                kind: str = "noise") -> np.ndarray:
    """Request images, NHWC, one independent Philox stream per (request id, sub-seed).

    kind "noise": every element ~ N(0,1).  kind "structured": a per-request coarse pattern (a STRUCT_GRID x STRUCT_GRID
    grid of N(0,1) values per channel, each cell covering a block of pixels) plus N(0, STRUCT_NOISE_STD^2) pixel noise.
    Pure-noise images all look alike to an expert after its global pooling (every request gets nearly the same logits);
    the coarse pattern gives each request features of its own, as the images of a real workload have.

    Returns uint16 bf16 bit patterns [n][H][W][C] for bf16 architectures, float32 otherwise.  A request whose
    routing margin is too small for a well-posed argmax is re-drawn by bumping its sub-seed."""
    assert kind in ("noise", "structured")
    n = len(request_ids)
    elems = arch.input_elems
    out = np.empty((n, elems), dtype=np.uint16 if arch.dtype == DT_BF16 else np.float32)
    ids = [int(r) for r in request_ids]
    # pixel row / column -> cell of the coarse grid
    cell_h = (np.arange(arch.in_h) * STRUCT_GRID) // arch.in_h
    cell_w = (np.arange(arch.in_w) * STRUCT_GRID) // arch.in_w

    def draw(i):
        ss = 0 if subseeds is None else int(subseeds[i])
        g = _stream(seed, _KIND_INPUT, ids[i], ss)
        if kind == "structured":
            coarse = g.standard_normal((STRUCT_GRID, STRUCT_GRID, arch.in_c), dtype=np.float32)
            v = g.standard_normal(elems, dtype=np.float32) * np.float32(STRUCT_NOISE_STD)
            v = (v.reshape(arch.in_h, arch.in_w, arch.in_c) + coarse[cell_h][:, cell_w]).reshape(elems)
        else:
            v = g.standard_normal(elems, dtype=np.float32)
        out[i] = f32_to_bf16_bits(v) if arch.dtype == DT_BF16 else v

    if n * elems > (1 << 24):      # large batches: numpy releases the GIL inside the generator
        from concurrent.futures import ThreadPoolExecutor
        with ThreadPoolExecutor(max_workers=min(16, os.cpu_count() or 1)) as ex:
            list(ex.map(draw, range(n)))
    else:
        for i in range(n):
            draw(i)
    return out.reshape(n, arch.in_h, arch.in_w, arch.in_c)


# ----------------------------------------------------------------------------
# dependency graphs (CSR successor lists; the argmax over the first n_route classes indexes the list)
# ----------------------------------------------------------------------------
@dataclasses.dataclass
class Graph:
    n_experts: int
    succ_off: np.ndarray  # int32 [E+1]
    succ: np.ndarray      # int32 [nnz], expert id or -1 (= final)

    def successors(self, e: int) -> np.ndarray:
        return self.succ[self.succ_off[e]:self.succ_off[e + 1]]


def graph_from_lists(lists: Sequence[Sequence[int]]) -> Graph:
    off = np.zeros(len(lists) + 1, dtype=np.int32)
    for i, l in enumerate(lists):
        off[i + 1] = off[i] + len(l)
    succ = np.array([v for l in lists for v in l], dtype=np.int32)
    return Graph(len(lists), off, succ)


def tree_graph(n_experts: int) -> Graph:
    """Expert 0 routes to experts 1..E-1 (class c -> expert c+1); leaves are final."""
    return graph_from_lists([list(range(1, n_experts))] + [[] for _ in range(n_experts - 1)])


def zipf_probs(n: int, s: float) -> np.ndarray:
    w = 1.0 / np.arange(1, n + 1, dtype=np.float64) ** s
    return w / w.sum()


# ----------------------------------------------------------------------------
# whole workloads
# ----------------------------------------------------------------------------
@dataclasses.dataclass
class Workload:
    name: str
    seed: int
    archs: List[Arch]
    expert_arch: List[int]            # arch index per expert
    usage_prob: List[float]
    graph: Graph
    n_requests: int
    first_expert: Optional[np.ndarray]  # int32 [n] or None (single root = expert 0)
    cache_cap_experts: int            # 0 = uncapped
    arrival_batch: int                # requests per coe_submit
    head_bias: Dict[int, np.ndarray]  # expert id -> calibrated head bias
    max_stages: int
    input_kind: str = "noise"         # see make_inputs

    def blob(self, e: int) -> np.ndarray:
        return make_expert_blob(self.archs[self.expert_arch[e]], self.seed, e, self.head_bias.get(e))

    def inputs(self, request_ids, subseeds=None) -> np.ndarray:
        return make_inputs(self.archs[0], self.seed, request_ids, subseeds, self.input_kind)

    @property
    def max_classes(self) -> int:
        return max(a.n_classes for a in self.archs)


_CALIB_DIR = os.path.join(os.path.dirname(os.path.abspath(__file__)), "calib")


def load_calibration(name: str) -> Dict[int, np.ndarray]:
    """Head-bias offsets written by the oracle-side calibration script; empty if none was stored."""
    path = os.path.join(_CALIB_DIR, name + ".json")
    if not os.path.exists(path):
        return {}
    with open(path) as f:
        d = json.load(f)
    return {int(k): np.array(v, dtype=np.float32) for k, v in d["head_bias"].items()}


def config1(n_requests: int = 256, hw: int = 64, calibrated: bool = True) -> Workload:
    """Four fp32 tiny-CNN experts, two stages: expert 0's argmax over classes 0-2 routes to experts 1-3."""
    a = tiny_cnn(4, hw, DT_F32)
    name = "config1" if hw == 64 else f"config1_hw{hw}"
    g = graph_from_lists([[1, 2, 3], [], [], []])
    return Workload(name, 0xC0E1, [a], [0] * 4, [1.0, 1 / 3, 1 / 3, 1 / 3], g, n_requests, None, 0, n_requests,
                    load_calibration(name) if calibrated else {}, 2)


def config2(n_requests: int = 4096, hw: int = 224, n_experts: int = 16, width: int = 64,
            calibrated: bool = True) -> Workload:
    """ResNet-18-shaped bf16 experts, one root routing 15 ways (16 logits, the first 15 route), all resident."""
    a = resnet18(16, hw, DT_BF16, width)
    name = "config2" if (hw, n_experts, width) == (224, 16, 64) else f"config2_hw{hw}_e{n_experts}_w{width}"
    g = tree_graph(n_experts)
    p = [1.0] + [1.0 / (n_experts - 1)] * (n_experts - 1)
    return Workload(name, 0xC0E2, [a], [0] * n_experts, p, g, n_requests, None, 0, n_requests,
                    load_calibration(name) if calibrated else {}, 2)


def config3(n_requests: int = 16384, hw: int = 224, n_experts: int = 64, width: int = 64, cap: int = 16,
            arrival_batch: int = 512, calibrated: bool = True) -> Workload:
    """ResNet-50-shaped bf16 experts, root -> 63 leaves with Zipf(1.1) leaf usage, capped device cache."""
    a = resnet50(n_experts, hw, DT_BF16, width)
    name = "config3" if (hw, n_experts, width) == (224, 64, 64) else f"config3_hw{hw}_e{n_experts}_w{width}"
    g = tree_graph(n_experts)
    p = [1.0] + list(zipf_probs(n_experts - 1, 1.1))
    return Workload(name, 0xC0E3, [a], [0] * n_experts, p, g, n_requests, None, cap, arrival_batch,
                    load_calibration(name) if calibrated else {}, 2, "structured")


def config4(n_requests: int = 8192, hw: int = 224, tiers: Tuple[int, int, int] = (8, 32, 80), width: int = 64,
            fan: Tuple[int, int] = (6, 5), calibrated: bool = True) -> Workload:
    """Three-stage DAG of mixed ResNet-18/50-shaped experts with shared downstream experts and skewed groups.

    Stage-1 expert i routes to `fan[0]` stage-2 experts, stage-2 expert j to `fan[1]` stage-3 experts, chosen
    from seeded, overlapping windows so several upstream experts share one downstream expert.  Architecture
    alternates by expert id parity.  first_expert follows a Zipf(1.2) draw over the stage-1 experts."""
    n1, n2, n3 = tiers
    e_total = n1 + n2 + n3
    ncls = max(fan) + 1
    a18 = resnet18(ncls, hw, DT_BF16, width)
    a50 = resnet50(ncls, hw, DT_BF16, width)
    name = "config4" if (hw, tiers, width) == (224, (8, 32, 80), 64) else \
        f"config4_hw{hw}_t{n1}_{n2}_{n3}_w{width}"
    seed = 0xC0E4
    g = _stream(seed, _KIND_MISC, 1)
    lists: List[List[int]] = []
    for i in range(n1):
        start = (i * n2) // n1
        lists.append([n1 + (start + d * 3 + int(g.integers(0, 3))) % n2 for d in range(fan[0])])
    for j in range(n2):
        start = (j * n3) // n2
        lists.append([n1 + n2 + (start + d * 2 + int(g.integers(0, 2))) % n3 for d in range(fan[1])])
    for _ in range(n3):
        lists.append([])
    graph = graph_from_lists(lists)
    first = _stream(seed, _KIND_MISC, 2).choice(n1, size=n_requests, p=zipf_probs(n1, 1.2)).astype(np.int32)
    # usage probability: propagate the first-expert distribution down the DAG with uniform branch choice
    prob = np.zeros(e_total)
    prob[:n1] = zipf_probs(n1, 1.2)
    for e in range(n1 + n2):
        for s in lists[e]:
            prob[s] += prob[e] / len(lists[e])
    return Workload(name, seed, [a18, a50], [e % 2 for e in range(e_total)], list(prob), graph, n_requests, first,
                    0, n_requests, load_calibration(name) if calibrated else {}, 3, "structured")


def config5(n_requests: int = 4096, hw: int = 224, n_experts: int = 32, cap: int = 12, dim: int = 768,
            depth: int = 12, heads: int = 12, mlp: int = 3072, calibrated: bool = True) -> Workload:
    """ViT-B/16-shaped bf16 experts, root -> 31 leaves with uniform routing, capped device cache."""
    a = vit(n_experts, hw, 16, dim, depth, heads, mlp, DT_BF16)
    name = "config5" if (hw, n_experts, dim, depth) == (224, 32, 768, 12) else \
        f"config5_hw{hw}_e{n_experts}_d{dim}_l{depth}"
    g = tree_graph(n_experts)
    p = [1.0] + [1.0 / (n_experts - 1)] * (n_experts - 1)
    return Workload(name, 0xC0E5, [a], [0] * n_experts, p, g, n_requests, None, cap, n_requests,
                    load_calibration(name) if calibrated else {}, 2, "structured")


def config6(n_requests: int = 4096, hw: int = 224, n_classifiers: int = 4, n_detectors: int = 8, fan: int = 6, width: int = 64,
            det_width: int = 64, det_classes: int = 27, calibrated: bool = True) -> Workload:
    """Classifier -> detector DAG in the shape of the paper's own workload (Section 5.1: classification experts decide what a
    component is, object-detection experts inspect it; several upstream experts share one downstream expert).  Stage 1:
    `n_classifiers` ResNet-18-shaped classifiers (the first expert of a request follows Zipf(1.2)); each routes `fan` ways to
    detector-shaped experts drawn from seeded, overlapping windows of the `n_detectors` detectors, which are final: a request's
    result is its detector's best detection score per class."""
    e_total = n_classifiers + n_detectors
    a_cls = resnet18(fan + 2, hw, DT_BF16, width)
    a_det = detector(det_classes, hw, det_width, 3, DT_BF16)
    name = "config6" if (hw, n_classifiers, n_detectors, fan, width, det_width) == (224, 4, 8, 6, 64, 64) else \
        f"config6_hw{hw}_c{n_classifiers}_d{n_detectors}_f{fan}_w{width}_{det_width}"
    seed = 0xC0E6
    g = _stream(seed, _KIND_MISC, 1)
    lists: List[List[int]] = []
    for i in range(n_classifiers):
        start = (i * n_detectors) // n_classifiers
        lists.append([n_classifiers + (start + d + int(g.integers(0, 2))) % n_detectors for d in range(fan)])
    for _ in range(n_detectors):
        lists.append([])
    graph = graph_from_lists(lists)
    first = _stream(seed, _KIND_MISC, 2).choice(n_classifiers, size=n_requests, p=zipf_probs(n_classifiers, 1.2)).astype(np.int32)
    prob = np.zeros(e_total)
    prob[:n_classifiers] = zipf_probs(n_classifiers, 1.2)
    for e in range(n_classifiers):
        for s_ in lists[e]:
            prob[s_] += prob[e] / len(lists[e])
    return Workload(name, seed, [a_cls, a_det], [0] * n_classifiers + [1] * n_detectors, list(prob), graph, n_requests, first,
                    0, n_requests, load_calibration(name) if calibrated else {}, 2, "structured")

