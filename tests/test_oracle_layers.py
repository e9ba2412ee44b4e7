"""Pins for the oracle's layer arithmetic: each check is something other than the oracle's own formula
(a structurally different brute force, a closed form, an invariant or a hand-computed value)."""
import math

import numpy as np
import pytest

import bench
import coe_workloads as W


# ---------------------------------------------------------------------------------------------
# bf16 rounding
# ---------------------------------------------------------------------------------------------
def _nearest_even_bf16_f64(x32: np.ndarray) -> np.ndarray:
    """Nearest bf16 by exact distance in float64; ties go to the neighbour with an even last mantissa bit."""
    u = x32.view(np.uint32)
    lo_bits = u & np.uint32(0xFFFF0000)
    hi_bits = lo_bits + np.uint32(0x00010000)          # next bf16 away from zero (may become inf: fine)
    lo = lo_bits.view(np.float32).astype(np.float64)
    hi = hi_bits.view(np.float32).astype(np.float64)
    x = x32.astype(np.float64)
    dlo, dhi = np.abs(x - lo), np.abs(hi - x)
    lo_even = ((lo_bits >> np.uint32(16)) & np.uint32(1)) == 0
    pick_lo = (dlo < dhi) | ((dlo == dhi) & lo_even)
    return np.where(pick_lo, lo_bits, hi_bits).view(np.float32)


def _finite_patterns():
    hi = np.arange(0, 1 << 16, dtype=np.uint32)
    hi = hi[(hi & 0x7F80) != 0x7F80]                    # drop inf / nan exponents
    hi = hi[((hi + 1) & 0x7F80) != 0x7F80]              # and the largest finite bf16 (its upper neighbour is inf)
    lows = np.array([0x0000, 0x0001, 0x7FFF, 0x8000, 0x8001, 0xFFFF, 0x1234, 0xC000], dtype=np.uint32)
    return ((hi[:, None] << np.uint32(16)) | lows[None, :]).ravel().astype(np.uint32)


def test_generator_bf16_rounding_exhaustive():
    pats = _finite_patterns()
    x = pats.view(np.float32)
    got = W.bf16_bits_to_f32(W.f32_to_bf16_bits(x))
    want = _nearest_even_bf16_f64(x)
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))


def test_oracle_bf16_rounding(oracle):
    pats = _finite_patterns()[::7]                       # every 7th pattern still hits all low-half cases
    x = pats.view(np.float32)
    got = oracle.bf16_round(x)
    want = _nearest_even_bf16_f64(x)
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))
    # known ties: 1.00390625 (0x3F808000) is halfway between 0x3F80 (even) and 0x3F81 -> down;
    # 0x3F818000 is halfway between 0x3F81 (odd) and 0x3F82 (even) -> up
    ties = np.array([0x3F808000, 0x3F818000], dtype=np.uint32).view(np.float32)
    assert oracle.bf16_round(ties).view(np.uint32).tolist() == [0x3F800000, 0x3F820000]


# ---------------------------------------------------------------------------------------------
# convolution
# ---------------------------------------------------------------------------------------------
def _conv_im2col(x, w, bias, stride, pad):
    """Second, structurally different implementation: zero-padded copy, patch matrix, one float64 matmul."""
    H, Wd, C = x.shape
    K, R, S, _ = w.shape
    xp = np.zeros((H + 2 * pad, Wd + 2 * pad, C), np.float64)
    xp[pad:pad + H, pad:pad + Wd] = x
    P = (H + 2 * pad - R) // stride + 1
    Q = (Wd + 2 * pad - S) // stride + 1
    cols = np.empty((P * Q, R * S * C), np.float64)
    for p in range(P):
        for q in range(Q):
            cols[p * Q + q] = xp[p * stride:p * stride + R, q * stride:q * stride + S].reshape(-1)
    return (cols @ w.reshape(K, -1).astype(np.float64).T + bias.astype(np.float64)).reshape(P, Q, K)


@pytest.mark.parametrize("H,Wd,C,K,R,S,stride,pad", [
    (5, 7, 3, 4, 3, 3, 1, 1), (9, 6, 2, 5, 3, 3, 2, 1), (11, 13, 3, 2, 7, 7, 2, 3),
    (6, 5, 4, 3, 1, 1, 1, 0), (8, 7, 4, 3, 1, 1, 2, 0), (7, 9, 2, 3, 3, 1, 1, 0), (7, 9, 2, 3, 1, 3, 1, 1),
    (8, 8, 3, 6, 4, 4, 4, 0),
])
def test_conv_matches_im2col(oracle, H, Wd, C, K, R, S, stride, pad):
    rng = np.random.default_rng(H * 100 + Wd)
    x = rng.standard_normal((H, Wd, C)).astype(np.float32)
    w = rng.standard_normal((K, R, S, C)).astype(np.float32)
    b = rng.standard_normal(K).astype(np.float32)
    # the oracle takes R == S from the descriptor but its layer routine accepts R != S; both orders are exercised
    want = _conv_im2col(x, w, b, stride, pad)
    L = oracle.lib()
    P, Q = want.shape[:2]
    y = np.empty((P, Q, K), np.float32)
    import ctypes as Ct
    L.orc_conv2d(x.ctypes.data_as(Ct.c_void_p), H, Wd, C, w.ctypes.data_as(Ct.c_void_p), b.ctypes.data_as(Ct.c_void_p),
                 None, K, R, S, stride, pad, 0, 0, y.ctypes.data_as(Ct.c_void_p))
    np.testing.assert_allclose(y, want, rtol=2e-6, atol=2e-6)


def test_conv_hand_example(oracle):
    # 3x3 image, one channel, 2x2... use 3x3 kernel of ones with pad 1: every output = sum of the 3x3 neighbourhood
    x = np.arange(1, 10, dtype=np.float32).reshape(3, 3, 1)
    w = np.ones((1, 3, 3, 1), np.float32)
    y = oracle.conv2d(x, w, np.zeros(1, np.float32), stride=1, pad=1)[..., 0]
    want = np.array([[12, 21, 16], [27, 45, 33], [24, 39, 28]], np.float32)
    assert np.array_equal(y, want)
    # bias and ReLU: subtract 30 then clamp
    y = oracle.conv2d(x, w, np.full(1, -30, np.float32), stride=1, pad=1, act=1)[..., 0]
    assert np.array_equal(y, np.maximum(want - 30, 0))
    # residual is added before the activation
    res = np.full((3, 3, 1), 20, np.float32)
    y = oracle.conv2d(x, w, np.full(1, -30, np.float32), res=res, stride=1, pad=1, act=1)[..., 0]
    assert np.array_equal(y, np.maximum(want - 10, 0))


def test_conv_delta_kernel_is_shift(oracle):
    rng = np.random.default_rng(3)
    x = rng.standard_normal((6, 8, 2)).astype(np.float32)
    for (r, s) in [(0, 0), (0, 2), (2, 1), (1, 1)]:
        w = np.zeros((2, 3, 3, 2), np.float32)
        w[0, r, s, 0] = 1.0      # output channel 0 copies input channel 0 shifted by (r-1, s-1)
        w[1, r, s, 1] = 1.0
        y = oracle.conv2d(x, w, np.zeros(2, np.float32), stride=1, pad=1)
        want = np.zeros_like(x)
        for p in range(6):
            for q in range(8):
                ih, iw = p + r - 1, q + s - 1
                if 0 <= ih < 6 and 0 <= iw < 8:
                    want[p, q] = x[ih, iw]
        assert np.array_equal(y, want)


def test_conv_constant_image_closed_form(oracle):
    rng = np.random.default_rng(5)
    c0 = 1.5
    x = np.full((7, 7, 3), c0, np.float32)
    w = rng.standard_normal((4, 3, 3, 3)).astype(np.float32)
    y = oracle.conv2d(x, w, np.zeros(4, np.float32), stride=1, pad=1)
    full = c0 * w.astype(np.float64).sum(axis=(1, 2, 3))
    np.testing.assert_allclose(y[3, 3], full, rtol=1e-6)
    # top-left corner sees only kernel rows/cols 1..2
    corner = c0 * w[:, 1:, 1:, :].astype(np.float64).sum(axis=(1, 2, 3))
    np.testing.assert_allclose(y[0, 0], corner, rtol=1e-6, atol=1e-6)
    # bottom edge (not corner) sees kernel rows 0..1, all cols
    edge = c0 * w[:, :2, :, :].astype(np.float64).sum(axis=(1, 2, 3))
    np.testing.assert_allclose(y[6, 3], edge, rtol=1e-6, atol=1e-6)


def test_conv_linearity_and_stride_subsampling(oracle):
    rng = np.random.default_rng(7)
    x1 = rng.standard_normal((9, 9, 3)).astype(np.float32)
    x2 = rng.standard_normal((9, 9, 3)).astype(np.float32)
    w = rng.standard_normal((5, 3, 3, 3)).astype(np.float32)
    z = np.zeros(5, np.float32)
    y1 = oracle.conv2d(x1, w, z, pad=1); y2 = oracle.conv2d(x2, w, z, pad=1)
    y = oracle.conv2d((2 * x1 - 3 * x2).astype(np.float32), w, z, pad=1)
    np.testing.assert_allclose(y, 2 * y1 - 3 * y2, rtol=1e-4, atol=1e-4)
    ys2 = oracle.conv2d(x1, w, z, stride=2, pad=1)
    assert np.array_equal(ys2, y1[::2, ::2])


def test_conv_1x1_on_1x1_is_dot(oracle):
    x = np.array([1, 2, 3, 4], np.float32).reshape(1, 1, 4)
    w = np.array([[1, 0, -1, 2], [0.5, 0.5, 0.5, 0.5]], np.float32).reshape(2, 1, 1, 4)
    y = oracle.conv2d(x, w, np.array([10, 20], np.float32))
    assert y.reshape(-1).tolist() == [1 - 3 + 8 + 10, 5 + 20]


def test_conv_bf16_storage_rounding(oracle):
    # the stored result is the bf16 nearest to the exactly accumulated value
    rng = np.random.default_rng(11)
    x = W.bf16_bits_to_f32(W.f32_to_bf16_bits(rng.standard_normal((6, 6, 8)).astype(np.float32))).reshape(6, 6, 8)
    w = W.bf16_bits_to_f32(W.f32_to_bf16_bits(rng.standard_normal((4, 3, 3, 8)).astype(np.float32))).reshape(4, 3, 3, 8)
    b = rng.standard_normal(4).astype(np.float32)
    y = oracle.conv2d(x, w, b, pad=1, act=1, dtype=1)
    exact = np.maximum(_conv_im2col(x, w, b, 1, 1), 0).astype(np.float32)
    assert np.array_equal(y.view(np.uint32), _nearest_even_bf16_f64(exact).view(np.uint32))
    assert np.all((y.view(np.uint32) & 0xFFFF) == 0)


# ---------------------------------------------------------------------------------------------
# pooling, head
# ---------------------------------------------------------------------------------------------
def test_maxpool_brute_force_and_padding(oracle):
    rng = np.random.default_rng(13)
    x = (rng.standard_normal((9, 11, 3)) - 5.0).astype(np.float32)      # all negative: zero padding would win if wrong
    y = oracle.maxpool(x, 3, 2, 1)
    xp = np.full((11, 13, 3), -np.inf, np.float32); xp[1:10, 1:12] = x
    P, Q = (9 + 2 - 3) // 2 + 1, (11 + 2 - 3) // 2 + 1
    want = np.empty((P, Q, 3), np.float32)
    for p in range(P):
        for q in range(Q):
            want[p, q] = xp[2 * p:2 * p + 3, 2 * q:2 * q + 3].reshape(-1, 3).max(axis=0)
    assert y.shape == want.shape and np.array_equal(y, want)
    assert np.all(y < 0)


def test_gap_fc_closed_forms(oracle):
    x = np.zeros((2, 2, 2), np.float32)
    x[..., 0] = [[1, 2], [3, 4]]      # mean 2.5
    x[..., 1] = [[0, 0], [0, 8]]      # mean 2
    w = np.array([[1, 1], [2, -1], [0, 0]], np.float32)
    b = np.array([0, 0.5, -7], np.float32)
    assert oracle.gap_fc(x, w, b).tolist() == [4.5, 3.5, -7.0]
    const = np.full((5, 3, 4), 0.25, np.float32)
    rng = np.random.default_rng(1)
    w = rng.standard_normal((6, 4)).astype(np.float32)
    np.testing.assert_allclose(oracle.gap_fc(const, w, np.zeros(6, np.float32)), 0.25 * w.astype(np.float64).sum(1), rtol=1e-6)


# ---------------------------------------------------------------------------------------------
# transformer pieces
# ---------------------------------------------------------------------------------------------
def test_layernorm_invariants(oracle):
    rng = np.random.default_rng(17)
    x = (3 * rng.standard_normal((5, 64)) + 2).astype(np.float32)
    y = oracle.layernorm(x, np.ones(64, np.float32), np.zeros(64, np.float32))
    np.testing.assert_allclose(y.mean(1), 0, atol=1e-6)
    np.testing.assert_allclose(y.var(1), 1, rtol=1e-4)
    g = rng.standard_normal(64).astype(np.float32); b = rng.standard_normal(64).astype(np.float32)
    y2 = oracle.layernorm(x, g, b)
    np.testing.assert_allclose(y2, y * g + b, rtol=1e-5, atol=1e-5)
    # shift and positive scale of the input leave the output unchanged (up to the epsilon)
    y3 = oracle.layernorm((4 * x + 9).astype(np.float32), np.ones(64, np.float32), np.zeros(64, np.float32))
    np.testing.assert_allclose(y3, y, rtol=1e-4, atol=1e-4)


def test_attention_closed_forms(oracle):
    rng = np.random.default_rng(19)
    T, D, heads = 7, 8, 2
    qkv = rng.standard_normal((T, 3 * D)).astype(np.float32)
    # zero queries -> uniform weights -> every output row is the mean of v
    q0 = qkv.copy(); q0[:, :D] = 0
    y = oracle.attention(q0, heads)
    np.testing.assert_allclose(y, np.broadcast_to(q0[:, 2 * D:].mean(0), (T, D)), rtol=1e-5, atol=1e-6)
    # general case against a float64 softmax written with matrix products per head
    y = oracle.attention(qkv, heads)
    want = np.empty((T, D))
    dh = D // heads
    for h in range(heads):
        q = qkv[:, h * dh:(h + 1) * dh].astype(np.float64); k = qkv[:, D + h * dh:D + (h + 1) * dh].astype(np.float64)
        v = qkv[:, 2 * D + h * dh:2 * D + (h + 1) * dh].astype(np.float64)
        s = q @ k.T / math.sqrt(dh)
        p = np.exp(s - s.max(1, keepdims=True)); p /= p.sum(1, keepdims=True)
        np.testing.assert_allclose(p.sum(1), 1, rtol=1e-12)
        want[:, h * dh:(h + 1) * dh] = p @ v
    np.testing.assert_allclose(y, want, rtol=1e-5, atol=1e-6)
    # heads are independent: permuting the channels of one head's v only permutes that head's output
    perm = qkv.copy(); perm[:, 2 * D:2 * D + dh] = qkv[:, 2 * D:2 * D + dh][:, ::-1]
    y2 = oracle.attention(perm, heads)
    np.testing.assert_allclose(y2[:, :dh], y[:, :dh][:, ::-1], rtol=1e-6)
    np.testing.assert_allclose(y2[:, dh:], y[:, dh:], rtol=1e-6)


def test_attention_bf16_rounds_the_softmax_probabilities(oracle):
    """Hand-worked case, bf16 expert, three tokens, one head of width 1 (scores = q k, no scaling).
    Keys (0, 0, 1), values (1, 3, -2); queries 1, 0, 1.
    Query 1: scores (0, 0, 1), minus the maximum (-1, -1, 0), exponentials (1/e, 1/e, 1), their sum 1.7357588823...,
    probabilities (0.2119415576..., 0.2119415576..., 0.5761168847...).  As bf16 (8 significant bits):
    0.2119415576 = 1.69553 x 2^-3 -> 217/128 x 2^-3 = 0.2119140625; 0.5761168847 = 1.15223 x 2^-1 -> 147/256 = 0.57421875.
    Output = 0.2119140625 x (1 + 3) + 0.57421875 x (-2) = -0.30078125, which is a bf16 value (-154/512).
    Rounding the exponentials instead and dividing by their unrounded sum afterwards would give -0.306640625, rounding
    nothing before the sum -0.3046875: the three readings differ in the stored bits.
    Query 0: uniform probabilities 1/3 -> bf16 171/512 = 0.333984375; output 0.333984375 x (1 + 3 - 2) = 0.66796875."""
    qkv = np.array([[1, 0, 1], [0, 0, 3], [1, 1, -2]], np.float32)
    y = oracle.attention(qkv, 1, dtype=1).reshape(-1)
    assert y.tolist() == [-0.30078125, 0.66796875, -0.30078125]
    assert -0.30078125 != -0.306640625 != -0.3046875
    # the fp32 expert keeps the probabilities unrounded: -0.30466... to fp32 precision
    y32 = oracle.attention(qkv, 1, dtype=0).reshape(-1)
    e = math.exp(-1.0)
    want = (e * 1 + e * 3 - 2.0) / (1 + 2 * e)
    np.testing.assert_allclose(y32[[0, 2]], want, rtol=1e-6)
    assert abs(float(y32[0]) - (-0.30078125)) > 1e-3


def test_gelu_via_1x1_conv(oracle):
    # act=2 on an identity 1x1 conv exposes the activation: GELU(0)=0, GELU(x)->x for large x, GELU(x)-GELU(-x)=x
    xs = np.array([0.0, 1.0, -1.0, 6.0, -6.0, 0.5, -0.5], np.float32)
    x = xs.reshape(1, -1, 1)
    y = oracle.conv2d(x, np.ones((1, 1, 1, 1), np.float32), np.zeros(1, np.float32), act=2).reshape(-1)
    assert y[0] == 0
    np.testing.assert_allclose(y[1], 0.8413447460685429, rtol=1e-6)     # Phi(1)
    np.testing.assert_allclose(y[3], 6.0, rtol=1e-6)
    assert abs(y[4]) < 1e-7
    np.testing.assert_allclose(y[1] - y[2], 1.0, rtol=1e-6)
    np.testing.assert_allclose(y[5] - y[6], 0.5, rtol=1e-6)


def test_detector_ops(oracle):
    """Concatenation, upsampling, SiLU and the detection read-out of detector-shaped experts against closed forms."""
    rng = np.random.default_rng(23)
    a = rng.standard_normal((3, 5, 8)).astype(np.float32); b = rng.standard_normal((3, 5, 16)).astype(np.float32)
    assert np.array_equal(oracle.concat(a, b), np.concatenate([a, b], axis=2))
    up = oracle.upsample2(a)
    assert up.shape == (6, 10, 8) and np.array_equal(up[::2, ::2], a) and np.array_equal(up[1::2, 1::2], a)
    assert np.array_equal(up[::2, 1::2], a) and np.array_equal(up[1::2, ::2], a)
    # SiLU through an identity 1x1 conv: SiLU(0) = 0, SiLU(1) = 1 / (1 + 1/e), SiLU(x) -> x for large x, SiLU(x) - SiLU(-x) = x
    xs = np.array([0.0, 1.0, -1.0, 20.0, -20.0, 0.5, -0.5], np.float32).reshape(1, -1, 1)
    y = oracle.conv2d(xs, np.ones((1, 1, 1, 1), np.float32), np.zeros(1, np.float32), act=3).reshape(-1)
    assert y[0] == 0
    np.testing.assert_allclose(y[1], 1.0 / (1.0 + math.exp(-1.0)), rtol=1e-6)
    np.testing.assert_allclose(y[3], 20.0, rtol=1e-6)
    assert abs(y[4]) < 1e-6
    np.testing.assert_allclose(y[1] - y[2], 1.0, rtol=1e-6)
    np.testing.assert_allclose(y[5] - y[6], 0.5, rtol=1e-6)
    # detection read-out by hand: one anchor, two classes, boxes (x, y, w, h, objectness, class 0, class 1).
    # All-zero logits: sigmoid(0)^2 = 0.25 for both classes.  One confident box (objectness 30, class 1 logit 30): class 1 -> 1,
    # class 0 stays 0.25 unless a box beats it; a box with objectness ln 3 (sigmoid 0.75) and class 0 logit ln 3: 0.5625.
    m = np.zeros((2, 2, 7), np.float32)
    assert oracle.det_head([m], 1, 2).tolist() == [0.25, 0.25]
    m[0, 1, 4] = 30.0; m[0, 1, 6] = 30.0
    m[1, 0, 4] = math.log(3.0); m[1, 0, 5] = math.log(3.0)
    got = oracle.det_head([m], 1, 2)
    np.testing.assert_allclose(got, [0.5625, 1.0], rtol=1e-6)
    # a second map can only raise the scores; the order of positions does not matter; two anchors per position
    m2 = np.zeros((1, 1, 7), np.float32); m2[0, 0, 4] = 30.0; m2[0, 0, 5] = 30.0
    np.testing.assert_allclose(oracle.det_head([m, m2], 1, 2), [1.0, 1.0], rtol=1e-6)
    assert np.array_equal(oracle.det_head([m[::-1, ::-1].copy()], 1, 2), got)
    two = np.concatenate([m, m[::-1]], axis=2)                       # anchors side by side in the channel dimension
    np.testing.assert_allclose(oracle.det_head([two], 2, 2), got, rtol=1e-6)


def test_forward_detector_fp32_matches_numpy(oracle):
    # detector-shaped expert at 64x64 input, width 16: wiring of the cross-stage blocks, the pooling pyramid, the neck
    # (upsample + concatenation with the finer map) and the two-scale detection read-out against the independent walk
    a = W.detector(n_classes=3, hw=64, width=16, anchors=4, dtype=W.DT_F32)
    blob = W.make_expert_blob(a, 31, 0)
    x = W.make_inputs(a, 31, [4])[0]
    got = oracle.forward(a, blob, x)
    want = _np_forward_f64(a, blob, x)
    assert got.shape == (3,) and 0 < got.min() and got.max() < 1
    np.testing.assert_allclose(got, want, rtol=1e-4, atol=1e-6)


def test_forward_detector_bf16_close_to_unrounded(oracle):
    a = W.detector(n_classes=3, hw=64, width=16, anchors=4, dtype=W.DT_BF16)
    blob = W.make_expert_blob(a, 31, 0)
    xb = W.make_inputs(a, 31, [4])[0]
    got = oracle.forward(a, blob, xb)
    want = _np_forward_f64(a, blob, W.bf16_bits_to_f32(xb).reshape(xb.shape))
    assert np.max(np.abs(got - want)) / np.max(np.abs(want)) < 3e-2


def test_tokens(oracle):
    x = np.arange(6, dtype=np.float32).reshape(3, 2)
    cls = np.array([10, 20], np.float32)
    pos = np.arange(8, dtype=np.float32).reshape(4, 2) * 100
    y = oracle.tokens(x, cls, pos)
    assert y.tolist() == [[10, 120], [200, 301], [402, 503], [604, 705]]


# ---------------------------------------------------------------------------------------------
# whole-expert forward from descriptor + blob
# ---------------------------------------------------------------------------------------------
def _np_forward_f64(arch, blob, x, stop_at=-1):
    """Independent float64 walk of a conv/pool/head program using numpy matmul convolution, no rounding.
    stop_at >= 0: the tensor that layer wrote instead of the head's output."""
    bufs = {0: x.astype(np.float64)}
    for li, L in enumerate(arch.layers):
        op, src, dst, res, k, r, s, stride, pad, act = [int(v) for v in L[:10]]
        if li == stop_at + 1 and stop_at >= 0:
            return bufs[int(arch.layers[stop_at][2])]
        if op == W.OP_CONV:
            y = _conv_im2col(bufs[src], W.blob_tensor(arch, blob, li, "w"), W.blob_tensor(arch, blob, li, "b"), stride, pad)
            if res >= 0:
                y = y + bufs[res]
            if act == 1:
                y = np.maximum(y, 0)
            elif act == 2:
                y = 0.5 * y * (1.0 + np.vectorize(math.erf)(y / math.sqrt(2.0)))
            elif act == 3:
                y = y * (0.5 * (1.0 + np.tanh(0.5 * y)))          # x sigmoid(x), the logistic function written through tanh
            bufs[dst] = y
        elif op == W.OP_CONCAT:
            bufs[dst] = np.concatenate([bufs[src], bufs[res]], axis=2)
        elif op == W.OP_UPSAMPLE:
            bufs[dst] = np.repeat(np.repeat(bufs[src], 2, axis=0), 2, axis=1)
        elif op == W.OP_HEAD_DET:
            anchors = int(L[10])
            maps = [bufs[src]] + ([bufs[res]] if res >= 0 else [])
            boxes = np.concatenate([m.reshape(-1, 5 + k) for m in maps])          # [positions * anchors][5 + k]
            sig = lambda v: 0.5 * (1.0 + np.tanh(0.5 * v))
            return (sig(boxes[:, 4:5]) * sig(boxes[:, 5:])).max(axis=0)
        elif op == W.OP_TOKENS:
            t = bufs[src].reshape(-1, bufs[src].shape[2])
            t = np.concatenate([W.blob_tensor(arch, blob, li, "cls")[None].astype(np.float64), t], 0)
            bufs[dst] = (t + W.blob_tensor(arch, blob, li, "pos"))[:, None, :]
        elif op == W.OP_LAYERNORM:
            t = bufs[src]
            mu = t.mean(-1, keepdims=True); var = ((t - mu) ** 2).mean(-1, keepdims=True)
            bufs[dst] = (t - mu) / np.sqrt(var + 1e-6) * W.blob_tensor(arch, blob, li, "gamma") + W.blob_tensor(arch, blob, li, "beta")
        elif op == W.OP_ATTENTION:
            t = bufs[src][:, 0, :]; T, D3 = t.shape; D = D3 // 3; heads = int(L[10]); dh = D // heads
            y = np.empty((T, D))
            for h in range(heads):
                q = t[:, h * dh:(h + 1) * dh]; kk = t[:, D + h * dh:D + (h + 1) * dh]; v = t[:, 2 * D + h * dh:2 * D + (h + 1) * dh]
                sc = q @ kk.T / math.sqrt(dh)
                pr = np.exp(sc - sc.max(1, keepdims=True)); pr /= pr.sum(1, keepdims=True)
                y[:, h * dh:(h + 1) * dh] = pr @ v
            bufs[dst] = y[:, None, :]
        elif op == W.OP_HEAD_CLS:
            t = bufs[src][0, 0]
            mu = t.mean(); var = ((t - mu) ** 2).mean()
            nrm = (t - mu) / math.sqrt(var + 1e-6) * W.blob_tensor(arch, blob, li, "gamma") + W.blob_tensor(arch, blob, li, "beta")
            return W.blob_tensor(arch, blob, li, "w").astype(np.float64) @ nrm + W.blob_tensor(arch, blob, li, "b")
        elif op == W.OP_MAXPOOL:
            xin = bufs[src]; H, Wd, C = xin.shape
            xp = np.full((H + 2 * pad, Wd + 2 * pad, C), -np.inf); xp[pad:pad + H, pad:pad + Wd] = xin
            P = (H + 2 * pad - r) // stride + 1; Q = (Wd + 2 * pad - s) // stride + 1
            y = np.empty((P, Q, C))
            for p in range(P):
                for q in range(Q):
                    y[p, q] = xp[p * stride:p * stride + r, q * stride:q * stride + s].reshape(-1, C).max(0)
            bufs[dst] = y
        elif op == W.OP_HEAD:
            f = bufs[src].reshape(-1, bufs[src].shape[2]).mean(0)
            return W.blob_tensor(arch, blob, li, "w").astype(np.float64) @ f + W.blob_tensor(arch, blob, li, "b")
    raise AssertionError


def test_forward_tiny_cnn_fp32_matches_numpy(oracle):
    a = W.tiny_cnn(4, 16)
    blob = W.make_expert_blob(a, 99, 2)
    x = W.make_inputs(a, 99, [5])[0]
    got = oracle.forward(a, blob, x)
    want = _np_forward_f64(a, blob, x)
    np.testing.assert_allclose(got, want, rtol=1e-5, atol=1e-6)


def test_forward_resnet18_fp32_matches_numpy(oracle):
    # fp32 variant of the ResNet-18-shaped program at 32x32 input, width 8: checks wiring of residuals,
    # shortcuts, strides and blob offsets against the independent walk
    a = W.resnet18(5, 32, W.DT_F32, 8)
    blob = W.make_expert_blob(a, 7, 0)
    x = W.make_inputs(a, 7, [1])[0]
    np.testing.assert_allclose(oracle.forward(a, blob, x), _np_forward_f64(a, blob, x), rtol=1e-4, atol=1e-5)


def test_forward_resnet50_fp32_matches_numpy(oracle):
    a = W.resnet50(6, 32, W.DT_F32, 4)
    blob = W.make_expert_blob(a, 8, 3)
    x = W.make_inputs(a, 8, [2])[0]
    np.testing.assert_allclose(oracle.forward(a, blob, x), _np_forward_f64(a, blob, x), rtol=1e-4, atol=1e-5)


def test_forward_vit_fp32_matches_numpy(oracle):
    # small ViT-shaped expert (4x4 patches of 8x8, dim 32, 2 blocks, 2 heads): wiring of tokens, pre-LN blocks,
    # attention, GELU MLP, residuals, class-token head and blob offsets against the independent walk
    a = W.vit(5, hw=32, patch=8, dim=32, depth=2, heads=2, mlp=64, dtype=W.DT_F32)
    blob = W.make_expert_blob(a, 21, 0)
    x = W.make_inputs(a, 21, [3])[0]
    np.testing.assert_allclose(oracle.forward(a, blob, x), _np_forward_f64(a, blob, x), rtol=1e-4, atol=1e-5)


@pytest.mark.parametrize("make", [lambda: W.resnet18(5, 32, W.DT_F32, 8),
                                  lambda: W.vit(5, hw=32, patch=8, dim=32, depth=2, heads=2, mlp=64, dtype=W.DT_F32),
                                  lambda: W.detector(3, hw=32, width=8, anchors=4, dtype=W.DT_F32)])
def test_forward_layer_matches_numpy_at_every_layer(oracle, make):
    # the per-layer read-out used for the layer-wise error budget: every intermediate tensor of a forward against the
    # independent walk stopped at the same layer
    a = make()
    blob = W.make_expert_blob(a, 31, 1)
    x = W.make_inputs(a, 31, [4])[0]
    for li in range(a.n_layers - 1):
        got = oracle.forward_layer(a, blob, x, li)
        want = _np_forward_f64(a, blob, x, stop_at=li)
        assert got.shape == want.shape, li
        np.testing.assert_allclose(got, want, rtol=2e-4, atol=2e-5, err_msg=f"layer {li}")


def test_forward_vit_bf16_close_to_unrounded(oracle):
    a = W.vit(5, hw=32, patch=8, dim=32, depth=2, heads=2, mlp=64, dtype=W.DT_BF16)
    blob = W.make_expert_blob(a, 21, 0)
    xb = W.make_inputs(a, 21, [3])[0]
    got = oracle.forward(a, blob, xb)
    want = _np_forward_f64(a, blob, W.bf16_bits_to_f32(xb).reshape(xb.shape))
    assert np.max(np.abs(got - want)) / np.max(np.abs(want)) < 3e-2


def test_forward_bf16_close_to_unrounded(oracle):
    # bf16 storage rounding perturbs logits by O(2^-8) relative, not more: catches a wrong rounding point (e.g. truncation
    # bias) without depending on the oracle's own arithmetic
    a = W.resnet18(5, 32, W.DT_BF16, 8)
    blob = W.make_expert_blob(a, 7, 0)
    xb = W.make_inputs(a, 7, [1])[0]
    got = oracle.forward(a, blob, xb)
    want = _np_forward_f64(a, blob, W.bf16_bits_to_f32(xb).reshape(xb.shape))
    assert np.max(np.abs(got - want)) / np.max(np.abs(want)) < 2e-2


def test_macs_match_published_tables():
    # standard layer tables: ResNet-18 1.814 GMAC, ResNet-50 (stride on the 3x3) 4.087 GMAC, ViT-B/16 17.56 GMAC
    assert abs(bench.arch_macs(W.resnet18(1000)) / 1e9 - 1.8141) < 2e-3
    assert abs(bench.arch_macs(W.resnet50(1000)) / 1e9 - 4.0891) < 2e-3
    assert abs(bench.arch_macs(W.vit(1000)) / 1e9 - 17.5638) < 2e-3
    assert bench.arch_macs(W.tiny_cnn()) == 64 * 64 * 9 * (3 * 16 + 16 * 32 + 32 * 64) + 64 * 4
