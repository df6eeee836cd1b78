"""Pins of the numeric oracle (oracle/conv_ref.c) against things other than itself:
library matrix products, closed forms, invariants and hand-rounded bit patterns."""
import os

import numpy as np
import pytest

import synth
from oracle import numeric as on

GOLD = os.path.join(os.path.dirname(__file__), "golden")
rs = np.random.RandomState(7)


def _bn_identity(C):
    # gamma=1, beta=0, mean=0, var=1-eps  =>  u = z exactly
    return dict(gamma=np.ones(C, np.float32), beta=np.zeros(C, np.float32),
                mean=np.zeros(C, np.float32), var=np.full(C, 1.0, np.float32), eps=0.0)


def test_1x1_is_a_matrix_product():
    x = rs.randn(2, 5, 7, 12).astype(np.float32)
    w = rs.randn(9, 1, 1, 12).astype(np.float32)
    _, y64 = on.conv_bn_act(x, w, None, relu=False, want_f64=True)
    ref = x.reshape(-1, 12).astype(np.float64) @ w.reshape(9, 12).astype(np.float64).T
    np.testing.assert_allclose(y64.reshape(-1, 9), ref, rtol=1e-13, atol=1e-13)


def test_kxk_against_explicit_im2col_matmul():
    # independent formulation: gather patches with numpy slicing, then one matmul
    N, H, W, C, K, R, S, stride, pad = 2, 9, 8, 5, 4, 3, 3, 2, 1
    x = rs.randn(N, H, W, C).astype(np.float32)
    w = rs.randn(K, R, S, C).astype(np.float32)
    _, y64 = on.conv_bn_act(x, w, None, stride=stride, pad=pad, relu=False, want_f64=True)
    xp = np.zeros((N, H + 2 * pad, W + 2 * pad, C))
    xp[:, pad:pad + H, pad:pad + W] = x
    P, Q = (H + 2 * pad - R) // stride + 1, (W + 2 * pad - S) // stride + 1
    cols = np.stack([xp[:, r:r + stride * P:stride, s:s + stride * Q:stride]
                     for r in range(R) for s in range(S)], axis=3)      # N,P,Q,RS,C
    ref = cols.reshape(N * P * Q, R * S * C) @ w.reshape(K, -1).astype(np.float64).T
    assert y64.shape == (N, P, Q, K)
    np.testing.assert_allclose(y64.reshape(-1, K), ref, rtol=1e-12, atol=1e-12)


def test_centre_tap_identity_reproduces_input():
    C = 6
    x = rs.randn(1, 7, 7, C).astype(np.float32)
    w = np.zeros((C, 3, 3, C), np.float32)
    for c in range(C):
        w[c, 1, 1, c] = 1.0
    y = on.conv_bn_act(x, w, None, pad=1, relu=False)
    assert np.array_equal(y, x)


def test_off_centre_tap_shifts_the_right_way():
    # w[k, r=0, s=2] = 1 picks x[p-1, q+1]: catches transposed r/s or a wrong sign of the shift
    x = rs.randn(1, 6, 6, 1).astype(np.float32)
    w = np.zeros((1, 3, 3, 1), np.float32)
    w[0, 0, 2, 0] = 1.0
    y = on.conv_bn_act(x, w, None, pad=1, relu=False)
    ref = np.zeros_like(x)
    ref[0, 1:, :-1, 0] = x[0, :-1, 1:, 0]
    assert np.array_equal(y, ref)


def test_all_ones_counts_padding():
    C = 4
    x = np.ones((1, 5, 6, C), np.float32)
    w = np.ones((2, 3, 3, C), np.float32)
    y = on.conv_bn_act(x, w, None, pad=1, relu=False)
    assert np.all(y[0, 1:-1, 1:-1] == 9 * C)
    assert np.all(y[0, 0, 1:-1] == 6 * C) and np.all(y[0, 1:-1, 0] == 6 * C)
    for (p, q) in ((0, 0), (0, -1), (-1, 0), (-1, -1)):
        assert np.all(y[0, p, q] == 4 * C)


def test_linearity_in_fp64():
    w = rs.randn(5, 3, 3, 3).astype(np.float32)
    a, b = 2.0, -0.5
    f = lambda x: on.conv_bn_act(x, w, None, pad=1, relu=False, want_f64=True)[1]
    # use inputs whose combination is exactly representable: small integers
    x1 = rs.randint(-8, 8, (1, 6, 6, 3)).astype(np.float32)
    x2 = rs.randint(-8, 8, (1, 6, 6, 3)).astype(np.float32)
    np.testing.assert_allclose(f(a * x1 + b * x2), a * f(x1) + b * f(x2), rtol=1e-13, atol=1e-12)


def test_stride2_is_subsampled_stride1():
    x = rs.randn(2, 9, 9, 4).astype(np.float32)
    w = rs.randn(3, 3, 3, 4).astype(np.float32)
    y1 = on.conv_bn_act(x, w, None, stride=1, pad=1, relu=False)
    y2 = on.conv_bn_act(x, w, None, stride=2, pad=1, relu=False)
    assert np.array_equal(y2, y1[:, ::2, ::2])
    w1 = rs.randn(3, 1, 1, 4).astype(np.float32)
    assert np.array_equal(on.conv_bn_act(x, w1, None, stride=2, relu=False),
                          on.conv_bn_act(x, w1, None, stride=1, relu=False)[:, ::2, ::2])


def test_bn_identity_and_closed_form():
    C = 5
    x = rs.randn(1, 4, 4, C).astype(np.float32)
    w = np.zeros((C, 1, 1, C), np.float32)
    w[np.arange(C), 0, 0, np.arange(C)] = 1.0
    assert np.array_equal(on.conv_bn_act(x, w, _bn_identity(C), relu=False), x)
    # constants: z = 3 everywhere; u = gamma*(3-mean)/sqrt(var+eps)+beta
    x = np.full((1, 2, 2, 1), 3.0, np.float32)
    w = np.ones((2, 1, 1, 1), np.float32)
    bn = dict(gamma=np.array([2.0, 0.5], np.float32), beta=np.array([1.0, -1.0], np.float32),
              mean=np.array([1.0, 5.0], np.float32), var=np.array([3.0, 0.25 - 1e-5], np.float32),
              eps=1.0)
    _, y64 = on.conv_bn_act(x, w, bn, relu=False, want_f64=True)
    np.testing.assert_allclose(y64[0, 0, 0, 0], 2.0 * 2.0 / 2.0 + 1.0, rtol=1e-15)
    v1 = float(np.float32(0.25 - 1e-5)) + 1.0
    np.testing.assert_allclose(y64[0, 0, 0, 1], 0.5 * (-2.0) / np.sqrt(v1) - 1.0, rtol=1e-15)


def test_relu_and_residual():
    C = 3
    x = rs.randn(1, 4, 4, C).astype(np.float32)
    w = np.zeros((C, 1, 1, C), np.float32)
    res = rs.randn(1, 4, 4, C).astype(np.float32)
    bn = _bn_identity(C)
    bn["beta"] = np.array([0.5, -0.5, 0.0], np.float32)
    # zero weights: y = relu(shift + residual); residual is added BEFORE the ReLU
    y = on.conv_bn_act(x, w, bn, res=res, relu=True)
    ref = np.maximum(res.astype(np.float64) + bn["beta"].astype(np.float64), 0).astype(np.float32)
    assert np.array_equal(y, ref)
    # idempotent
    eye = np.zeros((C, 1, 1, C), np.float32)
    eye[np.arange(C), 0, 0, np.arange(C)] = 1.0
    assert np.array_equal(on.conv_bn_act(y, eye, None, relu=True), y)
    # without relu negative values survive
    y2 = on.conv_bn_act(x, eye, None, relu=False)
    assert (y2 < 0).any() and np.array_equal(y2, x)


def test_bf16_rounding_golden():
    for line in open(os.path.join(GOLD, "bf16_rounding.txt")):
        if line.startswith("#") or not line.strip():
            continue
        f32, b16 = line.split()[:2]
        v = np.array([int(f32, 16)], np.uint32).view(np.float32)[0]
        assert on.double_to_bf16(float(v)) == int(b16, 16), line
        # the input generator's rounding must agree on the same patterns
        assert int(synth.f32_to_bf16_bits(np.array([v], np.float32))[0]) == int(b16, 16), line
    assert on.double_to_bf16(float("nan")) & 0x7FC0 == 0x7FC0
    # a double that fp32 would round first the wrong way: 1 + 2^-8 + 2^-30 (above the tie)
    assert on.double_to_bf16(1.0 + 2.0**-8 + 2.0**-30) == 0x3F81
    assert on.double_to_bf16(1.0 + 2.0**-8) == 0x3F80
    for b in (0x0000, 0x3F80, 0xC049, 0x0001, 0x7F7F):
        assert on.double_to_bf16(on.bf16_to_double(b)) == b


def test_bf16_layer_uses_stored_bits_and_rounds_once():
    x = synth.f32_to_bf16_bits(rs.randn(1, 5, 5, 8).astype(np.float32)).reshape(1, 5, 5, 8)
    w = synth.f32_to_bf16_bits(rs.randn(4, 3, 3, 8).astype(np.float32)).reshape(4, 3, 3, 8)
    y, y64 = on.conv_bn_act(x, w, None, pad=1, relu=True, dtype="bf16", want_f64=True)
    xf, wf = on.to_f64(x, "bf16"), on.to_f64(w, "bf16")
    _, ref64 = on.conv_bn_act(xf.astype(np.float32), wf.astype(np.float32), None, pad=1,
                              relu=True, dtype="f32", want_f64=True)
    np.testing.assert_array_equal(y64, ref64)           # same operands, same fp64 arithmetic
    back = on.to_f64(y, "bf16")
    assert np.all(np.abs(back - y64) <= np.abs(y64) * 2.0**-8 + 1e-38)   # half an ulp


def test_maxpool_and_avgpool():
    x = rs.randn(2, 6, 6, 3).astype(np.float32)
    y = on.maxpool(x, 3, 3, 2, 1)
    xp = np.full((2, 8, 8, 3), -np.inf, np.float32)
    xp[:, 1:7, 1:7] = x
    ref = np.max(np.stack([xp[:, r:r + 6:2, s:s + 6:2] for r in range(3) for s in range(3)]), axis=0)
    assert np.array_equal(y, ref)
    a = on.avgpool(x)
    np.testing.assert_allclose(a[:, 0, 0], x.astype(np.float64).mean(axis=(1, 2)), rtol=1e-6)


def test_rerun_is_bit_identical():
    L = synth.bottleneck_stack(1, 8, 8)[:2]
    P = {l.name: synth.make_params(3, l, "f32") for l in L}
    x = synth.make_input(3, (1, 8, 8, 64), "f32")
    a = on.run_layers(L, P, x, "f32")
    b = on.run_layers(L, P, x, "f32")
    for k in a:
        assert a[k].tobytes() == b[k].tobytes()


def test_rejects_bad_arguments():
    x = np.zeros((1, 2, 2, 1), np.float32)
    w = np.zeros((1, 5, 5, 1), np.float32)
    with pytest.raises(ValueError):
        on.conv_bn_act(x, w, None)      # kernel larger than the unpadded image


def test_softmax_cross_entropy_closed_forms():
    # uniform logits: every class has probability 1/C, the loss is ln C whatever the labels
    C, N = 37, 5
    z = np.full((N, C), 2.5, np.float32)
    labels = np.arange(N) % C
    np.testing.assert_allclose(on.softmax_ce(z, labels)[0], np.log(C), rtol=1e-6)
    # two classes: loss = log(1 + exp(-(z_label - z_other)))
    z = np.array([[3.0, 1.0], [0.5, 2.0]], np.float32)
    want = np.mean([np.log1p(np.exp(-2.0)), np.log1p(np.exp(1.5))])
    np.testing.assert_allclose(on.softmax_ce(z, np.array([0, 0]))[0], want, rtol=1e-6)
    # shift invariance and a dominant correct class
    z = rs.randn(4, 9).astype(np.float32)
    lab = np.array([1, 2, 3, 4])
    np.testing.assert_allclose(on.softmax_ce(z + 100.0, lab)[0], on.softmax_ce(z, lab)[0], rtol=1e-4)
    z[np.arange(4), lab] = 60.0
    assert on.softmax_ce(z, lab)[0] < 1e-12 + 1e-6
    # bf16 logits are read at their stored value
    zb = synth.f32_to_bf16_bits(z).reshape(z.shape)
    np.testing.assert_allclose(on.softmax_ce(zb, lab, "bf16")[0],
                               on.softmax_ce(synth.bf16_bits_to_f32(zb).reshape(z.shape), lab)[0], rtol=1e-7)


def test_classifier_is_matmul_plus_bias():
    l = synth.LayerSpec("fc", "fc", "x0", None, "logits", 3, 1, 1, 16, 24, 1, 1, 1, 0, False)
    l.index = 1
    p = {"fc": synth.make_params(9, l, "f32")}
    x = synth.make_input(9, (3, 1, 1, 16), "f32")
    got = on.run_layers([l], p, x, "f32")["logits"].reshape(3, 24)
    ref = x.reshape(3, 16).astype(np.float64) @ p["fc"]["w"].reshape(24, 16).astype(np.float64).T + p["fc"]["bias"]
    np.testing.assert_allclose(got, ref, rtol=1e-6, atol=1e-6)
