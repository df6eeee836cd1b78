"""Pins of the operator-granular oracle (oracle/opgranular.py): training-mode batch normalisation
against hand-computed values, its defining moments and invariances and PyTorch's CPU float64
routine; ReLU and add against numpy; the operator chain against the fused oracle where the two
must agree."""
import math

import numpy as np
import pytest

import synth
from oracle import numeric as on
from oracle import opgranular as og


def test_bn_train_hand_computed():
    # two channels, four positions: channel 0 = [1,2,3,4] (mean 2.5, var 1.25), channel 1 = [0,2,0,2] (mean 1, var 1)
    x = np.array([[1, 0], [2, 2], [3, 0], [4, 2]], np.float32).reshape(2, 2, 1, 2)
    y = on.to_f64(og.bn_train(x, np.ones(2, np.float32), np.zeros(2, np.float32), 0.0, "f32"), "f32").reshape(4, 2)
    r = 1.0 / math.sqrt(1.25)
    assert np.allclose(y[:, 0], [-1.5 * r, -0.5 * r, 0.5 * r, 1.5 * r], rtol=0, atol=1e-7)
    assert np.allclose(y[:, 1], [-1, 1, -1, 1], rtol=0, atol=1e-7)
    # eps under the root (variance 1, eps 3 -> /2); gamma and beta per channel
    y = on.to_f64(og.bn_train(x, np.array([1, 4], np.float32), np.array([0, 10], np.float32), 3.0, "f32"), "f32").reshape(4, 2)
    assert np.allclose(y[:, 1], [8, 12, 8, 12], rtol=0, atol=1e-6)
    # statistics are over the batch AND the positions, per channel: one image alone gives other numbers
    y1 = on.to_f64(og.bn_train(x[:1], np.ones(2, np.float32), np.zeros(2, np.float32), 0.0, "f32"), "f32").reshape(2, 2)
    assert np.allclose(y1[:, 0], [-1, 1], rtol=0, atol=1e-7)
    # a constant channel: variance 0, beta comes out
    c = np.full((2, 3, 3, 1), 7.0, np.float32)
    assert np.array_equal(on.to_f64(og.bn_train(c, np.array([2], np.float32), np.array([5], np.float32), 1e-5, "f32"), "f32"),
                          np.full((2, 3, 3, 1), 5.0))


def test_bn_train_moments_invariance_and_torch():
    torch = pytest.importorskip("torch")
    N, H, W, C = 3, 5, 4, 6
    x = (synth.normal(81, 1, N * H * W * C).reshape(N, H, W, C) * 2 + 0.7).astype(np.float32)
    one, zero = np.ones(C, np.float32), np.zeros(C, np.float32)
    y = on.to_f64(og.bn_train(x, one, zero, 0.0, "f32"), "f32")
    assert np.max(np.abs(y.mean(axis=(0, 1, 2)))) < 1e-6 and np.max(np.abs(y.var(axis=(0, 1, 2)) - 1)) < 1e-5
    a = np.array([0.5, 2, 4, 1, 8, 0.25], np.float32)
    c = np.array([1, -2, 0.5, 0, 3, -1], np.float32)
    y2 = on.to_f64(og.bn_train(x * a + c, one, zero, 0.0, "f32"), "f32")     # per-channel affine map of the input
    assert np.max(np.abs(y - y2)) < 2e-5
    g = synth.uniform(81, 2, C, 0.5, 1.5).astype(np.float32)
    b = synth.normal(81, 3, C, 0.0, 0.1).astype(np.float32)
    got = on.to_f64(og.bn_train(x, g, b, 1e-5, "f32"), "f32")
    xt = torch.from_numpy(x).double().permute(0, 3, 1, 2)
    ref = torch.nn.functional.batch_norm(xt, None, None, torch.from_numpy(g).double(), torch.from_numpy(b).double(),
                                         training=True, eps=1e-5).permute(0, 2, 3, 1).numpy()
    assert np.max(np.abs(got - ref)) < 1e-6


def test_relu_and_add_are_the_numpy_operations_rounded_once():
    x = synth.f32_to_bf16_bits(synth.normal(82, 1, 64).astype(np.float32))
    r = synth.f32_to_bf16_bits(synth.normal(82, 2, 64).astype(np.float32))
    xf, rf = synth.bf16_bits_to_f32(x).astype(np.float64), synth.bf16_bits_to_f32(r).astype(np.float64)
    assert np.array_equal(on.to_f64(og.relu(x, "bf16"), "bf16"), np.where(xf > 0, xf, 0.0))
    s = on.to_f64(og.add(x, r, "bf16"), "bf16")
    assert np.max(np.abs(s - (xf + rf))) <= 2.0 ** -8 * np.max(np.abs(xf + rf))
    assert int(og.add(np.array([0x3F80], np.uint16), np.array([0x3B80], np.uint16), "bf16")[0]) == 0x3F80   # 1 + 2^-8: tie to even


def test_chain_equals_the_fused_layer_when_the_statistics_are_given():
    """conv -> bn -> add -> relu with the batch's own statistics equals the fused oracle layer that
    is handed those statistics as its frozen ones (float32 storage: the fused layer rounds once,
    the chain after every operator, so agreement is to float32 rounding)."""
    layers = synth.bottleneck_stack(2, 6, 6, cin=8, mid=8, cout=16, nblocks=1)
    x0 = synth.make_input(83, (2, 6, 6, 8), "f32")
    params = {l.name: synth.make_params(83, l, "f32") for l in layers}
    acts = og.run_ops(layers, params, x0, "f32")
    alias = {"x0": "x0"}
    for l in layers:
        conv = on.to_f64(acts[l.name + ".conv"], "f32")
        p = dict(params[l.name])
        p["mean"] = conv.mean(axis=(0, 1, 2)).astype(np.float32)
        p["var"] = conv.var(axis=(0, 1, 2)).astype(np.float32)
        fused = on.conv_bn_act(acts[alias[l.x]], p["w"], p, res=acts[alias[l.res]] if l.res else None, stride=l.stride,
                               pad=l.pad, relu=l.relu, dtype="f32")
        last = l.name + (".relu" if l.relu else (".add" if l.res else ".bn"))
        alias[l.y] = last
        err = np.max(np.abs(on.to_f64(fused, "f32") - on.to_f64(acts[last], "f32")))
        assert err < 1e-4, (l.name, err)
    names = set(acts)
    assert {"b1.out.conv", "b1.out.bn", "b1.out.add", "b1.out.relu"} <= names or any(n.endswith(".add") for n in names)


def test_bn_train_bwd_hand_computed():
    # one channel, two positions x = [0, 2]: mu 1, var 1, eps 0 -> xhat = [-1, 1]; y does not change when
    # x moves (two points always normalise to -1, +1), so gx = 0 whatever gy is
    x = np.array([0, 2], np.float32).reshape(2, 1, 1, 1)
    gy = np.array([3, -5], np.float32).reshape(2, 1, 1, 1)
    gx, dg, db = og.bn_train_bwd(x, np.array([2], np.float32), gy, 0.0, "f32")
    assert np.max(np.abs(on.to_f64(gx, "f32"))) < 1e-12
    assert abs(dg[0] - (3 * -1 + -5 * 1)) < 1e-12 and abs(db[0] - (-2)) < 1e-12
    # with eps = 3 the two points sit at -1/2, +1/2 and do move: y_i = gamma (x_i - mu) / sqrt(var + 3),
    # var = d^2/4 with d = x1 - x0 = 2; y1 = gamma (d/2) / sqrt(d^2/4 + 3) -> dy1/dd = gamma * (3/2) / (d^2/4+3)^(3/2)
    # = 2 * 1.5 / 8 = 0.375; dy0/dd = -0.375; dL/dd = gy1 * .375 - gy0 * .375 = -3; gx = [-dL/dd, dL/dd] = [3, -3]
    gx, dg, db = og.bn_train_bwd(x, np.array([2], np.float32), gy, 3.0, "f32")
    assert np.allclose(on.to_f64(gx, "f32").reshape(2), [3.0, -3.0], rtol=0, atol=1e-6)
    assert abs(dg[0] - (3 * -0.5 + -5 * 0.5)) < 1e-12


def test_bn_train_bwd_finite_differences_invariants_and_torch():
    torch = pytest.importorskip("torch")
    N, H, W, C = 2, 3, 4, 5
    x = (synth.normal(83, 1, N * H * W * C).reshape(N, H, W, C) * 1.5 + 0.4).astype(np.float32)
    gy = synth.normal(83, 2, N * H * W * C).reshape(N, H, W, C).astype(np.float32)
    g = synth.uniform(83, 3, C, 0.5, 1.5).astype(np.float32)
    b = synth.normal(83, 4, C, 0.0, 0.1).astype(np.float32)
    eps = 1e-3
    gx, dg, db = og.bn_train_bwd(x, g, gy, eps, "f32")
    gx = on.to_f64(gx, "f32")
    # central differences of L = sum gy * bn(x) on the unrounded forward, every element of x
    v = x.astype(np.float64)
    w = gy.astype(np.float64)
    h = 1e-5
    num = np.empty_like(v)
    for i in np.ndindex(*v.shape):
        vp, vm = v.copy(), v.copy()
        vp[i] += h
        vm[i] -= h
        num[i] = ((w * og.bn_train_f64(vp, g, b, eps)).sum() - (w * og.bn_train_f64(vm, g, b, eps)).sum()) / (2 * h)
    assert np.max(np.abs(gx - num)) < 1e-6
    # gamma and beta by differences too (the forward is linear in both: exact up to the float32 rounding of g + 1, b + 1)
    for c in range(C):
        e = np.zeros(C, np.float32)
        e[c] = 1
        assert abs((w * (og.bn_train_f64(v, g + e, b, eps) - og.bn_train_f64(v, g, b, eps))).sum() - dg[c]) < 1e-5
        assert abs((w * (og.bn_train_f64(v, g, b + e, eps) - og.bn_train_f64(v, g, b, eps))).sum() - db[c]) < 1e-5
    # the output is unchanged by a shift or (eps = 0) a rescaling of a channel, so gx has no component along 1 or x - mu
    gx0 = on.to_f64(og.bn_train_bwd(x, g, gy, 0.0, "f32")[0], "f32")
    assert np.max(np.abs(gx.sum(axis=(0, 1, 2)))) < 1e-5
    assert np.max(np.abs((gx0 * (v - v.mean(axis=(0, 1, 2)))).sum(axis=(0, 1, 2)))) < 1e-5
    # PyTorch's CPU float64 autograd through its own batch-norm routine
    xt = torch.from_numpy(x).double().permute(0, 3, 1, 2).requires_grad_(True)
    gt = torch.from_numpy(g).double().requires_grad_(True)
    bt = torch.from_numpy(b).double().requires_grad_(True)
    yt = torch.nn.functional.batch_norm(xt, None, None, gt, bt, training=True, eps=eps)
    (yt * torch.from_numpy(gy).double().permute(0, 3, 1, 2)).sum().backward()
    assert np.max(np.abs(gx - xt.grad.permute(0, 2, 3, 1).numpy())) < 1e-6
    assert np.max(np.abs(dg - gt.grad.numpy())) < 1e-9 and np.max(np.abs(db - bt.grad.numpy())) < 1e-9


def test_relu_bwd_masks_on_the_stored_output():
    y = synth.f32_to_bf16_bits(np.array([1.5, 0.0, -0.0, -2.0, 3e-39, 7.0], np.float32))
    gy = synth.f32_to_bf16_bits(np.array([1, 2, 3, 4, 5, -6], np.float32))
    got = on.to_f64(og.relu_bwd(y, gy, "bf16"), "bf16")
    assert np.array_equal(got[[0, 1, 2, 3, 5]], [1, 0, 0, 0, -6])
