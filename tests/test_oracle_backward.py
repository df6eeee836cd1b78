"""Pins for the oracle's backward of the fused layer (CPU only).

Nothing here re-types the oracle's loops: the gradient is checked against central finite
differences of the oracle's own *forward* (already pinned in test_oracle_numeric.py), against
the adjoint identity of a linear map, against library matrix products in the 1x1 case, and
against hand-made cases whose answer is known in closed form.  A dropped term, a wrong sign,
a transposed operand or a wrong tap index fails at least one of them."""
import numpy as np
import pytest

import synth
from oracle import numeric as on


def _rand(shape, seed, scale=1.0):
    """Seeded normals on a grid of 2^-8, so that adding or subtracting a finite-difference step
    that is a power of two (>= 2^-12) is exact in fp32."""
    n = int(np.prod(shape))
    return (np.round(synth.normal(seed, 7, n) * scale * 256.0) / 256.0).astype(np.float32).reshape(shape)


def _bn(C, seed):
    return {"gamma": (1.0 + 0.25 * synth.normal(seed, 1, C)).astype(np.float32),
            "beta": (0.1 * synth.normal(seed, 2, C)).astype(np.float32),
            "mean": (0.1 * synth.normal(seed, 3, C)).astype(np.float32),
            "var": synth.uniform(seed, 4, C, 1.0, 1.5).astype(np.float32), "eps": 1e-5}


def _loss(x, w, bn, R_, stride, pad, relu, res=None):
    """L = sum(y * R_) with y the oracle's forward before its final rounding (fp64)."""
    _, y64 = on.conv_bn_act(x, w, bn, res=res, stride=stride, pad=pad, relu=relu, dtype="f32", want_f64=True)
    return float(np.sum(y64 * R_))


CASES = [
    # N  H  W  Cin Cout R stride pad
    (2, 5, 6, 3, 4, 3, 1, 1),
    (1, 7, 7, 2, 3, 3, 2, 1),       # stride 2
    (2, 4, 4, 5, 2, 1, 1, 0),       # 1x1
    (1, 6, 5, 2, 2, 1, 2, 0),       # 1x1 stride 2
    (1, 6, 6, 2, 3, 5, 1, 2),       # 5x5
]


@pytest.mark.parametrize("case", CASES)
def test_gradients_match_finite_differences_of_the_forward(case):
    """No ReLU (the forward is then linear in x and in w, so central differences are exact up
    to rounding): dL/dx and dL/dw for L = <y, R>."""
    N, H, W, Cin, Cout, R, stride, pad = case
    x = _rand((N, H, W, Cin), 11)
    w = _rand((Cout, R, R, Cin), 12, 0.5)
    bn = _bn(Cout, 13)
    P = (H + 2 * pad - R) // stride + 1
    Q = (W + 2 * pad - R) // stride + 1
    Rw = _rand((N, P, Q, Cout), 14)
    gx, gw, gpre = on.conv_bn_act_bwd(x, w, bn, None, Rw, stride=stride, pad=pad, relu=False, dtype="f32")
    assert np.array_equal(gpre, Rw.astype(np.float64))
    h = 2.0 ** -6                    # exactly representable steps keep x +- h in fp32
    rng = np.random.default_rng(5)
    for _ in range(12):
        idx = tuple(int(rng.integers(0, s)) for s in x.shape)
        xp, xm = x.copy(), x.copy()
        xp[idx] += h
        xm[idx] -= h
        fd = (_loss(xp, w, bn, Rw, stride, pad, False) - _loss(xm, w, bn, Rw, stride, pad, False)) / (2 * h)
        assert abs(fd - gx[idx]) <= 1e-7 * max(1.0, abs(fd)), (idx, fd, gx[idx])
    for _ in range(12):
        idx = tuple(int(rng.integers(0, s)) for s in w.shape)
        wp, wm = w.copy(), w.copy()
        wp[idx] += h
        wm[idx] -= h
        fd = (_loss(x, wp, bn, Rw, stride, pad, False) - _loss(x, wm, bn, Rw, stride, pad, False)) / (2 * h)
        assert abs(fd - gw[idx]) <= 1e-7 * max(1.0, abs(fd)), (idx, fd, gw[idx])


def test_relu_mask_uses_the_stored_output_and_residual_gets_the_masked_gradient():
    """With ReLU and a residual: finite differences where the pre-activation is away from the
    kink; entries with y = 0 get no gradient; dL/dres equals the masked gradient."""
    N, H, W, Cin, Cout, R, stride, pad = 2, 5, 5, 3, 4, 3, 1, 1
    x = _rand((N, H, W, Cin), 21)
    w = _rand((Cout, R, R, Cin), 22, 0.5)
    bn = _bn(Cout, 23)
    res = _rand((N, H, W, Cout), 24)
    Rw = _rand((N, H, W, Cout), 25)
    y, y64 = on.conv_bn_act(x, w, bn, res=res, stride=stride, pad=pad, relu=True, dtype="f32", want_f64=True)
    gx, gw, gpre = on.conv_bn_act_bwd(x, w, bn, y, Rw, stride=stride, pad=pad, relu=True, dtype="f32")
    assert np.array_equal(gpre, np.where(y > 0, Rw, 0).astype(np.float64))
    assert (y == 0).any() and (y > 0).any()
    # finite differences with a step small against the distance of every pre-activation to 0
    _, v64 = on.conv_bn_act(x, w, bn, res=res, stride=stride, pad=pad, relu=False, dtype="f32", want_f64=True)
    margin = np.min(np.abs(v64))
    h = 2.0 ** -12
    a_max = float(np.max(np.abs(bn["gamma"]) / np.sqrt(bn["var"])))
    assert margin > 4 * h * max(1.0, float(np.max(np.abs(w))) * a_max)   # no pre-activation crosses 0 within +-h
    rng = np.random.default_rng(6)
    for _ in range(10):
        idx = tuple(int(rng.integers(0, s)) for s in x.shape)
        xp, xm = x.copy(), x.copy()
        xp[idx] += h
        xm[idx] -= h
        fd = (_loss(xp, w, bn, Rw, stride, pad, True, res) - _loss(xm, w, bn, Rw, stride, pad, True, res)) / (2 * h)
        assert abs(fd - gx[idx]) <= 1e-6 * max(1.0, abs(fd)), (idx, fd, gx[idx])
    # residual: dL/dres by finite differences at a few positions
    for _ in range(6):
        idx = tuple(int(rng.integers(0, s)) for s in res.shape)
        rp, rm = res.copy(), res.copy()
        rp[idx] += h
        rm[idx] -= h
        fd = (_loss(x, w, bn, Rw, stride, pad, True, rp) - _loss(x, w, bn, Rw, stride, pad, True, rm)) / (2 * h)
        assert abs(fd - gpre[idx]) <= 1e-6 * max(1.0, abs(fd))


@pytest.mark.parametrize("case", CASES)
def test_adjoint_identity(case):
    """Without batch-norm and ReLU the layer is the linear map x -> conv(x, w); its backward is
    the transpose: <g, conv(x', w)> = <conv^T(g), x'> and = <dL/dw(g, x'), w> for any x'."""
    N, H, W, Cin, Cout, R, stride, pad = case
    w = _rand((Cout, R, R, Cin), 31, 0.5)
    xq = _rand((N, H, W, Cin), 32)
    P = (H + 2 * pad - R) // stride + 1
    Q = (W + 2 * pad - R) // stride + 1
    g = _rand((N, P, Q, Cout), 33)
    _, y64 = on.conv_bn_act(xq, w, None, stride=stride, pad=pad, relu=False, dtype="f32", want_f64=True)
    gx, gw, _ = on.conv_bn_act_bwd(xq, w, None, None, g, stride=stride, pad=pad, relu=False, dtype="f32")
    lhs = float(np.sum(g.astype(np.float64) * y64))
    assert abs(lhs - float(np.sum(gx * xq))) <= 1e-11 * max(1.0, abs(lhs))
    assert abs(lhs - float(np.sum(gw * w))) <= 1e-11 * max(1.0, abs(lhs))


def test_1x1_case_is_two_matrix_products():
    N, H, W, Cin, Cout = 2, 3, 4, 6, 5
    x = _rand((N, H, W, Cin), 41)
    w = _rand((Cout, 1, 1, Cin), 42)
    bn = _bn(Cout, 43)
    g = _rand((N, H, W, Cout), 44)
    gx, gw, _ = on.conv_bn_act_bwd(x, w, bn, None, g, relu=False, dtype="f32")
    a = bn["gamma"].astype(np.float64) / np.sqrt(bn["var"].astype(np.float64) + bn["eps"])
    gz = g.reshape(-1, Cout).astype(np.float64) * a
    np.testing.assert_allclose(gx.reshape(-1, Cin), gz @ w.reshape(Cout, Cin).astype(np.float64), rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(gw.reshape(Cout, Cin), gz.T @ x.reshape(-1, Cin).astype(np.float64), rtol=1e-12, atol=1e-12)


def test_single_tap_weight_gradient_counts_the_padding():
    """x = 1 everywhere, gy = 1 everywhere, no BN: dL/dw[k,r,s,c] is the number of output pixels
    whose tap (r,s) falls inside the image - (H - |r-1|) * (W - |s-1|) for 3x3, pad 1, stride 1;
    dL/dx at an interior pixel is the sum of all weights that reach it."""
    N, H, W, C, K = 2, 5, 4, 2, 3
    x = np.ones((N, H, W, C), np.float32)
    w = _rand((K, 3, 3, C), 51)
    g = np.ones((N, H, W, K), np.float32)
    gx, gw, _ = on.conv_bn_act_bwd(x, w, None, None, g, stride=1, pad=1, relu=False, dtype="f32")
    for r in range(3):
        for s in range(3):
            assert np.all(gw[:, r, s, :] == N * (H - abs(r - 1)) * (W - abs(s - 1)))
    np.testing.assert_allclose(gx[0, 2, 2, :], w.astype(np.float64).sum(axis=(0, 1, 2)), rtol=1e-12)
    # a corner pixel (0,0) is reached by output pixels (p,q) in {0,1}^2 through taps (1-p, 1-q)
    want = sum(w[:, 1 - p, 1 - q, :].astype(np.float64).sum(axis=0) for p in (0, 1) for q in (0, 1))
    np.testing.assert_allclose(gx[0, 0, 0, :], want, rtol=1e-12)


def test_bf16_operands_are_taken_at_their_stored_values():
    """bf16 storage: the backward widens the stored bit patterns exactly; with operands that are
    bf16-representable the bf16 and fp32 paths agree to the last bit of fp64."""
    N, H, W, Cin, Cout = 1, 4, 4, 4, 4
    xb = synth.f32_to_bf16_bits(_rand((N, H, W, Cin), 61)).reshape(N, H, W, Cin)
    wb = synth.f32_to_bf16_bits(_rand((Cout, 3, 3, Cin), 62)).reshape(Cout, 3, 3, Cin)
    gb = synth.f32_to_bf16_bits(_rand((N, H, W, Cout), 63)).reshape(N, H, W, Cout)
    bn = _bn(Cout, 64)
    yb = on.conv_bn_act(xb, wb, bn, stride=1, pad=1, relu=True, dtype="bf16")
    a = on.conv_bn_act_bwd(xb, wb, bn, yb, gb, stride=1, pad=1, relu=True, dtype="bf16")
    f = lambda t: on.to_f64(t, "bf16").astype(np.float32)
    b = on.conv_bn_act_bwd(f(xb), f(wb), bn, f(yb), f(gb), stride=1, pad=1, relu=True, dtype="f32")
    for u, v in zip(a, b):
        assert np.array_equal(u, v)


def test_maxpool_backward_routes_to_the_first_maximum():
    """Finite differences of the (pinned) forward on tie-free data; conservation of the gradient
    sum; and the tie rule on a hand-made window."""
    N, H, W, C = 2, 7, 6, 3
    n = N * H * W * C
    order = np.argsort(synth.normal(71, 7, n))              # a seeded permutation
    x = ((order.astype(np.float64) - n / 2) / 256.0).astype(np.float32).reshape(N, H, W, C)
    assert len(np.unique(x)) == x.size                      # distinct values, gaps of 2^-8
    y = on.maxpool(x, 3, 3, 2, 1, "f32")
    g = _rand(y.shape, 72)
    gx = on.maxpool_bwd(x, g, 3, 3, 2, 1, "f32")
    assert abs(gx.sum() - g.astype(np.float64).sum()) < 1e-9
    h = 2.0 ** -12                                           # far below the smallest gap (2^-8)
    rng = np.random.default_rng(7)
    for _ in range(20):
        idx = tuple(int(rng.integers(0, s)) for s in x.shape)
        xp, xm = x.copy(), x.copy()
        xp[idx] += h
        xm[idx] -= h
        fd = (np.sum(on.maxpool(xp, 3, 3, 2, 1, "f32").astype(np.float64) * g)
              - np.sum(on.maxpool(xm, 3, 3, 2, 1, "f32").astype(np.float64) * g)) / (2 * h)
        assert abs(fd - gx[idx]) <= 1e-6 * max(1.0, abs(fd))
    # ties: a constant image; window (p,q) scans rows r then columns s, padding skipped, so its
    # first maximum is its top-left valid pixel
    xc = np.ones((1, 4, 4, 1), np.float32)
    gc = np.arange(1, 5, dtype=np.float32).reshape(1, 2, 2, 1)
    gxc = on.maxpool_bwd(xc, gc, 3, 3, 2, 1, "f32")[0, :, :, 0]
    want = np.zeros((4, 4))
    want[0, 0], want[0, 1], want[1, 0], want[1, 1] = 1, 2, 3, 4   # windows start at (-1,-1),(-1,1),(1,-1),(1,1)
    assert np.array_equal(gxc, want)


def test_avgpool_and_softmax_backward():
    g = _rand((3, 1, 1, 5), 81)
    gx = on.avgpool_bwd(g, 4, 6, "f32")
    assert gx.shape == (3, 4, 6, 5)
    np.testing.assert_allclose(gx[1, 2, 3, :], g[1, 0, 0, :].astype(np.float64) / 24.0, rtol=1e-15)
    # cross-entropy: finite differences of the pinned forward formula, rows sum to zero
    N, C = 4, 7
    z = _rand((N, C), 82, 2.0)
    labels = synth.make_labels(83, N, C)
    gz = on.softmax_ce_bwd(z, labels, "f32")
    np.testing.assert_allclose(gz.sum(axis=1), 0.0, atol=1e-15)

    def loss64(zz):
        zz = zz.astype(np.float64)
        mx = zz.max(axis=1)
        return float(np.mean(mx + np.log(np.exp(zz - mx[:, None]).sum(axis=1)) - zz[np.arange(N), labels]))
    assert abs(loss64(z) - float(on.softmax_ce(z, labels, "f32")[0])) < 1e-6   # the same function as the forward
    h = 2.0 ** -10
    for i in range(N):
        for k in (0, 3, int(labels[i])):
            zp, zm = z.copy(), z.copy()
            zp[i, k] += h
            zm[i, k] -= h
            fd = (loss64(zp) - loss64(zm)) / (2 * h)
            assert abs(fd - gz[i, k]) <= 1e-6
    # uniform logits: (1/C - onehot) / N
    gu = on.softmax_ce_bwd(np.zeros((2, 4), np.float32), np.array([1, 3]), "f32")
    assert np.allclose(gu[0], np.array([0.25, -0.75, 0.25, 0.25]) / 2)


def test_classifier_backward_is_three_matrix_products():
    N, Cin, Cout = 5, 8, 6
    x = _rand((N, 1, 1, Cin), 91)
    w = _rand((Cout, 1, 1, Cin), 92)
    g = _rand((N, 1, 1, Cout), 93)
    gx, gw, gb = on.fc_bwd(x, w, g, "f32")
    G, X, Wm = (a.astype(np.float64) for a in (g.reshape(N, Cout), x.reshape(N, Cin), w.reshape(Cout, Cin)))
    np.testing.assert_allclose(gx.reshape(N, Cin), G @ Wm, rtol=1e-13)
    np.testing.assert_allclose(gw.reshape(Cout, Cin), G.T @ X, rtol=1e-13)
    np.testing.assert_allclose(gb, G.sum(axis=0), rtol=1e-13)


@pytest.mark.parametrize("case", CASES)
def test_single_entry_sums_agree_with_the_whole_gradients(case):
    """wgrad_entries / dgrad_pixels (the defining sums of single gradient entries, used on tensors
    too large to differentiate whole) against the full backward oracle, which is pinned above by
    finite differences: every entry of dL/dw and every pixel of dL/dx on small layers, strides and
    paddings included."""
    N, H, W, Cin, Cout, R, stride, pad = case
    x = _rand((N, H, W, Cin), 21)
    w = _rand((Cout, R, R, Cin), 22, 0.5)
    bn = _bn(Cout, 23)
    P = (H + 2 * pad - R) // stride + 1
    Q = (W + 2 * pad - R) // stride + 1
    g = _rand((N, P, Q, Cout), 24)
    gx, gw, gpre = on.conv_bn_act_bwd(x, w, bn, None, g, stride=stride, pad=pad, relu=False, dtype="f32")
    scale = (bn["gamma"].astype(np.float64) / np.sqrt(bn["var"].astype(np.float64) + bn["eps"])).astype(np.float32)
    entries = [(k, r, s, c) for k in range(Cout) for r in range(R) for s in range(R) for c in range(Cin)]
    got_w = np.array(on.wgrad_entries(x, g, scale, entries, stride, pad, "f32")).reshape(gw.shape)
    assert np.max(np.abs(got_w - gw)) <= 1e-6 * max(1.0, np.max(np.abs(gw)))     # scale rounded to float32 here
    pixels = [(n, h, v) for n in range(N) for h in range(H) for v in range(W)]
    got_x = on.dgrad_pixels(g, w, scale, pixels, stride, pad, H, W, "f32").reshape(gx.shape)
    assert np.max(np.abs(got_x - gx)) <= 1e-6 * max(1.0, np.max(np.abs(gx)))
