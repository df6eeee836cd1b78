"""Pins of the transformer oracle (oracle/transformer.py) to things other than itself: values
fixed by the definitions (closed forms, hand-computed rows), invariances, brute force with scalar
Python arithmetic on tiny inputs, PyTorch's CPU float64 routines as an independent implementation,
and the C oracle's bf16 rounding."""
import math

import numpy as np
import pytest

import synth
from oracle import numeric as on
from oracle import transformer as ot


def _f32(a):
    return np.asarray(a, dtype=np.float32)


# ------------------------------------------------------------------ storage rounding
def test_bf16_rounding_ties_to_even_and_is_taken_from_the_float64_value():
    cases = [
        (1.0, 0x3F80),
        (1.0 + 2.0 ** -8, 0x3F80),                  # exact tie: even neighbour below
        (1.0 + 3 * 2.0 ** -8, 0x3F82),              # exact tie: even neighbour above
        (1.0 + 2.0 ** -8 + 2.0 ** -30, 0x3F81),     # just above a tie; float32 cannot see the 2^-30
        (1.0 + 3 * 2.0 ** -8 - 2.0 ** -30, 0x3F81),  # just below a tie
        (-(1.0 + 2.0 ** -8 + 2.0 ** -30), 0xBF81),
        (0.0, 0x0000),
        (3.0e38 * 2, 0x7F80),                       # overflow to +inf
    ]
    for v, want in cases:
        assert int(ot.to_storage(np.array([v]), "bf16")[0]) == want, (v, hex(want))
    # the C oracle's scalar rounding is separate code: agree on random doubles and on every tie
    vals = synth.normal(5, 1, 4000) * np.exp(synth.uniform(5, 2, 4000, -20.0, 20.0))
    ties = (np.arange(0x3F00, 0x3F40).astype(np.uint32) << 16 | 0x8000).view(np.float32).astype(np.float64)
    for v in np.concatenate([vals, ties, -ties]):
        assert int(ot.to_storage(np.array([v]), "bf16")[0]) == on.double_to_bf16(float(v)), v
    assert np.array_equal(ot.to_f64(ot.to_storage(ties[:4], "f32"), "f32"), ties[:4])


# ------------------------------------------------------------------ GELU
def _phi_by_quadrature(x, n=4000):
    """Standard normal CDF from Simpson's rule on the density: no erf involved."""
    t = np.linspace(0.0, x, n + 1)
    f = np.exp(-0.5 * t * t) / math.sqrt(2.0 * math.pi)
    h = x / n
    return 0.5 + h / 3.0 * (f[0] + f[-1] + 4.0 * f[1:-1:2].sum() + 2.0 * f[2:-1:2].sum())


def test_gelu_closed_forms():
    assert ot.gelu(np.array([0.0]))[0] == 0.0
    assert abs(ot.gelu(np.array([1.0]))[0] - 0.8413447460685429) < 1e-15       # Phi(1)
    assert abs(ot.gelu(np.array([-1.0]))[0] + 0.15865525393145707) < 1e-15     # -(1 - Phi(1))
    x = np.linspace(-6.0, 6.0, 97)
    assert np.max(np.abs(ot.gelu(x) - ot.gelu(-x) - x)) < 1e-14                # x (Phi(x) + Phi(-x)) = x
    for v in (0.3, 1.7, 2.5, -0.9):
        assert abs(ot.gelu(np.array([v]))[0] - v * _phi_by_quadrature(v)) < 1e-12
    assert abs(ot.gelu(np.array([12.0]))[0] - 12.0) < 1e-12 and abs(ot.gelu(np.array([-12.0]))[0]) < 1e-12
    h = 1e-6
    assert abs((ot.gelu(np.array([h]))[0] - ot.gelu(np.array([-h]))[0]) / (2 * h) - 0.5) < 1e-9


# ------------------------------------------------------------------ LayerNorm
def test_layernorm_hand_computed_rows():
    x = _f32([[1, 2, 3, 4], [0, 2, 0, 2]])
    one, zero = _f32([1, 1, 1, 1]), _f32([0, 0, 0, 0])
    y = ot.to_f64(ot.layernorm(x, one, zero, 0.0, "f32"), "f32")
    r = 1.0 / math.sqrt(1.25)
    assert np.allclose(y[0], [-1.5 * r, -0.5 * r, 0.5 * r, 1.5 * r], rtol=0, atol=1e-7)
    assert np.allclose(y[1], [-1, 1, -1, 1], rtol=0, atol=1e-7)
    # eps enters under the root: variance 1, eps 3 -> divide by 2
    y = ot.to_f64(ot.layernorm(x[1:], one, zero, 3.0, "f32"), "f32")
    assert np.allclose(y[0], [-0.5, 0.5, -0.5, 0.5], rtol=0, atol=1e-7)
    # gamma scales, beta shifts, per column
    g, b = _f32([2, 1, 0.5, -1]), _f32([10, 20, 30, 40])
    y = ot.to_f64(ot.layernorm(x[1:], g, b, 0.0, "f32"), "f32")
    assert np.allclose(y[0], [8, 21, 29.5, 39], rtol=0, atol=1e-6)
    # a constant row has variance 0: beta comes out (eps keeps the division finite)
    y = ot.to_f64(ot.layernorm(_f32([[7, 7, 7, 7]]), g, b, 1e-12, "f32"), "f32")
    assert np.array_equal(y[0], [10, 20, 30, 40])


def test_layernorm_invariances_and_moments():
    x = synth.normal(11, 1, 6 * 96).reshape(6, 96).astype(np.float32) * 3 + 1.5
    one, zero = np.ones(96, np.float32), np.zeros(96, np.float32)
    y = ot.to_f64(ot.layernorm(x, one, zero, 0.0, "f32"), "f32")
    assert np.max(np.abs(y.mean(axis=1))) < 1e-6 and np.max(np.abs(y.var(axis=1) - 1.0)) < 1e-5
    x2 = (x.astype(np.float64) * 4.0 - 8.0).astype(np.float32)               # exact in float32 here? not needed:
    y2 = ot.to_f64(ot.layernorm(x2, one, zero, 0.0, "f32"), "f32")           # invariance holds up to rounding
    assert np.max(np.abs(y - y2)) < 2e-5
    # rows are independent: permuting rows permutes outputs
    perm = np.array([3, 0, 5, 1, 4, 2])
    assert np.array_equal(ot.layernorm(x[perm], one, zero, 1e-5, "f32"), ot.layernorm(x, one, zero, 1e-5, "f32")[perm])


# ------------------------------------------------------------------ linear
def test_linear_brute_force_with_bias_residual_and_activations():
    M, Cin, Cout = 3, 5, 2
    x = (synth.normal(21, 1, M * Cin).reshape(M, Cin)).astype(np.float32)
    w = (synth.normal(21, 2, Cout * Cin).reshape(Cout, Cin)).astype(np.float32)      # [out][in]: not square
    b = _f32([0.25, -1.5])
    res = (synth.normal(21, 3, M * Cout).reshape(M, Cout)).astype(np.float32)
    for act in (None, "relu", "gelu"):
        for r in (None, res):
            got = ot.to_f64(ot.linear(x, w, b, act=act, res=r, dtype="f32"), "f32")
            for m in range(M):
                for k in range(Cout):
                    v = float(b[k])
                    for c in range(Cin):
                        v += float(x[m, c]) * float(w[k, c])
                    if r is not None:
                        v += float(r[m, k])
                    if act == "relu":
                        v = max(v, 0.0)
                    elif act == "gelu":
                        v = 0.5 * v * (1.0 + math.erf(v / math.sqrt(2.0)))
                    assert abs(got[m, k] - v) <= 1e-6 * max(1.0, abs(v)), (act, m, k)


def test_linear_bf16_products_are_exact_and_rounded_once():
    # x, w exactly representable: the sum is exact in float64 and the result is its bf16 rounding
    x = ot.to_storage(np.array([[1.5, -2.0, 0.25]]), "bf16")
    w = ot.to_storage(np.array([[2.0, 0.5, 4.0], [1.0, 1.0, 1.0]]), "bf16")
    y = ot.linear(x, w, _f32([0.0, 2.0 ** -9]), dtype="bf16")
    assert ot.to_f64(y, "bf16")[0, 0] == 3.0
    assert int(y[0, 1]) == on.double_to_bf16(-0.25 + 2.0 ** -9)


# ------------------------------------------------------------------ attention
def _qkv(N, S, heads, d, master=31, scale=1.0):
    H = heads * d
    a = synth.normal(master, 1, N * S * 3 * H).reshape(N, S, 3 * H) * scale
    return a.astype(np.float32), H


def test_attention_rows_of_probabilities_sum_to_one_and_identical_keys_average_the_values():
    a, H = _qkv(2, 7, 3, 4)
    a1 = a.copy()
    a1[:, :, 2 * H:] = 1.0                                   # v = 1 everywhere
    assert np.allclose(ot.attention_f64(a1, 3, "f32"), 1.0, rtol=0, atol=1e-12)
    a2 = a.copy()
    a2[:, :, H:2 * H] = a2[:, :1, H:2 * H]                   # every position has the same key
    want = np.broadcast_to(a2[:, :, 2 * H:].astype(np.float64).mean(axis=1, keepdims=True), (2, 7, H))
    assert np.allclose(ot.attention_f64(a2, 3, "f32"), want, rtol=0, atol=1e-12)


def test_attention_two_keys_closed_form_pins_the_scale():
    d = 4
    a = np.zeros((1, 2, 3 * d), np.float32)
    a[0, :, 0:d] = [[2, 0, 0, 0], [0, 4, 0, 0]]              # queries
    a[0, :, d:2 * d] = [[1, 0, 0, 0], [0, 0, 0, 0]]          # keys
    a[0, :, 2 * d:] = [[1, 10, 100, 1000], [0, 0, 0, 0]]     # values
    ctx = ot.attention_f64(a, 1, "f32")
    p0 = math.e / (1.0 + math.e)                             # scores (2*1)/sqrt(4) = 1 and 0
    assert np.allclose(ctx[0, 0], p0 * np.array([1, 10, 100, 1000.0]), rtol=1e-14, atol=0)
    assert np.allclose(ctx[0, 1], 0.5 * np.array([1, 10, 100, 1000.0]), rtol=1e-14, atol=0)   # both scores 0


def test_attention_brute_force_heads_and_column_layout():
    N, S, heads, d = 2, 3, 2, 2
    a, H = _qkv(N, S, heads, d, master=33)
    got = ot.attention_f64(a, heads, "f32")
    for n in range(N):
        for h in range(heads):
            for i in range(S):
                sc = []
                for j in range(S):
                    sc.append(sum(float(a[n, i, h * d + e]) * float(a[n, j, H + h * d + e]) for e in range(d)) / math.sqrt(d))
                mx = max(sc)
                ex = [math.exp(v - mx) for v in sc]
                z = sum(ex)
                for e in range(d):
                    want = sum(ex[j] / z * float(a[n, j, 2 * H + h * d + e]) for j in range(S))
                    assert abs(got[n, i, h * d + e] - want) < 1e-12
    # heads do not see each other: changing head 1's keys and values leaves head 0's output alone
    b = a.copy()
    b[:, :, H + d:2 * H] += 1.0
    b[:, :, 2 * H + d:] *= 3.0
    got_b = ot.attention_f64(b, heads, "f32")
    assert np.array_equal(got_b[:, :, :d], got[:, :, :d]) and not np.allclose(got_b[:, :, d:], got[:, :, d:])
    # and images do not either
    assert np.array_equal(ot.attention_f64(a[1:], heads, "f32"), got[1:])


def test_attention_invariances():
    a, H = _qkv(1, 9, 2, 8, master=35)
    base = ot.attention_f64(a, 2, "f32")
    perm = np.array([4, 0, 8, 2, 6, 1, 7, 3, 5])
    b = a.copy()
    b[:, :, H:] = a[:, perm, H:]                              # keys and values move together
    assert np.allclose(ot.attention_f64(b, 2, "f32"), base, rtol=0, atol=1e-13)
    c = a.astype(np.float64).copy()
    c[:, :, H:2 * H] += 0.5                                   # q.(k + c) = q.k + q.c: constant per query
    assert np.allclose(ot.attention_f64(c.astype(np.float32), 2, "f32"), base, rtol=0, atol=1e-6)
    big = a.copy()
    big[:, :, :H] *= 200.0                                    # huge scores: the max is subtracted, no overflow
    assert np.isfinite(ot.attention_f64(big, 2, "f32")).all()


# ------------------------------------------------------------------ the layer against PyTorch's CPU float64 routines
def test_encoder_layer_matches_torch_float64():
    torch = pytest.importorskip("torch")
    F = torch.nn.functional
    N, S, H, heads, FF = 2, 10, 24, 3, 40
    p = synth.make_encoder_params(41, 0, H, FF, "f32")
    x = synth.normal(41, 999, N * S * H).reshape(N, S, H).astype(np.float32)
    out = ot.encoder_layer(x, p, heads, 1e-12, "f32")
    t = lambda a: torch.from_numpy(np.asarray(a, dtype=np.float32)).double()
    X = t(x).reshape(N * S, H)
    qkv = F.linear(X, t(p["wqkv"]), t(p["bqkv"]))
    q, k, v = [z.reshape(N, S, heads, H // heads).transpose(1, 2) for z in qkv.split(H, dim=1)]
    ctx = F.scaled_dot_product_attention(q, k, v).transpose(1, 2).reshape(N * S, H)
    ao = F.linear(ctx, t(p["wo"]), t(p["bo"])) + X
    ln1 = F.layer_norm(ao, (H,), t(p["g1"]), t(p["be1"]), 1e-12)
    f1 = F.gelu(F.linear(ln1, t(p["w1"]), t(p["b1"])))
    f2 = F.linear(f1, t(p["w2"]), t(p["b2"])) + ln1
    ln2 = F.layer_norm(f2, (H,), t(p["g2"]), t(p["be2"]), 1e-12)
    for name, ref in (("qkv", qkv), ("ctx", ctx), ("ao", ao), ("ln1", ln1), ("f1", f1), ("f2", f2), ("ln2", ln2)):
        got = ot.to_f64(out[name], "f32")
        err = float(np.max(np.abs(got - ref.numpy())) / np.max(np.abs(ref.numpy())))
        assert err < 2e-6, (name, err)                       # float32 storage roundings only
    assert out["ln2"].shape == (N * S, H) and out["f1"].shape == (N * S, FF)
