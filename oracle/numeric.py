"""numpy front end of the numeric oracle (oracle/conv_ref.c).

Arrays: activations NHWC, weights KRSC.  dtype 'f32' uses float32 arrays,
'bf16' uses uint16 arrays holding bf16 bit patterns.  See conv_ref.c for the
definition that is computed and the tests that pin it.
"""
import ctypes

import numpy as np

from . import build as _build

_lib = None


def lib():
    global _lib
    if _lib is None:
        L = ctypes.CDLL(_build.build())
        L.oracle_conv_bn_act.restype = ctypes.c_int
        L.oracle_conv_bn_act.argtypes = ([ctypes.c_int] + [ctypes.c_void_p] * 7 + [ctypes.c_double]
                                         + [ctypes.c_int] * 10 + [ctypes.c_void_p] * 2)
        L.oracle_maxpool.restype = ctypes.c_int
        L.oracle_conv_bn_act_bwd.argtypes = ([ctypes.c_int] + [ctypes.c_void_p] * 6 + [ctypes.c_double]
                                             + [ctypes.c_int] * 10 + [ctypes.c_void_p] * 3)
        L.oracle_conv_bn_act_bwd.restype = ctypes.c_int
        L.oracle_maxpool.argtypes = [ctypes.c_int, ctypes.c_void_p] + [ctypes.c_int] * 8 + [ctypes.c_void_p]
        L.oracle_avgpool.restype = ctypes.c_int
        L.oracle_avgpool.argtypes = [ctypes.c_int, ctypes.c_void_p] + [ctypes.c_int] * 4 + [ctypes.c_void_p]
        L.oracle_double_to_bf16.restype = ctypes.c_uint16
        L.oracle_double_to_bf16.argtypes = [ctypes.c_double]
        L.oracle_bf16_to_double.restype = ctypes.c_double
        L.oracle_bf16_to_double.argtypes = [ctypes.c_uint16]
        L.oracle_num_threads.restype = ctypes.c_int
        _lib = L
    return _lib


def _code(dtype):
    return {"f32": 0, "bf16": 1}[dtype]


def _np(dtype):
    return np.float32 if dtype == "f32" else np.uint16


def _ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def num_threads():
    return int(lib().oracle_num_threads())


def double_to_bf16(v):
    return int(lib().oracle_double_to_bf16(float(v)))


def bf16_to_double(b):
    return float(lib().oracle_bf16_to_double(int(b)))


def to_f64(a, dtype):
    """Exact widening of a stored array to float64."""
    if dtype == "f32":
        return np.asarray(a, dtype=np.float32).astype(np.float64)
    b = np.ascontiguousarray(a, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def conv_bn_act(x, w, bn, res=None, stride=1, pad=0, relu=True, dtype="f32", want_f64=False):
    """One fused layer; bn = dict(gamma, beta, mean, var, eps) or None.  Returns y
    (storage dtype) or (y, y64) where y64 holds the values before the final rounding."""
    x = np.ascontiguousarray(x, dtype=_np(dtype))
    w = np.ascontiguousarray(w, dtype=_np(dtype))
    N, H, W, Cin = x.shape
    Cout, R, S, Cin2 = w.shape
    assert Cin == Cin2
    P = (H + 2 * pad - R) // stride + 1
    Q = (W + 2 * pad - S) // stride + 1
    y = np.empty((N, P, Q, Cout), dtype=_np(dtype))
    y64 = np.empty((N, P, Q, Cout), dtype=np.float64) if want_f64 else None
    if res is not None:
        res = np.ascontiguousarray(res, dtype=_np(dtype))
        assert res.shape == y.shape
    if bn is not None:
        g, b, m, v = (np.ascontiguousarray(bn[k], dtype=np.float32) for k in ("gamma", "beta", "mean", "var"))
        assert g.shape == b.shape == m.shape == v.shape == (Cout,)
        eps = float(bn["eps"])
    else:
        g = b = m = v = None
        eps = 0.0
    rc = lib().oracle_conv_bn_act(_code(dtype), _ptr(x), _ptr(w), _ptr(res), _ptr(g), _ptr(b),
                                  _ptr(m), _ptr(v), eps, N, H, W, Cin, Cout, R, S, stride, pad,
                                  1 if relu else 0, _ptr(y), _ptr(y64))
    if rc != 0:
        raise ValueError("oracle_conv_bn_act rejected its arguments")
    return (y, y64) if want_f64 else y


def conv_bn_act_bwd(x, w, bn, y, gy, stride=1, pad=0, relu=True, dtype="f32"):
    """Backward of one fused layer (frozen batch-norm statistics).  x, w, y (stored forward
    output; only read when relu) and gy = dL/dy at storage precision.  Returns float64 arrays
    (gx, gw, gpre): dL/dx, dL/dw and dL/d(pre-activation), which is also dL/dres."""
    x = np.ascontiguousarray(x, dtype=_np(dtype))
    w = np.ascontiguousarray(w, dtype=_np(dtype))
    gy = np.ascontiguousarray(gy, dtype=_np(dtype))
    N, H, W, Cin = x.shape
    Cout, R, S, Cin2 = w.shape
    assert Cin == Cin2
    P = (H + 2 * pad - R) // stride + 1
    Q = (W + 2 * pad - S) // stride + 1
    assert gy.shape == (N, P, Q, Cout)
    if relu:
        y = np.ascontiguousarray(y, dtype=_np(dtype))
        assert y.shape == gy.shape
    else:
        y = None
    if bn is not None:
        g, v = (np.ascontiguousarray(bn[k], dtype=np.float32) for k in ("gamma", "var"))
        eps = float(bn["eps"])
    else:
        g = v = None
        eps = 0.0
    gx = np.empty(x.shape, dtype=np.float64)
    gw = np.empty(w.shape, dtype=np.float64)
    gpre = np.empty(gy.shape, dtype=np.float64)
    rc = lib().oracle_conv_bn_act_bwd(_code(dtype), _ptr(x), _ptr(w), _ptr(y), _ptr(gy), _ptr(g), _ptr(v),
                                      eps, N, H, W, Cin, Cout, R, S, stride, pad, 1 if relu else 0,
                                      _ptr(gx), _ptr(gw), _ptr(gpre))
    if rc != 0:
        raise ValueError("oracle_conv_bn_act_bwd rejected its arguments")
    return gx, gw, gpre


def wgrad_entries(x, gpre, scale, entries, stride, pad, dtype="f32"):
    """Single entries of dL/dw of one fused layer, each written out as its defining sum
    (for checking tensors too large to differentiate whole):
        gw[k, r, s, c] = scale_k * sum over n, p, q of gpre[n, p, q, k] * x[n, p*stride + r - pad, q*stride + s - pad, c]
    x [N,H,W,Cin] and gpre [N,P,Q,Cout] (dL/d pre-activation at the OUTPUT's resolution) at storage
    precision, scale float32 [Cout] or None; entries: (k, r, s, c) tuples.  float64 list."""
    xd, gd = to_f64(x, dtype), to_f64(gpre, dtype)
    N, H, W, _ = xd.shape
    _, P, Q, _ = gd.shape
    out = []
    for (k, r, s_, c) in entries:
        ps = [p for p in range(P) if 0 <= p * stride + r - pad < H]
        qs = [q for q in range(Q) if 0 <= q * stride + s_ - pad < W]
        if not ps or not qs:
            out.append(0.0)
            continue
        hs = [p * stride + r - pad for p in ps]
        ws = [q * stride + s_ - pad for q in qs]
        a = gd[:, ps][:, :, qs][..., k]
        b = xd[:, hs][:, :, ws][..., c]
        v = float((a * b).sum())
        out.append(v * (float(np.float32(scale[k])) if scale is not None else 1.0))
    return out


def dgrad_pixels(gpre, w, scale, pixels, stride, pad, H, W, dtype="f32"):
    """dL/dx of one fused layer at single input pixels, each written out as its defining sum:
        gx[n, h, w, c] = sum over k, r, s with (h + pad - r, w + pad - s) = stride * (p, q), p, q in range,
                         of gpre[n, p, q, k] * scale_k * w[k, r, s, c]
    gpre [N,P,Q,Cout] at the output's resolution and w [Cout,R,S,Cin] at storage precision; pixels:
    (n, h, w) tuples; H, W: the input's size.  float64 [len(pixels), Cin]."""
    gd, wd = to_f64(gpre, dtype), to_f64(w, dtype)
    Cout, R, S, Cin = wd.shape
    _, P, Q, _ = gd.shape
    sc = np.asarray(scale, dtype=np.float32).astype(np.float64) if scale is not None else np.ones(Cout)
    out = np.zeros((len(pixels), Cin))
    for i, (n, h, w_) in enumerate(pixels):
        assert 0 <= h < H and 0 <= w_ < W
        for r in range(R):
            for s_ in range(S):
                hp, wq = h + pad - r, w_ + pad - s_
                if hp % stride or wq % stride:
                    continue
                p, q = hp // stride, wq // stride
                if 0 <= p < P and 0 <= q < Q:
                    out[i] += (gd[n, p, q, :] * sc) @ wd[:, r, s_, :]
    return out


def maxpool(x, R, S, stride, pad, dtype="f32"):
    x = np.ascontiguousarray(x, dtype=_np(dtype))
    N, H, W, C = x.shape
    P = (H + 2 * pad - R) // stride + 1
    Q = (W + 2 * pad - S) // stride + 1
    y = np.empty((N, P, Q, C), dtype=_np(dtype))
    if lib().oracle_maxpool(_code(dtype), _ptr(x), N, H, W, C, R, S, stride, pad, _ptr(y)) != 0:
        raise ValueError("oracle_maxpool rejected its arguments")
    return y


def avgpool(x, dtype="f32"):
    x = np.ascontiguousarray(x, dtype=_np(dtype))
    N, H, W, C = x.shape
    y = np.empty((N, 1, 1, C), dtype=_np(dtype))
    if lib().oracle_avgpool(_code(dtype), _ptr(x), N, H, W, C, _ptr(y)) != 0:
        raise ValueError("oracle_avgpool rejected its arguments")
    return y


def softmax_ce(logits, labels, dtype="f32"):
    """Mean over images of logsumexp(z_i) - z_i[label_i], in float64; returned as float32 [1]."""
    z = to_f64(logits, dtype).reshape(len(labels), -1)
    mx = z.max(axis=1)
    lse = mx + np.log(np.exp(z - mx[:, None]).sum(axis=1))
    picked = z[np.arange(len(labels)), np.asarray(labels, dtype=np.int64)]
    return np.array([np.mean(lse - picked)], dtype=np.float32)


def maxpool_bwd(x, gy, R, S, stride, pad, dtype="f32"):
    """Backward of max pooling: the gradient of an output pixel goes to the maximal element of its
    window; among equal maxima to the first in scan order (r, then s) - the element the forward's
    scan `if v > m` keeps.  Padding never receives anything.  float64 [N,H,W,C]."""
    xd, gd = to_f64(x, dtype), to_f64(gy, dtype)
    N, H, W, C = xd.shape
    P = (H + 2 * pad - R) // stride + 1
    Q = (W + 2 * pad - S) // stride + 1
    assert gd.shape == (N, P, Q, C)
    gx = np.zeros_like(xd)
    n_idx, c_idx = np.meshgrid(np.arange(N), np.arange(C), indexing="ij")
    for p in range(P):
        for q in range(Q):
            hs = [p * stride + r - pad for r in range(R)]
            ws = [q * stride + s_ - pad for s_ in range(S)]
            cand = [(h, w) for h in hs for w in ws if 0 <= h < H and 0 <= w < W]   # scan order
            vals = np.stack([xd[:, h, w, :] for (h, w) in cand], axis=0)            # [cand, N, C]
            first = np.argmax(vals, axis=0)                                         # first maximum
            for i, (h, w) in enumerate(cand):
                gx[:, h, w, :] += np.where(first == i, gd[:, p, q, :], 0.0)
    return gx


def avgpool_bwd(gy, H, W, dtype="f32"):
    """Backward of the global average: every pixel receives gy / (H W).  float64 [N,H,W,C]."""
    gd = to_f64(gy, dtype)
    N, C = gd.shape[0], gd.shape[-1]
    return np.broadcast_to(gd.reshape(N, 1, 1, C) / float(H * W), (N, H, W, C)).copy()


def softmax_ce_bwd(logits, labels, dtype="f32"):
    """Gradient of the mean cross-entropy with respect to the logits:
    (softmax(z_i) - onehot(label_i)) / N.  float64 [N, classes]."""
    z = to_f64(logits, dtype).reshape(len(labels), -1)
    e = np.exp(z - z.max(axis=1, keepdims=True))
    g = e / e.sum(axis=1, keepdims=True)
    g[np.arange(len(labels)), np.asarray(labels, dtype=np.int64)] -= 1.0
    return g / float(len(labels))


def fc_bwd(x, w, gy, dtype="f32"):
    """Backward of z = x w^T + bias (the classifier): returns float64 (gx, gw, gbias)."""
    gx, gw, _ = conv_bn_act_bwd(x, w, None, None, gy, stride=1, pad=0, relu=False, dtype=dtype)
    return gx, gw, to_f64(gy, dtype).reshape(-1, gy.shape[-1]).sum(axis=0)


def run_layers(layers, params, x0, dtype, labels=None, acts=None):
    """Forward of a list of synth.LayerSpec layers; returns {tensor name: stored array}.  With
    `labels`, the mean cross-entropy of the last layer's output is added as "loss".  `acts`
    (instead of x0): stored tensors the layers may read, by name."""
    acts = dict(acts) if acts is not None else {"x0": x0}
    for l in layers:
        if l.kind == "conv":
            acts[l.y] = conv_bn_act(acts[l.x], params[l.name]["w"], params[l.name],
                                    res=acts[l.res] if l.res else None, stride=l.stride,
                                    pad=l.pad, relu=l.relu, dtype=dtype)
        elif l.kind == "maxpool":
            acts[l.y] = maxpool(acts[l.x], l.R, l.S, l.stride, l.pad, dtype)
        elif l.kind == "avgpool":
            acts[l.y] = avgpool(acts[l.x], dtype)
        elif l.kind == "fc":                    # z + bias: a 1x1 convolution with identity statistics
            C = l.Cout
            bn = dict(gamma=np.ones(C, np.float32), beta=params[l.name]["bias"],
                      mean=np.zeros(C, np.float32), var=np.ones(C, np.float32), eps=0.0)
            acts[l.y] = conv_bn_act(acts[l.x], params[l.name]["w"], bn, relu=False, dtype=dtype)
        else:
            raise ValueError("no oracle for layer kind %r" % l.kind)
    if labels is not None:
        acts["labels"] = np.asarray(labels, dtype=np.int64)
        acts["loss"] = softmax_ce(acts[layers[-1].y], labels, dtype)
    return acts
