"""Oracle for the transformer encoder layer of benchmark configuration 5 (BERT-base shapes).

TEST INFRASTRUCTURE ONLY: the product never imports this module.

The paper trains BERT-base (Sec. 5.2, the BERT column of its memory table) but does not restate
what an encoder layer computes; this file writes out the published definition of the post-LN
encoder layer (Devlin et al. 2018; Vaswani et al. 2017, Sec. 3.2-3.3), without dropout, in
float64 numpy, one plain step after the other:

    q|k|v = x Wqkv^T + bqkv                      (one matrix: rows [0,H) -> q, [H,2H) -> k, [2H,3H) -> v)
    ctx   = concat_h softmax(q_h k_h^T / sqrt(d)) v_h        d = H / heads
    ao    = ctx Wo^T + bo + x
    ln1   = LayerNorm(ao)
    f1    = gelu(ln1 W1^T + b1)                  gelu(v) = v/2 (1 + erf(v / sqrt 2))
    f2    = f1 W2^T + b2 + ln1
    ln2   = LayerNorm(f2)
    LayerNorm(v) = (v - mean) / sqrt(var + eps) * gamma + beta     (biased variance over the row)

Each tensor that the executed graph stores is rounded to the storage type (bf16 bit patterns in
uint16 arrays, or float32) where it is produced; scores and probabilities are never stored (the
kernels keep them on chip), so they are not rounded here either.  numpy's matmul and scipy's erf
are the library primitives; nothing is blocked, fused or reordered.

Pins: tests/test_oracle_transformer.py (closed forms, invariances, brute force on tiny inputs).
"""
import numpy as np
from scipy.special import erf


def to_f64(a, dtype):
    """Storage array -> float64 (bf16 bit patterns are widened exactly)."""
    if dtype == "bf16":
        return (np.asarray(a, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    return np.asarray(a, dtype=np.float32).astype(np.float64)


def to_storage(v, dtype):
    """float64 -> storage type, round to nearest, ties to even, straight from the float64 value."""
    v = np.asarray(v, dtype=np.float64)
    with np.errstate(over="ignore"):
        f = v.astype(np.float32)                   # nearest float32 (ties to even); overflow -> inf
    if dtype != "bf16":
        return f
    bits = f.view(np.uint32).astype(np.uint64)
    low = bits & 0xFFFF
    trunc = bits >> 16
    # which side of the float32 value the float64 one lies on (by magnitude): breaks what would
    # otherwise look like a tie after the first rounding
    with np.errstate(invalid="ignore"):            # inf - inf for infinite inputs: their low bits are 0 anyway
        resid = (np.abs(v) - np.abs(f.astype(np.float64)))
    up = (low > 0x8000) | ((low == 0x8000) & ((resid > 0) | ((resid == 0) & ((trunc & 1) == 1))))
    out = (trunc + up.astype(np.uint64)).astype(np.uint16)
    nan = np.isnan(v)
    if nan.any():
        out = np.where(nan, np.uint16(0x7FC0), out)
    return out


def gelu(v):
    """Exact (erf) GELU, elementwise, float64."""
    v = np.asarray(v, dtype=np.float64)
    return 0.5 * v * (1.0 + erf(v / np.sqrt(2.0)))


def linear(x, w, b, act=None, res=None, dtype="bf16"):
    """y = act(x w^T + b + res).  x [M, Cin], w [Cout, Cin] (storage), b [Cout] float32,
    res [M, Cout] (storage) or None; act None | 'relu' | 'gelu'.  Returns storage."""
    y = to_f64(x, dtype) @ to_f64(w, dtype).T + np.asarray(b, dtype=np.float32).astype(np.float64)[None, :]
    if res is not None:
        y = y + to_f64(res, dtype)
    if act == "relu":
        y = np.maximum(y, 0.0)
    elif act == "gelu":
        y = gelu(y)
    elif act is not None:
        raise ValueError(act)
    return to_storage(y, dtype)


def attention_f64(qkv, heads, dtype="bf16"):
    """Scaled dot-product self-attention over all positions (no mask), float64, unrounded.
    qkv [N, S, 3H]: q = [..., 0:H], k = [..., H:2H], v = [..., 2H:3H]; head h owns columns
    [h d, (h+1) d) of each.  Returns ctx [N, S, H]."""
    a = to_f64(qkv, dtype)
    N, S, H3 = a.shape
    H = H3 // 3
    d = H // heads
    assert H * 3 == H3 and d * heads == H
    ctx = np.empty((N, S, H))
    for n in range(N):
        for h in range(heads):
            q = a[n, :, h * d:(h + 1) * d]
            k = a[n, :, H + h * d:H + (h + 1) * d]
            v = a[n, :, 2 * H + h * d:2 * H + (h + 1) * d]
            s = (q @ k.T) / np.sqrt(float(d))
            s = s - s.max(axis=1, keepdims=True)
            p = np.exp(s)
            p = p / p.sum(axis=1, keepdims=True)
            ctx[n, :, h * d:(h + 1) * d] = p @ v
    return ctx


def attention(qkv, heads, dtype="bf16"):
    return to_storage(attention_f64(qkv, heads, dtype), dtype)


def layernorm(x, gamma, beta, eps, dtype="bf16"):
    """Row-wise layer normalisation of x [M, C] (storage); gamma, beta float32 [C]."""
    v = to_f64(x, dtype)
    mean = v.mean(axis=1, keepdims=True)
    var = ((v - mean) ** 2).mean(axis=1, keepdims=True)
    g = np.asarray(gamma, dtype=np.float32).astype(np.float64)
    b = np.asarray(beta, dtype=np.float32).astype(np.float64)
    return to_storage((v - mean) / np.sqrt(var + float(eps)) * g[None, :] + b[None, :], dtype)


def encoder_layer(x, p, heads, eps, dtype="bf16"):
    """One encoder layer on x [N, S, H] (storage).  p: dict with wqkv [3H,H], bqkv, wo [H,H], bo,
    g1, be1, w1 [F,H], b1, w2 [H,F], b2, g2, be2.  Returns the stored tensors by name."""
    N, S, H = x.shape
    x2 = x.reshape(N * S, H)
    out = {}
    out["qkv"] = linear(x2, p["wqkv"], p["bqkv"], dtype=dtype)
    out["ctx"] = attention(out["qkv"].reshape(N, S, 3 * H), heads, dtype).reshape(N * S, H)
    out["ao"] = linear(out["ctx"], p["wo"], p["bo"], res=x2, dtype=dtype)
    out["ln1"] = layernorm(out["ao"], p["g1"], p["be1"], eps, dtype)
    out["f1"] = linear(out["ln1"], p["w1"], p["b1"], act="gelu", dtype=dtype)
    out["f2"] = linear(out["f1"], p["w2"], p["b2"], res=out["ln1"], dtype=dtype)
    out["ln2"] = layernorm(out["f2"], p["g2"], p["be2"], eps, dtype)
    return out
