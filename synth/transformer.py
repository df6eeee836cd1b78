"""Shapes and seeded parameters of the transformer encoder of benchmark configuration 5
(BERT-base: 12 layers, hidden 768, 12 heads, feed-forward 3072, sequences of 512, batch 32), at the
granularity that is executed: attention is one fused layer, so scores and probabilities are not
tensors of this graph (synth.transformer_graph lists them for the planner-only workload).

No arithmetic of the method here: layer lists, array shapes and random draws only.
"""
import numpy as np

from . import rng
from .resnet import LayerSpec

LN_EPS = 1e-12          # BERT's layer-norm epsilon
W_STD = 0.02            # BERT's initialiser: N(0, 0.02^2)


def encoder_layers(N, S, hidden=768, heads=12, ffn=3072, nlayers=12, x0="x0"):
    """Post-LN encoder layers on x0 [N, S, hidden].  Linear layers are 1x1 'convolutions' over an
    N x S x 1 image (rows = tokens): y = act(x w^T + bias + res)."""
    layers = []
    x = x0

    def add(name, kind, xin, res, cin, cout, **kw):
        l = LayerSpec(name, kind, xin, res, name, N, S, 1, cin, cout, relu=False, **kw)
        l.index = len(layers) + 1
        layers.append(l)
        return name

    for i in range(nlayers):
        p = "l%d." % i
        qkv = add(p + "qkv", "linear", x, None, hidden, 3 * hidden)
        ctx = add(p + "ctx", "attention", qkv, None, 3 * hidden, hidden, R=heads)
        ao = add(p + "ao", "linear", ctx, x, hidden, hidden)
        ln1 = add(p + "ln1", "layernorm", ao, None, hidden, hidden)
        f1 = add(p + "f1", "linear", ln1, None, hidden, ffn, act="gelu")
        f2 = add(p + "f2", "linear", f1, ln1, ffn, hidden)
        x = add(p + "ln2", "layernorm", f2, None, hidden, hidden)
    return layers


def make_layer_params(master, layer, dtype):
    """linear: w [Cout, Cin] ~ N(0, 0.02^2) in the storage type and a float32 bias ~ N(0, 0.02^2);
    layernorm: gamma ~ U(0.5, 1.5), beta ~ N(0, 0.1^2), float32; attention: nothing."""
    base = layer.index * 16
    if layer.kind == "linear":
        w = rng.normal(master, base + 0, layer.Cout * layer.Cin, 0.0, W_STD).astype(np.float32)
        w = w.reshape(layer.Cout, layer.Cin)
        if dtype == "bf16":
            w = rng.f32_to_bf16_bits(w).reshape(layer.Cout, layer.Cin)
        return {"w": w, "bias": rng.normal(master, base + 2, layer.Cout, 0.0, W_STD).astype(np.float32)}
    if layer.kind == "layernorm":
        return {"gamma": rng.uniform(master, base + 1, layer.Cin, 0.5, 1.5).astype(np.float32),
                "beta": rng.normal(master, base + 2, layer.Cin, 0.0, 0.1).astype(np.float32), "eps": LN_EPS}
    return {}


def make_encoder_params(master, i, hidden, ffn, dtype, heads=1):
    """The parameters of encoder layer `i` as one dict (wqkv, bqkv, wo, bo, g1, be1, w1, b1, w2, b2,
    g2, be2): the same draws as make_layer_params gives layer by layer."""
    ls = encoder_layers(1, 1, hidden, heads, ffn, nlayers=i + 1)[7 * i:]
    by = {l.name.split(".")[1]: make_layer_params(master, l, dtype) for l in ls}
    return {"wqkv": by["qkv"]["w"], "bqkv": by["qkv"]["bias"], "wo": by["ao"]["w"], "bo": by["ao"]["bias"],
            "g1": by["ln1"]["gamma"], "be1": by["ln1"]["beta"], "w1": by["f1"]["w"], "b1": by["f1"]["bias"],
            "w2": by["f2"]["w"], "b2": by["f2"]["bias"], "g2": by["ln2"]["gamma"], "be2": by["ln2"]["beta"]}
