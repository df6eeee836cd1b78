"""Oracle for the operator-granular ResNet with training-mode batch normalisation.

TEST INFRASTRUCTURE ONLY: the product never imports this module.

The paper's framework manages the outputs of separate operators - ConvForward, BNForward,
PoolingForward are the tensors its Director's cost table lists (Sec. 5.5, the recompute-vs-swap
cost table) - and trains, so batch normalisation uses the statistics of the batch.  The paper
does not restate the operator; this is its published definition (Ioffe & Szegedy 2015, Alg. 1),
float64 numpy, one plain step after the other:

    mu_c  = mean over (n, h, w) of x[n,h,w,c]
    var_c = mean over (n, h, w) of (x[n,h,w,c] - mu_c)^2            (biased)
    y     = gamma_c (x - mu_c) / sqrt(var_c + eps) + beta_c

Running statistics are not part of the activations the memory manager handles and are not
modelled.  ReLU and the residual add are separate operators at this granularity; every stored
tensor is rounded to the storage type where it is produced.

Pins: tests/test_oracle_opgranular.py.
"""
import numpy as np

from . import numeric as on
from .transformer import to_storage


def bn_train(x, gamma, beta, eps, dtype="bf16"):
    """x [N,H,W,C] (storage); gamma, beta float32 [C].  Returns y (storage)."""
    v = on.to_f64(x, dtype)
    mu = v.mean(axis=(0, 1, 2), keepdims=True)
    var = ((v - mu) ** 2).mean(axis=(0, 1, 2), keepdims=True)
    g = np.asarray(gamma, dtype=np.float32).astype(np.float64)
    b = np.asarray(beta, dtype=np.float32).astype(np.float64)
    return to_storage(g * (v - mu) / np.sqrt(var + float(eps)) + b, dtype)


def relu(x, dtype="bf16"):
    return to_storage(np.maximum(on.to_f64(x, dtype), 0.0), dtype)


def add(x, r, dtype="bf16"):
    return to_storage(on.to_f64(x, dtype) + on.to_f64(r, dtype), dtype)


def run_ops(layers, params, x0, dtype):
    """Forward of synth.LayerSpec layers at operator granularity; tensor names as in
    synth.opgranular_graph (<layer>.conv, .bn, .add, .relu; pooling and classifier by layer name)."""
    acts = {"x0": x0}
    alias = {"x0": "x0"}
    for l in layers:
        x = acts[alias[l.x]]
        p = params.get(l.name)
        if l.kind == "conv":
            t = l.name + ".conv"
            acts[t] = on.conv_bn_act(x, p["w"], None, stride=l.stride, pad=l.pad, relu=False, dtype=dtype)
            acts[l.name + ".bn"] = bn_train(acts[t], p["gamma"], p["beta"], p["eps"], dtype)
            t = l.name + ".bn"
            if l.res:
                acts[l.name + ".add"] = add(acts[t], acts[alias[l.res]], dtype)
                t = l.name + ".add"
            if l.relu:
                acts[l.name + ".relu"] = relu(acts[t], dtype)
                t = l.name + ".relu"
        elif l.kind == "maxpool":
            t = l.name
            acts[t] = on.maxpool(x, l.R, l.S, l.stride, l.pad, dtype)
        elif l.kind == "avgpool":
            t = l.name
            acts[t] = on.avgpool(x, dtype)
        elif l.kind == "fc":
            t = l.name
            C = l.Cout
            bn = dict(gamma=np.ones(C, np.float32), beta=p["bias"], mean=np.zeros(C, np.float32),
                      var=np.ones(C, np.float32), eps=0.0)
            acts[t] = on.conv_bn_act(x, p["w"], bn, relu=False, dtype=dtype)
        else:
            raise ValueError("no oracle for layer kind %r" % l.kind)
        alias[l.y] = t
    return acts
