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

Its backward is the chain rule through those three lines, in the order the same publication
lists it (its Sec. 3): with xhat = (x - mu) / sqrt(var + eps), M = N H W positions per channel,

    dxhat  = gy gamma_c
    dvar_c = sum dxhat (x - mu_c) * (-1/2) (var_c + eps)^(-3/2)
    dmu_c  = -sum dxhat / sqrt(var_c + eps)  +  dvar_c * (-2/M) sum (x - mu_c)
    gx     = dxhat / sqrt(var_c + eps) + dvar_c * 2 (x - mu_c) / M + dmu_c / M
    dgamma_c = sum gy xhat            dbeta_c = sum gy

ReLU's backward passes gy where the stored output is positive.  Running statistics are not part
of the activations the memory manager handles and are not modelled.  ReLU and the residual add
are separate operators at this granularity; every stored tensor is rounded to the storage type
where it is produced.

Pins: tests/test_oracle_opgranular.py.
"""
import numpy as np

from . import numeric as on
from .transformer import to_storage


def bn_train_f64(v, gamma, beta, eps):
    """The operator on float64 values v [N,H,W,C], unrounded."""
    mu = v.mean(axis=(0, 1, 2), keepdims=True)
    var = ((v - mu) ** 2).mean(axis=(0, 1, 2), keepdims=True)
    g = np.asarray(gamma, dtype=np.float32).astype(np.float64)
    b = np.asarray(beta, dtype=np.float32).astype(np.float64)
    return g * (v - mu) / np.sqrt(var + float(eps)) + b


def bn_train(x, gamma, beta, eps, dtype="bf16"):
    """x [N,H,W,C] (storage); gamma, beta float32 [C].  Returns y (storage)."""
    return to_storage(bn_train_f64(on.to_f64(x, dtype), gamma, beta, eps), dtype)


def bn_train_bwd(x, gamma, gy, eps, dtype="bf16"):
    """Backward of bn_train.  x, gy [N,H,W,C] (storage); gamma float32 [C].
    Returns (gx storage, dgamma float64 [C], dbeta float64 [C])."""
    v, g = on.to_f64(x, dtype), on.to_f64(gy, dtype)
    M = v.shape[0] * v.shape[1] * v.shape[2]
    ax = (0, 1, 2)
    gam = np.asarray(gamma, dtype=np.float32).astype(np.float64)
    mu = v.mean(axis=ax, keepdims=True)
    var = ((v - mu) ** 2).mean(axis=ax, keepdims=True)
    ve = var + float(eps)
    xhat = (v - mu) / np.sqrt(ve)
    dxhat = g * gam
    dvar = (dxhat * (v - mu)).sum(axis=ax, keepdims=True) * (-0.5) * ve ** (-1.5)
    dmu = -(dxhat.sum(axis=ax, keepdims=True)) / np.sqrt(ve) + dvar * (-2.0 / M) * (v - mu).sum(axis=ax, keepdims=True)
    gx = dxhat / np.sqrt(ve) + dvar * 2.0 * (v - mu) / M + dmu / M
    return to_storage(gx, dtype), (g * xhat).sum(axis=ax), g.sum(axis=ax)


def relu(x, dtype="bf16"):
    return to_storage(np.maximum(on.to_f64(x, dtype), 0.0), dtype)


def relu_bwd(y, gy, dtype="bf16"):
    """gx = gy where the stored output y is positive, else 0 (storage in, storage out)."""
    return to_storage(np.where(on.to_f64(y, dtype) > 0, on.to_f64(gy, dtype), 0.0), dtype)


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
