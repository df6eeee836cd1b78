"""Workload definitions: layer lists, parameter draws and planner graphs.

Everything here is shape bookkeeping and random draws.  Layer arithmetic lives
in the oracle (CPU) and in the HIP library (GPU), never here.
"""
from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np

from . import rng

FLAG_UNCOMPUTABLE = 1
FLAG_EVICT_PINNED = 2
FLAG_OFFLOAD_PINNED = 4

BN_EPS = 1e-5


def master_seed(cfg: int) -> int:
    return 0xDE17A000 + int(cfg)


@dataclass
class LayerSpec:
    """One fused layer: y = relu?(bn(conv(x, w)) + res?), NHWC activations, KRSC weights."""
    name: str
    kind: str               # 'conv' | 'maxpool' | 'avgpool' | 'fc' | 'input' | 'loss' | transformer.py's kinds
    x: Optional[str]
    res: Optional[str]
    y: str
    N: int
    H: int
    W: int
    Cin: int
    Cout: int
    R: int = 1
    S: int = 1
    stride: int = 1
    pad: int = 0
    relu: bool = True
    index: int = 0          # position in the network, used to derive array ids
    act: str = ""           # 'gelu' for a linear layer that ends in GELU

    @property
    def P(self):
        if self.kind in ("attention", "layernorm"):          # R is the number of heads there
            return self.H
        return (self.H + 2 * self.pad - self.R) // self.stride + 1

    @property
    def Q(self):
        if self.kind in ("attention", "layernorm"):
            return self.W
        return (self.W + 2 * self.pad - self.S) // self.stride + 1

    @property
    def M(self):
        return self.N * self.P * self.Q

    @property
    def flops(self):
        if self.kind in ("conv", "fc", "linear"):
            return 2 * self.M * self.R * self.S * self.Cin * self.Cout
        if self.kind == "attention":                 # q k^T and p v: 2 * 2 * N * S^2 * hidden
            return 4 * self.N * self.H * self.H * self.Cout
        if self.kind == "layernorm":
            return 8 * self.N * self.H * self.W * self.Cin
        if self.kind == "maxpool":
            return self.M * self.R * self.S * self.Cout
        if self.kind == "avgpool":
            return self.N * self.H * self.W * self.Cin
        return 0

    def out_elems(self):
        return self.M * self.Cout

    def in_elems(self):
        return self.N * self.H * self.W * self.Cin


def _bottleneck(layers, prefix, x, N, H, W, cin, mid, cout, stride, project):
    """Append one ResNet-v1 bottleneck; returns (out tensor name, H_out, W_out)."""
    a1 = LayerSpec(prefix + ".a1", "conv", x, None, prefix + ".a1", N, H, W, cin, mid, 1, 1, 1, 0, True)
    a2 = LayerSpec(prefix + ".a2", "conv", a1.y, None, prefix + ".a2", N, H, W, mid, mid, 3, 3, stride, 1, True)
    Ho, Wo = a2.P, a2.Q
    layers += [a1, a2]
    if project:
        sc = LayerSpec(prefix + ".sc", "conv", x, None, prefix + ".sc", N, H, W, cin, cout, 1, 1, stride, 0, False)
        layers.append(sc)
        res = sc.y
    else:
        res = x
    out = LayerSpec(prefix + ".out", "conv", a2.y, res, prefix + ".out", N, Ho, Wo, mid, cout, 1, 1, 1, 0, True)
    layers.append(out)
    return out.y, Ho, Wo


def bottleneck_stack(N, H, W, cin=64, mid=64, cout=256, nblocks=3):
    """Configs 1 and 2: three bottleneck blocks, the first with a projection shortcut."""
    layers: List[LayerSpec] = []
    x, c = "x0", cin
    for b in range(nblocks):
        x, H, W = _bottleneck(layers, "b%d" % (b + 1), x, N, H, W, c, mid, cout, 1, b == 0)
        c = cout
    for i, l in enumerate(layers):
        l.index = i + 1
    return layers


def identity_block(N, H, W, cin=256, mid=64, prefix="blk"):
    """One bottleneck with an identity shortcut on an input of `cin` channels (blocks 2 and 3 of
    conv2_x): a1 (1x1), a2 (3x3), out (1x1 + x0)."""
    layers: List[LayerSpec] = []
    _bottleneck(layers, prefix, "x0", N, H, W, cin, mid, cin, 1, False)
    for i, l in enumerate(layers):
        l.index = i + 1
    return layers


def resnet_layers(N, depths=(3, 4, 6, 3), image=224, classes=1000):
    """Full ResNet-v1 (50: 3/4/6/3, 101: 3/4/23/3) as fused layers."""
    layers: List[LayerSpec] = []
    stem = LayerSpec("stem", "conv", "x0", None, "stem", N, image, image, 3, 64, 7, 7, 2, 3, True)
    layers.append(stem)
    H = W = stem.P
    pool = LayerSpec("maxpool", "maxpool", stem.y, None, "maxpool", N, H, W, 64, 64, 3, 3, 2, 1, False)
    layers.append(pool)
    H = W = pool.P
    x, c = pool.y, 64
    for s, depth in enumerate(depths):
        mid, cout = 64 << s, 256 << s
        for b in range(depth):
            stride = 2 if (b == 0 and s > 0) else 1
            x, H, W = _bottleneck(layers, "s%d.b%d" % (s + 2, b + 1), x, N, H, W, c, mid, cout,
                                  stride, b == 0)
            c = cout
    layers.append(LayerSpec("avgpool", "avgpool", x, None, "avgpool", N, H, W, c, c, H, W, 1, 0, False))
    layers.append(LayerSpec("fc", "fc", "avgpool", None, "logits", N, 1, 1, c, classes, 1, 1, 1, 0, False))
    for i, l in enumerate(layers):
        l.index = i + 1
    return layers


# --------------------------------------------------------------------------- draws

def make_input(master, shape, dtype):
    """x ~ N(0,1) in NHWC; dtype 'f32' -> float32 array, 'bf16' -> uint16 bit patterns."""
    n = int(np.prod(shape))
    a = rng.normal(master, 0xFFFF0000, n).astype(np.float32).reshape(shape)
    return a if dtype == "f32" else rng.f32_to_bf16_bits(a).reshape(shape)


def make_params(master, layer: LayerSpec, dtype):
    """Kaiming-normal (fan-in) weights in KRSC order and the four BN vectors (fp32)."""
    base = layer.index * 16
    fan_in = layer.R * layer.S * layer.Cin
    nw = layer.Cout * fan_in
    w = rng.normal(master, base + 0, nw, 0.0, float(np.sqrt(2.0 / fan_in))).astype(np.float32)
    w = w.reshape(layer.Cout, layer.R, layer.S, layer.Cin)
    if dtype == "bf16":
        w = rng.f32_to_bf16_bits(w).reshape(layer.Cout, layer.R, layer.S, layer.Cin)
    C = layer.Cout
    if layer.kind == "fc":                      # classifier: weights and a bias, no batch-norm
        bias = rng.normal(master, base + 2, C, 0.0, 0.1).astype(np.float32)
        return {"w": w, "bias": bias}
    gamma = rng.uniform(master, base + 1, C, 0.5, 1.5).astype(np.float32)
    beta = rng.normal(master, base + 2, C, 0.0, 0.1).astype(np.float32)
    mean = rng.normal(master, base + 3, C, 0.0, 0.1).astype(np.float32)
    var = rng.uniform(master, base + 4, C, 0.5, 1.5).astype(np.float32)
    return {"w": w, "gamma": gamma, "beta": beta, "mean": mean, "var": var, "eps": BN_EPS}


def make_labels(master, n, classes):
    """Synthetic labels, uniform over the classes (int64)."""
    return rng.integers(master, 0xFFFF0001, n, classes)


# --------------------------------------------------------------------------- graphs

def cost_model_ns(flops: int, nbytes: int) -> int:
    """Deterministic stand-in for a measured operator time (integer ns).

    max(flops at 1.25e6 flop/ns (half the bf16 matrix peak), bytes at 4000 B/ns (half the
    HBM peak)) + 2000 ns of launch latency.
    It is an *input* to both planners; bench.py replaces it by measured times.
    """
    return max(-(-int(flops) // 1250000), -(-int(nbytes) // 4000)) + 2000


@dataclass
class Graph:
    """Planner input in production order.  tensors[i] = dict(name, bytes, cost_ns, flops,
    flags, parents[list of ids < i]); steps[k] = dict(produces (id or -1), reads, cost_ns)."""
    tensors: list = field(default_factory=list)
    steps: list = field(default_factory=list)
    n_fwd: int = 0
    names: dict = field(default_factory=dict)

    def total_bytes(self):
        return sum(t["bytes"] for t in self.tensors)

    def add_tensor(self, name, nbytes, cost_ns, flops, flags, parents):
        tid = len(self.tensors)
        assert all(p < tid for p in parents)
        self.tensors.append(dict(name=name, bytes=int(nbytes), cost_ns=int(cost_ns),
                                 flops=int(flops), flags=int(flags), parents=sorted(set(parents))))
        self.names[name] = tid
        return tid

    def add_fwd(self, produces, reads, cost_ns):
        assert self.n_fwd == len(self.steps)
        self.steps.append(dict(produces=int(produces), reads=sorted(set(reads)), cost_ns=int(cost_ns)))
        self.n_fwd += 1

    def add_bwd(self, reads, cost_ns):
        self.steps.append(dict(produces=-1, reads=sorted(set(reads)), cost_ns=int(cost_ns)))


def _esize(dtype):
    return 4 if dtype == "f32" else 2


def fused_graph(layers: List[LayerSpec], dtype, with_loss=False, costs=None, rebuild=None) -> Graph:
    """One tensor per fused layer output.  Backward is an access trace: the backward of a
    layer reads its input (weight gradient) and, when it ends in ReLU or is a max-pool,
    its output (mask).  `costs` optionally maps layer name -> measured ns.
    `rebuild` optionally maps a tensor name -> dict(parents=[tensor names], flops, bytes) where a
    recomputation regenerates the tensor by another route than its forward step (a kernel that
    runs several layers from an earlier tensor): the tensor record then carries those parents and
    that route's cost (`costs[name + "@rebuild"]` when measured), the forward step keeps the
    layer's own reads and cost."""
    g = Graph()
    es = _esize(dtype)
    first = layers[0]
    x0 = g.add_tensor("x0", first.in_elems() * es, 0, 0, FLAG_UNCOMPUTABLE, [])
    g.add_fwd(x0, [], 0)
    fwd_cost = {}
    for l in layers:
        reads = [g.names[l.x]] + ([g.names[l.res]] if l.res else [])
        nbytes = l.out_elems() * es
        traffic = l.in_elems() * es + nbytes + (nbytes if l.res else 0)
        c = costs[l.name] if costs and l.name in costs else cost_model_ns(l.flops, traffic)
        rb = rebuild.get(l.y) if rebuild else None
        if rb:
            key = l.name + "@rebuild"
            rc = costs[key] if costs and key in costs else cost_model_ns(rb["flops"], rb["bytes"])
            t = g.add_tensor(l.y, nbytes, rc, rb["flops"], 0, [g.names[p] for p in rb["parents"]])
        else:
            t = g.add_tensor(l.y, nbytes, c, l.flops, 0, reads)
        g.add_fwd(t, reads, c)
        fwd_cost[l.y] = c
    if with_loss:
        lab = g.add_tensor("labels", first.N * 8, 0, 0, FLAG_UNCOMPUTABLE, [])
        g.add_fwd(lab, [], 0)
        logits = g.names[layers[-1].y]
        loss = g.add_tensor("loss", 4, 2000, 0, 0, [logits, lab])
        g.add_fwd(loss, [logits, lab], 2000)
        g.add_bwd([logits, lab], 2000)
    for l in reversed(layers):
        reads = []
        if l.kind in ("conv", "fc", "maxpool", "linear", "attention", "layernorm"):
            reads.append(g.names[l.x])
        if (l.kind == "conv" and l.relu) or l.kind in ("maxpool", "attention") or (l.kind == "linear" and l.act):
            reads.append(g.names[l.y])
        g.add_bwd(reads, 2 * fwd_cost[l.y])
    return g


def opgranular_graph(layers: List[LayerSpec], dtype, with_loss=True, costs=None) -> Graph:
    """Operator granularity: convolution, batch-norm, residual add and ReLU outputs are separate
    tensors (about 177 for ResNet-50).  `costs` optionally maps tensor name -> measured ns."""
    g = Graph()
    es = _esize(dtype)
    first = layers[0]
    x0 = g.add_tensor("x0", first.in_elems() * es, 0, 0, FLAG_UNCOMPUTABLE, [])
    g.add_fwd(x0, [], 0)
    alias = {"x0": x0}
    bwd = []

    def emit(name, nbytes, flops, traffic, parents, bwd_reads):
        c = costs[name] if costs and name in costs else cost_model_ns(flops, traffic)
        t = g.add_tensor(name, nbytes, c, flops, 0, parents)
        g.add_fwd(t, parents, c)
        bwd.append((bwd_reads, 2 * c))
        return t

    for l in layers:
        xin = alias[l.x]
        nb = l.out_elems() * es
        if l.kind == "conv":
            t = emit(l.name + ".conv", nb, l.flops, l.in_elems() * es + nb, [xin], [xin])
            t = emit(l.name + ".bn", nb, 2 * l.out_elems(), 2 * nb, [t], [t])
            if l.res:
                t = emit(l.name + ".add", nb, l.out_elems(), 3 * nb, [t, alias[l.res]], [])
            if l.relu:
                cur = len(g.tensors)
                t = emit(l.name + ".relu", nb, l.out_elems(), 2 * nb, [t], [cur])
        elif l.kind == "maxpool":
            cur = len(g.tensors)
            t = emit(l.name, nb, l.flops, l.in_elems() * es + nb, [xin], [xin, cur])
        elif l.kind == "avgpool":
            t = emit(l.name, nb, l.flops, l.in_elems() * es + nb, [xin], [])
        else:
            t = emit(l.name, nb, l.flops, l.in_elems() * es + nb, [xin], [xin])
        alias[l.y] = t
    if with_loss:
        lab = g.add_tensor("labels", first.N * 8, 0, 0, FLAG_UNCOMPUTABLE, [])
        g.add_fwd(lab, [], 0)
        logits = alias[layers[-1].y]
        loss = g.add_tensor("loss", 4, 2000, 0, 0, [logits, lab])
        g.add_fwd(loss, [logits, lab], 2000)
        g.add_bwd([logits, lab], 2000)
    for reads, c in reversed(bwd):
        g.add_bwd(reads, c)
    return g


def transformer_graph(batch=32, seq=512, hidden=768, heads=12, ffn=3072, nlayers=12) -> Graph:
    """Config 5 (planner and swap sizes only): post-LN encoder, bf16 activations."""
    g = Graph()
    tok = batch * seq
    act = tok * hidden * 2
    att = batch * heads * seq * seq * 2
    ids = g.add_tensor("ids", tok * 8, 0, 0, FLAG_UNCOMPUTABLE, [])
    g.add_fwd(ids, [], 0)
    bwd = []

    def emit(name, nbytes, flops, traffic, parents, bwd_reads):
        c = cost_model_ns(flops, traffic)
        t = g.add_tensor(name, nbytes, c, flops, 0, parents)
        g.add_fwd(t, parents, c)
        bwd.append((bwd_reads, 2 * c))
        return t

    x = emit("emb", act, tok * hidden, 2 * act, [ids], [ids])
    for i in range(nlayers):
        p = "l%d." % i
        gemm = 2 * tok * hidden * hidden
        q = emit(p + "q", act, gemm, 2 * act, [x], [x])
        k = emit(p + "k", act, gemm, 2 * act, [x], [x])
        v = emit(p + "v", act, gemm, 2 * act, [x], [x])
        sc = emit(p + "scores", att, 2 * tok * seq * hidden, 2 * act + att, [q, k], [q, k])
        cur = len(g.tensors)
        pr = emit(p + "probs", att, 5 * batch * heads * seq * seq, 2 * att, [sc], [cur])
        ctx = emit(p + "ctx", act, 2 * tok * seq * hidden, act + att + act, [pr, v], [pr, v])
        proj = emit(p + "proj", act, gemm, 2 * act, [ctx], [ctx])
        cur = len(g.tensors)
        ln1 = emit(p + "ln1", act, 8 * tok * hidden, 3 * act, [x, proj], [cur])
        f1 = emit(p + "ffn1", tok * ffn * 2, 2 * tok * hidden * ffn, act + tok * ffn * 2, [ln1], [ln1])
        ge = emit(p + "gelu", tok * ffn * 2, 8 * tok * ffn, 2 * tok * ffn * 2, [f1], [f1])
        f2 = emit(p + "ffn2", act, 2 * tok * hidden * ffn, act + tok * ffn * 2, [ge], [ge])
        cur = len(g.tensors)
        x = emit(p + "ln2", act, 8 * tok * hidden, 3 * act, [ln1, f2], [cur])
    for reads, c in reversed(bwd):
        g.add_bwd(reads, c)
    return g


def config_graph(cfg: int, costs=None) -> Graph:
    """Planner graph of benchmark configuration 1..5 (fused granularity for 1-4)."""
    if cfg == 1:
        return fused_graph(bottleneck_stack(2, 32, 32), "f32", costs=costs)
    if cfg == 2:
        return fused_graph(bottleneck_stack(32, 56, 56), "bf16", costs=costs)
    if cfg == 3:
        return fused_graph(resnet_layers(128, (3, 4, 6, 3)), "bf16", with_loss=True, costs=costs)
    if cfg == 4:
        return fused_graph(resnet_layers(256, (3, 4, 23, 3)), "bf16", with_loss=True, costs=costs)
    if cfg == 5:
        return transformer_graph()
    raise ValueError("config must be 1..5")
