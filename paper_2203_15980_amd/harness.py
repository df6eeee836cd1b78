"""Step driver around the C ABI: puts a synthetic network on the GPU, runs its forward
pass through delta_recompute_segment and replays a plan (the event list of delta_plan)
against the arena.  torch is used for device memory, streams and events only; every layer
runs in the library's kernels.  Used by the GPU tests, bench.py and the smoke entry."""
import numpy as np
import torch

import synth

from . import binding as B

_OPS = {"conv": B.OP_CONV, "fc": B.OP_CONV, "maxpool": B.OP_MAXPOOL, "avgpool": B.OP_AVGPOOL}


def _dev(a, device):
    return torch.from_numpy(np.ascontiguousarray(a)).to(device)


class Net:
    """Weights, folded batch-norm factors and layer descriptors of a list of synth.LayerSpec
    layers, resident on the GPU.  Tensor ids follow synth.fused_graph (x0 is 0; with
    `with_loss` the labels and the loss come last)."""

    def __init__(self, delta, layers, dtype, master, device="cuda:0", with_loss=False):
        self.delta, self.layers, self.dtype, self.master = delta, layers, dtype, master
        self.device = device
        self.es = 4 if dtype == "f32" else 2
        self.graph = synth.fused_graph(layers, dtype, with_loss=with_loss)
        self.ids = dict(self.graph.names)
        self.sizes = [t["bytes"] for t in self.graph.tensors]
        self.params_np = {}
        self.keep = []
        self.desc = {}
        self.shapes = {}
        self.np_dtype = {}
        self.sources = {}                     # uncomputable tensors: id -> device bytes to copy in
        first = layers[0]
        code = B.DTYPE_F32 if dtype == "f32" else B.DTYPE_BF16
        store = np.float32 if dtype == "f32" else np.uint16
        self.in_shape = (first.N, first.H, first.W, first.Cin)
        self.x0_np = synth.make_input(master, self.in_shape, dtype)
        self.shapes["x0"], self.np_dtype["x0"] = self.in_shape, store
        self.sources[0] = _dev(self.x0_np.view(np.uint8).reshape(-1), device)
        for l in layers:
            if l.kind not in _OPS:
                raise ValueError("layer kind %r has no kernel" % l.kind)
            w = scale = shift = None
            if l.kind in ("conv", "fc"):
                p = synth.make_params(master, l, dtype)
                self.params_np[l.name] = p
                w = _dev(p["w"], device)
                if l.kind == "conv":
                    bn = [_dev(p[k], device) for k in ("gamma", "beta", "mean", "var")]
                    scale = torch.empty(l.Cout, dtype=torch.float32, device=device)
                    shift = torch.empty(l.Cout, dtype=torch.float32, device=device)
                    delta.bn_fold(bn[0].data_ptr(), bn[1].data_ptr(), bn[2].data_ptr(), bn[3].data_ptr(),
                                  float(p["eps"]), l.Cout, scale.data_ptr(), shift.data_ptr())
                    self.keep += bn
                else:
                    scale = torch.ones(l.Cout, dtype=torch.float32, device=device)
                    shift = _dev(p["bias"], device)
                self.keep += [w, scale, shift]
            d = B.LayerDesc(x=self.ids[l.x], res=self.ids[l.res] if l.res else B.NO_TENSOR,
                            y=self.ids[l.y], dtype=code, w=w.data_ptr() if w is not None else None,
                            scale=scale.data_ptr() if scale is not None else None,
                            shift=shift.data_ptr() if shift is not None else None,
                            N=l.N, H=l.H, W=l.W, Cin=l.Cin, Cout=l.Cout, R=l.R, S=l.S,
                            stride=l.stride, pad=l.pad, relu=1 if (l.relu and l.kind == "conv") else 0,
                            op=_OPS[l.kind])
            self.desc[l.y] = B.layer_array([d])
            self.shapes[l.y], self.np_dtype[l.y] = (l.N, l.P, l.Q, l.Cout), store
        order = [self.desc[l.y][0] for l in layers]
        if with_loss:
            last = layers[-1]
            self.labels_np = synth.make_labels(master, last.N, last.Cout)
            self.sources[self.ids["labels"]] = _dev(self.labels_np.view(np.uint8).reshape(-1), device)
            self.shapes["labels"], self.np_dtype["labels"] = (last.N,), np.int64
            d = B.LayerDesc(x=self.ids[last.y], res=self.ids["labels"], y=self.ids["loss"], dtype=code,
                            w=None, scale=None, shift=None, N=last.N, H=1, W=1, Cin=last.Cout, Cout=1,
                            R=1, S=1, stride=1, pad=0, relu=0, op=B.OP_SOFTMAX_CE)
            self.desc["loss"] = B.layer_array([d])
            self.shapes["loss"], self.np_dtype["loss"] = (1,), np.float32
        self.all_layers = B.layer_array(order)
        self.by_tensor = {self.ids[l.y]: l for l in layers}
        torch.cuda.synchronize()

    # -- raw access to arena contents
    def _view(self, tensor_id):
        ptr = self.delta.tensor_ptr(tensor_id)
        off = ptr - self.delta.arena.data_ptr()
        return self.delta.arena[off:off + self.sizes[tensor_id]]

    def read(self, name):
        """Stored bits of a resident tensor as a numpy array (float32, uint16 bf16 bits, ...)."""
        raw = self._view(self.ids[name])
        torch.cuda.current_stream().synchronize()
        return raw.cpu().numpy().view(self.np_dtype[name]).reshape(self.shapes[name])

    def load_source(self, tensor_id):
        """Brings an uncomputable tensor (network input, labels) onto the GPU."""
        self.delta.alloc(tensor_id)
        self._view(tensor_id).copy_(self.sources[tensor_id], non_blocking=True)

    def load_input(self):
        self.load_source(0)

    def forward(self):
        """Inputs plus every layer (and the loss when present), nothing released."""
        self.load_input()
        self.delta.recompute_segment(self.all_layers)
        if "loss" in self.desc:
            self.load_source(self.ids["labels"])
            self.delta.recompute_segment(self.desc["loss"])

    def recompute(self, name):
        self.delta.recompute_segment(self.desc[name])

    # -- backward pass (convolution layers with stride 1 and "same" padding)
    def enable_backward(self, input_gradient=False):
        """Adds the gradient tensors to the tensor table (re-binds: call while nothing is
        resident), prepares the data-gradient weights, the fp32 weight-gradient buffers and the
        shared workspace.  Gradient tensors are transient: allocated when written, released
        after their last use; they are not part of the planned graph.  `input_gradient`: also
        compute dL/dx0."""
        d, dev = self.delta, self.device
        self.n_graph = len(self.sizes)
        self.bwd_ids, self.bwd_layers = {}, []
        extra = []

        def new_tensor(name, nbytes, shape):
            self.bwd_ids[name] = self.n_graph + len(extra)
            extra.append(nbytes)
            self.shapes[name], self.np_dtype[name] = shape, (np.float32 if self.dtype == "f32" else np.uint16)
            return self.bwd_ids[name]

        top = self.layers[-1]
        new_tensor("g:" + top.y, self.sizes[self.ids[top.y]], self.shapes[top.y])
        for l in self.layers:
            if l.kind != "conv":
                raise ValueError("backward: layer kind %r has no backward kernel" % l.kind)
            if l.relu:
                new_tensor("gp:" + l.name, self.sizes[self.ids[l.y]], self.shapes[l.y])
            if l.x != "x0" or input_gradient:
                new_tensor("g:" + l.x + ":" + l.name, self.sizes[self.ids[l.x]], self.shapes[l.x])
        self.all_sizes = self.sizes + extra
        for name, tid in self.bwd_ids.items():
            self.ids[name] = tid
        self.sizes = self.all_sizes
        d.bind(self.all_sizes)
        self.wt, self.gw = {}, {}
        ws_bytes = 16
        for l in self.layers:
            fwd = self.desc[l.y][0]
            n = l.Cout * l.R * l.S * l.Cin
            self.wt[l.name] = torch.empty(n * self.es, dtype=torch.uint8, device=dev)
            d.bwd_weights(fwd, self.wt[l.name].data_ptr())
            self.gw[l.name] = torch.zeros(n, dtype=torch.float32, device=dev)
            ws_bytes = max(ws_bytes, d.backward_workspace(fwd))
        self.bwd_workspace = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
        self.input_gradient = input_gradient
        self.top_gradient_np = synth.f32_to_bf16_bits(
            synth.normal(self.master, 7001, int(np.prod(self.shapes[top.y]))).astype(np.float32)
        ).reshape(self.shapes[top.y]) if self.dtype == "bf16" else synth.normal(
            self.master, 7001, int(np.prod(self.shapes[top.y]))).astype(np.float32).reshape(self.shapes[top.y])
        self.sources[self.ids["g:" + top.y]] = _dev(self.top_gradient_np.view(np.uint8).reshape(-1), dev)
        self.pending = {}
        torch.cuda.synchronize()

    def backward_begin(self):
        """Loads the gradient of the last layer's output (seeded, synthetic: it stands in for the
        loss's gradient)."""
        top = self.layers[-1]
        self.load_source(self.ids["g:" + top.y])
        self.pending = {top.y: "g:" + top.y}
        self.bwd_trace = []

    def backward_layer(self, l, keep=False):
        """Backward of layer `l`; every consumer of l.y must have run its backward already.
        Frees gradient tensors after their last use unless `keep` (tests read them back)."""
        d = self.delta
        fwd = self.desc[l.y][0]
        gy_name = self.pending.pop(l.y)
        gpre_name = "gp:" + l.name if l.relu else gy_name
        want_gx = l.x != "x0" or self.input_gradient
        gx_name = "g:" + l.x + ":" + l.name if want_gx else None
        add_name = self.pending.get(l.x) if want_gx else None
        desc = B.BwdDesc(fwd=fwd, gy=self.ids[gy_name], gpre=self.ids[gpre_name],
                         gx=self.ids[gx_name] if gx_name else B.NO_TENSOR,
                         gx_add=self.ids[add_name] if add_name else B.NO_TENSOR,
                         wt=self.wt[l.name].data_ptr(),
                         gw=self.gw[l.name].data_ptr() if self.dtype == "bf16" else None,   # weight gradient: bf16 only
                         workspace=self.bwd_workspace.data_ptr(), workspace_bytes=self.bwd_workspace.numel())
        d.backward_segment([desc])
        self.bwd_trace.append((l.name, gy_name, gpre_name, gx_name, add_name))
        dead = []
        if gx_name:
            self.pending[l.x] = gx_name
            if add_name:
                dead.append(add_name)
        if l.res:
            # the residual branch receives gpre; in a ResNet this is its first contribution
            assert l.res not in self.pending, "residual gradient would need an add kernel"
            self.pending[l.res] = gpre_name
        elif gpre_name != gy_name:
            dead.append(gpre_name)
        if gpre_name != gy_name or not l.res:
            dead.append(gy_name)
        if not keep:
            for name in dict.fromkeys(dead):
                d.release(self.ids[name], B.EV_FREE)

    def backward(self, keep=False):
        """Whole backward pass, last layer first (forward activations must be resident)."""
        self.backward_begin()
        for l in reversed(self.layers):
            self.backward_layer(l, keep=keep)


def run_plan(net, graph, events, backward_proxy=None):
    """One training-step replay.  Forward steps run their layer, backward steps call
    `backward_proxy(step_index)` when given; the plan's events are applied around them in
    issue order (everything of a step before it runs, FREE after)."""
    d = net.delta
    by_step = {}
    for (k, a, t) in events:
        by_step.setdefault(k, []).append((a, t))
    names = [t["name"] for t in graph.tensors]
    for k, st in enumerate(graph.steps):
        post = []
        for (a, t) in by_step.get(k, ()):
            if a == B.EV_FREE:
                post.append(t)
            elif a in (B.EV_EVICT, B.EV_OFFLOAD, B.EV_DROP_TEMP):
                d.release(t, a)
            elif a == B.EV_RECOMPUTE:
                d.recompute_segment(net.desc[names[t]])
            else:
                d.prefetch(t)
        if st["produces"] >= 0:
            if st["produces"] in net.sources:
                net.load_source(st["produces"])
            else:
                d.recompute_segment(net.desc[names[st["produces"]]])
        elif backward_proxy is not None:
            backward_proxy(k)
        for t in post:
            d.release(t, B.EV_FREE)
