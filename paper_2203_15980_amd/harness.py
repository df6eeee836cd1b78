"""Step driver around the C ABI: puts a synthetic network on the GPU, runs its forward
pass through delta_recompute_segment and replays a plan (the event list of delta_plan)
against the arena.  torch is used for device memory, streams and events only; every layer
runs in the library's kernels.  Used by the GPU tests, bench.py and the smoke entry."""
import ctypes

import numpy as np
import torch

import synth

from . import binding as B


def _dev(a, device):
    return torch.from_numpy(np.ascontiguousarray(a)).to(device)


class Net:
    """Weights, folded batch-norm factors and layer descriptors of a list of synth.LayerSpec
    conv layers, resident on the GPU.  Tensor ids follow synth.fused_graph (x0 is 0)."""

    def __init__(self, delta, layers, dtype, master, device="cuda:0"):
        self.delta, self.layers, self.dtype, self.master = delta, layers, dtype, master
        self.device = device
        self.es = 4 if dtype == "f32" else 2
        self.graph = synth.fused_graph(layers, dtype)
        self.ids = dict(self.graph.names)
        self.sizes = [t["bytes"] for t in self.graph.tensors]
        self.params_np = {}
        self.keep = []
        self.desc = {}
        first = layers[0]
        self.in_shape = (first.N, first.H, first.W, first.Cin)
        self.x0_np = synth.make_input(master, self.in_shape, dtype)
        self.x0_dev = _dev(self.x0_np.view(np.uint8).reshape(-1), device)
        for l in layers:
            if l.kind != "conv":
                raise ValueError("layer kind %r has no kernel" % l.kind)
            p = synth.make_params(master, l, dtype)
            self.params_np[l.name] = p
            w = _dev(p["w"], device)
            bn = [_dev(p[k], device) for k in ("gamma", "beta", "mean", "var")]
            scale = torch.empty(l.Cout, dtype=torch.float32, device=device)
            shift = torch.empty(l.Cout, dtype=torch.float32, device=device)
            delta.bn_fold(bn[0].data_ptr(), bn[1].data_ptr(), bn[2].data_ptr(), bn[3].data_ptr(),
                          float(p["eps"]), l.Cout, scale.data_ptr(), shift.data_ptr())
            self.keep += [w, scale, shift] + bn
            d = B.LayerDesc(x=self.ids[l.x], res=self.ids[l.res] if l.res else B.NO_TENSOR,
                            y=self.ids[l.y], dtype=B.DTYPE_F32 if dtype == "f32" else B.DTYPE_BF16,
                            w=w.data_ptr(), scale=scale.data_ptr(), shift=shift.data_ptr(),
                            N=l.N, H=l.H, W=l.W, Cin=l.Cin, Cout=l.Cout, R=l.R, S=l.S,
                            stride=l.stride, pad=l.pad, relu=1 if l.relu else 0)
            self.desc[l.y] = B.layer_array([d])
        self.by_tensor = {self.ids[l.y]: l for l in layers}
        self.all_layers = B.layer_array([self.desc[l.y][0] for l in layers])
        torch.cuda.synchronize()

    # -- raw access to arena contents
    def _view(self, tensor_id):
        ptr = self.delta.tensor_ptr(tensor_id)
        off = ptr - self.delta.arena.data_ptr()
        return self.delta.arena[off:off + self.sizes[tensor_id]]

    def read(self, name):
        """Stored bits of a resident tensor as a numpy array (float32 or uint16 bf16 bits)."""
        tid = self.ids[name]
        raw = self._view(tid)
        torch.cuda.current_stream().synchronize()
        a = raw.cpu().numpy()
        l = self.by_tensor.get(tid)
        shape = self.in_shape if l is None else (l.N, l.P, l.Q, l.Cout)
        return a.view(np.float32 if self.dtype == "f32" else np.uint16).reshape(shape)

    def load_input(self):
        self.delta.alloc(0)
        self._view(0).copy_(self.x0_dev, non_blocking=True)

    def forward(self):
        """x0 plus every layer, nothing released."""
        self.load_input()
        self.delta.recompute_segment(self.all_layers)

    def recompute(self, name):
        self.delta.recompute_segment(self.desc[name])


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
            if st["produces"] == 0:
                net.load_input()
            else:
                d.recompute_segment(net.desc[names[st["produces"]]])
        elif backward_proxy is not None:
            backward_proxy(k)
        for t in post:
            d.release(t, B.EV_FREE)
