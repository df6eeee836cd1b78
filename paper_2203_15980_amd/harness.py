"""Step driver around the C ABI: puts a synthetic network on the GPU, runs its forward
pass through delta_recompute_segment and replays a plan (the event list of delta_plan)
against the arena.  torch is used for device memory, streams and events only; every layer
runs in the library's kernels.  Used by the GPU tests, bench.py and the smoke entry."""
import numpy as np
import torch

import synth

from . import binding as B

_OPS = {"conv": B.OP_CONV, "fc": B.OP_CONV, "maxpool": B.OP_MAXPOOL, "avgpool": B.OP_AVGPOOL,
        "linear": B.OP_CONV, "attention": B.OP_ATTENTION, "layernorm": B.OP_LAYERNORM}


def _dev(a, device):
    return torch.from_numpy(np.ascontiguousarray(a)).to(device)


def find_blocks(layers, dtype="bf16"):
    """Bottlenecks the block kernel takes, {name prefix: its tensors in production order}: 1x1 256 -> 64, 3x3
    64 -> 64, 1x1 64 -> 256 + the block's input, ReLU after each, bf16 (.a1, .a2, .out); or the stage's first
    block, 64 input channels, whose shortcut is the projection sc = bn(w . x), 1x1 64 -> 256 without ReLU
    (.a1, .a2, .sc, .out)."""
    blocks = {}
    by_y = {l.y: l for l in layers}
    for l in layers:
        if not l.y.endswith(".a1") or dtype != "bf16":
            continue
        pre = l.y[:-3]
        a2, out = by_y.get(pre + ".a2"), by_y.get(pre + ".out")
        if a2 is None or out is None:
            continue
        if (a2.kind, a2.R, a2.stride, a2.pad, a2.Cin, a2.Cout, a2.relu, a2.x) != ("conv", 3, 1, 1, 64, 64, True, l.y):
            continue
        if (l.kind, l.R, l.stride, l.Cin, l.Cout, l.relu) == ("conv", 1, 1, 256, 64, True):
            if (out.kind, out.R, out.stride, out.Cin, out.Cout, out.relu, out.x, out.res) != ("conv", 1, 1, 64, 256, True, a2.y, l.x):
                continue
            blocks[pre] = (l.y, a2.y, out.y)
        elif (l.kind, l.R, l.stride, l.Cin, l.Cout, l.relu) == ("conv", 1, 1, 64, 64, True):
            sc = by_y.get(pre + ".sc")
            if sc is None or (sc.kind, sc.R, sc.stride, sc.Cin, sc.Cout, bool(sc.relu), sc.x, sc.res) != ("conv", 1, 1, 64, 256, False, l.x, None):
                continue
            if (out.kind, out.R, out.stride, out.Cin, out.Cout, out.relu, out.x, out.res) != ("conv", 1, 1, 64, 256, True, a2.y, sc.y):
                continue
            blocks[pre] = (l.y, a2.y, sc.y, out.y)
    return blocks


def block_rebuild(layers, dtype="bf16"):
    """What a recomputation needs for the tensors of such blocks, for `synth.fused_graph(rebuild=...)`: the block
    kernel regenerates any of them from the block's input alone (DELTA's Recompute action, Sec. 3, Table 1, with
    the block as the recompute segment), so .a2 and .out get that input as their only parent - rebuilding .out
    then needs neither .a1 nor .a2 (nor .sc) in memory - with the flops of every layer the kernel runs for them
    and the bytes of the input and the tensor itself.  .a1 and .sc already come from the input alone."""
    by_y = {l.y: l for l in layers}
    es = 2
    out = {}
    for pre, chain in find_blocks(layers, dtype).items():
        first = by_y[chain[0]]
        for j, n in enumerate(chain):
            l = by_y[n]
            if l.x == first.x and not l.res:
                continue
            runs = [by_y[m] for m in chain[:j + 1] if not (m.endswith(".sc") and not n.endswith(".out"))]
            out[n] = dict(parents=[first.x], flops=sum(m.flops for m in runs),
                          bytes=(first.in_elems() + l.out_elems()) * es)
    return out


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
            elif l.kind in ("linear", "layernorm"):
                p = synth.make_layer_params(master, l, dtype)
                self.params_np[l.name] = p
                if l.kind == "linear":
                    w = _dev(p["w"], device)
                    scale = torch.ones(l.Cout, dtype=torch.float32, device=device)
                    shift = _dev(p["bias"], device)
                    self.keep += [w, scale, shift]
                else:
                    scale, shift = _dev(p["gamma"], device), _dev(p["beta"], device)
                    self.keep += [scale, shift]
            act = 1 if (l.relu and l.kind == "conv") else (B.ACT_GELU if l.act == "gelu" else 0)
            d = B.LayerDesc(x=self.ids[l.x], res=self.ids[l.res] if l.res else B.NO_TENSOR,
                            y=self.ids[l.y], dtype=code, w=w.data_ptr() if w is not None else None,
                            scale=scale.data_ptr() if scale is not None else None,
                            shift=shift.data_ptr() if shift is not None else None,
                            N=l.N, H=l.H, W=l.W, Cin=l.Cin, Cout=l.Cout, R=l.R, S=l.S,
                            stride=l.stride, pad=l.pad, relu=act, op=_OPS[l.kind],
                            eps=float(self.params_np[l.name]["eps"]) if l.kind == "layernorm" else 0.0)
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
        # bottlenecks the block kernel takes: their tensors carry the bits of the per-layer kernels, so wherever all
        # the block's layers run back to back they run as one launch
        self.blocks = find_blocks(layers, dtype)
        self.block_rebuild = False            # True: the plan was made on a graph with `block_rebuild` (see run_plan)
        self._block_descs = {}
        fused = B.layer_array([B.LayerDesc.from_buffer_copy(dsc) for dsc in order])
        pos = {l.y: i for i, l in enumerate(layers)}
        for pre, chain in self.blocks.items():
            if all(pos[chain[j]] == pos[chain[0]] + j for j in range(len(chain))):
                fused[pos[chain[0]]].fuse = B.FUSE_BLOCK
        self.all_layers_fused = fused
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
        self.delta.recompute_segment(self.all_layers_fused)
        if "loss" in self.desc:
            self.load_source(self.ids["labels"])
            self.delta.recompute_segment(self.desc["loss"])

    def recompute(self, name):
        self.delta.recompute_segment(self.desc[name])

    def block_desc(self, prefix, store=None):
        """The layers of bottleneck `prefix` (.a1 / .a2 / .out of an identity block; .a1 / .a2 / .sc / .out of a
        block with a projection shortcut) as one launch of the block kernel; `store`: the tensor names to
        write (default: all).  A fresh array each time."""
        names = list(self.blocks[prefix])
        store = names if store is None else store
        arr = B.layer_array([B.LayerDesc.from_buffer_copy(self.desc[n][0]) for n in names])
        for i, n in enumerate(names):
            arr[i].fuse = (B.FUSE_BLOCK if i == 0 else 0) | (0 if n in store else B.FUSE_NO_STORE)
        return arr

    def _block_launch(self, prefix, stored):
        """`block_desc` for the first `stored` tensors of the block (an int) or for the given tensor names, built
        once (replays call it per step)."""
        names = tuple(self.blocks[prefix][:stored]) if isinstance(stored, int) else tuple(sorted(stored))
        key = (prefix, names)
        arr = self._block_descs.get(key)
        if arr is None:
            arr = self._block_descs[key] = self.block_desc(prefix, store=list(names))
        return arr

    # -- backward pass
    def _is_stem(self, l):
        return l.kind == "conv" and l.R == 7 and l.Cin == 3

    def _gy_masked(self, l):
        return bool(l.relu) and l.y in self.masked_by

    def _by_class(self, l):
        """A 3x3 stride-2 layer whose incoming gradient needs no mask of its own and whose channel
        counts the class-wise weight gradient takes: both gradients run at the output's resolution
        (by parity class of the input pixels), so no zero-filled copy of dL/dy is needed."""
        return (l.kind == "conv" and l.stride == 2 and l.R == 3 and l.S == 3 and l.pad == 1 and self.dtype == "bf16" and
                l.Cin % 128 == 0 and l.Cout % 128 == 0 and (not l.relu or self._gy_masked(l)))

    def _own_gpre(self, l):
        if l.kind != "conv":
            return False
        if self._is_stem(l):
            return bool(l.relu) and not self._gy_masked(l)
        return (l.relu and not self._gy_masked(l)) or (l.stride > 1 and l.R > 1 and not self._by_class(l))

    def _plan_mask_fusion(self):
        """tensor name -> the layer that applies the ReLU mask of the tensor's producer while it
        writes the tensor's gradient: the consumer whose backward runs last (the first in forward
        order), if it is a convolution reading the tensor as its input - its data gradient
        already holds every other consumer's contribution (gx_add) at that point - or a max-pool
        that is the tensor's only consumer (the stem's output in a ResNet)."""
        masked_by = {}
        for prod in self.layers:
            if prod.kind != "conv" or not prod.relu:
                continue
            users = [l for l in self.layers if l.x == prod.y or l.res == prod.y]
            if not users or users[0].x != prod.y:
                continue
            if users[0].kind == "conv" and not self._is_stem(users[0]) and not self._is_stem(prod):
                masked_by[prod.y] = users[0].name
            elif users[0].kind == "maxpool" and len(users) == 1 and self.dtype == "bf16":
                masked_by[prod.y] = users[0].name
        return masked_by

    def enable_backward(self, input_gradient=False, fuse_masks=True):
        """Adds the gradient tensors to the tensor table (re-binds: call while nothing is
        resident), prepares the data-gradient weights, the fp32 weight-gradient buffers and the
        shared workspace.  Gradient tensors are transient: allocated when written, released
        after their last use; they are not part of the planned graph.  `input_gradient`: also
        compute dL/dx0.  `fuse_masks`: a ReLU layer's mask is applied by the data-gradient
        kernel of its output's last consumer where that is a convolution (no separate mask
        kernel, no unmasked gradient tensor).  The 7x7 stem (bf16) has a weight gradient only."""
        d, dev = self.delta, self.device
        if self.dtype != "bf16" and any(l.kind != "conv" for l in self.layers):
            raise ValueError("backward of pooling, classifier and loss is bf16 only")
        self.n_graph = len(self.sizes)
        self.masked_by = self._plan_mask_fusion() if fuse_masks else {}
        self.bwd_ids = {}
        extra = []
        store = np.float32 if self.dtype == "f32" else np.uint16

        def new_tensor(name, nbytes, shape):
            self.bwd_ids[name] = self.n_graph + len(extra)
            extra.append(nbytes)
            self.shapes[name], self.np_dtype[name] = shape, store
            return self.bwd_ids[name]

        top = self.layers[-1]
        self.has_loss = "loss" in self.desc
        new_tensor("g:" + top.y, self.sizes[self.ids[top.y]], self.shapes[top.y])
        for l in self.layers:
            if self._is_stem(l) and (input_gradient or self.dtype != "bf16"):
                raise ValueError("the stem's backward is its bf16 weight gradient only")
            if self._own_gpre(l):
                # at the input's resolution; a 1x1 layer's and the stem's at the output's
                shape = (l.N, l.H, l.W, l.Cout) if (l.R > 1 and not self._is_stem(l)) else self.shapes[l.y]
                new_tensor("gp:" + l.name, int(np.prod(shape)) * self.es, shape)
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
            if l.kind == "fc":
                self.gw[l.name] = torch.zeros(l.Cout * l.Cin + l.Cout, dtype=torch.float32, device=dev)
            elif l.kind == "conv":
                n = l.Cout * l.R * l.S * l.Cin
                if not self._is_stem(l):                  # the data gradient's weights
                    self.wt[l.name] = torch.empty(n * self.es, dtype=torch.uint8, device=dev)
                    d.bwd_weights(fwd, self.wt[l.name].data_ptr())
                self.gw[l.name] = torch.zeros(n, dtype=torch.float32, device=dev)
                ws_bytes = max(ws_bytes, d.backward_workspace(fwd))
        # twice the largest single need: room for the largest partial sums and the largest staging
        # tensor side by side, so that no layer has to wait for weight gradients still in flight
        self.bwd_workspace = torch.empty(2 * ws_bytes, dtype=torch.uint8, device=dev)
        self.input_gradient = input_gradient
        if not self.has_loss:
            n = int(np.prod(self.shapes[top.y]))
            g = synth.normal(self.master, 7001, n).astype(np.float32)
            self.top_gradient_np = (synth.f32_to_bf16_bits(g) if self.dtype == "bf16" else g).reshape(self.shapes[top.y])
            self.sources[self.ids["g:" + top.y]] = _dev(self.top_gradient_np.view(np.uint8).reshape(-1), dev)
        self.pending = {}
        self.by_name = {l.name: l for l in self.layers}
        torch.cuda.synchronize()

    def enable_backward_proxy(self):
        """For networks whose layers have no backward kernels (the transformer encoder): each
        backward step then runs a compute PROXY - the layer's forward kernel twice, without its
        residual operand, into a scratch tensor - which reads what the access trace says the
        backward reads and costs about what a backward costs.  Adds one scratch tensor per
        output size to the tensor table (re-binds: call while nothing is resident)."""
        self.n_graph = len(self.sizes)
        self.proxy_desc = {}
        scratch = {}
        extra = []
        for l in self.layers:
            nbytes = self.sizes[self.ids[l.y]]
            if nbytes not in scratch:
                scratch[nbytes] = self.n_graph + len(extra)
                extra.append(nbytes)
            dsc = B.LayerDesc.from_buffer_copy(self.desc[l.y][0])
            dsc.y, dsc.res = scratch[nbytes], B.NO_TENSOR
            self.proxy_desc[l.name] = (B.layer_array([dsc]), scratch[nbytes])
        self.sizes = self.sizes + extra
        self.delta.bind(self.sizes)

    def backward_proxy_step(self, graph, k):
        """Backward step `k` of synth.fused_graph's step list, as the compute proxy."""
        l = self.layers[len(self.layers) - 1 - (k - graph.n_fwd)]
        arr, sid = self.proxy_desc[l.name]
        self.delta.recompute_segment(arr)
        self.delta.recompute_segment(arr)
        self.delta.release(sid, B.EV_FREE)

    def rebind(self, delta):
        """Moves the net to another context (same tensor table); nothing may be resident."""
        self.delta = delta
        delta.bind(self.sizes)

    def _bwd_plan(self, l, pending):
        """What the backward of layer `l` reads, writes and frees, given the partial gradients
        `pending` (tensor name -> gradient tensor name).  Pure bookkeeping (no GPU call):
        returns (gy, gpre, gx, add, dead, new_pending_entries)."""
        gy = pending[l.y]
        gpre = "gp:" + l.name if self._own_gpre(l) else gy
        want_gx = l.x != "x0" or self.input_gradient
        gx = "g:" + l.x + ":" + l.name if want_gx else None
        add = pending.get(l.x) if want_gx else None
        if add is not None and l.kind != "conv":
            raise ValueError("gradient accumulation at the input of a %s layer needs an add kernel" % l.kind)
        dead, new = [], {}
        if gx:
            new[l.x] = gx
            if add:
                dead.append(add)
        if l.res:
            if l.res in pending:
                raise ValueError("residual gradient would need an add kernel")
            new[l.res] = gpre                     # the shortcut receives gpre; first contribution
        elif gpre != gy:
            dead.append(gpre)
        if gpre != gy or not l.res:
            dead.append(gy)
        return gy, gpre, gx, add, list(dict.fromkeys(dead)), new

    def backward_peak_bytes(self):
        """Largest sum of gradient-tensor bytes alive at once during `backward` (a dry run of the
        bookkeeping): what the arena must hold beyond the activations."""
        top = self.layers[-1]
        first = "g:" + top.y
        live = {first: self.sizes[self.ids[first]]}
        pending = {top.y: first}
        peak = sum(live.values())
        for l in reversed(self.layers):
            gy, gpre, gx, add, dead, new = self._bwd_plan(l, pending)
            for nm in (gpre, gx):
                if nm and nm not in live:
                    live[nm] = self.sizes[self.ids[nm]]
            peak = max(peak, sum(live.values()))
            pending.pop(l.y)
            pending.update(new)
            for nm in dead:
                live.pop(nm, None)
        return peak

    def backward_begin(self):
        """The gradient of the last layer's output: from the loss's backward when the net has a
        loss (logits and labels must be resident), else a seeded synthetic tensor."""
        top = self.layers[-1]
        first = "g:" + top.y
        if self.has_loss:
            desc = B.BwdDesc(fwd=self.desc["loss"][0], gy=B.NO_TENSOR, gpre=B.NO_TENSOR, gx=self.ids[first],
                             gx_add=B.NO_TENSOR, wt=None, gw=None, workspace=None, workspace_bytes=0)
            self.delta.backward_segment([desc])
        else:
            self.load_source(self.ids[first])
        self.pending = {top.y: first}
        self.bwd_trace = []

    def backward_layer(self, l, keep=False):
        """Backward of layer `l`; every consumer of l.y must have run its backward already.
        Frees gradient tensors after their last use unless `keep` (tests read them back)."""
        d = self.delta
        gy, gpre, gx, add, dead, new = self._bwd_plan(l, self.pending)
        self.pending.pop(l.y)
        conv = l.kind == "conv"
        mask_gx = gx is not None and self.masked_by.get(l.x) == l.name
        desc = B.BwdDesc(fwd=self.desc[l.y][0], gy=self.ids[gy], gpre=self.ids[gpre],
                         gx=self.ids[gx] if gx else B.NO_TENSOR, gx_add=self.ids[add] if add else B.NO_TENSOR,
                         mask_gx=int(mask_gx), gy_masked=int(conv and self._gy_masked(l)),
                         wt=self.wt[l.name].data_ptr() if l.name in self.wt else None,
                         gw=self.gw[l.name].data_ptr() if l.name in self.gw else None,
                         workspace=self.bwd_workspace.data_ptr() if conv else None,
                         workspace_bytes=self.bwd_workspace.numel() if conv else 0)
        d.backward_segment([desc])
        self.bwd_trace.append((l.name, gy, gpre, gx, add, bool(mask_gx)))
        self.pending.update(new)
        if not keep:
            for name in dead:
                d.release(self.ids[name], B.EV_FREE)

    def backward(self, keep=False):
        """Whole backward pass, last layer first (forward activations must be resident)."""
        self.backward_begin()
        for l in reversed(self.layers):
            self.backward_layer(l, keep=keep)
        self.delta.backward_join()                 # weight gradients are visible to the compute stream from here

    def backward_step(self, graph, k):
        """Backward step `k` of synth.fused_graph's step list: the loss first (when present),
        then the layers in reverse order.  For use as run_plan's `backward` callback."""
        j = k - graph.n_fwd
        if self.has_loss:
            if j == 0:
                self.backward_begin()
                return
            j -= 1
        elif j == 0:
            self.backward_begin()
        self.backward_layer(self.layers[len(self.layers) - 1 - j])
        if j == len(self.layers) - 1:
            self.delta.backward_join()


def run_plan(net, graph, events, backward_proxy=None):
    """One training-step replay.  Forward steps run their layer, backward steps call
    `backward_proxy(step_index)` when given; the plan's events are applied around them in
    issue order (everything of a step before it runs, FREE after).
    Where the three layers of an identity bottleneck that the block kernel takes run back to back with
    nothing of the plan between them - three forward steps without events, or three RECOMPUTE events in
    a row - they run as one launch (the same bits, `Net.blocks`).
    With `net.block_rebuild` (the plan was made on `synth.fused_graph(rebuild=block_rebuild(layers))`: a block's
    tensors have the block's input as their only parent) every RECOMPUTE of .a2 / .out, and every run of RECOMPUTE
    events of one block, is one launch of the block kernel that stores exactly those tensors."""
    d = net.delta
    by_step = {}
    for (k, a, t) in events:
        by_step.setdefault(k, []).append((a, t))
    names = [t["name"] for t in graph.tensors]
    blocks = getattr(net, "blocks", {})
    first_of = {net.ids[chain[0]]: pre for pre, chain in blocks.items()}
    member_of = {net.ids[n]: pre for pre, chain in blocks.items() for n in chain} if getattr(net, "block_rebuild", False) else {}
    from_input = {net.ids[n] for chain in blocks.values() for n in chain
                  if n.endswith((".a1", ".sc"))}            # their per-layer kernel reads the block's input alone
    steps = graph.steps
    fused_away = set()                              # forward steps whose tensor an earlier block launch produced
    for k, st in enumerate(steps):
        post = []
        evs = by_step.get(k, ())
        i = 0
        while i < len(evs):
            a, t = evs[i]
            if a == B.EV_FREE:
                post.append(t)
            elif a in (B.EV_EVICT, B.EV_OFFLOAD, B.EV_DROP_TEMP):
                d.release(t, a)
            elif a == B.EV_RECOMPUTE:
                pre = member_of.get(t)
                if pre is not None:
                    run = [t]
                    while i + len(run) < len(evs) and evs[i + len(run)][0] == B.EV_RECOMPUTE and \
                            member_of.get(evs[i + len(run)][1]) == pre:
                        run.append(evs[i + len(run)][1])
                    if len(run) > 1 or t not in from_input:
                        d.recompute_segment(net._block_launch(pre, [names[r] for r in run]))
                        i += len(run)
                        continue
                    d.recompute_segment(net.desc[names[t]])
                    i += 1
                    continue
                pre = first_of.get(t)
                chain = [net.ids[n] for n in blocks[pre]] if pre is not None else []
                run = 0
                while run < len(chain) and i + run < len(evs) and evs[i + run] == (B.EV_RECOMPUTE, chain[run]):
                    run += 1
                if run >= 2:                        # a1 + a2 (+ out) regenerated from the block's input in one launch
                    d.recompute_segment(net._block_launch(pre, run))
                    i += run
                    continue
                d.recompute_segment(net.desc[names[t]])
            else:
                d.prefetch(t)
            i += 1
        p = st["produces"]
        if p >= 0:
            if p in net.sources:
                net.load_source(p)
            elif k in fused_away:
                pass
            else:
                pre = first_of.get(p)
                fuse = False
                c = [net.ids[n] for n in blocks[pre]] if pre is not None else []
                if pre is not None and k + len(c) - 1 < len(steps):
                    # the next steps produce the block's other tensors, the plan does nothing before them and frees
                    # nothing until after the last: the block's memory is the same a few steps early
                    last = k + len(c) - 1
                    fuse = (all(steps[k + j]["produces"] == c[j] for j in range(1, len(c))) and not post
                            and not any(by_step.get(k + j) for j in range(1, len(c) - 1))
                            and all(a == B.EV_FREE for (a, _) in by_step.get(last, ())))
                if fuse:
                    d.recompute_segment(net._block_launch(pre, len(c)))
                    fused_away.update(range(k + 1, k + len(c)))
                else:
                    d.recompute_segment(net.desc[names[p]])
        elif backward_proxy is not None:
            backward_proxy(k)
        for t in post:
            d.release(t, B.EV_FREE)


class OpNet:
    """A ResNet at OPERATOR granularity (synth.opgranular_graph): convolution, batch normalisation
    with the statistics of the batch, residual add and ReLU are separate launches and separate
    tensors (bf16).  Same interface as Net towards run_plan (delta, desc, sources, load_source).
    Backward, either of two: `enable_backward` - every operator's own backward kernel (convolution
    data and weight gradients, batch normalisation through its batch statistics, ReLU mask,
    pooling, classifier, loss; the add only hands its gradient to both inputs), reading exactly the
    activations the access trace of synth.opgranular_graph names; or `enable_backward_proxy` - the
    operator's forward kernel twice into a scratch tensor where the trace gives it an input."""

    def __init__(self, delta, layers, master, device="cuda:0", with_loss=True):
        self.delta, self.layers, self.master, self.device = delta, layers, master, device
        self.dtype, self.es = "bf16", 2
        self.graph = g = synth.opgranular_graph(layers, "bf16", with_loss=with_loss)
        self.ids = dict(g.names)
        self.sizes = [t["bytes"] for t in g.tensors]
        self.params_np, self.keep, self.desc, self.shapes, self.np_dtype, self.sources = {}, [], {}, {}, {}, {}
        first = layers[0]
        code = B.DTYPE_BF16
        self.x0_np = synth.make_input(master, (first.N, first.H, first.W, first.Cin), "bf16")
        self.shapes["x0"], self.np_dtype["x0"] = self.x0_np.shape, np.uint16
        self.sources[0] = _dev(self.x0_np.view(np.uint8).reshape(-1), device)
        cmax = max(l.Cout for l in layers)
        ones = torch.ones(cmax, dtype=torch.float32, device=device)
        zeros = torch.zeros(cmax, dtype=torch.float32, device=device)
        self.keep += [ones, zeros]
        self.op_names = []                        # in production order
        self.proxy_src = {}                       # op tensor -> the tensor its proxy reads (None: no proxy)
        self.op_inputs = {}                       # op tensor -> (x tensor name, second input's name or None)
        self.op_layer = {}                        # op tensor -> the LayerSpec it comes from
        alias = {"x0": "x0"}
        names_by_id = {v: k for k, v in self.ids.items()}

        def emit(name, shape, proxy_x, **kw):
            self.desc[name] = B.layer_array([B.LayerDesc(y=self.ids[name], dtype=code, **kw)])
            self.shapes[name], self.np_dtype[name] = shape, np.uint16
            self.op_names.append(name)
            self.proxy_src[name] = proxy_x
            self.op_inputs[name] = (names_by_id[kw["x"]], names_by_id[kw["res"]] if kw["res"] != B.NO_TENSOR else None)
            self.op_layer[name] = l

        for l in layers:
            xin = alias[l.x]
            geo = dict(N=l.N, H=l.H, W=l.W, Cin=l.Cin, Cout=l.Cout, R=l.R, S=l.S, stride=l.stride, pad=l.pad)
            oshape = (l.N, l.P, l.Q, l.Cout)
            same = dict(N=l.N, H=l.P, W=l.Q, Cin=l.Cout, Cout=l.Cout, R=1, S=1, stride=1, pad=0)
            if l.kind == "conv":
                p = synth.make_params(master, l, "bf16")
                self.params_np[l.name] = p
                w, gamma, beta = _dev(p["w"], device), _dev(p["gamma"], device), _dev(p["beta"], device)
                self.keep += [w, gamma, beta]
                t = l.name + ".conv"
                emit(t, oshape, xin, x=self.ids[xin], res=B.NO_TENSOR, w=w.data_ptr(), scale=ones.data_ptr(),
                     shift=zeros.data_ptr(), relu=0, op=B.OP_CONV, **geo)
                emit(l.name + ".bn", oshape, t, x=self.ids[t], res=B.NO_TENSOR, w=None, scale=gamma.data_ptr(),
                     shift=beta.data_ptr(), relu=0, op=B.OP_BATCHNORM, eps=float(p["eps"]), **same)
                t = l.name + ".bn"
                if l.res:
                    emit(l.name + ".add", oshape, None, x=self.ids[t], res=self.ids[alias[l.res]], w=None, scale=None,
                         shift=None, relu=0, op=B.OP_ADD, **same)
                    t = l.name + ".add"
                if l.relu:
                    emit(l.name + ".relu", oshape, l.name + ".relu", x=self.ids[t], res=B.NO_TENSOR, w=None, scale=None,
                         shift=None, relu=0, op=B.OP_RELU, **same)
                    t = l.name + ".relu"
            elif l.kind in ("maxpool", "avgpool"):
                t = l.name
                emit(t, oshape, xin if l.kind == "maxpool" else None, x=self.ids[xin], res=B.NO_TENSOR, w=None, scale=None,
                     shift=None, relu=0, op=_OPS[l.kind], **geo)
            elif l.kind == "fc":
                p = synth.make_params(master, l, "bf16")
                self.params_np[l.name] = p
                w, bias = _dev(p["w"], device), _dev(p["bias"], device)
                self.keep += [w, bias]
                t = l.name
                emit(t, oshape, xin, x=self.ids[xin], res=B.NO_TENSOR, w=w.data_ptr(), scale=ones.data_ptr(),
                     shift=bias.data_ptr(), relu=0, op=B.OP_CONV, **geo)
            else:
                raise ValueError("layer kind %r has no operator-granular form" % l.kind)
            alias[l.y] = t
        self.alias = alias
        self.with_loss = with_loss
        if with_loss:
            last = layers[-1]
            self.labels_np = synth.make_labels(master, last.N, last.Cout)
            self.sources[self.ids["labels"]] = _dev(self.labels_np.view(np.uint8).reshape(-1), device)
            self.shapes["labels"], self.np_dtype["labels"] = (last.N,), np.int64
            d = B.LayerDesc(x=self.ids[alias[last.y]], res=self.ids["labels"], y=self.ids["loss"], dtype=code,
                            w=None, scale=None, shift=None, N=last.N, H=1, W=1, Cin=last.Cout, Cout=1,
                            R=1, S=1, stride=1, pad=0, relu=0, op=B.OP_SOFTMAX_CE)
            self.desc["loss"] = B.layer_array([d])
            self.shapes["loss"], self.np_dtype["loss"] = (1,), np.float32
        self.all_ops = B.layer_array([self.desc[n][0] for n in self.op_names])
        torch.cuda.synchronize()

    _view = Net._view
    read = Net.read
    load_source = Net.load_source
    rebind = Net.rebind

    def forward(self):
        self.load_source(0)
        self.delta.recompute_segment(self.all_ops)
        if self.with_loss:
            self.load_source(self.ids["labels"])
            self.delta.recompute_segment(self.desc["loss"])

    def enable_backward_proxy(self):
        """Adds one scratch tensor per output size (re-binds: call while nothing is resident)."""
        n_graph = len(self.sizes)
        scratch, extra, self.proxy_desc = {}, [], {}
        for name in self.op_names:
            src = self.proxy_src[name]
            if src is None:
                continue
            nbytes = self.sizes[self.ids[name]]
            if nbytes not in scratch:
                scratch[nbytes] = n_graph + len(extra)
                extra.append(nbytes)
            dsc = B.LayerDesc.from_buffer_copy(self.desc[name][0])
            dsc.x, dsc.y = self.ids[src], scratch[nbytes]
            self.proxy_desc[name] = (B.layer_array([dsc]), scratch[nbytes])
        self.sizes = self.sizes + extra
        self.delta.bind(self.sizes)

    def backward_proxy_step(self, graph, k):
        j = k - graph.n_fwd
        if self.with_loss:
            if j == 0:
                return                            # the loss's backward: one tiny kernel, not modelled
            j -= 1
        name = self.op_names[len(self.op_names) - 1 - j]
        if name not in self.proxy_desc:
            return
        arr, sid = self.proxy_desc[name]
        self.delta.recompute_segment(arr)
        self.delta.recompute_segment(arr)
        self.delta.release(sid, B.EV_FREE)

    # ---------------------------------------------------------------- true backward
    def _kind(self, name):
        op = self.desc[name][0].op
        if op == B.OP_CONV:
            return "fc" if self.op_layer[name].kind == "fc" else "conv"
        return {B.OP_BATCHNORM: "bn", B.OP_RELU: "relu", B.OP_ADD: "add", B.OP_MAXPOOL: "maxpool",
                B.OP_AVGPOOL: "avgpool"}[op]

    def _dilated(self, name):
        """A strided convolution wider than 1x1 (the stem aside, which has no data gradient)."""
        l = self.op_layer[name]
        by_class = l.stride == 2 and l.R == 3 and l.S == 3 and l.pad == 1 and l.Cin % 128 == 0 and l.Cout % 128 == 0
        return self._kind(name) == "conv" and l.stride > 1 and l.R > 1 and self.op_inputs[name][0] != "x0" and not by_class

    def enable_backward(self):
        """Adds the gradient tensors to the tensor table (re-binds: call while nothing is
        resident), prepares the data gradients' weights and allocates the parameter gradients
        (outside the arena, fp32) and the workspace.  The network's input gets no gradient."""
        d, dev = self.delta, self.device
        self.n_graph = len(self.sizes)
        extra = []

        def new_tensor(name, like):
            self.ids[name] = self.n_graph + len(extra)
            extra.append(self.sizes[self.ids[like]])
            self.shapes[name], self.np_dtype[name] = self.shapes[like], np.uint16

        top = self.op_names[-1]
        if not self.with_loss:
            raise ValueError("the operator-granular backward starts from the loss")
        new_tensor("g:" + top, top)
        for name in self.op_names:
            x, res = self.op_inputs[name]
            if self._kind(name) != "add" and x != "x0":
                new_tensor("g:" + x + ":" + name, x)
            if self._dilated(name):               # dL/dy spread to the input's resolution
                l = self.op_layer[name]
                self.ids["gp:" + name] = self.n_graph + len(extra)
                extra.append(l.N * l.H * l.W * l.Cout * 2)
                self.shapes["gp:" + name], self.np_dtype["gp:" + name] = (l.N, l.H, l.W, l.Cout), np.uint16
        self.sizes = self.sizes + extra
        d.bind(self.sizes)
        self.wt, self.gw = {}, {}
        ws_bytes = 16
        for name in self.op_names:
            kind, fwd, l = self._kind(name), self.desc[name][0], self.op_layer[name]
            if kind == "fc":
                self.gw[name] = torch.zeros(l.Cout * l.Cin + l.Cout, dtype=torch.float32, device=dev)
            elif kind == "bn":
                self.gw[name] = torch.zeros(2 * l.Cout, dtype=torch.float32, device=dev)
            elif kind == "conv":
                n = l.Cout * l.R * l.S * l.Cin
                if self.op_inputs[name][0] != "x0":
                    self.wt[name] = torch.empty(n * 2, dtype=torch.uint8, device=dev)
                    d.bwd_weights(fwd, self.wt[name].data_ptr())
                self.gw[name] = torch.zeros(n, dtype=torch.float32, device=dev)
                ws_bytes = max(ws_bytes, d.backward_workspace(fwd))
        self.bwd_workspace = torch.empty(2 * ws_bytes, dtype=torch.uint8, device=dev)
        torch.cuda.synchronize()

    def _bwd_plan(self, name, pending, refs):
        """Bookkeeping of one operator's backward given `pending` (tensor -> name of the gradient
        accumulated so far) and `refs` (gradient tensor -> readers left).  No GPU call.
        Returns (gy, gx, add, dead gradient tensors)."""
        kind = self._kind(name)
        x, res = self.op_inputs[name]
        gy = pending.pop(name)
        dead = []
        if kind == "add":                          # both inputs receive gy itself
            for t in (x, res):
                if t in pending:
                    raise ValueError("gradient accumulation at %s would need an add kernel" % t)
                pending[t] = gy
            refs[gy] += 1                          # one reader became two
            return gy, None, None, dead
        gx = add = None
        if x != "x0":
            gx = "g:" + x + ":" + name
            add = pending.get(x)
            if add is not None and kind != "conv":
                raise ValueError("gradient accumulation at the input of %s needs an add kernel" % name)
            pending[x] = gx
            refs[gx] = 1
            if add is not None:
                refs[add] -= 1
                if refs[add] == 0:
                    dead.append(add)
        refs[gy] -= 1
        if refs[gy] == 0:
            dead.append(gy)
        return gy, gx, add, dead

    def backward_peak_bytes(self):
        """Largest sum of gradient-tensor bytes alive at once during the backward pass (dry run)."""
        first = "g:" + self.op_names[-1]
        pending, refs = {self.op_names[-1]: first}, {first: 1}
        live = {first}
        size = lambda n: self.sizes[self.ids[n]]
        peak = size(first)
        for name in reversed(self.op_names):
            gy, gx, add, dead = self._bwd_plan(name, pending, refs)
            if gx:
                live.add(gx)
            peak = max(peak, sum(size(n) for n in live) + (size("gp:" + name) if self._dilated(name) else 0))
            live.difference_update(dead)
        return peak

    def backward_begin(self):
        first = "g:" + self.op_names[-1]
        desc = B.BwdDesc(fwd=self.desc["loss"][0], gy=B.NO_TENSOR, gpre=B.NO_TENSOR, gx=self.ids[first],
                         gx_add=B.NO_TENSOR, wt=None, gw=None, workspace=None, workspace_bytes=0)
        self.delta.backward_segment([desc])
        self.pending, self.refs = {self.op_names[-1]: first}, {first: 1}
        self.bwd_trace = []

    def backward_op(self, name, keep=False):
        """Backward of the operator that produces `name` (all its consumers have run theirs)."""
        d = self.delta
        gy, gx, add, dead = self._bwd_plan(name, self.pending, self.refs)
        kind = self._kind(name)
        self.bwd_trace.append((name, kind, gy, gx, add))
        if kind != "add":
            conv = kind == "conv"
            gpre = "gp:" + name if self._dilated(name) else gy
            if gpre != gy:
                dead = dead + [gpre]
            desc = B.BwdDesc(fwd=self.desc[name][0], gy=self.ids[gy], gpre=self.ids[gpre],
                             gx=self.ids[gx] if gx else B.NO_TENSOR, gx_add=self.ids[add] if add else B.NO_TENSOR,
                             mask_gx=0, gy_masked=0,
                             wt=self.wt[name].data_ptr() if name in self.wt else None,
                             gw=self.gw[name].data_ptr() if name in self.gw else None,
                             workspace=self.bwd_workspace.data_ptr() if conv else None,
                             workspace_bytes=self.bwd_workspace.numel() if conv else 0)
            d.backward_segment([desc])
        if not keep:
            for g in dead:
                d.release(self.ids[g], B.EV_FREE)

    def backward(self, keep=False):
        self.backward_begin()
        for name in reversed(self.op_names):
            self.backward_op(name, keep=keep)
        self.delta.backward_join()

    def backward_step(self, graph, k):
        """Backward step `k` of synth.opgranular_graph's step list: the loss, then the operators in
        reverse order.  For use as run_plan's backward callback."""
        j = k - graph.n_fwd
        if j == 0:
            self.backward_begin()
            return
        self.backward_op(self.op_names[len(self.op_names) - j])
        if j == len(self.op_names):
            self.delta.backward_join()
