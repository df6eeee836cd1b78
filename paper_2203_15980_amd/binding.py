"""ctypes binding of include/delta.h.  Same names as the C entry points, minus the prefix."""
import ctypes as C
import os

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libdelta.so")

OK, ERR_INVALID, ERR_INFEASIBLE, ERR_OOM_ARENA = 0, -1, -2, -3
ERR_OOM_PINNED, ERR_STATE, ERR_BUFFER, ERR_HIP = -4, -5, -6, -7
F_UNCOMPUTABLE, F_EVICT_PINNED, F_OFFLOAD_PINNED = 1, 2, 4
FILTER_BASE, FILTER_LRU, FILTER_GREEDY = 0, 1, 2
EV_EVICT, EV_OFFLOAD, EV_RECOMPUTE, EV_RELOAD_PREFETCH = 1, 2, 3, 4
EV_RELOAD_DEMAND, EV_FREE, EV_DROP_TEMP = 5, 6, 7
DTYPE_F32, DTYPE_BF16 = 0, 1
SYNC_D2H, SYNC_H2D, SYNC_COMPUTE, SYNC_ALL = 1, 2, 4, 7
DIR_D2H, DIR_H2D, DIR_BOTH = 0, 1, 2
NO_TENSOR = 0xFFFFFFFF
OP_CONV, OP_MAXPOOL, OP_AVGPOOL, OP_SOFTMAX_CE, OP_ATTENTION, OP_LAYERNORM = 0, 1, 2, 3, 4, 5
OP_BATCHNORM, OP_RELU, OP_ADD = 6, 7, 8
ACT_NONE, ACT_RELU, ACT_GELU = 0, 1, 2
FUSE_NONE, FUSE_BLOCK, FUSE_NO_STORE = 0, 1, 2

EXPORTS = ["delta_create", "delta_destroy", "delta_last_error", "delta_plan", "delta_bind",
           "delta_alloc", "delta_tensor_ptr", "delta_release", "delta_swap_out", "delta_prefetch",
           "delta_recompute_segment", "delta_sync", "delta_bn_fold", "delta_stats",
           "delta_stats_reset", "delta_set_skip_copies", "delta_probe_hostlink",
           "delta_probe_hbm", "delta_probe_mfma", "delta_layer_kernel", "delta_bwd_weights",
           "delta_backward_workspace", "delta_backward_segment", "delta_backward_join",
           "delta_batchnorm_static", "delta_reserve_pinned"]


class TensorDesc(C.Structure):
    _fields_ = [("bytes", C.c_uint64), ("cost_ns", C.c_uint64), ("flops", C.c_uint64),
                ("flags", C.c_uint32), ("n_parents", C.c_uint32), ("parents", C.POINTER(C.c_uint32))]


class StepDesc(C.Structure):
    _fields_ = [("produces", C.c_int32), ("n_reads", C.c_uint32), ("reads", C.POINTER(C.c_uint32)),
                ("cost_ns", C.c_uint64)]


class PlanParams(C.Structure):
    _fields_ = [("budget_bytes", C.c_uint64), ("trigger_num", C.c_uint32), ("trigger_den", C.c_uint32),
                ("filter", C.c_uint32), ("prefetch_distance", C.c_uint32), ("max_reloads", C.c_uint32),
                ("n_fwd_steps", C.c_uint32), ("bw_d2h_Bps", C.c_uint64), ("bw_h2d_Bps", C.c_uint64),
                ("release_when_short", C.c_uint32), ("repair_rounds", C.c_uint32),
                ("prefetch_rebuild_reads", C.c_uint32)]


class Event(C.Structure):
    _fields_ = [("step", C.c_uint32), ("action", C.c_uint32), ("tensor", C.c_uint32), ("pad", C.c_uint32)]


class LayerDesc(C.Structure):
    _fields_ = [("x", C.c_uint32), ("res", C.c_uint32), ("y", C.c_uint32), ("dtype", C.c_uint32),
                ("w", C.c_void_p), ("scale", C.c_void_p), ("shift", C.c_void_p),
                ("N", C.c_int32), ("H", C.c_int32), ("W", C.c_int32), ("Cin", C.c_int32),
                ("Cout", C.c_int32), ("R", C.c_int32), ("S", C.c_int32), ("stride", C.c_int32),
                ("pad", C.c_int32), ("relu", C.c_uint32), ("op", C.c_uint32), ("eps", C.c_float),
                ("fuse", C.c_uint32)]


class BwdDesc(C.Structure):
    _fields_ = [("fwd", LayerDesc), ("gy", C.c_uint32), ("gpre", C.c_uint32), ("gx", C.c_uint32),
                ("gx_add", C.c_uint32), ("mask_gx", C.c_uint32), ("gy_masked", C.c_uint32), ("wt", C.c_void_p), ("gw", C.c_void_p), ("workspace", C.c_void_p),
                ("workspace_bytes", C.c_uint64)]


class Stats(C.Structure):
    _fields_ = [("arena_bytes", C.c_uint64), ("arena_in_use", C.c_uint64), ("arena_high_water", C.c_uint64),
                ("d2h_bytes", C.c_uint64), ("h2d_bytes", C.c_uint64), ("d2h_copies", C.c_uint64),
                ("h2d_copies", C.c_uint64), ("d2h_ms", C.c_double), ("h2d_ms", C.c_double),
                ("recompute_launches", C.c_uint64), ("recompute_flops", C.c_uint64),
                ("releases_evict", C.c_uint64), ("releases_offload", C.c_uint64),
                ("releases_free", C.c_uint64), ("pinned_bytes", C.c_uint64),
                ("arena_extent_high_water", C.c_uint64), ("arena_top_extent_high_water", C.c_uint64)]

    def as_dict(self):
        return {k: getattr(self, k) for k, _ in self._fields_}


class DeltaError(RuntimeError):
    def __init__(self, status, message):
        super().__init__("delta status %d: %s" % (status, message))
        self.status = status
        self.message = message


_lib = None


def load_library():
    """Loads the in-tree libdelta.so.  Fails loudly when it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    # PyTorch ships its own HIP runtime.  It must be the one already mapped when libdelta.so is
    # loaded, so that the arena pointers and streams torch hands over belong to the same
    # runtime instance as the library's own HIP calls.
    try:
        import torch  # noqa: F401
    except ImportError:
        pass
    if not os.path.exists(LIB_PATH):
        raise RuntimeError("%s is missing: build it with `python -m paper_2203_15980_amd.build` "
                           "(there is no CPU fallback)" % LIB_PATH)
    L = C.CDLL(LIB_PATH)
    vp, u32, u64, i32 = C.c_void_p, C.c_uint32, C.c_uint64, C.c_int32
    sig = {
        "delta_create": (i32, [vp, u64, vp, C.POINTER(vp)]),
        "delta_destroy": (None, [vp]),
        "delta_last_error": (C.c_char_p, [vp]),
        "delta_plan": (i32, [vp, C.POINTER(TensorDesc), u32, C.POINTER(StepDesc), u32,
                             C.POINTER(PlanParams), C.POINTER(Event), u32, C.POINTER(u32),
                             C.POINTER(u64)]),
        "delta_bind": (i32, [vp, C.POINTER(u64), u32]),
        "delta_alloc": (i32, [vp, u32, C.POINTER(vp)]),
        "delta_tensor_ptr": (i32, [vp, u32, C.POINTER(vp)]),
        "delta_release": (i32, [vp, u32, u32]),
        "delta_swap_out": (i32, [vp, u32]),
        "delta_prefetch": (i32, [vp, u32]),
        "delta_recompute_segment": (i32, [vp, C.POINTER(LayerDesc), u32]),
        "delta_sync": (i32, [vp, u32]),
        "delta_bn_fold": (i32, [vp, vp, vp, vp, vp, C.c_float, u32, vp, vp]),
        "delta_stats": (i32, [vp, C.POINTER(Stats)]),
        "delta_stats_reset": (i32, [vp]),
        "delta_set_skip_copies": (i32, [vp, i32]),
        "delta_probe_hostlink": (i32, [vp, u64, u32, u32, C.POINTER(C.c_double)]),
        "delta_probe_hbm": (i32, [vp, u64, u32, C.POINTER(C.c_double)]),
        "delta_probe_mfma": (i32, [vp, u32, C.POINTER(C.c_double)]),
        "delta_layer_kernel": (i32, [vp, C.POINTER(LayerDesc), C.c_char_p, u64]),
        "delta_bwd_weights": (i32, [vp, C.POINTER(LayerDesc), vp]),
        "delta_backward_workspace": (i32, [vp, C.POINTER(LayerDesc), C.POINTER(u64)]),
        "delta_backward_segment": (i32, [vp, C.POINTER(BwdDesc), u32]),
        "delta_backward_join": (i32, [vp]),
        "delta_batchnorm_static": (i32, [vp, vp, vp, vp, vp, u64, u32, C.c_float]),
        "delta_reserve_pinned": (i32, [vp, u64]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(L, name)
        fn.restype, fn.argtypes = res, args
    _lib = L
    return L


def layer_array(descs):
    """Packs a list of LayerDesc (or dicts of its fields) into a contiguous ctypes array."""
    arr = (LayerDesc * len(descs))()
    for i, d in enumerate(descs):
        arr[i] = d if isinstance(d, LayerDesc) else LayerDesc(**d)
    return arr


_OPTIONAL_PLAN_PARAMS = ("release_when_short", "repair_rounds", "prefetch_rebuild_reads")   # 0 when the caller leaves them out


def _plan_params(params):
    return PlanParams(**{k: int(params.get(k, 0) if k in _OPTIONAL_PLAN_PARAMS else params[k])
                         for k, _ in PlanParams._fields_})


def _marshal_graph(tensors, steps, params):
    keep = []
    td = (TensorDesc * len(tensors))()
    for i, t in enumerate(tensors):
        par = (C.c_uint32 * len(t["parents"]))(*t["parents"])
        keep.append(par)
        td[i] = TensorDesc(t["bytes"], t["cost_ns"], t.get("flops", 0), t["flags"], len(t["parents"]),
                           C.cast(par, C.POINTER(C.c_uint32)))
    sd = (StepDesc * len(steps))()
    for i, s in enumerate(steps):
        rd = (C.c_uint32 * len(s["reads"]))(*s["reads"])
        keep.append(rd)
        sd[i] = StepDesc(s["produces"], len(s["reads"]), C.cast(rd, C.POINTER(C.c_uint32)), s["cost_ns"])
    pp = _plan_params(params)
    return td, sd, pp, keep


class Delta:
    """One delta_ctx.  `arena` is a torch uint8 CUDA tensor (kept alive here) or None for a
    planner-only context; `stream` is a hipStream_t handle as an int (0 = default stream)."""

    def __init__(self, arena=None, stream=0):
        self.lib = load_library()
        self.arena = arena
        self.ctx = C.c_void_p()
        ptr, nbytes = (arena.data_ptr(), arena.numel() * arena.element_size()) if arena is not None else (None, 0)
        rc = self.lib.delta_create(ptr, nbytes, stream or None, C.byref(self.ctx))
        if rc != OK:
            raise DeltaError(rc, "delta_create failed")

    def close(self):
        if self.ctx:
            self.lib.delta_destroy(self.ctx)
            self.ctx = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, rc):
        if rc != OK:
            raise DeltaError(rc, self.last_error())

    def last_error(self):
        return (self.lib.delta_last_error(self.ctx) or b"").decode()

    # -- planning
    def prepare_graph(self, tensors, steps):
        """Marshals a graph once; pass the result to plan() in place of (tensors, steps)."""
        td, sd, _, keep = _marshal_graph(tensors, steps, dict.fromkeys([k for k, _ in PlanParams._fields_], 0))
        return ("prepared", td, sd, keep, len(tensors), len(steps))

    def plan(self, tensors, steps, params):
        """Returns (events, peak): events as (step, action, tensor) tuples.  `tensors` may be
        the result of prepare_graph() (then `steps` is ignored)."""
        if isinstance(tensors, tuple) and tensors and tensors[0] == "prepared":
            _, td, sd, keep, nt, ns = tensors
            pp = _plan_params(params)
            tensors, steps = range(nt), range(ns)
        else:
            td, sd, pp, keep = _marshal_graph(tensors, steps, params)
        cap = 64 + 8 * (len(tensors) + len(steps))
        while True:
            ev = (Event * cap)()
            n, peak = C.c_uint32(), C.c_uint64()
            rc = self.lib.delta_plan(self.ctx, td, len(tensors), sd, len(steps), C.byref(pp), ev, cap,
                                     C.byref(n), C.byref(peak))
            if rc == ERR_BUFFER:
                cap = n.value
                continue
            self._check(rc)
            return [(ev[i].step, ev[i].action, ev[i].tensor) for i in range(n.value)], peak.value

    # -- run time
    def bind(self, sizes):
        arr = (C.c_uint64 * len(sizes))(*[int(s) for s in sizes])
        self._check(self.lib.delta_bind(self.ctx, arr, len(sizes)))

    def reserve_pinned(self, nbytes):
        self._check(self.lib.delta_reserve_pinned(self.ctx, int(nbytes)))

    def alloc(self, tensor):
        p = C.c_void_p()
        self._check(self.lib.delta_alloc(self.ctx, tensor, C.byref(p)))
        return p.value

    def tensor_ptr(self, tensor):
        p = C.c_void_p()
        self._check(self.lib.delta_tensor_ptr(self.ctx, tensor, C.byref(p)))
        return p.value

    def release(self, tensor, action):
        self._check(self.lib.delta_release(self.ctx, tensor, action))

    def swap_out(self, tensor):
        self._check(self.lib.delta_swap_out(self.ctx, tensor))

    def prefetch(self, tensor):
        self._check(self.lib.delta_prefetch(self.ctx, tensor))

    def recompute_segment(self, layers, n=None):
        """`layers`: a ctypes array from layer_array() (or a list, packed on the fly)."""
        if isinstance(layers, (list, tuple)):
            layers = layer_array(layers)
        self._check(self.lib.delta_recompute_segment(self.ctx, layers, len(layers) if n is None else n))

    def bwd_weights(self, layer, wt_ptr):
        """Writes the data-gradient weights of `layer` (a LayerDesc) to device memory at wt_ptr."""
        self._check(self.lib.delta_bwd_weights(self.ctx, layer_array([layer]), wt_ptr))

    def backward_workspace(self, layer):
        v = C.c_uint64()
        self._check(self.lib.delta_backward_workspace(self.ctx, layer_array([layer]), C.byref(v)))
        return v.value

    def backward_segment(self, descs):
        """`descs`: a list of BwdDesc."""
        arr = (BwdDesc * len(descs))(*descs)
        self._check(self.lib.delta_backward_segment(self.ctx, arr, len(descs)))

    def backward_join(self):
        self._check(self.lib.delta_backward_join(self.ctx))

    def batchnorm_static(self, x_ptr, y_ptr, gamma_ptr, beta_ptr, rows, channels, eps):
        """Batch normalisation with batch statistics on caller-owned device buffers; allocates nothing."""
        self._check(self.lib.delta_batchnorm_static(self.ctx, x_ptr, y_ptr, gamma_ptr, beta_ptr, rows, channels, eps))

    def sync(self, which=SYNC_ALL):
        self._check(self.lib.delta_sync(self.ctx, which))

    def bn_fold(self, gamma, beta, mean, var, eps, C_, scale, shift):
        self._check(self.lib.delta_bn_fold(self.ctx, gamma, beta, mean, var, eps, C_, scale, shift))

    def stats(self):
        s = Stats()
        self._check(self.lib.delta_stats(self.ctx, C.byref(s)))
        return s.as_dict()

    def stats_reset(self):
        self._check(self.lib.delta_stats_reset(self.ctx))

    def set_skip_copies(self, skip):
        self._check(self.lib.delta_set_skip_copies(self.ctx, 1 if skip else 0))

    def probe_hostlink(self, nbytes, iters, direction):
        v = C.c_double()
        self._check(self.lib.delta_probe_hostlink(self.ctx, nbytes, iters, direction, C.byref(v)))
        return v.value

    def probe_hbm(self, nbytes, iters):
        v = C.c_double()
        self._check(self.lib.delta_probe_hbm(self.ctx, nbytes, iters, C.byref(v)))
        return v.value

    def layer_kernel(self, desc):
        """Name of the kernel variant a layer descriptor dispatches to."""
        arr = layer_array([desc])
        buf = C.create_string_buffer(128)
        self._check(self.lib.delta_layer_kernel(self.ctx, arr, buf, 128))
        return buf.value.decode()

    def probe_mfma(self, iters):
        v = C.c_double()
        self._check(self.lib.delta_probe_mfma(self.ctx, iters, C.byref(v)))
        return v.value


def plan(tensors, steps, params):
    """delta_plan on a throw-away planner-only context."""
    d = Delta()
    try:
        return d.plan(tensors, steps, params)
    finally:
        d.close()
