"""GPU parity of the backward kernels (through the C ABI) against the CPU oracle.

The ReLU mask is decided from the *stored* forward output, so the oracle is given the GPU's own y
(both sides then take that decision on the same bits) and gpre must match bit for bit.  dL/dx is
stored in bf16 from fp32 sums of bf16 products, with weights that carry one extra bf16 rounding
(w * scale): 2e-2 of the tensor's maximum, as for the forward.  dL/dw is fp32 sums of exact
products: 2e-4 of its maximum."""
import numpy as np
import pytest

import synth
from oracle import numeric as on

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def torch_mod():
    import torch
    assert torch.cuda.is_available()
    return torch


def _dev(torch, a):
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")


CASES = [
    # name        N   H   W  Cin Cout R relu res  add  stride
    ("1x1_64_256", 2, 12, 12,  64, 256, 1, True, True, False, 1),
    ("1x1_256_64", 3,  9, 11, 256,  64, 1, True, False, True, 1),
    ("1x1_norelu", 2,  7,  7,  64,  64, 1, False, False, False, 1),
    ("3x3_64",     2, 14, 14,  64,  64, 3, True, False, False, 1),
    ("3x3_128",    1,  9, 11, 128, 128, 3, True, False, True, 1),     # non-square, accumulate into gx
    ("3x3_wide",   1,  3, 56,  64,  64, 3, True, False, False, 1),    # config 2's row length
    ("1x1_128_128", 2, 10, 10, 128, 128, 1, True, False, False, 1),
    ("3x3_s2",     2, 14, 14,  64, 128, 3, True, False, False, 2),    # strided: gpre at the input's resolution
    ("3x3_s2_odd", 1,  9, 13, 128,  64, 3, True, False, True, 2),     # odd image sizes
    ("1x1_s2",     2, 12, 12, 128, 256, 1, False, False, False, 2),   # the projection shortcut: at the output's resolution
    ("1x1_s2_odd", 2,  9, 13, 128,  64, 1, True, False, True, 2),     # with ReLU, gx_add, odd image sizes
    ("1x1_s2_fx",  1, 10, 10,  64, 128, 1, False, False, True, 2, "x"),
    # fused masks ("x": this layer masks gx with [x > 0]; "y": gy arrives already masked)
    ("1x1_64_256_fx",  2, 12, 12,  64, 256, 1, True, True, False, 1, "x"),    # data gradient: streaming kernel
    ("1x1_256_64_fxy", 3,  9, 11, 256,  64, 1, True, False, True, 1, "xy"),   # streaming kernel, sliced, with gx_add
    ("1x1_128_256_fx", 2, 10, 10, 128, 256, 1, True, False, True, 1, "x"),    # tiled kernel
    ("3x3_64_fxy",     2, 14, 14,  64,  64, 3, True, False, False, 1, "xy"),  # halo kernel
    ("3x3_s2_fy",      2, 14, 14,  64, 128, 3, True, False, False, 2, "y"),   # strided: masked gy is only spread out;
                                                                               # data gradient by parity class
    ("3x3_s2_odd_fxy", 2,  9, 13, 128,  64, 3, True, False, True, 2, "xy"),   # the same on odd sizes, + gx_add, + mask_gx
    ("3x3_s2_norelu",  1, 12, 10,  64,  64, 3, False, False, True, 2, "x"),   # no mask of its own either
    ("3x3_s2_1row",    3,  1,  8,  64,  64, 3, True, False, False, 2, "y"),   # a single input row: no odd rows
    # channel counts the class-wise weight gradient takes ("g": gpre = gy, nothing is spread out)
    ("3x3_s2_cls",     2, 14, 14, 128, 128, 3, True, False, False, 2, "y"),   # both gradients by class, gpre still written
    ("3x3_s2_cls_g",   2, 14, 14, 128, 128, 3, True, False, True, 2, "xyg"),
    ("3x3_s2_cls_odd", 1,  9, 13, 128, 256, 3, False, False, True, 2, "xg"),  # odd sizes: classes of unequal size
    ("3x3_s2_cls_1col", 3, 6,  1, 256, 128, 3, True, False, False, 2, "yg"),  # a single input column: no odd columns
]


@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
def test_layer_backward_matches_oracle(torch_mod, case):
    torch = torch_mod
    import paper_2203_15980_amd as dl
    name, N, H, W, Cin, Cout, R, relu, has_res, has_add, stride = case[:11]
    fuse = case[11] if len(case) > 11 else ""
    mask_gx, gy_masked = "x" in fuse, "y" in fuse
    print("case", name, flush=True)
    pad = (R - 1) // 2
    l = synth.LayerSpec(name, "conv", "x0", "r0" if has_res else None, name, N, H, W, Cin, Cout, R, R, stride, pad, relu)
    P, Q = l.P, l.Q
    l.index = 1
    master = 91
    x = synth.make_input(master, (N, H, W, Cin), "bf16")
    p = synth.make_params(master, l, "bf16")
    yshape = (N, P, Q, Cout)
    direct = R == 1 and stride > 1                        # handled at the output's resolution
    gpshape = yshape if direct else (N, H, W, Cout)
    bits = lambda aid, shape: synth.f32_to_bf16_bits(
        synth.normal(master, aid, int(np.prod(shape))).astype(np.float32)).reshape(shape)
    res = bits(901, yshape) if has_res else None
    gy = bits(902, yshape)
    add = bits(903, x.shape) if has_add else None

    arena = torch.empty(96 << 20, dtype=torch.uint8, device="cuda:0")
    d = dl.Delta(arena, torch.cuda.current_stream().cuda_stream)
    ysz, xsz, gpsz = int(np.prod(yshape)) * 2, x.nbytes, int(np.prod(gpshape)) * 2
    # tensors: 0 x, 1 res, 2 y, 3 gy, 4 gpre, 5 gx, 6 gx_add
    d.bind([xsz, ysz, ysz, ysz, gpsz, xsz, xsz])
    base = d.arena.data_ptr()

    def put(tid, a):
        ptr = d.alloc(tid)
        d.arena[ptr - base:ptr - base + a.nbytes].copy_(_dev(torch, a.view(np.uint8).reshape(-1)))

    def get(tid, shape, dtype=np.uint16):
        ptr = d.tensor_ptr(tid)
        n = int(np.prod(shape)) * np.dtype(dtype).itemsize
        return d.arena[ptr - base:ptr - base + n].cpu().numpy().view(dtype).reshape(shape)

    put(0, x)
    if has_res:
        put(1, res)
    put(3, gy)
    if has_add:
        put(6, add)
    w = _dev(torch, p["w"])
    bn = [_dev(torch, p[k]) for k in ("gamma", "beta", "mean", "var")]
    scale = torch.empty(Cout, dtype=torch.float32, device="cuda:0")
    shift = torch.empty(Cout, dtype=torch.float32, device="cuda:0")
    d.bn_fold(bn[0].data_ptr(), bn[1].data_ptr(), bn[2].data_ptr(), bn[3].data_ptr(), float(p["eps"]),
              Cout, scale.data_ptr(), shift.data_ptr())
    fwd = dl.LayerDesc(x=0, res=1 if has_res else dl.NO_TENSOR, y=2, dtype=dl.DTYPE_BF16, w=w.data_ptr(),
                       scale=scale.data_ptr(), shift=shift.data_ptr(), N=N, H=H, W=W, Cin=Cin, Cout=Cout,
                       R=R, S=R, stride=stride, pad=pad, relu=1 if relu else 0)
    d.recompute_segment([fwd])                           # the forward, so that y is the GPU's own
    if gy_masked:                                        # what a consumer running with mask_gx would have left
        d.sync()
        gy = np.where(on.to_f64(get(2, yshape), "bf16") > 0, gy, np.uint16(0)).astype(np.uint16)
        put_again = d.tensor_ptr(3)
        d.arena[put_again - base:put_again - base + gy.nbytes].copy_(_dev(torch, gy.view(np.uint8).reshape(-1)))
    wt = torch.empty(Cout * R * R * Cin, dtype=torch.uint16, device="cuda:0")
    d.bwd_weights(fwd, wt.data_ptr())
    ws_bytes = d.backward_workspace(fwd)
    assert ws_bytes > 0
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda:0")
    gw = torch.full((Cout, R, R, Cin), float("nan"), dtype=torch.float32, device="cuda:0")
    own_gpre = ((relu and not gy_masked) or (stride > 1 and not direct)) and "g" not in fuse
    desc = dl.BwdDesc(fwd=fwd, gy=3, gpre=4 if own_gpre else 3, gx=5, gx_add=6 if has_add else dl.NO_TENSOR,
                      mask_gx=int(mask_gx), gy_masked=int(gy_masked),
                      wt=wt.data_ptr(), gw=gw.data_ptr(), workspace=ws.data_ptr(), workspace_bytes=ws_bytes)
    d.backward_segment([desc])
    d.sync()

    y_gpu = get(2, yshape)
    ref_gx, ref_gw, ref_gpre = on.conv_bn_act_bwd(x, p["w"], p, y_gpu, gy, stride=stride, pad=pad, relu=relu,
                                                  dtype="bf16")
    if has_add:
        ref_gx = ref_gx + on.to_f64(add, "bf16")
    if mask_gx:                                          # the producer's ReLU mask: x is its output
        keep = on.to_f64(x, "bf16") > 0
        assert keep.any() and not keep.all()
        ref_gx = np.where(keep, ref_gx, 0.0)
    # gpre: pure masking, bit for bit
    if "g" in fuse:                                      # not spread out: gy itself, untouched
        assert np.array_equal(get(3, yshape), gy)
    else:
        gpre_gpu = on.to_f64(get(4 if own_gpre else 3, gpshape), "bf16")
        want_gpre = np.zeros(gpshape)
        if direct:
            want_gpre = ref_gpre
        else:
            want_gpre[:, 0:stride * P:stride, 0:stride * Q:stride, :] = ref_gpre     # at the input's resolution
        assert np.array_equal(gpre_gpu, want_gpre)
    if relu:
        assert (ref_gpre == 0).any() and (ref_gpre != 0).any()
    # the transformed weights: w[k][r][s][c] * scale[k], flipped and transposed, one bf16 rounding
    s64 = p["gamma"].astype(np.float64) / np.sqrt(p["var"].astype(np.float64) + p["eps"])
    want_wt = (on.to_f64(p["w"], "bf16") * s64[:, None, None, None])[:, ::-1, ::-1, :].transpose(3, 1, 2, 0)
    got_wt = on.to_f64(wt.cpu().numpy().reshape(Cin, R, R, Cout), "bf16")
    assert np.max(np.abs(got_wt - want_wt)) <= 2.0 ** -8 * np.max(np.abs(want_wt))
    gx_gpu = on.to_f64(get(5, x.shape), "bf16")
    err_x = float(np.max(np.abs(gx_gpu - ref_gx)) / np.max(np.abs(ref_gx)))
    gw_gpu = gw.cpu().numpy().astype(np.float64)
    assert np.isfinite(gw_gpu).all()
    err_w = float(np.max(np.abs(gw_gpu - ref_gw)) / np.max(np.abs(ref_gw)))
    if mask_gx:
        assert np.array_equal(gx_gpu[~keep], np.zeros(int((~keep).sum())))
    print("  gx err %.2e  gw err %.2e" % (err_x, err_w), flush=True)
    assert err_x <= 2e-2, (name, err_x)
    assert err_w <= 2e-4, (name, err_w)
    d.close()


@pytest.mark.parametrize("N,H,W,relu", [(2, 32, 32, True), (1, 37, 45, True), (3, 64, 48, False)])
def test_stem_weight_gradient_matches_oracle(torch_mod, N, H, W, relu):
    """7x7 stride-2 stem: gpre bit-exact, dL/dw against the oracle (fp32 sums of exact bf16 products).
    Odd image sizes give partial tiles and padding on every side."""
    torch = torch_mod
    import paper_2203_15980_amd as dl
    print("stem", N, H, W, relu, flush=True)
    l = synth.LayerSpec("stem", "conv", "x0", None, "stem", N, H, W, 3, 64, 7, 7, 2, 3, relu)
    l.index = 1
    P, Q = l.P, l.Q
    master = 97
    x = synth.make_input(master, (N, H, W, 3), "bf16")
    p = synth.make_params(master, l, "bf16")
    gy = synth.f32_to_bf16_bits(synth.normal(master, 902, N * P * Q * 64).astype(np.float32)).reshape(N, P, Q, 64)
    ysz = gy.nbytes
    arena = torch.empty(32 << 20, dtype=torch.uint8, device="cuda:0")
    d = dl.Delta(arena, torch.cuda.current_stream().cuda_stream)
    d.bind([x.nbytes, ysz, ysz, ysz])               # 0 x, 1 y, 2 gy, 3 gpre
    base = d.arena.data_ptr()

    def put(tid, a):
        ptr = d.alloc(tid)
        d.arena[ptr - base:ptr - base + a.nbytes].copy_(_dev(torch, a.view(np.uint8).reshape(-1)))

    def get(tid, shape):
        ptr = d.tensor_ptr(tid)
        n = int(np.prod(shape)) * 2
        return d.arena[ptr - base:ptr - base + n].cpu().numpy().view(np.uint16).reshape(shape)

    put(0, x)
    put(2, gy)
    w = _dev(torch, p["w"])
    bn = [_dev(torch, p[k]) for k in ("gamma", "beta", "mean", "var")]
    scale = torch.empty(64, dtype=torch.float32, device="cuda:0")
    shift = torch.empty(64, dtype=torch.float32, device="cuda:0")
    d.bn_fold(bn[0].data_ptr(), bn[1].data_ptr(), bn[2].data_ptr(), bn[3].data_ptr(), float(p["eps"]), 64,
              scale.data_ptr(), shift.data_ptr())
    fwd = dl.LayerDesc(x=0, res=dl.NO_TENSOR, y=1, dtype=dl.DTYPE_BF16, w=w.data_ptr(), scale=scale.data_ptr(),
                       shift=shift.data_ptr(), N=N, H=H, W=W, Cin=3, Cout=64, R=7, S=7, stride=2, pad=3, relu=1 if relu else 0)
    d.recompute_segment([fwd])
    ws_bytes = d.backward_workspace(fwd)
    assert ws_bytes > 0
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda:0")
    gw = torch.full((64, 7, 7, 3), float("nan"), dtype=torch.float32, device="cuda:0")
    desc = dl.BwdDesc(fwd=fwd, gy=2, gpre=3 if relu else 2, gx=dl.NO_TENSOR, gx_add=dl.NO_TENSOR, wt=None,
                      gw=gw.data_ptr(), workspace=ws.data_ptr(), workspace_bytes=ws_bytes)
    d.backward_segment([desc])
    d.sync()
    y_gpu = get(1, (N, P, Q, 64))
    _, ref_gw, ref_gpre = on.conv_bn_act_bwd(x, p["w"], p, y_gpu, gy, stride=2, pad=3, relu=relu, dtype="bf16")
    assert np.array_equal(on.to_f64(get(3 if relu else 2, (N, P, Q, 64)), "bf16"), ref_gpre)
    got = gw.cpu().numpy().astype(np.float64)
    assert np.isfinite(got).all()
    err = float(np.max(np.abs(got - ref_gw)) / np.max(np.abs(ref_gw)))
    print("  gw err %.2e" % err, flush=True)
    assert err <= 2e-4, err
    with pytest.raises(dl.DeltaError):                      # the stem has no data gradient
        d.backward_segment([dl.BwdDesc(fwd=fwd, gy=2, gpre=3 if relu else 2, gx=0, gx_add=dl.NO_TENSOR, wt=None,
                                       gw=gw.data_ptr(), workspace=ws.data_ptr(), workspace_bytes=ws_bytes)])
    d.close()


def test_backward_rejects_what_it_does_not_support(torch_mod):
    torch = torch_mod
    import paper_2203_15980_amd as dl
    arena = torch.empty(8 << 20, dtype=torch.uint8, device="cuda:0")
    d = dl.Delta(arena, torch.cuda.current_stream().cuda_stream)
    N, H, W, C = 1, 8, 8, 64
    xs, ys = N * H * W * C * 2, N * 4 * 4 * C * 2
    d.bind([xs, ys, ys, ys, xs])
    for t in (0, 2):
        d.alloc(t)
    dummy = torch.zeros(C * 9 * C + 64, dtype=torch.uint16, device="cuda:0")
    f32 = torch.zeros(C, dtype=torch.float32, device="cuda:0")
    s2 = dl.LayerDesc(x=0, res=dl.NO_TENSOR, y=1, dtype=dl.DTYPE_BF16, w=dummy.data_ptr(), scale=f32.data_ptr(),
                      shift=f32.data_ptr(), N=N, H=H, W=W, Cin=C, Cout=C, R=3, S=3, stride=2, pad=1, relu=1)
    with pytest.raises(dl.DeltaError) as e:              # a strided layer with a mask to apply needs its own gpre tensor
        d.backward_segment([dl.BwdDesc(fwd=s2, gy=2, gpre=2, gx=4, gx_add=dl.NO_TENSOR, wt=dummy.data_ptr(),
                                       gw=None, workspace=None, workspace_bytes=0)])
    assert e.value.status == dl.ERR_INVALID
    d.close()
    d = dl.Delta(arena, torch.cuda.current_stream().cuda_stream)
    ys = N * 6 * 6 * C * 2
    d.bind([xs, ys, ys, ys, xs])
    for t in (0, 2):
        d.alloc(t)
    p0 = dl.LayerDesc(x=0, res=dl.NO_TENSOR, y=1, dtype=dl.DTYPE_BF16, w=dummy.data_ptr(), scale=f32.data_ptr(),
                      shift=f32.data_ptr(), N=N, H=H, W=W, Cin=C, Cout=C, R=3, S=3, stride=1, pad=0, relu=0)
    with pytest.raises(dl.DeltaError) as e:              # 3x3 without padding: 2*pad != R-1
        d.backward_segment([dl.BwdDesc(fwd=p0, gy=2, gpre=2, gx=4, gx_add=dl.NO_TENSOR, wt=dummy.data_ptr(),
                                       gw=None, workspace=None, workspace_bytes=0)])
    assert e.value.status == dl.ERR_INVALID
    d.close()


@pytest.mark.parametrize("fuse", [False, True], ids=["separate_masks", "fused_masks"])
def test_bottleneck_stack_backward_layer_by_layer_and_end_to_end(torch_mod, fuse):
    """Three bottleneck blocks (config 2's layer shapes at 2 x 16 x 16): the whole backward pass
    through the harness.  Layer by layer, the oracle is given exactly what the GPU's layer was
    given (its stored x, y and incoming gradient) and must reproduce what the layer wrote; end
    to end, the oracle runs its own chain and dL/dx0 must agree within the bf16 tolerance."""
    torch = torch_mod
    import paper_2203_15980_amd as dl
    from paper_2203_15980_amd.harness import Net
    layers = synth.bottleneck_stack(2, 16, 16)
    g = synth.fused_graph(layers, "bf16")
    arena = torch.empty(64 << 20, dtype=torch.uint8, device="cuda:0")
    d = dl.Delta(arena, torch.cuda.current_stream().cuda_stream)
    d.bind([t["bytes"] for t in g.tensors])
    net = Net(d, layers, "bf16", synth.master_seed(2))
    net.enable_backward(input_gradient=True, fuse_masks=fuse)
    assert bool(net.masked_by) == fuse
    net.forward()
    net.backward(keep=True)
    d.sync()
    acts = {"x0": net.x0_np}
    for l in layers:
        acts[l.y] = net.read(l.y)
    by_name = {l.name: l for l in layers}
    for (lname, gy_name, gpre_name, gx_name, add_name, masks_gx) in net.bwd_trace:
        l = by_name[lname]
        p = net.params_np[lname]
        gy = net.read(gy_name)
        # a gy that arrives masked is unchanged by the oracle's own mask (same y, same test)
        ref_gx, ref_gw, ref_gpre = on.conv_bn_act_bwd(acts[l.x], p["w"], p, acts[l.y], gy, stride=l.stride,
                                                      pad=l.pad, relu=l.relu, dtype="bf16")
        assert np.array_equal(on.to_f64(net.read(gpre_name), "bf16"), ref_gpre), lname
        if add_name:
            ref_gx = ref_gx + on.to_f64(net.read(add_name), "bf16")
        if masks_gx:
            ref_gx = np.where(on.to_f64(acts[l.x], "bf16") > 0, ref_gx, 0.0)
        got_gx = on.to_f64(net.read(gx_name), "bf16")
        ex = float(np.max(np.abs(got_gx - ref_gx)) / np.max(np.abs(ref_gx)))
        got_gw = net.gw[lname].cpu().numpy().astype(np.float64).reshape(ref_gw.shape)
        ew = float(np.max(np.abs(got_gw - ref_gw)) / np.max(np.abs(ref_gw)))
        print("  %-8s gx %.2e gw %.2e" % (lname, ex, ew), flush=True)
        assert ex <= 2e-2 and ew <= 2e-4, (lname, ex, ew)
    # end to end: the oracle's own forward (bf16 storage) and backward chain
    ref = on.run_layers(layers, net.params_np, net.x0_np, "bf16")
    grads = {layers[-1].y: on.to_f64(net.top_gradient_np, "bf16")}
    rnd = lambda a: on.to_f64(synth.f32_to_bf16_bits(a.astype(np.float32)), "bf16")   # gradients are stored in bf16
    for l in reversed(layers):
        p = net.params_np[l.name]
        gy_bits = synth.f32_to_bf16_bits(grads.pop(l.y).astype(np.float32)).reshape(ref[l.y].shape)
        x_in = net.x0_np if l.x == "x0" else ref[l.x]
        gx, gw, gpre = on.conv_bn_act_bwd(x_in, p["w"], p, ref[l.y], gy_bits, stride=l.stride, pad=l.pad,
                                          relu=l.relu, dtype="bf16")
        if l.res:
            grads[l.res] = grads.get(l.res, 0) + gpre
        grads[l.x] = rnd(grads.get(l.x, 0) + gx)
    assert any(t[5] for t in net.bwd_trace) == fuse
    last = net.bwd_trace[-1]
    got = on.to_f64(net.read(last[3]), "bf16")
    err = float(np.max(np.abs(got - grads["x0"])) / np.max(np.abs(grads["x0"])))
    print("  end to end dL/dx0 err %.2e" % err, flush=True)
    # Not the per-tensor parity bar (that is the 2e-2 asserted layer by layer above, each layer on
    # the GPU's own inputs): here the oracle walks its OWN chain, ten stored activations and ten
    # stored gradients deep, each rounded to bf16 independently of the GPU's (up to 2^-9 of the
    # tensor's maximum per rounding: 20 x 2^-9 = 3.9e-2), and ReLU masks taken on those
    # independently rounded activations may differ at activations next to zero.  5e-2 bounds that drift.
    assert err <= 5e-2, err
    d.close()


def _small_ctx(torch, sizes, mb=32):
    import paper_2203_15980_amd as dl
    arena = torch.empty(mb << 20, dtype=torch.uint8, device="cuda:0")
    d = dl.Delta(arena, torch.cuda.current_stream().cuda_stream)
    d.bind(sizes)
    base = d.arena.data_ptr()

    def put(tid, a):
        ptr = d.alloc(tid)
        d.arena[ptr - base:ptr - base + a.nbytes].copy_(_dev(torch, np.ascontiguousarray(a).view(np.uint8).reshape(-1)))

    def get(tid, shape, dtype=np.uint16):
        ptr = d.tensor_ptr(tid)
        n = int(np.prod(shape)) * np.dtype(dtype).itemsize
        return d.arena[ptr - base:ptr - base + n].cpu().numpy().view(dtype).reshape(shape)
    return d, put, get


def _bits(master, aid, shape, scale=1.0):
    return synth.f32_to_bf16_bits((synth.normal(master, aid, int(np.prod(shape))) * scale).astype(np.float32)).reshape(shape)


F32_CASES = [
    # name          N   H   W  Cin Cout R relu res  add  stride
    ("f32_1x1_res",  2, 12, 12,  64, 256, 1, True, True, False, 1),
    ("f32_1x1_tail", 3,  9, 11,  96,  32, 1, False, False, True, 1),    # 297 positions: a ragged last chunk of 64
    ("f32_3x3",      2, 14, 14,  64,  64, 3, True, False, False, 1),
    ("f32_3x3_odd",  1,  9, 11,  32,  96, 3, True, False, True, 1),
    ("f32_3x3_s2",   2, 13, 14,  64,  32, 3, True, False, False, 2),    # strided: gpre at the input's resolution
    ("f32_1x1_s2",   2, 12, 13,  64, 128, 1, False, False, True, 2),    # the projection shortcut
]


@pytest.mark.parametrize("case", F32_CASES, ids=[c[0] for c in F32_CASES])
def test_layer_backward_fp32_matches_oracle(torch_mod, case):
    """The fp32 storage type (config 1's): data gradient through the same kernels as bf16, weight
    gradient through the plain fp32 kernel; both within 1e-4 of the float64 oracle."""
    torch = torch_mod
    import paper_2203_15980_amd as dl
    name, N, H, W, Cin, Cout, R, relu, has_res, has_add, stride = case
    print("case", name, flush=True)
    pad = (R - 1) // 2
    l = synth.LayerSpec(name, "conv", "x0", "r0" if has_res else None, name, N, H, W, Cin, Cout, R, R, stride, pad, relu)
    P, Q = l.P, l.Q
    l.index = 1
    master = 92
    x = synth.make_input(master, (N, H, W, Cin), "f32")
    p = synth.make_params(master, l, "f32")
    yshape = (N, P, Q, Cout)
    direct = R == 1 and stride > 1
    gpshape = yshape if direct else (N, H, W, Cout)
    rnd = lambda aid, shape: synth.normal(master, aid, int(np.prod(shape))).astype(np.float32).reshape(shape)
    res = rnd(901, yshape) if has_res else None
    gy = rnd(902, yshape)
    add = rnd(903, x.shape) if has_add else None
    ysz, xsz, gpsz = int(np.prod(yshape)) * 4, x.nbytes, int(np.prod(gpshape)) * 4
    d, put, get = _small_ctx(torch, [xsz, ysz, ysz, ysz, gpsz, xsz, xsz])
    put(0, x)
    if has_res:
        put(1, res)
    put(3, gy)
    if has_add:
        put(6, add)
    w = _dev(torch, p["w"])
    bn = [_dev(torch, p[k]) for k in ("gamma", "beta", "mean", "var")]
    scale = torch.empty(Cout, dtype=torch.float32, device="cuda:0")
    shift = torch.empty(Cout, dtype=torch.float32, device="cuda:0")
    d.bn_fold(bn[0].data_ptr(), bn[1].data_ptr(), bn[2].data_ptr(), bn[3].data_ptr(), float(p["eps"]),
              Cout, scale.data_ptr(), shift.data_ptr())
    fwd = dl.LayerDesc(x=0, res=1 if has_res else dl.NO_TENSOR, y=2, dtype=dl.DTYPE_F32, w=w.data_ptr(),
                       scale=scale.data_ptr(), shift=shift.data_ptr(), N=N, H=H, W=W, Cin=Cin, Cout=Cout,
                       R=R, S=R, stride=stride, pad=pad, relu=1 if relu else 0)
    d.recompute_segment([fwd])
    wt = torch.empty(Cout * R * R * Cin, dtype=torch.float32, device="cuda:0")
    d.bwd_weights(fwd, wt.data_ptr())
    ws_bytes = max(d.backward_workspace(fwd), 256)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda:0")
    gw = torch.full((Cout, R, R, Cin), float("nan"), dtype=torch.float32, device="cuda:0")
    own_gpre = relu or (stride > 1 and not direct)
    desc = dl.BwdDesc(fwd=fwd, gy=3, gpre=4 if own_gpre else 3, gx=5, gx_add=6 if has_add else dl.NO_TENSOR,
                      mask_gx=0, gy_masked=0, wt=wt.data_ptr(), gw=gw.data_ptr(), workspace=ws.data_ptr(),
                      workspace_bytes=ws_bytes)
    d.backward_segment([desc])
    d.sync()
    y_gpu = get(2, yshape, np.float32)
    ref_gx, ref_gw, ref_gpre = on.conv_bn_act_bwd(x, p["w"], p, y_gpu, gy, stride=stride, pad=pad, relu=relu, dtype="f32")
    if has_add:
        ref_gx = ref_gx + add.astype(np.float64)
    gpre_gpu = get(4 if own_gpre else 3, gpshape, np.float32).astype(np.float64)
    want_gpre = np.zeros(gpshape)
    if direct:
        want_gpre = ref_gpre
    else:
        want_gpre[:, 0:stride * P:stride, 0:stride * Q:stride, :] = ref_gpre
    assert np.array_equal(gpre_gpu, want_gpre)               # pure masking: bit for bit
    if relu:
        assert (ref_gpre == 0).any() and (ref_gpre != 0).any()
    gx_gpu = get(5, x.shape, np.float32).astype(np.float64)
    err_x = float(np.max(np.abs(gx_gpu - ref_gx)) / np.max(np.abs(ref_gx)))
    gw_gpu = gw.cpu().numpy().astype(np.float64)
    assert np.isfinite(gw_gpu).all()
    err_w = float(np.max(np.abs(gw_gpu - ref_gw)) / np.max(np.abs(ref_gw)))
    print("  gx err %.2e  gw err %.2e" % (err_x, err_w), flush=True)
    assert err_x <= 1e-4 and err_w <= 1e-4, (name, err_x, err_w)
    d.close()


def test_config1_backward_fp32_layer_by_layer(torch_mod):
    """Config 1 (three bottleneck blocks, fp32, 2 x 32 x 32 x 64): the whole backward pass through
    the harness; every layer's gradients against the oracle given the same stored tensors."""
    torch = torch_mod
    import paper_2203_15980_amd as dl
    from paper_2203_15980_amd.harness import Net
    layers = synth.bottleneck_stack(2, 32, 32)
    g = synth.fused_graph(layers, "f32")
    arena = torch.empty(128 << 20, dtype=torch.uint8, device="cuda:0")
    d = dl.Delta(arena, torch.cuda.current_stream().cuda_stream)
    d.bind([t["bytes"] for t in g.tensors])
    net = Net(d, layers, "f32", synth.master_seed(1))
    net.enable_backward(input_gradient=True, fuse_masks=False)
    net.forward()
    net.backward(keep=True)
    d.sync()
    acts = {"x0": net.x0_np}
    for l in layers:
        acts[l.y] = net.read(l.y)
    by_name = {l.name: l for l in layers}
    assert len(net.bwd_trace) == len(layers)
    for (lname, gy_name, gpre_name, gx_name, add_name, masks_gx) in net.bwd_trace:
        l = by_name[lname]
        p = net.params_np[lname]
        ref_gx, ref_gw, ref_gpre = on.conv_bn_act_bwd(acts[l.x], p["w"], p, acts[l.y], net.read(gy_name), stride=l.stride,
                                                      pad=l.pad, relu=l.relu, dtype="f32")
        assert not masks_gx
        assert np.array_equal(net.read(gpre_name).astype(np.float64), ref_gpre), lname
        if add_name:
            ref_gx = ref_gx + net.read(add_name).astype(np.float64)
        ex = float(np.max(np.abs(net.read(gx_name).astype(np.float64) - ref_gx)) / np.max(np.abs(ref_gx)))
        got_gw = net.gw[lname].cpu().numpy().astype(np.float64).reshape(ref_gw.shape)
        ew = float(np.max(np.abs(got_gw - ref_gw)) / np.max(np.abs(ref_gw)))
        print("  %-8s gx %.2e gw %.2e" % (lname, ex, ew), flush=True)
        assert ex <= 1e-4 and ew <= 1e-4, (lname, ex, ew)
    d.close()


def test_pooling_backward_matches_oracle(torch_mod):
    torch = torch_mod
    import paper_2203_15980_amd as dl
    # max pooling 3x3 / 2 / 1 on a ReLU-like input (many exact ties at 0): the routing must be the
    # oracle's (same zero pattern), the sums agree to bf16 rounding
    N, H, W, C = 2, 12, 10, 64
    x = _bits(5, 1, (N, H, W, C))
    x = np.where(on.to_f64(x, "bf16") > 0, x, 0).astype(np.uint16)           # zeros tie
    P, Q = (H + 2 - 3) // 2 + 1, (W + 2 - 3) // 2 + 1
    gy = _bits(5, 2, (N, P, Q, C))
    xs, ys = x.nbytes, gy.nbytes
    d, put, get = _small_ctx(torch, [xs, ys, ys, xs])
    put(0, x)
    put(2, gy)
    fwd = dl.LayerDesc(x=0, res=dl.NO_TENSOR, y=1, dtype=dl.DTYPE_BF16, w=None, scale=None, shift=None, N=N, H=H, W=W,
                       Cin=C, Cout=C, R=3, S=3, stride=2, pad=1, relu=0, op=dl.OP_MAXPOOL)
    d.backward_segment([dl.BwdDesc(fwd=fwd, gy=2, gpre=2, gx=3, gx_add=dl.NO_TENSOR, wt=None, gw=None,
                                   workspace=None, workspace_bytes=0)])
    d.sync()
    got = on.to_f64(get(3, x.shape), "bf16")
    ref = on.maxpool_bwd(x, gy, 3, 3, 2, 1, "bf16")
    assert np.array_equal(got == 0, ref == 0)
    assert np.max(np.abs(got - ref)) <= 2.0 ** -8 * np.max(np.abs(ref))
    d.close()
    # the same with the producer's ReLU mask applied on the way out (mask_gx), on an input of mixed
    # signs so that maxima at or below zero exist: their gradient is dropped
    x = _bits(5, 3, (N, H, W, C))
    x[0, 0, 0, :8] = [0x8000, 0x0000, 0x7FC0, 0x0001, 0xBF80, 0x3F80, 0x8001, 0x7F80]     # -0, 0, NaN, tiny, -1, 1, -tiny, inf
    d, put, get = _small_ctx(torch, [xs, ys, ys, xs])
    put(0, x)
    put(2, gy)
    d.backward_segment([dl.BwdDesc(fwd=fwd, gy=2, gpre=2, gx=3, gx_add=dl.NO_TENSOR, mask_gx=1, wt=None, gw=None,
                                   workspace=None, workspace_bytes=0)])
    d.sync()
    got = on.to_f64(get(3, x.shape), "bf16")
    ref = np.where(on.to_f64(x, "bf16") > 0, on.maxpool_bwd(x, gy, 3, 3, 2, 1, "bf16"), 0.0)
    assert np.array_equal(got == 0, ref == 0) and (ref != 0).any() and (ref == 0).any()
    assert np.max(np.abs(got - ref)) <= 2.0 ** -8 * np.max(np.abs(ref))
    d.close()
    # global average
    N, H, W, C = 3, 7, 7, 128
    gy = _bits(6, 1, (N, 1, 1, C))
    d, put, get = _small_ctx(torch, [N * H * W * C * 2, gy.nbytes, gy.nbytes, N * H * W * C * 2])
    put(2, gy)
    fwd = dl.LayerDesc(x=0, res=dl.NO_TENSOR, y=1, dtype=dl.DTYPE_BF16, w=None, scale=None, shift=None, N=N, H=H, W=W,
                       Cin=C, Cout=C, R=H, S=W, stride=1, pad=0, relu=0, op=dl.OP_AVGPOOL)
    d.backward_segment([dl.BwdDesc(fwd=fwd, gy=2, gpre=2, gx=3, gx_add=dl.NO_TENSOR, wt=None, gw=None,
                                   workspace=None, workspace_bytes=0)])
    d.sync()
    got = on.to_f64(get(3, (N, H, W, C)), "bf16")
    ref = on.avgpool_bwd(gy, H, W, "bf16")
    assert np.max(np.abs(got - ref)) <= 2.0 ** -8 * np.max(np.abs(ref))
    d.close()


@pytest.mark.parametrize("shape", [(8, 128, 1000), (7, 576, 1000)], ids=["8x128x1000", "ragged_7x576x1000"])
def test_classifier_and_loss_backward_match_oracle(torch_mod, shape):
    """The second shape leaves a tail in the blockings of the two kernels: an odd number of images and
    72 chunks of input channels (the class count is a multiple of 8 in every layer the forward accepts)."""
    torch = torch_mod
    import paper_2203_15980_amd as dl
    N, Cin, Cout = shape
    x = _bits(7, 1, (N, 1, 1, Cin))
    w = _bits(7, 2, (Cout, 1, 1, Cin), 0.05)
    bias = (synth.normal(7, 3, Cout) * 0.1).astype(np.float32)
    labels = synth.make_labels(7, N, Cout)
    zs, xs = N * Cout * 2, x.nbytes
    # tensors: 0 x, 1 logits, 2 labels, 3 loss, 4 glogits, 5 gx
    d, put, get = _small_ctx(torch, [xs, zs, N * 8, 4, zs, xs])
    put(0, x)
    put(2, labels)
    wd, ones, bd = _dev(torch, w), torch.ones(Cout, dtype=torch.float32, device="cuda:0"), _dev(torch, bias)
    fc = dl.LayerDesc(x=0, res=dl.NO_TENSOR, y=1, dtype=dl.DTYPE_BF16, w=wd.data_ptr(), scale=ones.data_ptr(),
                      shift=bd.data_ptr(), N=N, H=1, W=1, Cin=Cin, Cout=Cout, R=1, S=1, stride=1, pad=0, relu=0)
    loss = dl.LayerDesc(x=1, res=2, y=3, dtype=dl.DTYPE_BF16, w=None, scale=None, shift=None, N=N, H=1, W=1,
                        Cin=Cout, Cout=1, R=1, S=1, stride=1, pad=0, relu=0, op=dl.OP_SOFTMAX_CE)
    d.recompute_segment([fc, loss])
    gw = torch.full((Cout * Cin + Cout,), float("nan"), dtype=torch.float32, device="cuda:0")
    d.backward_segment([
        dl.BwdDesc(fwd=loss, gy=dl.NO_TENSOR, gpre=dl.NO_TENSOR, gx=4, gx_add=dl.NO_TENSOR, wt=None, gw=None,
                   workspace=None, workspace_bytes=0),
        dl.BwdDesc(fwd=fc, gy=4, gpre=4, gx=5, gx_add=dl.NO_TENSOR, wt=None, gw=gw.data_ptr(), workspace=None,
                   workspace_bytes=0)])
    d.sync()
    logits = get(1, (N, Cout))
    gz_gpu = get(4, (N, Cout))
    ref_gz = on.softmax_ce_bwd(logits, labels, "bf16")                 # from the GPU's own logits
    assert np.max(np.abs(on.to_f64(gz_gpu, "bf16") - ref_gz)) <= 2.0 ** -8 * np.max(np.abs(ref_gz)) + 1e-7
    ref_gx, ref_gw, ref_gb = on.fc_bwd(x, w, gz_gpu.reshape(N, 1, 1, Cout), "bf16")
    got_gx = on.to_f64(get(5, (N, 1, 1, Cin)), "bf16")
    assert np.max(np.abs(got_gx - ref_gx)) <= 2e-2 * np.max(np.abs(ref_gx))
    g = gw.cpu().numpy().astype(np.float64)
    assert np.max(np.abs(g[:Cout * Cin].reshape(ref_gw.shape) - ref_gw)) <= 2e-4 * np.max(np.abs(ref_gw))
    assert np.max(np.abs(g[Cout * Cin:] - ref_gb)) <= 2e-4 * np.max(np.abs(ref_gb))
    d.close()


@pytest.mark.parametrize("fuse", [False, True], ids=["separate_masks", "fused_masks"])
def test_small_resnet_whole_backward_layer_by_layer(torch_mod, fuse):
    """ResNet with one bottleneck per stage on 2 x 64 x 64 x 3 with the loss: the whole backward
    pass through the harness (loss, classifier, average pool, strided and projection blocks,
    max-pool, the stem's weight gradient).  Every layer is checked against
    the oracle on exactly the tensors the GPU's layer was given."""
    torch = torch_mod
    import paper_2203_15980_amd as dl
    from paper_2203_15980_amd.harness import Net
    layers = synth.resnet_layers(2, (1, 1, 1, 1), image=64, classes=40)
    g = synth.fused_graph(layers, "bf16", with_loss=True)
    arena = torch.empty(96 << 20, dtype=torch.uint8, device="cuda:0")
    d = dl.Delta(arena, torch.cuda.current_stream().cuda_stream)
    d.bind([t["bytes"] for t in g.tensors])
    net = Net(d, layers, "bf16", 41, with_loss=True)
    net.enable_backward(fuse_masks=fuse)
    assert net.backward_peak_bytes() > 0
    net.forward()
    net.backward(keep=True)
    d.sync()
    acts = {"x0": net.x0_np}
    for l in layers:
        acts[l.y] = net.read(l.y)
    # the loss's gradient from the GPU's own logits
    top = layers[-1]
    gz = on.to_f64(net.read("g:" + top.y), "bf16").reshape(top.N, top.Cout)
    ref_gz = on.softmax_ce_bwd(acts[top.y], net.labels_np, "bf16")
    assert np.max(np.abs(gz - ref_gz)) <= 2.0 ** -8 * np.max(np.abs(ref_gz)) + 1e-7
    by_name = {l.name: l for l in layers}
    checked = set()
    for (lname, gy_name, gpre_name, gx_name, add_name, masks_gx) in net.bwd_trace:
        l = by_name[lname]
        if gx_name is None:                                 # the stem: weight gradient only
            p = net.params_np[lname]
            _, ref_gw, ref_gpre = on.conv_bn_act_bwd(acts[l.x], p["w"], p, acts[l.y], net.read(gy_name), stride=l.stride,
                                                     pad=l.pad, relu=l.relu, dtype="bf16")
            assert np.array_equal(on.to_f64(net.read(gpre_name), "bf16"), ref_gpre)
            got_gw = net.gw[lname].cpu().numpy().astype(np.float64).reshape(ref_gw.shape)
            ew = float(np.max(np.abs(got_gw - ref_gw)) / np.max(np.abs(ref_gw)))
            print("  %-10s stem     gw %.2e" % (lname, ew), flush=True)
            assert ew <= 2e-4, (lname, ew)
            checked.add("stem")
            continue
        gy = net.read(gy_name)
        got = on.to_f64(net.read(gx_name), "bf16")
        if l.kind == "conv":
            p = net.params_np[lname]
            ref_gx, ref_gw, ref_gpre = on.conv_bn_act_bwd(acts[l.x], p["w"], p, acts[l.y], gy, stride=l.stride,
                                                          pad=l.pad, relu=l.relu, dtype="bf16")
            if add_name:
                ref_gx = ref_gx + on.to_f64(net.read(add_name), "bf16")
            if masks_gx:
                ref_gx = np.where(on.to_f64(acts[l.x], "bf16") > 0, ref_gx, 0.0)
            got_gpre = on.to_f64(net.read(gpre_name), "bf16")
            if l.R > 1 and gpre_name != gy_name:            # at the input's resolution (unless both gradients run by class)
                got_gpre = got_gpre[:, ::l.stride, ::l.stride, :][:, :l.P, :l.Q, :]
            assert np.array_equal(got_gpre, ref_gpre), lname
            got_gw = net.gw[lname].cpu().numpy().astype(np.float64).reshape(ref_gw.shape)
            ew = float(np.max(np.abs(got_gw - ref_gw)) / np.max(np.abs(ref_gw)))
            assert ew <= 2e-4, (lname, ew)
        elif l.kind == "maxpool":
            ref_gx = on.maxpool_bwd(acts[l.x], gy, l.R, l.S, l.stride, l.pad, "bf16")
            if masks_gx:                                    # also the stem's ReLU mask
                ref_gx = np.where(on.to_f64(acts[l.x], "bf16") > 0, ref_gx, 0.0)
            assert masks_gx == fuse and np.array_equal(got == 0, ref_gx == 0)
        elif l.kind == "avgpool":
            ref_gx = on.avgpool_bwd(gy, l.H, l.W, "bf16")
        else:
            ref_gx, ref_gw, ref_gb = on.fc_bwd(acts[l.x], net.params_np[lname]["w"], gy, "bf16")
            gwb = net.gw[lname].cpu().numpy().astype(np.float64)
            n = l.Cout * l.Cin
            assert np.max(np.abs(gwb[:n].reshape(ref_gw.shape) - ref_gw)) <= 2e-4 * np.max(np.abs(ref_gw))
            assert np.max(np.abs(gwb[n:] - ref_gb)) <= 2e-4 * np.max(np.abs(ref_gb))
        ex = float(np.max(np.abs(got - ref_gx)) / np.max(np.abs(ref_gx)))
        print("  %-10s %-8s gx %.2e" % (lname, l.kind, ex), flush=True)
        assert ex <= 2e-2, (lname, ex)
        checked.add(l.kind)
    assert checked == {"conv", "maxpool", "avgpool", "fc", "stem"}
    assert any(by_name[t[0]].stride == 2 for t in net.bwd_trace)
    d.close()


def test_weight_gradient_survives_release_of_its_inputs(torch_mod):
    """The weight gradient runs beside the compute stream.  Its inputs are released straight after
    the launch and their blocks are handed to new tensors that the compute stream fills at once:
    the arena must hold those writers back until the weight gradient has read.  Weight gradients
    are a fixed function of the inputs, so the result must equal, bit for bit, that of a run
    that waits before releasing anything."""
    torch = torch_mod
    import paper_2203_15980_amd as dl
    N, H, W, Cin, Cout, R = 16, 56, 56, 64, 64, 3         # a long weight gradient: 50k positions, 9 taps
    l = synth.LayerSpec("wg", "conv", "x0", None, "wg", N, H, W, Cin, Cout, R, R, 1, 1, True)
    l.index = 1
    master = 17
    x = synth.make_input(master, (N, H, W, Cin), "bf16")
    p = synth.make_params(master, l, "bf16")
    gy = synth.f32_to_bf16_bits(synth.normal(master, 902, x.size).astype(np.float32)).reshape(x.shape)
    sz = x.nbytes
    arena = torch.empty(6 * sz + (1 << 20), dtype=torch.uint8, device="cuda:0")
    d = dl.Delta(arena, torch.cuda.current_stream().cuda_stream)
    # tensors: 0 x, 1 y, 2 gy, 3 gpre, 4 gx, 5..8 the tensors that take the four freed blocks
    d.bind([sz] * 9)
    base = d.arena.data_ptr()
    view = lambda ptr: d.arena[ptr - base:ptr - base + sz]
    w = _dev(torch, p["w"])
    scale = torch.ones(Cout, dtype=torch.float32, device="cuda:0")
    shift = torch.zeros(Cout, dtype=torch.float32, device="cuda:0")
    fwd = dl.LayerDesc(x=0, res=dl.NO_TENSOR, y=1, dtype=dl.DTYPE_BF16, w=w.data_ptr(), scale=scale.data_ptr(),
                       shift=shift.data_ptr(), N=N, H=H, W=W, Cin=Cin, Cout=Cout, R=R, S=R, stride=1, pad=1, relu=1)
    wt = torch.empty(Cout * R * R * Cin, dtype=torch.uint16, device="cuda:0")
    d.bwd_weights(fwd, wt.data_ptr())
    ws_bytes = d.backward_workspace(fwd)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda:0")
    xd, gyd = _dev(torch, x.view(np.uint8).reshape(-1)), _dev(torch, gy.view(np.uint8).reshape(-1))

    def run(release_at_once):
        for t, a in ((0, xd), (2, gyd)):
            view(d.alloc(t)).copy_(a)
        d.recompute_segment([fwd])
        gw = torch.full((Cout, R, R, Cin), float("nan"), dtype=torch.float32, device="cuda:0")
        desc = dl.BwdDesc(fwd=fwd, gy=2, gpre=3, gx=4, gx_add=dl.NO_TENSOR, mask_gx=0, gy_masked=0, wt=wt.data_ptr(),
                          gw=gw.data_ptr(), workspace=ws.data_ptr(), workspace_bytes=ws_bytes)
        d.backward_segment([desc])
        if not release_at_once:
            d.sync()
        for t in (0, 3, 1, 2):                            # x and gpre are what the weight gradient reads
            d.release(t, dl.EV_FREE)
        if release_at_once:
            for t in (5, 6, 7, 8):                        # best fit hands out the blocks just freed
                view(d.alloc(t)).fill_(0x7F)              # bf16 3.4e38 / NaN patterns: any early write shows
        d.backward_join()
        out = gw.clone()                                  # on the compute stream, after the join
        d.sync()
        for t in (4, 5, 6, 7, 8):
            if release_at_once or t == 4:
                d.release(t, dl.EV_FREE)
        d.sync()
        return out.cpu().numpy()

    ref = run(False)
    assert np.isfinite(ref).all() and np.abs(ref).max() > 0
    for rep in range(3):
        got = run(True)
        assert np.array_equal(got.view(np.uint32), ref.view(np.uint32)), "repeat %d" % rep
    d.close()


def test_config3_full_size_backward_sampled_entries(torch_mod):
    """Config 3 at full size (ResNet-50, batch 128, 224x224x3: the launch shapes bench.py times):
    forward and the whole backward pass, then for one layer of every backward code path sampled
    entries of dL/dw and sampled pixels of dL/dx against their defining sums (oracle
    wgrad_entries / dgrad_pixels) on the GPU's own x and gpre.  A whole gradient at this size is
    beyond the oracle; a sum over all 128 images per entry is not."""
    torch = torch_mod
    import paper_2203_15980_amd as dl
    from paper_2203_15980_amd.harness import Net
    N = 128
    layers = synth.resnet_layers(N)
    g = synth.fused_graph(layers, "bf16", with_loss=True)
    boot = torch.empty(1 << 20, dtype=torch.uint8, device="cuda:0")
    d = dl.Delta(boot, torch.cuda.current_stream().cuda_stream)
    d.bind([t["bytes"] for t in g.tensors])
    net = Net(d, layers, "bf16", synth.master_seed(3), with_loss=True)
    net.enable_backward()
    d.close()
    arena = torch.empty(sum(net.sizes) + (256 << 20), dtype=torch.uint8, device="cuda:0")   # everything kept
    d = dl.Delta(arena, torch.cuda.current_stream().cuda_stream)
    net.rebind(d)
    net.forward()
    net.backward(keep=True)
    d.sync()
    trace = {t[0]: t for t in net.bwd_trace}
    by_name = {l.name: l for l in layers}
    rng = np.random.default_rng(7)
    f64 = lambda a: on.to_f64(a, "bf16")
    # 3x3 | 1x1 with residual (flattened positions) | 3x3 stride 2 (dilated gpre) | 1x1 stride 2 (gathered) |
    # 3x3 on 7x7 images | a wide 1x1 on the GEMM kernel | block inputs that accumulate a second gradient | the stem
    seen_add = False
    for lname in ("s2.b1.a2", "s2.b1.out", "s3.b1.a2", "s3.b1.sc", "s5.b3.a2", "s4.b2.out", "s3.b1.a1", "s2.b2.a1", "stem"):
        l = by_name[lname]
        _, gy_name, gpre_name, gx_name, add_name, masks_gx = trace[lname]
        print("layer", lname, "gpre", gpre_name, "gx", gx_name, "add", add_name, "mask", masks_gx, flush=True)
        p = net.params_np[lname]
        scale = (p["gamma"].astype(np.float64) / np.sqrt(p["var"].astype(np.float64) + p["eps"])).astype(np.float32)
        x = net.read(l.x) if l.x != "x0" else net.x0_np
        gp = net.read(gpre_name)
        if gp.shape[1] != l.P:                             # written at the input's resolution, zeros between
            s = l.stride
            keep = np.zeros(gp.shape[1:3], dtype=bool)
            keep[::s, ::s] = True
            assert not gp[:, ~keep, :].any()
            gp = np.ascontiguousarray(gp[:, ::s, ::s, :][:, :l.P, :l.Q, :])
        assert gp.shape == (N, l.P, l.Q, l.Cout)
        gw = net.gw[lname].cpu().numpy().astype(np.float64).reshape(l.Cout, l.R, l.S, l.Cin)
        entries = [(int(rng.integers(l.Cout)), int(rng.integers(l.R)), int(rng.integers(l.S)), int(rng.integers(l.Cin)))
                   for _ in range(24)]
        ref = np.array(on.wgrad_entries(x, gp, scale, entries, l.stride, l.pad, "bf16"))
        got = np.array([gw[e] for e in entries])
        ew = float(np.max(np.abs(got - ref)) / np.max(np.abs(gw)))
        print("  dL/dw: 24 entries, max |gw| %.3g, err %.2e" % (np.max(np.abs(gw)), ew), flush=True)
        assert np.isfinite(gw).all() and ew <= 2e-4, (lname, ew)
        if gx_name is None:
            continue
        gx = net.read(gx_name)
        pixels = [(int(rng.integers(N)), int(rng.integers(l.H)), int(rng.integers(l.W))) for _ in range(12)]
        pixels += [(N - 1, l.H - 1, l.W - 1), (0, 0, 0), (1, 0, l.W - 1), (2, 1, 1)]        # corners, both parities
        ref = on.dgrad_pixels(gp, p["w"], scale, pixels, l.stride, l.pad, l.H, l.W, "bf16")
        if add_name is not None:
            a = net.read(add_name)
            ref = ref + np.stack([f64(a[px]) for px in pixels])
            seen_add = True
        if masks_gx:
            ref = ref * np.stack([f64(x[px]) > 0 for px in pixels])
        got = np.stack([f64(gx[px]) for px in pixels])
        ex = float(np.max(np.abs(got - ref)) / np.max(np.abs(f64(gx))))
        print("  dL/dx: %d pixels, err %.2e" % (len(pixels), ex), flush=True)
        assert ex <= 2e-2, (lname, ex)
    assert seen_add
    d.close()


def _random_backward_cases(seed, count):
    """Seeded random layer shapes for both gradients: 1x1 and 3x3, stride 1 and 2, 64 to 512 channels (192 among them),
    with and without ReLU, residual, an accumulated gx and the fused masks; the class-wise strided weight gradient
    ("g") where the channel counts allow it."""
    import random
    rnd = random.Random(seed)
    chs = [64, 128, 192, 256, 512]
    cases = []
    while len(cases) < count:
        R = rnd.choice([1, 1, 3]); stride = rnd.choice([1, 1, 1, 2]); pad = (R - 1) // 2
        Cin, Cout = rnd.choice(chs), rnd.choice(chs)
        N, H, W = rnd.randint(1, 3), rnd.randint(1, 24), rnd.randint(1, 24)
        P, Q = (H + 2 * pad - R) // stride + 1, (W + 2 * pad - R) // stride + 1
        if P < 1 or Q < 1 or N * H * W * Cin * Cout * R * R > 6e8:
            continue
        relu = rnd.random() < 0.7
        has_res = R == 1 and stride == 1 and rnd.random() < 0.4
        has_add = rnd.random() < 0.5
        fuse = rnd.choice(["", "x", "y", "xy"])
        if not relu:
            fuse = fuse.replace("y", "")
        if R == 3 and stride == 2 and Cin % 128 == 0 and Cout % 128 == 0 and rnd.random() < 0.5:
            fuse += "g"
            if "x" not in fuse and "y" not in fuse:
                fuse = ("y" if relu else "x") + fuse
        cases.append(("rnd%d" % len(cases), N, H, W, Cin, Cout, R, relu, has_res, has_add, stride, fuse))
    return cases


@pytest.mark.parametrize("case", _random_backward_cases(5, 12), ids=lambda c: "%s_%dx%dx%d_%d_%d_r%d_s%d%s" % (c[0], c[1], c[2], c[3], c[4], c[5], c[6], c[10], c[11]))
def test_random_layer_shapes_backward_match_oracle(torch_mod, case):
    """The single-layer backward comparison on seeded random shapes."""
    test_layer_backward_matches_oracle(torch_mod, case)
