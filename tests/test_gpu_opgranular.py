"""GPU parity of operator-granular execution (bare convolution, batch normalisation with batch
statistics, ReLU, add as separate launches and tensors) against the CPU oracle, through the C ABI.

Tolerances: ReLU is bit-exact; add and batch normalisation store bf16 rounded once from fp32
(2^-9 relative; the bar used is 2e-2 / 4 of the tensor's maximum); the network end to end 2e-2."""
import numpy as np
import pytest

import synth
from oracle import numeric as on
from oracle import opgranular as og
from oracle import planner as opl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def torch_mod():
    import torch
    assert torch.cuda.is_available()
    return torch


def _dev(torch, a):
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")


def _ctx(torch, sizes, mb):
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


def _bits(master, aid, shape, scale=1.0, shift=0.0):
    return synth.f32_to_bf16_bits((synth.normal(master, aid, int(np.prod(shape))) * scale + shift).astype(np.float32)).reshape(shape)


def _relerr(got, ref):
    return float(np.max(np.abs(got - ref)) / max(np.max(np.abs(ref)), 1e-30))


BN = [(2, 7, 7, 64), (3, 5, 9, 24), (1, 1, 1, 8), (4, 30, 30, 256), (2, 3, 3, 2048), (1, 2, 2, 4096), (16, 56, 56, 64)]


@pytest.mark.parametrize("shape", BN, ids=lambda s: "x".join(map(str, s)))
def test_batchnorm_with_batch_statistics_matches_oracle(torch_mod, shape):
    torch = torch_mod
    import paper_2203_15980_amd as dl
    print("shape", shape, flush=True)
    N, H, W, C = shape
    x = _bits(91, 1, shape, 2.0, 3.0)                      # mean 3, spread 2: the shifted sums matter
    gamma = synth.uniform(91, 2, C, 0.5, 1.5).astype(np.float32)
    beta = synth.normal(91, 3, C, 0.0, 0.1).astype(np.float32)
    d, put, get = _ctx(torch, [x.nbytes, x.nbytes], 64)
    put(0, x)
    g, b = _dev(torch, gamma), _dev(torch, beta)
    desc = dl.LayerDesc(x=0, res=dl.NO_TENSOR, y=1, dtype=dl.DTYPE_BF16, w=None, scale=g.data_ptr(), shift=b.data_ptr(),
                        N=N, H=H, W=W, Cin=C, Cout=C, R=1, S=1, stride=1, pad=0, relu=0, op=dl.OP_BATCHNORM, eps=1e-5)
    d.recompute_segment([desc])
    d.sync()
    first = get(1, shape).copy()
    ref = on.to_f64(og.bn_train(x, gamma, beta, 1e-5, "bf16"), "bf16")
    err = _relerr(on.to_f64(first, "bf16"), ref)
    print("  err %.2e" % err, flush=True)
    assert err <= 2e-2 / 4, (shape, err)
    d.recompute_segment([desc])                            # fixed reduction order: the same bits again
    d.sync()
    assert np.array_equal(get(1, shape), first)
    d.close()


def test_relu_and_add_match_oracle(torch_mod):
    torch = torch_mod
    import paper_2203_15980_amd as dl
    shape = (3, 9, 11, 40)
    x, r = _bits(92, 1, shape), _bits(92, 2, shape, 0.01)
    x.reshape(-1)[:6] = [0x0000, 0x8000, 0xFF80, 0x7F80, 0x8001, 0x0001]    # +-0, -inf, +inf, smallest denormals
    nb = x.nbytes
    d, put, get = _ctx(torch, [nb, nb, nb, nb], 8)
    put(0, x)
    put(1, r)
    geo = dict(dtype=dl.DTYPE_BF16, w=None, scale=None, shift=None, N=3, H=9, W=11, Cin=40, Cout=40, R=1, S=1, stride=1,
               pad=0, relu=0)
    d.recompute_segment([dl.LayerDesc(x=0, res=dl.NO_TENSOR, y=2, op=dl.OP_RELU, **geo),
                         dl.LayerDesc(x=0, res=1, y=3, op=dl.OP_ADD, **geo)])
    d.sync()
    assert np.array_equal(on.to_f64(get(2, shape), "bf16"), on.to_f64(og.relu(x, "bf16"), "bf16"))
    got, ref = on.to_f64(get(3, shape), "bf16").reshape(-1)[6:], on.to_f64(og.add(x, r, "bf16"), "bf16").reshape(-1)[6:]
    assert np.mean(got == ref) > 0.999 and _relerr(got, ref) <= 2.0 ** -8
    for bad in (dl.LayerDesc(x=0, res=1, y=2, op=dl.OP_RELU, **geo), dl.LayerDesc(x=0, res=dl.NO_TENSOR, y=3, op=dl.OP_ADD, **geo),
                dl.LayerDesc(x=0, res=dl.NO_TENSOR, y=2, op=dl.OP_BATCHNORM, **{**geo, "Cin": 20, "Cout": 20, "W": 22})):
        with pytest.raises(dl.DeltaError):
            d.recompute_segment([bad])
    d.close()


def _mini(torch, arena_bytes):
    import paper_2203_15980_amd as dl
    from paper_2203_15980_amd.harness import OpNet
    layers = synth.resnet_layers(2, (1, 1, 1, 1), image=64, classes=40)
    g = synth.opgranular_graph(layers, "bf16", with_loss=True)
    arena = torch.empty(arena_bytes or (g.total_bytes() + (1 << 20)), dtype=torch.uint8, device="cuda:0")
    d = dl.Delta(arena, torch.cuda.current_stream().cuda_stream)
    d.bind([t["bytes"] for t in g.tensors])
    return d, OpNet(d, layers, 93), layers, g


def test_small_resnet_operator_by_operator(torch_mod):
    """A ResNet with one bottleneck per stage on 2 x 64 x 64 x 3, 57 tensors: every operator is checked
    against the oracle on the GPU's own input tensor; the whole chain against the oracle's own."""
    d, net, layers, g = _mini(torch_mod, None)
    net.forward()
    d.sync()
    acts = {n: net.read(n) for n in ["x0"] + net.op_names}
    alias = {"x0": "x0"}
    for l in layers:
        x = acts[alias[l.x]]
        p = net.params_np.get(l.name)
        if l.kind == "conv":
            refs = [(l.name + ".conv", on.conv_bn_act(x, p["w"], None, stride=l.stride, pad=l.pad, relu=False, dtype="bf16"))]
            refs.append((l.name + ".bn", og.bn_train(acts[l.name + ".conv"], p["gamma"], p["beta"], p["eps"], "bf16")))
            t = l.name + ".bn"
            if l.res:
                refs.append((l.name + ".add", og.add(acts[t], acts[alias[l.res]], "bf16")))
                t = l.name + ".add"
            if l.relu:
                refs.append((l.name + ".relu", og.relu(acts[t], "bf16")))
                t = l.name + ".relu"
        elif l.kind == "maxpool":
            t, refs = l.name, [(l.name, on.maxpool(x, l.R, l.S, l.stride, l.pad, "bf16"))]
        elif l.kind == "avgpool":
            t, refs = l.name, [(l.name, on.avgpool(x, "bf16"))]
        else:
            t = l.name
            C = l.Cout
            bn = dict(gamma=np.ones(C, np.float32), beta=p["bias"], mean=np.zeros(C, np.float32), var=np.ones(C, np.float32), eps=0.0)
            refs = [(t, on.conv_bn_act(x, p["w"], bn, relu=False, dtype="bf16"))]
        alias[l.y] = t
        for name, ref in refs:
            err = _relerr(on.to_f64(acts[name], "bf16"), on.to_f64(ref, "bf16"))
            assert err <= 2e-2, (name, err)
    ref_all = og.run_ops(layers, net.params_np, net.x0_np, "bf16")
    last = alias[layers[-1].y]
    err = _relerr(on.to_f64(acts[last], "bf16"), on.to_f64(ref_all[last], "bf16"))
    print("  end to end (logits) err %.2e over %d operators" % (err, len(net.op_names)), flush=True)
    assert err <= 2e-2, err
    assert sum(n.endswith(".bn") for n in net.op_names) == 17 and any(n.endswith(".add") for n in net.op_names)
    d.close()


def test_operator_granular_plan_replay(torch_mod):
    """The 57-tensor operator-granular graph planned at half of its bytes (library plan = oracle plan)
    and replayed: every tensor a backward step reads is bit-identical to the unconstrained forward's
    (batch-norm statistics are recomputed in a fixed order).  Then once more with the proxy backward."""
    import paper_2203_15980_amd as dl
    from paper_2203_15980_amd.harness import run_plan
    d0, net0, layers, g = _mini(torch_mod, None)
    net0.forward()
    d0.sync()
    want = {t["name"]: net0.read(t["name"]).copy() for t in g.tensors}
    d0.close()
    budget = g.total_bytes() // 2
    p = opl.default_params(budget, g.n_fwd, bw_d2h_Bps=50 * 10**9, bw_h2d_Bps=50 * 10**9)
    ev, peak = dl.plan(g.tensors, g.steps, p)
    assert (ev, peak) == opl.plan(g.tensors, g.steps, p)
    d, net, layers, g = _mini(torch_mod, int(budget * 1.5) + (1 << 20))
    seen = set()

    def check(k):
        for t in g.steps[k]["reads"]:
            n = g.tensors[t]["name"]
            assert net.read(n).tobytes() == want[n].tobytes(), (k, n)
            seen.add(n)

    run_plan(net, g, ev, backward_proxy=check)
    d.sync()
    st = d.stats()
    kinds = {a for (_, a, _) in ev}
    print("events", sorted(kinds), "peak", peak, "budget", budget, flush=True)
    assert st["arena_in_use"] == 0 and st["arena_high_water"] <= budget
    assert dl.EV_RECOMPUTE in kinds and any(n.endswith(".conv") for n in seen) and any(n.endswith(".relu") for n in seen)
    net.enable_backward_proxy()
    run_plan(net, g, ev, backward_proxy=lambda k: net.backward_proxy_step(g, k))
    d.sync()
    assert d.stats()["arena_in_use"] == 0
    d.close()


# ------------------------------------------------------------------------------- backward

BN_BWD = [(2, 7, 7, 64), (3, 5, 9, 24), (1, 1, 2, 8), (4, 30, 30, 256), (2, 3, 3, 2048), (16, 56, 56, 64)]


@pytest.mark.parametrize("shape", BN_BWD, ids=lambda s: "x".join(map(str, s)))
def test_batchnorm_backward_matches_oracle(torch_mod, shape):
    """gx stored in bf16 from fp32 arithmetic on double-precision channel factors: 2e-2 / 4 of its
    maximum; dgamma, dbeta fp32 from fp32 partial sums combined in double: 2e-4 of their maximum
    (plus 1e-6 of sum |gy|, the rounding floor of a sum that nearly cancels)."""
    torch = torch_mod
    import paper_2203_15980_amd as dl
    print("shape", shape, flush=True)
    N, H, W, C = shape
    x = _bits(94, 1, shape, 2.0, 3.0)
    gy = _bits(94, 4, shape, 0.5, 0.1)
    gamma = synth.uniform(94, 2, C, 0.5, 1.5).astype(np.float32)
    d, put, get = _ctx(torch, [x.nbytes] * 4, 64)
    put(0, x)
    put(1, gy)
    g = _dev(torch, gamma)
    gw = torch.full((2 * C,), float("nan"), dtype=torch.float32, device="cuda:0")
    fwd = dl.LayerDesc(x=0, res=dl.NO_TENSOR, y=3, dtype=dl.DTYPE_BF16, w=None, scale=g.data_ptr(), shift=g.data_ptr(),
                       N=N, H=H, W=W, Cin=C, Cout=C, R=1, S=1, stride=1, pad=0, relu=0, op=dl.OP_BATCHNORM, eps=1e-5)
    desc = dl.BwdDesc(fwd=fwd, gy=1, gpre=1, gx=2, gx_add=dl.NO_TENSOR, mask_gx=0, gy_masked=0, wt=None,
                      gw=gw.data_ptr(), workspace=None, workspace_bytes=0)
    d.backward_segment([desc])
    d.sync()
    first = get(2, shape).copy()
    ref_gx, ref_dg, ref_db = og.bn_train_bwd(x, gamma, gy, 1e-5, "bf16")
    err = _relerr(on.to_f64(first, "bf16"), on.to_f64(ref_gx, "bf16"))
    got_w = gw.cpu().numpy().astype(np.float64)
    floor = 1e-6 * np.abs(on.to_f64(gy, "bf16")).sum(axis=(0, 1, 2)).max()
    eg = np.max(np.abs(got_w[:C] - ref_dg)) / (np.max(np.abs(ref_dg)) + floor)
    eb = np.max(np.abs(got_w[C:] - ref_db)) / (np.max(np.abs(ref_db)) + floor)
    print("  gx %.2e dgamma %.2e dbeta %.2e" % (err, eg, eb), flush=True)
    assert err <= 2e-2 / 4 and eg <= 2e-4 and eb <= 2e-4, (shape, err, eg, eb)
    d.backward_segment([desc])                             # fixed reduction order: the same bits again
    d.sync()
    assert np.array_equal(get(2, shape), first) and np.array_equal(gw.cpu().numpy().astype(np.float64), got_w)
    d.close()


def test_relu_backward_and_rejects(torch_mod):
    torch = torch_mod
    import paper_2203_15980_amd as dl
    shape = (3, 5, 7, 24)
    y = og.relu(_bits(95, 1, shape), "bf16")
    y.reshape(-1)[:3] = [0x8000, 0x7FC0, 0x0001]           # -0, NaN, the smallest positive value
    gy = _bits(95, 2, shape)
    d, put, get = _ctx(torch, [y.nbytes] * 4, 16)
    put(1, y)
    put(2, gy)
    geo = dict(dtype=dl.DTYPE_BF16, w=None, scale=None, shift=None, N=3, H=5, W=7, Cin=24, Cout=24, R=1, S=1, stride=1,
               pad=0, relu=0)
    fwd = dl.LayerDesc(x=0, res=dl.NO_TENSOR, y=1, op=dl.OP_RELU, **geo)     # x is not resident: not read
    mk = lambda **kw: dl.BwdDesc(**{**dict(fwd=fwd, gy=2, gpre=2, gx=3, gx_add=dl.NO_TENSOR, mask_gx=0, gy_masked=0, wt=None,
                                           gw=None, workspace=None, workspace_bytes=0), **kw})
    d.backward_segment([mk()])
    d.sync()
    got, ref = get(3, shape), og.relu_bwd(y, gy, "bf16")
    assert np.array_equal(got.reshape(-1)[3:], ref.reshape(-1)[3:])
    assert list(got.reshape(-1)[:3]) == [0, 0, gy.reshape(-1)[2]]
    g = torch.zeros(64, dtype=torch.float32, device="cuda:0")
    bn = dl.LayerDesc(x=1, res=dl.NO_TENSOR, y=0, op=dl.OP_BATCHNORM, eps=1e-5,
                      **{**geo, "scale": g.data_ptr(), "shift": g.data_ptr()})
    for bad in (mk(gx=2), mk(gx=1), mk(gpre=3), mk(gx_add=1), mk(mask_gx=1), mk(gw=g.data_ptr()),
                mk(fwd=bn, gw=g.data_ptr() + 4),
                mk(fwd=dl.LayerDesc(x=0, res=1, y=3, op=dl.OP_ADD, **geo))):
        with pytest.raises(dl.DeltaError):
            d.backward_segment([bad])
    d.release(1, dl.EV_FREE)
    with pytest.raises(dl.DeltaError):                     # the stored output is what the mask is read from
        d.backward_segment([mk()])
    d.close()


def test_small_resnet_operator_granular_backward(torch_mod):
    """Loss to stem through every operator's own backward kernel; each operator is checked against
    the oracle on the GPU's own tensors (activations and incoming gradient), parameter gradients
    included.  Then a replay under half the activation budget with this backward: the parameter
    gradients are bit-identical to the unconstrained run's (recomputation returns the same bits and
    every reduction has a fixed order)."""
    import paper_2203_15980_amd as dl
    from paper_2203_15980_amd.harness import run_plan
    torch = torch_mod
    d0, net, layers, g = _mini(torch, None)
    d0.close()
    net.delta = None
    arena = torch.empty(3 * g.total_bytes() + (8 << 20), dtype=torch.uint8, device="cuda:0")
    d = dl.Delta(arena, torch.cuda.current_stream().cuda_stream)
    net.rebind(d)
    net.enable_backward()
    net.forward()
    net.backward(keep=True)
    d.sync()
    acts = {n: net.read(n) for n in ["x0"] + net.op_names}
    f64 = lambda a: on.to_f64(a, "bf16")
    worst = {}
    for (name, kind, gy, gx, add) in net.bwd_trace:
        l = net.op_layer[name]
        x, res = net.op_inputs[name]
        if kind == "add":
            continue
        gyv = net.read(gy)
        p = net.params_np.get(l.name)
        ref_w = None
        if kind == "conv":
            ref, ref_w, _ = on.conv_bn_act_bwd(acts[x], p["w"], None, None, gyv, stride=l.stride, pad=l.pad, relu=False,
                                               dtype="bf16")
        elif kind == "bn":
            r, dg, db = og.bn_train_bwd(acts[x], p["gamma"], gyv, p["eps"], "bf16")
            ref, ref_w = f64(r), np.concatenate([dg, db])
        elif kind == "relu":
            ref = f64(og.relu_bwd(acts[name], gyv, "bf16"))
        elif kind == "maxpool":
            ref = on.maxpool_bwd(acts[x], gyv, l.R, l.S, l.stride, l.pad, "bf16")
        elif kind == "avgpool":
            ref = on.avgpool_bwd(gyv, l.H, l.W, "bf16")
        else:
            ref, w_, b_ = on.fc_bwd(acts[x], p["w"], gyv, "bf16")
            ref_w = np.concatenate([w_.reshape(-1), b_])
        if gx is not None:
            if add is not None:
                ref = ref + f64(net.read(add)).reshape(ref.shape)
            e = _relerr(f64(net.read(gx)).reshape(ref.shape), ref)
            worst[kind] = max(worst.get(kind, 0.0), e)
            assert e <= 2e-2, (name, e)
        if ref_w is not None:
            got_w = net.gw[name].cpu().numpy().astype(np.float64).reshape(-1)
            e = _relerr(got_w, ref_w.reshape(-1))
            worst[kind + ".w"] = max(worst.get(kind + ".w", 0.0), e)
            assert e <= 2e-4, (name, e)
    print("  worst", {k: "%.1e" % v for k, v in sorted(worst.items())}, flush=True)
    kinds = [t[1] for t in net.bwd_trace]
    assert kinds.count("bn") == 17 and kinds.count("add") == 4 and kinds.count("conv") == 17
    assert sum(1 for t in net.bwd_trace if t[4] is not None) == 4          # one accumulation per block input
    want = {n: t.clone() for n, t in net.gw.items()}
    d.close()                                              # kept tensors go with the context
    budget = g.total_bytes() // 2
    arena = torch.empty(int(budget * 1.5) + net.backward_peak_bytes() * 2 + (8 << 20), dtype=torch.uint8, device="cuda:0")
    d = dl.Delta(arena, torch.cuda.current_stream().cuda_stream)
    net.rebind(d)
    p = opl.default_params(budget, g.n_fwd, bw_d2h_Bps=50 * 10**9, bw_h2d_Bps=50 * 10**9)
    ev, peak = dl.plan(g.tensors, g.steps, p)
    for t in net.gw.values():
        t.fill_(float("nan"))
    run_plan(net, g, ev, backward_proxy=lambda k: net.backward_step(g, k))
    d.sync()
    assert d.stats()["arena_in_use"] == 0
    for n, t in net.gw.items():
        assert torch.equal(t.view(torch.int32), want[n].view(torch.int32)), n
    d.close()


def test_config3_full_size_operator_granular_sampled(torch_mod):
    """ResNet-50 at batch 128 at operator granularity (the launch shapes bench.py replays):
    forward and the whole backward; batch normalisation is independent per channel, so the oracle
    runs whole sampled channels (statistics over all 128 images) of a 205 MB, a 51 MB and a 13 MB
    tensor, forward and backward; one ReLU backward whole (bit-exact); one bare convolution's
    weight gradient on sampled entries."""
    import paper_2203_15980_amd as dl
    from paper_2203_15980_amd.harness import OpNet
    torch = torch_mod
    N = 128
    layers = synth.resnet_layers(N)
    g = synth.opgranular_graph(layers, "bf16", with_loss=True)
    boot = torch.empty(1 << 20, dtype=torch.uint8, device="cuda:0")
    d = dl.Delta(boot, torch.cuda.current_stream().cuda_stream)
    d.bind([t["bytes"] for t in g.tensors])
    net = OpNet(d, layers, synth.master_seed(3))
    net.enable_backward()
    d.close()
    arena = torch.empty(sum(net.sizes) + (256 << 20), dtype=torch.uint8, device="cuda:0")   # everything kept
    d = dl.Delta(arena, torch.cuda.current_stream().cuda_stream)
    net.rebind(d)
    net.forward()
    net.backward(keep=True)
    d.sync()
    trace = {t[0]: t for t in net.bwd_trace}
    rng = np.random.default_rng(11)
    f64 = lambda a: on.to_f64(a, "bf16")
    for lname in ("stem", "s2.b1.out", "s3.b2.a1", "s5.b3.out"):
        name = lname + ".bn"
        _, kind, gy_name, gx_name, _ = trace[name]
        assert kind == "bn"
        p = net.params_np[lname]
        x, y, gy, gx = net.read(lname + ".conv"), net.read(name), net.read(gy_name), net.read(gx_name)
        gw = net.gw[name].cpu().numpy().astype(np.float64)
        C = x.shape[-1]
        print("batch-norm", name, x.shape, flush=True)
        for c in sorted({0, C - 1, int(rng.integers(C))}):
            one = lambda a: np.ascontiguousarray(a[..., c:c + 1])
            ref_y = og.bn_train(one(x), p["gamma"][c:c + 1], p["beta"][c:c + 1], p["eps"], "bf16")
            ey = _relerr(f64(one(y)), f64(ref_y))
            ref_gx, dg, db = og.bn_train_bwd(one(x), p["gamma"][c:c + 1], one(gy), p["eps"], "bf16")
            ex = _relerr(f64(one(gx)), f64(ref_gx))
            floor = 1e-6 * np.abs(f64(one(gy))).sum()
            eg, eb = abs(gw[c] - dg[0]) / (abs(dg[0]) + floor), abs(gw[C + c] - db[0]) / (abs(db[0]) + floor)
            print("  channel %4d: y %.2e gx %.2e dgamma %.2e dbeta %.2e" % (c, ey, ex, eg, eb), flush=True)
            assert ey <= 2e-2 / 4 and ex <= 2e-2 / 4 and eg <= 2e-4 and eb <= 2e-4, (name, c, ey, ex, eg, eb)
    name = "s2.b1.out.relu"
    _, kind, gy_name, gx_name, _ = trace[name]
    assert kind == "relu" and np.array_equal(net.read(gx_name), og.relu_bwd(net.read(name), net.read(gy_name), "bf16"))
    name = "s2.b1.a2.conv"
    _, kind, gy_name, gx_name, add = trace[name]
    l = net.op_layer[name]
    gwc = net.gw[name].cpu().numpy().astype(np.float64).reshape(l.Cout, l.R, l.S, l.Cin)
    entries = [(int(rng.integers(l.Cout)), int(rng.integers(3)), int(rng.integers(3)), int(rng.integers(l.Cin))) for _ in range(16)]
    ref = np.array(on.wgrad_entries(net.read(net.op_inputs[name][0]), net.read(gy_name), None, entries, 1, 1, "bf16"))
    ew = float(np.max(np.abs(np.array([gwc[e] for e in entries]) - ref)) / np.max(np.abs(gwc)))
    print("bare convolution dL/dw: 16 entries, err %.2e" % ew, flush=True)
    assert ew <= 2e-4
    d.close()
