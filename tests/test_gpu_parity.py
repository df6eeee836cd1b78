"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by element.

Tolerances (max |gpu - oracle| / max |oracle| per tensor): 1e-4 for fp32, 2e-2 for bf16.
Recomputed tensors must equal the GPU's own forward bit for bit; swapped tensors byte for
byte; every operand a replayed plan hands to a step must carry its forward bits."""
import numpy as np
import pytest

import synth
from oracle import numeric as on
from oracle import planner as opl

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-4, "bf16": 2e-2}


@pytest.fixture(scope="module")
def torch_mod():
    import torch
    assert torch.cuda.is_available()
    return torch


def make_delta(torch, arena_bytes):
    import paper_2203_15980_amd as dl
    arena = torch.empty(int(arena_bytes), dtype=torch.uint8, device="cuda:0")
    return dl.Delta(arena, torch.cuda.current_stream().cuda_stream)


def rel_err(gpu, ref, dtype):
    g, r = on.to_f64(gpu, dtype), on.to_f64(ref, dtype)
    return float(np.max(np.abs(g - r)) / max(np.max(np.abs(r)), 1e-30))


def single(name, N, H, W, Cin, Cout, R, stride, pad, relu, res):
    l = synth.LayerSpec(name, "conv", "x0", "r0" if res else None, name, N, H, W, Cin, Cout, R, R, stride, pad, relu)
    l.index = 1
    return l


CASES = [
    # name            N   H   W  Cin Cout R st pad relu  res
    ("1x1_64_64",     3, 13, 13,  64,  64, 1, 1, 0, True, False),   # M = 507: ragged tail
    ("1x1_64_256",    2, 17, 11,  64, 256, 1, 1, 0, False, False),
    ("1x1_256_64",    1, 20, 20, 256,  64, 1, 1, 0, True, False),   # several reduction slices
    ("1x1_res",       2, 12, 12,  64, 256, 1, 1, 0, True, True),
    ("3x3_s1",        2, 14, 14,  64,  64, 3, 1, 1, True, False),
    ("3x3_s2",        2, 15, 15,  64, 128, 3, 2, 1, True, False),
    ("1x1_s2",        2, 14, 14, 128, 128, 1, 2, 0, False, False),
    ("3x3_128",       1,  9,  9, 128, 128, 3, 1, 1, True, True),
    ("tiny",          1,  1,  1,  64,  64, 1, 1, 0, True, False),   # one pixel
    ("5x5_pad2",      1,  8,  8,  64,  64, 5, 1, 2, False, False),
    # 1x1 with more output channels than one LDS-resident weight slice (bf16: sliced streaming)
    ("1x1_sl_64_512",  2, 12, 12,  64,  512, 1, 1, 0, True, False),  # 2 slices of 256
    ("1x1_sl_128_512", 2, 13, 11, 128,  512, 1, 1, 0, True, True),   # residual, ragged
    ("1x1_sl_128_768", 2, 14, 14, 128,  768, 1, 2, 0, False, False), # stride 2, 3 slices of 256
    ("1x1_sl_64_1k",   1, 14, 14,  64, 1024, 1, 1, 0, True, True),   # 4 slices
    ("1x1_sl_128_192", 2, 10, 10, 128,  192, 1, 1, 0, False, False), # 3 slices of 64
    ("1x1_256_1k",     1, 14, 14, 256, 1024, 1, 1, 0, True, True),   # tiled kernel, 8 channel tiles
    ("1x1_512_128",    3,  9,  9, 512,  128, 1, 1, 0, True, False),
    # a projection shortcut's shape: stride 2 on an odd image, enough tiles for the GEMM kernel (bf16), ragged last tile
    ("1x1_s2_256_512", 3, 147, 147, 256, 512, 1, 2, 0, False, False),
    # 3x3 stride 1 (bf16: the LDS-halo kernel): image borders inside a pixel tile, ragged tail,
    # odd step count, non-square images, wide rows
    ("3x3_halo_res",  3, 13, 13, 128,  64, 3, 1, 1, True, True),    # M = 507: two tiles, ragged
    ("3x3_halo_192",  5, 16, 16, 192, 128, 3, 1, 1, True, False),   # three channel blocks: 27 steps
    ("3x3_halo_5x7",  1,  5,  7,  64, 128, 3, 1, 1, False, False),  # one small non-square image
    ("3x3_halo_wide", 2,  4, 60,  64,  64, 3, 1, 1, True, False),   # W = 60: longest halo variant
    ("3x3_halo_1px",  3,  1,  1,  64,  64, 3, 1, 1, False, False),  # only the centre tap is valid
]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
def test_single_layer_matches_oracle(torch_mod, dtype, case):
    torch = torch_mod
    import paper_2203_15980_amd as dl
    name, N, H, W, Cin, Cout, R, stride, pad, relu, res = case
    print("case", name, dtype, flush=True)
    l = single(name, N, H, W, Cin, Cout, R, stride, pad, relu, res)
    es = 4 if dtype == "f32" else 2
    master = 77
    x = synth.make_input(master, (N, H, W, Cin), dtype)
    p = synth.make_params(master, l, dtype)
    rshape = (N, l.P, l.Q, Cout)
    r = None
    if res:
        r = synth.normal(master, 999, int(np.prod(rshape))).astype(np.float32).reshape(rshape)
        r = r if dtype == "f32" else synth.f32_to_bf16_bits(r).reshape(rshape)
    ref = on.conv_bn_act(x, p["w"], p, res=r, stride=stride, pad=pad, relu=relu, dtype=dtype)

    sizes = [x.nbytes, int(np.prod(rshape)) * es, int(np.prod(rshape)) * es]     # x, res, y
    d = make_delta(torch, max(64 << 20, sum(sizes) + (8 << 20)))
    d.bind(sizes)
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")
    w = dev(p["w"])
    bn = [dev(p[k]) for k in ("gamma", "beta", "mean", "var")]
    scale = torch.empty(Cout, dtype=torch.float32, device="cuda:0")
    shift = torch.empty(Cout, dtype=torch.float32, device="cuda:0")
    d.bn_fold(bn[0].data_ptr(), bn[1].data_ptr(), bn[2].data_ptr(), bn[3].data_ptr(), float(p["eps"]),
              Cout, scale.data_ptr(), shift.data_ptr())
    base = d.arena.data_ptr()
    px = d.alloc(0)
    d.arena[px - base:px - base + sizes[0]].copy_(dev(x.view(np.uint8).reshape(-1)))
    if res:
        pr = d.alloc(1)
        d.arena[pr - base:pr - base + sizes[1]].copy_(dev(r.view(np.uint8).reshape(-1)))
    desc = dl.LayerDesc(x=0, res=1 if res else dl.NO_TENSOR, y=2,
                        dtype=dl.DTYPE_F32 if dtype == "f32" else dl.DTYPE_BF16, w=w.data_ptr(),
                        scale=scale.data_ptr(), shift=shift.data_ptr(), N=N, H=H, W=W, Cin=Cin, Cout=Cout,
                        R=R, S=R, stride=stride, pad=pad, relu=1 if relu else 0)
    if name == "1x1_s2_256_512" and dtype == "bf16":
        assert "gemm_nt" in d.layer_kernel(desc), d.layer_kernel(desc)
    d.recompute_segment([desc])
    py = d.tensor_ptr(2)
    d.sync()
    got = d.arena[py - base:py - base + sizes[2]].cpu().numpy().view(np.float32 if dtype == "f32" else np.uint16)
    got = got.reshape(rshape)
    err = rel_err(got, ref, dtype)
    assert err <= TOL[dtype], (name, dtype, err)
    # folded scale/shift against the textbook form
    s_ref = p["gamma"].astype(np.float64) / np.sqrt(p["var"].astype(np.float64) + p["eps"])
    np.testing.assert_allclose(scale.cpu().numpy(), s_ref, rtol=1e-6)
    d.close()


def test_conv3x3_c64_persistent_workgroups_on_sampled_images(torch_mod):
    """The 64 -> 64 channel 3x3 kernel keeps its workgroups alive over several tiles once there are more
    than 256 tiles: 40 images of 56 x 56 make 506 tiles of 248 pixels (two rounds, the second ragged).
    With residual and ReLU; the oracle computes the first and the last image (a convolution with frozen
    statistics treats images independently).  Recomputation gives the same bits."""
    torch = torch_mod
    import paper_2203_15980_amd as dl
    N, H, W, C = 40, 56, 56, 64
    l = single("c64_rounds", N, H, W, C, C, 3, 1, 1, True, True)
    x = synth.make_input(78, (N, H, W, C), "bf16")
    p = synth.make_params(78, l, "bf16")
    r = synth.f32_to_bf16_bits(synth.normal(78, 999, N * H * W * C).astype(np.float32)).reshape(N, H, W, C)
    d = make_delta(torch, 64 << 20)
    d.bind([x.nbytes] * 3)
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")
    w = dev(p["w"])
    bn = [dev(p[k]) for k in ("gamma", "beta", "mean", "var")]
    scale = torch.empty(C, dtype=torch.float32, device="cuda:0")
    shift = torch.empty(C, dtype=torch.float32, device="cuda:0")
    d.bn_fold(bn[0].data_ptr(), bn[1].data_ptr(), bn[2].data_ptr(), bn[3].data_ptr(), float(p["eps"]), C,
              scale.data_ptr(), shift.data_ptr())
    base = d.arena.data_ptr()
    for tid, a in ((0, x), (1, r)):
        ptr = d.alloc(tid)
        d.arena[ptr - base:ptr - base + a.nbytes].copy_(dev(a.view(np.uint8).reshape(-1)))
    desc = dl.LayerDesc(x=0, res=1, y=2, dtype=dl.DTYPE_BF16, w=w.data_ptr(), scale=scale.data_ptr(),
                        shift=shift.data_ptr(), N=N, H=H, W=W, Cin=C, Cout=C, R=3, S=3, stride=1, pad=1, relu=1)
    assert "c64" in d.layer_kernel(desc)
    d.recompute_segment([desc])
    py = d.tensor_ptr(2)
    d.sync()
    got = d.arena[py - base:py - base + x.nbytes].cpu().numpy().view(np.uint16).reshape(N, H, W, C).copy()
    for img in (0, N - 1):
        ref = on.conv_bn_act(x[img:img + 1], p["w"], p, res=r[img:img + 1], stride=1, pad=1, relu=True, dtype="bf16")
        err = rel_err(got[img:img + 1], ref, "bf16")
        print("image %d err %.2e" % (img, err), flush=True)
        assert err <= TOL["bf16"], (img, err)
    d.release(2, dl.EV_EVICT)
    filler = d.alloc(2)                                       # a recomputation at another address
    d.release(2, dl.EV_FREE)
    d.recompute_segment([desc])
    py2 = d.tensor_ptr(2)
    d.sync()
    again = d.arena[py2 - base:py2 - base + x.nbytes].cpu().numpy().view(np.uint16).reshape(N, H, W, C)
    assert np.array_equal(again, got)
    d.close()


def _stack(torch, N, HW, dtype, master, arena_mult=1.0):
    from paper_2203_15980_amd.harness import Net
    layers = synth.bottleneck_stack(N, HW, HW)
    g = synth.fused_graph(layers, dtype)
    d = make_delta(torch, int(g.total_bytes() * arena_mult) + (1 << 20))
    d.bind([t["bytes"] for t in g.tensors])
    return d, Net(d, layers, dtype, master), layers, g


def test_config1_stack_matches_oracle(torch_mod):
    """Config 1 in full: fp32, batch 2, 32x32x64, three bottleneck blocks."""
    d, net, layers, g = _stack(torch_mod, 2, 32, "f32", synth.master_seed(1))
    net.forward()
    ref = on.run_layers(layers, net.params_np, net.x0_np, "f32")
    for l in layers:
        err = rel_err(net.read(l.y), ref[l.y], "f32")
        print(l.y, err, flush=True)
        assert err <= 1e-4, (l.y, err)
    d.close()


def test_bf16_stack_matches_oracle_and_layerwise(torch_mod):
    """bf16 stack at 2x56x56 (config 2's layer shapes, smaller batch): end to end and, with
    the GPU's own stored input fed to the oracle, layer by layer."""
    d, net, layers, g = _stack(torch_mod, 2, 56, "bf16", synth.master_seed(2))
    net.forward()
    ref = on.run_layers(layers, net.params_np, net.x0_np, "bf16")
    acts = {"x0": net.x0_np}
    for l in layers:
        acts[l.y] = net.read(l.y)
        assert rel_err(acts[l.y], ref[l.y], "bf16") <= 2e-2, l.y
        p = net.params_np[l.name]
        one = on.conv_bn_act(acts[l.x], p["w"], p, res=acts[l.res] if l.res else None, stride=l.stride,
                             pad=l.pad, relu=l.relu, dtype="bf16")
        e = rel_err(acts[l.y], one, "bf16")
        assert e <= 2.0**-7, (l.y, e)            # same inputs: at most about one bf16 ulp of the max
    d.close()


def test_config2_full_size_sampled_images(torch_mod):
    """Config 2 at full size (batch 32, 56x56, the launch shape bench.py times).  Frozen
    batch-norm makes images independent, so the oracle runs the first and the last image
    and is compared with those images of the full-batch GPU result."""
    d, net, layers, g = _stack(torch_mod, 32, 56, "bf16", synth.master_seed(2))
    net.forward()
    sub = synth.bottleneck_stack(2, 56, 56)
    x_sub = np.ascontiguousarray(net.x0_np[[0, 31]])
    ref = on.run_layers(sub, net.params_np, x_sub, "bf16")
    for l in layers:
        got = net.read(l.y)[[0, 31]]
        err = rel_err(got, ref[l.y], "bf16")
        print(l.y, err, flush=True)
        assert err <= 2e-2, (l.y, err)
    d.close()


def test_recompute_is_bit_identical_to_forward(torch_mod):
    import paper_2203_15980_amd as dl
    for dtype in ("f32", "bf16"):
        d, net, layers, g = _stack(torch_mod, 2, 32, dtype, 5, arena_mult=1.5)
        net.forward()
        saved = {l.y: net.read(l.y).copy() for l in layers}
        old_ptr = {n: d.tensor_ptr(net.ids[n]) for n in ("b1.a1", "b1.a2", "b2.a1")}
        for n in ("b1.a1", "b1.a2", "b1.sc", "b2.a1", "b2.a2", "b3.a1"):
            d.release(net.ids[n], dl.EV_EVICT)
        # best fit sends b1.a1 into the hole b3.a1 left and b1.a2 into b2's: new addresses
        for n in ("b1.a1", "b1.a2", "b1.sc", "b2.a1", "b2.a2", "b3.a1"):
            net.recompute(n)
        moved = sum(d.tensor_ptr(net.ids[n]) != old_ptr[n] for n in old_ptr)
        for n in ("b1.a1", "b1.a2", "b1.sc", "b2.a1", "b2.a2", "b3.a1"):
            assert net.read(n).tobytes() == saved[n].tobytes(), (dtype, n)
        assert moved >= 1, "no tensor changed address; the test lost its point"
        # recomputing in place gives the same bits as well
        net.recompute("b3.out")
        assert net.read("b3.out").tobytes() == saved["b3.out"].tobytes()
        d.close()


def test_swap_round_trip_is_byte_exact(torch_mod):
    import paper_2203_15980_amd as dl
    d, net, layers, g = _stack(torch_mod, 2, 32, "bf16", 9)
    net.forward()
    names = ["x0", "b1.a1", "b1.out", "b2.a2"]
    saved = {n: net.read(n).copy() for n in names}
    for n in names:
        d.release(net.ids[n], dl.EV_OFFLOAD)
    # reuse the freed blocks for something else while the copies may still be in flight
    d.release(net.ids["b3.a1"], dl.EV_EVICT)
    net.recompute("b3.a1")                       # lands in a block whose Offload may still run
    for n in reversed(names):
        d.prefetch(net.ids[n])
    for n in names:
        assert net.read(n).tobytes() == saved[n].tobytes(), n
    st = d.stats()
    total = sum(net.sizes[net.ids[n]] for n in names)
    assert st["d2h_bytes"] == total and st["h2d_bytes"] == total
    assert st["d2h_copies"] == 4 and st["h2d_copies"] == 4 and st["d2h_ms"] > 0 and st["h2d_ms"] > 0
    # swap_out without release keeps the tensor usable and makes a later Offload free
    d.swap_out(net.ids["b3.a1"])
    d.release(net.ids["b3.a1"], dl.EV_OFFLOAD)
    assert d.stats()["d2h_copies"] == 5
    d.close()


def test_swap_round_trip_of_tensors_larger_than_one_copy_piece(torch_mod):
    """Tensors above 32 MiB travel as four copies: a Reload issued right behind the Offload follows it
    piece by piece, one issued after a sync takes the plain path; both return the bytes, also with a
    ragged last piece and with sizes at and just above the boundary."""
    torch = torch_mod
    import paper_2203_15980_amd as dl
    whole = 32 << 20
    sizes = [2 * whole + 4096 + 256, whole, whole + 256, whole + whole // 2, 1 << 20]
    # twice the tensors' bytes, pre-filled: the Reloads of the first round land in blocks nobody reads
    # any more (the untouched half), so a piece that was not copied would show as the fill pattern
    arena = torch.full((2 * sum(sizes) + (1 << 20),), 0xA5, dtype=torch.uint8, device="cuda:0")
    d = dl.Delta(arena, torch.cuda.current_stream().cuda_stream)
    d.bind(sizes)
    base = d.arena.data_ptr()
    gen = torch.Generator(device="cuda:0")
    gen.manual_seed(77)
    want = []
    for t, n in enumerate(sizes):
        ptr = d.alloc(t)
        v = torch.randint(0, 256, (n,), dtype=torch.uint8, device="cuda:0", generator=gen)
        d.arena[ptr - base:ptr - base + n].copy_(v)
        want.append(v.cpu())
    torch.cuda.synchronize()

    def check():
        for t, n in enumerate(sizes):
            ptr = d.tensor_ptr(t)
            assert torch.equal(d.arena[ptr - base:ptr - base + n].cpu(), want[t]), t

    for rnd in range(2):
        for t in range(len(sizes)):
            d.release(t, dl.EV_OFFLOAD)
        if rnd == 1:
            d.sync()                                          # the Offloads are complete: no pieces to follow
            d.arena.fill_(0x5A)                               # nothing resident, no copy in flight: wipe the device side
            torch.cuda.synchronize()
        for t in range(len(sizes)):
            d.prefetch(t)
        d.sync()
        check()
    st = d.stats()
    # the second round's Offloads are free: the host copies are still valid
    assert st["d2h_bytes"] == sum(sizes) and st["h2d_bytes"] == 2 * sum(sizes)
    assert st["d2h_copies"] == len(sizes) and st["h2d_copies"] == 2 * len(sizes)
    d.close()


def test_replay_with_prefetch_for_recomputations_hands_every_step_its_forward_bits(torch_mod):
    """prefetch_rebuild_reads: a plan in which the Prefetcher brings a tensor back for a recomputation (ahead of
    the step that reads the recomputed tensor, and possibly after the tensor's own last read) replays with the bits
    of the unconstrained forward at every backward step.  The plan is the first, over filters, links and budgets,
    that the switch changes; it equals the oracle's."""
    import paper_2203_15980_amd as dl
    from paper_2203_15980_amd.harness import Net, run_plan
    torch = torch_mod
    layers = synth.bottleneck_stack(4, 56, 56)
    g = synth.fused_graph(layers, "bf16")
    d0 = make_delta(torch, g.total_bytes() + (1 << 20))
    d0.bind([t["bytes"] for t in g.tensors])
    net0 = Net(d0, layers, "bf16", 21)
    net0.forward()
    want = {t["name"]: net0.read(t["name"]).copy() for t in g.tensors}
    d0.close()
    found = None
    for frac in (0.5, 0.6, 0.7, 0.45):
        for kind in (dl.FILTER_BASE, dl.FILTER_LRU, dl.FILTER_GREEDY):
            for bw in (2 * 10**9, 20 * 10**9, 10**12):
                p = opl.default_params(int(g.total_bytes() * frac), g.n_fwd, filter=kind, bw_d2h_Bps=bw, bw_h2d_Bps=bw,
                                       prefetch_distance=2, max_reloads=2, release_when_short=1, repair_rounds=4,
                                       prefetch_rebuild_reads=1)
                try:
                    ev, peak = dl.plan(g.tensors, g.steps, p)
                    ev0, _ = dl.plan(g.tensors, g.steps, dict(p, prefetch_rebuild_reads=0))
                except dl.DeltaError as e:
                    assert e.status == dl.ERR_INFEASIBLE
                    continue
                if ev != ev0 and found is None:
                    assert (ev, peak) == opl.plan(g.tensors, g.steps, p)
                    found = (ev, p)
    assert found is not None, "the switch changed no plan of this graph"
    ev, p = found
    pre = [(k, g.tensors[t]["name"]) for (k, a, t) in ev if a == dl.EV_RELOAD_PREFETCH]
    print("budget", p["budget_bytes"], "filter", p["filter"], "link", p["bw_d2h_Bps"], "prefetches", pre, flush=True)
    d = make_delta(torch, p["budget_bytes"] * 3 // 2)
    d.bind([t["bytes"] for t in g.tensors])
    net = Net(d, layers, "bf16", 21)
    checked = []

    def proxy(k):
        for t in g.steps[k]["reads"]:
            n = g.tensors[t]["name"]
            assert net.read(n).tobytes() == want[n].tobytes(), (k, n)
            checked.append(n)

    run_plan(net, g, ev, backward_proxy=proxy)
    d.sync()
    st = d.stats()
    assert checked and st["arena_in_use"] == 0
    assert st["arena_high_water"] <= p["budget_bytes"]
    d.close()


@pytest.mark.parametrize("dtype,N,HW", [("f32", 2, 32), ("bf16", 4, 56)])
def test_plan_replay_hands_every_step_its_forward_bits(torch_mod, dtype, N, HW):
    """Plan with delta_plan at a 50 % budget, replay it in an arena of exactly that size, and
    at every backward step compare each operand with the value of the unconstrained forward."""
    import paper_2203_15980_amd as dl
    from paper_2203_15980_amd.harness import Net, run_plan
    torch = torch_mod
    layers = synth.bottleneck_stack(N, HW, HW)
    g = synth.fused_graph(layers, dtype)
    # reference forward, nothing released
    d0 = make_delta(torch, g.total_bytes() + (1 << 20))
    d0.bind([t["bytes"] for t in g.tensors])
    net0 = Net(d0, layers, dtype, 21)
    net0.forward()
    want = {t["name"]: net0.read(t["name"]).copy() for t in g.tensors}
    d0.close()
    budget = g.total_bytes() // 2
    found = None
    for kind in (dl.FILTER_BASE, dl.FILTER_LRU, dl.FILTER_GREEDY):
        for bw in (50 * 10**9, 10**12, 0):
            p = opl.default_params(budget, g.n_fwd, filter=kind, bw_d2h_Bps=bw, bw_h2d_Bps=bw)
            try:
                ev, peak = dl.plan(g.tensors, g.steps, p)
            except dl.DeltaError as e:
                assert e.status == dl.ERR_INFEASIBLE
                continue
            assert (ev, peak) == opl.plan(g.tensors, g.steps, p)
            acts = {a for (_, a, _) in ev}
            if found is None or len(acts) > len(found[2]):
                found = (ev, peak, acts, p)
    assert found is not None, "no feasible plan at 50 %"
    ev, peak, acts, p = found
    print("plan actions:", sorted(acts), "peak", peak, "budget", budget, flush=True)
    # the arena gets slack for fragmentation; the budget is checked on bytes in use
    d = make_delta(torch, budget * 3 // 2)
    d.bind([t["bytes"] for t in g.tensors])
    net = Net(d, layers, dtype, 21)
    checked = []

    def proxy(k):
        for t in g.steps[k]["reads"]:
            n = g.tensors[t]["name"]
            assert net.read(n).tobytes() == want[n].tobytes(), (k, n)
            checked.append(n)

    run_plan(net, g, ev, backward_proxy=proxy)
    d.sync()
    st = d.stats()
    assert checked and st["arena_in_use"] == 0
    assert st["arena_high_water"] <= budget
    d.close()


def test_error_paths(torch_mod):
    import paper_2203_15980_amd as dl
    d, net, layers, g = _stack(torch_mod, 1, 8, "bf16", 3)
    with pytest.raises(dl.DeltaError) as e:
        net.recompute("b1.a1")                               # x0 not resident yet
    assert e.value.status == dl.ERR_STATE
    net.load_input()
    with pytest.raises(dl.DeltaError) as e:
        d.prefetch(net.ids["b1.a1"])                         # never offloaded
    assert e.value.status == dl.ERR_STATE
    with pytest.raises(dl.DeltaError) as e:
        d.release(net.ids["b1.a1"], dl.EV_EVICT)             # not resident
    assert e.value.status == dl.ERR_STATE
    with pytest.raises(dl.DeltaError) as e:
        d.release(0, dl.EV_RECOMPUTE)                        # not a release action
    assert e.value.status == dl.ERR_INVALID
    with pytest.raises(dl.DeltaError) as e:
        d.tensor_ptr(10**6)
    assert e.value.status == dl.ERR_INVALID
    bad = dl.LayerDesc.from_buffer_copy(net.desc["b1.a1"][0])
    bad.Cin = 48                                             # not a multiple of 64
    with pytest.raises(dl.DeltaError) as e:
        d.recompute_segment([bad])
    assert e.value.status == dl.ERR_INVALID
    wide = dl.LayerDesc.from_buffer_copy(net.desc["b1.a1"][0])
    wide.pad = 1                                             # 1x1 window with padding 1: rejected
    with pytest.raises(dl.DeltaError) as e:
        d.recompute_segment([wide])
    assert e.value.status == dl.ERR_INVALID
    # the kernel a layer dispatches to, by name
    assert "conv1x1_stream" in d.layer_kernel(net.desc["b1.a1"][0])
    assert "conv3x3_c64" in d.layer_kernel(net.desc["b1.a2"][0])           # 64 -> 64 channels: the weights stay in LDS
    d.close()
    # arena too small for the second tensor
    small = make_delta(torch_mod, 4096)
    small.bind([4096, 4096])
    small.alloc(0)
    with pytest.raises(dl.DeltaError) as e:
        small.alloc(1)
    assert e.value.status == dl.ERR_OOM_ARENA
    small.close()


def test_probes_report_plausible_rooflines(torch_mod):
    d = make_delta(torch_mod, 1 << 20)
    d2h = d.probe_hostlink(64 << 20, 5, 0)
    h2d = d.probe_hostlink(64 << 20, 5, 1)
    hbm = d.probe_hbm(256 << 20, 5)
    mfma = d.probe_mfma(2000)
    print("probes: d2h %.1f GB/s, h2d %.1f GB/s, hbm %.0f GB/s, mfma %.0f TFLOP/s" % (d2h, h2d, hbm, mfma), flush=True)
    assert 1 < d2h < 200 and 1 < h2d < 200 and 500 < hbm < 10000 and 100 < mfma < 3000
    d.close()


def test_degenerate_inputs(torch_mod):
    """Empty segments are no-ops; a one-pixel image and a one-row tensor go through every operator
    family without touching memory outside their tensors (checked by guard bytes around them)."""
    import paper_2203_15980_amd as dl
    from oracle import opgranular as og
    from oracle import transformer as ot
    torch = torch_mod
    d = make_delta(torch, 1 << 20)
    # guard tensors 0, 2, 4, 6, 8 of 256 bytes around the working tensors
    C = 64
    row = C * 2
    d.bind([256, row, 256, row, 256, 3 * row, 256, row, 256])
    d.recompute_segment([])                                  # nothing to do
    d.backward_segment([])
    base = d.arena.data_ptr()
    for t in range(9):
        ptr = d.alloc(t)
        n = [256, row, 256, row, 256, 3 * row, 256, row, 256][t]
        d.arena[ptr - base:ptr - base + n] = 0xA5 if t % 2 == 0 else 0
    x = synth.f32_to_bf16_bits(synth.normal(7, 1, C).astype(np.float32))
    ptr = d.tensor_ptr(1)
    d.arena[ptr - base:ptr - base + row].copy_(torch.from_numpy(x.view(np.uint8)).to("cuda:0"))
    g = torch.ones(C, dtype=torch.float32, device="cuda:0")
    z = torch.zeros(C, dtype=torch.float32, device="cuda:0")
    w = synth.f32_to_bf16_bits((synth.normal(7, 2, C * C) / 8).astype(np.float32)).reshape(C, C)
    wd = torch.from_numpy(w.view(np.uint8).reshape(-1)).to("cuda:0")
    geo = dict(dtype=dl.DTYPE_BF16, N=1, H=1, W=1, Cin=C, Cout=C, R=1, S=1, stride=1, pad=0)
    d.recompute_segment([
        dl.LayerDesc(x=1, res=dl.NO_TENSOR, y=3, w=wd.data_ptr(), scale=g.data_ptr(), shift=z.data_ptr(), relu=1,
                     op=dl.OP_CONV, **geo),                                          # one pixel through the 1x1 kernel
        dl.LayerDesc(x=1, res=dl.NO_TENSOR, y=7, w=None, scale=g.data_ptr(), shift=z.data_ptr(), relu=0,
                     op=dl.OP_LAYERNORM, eps=1e-5, **geo)])                          # one row
    d.sync()

    def get(t, n):
        p = d.tensor_ptr(t)
        return d.arena[p - base:p - base + n].cpu().numpy()

    y = get(3, row).view(np.uint16)
    ref = ot.linear(x.reshape(1, C), w, z.cpu().numpy(), act="relu", dtype="bf16")[0]
    assert np.max(np.abs(ot.to_f64(y, "bf16") - ot.to_f64(ref, "bf16"))) <= 2e-2 * max(1e-6, np.max(np.abs(ot.to_f64(ref, "bf16"))))
    ln = get(7, row).view(np.uint16)
    ref_ln = ot.layernorm(x.reshape(1, C), np.ones(C, np.float32), np.zeros(C, np.float32), 1e-5, "bf16")[0]
    assert np.max(np.abs(ot.to_f64(ln, "bf16") - ot.to_f64(ref_ln, "bf16"))) <= 2e-2
    # batch normalisation over a single position: variance 0, the output is beta (= 0)
    d.recompute_segment([dl.LayerDesc(x=1, res=dl.NO_TENSOR, y=3, w=None, scale=g.data_ptr(), shift=z.data_ptr(), relu=0,
                                      op=dl.OP_BATCHNORM, eps=1e-5, **geo)])
    d.sync()
    assert np.array_equal(ot.to_f64(get(3, row).view(np.uint16), "bf16"), np.zeros(C))
    # attention over a single position: the softmax of one score is 1, ctx = v
    qkv = synth.f32_to_bf16_bits(synth.normal(7, 3, 3 * C).astype(np.float32))
    p5 = d.tensor_ptr(5)
    d.arena[p5 - base:p5 - base + 3 * row].copy_(torch.from_numpy(qkv.view(np.uint8)).to("cuda:0"))
    d.recompute_segment([dl.LayerDesc(x=5, res=dl.NO_TENSOR, y=3, dtype=dl.DTYPE_BF16, w=None, scale=None, shift=None, N=1, H=1,
                                      W=1, Cin=3 * C, Cout=C, R=1, S=1, stride=1, pad=0, relu=0, op=dl.OP_ATTENTION)])
    d.sync()
    assert np.array_equal(get(3, row).view(np.uint16), qkv[2 * C:])
    for t in (0, 2, 4, 6, 8):                                # nothing wrote outside its tensor
        assert (get(t, 256) == 0xA5).all(), t
    d.close()


def _random_layer_cases(seed, count):
    """Seeded random layer shapes the library takes: 1x1 and 3x3, stride 1 and 2, channel counts from 64 to 1024
    (192 and 320 among them), up to 4 images of up to 40 x 40, with and without residual and ReLU; small enough for
    the oracle (at most 1.5e9 multiply-adds each)."""
    import random
    rnd = random.Random(seed)
    chs = [64, 128, 192, 256, 320, 512, 1024]
    cases = []
    while len(cases) < count:
        R = rnd.choice([1, 1, 3]); stride = rnd.choice([1, 1, 2]); pad = (R - 1) // 2
        Cin, Cout = rnd.choice(chs), rnd.choice(chs)
        N, H, W = rnd.randint(1, 4), rnd.randint(1, 40), rnd.randint(1, 40)
        P, Q = (H + 2 * pad - R) // stride + 1, (W + 2 * pad - R) // stride + 1
        if P < 1 or Q < 1 or N * P * Q * Cin * Cout * R * R > 1.5e9:
            continue
        cases.append(("rnd%d" % len(cases), N, H, W, Cin, Cout, R, stride, pad, rnd.random() < 0.6, rnd.random() < 0.4))
    return cases


@pytest.mark.parametrize("case", _random_layer_cases(11, 16), ids=lambda c: "%s_%dx%dx%d_%d_%d_r%d_s%d" % (c[0], c[1], c[2], c[3], c[4], c[5], c[6], c[7]))
def test_random_layer_shapes_match_oracle(torch_mod, case):
    """The single-layer comparison on seeded random shapes: whatever kernel the dispatch picks for them (streaming,
    GEMM tiles with two to four slice buffers, halo, tiled), ragged tiles and odd image sizes included."""
    test_single_layer_matches_oracle(torch_mod, "bf16", case)
