"""GPU parity of the block kernel (one bottleneck 1x1 -> 3x3 -> 1x1 + shortcut in a single launch, selected
with DELTA_FUSE_BLOCK: the identity blocks, and the stage's first block with its projection shortcut) against
the CPU oracle's layer chain, through the C ABI.

Bars: every stored tensor within 2e-2 (bf16) of the oracle's; whatever subset of {a1, a2, out} a
launch stores, the stored tensors carry the same bits; a recomputation after a release (at
another arena address) reproduces the forward bit for bit."""
import itertools

import numpy as np
import pytest

import synth
from oracle import numeric as on

pytestmark = pytest.mark.gpu

NAMES = ("blk.a1", "blk.a2", "blk.out")


@pytest.fixture(scope="module")
def torch_mod():
    import torch
    assert torch.cuda.is_available()
    return torch


def _net(torch, N, H, W, master=61, extra=4):
    import paper_2203_15980_amd as dl
    from paper_2203_15980_amd.harness import Net
    layers = synth.identity_block(N, H, W)
    g = synth.fused_graph(layers, "bf16")
    arena = torch.empty(extra * g.total_bytes() + (1 << 20), dtype=torch.uint8, device="cuda:0")
    d = dl.Delta(arena, torch.cuda.current_stream().cuda_stream)
    d.bind([t["bytes"] for t in g.tensors])
    return d, Net(d, layers, "bf16", master), layers


def _rel(got, ref):
    g, r = on.to_f64(got, "bf16"), on.to_f64(ref, "bf16")
    return float(np.max(np.abs(g - r)) / max(np.max(np.abs(r)), 1e-30))


def test_block_kernel_carries_the_bits_of_the_per_layer_kernels(torch_mod):
    """The same three tensors from three per-layer launches and from one block launch: equal bit for bit
    (every reduction runs in the same order), so a plan may mix the two."""
    torch = torch_mod
    import paper_2203_15980_amd as dl
    for shape in [(2, 7, 7), (3, 9, 11), (8, 56, 56), (1, 4, 224), (2, 15, 29)]:
        print("shape", shape, flush=True)
        d, net, layers = _net(torch, *shape)
        net.load_input()
        d.recompute_segment(net.all_layers)
        d.sync()
        per_layer = {n: net.read(n).copy() for n in NAMES}
        for n in NAMES:
            d.release(net.ids[n], dl.EV_EVICT)
        d.recompute_segment(net.block_desc("blk"))
        d.sync()
        for n in NAMES:
            assert np.array_equal(net.read(n), per_layer[n]), (shape, n)
        d.close()


SHAPES = [(2, 7, 7), (1, 14, 14), (3, 9, 11), (1, 1, 1), (2, 3, 100), (1, 5, 223), (5, 56, 56), (2, 15, 29), (1, 28, 28)]


@pytest.mark.parametrize("shape", SHAPES, ids=lambda s: "x".join(map(str, s)))
def test_block_kernel_matches_the_oracle_chain(torch_mod, shape):
    torch = torch_mod
    import paper_2203_15980_amd as dl
    print("shape", shape, flush=True)
    d, net, layers = _net(torch, *shape)
    net.load_input()
    ref = on.run_layers(layers, net.params_np, net.x0_np, "bf16")
    d.recompute_segment(net.block_desc("blk"))
    d.sync()
    first = {n: net.read(n).copy() for n in NAMES}
    for n in NAMES:
        err = _rel(first[n], ref[n])
        print("  %s err %.2e" % (n, err), flush=True)
        assert err <= 2e-2, (shape, n, err)
    # every subset of stored outputs: same bits; what is not stored is not allocated
    for k in (1, 2):
        for keep in itertools.combinations(NAMES, k):
            for n in NAMES:
                d.release(net.ids[n], dl.EV_EVICT)
            filler = d.alloc(net.ids["blk.a1"]) if "blk.a1" not in keep else None     # shifts the addresses
            if filler is not None:
                d.release(net.ids["blk.a1"], dl.EV_FREE)
            d.recompute_segment(net.block_desc("blk", store=keep))
            d.sync()
            for n in NAMES:
                if n in keep:
                    assert np.array_equal(net.read(n), first[n]), (shape, keep, n)
                else:
                    with pytest.raises(dl.DeltaError) as e:
                        d.tensor_ptr(net.ids[n])
                    assert e.value.status == dl.ERR_STATE
            for n in keep:
                d.release(net.ids[n], dl.EV_EVICT)
            d.recompute_segment(net.block_desc("blk"))                               # all three back for the next round
    d.sync()
    st = d.stats()
    assert st["recompute_launches"] == 1 + 2 * 6
    d.close()


PROJ_NAMES = ("b1.a1", "b1.a2", "b1.sc", "b1.out")


def _proj_net(torch, N, H, W, master=61, extra=4):
    """The first block of a stage: 64 input channels and a projection shortcut (config 2's block 1)."""
    import paper_2203_15980_amd as dl
    from paper_2203_15980_amd.harness import Net
    layers = synth.bottleneck_stack(N, H, W, nblocks=1)
    g = synth.fused_graph(layers, "bf16")
    arena = torch.empty(extra * g.total_bytes() + (1 << 20), dtype=torch.uint8, device="cuda:0")
    d = dl.Delta(arena, torch.cuda.current_stream().cuda_stream)
    d.bind([t["bytes"] for t in g.tensors])
    net = Net(d, layers, "bf16", master)
    assert net.blocks == {"b1": PROJ_NAMES}
    return d, net, layers


@pytest.mark.parametrize("shape", [(2, 7, 7), (3, 9, 11), (1, 1, 1), (2, 15, 29), (5, 56, 56), (1, 4, 224)],
                         ids=lambda s: "x".join(map(str, s)))
def test_projection_block_carries_the_per_layer_bits_and_matches_the_oracle(torch_mod, shape):
    """The block with a projection shortcut (1x1 64 -> 64, 3x3, the projection 1x1 64 -> 256 of the block's input, 1x1
    64 -> 256 + the projection) in one launch: within 2e-2 of the oracle's chain, and every subset of its four
    tensors carries the bits of the four per-layer launches; what is not stored is not allocated."""
    torch = torch_mod
    import paper_2203_15980_amd as dl
    print("shape", shape, flush=True)
    d, net, layers = _proj_net(torch, *shape)
    net.load_input()
    d.recompute_segment(net.all_layers)
    d.sync()
    per_layer = {n: net.read(n).copy() for n in PROJ_NAMES}
    ref = on.run_layers(layers, net.params_np, net.x0_np, "bf16")
    for n in PROJ_NAMES:
        err = _rel(per_layer[n], ref[n])
        print("  %s err %.2e" % (n, err), flush=True)
        assert err <= 2e-2, (shape, n, err)
    launches = 0
    for k in (1, 2, 3, 4):
        for keep in itertools.combinations(PROJ_NAMES, k):
            for n in PROJ_NAMES:
                d.release(net.ids[n], dl.EV_EVICT)
            d.stats_reset()
            d.recompute_segment(net.block_desc("b1", store=keep))
            d.sync()
            launches += d.stats()["recompute_launches"]
            for n in PROJ_NAMES:
                if n in keep:
                    assert np.array_equal(net.read(n), per_layer[n]), (shape, keep, n)
                else:
                    with pytest.raises(dl.DeltaError) as e:
                        d.tensor_ptr(net.ids[n])
                    assert e.value.status == dl.ERR_STATE
            for n in keep:
                d.release(net.ids[n], dl.EV_EVICT)
            d.recompute_segment(net.all_layers)                                     # all four back for the next round
    assert launches == 15
    d.close()


def test_projection_block_at_config2_size_on_sampled_images(torch_mod):
    """Config 2's block 1 at its launch shape (batch 32, 56 x 56); the oracle computes the first and the last image."""
    torch = torch_mod
    d, net, layers = _proj_net(torch, 32, 56, 56, extra=2)
    net.load_input()
    d.recompute_segment(net.block_desc("b1"))
    d.sync()
    for img in (0, 31):
        sub = synth.bottleneck_stack(1, 56, 56, nblocks=1)
        ref = on.run_layers(sub, net.params_np, net.x0_np[img:img + 1], "bf16")
        for n in PROJ_NAMES:
            err = _rel(net.read(n)[img:img + 1], ref[n])
            print("image %d %s err %.2e" % (img, n, err), flush=True)
            assert err <= 2e-2, (img, n, err)
    d.close()


def test_projection_block_refuses_a_broken_chain(torch_mod):
    torch = torch_mod
    import paper_2203_15980_amd as dl
    d, net, layers = _proj_net(torch, 2, 6, 6)
    net.load_input()
    arr = net.block_desc("b1")
    arr[3].res = dl.NO_TENSOR                                  # the last layer must add the projection
    with pytest.raises(dl.DeltaError) as e:
        d.recompute_segment(arr)
    assert e.value.status == dl.ERR_INVALID
    arr = net.block_desc("b1")
    arr[2].relu = 1                                            # the projection has no ReLU
    with pytest.raises(dl.DeltaError) as e:
        d.recompute_segment(arr)
    assert e.value.status == dl.ERR_INVALID
    arr = net.block_desc("b1")
    arr[2].x = arr[1].y                                        # ... and reads the block's input
    with pytest.raises(dl.DeltaError) as e:
        d.recompute_segment(arr)
    assert e.value.status == dl.ERR_INVALID
    with pytest.raises(dl.DeltaError) as e:                   # a block cut short
        d.recompute_segment(net.block_desc("b1"), 3)
    assert e.value.status == dl.ERR_INVALID
    with pytest.raises(dl.DeltaError) as e:
        d.recompute_segment(net.block_desc("b1", store=()))
    assert e.value.status == dl.ERR_INVALID
    d.recompute_segment(net.block_desc("b1"))                  # and the intact chain runs
    d.sync()
    d.close()


def test_step_replay_runs_a_projection_block_as_one_launch(torch_mod):
    """`run_plan` on config 2's stack (block 1 with a projection, blocks 2 and 3 identity): without plan events the
    forward is three launches; RECOMPUTE events for a1, a2, sc, out of block 1 in a row are one launch; the bits are
    those of the per-layer launches."""
    torch = torch_mod
    import paper_2203_15980_amd as dl
    from paper_2203_15980_amd.harness import Net, run_plan
    layers = synth.bottleneck_stack(2, 20, 17)
    g = synth.fused_graph(layers, "bf16")
    arena = torch.empty(4 * g.total_bytes() + (1 << 20), dtype=torch.uint8, device="cuda:0")
    d = dl.Delta(arena, torch.cuda.current_stream().cuda_stream)
    d.bind([t["bytes"] for t in g.tensors])
    net = Net(d, layers, "bf16", 61)
    assert set(net.blocks) == {"b1", "b2", "b3"} and len(net.blocks["b1"]) == 4
    names = [t["name"] for t in g.tensors]
    net.load_input()
    d.recompute_segment(net.all_layers)
    d.sync()
    ref = {n: net.read(n).copy() for n in names if n != "x0"}
    for t in range(len(names)):
        d.release(t, dl.EV_FREE)
    d.stats_reset()
    run_plan(net, g, [])
    d.sync()
    assert d.stats()["recompute_launches"] == 3
    for n in ref:
        assert np.array_equal(net.read(n), ref[n]), n
    for t in range(len(names)):
        d.release(t, dl.EV_FREE)
    ids = [net.ids[n] for n in net.blocks["b1"]]
    k_bwd = g.n_fwd
    events = [(k_bwd, dl.EV_EVICT, t) for t in ids] + [(k_bwd, dl.EV_RECOMPUTE, t) for t in ids]
    d.stats_reset()
    run_plan(net, g, events)
    d.sync()
    assert d.stats()["recompute_launches"] == 3 + 1
    for n in ref:
        assert np.array_equal(net.read(n), ref[n]), n
    d.close()


def test_block_kernel_at_config2_size_on_sampled_images(torch_mod):
    """The launch shape bench.py times (batch 32, 56 x 56: one workgroup of 392 pixels per CU);
    the oracle computes the first and the last image (frozen statistics: images are independent)."""
    torch = torch_mod
    d, net, layers = _net(torch, 32, 56, 56, extra=2)
    net.load_input()
    d.recompute_segment(net.block_desc("blk"))
    d.sync()
    for img in (0, 31):
        sub = synth.identity_block(1, 56, 56)
        ref = on.run_layers(sub, net.params_np, net.x0_np[img:img + 1], "bf16")
        for n in NAMES:
            err = _rel(net.read(n)[img:img + 1], ref[n])
            print("image %d %s err %.2e" % (img, n, err), flush=True)
            assert err <= 2e-2, (img, n, err)
    d.close()


def test_block_kernel_refuses_what_it_does_not_take(torch_mod):
    torch = torch_mod
    import paper_2203_15980_amd as dl
    d, net, layers = _net(torch, 2, 6, 6)
    net.load_input()
    with pytest.raises(dl.DeltaError) as e:
        d.recompute_segment(net.block_desc("blk", store=()))
    assert e.value.status == dl.ERR_INVALID
    arr = net.block_desc("blk")
    arr[2].res = dl.NO_TENSOR                                  # the shortcut is part of the block
    with pytest.raises(dl.DeltaError) as e:
        d.recompute_segment(arr)
    assert e.value.status == dl.ERR_INVALID
    arr = net.block_desc("blk")
    with pytest.raises(dl.DeltaError) as e:                   # a block cut short
        d.recompute_segment(arr, 2)
    assert e.value.status == dl.ERR_INVALID
    lone = dl.layer_array([dl.LayerDesc.from_buffer_copy(net.desc["blk.a1"][0])])
    lone[0].fuse = dl.FUSE_NO_STORE                            # the flag means nothing outside a block
    with pytest.raises(dl.DeltaError) as e:
        d.recompute_segment(lone)
    assert e.value.status == dl.ERR_INVALID
    net.delta.release(0, dl.EV_FREE)
    with pytest.raises(dl.DeltaError) as e:                   # the block's input must be resident
        d.recompute_segment(net.block_desc("blk"))
    assert e.value.status == dl.ERR_STATE
    d.close()


def test_step_replay_runs_adjacent_block_layers_as_one_launch(torch_mod):
    """`run_plan` on a graph with an identity bottleneck: three forward steps with no plan event between
    them, and RECOMPUTE events for a1 and a2 in a row, each become one launch of the block kernel; a plan
    event in between keeps the per-layer launches.  Every tensor carries the same bits either way."""
    torch = torch_mod
    import paper_2203_15980_amd as dl
    from paper_2203_15980_amd.harness import run_plan
    d, net, layers = _net(torch, 3, 20, 17)
    g = synth.fused_graph(layers, "bf16")
    ids = [net.ids[n] for n in NAMES]
    assert net.blocks == {"blk": NAMES}

    def launches():
        return d.stats()["recompute_launches"]

    # per-layer reference bits
    net.load_input()
    d.recompute_segment(net.all_layers)
    d.sync()
    ref = {n: net.read(n).copy() for n in NAMES}
    for t in [0] + ids:
        d.release(t, dl.EV_FREE)

    # (a) no events: the forward's three steps fuse
    d.stats_reset()
    run_plan(net, g, [])
    d.sync()
    fused_launches = launches()
    for n in NAMES:
        assert np.array_equal(net.read(n), ref[n]), n
    for t in [0] + ids:
        d.release(t, dl.EV_FREE)

    # (b) an event before the second layer: per-layer launches; later a1 and a2 are evicted and regenerated in a row
    k_a2 = [k for k, st in enumerate(g.steps) if st["produces"] == ids[1]][0]
    k_bwd = g.n_fwd                                  # the first backward step
    events = [(k_a2, dl.EV_EVICT, ids[0]), (k_a2, dl.EV_RECOMPUTE, ids[0]),
              (k_bwd, dl.EV_EVICT, ids[0]), (k_bwd, dl.EV_EVICT, ids[1]),
              (k_bwd, dl.EV_RECOMPUTE, ids[0]), (k_bwd, dl.EV_RECOMPUTE, ids[1])]
    d.stats_reset()
    run_plan(net, g, events)
    d.sync()
    for n in NAMES:
        assert np.array_equal(net.read(n), ref[n]), n
    # forward: 3 per-layer launches + 1 recomputation of a1; backward step: one block launch for a1 + a2
    assert launches() - fused_launches == 4, (launches(), fused_launches)
    d.close()


@pytest.mark.parametrize("frac", [0.5, 0.4])
def test_single_pass_plan_with_blocks_rebuilt_from_their_input_replays_with_forward_bits(torch_mod, frac):
    """Config 2's stack planned on the graph in which the block kernel is the recompute route (`block_rebuild`): the
    single greedy pass (no repair rounds) plans it at 50 % and 40 %, where the per-layer graph is infeasible; the
    replay keeps the bytes in use within the budget, every RECOMPUTE of .a2 / .out is one block-kernel launch that stores only
    that tensor (its block-mates stay released), and every backward step finds the bits of the unconstrained forward."""
    torch = torch_mod
    import paper_2203_15980_amd as dl
    from oracle import planner as opl
    from paper_2203_15980_amd.harness import Net, run_plan, block_rebuild
    layers = synth.bottleneck_stack(4, 56, 56)
    g0 = synth.fused_graph(layers, "bf16")
    g = synth.fused_graph(layers, "bf16", rebuild=block_rebuild(layers))
    total = g.total_bytes()
    arena = torch.empty(total + (1 << 20), dtype=torch.uint8, device="cuda:0")
    d0 = dl.Delta(arena, torch.cuda.current_stream().cuda_stream)
    d0.bind([t["bytes"] for t in g.tensors])
    net0 = Net(d0, layers, "bf16", 23)
    net0.forward()
    want = {t["name"]: net0.read(t["name"]).copy() for t in g.tensors}
    d0.close()
    del net0, d0, arena
    p = opl.default_params(int(total * frac), g.n_fwd, bw_d2h_Bps=48 * 10**9, bw_h2d_Bps=52 * 10**9,
                           prefetch_distance=2, max_reloads=2, release_when_short=1)
    with pytest.raises(dl.DeltaError) as e:
        dl.plan(g0.tensors, g0.steps, p)
    assert e.value.status == dl.ERR_INFEASIBLE
    ev, peak = dl.plan(g.tensors, g.steps, p)
    assert (ev, peak) == opl.plan(g.tensors, g.steps, p)
    rebuilt = [g.tensors[t]["name"] for (_, a, t) in ev if a == dl.EV_RECOMPUTE]
    print("frac", frac, "events", len(ev), "recomputed", rebuilt, flush=True)
    assert any(n.endswith((".a2", ".out")) for n in rebuilt)
    arena = torch.empty(p["budget_bytes"] * 3 // 2, dtype=torch.uint8, device="cuda:0")   # room for placement; the bytes in use are checked below
    d = dl.Delta(arena, torch.cuda.current_stream().cuda_stream)
    d.bind([t["bytes"] for t in g.tensors])
    net = Net(d, layers, "bf16", 23)
    net.block_rebuild = True
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


def _random_block_shapes(seed, count):
    import random
    rnd = random.Random(seed)
    return [(i % 2 == 0, rnd.randint(1, 5), rnd.randint(1, 61), rnd.randint(1, 61), rnd.randint(0, 10**6)) for i in range(count)]


@pytest.mark.parametrize("case", _random_block_shapes(7, 12), ids=lambda c: "%s_%dx%dx%d" % ("proj" if c[0] else "ident", c[1], c[2], c[3]))
def test_block_kernels_carry_the_per_layer_bits_on_random_shapes(torch_mod, case):
    """Both forms of the block kernel on seeded random image sizes (tiles cut by every border, single rows and
    columns): one random subset of each size of the block's tensors, bit for bit against the per-layer launches."""
    import random
    torch = torch_mod
    import paper_2203_15980_amd as dl
    from paper_2203_15980_amd.harness import Net
    proj, N, H, W, sub = case
    print("case", case, flush=True)
    rnd = random.Random(sub)
    layers = synth.bottleneck_stack(N, H, W, nblocks=1) if proj else synth.identity_block(N, H, W)
    g = synth.fused_graph(layers, "bf16")
    arena = torch.empty(4 * g.total_bytes() + (1 << 20), dtype=torch.uint8, device="cuda:0")
    d = dl.Delta(arena, torch.cuda.current_stream().cuda_stream)
    d.bind([t["bytes"] for t in g.tensors])
    net = Net(d, layers, "bf16", 100 + sub % 1000)
    (pre, chain), = net.blocks.items()
    net.load_input()
    d.recompute_segment(net.all_layers)
    d.sync()
    ref = {n: net.read(n).copy() for n in chain}
    for k in range(1, len(chain) + 1):
        keep = rnd.sample(chain, k)
        for n in chain:
            d.release(net.ids[n], dl.EV_EVICT)
        d.recompute_segment(net.block_desc(pre, store=keep))
        d.sync()
        for n in keep:
            assert np.array_equal(net.read(n), ref[n]), (case, keep, n)
        for n in keep:
            d.release(net.ids[n], dl.EV_EVICT)
        d.recompute_segment(net.all_layers)
    d.close()
