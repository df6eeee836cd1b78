"""GPU parity of the transformer-layer operators (through the C ABI) against the float64 oracle.

Tolerance: every stored tensor is bf16 (relative rounding 2^-9); the linear layers and the layer
normalisation round once from fp32, the attention kernel additionally rounds the probabilities to
bf16 before they multiply v: 2e-2 of the tensor's maximum, the bar of the convolution layers."""
import numpy as np
import pytest

import synth
from oracle import transformer as ot

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


def _bits(master, aid, shape, scale=1.0):
    return synth.f32_to_bf16_bits((synth.normal(master, aid, int(np.prod(shape))) * scale).astype(np.float32)).reshape(shape)


def _relerr(got, ref):
    return float(np.max(np.abs(got - ref)) / np.max(np.abs(ref)))


ATT = [
    # name            N    S  heads scale
    ("tiny",          3,   33, 2, 1.0),     # one ragged chunk
    ("ragged150",     2,  150, 3, 1.0),     # two chunks, the second ragged; one query block, partly empty
    ("peaked",        1,  256, 2, 2.5),     # scores with a spread of ~6: the running maximum moves
    ("full512",       1,  512, 2, 1.0),     # config 5's sequence length: two query blocks, K/V fill the LDS
    ("two_kblocks",   1,  700, 1, 1.0),     # more keys than fit at once: second key block, ragged
]


@pytest.mark.parametrize("case", ATT, ids=[c[0] for c in ATT])
def test_attention_matches_oracle(torch_mod, case):
    torch = torch_mod
    import paper_2203_15980_amd as dl
    name, N, S, heads, scale = case
    print("case", name, flush=True)
    H = heads * 64
    qkv = _bits(61, 1, (N, S, 3 * H), scale)
    d, put, get = _ctx(torch, [qkv.nbytes, N * S * H * 2], 32)
    put(0, qkv)
    desc = dl.LayerDesc(x=0, res=dl.NO_TENSOR, y=1, dtype=dl.DTYPE_BF16, w=None, scale=None, shift=None,
                        N=N, H=S, W=1, Cin=3 * H, Cout=H, R=heads, S=1, stride=1, pad=0, relu=0, op=dl.OP_ATTENTION)
    assert "attention" in d.layer_kernel(desc)
    d.recompute_segment([desc])
    d.sync()
    got = ot.to_f64(get(1, (N, S, H)), "bf16")
    ref = ot.attention_f64(qkv, heads, "bf16")
    err = _relerr(got, ref)
    print("  err %.2e" % err, flush=True)
    assert err <= 2e-2, (name, err)
    # recomputation is bit-identical
    first = get(1, (N, S, H)).copy()
    d.recompute_segment([desc])
    d.sync()
    assert np.array_equal(get(1, (N, S, H)), first)
    d.close()


@pytest.mark.parametrize("rows,C", [(37, 768), (5, 2048), (130, 64), (9, 8)])
def test_layernorm_matches_oracle(torch_mod, rows, C):
    torch = torch_mod
    import paper_2203_15980_amd as dl
    print("rows", rows, "C", C, flush=True)
    x = _bits(62, 1, (rows, C), 3.0)
    x = synth.f32_to_bf16_bits((synth.bf16_bits_to_f32(x) + 1.5).astype(np.float32)).reshape(rows, C)   # a mean to remove
    gamma = synth.uniform(62, 2, C, 0.5, 1.5).astype(np.float32)
    beta = synth.normal(62, 3, C, 0.0, 0.1).astype(np.float32)
    d, put, get = _ctx(torch, [x.nbytes, x.nbytes], 8)
    put(0, x)
    g, b = _dev(torch, gamma), _dev(torch, beta)
    desc = dl.LayerDesc(x=0, res=dl.NO_TENSOR, y=1, dtype=dl.DTYPE_BF16, w=None, scale=g.data_ptr(), shift=b.data_ptr(),
                        N=1, H=rows, W=1, Cin=C, Cout=C, R=1, S=1, stride=1, pad=0, relu=0, op=dl.OP_LAYERNORM, eps=1e-12)
    d.recompute_segment([desc])
    d.sync()
    got = ot.to_f64(get(1, (rows, C)), "bf16")
    ref = ot.to_f64(ot.layernorm(x, gamma, beta, 1e-12, "bf16"), "bf16")
    err = _relerr(got, ref)
    print("  err %.2e" % err, flush=True)
    assert err <= 2e-2 / 4, err                 # one rounding from fp32: well inside the bar
    d.close()


@pytest.mark.parametrize("case", [("gelu", 2, 70, 128, 192, "gelu", False), ("res", 1, 45, 768, 64, None, True),
                                  ("plain", 3, 33, 64, 256, None, False),
                                  # few tiles and a long reduction: the GEMM kernel's 128 x 128 tile with four slice
                                  # buffers (8, 16 and 20 slices; one tile, ragged rows, ragged channels)
                                  ("gemm4_ffn2", 1, 40, 512, 128, None, True),
                                  ("gemm4_ragged", 3, 211, 1024, 200, "gelu", True),
                                  ("gemm4_short_tail", 1, 300, 1280, 136, "relu", False),
                                  # large enough for the 256 x 256-tiled GEMM kernel; ragged rows and channels
                                  ("gemm_gelu", 1, 8465, 256, 1024, "gelu", False),
                                  ("gemm_res_ragged_n", 1, 8300, 768, 776, None, True),
                                  ("gemm_one_column_of_tiles", 1, 32800, 256, 256, "relu", False)],
                         ids=lambda c: c[0])
def test_linear_layers_match_oracle(torch_mod, case):
    torch = torch_mod
    import paper_2203_15980_amd as dl
    name, N, S, Cin, Cout, act, has_res = case
    print("case", name, flush=True)
    M = N * S
    x = _bits(63, 1, (M, Cin))
    w = _bits(63, 2, (Cout, Cin), 1.0 / np.sqrt(Cin) * 1.5)
    bias = synth.normal(63, 3, Cout, 0.0, 0.5).astype(np.float32)
    res = _bits(63, 4, (M, Cout)) if has_res else None
    d, put, get = _ctx(torch, [x.nbytes, M * Cout * 2, M * Cout * 2], 96)
    put(0, x)
    if has_res:
        put(1, res)
    wd, ones, bd = _dev(torch, w), torch.ones(Cout, dtype=torch.float32, device="cuda:0"), _dev(torch, bias)
    desc = dl.LayerDesc(x=0, res=1 if has_res else dl.NO_TENSOR, y=2, dtype=dl.DTYPE_BF16, w=wd.data_ptr(),
                        scale=ones.data_ptr(), shift=bd.data_ptr(), N=N, H=S, W=1, Cin=Cin, Cout=Cout, R=1, S=1,
                        stride=1, pad=0, relu={"gelu": dl.ACT_GELU, "relu": dl.ACT_RELU, None: dl.ACT_NONE}[act], op=dl.OP_CONV)
    assert ("gemm_nt" in d.layer_kernel(desc)) == name.startswith("gemm"), d.layer_kernel(desc)
    d.recompute_segment([desc])
    d.sync()
    got = ot.to_f64(get(2, (M, Cout)), "bf16")
    ref = ot.to_f64(ot.linear(x, w, bias, act=act, res=res, dtype="bf16"), "bf16")
    err = _relerr(got, ref)
    print("  err %.2e" % err, flush=True)
    assert err <= 2e-2 / 4, (name, err)
    if act == "gelu":
        assert (ref < 0).any() and (ref > 1).any()          # both branches of the curve are exercised
    d.close()


def test_transformer_ops_reject_what_they_do_not_support(torch_mod):
    torch = torch_mod
    import paper_2203_15980_amd as dl
    S, H = 40, 128
    d, put, get = _ctx(torch, [S * 3 * H * 2, S * H * 2, S * H * 2, S * 2056 * 2, S * 2056 * 2], 8)
    put(0, _bits(64, 1, (S, 3 * H)))
    ones = torch.ones(4096, dtype=torch.float32, device="cuda:0")
    att = dict(x=0, res=dl.NO_TENSOR, y=1, dtype=dl.DTYPE_BF16, w=None, scale=None, shift=None, N=1, H=S, W=1,
               Cin=3 * H, Cout=H, R=2, S=1, stride=1, pad=0, relu=0, op=dl.OP_ATTENTION)
    for bad in (dict(R=3), dict(Cin=2 * H), dict(dtype=dl.DTYPE_F32), dict(W=2), dict(res=2)):
        with pytest.raises(dl.DeltaError) as e:
            d.recompute_segment([dl.LayerDesc(**{**att, **bad})])
        assert e.value.status in (dl.ERR_INVALID,), bad
    ln = dict(x=3, res=dl.NO_TENSOR, y=4, dtype=dl.DTYPE_BF16, w=None, scale=ones.data_ptr(), shift=ones.data_ptr(),
              N=1, H=S, W=1, Cin=2056, Cout=2056, R=1, S=1, stride=1, pad=0, relu=0, op=dl.OP_LAYERNORM, eps=1e-5)
    put(3, _bits(64, 2, (S, 2056)))
    with pytest.raises(dl.DeltaError):                      # more channels than a wavefront keeps in registers
        d.recompute_segment([dl.LayerDesc(**ln)])
    with pytest.raises(dl.DeltaError):                      # no backward for these operators
        d.backward_segment([dl.BwdDesc(fwd=dl.LayerDesc(**att), gy=1, gpre=1, gx=2, gx_add=dl.NO_TENSOR, wt=None,
                                       gw=None, workspace=None, workspace_bytes=0)])
    with pytest.raises(dl.DeltaError):                      # unknown activation code
        d.recompute_segment([dl.LayerDesc(x=1, res=dl.NO_TENSOR, y=2, dtype=dl.DTYPE_BF16, w=ones.data_ptr(),
                                          scale=ones.data_ptr(), shift=ones.data_ptr(), N=1, H=S, W=1, Cin=H, Cout=H,
                                          R=1, S=1, stride=1, pad=0, relu=3, op=dl.OP_CONV)])
    d.close()


def test_encoder_layers_through_the_harness(torch_mod):
    """Two encoder layers (hidden 128, 2 heads, feed-forward 256) on 2 x 150 tokens.  Layer by
    layer the oracle is given the GPU's own input of that layer; end to end it runs its own chain."""
    torch = torch_mod
    import paper_2203_15980_amd as dl
    from paper_2203_15980_amd.harness import Net
    N, S, H, heads, FF = 2, 150, 128, 2, 256
    layers = synth.encoder_layers(N, S, H, heads, FF, nlayers=2)
    g = synth.fused_graph(layers, "bf16")
    arena = torch.empty(32 << 20, dtype=torch.uint8, device="cuda:0")
    d = dl.Delta(arena, torch.cuda.current_stream().cuda_stream)
    d.bind([t["bytes"] for t in g.tensors])
    net = Net(d, layers, "bf16", 71)
    net.forward()
    d.sync()
    acts = {"x0": net.x0_np.reshape(N * S, H)}
    for l in layers:
        acts[l.y] = net.read(l.y).reshape(N * S, l.Cout)
    for l in layers:
        p = net.params_np.get(l.name)
        x = acts[l.x]
        if l.kind == "linear":
            ref = ot.linear(x, p["w"], p["bias"], act=l.act or None, res=acts[l.res] if l.res else None, dtype="bf16")
        elif l.kind == "attention":
            ref = ot.attention(x.reshape(N, S, 3 * H), heads, "bf16").reshape(N * S, H)
        else:
            ref = ot.layernorm(x, p["gamma"], p["beta"], p["eps"], "bf16")
        err = _relerr(ot.to_f64(acts[l.y], "bf16"), ot.to_f64(ref, "bf16"))
        print("  %-8s %-10s err %.2e" % (l.name, l.kind, err), flush=True)
        assert err <= 2e-2, (l.name, err)
    x = net.x0_np.reshape(N, S, H)
    for i in range(2):
        out = ot.encoder_layer(x, synth.make_encoder_params(71, i, H, FF, "bf16", heads), heads, synth.LN_EPS, "bf16")
        for k, v in out.items():                              # the harness and the oracle drew the same parameters
            err = _relerr(ot.to_f64(acts["l%d.%s" % (i, k)], "bf16"), ot.to_f64(v, "bf16"))
            assert err <= 2e-2, (i, k, err)
        x = out["ln2"].reshape(N, S, H)
    print("  end to end err %.2e" % err, flush=True)
    d.close()


def test_attention_at_config5_size_on_sampled_heads(torch_mod):
    """BERT-base attention at the benchmark's size (batch 32, 512 positions, 12 heads), in the launch
    configuration the bench times; the oracle checks sampled (image, head) pairs."""
    torch = torch_mod
    import paper_2203_15980_amd as dl
    N, S, heads = 32, 512, 12
    H = heads * 64
    # one image's worth of random rows, tiled with a per-image scale: cheap to draw, different per image
    one = synth.normal(65, 1, S * 3 * H).astype(np.float32).reshape(S, 3 * H)
    scales = (0.5 + 0.05 * np.arange(N)).astype(np.float32)
    qkv = synth.f32_to_bf16_bits((one[None] * scales[:, None, None]).astype(np.float32).reshape(-1)).reshape(N, S, 3 * H)
    d, put, get = _ctx(torch, [qkv.nbytes, N * S * H * 2], 160)
    put(0, qkv)
    desc = dl.LayerDesc(x=0, res=dl.NO_TENSOR, y=1, dtype=dl.DTYPE_BF16, w=None, scale=None, shift=None,
                        N=N, H=S, W=1, Cin=3 * H, Cout=H, R=heads, S=1, stride=1, pad=0, relu=0, op=dl.OP_ATTENTION)
    d.recompute_segment([desc])
    d.sync()
    got = get(1, (N, S, H))
    for (n, h) in ((0, 0), (13, 5), (31, 11), (7, 3)):
        sub = np.concatenate([qkv[n:n + 1, :, k * H + h * 64:k * H + (h + 1) * 64] for k in range(3)], axis=2)
        ref = ot.attention_f64(sub, 1, "bf16")[0]
        err = _relerr(ot.to_f64(got[n, :, h * 64:(h + 1) * 64], "bf16"), ref)
        print("  image %d head %d err %.2e" % (n, h, err), flush=True)
        assert err <= 2e-2, (n, h, err)
    d.close()


def test_encoder_plan_replay_restores_every_backward_operand(torch_mod):
    """Plan three small encoder layers at 40 % of their activation bytes (library plan = oracle plan),
    replay it, and compare every tensor a backward step reads with the unconstrained forward's, bit
    for bit: evicted tensors are rebuilt by the attention / linear / LayerNorm kernels, offloaded
    ones come back over the link.  Then the same plan once more with the compute-proxy backward."""
    torch = torch_mod
    import paper_2203_15980_amd as dl
    from oracle import planner as opl
    from paper_2203_15980_amd.harness import Net, run_plan
    N, S, H, heads, FF = 2, 150, 128, 2, 256
    layers = synth.encoder_layers(N, S, H, heads, FF, nlayers=3)
    g = synth.fused_graph(layers, "bf16")
    sizes = [t["bytes"] for t in g.tensors]

    def make(arena_bytes):
        arena = torch.empty(arena_bytes, dtype=torch.uint8, device="cuda:0")
        d = dl.Delta(arena, torch.cuda.current_stream().cuda_stream)
        d.bind(sizes)
        return d, Net(d, layers, "bf16", 73)

    d0, net0 = make(g.total_bytes() + (1 << 20))
    net0.forward()
    want = {t["name"]: net0.read(t["name"]).copy() for t in g.tensors}
    d0.close()
    budget = int(g.total_bytes() * 0.4)
    p = opl.default_params(budget, g.n_fwd, bw_d2h_Bps=50 * 10**9, bw_h2d_Bps=50 * 10**9)
    ev, peak = dl.plan(g.tensors, g.steps, p)
    assert (ev, peak) == opl.plan(g.tensors, g.steps, p)
    d, net = make(int(budget * 1.5) + (1 << 20))
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
    print("events", sorted(kinds), "peak", peak, "budget", budget, "recompute launches", st["recompute_launches"], flush=True)
    assert st["arena_in_use"] == 0 and st["arena_high_water"] <= budget
    assert dl.EV_RECOMPUTE in kinds and any(n.endswith("ctx") for n in seen)
    # the proxy backward: same plan, every backward step runs its operator's forward kernel twice
    net.enable_backward_proxy()
    run_plan(net, g, ev, backward_proxy=lambda k: net.backward_proxy_step(g, k))
    d.sync()
    assert d.stats()["arena_in_use"] == 0
    d.close()
