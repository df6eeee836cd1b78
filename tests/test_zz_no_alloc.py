"""delta_batchnorm_static, the entry point that allocates nothing (its scratch is a file-scope device
array inside the library), against the DELTA_OP_BATCHNORM operator of delta_recompute_segment, through
the C ABI: the same kernels and decomposition, so the bar is bit equality; and against the CPU oracle
within the batch-norm bar of the operator-granular tests (2e-2 / 4 of the tensor's maximum).  Two calls
in a row on one context, the second with a smaller input, so that whatever the first left in the
shared scratch would show."""
import numpy as np
import pytest

import synth
from oracle import numeric as on
from oracle import opgranular as og

pytestmark = pytest.mark.gpu


def _dev(torch, a):
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")


def _bits(master, aid, shape, scale=1.0, shift=0.0):
    return synth.f32_to_bf16_bits((synth.normal(master, aid, int(np.prod(shape))) * scale + shift).astype(np.float32)).reshape(shape)


def test_batchnorm_static_matches_the_allocating_entry_point_twice_in_a_row():
    import torch
    import paper_2203_15980_amd as dl
    assert torch.cuda.is_available()
    arena = torch.empty(64 << 20, dtype=torch.uint8, device="cuda:0")
    d = dl.Delta(arena, torch.cuda.current_stream().cuda_stream)
    base = arena.data_ptr()
    for call, shape in enumerate([(16, 56, 56, 64), (3, 5, 9, 24)]):       # second call: smaller input
        print("call", call, "shape", shape, flush=True)
        N, H, W, C = shape
        x = _bits(97, 10 + call, shape, 2.0, 3.0)
        gamma = synth.uniform(97, 20 + call, C, 0.5, 1.5).astype(np.float32)
        beta = synth.normal(97, 30 + call, C, 0.0, 0.1).astype(np.float32)
        g, b = _dev(torch, gamma), _dev(torch, beta)
        # the existing entry point, on arena tensors
        d.bind([x.nbytes, x.nbytes])
        ptr = d.alloc(0)
        arena[ptr - base:ptr - base + x.nbytes].copy_(_dev(torch, x.view(np.uint8).reshape(-1)))
        desc = dl.LayerDesc(x=0, res=dl.NO_TENSOR, y=1, dtype=dl.DTYPE_BF16, w=None, scale=g.data_ptr(), shift=b.data_ptr(),
                            N=N, H=H, W=W, Cin=C, Cout=C, R=1, S=1, stride=1, pad=0, relu=0, op=dl.OP_BATCHNORM, eps=1e-5)
        d.recompute_segment([desc])
        d.sync()
        yp = d.tensor_ptr(1)
        want = arena[yp - base:yp - base + x.nbytes].cpu().numpy().view(np.uint16).reshape(shape).copy()
        # the entry point that allocates nothing, on the caller's own buffers
        xs = _dev(torch, x.view(np.int16).reshape(-1))
        ys = torch.full_like(xs, 0x7FC0)                                     # NaN pattern: every element must be written
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated()
        d.batchnorm_static(xs.data_ptr(), ys.data_ptr(), g.data_ptr(), b.data_ptr(), N * H * W, C, 1e-5)
        d.sync()
        assert torch.cuda.memory_allocated() == before
        got = ys.cpu().numpy().view(np.uint16).reshape(shape)
        assert np.array_equal(got, want), (shape, int(np.sum(got != want)))
        ref = on.to_f64(og.bn_train(x, gamma, beta, 1e-5, "bf16"), "bf16")
        err = float(np.max(np.abs(on.to_f64(got, "bf16") - ref)) / np.max(np.abs(ref)))
        print("  err vs oracle %.2e" % err, flush=True)
        assert err <= 2e-2 / 4, (shape, err)
    # sizes beyond what the static scratch is sized for are refused before anything is launched
    big = torch.zeros(8200 * 2, dtype=torch.int16, device="cuda:0")
    f = torch.zeros(8200, dtype=torch.float32, device="cuda:0")
    with pytest.raises(dl.DeltaError) as e:
        d.batchnorm_static(big.data_ptr(), big.data_ptr() + 8200 * 2, f.data_ptr(), f.data_ptr(), 1, 8200, 1e-5)
    assert e.value.status == dl.ERR_INVALID and "8192" in e.value.message
    d.close()
