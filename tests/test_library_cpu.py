"""CPU-side checks of the HIP library: it loads, exports what include/delta.h declares, and
its planner (C++) produces byte-identical plans to the oracle planner (Python)."""
import os
import random
import re
import subprocess

import pytest

import paper_2203_15980_amd as dl
import synth
from oracle import checker, planner as pl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "delta.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(delta_[a-z_0-9]+)\s*\(", hdr))
    assert len(declared) >= 19
    lib = dl.load_library()
    nm = subprocess.check_output(["nm", "-D", "--defined-only", dl.binding.LIB_PATH]).decode()
    exported = set(re.findall(r" T (delta_[a-z_0-9]+)", nm))
    assert declared <= exported, declared - exported
    assert declared == set(dl.EXPORTS)
    for name in declared:
        assert getattr(lib, name) is not None


def test_planner_only_context_rejects_gpu_calls():
    d = dl.Delta()
    for call in (lambda: d.bind([16]), lambda: d.alloc(0), lambda: d.release(0, dl.EV_FREE), lambda: d.prefetch(0),
                 lambda: d.swap_out(0), lambda: d.sync(), lambda: d.backward_join(), lambda: d.backward_segment([]),
                 lambda: d.recompute_segment([])):
        with pytest.raises(dl.DeltaError) as e:
            call()
        assert e.value.status == dl.ERR_STATE
    d.close()


@pytest.mark.parametrize("cfg,frac", [(1, 0.5), (3, 0.5), (4, 0.4), (5, 0.3)])
def test_plans_match_oracle_on_configs(cfg, frac):
    g = synth.config_graph(cfg)
    B = int(frac * g.total_bytes())
    for kind in (pl.FILTER_BASE, pl.FILTER_LRU, pl.FILTER_GREEDY):
        for bw in (0, 20 * 10**9, 55 * 10**9, 10**13):
            for d in (0, 1, 4):
                p = pl.default_params(B, g.n_fwd, filter=kind, bw_d2h_Bps=bw, bw_h2d_Bps=bw * 9 // 10,
                                      prefetch_distance=d, max_reloads=d)
                try:
                    want = pl.plan(g.tensors, g.steps, p)
                except pl.Infeasible as e:
                    with pytest.raises(dl.DeltaError) as got:
                        dl.plan(g.tensors, g.steps, p)
                    assert got.value.status == dl.ERR_INFEASIBLE
                    assert ("step %d:" % e.step) in got.value.message
                    continue
                assert dl.plan(g.tensors, g.steps, p) == want


def test_config2_plans_in_a_single_pass_when_a_block_is_rebuilt_from_its_input():
    """The block kernel regenerates any tensor of a bottleneck from the block's input alone.  With that as the
    tensors' recompute route (`block_rebuild`: .a2 and .out have the block's input as their only parent) the single
    greedy pass of Algorithms 1-4 plans config 2 from 60 % down to 40 % of its activation bytes; with per-layer
    parents it fails at step 14 below 60 % (rebuilding b*.out drags a1 and a2 back into memory).  Library and
    oracle agree event by event on both graphs, the checker accepts every plan, and ResNet-50 with its three such
    blocks plans alike."""
    from paper_2203_15980_amd.harness import block_rebuild, find_blocks
    layers = synth.bottleneck_stack(32, 56, 56)
    assert sorted(find_blocks(layers)) == ["b1", "b2", "b3"]
    rb = block_rebuild(layers)
    assert sorted(rb) == ["b1.a2", "b1.out", "b2.a2", "b2.out", "b3.a2", "b3.out"]
    assert rb["b2.out"]["parents"] == ["b1.out"] and rb["b1.out"]["parents"] == ["x0"]
    by = {l.y: l for l in layers}
    assert rb["b2.out"]["flops"] == by["b2.a1"].flops + by["b2.a2"].flops + by["b2.out"].flops
    assert rb["b1.out"]["flops"] == sum(by["b1." + k].flops for k in ("a1", "a2", "sc", "out"))
    assert rb["b1.a2"]["flops"] == by["b1.a1"].flops + by["b1.a2"].flops
    per_layer = synth.fused_graph(layers, "bf16")
    block = synth.fused_graph(layers, "bf16", rebuild=rb)
    assert [t["bytes"] for t in block.tensors] == [t["bytes"] for t in per_layer.tensors]
    assert block.steps == per_layer.steps                     # the forward and backward steps are the same
    total = per_layer.total_bytes()
    for frac in (0.6, 0.55, 0.5, 0.45, 0.4):
        for kind in (pl.FILTER_BASE, pl.FILTER_LRU, pl.FILTER_GREEDY):
            p = pl.default_params(int(frac * total), block.n_fwd, filter=kind, bw_d2h_Bps=48 * 10**9, bw_h2d_Bps=52 * 10**9,
                                  prefetch_distance=2, max_reloads=2, release_when_short=1)
            want = pl.plan(block.tensors, block.steps, p)
            assert dl.plan(block.tensors, block.steps, p) == want
            st = checker.check(block.tensors, block.steps, p, want[0])
            assert st["peak"] <= p["budget_bytes"]
            if frac < 0.6 and kind == pl.FILTER_BASE:
                with pytest.raises(pl.Infeasible) as e:
                    pl.plan(per_layer.tensors, per_layer.steps, p)
                assert e.value.step == 14
                with pytest.raises(dl.DeltaError) as got:
                    dl.plan(per_layer.tensors, per_layer.steps, p)
                assert got.value.status == dl.ERR_INFEASIBLE
    r50 = synth.resnet_layers(128, (3, 4, 6, 3))
    rb = block_rebuild(r50)
    assert len(rb) == 6
    g = synth.fused_graph(r50, "bf16", with_loss=True, rebuild=rb)
    for frac in (0.5, 0.3):
        p = pl.default_params(int(frac * g.total_bytes()), g.n_fwd, bw_d2h_Bps=48 * 10**9, bw_h2d_Bps=52 * 10**9,
                              prefetch_distance=2, max_reloads=2, release_when_short=1, repair_rounds=8)
        try:
            want = pl.plan(g.tensors, g.steps, p)
        except pl.Infeasible:
            with pytest.raises(dl.DeltaError):
                dl.plan(g.tensors, g.steps, p)
            continue
        assert dl.plan(g.tensors, g.steps, p) == want
        checker.check(g.tensors, g.steps, p, want[0])


@pytest.mark.parametrize("cfg,frac", [(2, 0.5), (2, 0.4), (3, 0.3), (4, 0.25), (5, 0.2)])
def test_plans_match_oracle_with_the_optional_switches(cfg, frac):
    """release_when_short and repair_rounds, alone and together, at budgets where the single
    greedy pass struggles: same events, same peak, or the same failing step."""
    g = synth.config_graph(cfg)
    B = int(frac * g.total_bytes())
    for rws in (0, 1):
        for rounds in (0, 2, 8):
            for bw in (0, 55 * 10**9):
                p = pl.default_params(B, g.n_fwd, bw_d2h_Bps=bw, bw_h2d_Bps=bw, release_when_short=rws,
                                      repair_rounds=rounds)
                try:
                    want = pl.plan(g.tensors, g.steps, p)
                except pl.Infeasible as e:
                    with pytest.raises(dl.DeltaError) as got:
                        dl.plan(g.tensors, g.steps, p)
                    assert got.value.status == dl.ERR_INFEASIBLE
                    assert ("step %d:" % e.step) in got.value.message
                    continue
                assert dl.plan(g.tensors, g.steps, p) == want
                checker.check(g.tensors, g.steps, p, want[0])


def test_library_planner_reproduces_the_hand_worked_traces():
    """The event lists worked by hand from Algorithms 1-4 (tests/test_oracle_planner.py pins the
    oracle with them) also pin the library's planner directly, not only through the oracle."""
    import test_oracle_planner as top
    seen = []

    class Both:
        """Stands in for the oracle module inside the trace tests: every plan is made by both."""
        def __getattr__(self, name):
            return getattr(pl, name)

        @staticmethod
        def plan(tensors, steps, params):
            want = pl.plan(tensors, steps, params)
            assert dl.plan(tensors, steps, params) == (want[0], want[1])
            seen.append(len(want[0]))
            return want

        @staticmethod
        def plan_with_pins(tensors, steps, params):
            want = pl.plan_with_pins(tensors, steps, params)
            assert dl.plan(tensors, steps, params) == (want[0], want[1])
            seen.append(len(want[0]))
            return want

    saved = top.pl
    top.pl = Both()
    try:
        for name in sorted(dir(top)):
            if name.startswith("test_handworked_"):
                getattr(top, name)()
    finally:
        top.pl = saved
    assert len(seen) >= 12


def test_opgranular_resnet50_plan_matches_oracle():
    g = synth.opgranular_graph(synth.resnet_layers(128), "bf16")
    assert 150 <= len(g.tensors) <= 190
    p = pl.default_params(g.total_bytes() // 2, g.n_fwd)
    want = pl.plan(g.tensors, g.steps, p)
    assert dl.plan(g.tensors, g.steps, p) == want
    checker.check(g.tensors, g.steps, p, want[0])


def _random_graph(rnd, n):
    T = [dict(bytes=rnd.choice([256, 512, 1024]), cost_ns=0, flops=0, flags=pl.UNCOMPUTABLE, parents=[])]
    for i in range(1, n):
        par = {i - 1} | ({rnd.randrange(i)} if rnd.random() < 0.35 else set())
        flags = 0
        r = rnd.random()
        if r < 0.08:
            flags = pl.EVICT_PINNED
        elif r < 0.16:
            flags = pl.OFFLOAD_PINNED
        T.append(dict(bytes=rnd.choice([256, 512, 1024, 4096]), cost_ns=rnd.randint(1, 3000), flops=0,
                      flags=flags, parents=sorted(par)))
    S = [dict(produces=0, reads=[], cost_ns=0)]
    S += [dict(produces=i, reads=list(T[i]["parents"]), cost_ns=T[i]["cost_ns"]) for i in range(1, n)]
    for i in range(n - 1, 0, -1):
        if rnd.random() < 0.85:
            S.append(dict(produces=-1, reads=sorted(set(T[i]["parents"]) | {i}), cost_ns=2 * T[i]["cost_ns"]))
    return T, S, n


def test_plans_match_oracle_on_random_graphs():
    rnd = random.Random(2203)
    ok = bad = 0
    for trial in range(900):                    # the last 600 also draw the two optional switches
        T, S, n_fwd = _random_graph(rnd, rnd.randint(3, 40))
        total = sum(t["bytes"] for t in T)
        p = pl.default_params(int(total * rnd.uniform(0.15, 0.9)), n_fwd,
                              filter=rnd.randrange(3), prefetch_distance=rnd.randrange(5),
                              max_reloads=rnd.randrange(4),
                              trigger_num=rnd.choice([1, 3, 3, 7]), trigger_den=rnd.choice([1, 4, 8]),
                              bw_d2h_Bps=rnd.choice([0, 10**9, 10**12]), bw_h2d_Bps=rnd.choice([0, 10**9, 10**12]),
                              release_when_short=rnd.randrange(2) if trial >= 300 else 0,
                              repair_rounds=rnd.choice([0, 1, 4]) if trial >= 300 else 0)
        if p["trigger_num"] > p["trigger_den"]:
            p["trigger_num"] = p["trigger_den"]
        try:
            want = pl.plan(T, S, p)
        except pl.Infeasible as e:
            with pytest.raises(dl.DeltaError) as got:
                dl.plan(T, S, p)
            assert got.value.status == dl.ERR_INFEASIBLE and ("step %d:" % e.step) in got.value.message
            bad += 1
            continue
        assert dl.plan(T, S, p) == want
        checker.check(T, S, p, want[0])
        ok += 1
    assert ok > 300 and bad > 30        # both outcomes are exercised


def test_plans_match_oracle_with_rebuild_aware_prefetch():
    """prefetch_rebuild_reads: the library's reading of "wanted by a recomputation" against the oracle's, on
    random graphs (every switch drawn), on the configurations, and on the two hand-worked traces."""
    rnd = random.Random(1598)
    ok = bad = moved = 0
    for trial in range(700):
        T, S, n_fwd = _random_graph(rnd, rnd.randint(3, 40))
        total = sum(t["bytes"] for t in T)
        p = pl.default_params(int(total * rnd.uniform(0.15, 0.9)), n_fwd,
                              filter=rnd.randrange(3), prefetch_distance=rnd.randrange(1, 6),
                              max_reloads=rnd.randrange(1, 4),
                              trigger_num=rnd.choice([1, 3, 3, 7]), trigger_den=rnd.choice([4, 8]),
                              bw_d2h_Bps=rnd.choice([10**8, 10**9, 10**12]), bw_h2d_Bps=rnd.choice([10**8, 10**9, 10**12]),
                              release_when_short=rnd.randrange(2), repair_rounds=rnd.choice([0, 1, 4]),
                              prefetch_rebuild_reads=1)
        p["trigger_num"] = min(p["trigger_num"], p["trigger_den"])
        try:
            ev, peak, pins = pl.plan_with_pins(T, S, p)
            want = (ev, peak)
        except pl.Infeasible as e:
            with pytest.raises(dl.DeltaError) as got:
                dl.plan(T, S, p)
            assert got.value.status == dl.ERR_INFEASIBLE and ("step %d:" % e.step) in got.value.message
            bad += 1
            continue
        assert dl.plan(T, S, p) == want
        # the checker sees the graph as the last repair round planned it (its learned offload-only tensors)
        checker.check([dict(t, flags=t["flags"] | pl.UNCOMPUTABLE) if i in pins else t for i, t in enumerate(T)], S, p, ev)
        ok += 1
        try:
            moved += pl.plan(T, S, dict(p, prefetch_rebuild_reads=0)) != want
        except pl.Infeasible:
            moved += 1
    assert ok > 300 and bad > 10 and moved > 25, (ok, bad, moved)
    for cfg, frac in [(3, 0.5), (4, 0.4), (5, 0.3)]:
        g = synth.config_graph(cfg)
        for bw in (20 * 10**9, 55 * 10**9):
            p = pl.default_params(int(frac * g.total_bytes()), g.n_fwd, bw_d2h_Bps=bw, bw_h2d_Bps=bw, prefetch_distance=2,
                                  max_reloads=2, release_when_short=1, repair_rounds=8, prefetch_rebuild_reads=1)
            want = pl.plan(g.tensors, g.steps, p)
            assert dl.plan(g.tensors, g.steps, p) == want
            checker.check(g.tensors, g.steps, p, want[0])
    with pytest.raises(dl.DeltaError):
        dl.plan(g.tensors, g.steps, dict(p, prefetch_rebuild_reads=2))


def test_plan_rejects_malformed_graphs():
    g = synth.config_graph(1)
    p = pl.default_params(g.total_bytes(), g.n_fwd)
    bad = [dict(t) for t in g.tensors]
    bad[3] = dict(bad[3], parents=[5])                      # parent id above own id
    with pytest.raises(dl.DeltaError) as e:
        dl.plan(bad, g.steps, p)
    assert e.value.status == dl.ERR_INVALID
    steps = [dict(s) for s in g.steps]
    steps[2] = dict(steps[2], reads=[9])                    # reads a tensor not produced yet
    with pytest.raises(dl.DeltaError) as e:
        dl.plan(g.tensors, steps, p)
    assert e.value.status == dl.ERR_INVALID
    with pytest.raises(dl.DeltaError) as e:
        dl.plan(g.tensors, g.steps, dict(p, trigger_den=0))
    assert e.value.status == dl.ERR_INVALID


def test_heuristic_sweep_reproduces_the_papers_ordering():
    """Sec. 5.7 / Fig. 7-8 (qualitative): at small budgets base and LRU get by with less memory
    than GREEDY on ResNet-50, and LRU moves more tensors than base."""
    from paper_2203_15980_amd import sweep
    res = sweep.run(configs=(3,), fracs=(0.5,))["config3"]
    assert res["base"]["min_budget_frac"] <= res["greedy"]["min_budget_frac"]
    assert res["lru"]["min_budget_frac"] <= res["greedy"]["min_budget_frac"]
    moved = lambda r: r["at"]["0.5"]["evict"] + r["at"]["0.5"]["offload"]
    assert moved(res["lru"]) >= moved(res["base"])


def test_binding_structs_have_the_headers_layout(tmp_path):
    """The ctypes structures must match include/delta.h field for field: a C program built against
    the header prints sizes and offsets, the binding is compared with it."""
    import ctypes as C
    from paper_2203_15980_amd import binding as B
    fields = {"delta_plan_params": [f for f, _ in B.PlanParams._fields_],
              "delta_layer_desc": [f for f, _ in B.LayerDesc._fields_],
              "delta_bwd_desc": [f for f, _ in B.BwdDesc._fields_],
              "delta_stats_t": [f for f, _ in B.Stats._fields_]}
    src = ["#include <stdio.h>", "#include <stddef.h>", '#include "delta.h"', "int main(void) {"]
    for st, fs in fields.items():
        src.append('printf("%s %%zu\\n", sizeof(%s));' % (st, st))
        for f in fs:
            src.append('printf("%s.%s %%zu\\n", offsetof(%s, %s));' % (st, f, st, f))
    src += ["return 0;", "}"]
    c_file = tmp_path / "layout.c"
    c_file.write_text("\n".join(src))
    exe = tmp_path / "layout"
    subprocess.check_call(["gcc", "-I", os.path.join(ROOT, "include"), str(c_file), "-o", str(exe)])
    want = dict(line.split() for line in subprocess.check_output([str(exe)]).decode().splitlines())
    classes = {"delta_plan_params": B.PlanParams, "delta_layer_desc": B.LayerDesc, "delta_bwd_desc": B.BwdDesc,
               "delta_stats_t": B.Stats}
    for st, cls in classes.items():
        assert C.sizeof(cls) == int(want[st]), st
        for f in fields[st]:
            assert getattr(cls, f).offset == int(want["%s.%s" % (st, f)]), (st, f)
    # and the enumerators the binding restates
    hdr = open(os.path.join(ROOT, "include", "delta.h")).read()
    for name, val in (("OP_ATTENTION", B.OP_ATTENTION), ("OP_LAYERNORM", B.OP_LAYERNORM), ("OP_BATCHNORM", B.OP_BATCHNORM),
                      ("OP_RELU", B.OP_RELU), ("OP_ADD", B.OP_ADD), ("OP_SOFTMAX_CE", B.OP_SOFTMAX_CE),
                      ("ACT_GELU", B.ACT_GELU), ("ACT_RELU", B.ACT_RELU)):
        m = re.search(r"DELTA_%s\s*=\s*(\d+)" % name, hdr)
        assert m and int(m.group(1)) == val, name


def test_executed_encoder_plan_matches_oracle():
    """The graph bench.py replays for config 5 (12 BERT-base layers as 84 fused operators, no score
    tensors): library plan = oracle plan at 30 % and 50 %, and the plans pass the checker."""
    layers = synth.encoder_layers(32, 512, nlayers=12)
    g = synth.fused_graph(layers, "bf16")
    assert len(g.tensors) == 85 and g.total_bytes() == 3649044480
    for frac in (0.3, 0.5):
        p = pl.default_params(int(frac * g.total_bytes()), g.n_fwd, bw_d2h_Bps=55 * 10**9, bw_h2d_Bps=55 * 10**9)
        want = pl.plan(g.tensors, g.steps, p)
        assert dl.plan(g.tensors, g.steps, p) == want
        st = checker.check(g.tensors, g.steps, p, want[0])
        assert st["peak"] == want[1] <= p["budget_bytes"]


def test_bench_refuses_more_than_one_gpu():
    r = subprocess.run(["python", os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "one GPU" in r.stderr and r.stdout.strip() == ""


def test_max_batch_search_brackets_feasibility():
    """Sec. 5.3's question on synthetic graphs: under a fixed number of activation bytes the planner
    admits a larger batch than keeping everything; the returned batches are exactly the last that fit."""
    import synth
    from paper_2203_15980_amd import sweep
    from paper_2203_15980_amd import binding as B
    arena = 1 << 30
    depths = (3, 4, 6, 3)
    d = B.Delta()
    plain, planned = sweep.max_batch(d, depths, arena)
    assert 0 < plain < planned

    def plan(n, budget):
        g = synth.fused_graph(synth.resnet_layers(n, depths), "bf16", with_loss=True)
        return d.plan(g.tensors, g.steps, sweep._params(budget, g.n_fwd, B.FILTER_BASE))

    assert plan(plain, 10**15)[1] <= arena < plan(plain + 1, 10**15)[1]
    assert plan(planned, arena)[1] <= arena
    with pytest.raises(B.DeltaError) as e:
        plan(planned + 1, arena)
    assert e.value.status == B.ERR_INFEASIBLE
    d.close()
