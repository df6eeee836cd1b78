"""Pins of the planner oracle: the paper's Table 5, the special cases its text fixes,
closed forms, hand-worked traces, the independent checker and exhaustive search."""
import os
import random

import pytest

import synth
from oracle import brute, checker, planner as pl

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def T(m, cost, parents=(), flags=0):
    return dict(bytes=m, cost_ns=cost, flops=0, flags=flags, parents=list(parents))


def chain(n, m=4, cost=10, src_flags=pl.UNCOMPUTABLE, src_cost=0):
    """t0 -> t1 -> ... ; forward step i produces t_i from t_{i-1}; backward of layer i
    (i = n-1 .. 1) reads t_{i-1} and t_i."""
    tensors = [T(m, src_cost, (), src_flags)] + [T(m, cost, (i - 1,)) for i in range(1, n)]
    steps = [dict(produces=0, reads=[], cost_ns=src_cost)]
    steps += [dict(produces=i, reads=[i - 1], cost_ns=cost) for i in range(1, n)]
    steps += [dict(produces=-1, reads=[i - 1, i], cost_ns=2 * cost) for i in range(n - 1, 0, -1)]
    return tensors, steps, n


def names(events):
    return [(k, pl.EVENT_NAMES[a], t) for (k, a, t) in events]


# ------------------------------------------------------------------ Director (Alg. 3, Eq. 4-6)

def _director(c_r_ns, m, bw, flags=0):
    sim = pl._Sim([T(m, c_r_ns, (), flags)], [dict(produces=0, reads=[], cost_ns=0)],
                  pl.default_params(10**12, 1, bw_d2h_Bps=bw, bw_h2d_Bps=bw))
    sim.resident[0] = True
    return sim.director(0)


def test_table5_pairs_all_evict():
    """Sec. 5.5, Table 5: for each printed (c_s, c_r) pair recomputation is far cheaper, so
    F = c_r / c_s < 1 and the Director must answer Evict."""
    rows = [l.split() for l in open(os.path.join(GOLD, "table5_costs.txt"))
            if l.strip() and not l.startswith("#")]
    assert len(rows) == 6
    for name, cs_us, cr_us in rows:
        cs_ns, cr_ns = int(cs_us) * 1000, int(cr_us) * 1000
        # choose m and b so that c_s = m/b + m/b equals the printed value exactly
        m, bw = cs_ns // 2, 10**9           # 1 byte per ns each way
        assert pl.swap_cost_ns(m, bw, bw) == cs_ns
        assert _director(cr_ns, m, bw) == pl.EV_EVICT, name
        # and the same tensors flip to Offload once recomputation costs more than the swap
        assert _director(cs_ns + 1, m, bw) == pl.EV_OFFLOAD, name


def test_director_pins_override_costs():
    """Sec. 4.3: evict_pinned -> Offload, offload_pinned -> Evict, whatever the costs."""
    assert _director(1, 10**6, 10**9, pl.EVICT_PINNED) == pl.EV_OFFLOAD
    assert _director(1, 10**6, 10**9, pl.UNCOMPUTABLE) == pl.EV_OFFLOAD
    assert _director(10**15, 10**6, 10**9, pl.OFFLOAD_PINNED) == pl.EV_EVICT


def test_director_tie_and_limits():
    m, bw = 500, 10**9                      # c_s = 500 + 500 ns
    assert _director(1000, m, bw) == pl.EV_EVICT        # F = 1 -> Evict (Alg. 3: s_d <= 1)
    assert _director(1001, m, bw) == pl.EV_OFFLOAD
    assert _director(10**18, m, 0) == pl.EV_EVICT       # b -> 0: swap never pays (DTR limit)
    assert _director(1, m, 10**18) == pl.EV_EVICT       # c_s rounds up to 2 ns, c_r = 1
    assert _director(3, m, 10**18) == pl.EV_OFFLOAD     # b -> infinity: everything offloads


def test_recompute_cost_counts_missing_ancestors_once():
    # diamond: 0 -> 1 -> 3, 0 -> 2 -> 3 ; c_r(3) with 1, 2 and 0 absent counts 0 once
    tensors = [T(8, 5), T(8, 7, (0,)), T(8, 11, (0,)), T(8, 13, (1, 2))]
    sim = pl._Sim(tensors, [dict(produces=-1, reads=[], cost_ns=0)], pl.default_params(100, 0))
    sim.resident = [False, False, False, True]
    assert sim.recompute_cost(3) == 13 + 7 + 11 + 5
    sim.resident = [False, True, False, True]
    assert sim.recompute_cost(3) == 13 + 11 + 5
    sim.resident = [False, True, True, True]
    assert sim.recompute_cost(3) == 13                   # resident parents stop the walk
    # an uncomputable missing ancestor costs its reload time
    tensors[0] = T(8, 5, (), pl.UNCOMPUTABLE)
    sim = pl._Sim(tensors, [dict(produces=-1, reads=[], cost_ns=0)],
                  pl.default_params(100, 0, bw_h2d_Bps=2 * 10**9))
    sim.resident = [False, False, True, True]
    assert sim.recompute_cost(3) == 13 + 7 + 4


# ------------------------------------------------------------------ Filter (Alg. 2, Eq. 1-3)

def _filter(kind, ms, stale):
    tensors = [T(m, 1) for m in ms]
    sim = pl._Sim(tensors, [dict(produces=-1, reads=[], cost_ns=0)],
                  pl.default_params(10**9, 0, filter=kind))
    sim.tau = 1000
    sim.last_access = [1000 - s for s in stale]
    return sim.filter(list(range(len(ms))))


def test_filter_is_argmin_of_the_printed_heuristics():
    ms, st = [10, 40, 20, 40], [7, 2, 5, 3]
    from fractions import Fraction as F
    h = {pl.FILTER_BASE: lambda m, s: F(1, m * s), pl.FILTER_LRU: lambda m, s: F(1, s),
         pl.FILTER_GREEDY: lambda m, s: F(1, m)}
    for kind, fn in h.items():
        scores = [fn(m, s) for m, s in zip(ms, st)]
        assert _filter(kind, ms, st) == scores.index(min(scores))     # first minimum: lowest id
    assert _filter(pl.FILTER_BASE, ms, st) == 3        # 40*3 = 120 beats 10*7, 40*2, 20*5
    assert _filter(pl.FILTER_LRU, ms, st) == 0
    assert _filter(pl.FILTER_GREEDY, ms, st) == 1      # tie 40/40 -> lowest id


def test_filter_equal_m_is_lru_equal_s_is_greedy_and_zero_staleness_is_last():
    rnd = random.Random(3)
    for _ in range(50):
        st = [rnd.randint(1, 99) for _ in range(6)]
        ms = [rnd.randint(1, 99) for _ in range(6)]
        assert _filter(pl.FILTER_BASE, [16] * 6, st) == _filter(pl.FILTER_LRU, [16] * 6, st)
        assert _filter(pl.FILTER_BASE, ms, [9] * 6) == _filter(pl.FILTER_GREEDY, ms, [9] * 6)
    assert _filter(pl.FILTER_BASE, [10**9, 1], [0, 1]) == 1      # s = 0 -> H = infinity
    # 128-bit product: 2^63 * 3 > 2^64 must not wrap
    assert _filter(pl.FILTER_BASE, [2**63, 2**62], [3, 5]) == 0


# ------------------------------------------------------------------ hand-worked traces

def test_handworked_chain_offload_evict_prefetch():
    """Chain t0..t4, m = 4 each, cost 10, B = 12, trigger 1/1, b = 0 (swap never pays),
    t0 uncomputable, d = n = 1.  By hand from Alg. 1-4:
      step 3 (make t3): live 12 + 4 > 12; candidates t0 (m*s = 4*10) and t1 (4*0); the
        Filter takes t0; it is uncomputable so the Director says Offload.
      step 4 (make t4): candidates t1 (s = 10) and t2 (s = 0) -> t1, Evict (c_s infinite).
      step 5, 6: backward of layers 4, 3; t4 and t3 die.
      step 7 reads t1, t2: t0's next use is step 8 <= 7 + d and 4 + 4 <= 12 -> prefetch t0;
        t1 is evicted -> Recompute (its parent t0 is back); t2 dies.
      step 8 reads t0, t1; both die."""
    tensors, steps, n_fwd = chain(5)
    p = pl.default_params(12, n_fwd, trigger_num=1, trigger_den=1, bw_d2h_Bps=0, bw_h2d_Bps=0,
                          prefetch_distance=1, max_reloads=1)
    ev, peak = pl.plan(tensors, steps, p)
    assert names(ev) == [(3, "OFFLOAD", 0), (4, "EVICT", 1), (5, "FREE", 4), (6, "FREE", 3),
                         (7, "RELOAD_PREFETCH", 0), (7, "RECOMPUTE", 1), (7, "FREE", 2),
                         (8, "FREE", 0), (8, "FREE", 1)]
    assert peak == 12
    checker.check(tensors, steps, p, ev)


def test_handworked_chain_recompute_keeps_needed_parent():
    """Same chain but t0 is a recomputable source (cost 5).  Steps 3 and 4 evict t0 and t1.
    At step 7 rebuilding t1 first rebuilds t0; t0 is read at step 8, so it stays (no
    DROP_TEMP) and step 8 finds both on the GPU."""
    tensors, steps, n_fwd = chain(5, src_flags=0, src_cost=5)
    p = pl.default_params(12, n_fwd, trigger_num=1, trigger_den=1, bw_d2h_Bps=0, bw_h2d_Bps=0)
    ev, peak = pl.plan(tensors, steps, p)
    assert names(ev) == [(3, "EVICT", 0), (4, "EVICT", 1), (5, "FREE", 4), (6, "FREE", 3),
                         (7, "RECOMPUTE", 0), (7, "RECOMPUTE", 1), (7, "FREE", 2),
                         (8, "FREE", 0), (8, "FREE", 1)]
    assert peak == 12
    checker.check(tensors, steps, p, ev)


def test_handworked_temporaries_without_a_reader_are_dropped():
    """t0 -> t1 -> t2 -> t3 -> t4, m = 4, B = 8; the backward pass reads only t4, t3, t2.
    t0 and t1 die in the forward pass.  Step 4 must evict t2 (only candidate).  Step 7 reads
    t2: rebuild t0, t1 (drop t0: nobody reads it), t2 (drop t1)."""
    tensors = [T(4, 5)] + [T(4, 10, (i - 1,)) for i in range(1, 5)]
    steps = [dict(produces=0, reads=[], cost_ns=5)]
    steps += [dict(produces=i, reads=[i - 1], cost_ns=10) for i in range(1, 5)]
    steps += [dict(produces=-1, reads=[t], cost_ns=20) for t in (4, 3, 2)]
    p = pl.default_params(8, 5, trigger_num=1, trigger_den=1, bw_d2h_Bps=0, bw_h2d_Bps=0)
    ev, peak = pl.plan(tensors, steps, p)
    assert names(ev) == [(1, "FREE", 0), (2, "FREE", 1), (4, "EVICT", 2), (5, "FREE", 4),
                         (6, "FREE", 3), (7, "RECOMPUTE", 0), (7, "RECOMPUTE", 1),
                         (7, "DROP_TEMP", 0), (7, "RECOMPUTE", 2), (7, "DROP_TEMP", 1),
                         (7, "FREE", 2)]
    assert peak == 8
    checker.check(tensors, steps, p, ev)


def test_chain_victims_leave_in_production_order():
    """Equal m and cost on a chain: the stalest resident tensor is always the oldest one,
    so base, LRU and (by the lowest-id tie-break) GREEDY all release t0, t1, t2, ..."""
    tensors, steps, n_fwd = chain(10, src_flags=0, src_cost=10)
    for kind in (pl.FILTER_BASE, pl.FILTER_LRU, pl.FILTER_GREEDY):
        p = pl.default_params(3 * 4, n_fwd, trigger_num=1, trigger_den=1, filter=kind,
                              bw_d2h_Bps=0, bw_h2d_Bps=0)
        ev, _ = pl.plan(tensors, steps, p)
        victims = [t for (k, a, t) in ev if a == pl.EV_EVICT]
        assert victims == list(range(len(victims))) and len(victims) == 7


# ------------------------------------------------------------------ whole plans

@pytest.mark.parametrize("cfg,frac", [(1, 0.5), (3, 0.5), (4, 0.4), (5, 0.3)])
def test_config_plans_pass_the_checker(cfg, frac):
    g = synth.config_graph(cfg)
    B = int(frac * g.total_bytes())
    for bw in (50 * 10**9, 5 * 10**12):
        p = pl.default_params(B, g.n_fwd, bw_d2h_Bps=bw, bw_h2d_Bps=bw)
        ev, peak = pl.plan(g.tensors, g.steps, p)
        st = checker.check(g.tensors, g.steps, p, ev)
        assert st["peak"] == peak <= B
        assert not any(a in (pl.EV_EVICT, pl.EV_OFFLOAD) and k >= g.n_fwd for (k, a, t) in ev)


def test_large_budget_gives_an_empty_plan():
    """With B >= 4/3 of the no-release peak the 3/4 trigger never fires."""
    for cfg in (1, 2, 3):
        g = synth.config_graph(cfg)
        big = pl.default_params(10**15, g.n_fwd)
        _, base_peak = pl.plan(g.tensors, g.steps, big)
        p = pl.default_params(-(-base_peak * 4 // 3), g.n_fwd)
        ev, peak = pl.plan(g.tensors, g.steps, p)
        assert all(a == pl.EV_FREE for (_, a, _) in ev) and peak == base_peak
        p = pl.default_params(base_peak * 4 // 3 - 8, g.n_fwd)
        ev, _ = pl.plan(g.tensors, g.steps, p)
        assert any(a in (pl.EV_EVICT, pl.EV_OFFLOAD) for (_, a, _) in ev)


def test_bandwidth_limits_flip_every_decision():
    g = synth.config_graph(3)
    B = g.total_bytes() // 2
    ev0, _ = pl.plan(g.tensors, g.steps, pl.default_params(B, g.n_fwd, bw_d2h_Bps=0, bw_h2d_Bps=0))
    rel = [(a, t) for (_, a, t) in ev0 if a in (pl.EV_EVICT, pl.EV_OFFLOAD)]
    assert rel and all(a == pl.EV_EVICT or g.tensors[t]["flags"] & pl.UNCOMPUTABLE for a, t in rel)
    evi, _ = pl.plan(g.tensors, g.steps,
                     pl.default_params(B, g.n_fwd, bw_d2h_Bps=10**18, bw_h2d_Bps=10**18))
    rel = [a for (_, a, t) in evi if a in (pl.EV_EVICT, pl.EV_OFFLOAD)]
    assert rel and all(a == pl.EV_OFFLOAD for a in rel)


def test_infeasible_budget_is_reported():
    g = synth.config_graph(1)
    with pytest.raises(pl.Infeasible):
        pl.plan(g.tensors, g.steps, pl.default_params(2 * 2**20, g.n_fwd))


def test_checker_rejects_planted_mistakes():
    g = synth.config_graph(1)
    p = pl.default_params(g.total_bytes() // 2, g.n_fwd)
    ev, _ = pl.plan(g.tensors, g.steps, p)
    checker.check(g.tensors, g.steps, p, ev)
    rel = [i for i, e in enumerate(ev) if e[1] in (pl.EV_EVICT, pl.EV_OFFLOAD)]
    rec = [i for i, e in enumerate(ev) if e[1] in (pl.EV_RECOMPUTE, pl.EV_RELOAD_PREFETCH,
                                                   pl.EV_RELOAD_DEMAND)]
    bad = []
    bad.append(ev[:rel[0]] + ev[rel[0] + 1:])                     # a release goes missing
    bad.append(ev[:rec[0]] + ev[rec[0] + 1:])                     # a tensor never comes back
    k_b = g.n_fwd
    bad.append(sorted(ev + [(k_b, pl.EV_EVICT, 10)], key=lambda e: e[0]))   # release in backward
    e = ev[rel[0]]
    bad.append([(e[0], e[1], 0) if i == rel[0] and e[1] == pl.EV_EVICT else x
                for i, x in enumerate(ev)] if e[1] == pl.EV_EVICT else
               ev[:rel[0]] + [(e[0], pl.EV_EVICT, 0)] + ev[rel[0]:])        # evicts the input
    for b in bad:
        with pytest.raises(checker.PlanError):
            checker.check(g.tensors, g.steps, p, b)
    small = dict(p, budget_bytes=p["budget_bytes"] // 2)
    with pytest.raises(checker.PlanError):
        checker.check(g.tensors, g.steps, small, ev)              # over a tighter budget


# ------------------------------------------------------------------ exhaustive search

def _random_graph(rnd, n):
    tensors = [T(rnd.choice([2, 4, 8]), 0, (), pl.UNCOMPUTABLE)]
    for i in range(1, n):
        par = {i - 1} | ({rnd.randrange(i)} if rnd.random() < 0.4 else set())
        tensors.append(T(rnd.choice([2, 4, 8, 16]), rnd.randint(1, 50), sorted(par)))
    steps = [dict(produces=0, reads=[], cost_ns=0)]
    steps += [dict(produces=i, reads=list(tensors[i]["parents"]), cost_ns=tensors[i]["cost_ns"])
              for i in range(1, n)]
    for i in range(n - 1, 0, -1):
        steps.append(dict(produces=-1, reads=sorted(set(tensors[i]["parents"]) | {i}),
                          cost_ns=2 * tensors[i]["cost_ns"]))
    return tensors, steps, n


def test_brute_force_agrees_with_checker_and_is_monotone():
    rnd = random.Random(11)
    for trial in range(12):
        tensors, steps, n_fwd = _random_graph(rnd, rnd.randint(4, 8))
        total = sum(t["bytes"] for t in tensors)
        prev = None
        for B in range(total, 0, -max(1, total // 6)):
            p = pl.default_params(B, n_fwd, bw_d2h_Bps=10**9, bw_h2d_Bps=10**9)
            o = brute.optimum(tensors, steps, p)
            if o is None:
                prev = None
                continue
            st = checker.check(tensors, steps, p, o["events"], check_trigger=False)
            assert st["peak"] == o["peak"] <= B          # two independent replays agree
            assert st["cost_ns"] == o["cost"]
            if prev is not None:
                assert o["cost"] >= prev                 # less memory never gets cheaper
            prev = o["cost"]
        # with the whole graph's bytes as budget nothing needs to move
        p = pl.default_params(total, n_fwd, bw_d2h_Bps=10**9, bw_h2d_Bps=10**9)
        assert brute.optimum(tensors, steps, p)["cost"] == 0


def test_heuristic_cost_is_bounded_below_where_the_static_class_covers_it():
    """On chains every tensor the heuristic can release has already had its last forward
    read, so with prefetch off its plan is a static plan (release after last forward use,
    restore at first backward use) and cannot beat the exhaustive optimum."""
    for n, B in ((6, 12), (7, 16), (8, 12)):
        tensors, steps, n_fwd = chain(n, src_flags=0, src_cost=10)
        p = pl.default_params(B, n_fwd, trigger_num=1, trigger_den=1, bw_d2h_Bps=0, bw_h2d_Bps=0,
                              prefetch_distance=0, max_reloads=0)
        ev, _ = pl.plan(tensors, steps, p)
        st = checker.check(tensors, steps, p, ev)
        o = brute.optimum(tensors, steps, p)
        assert o is not None and st["cost_ns"] >= o["cost"] > 0


def test_config1_optimum_and_heuristic_gap():
    g = synth.config_graph(1)
    p = pl.default_params(g.total_bytes() // 2, g.n_fwd)
    o = brute.optimum(g.tensors, g.steps, p)
    assert o is not None
    st = checker.check(g.tensors, g.steps, p, o["events"], check_trigger=False)
    assert st["cost_ns"] == o["cost"] and st["peak"] <= p["budget_bytes"]
    ev, _ = pl.plan(g.tensors, g.steps, p)
    h = checker.check(g.tensors, g.steps, p, ev)
    print("config 1: heuristic cost %d ns, static optimum %d ns" % (h["cost_ns"], o["cost"]))
