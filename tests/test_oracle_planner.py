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


def test_handworked_leftovers_give_way_farthest_next_use_first_lowest_id_on_ties():
    """Three leftovers of a recomputation with next uses 10, 11, 10 and an allocation that
    needs the room of two of them (reading: rebuilt parents stay while a later step reads them
    and go farthest next use first, ties to the lowest id).
    t0 (m 4, never releasable: both pin flags) feeds t1, t2, t3 (m 4); t4 = f(t1, t2, t3);
    t5 = f(t0), m 8; t6 = f(t4, t5); t7 = f(t6), m 8.  B = 20, trigger 1/1, no link.
      step 4 fills the budget (t0..t4 = 20).  step 5 (t5 needs 8): t1..t4 all have s = 0, so
        every product m*s is 0 and the lowest ids go: Evict t1, t2.  step 6: only t3 (s = 10)
        is free to go.  step 7 (t7 needs 8): t4 then t5 (both s = 0, lowest id first); t6 and
        t7 die at once.
      step 8 reads t4: t1, t2, t3 are rebuilt first (live 20); they are read again at steps
        10, 11, 10, so they stay as leftovers.
      step 9 reads t5 (8 bytes, live 20): the farthest leftover t2 (step 11) goes first, then
        the tie t1/t3 (step 10) goes to the lowest id, t1.
    One-line mutations that turn this red: `nr > best_nr` -> `nr < best_nr` in grow (drops
    t1, t3); `nr >= best_nr` (drops t2, t3); ignoring nr altogether (drops t1, t2)."""
    both = pl.EVICT_PINNED | pl.OFFLOAD_PINNED
    tensors = [T(4, 1, (), both), T(4, 10, (0,)), T(4, 10, (0,)), T(4, 10, (0,)),
               T(4, 10, (1, 2, 3)), T(8, 10, (0,)), T(4, 10, (4, 5)), T(8, 10, (6,))]
    steps = [dict(produces=0, reads=[], cost_ns=1)]
    steps += [dict(produces=i, reads=list(tensors[i]["parents"]), cost_ns=10) for i in range(1, 8)]
    steps += [dict(produces=-1, reads=r, cost_ns=20) for r in ([4], [5], [1, 3], [2], [0, 4])]
    p = pl.default_params(20, 8, trigger_num=1, trigger_den=1, bw_d2h_Bps=0, bw_h2d_Bps=0)
    ev, peak = pl.plan(tensors, steps, p)
    assert names(ev) == [
        (5, "EVICT", 1), (5, "EVICT", 2), (6, "EVICT", 3), (7, "EVICT", 4), (7, "EVICT", 5),
        (7, "FREE", 6), (7, "FREE", 7),
        (8, "RECOMPUTE", 1), (8, "RECOMPUTE", 2), (8, "RECOMPUTE", 3), (8, "RECOMPUTE", 4),
        (9, "DROP_TEMP", 2), (9, "DROP_TEMP", 1), (9, "RECOMPUTE", 5), (9, "FREE", 5),
        (10, "RECOMPUTE", 1), (10, "FREE", 1), (10, "FREE", 3),
        (11, "RECOMPUTE", 2), (11, "FREE", 2), (12, "FREE", 0), (12, "FREE", 4)]
    assert peak == 20
    checker.check(tensors, steps, p, ev)


def test_handworked_leftover_goes_before_the_filter_is_asked_in_the_forward_pass():
    """A forward operator with a skip connection reads an evicted tensor; the parent rebuilt
    for it is a leftover and must leave (DROP_TEMP) before Filter and Director release anything.
    Chain t0..t5 (m 4, cost 10; t0 never releasable), t6 = f(t2, t5).  B = 24, trigger 3/4
    (release while 4 (live + need) > 72), no link.
      step 4: 4*20 > 72; t1 (s = 10) beats t2 (s = 0): Evict t1.  step 5: Evict t2
        (s = 10; c_r = 10 + 10 for the missing t1).
      step 6 reads t2: rebuild t1 (live 20), t2 (live 24); t1 is read again by the backward
        pass, so it stays as a leftover.  Then the trigger: 4*(24 + 4) > 72: the leftover t1
        goes first; 4*24 > 72 still: now the Filter: t3 (m*s = 4*30) beats t4 (4*20): Evict
        t3, then Evict t4 (4*20 > 72 still); 4*16 <= 72 stops it.
      backward: 7 [2,5,6], 8 [4,5] rebuilds t3 (leftover, read at 9) and t4, 9 [3,4],
        10 [2,3], 11 [1,2] rebuilds t1, 12 [0,1].
    Mutation: skipping the `if prov:` branch of step() makes the Filter evict t1 (m*s = 4*50)
    as an ordinary EVICT."""
    both = pl.EVICT_PINNED | pl.OFFLOAD_PINNED
    tensors = [T(4, 1, (), both)] + [T(4, 10, (i - 1,)) for i in range(1, 6)] + [T(4, 10, (2, 5))]
    steps = [dict(produces=0, reads=[], cost_ns=1)]
    steps += [dict(produces=i, reads=list(tensors[i]["parents"]), cost_ns=10) for i in range(1, 7)]
    steps += [dict(produces=-1, reads=r, cost_ns=20)
              for r in ([2, 5, 6], [4, 5], [3, 4], [2, 3], [1, 2], [0, 1])]
    p = pl.default_params(24, 7, bw_d2h_Bps=0, bw_h2d_Bps=0)
    ev, peak = pl.plan(tensors, steps, p)
    assert names(ev) == [
        (4, "EVICT", 1), (5, "EVICT", 2),
        (6, "RECOMPUTE", 1), (6, "RECOMPUTE", 2), (6, "DROP_TEMP", 1), (6, "EVICT", 3), (6, "EVICT", 4),
        (7, "FREE", 6), (8, "RECOMPUTE", 3), (8, "RECOMPUTE", 4), (8, "FREE", 5), (9, "FREE", 4),
        (10, "FREE", 3), (11, "RECOMPUTE", 1), (11, "FREE", 2), (12, "FREE", 0), (12, "FREE", 1)]
    assert peak == 24
    checker.check(tensors, steps, p, ev)


def _offloaded_chain(sizes, budget, num, den):
    """Chain t0..t5 with the given sizes and an effectively infinite link, so that every release is
    an Offload (c_s = 2 ns); the early trigger num/den makes the forward pass offload t0, t1, t2
    while the budget leaves the backward pass room to bring them back."""
    tensors, steps, n_fwd = chain(6)
    for t, m in zip(tensors, sizes):
        t["bytes"] = m
    return tensors, steps, pl.default_params(budget, n_fwd, trigger_num=num, trigger_den=den,
                                             bw_d2h_Bps=10**18, bw_h2d_Bps=10**18)


def test_handworked_prefetcher_window_admits_two_and_n_caps():
    """Algorithm 4 with three queued tensors.  Chain of six, m = 4, B = 24, trigger 1/2: the
    forward pass releases while live + need > 12, exactly as with a budget of 12: t0 at step 3
    (uncomputable), t1 at step 4 (c_r = 10 + 1 > c_s = 2), t2 at step 5 -- all Offload.
    The queue, by next use: t2 (step 8), t1 (9), t0 (10).  Backward steps 6 [4,5], 7 [3,4],
    8 [2,3], 9 [1,2], 10 [0,1]; live is 12 when the backward pass starts.
      d = 3, n = 2: step 6 sees uses up to step 9: t2 and t1 come back (live 20), t0 (step 10)
        is outside the window; step 7: t0.
      d = 4, n = 1: the window would admit t2 and t1 at step 6 and both fit, but one reload
        per step: t2 at 6, t1 at 7, t0 at 8.
    Mutations: dropping `issued < n` (two reloads at step 6 of the second case); `nr > k + d`
    -> `nr >= k + d` (t1 waits for step 7 in the first case)."""
    tensors, steps, p = _offloaded_chain([4] * 6, 24, 1, 2)
    fwd = [(3, "OFFLOAD", 0), (4, "OFFLOAD", 1), (5, "OFFLOAD", 2)]
    frees = {6: 5, 7: 4, 8: 3, 9: 2}
    ev, peak = pl.plan(tensors, steps, dict(p, prefetch_distance=3, max_reloads=2))
    assert names(ev) == fwd + [
        (6, "RELOAD_PREFETCH", 2), (6, "RELOAD_PREFETCH", 1), (6, "FREE", 5),
        (7, "RELOAD_PREFETCH", 0), (7, "FREE", 4), (8, "FREE", 3), (9, "FREE", 2),
        (10, "FREE", 0), (10, "FREE", 1)]
    assert peak == 20
    checker.check(tensors, steps, dict(p, prefetch_distance=3, max_reloads=2), ev)
    ev, peak = pl.plan(tensors, steps, dict(p, prefetch_distance=4, max_reloads=1))
    assert names(ev) == fwd + [
        (6, "RELOAD_PREFETCH", 2), (6, "FREE", 5), (7, "RELOAD_PREFETCH", 1), (7, "FREE", 4),
        (8, "RELOAD_PREFETCH", 0), (8, "FREE", 3), (9, "FREE", 2), (10, "FREE", 0), (10, "FREE", 1)]
    assert peak == 16 and frees
    checker.check(tensors, steps, dict(p, prefetch_distance=4, max_reloads=1), ev)


def test_handworked_prefetcher_stops_at_a_head_that_does_not_fit():
    """The head of the queue blocks what stands behind it.  Sizes 4, 4, 12, 4, 4, 4; B = 20,
    trigger 3/5 (release while live + need > 12).  Forward: step 2 (t2 needs 12, live 8):
    only t0 may go (Offload), then nothing is left and 16 <= 20 is allowed; step 3: Offload t1;
    step 4: Offload t2 (c_r = 10 + 10 + 1 > 2).  Backward starts with t3, t4, t5 = 12 bytes.
    d = 4, n = 3.  step 6: the head t2 (12 bytes, used at step 8) does not fit (24 > 20), and
    although t1 (4 bytes, used at step 9, inside the window) would, nothing is reloaded.
    step 7 (live 8): t2 fits exactly; t1 no longer does.  step 8: t1; step 9: t0.
    Mutation: `break` -> skip to the next queued tensor reloads t1 at step 6."""
    tensors, steps, p = _offloaded_chain([4, 4, 12, 4, 4, 4], 20, 3, 5)
    p = dict(p, prefetch_distance=4, max_reloads=3)
    ev, peak = pl.plan(tensors, steps, p)
    assert names(ev) == [
        (2, "OFFLOAD", 0), (3, "OFFLOAD", 1), (4, "OFFLOAD", 2), (6, "FREE", 5),
        (7, "RELOAD_PREFETCH", 2), (7, "FREE", 4), (8, "RELOAD_PREFETCH", 1), (8, "FREE", 3),
        (9, "RELOAD_PREFETCH", 0), (9, "FREE", 2), (10, "FREE", 0), (10, "FREE", 1)]
    assert peak == 20
    checker.check(tensors, steps, p, ev)


def test_handworked_demand_reload_of_an_uncomputable_parent_inside_a_recomputation():
    """The first hand-worked chain with the Prefetcher switched off (n = 0): at step 7 the
    evicted t1 is rebuilt, its parent t0 is offloaded and cannot be recomputed, so it comes
    back by a demand reload inside the recomputation (Algorithm 1: Reload when uncomputable),
    and stays because step 8 reads it.  When step 8 reads t1 only, t0 is dead after step 1, is
    freed there and never offloaded, so the rebuild of t1 at step 7 has no way to get its
    parent: the plan fails at step 7.
    Mutation: raising on an uncomputable parent, or recomputing it, changes event (7, ., 0)."""
    tensors, steps, n_fwd = chain(5)
    p = pl.default_params(12, n_fwd, trigger_num=1, trigger_den=1, bw_d2h_Bps=0, bw_h2d_Bps=0,
                          prefetch_distance=1, max_reloads=0)
    ev, peak = pl.plan(tensors, steps, p)
    assert names(ev) == [(3, "OFFLOAD", 0), (4, "EVICT", 1), (5, "FREE", 4), (6, "FREE", 3),
                         (7, "RELOAD_DEMAND", 0), (7, "RECOMPUTE", 1), (7, "FREE", 2),
                         (8, "FREE", 0), (8, "FREE", 1)]
    assert peak == 12
    checker.check(tensors, steps, p, ev)
    steps[8]["reads"] = [1]
    with pytest.raises(pl.Infeasible) as e:
        pl.plan(tensors, steps, p)
    assert e.value.step == 7


def _late_source_chain(n, extra):
    """chain(n), but `extra` backward steps that read t1 alone stand between the backward of layer 2
    and the one step that reads the source t0: its own next use lies far behind the recomputation
    that needs it."""
    tensors, steps, n_fwd = chain(n)
    steps = steps[:-1] + [dict(produces=-1, reads=[1], cost_ns=20) for _ in range(extra)] + steps[-1:]
    return tensors, steps, n_fwd


def test_handworked_prefetch_for_a_recomputation_one_generation():
    """t0 (source, uncomputable) -> t1 -> ... -> t4, m = 4 each, B = 12 (three tensors), no link (every computable
    tensor is evicted, t0 can only be offloaded), release loop at B, d = n = 1.  Backward steps: 5 reads (t3, t4),
    6 (t2, t3), 7 (t1, t2), 8 and 9 t1 alone, 10 (t0, t1).
    Forward: step 3 needs room: t0 (staleness 10) against t1 (0): OFFLOAD t0; step 4: t1 (10) against t2 (0): EVICT t1.
    Algorithm 4 as printed looks at t0's own next read, step 10: nothing is prefetched before step 9, and at step 7
    the recomputation of t1 reloads t0 on demand.  With prefetch_rebuild_reads t0 is wanted at step 7 - t1 is neither on
    the GPU nor in host memory, step 7 reads it, its recomputation accesses t0 - so it is prefetched at step 6 = 7 - d
    (8 bytes in use + 4 fit), and step 7 recomputes t1 without a reload.
    Mutation: looking at own reads only moves the reload to (7, RELOAD_DEMAND, 0)."""
    tensors, steps, n_fwd = _late_source_chain(5, 2)
    p = pl.default_params(12, n_fwd, trigger_num=1, trigger_den=1, bw_d2h_Bps=0, bw_h2d_Bps=0,
                          prefetch_distance=1, max_reloads=1)
    ev, peak = pl.plan(tensors, steps, p)
    assert names(ev) == [(3, "OFFLOAD", 0), (4, "EVICT", 1), (5, "FREE", 4), (6, "FREE", 3),
                         (7, "RELOAD_DEMAND", 0), (7, "RECOMPUTE", 1), (7, "FREE", 2),
                         (10, "FREE", 0), (10, "FREE", 1)]
    checker.check(tensors, steps, p, ev)
    p = dict(p, prefetch_rebuild_reads=1)
    ev, peak = pl.plan(tensors, steps, p)
    assert names(ev) == [(3, "OFFLOAD", 0), (4, "EVICT", 1), (5, "FREE", 4), (6, "RELOAD_PREFETCH", 0),
                         (6, "FREE", 3), (7, "RECOMPUTE", 1), (7, "FREE", 2), (10, "FREE", 0), (10, "FREE", 1)]
    assert peak == 12
    checker.check(tensors, steps, p, ev)
    with pytest.raises(checker.PlanError):               # the same events are outside Algorithm 4's own window
        checker.check(tensors, steps, dict(p, prefetch_rebuild_reads=0), ev)


def test_handworked_prefetch_for_a_recomputation_two_generations_and_it_is_a_leftover():
    """The same with six tensors: forward OFFLOAD t0 (step 3), EVICT t1 (4), EVICT t2 (5).  Backward: 6 reads
    (t4, t5), 7 (t3, t4), 8 (t2, t3), 9 (t1, t2), 10 t1 alone, 11 (t0, t1).
    Step 8 reads t2, which is gone; its recomputation accesses t1, gone as well, whose recomputation accesses t0:
    t0 is wanted at step 8 and prefetched at step 7 (8 bytes in use + 4 fit).  It is back for a recomputation, not
    for a step of its own, so it is a leftover: at step 8, after t1 is rebuilt (12 bytes in use), the allocation of
    t2 does not fit and t0 - not an operand of the recomputation still in progress - gives way (DROP_TEMP, as after a
    demand reload), t1 stays as a leftover for step 9, and t0 returns at step 10 for its own read at step 11.
    Mutation: stopping at the first generation (t1's own read is step 9) prefetches nothing at step 7 and reloads
    on demand at step 8; not marking the prefetched tensor a leftover makes step 8 infeasible."""
    tensors, steps, n_fwd = _late_source_chain(6, 1)
    p = pl.default_params(12, n_fwd, trigger_num=1, trigger_den=1, bw_d2h_Bps=0, bw_h2d_Bps=0,
                          prefetch_distance=1, max_reloads=1, prefetch_rebuild_reads=1)
    ev, peak = pl.plan(tensors, steps, p)
    assert names(ev) == [(3, "OFFLOAD", 0), (4, "EVICT", 1), (5, "EVICT", 2), (6, "FREE", 5),
                         (7, "RELOAD_PREFETCH", 0), (7, "FREE", 4),
                         (8, "RECOMPUTE", 1), (8, "DROP_TEMP", 0), (8, "RECOMPUTE", 2), (8, "FREE", 3),
                         (9, "FREE", 2), (10, "RELOAD_PREFETCH", 0), (11, "FREE", 0), (11, "FREE", 1)]
    assert peak == 12
    checker.check(tensors, steps, p, ev)
    ev0, _ = pl.plan(tensors, steps, dict(p, prefetch_rebuild_reads=0))
    assert (8, "RELOAD_DEMAND", 0) in names(ev0) and (7, "RELOAD_PREFETCH", 0) not in names(ev0)


def test_handworked_release_when_memory_is_short_in_the_backward_pass():
    """Algorithm 1 taken literally (release_when_short): its release loop also runs when an
    allocation of the backward pass does not fit.  t0 (m 4, cost 5) -> t1 -> t2 -> t3 (m 8,
    cost 10); backward steps 4 [0,2], 5 [2,3], 6 [0,3], 7 [3]; B = 16, trigger 1/1, no link.
      step 2: t0 is the only tensor free to go: Evict; t1 dies.  step 3 fills the budget.
      step 4 needs t0 back (4 bytes, live 16): no leftover to drop; the only resident tensor
        that the step does not use and that is read later is t3: Evict t3, Recompute t0.
      step 5 needs t3 back (8 bytes, live 12): t0 (read again at 6) goes: Evict, Recompute t3.
      step 6: Recompute t0.
    With the switch off (Assumption 2 to the letter) step 4 cannot be planned."""
    tensors = [T(4, 5), T(8, 10, (0,)), T(8, 10, (1,)), T(8, 10, (2,))]
    steps = [dict(produces=0, reads=[], cost_ns=5)]
    steps += [dict(produces=i, reads=[i - 1], cost_ns=10) for i in (1, 2, 3)]
    steps += [dict(produces=-1, reads=r, cost_ns=20) for r in ([0, 2], [2, 3], [0, 3], [3])]
    p = pl.default_params(16, 4, trigger_num=1, trigger_den=1, bw_d2h_Bps=0, bw_h2d_Bps=0)
    with pytest.raises(pl.Infeasible) as e:
        pl.plan(tensors, steps, p)
    assert e.value.step == 4
    p = dict(p, release_when_short=1)
    ev, peak = pl.plan(tensors, steps, p)
    assert names(ev) == [(2, "EVICT", 0), (2, "FREE", 1), (4, "EVICT", 3), (4, "RECOMPUTE", 0),
                         (5, "EVICT", 0), (5, "RECOMPUTE", 3), (5, "FREE", 2),
                         (6, "RECOMPUTE", 0), (6, "FREE", 0), (7, "FREE", 3)]
    assert peak == 16
    checker.check(tensors, steps, p, ev)
    with pytest.raises(checker.PlanError):          # the same events are no plan under Assumption 2
        checker.check(tensors, steps, dict(p, release_when_short=0), ev)
    # a release in the backward pass that no allocation needs is refused even with the switch on
    big = dict(p, budget_bytes=64)
    evb, _ = pl.plan(tensors, steps, big)
    bad = sorted(evb + [(5, pl.EV_EVICT, 0)], key=lambda x: (x[0], x[1] == pl.EV_FREE))
    with pytest.raises(checker.PlanError):
        checker.check(tensors, steps, big, bad)


def test_handworked_repair_round_makes_the_failing_operand_offload_only():
    """repair_rounds (our addition): t0 (m 4) -> t1 (m 8) -> t2 (m 4) -> t3 (m 8); backward
    steps 4 [1], 5 [1,3]; B = 16, trigger 1/1, no link, Prefetcher off.
    First pass: t0 dies at step 1; step 3 evicts t1 (the only tensor free to go), t2 dies.
    Step 4 must rebuild t1, which first rebuilds t0 (live 8 + 4), and then t1's 8 bytes do not
    fit: the plan fails with t1 as the operand that could not be brought back.
    Second pass: t1 counts as uncomputable, so step 3 offloads it and step 4 reloads it (8
    bytes fit beside t3)."""
    tensors = [T(4, 5), T(8, 10, (0,)), T(4, 10, (1,)), T(8, 10, (2,))]
    steps = [dict(produces=0, reads=[], cost_ns=5)]
    steps += [dict(produces=i, reads=[i - 1], cost_ns=10) for i in (1, 2, 3)]
    steps += [dict(produces=-1, reads=r, cost_ns=20) for r in ([1], [1, 3])]
    p = pl.default_params(16, 4, trigger_num=1, trigger_den=1, bw_d2h_Bps=0, bw_h2d_Bps=0,
                          max_reloads=0)
    with pytest.raises(pl.Infeasible) as e:
        pl.plan(tensors, steps, p)
    assert e.value.step == 4 and e.value.operand == 1
    p = dict(p, repair_rounds=1)
    ev, peak, learned = pl.plan_with_pins(tensors, steps, p)
    assert learned == [1]
    assert names(ev) == [(1, "FREE", 0), (3, "OFFLOAD", 1), (3, "FREE", 2),
                         (4, "RELOAD_DEMAND", 1), (5, "FREE", 1), (5, "FREE", 3)]
    assert peak == 16
    checker.check(tensors, steps, p, ev)


@pytest.mark.parametrize("frac", [0.6, 0.55, 0.5, 0.45, 0.4])
def test_config2_plans_wherever_a_static_plan_exists(frac):
    """The conv2_x stage (config 2): the exhaustive search finds a static plan at every one of
    these budgets.  The single greedy pass does not below 60 % (it evicts b2.a1 and b1.out, and
    rebuilding b2.a2 then needs b1.a2 + b1.sc + b1.out next to the locked b2.out: 167 MB); with
    repair rounds the heuristic plans all of them.  The gap to the optimum is printed."""
    g = synth.config_graph(2)
    B = int(frac * g.total_bytes())
    p = pl.default_params(B, g.n_fwd, repair_rounds=8)
    o = brute.optimum(g.tensors, g.steps, p)
    assert o is not None
    if frac < 0.6:
        with pytest.raises(pl.Infeasible):
            pl.plan(g.tensors, g.steps, dict(p, repair_rounds=0))
        with pytest.raises(pl.Infeasible):          # the literal reading of Algorithm 1 alone does not help
            pl.plan(g.tensors, g.steps, dict(p, repair_rounds=0, release_when_short=1))
    ev, peak, learned = pl.plan_with_pins(g.tensors, g.steps, p)
    st = checker.check(g.tensors, g.steps, p, ev)
    assert st["peak"] == peak <= B
    print("config 2 at %.0f %%: heuristic %d ns (offload-only: %s), static optimum %d ns"
          % (100 * frac, st["cost_ns"], [g.tensors[t]["name"] for t in learned], o["cost"]))


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


def test_handworked_recomputation_follows_the_tensor_parents_not_the_forward_reads():
    """A tensor's parents say what its recomputation reads; they need not be what its forward step read (a kernel that
    regenerates t2 from t0 directly, while the forward step of t2 read t1).  t0 (source) -> ... -> t5, m = 4, B = 12,
    no link, release loop at B, no prefetch.  Forward, as with per-layer parents: OFFLOAD t0 (step 3), EVICT t1 (4),
    EVICT t2 (5).  Backward: 6 reads (t4, t5), 7 (t3, t4), 8 (t2, t3), 9 (t1, t2), 10 (t0, t1).
    Per-layer parents: step 8 rebuilds t2 through t1: t0 back on demand, t1 recomputed (12 bytes in use), t0 gives way
    for t2 (DROP_TEMP), t1 stays for step 9, and step 10 reloads t0 once more.
    t2's parents = (t0): step 8 reloads t0 and recomputes t2 from it (t3, t0, t2 = 12 bytes: nothing gives way), t0
    stays because step 10 reads it, step 9 recomputes t1 from it, and there is no second reload.
    Mutation: following the forward step's reads in the recomputation gives the first event list for both graphs."""
    tensors, steps, n_fwd = chain(6)
    p = pl.default_params(12, n_fwd, trigger_num=1, trigger_den=1, bw_d2h_Bps=0, bw_h2d_Bps=0,
                          prefetch_distance=1, max_reloads=0)
    ev, peak = pl.plan(tensors, steps, p)
    assert names(ev) == [(3, "OFFLOAD", 0), (4, "EVICT", 1), (5, "EVICT", 2), (6, "FREE", 5), (7, "FREE", 4),
                         (8, "RELOAD_DEMAND", 0), (8, "RECOMPUTE", 1), (8, "DROP_TEMP", 0), (8, "RECOMPUTE", 2),
                         (8, "FREE", 3), (9, "FREE", 2), (10, "RELOAD_DEMAND", 0), (10, "FREE", 0), (10, "FREE", 1)]
    assert peak == 12
    checker.check(tensors, steps, p, ev)
    tensors[2] = dict(tensors[2], parents=[0])
    assert steps[2]["reads"] == [1]
    ev, peak = pl.plan(tensors, steps, p)
    assert names(ev) == [(3, "OFFLOAD", 0), (4, "EVICT", 1), (5, "EVICT", 2), (6, "FREE", 5), (7, "FREE", 4),
                         (8, "RELOAD_DEMAND", 0), (8, "RECOMPUTE", 2), (8, "FREE", 3),
                         (9, "RECOMPUTE", 1), (9, "FREE", 2), (10, "FREE", 0), (10, "FREE", 1)]
    assert peak == 12
    checker.check(tensors, steps, p, ev)
