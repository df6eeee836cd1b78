"""Planner-only sweep over Filter heuristics and budgets (DELTA Sec. 5.7, Fig. 7-8): for each
synthetic graph and each of base / LRU / GREEDY, plan at a grid of budgets with the library's
delta_plan and report what the plan does, plus the smallest budget each heuristic can still
plan for (bisection).  Then the analogue of the paper's maximum-batch tables (Sec. 5.3): under a
fixed number of bytes for activations, the largest batch whose whole-ResNet graph still fits
without any release, and the largest one the planner still finds a plan for (bisection over the
batch; every tensor and every cost grows linearly with it).  Needs no GPU.
Run: python -m paper_2203_15980_amd.sweep"""
import json
import sys

import synth

from . import binding as B

FILTERS = (("base", B.FILTER_BASE), ("lru", B.FILTER_LRU), ("greedy", B.FILTER_GREEDY))


def _params(budget, n_fwd, filt, bw=55 * 10**9, d=2):
    return dict(budget_bytes=int(budget), trigger_num=3, trigger_den=4, filter=filt, prefetch_distance=d,
                max_reloads=d, n_fwd_steps=n_fwd, bw_d2h_Bps=bw, bw_h2d_Bps=bw)


def describe(delta, graph, prepared, budget, filt):
    total_cost = sum(s["cost_ns"] for s in graph.steps)
    try:
        ev, peak = delta.plan(prepared, None, _params(budget, graph.n_fwd, filt))
    except B.DeltaError as e:
        if e.status != B.ERR_INFEASIBLE:
            raise
        return None
    cnt = {}
    rec_ns = off_bytes = 0
    for (_, a, t) in ev:
        cnt[a] = cnt.get(a, 0) + 1
        if a == B.EV_RECOMPUTE:
            rec_ns += graph.tensors[t]["cost_ns"]
        elif a == B.EV_OFFLOAD:
            off_bytes += graph.tensors[t]["bytes"]
    return dict(peak_frac=peak / graph.total_bytes(), evict=cnt.get(B.EV_EVICT, 0), offload=cnt.get(B.EV_OFFLOAD, 0),
                recompute=cnt.get(B.EV_RECOMPUTE, 0), reload=cnt.get(B.EV_RELOAD_PREFETCH, 0) + cnt.get(B.EV_RELOAD_DEMAND, 0),
                recompute_cost_frac=rec_ns / total_cost, offload_bytes=off_bytes)


def min_budget(delta, graph, prepared, filt):
    """Smallest budget (as a fraction of all activation bytes, to 1/256) that still plans."""
    lo, hi = 0, 256
    total = graph.total_bytes()
    while hi - lo > 1:
        mid = (lo + hi) // 2
        if describe(delta, graph, prepared, total * mid // 256, filt) is None:
            lo = mid
        else:
            hi = mid
    return hi / 256.0


def max_batch(delta, depths, arena_bytes, filt=B.FILTER_BASE, hi=1 << 14):
    """Largest batch of the fused ResNet graph (bf16, 224 x 224, with loss) that fits `arena_bytes`
    of activations: (without releasing anything, with a plan).  A batch "fits" without releases when
    the peak of the unconstrained plan is within the arena; with releases when delta_plan succeeds
    at budget = arena."""
    def fits(n, release):
        g = synth.fused_graph(synth.resnet_layers(n, depths), "bf16", with_loss=True)
        try:
            _, peak = delta.plan(g.tensors, g.steps, _params(arena_bytes if release else 10**15, g.n_fwd, filt))
        except B.DeltaError as e:
            if e.status != B.ERR_INFEASIBLE:
                raise
            return False
        return peak <= arena_bytes

    out = []
    for release in (False, True):
        lo, top = 0, hi                            # lo fits (0 = nothing), top does not
        if fits(top, release):
            out.append(top)
            continue
        while top - lo > 1:
            mid = (lo + top) // 2
            if fits(mid, release):
                lo = mid
            else:
                top = mid
        out.append(lo)
    return tuple(out)


def run_max_batch(arenas_gib=(8, 16, 32), nets=(("resnet50", (3, 4, 6, 3)), ("resnet101", (3, 4, 23, 3)))):
    delta = B.Delta()
    out = {}
    for name, depths in nets:
        for gib in arenas_gib:
            plain, planned = max_batch(delta, depths, gib << 30)
            out["%s@%dGiB" % (name, gib)] = {"no_release": plain, "planned": planned,
                                            "ratio": planned / plain if plain else None}
    delta.close()
    return out


def run(configs=(3, 4, 5), fracs=(0.8, 0.6, 0.5, 0.4, 0.3, 0.25)):
    delta = B.Delta()
    out = {}
    for cfg in configs:
        g = synth.config_graph(cfg)
        prepared = delta.prepare_graph(g.tensors, g.steps)
        rows = {}
        for name, filt in FILTERS:
            rows[name] = {"min_budget_frac": min_budget(delta, g, prepared, filt),
                          "at": {str(f): describe(delta, g, prepared, int(g.total_bytes() * f), filt) for f in fracs}}
        out["config%d" % cfg] = rows
    delta.close()
    return out


def main():
    res = run()
    for cfg, rows in res.items():
        print(cfg)
        for name, r in rows.items():
            print("  %-6s smallest plannable budget %.3f of the activation bytes" % (name, r["min_budget_frac"]))
            for f, dsc in r["at"].items():
                if dsc is None:
                    print("     %4s  infeasible" % f)
                else:
                    print("     %4s  peak %.3f  evict %3d  offload %3d  recompute %3d  reload %3d  "
                          "recompute cost %.3f of step  offloaded %.2f GB"
                          % (f, dsc["peak_frac"], dsc["evict"], dsc["offload"], dsc["recompute"], dsc["reload"],
                             dsc["recompute_cost_frac"], dsc["offload_bytes"] / 1e9))
    mb = run_max_batch()
    print("largest batch under a fixed number of activation bytes (fused graph, bf16, base Filter)")
    for key, r in mb.items():
        print("  %-18s no release %5d   planned %5d   x%.2f" % (key, r["no_release"], r["planned"], r["ratio"]))
    if "--json" in sys.argv:
        print(json.dumps({"sweep": res, "max_batch": mb}))


if __name__ == "__main__":
    main()
