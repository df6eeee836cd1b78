"""CPU oracle: independent plan checker.

TEST INFRASTRUCTURE ONLY.  Replays any event list against the graph and fails
on the first violated rule.  It knows nothing about how a plan was produced, so
it pins the planners to what the paper fixes:

  * the budget: live activation bytes never exceed B (DELTA Sec. 5.1, budget);
  * the early start: before a forward operator runs, either at most 3/4 of B is
    in use or nothing releasable was left (Algorithm 1 and Sec. 4.3);
  * Assumption 2: no Evict/Offload once the forward pass is over -- or, when the plan was
    made with release_when_short (Algorithm 1 taken literally), only where the allocation
    that follows in the same step would not fit without it;
  * Table 1 semantics: Recompute needs every parent on the GPU, Reload needs a
    host copy made by an earlier Offload, Evict/Offload need a resident tensor;
  * pins (Sec. 4.3 flag meanings): evict_pinned/uncomputable tensors are never
    evicted, offload_pinned never offloaded;
  * every operand of every step is resident when the step runs;
  * DROP_TEMP only removes a tensor that is on the GPU as a leftover operand of a
    recomputation and that no step has read since (it is not a Release).
"""
from .planner import (EV_DROP_TEMP, EV_EVICT, EV_FREE, EV_OFFLOAD, EV_RECOMPUTE,
                      EV_RELOAD_DEMAND, EV_RELOAD_PREFETCH, EVICT_PINNED, OFFLOAD_PINNED,
                      UNCOMPUTABLE, transfer_ns)


class PlanError(AssertionError):
    pass


def check(tensors, steps, params, events, check_trigger=True, check_prefetch_window=True):
    """Returns a dict of statistics (peak, counts, modelled cost).  Raises PlanError."""
    B = params["budget_bytes"]
    n_fwd = params["n_fwd_steps"]
    nT = len(tensors)
    last_read = [-1] * nT
    for k, st in enumerate(steps):
        for t in st["reads"]:
            last_read[t] = k
    children = [[] for _ in range(nT)]
    for c, tc in enumerate(tensors):
        for q in tc["parents"]:
            children[q].append(c)
    resident = [False] * nT
    host = [False] * nT
    provisional = [False] * nT      # on the GPU only as a leftover operand of a recomputation
    live = peak = 0
    stats = dict(peak=0, evict=0, offload=0, recompute=0, reload_prefetch=0, reload_demand=0,
                 free=0, drop_temp=0, recompute_ns=0, d2h_bytes=0, h2d_bytes=0, cost_ns=0)

    def fail(k, msg):
        raise PlanError("step %d: %s" % (k, msg))

    def wanted(t, k, seen):
        """First step >= k that reads t; with prefetch_rebuild_reads also through the recomputation of
        a tensor that is on neither side of the link (such a tensor is rebuilt from its parents)."""
        first = min([s for s in range(k, len(steps)) if t in steps[s]["reads"]], default=None)
        if params.get("prefetch_rebuild_reads") and t not in seen:
            seen = seen | {t}
            for c in children[t]:
                if not resident[c] and not host[c] and not (tensors[c]["flags"] & UNCOMPUTABLE):
                    u = wanted(c, k, seen)
                    if u is not None and (first is None or u < first):
                        first = u
        return first

    by_step = [[] for _ in steps]
    prev = 0
    for (k, a, t) in events:
        if not (0 <= k < len(steps)) or k < prev:
            fail(k, "events out of step order")
        if not (0 <= t < nT):
            fail(k, "bad tensor id %d" % t)
        prev = k
        by_step[k].append((a, t))

    for k, st in enumerate(steps):
        fwd = k < n_fwd
        locked = set(st["reads"]) | ({st["produces"]} if st["produces"] >= 0 else set())
        prefetched = 0
        ev = by_step[k]
        pre = [e for e in ev if e[0] != EV_FREE]
        post = [e for e in ev if e[0] == EV_FREE]
        if ev != pre + post:
            fail(k, "FREE must follow every other event of the step")
        for i, (a, t) in enumerate(pre):
            m = tensors[t]["bytes"]
            fl = tensors[t]["flags"]
            if a in (EV_EVICT, EV_OFFLOAD):
                if not fwd:
                    if not params.get("release_when_short"):
                        fail(k, "release of %d in the backward pass" % t)
                    nxt = [tensors[u]["bytes"] for (b, u) in pre[i + 1:]
                           if b in (EV_RECOMPUTE, EV_RELOAD_DEMAND)]
                    if not nxt or live + nxt[0] <= B:
                        fail(k, "release of %d in the backward pass without an allocation "
                                "that needs the room" % t)
                if not resident[t] or t in locked or provisional[t]:
                    fail(k, "release of non-resident, in-use or provisional tensor %d" % t)
                if a == EV_EVICT and fl & (EVICT_PINNED | UNCOMPUTABLE):
                    fail(k, "evicted a tensor that may only be offloaded: %d" % t)
                if a == EV_OFFLOAD and fl & OFFLOAD_PINNED:
                    fail(k, "offloaded a tensor that may only be evicted: %d" % t)
                resident[t] = False
                live -= m
                if a == EV_OFFLOAD:
                    if not host[t]:
                        stats["d2h_bytes"] += m
                        stats["cost_ns"] += transfer_ns(m, params["bw_d2h_Bps"])
                    host[t] = True
                    stats["offload"] += 1
                else:
                    host[t] = False
                    stats["evict"] += 1
            elif a == EV_RECOMPUTE:
                if resident[t] or fl & UNCOMPUTABLE:
                    fail(k, "recompute of resident or uncomputable tensor %d" % t)
                for p in tensors[t]["parents"]:
                    if not resident[p]:
                        fail(k, "recompute of %d with parent %d missing" % (t, p))
                resident[t] = True
                provisional[t] = t not in locked
                live += m
                stats["recompute"] += 1
                stats["recompute_ns"] += tensors[t]["cost_ns"]
                stats["cost_ns"] += tensors[t]["cost_ns"]
            elif a in (EV_RELOAD_PREFETCH, EV_RELOAD_DEMAND):
                if resident[t] or not host[t]:
                    fail(k, "reload of %d without a host copy (or already resident)" % t)
                if a == EV_RELOAD_PREFETCH:
                    prefetched += 1
                    if check_prefetch_window:
                        if fwd:
                            fail(k, "prefetch in the forward pass")
                        nxt = wanted(t, k, frozenset())
                        if nxt is None or nxt > k + params["prefetch_distance"]:
                            fail(k, "prefetch of %d outside the look-ahead window" % t)
                        if prefetched > params["max_reloads"]:
                            fail(k, "more than n prefetches in one step")
                        own = min([s for s in range(k, len(steps)) if t in steps[s]["reads"]], default=None)
                        if own is None or nxt < own:     # back for a recomputation: a leftover like the operands it reloads
                            provisional[t] = True
                    stats["reload_prefetch"] += 1
                else:
                    provisional[t] = t not in locked
                    stats["reload_demand"] += 1
                resident[t] = True
                live += m
                stats["h2d_bytes"] += m
                stats["cost_ns"] += transfer_ns(m, params["bw_h2d_Bps"])
            elif a == EV_DROP_TEMP:
                if not resident[t] or t in locked or not provisional[t]:
                    fail(k, "DROP_TEMP of %d, which is not a leftover of a recomputation" % t)
                if (fl & UNCOMPUTABLE) and not host[t]:
                    fail(k, "dropping %d would lose it" % t)
                resident[t] = False
                provisional[t] = False
                live -= m
                stats["drop_temp"] += 1
            else:
                fail(k, "unknown action %d" % a)
            if live > B:
                fail(k, "live %d exceeds budget %d" % (live, B))
            peak = max(peak, live)
        for t in st["reads"]:
            if not resident[t]:
                fail(k, "operand %d is not on the GPU" % t)
            provisional[t] = False
        need = tensors[st["produces"]]["bytes"] if st["produces"] >= 0 else 0
        if fwd and check_trigger:
            num, den = params["trigger_num"], params["trigger_den"]
            if den * (live + need) > num * B:
                for t in range(nT):
                    fl = tensors[t]["flags"]
                    pinned_both = (fl & (EVICT_PINNED | UNCOMPUTABLE)) and (fl & OFFLOAD_PINNED)
                    if (resident[t] and t not in locked and last_read[t] > k
                            and (provisional[t] or not pinned_both)):
                        fail(k, "over the trigger with releasable tensor %d left" % t)
        if st["produces"] >= 0:
            if resident[st["produces"]]:
                fail(k, "produced tensor already resident")
            resident[st["produces"]] = True
            live += need
            if live > B:
                fail(k, "live %d exceeds budget %d after allocation" % (live, B))
            peak = max(peak, live)
        for (a, t) in post:
            if not resident[t] or last_read[t] > k:
                fail(k, "FREE of %d that is absent or still needed" % t)
            resident[t] = False
            live -= tensors[t]["bytes"]
            stats["free"] += 1
        for t in range(nT):
            if resident[t] and last_read[t] <= k:
                # prefetch_rebuild_reads: a tensor may wait for the recomputation it was prefetched for
                if not (provisional[t] and wanted(t, k + 1, frozenset()) is not None):
                    fail(k, "dead tensor %d left on the GPU" % t)
    if live != 0:
        fail(len(steps) - 1, "memory not returned at the end")
    stats["peak"] = peak
    return stats
