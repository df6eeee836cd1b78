"""CPU oracle: exhaustive search over static plans on small graphs (<= 12 tensors).

TEST INFRASTRUCTURE ONLY.  The paper gives no objective for an "optimal plan";
the class searched here is the one its Table 1 actions and Assumption 2 allow
once every decision is fixed ahead of time:

  * each tensor is KEEP, EVICT or OFFLOAD (respecting the pin flags);
  * a released tensor leaves the GPU right after its last forward read (or
    right after it is produced when the forward pass never reads it) -- never
    during the backward pass (Assumption 2);
  * it comes back at its first backward read: EVICT by recomputation, which
    first brings in missing parents; OFFLOAD by reload.  A missing operand of a
    recomputation is reloaded when a host copy exists and recomputed otherwise.
    Rebuilt operands that a later step reads stay while they fit and give way
    (farthest next use first) when an allocation needs the room; those nobody
    reads are dropped at once;
  * feasible iff live bytes <= B at every moment;
  * cost = sum of recompute costs paid + offload (D2H) times + reload (H2D)
    times, i.e. c_r at the time of need for EVICT and c_s for OFFLOAD (Sec. 3).

The optimum is the cheapest feasible vector; ties go to the lexicographically
smallest vector with KEEP < EVICT < OFFLOAD.  This validates the memory and
cost model that planner.py and checker.py share with it only by definition,
not by code: brute.py imports nothing but the event codes.
"""
import itertools

from .planner import (EV_DROP_TEMP, EV_EVICT, EV_FREE, EV_OFFLOAD, EV_RECOMPUTE, EV_RELOAD_DEMAND,
                      EVICT_PINNED, OFFLOAD_PINNED, UNCOMPUTABLE, transfer_ns)

KEEP, EVICT, OFFLOAD = 0, 1, 2


def choices(tensors, steps, n_fwd):
    """Allowed decisions per tensor."""
    out = []
    for t, d in enumerate(tensors):
        fr = [k for k, st in enumerate(steps) if t in st["reads"] and k < n_fwd]
        br = [k for k, st in enumerate(steps) if t in st["reads"] and k >= n_fwd]
        prod = [k for k, st in enumerate(steps) if st["produces"] == t][0]
        rel_at = (max(fr) if fr else prod) + 1          # first step that no longer sees it
        opts = [KEEP]
        if br and rel_at < n_fwd:
            f = d["flags"]
            if not f & (EVICT_PINNED | UNCOMPUTABLE):
                opts.append(EVICT)
            if not f & OFFLOAD_PINNED:
                opts.append(OFFLOAD)
        out.append(opts)
    return out


def simulate(tensors, steps, params, vec):
    """Returns (cost_ns, peak, events) for a decision vector, or None when infeasible."""
    B, n_fwd = params["budget_bytes"], params["n_fwd_steps"]
    nT = len(tensors)
    last_read = [-1] * nT
    last_fwd_read = [-1] * nT
    for k, st in enumerate(steps):
        for t in st["reads"]:
            last_read[t] = k
            if k < n_fwd:
                last_fwd_read[t] = k
    produced_at = {st["produces"]: k for k, st in enumerate(steps) if st["produces"] >= 0}
    release_at = [[] for _ in steps]
    for t in range(nT):
        if vec[t] != KEEP:
            release_at[max(last_fwd_read[t], produced_at[t]) + 1].append(t)
    resident = [False] * nT
    host = [False] * nT
    state = dict(live=0, peak=0, cost=0)
    events = []

    class Over(Exception):
        pass

    reads_of = [[k for k, st in enumerate(steps) if t in st["reads"]] for t in range(nT)]
    provisional = [False] * nT
    held = []                         # parent lists of the recomputations in progress

    def next_use(t, k):
        return min((s for s in reads_of[t] if s >= k), default=None)

    def grow(k, m, locked):
        while state["live"] + m > B:
            # leftovers of earlier recomputations go first, farthest next use first
            c = [(next_use(t, k), -t) for t in range(nT)
                 if provisional[t] and t not in locked and not any(t in h for h in held)]
            if not c:
                raise Over()
            v = -max(c)[1]
            events.append((k, EV_DROP_TEMP, v))
            resident[v] = provisional[v] = False
            state["live"] -= tensors[v]["bytes"]
        state["live"] += m
        state["peak"] = max(state["peak"], state["live"])

    def bring(k, t, locked):
        """Make t resident for a recomputation or a read."""
        if host[t]:
            grow(k, tensors[t]["bytes"], locked)
            events.append((k, EV_RELOAD_DEMAND, t))
            state["cost"] += transfer_ns(tensors[t]["bytes"], params["bw_h2d_Bps"])
        elif not tensors[t]["flags"] & UNCOMPUTABLE:
            temps = []
            held.append(tensors[t]["parents"])
            for p in tensors[t]["parents"]:
                if not resident[p]:
                    bring(k, p, locked)
                    temps.append(p)
            grow(k, tensors[t]["bytes"], locked)
            events.append((k, EV_RECOMPUTE, t))
            state["cost"] += tensors[t]["cost_ns"]
            held.pop()
            for p in temps:
                if p in locked:
                    continue
                if next_use(p, k + 1) is None:
                    events.append((k, EV_DROP_TEMP, p))
                    resident[p] = False
                    state["live"] -= tensors[p]["bytes"]
                else:
                    provisional[p] = True      # a later step reads it: keep while it fits
        else:
            raise Over()
        resident[t] = True

    try:
        for k, st in enumerate(steps):
            for t in release_at[k]:
                if vec[t] == EVICT:
                    events.append((k, EV_EVICT, t))
                else:
                    events.append((k, EV_OFFLOAD, t))
                    host[t] = True
                    state["cost"] += transfer_ns(tensors[t]["bytes"], params["bw_d2h_Bps"])
                resident[t] = False
                state["live"] -= tensors[t]["bytes"]
            locked = set(st["reads"])
            for t in st["reads"]:
                if not resident[t]:
                    bring(k, t, locked)
                provisional[t] = False
            if st["produces"] >= 0:
                grow(k, tensors[st["produces"]]["bytes"], locked)
                resident[st["produces"]] = True
            touched = sorted(set(st["reads"]) | ({st["produces"]} if st["produces"] >= 0 else set()))
            for t in touched:
                if last_read[t] <= k and resident[t]:
                    events.append((k, EV_FREE, t))
                    resident[t] = provisional[t] = False
                    state["live"] -= tensors[t]["bytes"]
    except Over:
        return None
    return state["cost"], state["peak"], events


def optimum(tensors, steps, params):
    """Exhaustive search.  Returns dict(cost, vec, peak, events, searched) or None when no
    static plan fits the budget."""
    if len(tensors) > 12:
        raise ValueError("brute force is limited to 12 tensors")
    opts = choices(tensors, steps, params["n_fwd_steps"])
    best = None
    n = 0
    for vec in itertools.product(*opts):                 # lexicographic order
        n += 1
        r = simulate(tensors, steps, params, vec)
        if r is not None and (best is None or r[0] < best["cost"]):
            best = dict(cost=r[0], vec=vec, peak=r[1], events=r[2])
    if best is not None:
        best["searched"] = n
    return best
