"""CPU oracle, planner half: DELTA's main loop, Filter, Director and Prefetcher
simulated over a static operator trace.

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).  Pure Python integers, so
the 128-bit products the C++ planner needs are exact here for free.

The algorithm is a heuristic, so this follows the paper's steps in its order
and notation:

  * Main loop (DELTA Algorithm 1): on access, an evicted tensor is recomputed;
    an offloaded tensor that is not on the GPU is recomputed when it can be and
    reloaded otherwise; then, while three quarters of the budget is used or
    memory is short, Filter picks a tensor, Director picks Evict or Offload.
  * Filter (Algorithm 2, Eq. 1-3): the resident tensor with the minimum
    H = 1/(m*s) (base), 1/s (LRU) or 1/m (GREEDY), i.e. the maximum of m*s, s
    or m; ties go to the lowest id; s = 0 gives H = infinity (least preferred)
    without ever dividing.
  * Director (Algorithm 3, Eq. 4-6): evict_pinned -> Offload, offload_pinned ->
    Evict, otherwise F = h_r/h_o = c_r/c_s and F <= 1 -> Evict else Offload.
    c_s is the time to offload plus the time to reload (Sec. 3); c_r is the
    tensor's own cost plus that of its non-resident ancestors (Sec. 3, Eq. 5).
  * Prefetcher (Algorithm 4): reload the head of the offloaded queue while
    memory allows and fewer than n reloads have been issued.  With the parameter
    prefetch_rebuild_reads the "next use" that orders the queue and is held against
    the look-ahead also counts the accesses Algorithm 1 makes on the way to a
    recomputation: an offloaded tensor is needed as soon as a step reads a tensor
    that is neither on the GPU nor in host memory and whose recomputation reaches
    it through such tensors.  A tensor reloaded for that reason is a leftover of a
    recomputation like the operands a recomputation reloads itself (it gives way
    first when an allocation does not fit).
  * Assumption 2: no Evict/Offload after the last forward step -- unless the
    parameter release_when_short is set: then Algorithm 1 is taken literally
    (its release loop stands behind every access, and "memory is not enough" is
    one of its two conditions): whenever an allocation does not fit, in either
    pass, and no leftover of a recomputation can give way, Filter and Director
    release resident tensors that the running step and the recomputations in
    progress do not use.  The early 3/4 trigger stays a forward-pass rule.

Readings taken where the paper is silent (each listed in the design notes):
logical clock = sum of executed operator costs; queue ordered by next use;
prefetch guard is "and"; release stops at 3/4 of the budget or when no candidate
is left, failing only above the full budget; parents rebuilt only as operands of a
recomputation stay on the GPU as provisional tensors while a later step still
reads them, and are the first to go (DROP_TEMP, farthest next use first) when
an allocation does not fit or the 3/4 trigger fires.

Pins (tests/test_oracle_planner.py): Table 5 cost pairs give Evict; pin flags
override; b = 0 gives all Evict, huge b all Offload; tie gives Evict; equal m
makes base = LRU, equal s makes base = GREEDY; closed-form victim order on a
chain; budget >= 4/3 of the peak gives an empty plan; every plan passes the
independent checker (oracle/checker.py); brute force on <= 12 tensors
(oracle/brute.py) bounds the plan cost from below.  The greedy sequence beyond
those cases has no printed example in the paper: parity unpinned.
"""

UNCOMPUTABLE, EVICT_PINNED, OFFLOAD_PINNED = 1, 2, 4
FILTER_BASE, FILTER_LRU, FILTER_GREEDY = 0, 1, 2
EV_EVICT, EV_OFFLOAD, EV_RECOMPUTE, EV_RELOAD_PREFETCH = 1, 2, 3, 4
EV_RELOAD_DEMAND, EV_FREE, EV_DROP_TEMP = 5, 6, 7
EVENT_NAMES = {1: "EVICT", 2: "OFFLOAD", 3: "RECOMPUTE", 4: "RELOAD_PREFETCH",
               5: "RELOAD_DEMAND", 6: "FREE", 7: "DROP_TEMP"}
U64_MAX = (1 << 64) - 1


class Infeasible(Exception):
    """The budget cannot hold what one step needs.  `operand` is the operand of the step whose
    way back onto the GPU (recomputation with its missing ancestors, or reload) did not fit;
    None when the step failed elsewhere."""

    def __init__(self, step, msg, operand=None):
        super().__init__("step %d: %s" % (step, msg))
        self.step = step
        self.operand = operand


def ceil_div(a, b):
    return -(-a // b)


def transfer_ns(nbytes, bw_Bps):
    """Time to move nbytes at bw bytes/s, in ns, rounded up; bw = 0 means never (saturates)."""
    if bw_Bps == 0:
        return U64_MAX
    return min(ceil_div(nbytes * 10**9, bw_Bps), U64_MAX)


def swap_cost_ns(nbytes, bw_d2h, bw_h2d):
    """c_s(t): offload time plus reload time (Sec. 3), saturating at 2^64 - 1."""
    return min(transfer_ns(nbytes, bw_d2h) + transfer_ns(nbytes, bw_h2d), U64_MAX)


def default_params(budget, n_fwd, **kw):
    p = dict(budget_bytes=int(budget), trigger_num=3, trigger_den=4, filter=FILTER_BASE,
             prefetch_distance=2, max_reloads=2, bw_d2h_Bps=50 * 10**9, bw_h2d_Bps=50 * 10**9,
             n_fwd_steps=int(n_fwd), release_when_short=0, prefetch_rebuild_reads=0)
    p.update(kw)
    return p


class _Held:
    """Stack of parent lists of the recomputations in progress; `in` looks through all."""

    def __init__(self):
        self.frames = []

    def append(self, frame):
        self.frames.append(frame)

    def pop(self):
        self.frames.pop()

    def __contains__(self, t):
        return any(t in f for f in self.frames)


class _Sim:
    def __init__(self, tensors, steps, params):
        self.T = tensors
        self.S = steps
        self.p = params
        self.B = params["budget_bytes"]
        n = len(tensors)
        self.resident = [False] * n
        self.evicted = [False] * n
        self.swapout = [False] * n
        self.last_access = [0] * n
        self.reads_at = [[] for _ in range(n)]       # ascending step indices
        for k, st in enumerate(steps):
            for t in st["reads"]:
                self.reads_at[t].append(k)
        self.children = [[] for _ in range(n)]
        for c, t in enumerate(tensors):
            for q in t["parents"]:
                self.children[q].append(c)
        self.tau = 0
        self.live = 0
        self.peak = 0
        self.events = []
        self.k = 0
        self.locked = set()
        self.provisional = [False] * n
        self.held = _Held()
        self.bringing_back = None                    # operand of the running step on its way back

    # -- bookkeeping -------------------------------------------------------
    def emit(self, action, t):
        self.events.append((self.k, action, t))

    def grow(self, nbytes):
        """Allocate nbytes.  Tensors that sit on the GPU only as leftovers of an earlier
        recomputation (provisional) give way first: the one needed farthest in the future
        goes first, ties to the lowest id.  When none is left and release_when_short is
        set, the release loop of Algorithm 1 runs ("memory is not enough"): Filter picks
        among the resident tensors that neither the running step nor a recomputation in
        progress uses, Director says Evict or Offload."""
        while self.live + nbytes > self.B:
            best, best_nr = None, None
            for t in range(len(self.T)):
                if self.provisional[t] and t not in self.locked and t not in self.held:
                    nr = self.next_read(t, self.k)
                    if best is None or nr > best_nr:
                        best, best_nr = t, nr
            if best is not None:
                self.drop(best)
                continue
            cands = []
            if self.p.get("release_when_short"):
                cands = [t for t in range(len(self.T))
                         if self.resident[t] and not self.provisional[t] and t not in self.locked
                         and t not in self.held and not self.doubly_pinned(t)
                         and self.next_read(t, self.k + 1) is not None]
            if not cands:
                raise Infeasible(self.k, "live %d + %d exceeds budget %d"
                                 % (self.live, nbytes, self.B), self.bringing_back)
            self.release(self.filter(cands))
        self.live += nbytes
        self.peak = max(self.peak, self.live)

    def release(self, v):
        """Algorithm 1, the body of its release loop: Director decides, the tensor leaves."""
        act = self.director(v)
        self.emit(act, v)
        self.live -= self.T[v]["bytes"]
        self.resident[v] = False
        if act == EV_EVICT:
            self.evicted[v], self.swapout[v] = True, False
        else:
            self.swapout[v] = True

    def drop(self, t):
        self.emit(EV_DROP_TEMP, t)
        self.live -= self.T[t]["bytes"]
        self.resident[t] = False
        self.provisional[t] = False

    def next_read(self, t, from_step):
        for s in self.reads_at[t]:
            if s >= from_step:
                return s
        return None

    def computable(self, t):
        return not (self.T[t]["flags"] & UNCOMPUTABLE)

    # -- Algorithm 1, access part -----------------------------------------
    def materialise(self, t):
        """Bring t onto the GPU (Recompute when it can be recomputed, Reload otherwise).
        Missing parents are brought in first; they stay afterwards as provisional tensors
        when a later step reads them and are dropped at once when none does."""
        if self.computable(t):
            parents = self.T[t]["parents"]
            self.held.append(parents)
            mine = []
            for p in parents:                           # ascending id
                if not self.resident[p]:
                    self.materialise(p)
                    mine.append(p)
            self.grow(self.T[t]["bytes"])
            self.emit(EV_RECOMPUTE, t)
            self.tau += self.T[t]["cost_ns"]
            self.held.pop()
            for p in mine:
                if p in self.locked:
                    continue
                if self.next_read(p, self.k + 1) is None:
                    self.drop(p)
                else:
                    self.provisional[p] = True
            for p in parents:
                # a parent that was prefetched for this recomputation (prefetch_rebuild_reads) and that
                # no step reads goes the way of the parents the recomputation brought back itself
                if (p not in mine and self.provisional[p] and p not in self.locked and p not in self.held
                        and self.next_read(p, self.k + 1) is None):
                    self.drop(p)
        elif self.swapout[t]:
            self.grow(self.T[t]["bytes"])
            self.emit(EV_RELOAD_DEMAND, t)
        else:
            raise Infeasible(self.k, "tensor %d cannot be recomputed and has no host copy" % t)
        self.resident[t] = True

    # -- Algorithm 2 -------------------------------------------------------
    def filter(self, cands):
        kind = self.p["filter"]
        best, best_key = None, None
        for t in cands:                                  # ascending id: first maximum wins
            m = self.T[t]["bytes"]
            s = self.tau - self.last_access[t]
            key = m * s if kind == FILTER_BASE else (s if kind == FILTER_LRU else m)
            if best is None or key > best_key:
                best, best_key = t, key
        return best

    # -- Algorithm 3 -------------------------------------------------------
    def recompute_cost(self, t):
        """c_r(t): own cost plus every non-resident ancestor reached through non-resident
        tensors (its compute cost, or its reload time when it cannot be recomputed)."""
        total = self.T[t]["cost_ns"]
        seen = set()
        stack = list(self.T[t]["parents"])
        while stack:
            a = stack.pop()
            if a in seen or self.resident[a]:
                continue
            seen.add(a)
            if self.computable(a):
                total += self.T[a]["cost_ns"]
                stack.extend(self.T[a]["parents"])
            else:
                total += transfer_ns(self.T[a]["bytes"], self.p["bw_h2d_Bps"])
        return min(total, U64_MAX)

    def director(self, t):
        f = self.T[t]["flags"]
        if f & (EVICT_PINNED | UNCOMPUTABLE):
            return EV_OFFLOAD
        if f & OFFLOAD_PINNED:
            return EV_EVICT
        c_s = swap_cost_ns(self.T[t]["bytes"], self.p["bw_d2h_Bps"], self.p["bw_h2d_Bps"])
        return EV_EVICT if self.recompute_cost(t) <= c_s else EV_OFFLOAD

    # -- Algorithm 4 -------------------------------------------------------
    def rebuild_read(self, t, memo):
        """Earliest step from the running one on that reads t or, through tensors that are neither
        on the GPU nor in host memory (an access recomputes them, Algorithm 1, and a recomputation
        accesses its parents), a descendant of t; None when there is none."""
        if t in memo:
            return memo[t]
        best = self.next_read(t, self.k)
        for c in self.children[t]:
            if not self.resident[c] and not self.swapout[c] and self.computable(c):
                u = self.rebuild_read(c, memo)
                if u is not None and (best is None or u < best):
                    best = u
        memo[t] = best
        return best

    def prefetch(self):
        d, n = self.p["prefetch_distance"], self.p["max_reloads"]
        wide = bool(self.p.get("prefetch_rebuild_reads"))
        issued = 0
        while issued < n:
            q = []
            memo = {}
            for t in range(len(self.T)):
                if self.swapout[t] and not self.resident[t]:
                    nr = self.rebuild_read(t, memo) if wide else self.next_read(t, self.k)
                    if nr is not None:
                        q.append((nr, t))
            if not q:
                break
            nr, head = min(q)
            if nr > self.k + d or self.live + self.T[head]["bytes"] > self.B:
                break
            self.emit(EV_RELOAD_PREFETCH, head)
            self.live += self.T[head]["bytes"]
            self.peak = max(self.peak, self.live)
            self.resident[head] = True
            own = self.next_read(head, self.k)
            if own is None or nr < own:                  # back for a recomputation, not for a step of its own
                self.provisional[head] = True
            issued += 1

    # -- one step ----------------------------------------------------------
    def doubly_pinned(self, t):
        f = self.T[t]["flags"]
        return bool(f & (EVICT_PINNED | UNCOMPUTABLE)) and bool(f & OFFLOAD_PINNED)

    def step(self, k):
        self.k = k
        st = self.S[k]
        fwd = k < self.p["n_fwd_steps"]
        if not fwd:
            self.prefetch()
        self.locked = set(st["reads"])
        if st["produces"] >= 0:
            self.locked.add(st["produces"])
        for t in st["reads"]:                           # ascending id
            if not self.resident[t]:
                self.bringing_back = t
                self.materialise(t)
                self.bringing_back = None
            self.provisional[t] = False
            self.evicted[t] = False
        need = self.T[st["produces"]]["bytes"] if st["produces"] >= 0 else 0
        if fwd:
            num, den = self.p["trigger_num"], self.p["trigger_den"]
            while den * (self.live + need) > num * self.B:
                prov = [(self.next_read(t, k), -t) for t in range(len(self.T))
                        if self.provisional[t] and t not in self.locked]
                if prov:
                    self.drop(-max(prov)[1])
                    continue
                cands = [t for t in range(len(self.T))
                         if self.resident[t] and t not in self.locked
                         and not self.doubly_pinned(t) and self.next_read(t, k + 1) is not None]
                if not cands:
                    if self.live + need <= self.B:
                        break
                    raise Infeasible(k, "nothing left to release")
                self.release(self.filter(cands))
        if st["produces"] >= 0:
            self.grow(need)
            self.resident[st["produces"]] = True
        self.tau += st["cost_ns"]
        touched = list(st["reads"]) + ([st["produces"]] if st["produces"] >= 0 else [])
        for t in touched:
            self.last_access[t] = self.tau
        for t in sorted(set(touched)):
            if self.next_read(t, k + 1) is None:
                self.emit(EV_FREE, t)
                self.live -= self.T[t]["bytes"]
                self.resident[t] = False
                self.provisional[t] = False
                self.evicted[t] = True
        self.locked = set()


def plan(tensors, steps, params):
    """Returns (events, peak_bytes); events are (step, action, tensor) in issue order.
    Raises Infeasible when some step cannot fit into the budget.

    repair_rounds > 0 (our addition; the paper's manager would simply run out of memory):
    the operator sequence repeats every iteration (Assumption 1), so an iteration that
    fails teaches the next one.  When an operand of a step cannot be brought back because
    rebuilding it with its missing ancestors does not fit, that operand is treated as
    uncomputable from then on -- the Director may only offload it (Sec. 4.3, the pin flags)
    and it comes back by reload, which needs no more than its own bytes -- and the whole
    iteration is planned again, at most repair_rounds times.  A failure anywhere else is final."""
    return plan_with_pins(tensors, steps, params)[:2]


def plan_with_pins(tensors, steps, params):
    """plan() plus the list of tensors that the repair rounds made offload-only."""
    learned = []
    while True:
        T = tensors
        if learned:
            T = [dict(t, flags=t["flags"] | UNCOMPUTABLE) if i in learned else t
                 for i, t in enumerate(tensors)]
        sim = _Sim(T, steps, params)
        try:
            for k in range(len(steps)):
                sim.step(k)
            return sim.events, sim.peak, learned
        except Infeasible as e:
            o = e.operand
            if (o is None or len(learned) >= params.get("repair_rounds", 0)
                    or T[o]["flags"] & UNCOMPUTABLE):
                raise
            learned.append(o)
