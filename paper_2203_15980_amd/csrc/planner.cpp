// Planner behind delta_plan: DELTA's main loop (Algorithm 1) simulated over a static
// operator trace, with the Filter (Algorithm 2, Eq. 1-3), the Director (Algorithm 3,
// Eq. 4-6) and the Prefetcher (Algorithm 4).  Integer arithmetic only.
//
// Readings taken where the paper leaves room (all stated in the design notes):
//   staleness s(t) runs on a logical clock that advances by the cost of every executed or
//   recomputed operator, transfers do not advance it (Assumption 3); c_s = offload time +
//   reload time (Sec. 3); F <= 1 evicts (Algorithm 3); the offloaded queue is ordered by
//   next use; the Prefetcher reloads while memory allows AND fewer than n were issued; the
//   release loop runs in the forward pass only (Assumption 2), down to trigger*B or until
//   nothing releasable is left, and fails only above B; parents rebuilt as operands of a
//   recomputation stay as provisional tensors while a later step reads them and go first
//   (farthest next use first) when room is needed.
#include "planner.hpp"

#include <algorithm>
#include <cstdio>
#include <limits>

namespace delta {

typedef unsigned __int128 u128;
static const uint64_t kU64Max = std::numeric_limits<uint64_t>::max();

static uint64_t transfer_ns(uint64_t bytes, uint64_t bw) {
    if (bw == 0) return kU64Max;
    u128 q = ((u128)bytes * 1000000000u + (bw - 1)) / bw;
    return q > (u128)kU64Max ? kU64Max : (uint64_t)q;
}

static uint64_t sat_add(uint64_t a, uint64_t b) { return a > kU64Max - b ? kU64Max : a + b; }

namespace {

struct Sim {
    const std::vector<PlanTensor> &T;
    const std::vector<PlanStep> &S;
    const delta_plan_params &P;
    uint32_t nT;
    std::vector<uint8_t> resident, swapout, provisional, locked, hold;
    std::vector<uint64_t> last_access;
    std::vector<std::vector<uint32_t>> reads_at;   // per tensor: steps that read it, ascending
    std::vector<uint32_t> cursor;                  // per tensor: first entry of reads_at >= current step
    uint64_t tau = 0, live = 0, peak = 0;
    uint32_t k = 0;
    std::vector<delta_event> ev;
    std::string err;
    bool failed = false;

    Sim(const std::vector<PlanTensor> &t, const std::vector<PlanStep> &s, const delta_plan_params &p)
        : T(t), S(s), P(p), nT((uint32_t)t.size()), resident(nT, 0), swapout(nT, 0),
          provisional(nT, 0), locked(nT, 0), hold(nT, 0), last_access(nT, 0), reads_at(nT),
          cursor(nT, 0) {
        for (uint32_t i = 0; i < S.size(); ++i)
            for (uint32_t r : S[i].reads) reads_at[r].push_back(i);
    }

    static const uint32_t kNever = 0xFFFFFFFFu;

    // first step >= from that reads t, or kNever
    uint32_t next_read(uint32_t t, uint32_t from) const {
        const std::vector<uint32_t> &v = reads_at[t];
        std::vector<uint32_t>::const_iterator it = std::lower_bound(v.begin(), v.end(), from);
        return it == v.end() ? kNever : *it;
    }

    bool computable(uint32_t t) const { return !(T[t].flags & DELTA_F_UNCOMPUTABLE); }

    void emit(uint32_t action, uint32_t t) {
        delta_event e = {k, action, t, 0};
        ev.push_back(e);
    }

    void fail(const char *what, uint64_t a = 0, uint64_t b = 0) {
        if (failed) return;
        char buf[256];
        snprintf(buf, sizeof buf, "step %u: %s (%llu, %llu; budget %llu)", k, what,
                 (unsigned long long)a, (unsigned long long)b, (unsigned long long)P.budget_bytes);
        err = buf;
        failed = true;
    }

    void drop(uint32_t t) {
        emit(DELTA_EV_DROP_TEMP, t);
        live -= T[t].bytes;
        resident[t] = 0;
        provisional[t] = 0;
    }

    // provisional tensor with the farthest next use (lowest id on ties) that is neither an
    // operand of the running step nor of a recomputation in progress; nT when none
    uint32_t farthest_provisional(bool respect_hold) const {
        uint32_t best = nT, best_nr = 0;
        for (uint32_t t = 0; t < nT; ++t) {
            if (!provisional[t] || locked[t] || (respect_hold && hold[t])) continue;
            uint32_t nr = next_read(t, k);
            if (best == nT || nr > best_nr) { best = t; best_nr = nr; }
        }
        return best;
    }

    void grow(uint64_t bytes) {
        while (!failed && live + bytes > P.budget_bytes) {
            uint32_t v = farthest_provisional(true);
            if (v == nT) { fail("allocation does not fit", live, bytes); return; }
            drop(v);
        }
        live += bytes;
        if (live > peak) peak = live;
    }

    // Algorithm 1, lines on the accessed tensor: Recompute when possible, else Reload.
    void materialise(uint32_t t) {
        if (failed) return;
        if (computable(t)) {
            const std::vector<uint32_t> &par = T[t].parents;
            for (uint32_t p : par) ++hold[p];
            std::vector<uint32_t> mine;
            for (uint32_t p : par) {
                if (!resident[p]) {
                    materialise(p);
                    if (failed) return;
                    mine.push_back(p);
                }
            }
            grow(T[t].bytes);
            if (failed) return;
            emit(DELTA_EV_RECOMPUTE, t);
            tau += T[t].cost_ns;
            for (uint32_t p : par) --hold[p];
            for (uint32_t p : mine) {
                if (locked[p]) continue;
                if (next_read(p, k + 1) == kNever) drop(p);
                else provisional[p] = 1;
            }
        } else if (swapout[t]) {
            grow(T[t].bytes);
            if (failed) return;
            emit(DELTA_EV_RELOAD_DEMAND, t);
        } else {
            fail("tensor can neither be recomputed nor reloaded", t);
            return;
        }
        resident[t] = 1;
    }

    // Algorithm 2: minimum of 1/(m*s), 1/s or 1/m == maximum of m*s, s or m.
    uint32_t filter(const std::vector<uint32_t> &cands) const {
        uint32_t best = cands[0];
        u128 best_key = 0;
        bool first = true;
        for (uint32_t t : cands) {
            uint64_t s = tau - last_access[t];
            u128 key = P.filter == DELTA_FILTER_BASE ? (u128)T[t].bytes * s
                     : P.filter == DELTA_FILTER_LRU  ? (u128)s
                                                     : (u128)T[t].bytes;
            if (first || key > best_key) { best = t; best_key = key; first = false; }
        }
        return best;
    }

    // c_r(t), Eq. (5): own cost plus missing ancestors reached through missing tensors.
    uint64_t recompute_cost(uint32_t t) const {
        uint64_t total = T[t].cost_ns;
        std::vector<uint8_t> seen(nT, 0);
        std::vector<uint32_t> stack(T[t].parents.begin(), T[t].parents.end());
        while (!stack.empty()) {
            uint32_t a = stack.back();
            stack.pop_back();
            if (seen[a] || resident[a]) continue;
            seen[a] = 1;
            if (computable(a)) {
                total = sat_add(total, T[a].cost_ns);
                stack.insert(stack.end(), T[a].parents.begin(), T[a].parents.end());
            } else {
                total = sat_add(total, transfer_ns(T[a].bytes, P.bw_h2d_Bps));
            }
        }
        return total;
    }

    // Algorithm 3.
    uint32_t director(uint32_t t) const {
        uint32_t f = T[t].flags;
        if (f & (DELTA_F_EVICT_PINNED | DELTA_F_UNCOMPUTABLE)) return DELTA_EV_OFFLOAD;
        if (f & DELTA_F_OFFLOAD_PINNED) return DELTA_EV_EVICT;
        uint64_t c_s = sat_add(transfer_ns(T[t].bytes, P.bw_d2h_Bps),
                               transfer_ns(T[t].bytes, P.bw_h2d_Bps));
        return recompute_cost(t) <= c_s ? DELTA_EV_EVICT : DELTA_EV_OFFLOAD;
    }

    // Algorithm 4.
    void prefetch() {
        for (uint32_t issued = 0; issued < P.max_reloads; ++issued) {
            uint32_t head = nT, head_nr = kNever;
            for (uint32_t t = 0; t < nT; ++t) {
                if (!swapout[t] || resident[t]) continue;
                uint32_t nr = next_read(t, k);
                if (nr != kNever && (head == nT || nr < head_nr)) { head = t; head_nr = nr; }
            }
            if (head == nT) return;
            if ((uint64_t)head_nr > (uint64_t)k + P.prefetch_distance) return;
            if (live + T[head].bytes > P.budget_bytes) return;
            emit(DELTA_EV_RELOAD_PREFETCH, head);
            live += T[head].bytes;
            if (live > peak) peak = live;
            resident[head] = 1;
        }
    }

    bool doubly_pinned(uint32_t t) const {
        uint32_t f = T[t].flags;
        return (f & (DELTA_F_EVICT_PINNED | DELTA_F_UNCOMPUTABLE)) && (f & DELTA_F_OFFLOAD_PINNED);
    }

    void step(uint32_t idx) {
        k = idx;
        const PlanStep &st = S[k];
        const bool fwd = k < P.n_fwd_steps;
        if (!fwd) prefetch();
        for (uint32_t r : st.reads) locked[r] = 1;
        if (st.produces >= 0) locked[st.produces] = 1;
        for (uint32_t r : st.reads) {
            if (!resident[r]) materialise(r);
            if (failed) return;
            provisional[r] = 0;
        }
        const uint64_t need = st.produces >= 0 ? T[st.produces].bytes : 0;
        if (fwd) {
            while ((u128)P.trigger_den * (live + need) > (u128)P.trigger_num * P.budget_bytes) {
                uint32_t pv = farthest_provisional(false);
                if (pv != nT) { drop(pv); continue; }
                std::vector<uint32_t> cands;
                for (uint32_t t = 0; t < nT; ++t)
                    if (resident[t] && !locked[t] && !doubly_pinned(t) &&
                        next_read(t, k + 1) != kNever)
                        cands.push_back(t);
                if (cands.empty()) {
                    if (live + need <= P.budget_bytes) break;
                    fail("nothing left to release", live, need);
                    return;
                }
                uint32_t v = filter(cands);
                uint32_t act = director(v);
                emit(act, v);
                live -= T[v].bytes;
                resident[v] = 0;
                swapout[v] = act == DELTA_EV_OFFLOAD ? 1 : 0;
            }
        }
        if (st.produces >= 0) {
            grow(need);
            if (failed) return;
            resident[st.produces] = 1;
        }
        tau += st.cost_ns;
        std::vector<uint32_t> touched(st.reads);
        if (st.produces >= 0) touched.push_back((uint32_t)st.produces);
        std::sort(touched.begin(), touched.end());
        touched.erase(std::unique(touched.begin(), touched.end()), touched.end());
        for (uint32_t t : touched) last_access[t] = tau;
        for (uint32_t t : touched) {
            if (next_read(t, k + 1) == kNever) {
                emit(DELTA_EV_FREE, t);
                live -= T[t].bytes;
                resident[t] = 0;
                provisional[t] = 0;
            }
        }
        for (uint32_t t : touched) locked[t] = 0;
    }
};

}  // namespace

delta_status run_plan(const std::vector<PlanTensor> &tensors, const std::vector<PlanStep> &steps,
                      const delta_plan_params &params, std::vector<delta_event> &events,
                      uint64_t &peak, std::string &err) {
    Sim sim(tensors, steps, params);
    for (uint32_t i = 0; i < steps.size(); ++i) {
        sim.step(i);
        if (sim.failed) {
            err = sim.err;
            events.swap(sim.ev);
            peak = sim.peak;
            return DELTA_ERR_INFEASIBLE;
        }
    }
    events.swap(sim.ev);
    peak = sim.peak;
    return DELTA_OK;
}

// Validates and copies the caller's graph.
delta_status load_graph(const delta_tensor_desc *tensors, uint32_t n_tensors,
                        const delta_step_desc *steps, uint32_t n_steps,
                        const delta_plan_params *params, std::vector<PlanTensor> &T,
                        std::vector<PlanStep> &S, std::string &err) {
    if ((!tensors && n_tensors) || (!steps && n_steps) || !params) {
        err = "null argument";
        return DELTA_ERR_INVALID;
    }
    if (params->trigger_den == 0 || params->trigger_num > params->trigger_den ||
        params->filter > DELTA_FILTER_GREEDY || params->n_fwd_steps > n_steps) {
        err = "bad plan parameters";
        return DELTA_ERR_INVALID;
    }
    T.resize(n_tensors);
    for (uint32_t i = 0; i < n_tensors; ++i) {
        const delta_tensor_desc &d = tensors[i];
        if (d.n_parents && !d.parents) { err = "null parents"; return DELTA_ERR_INVALID; }
        T[i].bytes = d.bytes;
        T[i].cost_ns = d.cost_ns;
        T[i].flags = d.flags;
        T[i].parents.assign(d.parents, d.parents + d.n_parents);
        for (uint32_t j = 0; j < d.n_parents; ++j)
            if (d.parents[j] >= i || (j && d.parents[j] <= d.parents[j - 1])) {
                err = "parents must be ascending ids below the tensor's own id";
                return DELTA_ERR_INVALID;
            }
    }
    std::vector<uint8_t> produced(n_tensors, 0);
    S.resize(n_steps);
    for (uint32_t i = 0; i < n_steps; ++i) {
        const delta_step_desc &d = steps[i];
        if (d.n_reads && !d.reads) { err = "null reads"; return DELTA_ERR_INVALID; }
        S[i].produces = d.produces;
        S[i].cost_ns = d.cost_ns;
        S[i].reads.assign(d.reads, d.reads + d.n_reads);
        for (uint32_t j = 0; j < d.n_reads; ++j)
            if (d.reads[j] >= n_tensors || (j && d.reads[j] <= d.reads[j - 1]) ||
                !produced[d.reads[j]]) {
                err = "reads must be ascending ids of tensors produced earlier";
                return DELTA_ERR_INVALID;
            }
        if (d.produces >= 0) {
            if ((uint32_t)d.produces >= n_tensors || produced[d.produces] ||
                i >= params->n_fwd_steps) {
                err = "bad produces (unknown id, produced twice, or in the backward pass)";
                return DELTA_ERR_INVALID;
            }
            produced[d.produces] = 1;
        } else if (d.produces != -1) {
            err = "produces must be a tensor id or -1";
            return DELTA_ERR_INVALID;
        }
    }
    return DELTA_OK;
}

}  // namespace delta
