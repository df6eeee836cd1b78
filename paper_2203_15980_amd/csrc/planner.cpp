// Planner behind delta_plan.
//
// The paper describes DELTA as a manager that sits under a framework's executor and is called
// once per tensor access (Algorithm 1): bring the accessed tensor back if it is gone, then,
// while memory is tight, let the Filter (Algorithm 2, Eq. 1-3) pick a resident tensor and the
// Director (Algorithm 3, Eq. 4-6) decide between Evict and Offload; before the backward pass's
// operators the Prefetcher (Algorithm 4) reloads offloaded tensors.  This file is that manager
// (class Manager: on_access, make_room, pick_victim, decide, prefetch) plus an executor stand-in
// (run_iteration) that walks the operator sequence of one training iteration (Assumption 1) and
// records what the manager does as plan events.  Integer arithmetic only: products of bytes and
// time are 128-bit, costs saturate at 2^64 - 1.
//
// Where the paper leaves room, the choices are:
//   * time runs on a logical clock that advances by the cost of every operator that runs,
//     recomputations included; copies do not advance it (Assumption 3).  Staleness s(t) is the
//     clock minus the tensor's last access by an operator of the sequence;
//   * c_s(t) is the offload time plus the reload time (Sec. 3), each rounded up to a nanosecond;
//     c_r(t) is t's own cost plus, once each, the cost of every missing ancestor reached through
//     missing tensors (reload time for one that cannot be recomputed); F <= 1 evicts;
//   * the release loop runs before a forward operator's output is allocated and stops at the
//     early-start level (3/4 of the budget in the paper, Sec. 4.3) or when nothing releasable is
//     left; only a step that does not fit into the whole budget fails.  After the forward pass no
//     Evict or Offload is issued (Assumption 2), unless release_when_short asks for Algorithm 1
//     to the letter: then the same loop also runs whenever an allocation does not fit;
//   * parents that were rebuilt only to recompute a tensor stay on the GPU as leftovers while
//     some later operator reads them, and are the first to give way (latest next use first, ties to
//     the lowest id); one nobody reads again leaves at once;
//   * the Prefetcher's queue is ordered by next use (ties: lowest id); it looks d steps ahead,
//     issues at most n reloads per step, and stops at the first tensor that does not fit;
//   * repair_rounds: an iteration whose operand could not be brought back is planned again with
//     that operand offload-only (it then returns by reload, which needs only its own bytes).
#include "planner.hpp"

#include <algorithm>
#include <cstdio>
#include <limits>

namespace delta {

namespace {

typedef unsigned __int128 u128;
const uint64_t kForever = std::numeric_limits<uint64_t>::max();
const uint32_t kNoStep = 0xFFFFFFFFu;
const uint32_t kNoTensor = 0xFFFFFFFFu;

uint64_t saturating_sum(uint64_t a, uint64_t b) { return b > kForever - a ? kForever : a + b; }

// ceil(bytes / bandwidth) in ns; a link of 0 B/s never finishes
uint64_t copy_ns(uint64_t bytes, uint64_t bytes_per_s) {
    if (!bytes_per_s) return kForever;
    const u128 ns = ((u128)bytes * 1000000000ull + bytes_per_s - 1) / bytes_per_s;
    return ns > (u128)kForever ? kForever : (uint64_t)ns;
}

// The fields of the paper's struct DELTATensor (Sec. 4.3) that the planner needs, plus the
// trace knowledge a static plan has: when the tensor is used.
struct Record {
    uint64_t memory = 0, compute_cost = 0;
    bool uncomputable = false, evict_pinned = false, offload_pinned = false;
    bool on_gpu = false;
    bool host_copy = false;        // "swapout": a valid copy sits in host memory
    bool leftover = false;         // on the GPU only because a recomputation needed it
    bool operand = false;          // read or produced by the operator that is running
    uint32_t rebuilding = 0;       // number of recomputations in progress that hold it as a parent
    uint64_t last_access = 0;
    std::vector<uint32_t> uses;    // steps that read it, ascending
    size_t seen = 0;               // uses[0 .. seen) lie before the running step
    const std::vector<uint32_t> *parents = nullptr;

    // first use at or after the running step / strictly after it
    uint32_t use_from_now() const { return seen < uses.size() ? uses[seen] : kNoStep; }
    uint32_t use_after(uint32_t now) const {
        size_t i = seen;
        if (i < uses.size() && uses[i] == now) ++i;
        return i < uses.size() ? uses[i] : kNoStep;
    }
    bool may_never_leave() const { return (evict_pinned || uncomputable) && offload_pinned; }
};

struct OutOfMemory {
    uint32_t step;
    uint32_t operand;              // the step's operand that was on its way back, or kNoTensor
    std::string what;
};

class Manager {
  public:
    Manager(const std::vector<PlanTensor> &tensors, const std::vector<PlanStep> &steps,
            const delta_plan_params &params, const std::vector<uint8_t> &offload_only)
        : steps_(steps), cfg_(params), rec_(tensors.size()), mark_(tensors.size(), 0) {
        for (size_t t = 0; t < tensors.size(); ++t) {
            Record &r = rec_[t];
            r.memory = tensors[t].bytes;
            r.compute_cost = tensors[t].cost_ns;
            r.uncomputable = (tensors[t].flags & DELTA_F_UNCOMPUTABLE) || offload_only[t];
            r.evict_pinned = tensors[t].flags & DELTA_F_EVICT_PINNED;
            r.offload_pinned = tensors[t].flags & DELTA_F_OFFLOAD_PINNED;
            r.parents = &tensors[t].parents;
        }
        for (uint32_t k = 0; k < steps.size(); ++k)
            for (uint32_t t : steps[k].reads) rec_[t].uses.push_back(k);
        if (cfg_.prefetch_rebuild_reads) {
            consumers_.resize(tensors.size());
            for (uint32_t t = 0; t < tensors.size(); ++t)
                for (uint32_t p : tensors[t].parents) consumers_[p].push_back(t);
            wanted_.resize(tensors.size());
        }
    }

    // One operator of the sequence.  Throws OutOfMemory.
    void run_step(uint32_t k) {
        now_ = k;
        const PlanStep &op = steps_[k];
        const bool forward = k < cfg_.n_fwd_steps;
        for (Record &r : rec_)
            while (r.seen < r.uses.size() && r.uses[r.seen] < k) ++r.seen;
        if (!forward) prefetch();
        for (uint32_t t : op.reads) rec_[t].operand = true;
        if (op.produces >= 0) rec_[op.produces].operand = true;
        for (uint32_t t : op.reads) {
            on_access(t);
            rec_[t].leftover = false;
        }
        if (op.produces >= 0) {
            Record &out = rec_[op.produces];
            if (forward) early_release(out.memory);
            make_room(out.memory, kNoTensor);
            occupy(out.memory);
            out.on_gpu = true;
        }
        clock_ += op.cost_ns;
        // ids in ascending order, each once: reads are ascending, the output is a new id
        std::vector<uint32_t> touched(op.reads);
        if (op.produces >= 0)
            touched.insert(std::upper_bound(touched.begin(), touched.end(), (uint32_t)op.produces), (uint32_t)op.produces);
        for (uint32_t t : touched) rec_[t].last_access = clock_;
        for (uint32_t t : touched) {
            Record &r = rec_[t];
            r.operand = false;
            if (r.use_after(k) == kNoStep) {            // its last use has passed
                note(DELTA_EV_FREE, t);
                vacate(r);
            }
        }
    }

    std::vector<delta_event> events;
    uint64_t peak = 0;

  private:
    const std::vector<PlanStep> &steps_;
    const delta_plan_params &cfg_;
    std::vector<Record> rec_;
    std::vector<uint32_t> mark_;       // visit stamps of the ancestor walk
    std::vector<std::vector<uint32_t>> consumers_;   // prefetch_rebuild_reads: the tensors computed from each tensor
    std::vector<uint32_t> wanted_;     // ... and, per prefetch round, when each tensor is wanted (kNoStep - 1: not worked out yet)
    uint32_t stamp_ = 0;
    uint32_t now_ = 0;
    uint64_t clock_ = 0, in_use_ = 0;

    void note(uint32_t action, uint32_t t) {
        const delta_event e = {now_, action, t, 0};
        events.push_back(e);
    }
    void occupy(uint64_t bytes) {
        in_use_ += bytes;
        if (in_use_ > peak) peak = in_use_;
    }
    void vacate(Record &r) {
        in_use_ -= r.memory;
        r.on_gpu = false;
        r.leftover = false;
    }

    // ---- Algorithm 1, first half: the accessed tensor must be on the GPU.
    // A missing tensor that can be recomputed is recomputed, after its missing parents (depth
    // first, ascending ids); one that cannot is reloaded from its host copy.  Written as a loop
    // over an explicit stack of recomputations in progress.
    struct Rebuild {
        uint32_t tensor;
        size_t next_parent;
        std::vector<uint32_t> fetched;     // parents this recomputation had to bring back
    };

    void on_access(uint32_t wanted) {
        if (rec_[wanted].on_gpu) return;
        std::vector<Rebuild> stack;
        open_rebuild(stack, wanted, wanted);
        while (!stack.empty()) {
            Rebuild &top = stack.back();
            Record &r = rec_[top.tensor];
            const std::vector<uint32_t> &parents = *r.parents;
            if (top.next_parent < parents.size()) {
                const uint32_t p = parents[top.next_parent++];
                if (!rec_[p].on_gpu) {
                    top.fetched.push_back(p);
                    open_rebuild(stack, p, wanted);     // may invalidate `top`
                }
                continue;
            }
            // all parents are here: run the operator again
            make_room(r.memory, wanted);
            occupy(r.memory);
            note(DELTA_EV_RECOMPUTE, top.tensor);
            clock_ += r.compute_cost;
            r.on_gpu = true;
            for (uint32_t p : parents) --rec_[p].rebuilding;
            for (uint32_t p : top.fetched) {
                Record &q = rec_[p];
                if (q.operand) continue;                // the running operator reads it anyway
                if (q.use_after(now_) == kNoStep) {
                    note(DELTA_EV_DROP_TEMP, p);
                    vacate(q);
                } else {
                    q.leftover = true;
                }
            }
            // a parent that the Prefetcher brought back for this recomputation (prefetch_rebuild_reads)
            // and that no operator reads leaves like the ones the recomputation fetched itself
            for (uint32_t p : parents) {
                Record &q = rec_[p];
                if (!q.on_gpu || !q.leftover || q.operand || q.rebuilding || q.use_after(now_) != kNoStep) continue;
                if (std::find(top.fetched.begin(), top.fetched.end(), p) != top.fetched.end()) continue;
                note(DELTA_EV_DROP_TEMP, p);
                vacate(q);
            }
            stack.pop_back();
        }
    }

    // Starts bringing `t` back: a reload completes at once, a recomputation goes on the stack.
    void open_rebuild(std::vector<Rebuild> &stack, uint32_t t, uint32_t wanted) {
        Record &r = rec_[t];
        if (!r.uncomputable) {
            for (uint32_t p : *r.parents) ++rec_[p].rebuilding;
            Rebuild f;
            f.tensor = t;
            f.next_parent = 0;
            stack.push_back(f);
            return;
        }
        if (!r.host_copy) {
            char msg[96];
            snprintf(msg, sizeof msg, "tensor %u can neither be recomputed nor reloaded", t);
            throw OutOfMemory{now_, kNoTensor, msg};
        }
        make_room(r.memory, wanted);
        occupy(r.memory);
        note(DELTA_EV_RELOAD_DEMAND, t);
        r.on_gpu = true;
    }

    // ---- Algorithm 1, second half: the release loop.
    bool idle(const Record &r) const { return !r.operand && r.rebuilding == 0; }

    // the leftover to drop next: latest next use, lowest id among equals
    uint32_t next_leftover() const {
        uint32_t best = kNoTensor, best_use = 0;
        for (uint32_t t = 0; t < rec_.size(); ++t) {
            const Record &r = rec_[t];
            if (!r.leftover || !idle(r)) continue;
            const uint32_t u = r.use_from_now();
            if (best == kNoTensor || u > best_use) {
                best = t;
                best_use = u;
            }
        }
        return best;
    }

    // Algorithm 2.  The minimum of H = 1/(m s), 1/s or 1/m is the maximum of m s, s or m; the
    // first of equal scores wins; s = 0 scores lowest without a division.
    uint32_t pick_victim() const {
        uint32_t best = kNoTensor;
        u128 best_score = 0;
        for (uint32_t t = 0; t < rec_.size(); ++t) {
            const Record &r = rec_[t];
            if (!r.on_gpu || r.leftover || !idle(r) || r.may_never_leave() || r.use_after(now_) == kNoStep) continue;
            const uint64_t stale = clock_ - r.last_access;
            u128 score;
            switch (cfg_.filter) {
            case DELTA_FILTER_LRU: score = stale; break;
            case DELTA_FILTER_GREEDY: score = r.memory; break;
            default: score = (u128)r.memory * stale; break;
            }
            if (best == kNoTensor || score > best_score) {
                best = t;
                best_score = score;
            }
        }
        return best;
    }

    // c_r(t) of Eq. (5)
    uint64_t rebuild_cost(uint32_t t) {
        ++stamp_;
        uint64_t total = rec_[t].compute_cost;
        std::vector<uint32_t> todo(rec_[t].parents->rbegin(), rec_[t].parents->rend());
        while (!todo.empty()) {
            const uint32_t a = todo.back();
            todo.pop_back();
            if (rec_[a].on_gpu || mark_[a] == stamp_) continue;
            mark_[a] = stamp_;
            if (rec_[a].uncomputable) {
                total = saturating_sum(total, copy_ns(rec_[a].memory, cfg_.bw_h2d_Bps));
            } else {
                total = saturating_sum(total, rec_[a].compute_cost);
                todo.insert(todo.end(), rec_[a].parents->rbegin(), rec_[a].parents->rend());
            }
        }
        return total;
    }

    // Algorithm 3
    uint32_t decide(uint32_t t) {
        const Record &r = rec_[t];
        if (r.evict_pinned || r.uncomputable) return DELTA_EV_OFFLOAD;
        if (r.offload_pinned) return DELTA_EV_EVICT;
        const uint64_t c_s = saturating_sum(copy_ns(r.memory, cfg_.bw_d2h_Bps), copy_ns(r.memory, cfg_.bw_h2d_Bps));
        return rebuild_cost(t) <= c_s ? DELTA_EV_EVICT : DELTA_EV_OFFLOAD;
    }

    void release(uint32_t t) {
        const uint32_t action = decide(t);
        note(action, t);
        rec_[t].host_copy = action == DELTA_EV_OFFLOAD;
        vacate(rec_[t]);
    }

    // "3/4 of the memory is used": before a forward operator's output of `incoming` bytes
    void early_release(uint64_t incoming) {
        while ((u128)cfg_.trigger_den * ((u128)in_use_ + incoming) > (u128)cfg_.trigger_num * cfg_.budget_bytes) {
            uint32_t t = next_leftover();
            if (t != kNoTensor) {
                note(DELTA_EV_DROP_TEMP, t);
                vacate(rec_[t]);
                continue;
            }
            t = pick_victim();
            if (t == kNoTensor) {
                if (in_use_ + incoming <= cfg_.budget_bytes) return;
                char msg[128];
                snprintf(msg, sizeof msg, "nothing left to release (%llu in use + %llu; budget %llu)",
                         (unsigned long long)in_use_, (unsigned long long)incoming, (unsigned long long)cfg_.budget_bytes);
                throw OutOfMemory{now_, kNoTensor, msg};
            }
            release(t);
        }
    }

    // "memory is not enough": `incoming` bytes must fit into the budget
    void make_room(uint64_t incoming, uint32_t wanted) {
        while (in_use_ + incoming > cfg_.budget_bytes) {
            uint32_t t = next_leftover();
            if (t != kNoTensor) {
                note(DELTA_EV_DROP_TEMP, t);
                vacate(rec_[t]);
                continue;
            }
            t = cfg_.release_when_short ? pick_victim() : kNoTensor;
            if (t == kNoTensor) {
                char msg[128];
                snprintf(msg, sizeof msg, "allocation does not fit (%llu in use + %llu; budget %llu)",
                         (unsigned long long)in_use_, (unsigned long long)incoming, (unsigned long long)cfg_.budget_bytes);
                throw OutOfMemory{now_, wanted, msg};
            }
            release(t);
        }
    }

    // ---- Algorithm 4
    // When a tensor is wanted next: by a step that reads it, or - prefetch_rebuild_reads - by the
    // recomputation of a tensor that a step reads: a tensor that is neither on the GPU nor in host
    // memory is recomputed when it is accessed (Algorithm 1), and the recomputation accesses its parents.
    uint32_t wanted_from_now(uint32_t t) {
        const Record &r = rec_[t];
        if (!cfg_.prefetch_rebuild_reads) return r.use_from_now();
        if (wanted_[t] != kNoStep - 1) return wanted_[t];
        uint32_t first = r.use_from_now();
        for (uint32_t c : consumers_[t]) {
            const Record &rc = rec_[c];
            if (rc.on_gpu || rc.host_copy || rc.uncomputable) continue;
            first = std::min(first, wanted_from_now(c));
        }
        wanted_[t] = first;
        return first;
    }

    void prefetch() {
        for (uint32_t issued = 0; issued < cfg_.max_reloads; ++issued) {
            if (cfg_.prefetch_rebuild_reads) std::fill(wanted_.begin(), wanted_.end(), kNoStep - 1);
            uint32_t head = kNoTensor, head_use = kNoStep;
            for (uint32_t t = 0; t < rec_.size(); ++t) {
                const Record &r = rec_[t];
                if (r.on_gpu || !r.host_copy) continue;
                const uint32_t u = wanted_from_now(t);
                if (u < head_use) {                      // kNoStep (never used again) is never below
                    head = t;
                    head_use = u;
                }
            }
            if (head == kNoTensor) return;
            if ((uint64_t)head_use - now_ > cfg_.prefetch_distance) return;
            if (in_use_ + rec_[head].memory > cfg_.budget_bytes) return;
            note(DELTA_EV_RELOAD_PREFETCH, head);
            occupy(rec_[head].memory);
            rec_[head].on_gpu = true;
            // back for a recomputation rather than for a step of its own: a leftover, first to give way
            if (head_use < rec_[head].use_from_now()) rec_[head].leftover = true;
        }
    }
};

}  // namespace

delta_status run_plan(const std::vector<PlanTensor> &tensors, const std::vector<PlanStep> &steps,
                      const delta_plan_params &params, std::vector<delta_event> &events,
                      uint64_t &peak, std::string &err) {
    std::vector<uint8_t> offload_only(tensors.size(), 0);
    for (uint32_t round = 0;; ++round) {
        Manager m(tensors, steps, params, offload_only);
        try {
            for (uint32_t k = 0; k < steps.size(); ++k) m.run_step(k);
            events.swap(m.events);
            peak = m.peak;
            return DELTA_OK;
        } catch (const OutOfMemory &oom) {
            const uint32_t o = oom.operand;
            const bool can_learn = o != kNoTensor && round < params.repair_rounds && !offload_only[o] &&
                                   !(tensors[o].flags & DELTA_F_UNCOMPUTABLE);
            if (can_learn) {
                offload_only[o] = 1;
                continue;
            }
            char head[32];
            snprintf(head, sizeof head, "step %u: ", oom.step);
            err = head + oom.what;
            events.swap(m.events);
            peak = m.peak;
            return DELTA_ERR_INFEASIBLE;
        }
    }
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
        params->filter > DELTA_FILTER_GREEDY || params->n_fwd_steps > n_steps ||
        params->release_when_short > 1 || params->prefetch_rebuild_reads > 1) {
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
