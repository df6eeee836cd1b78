// C ABI of the library (include/delta.h): context, arena sub-allocator, swap engine,
// recompute dispatch and measurement probes.  The planner lives in planner.cpp, the
// kernels in conv_igemm.hip.
//
// Stream model (DELTA Sec. 4.2: copies run on a memory stream of their own so that they
// overlap the computation stream).  Three streams: the caller's compute stream, a D2H
// stream for Offload and an H2D stream for Reload -- two copy streams so that both
// directions of the host link can be busy at once.  Nothing here blocks the host except
// delta_sync / delta_stats / delta_bind / delta_destroy.  Ordering between streams is
// carried by events:
//   - every arena block remembers, per stream, the last event after which its old
//     contents are no longer touched (a "fence"); whoever receives the block makes its
//     own stream wait for the fences of the other streams before writing;
//   - a reloaded tensor carries the event of its H2D copy; the compute stream waits for it
//     at the first use;
//   - an offloaded tensor carries the event of its D2H copy; a reload waits for it.
#include <hip/hip_runtime.h>

#include <chrono>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <deque>
#include <map>
#include <new>
#include <string>
#include <vector>

#include "../../include/delta.h"
#include "kernels.hpp"
#include "planner.hpp"

namespace {

// S_AUX carries the weight gradients of convolutions: nothing later in the backward pass reads
// them, so they run beside the data-gradient chain instead of inside it.
enum { S_COMPUTE = 0, S_D2H = 1, S_H2D = 2, S_AUX = 3, N_STREAMS = 4 };
const uint64_t kAlign = 256;
// The swap engine sends a tensor of more than kCopyWhole bytes as four copy commands (pieces).
const uint64_t kCopyWhole = 32ull << 20;
inline uint64_t copy_piece_bytes(uint64_t bytes) {
    if (bytes <= kCopyWhole) return bytes ? bytes : 1;
    return ((bytes + 3) / 4 + kAlign - 1) / kAlign * kAlign;
}

// An ordering event plus its position in the order of recording: of two events recorded on
// the same stream, waiting for the one with the larger seq covers the other.
struct Ev {
    hipEvent_t e;
    uint64_t seq;
    Ev() : e(nullptr), seq(0) {}
    explicit operator bool() const { return e != nullptr; }
};

struct Fence {
    Ev ev[N_STREAMS];
};

struct Block {
    uint64_t size;
    Fence fence;
};

// A freed block that stays out of the free list for a while (see arena_free).
struct Resting {
    uint64_t offset, order;         // order: its place in the sequence of all frees
    Block block;
};

struct Tensor {
    uint64_t bytes = 0;
    bool resident = false;
    uint64_t offset = 0;            // arena offset when resident
    void *host = nullptr;           // pinned buffer (lazily allocated, kept for reuse)
    bool host_valid = false;
    Ev d2h_done;                    // last Offload copy of this tensor
    std::vector<Ev> d2h_piece;      // when that copy went out in pieces: one per piece but the last
    Ev h2d_done;                    // pending Reload the compute stream has not waited for
    Ev aux_done;                    // last weight-gradient launch on S_AUX that reads this tensor
};

struct Timed {
    hipEvent_t start, stop;
    int dir;
};

// One allocation of pinned host memory; tensors' host buffers are carved out of slabs in order.
struct Slab {
    unsigned char *base;
    uint64_t size, used;
};
const uint64_t kSlabMin = 64ull << 20;

}  // namespace

// Scratch of delta_batchnorm_static, the entry point that allocates nothing: the partial sums and the
// per-channel factors of the batch-norm kernels.  One copy per GPU, at its own address, held until the
// process ends.  In host code this name only stands for the symbol: the device address of the current
// GPU's copy comes from hipGetSymbolAddress (static_scratch_for below) and only that pointer is ever
// handed to a kernel.
constexpr size_t kStaticScratchBytes = ((size_t)4 << 20) + ((size_t)64 << 10);
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
static void *g_static_scratch[kMaxDevices];        // per device ordinal: where that GPU keeps its copy

struct delta_ctx {
    unsigned char *arena = nullptr;
    uint64_t arena_bytes = 0;
    int device = -1;
    hipStream_t stream[N_STREAMS] = {nullptr, nullptr, nullptr, nullptr};
    Ev aux_tail;                                   // last launch on S_AUX the compute stream has not joined
    uintptr_t aux_lo = 0, aux_hi = 0;              // caller memory (workspace) those launches use: [aux_lo, aux_hi)
    Ev stg_tail;                                   // last launch on S_AUX that used a staging range, and that range
    uintptr_t stg_lo = 0, stg_hi = 0;
    std::map<uint64_t, Block> free_blocks;         // offset -> block, coalesced
    std::deque<Resting> cooling;                   // freed blocks the weight-gradient stream may still read, oldest first
    std::deque<Resting> copying;                   // freed blocks a copy may still touch, oldest first
    uint64_t free_seq = 0;                         // blocks freed so far
    std::map<uint64_t, uint64_t> used;             // offset -> size
    std::vector<Tensor> tensors;
    std::vector<Slab> slabs;                       // the pinned host pool: kept across delta_bind, freed by delta_destroy
    std::vector<hipEvent_t> ev_pool, ev_live;      // ordering events (no timing)
    std::vector<hipEvent_t> tev_pool;              // timing events
    std::vector<Timed> timed;
    delta_stats_t st;
    bool skip_copies = false;
    void *bn_scratch = nullptr;                    // partial sums of DELTA_OP_BATCHNORM, allocated on first use
    void *static_scratch = nullptr;                // this GPU's copy of the file-scope scratch array (delta_batchnorm_static)
    float *ones = nullptr, *zeros = nullptr;       // kMaxChannels floats each (identity scale/shift of the data gradient)
    uint64_t ev_seq = 0;
    std::string err;

    delta_ctx() { memset(&st, 0, sizeof st); }
};

namespace {

delta_status fail(delta_ctx *c, delta_status code, const char *fmt, ...) {
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    if (c) c->err = buf;
    return code;
}

#define HIP_TRY(c, call)                                                                       \
    do {                                                                                       \
        hipError_t e_ = (call);                                                                \
        if (e_ != hipSuccess)                                                                  \
            return fail((c), DELTA_ERR_HIP, "%s failed: %s", #call, hipGetErrorString(e_));    \
    } while (0)

delta_status need_gpu(delta_ctx *c) {
    if (!c) return DELTA_ERR_INVALID;
    if (!c->arena) return fail(c, DELTA_ERR_STATE, "planner-only context: no arena was given");
    return DELTA_OK;
}

// ---- events

delta_status new_event(delta_ctx *c, hipStream_t s, Ev *out) {
    hipEvent_t e;
    if (!c->ev_pool.empty()) {
        e = c->ev_pool.back();
        c->ev_pool.pop_back();
    } else {
        HIP_TRY(c, hipEventCreateWithFlags(&e, hipEventDisableTiming));
    }
    c->ev_live.push_back(e);
    HIP_TRY(c, hipEventRecord(e, s));
    out->e = e;
    out->seq = ++c->ev_seq;
    return DELTA_OK;
}

delta_status new_timing_event(delta_ctx *c, hipStream_t s, hipEvent_t *out) {
    hipEvent_t e;
    if (!c->tev_pool.empty()) {
        e = c->tev_pool.back();
        c->tev_pool.pop_back();
    } else {
        HIP_TRY(c, hipEventCreate(&e));
    }
    HIP_TRY(c, hipEventRecord(e, s));
    *out = e;
    return DELTA_OK;
}

// Folds finished copy timings into the statistics.  Streams must be idle.
delta_status harvest_timings(delta_ctx *c) {
    for (size_t i = 0; i < c->timed.size(); ++i) {
        float ms = 0.f;
        HIP_TRY(c, hipEventElapsedTime(&ms, c->timed[i].start, c->timed[i].stop));
        (c->timed[i].dir == DELTA_DIR_D2H ? c->st.d2h_ms : c->st.h2d_ms) += ms;
        c->tev_pool.push_back(c->timed[i].start);
        c->tev_pool.push_back(c->timed[i].stop);
    }
    c->timed.clear();
    return DELTA_OK;
}

void flush_cooling(delta_ctx *c);

// After all streams are idle every fence is satisfied: recycle the events.
void retire_events(delta_ctx *c) {
    for (size_t i = 0; i < c->cooling.size(); ++i) c->cooling[i].block.fence = Fence();
    for (size_t i = 0; i < c->copying.size(); ++i) c->copying[i].block.fence = Fence();
    for (std::map<uint64_t, Block>::iterator it = c->free_blocks.begin(); it != c->free_blocks.end(); ++it)
        it->second.fence = Fence();
    for (size_t i = 0; i < c->tensors.size(); ++i) {
        c->tensors[i].d2h_done = c->tensors[i].h2d_done = c->tensors[i].aux_done = Ev();
        c->tensors[i].d2h_piece.clear();
    }
    c->aux_tail = c->stg_tail = Ev();              // every stream is idle: nothing in flight uses the caller's workspace
    c->aux_lo = c->aux_hi = c->stg_lo = c->stg_hi = 0;
    c->ev_pool.insert(c->ev_pool.end(), c->ev_live.begin(), c->ev_live.end());
    c->ev_live.clear();
}

delta_status sync_all(delta_ctx *c) {
    for (int s = 0; s < N_STREAMS; ++s) HIP_TRY(c, hipStreamSynchronize(c->stream[s]));
    delta_status r = harvest_timings(c);
    if (r != DELTA_OK) return r;
    retire_events(c);
    flush_cooling(c);                              // nothing is in flight: resting blocks rejoin the free list
    return DELTA_OK;
}

// ---- arena: first fit over an offset-ordered free list, coalescing on free

Ev later(const Ev &a, const Ev &b) { return a.seq > b.seq ? a : b; }

// Placement.  Two populations share the arena: the planned activations, which live long, and the
// gradient tensors of the backward pass, which come and go.  Activations (top = false) are placed
// from the bottom of the arena upwards, gradients (top = true) from its end downwards, so that the
// two do not cut up each other's free space; with that an arena of little more than the activation
// budget plus the gradient peak is enough (the early start of Sec. 4.3 keeps a quarter of the
// budget free, which is what leaves a choice at all).  Best fit; among equals the block nearest
// the population's own end.
// A freed block that a copy or a weight gradient of another stream may still be touching would
// stall the stream that receives it.  Such blocks rest outside the free list first: one that a
// weight gradient reads, in a short queue (kCooling blocks, in order of release), by which time
// that stream has usually passed it; one that an Offload or Reload copy still touches - the link
// is three orders slower than HBM - until nothing else fits.  When nothing in the free list fits,
// the blocks that rest rejoin it one by one, the longest-resting first, until something fits, so
// the arena never fails while a fitting block exists (at the price of some fragmentation: resting
// blocks do not merge with their neighbours).  Which block a tensor gets depends on the order of
// calls only, never on timing: a replay that fits once fits every time.
const size_t kCooling = 4;

void insert_free(delta_ctx *c, uint64_t off, Block b) {
    // Fences that have completed by now are dropped before they can spread to the neighbours the block
    // merges with (this only spares later waits; it has no part in where anything is placed).
    for (int s = 0; s < N_STREAMS; ++s)
        if (b.fence.ev[s] && s != S_COMPUTE) {
            if (hipEventQuery(b.fence.ev[s].e) == hipSuccess) b.fence.ev[s] = Ev();
            else (void)hipGetLastError();                       // hipErrorNotReady is not an error here
        }
    uint64_t o = off;
    std::map<uint64_t, Block>::iterator nx = c->free_blocks.lower_bound(off);   // first block above
    if (nx != c->free_blocks.begin()) {
        std::map<uint64_t, Block>::iterator pv = nx;
        --pv;
        if (pv->first + pv->second.size == off) {                               // merge downwards
            o = pv->first;
            b.size += pv->second.size;
            for (int s = 0; s < N_STREAMS; ++s) b.fence.ev[s] = later(pv->second.fence.ev[s], b.fence.ev[s]);
            c->free_blocks.erase(pv);
        }
    }
    if (nx != c->free_blocks.end() && o + b.size == nx->first) {                // merge upwards
        b.size += nx->second.size;
        for (int s = 0; s < N_STREAMS; ++s) b.fence.ev[s] = later(nx->second.fence.ev[s], b.fence.ev[s]);
        c->free_blocks.erase(nx);
    }
    c->free_blocks[o] = b;
}

// The streams are drained: nothing needs to rest any more.
void flush_cooling(delta_ctx *c) {
    for (size_t i = 0; i < c->cooling.size(); ++i) insert_free(c, c->cooling[i].offset, c->cooling[i].block);
    c->cooling.clear();
    for (size_t i = 0; i < c->copying.size(); ++i) insert_free(c, c->copying[i].offset, c->copying[i].block);
    c->copying.clear();
}

// The block that has rested longest joins the free list; false when nothing rests.
bool wake_oldest(delta_ctx *c) {
    const bool a = !c->cooling.empty(), b = !c->copying.empty();
    if (!a && !b) return false;
    std::deque<Resting> &q = (a && (!b || c->cooling.front().order < c->copying.front().order)) ? c->cooling : c->copying;
    insert_free(c, q.front().offset, q.front().block);
    q.pop_front();
    return true;
}

delta_status arena_alloc(delta_ctx *c, uint64_t bytes, int for_stream, uint64_t *off, bool top = false) {
    const uint64_t need = (bytes + kAlign - 1) / kAlign * kAlign;
    std::map<uint64_t, Block>::iterator pick = c->free_blocks.end();
    for (;;) {
        // the map runs bottom-up: for the bottom population the first of equals stays, for the top one the last
        for (std::map<uint64_t, Block>::iterator it = c->free_blocks.begin(); it != c->free_blocks.end(); ++it) {
            if (it->second.size < need) continue;
            if (pick == c->free_blocks.end() || it->second.size < pick->second.size ||
                (top && it->second.size == pick->second.size))
                pick = it;
        }
        if (pick != c->free_blocks.end() || !wake_oldest(c)) break;   // nothing fits: the longest-resting block returns
    }
    if (pick == c->free_blocks.end())
        return fail(c, DELTA_ERR_OOM_ARENA, "no arena block of %llu bytes (in use %llu of %llu)",
                    (unsigned long long)need, (unsigned long long)c->st.arena_in_use,
                    (unsigned long long)c->arena_bytes);
    const uint64_t o = pick->first;
    Block b = pick->second;
    c->free_blocks.erase(pick);
    const uint64_t at = top ? o + b.size - need : o;             // the end of the block that faces the population's side
    if (b.size > need) {
        Block rest;
        rest.size = b.size - need;
        rest.fence = b.fence;
        c->free_blocks[top ? o : o + need] = rest;
    }
    for (int s = 0; s < N_STREAMS; ++s)
        if (s != for_stream && b.fence.ev[s])
            HIP_TRY(c, hipStreamWaitEvent(c->stream[for_stream], b.fence.ev[s].e, 0));
    c->used[at] = need;
    c->st.arena_in_use += need;
    if (c->st.arena_in_use > c->st.arena_high_water) c->st.arena_high_water = c->st.arena_in_use;
    if (top) {
        if (c->arena_bytes - at > c->st.arena_top_extent_high_water) c->st.arena_top_extent_high_water = c->arena_bytes - at;
    } else if (at + need > c->st.arena_extent_high_water) {
        c->st.arena_extent_high_water = at + need;
    }
    *off = at;
    return DELTA_OK;
}

void arena_free(delta_ctx *c, uint64_t off, const Fence &f) {
    std::map<uint64_t, uint64_t>::iterator u = c->used.find(off);
    if (u == c->used.end()) return;
    Resting r;
    r.offset = off;
    r.block.size = u->second;
    r.block.fence = f;
    r.order = ++c->free_seq;
    c->st.arena_in_use -= r.block.size;
    c->used.erase(u);
    if (f.ev[S_D2H] || f.ev[S_H2D]) {                           // a copy may still be at it: rest until needed
        c->copying.push_back(r);
    } else if (f.ev[S_AUX]) {                                    // a weight gradient may still read it: rest a while
        c->cooling.push_back(r);
        if (c->cooling.size() > kCooling) {
            insert_free(c, c->cooling.front().offset, c->cooling.front().block);
            c->cooling.pop_front();
        }
    } else {
        insert_free(c, off, r.block);
    }
}

// Device address of the file-scope scratch array on the context's GPU, resolved once per device.
// The context's device must be the current one: every GPU holds its own copy at its own address.
hipError_t static_scratch_for(int device, void **out) {
    if (device < 0 || device >= kMaxDevices) return hipErrorInvalidDevice;
    if (!g_static_scratch[device]) {
        int cur = -1;
        hipError_t e = hipGetDevice(&cur);
        if (e != hipSuccess) return e;
        if (cur != device) return hipErrorInvalidDevice;
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        g_static_scratch[device] = p;
    }
    *out = g_static_scratch[device];
    return hipSuccess;
}

delta_status check_id(delta_ctx *c, uint32_t t) {
    if (t >= c->tensors.size()) return fail(c, DELTA_ERR_INVALID, "tensor id %u out of range (%zu bound)", t, c->tensors.size());
    return DELTA_OK;
}

// The compute stream is about to touch tensor t: wait for a reload still in flight.
delta_status compute_uses(delta_ctx *c, Tensor &t) {
    if (t.h2d_done) {
        HIP_TRY(c, hipStreamWaitEvent(c->stream[S_COMPUTE], t.h2d_done.e, 0));
        t.h2d_done = Ev();
    }
    return DELTA_OK;
}

// Returns the tensor's block to the arena.  Its next owner must wait for: everything the
// compute stream was told to do with it so far, an Offload copy still reading it, and a
// Reload nobody waited for yet that still writes it.
delta_status drop_block(delta_ctx *c, Tensor &t) {
    Fence f;
    delta_status r = new_event(c, c->stream[S_COMPUTE], &f.ev[S_COMPUTE]);
    if (r != DELTA_OK) return r;
    f.ev[S_D2H] = t.d2h_done;
    f.ev[S_H2D] = t.h2d_done;
    f.ev[S_AUX] = t.aux_done;
    t.h2d_done = t.aux_done = Ev();
    arena_free(c, t.offset, f);
    t.resident = false;
    return DELTA_OK;
}

// Adds a slab of at least `bytes` to the pinned pool.
delta_status pool_grow(delta_ctx *c, uint64_t bytes) {
    Slab sl;
    sl.size = bytes < kSlabMin ? kSlabMin : (bytes + kAlign - 1) / kAlign * kAlign;
    sl.used = 0;
    void *p = nullptr;
    hipError_t e = hipHostMalloc(&p, sl.size, hipHostMallocDefault);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        return fail(c, DELTA_ERR_OOM_PINNED, "hipHostMalloc(%llu) failed: %s", (unsigned long long)sl.size, hipGetErrorString(e));
    }
    sl.base = static_cast<unsigned char *>(p);
    c->slabs.push_back(sl);
    c->st.pinned_bytes += sl.size;
    return DELTA_OK;
}

// A host buffer for tensor t from the pool (first slab with room; a new slab when none has: the
// only place where a replay can still reach hipHostMalloc, and delta_reserve_pinned avoids it).
delta_status pool_take(delta_ctx *c, Tensor &t) {
    const uint64_t need = ((t.bytes ? t.bytes : 1) + kAlign - 1) / kAlign * kAlign;
    for (int pass = 0; pass < 2; ++pass) {
        for (size_t i = 0; i < c->slabs.size(); ++i) {
            Slab &sl = c->slabs[i];
            if (sl.size - sl.used >= need) {
                t.host = sl.base + sl.used;
                sl.used += need;
                return DELTA_OK;
            }
        }
        delta_status r = pool_grow(c, need);
        if (r != DELTA_OK) return r;
    }
    return fail(c, DELTA_ERR_OOM_PINNED, "pinned pool: no room for %llu bytes", (unsigned long long)need);
}

delta_status swap_out_impl(delta_ctx *c, uint32_t id) {
    Tensor &t = c->tensors[id];
    if (!t.resident) return fail(c, DELTA_ERR_STATE, "swap_out: tensor %u is not resident", id);
    if (!t.host) {
        delta_status pr = pool_take(c, t);
        if (pr != DELTA_OK) return pr;
    }
    Ev produced;
    delta_status r = new_event(c, c->stream[S_COMPUTE], &produced);
    if (r != DELTA_OK) return r;
    HIP_TRY(c, hipStreamWaitEvent(c->stream[S_D2H], produced.e, 0));
    if (t.h2d_done) HIP_TRY(c, hipStreamWaitEvent(c->stream[S_D2H], t.h2d_done.e, 0));
    // A large tensor goes out as four copies, each followed by an event of its own, so that a Reload of
    // the same tensor can follow its Offload piece by piece instead of waiting for the whole of it
    // (both directions of the link are then busy).  Four pieces whatever the size, and none below
    // 32 MiB: cutting every 16 MiB cost the large copies of the link-bound replays 6 % of their rate,
    // pieces of 6 MB cost the encoder's 24 MB tensors 9 %.
    t.d2h_piece.clear();
    if (!c->skip_copies && t.bytes) {
        const uint64_t piece = copy_piece_bytes(t.bytes);
        Timed tm;
        tm.dir = DELTA_DIR_D2H;
        if ((r = new_timing_event(c, c->stream[S_D2H], &tm.start)) != DELTA_OK) return r;
        for (uint64_t o = 0; o < t.bytes; o += piece) {
            const uint64_t nb = t.bytes - o < piece ? t.bytes - o : piece;
            HIP_TRY(c, hipMemcpyAsync(static_cast<unsigned char *>(t.host) + o, c->arena + t.offset + o, nb,
                                      hipMemcpyDeviceToHost, c->stream[S_D2H]));
            if (piece < t.bytes && o + nb < t.bytes) {           // the last piece's event is d2h_done
                Ev done;
                if ((r = new_event(c, c->stream[S_D2H], &done)) != DELTA_OK) return r;
                t.d2h_piece.push_back(done);
            }
        }
        if ((r = new_timing_event(c, c->stream[S_D2H], &tm.stop)) != DELTA_OK) return r;
        c->timed.push_back(tm);
    }
    if ((r = new_event(c, c->stream[S_D2H], &t.d2h_done)) != DELTA_OK) return r;
    t.host_valid = true;
    c->st.d2h_bytes += t.bytes;
    c->st.d2h_copies += 1;
    return DELTA_OK;
}

// Forgets every tensor's host buffer; the slabs stay (delta_bind) or go (delta_destroy).
void free_host_buffers(delta_ctx *c, bool slabs_too) {
    for (size_t i = 0; i < c->tensors.size(); ++i) c->tensors[i].host = nullptr;
    for (size_t i = 0; i < c->slabs.size(); ++i) {
        c->slabs[i].used = 0;
        if (slabs_too) (void)hipHostFree(c->slabs[i].base);
    }
    if (slabs_too) {
        c->slabs.clear();
        c->st.pinned_bytes = 0;
    }
}

}  // namespace

// =========================================================================== C ABI

extern "C" {

delta_status delta_create(void *arena_dev, uint64_t arena_bytes, void *compute_stream, delta_ctx **out) {
    if (!out) return DELTA_ERR_INVALID;
    *out = nullptr;
    delta_ctx *c = new (std::nothrow) delta_ctx();
    if (!c) return DELTA_ERR_INVALID;
    if (arena_dev) {
        if (((uintptr_t)arena_dev % kAlign) || arena_bytes < kAlign) {
            delete c;
            return DELTA_ERR_INVALID;
        }
        if (hipGetDevice(&c->device) != hipSuccess) {
            delete c;
            return DELTA_ERR_HIP;
        }
        c->arena = static_cast<unsigned char *>(arena_dev);
        c->arena_bytes = arena_bytes / kAlign * kAlign;
        c->st.arena_bytes = c->arena_bytes;
        c->stream[S_COMPUTE] = static_cast<hipStream_t>(compute_stream);
        if (hipStreamCreateWithFlags(&c->stream[S_D2H], hipStreamNonBlocking) != hipSuccess ||
            hipStreamCreateWithFlags(&c->stream[S_H2D], hipStreamNonBlocking) != hipSuccess ||
            hipStreamCreateWithFlags(&c->stream[S_AUX], hipStreamNonBlocking) != hipSuccess) {
            delete c;
            return DELTA_ERR_HIP;
        }
        if (static_scratch_for(c->device, &c->static_scratch) != hipSuccess) {
            (void)hipGetLastError();
            c->static_scratch = nullptr;            // delta_batchnorm_static reports it; everything else works
        }
        Block b;
        b.size = c->arena_bytes;
        c->free_blocks[0] = b;
    }
    *out = c;
    return DELTA_OK;
}

void delta_destroy(delta_ctx *c) {
    if (!c) return;
    if (c->arena) {
        for (int s = 0; s < N_STREAMS; ++s) (void)hipStreamSynchronize(c->stream[s]);
        free_host_buffers(c, true);
        for (size_t i = 0; i < c->ev_live.size(); ++i) (void)hipEventDestroy(c->ev_live[i]);
        for (size_t i = 0; i < c->ev_pool.size(); ++i) (void)hipEventDestroy(c->ev_pool[i]);
        for (size_t i = 0; i < c->tev_pool.size(); ++i) (void)hipEventDestroy(c->tev_pool[i]);
        for (size_t i = 0; i < c->timed.size(); ++i) {
            (void)hipEventDestroy(c->timed[i].start);
            (void)hipEventDestroy(c->timed[i].stop);
        }
        if (c->bn_scratch) (void)hipFree(c->bn_scratch);
        if (c->ones) (void)hipFree(c->ones);
        if (c->zeros) (void)hipFree(c->zeros);
        (void)hipStreamDestroy(c->stream[S_D2H]);
        (void)hipStreamDestroy(c->stream[S_H2D]);
        (void)hipStreamDestroy(c->stream[S_AUX]);
    }
    delete c;
}

const char *delta_last_error(delta_ctx *c) { return c ? c->err.c_str() : "null context"; }

delta_status delta_plan(delta_ctx *c, const delta_tensor_desc *tensors, uint32_t n_tensors,
                        const delta_step_desc *steps, uint32_t n_steps, const delta_plan_params *params,
                        delta_event *out_events, uint32_t capacity, uint32_t *out_count, uint64_t *out_peak) {
    if (!c) return DELTA_ERR_INVALID;
    if (!out_count || (capacity && !out_events)) return fail(c, DELTA_ERR_INVALID, "null output argument");
    std::vector<delta::PlanTensor> T;
    std::vector<delta::PlanStep> S;
    std::string err;
    delta_status r = delta::load_graph(tensors, n_tensors, steps, n_steps, params, T, S, err);
    if (r != DELTA_OK) return fail(c, r, "%s", err.c_str());
    std::vector<delta_event> ev;
    uint64_t peak = 0;
    r = delta::run_plan(T, S, *params, ev, peak, err);
    *out_count = (uint32_t)ev.size();
    if (out_peak) *out_peak = peak;
    if (r != DELTA_OK) return fail(c, r, "%s", err.c_str());
    if (ev.size() > capacity)
        return fail(c, DELTA_ERR_BUFFER, "plan has %zu events, buffer holds %u", ev.size(), capacity);
    if (!ev.empty()) memcpy(out_events, ev.data(), ev.size() * sizeof(delta_event));
    return DELTA_OK;
}

delta_status delta_bind(delta_ctx *c, const uint64_t *bytes, uint32_t n) {
    delta_status r = need_gpu(c);
    if (r != DELTA_OK) return r;
    if (!bytes && n) return fail(c, DELTA_ERR_INVALID, "null sizes");
    if ((r = sync_all(c)) != DELTA_OK) return r;
    free_host_buffers(c, false);
    c->tensors.assign(n, Tensor());
    for (uint32_t i = 0; i < n; ++i) c->tensors[i].bytes = bytes[i];
    c->free_blocks.clear();
    c->used.clear();
    c->cooling.clear();
    c->copying.clear();
    Block b;
    b.size = c->arena_bytes;
    c->free_blocks[0] = b;
    c->st.arena_in_use = 0;
    return DELTA_OK;
}

delta_status delta_reserve_pinned(delta_ctx *c, uint64_t bytes) {
    delta_status r = need_gpu(c);
    if (r != DELTA_OK) return r;
    uint64_t room = 0;
    for (size_t i = 0; i < c->slabs.size(); ++i) room += c->slabs[i].size - c->slabs[i].used;
    // every tensor's buffer is rounded up to 256 bytes and must lie within one slab: one slab for the shortfall
    return room >= bytes ? DELTA_OK : pool_grow(c, bytes - room + kAlign * (uint64_t)c->tensors.size());
}

delta_status delta_alloc(delta_ctx *c, uint32_t id, void **dev_out) {
    delta_status r = need_gpu(c);
    if (r != DELTA_OK) return r;
    if ((r = check_id(c, id)) != DELTA_OK) return r;
    Tensor &t = c->tensors[id];
    if (t.resident) return fail(c, DELTA_ERR_STATE, "alloc: tensor %u is already resident", id);
    if ((r = arena_alloc(c, t.bytes, S_COMPUTE, &t.offset)) != DELTA_OK) return r;
    t.resident = true;
    t.host_valid = false;
    if (dev_out) *dev_out = c->arena + t.offset;
    return DELTA_OK;
}

delta_status delta_tensor_ptr(delta_ctx *c, uint32_t id, void **dev_out) {
    delta_status r = need_gpu(c);
    if (r != DELTA_OK) return r;
    if ((r = check_id(c, id)) != DELTA_OK) return r;
    if (!dev_out) return fail(c, DELTA_ERR_INVALID, "null output argument");
    Tensor &t = c->tensors[id];
    if (!t.resident) {
        *dev_out = nullptr;
        return fail(c, DELTA_ERR_STATE, "tensor %u is not resident", id);
    }
    if ((r = compute_uses(c, t)) != DELTA_OK) return r;
    *dev_out = c->arena + t.offset;
    return DELTA_OK;
}

delta_status delta_swap_out(delta_ctx *c, uint32_t id) {
    delta_status r = need_gpu(c);
    if (r != DELTA_OK) return r;
    if ((r = check_id(c, id)) != DELTA_OK) return r;
    return swap_out_impl(c, id);
}

delta_status delta_release(delta_ctx *c, uint32_t id, uint32_t action) {
    delta_status r = need_gpu(c);
    if (r != DELTA_OK) return r;
    if ((r = check_id(c, id)) != DELTA_OK) return r;
    Tensor &t = c->tensors[id];
    if (!t.resident) return fail(c, DELTA_ERR_STATE, "release: tensor %u is not resident", id);
    switch (action) {
    case DELTA_EV_EVICT:
        t.host_valid = false;
        c->st.releases_evict += 1;
        return drop_block(c, t);
    case DELTA_EV_OFFLOAD:
        if (!t.host_valid && (r = swap_out_impl(c, id)) != DELTA_OK) return r;
        c->st.releases_offload += 1;
        return drop_block(c, t);
    case DELTA_EV_FREE:
    case DELTA_EV_DROP_TEMP:
        c->st.releases_free += 1;
        return drop_block(c, t);
    default:
        return fail(c, DELTA_ERR_INVALID, "release: action %u is not a release", action);
    }
}

delta_status delta_prefetch(delta_ctx *c, uint32_t id) {
    delta_status r = need_gpu(c);
    if (r != DELTA_OK) return r;
    if ((r = check_id(c, id)) != DELTA_OK) return r;
    Tensor &t = c->tensors[id];
    if (t.resident) return fail(c, DELTA_ERR_STATE, "prefetch: tensor %u is already resident", id);
    if (!t.host_valid || !t.host) return fail(c, DELTA_ERR_STATE, "prefetch: tensor %u has no host copy", id);
    if ((r = arena_alloc(c, t.bytes, S_H2D, &t.offset)) != DELTA_OK) return r;
    t.resident = true;
    // piece by piece behind an Offload of this tensor that may still be running (see swap_out_impl);
    // each piece is then timed on its own, so that the waits between them do not count as copy time
    const uint64_t piece = copy_piece_bytes(t.bytes);
    const uint64_t npieces = t.bytes ? (t.bytes + piece - 1) / piece : 0;
    const bool follow = t.d2h_done && !c->skip_copies && npieces > 1 && t.d2h_piece.size() == npieces - 1;
    if (t.d2h_done && !follow) HIP_TRY(c, hipStreamWaitEvent(c->stream[S_H2D], t.d2h_done.e, 0));
    if (!c->skip_copies && t.bytes) {
        Timed tm;
        tm.dir = DELTA_DIR_H2D;
        if (!follow && (r = new_timing_event(c, c->stream[S_H2D], &tm.start)) != DELTA_OK) return r;
        uint64_t j = 0;
        for (uint64_t o = 0; o < t.bytes; o += piece, ++j) {
            const uint64_t nb = t.bytes - o < piece ? t.bytes - o : piece;
            if (follow) {
                HIP_TRY(c, hipStreamWaitEvent(c->stream[S_H2D], (j + 1 < npieces ? t.d2h_piece[j] : t.d2h_done).e, 0));
                if ((r = new_timing_event(c, c->stream[S_H2D], &tm.start)) != DELTA_OK) return r;
            }
            HIP_TRY(c, hipMemcpyAsync(c->arena + t.offset + o, static_cast<const unsigned char *>(t.host) + o, nb,
                                      hipMemcpyHostToDevice, c->stream[S_H2D]));
            if (follow) {
                if ((r = new_timing_event(c, c->stream[S_H2D], &tm.stop)) != DELTA_OK) return r;
                c->timed.push_back(tm);
            }
        }
        if (!follow) {
            if ((r = new_timing_event(c, c->stream[S_H2D], &tm.stop)) != DELTA_OK) return r;
            c->timed.push_back(tm);
        }
    }
    if ((r = new_event(c, c->stream[S_H2D], &t.h2d_done)) != DELTA_OK) return r;
    c->st.h2d_bytes += t.bytes;
    c->st.h2d_copies += 1;
    return DELTA_OK;
}

// Shape and size checks of one layer; fills the launch arguments except device addresses.
static delta_status prepare_layer(delta_ctx *c, const delta_layer_desc &L, uint32_t i, delta::ConvArgs &a,
                                  delta::PoolArgs &pa, uint64_t &flops) {
    const size_t nt = c->tensors.size();
    if (L.x >= nt || L.y >= nt || (L.res != DELTA_NO_TENSOR && L.res >= nt))
        return fail(c, DELTA_ERR_INVALID, "layer %u: tensor id out of range", i);
    if (L.dtype != DELTA_DTYPE_F32 && L.dtype != DELTA_DTYPE_BF16)
        return fail(c, DELTA_ERR_INVALID, "layer %u: unknown dtype %u", i, L.dtype);
    if (L.y == L.x || L.y == L.res) return fail(c, DELTA_ERR_INVALID, "layer %u: output aliases an input", i);
    if (L.N <= 0 || L.H <= 0 || L.W <= 0 || L.Cin <= 0)
        return fail(c, DELTA_ERR_INVALID, "layer %u: non-positive dimension", i);
    const bool bf16 = L.dtype == DELTA_DTYPE_BF16;
    const uint64_t es = bf16 ? 2 : 4;
    const uint64_t xbytes = (uint64_t)L.N * L.H * L.W * L.Cin * es;
    if (c->tensors[L.x].bytes != xbytes)
        return fail(c, DELTA_ERR_INVALID, "layer %u: input tensor %u has %llu bytes, layer needs %llu", i, L.x,
                    (unsigned long long)c->tensors[L.x].bytes, (unsigned long long)xbytes);
    memset(&a, 0, sizeof a);
    memset(&pa, 0, sizeof pa);
    flops = 0;
    uint64_t ybytes = 0;
    switch (L.op) {
    case DELTA_OP_CONV: {
        if (L.stride <= 0 || L.R <= 0 || L.S <= 0 || L.pad < 0 || L.Cout <= 0)
            return fail(c, DELTA_ERR_INVALID, "layer %u: non-positive dimension", i);
        a.N = L.N; a.H = L.H; a.W = L.W; a.Cin = L.Cin; a.Cout = L.Cout; a.R = L.R; a.S = L.S;
        if (L.relu > DELTA_ACT_GELU) return fail(c, DELTA_ERR_INVALID, "layer %u: unknown activation %u", i, L.relu);
        a.stride = L.stride; a.pad = L.pad; a.relu = (int)L.relu; a.bf16 = bf16;
        a.P = (L.H + 2 * L.pad - L.R) / L.stride + 1;
        a.Q = (L.W + 2 * L.pad - L.S) / L.stride + 1;
        const long long M = (long long)L.N * a.P * a.Q;
        a.M = (M > 0 && M <= 0x7FFFFFFFLL) ? (int)M : -1;
        a.x = a.y = c->arena;                      // placeholders for the alignment checks
        a.res = nullptr;
        a.w = L.w; a.scale = L.scale; a.shift = L.shift;
        const char *why = delta::stem_applies(a) ? delta::stem_check(a) : delta::conv_check(a);
        if (why) return fail(c, DELTA_ERR_INVALID, "layer %u: %s", i, why);
        ybytes = (uint64_t)M * L.Cout * es;
        if (L.res != DELTA_NO_TENSOR) {
            if (delta::stem_applies(a)) return fail(c, DELTA_ERR_INVALID, "layer %u: the stem takes no residual", i);
            if (c->tensors[L.res].bytes != ybytes)
                return fail(c, DELTA_ERR_INVALID, "layer %u: residual tensor %u has the wrong size", i, L.res);
        }
        flops = 2ull * (uint64_t)M * L.R * L.S * L.Cin * L.Cout;
        break;
    }
    case DELTA_OP_MAXPOOL:
    case DELTA_OP_AVGPOOL: {
        pa.N = L.N; pa.H = L.H; pa.W = L.W; pa.C = L.Cin; pa.bf16 = bf16;
        pa.x = pa.y = c->arena;
        if (L.op == DELTA_OP_MAXPOOL) {
            if (L.stride <= 0 || L.R <= 0 || L.S <= 0 || L.pad < 0)
                return fail(c, DELTA_ERR_INVALID, "layer %u: bad pooling window", i);
            pa.R = L.R; pa.S = L.S; pa.stride = L.stride; pa.pad = L.pad;
            pa.P = (L.H + 2 * L.pad - L.R) / L.stride + 1;
            pa.Q = (L.W + 2 * L.pad - L.S) / L.stride + 1;
        } else {
            pa.P = pa.Q = 1;
        }
        const char *why = delta::pool_check(pa, L.op == DELTA_OP_AVGPOOL);
        if (why) return fail(c, DELTA_ERR_INVALID, "layer %u: %s", i, why);
        if (L.res != DELTA_NO_TENSOR) return fail(c, DELTA_ERR_INVALID, "layer %u: pooling takes no second input", i);
        ybytes = (uint64_t)L.N * pa.P * pa.Q * L.Cin * es;
        break;
    }
    case DELTA_OP_SOFTMAX_CE:
        if (L.H != 1 || L.W != 1) return fail(c, DELTA_ERR_INVALID, "layer %u: logits must be [N, classes]", i);
        if (L.res == DELTA_NO_TENSOR || c->tensors[L.res].bytes != (uint64_t)L.N * 8)
            return fail(c, DELTA_ERR_INVALID, "layer %u: labels tensor must hold N int64 values", i);
        ybytes = 4;
        break;
    case DELTA_OP_ATTENTION: {
        if (L.W != 1 || L.R <= 0 || L.Cout != 64 * L.R || L.Cin != 3 * L.Cout)
            return fail(c, DELTA_ERR_INVALID, "layer %u: attention needs W = 1, R heads of 64, Cout = 64 R, Cin = 3 Cout", i);
        if (L.res != DELTA_NO_TENSOR) return fail(c, DELTA_ERR_INVALID, "layer %u: attention takes no second input", i);
        const char *why = delta::attention_check(c->arena, c->arena, L.N, L.H, L.R, bf16);
        if (why) return fail(c, DELTA_ERR_INVALID, "layer %u: %s", i, why);
        ybytes = (uint64_t)L.N * L.H * L.Cout * es;
        flops = 4ull * (uint64_t)L.N * L.H * L.H * L.Cout;
        break;
    }
    case DELTA_OP_LAYERNORM: {
        if (L.Cout != L.Cin) return fail(c, DELTA_ERR_INVALID, "layer %u: layer normalisation keeps the shape", i);
        if (L.res != DELTA_NO_TENSOR) return fail(c, DELTA_ERR_INVALID, "layer %u: layer normalisation takes no second input", i);
        if (!(L.eps >= 0.f)) return fail(c, DELTA_ERR_INVALID, "layer %u: eps must be >= 0", i);
        const char *why = delta::layernorm_check(c->arena, c->arena, L.scale, L.shift, (long long)L.N * L.H * L.W, L.Cin, bf16);
        if (why) return fail(c, DELTA_ERR_INVALID, "layer %u: %s", i, why);
        ybytes = xbytes;
        break;
    }
    case DELTA_OP_BATCHNORM:
    case DELTA_OP_RELU:
    case DELTA_OP_ADD: {
        if (!bf16) return fail(c, DELTA_ERR_INVALID, "layer %u: this operator is bf16 only", i);
        if (L.Cout != L.Cin || L.Cin % 8) return fail(c, DELTA_ERR_INVALID, "layer %u: Cout = Cin, a multiple of 8", i);
        if ((L.op == DELTA_OP_ADD) != (L.res != DELTA_NO_TENSOR))
            return fail(c, DELTA_ERR_INVALID, "layer %u: add needs a second input, the others take none", i);
        if (L.op == DELTA_OP_ADD && c->tensors[L.res].bytes != xbytes)
            return fail(c, DELTA_ERR_INVALID, "layer %u: second input tensor %u has the wrong size", i, L.res);
        if (L.op == DELTA_OP_BATCHNORM) {
            if (!(L.eps >= 0.f)) return fail(c, DELTA_ERR_INVALID, "layer %u: eps must be >= 0", i);
            const char *why = delta::bn_train_check(c->arena, c->arena, L.scale, L.shift, (long long)L.N * L.H * L.W, L.Cin, bf16);
            if (why) return fail(c, DELTA_ERR_INVALID, "layer %u: %s", i, why);
        }
        ybytes = xbytes;
        break;
    }
    default:
        return fail(c, DELTA_ERR_INVALID, "layer %u: unknown operator %u", i, L.op);
    }
    if (c->tensors[L.y].bytes != ybytes)
        return fail(c, DELTA_ERR_INVALID, "layer %u: output tensor %u has %llu bytes, layer produces %llu", i, L.y,
                    (unsigned long long)c->tensors[L.y].bytes, (unsigned long long)ybytes);
    return DELTA_OK;
}

// The layers of a bottleneck that the block kernel runs in one launch (layers[i] carries DELTA_FUSE_BLOCK):
// three of an identity block (1x1 256 -> 64, 3x3, 1x1 64 -> 256 + the block's input), or four of a stage's
// first block (1x1 64 -> 64, 3x3, the projection shortcut 1x1 64 -> 256 of the block's input, 1x1 64 -> 256 +
// the projection).  Validates the chain and fills the launch arguments except device addresses; `n_block`
// is the number of layers the block takes.
static delta_status prepare_block(delta_ctx *c, const delta_layer_desc *layers, uint32_t n_layers, uint32_t i,
                                  delta::BlockArgs &b, uint64_t (&flops)[4], uint32_t &n_block) {
    if (i + 3 > n_layers) return fail(c, DELTA_ERR_INVALID, "layer %u: a fused block needs three or four layers", i);
    const bool proj = layers[i].Cin == 64;
    n_block = proj ? 4 : 3;
    if (i + n_block > n_layers) return fail(c, DELTA_ERR_INVALID, "layer %u: a fused block with a projection needs four layers", i);
    const delta_layer_desc &L1 = layers[i], &L2 = layers[i + 1], &L3 = layers[i + n_block - 1];
    delta::ConvArgs a;
    delta::PoolArgs pa;
    flops[3] = 0;
    for (uint32_t j = 0; j < n_block; ++j) {
        const delta_layer_desc &L = layers[i + j];
        if (L.op != DELTA_OP_CONV || L.dtype != DELTA_DTYPE_BF16)
            return fail(c, DELTA_ERR_INVALID, "layer %u: the block kernel takes bf16 convolutions", i + j);
        if (L.fuse & ~(uint32_t)(DELTA_FUSE_BLOCK | DELTA_FUSE_NO_STORE) || (j && (L.fuse & DELTA_FUSE_BLOCK)))
            return fail(c, DELTA_ERR_INVALID, "layer %u: bad fuse flags %u", i + j, L.fuse);
        delta_status r = prepare_layer(c, L, i + j, a, pa, flops[j]);
        if (r != DELTA_OK) return r;
    }
    auto one_by_one = [](const delta_layer_desc &L, int cin, int cout) {
        return L.R == 1 && L.S == 1 && L.stride == 1 && L.pad == 0 && (int)L.Cin == cin && (int)L.Cout == cout;
    };
    auto same_image = [&](const delta_layer_desc &L) { return L.N == L1.N && L.H == L1.H && L.W == L1.W; };
    bool geo = one_by_one(L1, proj ? 64 : 256, 64) && L2.R == 3 && L2.S == 3 && L2.stride == 1 && L2.pad == 1 && L2.Cin == 64 &&
               L2.Cout == 64 && one_by_one(L3, 64, 256) && same_image(L2) && same_image(L3);
    bool chain = L2.x == L1.y && L3.x == L2.y && L1.res == DELTA_NO_TENSOR && L2.res == DELTA_NO_TENSOR &&
                 L1.relu == DELTA_ACT_RELU && L2.relu == DELTA_ACT_RELU && L3.relu == DELTA_ACT_RELU;
    bool distinct = L1.y != L1.x && L2.y != L1.x && L3.y != L1.x && L1.y != L2.y && L1.y != L3.y && L2.y != L3.y;
    if (proj) {
        const delta_layer_desc &Lc = layers[i + 2];
        geo = geo && one_by_one(Lc, 64, 256) && same_image(Lc);
        chain = chain && Lc.x == L1.x && Lc.res == DELTA_NO_TENSOR && Lc.relu == DELTA_ACT_NONE && L3.res == Lc.y;
        distinct = distinct && Lc.y != L1.x && Lc.y != L1.y && Lc.y != L2.y && Lc.y != L3.y;
    } else {
        chain = chain && L3.res == L1.x;
    }
    if (!geo || !chain)
        return fail(c, DELTA_ERR_INVALID, "layer %u: not a bottleneck the block kernel takes (1x1 256->64, 3x3 64->64 s1 p1, "
                    "1x1 64->256 + the block's input, ReLU after each; or 1x1 64->64, 3x3, the projection 1x1 64->256 of the "
                    "block's input without ReLU, 1x1 64->256 + the projection)", i);
    if (!distinct) return fail(c, DELTA_ERR_INVALID, "layer %u: the block's tensors must be distinct", i);
    uint32_t all_skipped = DELTA_FUSE_NO_STORE;
    for (uint32_t j = 0; j < n_block; ++j) all_skipped &= layers[i + j].fuse;
    if (all_skipped) return fail(c, DELTA_ERR_INVALID, "layer %u: the block stores nothing", i);
    memset(&b, 0, sizeof b);
    b.N = L1.N; b.H = L1.H; b.W = L1.W;
    b.M = (int)((long long)L1.N * L1.H * L1.W);
    b.w1 = L1.w; b.w2 = L2.w; b.w3 = L3.w;
    b.s1 = L1.scale; b.h1 = L1.shift; b.s2 = L2.scale; b.h2 = L2.shift; b.s3 = L3.scale; b.h3 = L3.shift;
    if (proj) {
        const delta_layer_desc &Lc = layers[i + 2];
        b.proj = 1; b.wsc = Lc.w; b.ssc = Lc.scale; b.hsc = Lc.shift;
    }
    b.x = c->arena;                                  // placeholders for the checks
    b.out = c->arena;
    const char *why = delta::bottleneck_block_check(b);
    if (why) return fail(c, DELTA_ERR_INVALID, "layer %u: %s", i, why);
    return DELTA_OK;
}

// Makes tensor `y` ready to be written on the compute stream: a fresh block, or its own one once
// nobody else is still reading it.
static delta_status claim_output(delta_ctx *c, Tensor &ty) {
    delta_status r;
    if (!ty.resident) {
        if ((r = arena_alloc(c, ty.bytes, S_COMPUTE, &ty.offset)) != DELTA_OK) return r;
        ty.resident = true;
    } else {
        if ((r = compute_uses(c, ty)) != DELTA_OK) return r;
        if (ty.d2h_done)                            // an Offload copy may still be reading it
            HIP_TRY(c, hipStreamWaitEvent(c->stream[S_COMPUTE], ty.d2h_done.e, 0));
        if (ty.aux_done)                            // and so may a weight gradient
            HIP_TRY(c, hipStreamWaitEvent(c->stream[S_COMPUTE], ty.aux_done.e, 0));
    }
    ty.host_valid = false;                          // the host copy, if any, is of older contents
    return DELTA_OK;
}

delta_status delta_recompute_segment(delta_ctx *c, const delta_layer_desc *layers, uint32_t n_layers) {
    delta_status r = need_gpu(c);
    if (r != DELTA_OK) return r;
    if (!layers && n_layers) return fail(c, DELTA_ERR_INVALID, "null layers");
    delta::ConvArgs a;
    delta::PoolArgs pa;
    delta::BlockArgs blk;
    uint64_t flops, bflops[4];
    uint32_t nb = 0;
    // Pass 1: validate everything before anything is launched or allocated.
    std::vector<uint8_t> will_exist(c->tensors.size(), 0);
    for (uint32_t i = 0; i < n_layers; ++i) {
        const delta_layer_desc &L = layers[i];
        if (L.op == DELTA_OP_CONV && (L.fuse & DELTA_FUSE_BLOCK)) {
            if ((r = prepare_block(c, layers, n_layers, i, blk, bflops, nb)) != DELTA_OK) return r;
            if (!c->tensors[L.x].resident && !will_exist[L.x])
                return fail(c, DELTA_ERR_STATE, "layer %u: input tensor %u is not resident", i, L.x);
            for (uint32_t j = 0; j < nb; ++j)
                if (!(layers[i + j].fuse & DELTA_FUSE_NO_STORE)) will_exist[layers[i + j].y] = 1;
            i += nb - 1;
            continue;
        }
        if (L.fuse) return fail(c, DELTA_ERR_INVALID, "layer %u: fuse flags %u outside a fused block", i, L.fuse);
        if ((r = prepare_layer(c, L, i, a, pa, flops)) != DELTA_OK) return r;
        if (!c->tensors[L.x].resident && !will_exist[L.x])
            return fail(c, DELTA_ERR_STATE, "layer %u: input tensor %u is not resident", i, L.x);
        if (L.res != DELTA_NO_TENSOR && !c->tensors[L.res].resident && !will_exist[L.res])
            return fail(c, DELTA_ERR_STATE, "layer %u: second input tensor %u is not resident", i, L.res);
        will_exist[L.y] = 1;
    }
    // Pass 2: allocate outputs and launch, in order, on the compute stream.
    for (uint32_t i = 0; i < n_layers; ++i) {
        const delta_layer_desc &L = layers[i];
        if (L.op == DELTA_OP_CONV && (L.fuse & DELTA_FUSE_BLOCK)) {
            if ((r = prepare_block(c, layers, n_layers, i, blk, bflops, nb)) != DELTA_OK) return r;
            Tensor &tx = c->tensors[L.x];
            if ((r = compute_uses(c, tx)) != DELTA_OK) return r;
            void *outp[4] = {nullptr, nullptr, nullptr, nullptr};
            for (uint32_t j = 0; j < nb; ++j) {
                if (layers[i + j].fuse & DELTA_FUSE_NO_STORE) continue;
                Tensor &ty = c->tensors[layers[i + j].y];
                if ((r = claim_output(c, ty)) != DELTA_OK) return r;
                outp[j] = c->arena + ty.offset;
            }
            blk.x = c->arena + tx.offset;
            blk.a1 = outp[0]; blk.a2 = outp[1];
            if (nb == 4) {                          // a1, a2, the projection, out
                blk.sc = outp[2]; blk.out = outp[3];
                c->st.recompute_flops += bflops[0] + ((outp[1] || outp[2] || outp[3]) ? bflops[1] : 0) +
                                         ((outp[2] || outp[3]) ? bflops[2] : 0) + (outp[3] ? bflops[3] : 0);
            } else {
                blk.out = outp[2];
                c->st.recompute_flops += bflops[0] + ((outp[1] || outp[2]) ? bflops[1] : 0) + (outp[2] ? bflops[2] : 0);
            }
            HIP_TRY(c, delta::launch_bottleneck_block(blk, c->stream[S_COMPUTE]));
            c->st.recompute_launches += 1;
            i += nb - 1;
            continue;
        }
        if ((r = prepare_layer(c, L, i, a, pa, flops)) != DELTA_OK) return r;
        Tensor &tx = c->tensors[L.x];
        Tensor &ty = c->tensors[L.y];
        if ((r = compute_uses(c, tx)) != DELTA_OK) return r;
        if (L.res != DELTA_NO_TENSOR && (r = compute_uses(c, c->tensors[L.res])) != DELTA_OK) return r;
        if ((r = claim_output(c, ty)) != DELTA_OK) return r;
        unsigned char *xp = c->arena + tx.offset, *yp = c->arena + ty.offset;
        unsigned char *rp = L.res != DELTA_NO_TENSOR ? c->arena + c->tensors[L.res].offset : nullptr;
        switch (L.op) {
        case DELTA_OP_CONV:
            a.x = xp; a.y = yp; a.res = rp;
            if (delta::stem_applies(a)) HIP_TRY(c, delta::launch_stem(a, c->stream[S_COMPUTE]));
            else HIP_TRY(c, delta::launch_conv(a, c->stream[S_COMPUTE]));
            break;
        case DELTA_OP_MAXPOOL:
            pa.x = xp; pa.y = yp;
            HIP_TRY(c, delta::launch_maxpool(pa, c->stream[S_COMPUTE]));
            break;
        case DELTA_OP_AVGPOOL:
            pa.x = xp; pa.y = yp;
            HIP_TRY(c, delta::launch_avgpool(pa, c->stream[S_COMPUTE]));
            break;
        case DELTA_OP_ATTENTION:
            HIP_TRY(c, delta::launch_attention(xp, yp, L.N, L.H, L.R, L.dtype == DELTA_DTYPE_BF16, c->stream[S_COMPUTE]));
            break;
        case DELTA_OP_BATCHNORM:
            if (!c->bn_scratch) HIP_TRY(c, hipMalloc(&c->bn_scratch, delta::bn_train_scratch_bytes()));
            HIP_TRY(c, delta::launch_bn_train(xp, yp, L.scale, L.shift, (long long)L.N * L.H * L.W, L.Cin, L.eps, 1,
                                              c->bn_scratch, delta::bn_train_scratch_bytes(), c->stream[S_COMPUTE]));
            break;
        case DELTA_OP_RELU:
            HIP_TRY(c, delta::launch_relu(xp, yp, ty.bytes, 1, c->stream[S_COMPUTE]));
            break;
        case DELTA_OP_ADD:
            HIP_TRY(c, delta::launch_add(xp, rp, yp, ty.bytes, 1, c->stream[S_COMPUTE]));
            break;
        case DELTA_OP_LAYERNORM:
            HIP_TRY(c, delta::launch_layernorm(xp, yp, L.scale, L.shift, (long long)L.N * L.H * L.W, L.Cin, L.eps,
                                               L.dtype == DELTA_DTYPE_BF16, c->stream[S_COMPUTE]));
            break;
        default:
            HIP_TRY(c, delta::launch_softmax_ce(xp, rp, L.N, L.Cin, L.dtype == DELTA_DTYPE_BF16,
                                                reinterpret_cast<float *>(yp), c->stream[S_COMPUTE]));
            break;
        }
        c->st.recompute_launches += 1;
        c->st.recompute_flops += flops;
    }
    return DELTA_OK;
}

delta_status delta_batchnorm_static(delta_ctx *c, const void *x, void *y, const float *gamma, const float *beta,
                                    uint64_t rows, uint32_t channels, float eps) {
    delta_status r = need_gpu(c);
    if (r != DELTA_OK) return r;
    if (channels == 0 || channels % 8 || channels > 8192)
        return fail(c, DELTA_ERR_INVALID, "batchnorm_static: %u channels: must be a multiple of 8 and at most 8192 "
                    "(the static scratch of %zu bytes is sized for that)", channels, kStaticScratchBytes);
    if (rows == 0 || rows > (uint64_t)1 << 40) return fail(c, DELTA_ERR_INVALID, "batchnorm_static: bad row count");
    if (!(eps >= 0.f)) return fail(c, DELTA_ERR_INVALID, "batchnorm_static: eps must be >= 0");
    if (x == y) return fail(c, DELTA_ERR_INVALID, "batchnorm_static: output aliases the input");
    const char *why = delta::bn_train_check(x, y, gamma, beta, (long long)rows, (int)channels, 1);
    if (why) return fail(c, DELTA_ERR_INVALID, "batchnorm_static: %s", why);
    if (delta::bn_train_fwd_scratch_bytes() > kStaticScratchBytes)
        return fail(c, DELTA_ERR_INVALID, "batchnorm_static: the kernels need more scratch than the static array holds");
    if (!c->static_scratch) {
        hipError_t e = static_scratch_for(c->device, &c->static_scratch);
        if (e != hipSuccess) {
            (void)hipGetLastError();
            return fail(c, DELTA_ERR_HIP, "batchnorm_static: hipGetSymbolAddress(scratch) failed: %s", hipGetErrorString(e));
        }
    }
    // Nothing in the scratch has to start at zero: every partial sum and factor the later kernels of
    // this call read is written by an earlier kernel of this call.
    HIP_TRY(c, delta::launch_bn_train(x, y, gamma, beta, (long long)rows, (int)channels, eps, 1, c->static_scratch,
                                      kStaticScratchBytes, c->stream[S_COMPUTE]));
    return DELTA_OK;
}

delta_status delta_sync(delta_ctx *c, uint32_t which) {
    delta_status r = need_gpu(c);
    if (r != DELTA_OK) return r;
    if (which == 0 || (which & ~(uint32_t)DELTA_SYNC_ALL)) return fail(c, DELTA_ERR_INVALID, "bad sync mask %u", which);
    if (which == DELTA_SYNC_ALL) return sync_all(c);
    if (which & DELTA_SYNC_COMPUTE) {
        HIP_TRY(c, hipStreamSynchronize(c->stream[S_COMPUTE]));
        HIP_TRY(c, hipStreamSynchronize(c->stream[S_AUX]));
    }
    if (which & DELTA_SYNC_D2H) HIP_TRY(c, hipStreamSynchronize(c->stream[S_D2H]));
    if (which & DELTA_SYNC_H2D) HIP_TRY(c, hipStreamSynchronize(c->stream[S_H2D]));
    return DELTA_OK;
}

delta_status delta_bn_fold(delta_ctx *c, const float *gamma, const float *beta, const float *mean,
                           const float *var, float eps, uint32_t C, float *scale, float *shift) {
    delta_status r = need_gpu(c);
    if (r != DELTA_OK) return r;
    if (!gamma || !beta || !mean || !var || !scale || !shift) return fail(c, DELTA_ERR_INVALID, "null pointer");
    HIP_TRY(c, delta::launch_bn_fold(gamma, beta, mean, var, eps, C, scale, shift, c->stream[S_COMPUTE]));
    return DELTA_OK;
}

delta_status delta_stats(delta_ctx *c, delta_stats_t *out) {
    delta_status r = need_gpu(c);
    if (r != DELTA_OK) return r;
    if (!out) return fail(c, DELTA_ERR_INVALID, "null output argument");
    HIP_TRY(c, hipStreamSynchronize(c->stream[S_D2H]));
    HIP_TRY(c, hipStreamSynchronize(c->stream[S_H2D]));
    if ((r = harvest_timings(c)) != DELTA_OK) return r;
    *out = c->st;
    return DELTA_OK;
}

delta_status delta_stats_reset(delta_ctx *c) {
    delta_status r = need_gpu(c);
    if (r != DELTA_OK) return r;
    HIP_TRY(c, hipStreamSynchronize(c->stream[S_D2H]));
    HIP_TRY(c, hipStreamSynchronize(c->stream[S_H2D]));
    if ((r = harvest_timings(c)) != DELTA_OK) return r;
    const uint64_t ab = c->st.arena_bytes, iu = c->st.arena_in_use, pb = c->st.pinned_bytes;
    memset(&c->st, 0, sizeof c->st);
    c->st.arena_bytes = ab;
    c->st.arena_in_use = c->st.arena_high_water = iu;
    // what is resident now counts towards the bottom population's extent (a replay starts from an empty arena)
    for (std::map<uint64_t, uint64_t>::iterator u = c->used.begin(); u != c->used.end(); ++u)
        if (u->first + u->second > c->st.arena_extent_high_water) c->st.arena_extent_high_water = u->first + u->second;
    c->st.pinned_bytes = pb;
    return DELTA_OK;
}

delta_status delta_set_skip_copies(delta_ctx *c, int32_t skip) {
    delta_status r = need_gpu(c);
    if (r != DELTA_OK) return r;
    c->skip_copies = skip != 0;
    return DELTA_OK;
}

// ---- probes

delta_status delta_probe_hostlink(delta_ctx *c, uint64_t bytes, uint32_t iters, uint32_t dir, double *out) {
    delta_status r = need_gpu(c);
    if (r != DELTA_OK) return r;
    if (!out || !bytes || !iters || dir > DELTA_DIR_BOTH) return fail(c, DELTA_ERR_INVALID, "bad probe arguments");
    void *h[2] = {nullptr, nullptr}, *d[2] = {nullptr, nullptr};
    delta_status rc = DELTA_OK;
    for (int i = 0; i < 2 && rc == DELTA_OK; ++i) {
        if (hipHostMalloc(&h[i], bytes, hipHostMallocDefault) != hipSuccess) rc = fail(c, DELTA_ERR_OOM_PINNED, "probe: hipHostMalloc failed");
        else if (hipMalloc(&d[i], bytes) != hipSuccess) rc = fail(c, DELTA_ERR_HIP, "probe: hipMalloc failed");
        else memset(h[i], 1, bytes);
    }
    if (rc == DELTA_OK) {
        const bool down = dir == DELTA_DIR_D2H || dir == DELTA_DIR_BOTH;
        const bool up = dir == DELTA_DIR_H2D || dir == DELTA_DIR_BOTH;
        hipError_t e = hipSuccess;
        for (int rep = 0; rep < 2 && e == hipSuccess; ++rep) {      // rep 0 warms up
            const uint32_t n = rep == 0 ? 2 : iters;
            (void)hipStreamSynchronize(c->stream[S_D2H]);
            (void)hipStreamSynchronize(c->stream[S_H2D]);
            std::chrono::steady_clock::time_point t0 = std::chrono::steady_clock::now();
            for (uint32_t i = 0; i < n && e == hipSuccess; ++i) {
                if (down) e = hipMemcpyAsync(h[0], d[0], bytes, hipMemcpyDeviceToHost, c->stream[S_D2H]);
                if (up && e == hipSuccess) e = hipMemcpyAsync(d[1], h[1], bytes, hipMemcpyHostToDevice, c->stream[S_H2D]);
            }
            if (e == hipSuccess) e = hipStreamSynchronize(c->stream[S_D2H]);
            if (e == hipSuccess) e = hipStreamSynchronize(c->stream[S_H2D]);
            const double sec = std::chrono::duration<double>(std::chrono::steady_clock::now() - t0).count();
            if (rep == 1) *out = (double)bytes * n * ((down ? 1 : 0) + (up ? 1 : 0)) / sec / 1e9;
        }
        if (e != hipSuccess) rc = fail(c, DELTA_ERR_HIP, "probe copy failed: %s", hipGetErrorString(e));
    }
    for (int i = 0; i < 2; ++i) {
        if (h[i]) (void)hipHostFree(h[i]);
        if (d[i]) (void)hipFree(d[i]);
    }
    return rc;
}

delta_status delta_probe_hbm(delta_ctx *c, uint64_t bytes, uint32_t iters, double *out) {
    delta_status r = need_gpu(c);
    if (r != DELTA_OK) return r;
    if (!out || bytes < 16 || !iters) return fail(c, DELTA_ERR_INVALID, "bad probe arguments");
    void *a = nullptr, *b = nullptr;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    delta_status rc = DELTA_OK;
    hipStream_t s = c->stream[S_COMPUTE];
    if (hipMalloc(&a, bytes) != hipSuccess || hipMalloc(&b, bytes) != hipSuccess) rc = fail(c, DELTA_ERR_HIP, "probe: hipMalloc failed");
    if (rc == DELTA_OK && (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess)) rc = fail(c, DELTA_ERR_HIP, "probe: event");
    if (rc == DELTA_OK) {
        hipError_t e = hipMemsetAsync(a, 1, bytes, s);
        for (int i = 0; i < 2 && e == hipSuccess; ++i) e = delta::launch_copy(a, b, bytes, s);
        if (e == hipSuccess) e = hipEventRecord(e0, s);
        for (uint32_t i = 0; i < iters && e == hipSuccess; ++i) e = delta::launch_copy(a, b, bytes, s);
        if (e == hipSuccess) e = hipEventRecord(e1, s);
        if (e == hipSuccess) e = hipEventSynchronize(e1);
        float ms = 0.f;
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
        if (e != hipSuccess) rc = fail(c, DELTA_ERR_HIP, "probe failed: %s", hipGetErrorString(e));
        else *out = 2.0 * (double)(bytes / 16 * 16) * iters / (ms * 1e-3) / 1e9;
    }
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    if (a) (void)hipFree(a);
    if (b) (void)hipFree(b);
    return rc;
}

// ---------------------------------------------------------------- backward of a layer
namespace {

constexpr uint32_t kMaxChannels = 8192;

delta_status need_identity_factors(delta_ctx *c) {
    if (c->ones) return DELTA_OK;
    HIP_TRY(c, hipMalloc((void **)&c->ones, kMaxChannels * sizeof(float)));
    HIP_TRY(c, hipMalloc((void **)&c->zeros, kMaxChannels * sizeof(float)));
    std::vector<float> one(kMaxChannels, 1.0f);
    HIP_TRY(c, hipMemcpy(c->ones, one.data(), kMaxChannels * sizeof(float), hipMemcpyHostToDevice));
    HIP_TRY(c, hipMemset(c->zeros, 0, kMaxChannels * sizeof(float)));
    return DELTA_OK;
}

enum BwdKind { BK_CONV, BK_DENSE, BK_MAXPOOL, BK_AVGPOOL, BK_LOSS, BK_STEM, BK_BATCHNORM, BK_RELU };

bool is_stem(const delta_layer_desc &L) {
    return L.op == DELTA_OP_CONV && L.dtype == DELTA_DTYPE_BF16 && L.R == 7 && L.S == 7 && L.stride == 2 && L.pad == 3 &&
           L.Cin == 3 && L.Cout == 64 && L.res == DELTA_NO_TENSOR;
}

// The classifier (one pixel per image, a channel count the matrix-core kernels do not take) has its
// own small kernels; every other convolution goes through the convolution backward.
BwdKind bwd_kind(const delta_layer_desc &L) {
    if (L.op == DELTA_OP_MAXPOOL) return BK_MAXPOOL;
    if (L.op == DELTA_OP_AVGPOOL) return BK_AVGPOOL;
    if (L.op == DELTA_OP_SOFTMAX_CE) return BK_LOSS;
    if (L.op == DELTA_OP_BATCHNORM) return BK_BATCHNORM;
    if (L.op == DELTA_OP_RELU) return BK_RELU;
    if (is_stem(L)) return BK_STEM;
    if (L.H == 1 && L.W == 1 && L.R == 1 && L.S == 1 && L.stride == 1 && L.pad == 0 && L.Cout % 64 != 0) return BK_DENSE;
    return BK_CONV;
}

// The stem: weight gradient only (its input is the network's input).
delta_status prepare_backward_stem(delta_ctx *c, const delta_bwd_desc &D, uint32_t i, delta::ConvArgs &fa) {
    delta::PoolArgs pa;
    uint64_t flops = 0;
    const delta_layer_desc &L = D.fwd;
    delta_status r = prepare_layer(c, L, i, fa, pa, flops);
    if (r != DELTA_OK) return r;
    const size_t nt = c->tensors.size();
    if (D.gx != DELTA_NO_TENSOR || D.gx_add != DELTA_NO_TENSOR || D.mask_gx)
        return fail(c, DELTA_ERR_INVALID, "backward %u: the stem has a weight gradient only (gx, gx_add, mask_gx unused)", i);
    if (!D.gw || ((uintptr_t)D.gw & 15)) return fail(c, DELTA_ERR_INVALID, "backward %u: gw missing or misaligned", i);
    const uint64_t ybytes = c->tensors[L.y].bytes;
    if (D.gy >= nt || D.gpre >= nt || c->tensors[D.gy].bytes != ybytes || c->tensors[D.gpre].bytes != ybytes)
        return fail(c, DELTA_ERR_INVALID, "backward %u: gy and gpre must have the bytes of y", i);
    const bool own_mask = L.relu && !D.gy_masked;
    if (own_mask ? (D.gpre == D.gy || D.gpre == L.y || D.gpre == L.x) : D.gpre != D.gy)
        return fail(c, DELTA_ERR_INVALID, "backward %u: gpre must be a separate tensor exactly when a ReLU mask is applied", i);
    if (!D.workspace || ((uintptr_t)D.workspace & 255) || D.workspace_bytes < delta::stem_wgrad_workspace_bytes(fa))
        return fail(c, DELTA_ERR_INVALID, "backward %u: workspace missing, not 256-byte aligned or too small", i);
    return DELTA_OK;
}

// Pooling, classifier, loss, batch normalisation with batch statistics and ReLU: validation only
// (bf16).  gx is required; gpre must be gy; no gx_add.
delta_status prepare_backward_other(delta_ctx *c, const delta_bwd_desc &D, uint32_t i, BwdKind kind,
                                    delta::ConvArgs &fa, delta::PoolArgs &pa) {
    uint64_t flops = 0;
    const delta_layer_desc &L = D.fwd;
    delta_status r = prepare_layer(c, L, i, fa, pa, flops);
    if (r != DELTA_OK) return r;
    if (L.dtype != DELTA_DTYPE_BF16) return fail(c, DELTA_ERR_INVALID, "backward %u: this operator's backward is bf16 only", i);
    const size_t nt = c->tensors.size();
    if (D.gx == DELTA_NO_TENSOR && !(kind == BK_DENSE && D.gw))
        return fail(c, DELTA_ERR_INVALID, "backward %u: nothing to compute", i);
    if (D.gx != DELTA_NO_TENSOR &&
        (D.gx >= nt || c->tensors[D.gx].bytes != c->tensors[L.x].bytes || D.gx == L.x || D.gx == L.y || D.gx == D.gy))
        return fail(c, DELTA_ERR_INVALID, "backward %u: gx must be another tensor with the bytes of x", i);
    if (D.gx_add != DELTA_NO_TENSOR || (D.mask_gx && kind != BK_MAXPOOL) || D.gy_masked)
        return fail(c, DELTA_ERR_INVALID, "backward %u: gx_add and gy_masked are for convolutions only, mask_gx for "
                    "convolutions and max pooling", i);
    if (kind == BK_LOSS) {
        if (D.gy != DELTA_NO_TENSOR || D.gpre != DELTA_NO_TENSOR || D.gw)
            return fail(c, DELTA_ERR_INVALID, "backward %u: the loss takes no incoming gradient and has no weights", i);
        return DELTA_OK;
    }
    if (D.gy >= nt || c->tensors[D.gy].bytes != c->tensors[L.y].bytes || D.gpre != D.gy)
        return fail(c, DELTA_ERR_INVALID, "backward %u: gy must have the bytes of y and gpre must be gy", i);
    if (kind == BK_DENSE) {
        if (L.relu || L.res != DELTA_NO_TENSOR) return fail(c, DELTA_ERR_INVALID, "backward %u: classifier with ReLU or residual", i);
        if (D.gw && ((uintptr_t)D.gw & 15)) return fail(c, DELTA_ERR_INVALID, "backward %u: gw misaligned", i);
    } else if (kind == BK_BATCHNORM) {
        if (D.gw && ((uintptr_t)D.gw & 15)) return fail(c, DELTA_ERR_INVALID, "backward %u: gw misaligned", i);
    } else if (D.gw) {
        return fail(c, DELTA_ERR_INVALID, "backward %u: this operator has no weights", i);
    }
    return DELTA_OK;
}

// Validates one backward descriptor; fills the forward geometry (fa) and, if gx is asked for, the
// convolution that computes the data gradient (da).  Pointers in fa/da are placeholders.
// A 1x1 layer with stride > 1 touches only the input pixels (stride p, stride q): its gradients are
// computed at the output's resolution (input pixels gathered, data gradient spread back out).
bool strided_1x1(const delta_layer_desc &L) { return L.stride > 1 && L.R == 1 && L.S == 1 && L.pad == 0; }

// A 3x3 stride-2 pad-1 layer whose incoming gradient needs no mask of its own: input pixel (2i+a, 2j+b)
// only receives from the taps with r = a + 1 (mod 2) and s = b + 1 (mod 2), so its data gradient is four
// small convolutions of gy at the OUTPUT's resolution (1, 2, 2 and 4 taps: the nine taps once, where
// the stride-1 convolution of the zero-filled gradient does four times that work), each storing to
// its own parity class of gx.
bool class_dgrad(const delta_bwd_desc &D) {
    const delta_layer_desc &L = D.fwd;
    return L.stride == 2 && L.R == 3 && L.S == 3 && L.pad == 1 && D.gx != DELTA_NO_TENSOR && (!L.relu || D.gy_masked);
}

// The same layers' weight gradient by parity class (delta::launch_wgrad_s2): bf16, channel counts that
// are multiples of 128.  `fo`: the forward layer's own arguments.
bool class_layer(const delta_bwd_desc &D) {
    const delta_layer_desc &L = D.fwd;
    return L.stride == 2 && L.R == 3 && L.S == 3 && L.pad == 1 && (!L.relu || D.gy_masked);
}
bool class_wgrad(const delta_bwd_desc &D, const delta::ConvArgs &fo) { return D.gw && class_layer(D) && delta::wgrad_s2_applies(fo); }
// Everything such a layer was asked for runs at the output's resolution: no zero-filled copy of gy is
// needed, and the caller may say so by passing gpre = gy.
bool class_only(const delta_bwd_desc &D, const delta::ConvArgs &fo) {
    return class_layer(D) && (!D.gw || delta::wgrad_s2_applies(fo));
}

// Geometry of class (a, b): a convolution of gy [N,P,Q,Cout] with window (1+a) x (1+b) starting at
// the output pixel; tap t along a dimension of class 1 is r = 2 - 2t, i.e. index 2t of the flipped
// weights delta_bwd_weights prepares; class 0 uses r = 1, index 1.
void class_args(const delta_layer_desc &L, int bf16, int a, int b, delta::ConvArgs &ca) {
    memset(&ca, 0, sizeof ca);
    const int P = (L.H + 2 - 3) / 2 + 1, Q = (L.W + 2 - 3) / 2 + 1;
    ca.N = L.N; ca.H = P; ca.W = Q; ca.Cin = L.Cout; ca.Cout = L.Cin;
    ca.R = 1 + a; ca.S = 1 + b; ca.stride = 1; ca.pad = 0;
    ca.P = (L.H - a + 1) / 2; ca.Q = (L.W - b + 1) / 2;
    ca.M = ca.N * ca.P * ca.Q;
    ca.relu = 0; ca.bf16 = bf16;
    ca.oy_s = 2; ca.oy_a = a; ca.oy_b = b; ca.OH = L.H; ca.OW = L.W;
    ca.wR = 3; ca.wS = 3; ca.w_r0 = a ? 0 : 1; ca.w_s0 = b ? 0 : 1; ca.w_step = 2;
}

// `fa` (the forward layer's arguments) as the weight gradient sees the layer: stride 1.
void as_stride_1(const delta_layer_desc &L, delta::ConvArgs &fa) {
    if (strided_1x1(L)) { fa.H = fa.P; fa.W = fa.Q; }
    else { fa.P = L.H; fa.Q = L.W; }
    fa.stride = 1;
    fa.M = L.N * fa.P * fa.Q;
}

// Bytes of the staging tensor of a strided 1x1 layer (the gathered input pixels, and before that
// the data gradient at the output's resolution): N*P*Q*Cin elements, after the weight gradient's
// partial sums in the workspace.
uint64_t staging_bytes(const delta_layer_desc &L, const delta::ConvArgs &fa) {
    if (!strided_1x1(L)) return 0;
    const uint64_t b = (uint64_t)L.N * fa.P * fa.Q * L.Cin * (fa.bf16 ? 2 : 4);
    return (b + 255) / 256 * 256;
}
uint64_t partials_bytes(const delta::ConvArgs &fa) { return ((uint64_t)delta::wgrad_workspace_bytes(fa) + 255) / 256 * 256; }
// `fa` after as_stride_1
uint64_t backward_workspace_bytes(const delta_layer_desc &L, const delta::ConvArgs &fa) {
    uint64_t need = partials_bytes(fa) + staging_bytes(L, fa);
    if (L.stride == 2 && L.R == 3 && L.S == 3 && L.pad == 1) {          // whichever way the weight gradient goes
        delta::ConvArgs fo = fa;
        fo.stride = 2; fo.P = (L.H - 1) / 2 + 1; fo.Q = (L.W - 1) / 2 + 1; fo.M = L.N * fo.P * fo.Q;
        const uint64_t by_class = delta::wgrad_s2_workspace_bytes(fo);
        need = by_class > need ? by_class : need;
    }
    return need;
}

delta_status prepare_backward(delta_ctx *c, const delta_bwd_desc &D, uint32_t i, delta::ConvArgs &fa,
                              delta::ConvArgs &da) {
    delta::PoolArgs pa;
    uint64_t flops = 0;
    const delta_layer_desc &L = D.fwd;
    delta_status r = prepare_layer(c, L, i, fa, pa, flops);
    if (r != DELTA_OK) return r;
    if (L.op != DELTA_OP_CONV) return fail(c, DELTA_ERR_INVALID, "backward %u: operator %u has no backward here", i, L.op);
    if (delta::stem_applies(fa)) return fail(c, DELTA_ERR_INVALID, "backward %u: the stem convolution has no backward here", i);
    if (L.relu > DELTA_ACT_RELU) return fail(c, DELTA_ERR_INVALID, "backward %u: only ReLU layers have a backward here", i);
    if (2 * L.pad != L.R - 1 || 2 * L.pad != L.S - 1)
        return fail(c, DELTA_ERR_INVALID, "backward %u: needs 2*pad == R-1 == S-1", i);
    if (L.stride > 1 && L.res != DELTA_NO_TENSOR)
        return fail(c, DELTA_ERR_INVALID, "backward %u: a strided layer with a residual has no backward here", i);
    const size_t nt = c->tensors.size();
    const uint64_t ybytes = c->tensors[L.y].bytes, xbytes = c->tensors[L.x].bytes;
    // gpre lives at the input's resolution (for stride 1 that is y's), except for strided 1x1
    // layers, which are handled at the output's resolution
    const bool direct = strided_1x1(L);
    const delta::ConvArgs fo = fa;                       // the forward layer as it is (fa becomes its stride-1 view below)
    const bool no_spread = D.gpre == D.gy && class_only(D, fo);
    const uint64_t gpbytes = direct || no_spread ? ybytes : (uint64_t)L.N * L.H * L.W * L.Cout * (fa.bf16 ? 2 : 4);
    if (D.gy >= nt || D.gpre >= nt || c->tensors[D.gy].bytes != ybytes || c->tensors[D.gpre].bytes != gpbytes)
        return fail(c, DELTA_ERR_INVALID, "backward %u: gy must have the bytes of y, gpre N*H*W*Cout elements "
                    "(the bytes of y for a 1x1 layer)", i);
    const bool writes_gpre = (L.relu && !D.gy_masked) || (L.stride > 1 && !direct && !no_spread);
    if (!writes_gpre && D.gpre != D.gy)
        return fail(c, DELTA_ERR_INVALID, "backward %u: without a ReLU mask to apply and stride gpre must be gy itself", i);
    if (D.mask_gx && D.gx == DELTA_NO_TENSOR)
        return fail(c, DELTA_ERR_INVALID, "backward %u: mask_gx without gx", i);
    if (writes_gpre && (D.gpre == D.gy || D.gpre == L.y || D.gpre == L.x))
        return fail(c, DELTA_ERR_INVALID, "backward %u: gpre aliases another operand", i);
    if (D.gx != DELTA_NO_TENSOR) {
        if (D.gx >= nt || c->tensors[D.gx].bytes != xbytes)
            return fail(c, DELTA_ERR_INVALID, "backward %u: gx must be a tensor with the bytes of x", i);
        if (D.gx == D.gy || D.gx == D.gpre || D.gx == L.x || D.gx == L.y)
            return fail(c, DELTA_ERR_INVALID, "backward %u: gx aliases another operand", i);
        if (D.gx_add != DELTA_NO_TENSOR && (D.gx_add >= nt || c->tensors[D.gx_add].bytes != xbytes || D.gx_add == D.gx))
            return fail(c, DELTA_ERR_INVALID, "backward %u: gx_add must be another tensor with the bytes of x", i);
        if (!D.wt || ((uintptr_t)D.wt & 15)) return fail(c, DELTA_ERR_INVALID, "backward %u: wt missing or misaligned", i);
        if ((uint32_t)L.Cin > kMaxChannels) return fail(c, DELTA_ERR_INVALID, "backward %u: too many channels", i);
        memset(&da, 0, sizeof da);
        da.N = L.N; da.H = L.H; da.W = L.W; da.Cin = L.Cout; da.Cout = L.Cin; da.R = L.R; da.S = L.S;
        if (direct) { da.H = fa.P; da.W = fa.Q; }
        da.stride = 1; da.pad = L.R - 1 - L.pad; da.P = da.H; da.Q = da.W; da.M = L.N * da.H * da.W;
        da.relu = 0; da.bf16 = fa.bf16;
        da.x = da.y = c->arena; da.w = D.wt; da.scale = da.shift = reinterpret_cast<const float *>(c->arena);
        const char *why = delta::conv_check(da);
        if (why) return fail(c, DELTA_ERR_INVALID, "backward %u: data gradient: %s", i, why);
        if (class_dgrad(D)) {
            for (int cls = 0; cls < 4; ++cls) {
                delta::ConvArgs ca;
                class_args(L, fa.bf16, cls >> 1, cls & 1, ca);
                if (ca.P <= 0 || ca.Q <= 0) continue;              // a one-pixel-high or -wide input has no odd rows / columns
                ca.x = ca.y = c->arena; ca.w = D.wt; ca.scale = ca.shift = reinterpret_cast<const float *>(c->arena);
                if ((why = delta::conv_scatter_check(ca)) != nullptr)
                    return fail(c, DELTA_ERR_INVALID, "backward %u: data gradient by parity class: %s", i, why);
            }
        }
    } else if (D.gx_add != DELTA_NO_TENSOR) {
        return fail(c, DELTA_ERR_INVALID, "backward %u: gx_add without gx", i);
    }
    // the weight gradient sees the layer at stride 1 (gpre is at the input's resolution; a strided
    // 1x1 layer at the output's, on the gathered input pixels)
    as_stride_1(L, fa);
    if (D.gw) {
        const char *why = class_wgrad(D, fo) ? nullptr : delta::wgrad_check(fa);
        if (why) return fail(c, DELTA_ERR_INVALID, "backward %u: %s", i, why);
        if ((uintptr_t)D.gw & 15) return fail(c, DELTA_ERR_INVALID, "backward %u: gw misaligned", i);
    }
    if (D.gw || (direct && D.gx != DELTA_NO_TENSOR)) {
        if (!D.workspace || ((uintptr_t)D.workspace & 255) || D.workspace_bytes < backward_workspace_bytes(L, fa))
            return fail(c, DELTA_ERR_INVALID, "backward %u: workspace missing, not 256-byte aligned or too small", i);
    }
    return DELTA_OK;
}

// An output tensor of a launch on the compute stream: allocate it, or order the launch after
// whatever still touches its block.
delta_status compute_writes(delta_ctx *c, Tensor &t) {
    delta_status r;
    if (!t.resident) {
        if ((r = arena_alloc(c, t.bytes, S_COMPUTE, &t.offset, /*top=*/true)) != DELTA_OK) return r;   // a gradient tensor
        t.resident = true;
    } else {
        if ((r = compute_uses(c, t)) != DELTA_OK) return r;
        if (t.d2h_done) HIP_TRY(c, hipStreamWaitEvent(c->stream[S_COMPUTE], t.d2h_done.e, 0));
        if (t.aux_done) HIP_TRY(c, hipStreamWaitEvent(c->stream[S_COMPUTE], t.aux_done.e, 0));
    }
    t.host_valid = false;
    return DELTA_OK;
}

// Orders the compute stream after every weight gradient launched so far.
delta_status join_aux(delta_ctx *c) {
    if (c->aux_tail) {
        HIP_TRY(c, hipStreamWaitEvent(c->stream[S_COMPUTE], c->aux_tail.e, 0));
        c->aux_tail = Ev();
    }
    c->aux_lo = c->aux_hi = 0;
    c->stg_tail = Ev();
    c->stg_lo = c->stg_hi = 0;
    return DELTA_OK;
}

// Workspace bytes [p, p + n) are about to be used by a weight gradient on S_AUX / by the compute stream.
void aux_claims(delta_ctx *c, const void *p, uint64_t n) {
    const uintptr_t lo = (uintptr_t)p, hi = lo + n;
    if (c->aux_lo == c->aux_hi) { c->aux_lo = lo; c->aux_hi = hi; return; }
    if (lo < c->aux_lo) c->aux_lo = lo;
    if (hi > c->aux_hi) c->aux_hi = hi;
}
bool aux_holds(const delta_ctx *c, const void *p, uint64_t n) {
    const uintptr_t lo = (uintptr_t)p, hi = lo + n;
    return c->aux_tail && lo < c->aux_hi && c->aux_lo < hi;
}

}  // namespace

delta_status delta_bwd_weights(delta_ctx *c, const delta_layer_desc *layer, void *wt) {
    delta_status r = need_gpu(c);
    if (r != DELTA_OK) return r;
    if (!layer || !wt || ((uintptr_t)wt & 15)) return fail(c, DELTA_ERR_INVALID, "null or misaligned argument");
    const delta_layer_desc &L = *layer;
    if (L.op != DELTA_OP_CONV || !L.w || !L.scale || L.Cout <= 0 || L.Cin <= 0 || L.R <= 0 || L.S <= 0 ||
        (L.dtype != DELTA_DTYPE_F32 && L.dtype != DELTA_DTYPE_BF16))
        return fail(c, DELTA_ERR_INVALID, "not a convolution layer with weights and scale");
    HIP_TRY(c, delta::launch_bwd_weights(L.w, L.scale, wt, L.Cout, L.R, L.S, L.Cin, L.dtype == DELTA_DTYPE_BF16,
                                         c->stream[S_COMPUTE]));
    return DELTA_OK;
}

delta_status delta_backward_workspace(delta_ctx *c, const delta_layer_desc *layer, uint64_t *out_bytes) {
    delta_status r = need_gpu(c);
    if (r != DELTA_OK) return r;
    if (!layer || !out_bytes) return fail(c, DELTA_ERR_INVALID, "null argument");
    delta::ConvArgs a;
    delta::PoolArgs pa;
    uint64_t flops = 0;
    if ((r = prepare_layer(c, *layer, 0, a, pa, flops)) != DELTA_OK) return r;
    if (layer->op != DELTA_OP_CONV) { *out_bytes = 0; return DELTA_OK; }
    if (is_stem(*layer)) { *out_bytes = delta::stem_wgrad_workspace_bytes(a); return DELTA_OK; }
    as_stride_1(*layer, a);
    *out_bytes = backward_workspace_bytes(*layer, a);
    return DELTA_OK;
}

delta_status delta_backward_segment(delta_ctx *c, const delta_bwd_desc *descs, uint32_t n) {
    delta_status r = need_gpu(c);
    if (r != DELTA_OK) return r;
    if (!descs && n) return fail(c, DELTA_ERR_INVALID, "null descriptors");
    delta::ConvArgs fa, da;
    // Pass 1: validate everything, including residency as it will be when each step runs.
    std::vector<uint8_t> will_exist(c->tensors.size(), 0);
    auto there = [&](uint32_t t) { return c->tensors[t].resident || will_exist[t]; };
    for (uint32_t i = 0; i < n; ++i) {
        const delta_bwd_desc &D = descs[i];
        const BwdKind kind = bwd_kind(D.fwd);
        if (kind == BK_STEM) {
            if ((r = prepare_backward_stem(c, D, i, fa)) != DELTA_OK) return r;
            if (!there(D.gy)) return fail(c, DELTA_ERR_STATE, "backward %u: gy tensor %u is not resident", i, D.gy);
            if (!there(D.fwd.x)) return fail(c, DELTA_ERR_STATE, "backward %u: x tensor %u is not resident", i, D.fwd.x);
            if (D.fwd.relu && !D.gy_masked && !there(D.fwd.y))
                return fail(c, DELTA_ERR_STATE, "backward %u: y tensor %u is not resident", i, D.fwd.y);
            will_exist[D.gpre] = 1;
            continue;
        }
        if (kind != BK_CONV) {
            delta::PoolArgs pa;
            if ((r = prepare_backward_other(c, D, i, kind, fa, pa)) != DELTA_OK) return r;
            if (kind != BK_LOSS && !there(D.gy)) return fail(c, DELTA_ERR_STATE, "backward %u: gy tensor %u is not resident", i, D.gy);
            const bool needs_x = kind == BK_MAXPOOL || kind == BK_LOSS || kind == BK_BATCHNORM || (kind == BK_DENSE && D.gw);
            if (needs_x && !there(D.fwd.x)) return fail(c, DELTA_ERR_STATE, "backward %u: x tensor %u is not resident", i, D.fwd.x);
            if (kind == BK_RELU && !there(D.fwd.y)) return fail(c, DELTA_ERR_STATE, "backward %u: y tensor %u is not resident", i, D.fwd.y);
            if (kind == BK_LOSS && !there(D.fwd.res)) return fail(c, DELTA_ERR_STATE, "backward %u: labels are not resident", i);
            if (D.gx != DELTA_NO_TENSOR) will_exist[D.gx] = 1;
            continue;
        }
        if ((r = prepare_backward(c, D, i, fa, da)) != DELTA_OK) return r;
        if (!there(D.gy)) return fail(c, DELTA_ERR_STATE, "backward %u: gy tensor %u is not resident", i, D.gy);
        if (D.fwd.relu && !D.gy_masked && !there(D.fwd.y))
            return fail(c, DELTA_ERR_STATE, "backward %u: y tensor %u is not resident", i, D.fwd.y);
        if ((D.gw || D.mask_gx) && !there(D.fwd.x))
            return fail(c, DELTA_ERR_STATE, "backward %u: x tensor %u is not resident", i, D.fwd.x);
        if (D.gx_add != DELTA_NO_TENSOR && !there(D.gx_add))
            return fail(c, DELTA_ERR_STATE, "backward %u: gx_add tensor %u is not resident", i, D.gx_add);
        will_exist[D.gpre] = 1;
        if (D.gx != DELTA_NO_TENSOR) will_exist[D.gx] = 1;
    }
    if ((r = need_identity_factors(c)) != DELTA_OK) return r;
    hipStream_t s = c->stream[S_COMPUTE];
    for (uint32_t i = 0; i < n; ++i) {
        const delta_bwd_desc &D = descs[i];
        const delta_layer_desc &L = D.fwd;
        const BwdKind kind = bwd_kind(L);
        if (kind == BK_STEM) {
            if ((r = prepare_backward_stem(c, D, i, fa)) != DELTA_OK) return r;
            Tensor &tgy = c->tensors[D.gy];
            if ((r = compute_uses(c, tgy)) != DELTA_OK) return r;
            if (L.relu && !D.gy_masked) {
                Tensor &ty = c->tensors[L.y];
                if ((r = compute_uses(c, ty)) != DELTA_OK) return r;
                if ((r = compute_writes(c, c->tensors[D.gpre])) != DELTA_OK) return r;
                HIP_TRY(c, delta::launch_relu_mask(c->arena + ty.offset, c->arena + tgy.offset,
                                                   c->arena + c->tensors[D.gpre].offset, tgy.bytes, 1, s));
            }
            Tensor &tx = c->tensors[L.x];
            if ((r = compute_uses(c, tx)) != DELTA_OK) return r;
            fa.x = c->arena + tx.offset;
            if ((r = join_aux(c)) != DELTA_OK) return r;          // the workspace is shared with the layers before
            HIP_TRY(c, delta::launch_stem_wgrad(fa, c->arena + c->tensors[D.gpre].offset, static_cast<float *>(D.gw),
                                                D.workspace, D.workspace_bytes, s));
            c->st.recompute_flops += 2ull * (uint64_t)fa.M * 7 * 7 * 3 * 64;
            c->st.recompute_launches += 1;
            continue;
        }
        if (kind != BK_CONV) {
            delta::PoolArgs pa;
            if ((r = prepare_backward_other(c, D, i, kind, fa, pa)) != DELTA_OK) return r;
            const unsigned char *gyp = nullptr, *xp = nullptr;
            if (kind != BK_LOSS) {
                if ((r = compute_uses(c, c->tensors[D.gy])) != DELTA_OK) return r;
                gyp = c->arena + c->tensors[D.gy].offset;
            }
            if (c->tensors[L.x].resident) {
                if ((r = compute_uses(c, c->tensors[L.x])) != DELTA_OK) return r;
                xp = c->arena + c->tensors[L.x].offset;
            }
            unsigned char *gxp = nullptr;
            if (D.gx != DELTA_NO_TENSOR) {
                if ((r = compute_writes(c, c->tensors[D.gx])) != DELTA_OK) return r;
                gxp = c->arena + c->tensors[D.gx].offset;
            }
            switch (kind) {
            case BK_MAXPOOL:
                pa.x = xp;
                HIP_TRY(c, delta::launch_maxpool_bwd(pa, gyp, gxp, D.mask_gx ? 1 : 0, s));
                break;
            case BK_AVGPOOL:
                HIP_TRY(c, delta::launch_avgpool_bwd(pa, gyp, gxp, s));
                break;
            case BK_LOSS: {
                Tensor &tl = c->tensors[L.res];
                if ((r = compute_uses(c, tl)) != DELTA_OK) return r;
                HIP_TRY(c, delta::launch_softmax_ce_bwd(xp, c->arena + tl.offset, L.N, L.Cin, gxp, s));
                break;
            }
            case BK_BATCHNORM:
                if (!c->bn_scratch) HIP_TRY(c, hipMalloc(&c->bn_scratch, delta::bn_train_scratch_bytes()));
                HIP_TRY(c, delta::launch_bn_train_bwd(xp, gyp, gxp, L.scale, static_cast<float *>(D.gw),
                                                      (long long)L.N * L.H * L.W, L.Cin, L.eps, 1, c->bn_scratch, s));
                break;
            case BK_RELU: {
                Tensor &ty = c->tensors[L.y];
                if ((r = compute_uses(c, ty)) != DELTA_OK) return r;
                HIP_TRY(c, delta::launch_relu_mask(c->arena + ty.offset, gyp, gxp, c->tensors[D.gy].bytes, 1, s));
                break;
            }
            default:
                if (gxp) HIP_TRY(c, delta::launch_dense_bwd(xp, L.w, L.scale, gyp, gxp, nullptr, L.N, L.Cin, L.Cout, s));
                if (D.gw) {                                     // the weight gradient beside the chain, like the convolutions'
                    Ev ready;
                    if ((r = new_event(c, s, &ready)) != DELTA_OK) return r;
                    HIP_TRY(c, hipStreamWaitEvent(c->stream[S_AUX], ready.e, 0));
                    HIP_TRY(c, delta::launch_dense_bwd(xp, L.w, L.scale, gyp, nullptr, static_cast<float *>(D.gw), L.N, L.Cin,
                                                       L.Cout, c->stream[S_AUX]));
                    if ((r = new_event(c, c->stream[S_AUX], &c->aux_tail)) != DELTA_OK) return r;
                    c->tensors[L.x].aux_done = c->tensors[D.gy].aux_done = c->aux_tail;
                }
                break;
            }
            c->st.recompute_launches += 1;
            continue;
        }
        if ((r = prepare_backward(c, D, i, fa, da)) != DELTA_OK) return r;
        Tensor &tgy = c->tensors[D.gy];
        if ((r = compute_uses(c, tgy)) != DELTA_OK) return r;
        const bool own_mask = L.relu && !D.gy_masked;
        const bool direct = strided_1x1(L);
        const int outP = (L.H + 2 * L.pad - L.R) / L.stride + 1, outQ = (L.W + 2 * L.pad - L.S) / L.stride + 1;
        // A strided 1x1 layer stages both of its gradients at the END of the workspace; weight gradients
        // still running on the other stream use its beginning.  Only if the two ranges meet (a
        // workspace no larger than this layer needs) does the compute stream wait for them.
        const uint64_t stg_bytes = direct ? staging_bytes(L, fa) : 0;
        unsigned char *staging =
            direct ? static_cast<unsigned char *>(D.workspace) + ((D.workspace_bytes - stg_bytes) & ~(uint64_t)255) : nullptr;
        if (direct) {
            const uintptr_t lo = (uintptr_t)staging, hi = lo + stg_bytes;
            if (aux_holds(c, staging, stg_bytes)) {
                if ((r = join_aux(c)) != DELTA_OK) return r;
            } else if (c->stg_tail && lo < c->stg_hi && c->stg_lo < hi) {
                // only an earlier strided 1x1 layer's weight gradient used these bytes: wait for that one launch
                HIP_TRY(c, hipStreamWaitEvent(s, c->stg_tail.e, 0));
                c->stg_tail = Ev();
            }
        }
        delta::ConvArgs fo = fa;                             // the forward layer's own geometry (fa is its stride-1 view)
        fo.stride = L.stride; fo.P = outP; fo.Q = outQ; fo.M = L.N * outP * outQ;
        const bool no_spread = D.gpre == D.gy && class_only(D, fo);
        if (own_mask || (L.stride > 1 && !direct && !no_spread)) {
            Tensor &tgp = c->tensors[D.gpre];
            const unsigned char *yp = nullptr;
            if (own_mask) {
                Tensor &ty = c->tensors[L.y];
                if ((r = compute_uses(c, ty)) != DELTA_OK) return r;
                yp = c->arena + ty.offset;
            }
            if ((r = compute_writes(c, tgp)) != DELTA_OK) return r;
            if (L.stride == 1 || direct)
                HIP_TRY(c, delta::launch_relu_mask(yp, c->arena + tgy.offset, c->arena + tgp.offset, tgp.bytes,
                                                   fa.bf16, s));
            else
                HIP_TRY(c, delta::launch_relu_mask_dilate(yp, c->arena + tgy.offset, c->arena + tgp.offset, L.N, L.H,
                                                          L.W, outP, outQ, L.Cout, L.stride, fa.bf16, s));
        }
        const unsigned char *gp = c->arena + c->tensors[D.gpre].offset;
        Ev ready;
        if (D.gw && !direct) {
            if ((r = compute_uses(c, c->tensors[L.x])) != DELTA_OK) return r;
            if ((r = new_event(c, s, &ready)) != DELTA_OK) return r;
        }
        if (D.gx != DELTA_NO_TENSOR) {
            Tensor &tgx = c->tensors[D.gx];
            const unsigned char *addp = nullptr;
            if (D.gx_add != DELTA_NO_TENSOR) {
                if ((r = compute_uses(c, c->tensors[D.gx_add])) != DELTA_OK) return r;
                addp = c->arena + c->tensors[D.gx_add].offset;
            }
            const unsigned char *maskp = nullptr;
            if (D.mask_gx) {
                if ((r = compute_uses(c, c->tensors[L.x])) != DELTA_OK) return r;
                maskp = c->arena + c->tensors[L.x].offset;
            }
            if ((r = compute_writes(c, tgx)) != DELTA_OK) return r;
            da.x = gp; da.w = D.wt; da.res = addp; da.mask = maskp; da.y = c->arena + tgx.offset;
            da.scale = c->ones; da.shift = c->zeros;
            if (direct) { da.res = nullptr; da.mask = nullptr; da.y = staging; }
            if (class_dgrad(D)) {
                for (int cls = 0; cls < 4; ++cls) {
                    delta::ConvArgs ca;
                    class_args(L, fa.bf16, cls >> 1, cls & 1, ca);
                    if (ca.P <= 0 || ca.Q <= 0) continue;
                    ca.x = c->arena + tgy.offset; ca.w = D.wt; ca.res = addp; ca.mask = maskp; ca.y = c->arena + tgx.offset;
                    ca.scale = c->ones; ca.shift = c->zeros;
                    HIP_TRY(c, delta::launch_conv_scatter(ca, s));
                }
            } else
            HIP_TRY(c, delta::launch_conv(da, s));
            if (direct)
                HIP_TRY(c, delta::launch_spread_add(staging, addp, maskp, c->arena + tgx.offset, L.N, L.H, L.W, outP, outQ,
                                                    L.Cin, L.stride, fa.bf16, s));
            c->st.recompute_flops += class_dgrad(D) ? 2ull * (uint64_t)L.N * outP * outQ * 9 * L.Cin * L.Cout
                                                    : 2ull * (uint64_t)da.M * da.R * da.S * da.Cin * da.Cout;
        }
        if (D.gw) {
            Tensor &tx = c->tensors[L.x];
            if ((r = compute_uses(c, tx)) != DELTA_OK) return r;
            fa.x = c->arena + tx.offset;
            // gpre and x are complete once the compute stream reaches `ready` (for a strided 1x1 layer:
            // and the data gradient has left the staging area); from there the weight gradient runs on
            // its own stream, and both tensors remember that reader.
            if (direct && (r = new_event(c, s, &ready)) != DELTA_OK) return r;
            HIP_TRY(c, hipStreamWaitEvent(c->stream[S_AUX], ready.e, 0));
            if (direct) {
                HIP_TRY(c, delta::launch_subsample(fa.x, staging, L.N, L.H, L.W, outP, outQ, L.Cin, L.stride, fa.bf16,
                                                   c->stream[S_AUX]));
                fa.x = staging;
            }
            if (class_wgrad(D, fo)) {
                // by parity class, from gy itself (it needs no mask of this layer's) and x
                fo.x = fa.x;
                const uint64_t need = delta::wgrad_s2_workspace_bytes(fo);
                HIP_TRY(c, delta::launch_wgrad_s2(fo, c->arena + tgy.offset, static_cast<float *>(D.gw), D.workspace, need,
                                                  c->stream[S_AUX]));
                aux_claims(c, D.workspace, need);
                if ((r = new_event(c, c->stream[S_AUX], &c->aux_tail)) != DELTA_OK) return r;
                tx.aux_done = tgy.aux_done = c->aux_tail;
                c->st.recompute_flops += 2ull * (uint64_t)fo.M * 9 * fo.Cin * fo.Cout;
            } else {
                HIP_TRY(c, delta::launch_wgrad(fa, gp, static_cast<float *>(D.gw), D.workspace, partials_bytes(fa),
                                               c->stream[S_AUX]));
                aux_claims(c, D.workspace, partials_bytes(fa));
                if ((r = new_event(c, c->stream[S_AUX], &c->aux_tail)) != DELTA_OK) return r;
                tx.aux_done = c->tensors[D.gpre].aux_done = c->aux_tail;
                if (direct) {                                   // the staging range is tracked on its own
                    c->stg_tail = c->aux_tail;
                    c->stg_lo = (uintptr_t)staging;
                    c->stg_hi = c->stg_lo + stg_bytes;
                }
                c->st.recompute_flops += 2ull * (uint64_t)fa.M * fa.R * fa.S * fa.Cin * fa.Cout;
            }
        }
        c->st.recompute_launches += 1;
    }
    return DELTA_OK;
}

delta_status delta_backward_join(delta_ctx *c) {
    delta_status r = need_gpu(c);
    if (r != DELTA_OK) return r;
    return join_aux(c);
}

delta_status delta_layer_kernel(delta_ctx *c, const delta_layer_desc *layer, char *out, uint64_t cap) {
    delta_status r = need_gpu(c);
    if (r != DELTA_OK) return r;
    if (!layer || !out || cap == 0) return fail(c, DELTA_ERR_INVALID, "null argument");
    delta::ConvArgs a;
    delta::PoolArgs pa;
    uint64_t flops = 0;
    r = prepare_layer(c, *layer, 0, a, pa, flops);
    if (r != DELTA_OK) return r;
    const char *name = "?";
    switch (layer->op) {
    case DELTA_OP_CONV: name = delta::stem_applies(a) ? "stem7x7 bf16" : delta::conv_kernel_name(a); break;
    case DELTA_OP_MAXPOOL: name = "maxpool"; break;
    case DELTA_OP_AVGPOOL: name = "avgpool"; break;
    case DELTA_OP_SOFTMAX_CE: name = "softmax_ce"; break;
    case DELTA_OP_ATTENTION: name = "attention bf16 (256 queries x 8 waves, K/V in LDS)"; break;
    case DELTA_OP_LAYERNORM: name = "layernorm bf16"; break;
    case DELTA_OP_BATCHNORM: name = "batchnorm (batch statistics) bf16: stats + finalize + apply"; break;
    case DELTA_OP_RELU: name = "relu bf16"; break;
    case DELTA_OP_ADD: name = "add bf16"; break;
    default: break;
    }
    snprintf(out, (size_t)cap, "%s", name);
    return DELTA_OK;
}

delta_status delta_probe_mfma(delta_ctx *c, uint32_t iters, double *out) {
    delta_status r = need_gpu(c);
    if (r != DELTA_OK) return r;
    if (!out || !iters || iters > (1u << 24)) return fail(c, DELTA_ERR_INVALID, "bad probe arguments");
    float *buf = nullptr;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    delta_status rc = DELTA_OK;
    hipStream_t s = c->stream[S_COMPUTE];
    const int blocks = 256 * 8;
    if (hipMalloc((void **)&buf, 256) != hipSuccess) rc = fail(c, DELTA_ERR_HIP, "probe: hipMalloc failed");
    if (rc == DELTA_OK && (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess)) rc = fail(c, DELTA_ERR_HIP, "probe: event");
    if (rc == DELTA_OK) {
        hipError_t e = delta::launch_mfma_probe(buf, 16, blocks, s);
        if (e == hipSuccess) e = hipEventRecord(e0, s);
        if (e == hipSuccess) e = delta::launch_mfma_probe(buf, (int)iters, blocks, s);
        if (e == hipSuccess) e = hipEventRecord(e1, s);
        if (e == hipSuccess) e = hipEventSynchronize(e1);
        float ms = 0.f;
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
        if (e != hipSuccess) rc = fail(c, DELTA_ERR_HIP, "probe failed: %s", hipGetErrorString(e));
        else {
            // per wavefront and iteration: 4 MFMAs of 32x32x16 = 4 * 2*32*32*16 flops
            const double flops = (double)blocks * 4 /*waves*/ * iters * 4.0 * 2.0 * 32 * 32 * 16;
            *out = flops / (ms * 1e-3) / 1e12;
        }
    }
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    if (buf) (void)hipFree(buf);
    return rc;
}

}  // extern "C"
