/*
 * delta.h -- C ABI of the MI355X hot path behind DELTA (arXiv 2203.15980,
 * "Dynamically Optimizing GPU Memory beyond Tensor Recomputation").
 *
 * The library covers what DELTA's Filter and Director trade against each other:
 *   - planning: which resident activation to Release, and whether to Evict or
 *     Offload it (Algorithms 1-4, Eq. 1-6);
 *   - Evict / Recompute: dropping an activation and regenerating it by re-running
 *     the fused conv + BN-affine (+ residual) + ReLU layers that produced it;
 *   - Offload / Reload: copying an activation to pinned host memory and back on
 *     side streams that overlap the compute stream (Sec. 4.2).
 *
 * Conventions for every entry point
 *   - Plain C: no exceptions cross the boundary; every call returns a
 *     delta_status (0 = DELTA_OK, negative = error) and leaves a message that
 *     delta_last_error() returns.
 *   - "device" pointers are HIP device addresses on the context's GPU, "host"
 *     pointers are ordinary process memory.  The caller owns every array it
 *     passes; the library copies what it keeps before the call returns.
 *   - The caller owns the device arena and the compute stream handed to
 *     delta_create().  The library owns the context, its copy streams, its
 *     events, its pinned host pool, and sub-allocates the arena: the arena
 *     size is the physical budget (planned activations from its bottom upwards,
 *     the backward pass's gradient tensors from its end downwards).
 *   - delta_swap_out, delta_prefetch, delta_release and delta_recompute_segment
 *     only enqueue work; delta_sync (and delta_destroy) block the host.
 *   - One context is used from one host thread at a time.
 *   - There is no CPU fallback: calls that need the GPU fail with
 *     DELTA_ERR_HIP when no device is usable.
 */
#ifndef DELTA_H
#define DELTA_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct delta_ctx delta_ctx;
typedef int32_t delta_status;

enum {
    DELTA_OK = 0,
    DELTA_ERR_INVALID = -1,     /* bad argument, id, shape or unsupported layer */
    DELTA_ERR_INFEASIBLE = -2,  /* delta_plan: some step cannot fit into the budget */
    DELTA_ERR_OOM_ARENA = -3,   /* no arena block large enough */
    DELTA_ERR_OOM_PINNED = -4,  /* pinned host allocation failed */
    DELTA_ERR_STATE = -5,       /* tensor not in the state the call needs */
    DELTA_ERR_BUFFER = -6,      /* delta_plan: out_events too small (count is still returned) */
    DELTA_ERR_HIP = -7          /* a HIP call failed */
};

/* Tensor flags: the pin flags of struct DELTATensor (Sec. 4.3). */
enum { DELTA_F_UNCOMPUTABLE = 1, DELTA_F_EVICT_PINNED = 2, DELTA_F_OFFLOAD_PINNED = 4 };
/* Filter heuristics: Eq. (1) base 1/(m*s), Eq. (2) LRU 1/s, Eq. (3) GREEDY 1/m. */
enum { DELTA_FILTER_BASE = 0, DELTA_FILTER_LRU = 1, DELTA_FILTER_GREEDY = 2 };
/* Plan events: the actions of Table 1, plus FREE (last use passed) and DROP_TEMP (a
 * tensor that was back on the GPU only as an operand of a recomputation leaves again). */
enum {
    DELTA_EV_EVICT = 1, DELTA_EV_OFFLOAD = 2, DELTA_EV_RECOMPUTE = 3,
    DELTA_EV_RELOAD_PREFETCH = 4, DELTA_EV_RELOAD_DEMAND = 5, DELTA_EV_FREE = 6,
    DELTA_EV_DROP_TEMP = 7
};
enum { DELTA_DTYPE_F32 = 0, DELTA_DTYPE_BF16 = 1 };
/* Operators a recompute segment can contain (the regenerated operators Sec. 5.5 names are
 * ConvForward, BNForward and PoolingForward; the classifier and the loss close the net). */
enum {
    DELTA_OP_CONV = 0,       /* fused conv + BN affine (+ residual) (+ ReLU); also the classifier */
    DELTA_OP_MAXPOOL = 1,    /* R x S window, stride, pad; padding never wins the maximum */
    DELTA_OP_AVGPOOL = 2,    /* global average over H x W */
    DELTA_OP_SOFTMAX_CE = 3, /* mean cross-entropy of logits x [N, Cin] against labels `res` */
    DELTA_OP_ATTENTION = 4,  /* fused multi-head self-attention of a transformer layer (bf16, heads of 64) */
    DELTA_OP_LAYERNORM = 5,  /* layer normalisation over the channel axis (bf16) */
    DELTA_OP_BATCHNORM = 6,  /* batch normalisation with the statistics of the batch (bf16) */
    DELTA_OP_RELU = 7,       /* y = max(x, 0) (bf16) */
    DELTA_OP_ADD = 8         /* y = x + res (bf16) */
};
enum { DELTA_SYNC_D2H = 1, DELTA_SYNC_H2D = 2, DELTA_SYNC_COMPUTE = 4, DELTA_SYNC_ALL = 7 };
enum { DELTA_DIR_D2H = 0, DELTA_DIR_H2D = 1, DELTA_DIR_BOTH = 2 };
#define DELTA_NO_TENSOR 0xFFFFFFFFu

/* One tensor of the planner graph (the cost fields of struct DELTATensor, Sec. 4.3).
 * Tensors are numbered in production order; parents[i] < own id. */
typedef struct {
    uint64_t bytes;        /* m(t) */
    uint64_t cost_ns;      /* time to compute t from resident parents */
    uint64_t flops;        /* informational */
    uint32_t flags;        /* DELTA_F_* */
    uint32_t n_parents;
    const uint32_t *parents;   /* host, ascending ids */
} delta_tensor_desc;

/* One operator of the per-iteration sequence (Assumption 1).  Steps [0, n_fwd_steps) are
 * the forward pass and produce one tensor each; later steps only read. */
typedef struct {
    int32_t produces;      /* tensor id, or -1 */
    uint32_t n_reads;
    const uint32_t *reads; /* host, ascending ids */
    uint64_t cost_ns;
} delta_step_desc;

typedef struct {
    uint64_t budget_bytes;                 /* B */
    uint32_t trigger_num, trigger_den;     /* early start, 3/4 in the paper (Sec. 4.3) */
    uint32_t filter;                       /* DELTA_FILTER_* */
    uint32_t prefetch_distance;            /* d: look-ahead of Algorithm 4, in steps */
    uint32_t max_reloads;                  /* n of Algorithm 4, per step */
    uint32_t n_fwd_steps;
    uint64_t bw_d2h_Bps, bw_h2d_Bps;       /* b of Eq. (6), per direction; 0 = no link */
    uint32_t release_when_short;           /* 0: Evict/Offload only in the forward pass's release loop
                                              (Assumption 2).  1: Algorithm 1 to the letter: the loop
                                              also runs whenever an allocation does not fit ("memory is
                                              not enough"), in either pass, over the tensors that the
                                              running operator and the recomputations in progress do
                                              not use */
    uint32_t repair_rounds;                /* > 0: when an operand of a step cannot be brought back
                                              because rebuilding it with its missing ancestors does not
                                              fit, plan the iteration again with that operand treated as
                                              uncomputable (offload-only, Sec. 4.3: it then returns by
                                              reload), at most this many times.  The operator sequence
                                              repeats every iteration (Assumption 1), so a failed
                                              iteration can teach the next.  0: fail at once */
    uint32_t prefetch_rebuild_reads;       /* 0: Algorithm 4's queue is ordered by, and its look-ahead held
                                              against, the next step that reads the offloaded tensor.
                                              1: an access by a recomputation counts as well (Algorithm 1
                                              accesses the parents of what it recomputes): the tensor is
                                              wanted as soon as a step reads a tensor that is neither on the
                                              GPU nor in host memory and whose recomputation reaches it
                                              through such tensors; reloaded for that reason it is a leftover
                                              of a recomputation (first to give way when memory is short) */
} delta_plan_params;

typedef struct { uint32_t step, action, tensor, pad; } delta_event;

/* Activation of a DELTA_OP_CONV layer (field `relu`). */
enum { DELTA_ACT_NONE = 0, DELTA_ACT_RELU = 1, DELTA_ACT_GELU = 2 /* x/2 (1 + erf(x / sqrt 2)) */ };

/* Field `fuse` of a DELTA_OP_CONV layer: the block kernel.  A layer with DELTA_FUSE_BLOCK is the first
 * of an identity bottleneck whose three layers stand next to each other in the segment and run in ONE
 * launch: [1x1, 256 -> 64, ReLU] [3x3, 64 -> 64, stride 1, pad 1, ReLU, x = the first layer's y]
 * [1x1, 64 -> 256, ReLU, x = the second layer's y, res = the first layer's x], bf16.
 * Or it is the first of a stage's first bottleneck (config 2's block 1), whose FOUR layers stand next
 * to each other: [1x1, 64 -> 64, ReLU] [3x3, 64 -> 64, stride 1, pad 1, ReLU, x = the first layer's y]
 * [the projection shortcut: 1x1, 64 -> 256, no activation, x = the first layer's x]
 * [1x1, 64 -> 256, ReLU, x = the second layer's y, res = the projection's y].
 * Only the first layer's x has to be resident: every output is regenerated from it, and an
 * output whose layer carries DELTA_FUSE_NO_STORE is neither allocated nor written (at least one
 * must be stored).  The arithmetic does not depend on which outputs are stored, and every
 * reduction runs in the order of the per-layer kernels: a tensor carries the same bits whether the
 * block kernel or the per-layer launches produced it, so a plan may regenerate it with either. */
enum { DELTA_FUSE_NONE = 0, DELTA_FUSE_BLOCK = 1, DELTA_FUSE_NO_STORE = 2 };

/* One layer.  DELTA_OP_CONV: y = act(scale_k * conv(x, w) + shift_k (+ res)), activations
 * NHWC, weights KRSC (w[k][r][s][c]), scale/shift fp32 per output channel (folded batch-norm
 * with frozen statistics; scale = 1, shift = bias for the classifier).  The pooling
 * operators use x, y, N, H, W, Cin (= Cout), R, S, stride, pad and ignore w/scale/shift/res.
 * DELTA_OP_SOFTMAX_CE reads logits x [N, Cin] (storage dtype) and int64 labels in tensor
 * `res` [N], and writes one fp32 (the mean loss) to y.  x, res, y are tensor ids of the
 * bound table.
 * Transformer encoder layers (the paper's BERT-base workload, Sec. 5.2; the layer itself is the
 * published post-LN encoder): a linear layer y = act(x w^T + bias + res) is DELTA_OP_CONV with
 * H = sequence length, W = R = S = stride = 1, pad = 0, w [Cout][Cin], scale = ones, shift = bias.
 * DELTA_OP_ATTENTION: x = qkv [N, H, Cin] with Cin = 3 * Cout (q | k | v, head h in columns
 * [64 h, 64 h + 64) of each), y = ctx [N, H, Cout] = concat_h softmax(q_h k_h^T / 8) v_h over all H
 * positions, no mask; R = number of heads, Cout = 64 * R; the scores never reach memory (fp32 on
 * chip, probabilities rounded to bf16 before they multiply v).  W = S = stride = 1, pad = 0.
 * DELTA_OP_LAYERNORM: y = (x - mean) / sqrt(var + eps) * scale + shift over the Cin (= Cout,
 * multiple of 8, <= 2048) channels of each of the N*H*W rows; scale = gamma, shift = beta.
 * Both are bf16 only and ignore w and res.
 * Operator granularity (the separate ConvForward / BNForward tensors of the paper's cost table,
 * Sec. 5.5; bf16 only, any N, H, W, Cin = Cout a multiple of 8): a bare convolution is
 * DELTA_OP_CONV with scale = ones, shift = zeros, relu = 0, no res.  DELTA_OP_BATCHNORM:
 * y = scale_c (x - mu_c) / sqrt(var_c + eps) + shift_c with mu_c, var_c (biased) the mean and
 * variance of channel c over the N*H*W positions of THIS batch; scale = gamma, shift = beta;
 * Cin <= 8192; running statistics are not kept.  DELTA_OP_RELU: y = max(x, 0).  DELTA_OP_ADD:
 * y = x + res (res required).  All are deterministic: recomputation gives the same bits. */
typedef struct {
    uint32_t x, res, y;        /* res = DELTA_NO_TENSOR when there is no residual */
    uint32_t dtype;            /* DELTA_DTYPE_*: storage type of x, res, y and w */
    const void *w;             /* device, 16-byte aligned */
    const float *scale;        /* device */
    const float *shift;        /* device */
    int32_t N, H, W, Cin, Cout, R, S, stride, pad;
    uint32_t relu;             /* DELTA_ACT_* (convolution / linear layers) */
    uint32_t op;               /* DELTA_OP_* */
    float eps;                 /* DELTA_OP_LAYERNORM and DELTA_OP_BATCHNORM */
    uint32_t fuse;             /* DELTA_FUSE_* bits (convolutions only; 0 everywhere else) */
} delta_layer_desc;

typedef struct {
    uint64_t arena_bytes, arena_in_use, arena_high_water;
    uint64_t d2h_bytes, h2d_bytes;         /* copied since the last delta_stats_reset */
    uint64_t d2h_copies, h2d_copies;
    double d2h_ms, h2d_ms;                 /* sum of copy durations (device timestamps) */
    uint64_t recompute_launches, recompute_flops;
    uint64_t releases_evict, releases_offload, releases_free;
    uint64_t pinned_bytes;
    uint64_t arena_extent_high_water;      /* highest arena offset handed to a tensor placed from the bottom (fragmentation) */
    uint64_t arena_top_extent_high_water;  /* deepest reach, measured from the arena's end, of the tensors placed from
                                              the top (the backward pass's gradient tensors) */
} delta_stats_t;

/* Creates a context on the current HIP device.  arena_dev: device, 256-byte aligned,
 * arena_bytes long, or NULL for a planner-only context (then every call but delta_plan,
 * delta_last_error and delta_destroy fails with DELTA_ERR_STATE).  compute_stream: a
 * hipStream_t (NULL = the default stream). */
delta_status delta_create(void *arena_dev, uint64_t arena_bytes, void *compute_stream,
                          delta_ctx **out);
/* Waits for all three streams, frees pinned buffers, events and streams.  NULL is a no-op. */
void delta_destroy(delta_ctx *ctx);
/* Message of the last failed call on ctx (ctx-owned, valid until the next call). */
const char *delta_last_error(delta_ctx *ctx);

/*
 * Filter + Director + Prefetcher over a static trace (Algorithms 1-4, Eq. 1-6,
 * Assumptions 1-2).  Pure CPU, integer arithmetic only, deterministic.
 * Writes at most `capacity` events in issue order and always sets *out_count to the
 * number the plan has (DELTA_ERR_BUFFER when capacity was too small) and *out_peak to the
 * peak of live bytes.  DELTA_ERR_INFEASIBLE: last_error names the failing step.
 */
delta_status delta_plan(delta_ctx *ctx, const delta_tensor_desc *tensors, uint32_t n_tensors,
                        const delta_step_desc *steps, uint32_t n_steps,
                        const delta_plan_params *params, delta_event *out_events,
                        uint32_t capacity, uint32_t *out_count, uint64_t *out_peak);

/* Declares the run-time tensor table: n tensors with the given byte sizes, none resident.
 * Drops every tensor and host copy of a previous table (after waiting for the streams). */
delta_status delta_bind(delta_ctx *ctx, const uint64_t *bytes, uint32_t n_tensors);
/* The pinned host pool (Offload's destination, Sec. 4.2) grows by whole slabs and keeps them until
 * delta_destroy; a tensor gets its host buffer from it at its first Offload.  This call makes sure that
 * `bytes` more fit without a further allocation, so that a replay whose offloaded tensors add up to at
 * most `bytes` never reaches hipHostMalloc.  delta_bind returns every buffer to the pool. */
delta_status delta_reserve_pinned(delta_ctx *ctx, uint64_t bytes);
/* Makes `tensor` resident in a fresh arena block without computing it (network input).
 * The block may be written on the compute stream right away. */
delta_status delta_alloc(delta_ctx *ctx, uint32_t tensor, void **dev_out);
/* Device address of a resident tensor, valid until it is released.  Makes the compute
 * stream wait for a pending reload of that tensor.  DELTA_ERR_STATE when not resident. */
delta_status delta_tensor_ptr(delta_ctx *ctx, uint32_t tensor, void **dev_out);

/*
 * Release (Table 1).  action DELTA_EV_EVICT: the block returns to the arena, a host copy
 * is forgotten.  DELTA_EV_OFFLOAD: delta_swap_out if no valid host copy exists, then the
 * block returns to the arena; whoever gets the block next waits for the copy on its own
 * stream, the host never blocks.  DELTA_EV_FREE / DELTA_EV_DROP_TEMP: the block returns, a
 * host copy stays valid.  DELTA_ERR_STATE when the tensor is not resident.
 */
delta_status delta_release(delta_ctx *ctx, uint32_t tensor, uint32_t action);
/* Offload without release: async copy to the tensor's pinned host buffer on the D2H
 * stream, ordered after everything enqueued so far on the compute stream (Sec. 4.2).
 * A tensor above 32 MiB goes out as four copies with an event after each. */
delta_status delta_swap_out(delta_ctx *ctx, uint32_t tensor);
/* Reload (Algorithm 4): fresh arena block, async copy from the host buffer on the H2D
 * stream; later uses of the tensor on the compute stream wait for the copy's event.
 * May be called while the tensor's Offload is still in flight: the copy back then follows
 * it (piece by piece for a tensor that went out in pieces), never overtakes it.
 * DELTA_ERR_STATE when the tensor is resident or has no valid host copy. */
delta_status delta_prefetch(delta_ctx *ctx, uint32_t tensor);
/*
 * Recompute (Table 1), also used for the first forward so that both produce the same
 * bits: runs the layers in order on the compute stream.  Every x / res must be resident;
 * y gets a fresh block when it is not resident and is overwritten when it is.
 * Supported convolutions: Cin a multiple of 64 (bf16) or 32 (fp32) and Cout a multiple of 8
 * (bf16) or 4 (fp32) with any R, S, stride, pad; plus the bf16 ResNet stem (7x7, stride 2,
 * pad 3, Cin 3, Cout 64).  Pooling: channels a multiple of 8 (bf16) or 4 (fp32).  Other
 * shapes return DELTA_ERR_INVALID before anything is launched.
 */
delta_status delta_recompute_segment(delta_ctx *ctx, const delta_layer_desc *layers,
                                     uint32_t n_layers);
/*
 * For callers that cannot allocate device memory: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  The DELTA_OP_BATCHNORM operator of delta_recompute_segment (which
 * allocates its partial-sum buffer on first use, and an arena block for the output) on buffers the
 * caller owns: y = gamma_c (x - mu_c) / sqrt(var_c + eps) + beta_c over x [rows, channels] bf16, with the
 * mean and biased variance of THIS batch; same kernels, same decomposition, so the same bits.
 * x, y, gamma, beta: device, 16-byte aligned, x != y; channels a multiple of 8 and at most 8192 (more:
 * DELTA_ERR_INVALID); any rows >= 1.  Runs on the compute stream; calls no hipMalloc / hipFree and no
 * other allocating routine.  Its scratch (partial sums and factors, at most 4 259 840 bytes) is a
 * file-scope device array inside the library: every GPU the library runs on holds one copy until the
 * process ends, and every call on a GPU shares that copy - calls that overlap on one GPU (two streams,
 * two contexts, two threads) race; calls enqueued on one stream do not.  Nothing in it needs clearing
 * between calls.
 */
delta_status delta_batchnorm_static(delta_ctx *ctx, const void *x, void *y, const float *gamma, const float *beta,
                                    uint64_t rows, uint32_t channels, float eps);
/* Blocks the host until the selected streams (DELTA_SYNC_* bit mask) are idle. */
delta_status delta_sync(delta_ctx *ctx, uint32_t which);

/* Folds frozen batch-norm statistics into scale = gamma / sqrt(var + eps) and
 * shift = beta - mean * scale (fp32, on the compute stream).  All pointers: device. */
delta_status delta_bn_fold(delta_ctx *ctx, const float *gamma, const float *beta,
                           const float *mean, const float *var, float eps, uint32_t C,
                           float *scale, float *shift);

delta_status delta_stats(delta_ctx *ctx, delta_stats_t *out);   /* waits for the copy streams */
delta_status delta_stats_reset(delta_ctx *ctx);
/* When skip != 0, swap-out and prefetch keep all their bookkeeping and stream ordering
 * but move no bytes: the replay then shows what the step costs without the link. */
delta_status delta_set_skip_copies(delta_ctx *ctx, int32_t skip);

/* ---- Backward of a fused convolution layer (frozen batch-norm statistics).
 * The backward half of the training iteration whose tensor accesses the planner follows
 * (DELTA Sec. 3, Assumptions 1-3: the backward pass reads the stored forward activations).
 * For y = relu?(scale_k * conv(x, w) + shift_k (+ res)) and gy = dL/dy:
 *     gpre = gy * [y > 0]  (gy itself without ReLU)      - also dL/dres
 *     gx   = conv^T(gpre * scale, w) (+ gx_add)           - dL/dx
 *     gw[k,r,s,c] = scale_k * sum_m gpre[m,k] * x[m+(r,s),c]   - dL/dw, fp32
 * Supported: DELTA_OP_CONV with 2*pad == R-1 == S-1; gx for bf16 and fp32; gw with R in {1,3}: bf16
 * with channel counts that are multiples of 64 (MFMA kernel), fp32 with any channel counts the
 * forward accepts (a plain fp32 kernel, one fixed summation order, no workspace bytes).  A layer with stride > 1 (no residual allowed)
 * and a window larger than 1x1 gets gpre at the INPUT's resolution: gpre[n, stride*p, stride*q, :] =
 * gy[n,p,q,:] * [y > 0], zero elsewhere, so that both gradients are stride-1 operations on it
 * (stride^2 times the arithmetic).  A 1x1 layer with stride > 1 only reads the input pixels
 * (stride*p, stride*q): gpre keeps the bytes of y, those pixels are gathered into the workspace for
 * the weight gradient, and the data gradient is computed at the output's resolution into the
 * workspace and then spread out (zeros between), gx_add added in a second bf16 rounding.
 * Other operators (bf16 only; gpre must be gy, gx_add unused):
 *   DELTA_OP_MAXPOOL   gx receives gy routed to the first maximal element of each window (scan order
 *                      r, then s); needs fwd.x resident.  With mask_gx, gx is also multiplied by [x > 0].
 *   DELTA_OP_AVGPOOL   gx = gy / (H W) at every pixel.
 *   the classifier     (DELTA_OP_CONV with H = W = R = S = 1 and Cout not a multiple of 64):
 *                      gx = gy . (scale * w); gw (optional, fp32) receives Cout*Cin weight gradients
 *                      followed by Cout bias gradients (sum of gy over the images).
 *   DELTA_OP_SOFTMAX_CE  gx (bytes of the logits) = (softmax(z) - onehot(label)) / N; gy and gpre
 *                      must be DELTA_NO_TENSOR; needs fwd.x (logits) and fwd.res (labels) resident.
 *   DELTA_OP_BATCHNORM (batch statistics, bf16) gx = a (gy - mean(gy) - (x - mu) S / ((var + eps) M)) per channel,
 *                      a = gamma / sqrt(var + eps), S = sum gy (x - mu), M = N*H*W, mu and var recomputed
 *                      from x; gw (optional, fp32) receives C values dgamma = S / sqrt(var + eps), then
 *                      C values dbeta = sum gy.  Needs fwd.x resident; fwd.scale = gamma; gpre = gy.
 *   DELTA_OP_RELU      (bf16) gx = gy * [y > 0] on the stored output; needs fwd.y resident; gpre = gy.
 *   the stem           (DELTA_OP_CONV, 7x7, stride 2, pad 3, 3 -> 64 channels, bf16): weight gradient only
 *                      (gw required, fp32 [64][7][7][3]; gx, gx_add must be unset); gpre (bytes of y) receives
 *                      gy * [y > 0] when fwd.relu, else gpre must be gy; needs fwd.x resident and a workspace.
 * Anything else: DELTA_ERR_INVALID. */
typedef struct delta_bwd_desc {
    delta_layer_desc fwd;      /* the forward layer; fwd.x must be resident when gw is asked for,
                                  fwd.y when fwd.relu != 0; fwd.res only says whether a residual exists */
    uint32_t gy;               /* tensor id of dL/dy, resident, bytes of y */
    uint32_t gpre;             /* tensor id that receives gpre: N*H*W*Cout elements (the bytes of y when
                                  stride == 1 or the layer is 1x1); allocated if not resident.  Must equal
                                  gy when there is nothing to write: no ReLU mask to apply (fwd.relu == 0
                                  or gy_masked) and stride == 1 or a 1x1 layer.  May equal gy with no mask
                                  to apply on a 3x3 stride-2 pad-1 layer whose gradients both run at the
                                  output's resolution (bf16; if gw is set, channel counts multiples of
                                  128): gy is then not spread out and gpre not written */
    uint32_t gx;               /* tensor id that receives dL/dx (bytes of x), or DELTA_NO_TENSOR */
    uint32_t gx_add;           /* resident tensor (bytes of x) added to dL/dx before it is stored: the
                                  contribution of another consumer of x; or DELTA_NO_TENSOR */
    uint32_t mask_gx;          /* convolutions and max pooling.  Non-zero: gx is stored as (dL/dx + gx_add) * [x > 0],
                                  i.e. this layer also applies the ReLU mask of the layer that produced x
                                  (x is that layer's y), in the epilogue of the data-gradient kernel;
                                  the caller sets it on the LAST consumer of x to run.  Needs fwd.x resident */
    uint32_t gy_masked;        /* convolutions only.  Non-zero: gy already carries this layer's ReLU mask
                                  (a consumer ran with mask_gx): fwd.y is not read; with stride 1 gpre must
                                  be gy, with stride > 1 gpre receives gy spread to the input's resolution */
    const void *wt;            /* device: weights prepared by delta_bwd_weights (needed when gx is set) */
    void *gw;                  /* device, fp32 [Cout][R][S][Cin]: receives dL/dw (overwritten), or NULL */
    void *workspace;           /* device scratch, 256-byte aligned: the weight gradient's partial sums (from
                                  its start) and, for a strided 1x1 layer, its staging tensor (at its
                                  end); needed when gw is set or (strided 1x1) gx is set.  A strided 1x1
                                  layer whose staging bytes overlap what weight gradients still in flight
                                  use makes the compute stream wait for them: one workspace of (largest
                                  partial sums + largest staging tensor) for all layers avoids that */
    uint64_t workspace_bytes;  /* at least what delta_backward_workspace reports */
} delta_bwd_desc;

/* wt[c][R-1-r][S-1-s][k] = w[k][r][s][c] * scale[k] in the layer's storage type (same byte count as
 * w): with these weights the data gradient is a forward convolution of gpre.  Device pointers;
 * runs on the compute stream. */
delta_status delta_bwd_weights(delta_ctx *ctx, const delta_layer_desc *layer, void *wt);
/* Bytes of workspace delta_backward_segment needs for this layer (0 for operators that need none). */
delta_status delta_backward_workspace(delta_ctx *ctx, const delta_layer_desc *layer, uint64_t *out_bytes);
/* Runs the descriptors in order on the compute stream.  Everything is validated before the first
 * launch.  Output tensors are allocated from the arena when not resident (DELTA_ERR_OOM_ARENA);
 * a non-resident input is DELTA_ERR_STATE.
 * Weight gradients of convolutions and of the classifier (gw) are the exception to "on the compute stream": nothing later
 * in the backward pass reads them, so they run on a stream of the library's own, beside the
 * data-gradient chain, each after the launches that produce its inputs.  The arena accounts for
 * these readers when a tensor is released or rewritten.  The gw buffers and the workspace are the
 * caller's: their contents are ordered for later work on the compute stream only after
 * delta_backward_join (or complete after delta_sync with DELTA_SYNC_COMPUTE), and descriptors of one
 * context must keep using the same workspace or join in between. */
delta_status delta_backward_segment(delta_ctx *ctx, const delta_bwd_desc *descs, uint32_t n);
/* Orders the compute stream after every weight gradient enqueued so far (no host wait): work given
 * to the compute stream afterwards may read the gw buffers and reuse the workspace. */
delta_status delta_backward_join(delta_ctx *ctx);

/* Name of the kernel variant that delta_recompute_segment would launch for this layer (the
 * operator DELTA re-runs, Sec. 3 / Table 1), written NUL-terminated into out[0..cap).  Validates
 * the descriptor exactly as delta_recompute_segment does; launches nothing.  Needs a context
 * with an arena and the tensors bound (delta_bind), since the descriptor names tensor ids. */
delta_status delta_layer_kernel(delta_ctx *ctx, const delta_layer_desc *layer, char *out, uint64_t cap);

/* Measurement probes (rooflines the hot path is reported against). */
/* Pinned host <-> device hipMemcpyAsync throughput for `bytes` per copy, `iters` copies,
 * direction DELTA_DIR_*; BOTH runs the two directions concurrently and reports their sum. */
delta_status delta_probe_hostlink(delta_ctx *ctx, uint64_t bytes, uint32_t iters, uint32_t dir,
                                  double *out_GBps);
/* Device copy kernel (read + write of `bytes` each) -> achieved HBM GB/s, counting both. */
delta_status delta_probe_hbm(delta_ctx *ctx, uint64_t bytes, uint32_t iters, double *out_GBps);
/* Register-resident bf16 MFMA loop -> achieved TFLOP/s. */
delta_status delta_probe_mfma(delta_ctx *ctx, uint32_t iters, double *out_TFLOPs);

#ifdef __cplusplus
}
#endif
#endif /* DELTA_H */
