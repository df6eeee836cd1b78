// Block kernel: one bottleneck of ResNet's conv2_x stage in a single launch (bf16, fp32 accumulate).
// The identity blocks:
//                a1 = relu(bn1(w1 . x))             1x1, 256 -> 64
//                a2 = relu(bn2(conv3x3(a1, w2)))    3x3, 64 -> 64, stride 1, pad 1
//                out = relu(bn3(w3 . a2) + x)       1x1, 64 -> 256, identity shortcut
// This is the recompute segment DELTA's Recompute action re-runs for a released activation of such
// a block (Sec. 3, Table 1): any subset of {a1, a2, out} is regenerated from the block's input x
// alone, the tensors that are not asked for never reach memory.  Three per-layer launches move
// 2 x (256 + 64 | 64 + 64 | 64 + 256 + 256) bytes per pixel; this kernel reads x once (plus the
// shortcut's re-read, which the caches serve) and writes only what is stored.
//
// A workgroup of 8 wavefronts owns a 14 x 14 tile of output pixels of one image (two workgroups share
// a CU's LDS) and walks three phases:
//   1. a1 on the tile's 16 x 16 halo (256 positions, one 32-position block per wavefront): x straight
//      from global memory into registers (64 bytes per lane and 128-byte slice), w1 from LDS; the
//      results go to LDS as bf16 rows of 128 bytes (pitch 144) - exactly the layout the 3x3 reads its
//      operand in; positions outside the image hold zeros (the 3x3's padding);
//   2. a2: seven wavefronts take 32 of the 196 pixels x 64 channels each; the nine taps read nine
//      shifted rows of the a1 tile in LDS, w2 passes through LDS three taps at a time (the next
//      three are fetched into registers under the current three's MFMAs); the result stays in
//      registers as bf16, 8 consecutive channels per piece;
//   3. out: those registers, after one exchange between the lane halves, are the MFMA's pixel
//      operand (a piece of 8 channels per step; w3's rows are read from LDS in the same channel
//      order), the shortcut is read from x in the same piece layout, and rows of 128 contiguous
//      bytes leave through a wavefront-private LDS tile.
// Everything the kernel stores leaves with non-temporal stores: nothing in this launch reads it again, and
// the rows of x that phase 3 reads a second time then stay in the caches more often (batch 128: all three
// tensors 161-168 -> 149-151 us, out alone 156-160 -> 128-143 us; batch 32, where everything fits the
// Infinity Cache anyway, unchanged).
// Orientation as in the per-layer kernels: output channels on the MFMA row axis, pixels on the
// column axis; lane half h owns bytes [64h, 64h + 64) of every 128-byte slice of both operands.
// The order of every sum is fixed and does not depend on which tensors are stored, so whatever
// this kernel produced in the forward pass it reproduces bit for bit in a recomputation.
// The stage's first block (template argument PROJ; 64 input channels) has a projection in place of the identity
// shortcut: sc = bn_sc(wsc . x), 1x1, 64 -> 256, no ReLU - a fourth tensor the launch can store.  Phase 1 then
// reads one 128-byte slice per position; phase 3 multiplies each 64-channel group twice, wsc . x (the lane's half of
// its pixel's x row, read again from the caches: 64 bytes) rounded to bf16 as the stored sc is, then w3 . a2 with
// that added; w3 and wsc share the weight region of LDS, 128 rows each at a time (the second halves travel in
// registers while the first are multiplied).
// Every reduction also runs in the order of the per-layer kernels (slices of the input channels in order,
// the 3x3's taps in order, lane half h supplying bytes [64 h, 64 h + 64) of each 128-byte operand slice),
// so the three tensors carry the bits the three per-layer launches produce: a plan may regenerate a
// tensor with either.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kernels.hpp"

namespace delta {
namespace block {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

static constexpr int kWaves = 8, kThreads = kWaves * 64;
static constexpr int kCin = 256, kMid = 64, kCout = 256;
static constexpr int kT = 14;                            // output tile: 14 x 14 pixels, its a1 halo 16 x 16 positions
static constexpr int kPitch = 144;                       // 128-byte rows, 4 banks apart
static constexpr int kW1Pitch = kCin * 2 + 16;           // 528
static constexpr int kTap = kMid * kPitch;               // one 64 x 64 tap of w2 in LDS: 9216 bytes
static constexpr int kRA = 256 * kPitch;                 // the a1 halo tile; later one store tile per wavefront
static constexpr int kRB = kCout * kPitch;               // w1, then three taps of w2 at a time, then w3
static constexpr int kRD = (2 * kMid + 2 * kMid + 2 * kCout + 2 * kCout) * 4;   // scale/shift of the three layers and of a projection shortcut
static constexpr int kLds = kRA + kRB + kRD;
static constexpr int kCinProj = 64;                      // input channels of the block with a projection shortcut
static_assert(kW1Pitch * kMid <= kRB && 3 * kTap <= kRB && kWaves * 32 * kPitch <= kRA, "LDS regions");
static_assert(2 * kLds <= 160 * 1024, "two workgroups per CU");
static_assert(kWaves * 32 == 256 && (kT + 2) * (kT + 2) == 256 && kT * kT <= (kWaves - 1) * 32, "tile geometry");

__device__ __forceinline__ uint32_t pack2(float lo, float hi) {
    const f32x2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}
__device__ __forceinline__ float lo16(uint32_t p) { return __uint_as_float(p << 16); }
__device__ __forceinline__ float hi16(uint32_t p) { return __uint_as_float(p & 0xFFFF0000u); }
__device__ __forceinline__ float relu_keep_nan(float v) { return v < 0.f ? 0.f : v; }
__device__ __forceinline__ void wave_fence() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}
__device__ __forceinline__ f32x16 mma(const u32x4 w, const u32x4 x, const f32x16 acc) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, w), __builtin_bit_cast(bf16x8, x), acc, 0, 0, 0);
}

// One 32-channel accumulator tile of a 32-pixel column block -> scale/shift, (ReLU), bf16, as two pieces of
// 8 consecutive channels: piece [i2] of lane (pixel, half) holds channels 16 i2 + 8 half .. + 8 of the tile for
// its pixel.  `add` (optional, the same layout; may be `piece` itself) is added before the ReLU.
template <bool HAS_ADD, bool RELU = true>
__device__ __forceinline__ void finish_tile(const f32x16 &acc, const float *scale, const float *shift, int half,
                                            const u32x4 *add, u32x4 *piece) {
    float v[16];
#pragma unroll
    for (int rb = 0; rb < 4; ++rb) {
        const f32x4 sc = *reinterpret_cast<const f32x4 *>(scale + 8 * rb + 4 * half);
        const f32x4 sh = *reinterpret_cast<const f32x4 *>(shift + 8 * rb + 4 * half);
        v[4 * rb + 0] = acc[4 * rb + 0] * sc.x + sh.x;
        v[4 * rb + 1] = acc[4 * rb + 1] * sc.y + sh.y;
        v[4 * rb + 2] = acc[4 * rb + 2] * sc.z + sh.z;
        v[4 * rb + 3] = acc[4 * rb + 3] * sc.w + sh.w;
    }
#pragma unroll
    for (int i2 = 0; i2 < 2; ++i2) {
        float o[8];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v[8 * i2 + j]), __float_as_uint(v[8 * i2 + 4 + j]),
                                                      false, false);
            o[j] = __uint_as_float(r[0]);
            o[4 + j] = __uint_as_float(r[1]);
        }
        if constexpr (HAS_ADD) {
            const u32x4 r4 = add[i2];
            o[0] += lo16(r4.x); o[1] += hi16(r4.x); o[2] += lo16(r4.y); o[3] += hi16(r4.y);
            o[4] += lo16(r4.z); o[5] += hi16(r4.z); o[6] += lo16(r4.w); o[7] += hi16(r4.w);
        }
        if constexpr (RELU) {
#pragma unroll
            for (int e = 0; e < 8; ++e) o[e] = relu_keep_nan(o[e]);
        }
        u32x4 out;
        out.x = pack2(o[0], o[1]); out.y = pack2(o[2], o[3]);
        out.z = pack2(o[4], o[5]); out.w = pack2(o[6], o[7]);
        piece[i2] = out;
    }
}

// Two such tiles (channels 32 u .. 32 u + 32 of a 64-channel group): piece [u][i2].
template <bool HAS_ADD, bool RELU = true>
__device__ __forceinline__ void finish_tiles(const f32x16 (&acc)[2], const float *scale, const float *shift, int half,
                                             const u32x4 (*add)[2], u32x4 (&piece)[2][2]) {
#pragma unroll
    for (int u = 0; u < 2; ++u)
        finish_tile<HAS_ADD, RELU>(acc[u], scale + u * 32, shift + u * 32, half, HAS_ADD ? add[u] : nullptr, piece[u]);
}

// One workgroup: the 14 x 14 output pixels (ty, tx) of image n.
// PROJ: the stage's first block - 64 input channels, and instead of the identity shortcut the projection
// sc = bn_sc(wsc . x) (1x1, 64 -> 256, no ReLU), which is the fourth tensor the block can store.
template <bool PROJ>
__global__ __launch_bounds__(kThreads, 4) void bottleneck_block_kernel(BlockArgs a, int tiles_y, int tiles_x) {
    constexpr int CIN = PROJ ? kCinProj : kCin, NS = CIN / 64;          // input channels, 128-byte slices of an x row
    constexpr int W1P = CIN * 2 + 16;                                   // LDS pitch of a w1 row
    extern __shared__ __align__(16) unsigned char lds[];
    unsigned char *ra = lds;                             // a1 halo tile, later the store tiles
    unsigned char *rb = lds + kRA;                       // w1, then three taps of w2 at a time, then w3
    float *f1s = reinterpret_cast<float *>(rb + kRB), *f1h = f1s + kMid, *f2s = f1h + kMid, *f2h = f2s + kMid,
          *f3s = f2h + kMid, *f3h = f3s + kCout, *fcs = f3h + kCout, *fch = fcs + kCout;

    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int l32 = lane & 31, half = lane >> 5;
    unsigned logical;                                    // neighbouring tiles (shared halo) on one XCD
    {
        const unsigned nb = gridDim.x, per = nb >> 3, rem = nb & 7u;
        const unsigned xcd = blockIdx.x & 7u, idx = blockIdx.x >> 3;
        logical = xcd < rem ? xcd * (per + 1) + idx : rem * (per + 1) + (xcd - rem) * per + idx;
    }
    const int H = a.H, W = a.W;
    const int per_image = tiles_y * tiles_x;
    const int n = (int)(logical / (unsigned)per_image), t2 = (int)(logical - (unsigned)n * per_image);
    const int y0 = (t2 / tiles_x) * kT, x0 = (t2 % tiles_x) * kT;
    const bool need3 = a.out != nullptr || (PROJ && a.sc != nullptr);
    const bool need2 = a.a2 != nullptr || need3;
    const unsigned char *xg = static_cast<const unsigned char *>(a.x);
    const size_t image = (size_t)n * H * W;

    // ---- phase 1 operand: halo position hp = 32 wv + l32 is pixel (y0 - 1 + hp / 16, x0 - 1 + hp % 16);
    // its x row goes into flight before anything is staged.  Positions outside the image hold zeros
    // (the 3x3's padding), whatever w1 . x would give there.
    const int hp = wv * 32 + l32, hy = hp >> 4, hx = hp & 15;
    const int py = y0 - 1 + hy, px = x0 - 1 + hx;
    const bool inside = (unsigned)py < (unsigned)H && (unsigned)px < (unsigned)W;
    // without the 3x3 only the tile's own pixels count
    const bool own = inside && hy >= 1 && hy <= kT && hx >= 1 && hx <= kT;
    const bool p1 = __builtin_amdgcn_ballot_w64(need2 ? inside : own) != 0;      // this wavefront has a position to compute
    u32x4 xf[NS][4];
    if (p1) {
        const size_t q = image + (size_t)(inside ? py : 0) * W + (inside ? px : 0);      // clamped rows are overwritten by zeros
        const unsigned char *xp = xg + q * (CIN * 2) + half * 64;
#pragma unroll
        for (int s = 0; s < NS; ++s)
#pragma unroll
            for (int j = 0; j < 4; ++j) xf[s][j] = *reinterpret_cast<const u32x4 *>(xp + s * 128 + j * 16);
    }

    // ---- stage w1 and the batch-norm factors
    {
        const unsigned char *w1g = static_cast<const unsigned char *>(a.w1);
        for (int c = tid; c < kMid * (CIN / 8); c += kThreads) {          // CIN / 8 pieces of 16 bytes per row
            const int row = c / (CIN / 8), seg = c % (CIN / 8);
            *reinterpret_cast<u32x4 *>(rb + row * W1P + seg * 16) = *reinterpret_cast<const u32x4 *>(w1g + (size_t)c * 16);
        }
        if (tid < kMid) {
            f1s[tid] = a.s1[tid]; f1h[tid] = a.h1[tid];
            f2s[tid] = a.s2[tid]; f2h[tid] = a.h2[tid];
        }
        if (tid < kCout) {
            f3s[tid] = a.s3[tid]; f3h[tid] = a.h3[tid];
            if constexpr (PROJ) { fcs[tid] = a.ssc[tid]; fch[tid] = a.hsc[tid]; }
        }
    }
    __syncthreads();

    // The weights of the later phases are requested as early as registers allow, so that their latency is
    // paid under the phases before them: taps 0-2 now, taps 3-8 and w3 as soon as phase 1 has freed x.
    const unsigned char *w2g = static_cast<const unsigned char *>(a.w2);
    auto fetch_taps = [&](int first, u32x4 (&dst)[3]) {   // 3 taps x 64 rows x 8 pieces = 1536 pieces, three per thread
#pragma unroll
        for (int j = 0; j < 3; ++j) {
            const int c = tid + j * kThreads;
            const int tap = first + c / (kMid * 8), rest = c % (kMid * 8), k = rest >> 3, seg = rest & 7;
            dst[j] = *reinterpret_cast<const u32x4 *>(w2g + ((size_t)(k * 9 + tap) * 8 + seg) * 16);
        }
    };
    auto deposit_taps = [&](const u32x4 (&src)[3]) {
#pragma unroll
        for (int j = 0; j < 3; ++j) {
            const int c = tid + j * kThreads;
            const int t = c / (kMid * 8), rest = c % (kMid * 8), k = rest >> 3, seg = rest & 7;
            *reinterpret_cast<u32x4 *>(rb + t * kTap + k * kPitch + seg * 16) = src[j];
        }
    };
    u32x4 wq0[3], wq1[3], wq2[3], w3q[PROJ ? 2 : 4], wcq[PROJ ? 2 : 1];   // with a projection: half of w3 / wsc at a time
    if (need2) fetch_taps(0, wq0);

    // ---- phase 1: a1 = relu(bn1(w1 . x)) for one 32-position tile per wavefront, into LDS
    {
        u32x4 piece[2][2] = {};
        if (p1) {
            f32x16 acc[2];
#pragma unroll
            for (int u = 0; u < 2; ++u)
#pragma unroll
                for (int e = 0; e < 16; ++e) acc[u][e] = 0.f;
            const unsigned char *wrow = rb + l32 * W1P + half * 64;
#pragma unroll
            for (int s = 0; s < NS; ++s)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const u32x4 w0 = *reinterpret_cast<const u32x4 *>(wrow + s * 128 + j * 16);
                    const u32x4 w1 = *reinterpret_cast<const u32x4 *>(wrow + 32 * W1P + s * 128 + j * 16);
                    acc[0] = mma(w0, xf[s][j], acc[0]);
                    acc[1] = mma(w1, xf[s][j], acc[1]);
                }
            finish_tiles<false>(acc, f1s, f1h, half, nullptr, piece);
        }
        if (need2) {
            fetch_taps(3, wq1);
            fetch_taps(6, wq2);
            if (a.out) {
                const unsigned char *w3g = static_cast<const unsigned char *>(a.w3);
#pragma unroll
                for (int j = 0; j < (PROJ ? 2 : 4); ++j) // 256 rows x 8 pieces = 2048 pieces: four per thread
                    w3q[j] = *reinterpret_cast<const u32x4 *>(w3g + (size_t)(tid + j * kThreads) * 16);
            }
        }
        unsigned char *row = ra + hp * kPitch;
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
            for (int i2 = 0; i2 < 2; ++i2)
                *reinterpret_cast<u32x4 *>(row + (u * 32 + 16 * i2 + 8 * half) * 2) =
                    (p1 && inside) ? piece[u][i2] : u32x4{0u, 0u, 0u, 0u};
    }
    __syncthreads();                                     // the a1 tile is complete; w1 is dead

    // ---- a1 leaves as rows of 128 contiguous bytes (8 lanes per pixel), if it is stored
    if (a.a1) {
        unsigned char *a1g = static_cast<unsigned char *>(a.a1);
        for (int c = tid; c < kT * kT * 8; c += kThreads) {
            const int i = c >> 3, seg = c & 7, iy = i / kT, ix = i - iy * kT;
            if (y0 + iy < H && x0 + ix < W)
                __builtin_nontemporal_store(*reinterpret_cast<const u32x4 *>(ra + ((iy + 1) * 16 + ix + 1) * kPitch + seg * 16),
                                            reinterpret_cast<u32x4 *>(a1g + (image + (size_t)(y0 + iy) * W + x0 + ix) * (kMid * 2) + seg * 16));
        }
    }
    if (!need2) return;

    // ---- phase 2: a2 = relu(bn2(conv3x3(a1))), three taps of w2 at a time through LDS (all nine, and w3,
    // are already on their way in registers).
    // This lane's output pixel: pi = 32 wv + l32 < 196 is pixel (pi / 14, pi % 14) of the tile.
    const int pi = wv * 32 + l32;
    const bool p2 = wv * 32 < kT * kT;                   // wavefronts 0 .. 6
    const int iy = pi < kT * kT ? pi / kT : 0, ix = pi < kT * kT ? pi - (pi / kT) * kT : 0;   // lanes past the tile read row 0
    const bool mine = pi < kT * kT && y0 + iy < H && x0 + ix < W;
    f32x16 acc2[2];
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc2[u][e] = 0.f;
#pragma unroll
    for (int g = 0; g < 3; ++g) {
        deposit_taps(g == 0 ? wq0 : (g == 1 ? wq1 : wq2));   // the region is free: w1 / the previous taps are behind a barrier
        if constexpr (PROJ) {
            if (g == 2 && need3) {                           // the tap registers are free: the projection's weights take them
                const unsigned char *wcg = static_cast<const unsigned char *>(a.wsc);
#pragma unroll
                for (int j = 0; j < 2; ++j)                  // rows 0 .. 127 (1024 pieces: two per thread); the rest follows in phase 3
                    wcq[j] = *reinterpret_cast<const u32x4 *>(wcg + (size_t)(tid + j * kThreads) * 16);
            }
        }
        __syncthreads();
        if (p2) {
            // 12 steps (tap t, 16-byte piece q), tap 3 g + t being window position (g, t); the three operand
            // pieces of the next step are read while this step's two MFMAs issue
            u32x4 xv[2], w0[2], w1[2];
            auto read_step = [&](int st, int f) {
                const int t = st >> 2, q = st & 3;
                const unsigned char *xp = ra + ((iy + g) * 16 + ix + t) * kPitch + half * 64;
                const unsigned char *wp = rb + t * kTap + l32 * kPitch + half * 64;
                xv[f] = *reinterpret_cast<const u32x4 *>(xp + q * 16);
                w0[f] = *reinterpret_cast<const u32x4 *>(wp + q * 16);
                w1[f] = *reinterpret_cast<const u32x4 *>(wp + 32 * kPitch + q * 16);
            };
            read_step(0, 0);
#pragma unroll
            for (int st = 0; st < 12; ++st) {
                if (st + 1 < 12) read_step(st + 1, (st + 1) & 1);
                acc2[0] = mma(w0[st & 1], xv[st & 1], acc2[0]);
                acc2[1] = mma(w1[st & 1], xv[st & 1], acc2[1]);
                if (st + 1 < 12) {
                    __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                    __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                }
            }
        }
        __syncthreads();                                 // everyone is done with these taps (and, after the last, with a1)
    }
    u32x4 a2p[2][2];                                     // this lane's pixel of a2: four pieces of 8 channels
    if (p2) finish_tiles<false>(acc2, f2s, f2h, half, nullptr, a2p);
    if constexpr (PROJ) {
        // ---- phase 3 with a projection shortcut: sc = bn_sc(wsc . x) and out = relu(bn3(w3 . a2) + sc), 64 output
        // channels at a time.  w3 and wsc (256 rows of 128 bytes each) pass through the weight region in two
        // halves of 128 rows; every wavefront takes part in the barriers between them.
        const size_t rm = image + (size_t)(mine ? y0 + iy : 0) * W + (mine ? x0 + ix : 0);   // clamp: the loads stay in bounds
        u32x4 xs[4];                                         // this lane's half of its pixel's x row: the projection's operand
        if (need3 && p2) {
#pragma unroll
            for (int j = 0; j < 4; ++j)
                xs[j] = *reinterpret_cast<const u32x4 *>(xg + rm * (kCinProj * 2) + half * 64 + j * 16);
        }
        unsigned char *ttile = ra + wv * (32 * kPitch);      // wavefront-private: pieces in, rows out
        const int trow = lane >> 3, tseg = lane & 7;
        int srow[4];                                         // pixel index (below 2^30) or -1
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const int sp = wv * 32 + trow + 8 * t, sy = sp / kT, sx = sp - sy * kT;
            srow[t] = sp < kT * kT && y0 + sy < H && x0 + sx < W ? (int)(image + (size_t)(y0 + sy) * W + x0 + sx) : -1;
        }
        auto put_rows = [&](const u32x4 (&piece)[2][2], unsigned char *dst, int row_bytes, int col_bytes) {
#pragma unroll
            for (int u = 0; u < 2; ++u)
#pragma unroll
                for (int i2 = 0; i2 < 2; ++i2)
                    *reinterpret_cast<u32x4 *>(ttile + l32 * kPitch + (u * 32 + 16 * i2 + 8 * half) * 2) = piece[u][i2];
            wave_fence();
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const u32x4 o4 = *reinterpret_cast<const u32x4 *>(ttile + (trow + 8 * t) * kPitch + tseg * 16);
                if (srow[t] >= 0) __builtin_nontemporal_store(o4, reinterpret_cast<u32x4 *>(dst + (size_t)srow[t] * row_bytes + col_bytes + tseg * 16));
            }
            wave_fence();
        };
        if (p2 && a.a2) put_rows(a2p, static_cast<unsigned char *>(a.a2), kMid * 2, 0);
        if (!need3) return;
        if (p2 && a.out) {                                   // the two lanes of a pixel trade pieces (see the identity block below)
#pragma unroll
            for (int i2 = 0; i2 < 2; ++i2) {
                uint32_t *pa = reinterpret_cast<uint32_t *>(&a2p[0][i2]), *pb = reinterpret_cast<uint32_t *>(&a2p[1][i2]);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    auto r = __builtin_amdgcn_permlane32_swap(pa[e], pb[e], false, false);
                    pa[e] = r[0];
                    pb[e] = r[1];
                }
            }
        }
        constexpr int kHalfRows = 128, kHalfBytes = kHalfRows * kPitch;
        unsigned char *og = static_cast<unsigned char *>(a.out), *cg = static_cast<unsigned char *>(a.sc);
#pragma unroll
        for (int round = 0; round < 2; ++round) {
            if (round) __syncthreads();                      // everyone has read the first halves
#pragma unroll
            for (int jj = 0; jj < 2; ++jj) {                 // piece jj of a thread is row 64 jj + tid / 8 of this half
                const int c = tid + jj * kThreads, row = c >> 3, seg = c & 7;
                if (a.out) *reinterpret_cast<u32x4 *>(rb + row * kPitch + seg * 16) = w3q[jj];
                *reinterpret_cast<u32x4 *>(rb + kHalfBytes + row * kPitch + seg * 16) = wcq[jj];
            }
            if (round == 0) {                                // the second halves travel while the first are multiplied
                const unsigned char *w3g = static_cast<const unsigned char *>(a.w3), *wcg = static_cast<const unsigned char *>(a.wsc);
#pragma unroll
                for (int jj = 0; jj < 2; ++jj) {
                    const size_t c = (size_t)(tid + (2 + jj) * kThreads) * 16;
                    if (a.out) w3q[jj] = *reinterpret_cast<const u32x4 *>(w3g + c);
                    wcq[jj] = *reinterpret_cast<const u32x4 *>(wcg + c);
                }
            }
            __syncthreads();
            if (p2) {
#pragma unroll
                for (int gg = 0; gg < 2; ++gg) {
                    const int g = 2 * round + gg;
                    const unsigned char *wrow = rb + (gg * 64 + l32) * kPitch + half * 64;
                    // one 32-channel tile at a time: a single accumulator tile is live beside x, a2 and the pieces
                    u32x4 scp[2][2];
#pragma unroll
                    for (int u = 0; u < 2; ++u) {            // the projection: one 128-byte slice of x, pieces in order
                        f32x16 acc;
#pragma unroll
                        for (int e = 0; e < 16; ++e) acc[e] = 0.f;
#pragma unroll
                        for (int j = 0; j < 4; ++j)
                            acc = mma(*reinterpret_cast<const u32x4 *>(wrow + kHalfBytes + u * 32 * kPitch + j * 16), xs[j], acc);
                        finish_tile<false, false>(acc, fcs + g * 64 + u * 32, fch + g * 64 + u * 32, half, nullptr, scp[u]);
                    }
                    if (a.sc) put_rows(scp, cg, kCout * 2, g * 128);
                    if (a.out) {
#pragma unroll
                        for (int u = 0; u < 2; ++u) {
                            f32x16 acc;
#pragma unroll
                            for (int e = 0; e < 16; ++e) acc[e] = 0.f;
#pragma unroll
                            for (int j = 0; j < 4; ++j)
                                acc = mma(*reinterpret_cast<const u32x4 *>(wrow + u * 32 * kPitch + j * 16), a2p[j & 1][j >> 1], acc);
                            // in place: each piece is read, then written
                            finish_tile<true>(acc, f3s + g * 64 + u * 32, f3h + g * 64 + u * 32, half, scp[u], scp[u]);
                        }
                        put_rows(scp, og, kCout * 2, g * 128);
                    }
                }
            }
        }
        return;
    } else {
    // the shortcut rows of the first two channel groups go into flight before the barrier that publishes w3
    const size_t rm = image + (size_t)(mine ? y0 + iy : 0) * W + (mine ? x0 + ix : 0);   // clamp: the loads stay in bounds
    const unsigned char *xres = xg + rm * (kCin * 2);
    u32x4 rv[2][2][2];
    auto load_res = [&](int g, u32x4 (&dst)[2][2]) {
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
            for (int i2 = 0; i2 < 2; ++i2)
                dst[u][i2] = *reinterpret_cast<const u32x4 *>(xres + (size_t)(g * 64 + u * 32 + 16 * i2 + 8 * half) * 2);
    };
    if (need3) {
        if (p2) { load_res(0, rv[0]); load_res(1, rv[1]); }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int c = tid + j * kThreads, row = c >> 3, seg = c & 7;
            *reinterpret_cast<u32x4 *>(rb + row * kPitch + seg * 16) = w3q[j];
        }
    }
    __syncthreads();                                     // w3 is in place
    if (!p2) return;

    unsigned char *ttile = ra + wv * (32 * kPitch);      // wavefront-private: pieces in, rows out
    const int trow = lane >> 3, tseg = lane & 7;
    // the pixels this lane stores rows of: pr = trow + 8 t of the wavefront's 32
    long long srow[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        const int sp = wv * 32 + trow + 8 * t, sy = sp / kT, sx = sp - sy * kT;
        srow[t] = sp < kT * kT && y0 + sy < H && x0 + sx < W ? (long long)(image + (size_t)(y0 + sy) * W + x0 + sx) : -1;
    }
    if (a.a2) {
        unsigned char *a2g = static_cast<unsigned char *>(a.a2);
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
            for (int i2 = 0; i2 < 2; ++i2)
                *reinterpret_cast<u32x4 *>(ttile + l32 * kPitch + (u * 32 + 16 * i2 + 8 * half) * 2) = a2p[u][i2];
        wave_fence();
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const u32x4 o4 = *reinterpret_cast<const u32x4 *>(ttile + (trow + 8 * t) * kPitch + tseg * 16);
            if (srow[t] >= 0) __builtin_nontemporal_store(o4, reinterpret_cast<u32x4 *>(a2g + (size_t)srow[t] * (kMid * 2) + tseg * 16));
        }
        wave_fence();
    }
    if (!need3) return;

    // ---- phase 3: out = relu(bn3(w3 . a2) + x), 64 output channels at a time.
    // The two lanes of a pixel first trade pieces so that lane half h holds channels 32 h .. 32 h + 32 in
    // order (bytes [64 h, 64 h + 64) of the a2 row, as a kernel that reads a2 from memory would): step j of
    // the reduction then multiplies channels 8 j .. + 8 and 32 + 8 j .. + 8, the same sixteen products per
    // MFMA, in the same order, as the per-layer 1x1 kernel - and so the same bits.
    //   before: half 0 holds [0,8) [16,24) [32,40) [48,56), half 1 holds [8,16) [24,32) [40,48) [56,64)
    //   after:  half 0 holds [0,8) [16,24) [8,16) [24,32),  half 1 holds [32,40) [48,56) [40,48) [56,64)
    {
        auto trade = [](u32x4 &lo_keeps, u32x4 &hi_keeps) {   // upper half of the first <-> lower half of the second
            uint32_t *pa = reinterpret_cast<uint32_t *>(&lo_keeps), *pb = reinterpret_cast<uint32_t *>(&hi_keeps);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                auto r = __builtin_amdgcn_permlane32_swap(pa[e], pb[e], false, false);
                pa[e] = r[0];
                pb[e] = r[1];
            }
        };
        trade(a2p[0][0], a2p[1][0]);
        trade(a2p[0][1], a2p[1][1]);
    }
    unsigned char *og = static_cast<unsigned char *>(a.out);
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        f32x16 acc[2];
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[u][e] = 0.f;
        const unsigned char *wrow = rb + (g * 64 + l32) * kPitch + half * 64;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            // step j: channels 32 half + 8 j .. + 8 - after the trade that is piece [j & 1][j >> 1]
            const u32x4 w0 = *reinterpret_cast<const u32x4 *>(wrow + j * 16);
            const u32x4 w1 = *reinterpret_cast<const u32x4 *>(wrow + 32 * kPitch + j * 16);
            acc[0] = mma(w0, a2p[j & 1][j >> 1], acc[0]);
            acc[1] = mma(w1, a2p[j & 1][j >> 1], acc[1]);
        }
        u32x4 piece[2][2];
        finish_tiles<true>(acc, f3s + g * 64, f3h + g * 64, half, rv[g & 1], piece);
        if (g + 2 < 4) load_res(g + 2, rv[g & 1]);       // two groups ahead
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
            for (int i2 = 0; i2 < 2; ++i2)
                *reinterpret_cast<u32x4 *>(ttile + l32 * kPitch + (u * 32 + 16 * i2 + 8 * half) * 2) = piece[u][i2];
        wave_fence();
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const u32x4 o4 = *reinterpret_cast<const u32x4 *>(ttile + (trow + 8 * t) * kPitch + tseg * 16);
            if (srow[t] >= 0) __builtin_nontemporal_store(o4, reinterpret_cast<u32x4 *>(og + ((size_t)srow[t] * kCout + g * 64) * 2 + tseg * 16));
        }
        wave_fence();
    }
    }
}

}  // namespace block

const char *bottleneck_block_check(const BlockArgs &a) {
    if (a.N <= 0 || a.H <= 0 || a.W <= 0) return "non-positive dimension";
    const long long M = (long long)a.N * a.H * a.W;
    if (M != a.M || M > 0x7FFFFFFFLL / 2) return "pixel count out of range";
    if (!a.x || !a.w1 || !a.w2 || !a.w3 || !a.s1 || !a.h1 || !a.s2 || !a.h2 || !a.s3 || !a.h3) return "null operand";
    if (a.proj ? (!a.wsc || !a.ssc || !a.hsc) : (a.wsc || a.ssc || a.hsc || a.sc)) return "projection operands do not match the block's kind";
    if (!a.a1 && !a.a2 && !a.out && !a.sc) return "nothing to store";
    const uintptr_t all = (uintptr_t)a.x | (uintptr_t)a.a1 | (uintptr_t)a.a2 | (uintptr_t)a.out | (uintptr_t)a.w1 |
                          (uintptr_t)a.w2 | (uintptr_t)a.w3 | (uintptr_t)a.s1 | (uintptr_t)a.h1 | (uintptr_t)a.s2 |
                          (uintptr_t)a.h2 | (uintptr_t)a.s3 | (uintptr_t)a.h3 | (uintptr_t)a.wsc | (uintptr_t)a.ssc |
                          (uintptr_t)a.hsc | (uintptr_t)a.sc;
    if (all & 15) return "pointers must be 16-byte aligned";
    const long long tiles = (long long)a.N * ((a.H + block::kT - 1) / block::kT) * ((a.W + block::kT - 1) / block::kT);
    if (tiles > 0x7FFFFFF0LL) return "too many tiles";
    return nullptr;
}

hipError_t launch_bottleneck_block(const BlockArgs &a, hipStream_t stream) {
    if (bottleneck_block_check(a)) return hipErrorInvalidValue;
    const int tiles_y = (a.H + block::kT - 1) / block::kT, tiles_x = (a.W + block::kT - 1) / block::kT;
    static const hipError_t raised = hipFuncSetAttribute(reinterpret_cast<const void *>(block::bottleneck_block_kernel<false>),
                                                         hipFuncAttributeMaxDynamicSharedMemorySize, block::kLds);
    static const hipError_t raised_proj = hipFuncSetAttribute(reinterpret_cast<const void *>(block::bottleneck_block_kernel<true>),
                                                              hipFuncAttributeMaxDynamicSharedMemorySize, block::kLds);
    if (raised != hipSuccess) return raised;
    if (raised_proj != hipSuccess) return raised_proj;
    const long long blocks = (long long)a.N * tiles_y * tiles_x;
    if (a.proj)
        block::bottleneck_block_kernel<true><<<dim3((unsigned)blocks), dim3(block::kThreads), block::kLds, stream>>>(a, tiles_y, tiles_x);
    else
        block::bottleneck_block_kernel<false><<<dim3((unsigned)blocks), dim3(block::kThreads), block::kLds, stream>>>(a, tiles_y, tiles_x);
    return hipGetLastError();
}

}  // namespace delta
