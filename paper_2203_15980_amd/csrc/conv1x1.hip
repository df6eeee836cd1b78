// Streaming kernel for 1x1 convolutions with small weights (bf16, fp32 accumulate):
// y = relu?(scale_k * (x . w_k) + shift_k (+ res)).
//
// These are the HBM-bound layers of a bottleneck (28-51 flop per byte against a ridge of
// about 310 on MI355X): the job is to keep as many bytes in flight as possible, not to
// feed the matrix cores.  So, unlike the tiled kernel in conv_igemm.hip:
//   - the weight rows of a slice of NG * 64 output channels (plus their scale/shift) are staged
//     once per workgroup in LDS; a layer with more channels than one slice holds runs one
//     workgroup per (pixel group, slice), the slices of a pixel group on the same XCD so that
//     they share the activations in its L2;
//   - after that single barrier every wavefront works alone on its own 32 pixels: it
//     loads its activation operand straight from global memory into registers (each lane
//     64 contiguous bytes per 128-byte slice of Cin, issued before the staging so that the
//     latency overlaps it), so there is no barrier on the streaming side, and many
//     wavefronts per CU overlap freely;
//   - output channels are processed 64 at a time (two 32x32 accumulators, 32 registers),
//     which keeps the kernel under 128 VGPRs: 16 wavefronts per CU.
// Orientation as in conv_igemm.hip: channels on the MFMA row axis, pixels on the column
// axis, so a lane owns 4 consecutive channels of one pixel in each 8-row block.  One
// v_permlane32_swap per register pair then gives every lane 8 consecutive channels
// (16 bytes of bf16).  Those 16-byte pieces pass through a small wavefront-private LDS tile
// (32 pixels x 128 bytes) that turns them into rows, so that y is stored with 128 contiguous
// bytes per pixel (8 lanes x 16 bytes): with 32-byte store runs the same kernel reached
// 5.2 TB/s on the residual layer, with full lines 6.3 TB/s.
// The summation order is fixed (slices of Cin in order, MFMA internal order), so forward
// and recomputation give the same bits.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kernels.hpp"

namespace delta {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

namespace {

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
// two fp32 -> packed bf16, round to nearest even (v_cvt_pk_bf16_f32)
__device__ __forceinline__ uint32_t pack2(float lo, float hi) {
    const f32x2_t v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}
__device__ __forceinline__ float lo16(uint32_t p) { return __uint_as_float(p << 16); }
__device__ __forceinline__ float hi16(uint32_t p) { return __uint_as_float(p & 0xFFFF0000u); }
__device__ __forceinline__ float relu_keep_nan(float v) { return v < 0.f ? 0.f : v; }   // NaN stays NaN
// LDS instructions of one wavefront execute in order; this only keeps the compiler from moving
// accesses across the point where lanes exchange data through their private LDS tile.
__device__ __forceinline__ void wave_fence() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

}  // namespace

static constexpr int kTPitch = 144;

// NS = Cin / 64 (128-byte slices of the reduction axis), NG = channels of one slice / 64.
// Dynamic LDS: weights [NG*64][Cin*2 + 16 bytes], scale, shift (fp32) of the slice, then one
// transposition tile per wavefront.
// Persistent workgroups: the grid is `nworkers` workgroups per channel slice (about one per CU),
// each stages its weights once and its wavefronts then walk the 32-pixel tiles
// worker + nworkers * (wavefront + WAVES * k): consecutive tiles go to different CUs, so that
// whatever number of tiles there is, every CU gets its share to within one tile per wavefront
// (one workgroup per 512 pixels left 60 of 256 CUs idle at batch 32 and ran 3.06 rounds as 4 at
// batch 128).  While a tile's last channel group is finished the next tile's rows are already in flight.
// Grid: 8 * ceil(nworkers / 8) * slices workgroups.
template <int NS, int NG, int WAVES, bool HAS_RES, bool SLICED, bool HAS_MASK = false>
__global__ __launch_bounds__(WAVES * 64) void conv1x1_stream_kernel(ConvArgs a, int nworkers) {
    constexpr int THREADS = WAVES * 64;
    constexpr int Cout = NG * 64;               // channels of this workgroup's slice
    // The next tile's rows are requested while the current tile's last group is finished - where a
    // lane has the registers for them to wait in: not with a residual at 16 wavefronts (128
    // registers) or with residual and mask, and not with four operand slices.
    constexpr bool AHEAD = !(HAS_RES && (WAVES > 12 || HAS_MASK)) && NS <= 2;
    extern __shared__ __align__(16) unsigned char lds[];
    // workgroup -> (worker, channel slice): consecutive workgroups go to consecutive XCDs,
    // so the slices of worker g all land on XCD g % 8 and share the activations in its L2.
    // A layer that is one slice keeps the channel count a compile-time constant (cheaper
    // addressing, fewer registers).
    int worker, n0;
    if constexpr (SLICED) {
        const int nslices = a.Cout / Cout;
        const unsigned xcd = blockIdx.x & 7u, rest = blockIdx.x >> 3;
        worker = (int)(rest / (unsigned)nslices) * 8 + (int)xcd;
        if (worker >= nworkers) return;          // whole workgroup, before the barrier
        n0 = (int)(rest % (unsigned)nslices) * Cout;
    } else {
        worker = blockIdx.x;
        n0 = 0;
    }
    const int Ctot = SLICED ? a.Cout : Cout;
    constexpr int WPITCH = NS * 128 + 16;       // rows 4 banks apart: conflict-free b128 reads
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int l32 = lane & 31, half = lane >> 5;
    float *lscale = reinterpret_cast<float *>(lds + (size_t)Cout * WPITCH);
    float *lshift = lscale + Cout;
    // wavefront-private transposition tile: 32 pixel rows of 128 bytes, pitch 144
    unsigned char *ttile = reinterpret_cast<unsigned char *>(lshift + Cout) + wv * (32 * kTPitch);

    // tile numbers fit 32 bits with room to spare (M < 2^31, at most 2^26 tiles, step <= 4096)
    const int ntiles = (int)(((long long)a.M + 31) / 32);
    const int step = nworkers * WAVES;
    int tile = worker + nworkers * wv;
    const bool active = tile < ntiles;           // wavefronts without a tile only help staging

    // This lane's pixel of a tile (clamped: loads stay in bounds, such rows are never stored)
    auto pixel = [&](int t) -> long long {
        const long long m = (long long)t * 32 + l32;
        return m < a.M ? m : (long long)a.M - 1;
    };
    // operand straight into registers: lane (pixel l32, half) takes bytes [64*half, 64*half + 64)
    // of each 128-byte slice of its pixel (routing these loads through the LDS tile as rows
    // helped the smallest layer only and cost registers everywhere else)
    auto load_x = [&](int t, u32x4_t (&dst)[NS][4]) {
        const long long mm = pixel(t);
        size_t xpix;
        if (a.stride == 1) {
            xpix = (size_t)mm;
        } else {
            const int PQ = a.P * a.Q;
            const int n = (int)(mm / PQ), pq = (int)(mm - (long long)n * PQ);
            const int p = pq / a.Q, q = pq - p * a.Q;
            xpix = ((size_t)n * a.H + (size_t)p * a.stride) * a.W + (size_t)q * a.stride;
        }
        const unsigned char *xp = static_cast<const unsigned char *>(a.x) + xpix * (NS * 128) + half * 64;
#pragma unroll
        for (int s = 0; s < NS; ++s)
#pragma unroll
            for (int j = 0; j < 4; ++j) dst[s][j] = *reinterpret_cast<const u32x4_t *>(xp + s * 128 + j * 16);
    };
    // the slice offset is folded into the (uniform) base pointers
    unsigned char *yg = static_cast<unsigned char *>(a.y) + (size_t)n0 * 2;
    const unsigned char *rg = static_cast<const unsigned char *>(a.res) + (size_t)n0 * 2;
    const unsigned char *mg = static_cast<const unsigned char *>(a.mask) + (size_t)n0 * 2;   // HAS_MASK only
    // residual in the post-swap layout, straight into registers: piece (u, i2) of group g
    // covers channels g*64 + u*32 + 16*i2 + 8*half .. +8 of this lane's pixel (32-byte runs per
    // pixel; routing the reads through the LDS tile as well measured slower).  Two groups are
    // held: the one being finished and the next one (of this tile or the next), already in flight.
    u32x4_t rv[2][2][2];
    auto load_res = [&](int t, int g, u32x4_t (&dst)[2][2]) {
        const size_t orow = (size_t)pixel(t) * Ctot * 2;
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
            for (int i2 = 0; i2 < 2; ++i2)
                dst[u][i2] = *reinterpret_cast<const u32x4_t *>(
                    rg + orow + (size_t)(g * 64 + u * 32 + 16 * i2 + 8 * half) * 2);
    };
    // Everything the first tile reads from HBM goes into flight before the staging, so that the
    // latency overlaps it.
    u32x4_t xf[NS][4];
    load_x(tile, xf);
    if constexpr (HAS_RES) load_res(tile, 0, rv[0]);

    // ---- stage weights and batch-norm factors (once per workgroup)
    {
        constexpr int SEGS = NS * 8;             // 16-byte pieces per weight row
        const unsigned char *wg = static_cast<const unsigned char *>(a.w) + (size_t)n0 * SEGS * 16;
        constexpr int pieces = Cout * SEGS;
        for (int c = tid; c < pieces; c += THREADS) {
            const int row = c / SEGS, seg = c - row * SEGS;
            *reinterpret_cast<u32x4_t *>(lds + row * WPITCH + seg * 16) =
                *reinterpret_cast<const u32x4_t *>(wg + ((size_t)row * SEGS + seg) * 16);
        }
        for (int c = tid; c < Cout; c += THREADS) {
            lscale[c] = a.scale[n0 + c];
            lshift[c] = a.shift[n0 + c];
        }
    }
    __syncthreads();                             // the only barrier
    if (!active) return;
    const int relu = a.relu;

    for (;;) {
        const int next = tile + step;
        const bool more = next < ntiles;         // the same for the whole wavefront
        // with a mask operand the lane-derived offsets are recomputed per tile (a handful of integer
        // operations) instead of being carried across the loop: those variants have no register to spare
        int lz = lane;
        if constexpr (HAS_MASK) asm volatile("" : "+v"(lz));
        const int l32 = lz & 31, half = lz >> 5, trow = lz >> 3, tseg = lz & 7;
        const long long mbase = (long long)tile * 32;
#pragma unroll
        for (int g = 0; g < NG; ++g) {
            if constexpr (HAS_RES) {
                if (g + 1 < NG) load_res(tile, g + 1, rv[(g + 1) & 1]);
                else if (AHEAD && more) load_res(next, 0, rv[NG & 1]);
            }
            f32x16_t acc[2];
#pragma unroll
            for (int u = 0; u < 2; ++u)
#pragma unroll
                for (int e = 0; e < 16; ++e) acc[u][e] = 0.f;
            const unsigned char *wrow = lds + (size_t)(g * 64 + l32) * WPITCH + half * 64;
#pragma unroll
            for (int s = 0; s < NS; ++s)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const u32x4_t w0 = *reinterpret_cast<const u32x4_t *>(wrow + s * 128 + j * 16);
                    const u32x4_t w1 = *reinterpret_cast<const u32x4_t *>(wrow + 32 * WPITCH + s * 128 + j * 16);
                    acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, w0),
                                                                     __builtin_bit_cast(bf16x8_t, xf[s][j]), acc[0], 0, 0, 0);
                    acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, w1),
                                                                     __builtin_bit_cast(bf16x8_t, xf[s][j]), acc[1], 0, 0, 0);
                }
            // the operand registers are free after the last group's products: the next tile's rows
            // go into flight under this group's epilogue and stores
            if constexpr (AHEAD) {
                if (g == NG - 1 && more) load_x(next, xf);
            }
            // ---- epilogue of the two 32-channel tiles
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const int cb = g * 64 + u * 32;
                float v[16];
#pragma unroll
                for (int rb = 0; rb < 4; ++rb) {
                    const f32x4_t sc = *reinterpret_cast<const f32x4_t *>(lscale + cb + 8 * rb + 4 * half);
                    const f32x4_t sh = *reinterpret_cast<const f32x4_t *>(lshift + cb + 8 * rb + 4 * half);
                    v[4 * rb + 0] = acc[u][4 * rb + 0] * sc.x + sh.x;
                    v[4 * rb + 1] = acc[u][4 * rb + 1] * sc.y + sh.y;
                    v[4 * rb + 2] = acc[u][4 * rb + 2] * sc.z + sh.z;
                    v[4 * rb + 3] = acc[u][4 * rb + 3] * sc.w + sh.w;
                }
#pragma unroll
                for (int i2 = 0; i2 < 2; ++i2) {
                    // blocks 2*i2 and 2*i2+1: after the swap the lower half-wave holds channels
                    // cb + 16*i2 .. +8 and the upper half-wave the next eight, in order
                    float o[8];
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v[8 * i2 + j]),
                                                                  __float_as_uint(v[8 * i2 + 4 + j]), false, false);
                        o[j] = __uint_as_float(r[0]);
                        o[4 + j] = __uint_as_float(r[1]);
                    }
                    if constexpr (HAS_RES) {
                        const u32x4_t r4 = rv[g & 1][u][i2];
                        o[0] += lo16(r4.x); o[1] += hi16(r4.x); o[2] += lo16(r4.y); o[3] += hi16(r4.y);
                        o[4] += lo16(r4.z); o[5] += hi16(r4.z); o[6] += lo16(r4.w); o[7] += hi16(r4.w);
                    }
                    if (relu) {
#pragma unroll
                        for (int e = 0; e < 8; ++e) o[e] = relu_keep_nan(o[e]);
                    }
                    u32x4_t out;
                    out.x = pack2(o[0], o[1]); out.y = pack2(o[2], o[3]);
                    out.z = pack2(o[4], o[5]); out.w = pack2(o[6], o[7]);
                    *reinterpret_cast<u32x4_t *>(ttile + l32 * kTPitch + (u * 32 + 16 * i2 + 8 * half) * 2) = out;
                }
            }
            // pieces -> rows: 8 lanes store 128 contiguous bytes of one pixel
            wave_fence();
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const int pr = trow + 8 * t;
                u32x4_t o4 = *reinterpret_cast<const u32x4_t *>(ttile + pr * kTPitch + tseg * 16);
                if (mbase + pr < a.M) {
                    const size_t off = ((size_t)(mbase + pr) * Ctot + g * 64) * 2 + tseg * 16;
                    if constexpr (HAS_MASK) {
                        const u32x4_t mv = *reinterpret_cast<const u32x4_t *>(mg + off);
                        o4.x = keep_where_positive_bf16(o4.x, mv.x); o4.y = keep_where_positive_bf16(o4.y, mv.y);
                        o4.z = keep_where_positive_bf16(o4.z, mv.z); o4.w = keep_where_positive_bf16(o4.w, mv.w);
                    }
                    *reinterpret_cast<u32x4_t *>(yg + off) = o4;
                }
            }
            wave_fence();
        }
        if (!more) break;
        tile = next;
        if constexpr (!AHEAD) {
            load_x(tile, xf);
            if constexpr (HAS_RES) load_res(tile, 0, rv[0]);
        }
        if constexpr (AHEAD && HAS_RES && (NG & 1)) {
#pragma unroll
            for (int u = 0; u < 2; ++u)
#pragma unroll
                for (int i2 = 0; i2 < 2; ++i2) rv[0][u][i2] = rv[1][u][i2];
        }
    }
}

// Channels per slice: the most 64-channel groups (4, 2 or 1) that divide Cout and whose weight
// rows fit next to the transposition tiles.
static int slice_groups(const ConvArgs &a) {
    const int groups = a.Cout / 64;
    for (int ng = 4; ng >= 1; ng >>= 1)
        if (groups % ng == 0 && (size_t)ng * 64 * ((size_t)a.Cin * 2 + 16 + 8) <= 72 * 1024) return ng;
    return 0;
}

// The streaming kernel applies to bf16 1x1 convolutions without padding with a short reduction
// axis.  Measured on MI355X (batch 128): with 64 or 128 input channels it beats the tiled kernel
// for any number of output slices (128 -> 512 at 28 x 28: 49 against 62 us); with 256 input
// channels only while all output channels fit one slice of 64 (each further slice re-reads a
// 512-byte activation row that the tiled kernel shares through LDS), and never with 512.
// (256 -> 128 at 56 x 56 with both 64-channel groups in one slice: 59 against 72 us for the GEMM kernel when the
// layer is repeated on its own, no difference inside the forward pass - left with the GEMM kernel.)
bool conv1x1_stream_applies(const ConvArgs &a) {
    if (!a.bf16 || a.R != 1 || a.S != 1 || a.pad != 0 || a.Cout % 64 || a.relu > 1) return false;
    if (a.Cin == 256) return a.Cout == 64;
    if (a.Cin != 64 && a.Cin != 128) return false;
    return slice_groups(a) != 0;
}

template <int NS, int NG, int WAVES, bool SLICED, bool HAS_MASK>
static hipError_t launch_stream_s(const ConvArgs &a, hipStream_t stream) {
    const long long tiles = ((long long)a.M + 31) / 32;
    const long long groups = (tiles + WAVES - 1) / WAVES;
    const int nslices = SLICED ? a.Cout / (NG * 64) : 1;
    // one workgroup per CU and slice set; fewer when there are not enough tiles for that.  The masked
    // variants are the backward pass's data gradients, which share the GPU with the weight-gradient
    // stream: workgroups that hold their CU for the whole launch were 1.5 % slower there than one
    // workgroup per WAVES tiles, which leaves and lets the other stream's workgroups in.
    long long cap = HAS_MASK ? groups : 256 / nslices;
    if (cap < 8) cap = 8;
    const long long nworkers = groups < cap ? groups : cap;
    const long long blocks = SLICED ? (nworkers + 7) / 8 * 8 * nslices : nworkers;
    if (blocks <= 0 || blocks > 0x7FFFFFFFLL) return hipErrorInvalidValue;
    const dim3 grid((unsigned)blocks), block(WAVES * 64);
    const size_t lds = (size_t)NG * 64 * ((size_t)NS * 128 + 16 + 8) + (size_t)WAVES * 32 * kTPitch;
    if (lds > 160 * 1024) return hipErrorInvalidValue;
    static bool raised = false;                  // more than the default 64 KB of dynamic LDS
    if (lds > 64 * 1024 && !raised) {
        hipError_t e = hipFuncSetAttribute(
            reinterpret_cast<const void *>(conv1x1_stream_kernel<NS, NG, WAVES, true, SLICED, HAS_MASK>),
            hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e == hipSuccess)
            e = hipFuncSetAttribute(
                reinterpret_cast<const void *>(conv1x1_stream_kernel<NS, NG, WAVES, false, SLICED, HAS_MASK>),
                hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e != hipSuccess) return e;
        raised = true;
    }
    if (a.res) conv1x1_stream_kernel<NS, NG, WAVES, true, SLICED, HAS_MASK><<<grid, block, lds, stream>>>(a, (int)nworkers);
    else conv1x1_stream_kernel<NS, NG, WAVES, false, SLICED, HAS_MASK><<<grid, block, lds, stream>>>(a, (int)nworkers);
    return hipGetLastError();
}

// The larger slices need more than the 128 registers that 16 wavefronts per CU leave a lane:
// those run 12 wavefronts (170 registers).
template <int NS, int NG, int WAVES>
static hipError_t launch_stream(const ConvArgs &a, hipStream_t stream) {
    // the variants that also apply a mask (the backward pass's data gradients) always take the
    // 12-wavefront budget: the 16-wavefront ones have no register to spare
    constexpr int W12 = WAVES > 12 ? 12 : WAVES;
    if (a.Cout == NG * 64) {
        constexpr int WV = NS * NG <= 4 ? WAVES : W12;
        if (a.mask) return launch_stream_s<NS, NG, W12, false, true>(a, stream);
        // two or four operand slices and a residual do not fit 128 registers
        if (NS > 1 && a.res) return launch_stream_s<NS, NG, W12, false, false>(a, stream);
        return launch_stream_s<NS, NG, WV, false, false>(a, stream);
    }
    constexpr int WV = NS * NG <= 2 ? WAVES : W12;
    if (a.mask) return launch_stream_s<NS, NG, W12, true, true>(a, stream);
    return launch_stream_s<NS, NG, WV, true, false>(a, stream);
}

template <int WAVES>
hipError_t launch_conv1x1_stream_t(const ConvArgs &a, hipStream_t stream) {
    if (conv_check(a) || !conv1x1_stream_applies(a)) return hipErrorInvalidValue;
    const int key = (a.Cin / 64) * 10 + slice_groups(a);
    switch (key) {
    case 11: return launch_stream<1, 1, WAVES>(a, stream);
    case 12: return launch_stream<1, 2, WAVES>(a, stream);
    case 14: return launch_stream<1, 4, WAVES>(a, stream);
    case 21: return launch_stream<2, 1, WAVES>(a, stream);
    case 22: return launch_stream<2, 2, WAVES>(a, stream);
    case 24: return launch_stream<2, 4, WAVES>(a, stream);
    case 41: return launch_stream<4, 1, WAVES>(a, stream);
    default: return hipErrorInvalidValue;
    }
}

hipError_t launch_conv1x1_stream(const ConvArgs &a, hipStream_t stream) {
    // Workgroups share one staged copy of the weights, so larger ones stage less; small
    // problems keep small workgroups so that every CU still gets one.
    const long long tiles = ((long long)a.M + 31) / 32;
    if (tiles >= 2048) return launch_conv1x1_stream_t<16>(a, stream);
    if (tiles >= 1024) return launch_conv1x1_stream_t<8>(a, stream);
    return launch_conv1x1_stream_t<4>(a, stream);
}

}  // namespace delta
