// y[M, N] = act(scale_n * (x[M, K] . w[N, K]^T) + shift_n (+ res)) (* [mask > 0]) for gfx950, bf16.
// Row m of x is pixel m of the input, or, for a strided 1x1 convolution, the input pixel under output pixel m.
//
// The dense layers of a recomputation segment whose reduction axis is long: the linear layers of a
// transformer encoder (the paper's BERT-base workload, Sec. 5.2) and the 1x1 stride-1 convolutions
// with many input channels - both are plain "NT" GEMMs (both operands contiguous along K), bound
// by the matrix cores.  The tiled convolution kernel treats them as a convolution (64 x 64 tiles
// per wavefront, slices staged through registers); this kernel is built for the GEMM:
//  * workgroup tile 256 x 256 (16 wavefronts as 4 x 4) or 256 x 192 (12 wavefronts) where the output is
//    at least 192 channels wide, 128 x 128 (4 wavefronts, two workgroups per CU) for 128 channels;
//    64 x 64 per
//    wavefront and at most 128 registers, so that four (three) wavefronts share a SIMD: with
//    128 x 64 per wavefront (8 | 6 wavefronts, two per SIMD, fewer operand reads per MFMA) the same
//    kernel was 5-13 % slower - a SIMD needs more than two wavefronts to keep its MFMA pipe fed
//    across the barrier and the operand reads; the width is the one that leaves fewer CUs idle
//    (768 output channels: 4 tiles of 192 fill the chip at 16384 rows, 3 tiles of 256 leave a
//    quarter of it idle);
//  * K slices of 64 go from global memory straight into LDS (global_load_lds, 16 bytes per lane,
//    no registers, no LDS store instructions) through TWO buffers of 64 KB (56 KB): a tile row is a
//    whole 128-byte line of the operand, one barrier per 64 of K, and the slice after the current one
//    is in flight while the current one is multiplied (2000 cycles of MFMA work per SIMD at full
//    rate).  The operand pieces of a 16-wide step are read from LDS into one of two register sets
//    while the other set's MFMAs issue (the barrier of a slice stands before its last step, so the
//    first pieces of the next slice are read under that step's MFMAs), and the scheduler is told to
//    alternate LDS reads and MFMAs: with LDS reads and MFMAs left to the compiler's order every
//    wavefront read all its pieces after the barrier and the matrix pipe idled meanwhile (3-9 % of a
//    layer's time; the loop alone, operands resident in LDS: 1.75 -> 2.1 PFLOP/s).  Measured against four buffers of 32 (two and three slices ahead, also with a fifth
//    buffer, also with the next slice's first operands read before the barrier): those were all the
//    same speed, this is 4-9 % faster on the encoder's and ResNet's shapes; with the loads switched
//    off the loop runs at 1.3-1.5 PFLOP/s and removing the barrier changes nothing: what holds the
//    kernel at about 1 PFLOP/s is the delivery of the operands, not the barrier or LDS (LDS
//    reads are a quarter of the cycles by the counters): with every slice served by the L2 the loop
//    below runs at 1.8 PFLOP/s, served by the Infinity Cache at 0.93, by HBM at 0.8-0.87 (the L2
//    delivers 35 TB/s, the two behind it 6-7 TB/s).  Re-measured inside ResNet-50's forward
//    pass, where a layer's operands come from HBM rather than the caches: slices of 32 through four
//    buffers, three of them in flight, were again 1 % slower.  Also measured and slower: the loads
//    of a slice spread over its four steps instead of issued at its start (5-8 %), and x three
//    slices deep with w two deep in the same 160 KB (3-8 %);
//  * a tile row is 128 bytes = 8 pieces of 16; piece p of row r lives in slot p ^ ((r >> 1) & 7):
//    the direct loads fix where a LANE's 16 bytes land, so the swizzle is applied to the global
//    address each lane fetches; 16 lanes reading one piece of 16 consecutive rows then touch all
//    64 banks once;
//  * workgroups are numbered so that each XCD (blockIdx % 8) walks a contiguous range of x-row
//    tiles with all their w tiles: x rows and the whole of w stay in that XCD's L2;
//  * epilogue: a wavefront-private fp32 tile in LDS turns channel-major accumulators into 128-byte
//    pixel rows; scale/shift, residual, activation (none / ReLU / GELU), optional mask, one rounding;
//    the residual and mask rows of the next 32 pixels are requested while the current ones are finished.
// Rows past M or N are fetched from the last valid row (never stored).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kernels.hpp"

namespace delta {
namespace gemm {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

static constexpr int kBK = 64;
static constexpr int kTM = 2, kTN = 2;                                  // 2 x 2 tiles of 32 x 32 per wavefront
static constexpr int kStgPitch = 64 * 4 + 16;                          // fp32 staging row: 64 channels + pad

__device__ __forceinline__ uint32_t pack2(float lo, float hi) {
    const f32x2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}
__device__ __forceinline__ float lo16(uint32_t p) { return __uint_as_float(p << 16); }
__device__ __forceinline__ float hi16(uint32_t p) { return __uint_as_float(p & 0xFFFF0000u); }

__device__ __forceinline__ void wave_lds_fence() {
    // LDS instructions of one wavefront execute in order; this only stops the compiler from moving
    // accesses across the point where lanes exchange data through LDS.
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

__device__ __forceinline__ float gelu_erf(float v) {     // v/2 (1 + erf(v / sqrt 2)); see conv_igemm.hip
    const float x = fabsf(v) * 0.70710678118654752f;
    const float t = __builtin_amdgcn_rcpf(1.0f + 0.3275911f * x);
    const float poly = t * (0.254829592f + t * (-0.284496736f + t * (1.421413741f + t * (-1.453152027f + t * 1.061405429f))));
    const float c = poly * __builtin_amdgcn_exp2f(-x * x * 1.4426950408889634f);
    return 0.5f * v * (v < 0.f ? c : 2.0f - c);
}

// BM: rows of x per workgroup, 256 or 128 (BM / 64 wavefront rows); BN: rows of w (output channels)
// per workgroup, 256, 192 or 128 (BN / 64 wavefront columns).
// S: LDS buffers of one K slice each (2 or 4); S - 1 slices are in flight while one is multiplied.
template <int BM, int BN, int S>
__global__ __launch_bounds__((BM / 64) * (BN / 64) * 64) void gemm_nt_kernel(ConvArgs a, int tiles_n, int tiles_total) {
    static_assert(S >= 2 && S <= 4, "two to four slice buffers");
    constexpr int kBM = BM, kBN = BN, kWM = BM / 64, kWN = BN / 64, kWaves = kWM * kWN;
    constexpr int kXBytes = kBM * kBK * 2;                  // x rows of one buffer
    constexpr int kStageBytes = kXBytes + BN * kBK * 2;
    constexpr int XI = (kBM / 8 + kWaves - 1) / kWaves, WI = (BN / 8 + kWaves - 1) / kWaves;   // direct loads per wavefront and slice
    extern __shared__ __align__(16) unsigned char smem[];
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int l32 = lane & 31, half = lane >> 5;
    const int wm = wv / kWN, wn = wv % kWN;
    const int M = a.M, N = a.Cout, K = a.Cin;
    // XCD-aware numbering: XCD x (= blockIdx % 8) takes logical tiles x * per .. (x + 1) * per
    const int per = (tiles_total + 7) / 8;
    const int logical = (blockIdx.x & 7) * per + (blockIdx.x >> 3);
    if (logical >= tiles_total) return;
    const int m0 = (logical / tiles_n) * kBM, n0 = (logical % tiles_n) * kBN;

    // ---- direct loads: one instruction fills 8 tile rows (1 KB); per slice a wavefront issues XI for
    // x and WI for w (when the rows do not divide evenly the last wavefronts repeat a neighbour's rows)
    const unsigned char *xg = static_cast<const unsigned char *>(a.x);
    const unsigned char *wg = static_cast<const unsigned char *>(a.w);
    const size_t krow = (size_t)K * 2;
    const unsigned char *xsrc[XI], *wsrc[WI];
    uint32_t xdst[XI], wdst[WI];
#pragma unroll
    for (int q = 0; q < XI; ++q) {
        int g = wv * XI + q;
        g = g < kBM / 8 ? g : kBM / 8 - 1;
        const int r = 8 * g + (lane >> 3);                              // row of the tile this lane fills
        const int piece = (lane & 7) ^ ((r >> 1) & 7);                 // which 16 bytes of the row land in this lane's slot
        int xr = m0 + r;
        xr = xr < M ? xr : M - 1;
        size_t xpix = (size_t)xr;
        if (a.stride != 1) {                                            // a strided 1x1 layer reads every stride-th pixel
            const int oq = xr % a.Q, t = xr / a.Q, op = t % a.P, n = t / a.P;
            xpix = ((size_t)n * a.H + (size_t)op * a.stride) * a.W + (size_t)oq * a.stride;
        }
        xsrc[q] = xg + xpix * krow + piece * 16;
        xdst[q] = (uint32_t)g * 1024u;
    }
#pragma unroll
    for (int q = 0; q < WI; ++q) {
        int g = wv * WI + q;
        g = g < BN / 8 ? g : BN / 8 - 1;
        const int r = 8 * g + (lane >> 3);
        const int piece = (lane & 7) ^ ((r >> 1) & 7);
        int wr = n0 + r;
        wr = wr < N ? wr : N - 1;
        wsrc[q] = wg + (size_t)wr * krow + piece * 16;
        wdst[q] = (uint32_t)kXBytes + (uint32_t)g * 1024u;
    }
    // The direct loads and the waits for them are written as inline assembly: the compiler does not
    // track what a direct load writes, the explicit waits below do.
    typedef __attribute__((address_space(3))) unsigned char *lptr_t;
    const uint32_t lds0 = (uint32_t)(uintptr_t)(lptr_t)smem;
    const int nslices = K / kBK;
    auto fetch = [&](int t, int buf) {
        const uint32_t sb = lds0 + (uint32_t)buf * kStageBytes;
#pragma unroll
        for (int q = 0; q < XI; ++q)
            asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off"
                         :: "v"(xsrc[q] + (size_t)t * 128), "s"(__builtin_amdgcn_readfirstlane(sb + xdst[q])) : "memory", "m0");
#pragma unroll
        for (int q = 0; q < WI; ++q)
            asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off"
                         :: "v"(wsrc[q] + (size_t)t * 128), "s"(__builtin_amdgcn_readfirstlane(sb + wdst[q])) : "memory", "m0");
    };
    f32x16 acc[kTM][kTN];
#pragma unroll
    for (int i = 0; i < kTM; ++i)
#pragma unroll
        for (int j = 0; j < kTN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    // operand reads: row (tile row of this lane), piece 2 * k2 + half, swizzled
    int xoff[kTM], woff[kTN], xsw[kTM], wsw[kTN];
#pragma unroll
    for (int i = 0; i < kTM; ++i) {
        const int r = wm * (32 * kTM) + i * 32 + l32;
        xoff[i] = r * 128;
        xsw[i] = (r >> 1) & 7;
    }
#pragma unroll
    for (int j = 0; j < kTN; ++j) {
        const int r = wn * 64 + j * 32 + l32;
        woff[j] = kXBytes + r * 128;
        wsw[j] = (r >> 1) & 7;
    }

    // Operand pieces of step q of the slice in buffer `buf`, into register set `f`
    u32x4 xf[2][kTM], wf[2][kTN];
    auto read_step = [&](int buf, int q, int f) {
        const unsigned char *base = smem + (size_t)buf * kStageBytes;
#pragma unroll
        for (int i = 0; i < kTM; ++i) xf[f][i] = *reinterpret_cast<const u32x4 *>(base + xoff[i] + (((2 * q + half) ^ xsw[i]) << 4));
#pragma unroll
        for (int j = 0; j < kTN; ++j) wf[f][j] = *reinterpret_cast<const u32x4 *>(base + woff[j] + (((2 * q + half) ^ wsw[j]) << 4));
    };
    // Direct loads complete in order: "at most n later slices outstanding" is vmcnt(n * loads per slice).
    constexpr int kLoads = XI + WI;
    auto wait_slices = [&](int later) {
        if (S == 2 || later <= 0) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        else if (later == 1) asm volatile("s_waitcnt vmcnt(%0)" :: "n"(kLoads) : "memory");
        else asm volatile("s_waitcnt vmcnt(%0)" :: "n"(2 * kLoads) : "memory");
    };
#pragma unroll
    for (int i = 0; i < S - 1; ++i)
        if (i < nslices) fetch(i, i);
    wait_slices((nslices - 1 < S - 2) ? nslices - 1 : S - 2);          // slice 0 has landed
    __syncthreads();
    if (S - 1 < nslices) fetch(S - 1, S - 1);
    read_step(0, 0, 0);
    for (int t = 0; t < nslices; ++t) {
        const int buf = t % S;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            if (q == 3) {
                // this wavefront's loads of slice t + 1 have landed (those of the slices after it may still
                // travel), and its last reads of buffer `buf` (step 3's pieces, requested during step 2) are
                // in registers
                {
                    const int last = t + S - 1 < nslices - 1 ? t + S - 1 : nslices - 1;   // last slice requested so far
                    wait_slices(last - (t + 1));
                }
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                __syncthreads();                   // everyone's have
                if (t + S < nslices) fetch(t + S, buf);
                if (t + 1 < nslices) read_step((t + 1) % S, 0, 0);
            } else {
                read_step(buf, q + 1, (q + 1) & 1);
            }
#pragma unroll
            for (int i = 0; i < kTM; ++i)
#pragma unroll
                for (int j = 0; j < kTN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, wf[q & 1][j]),
                                                                        __builtin_bit_cast(bf16x8, xf[q & 1][i]), acc[i][j], 0, 0, 0);
#pragma unroll
            for (int k = 0; k < kTM + kTN; ++k) {
                __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x008, (kTM * kTN) / (kTM + kTN), 0);
            }
        }
    }

    // ---- epilogue.  acc[i][j]: lane holds pixel (x row) l32 of tile i and channels 8*rb + 4*half + e of tile j
    unsigned char *stg = smem + (size_t)wv * (32 * kStgPitch);
    unsigned char *yg = static_cast<unsigned char *>(a.y);
    const unsigned char *rg = static_cast<const unsigned char *>(a.res);
    const unsigned char *mg = static_cast<const unsigned char *>(a.mask);
    const int prow = lane >> 3, cseg = lane & 7;
    const int chan = n0 + wn * 64 + cseg * 8;
    // scale / shift of this lane's 8 channels in the row-major phase (the same for every row)
    float sc[8], sh[8];
    {
        const int ch = chan < N ? chan : 0;          // N is a multiple of 8: the 8 channels are inside or outside together
        const f32x4 s0 = *reinterpret_cast<const f32x4 *>(a.scale + ch), s1 = *reinterpret_cast<const f32x4 *>(a.scale + ch + 4);
        const f32x4 h0 = *reinterpret_cast<const f32x4 *>(a.shift + ch), h1 = *reinterpret_cast<const f32x4 *>(a.shift + ch + 4);
        sc[0] = s0.x; sc[1] = s0.y; sc[2] = s0.z; sc[3] = s0.w; sc[4] = s1.x; sc[5] = s1.y; sc[6] = s1.z; sc[7] = s1.w;
        sh[0] = h0.x; sh[1] = h0.y; sh[2] = h0.z; sh[3] = h0.w; sh[4] = h1.x; sh[5] = h1.y; sh[6] = h1.z; sh[7] = h1.w;
    }
    // residual and mask rows of tile i + 1 are requested while tile i is finished (a workgroup is
    // alone on its CU: nothing else would cover their latency; it was most of a short-K layer's time)
    u32x4 rres[kTM > 2 ? 2 : 1][4], rmsk[kTM > 2 ? 2 : 1][4];
    auto request = [&](int i, u32x4 (&rr)[4], u32x4 (&rm)[4]) {
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const int m = m0 + wm * (32 * kTM) + i * 32 + prow + 8 * t;
            const bool ok = m < M && chan < N;
            const size_t off = ((size_t)(ok ? m : 0) * N + (ok ? chan : 0)) * 2;
            rr[t] = rg ? *reinterpret_cast<const u32x4 *>(rg + off) : u32x4{0u, 0u, 0u, 0u};
            rm[t] = mg ? *reinterpret_cast<const u32x4 *>(mg + off) : u32x4{0u, 0u, 0u, 0u};
        }
    };
    constexpr bool kAhead = kTM > 2;              // the 64-row wavefront tiles have no registers for a tile ahead
    request(0, rres[0], rmsk[0]);
#pragma unroll
    for (int i = 0; i < kTM; ++i) {
        if constexpr (kAhead) {
            if (i + 1 < kTM) request(i + 1, rres[(i + 1) & 1], rmsk[(i + 1) & 1]);
        } else {
            if (i > 0) request(i, rres[0], rmsk[0]);
        }
        wave_lds_fence();
#pragma unroll
        for (int j = 0; j < kTN; ++j)
#pragma unroll
            for (int rb = 0; rb < 4; ++rb) {
                const f32x16 &c = acc[i][j];
                const f32x4 v = {c[4 * rb + 0], c[4 * rb + 1], c[4 * rb + 2], c[4 * rb + 3]};
                *reinterpret_cast<f32x4 *>(stg + l32 * kStgPitch + (j * 32 + 8 * rb + 4 * half) * 4) = v;
            }
        wave_lds_fence();
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const int pr = prow + 8 * t;
            const int m = m0 + wm * (32 * kTM) + i * 32 + pr;
            if (m >= M || chan >= N) continue;
            const f32x4 f0 = *reinterpret_cast<const f32x4 *>(stg + pr * kStgPitch + cseg * 32);
            const f32x4 f1 = *reinterpret_cast<const f32x4 *>(stg + pr * kStgPitch + cseg * 32 + 16);
            float v[8] = {f0.x, f0.y, f0.z, f0.w, f1.x, f1.y, f1.z, f1.w};
#pragma unroll
            for (int e = 0; e < 8; ++e) v[e] = v[e] * sc[e] + sh[e];
            const size_t off = ((size_t)m * N + chan) * 2;
            if (rg) {
                const u32x4 rv = rres[kAhead ? (i & 1) : 0][t];
                v[0] += lo16(rv.x); v[1] += hi16(rv.x); v[2] += lo16(rv.y); v[3] += hi16(rv.y);
                v[4] += lo16(rv.z); v[5] += hi16(rv.z); v[6] += lo16(rv.w); v[7] += hi16(rv.w);
            }
            if (a.relu == 1) {
#pragma unroll
                for (int e = 0; e < 8; ++e) v[e] = v[e] < 0.f ? 0.f : v[e];
            } else if (a.relu == 2) {
#pragma unroll
                for (int e = 0; e < 8; ++e) v[e] = gelu_erf(v[e]);
            }
            u32x4 o;
            o.x = pack2(v[0], v[1]); o.y = pack2(v[2], v[3]); o.z = pack2(v[4], v[5]); o.w = pack2(v[6], v[7]);
            if (mg) {
                const u32x4 mv = rmsk[kAhead ? (i & 1) : 0][t];
                o.x = keep_where_positive_bf16(o.x, mv.x); o.y = keep_where_positive_bf16(o.y, mv.y);
                o.z = keep_where_positive_bf16(o.z, mv.z); o.w = keep_where_positive_bf16(o.w, mv.w);
            }
            *reinterpret_cast<u32x4 *>(yg + off) = o;
        }
    }
}

}  // namespace gemm

namespace {

// Workgroup tiles.  Measured at batch 128 on ResNet-50's 1x1 layers, us per launch when the layer is
// repeated on its own (operands warm in the caches) | inside the forward pass (operands cold):
//                         256x256      256x128      128x128      tiled convolution kernel
//   512 -> 128, 28 x 28     38.2         32.9       29.6 | 37.2    34.0 | 38.3
//   256 -> 128, 56 x 56    101.3         85.3       74.6 | 78.7    77.4 | 83.4
//   1024 -> 256, 14 x 14    30.1       22.1 | 30.2    22.6         25.3 | 28.0
//   2048 -> 512, 7 x 7         -         32.3       26.5 | 38.5    27.5 | 30.7
//   512 -> 256, 28 x 28   40.3 | 55.5    52.7         47.0
//   256 -> 1024, 14 x 14    31.4         38.6         34.2
//   1024 -> 512, 14 x 14    32.0         39.1         39.5
//   512 -> 2048, 7 x 7      22.5         27.5         26.3
// 128 x 256 for 1024 -> 256 at 14 x 14 (196 workgroups without padded columns instead of 196 with a third of their
// columns padding): 26 -> 22 us on its own, no change inside the pass with two slice buffers, 23 us less for the five
// layers inside the pass with THREE (two slices in flight per workgroup); the same tile on 512 -> 2048 at 7 x 7 and
// 1024 -> 512 at 14 x 14 was 20 % slower than 256 x 256.
// With cold operands the two-deep pipeline of this kernel is short: one slice ahead does not cover a
// miss to HBM, and the tiled kernel's three workgroups per CU cover each other's.  So the narrow tiles
// take only the layers with at most 128 output channels, where they win both ways.
struct Tile { int bm, bn, stages; };
const Tile kTiles[] = {{256, 256, 2}, {256, 192, 2}, {128, 128, 2}, {128, 128, 4}, {128, 256, 3}};

long long tiles_of(const ConvArgs &a, const Tile &t) {
    return (((long long)a.M + t.bm - 1) / t.bm) * ((a.Cout + t.bn - 1) / t.bn);
}

// Width of the w tile: the one whose number of rounds over the 256 CUs (one workgroup per CU) times
// its cost per tile is smaller; e.g. 768 output channels are 3 tiles of 256 (192 workgroups at
// batch 32 x 512: a quarter of the chip idle) but 4 tiles of 192 (256 workgroups, one full round).
const Tile &pick_tile(const ConvArgs &a) {
    if (a.Cout <= 128) return kTiles[2];
    if (a.Cout <= 256 && tiles_of(a, kTiles[0]) < 192) return kTiles[4];
    const long long c256 = ((tiles_of(a, kTiles[0]) + 255) / 256) * 256, c192 = ((tiles_of(a, kTiles[1]) + 255) / 256) * 192;
    return c192 < c256 ? kTiles[1] : kTiles[0];
}

// The tile a layer runs on, or nullptr where this kernel does not apply.  A layer that fills the chip
// takes the two-buffer tiles above.  One that does not (2048 -> 512 on 7 x 7 images: 196 tiles of
// 128 x 128; a classifier: 8) is a chain of slice latencies - about 0.8 us per slice of 64 on the tiled
// kernel, whatever else the chip does - so with a long reduction it takes 128 x 128 tiles with FOUR
// slice buffers: three slices in flight per workgroup (128 KB of LDS: one workgroup per CU, which is
// all such a layer has).
const Tile *choose_tile(const ConvArgs &a) {
    if (!a.bf16 || a.R != 1 || a.S != 1 || a.stride < 1 || a.pad != 0) return nullptr;
    if (a.Cin % 64 || a.Cin < 256 || a.Cout % 8 || a.Cout < 128) return nullptr;
    if (a.Cout <= 128 || a.Cout >= 192) {
        const Tile &t = pick_tile(a);
        const long long tiles = tiles_of(a, t);
        if (tiles > 0x3FFFFFF0LL) return nullptr;
        if (tiles >= (a.Cout <= 128 ? 512 : 128)) return &t;
    }
    if (a.Cin >= 512 && tiles_of(a, kTiles[3]) <= 512) return &kTiles[3];
    return nullptr;
}

template <int BM, int BN, int S>
hipError_t launch_tile(const ConvArgs &a, hipStream_t stream) {
    constexpr size_t pipe = (size_t)S * ((size_t)BM * gemm::kBK * 2 + (size_t)BN * gemm::kBK * 2);
    constexpr size_t stage_out = (size_t)(BM / 64) * (BN / 64) * 32 * gemm::kStgPitch;
    constexpr size_t lds = pipe > stage_out ? pipe : stage_out;
    static_assert(lds <= 160 * 1024, "LDS");
    constexpr int threads = (BM / 64) * (BN / 64) * 64;
    const int tiles_m = (a.M + BM - 1) / BM, tiles_n = (a.Cout + BN - 1) / BN;
    const long long total = (long long)tiles_m * tiles_n;
    const long long blocks = (total + 7) / 8 * 8;
    static bool raised = false;
    if (!raised) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(gemm::gemm_nt_kernel<BM, BN, S>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        raised = true;
    }
    gemm::gemm_nt_kernel<BM, BN, S><<<dim3((unsigned)blocks), dim3(threads), lds, stream>>>(a, tiles_n, (int)total);
    return hipGetLastError();
}

}  // namespace

// bf16 1x1 layers (rows of x contiguous) with a reduction axis of at least 256 and either enough
// output to fill the chip with the two-buffer tiles or a reduction long enough for the four-buffer one.
bool gemm_nt_applies(const ConvArgs &a) { return choose_tile(a) != nullptr; }

const char *gemm_nt_kernel_name(const ConvArgs &a) {
    const Tile *t = choose_tile(a);
    if (!t) return "";
    if (t->bm == 256)
        return t->bn == 256 ? "gemm_nt bf16 256x256 (64x64 per wave, direct-to-LDS)"
                            : "gemm_nt bf16 256x192 (64x64 per wave, direct-to-LDS)";
    if (t->bn == 256) return "gemm_nt bf16 128x256, three slice buffers (64x64 per wave, direct-to-LDS)";
    return t->stages == 4 ? "gemm_nt bf16 128x128, four slice buffers (64x64 per wave, direct-to-LDS)"
                          : "gemm_nt bf16 128x128 (64x64 per wave, direct-to-LDS)";
}

hipError_t launch_gemm_nt(const ConvArgs &a, hipStream_t stream) {
    const Tile *t = conv_check(a) ? nullptr : choose_tile(a);
    if (!t) return hipErrorInvalidValue;
    if (t->bm == 256) return t->bn == 256 ? launch_tile<256, 256, 2>(a, stream) : launch_tile<256, 192, 2>(a, stream);
    if (t->bn == 256) return launch_tile<128, 256, 3>(a, stream);
    return t->stages == 4 ? launch_tile<128, 128, 4>(a, stream) : launch_tile<128, 128, 2>(a, stream);
}

}  // namespace delta
