// Fused layer kernel for gfx950: y = relu?(scale_k * conv(x, w) + shift_k (+ res)).
//
// This is the operator that DELTA's Recompute action re-runs for a released activation
// (Sec. 3, Table 1; Sec. 5.5 names ConvForward / BNForward among the regenerated
// operators).  The first forward and every recomputation go through this same kernel
// with the same tiling and the same summation order, so a recomputed tensor is
// bit-identical to the original.
//
// Formulation: implicit GEMM  D[k][m] = sum_{r,s,c} w[k][r][s][c] * x[pixel m shifted by (r,s)][c]
// with the output channels on the MFMA row axis and the output pixels on the column
// axis.  In the 32x32 accumulator layout a lane then owns 4 consecutive channels of one
// pixel, which is what NHWC wants.
//
// Per workgroup (256 threads = 4 wavefronts of 64): BM output pixels x BN output channels.
// The reduction runs over (tap, 128-byte slice of Cin).  Each slice of the BM gathered input
// rows and of the BN weight rows is fetched with 16-byte buffer loads (8 lanes cover one
// 128-byte row) and staged in LDS with rows padded to 144 bytes (conflict-free ds_read_b128).
// Pipeline, one barrier per slice: slice t is multiplied out of LDS buffer t % 2 while slice
// t+1 moves from registers into the other buffer and slice t+3 is requested from memory.
// The fetches go through buffer descriptors: padding taps, rows past the last pixel, channel
// rows past Cout and slices past the last one are given an offset outside the descriptor, which
// loads zeros.  Nothing in a step is conditional, so the compiler knows how many loads are in
// flight at each wait and waits only for the slice it is about to store (with branches around
// the loads it waited for all of them, which halved the speed).
// Within a slice, lane half h owns bytes [64h, 64h+64) of every row for both operands, so the
// pairing of products is the same for w and x whatever the hardware's internal k order is.
//
// Epilogue: fp32 scale/shift in the accumulator layout, then through a wavefront-private
// fp32 LDS tile into row-major order, so that the residual is read and y is written with
// 16 bytes per lane and 128 contiguous bytes per pixel; residual add and ReLU in fp32, one
// rounding to the storage type.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kernels.hpp"

namespace delta {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));   // native vectors keep register arrays out of scratch

static constexpr int kThreads = 256;
static constexpr int kRowBytes = 128;   // bytes of the reduction axis per LDS row and slice
static constexpr int kRowPitch = 144;   // padded pitch: 16 consecutive rows hit 64 distinct banks

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
// two fp32 -> packed bf16, round to nearest even (v_cvt_pk_bf16_f32)
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
    const f32x2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

__device__ __forceinline__ float bf16_lo(uint32_t packed) { return __uint_as_float(packed << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t packed) { return __uint_as_float(packed & 0xFFFF0000u); }

template <bool BF16> struct Elem {
    static constexpr int size = BF16 ? 2 : 4;
    static constexpr int per_slice = kRowBytes / size;   // reduction elements per slice
    static constexpr int group = kRowBytes / size;       // output channels per 128-byte store row
};

// One 16-byte piece of both operands -> MFMAs.  a = weights (rows), b = activations (columns).
template <bool BF16>
__device__ __forceinline__ void mma16(const u32x4 a, const u32x4 b, f32x16 &acc) {
    if constexpr (BF16) {
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a),
                                                      __builtin_bit_cast(bf16x8, b), acc, 0, 0, 0);
    } else {
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.x), __uint_as_float(b.x), acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.y), __uint_as_float(b.y), acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.z), __uint_as_float(b.z), acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.w), __uint_as_float(b.w), acc, 0, 0, 0);
    }
}

__device__ __forceinline__ void wave_lds_fence() {
    // LDS instructions of one wavefront execute in order; this only stops the compiler
    // from moving accesses across the point where lanes exchange data through LDS.
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// offset that lies outside every buffer descriptor used here (their sizes stay below 2 GiB)
static constexpr int kOutOfRange = (int)0x80000000;

// GELU in its erf form, v/2 (1 + erf(v / sqrt 2)).  1 + erf(x) = erfc(-x): for x < 0 it is
// erfc(|x|), for x >= 0 it is 2 - erfc(x), and erfc(|x|) = poly(t) exp(-x^2), t = 1/(1 + p |x|)
// (Abramowitz & Stegun 7.1.26, absolute error 1.5e-7) - no cancellation in the negative tail, one
// exp and one reciprocal per element instead of the library erff's branches.
__device__ __forceinline__ float gelu_erf(float v) {
    const float x = fabsf(v) * 0.70710678118654752f;
    const float t = __builtin_amdgcn_rcpf(1.0f + 0.3275911f * x);
    const float poly = t * (0.254829592f + t * (-0.284496736f + t * (1.421413741f + t * (-1.453152027f + t * 1.061405429f))));
    const float c = poly * __builtin_amdgcn_exp2f(-x * x * 1.4426950408889634f);   // erfc(|x|)
    return 0.5f * v * (v < 0.f ? c : 2.0f - c);
}

// SCATTER: the scattered form described at ConvArgs (strided output pixels, a strided subset of the
// weight tensor's taps, residual read in the epilogue); HAS_RES is then false.
template <bool BF16, int BM, int BN, int WM, int WN, bool HAS_RES, bool SCATTER = false>
__global__ __launch_bounds__(kThreads) void conv_igemm_kernel(ConvArgs a) {
    using E = Elem<BF16>;
    constexpr int ES = E::size;
    constexpr int KC = E::per_slice;
    constexpr int CW = E::group;               // channels per store row (128 bytes of output)
    constexpr int TM = BM / WM / 32;           // 32-pixel tiles per wavefront
    constexpr int TN = BN / WN / 32;           // 32-channel tiles per wavefront
    constexpr int TG = CW / 32;                // channel tiles per staging group
    constexpr int XL = BM / 32;                // 16-byte loads per thread and slice, activations
    constexpr int WL = BN / 32;                // same, weights
    constexpr int STG_PITCH = CW * 4 + 16;
    constexpr int PITCH = kRowPitch;           // rows 4 banks apart
    constexpr int TILE_BYTES = 2 * (BM + BN) * PITCH;   // two buffers
    constexpr int STG_BYTES = 4 * 32 * STG_PITCH;
    constexpr int SMEM = TILE_BYTES > STG_BYTES ? TILE_BYTES : STG_BYTES;
    static_assert(WM * WN == 4 && TM >= 1 && TN >= 1 && TN % TG == 0, "bad tiling");

    __shared__ __align__(16) unsigned char smem[SMEM];
    __shared__ __align__(16) float sbn[2][BN];   // scale, shift of this tile's channels

    const int tid = threadIdx.x;
    const int lane = tid & 63, wv = tid >> 6;
    const int wm = wv % WM, wn = wv / WM;
    const int l32 = lane & 31, half = lane >> 5;

    // Workgroups are dealt round-robin to the 8 XCDs, each with its own L2.  Give every XCD a
    // contiguous run of logical tiles (channel tile fastest), so that the channel tiles of one
    // pixel tile, and neighbouring pixel tiles with their shared halo, meet in the same L2.
    unsigned logical;
    {
        const unsigned nb = gridDim.x, per = nb >> 3, rem = nb & 7u;
        const unsigned xcd = blockIdx.x & 7u, idx = blockIdx.x >> 3;
        logical = xcd < rem ? xcd * (per + 1) + idx : rem * (per + 1) + (xcd - rem) * per + idx;
    }
    const int tiles_n = (a.Cout + BN - 1) / BN;
    const int m0 = (int)(logical / tiles_n) * BM;
    const int n0 = (int)(logical % tiles_n) * BN;

    const unsigned char *xg = static_cast<const unsigned char *>(a.x);
    const unsigned char *wg = static_cast<const unsigned char *>(a.w);
    // folded batch-norm factors: fetched now, read in the epilogue (the barriers of the main
    // loop make them visible); channels past Cout get zeros
    if (tid < BN) {
        const int ch = n0 + tid;
        sbn[0][tid] = ch < a.Cout ? a.scale[ch] : 0.f;
        sbn[1][tid] = ch < a.Cout ? a.shift[ch] : 0.f;
    }

    // ---- per-thread gather coordinates: row = tid/8 + 32 i, 16-byte segment = tid%8.
    // Both operands are read through buffer descriptors with 32-bit offsets.  The activation
    // descriptor starts at the first input pixel this tile can touch (input pixel indices grow
    // with the output pixel index and with the tap), so offsets stay small whatever the tensor
    // size; an offset of kOutOfRange lies outside every descriptor and loads zeros.
    const int lrow = tid >> 3, seg = tid & 7;
    const size_t cin_bytes = (size_t)a.Cin * ES;
    const int PQ = a.P * a.Q;
    long long base_pix;
    {
        const int n = m0 / PQ, pq = m0 - n * PQ;
        const int p = pq / a.Q, q = pq - p * a.Q;
        base_pix = ((long long)n * a.H + (p * a.stride - a.pad)) * a.W + (q * a.stride - a.pad);
        if (base_pix < 0) base_pix = 0;
    }
    const unsigned long long xbytes = (unsigned long long)a.N * a.H * a.W * cin_bytes - (unsigned long long)base_pix * cin_bytes;
    const __amdgpu_buffer_rsrc_t xrsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<unsigned char *>(xg) + (size_t)base_pix * cin_bytes, 0,
        (int)(xbytes < 0x7FFFFFFFull ? xbytes : 0x7FFFFFFFull), 0x00020000);
    const int wtaps = SCATTER ? a.wR * a.wS : a.R * a.S;       // taps per output channel in memory
    const __amdgpu_buffer_rsrc_t wrsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<unsigned char *>(wg), 0, (int)((size_t)a.Cout * wtaps * cin_bytes), 0x00020000);
    int h0[XL], w0[XL];
    int xoff[XL];                  // byte offset of the row's tap (0,0) pixel, or kOutOfRange past M
#pragma unroll
    for (int i = 0; i < XL; ++i) {
        const int m = m0 + lrow + 32 * i;
        if (m < a.M) {
            const int n = m / PQ, pq = m - n * PQ;
            const int p = pq / a.Q, q = pq - p * a.Q;
            h0[i] = p * a.stride - a.pad;
            w0[i] = q * a.stride - a.pad;
            const long long pix = ((long long)n * a.H + h0[i]) * a.W + w0[i];
            xoff[i] = (int)((pix - base_pix) * (long long)cin_bytes) + seg * 16;
        } else {
            h0[i] = w0[i] = 0;
            xoff[i] = kOutOfRange;
        }
    }
    int woff[WL];
#pragma unroll
    for (int j = 0; j < WL; ++j) {
        const int k = n0 + lrow + 32 * j;
        woff[j] = k < a.Cout ? (int)((size_t)k * wtaps * cin_bytes) + seg * 16 : kOutOfRange;
    }
    const int cslices = a.Cin / KC;
    const int nslices = a.R * a.S * cslices;


    constexpr int TILE1 = (BM + BN) * PITCH;     // one buffer: x rows then w rows
    constexpr int D = 2;                          // slices in flight in registers
    constexpr int U = (D % 2 == 0) ? D : 2 * D;   // steps per unrolled round: buffer and register indices static
    u32x4 xr[D][XL], wr[D][WL];                   // register ring: set s holds a slice t with t % D == s

    // global -> registers for slice `it`.  Unconditional: a slice index past the end, padding,
    // rows past M and channel rows past Cout turn into out-of-range offsets, i.e. zeros, so the
    // number of loads in flight at every wait is a compile-time constant.
    auto fetch = [&](int it, u32x4 (&xd)[XL], u32x4 (&wd)[WL]) {
        const bool live = it < nslices;
        const int tap = it / cslices, cs = it - tap * cslices;
        const int r = tap / a.S, sx = tap - r * a.S;
        const int xadd = (r * a.W + sx) * (int)cin_bytes + cs * kRowBytes;
        const int wadd = (SCATTER ? (a.w_r0 + r * a.w_step) * a.wS + a.w_s0 + sx * a.w_step : r * a.S + sx) * (int)cin_bytes +
                         cs * kRowBytes;
#pragma unroll
        for (int i = 0; i < XL; ++i) {
            const int h = h0[i] + r, w = w0[i] + sx;
            const bool ok = live && xoff[i] != kOutOfRange && (unsigned)h < (unsigned)a.H && (unsigned)w < (unsigned)a.W;
            xd[i] = __builtin_amdgcn_raw_buffer_load_b128(xrsrc, ok ? xoff[i] + xadd : kOutOfRange, 0, 0);
        }
#pragma unroll
        for (int j = 0; j < WL; ++j)
            wd[j] = __builtin_amdgcn_raw_buffer_load_b128(
                wrsrc, live && woff[j] != kOutOfRange ? woff[j] + wadd : kOutOfRange, 0, 0);
    };
    auto store = [&](int buf, const u32x4 (&xd)[XL], const u32x4 (&wd)[WL]) {
        unsigned char *xb = smem + buf * TILE1, *wb = xb + BM * PITCH;
#pragma unroll
        for (int i = 0; i < XL; ++i) *reinterpret_cast<u32x4 *>(xb + (lrow + 32 * i) * PITCH + seg * 16) = xd[i];
#pragma unroll
        for (int j = 0; j < WL; ++j) *reinterpret_cast<u32x4 *>(wb + (lrow + 32 * j) * PITCH + seg * 16) = wd[j];
    };

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    auto mma = [&](int buf) {
        const unsigned char *xb = smem + buf * TILE1, *wb = xb + BM * PITCH;
#pragma unroll
        for (int j16 = 0; j16 < 4; ++j16) {
            const int koff = half * 64 + j16 * 16;
            u32x4 xf[TM], wf[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i)
                xf[i] = *reinterpret_cast<const u32x4 *>(xb + ((wm * TM + i) * 32 + l32) * PITCH + koff);
#pragma unroll
            for (int j = 0; j < TN; ++j)
                wf[j] = *reinterpret_cast<const u32x4 *>(wb + ((wn * TN + j) * 32 + l32) * PITCH + koff);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j) mma16<BF16>(wf[j], xf[i], acc[i][j]);
        }
    };

    // Pipeline, one barrier per slice: slice t is multiplied out of LDS buffer t % 2 while slice
    // t+1 moves from registers to the other buffer and slice t+1+D is requested into the
    // registers that frees.
#pragma unroll
    for (int i = 0; i < D; ++i) fetch(i, xr[i], wr[i]);
    // The residual rows of this wavefront's outputs are requested now, in the layout the
    // row-major phase of the epilogue uses, so that their latency hides behind the main loop
    // (a layer with few slices otherwise pays it again after its last MFMA).  Tile-relative
    // descriptor: rows past M lie past the end of the tensor, i.e. outside it.
    constexpr int CPL = CW / 8;                   // channels per lane in the row-major phase
    const int prow = lane >> 3, cseg = lane & 7;
    u32x4 rres[HAS_RES ? TN / TG : 1][HAS_RES ? TM : 1][4];
    if constexpr (HAS_RES) {
        const size_t row_bytes = (size_t)a.Cout * ES;
        const unsigned long long rbytes = (unsigned long long)(a.M - m0) * row_bytes;
        const __amdgpu_buffer_rsrc_t rrsrc = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<unsigned char *>(static_cast<const unsigned char *>(a.res)) + (size_t)m0 * row_bytes, 0,
            (int)(rbytes < 0x7FFFFFFFull ? rbytes : 0x7FFFFFFFull), 0x00020000);
#pragma unroll
        for (int g = 0; g < TN / TG; ++g) {
            const int chan = n0 + (wn * TN + g * TG) * 32 + cseg * CPL;
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    const int row = (wm * TM + i) * 32 + prow + 8 * t;
                    rres[g][i][t] = __builtin_amdgcn_raw_buffer_load_b128(
                        rrsrc, chan < a.Cout ? (int)(row * row_bytes + (size_t)chan * ES) : kOutOfRange, 0, 0);
                }
        }
    }
    store(0, xr[0], wr[0]);
    fetch(D, xr[0], wr[0]);
    for (int t0 = 0; t0 < nslices; t0 += U) {     // a last partial round runs on tiles of zeros
#pragma unroll
        for (int i = 0; i < U; ++i) {
            const int t = t0 + i;
            __syncthreads();                      // buffer t % 2 holds slice t; the other one is free
            store((i + 1) & 1, xr[(i + 1) % D], wr[(i + 1) % D]);
            fetch(t + 1 + D, xr[(i + 1) % D], wr[(i + 1) % D]);
            mma(i & 1);
        }
    }
    // ---- epilogue
    __syncthreads();                              // tiles are dead, LDS becomes staging space
    unsigned char *stg = smem + wv * (32 * STG_PITCH);
    unsigned char *yg = static_cast<unsigned char *>(a.y);

#pragma unroll
    for (int g = 0; g < TN / TG; ++g) {
        // folded batch-norm factors of this lane's channels in the accumulator layout
        f32x4 sc[TG][4], sh[TG][4];
#pragma unroll
        for (int u = 0; u < TG; ++u)
#pragma unroll
            for (int rb = 0; rb < 4; ++rb) {
                const int cl = (wn * TN + g * TG + u) * 32 + 8 * rb + 4 * half;   // channel within the tile
                sc[u][rb] = *reinterpret_cast<const f32x4 *>(&sbn[0][cl]);
                sh[u][rb] = *reinterpret_cast<const f32x4 *>(&sbn[1][cl]);
            }
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            wave_lds_fence();                     // earlier reads of the staging tile are done
#pragma unroll
            for (int u = 0; u < TG; ++u)
#pragma unroll
                for (int rb = 0; rb < 4; ++rb) {
                    const f32x16 &c = acc[i][g * TG + u];
                    f32x4 v;
                    v.x = c[4 * rb + 0] * sc[u][rb].x + sh[u][rb].x;
                    v.y = c[4 * rb + 1] * sc[u][rb].y + sh[u][rb].y;
                    v.z = c[4 * rb + 2] * sc[u][rb].z + sh[u][rb].z;
                    v.w = c[4 * rb + 3] * sc[u][rb].w + sh[u][rb].w;
                    *reinterpret_cast<f32x4 *>(stg + l32 * STG_PITCH + (u * 32 + 8 * rb + 4 * half) * 4) = v;
                }
            wave_lds_fence();
            const int chan = n0 + (wn * TN + g * TG) * 32 + cseg * CPL;
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const int pr = prow + 8 * t;
                const int m = m0 + (wm * TM + i) * 32 + pr;
                if (m >= a.M || chan >= a.Cout) continue;   // Cout is a multiple of CPL
                float v[CPL];
#pragma unroll
                for (int e = 0; e < CPL; e += 4) {
                    const f32x4 f = *reinterpret_cast<const f32x4 *>(stg + pr * STG_PITCH + (cseg * CPL + e) * 4);
                    v[e] = f.x; v[e + 1] = f.y; v[e + 2] = f.z; v[e + 3] = f.w;
                }
                size_t pixel = (size_t)m;
                if constexpr (SCATTER) {
                    const int n = m / PQ, pq = m - n * PQ;
                    const int p = pq / a.Q, q = pq - p * a.Q;
                    pixel = ((size_t)n * a.OH + (p * a.oy_s + a.oy_a)) * a.OW + (q * a.oy_s + a.oy_b);
                }
                const size_t off = (pixel * a.Cout + chan) * ES;
                if constexpr (SCATTER) {
                    if (a.res) {
                        const u32x4 rv = *reinterpret_cast<const u32x4 *>(static_cast<const unsigned char *>(a.res) + off);
                        if constexpr (BF16) {
                            v[0] += bf16_lo(rv.x); v[1] += bf16_hi(rv.x);
                            v[2] += bf16_lo(rv.y); v[3] += bf16_hi(rv.y);
                            v[4] += bf16_lo(rv.z); v[5] += bf16_hi(rv.z);
                            v[6] += bf16_lo(rv.w); v[7] += bf16_hi(rv.w);
                        } else {
                            v[0] += __uint_as_float(rv.x); v[1] += __uint_as_float(rv.y);
                            v[2] += __uint_as_float(rv.z); v[3] += __uint_as_float(rv.w);
                        }
                    }
                }
                if constexpr (HAS_RES) {
                    const u32x4 rv = rres[g][i][t];
                    if constexpr (BF16) {
                        v[0] += bf16_lo(rv.x); v[1] += bf16_hi(rv.x);
                        v[2] += bf16_lo(rv.y); v[3] += bf16_hi(rv.y);
                        v[4] += bf16_lo(rv.z); v[5] += bf16_hi(rv.z);
                        v[6] += bf16_lo(rv.w); v[7] += bf16_hi(rv.w);
                    } else {
                        v[0] += __uint_as_float(rv.x); v[1] += __uint_as_float(rv.y);
                        v[2] += __uint_as_float(rv.z); v[3] += __uint_as_float(rv.w);
                    }
                }
                if (a.relu == 1) {
#pragma unroll
                    for (int e = 0; e < CPL; ++e) v[e] = v[e] < 0.f ? 0.f : v[e];   // NaN stays NaN
                } else if (a.relu == 2) {
#pragma unroll
                    for (int e = 0; e < CPL; ++e) v[e] = gelu_erf(v[e]);
                }
                u32x4 o;
                if constexpr (BF16) {
                    o.x = pack_bf16(v[0], v[1]);
                    o.y = pack_bf16(v[2], v[3]);
                    o.z = pack_bf16(v[4], v[5]);
                    o.w = pack_bf16(v[6], v[7]);
                } else {
                    o.x = __float_as_uint(v[0]); o.y = __float_as_uint(v[1]);
                    o.z = __float_as_uint(v[2]); o.w = __float_as_uint(v[3]);
                }
                if (a.mask) {
                    const u32x4 mv = *reinterpret_cast<const u32x4 *>(static_cast<const unsigned char *>(a.mask) + off);
                    if constexpr (BF16) {
                        o.x = keep_where_positive_bf16(o.x, mv.x); o.y = keep_where_positive_bf16(o.y, mv.y);
                        o.z = keep_where_positive_bf16(o.z, mv.z); o.w = keep_where_positive_bf16(o.w, mv.w);
                    } else {
                        o.x = keep_where_positive_f32(o.x, mv.x); o.y = keep_where_positive_f32(o.y, mv.y);
                        o.z = keep_where_positive_f32(o.z, mv.z); o.w = keep_where_positive_f32(o.w, mv.w);
                    }
                }
                *reinterpret_cast<u32x4 *>(yg + off) = o;
            }
        }
    }
}

template <bool BF16, int BM, int BN, int WM, int WN>
static hipError_t launch(const ConvArgs &a, hipStream_t stream) {
    constexpr long long kMaxRowBytes = 0x7FFFFFFFLL / BM;   // residual offsets inside one tile
    if (a.res && (long long)a.Cout * (BF16 ? 2 : 4) > kMaxRowBytes) return hipErrorInvalidValue;
    const long long tiles_m = ((long long)a.M + BM - 1) / BM;
    const long long blocks = tiles_m * ((a.Cout + BN - 1) / BN);
    if (blocks <= 0 || blocks > 0x7FFFFFFFLL) return hipErrorInvalidValue;
    if (a.oy_s) conv_igemm_kernel<BF16, BM, BN, WM, WN, false, true><<<dim3((unsigned)blocks), dim3(kThreads), 0, stream>>>(a);
    else if (a.res) conv_igemm_kernel<BF16, BM, BN, WM, WN, true><<<dim3((unsigned)blocks), dim3(kThreads), 0, stream>>>(a);
    else conv_igemm_kernel<BF16, BM, BN, WM, WN, false><<<dim3((unsigned)blocks), dim3(kThreads), 0, stream>>>(a);
    return hipGetLastError();
}

// Channel tile: 128 when it divides Cout or wastes little, else 64.  Measured on MI355X,
// 128 pixels x 128 channels with 2 x 2 wavefronts (64 x 64 each) beats the wider tiles
// (256 x 128 and 128 x 256 with 8 wavefronts were level or slower on every ResNet-50 shape):
// two workgroups share a CU and cover each other's barriers.
static int conv_tile_n(const ConvArgs &a) {
    if (a.Cout % 128 == 0) return 128;
    if (a.Cout % 64 == 0) return 64;
    return a.Cout > 64 ? 128 : 64;
}

const char *conv_kernel_name(const ConvArgs &a) {
    if (conv1x1_stream_applies(a)) return "conv1x1_stream bf16";
    if (conv3x3_c64_applies(a)) return "conv3x3_c64 bf16 (persistent, nine taps resident in LDS)";
    if (conv3x3_halo_applies(a)) return "conv3x3_halo bf16 256x64 (4x1 waves)";
    if (gemm_nt_applies(a)) return gemm_nt_kernel_name(a);
    const int bn = conv_tile_n(a);
    if (a.bf16) return bn == 128 ? "conv_igemm bf16 128x128 (2x2 waves)" : "conv_igemm bf16 128x64 (4x1 waves)";
    return bn == 128 ? "conv_igemm f32 128x128 (2x2 waves)" : "conv_igemm f32 128x64 (4x1 waves)";
}

// Host-side shape check; the kernel assumes exactly this.
const char *conv_check(const ConvArgs &a) {
    const int kc = a.bf16 ? 64 : 32;
    if (a.N <= 0 || a.H <= 0 || a.W <= 0 || a.R <= 0 || a.S <= 0 || a.stride <= 0 || a.pad < 0)
        return "non-positive dimension";
    if (a.relu < 0 || a.relu > 2) return "unknown activation";
    // with more padding than half a window, input pixel indices would no longer grow with the
    // output pixel index, which the tiled kernel's tile-relative offsets rely on
    if (2 * a.pad > a.R - 1 || 2 * a.pad > a.S - 1) return "padding larger than half the window";
    if (a.Cin <= 0 || a.Cin % kc) return "Cin must be a multiple of 64 (bf16) or 32 (fp32)";
    if (a.Cout <= 0 || a.Cout % (a.bf16 ? 8 : 4)) return "Cout must be a multiple of 8 (bf16) or 4 (fp32)";
    if (a.P != (a.H + 2 * a.pad - a.R) / a.stride + 1 || a.Q != (a.W + 2 * a.pad - a.S) / a.stride + 1 ||
        a.P <= 0 || a.Q <= 0)
        return "inconsistent output size";
    if ((long long)a.N * a.P * a.Q != a.M || (long long)a.N * a.P * a.Q > 0x7FFFFFFFLL) return "bad M";
    if ((long long)a.N * a.H * a.W > 0x7FFFFFFFLL) return "input too large";
    {
        // 32-bit offsets of the tiled kernel: the weights as a whole, and the input pixels one
        // tile of 128 output pixels can touch, relative to the first of them (a loose bound:
        // the images the tile can reach into, plus two more for partial rows and the taps)
        const long long es = a.bf16 ? 2 : 4;
        if ((long long)a.Cout * a.R * a.S * a.Cin * es > 0x7FFFFFFFLL) return "weights exceed 2 GiB";
        const long long images = 127 / ((long long)a.P * a.Q) + 3;
        if (images * a.H * a.W * a.Cin * es + 256 > 0x7FFFFFFFLL) return "image too large for 32-bit tile offsets";
    }
    if (!a.x || !a.w || !a.y || !a.scale || !a.shift) return "null pointer";
    if (((uintptr_t)a.x | (uintptr_t)a.w | (uintptr_t)a.y | (uintptr_t)a.res | (uintptr_t)a.mask | (uintptr_t)a.scale |
         (uintptr_t)a.shift) & 15)
        return "pointers must be 16-byte aligned";
    return nullptr;
}

// The scattered form: stride 1, no padding, windows of at most 2 x 2 starting AT the output pixel
// (a tap past the input's last row or column reads zeros), P <= H and Q <= W given by the caller.
const char *conv_scatter_check(const ConvArgs &a) {
    const int kc = a.bf16 ? 64 : 32;
    if (a.N <= 0 || a.H <= 0 || a.W <= 0 || a.R < 1 || a.R > 2 || a.S < 1 || a.S > 2 || a.stride != 1 || a.pad != 0)
        return "scattered form: windows of 1 or 2, stride 1, no padding";
    if (a.relu) return "scattered form: no activation";
    if (a.Cin <= 0 || a.Cin % kc) return "Cin must be a multiple of 64 (bf16) or 32 (fp32)";
    if (a.Cout <= 0 || a.Cout % (a.bf16 ? 8 : 4)) return "Cout must be a multiple of 8 (bf16) or 4 (fp32)";
    if (a.P <= 0 || a.Q <= 0 || a.P > a.H || a.Q > a.W) return "output size must be within the input's";
    if ((long long)a.N * a.P * a.Q != a.M || (long long)a.N * a.P * a.Q > 0x7FFFFFFFLL) return "bad M";
    if (a.oy_s <= 0 || a.oy_a < 0 || a.oy_b < 0 || a.oy_a >= a.oy_s || a.oy_b >= a.oy_s ||
        (a.P - 1) * a.oy_s + a.oy_a >= a.OH || (a.Q - 1) * a.oy_s + a.oy_b >= a.OW)
        return "scattered output pixels leave the output tensor";
    if (a.w_step <= 0 || a.w_r0 < 0 || a.w_s0 < 0 || a.w_r0 + (a.R - 1) * a.w_step >= a.wR ||
        a.w_s0 + (a.S - 1) * a.w_step >= a.wS)
        return "taps leave the weight tensor";
    const long long es = a.bf16 ? 2 : 4;
    if ((long long)a.N * a.H * a.W > 0x7FFFFFFFLL || (long long)a.N * a.OH * a.OW > 0x7FFFFFFFLL) return "tensor too large";
    if ((long long)a.Cout * a.wR * a.wS * a.Cin * es > 0x7FFFFFFFLL) return "weights exceed 2 GiB";
    const long long images = 127 / ((long long)a.P * a.Q) + 3;
    if (images * a.H * a.W * a.Cin * es + 256 > 0x7FFFFFFFLL) return "image too large for 32-bit tile offsets";
    if (!a.x || !a.w || !a.y || !a.scale || !a.shift) return "null pointer";
    if (((uintptr_t)a.x | (uintptr_t)a.w | (uintptr_t)a.y | (uintptr_t)a.res | (uintptr_t)a.mask | (uintptr_t)a.scale |
         (uintptr_t)a.shift) & 15)
        return "pointers must be 16-byte aligned";
    return nullptr;
}

hipError_t launch_conv_scatter(const ConvArgs &a, hipStream_t stream) {
    if (conv_scatter_check(a)) return hipErrorInvalidValue;
    const int bn = conv_tile_n(a);
    if (a.bf16) {
        if (bn == 128) return launch<true, 128, 128, 2, 2>(a, stream);
        return launch<true, 128, 64, 4, 1>(a, stream);
    }
    if (bn == 128) return launch<false, 128, 128, 2, 2>(a, stream);
    return launch<false, 128, 64, 4, 1>(a, stream);
}

hipError_t launch_conv(const ConvArgs &a, hipStream_t stream) {
    if (conv_check(a) || a.oy_s) return hipErrorInvalidValue;
    if (conv1x1_stream_applies(a)) return launch_conv1x1_stream(a, stream);
    if (conv3x3_c64_applies(a)) return launch_conv3x3_c64(a, stream);
    if (conv3x3_halo_applies(a)) return launch_conv3x3_halo(a, stream);
    if (gemm_nt_applies(a)) return launch_gemm_nt(a, stream);
    const int bn = conv_tile_n(a);
    if (a.bf16) {
        if (bn == 128) return launch<true, 128, 128, 2, 2>(a, stream);
        return launch<true, 128, 64, 4, 1>(a, stream);
    }
    if (bn == 128) return launch<false, 128, 128, 2, 2>(a, stream);
    return launch<false, 128, 64, 4, 1>(a, stream);
}

// ---------------------------------------------------------------- small helpers

__global__ void bn_fold_kernel(const float *gamma, const float *beta, const float *mean,
                               const float *var, float eps, unsigned C, float *scale, float *shift) {
    const unsigned c = blockIdx.x * blockDim.x + threadIdx.x;
    if (c < C) {
        const float s = gamma[c] / sqrtf(var[c] + eps);
        scale[c] = s;
        shift[c] = beta[c] - mean[c] * s;
    }
}

hipError_t launch_bn_fold(const float *gamma, const float *beta, const float *mean, const float *var,
                          float eps, unsigned C, float *scale, float *shift, hipStream_t stream) {
    if (C == 0) return hipSuccess;
    bn_fold_kernel<<<dim3((C + 255) / 256), dim3(256), 0, stream>>>(gamma, beta, mean, var, eps, C, scale, shift);
    return hipGetLastError();
}

// Plain copy, 16 bytes per lane, grid-stride: the HBM roofline probe.
__global__ __launch_bounds__(256) void copy_kernel(const uint4 *__restrict__ src, uint4 *__restrict__ dst, size_t n16) {
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

hipError_t launch_copy(const void *src, void *dst, size_t bytes, hipStream_t stream) {
    const size_t n16 = bytes / 16;
    if (n16 == 0) return hipSuccess;
    size_t blocks = (n16 + 255) / 256;
    if (blocks > 256 * 32) blocks = 256 * 32;
    copy_kernel<<<dim3((unsigned)blocks), dim3(256), 0, stream>>>(static_cast<const uint4 *>(src),
                                                                 static_cast<uint4 *>(dst), n16);
    return hipGetLastError();
}

// Register-resident MFMA loop: the matrix-core roofline probe (bf16, 32x32x16).
__global__ __launch_bounds__(256) void mfma_probe_kernel(float *out, int iters) {
    bf16x8 a, b;
#pragma unroll
    for (int e = 0; e < 8; ++e) { a[e] = (__bf16)(float)(threadIdx.x % 3); b[e] = (__bf16)1.0f; }
    f32x16 c0 = {0}, c1 = {0}, c2 = {0}, c3 = {0};
    for (int i = 0; i < iters; ++i) {
        c0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c0, 0, 0, 0);
        c1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c1, 0, 0, 0);
        c2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c2, 0, 0, 0);
        c3 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c3, 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int e = 0; e < 16; ++e) s += c0[e] + c1[e] + c2[e] + c3[e];
    if (s == -1.f) out[0] = s;                   // never true; keeps the loop alive
}

hipError_t launch_mfma_probe(float *out, int iters, int blocks, hipStream_t stream) {
    mfma_probe_kernel<<<dim3(blocks), dim3(256), 0, stream>>>(out, iters);
    return hipGetLastError();
}

}  // namespace delta
