// 3x3, stride 1, pad 1 bf16 layer kernel that keeps the input halo of a pixel tile in LDS.
//
// Same operator as conv_igemm.hip, y = relu?(scale_k * conv(x, w) + shift_k (+ res)): the layer
// that DELTA's Recompute action re-runs (Sec. 3, Table 1), specialised for the 3x3 convolution in
// the middle of every ResNet bottleneck.  The nine taps of an output pixel read nine neighbouring
// input pixels, so a tile of BM consecutive pixels (NHW order) touches only BM + 2W + 2 consecutive
// input rows.  The generic kernel gathers those rows nine times from L2; this one stages them once
// per block of 64 input channels and lets the MFMA operand reads walk the taps inside LDS.  What
// still streams from L2 at every step is the BN x 64 weight tile of one tap.
//
// Layout: output channels on the MFMA row axis, pixels on the column axis, lane half h owns bytes
// [64h, 64h+64) of every 128-byte row for both operands (as in conv_igemm.hip).  A workgroup is
// (BM/64) x (BN/64) wavefronts of 64 pixels x 64 channels; 256 x 64 measured best on MI355X for
// every ResNet-50 shape (two workgroups share a CU).
// Pipeline: one step = one tap of one channel block = 16 MFMAs per wavefront and one barrier.
// Weight tiles are requested D = 4 steps ahead into a register ring and move to one of two LDS
// buffers a step before use; the halo of the next channel block is requested at tap 0 and stored
// after tap 8.  The operand pieces of a 16-wide step are read into one of two register sets while
// the other set's MFMAs issue; the barrier of a step stands before its last 16-wide step, so the
// first pieces of the next step are read under the last MFMAs of this one.  Taps outside the image are redirected to a row of zeros in LDS, so no
// operand needs masking.  The step order is fixed, so the first forward and every recomputation
// add in the same order and a recomputed tensor is bit-identical to the original.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kernels.hpp"

namespace delta {
namespace halo {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

static constexpr int kStgPitch = 64 * 4 + 16;

__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
    const f32x2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}
__device__ __forceinline__ float bf16_lo(uint32_t p) { return __uint_as_float(p << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t p) { return __uint_as_float(p & 0xFFFF0000u); }

__device__ __forceinline__ void wave_lds_fence() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

template <int BM, int BN, int HL>
__global__ __launch_bounds__((BM / 64) * (BN / 64) * 64) void conv3x3_halo_kernel(ConvArgs a, int HR) {
    constexpr int TP = 2;                         // 32-pixel tiles per wavefront (and 2 channel tiles)
    constexpr int KB = 128;                       // bytes of input channels per step (64 bf16)
    constexpr int WM = BM / (32 * TP), WN = BN / 64, NW = WM * WN, NT = NW * 64;
    constexpr int SEGS = KB / 16;                 // 16-byte segments per row (KB bytes of channels per step)
    constexpr int kPitch = KB + 16;               // 4 banks between rows: conflict-free ds_read_b128
    constexpr int WL = BN * SEGS / NT;            // 16-byte weight loads per thread and tap
    constexpr int WBUF = BN * kPitch;
    static_assert(BN * SEGS % NT == 0, "weight tile must divide over the threads");

    extern __shared__ __align__(16) unsigned char smem[];
    unsigned char *wbuf0 = smem;
    unsigned char *wbuf1 = smem + WBUF;
    unsigned char *hs = smem + 2 * WBUF;          // HR halo rows, then one row of zeros

    const int tid = threadIdx.x;
    const int lane = tid & 63, wv = tid >> 6;
    const int wm = wv % WM, wn = wv / WM;
    const int l32 = lane & 31, half = lane >> 5;

    unsigned logical;
    {
        const unsigned nb = gridDim.x, per = nb >> 3, rem = nb & 7u;
        const unsigned xcd = blockIdx.x & 7u, idx = blockIdx.x >> 3;
        logical = xcd < rem ? xcd * (per + 1) + idx : rem * (per + 1) + (xcd - rem) * per + idx;
    }
    const int tiles_n = a.Cout / BN;
    const int m0 = (int)(logical / tiles_n) * BM;
    const int n0 = (int)(logical % tiles_n) * BN;

    const unsigned char *xg = static_cast<const unsigned char *>(a.x);
    const unsigned char *wg = static_cast<const unsigned char *>(a.w);
    const int W = a.W, HW = a.H * a.W;
    const int CB = a.Cin * 2 / KB;                // channel blocks of KB bytes
    const int T = 9 * CB;                         // steps
    const uint32_t cin_bytes = (uint32_t)a.Cin * 2u;

    // ---- halo rows of this thread: chunk c covers row (tid + c NT) / 8, segment (tid + c NT) % 8
    uint32_t hoff[HL];                            // byte offset of the row's channel block 0 in x, or ~0u
#pragma unroll
    for (int c = 0; c < HL; ++c) {
        const int idx = tid + c * NT, row = idx / SEGS, seg = idx % SEGS;
        const long long q = (long long)m0 - (W + 1) + row;
        hoff[c] = (row < HR && q >= 0 && q < a.M) ? (uint32_t)q * cin_bytes + seg * 16u : 0xFFFFFFFFu;
    }
    // ---- weight rows of this thread
    uint32_t woff[WL];
#pragma unroll
    for (int j = 0; j < WL; ++j) {
        const int idx = tid + j * NT, krow = idx / SEGS, seg = idx % SEGS;
        woff[j] = (uint32_t)(n0 + krow) * 9u * cin_bytes + seg * 16u;
    }
    // ---- operand rows of this lane: two pixel columns, nine validity bits each
    int prow[TP];
    uint32_t valid[TP];
#pragma unroll
    for (int j = 0; j < TP; ++j) {
        const int i = wm * (32 * TP) + 32 * j + l32, m = m0 + i;
        prow[j] = i;
        uint32_t v = 0;
        if (m < a.M) {
            const int hw = m % HW, h = hw / W, w_ = hw - h * W;
#pragma unroll
            for (int r = 0; r < 3; ++r)
#pragma unroll
                for (int s = 0; s < 3; ++s)
                    if ((unsigned)(h + r - 1) < (unsigned)a.H && (unsigned)(w_ + s - 1) < (unsigned)W)
                        v |= 1u << (r * 3 + s);
        }
        valid[j] = v;
    }

    constexpr int D = 4;                          // weight tiles in flight
    constexpr int HALO_TAP = 0;                   // tap at which the next halo is requested
    static_assert(D % 2 == 0, "D must be even");
    u32x4 rh[HL], rw[D][WL];

    auto load_halo = [&](int cb) {
#pragma unroll
        for (int c = 0; c < HL; ++c)
            rh[c] = hoff[c] != 0xFFFFFFFFu
                        ? *reinterpret_cast<const u32x4 *>(xg + (size_t)hoff[c] + (size_t)cb * KB)
                        : u32x4{0u, 0u, 0u, 0u};
    };
    auto store_halo = [&]() {
#pragma unroll
        for (int c = 0; c < HL; ++c) {
            const int idx = tid + c * NT, row = idx / SEGS, seg = idx % SEGS;
            if (row < HR) *reinterpret_cast<u32x4 *>(hs + row * kPitch + seg * 16) = rh[c];
        }
    };
    auto load_w = [&](int t, u32x4 (&rw)[WL]) {
        const int cb = t / 9, tap = t - cb * 9;
        const uint32_t add = (uint32_t)tap * cin_bytes + (uint32_t)cb * KB;
#pragma unroll
        for (int j = 0; j < WL; ++j) rw[j] = *reinterpret_cast<const u32x4 *>(wg + (size_t)(woff[j] + add));
    };
    auto store_w = [&](unsigned char *wb, const u32x4 (&rw)[WL]) {
#pragma unroll
        for (int j = 0; j < WL; ++j) {
            const int idx = tid + j * NT, krow = idx / SEGS, seg = idx % SEGS;
            *reinterpret_cast<u32x4 *>(wb + krow * kPitch + seg * 16) = rw[j];
        }
    };

    f32x16 acc[TP][2];                            // [pixel tile][channel tile]
#pragma unroll
    for (int i = 0; i < TP; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    // Operand pieces.  `point` fixes the rows of a step (tap) in weight buffer wb; `read_pieces`
    // reads the pieces of its 16-wide step q into register set f; `mfmas` multiplies set f.
    const unsigned char *xp[TP], *wp;
    auto point = [&](const unsigned char *wb, int tap) {
        const int r = tap / 3, s = tap - 3 * r;
        const int shift_rows = r * W + s;
#pragma unroll
        for (int j = 0; j < TP; ++j) {
            const int row = ((valid[j] >> tap) & 1u) ? prow[j] + shift_rows : HR;
            xp[j] = hs + row * kPitch + half * (KB / 2);
        }
        wp = wb + (wn * 64 + l32) * kPitch + half * (KB / 2);
    };
    u32x4 wf[2][2], xf[2][TP];
    auto read_pieces = [&](int q, int f) {
#pragma unroll
        for (int c = 0; c < 2; ++c) wf[f][c] = *reinterpret_cast<const u32x4 *>(wp + c * 32 * kPitch + q * 16);
#pragma unroll
        for (int j = 0; j < TP; ++j) xf[f][j] = *reinterpret_cast<const u32x4 *>(xp[j] + q * 16);
    };
    auto mfmas = [&](int f) {
#pragma unroll
        for (int j = 0; j < TP; ++j)
#pragma unroll
            for (int c = 0; c < 2; ++c)
                acc[j][c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                    __builtin_bit_cast(bf16x8, wf[f][c]), __builtin_bit_cast(bf16x8, xf[f][j]), acc[j][c], 0, 0, 0);
    };
    auto interleave = [&]() {                     // one LDS read, one MFMA, ... (2-3 % on 28x28 and 7x7 images, 1 % slower on 14x14)
#pragma unroll
        for (int k = 0; k < 2 + TP; ++k) {
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x008, (2 * TP) / (2 + TP), 0);
        }
    };

    // ---- prologue: the weights of steps 0 and 1 to LDS, those of steps 2 .. D + 1 in flight in
    // registers (rw[i] holds the tile of a step t with t % D == i)
    if (tid < SEGS + 1) *reinterpret_cast<u32x4 *>(hs + HR * kPitch + tid * 16) = u32x4{0u, 0u, 0u, 0u};
    load_halo(0);
    load_w(0, rw[0]);
    if (1 < T) load_w(1, rw[1]);
    store_halo();
    store_w(wbuf0, rw[0]);
    if (1 < T) store_w(wbuf1, rw[1]);
#pragma unroll
    for (int i = 2; i < D + 2; ++i)
        if (i < T) load_w(i, rw[i % D]);
    __syncthreads();
    point(wbuf0, 0);
    read_pieces(0, 0);

    // Step t multiplies out of buffer t % 2.  Its barrier stands before its last 16-wide step, when every
    // wavefront holds that step's pieces in registers: from there on buffer t % 2 takes the weights of
    // step t + 2, and the first pieces of step t + 1 (stored a step earlier) are read under the last MFMAs.
    int tap = 0, cb = 0;
    for (int t0 = 0; t0 < T; t0 += D) {
#pragma unroll
        for (int i = 0; i < D; ++i) {
            const int t = t0 + i;
            if (t < T) {
                unsigned char *cur = (i & 1) ? wbuf1 : wbuf0;   // D is even: t % 2 == i % 2
                unsigned char *nxt = (i & 1) ? wbuf0 : wbuf1;
                const bool more = cb + 1 < CB;
                if (tap == HALO_TAP && more) load_halo(cb + 1);
                read_pieces(1, 1);
                mfmas(0);
                interleave();
                read_pieces(2, 0);
                mfmas(1);
                interleave();
                read_pieces(3, 1);
                mfmas(0);
                interleave();
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                __syncthreads();
                if (t + 2 < T) store_w(cur, rw[(i + 2) % D]);
                if (t + 2 + D < T) load_w(t + 2 + D, rw[(i + 2) % D]);
                if (tap == 8) {
                    if (more) {
                        store_halo();
                        __syncthreads();
                    }
                    tap = 0;
                    ++cb;
                } else {
                    ++tap;
                }
                if (t + 1 < T) {
                    point(nxt, tap);
                    read_pieces(0, 0);
                }
                mfmas(1);
            }
        }
    }

    // ---- epilogue: row-major through a wavefront-private fp32 tile, scale/shift, residual + ReLU
    // (+ mask), one rounding, 128 contiguous bytes per pixel.  The residual and mask rows are
    // requested before the barrier, so that their latency overlaps it and the transposition.
    unsigned char *yg = static_cast<unsigned char *>(a.y);
    const unsigned char *rg = static_cast<const unsigned char *>(a.res);
    const unsigned char *mg = static_cast<const unsigned char *>(a.mask);
    const int pr8 = lane >> 3, cseg = lane & 7;
    const int chan = n0 + wn * 64 + cseg * 8;
    u32x4 rres[TP][4], rmsk[TP][4];
#pragma unroll
    for (int i = 0; i < TP; ++i)
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const int m = m0 + wm * (32 * TP) + i * 32 + pr8 + 8 * t;
            const size_t off = ((size_t)(m < a.M ? m : 0) * a.Cout + chan) * 2;
            rres[i][t] = rg ? *reinterpret_cast<const u32x4 *>(rg + off) : u32x4{0u, 0u, 0u, 0u};
            rmsk[i][t] = mg ? *reinterpret_cast<const u32x4 *>(mg + off) : u32x4{0u, 0u, 0u, 0u};
        }
    float sc[8], sh[8];                             // this lane's 8 channels in the row-major phase
    {
        const f32x4 s0 = *reinterpret_cast<const f32x4 *>(a.scale + chan), s1 = *reinterpret_cast<const f32x4 *>(a.scale + chan + 4);
        const f32x4 h0 = *reinterpret_cast<const f32x4 *>(a.shift + chan), h1 = *reinterpret_cast<const f32x4 *>(a.shift + chan + 4);
        sc[0] = s0.x; sc[1] = s0.y; sc[2] = s0.z; sc[3] = s0.w; sc[4] = s1.x; sc[5] = s1.y; sc[6] = s1.z; sc[7] = s1.w;
        sh[0] = h0.x; sh[1] = h0.y; sh[2] = h0.z; sh[3] = h0.w; sh[4] = h1.x; sh[5] = h1.y; sh[6] = h1.z; sh[7] = h1.w;
    }
    __syncthreads();
    unsigned char *stg = smem + wv * (32 * kStgPitch);
#pragma unroll
    for (int i = 0; i < TP; ++i) {
        wave_lds_fence();
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
            for (int rb = 0; rb < 4; ++rb) {
                const f32x16 &c = acc[i][u];
                const f32x4 v = {c[4 * rb + 0], c[4 * rb + 1], c[4 * rb + 2], c[4 * rb + 3]};
                *reinterpret_cast<f32x4 *>(stg + l32 * kStgPitch + (u * 32 + 8 * rb + 4 * half) * 4) = v;
            }
        wave_lds_fence();
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const int pr = pr8 + 8 * t;
            const int m = m0 + wm * (32 * TP) + i * 32 + pr;
            if (m >= a.M) continue;
            const f32x4 f0 = *reinterpret_cast<const f32x4 *>(stg + pr * kStgPitch + cseg * 32);
            const f32x4 f1 = *reinterpret_cast<const f32x4 *>(stg + pr * kStgPitch + cseg * 32 + 16);
            float v[8] = {f0.x, f0.y, f0.z, f0.w, f1.x, f1.y, f1.z, f1.w};
#pragma unroll
            for (int e = 0; e < 8; ++e) v[e] = v[e] * sc[e] + sh[e];
            const size_t off = ((size_t)m * a.Cout + chan) * 2;
            if (rg) {
                const u32x4 rv = rres[i][t];
                v[0] += bf16_lo(rv.x); v[1] += bf16_hi(rv.x);
                v[2] += bf16_lo(rv.y); v[3] += bf16_hi(rv.y);
                v[4] += bf16_lo(rv.z); v[5] += bf16_hi(rv.z);
                v[6] += bf16_lo(rv.w); v[7] += bf16_hi(rv.w);
            }
            if (a.relu) {
#pragma unroll
                for (int e = 0; e < 8; ++e) v[e] = v[e] < 0.f ? 0.f : v[e];
            }
            u32x4 o;
            o.x = pack_bf16(v[0], v[1]);
            o.y = pack_bf16(v[2], v[3]);
            o.z = pack_bf16(v[4], v[5]);
            o.w = pack_bf16(v[6], v[7]);
            if (mg) {
                const u32x4 mv = rmsk[i][t];
                o.x = keep_where_positive_bf16(o.x, mv.x); o.y = keep_where_positive_bf16(o.y, mv.y);
                o.z = keep_where_positive_bf16(o.z, mv.z); o.w = keep_where_positive_bf16(o.w, mv.w);
            }
            *reinterpret_cast<u32x4 *>(yg + off) = o;
        }
    }
}

static constexpr int kBM = 256, kBN = 64;       // 4 wavefronts of 64 pixels x 64 channels
static constexpr int kNT = (kBM / 64) * (kBN / 64) * 64;
static constexpr int kMaxW = 127;                // halo rows per thread stay within 16 loads
static constexpr size_t kMaxLds = 160 * 1024;

static int halo_rows(const ConvArgs &a) { return kBM + 2 * a.W + 2; }

static size_t smem_bytes(int HR) {
    const size_t tiles = 2 * (size_t)kBN * 144 + (size_t)(HR + 1) * 144;
    const size_t stg = (size_t)(kNT / 64) * 32 * kStgPitch;
    return tiles > stg ? tiles : stg;
}

template <int HL>
static hipError_t launch_one(const ConvArgs &a, int HR, hipStream_t stream) {
    const size_t smem = smem_bytes(HR);
    static bool raised = false;                   // per instantiation
    if (!raised) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&conv3x3_halo_kernel<kBM, kBN, HL>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)kMaxLds);
        if (e != hipSuccess) return e;
        raised = true;
    }
    const long long blocks = (((long long)a.M + kBM - 1) / kBM) * (a.Cout / kBN);
    if (blocks <= 0 || blocks > 0x7FFFFFFFLL || smem > kMaxLds) return hipErrorInvalidValue;
    conv3x3_halo_kernel<kBM, kBN, HL><<<dim3((unsigned)blocks), dim3(kNT), smem, stream>>>(a, HR);
    return hipGetLastError();
}

}  // namespace halo

// bf16, 3x3, stride 1, pad 1, channel counts in whole 64-blocks, and offsets that fit 32 bits.
// conv_check() must have passed; everything the kernel assumes beyond it is tested here.
bool conv3x3_halo_applies(const ConvArgs &a) {
    if (!a.bf16 || a.R != 3 || a.S != 3 || a.stride != 1 || a.pad != 1) return false;
    if (a.Cin % 64 || a.Cout % 64 || a.W > halo::kMaxW) return false;
    if (a.P != a.H || a.Q != a.W) return false;
    if ((unsigned long long)a.M * a.Cin * 2ull >= 0xFFFFFFFFull) return false;        // x offsets
    if ((unsigned long long)a.Cout * 9ull * a.Cin * 2ull >= 0xFFFFFFFFull) return false;  // w offsets
    return halo::smem_bytes(halo::halo_rows(a)) <= halo::kMaxLds;
}

hipError_t launch_conv3x3_halo(const ConvArgs &a, hipStream_t stream) {
    if (conv_check(a) || !conv3x3_halo_applies(a)) return hipErrorInvalidValue;
    const int HR = halo::halo_rows(a);
    const int hl = (HR * 8 + halo::kNT - 1) / halo::kNT;      // 16-byte halo loads per thread
    if (hl <= 12) return halo::launch_one<12>(a, HR, stream);
    if (hl <= 16) return halo::launch_one<16>(a, HR, stream);
    return hipErrorInvalidValue;
}

}  // namespace delta
