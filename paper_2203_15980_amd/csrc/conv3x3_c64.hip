// 3x3, stride 1, pad 1, 64 -> 64 channels, bf16: the middle layer of conv2_x's bottlenecks (and its data
// gradient), y = relu?(scale_k * conv(x, w) + shift_k (+ res)) (* [mask > 0]).
//
// With 64 channels in and out all nine taps of the weights are 72 KB: they stay in LDS for the whole
// launch.  A workgroup of 16 wavefronts is persistent: it stages the weights once and then walks tiles of
// BM consecutive pixels (NHW order).  Per tile the BM + 2W + 2 input rows the nine taps touch are staged
// once (rows of 128 bytes, pitch 144; they were requested from memory while the previous tile was being
// multiplied), then every wavefront multiplies 32 pixels x 64 channels out of LDS - 72 MFMAs without a
// barrier in between; taps outside the image are redirected to a row of zeros - and stores its pixels
// itself.  Two barriers per tile, none per tap; the general halo kernel (conv3x3_halo.hip) re-stages a
// 64 x 64 weight tile from L2 and meets at a barrier for every tap.
// Orientation as in the other kernels: output channels on the MFMA row axis, pixels on the column axis,
// lane half h owns bytes [64h, 64h + 64) of every 128-byte row of both operands.  Fixed summation order
// (taps in order, 16 channels per MFMA step), so forward and recomputation give the same bits.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kernels.hpp"

namespace delta {
namespace c64 {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

static constexpr int kWaves = 16, kThreads = kWaves * 64;
static constexpr int kC = 64;
static constexpr int kPitch = 144;
static constexpr int kMaxRows = 512;                      // staged input rows per tile (4 pieces of 16 bytes per thread)
static constexpr int kTap = kC * kPitch;                  // 9216 bytes
static constexpr int kRA = (kMaxRows + 1) * kPitch;       // input rows + the row of zeros
static constexpr int kRW = 9 * kTap;
static constexpr int kRF = 2 * kC * 4;
static constexpr int kLds = kRA + kRW + kRF;
static_assert(kLds <= 160 * 1024, "LDS budget of a CU");

__device__ __forceinline__ uint32_t pack2(float lo, float hi) {
    const f32x2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}
__device__ __forceinline__ float lo16(uint32_t p) { return __uint_as_float(p << 16); }
__device__ __forceinline__ float hi16(uint32_t p) { return __uint_as_float(p & 0xFFFF0000u); }

// BM pixels per tile, HR = BM + 2W + 2 staged rows (<= 512), NT = ceil(BM / 32) <= 16 wavefronts with pixels.
template <bool HAS_RES, bool HAS_MASK>
__global__ __launch_bounds__(kThreads) void conv3x3_c64_kernel(ConvArgs a, int BM, int HR, int NT, int ntiles) {
    extern __shared__ __align__(16) unsigned char lds[];
    unsigned char *ra = lds;
    unsigned char *rw = lds + kRA;
    float *fs = reinterpret_cast<float *>(rw + kRW), *fh = fs + kC;

    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int l32 = lane & 31, half = lane >> 5;
    const int W = a.W, HW = a.H * a.W, M = a.M;
    const unsigned char *xg = static_cast<const unsigned char *>(a.x);
    // Tiles are dealt so that each of the 8 XCDs (consecutive workgroups go to consecutive XCDs) works on a
    // contiguous run of them per round: neighbouring tiles share 2W + 2 input rows through that XCD's L2.
    const unsigned nb = gridDim.x, per = nb >> 3, rem = nb & 7u;
    const unsigned xcd = blockIdx.x & 7u, idx = blockIdx.x >> 3;
    const unsigned logical = xcd < rem ? xcd * (per + 1) + idx : rem * (per + 1) + (xcd - rem) * per + idx;

    u32x4 hreg[4];
    auto fetch = [&](int tile) {                                 // input rows of `tile` into registers
        const long long q0 = (long long)tile * BM - (W + 1);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int c = tid + j * kThreads, row = c >> 3, seg = c & 7;
            const long long q = q0 + row;
            hreg[j] = (row < HR && q >= 0 && q < M) ? *reinterpret_cast<const u32x4 *>(xg + (size_t)q * (kC * 2) + seg * 16)
                                                     : u32x4{0u, 0u, 0u, 0u};
        }
    };
    int tile = (int)logical;
    if (tile < ntiles) fetch(tile);

    // ---- once per workgroup: all nine taps, the batch-norm factors, the row of zeros
    {
        const unsigned char *wg = static_cast<const unsigned char *>(a.w);
        for (int c = tid; c < 9 * kC * 8; c += kThreads) {       // (tap, k, seg)
            const int tap = c / (kC * 8), rest = c - tap * (kC * 8), k = rest >> 3, seg = rest & 7;
            *reinterpret_cast<u32x4 *>(rw + tap * kTap + k * kPitch + seg * 16) =
                *reinterpret_cast<const u32x4 *>(wg + ((size_t)(k * 9 + tap) * 8 + seg) * 16);
        }
        if (tid < kC) { fs[tid] = a.scale[tid]; fh[tid] = a.shift[tid]; }
        if (tid < 9) *reinterpret_cast<u32x4 *>(ra + kMaxRows * kPitch + tid * 16) = u32x4{0u, 0u, 0u, 0u};
    }
    const int relu = a.relu;
    unsigned char *yg = static_cast<unsigned char *>(a.y);
    const unsigned char *rg = static_cast<const unsigned char *>(a.res);
    const unsigned char *mg = static_cast<const unsigned char *>(a.mask);

    for (; tile < ntiles; tile += (int)nb) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int c = tid + j * kThreads, row = c >> 3, seg = c & 7;
            if (row < HR) *reinterpret_cast<u32x4 *>(ra + row * kPitch + seg * 16) = hreg[j];
        }
        __syncthreads();                                         // the tile's rows (and, the first time, the weights) are in place
        if (tile + (int)nb < ntiles) fetch(tile + (int)nb);      // the next tile travels while this one is multiplied
        if (wv < NT) {
            const long long m0 = (long long)tile * BM;
            const int pi = wv * 32 + l32;
            const long long pm = m0 + pi;
            const bool mine = pi < BM && pm < M;
            uint32_t valid = 0;
            if (mine) {
                const int hw = (int)(pm % HW), h = hw / W, w_ = hw - h * W;
#pragma unroll
                for (int r = 0; r < 3; ++r)
#pragma unroll
                    for (int s = 0; s < 3; ++s)
                        if ((unsigned)(h + r - 1) < (unsigned)a.H && (unsigned)(w_ + s - 1) < (unsigned)W) valid |= 1u << (r * 3 + s);
            }
            // residual and mask pieces in the layout the lane ends up holding: channels 32 u + 16 i2 + 8 half .. + 8
            const size_t orow = (size_t)(mine ? pm : 0) * (kC * 2);
            u32x4 rres[2][2], rmsk[2][2];
#pragma unroll
            for (int u = 0; u < 2; ++u)
#pragma unroll
                for (int i2 = 0; i2 < 2; ++i2) {
                    const size_t off = orow + (size_t)(u * 32 + 16 * i2 + 8 * half) * 2;
                    if constexpr (HAS_RES) rres[u][i2] = *reinterpret_cast<const u32x4 *>(rg + off);
                    if constexpr (HAS_MASK) rmsk[u][i2] = *reinterpret_cast<const u32x4 *>(mg + off);
                }
            f32x16 acc[2];
#pragma unroll
            for (int u = 0; u < 2; ++u)
#pragma unroll
                for (int e = 0; e < 16; ++e) acc[u][e] = 0.f;
            // 36 steps (tap, 16-byte piece q); the three operand pieces of step st + 1 are read while
            // step st's two MFMAs issue
            u32x4 xv[2], w0[2], w1[2];
            auto read_step = [&](int st, int f) {
                const int tap = st >> 2, q = st & 3;
                const int r = tap / 3, s = tap - 3 * r;
                const int row = ((valid >> tap) & 1u) ? pi + r * W + s : kMaxRows;
                const unsigned char *xp = ra + row * kPitch + half * 64;
                const unsigned char *wp = rw + tap * kTap + l32 * kPitch + half * 64;
                xv[f] = *reinterpret_cast<const u32x4 *>(xp + q * 16);
                w0[f] = *reinterpret_cast<const u32x4 *>(wp + q * 16);
                w1[f] = *reinterpret_cast<const u32x4 *>(wp + 32 * kPitch + q * 16);
            };
            read_step(0, 0);
#pragma unroll
            for (int st = 0; st < 36; ++st) {
                if (st + 1 < 36) read_step(st + 1, (st + 1) & 1);
                acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, w0[st & 1]),
                                                                 __builtin_bit_cast(bf16x8, xv[st & 1]), acc[0], 0, 0, 0);
                acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, w1[st & 1]),
                                                                 __builtin_bit_cast(bf16x8, xv[st & 1]), acc[1], 0, 0, 0);
                if (st + 1 < 36) {
                    __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                    __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                }
            }
            // ---- epilogue: scale/shift, lanes l and l + 32 swap so that each holds 8 consecutive channels,
            // residual, ReLU, one rounding, mask; each lane stores its four 16-byte pieces itself
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                float v[16];
#pragma unroll
                for (int rb = 0; rb < 4; ++rb) {
                    const f32x4 sc = *reinterpret_cast<const f32x4 *>(fs + u * 32 + 8 * rb + 4 * half);
                    const f32x4 sh = *reinterpret_cast<const f32x4 *>(fh + u * 32 + 8 * rb + 4 * half);
                    v[4 * rb + 0] = acc[u][4 * rb + 0] * sc.x + sh.x;
                    v[4 * rb + 1] = acc[u][4 * rb + 1] * sc.y + sh.y;
                    v[4 * rb + 2] = acc[u][4 * rb + 2] * sc.z + sh.z;
                    v[4 * rb + 3] = acc[u][4 * rb + 3] * sc.w + sh.w;
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
                    if constexpr (HAS_RES) {
                        const u32x4 r4 = rres[u][i2];
                        o[0] += lo16(r4.x); o[1] += hi16(r4.x); o[2] += lo16(r4.y); o[3] += hi16(r4.y);
                        o[4] += lo16(r4.z); o[5] += hi16(r4.z); o[6] += lo16(r4.w); o[7] += hi16(r4.w);
                    }
                    if (relu) {
#pragma unroll
                        for (int e = 0; e < 8; ++e) o[e] = o[e] < 0.f ? 0.f : o[e];
                    }
                    u32x4 out;
                    out.x = pack2(o[0], o[1]); out.y = pack2(o[2], o[3]);
                    out.z = pack2(o[4], o[5]); out.w = pack2(o[6], o[7]);
                    if constexpr (HAS_MASK) {
                        const u32x4 mv = rmsk[u][i2];
                        out.x = keep_where_positive_bf16(out.x, mv.x); out.y = keep_where_positive_bf16(out.y, mv.y);
                        out.z = keep_where_positive_bf16(out.z, mv.z); out.w = keep_where_positive_bf16(out.w, mv.w);
                    }
                    if (mine) *reinterpret_cast<u32x4 *>(yg + orow + (size_t)(u * 32 + 16 * i2 + 8 * half) * 2) = out;
                }
            }
        }
        __syncthreads();                                         // every wavefront is done with the rows
    }
}

static int max_tile(int W) { return (kMaxRows - 2 * W - 2) / 8 * 8; }

// as few rounds of one workgroup per CU as the staged rows allow, tiles of equal size
static int pick_tile(const ConvArgs &a) {
    const long long cap = max_tile(a.W);
    const long long rounds = (a.M + 256 * cap - 1) / (256 * cap);
    long long bm = (a.M + 256 * rounds - 1) / (256 * rounds);
    bm = (bm + 7) / 8 * 8;
    if (bm < 64) bm = 64;
    if (bm > cap) bm = cap;
    return (int)bm;
}

template <bool HAS_RES, bool HAS_MASK>
static hipError_t launch_t(const ConvArgs &a, hipStream_t stream) {
    static bool raised = false;
    if (!raised) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&conv3x3_c64_kernel<HAS_RES, HAS_MASK>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, kLds);
        if (e != hipSuccess) return e;
        raised = true;
    }
    const int BM = pick_tile(a), HR = BM + 2 * a.W + 2, NT = (BM + 31) / 32;
    const long long tiles = ((long long)a.M + BM - 1) / BM;
    if (HR > kMaxRows || NT > kWaves || tiles > 0x7FFFFFFFLL) return hipErrorInvalidValue;
    const unsigned grid = (unsigned)(tiles < 256 ? tiles : 256);
    conv3x3_c64_kernel<HAS_RES, HAS_MASK><<<dim3(grid), dim3(kThreads), kLds, stream>>>(a, BM, HR, NT, (int)tiles);
    return hipGetLastError();
}

}  // namespace c64

// conv_check() must have passed.
bool conv3x3_c64_applies(const ConvArgs &a) {
    if (!a.bf16 || a.R != 3 || a.S != 3 || a.stride != 1 || a.pad != 1 || a.relu > 1) return false;
    if (a.Cin != 64 || a.Cout != 64 || a.P != a.H || a.Q != a.W) return false;
    if (a.oy_s) return false;
    return c64::max_tile(a.W) >= 64;
}

hipError_t launch_conv3x3_c64(const ConvArgs &a, hipStream_t stream) {
    if (conv_check(a) || !conv3x3_c64_applies(a)) return hipErrorInvalidValue;
    if (a.res) return a.mask ? c64::launch_t<true, true>(a, stream) : c64::launch_t<true, false>(a, stream);
    return a.mask ? c64::launch_t<false, true>(a, stream) : c64::launch_t<false, false>(a, stream);
}

}  // namespace delta
