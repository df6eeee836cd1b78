// The operators of a ResNet that are not bottleneck convolutions: the 7x7 stem, max
// pooling, global average pooling and the mean softmax cross-entropy.  DELTA regenerates
// them like any other operator output (Sec. 5.5 lists PoolingForward among the tensors that
// are released and recomputed), so they go through delta_recompute_segment as well.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kernels.hpp"

namespace delta {

typedef __bf16 bf16x8_s __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2_s __attribute__((ext_vector_type(2)));
typedef float f32x2_s __attribute__((ext_vector_type(2)));
typedef float f32x16_s __attribute__((ext_vector_type(16)));
typedef float f32x4_s __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4_s __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2_s __attribute__((ext_vector_type(2)));

namespace {
__device__ __forceinline__ uint32_t pack2s(float lo, float hi) {
    const f32x2_s v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_s));
}
__device__ __forceinline__ float blo(uint32_t p) { return __uint_as_float(p << 16); }
__device__ __forceinline__ float bhi(uint32_t p) { return __uint_as_float(p & 0xFFFF0000u); }
}  // namespace

// ------------------------------------------------------------------------------ stem
// 7x7, stride 2, pad 3, Cin = 3, Cout = 64, bf16.  Implicit GEMM on the matrix cores with the
// reduction axis laid out as (r, s, c padded to 4): for a fixed kernel row r the 7 taps x 4
// channels of one output pixel are 28 contiguous elements of the input patch once its
// pixels are padded from 3 to 4 channels, starting at a 16-byte boundary (stride 2 x 4
// channels x 2 bytes).  Each row is rounded up to 32 elements -- the extra tap and the
// fourth channel carry zero weights -- so K = 7 x 32 = 224, fourteen 32x32x16 steps.
//
// The layer is bound by its 128 bytes of output per pixel (24.5 input bytes, 224 MFMA steps per
// 32 pixels), so the kernel is built around the memory side:
//  * a workgroup (4 wavefronts, two workgroups per CU) owns 8 output rows x 112 output columns at
//    a time and is persistent over such tiles; the 21 x 240 input pixels a tile needs are whole
//    16-byte-aligned runs of the image rows when the image width is a multiple of 8: a thread
//    fetches 8 pixels (48 bytes) with three 16-byte loads and writes them to LDS as 8 padded
//    pixels.  The next tile's pixels are requested before the current tile is multiplied and wait
//    in registers.  (Other widths take one pixel per thread and step.)
//  * the rearranged weights live in registers (112 per lane) for the whole launch, so the inner
//    loop is one 16-byte LDS read per two MFMAs;
//  * a wavefront finishes 32 pixels (2 rows x 16 columns) at a time through a private fp32 LDS tile
//    that turns channel-major accumulators into pixel rows; scale, shift, ReLU and the rounding
//    happen on the row side, where a lane's 8 channels are the same for every pixel (16 registers
//    instead of 32 LDS reads per 32 pixels), and stores are whole 128-byte lines.
static constexpr int kStemRO = 8, kStemCQ = 112;              // output rows x columns of a tile
static constexpr int kStemPRows = 2 * kStemRO + 5;             // 21 input rows
static constexpr int kStemGroups = (2 * kStemCQ + 16) / 8;     // 30 groups of 8 input pixels per row
// input pixel w of a tile whose first output column is q0 sits at position w - 2 q0 + 11 of its row:
// groups start at position 3, the taps of output column q at position 2 (q - q0) + 8 (16-byte aligned)
static constexpr int kStemPPitch = (3 + 8 * kStemGroups + 1) * 8;   // 1952 bytes
static constexpr int kStemPatch = kStemPRows * kStemPPitch;          // 40992 bytes
static constexpr int kStemTasks = kStemPRows * kStemGroups;          // 630 groups per tile
static constexpr int kStemTPitch = 64 * 4 + 16;                      // fp32 row of 64 channels + pad
static constexpr int kStemLds = kStemPatch + 4 * 32 * kStemTPitch;
static_assert(64 * (7 * 64 + 16) <= kStemPatch, "the weights are staged in the patch buffer first");

__global__ __launch_bounds__(256, 2) void stem7x7_kernel(ConvArgs a, int tiles_p, int tiles_q, int ntiles, int aligned) {
    __shared__ __align__(16) unsigned char lds[kStemLds];
    unsigned char *patch = lds;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int l32 = lane & 31, half = lane >> 5;
    unsigned char *ttile = lds + kStemPatch + wv * (32 * kStemTPitch);
    const uint16_t *wg = static_cast<const uint16_t *>(a.w);
    const uint16_t *xg = static_cast<const uint16_t *>(a.x);

    // ---- weights: wl[k][r][s*4 + c] = w[k][r][s][c], zero for s = 7 or c = 3; through LDS (the patch
    // buffer, not yet in use) into registers: wreg[r][hh][u] = 8 elements 16 hh + 8 half .. of row r of
    // output channel 32 u + l32
    {
        constexpr int WP = 7 * 64 + 16;
        for (int e = tid; e < 64 * 7 * 32; e += 256) {
            const int k = e / 224, rem = e - k * 224;
            const int r = rem >> 5, el = rem & 31;
            const int s = el >> 2, c = el & 3;
            uint16_t v = 0;
            if (s < 7 && c < 3) v = wg[((k * 7 + r) * 7 + s) * 3 + c];
            *reinterpret_cast<uint16_t *>(patch + k * WP + r * 64 + el * 2) = v;
        }
    }
    __syncthreads();
    u32x4_s wreg[7][2][2];
    {
        constexpr int WP = 7 * 64 + 16;
        const unsigned char *wrow = patch + l32 * WP + half * 16;
#pragma unroll
        for (int r = 0; r < 7; ++r)
#pragma unroll
            for (int hh = 0; hh < 2; ++hh) {
                wreg[r][hh][0] = *reinterpret_cast<const u32x4_s *>(wrow + r * 64 + hh * 32);
                wreg[r][hh][1] = *reinterpret_cast<const u32x4_s *>(wrow + 32 * WP + r * 64 + hh * 32);
            }
    }
    const int trow = lane >> 3, tseg = lane & 7;
    float sc[8], sh[8];                             // of channels 8 tseg .. + 8, the ones this lane finishes
    {
        const f32x4_s s0 = *reinterpret_cast<const f32x4_s *>(a.scale + tseg * 8), s1 = *reinterpret_cast<const f32x4_s *>(a.scale + tseg * 8 + 4);
        const f32x4_s h0 = *reinterpret_cast<const f32x4_s *>(a.shift + tseg * 8), h1 = *reinterpret_cast<const f32x4_s *>(a.shift + tseg * 8 + 4);
        sc[0] = s0.x; sc[1] = s0.y; sc[2] = s0.z; sc[3] = s0.w; sc[4] = s1.x; sc[5] = s1.y; sc[6] = s1.z; sc[7] = s1.w;
        sh[0] = h0.x; sh[1] = h0.y; sh[2] = h0.z; sh[3] = h0.w; sh[4] = h1.x; sh[5] = h1.y; sh[6] = h1.z; sh[7] = h1.w;
    }

    // ---- input staging.  Aligned form: task (row i, group g) = 8 pixels, three per thread and tile.
    u32x4_s pre[3][3];
    auto tile_origin = [&](int tile, int &n, int &p0, int &q0) {
        n = tile / (tiles_p * tiles_q);
        const int t2 = tile - n * tiles_p * tiles_q;
        p0 = (t2 / tiles_q) * kStemRO;
        q0 = (t2 % tiles_q) * kStemCQ;
    };
    // Every thread issues its three loads unconditionally (pieces outside the image or past the task list
    // read the first bytes of the image instead and are zeroed when they are written to LDS): nothing
    // depends on the loaded registers until then, so the loads stay in flight under the MFMAs.
    uint32_t pre_ok = 0;
    auto request = [&](int tile) {                   // aligned form only
        int n, p0, q0;
        tile_origin(tile, n, p0, q0);
        pre_ok = 0;
#pragma unroll
        for (int t = 0; t < 3; ++t) {
            const int idx = tid + 256 * t;
            const int i = idx / kStemGroups, g = idx - i * kStemGroups;
            const int h = 2 * p0 - 3 + i, w0 = 2 * q0 - 8 + 8 * g;
            const bool ok = idx < kStemTasks && (unsigned)h < (unsigned)a.H && w0 >= 0 && w0 + 8 <= a.W;
            pre_ok |= ok ? 1u << t : 0u;
            const u32x4_s *src = reinterpret_cast<const u32x4_s *>(xg + ((size_t)((size_t)n * a.H + (ok ? h : 0)) * a.W + (ok ? w0 : 0)) * 3);
#pragma unroll
            for (int q = 0; q < 3; ++q) pre[t][q] = src[q];
        }
    };
    auto deposit = [&]() {                           // 24 bf16 = 8 pixels x 3 channels -> 8 x (3 channels + 0)
#pragma unroll
        for (int t = 0; t < 3; ++t) {
            const int idx = tid + 256 * t;
            if (idx >= kStemTasks) continue;
            const int i = idx / kStemGroups, g = idx - i * kStemGroups;
            const uint32_t keep = (pre_ok >> t) & 1u ? 0xFFFFFFFFu : 0u;
            const uint32_t d[12] = {pre[t][0].x & keep, pre[t][0].y & keep, pre[t][0].z & keep, pre[t][0].w & keep,
                                    pre[t][1].x & keep, pre[t][1].y & keep, pre[t][1].z & keep, pre[t][1].w & keep,
                                    pre[t][2].x & keep, pre[t][2].y & keep, pre[t][2].z & keep, pre[t][2].w & keep};
            unsigned char *dst = patch + i * kStemPPitch + (3 + 8 * g) * 8;
#pragma unroll
            for (int px = 0; px < 8; ++px) {
                // elements 3 px, 3 px + 1, 3 px + 2 of the 24
                const int e0 = 3 * px;
                uint32_t lo, hi;
                if (e0 & 1) {                        // starts in the upper half of a dword
                    lo = (d[e0 >> 1] >> 16) | (d[(e0 >> 1) + 1] << 16);
                    hi = d[(e0 >> 1) + 1] >> 16;
                } else {
                    lo = d[e0 >> 1];
                    hi = d[(e0 >> 1) + 1] & 0xFFFFu;
                }
                *reinterpret_cast<u32x2_s *>(dst + px * 8) = u32x2_s{lo, hi};
            }
        }
    };
    auto stage_any = [&](int tile) {                 // any width: one pixel per thread and step
        int n, p0, q0;
        tile_origin(tile, n, p0, q0);
        constexpr int COLS = 8 * kStemGroups;
        for (int e = tid; e < kStemPRows * COLS; e += 256) {
            const int i = e / COLS, j = e - i * COLS;
            const int h = 2 * p0 - 3 + i, w = 2 * q0 - 8 + j;
            u32x2_s v = {0u, 0u};
            if ((unsigned)h < (unsigned)a.H && (unsigned)w < (unsigned)a.W) {
                const uint16_t *px = xg + ((size_t)((size_t)n * a.H + h) * a.W + w) * 3;
                v.x = (uint32_t)px[0] | ((uint32_t)px[1] << 16);
                v.y = (uint32_t)px[2];
            }
            *reinterpret_cast<u32x2_s *>(patch + i * kStemPPitch + (3 + j) * 8) = v;
        }
    };

    int tile = blockIdx.x;
    if (aligned && tile < ntiles) request(tile);
    for (; tile < ntiles; tile += gridDim.x) {
        int n, p0, q0;
        tile_origin(tile, n, p0, q0);
        __syncthreads();                             // the previous tile's patch (or the weights) is no longer read
        if (aligned) deposit(); else stage_any(tile);
        __syncthreads();
        if (aligned && tile + (int)gridDim.x < ntiles) request(tile + gridDim.x);   // in flight under the MFMAs

        // ---- 28 units of 2 rows x 16 columns, seven per wavefront
        for (int j = 0; j < 7; ++j) {
            const int unit = wv + 4 * j, ur = unit / 7, uc = unit - ur * 7;
            if (p0 + 2 * ur >= a.P || q0 + 16 * uc >= a.Q) continue;          // the same for the whole wavefront
            const int prow = 2 * ur + (l32 >> 4), pcol = 16 * uc + (l32 & 15);
            f32x16_s acc[2];
#pragma unroll
            for (int u = 0; u < 2; ++u)
#pragma unroll
                for (int e = 0; e < 16; ++e) acc[u][e] = 0.f;
            const unsigned char *xrow = patch + (2 * prow) * kStemPPitch + pcol * 16 + 64 + half * 16;
            // the pixel operand of step k + 4 is requested before step k is multiplied (a ring of four):
            // with two wavefronts per SIMD one read ahead does not cover the LDS latency
            u32x4_s xq[4];
#pragma unroll
            for (int k = 0; k < 4; ++k)
                xq[k] = *reinterpret_cast<const u32x4_s *>(xrow + (k >> 1) * kStemPPitch + (k & 1) * 32);
            __builtin_amdgcn_sched_barrier(0);       // (the scheduler would otherwise pull the reads back to one step ahead)
#pragma unroll
            for (int k = 0; k < 14; ++k) {
                const u32x4_s xb = xq[k & 3];
                if (k + 4 < 14)
                    xq[k & 3] = *reinterpret_cast<const u32x4_s *>(xrow + ((k + 4) >> 1) * kStemPPitch + ((k + 4) & 1) * 32);
                acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_s, wreg[k >> 1][k & 1][0]),
                                                                 __builtin_bit_cast(bf16x8_s, xb), acc[0], 0, 0, 0);
                acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_s, wreg[k >> 1][k & 1][1]),
                                                                 __builtin_bit_cast(bf16x8_s, xb), acc[1], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
            }
            // acc[u][4 rb + e] = channel 32 u + 8 rb + 4 half + e of pixel l32 -> fp32 rows in the private tile
#pragma unroll
            for (int u = 0; u < 2; ++u)
#pragma unroll
                for (int rb = 0; rb < 4; ++rb) {
                    const f32x4_s v = {acc[u][4 * rb], acc[u][4 * rb + 1], acc[u][4 * rb + 2], acc[u][4 * rb + 3]};
                    *reinterpret_cast<f32x4_s *>(ttile + l32 * kStemTPitch + (u * 32 + 8 * rb + 4 * half) * 4) = v;
                }
            // (LDS instructions of one wavefront execute in order; the fences only keep the compiler from
            // moving accesses across the exchange)
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const int pr = trow + 8 * t;         // pixel of the unit: row pr / 16, column pr % 16
                const f32x4_s f0 = *reinterpret_cast<const f32x4_s *>(ttile + pr * kStemTPitch + tseg * 32);
                const f32x4_s f1 = *reinterpret_cast<const f32x4_s *>(ttile + pr * kStemTPitch + tseg * 32 + 16);
                float o[8] = {f0.x, f0.y, f0.z, f0.w, f1.x, f1.y, f1.z, f1.w};
#pragma unroll
                for (int e = 0; e < 8; ++e) o[e] = o[e] * sc[e] + sh[e];
                if (a.relu) {
#pragma unroll
                    for (int e = 0; e < 8; ++e) o[e] = o[e] < 0.f ? 0.f : o[e];
                }
                u32x4_s o4;
                o4.x = pack2s(o[0], o[1]); o4.y = pack2s(o[2], o[3]);
                o4.z = pack2s(o[4], o[5]); o4.w = pack2s(o[6], o[7]);
                const int p = p0 + 2 * ur + (pr >> 4), q = q0 + 16 * uc + (pr & 15);
                if (p < a.P && q < a.Q)
                    *reinterpret_cast<u32x4_s *>(static_cast<unsigned char *>(a.y) +
                                                 ((size_t)((size_t)n * a.P + p) * a.Q + q) * 128 + tseg * 16) = o4;
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        }
    }
}

bool stem_applies(const ConvArgs &a) {
    return a.bf16 && a.R == 7 && a.S == 7 && a.stride == 2 && a.pad == 3 && a.Cin == 3 && a.Cout == 64 && !a.res;
}

const char *stem_check(const ConvArgs &a) {
    if (a.N <= 0 || a.H <= 0 || a.W <= 0) return "non-positive dimension";
    if (a.P != (a.H + 6 - 7) / 2 + 1 || a.Q != (a.W + 6 - 7) / 2 + 1 || a.P <= 0 || a.Q <= 0)
        return "inconsistent output size";
    if ((long long)a.N * a.P * a.Q != a.M || (long long)a.N * a.H * a.W > 0x7FFFFFFFLL) return "bad M";
    if (!a.x || !a.w || !a.y || !a.scale || !a.shift) return "null pointer";
    if (((uintptr_t)a.y | (uintptr_t)a.scale | (uintptr_t)a.shift) & 15) return "pointers must be 16-byte aligned";
    if (((uintptr_t)a.x | (uintptr_t)a.w) & 1) return "pointers must be 2-byte aligned";
    return nullptr;
}

hipError_t launch_stem(const ConvArgs &a, hipStream_t stream) {
    if (!stem_applies(a) || stem_check(a)) return hipErrorInvalidValue;
    const int tiles_p = (a.P + kStemRO - 1) / kStemRO, tiles_q = (a.Q + kStemCQ - 1) / kStemCQ;
    const long long ntiles = (long long)a.N * tiles_p * tiles_q;
    if (ntiles <= 0 || ntiles > 0x3FFFFFFFLL) return hipErrorInvalidValue;
    const int grid = (int)(ntiles < 512 ? ntiles : 512);            // two workgroups per CU
    // whole 16-byte runs of 8 pixels: rows start 16-byte aligned when the width is a multiple of 8
    const int aligned = a.W % 8 == 0 && ((uintptr_t)a.x & 15) == 0;
    stem7x7_kernel<<<dim3(grid), dim3(256), 0, stream>>>(a, tiles_p, tiles_q, (int)ntiles, aligned);
    return hipGetLastError();
}

// --------------------------------------------------------------------------- pooling

// One thread: 16 bytes of channels (8 bf16 or 4 fp32) of one output pixel.
template <bool BF16>
__global__ __launch_bounds__(256) void maxpool_kernel(PoolArgs a, long long total) {
    // Workgroups are dealt round-robin to the 8 XCDs; each XCD takes a contiguous range of outputs, so
    // that the input rows two neighbouring output rows share are fetched into one L2, once (with
    // neighbouring output rows on different XCDs the 3 x 3 stride-2 pool fetched 1.5 x its input).
    const unsigned nb = gridDim.x, per = nb >> 3, rem = nb & 7u;
    const unsigned xcd = blockIdx.x & 7u, slot = blockIdx.x >> 3;
    const unsigned logical = xcd < rem ? xcd * (per + 1) + slot : rem * (per + 1) + (xcd - rem) * per + slot;
    const long long idx = (long long)logical * 256 + threadIdx.x;
    if (idx >= total) return;
    constexpr int CPT = BF16 ? 8 : 4;
    const int chunks = a.C / CPT;
    const int ck = (int)(idx % chunks);
    long long pix = idx / chunks;
    const int q = (int)(pix % a.Q);
    pix /= a.Q;
    const int p = (int)(pix % a.P);
    const int n = (int)(pix / a.P);
    float m[CPT];
#pragma unroll
    for (int e = 0; e < CPT; ++e) m[e] = -INFINITY;
    const unsigned char *xg = static_cast<const unsigned char *>(a.x);
    for (int r = 0; r < a.R; ++r) {
        const int h = p * a.stride + r - a.pad;
        if ((unsigned)h >= (unsigned)a.H) continue;
        for (int s = 0; s < a.S; ++s) {
            const int w = q * a.stride + s - a.pad;
            if ((unsigned)w >= (unsigned)a.W) continue;
            const u32x4_s v = *reinterpret_cast<const u32x4_s *>(
                xg + (((size_t)((size_t)n * a.H + h) * a.W + w) * chunks + ck) * 16);
            if constexpr (BF16) {
                m[0] = fmaxf(m[0], blo(v.x)); m[1] = fmaxf(m[1], bhi(v.x));
                m[2] = fmaxf(m[2], blo(v.y)); m[3] = fmaxf(m[3], bhi(v.y));
                m[4] = fmaxf(m[4], blo(v.z)); m[5] = fmaxf(m[5], bhi(v.z));
                m[6] = fmaxf(m[6], blo(v.w)); m[7] = fmaxf(m[7], bhi(v.w));
            } else {
                m[0] = fmaxf(m[0], __uint_as_float(v.x)); m[1] = fmaxf(m[1], __uint_as_float(v.y));
                m[2] = fmaxf(m[2], __uint_as_float(v.z)); m[3] = fmaxf(m[3], __uint_as_float(v.w));
            }
        }
    }
    u32x4_s o;
    if constexpr (BF16) {
        o.x = pack2s(m[0], m[1]); o.y = pack2s(m[2], m[3]); o.z = pack2s(m[4], m[5]); o.w = pack2s(m[6], m[7]);
    } else {
        o.x = __float_as_uint(m[0]); o.y = __float_as_uint(m[1]); o.z = __float_as_uint(m[2]); o.w = __float_as_uint(m[3]);
    }
    *reinterpret_cast<u32x4_s *>(static_cast<unsigned char *>(a.y) + (size_t)idx * 16) = o;
}

// Global average: one thread per (image, 16 bytes of channels), fp32 accumulation in pixel order.
template <bool BF16>
__global__ __launch_bounds__(256) void avgpool_kernel(PoolArgs a, long long total) {
    const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= total) return;
    constexpr int CPT = BF16 ? 8 : 4;
    const int chunks = a.C / CPT;
    const int ck = (int)(idx % chunks);
    const int n = (int)(idx / chunks);
    float s[CPT];
#pragma unroll
    for (int e = 0; e < CPT; ++e) s[e] = 0.f;
    const unsigned char *xg = static_cast<const unsigned char *>(a.x);
    const int hw = a.H * a.W;
    for (int i = 0; i < hw; ++i) {
        const u32x4_s v = *reinterpret_cast<const u32x4_s *>(xg + (((size_t)n * hw + i) * chunks + ck) * 16);
        if constexpr (BF16) {
            s[0] += blo(v.x); s[1] += bhi(v.x); s[2] += blo(v.y); s[3] += bhi(v.y);
            s[4] += blo(v.z); s[5] += bhi(v.z); s[6] += blo(v.w); s[7] += bhi(v.w);
        } else {
            s[0] += __uint_as_float(v.x); s[1] += __uint_as_float(v.y);
            s[2] += __uint_as_float(v.z); s[3] += __uint_as_float(v.w);
        }
    }
    const float inv = 1.0f / (float)hw;
    u32x4_s o;
    if constexpr (BF16) {
        o.x = pack2s(s[0] * inv, s[1] * inv); o.y = pack2s(s[2] * inv, s[3] * inv);
        o.z = pack2s(s[4] * inv, s[5] * inv); o.w = pack2s(s[6] * inv, s[7] * inv);
    } else {
        o.x = __float_as_uint(s[0] * inv); o.y = __float_as_uint(s[1] * inv);
        o.z = __float_as_uint(s[2] * inv); o.w = __float_as_uint(s[3] * inv);
    }
    *reinterpret_cast<u32x4_s *>(static_cast<unsigned char *>(a.y) + (size_t)idx * 16) = o;
}

const char *pool_check(const PoolArgs &a, bool global_avg) {
    const int cpt = a.bf16 ? 8 : 4;
    if (a.N <= 0 || a.H <= 0 || a.W <= 0 || a.C <= 0) return "non-positive dimension";
    if (a.C % cpt) return "channels must be a multiple of 8 (bf16) or 4 (fp32)";
    if (!a.x || !a.y || (((uintptr_t)a.x | (uintptr_t)a.y) & 15)) return "pointers must be non-null and 16-byte aligned";
    if ((long long)a.N * a.H * a.W > 0x7FFFFFFFLL) return "input too large";
    if (!global_avg) {
        if (a.R <= 0 || a.S <= 0 || a.stride <= 0 || a.pad < 0 || a.pad >= a.R || a.pad >= a.S)
            return "bad window (padding must be smaller than the window)";
        if (a.P != (a.H + 2 * a.pad - a.R) / a.stride + 1 || a.Q != (a.W + 2 * a.pad - a.S) / a.stride + 1 ||
            a.P <= 0 || a.Q <= 0)
            return "inconsistent output size";
    }
    return nullptr;
}

hipError_t launch_maxpool(const PoolArgs &a, hipStream_t stream) {
    if (pool_check(a, false)) return hipErrorInvalidValue;
    const long long total = (long long)a.N * a.P * a.Q * (a.C / (a.bf16 ? 8 : 4));
    const long long blocks = (total + 255) / 256;
    if (blocks > 0x7FFFFFFFLL) return hipErrorInvalidValue;
    if (a.bf16) maxpool_kernel<true><<<dim3((unsigned)blocks), dim3(256), 0, stream>>>(a, total);
    else maxpool_kernel<false><<<dim3((unsigned)blocks), dim3(256), 0, stream>>>(a, total);
    return hipGetLastError();
}

hipError_t launch_avgpool(const PoolArgs &a, hipStream_t stream) {
    if (pool_check(a, true)) return hipErrorInvalidValue;
    const long long total = (long long)a.N * (a.C / (a.bf16 ? 8 : 4));
    const long long blocks = (total + 255) / 256;
    if (a.bf16) avgpool_kernel<true><<<dim3((unsigned)blocks), dim3(256), 0, stream>>>(a, total);
    else avgpool_kernel<false><<<dim3((unsigned)blocks), dim3(256), 0, stream>>>(a, total);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------ loss
// Mean over images of logsumexp(z_i) - z_i[label_i].  One workgroup of 16 wavefronts (the
// result is one float, so there is nothing to spread over the chip; what matters is that the
// loads of a wavefront are all in flight together).  A wavefront takes two images per round;
// a lane owns classes lane, lane + 64, ... and holds up to 16 of them per image in registers,
// so each logit is read once; more than 1024 classes fall back to re-reading loops.  Fixed
// reduction trees and a fixed image -> wavefront map: the result does not depend on timing.
// A label outside [0, classes) makes the result NaN, so that it cannot pass unnoticed.
template <bool BF16>
__device__ __forceinline__ float logit_at(const void *logits, size_t idx) {
    return BF16 ? __uint_as_float((uint32_t)static_cast<const uint16_t *>(logits)[idx] << 16)
                : static_cast<const float *>(logits)[idx];
}

template <bool BF16>
__global__ __launch_bounds__(1024) void softmax_ce_kernel(const void *logits, const long long *labels, int N,
                                                          int classes, float *out) {
    constexpr int WAVES = 16, IMGS = 2, KMAX = 16;
    __shared__ float part[WAVES];
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    float total = 0.f;
    if (classes <= 64 * KMAX) {
        for (int i0 = wv * IMGS; i0 < N; i0 += WAVES * IMGS) {
            float z[IMGS][KMAX], zl[IMGS];
#pragma unroll
            for (int u = 0; u < IMGS; ++u) {
                const int i = i0 + u;
#pragma unroll
                for (int k = 0; k < KMAX; ++k) {
                    const int c = lane + 64 * k;
                    z[u][k] = (i < N && c < classes) ? logit_at<BF16>(logits, (size_t)i * classes + c) : -INFINITY;
                }
                zl[u] = __builtin_nanf("");
                if (i < N) {
                    const long long lab = labels[i];
                    if (lab >= 0 && lab < classes) zl[u] = logit_at<BF16>(logits, (size_t)i * classes + lab);
                }
            }
#pragma unroll
            for (int u = 0; u < IMGS; ++u) {
                if (i0 + u >= N) break;                       // uniform over the wavefront
                float mx = -INFINITY;
#pragma unroll
                for (int k = 0; k < KMAX; ++k) mx = fmaxf(mx, z[u][k]);
#pragma unroll
                for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o));
                float se = 0.f;
#pragma unroll
                for (int k = 0; k < KMAX; ++k)
                    if (lane + 64 * k < classes) se += __expf(z[u][k] - mx);
#pragma unroll
                for (int o = 32; o > 0; o >>= 1) se += __shfl_xor(se, o);
                total += (mx + __logf(se)) - zl[u];
            }
        }
    } else {
        for (int i = wv; i < N; i += WAVES) {
            float mx = -INFINITY;
            for (int c = lane; c < classes; c += 64) mx = fmaxf(mx, logit_at<BF16>(logits, (size_t)i * classes + c));
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o));
            float se = 0.f;
            for (int c = lane; c < classes; c += 64) se += __expf(logit_at<BF16>(logits, (size_t)i * classes + c) - mx);
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) se += __shfl_xor(se, o);
            const long long lab = labels[i];
            float zl = __builtin_nanf("");
            if (lab >= 0 && lab < classes) zl = logit_at<BF16>(logits, (size_t)i * classes + lab);
            total += (mx + __logf(se)) - zl;
        }
    }
    if (lane == 0) part[wv] = total;
    __syncthreads();
    if (threadIdx.x == 0) {
        float sum = 0.f;
#pragma unroll
        for (int w = 0; w < WAVES; ++w) sum += part[w];
        out[0] = sum / (float)N;
    }
}

hipError_t launch_softmax_ce(const void *logits, const void *labels, int N, int classes, int bf16, float *out,
                             hipStream_t stream) {
    if (!logits || !labels || !out || N <= 0 || classes <= 0) return hipErrorInvalidValue;
    if (bf16) softmax_ce_kernel<true><<<dim3(1), dim3(1024), 0, stream>>>(logits, static_cast<const long long *>(labels), N, classes, out);
    else softmax_ce_kernel<false><<<dim3(1), dim3(1024), 0, stream>>>(logits, static_cast<const long long *>(labels), N, classes, out);
    return hipGetLastError();
}

}  // namespace delta
