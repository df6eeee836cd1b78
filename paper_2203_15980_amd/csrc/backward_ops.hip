// Backward of the layers around the bottleneck stack (bf16): max pooling, global average
// pooling, the classifier and the cross-entropy loss.  With backward.hip they make the backward
// half of a ResNet training iteration, the pass whose accesses to stored activations DELTA's
// planner follows (Sec. 3, Assumptions 1-3).  All of them are memory-bound and small next to the
// convolutions; they are written for bytes per thread and coalescing, not for the matrix cores.
// Nothing here uses atomics: every output element is produced by exactly one thread, in a fixed
// order of additions.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#include "kernels.hpp"

namespace delta {
namespace bops {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ float lo16(uint32_t p) { return __uint_as_float(p << 16); }
__device__ __forceinline__ float hi16(uint32_t p) { return __uint_as_float(p & 0xFFFF0000u); }
__device__ __forceinline__ uint32_t pack2(float lo, float hi) {
    const f32x2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}
__device__ __forceinline__ void unpack8(const u32x4 v, float (&f)[8]) {
    f[0] = lo16(v.x); f[1] = hi16(v.x); f[2] = lo16(v.y); f[3] = hi16(v.y);
    f[4] = lo16(v.z); f[5] = hi16(v.z); f[6] = lo16(v.w); f[7] = hi16(v.w);
}
__device__ __forceinline__ u32x4 pack8(const float (&f)[8]) {
    u32x4 o;
    o.x = pack2(f[0], f[1]); o.y = pack2(f[2], f[3]); o.z = pack2(f[4], f[5]); o.w = pack2(f[6], f[7]);
    return o;
}

// ---------------------------------------------------------------- max pooling
// A workgroup owns an 8 x 8 tile of INPUT pixels and 64 channels (8 chunks of 8), in three steps:
//  1. copy every pixel that a window touching the tile can reach (the tile plus R-1 / S-1 pixels
//     on each side) into LDS, and the gradients of those windows with them (one global round trip
//     for both; step 3 then reads each window's gradient from LDS instead of once per pixel);
//  2. one thread per (window, chunk): scan the window in the forward's order (r, then s, padding
//     skipped) and record, per channel, the position r*S + s of the first maximal element as
//     one byte (255: none) - each window is scanned once, not once per pixel it covers;
//  3. one thread per (pixel, chunk): for each of the at most ceil(R/stride) x ceil(S/stride)
//     windows containing the pixel, add the window's gradient where the recorded position is
//     the pixel's.  Sums in window order (p, then q), fp32.
// Every loop has a uniform trip count and selects instead of branches: a per-element `if`
// compiled to a branch per element and ran ten times slower.  The kernel is bound by its vector
// arithmetic (about 3300 wavefront instructions per tile): XCD-aware tile numbering and trip counts
// made uniform per wavefront by pixel parity class both left its time unchanged; scanning only the
// windows that can touch the tile (5 x 5 instead of 6 x 6 for the 3 x 3 stride-2 pool) took 16 % off.
static constexpr int kPoolTile = 8, kPoolChunks = 8;

// windows p with a pixel in kPoolTile consecutive rows: stride * p - pad in [h0 - R + 1, h0 + kPoolTile - 1],
// an interval of length kPoolTile + R - 2
__host__ __device__ inline int pool_windows_max(int R, int stride) { return (kPoolTile + R - 2) / stride + 1; }

// FIXED: the ResNet pool (3 x 3, stride 2, padding 1) with every loop unrolled.
template <bool FIXED>
__global__ __launch_bounds__(256) void maxpool_bwd_kernel(PoolArgs a, const void *gy, void *gx, int tiles_w, int tiles_h,
                                                          int mask_x) {
    if constexpr (FIXED) { a.R = 3; a.S = 3; a.stride = 2; a.pad = 1; }
    extern __shared__ __align__(16) unsigned char plds[];
    const int chunks = a.C / 8, cgroups = (chunks + kPoolChunks - 1) / kPoolChunks;
    int blk = blockIdx.x;
    const int cg = blk % cgroups; blk /= cgroups;
    const int tw = blk % tiles_w; blk /= tiles_w;
    const int th = blk % tiles_h;
    const int n = blk / tiles_h;
    const int h0 = th * kPoolTile, w0 = tw * kPoolTile;
    const int LH = kPoolTile + 2 * (a.R - 1), LW = kPoolTile + 2 * (a.S - 1);
    const int NWH = pool_windows_max(a.R, a.stride), NWW = pool_windows_max(a.S, a.stride);
    unsigned char *arg = plds + (size_t)LH * LW * kPoolChunks * 16;      // [NWH][NWW][chunk] x 8 bytes
    unsigned char *gys = arg + (size_t)NWH * NWW * kPoolChunks * 8;      // [NWH][NWW][chunk] x 16 bytes
    const unsigned char *xg = static_cast<const unsigned char *>(a.x);
    const unsigned char *gg = static_cast<const unsigned char *>(gy);
    // windows that contain a pixel of the tile: p in [pw0, pw0 + NWH) clipped to the image (likewise q)
    int pw0 = h0 + a.pad - a.R + 1;
    pw0 = pw0 <= 0 ? 0 : (pw0 + a.stride - 1) / a.stride;
    int qw0 = w0 + a.pad - a.S + 1;
    qw0 = qw0 <= 0 ? 0 : (qw0 + a.stride - 1) / a.stride;
    // step 1: LDS pixel (lh, lw) = image pixel (h0 - (R-1) + lh, w0 - (S-1) + lw); outside the image: zeros, unused
    for (int i = threadIdx.x; i < LH * LW * kPoolChunks; i += 256) {
        const int c = i % kPoolChunks, pix = i / kPoolChunks;
        const int lh = pix / LW, lw = pix - lh * LW;
        const int hh = h0 - (a.R - 1) + lh, ww = w0 - (a.S - 1) + lw, ck = cg * kPoolChunks + c;
        u32x4 v = {0u, 0u, 0u, 0u};
        if ((unsigned)hh < (unsigned)a.H && (unsigned)ww < (unsigned)a.W && ck < chunks)
            v = *reinterpret_cast<const u32x4 *>(xg + ((((size_t)n * a.H + hh) * a.W + ww) * chunks + ck) * 16);
        *reinterpret_cast<u32x4 *>(plds + (size_t)i * 16) = v;
    }
    for (int i = threadIdx.x; i < NWH * NWW * kPoolChunks; i += 256) {
        const int c = i % kPoolChunks, win = i / kPoolChunks;
        const int p = pw0 + win / NWW, q = qw0 + win % NWW, ck = cg * kPoolChunks + c;
        u32x4 v = {0u, 0u, 0u, 0u};
        if (p < a.P && q < a.Q && ck < chunks)
            v = *reinterpret_cast<const u32x4 *>(gg + ((((size_t)n * a.P + p) * a.Q + q) * chunks + ck) * 16);
        *reinterpret_cast<u32x4 *>(gys + (size_t)i * 16) = v;
    }
    __syncthreads();
    // step 2
    for (int i = threadIdx.x; i < NWH * NWW * kPoolChunks; i += 256) {
        const int c = i % kPoolChunks, win = i / kPoolChunks;
        const int wp = win / NWW, wq = win - wp * NWW;
        const int hb = (pw0 + wp) * a.stride - a.pad, wb = (qw0 + wq) * a.stride - a.pad;
        float m[8];
        uint32_t idx[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) { m[e] = -INFINITY; idx[e] = 255u; }
#pragma unroll
        for (int r = 0; r < a.R; ++r)
#pragma unroll
            for (int s = 0; s < a.S; ++s) {
                const int hh = hb + r, ww = wb + s;
                const bool inside = (unsigned)hh < (unsigned)a.H && (unsigned)ww < (unsigned)a.W;
                // windows beyond the tile's reach (or the image) are never consulted: clamp their reads
                int lh = hh - h0 + a.R - 1, lw = ww - w0 + a.S - 1;
                lh = lh < 0 ? 0 : (lh > LH - 1 ? LH - 1 : lh);
                lw = lw < 0 ? 0 : (lw > LW - 1 ? LW - 1 : lw);
                float v[8];
                unpack8(*reinterpret_cast<const u32x4 *>(plds + ((size_t)(lh * LW + lw) * kPoolChunks + c) * 16), v);
                const uint32_t pos = (uint32_t)(r * a.S + s);
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const bool take = inside && v[e] > m[e];
                    m[e] = take ? v[e] : m[e];
                    idx[e] = take ? pos : idx[e];
                }
            }
        u32x2 o;
        o.x = idx[0] | (idx[1] << 8) | (idx[2] << 16) | (idx[3] << 24);
        o.y = idx[4] | (idx[5] << 8) | (idx[6] << 16) | (idx[7] << 24);
        *reinterpret_cast<u32x2 *>(arg + (size_t)i * 8) = o;
    }
    __syncthreads();
    // step 3
    const int np = (a.R + a.stride - 1) / a.stride, nq = (a.S + a.stride - 1) / a.stride;
    for (int i = threadIdx.x; i < kPoolTile * kPoolTile * kPoolChunks; i += 256) {
        const int c = i % kPoolChunks, pix = i / kPoolChunks;
        const int h = h0 + pix / kPoolTile, w = w0 + pix % kPoolTile, ck = cg * kPoolChunks + c;
        const bool owned = h < a.H && w < a.W && ck < chunks;
        int p_lo = h + a.pad - a.R + 1;
        p_lo = p_lo <= 0 ? 0 : (p_lo + a.stride - 1) / a.stride;
        int p_hi = (h + a.pad) / a.stride;
        if (p_hi > a.P - 1) p_hi = a.P - 1;
        int q_lo = w + a.pad - a.S + 1;
        q_lo = q_lo <= 0 ? 0 : (q_lo + a.stride - 1) / a.stride;
        int q_hi = (w + a.pad) / a.stride;
        if (q_hi > a.Q - 1) q_hi = a.Q - 1;
        float acc[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] = 0.f;
#pragma unroll
        for (int dp = np - 1; dp >= 0; --dp)                       // ascending p, then q: the order of the sums
#pragma unroll
            for (int dq = nq - 1; dq >= 0; --dq) {
                const int p = p_hi - dp, q = q_hi - dq;
                const bool live = owned && p >= p_lo && q >= q_lo;  // this pixel lies in window (p, q)
                // clamped to the windows steps 1 and 2 covered: the LDS reads stay in bounds
                const int pc = p < pw0 ? pw0 : (p > pw0 + NWH - 1 ? pw0 + NWH - 1 : p);
                const int qc = q < qw0 ? qw0 : (q > qw0 + NWW - 1 ? qw0 + NWW - 1 : q);
                const size_t slot = (size_t)((pc - pw0) * NWW + (qc - qw0)) * kPoolChunks + c;
                const u32x2 am = *reinterpret_cast<const u32x2 *>(arg + slot * 8);
                float g[8];
                unpack8(*reinterpret_cast<const u32x4 *>(gys + slot * 16), g);
                const uint32_t my = (uint32_t)((h - (p * a.stride - a.pad)) * a.S + (w - (q * a.stride - a.pad)));
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const uint32_t pos = ((e < 4 ? am.x : am.y) >> (8 * (e & 3))) & 0xFFu;
                    acc[e] += (live && pos == my) ? g[e] : 0.f;
                }
            }
        if (owned) {
            u32x4 o = pack8(acc);
            if (mask_x) {                                           // also the ReLU mask of x's producer: x is its output
                const int lh = h - h0 + a.R - 1, lw = w - w0 + a.S - 1;
                const u32x4 xv = *reinterpret_cast<const u32x4 *>(plds + ((size_t)(lh * LW + lw) * kPoolChunks + c) * 16);
#pragma unroll
                for (int e = 0; e < 4; ++e) o[e] = keep_where_positive_bf16(o[e], xv[e]);
            }
            *reinterpret_cast<u32x4 *>(static_cast<unsigned char *>(gx) +
                                       ((((size_t)n * a.H + h) * a.W + w) * chunks + ck) * 16) = o;
        }
    }
}

// ---------------------------------------------------------------- global average pooling
// gx[n,h,w,c] = gy[n,c] / (H W); one thread per 8 channels of one input pixel.
__global__ __launch_bounds__(256) void avgpool_bwd_kernel(const void *gy, void *gx, int HW, int chunks, long long total) {
    const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= total) return;
    const int ck = (int)(idx % chunks);
    const long long n = idx / chunks / HW;
    float g[8];
    unpack8(*reinterpret_cast<const u32x4 *>(static_cast<const unsigned char *>(gy) + ((size_t)n * chunks + ck) * 16), g);
    const float inv = 1.0f / (float)HW;
#pragma unroll
    for (int e = 0; e < 8; ++e) g[e] *= inv;
    *reinterpret_cast<u32x4 *>(static_cast<unsigned char *>(gx) + (size_t)idx * 16) = pack8(g);
}

// ---------------------------------------------------------------- cross-entropy
// dL/dz[i,k] = (softmax(z_i)[k] - [k == label_i]) / N.  One wavefront per image, lanes stride over
// the classes; fixed reduction trees.
__global__ __launch_bounds__(256) void softmax_ce_bwd_kernel(const uint16_t *logits, const long long *labels, int N,
                                                             int classes, uint16_t *gz) {
    const int lane = threadIdx.x & 63;
    const int i = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (i >= N) return;
    const uint16_t *z = logits + (size_t)i * classes;
    float mx = -INFINITY;
    for (int c = lane; c < classes; c += 64) mx = fmaxf(mx, __uint_as_float((uint32_t)z[c] << 16));
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o));
    float se = 0.f;
    for (int c = lane; c < classes; c += 64) se += __expf(__uint_as_float((uint32_t)z[c] << 16) - mx);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) se += __shfl_xor(se, o);
    const float inv = 1.0f / se, invn = 1.0f / (float)N;
    const long long lab = labels[i];
    for (int c = lane; c < classes; c += 64) {
        float g = __expf(__uint_as_float((uint32_t)z[c] << 16) - mx) * inv;
        if (c == lab) g -= 1.0f;
        if (lab < 0 || lab >= classes) g = __builtin_nanf("");     // a bad label cannot pass unnoticed
        gz[(size_t)i * classes + c] = __builtin_bit_cast(uint16_t, (__bf16)(g * invn));
    }
}

// ---------------------------------------------------------------- classifier z = x w^T + bias
// gx[n][c] = sum_k gy[n][k] * scale_k * w[k][c].  A workgroup: one image, 32 x 8 input channels; its
// 8 wavefront-halves split the classes (group g takes k = g, g + 8, ...), then the 8 partial sums
// are added in group order.
__global__ __launch_bounds__(256) void dense_bwd_data_kernel(const uint16_t *gy, const void *w, const float *scale,
                                                             void *gx, int N, int Cin, int Cout) {
    __shared__ float part[8][32][8];
    const int chunks = Cin / 8, cblocks = (chunks + 31) / 32;
    const int n = blockIdx.x / cblocks, cb = blockIdx.x % cblocks;
    const int lane = threadIdx.x & 31, grp = threadIdx.x >> 5;
    const int ck = cb * 32 + lane;
    float acc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = 0.f;
    const unsigned char *wg = static_cast<const unsigned char *>(w);
    if (ck < chunks) {
#pragma unroll 4
        for (int k = grp; k < Cout; k += 8) {
            const float g = __uint_as_float((uint32_t)gy[(size_t)n * Cout + k] << 16) * scale[k];
            float v[8];
            unpack8(*reinterpret_cast<const u32x4 *>(wg + ((size_t)k * chunks + ck) * 16), v);
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[e] += g * v[e];
        }
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) part[grp][lane][e] = acc[e];
    __syncthreads();
    if (grp != 0 || ck >= chunks) return;
#pragma unroll
    for (int g = 1; g < 8; ++g)
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] += part[g][lane][e];
    *reinterpret_cast<u32x4 *>(static_cast<unsigned char *>(gx) + ((size_t)n * chunks + ck) * 16) = pack8(acc);
}

// gw[k][c] = scale_k * sum_n gy[n][k] * x[n][c] (fp32): one thread per (k, 8 input channels); n ascending.
// Threads with ck == 0 also write the bias gradient sum_n gy[n][k] behind the weights.
__global__ __launch_bounds__(256) void dense_bwd_weight_kernel(const uint16_t *gy, const void *x, const float *scale,
                                                               float *gw, int N, int Cin, int Cout) {
    const int chunks = Cin / 8;
    const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (long long)Cout * chunks) return;
    const int ck = (int)(idx % chunks), k = (int)(idx / chunks);
    float acc[8], gsum = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = 0.f;
    const unsigned char *xg = static_cast<const unsigned char *>(x);
#pragma unroll 8
    for (int n = 0; n < N; ++n) {
        const float g = __uint_as_float((uint32_t)gy[(size_t)n * Cout + k] << 16);
        gsum += g;
        float v[8];
        unpack8(*reinterpret_cast<const u32x4 *>(xg + ((size_t)n * chunks + ck) * 16), v);
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] += g * v[e];
    }
    const float sc = scale[k];
#pragma unroll
    for (int e = 0; e < 8; ++e) gw[(size_t)k * Cin + ck * 8 + e] = acc[e] * sc;
    if (ck == 0) gw[(size_t)Cout * Cin + k] = gsum;
}

}  // namespace bops

hipError_t launch_maxpool_bwd(const PoolArgs &a, const void *gy, void *gx, int mask_x, hipStream_t stream) {
    if (pool_check(a, false) || !a.bf16 || !gy || !gx) return hipErrorInvalidValue;
    const int tiles_h = (a.H + bops::kPoolTile - 1) / bops::kPoolTile, tiles_w = (a.W + bops::kPoolTile - 1) / bops::kPoolTile;
    const int cgroups = (a.C / 8 + bops::kPoolChunks - 1) / bops::kPoolChunks;
    const long long blocks = (long long)a.N * tiles_h * tiles_w * cgroups;
    if (a.R * a.S > 255) return hipErrorInvalidValue;                   // window positions are recorded as bytes
    const size_t lds = (size_t)(bops::kPoolTile + 2 * (a.R - 1)) * (bops::kPoolTile + 2 * (a.S - 1)) * bops::kPoolChunks * 16 +
                       (size_t)bops::pool_windows_max(a.R, a.stride) * bops::pool_windows_max(a.S, a.stride) * bops::kPoolChunks * (8 + 16);
    if (blocks <= 0 || blocks > 0x7FFFFFFFLL || lds > 64 * 1024) return hipErrorInvalidValue;
    if (a.R == 3 && a.S == 3 && a.stride == 2 && a.pad == 1)
        bops::maxpool_bwd_kernel<true><<<dim3((unsigned)blocks), dim3(256), lds, stream>>>(a, gy, gx, tiles_w, tiles_h, mask_x);
    else
        bops::maxpool_bwd_kernel<false><<<dim3((unsigned)blocks), dim3(256), lds, stream>>>(a, gy, gx, tiles_w, tiles_h, mask_x);
    return hipGetLastError();
}

hipError_t launch_avgpool_bwd(const PoolArgs &a, const void *gy, void *gx, hipStream_t stream) {
    if (pool_check(a, true) || !a.bf16 || !gy || !gx) return hipErrorInvalidValue;
    const long long total = (long long)a.N * a.H * a.W * (a.C / 8);
    const long long blocks = (total + 255) / 256;
    if (blocks <= 0 || blocks > 0x7FFFFFFFLL) return hipErrorInvalidValue;
    bops::avgpool_bwd_kernel<<<dim3((unsigned)blocks), dim3(256), 0, stream>>>(gy, gx, a.H * a.W, a.C / 8, total);
    return hipGetLastError();
}

hipError_t launch_softmax_ce_bwd(const void *logits, const void *labels, int N, int classes, void *gz, hipStream_t stream) {
    if (!logits || !labels || !gz || N <= 0 || classes <= 0) return hipErrorInvalidValue;
    bops::softmax_ce_bwd_kernel<<<dim3((unsigned)((N + 3) / 4)), dim3(256), 0, stream>>>(
        static_cast<const uint16_t *>(logits), static_cast<const long long *>(labels), N, classes,
        static_cast<uint16_t *>(gz));
    return hipGetLastError();
}

// Classifier: x [N][Cin], w [Cout][Cin] bf16, gy [N][Cout] bf16; gx [N][Cin] bf16 (or null),
// gw fp32 [Cout*Cin + Cout] (weights, then bias; or null).  Cin a multiple of 8.
hipError_t launch_dense_bwd(const void *x, const void *w, const float *scale, const void *gy, void *gx, float *gw,
                            int N, int Cin, int Cout, hipStream_t stream) {
    if (!w || !scale || !gy || N <= 0 || Cin <= 0 || Cout <= 0 || Cin % 8) return hipErrorInvalidValue;
    if (gx) {
        const long long t = (long long)N * ((Cin / 8 + 31) / 32);
        bops::dense_bwd_data_kernel<<<dim3((unsigned)t), dim3(256), 0, stream>>>(
            static_cast<const uint16_t *>(gy), w, scale, gx, N, Cin, Cout);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    if (gw) {
        if (!x) return hipErrorInvalidValue;
        const long long t = (long long)Cout * (Cin / 8);
        bops::dense_bwd_weight_kernel<<<dim3((unsigned)((t + 255) / 256)), dim3(256), 0, stream>>>(
            static_cast<const uint16_t *>(gy), x, scale, gw, N, Cin, Cout);
        return hipGetLastError();
    }
    return hipSuccess;
}

}  // namespace delta
