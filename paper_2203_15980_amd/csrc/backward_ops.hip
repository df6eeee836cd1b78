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
// One thread: 8 channels of one INPUT pixel.  For every window that contains the pixel, the
// window is scanned in the forward's order (r, then s, padding skipped); the pixel receives the
// window's gradient where it is the first maximal element.  Sums in window order (p, then q), fp32.
__global__ __launch_bounds__(256) void maxpool_bwd_kernel(PoolArgs a, const void *gy, void *gx, long long total) {
    const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= total) return;
    const int chunks = a.C / 8;
    const int ck = (int)(idx % chunks);
    long long pix = idx / chunks;
    const int w = (int)(pix % a.W);
    pix /= a.W;
    const int h = (int)(pix % a.H);
    const int n = (int)(pix / a.H);
    const unsigned char *xg = static_cast<const unsigned char *>(a.x);
    const unsigned char *gg = static_cast<const unsigned char *>(gy);
    float mine[8], acc[8];
    unpack8(*reinterpret_cast<const u32x4 *>(xg + (size_t)idx * 16), mine);
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = 0.f;
    // windows (p, q) with p*stride - pad <= h <= p*stride - pad + R - 1
    int p_lo = h + a.pad - a.R + 1;
    p_lo = p_lo <= 0 ? 0 : (p_lo + a.stride - 1) / a.stride;
    int p_hi = (h + a.pad) / a.stride;
    if (p_hi > a.P - 1) p_hi = a.P - 1;
    int q_lo = w + a.pad - a.S + 1;
    q_lo = q_lo <= 0 ? 0 : (q_lo + a.stride - 1) / a.stride;
    int q_hi = (w + a.pad) / a.stride;
    if (q_hi > a.Q - 1) q_hi = a.Q - 1;
    for (int p = p_lo; p <= p_hi; ++p)
        for (int q = q_lo; q <= q_hi; ++q) {
            // is (h, w) the first maximum of window (p, q)?  An element before it in scan order
            // beats it when it is >=, one after it only when it is >.
            bool first[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) first[e] = true;
            for (int r = 0; r < a.R; ++r) {
                const int hh = p * a.stride + r - a.pad;
                if ((unsigned)hh >= (unsigned)a.H) continue;
                for (int s = 0; s < a.S; ++s) {
                    const int ww = q * a.stride + s - a.pad;
                    if ((unsigned)ww >= (unsigned)a.W || (hh == h && ww == w)) continue;
                    float v[8];
                    unpack8(*reinterpret_cast<const u32x4 *>(
                                xg + ((((size_t)n * a.H + hh) * a.W + ww) * chunks + ck) * 16), v);
                    const bool before = hh < h || (hh == h && ww < w);
#pragma unroll
                    for (int e = 0; e < 8; ++e)
                        if (before ? v[e] >= mine[e] : v[e] > mine[e]) first[e] = false;
                }
            }
            float g[8];
            unpack8(*reinterpret_cast<const u32x4 *>(gg + ((((size_t)n * a.P + p) * a.Q + q) * chunks + ck) * 16), g);
#pragma unroll
            for (int e = 0; e < 8; ++e)
                if (first[e]) acc[e] += g[e];
        }
    *reinterpret_cast<u32x4 *>(static_cast<unsigned char *>(gx) + (size_t)idx * 16) = pack8(acc);
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
// gx[n][c] = sum_k gy[n][k] * scale_k * w[k][c]: one thread per (image, 8 input channels); k ascending.
__global__ __launch_bounds__(256) void dense_bwd_data_kernel(const uint16_t *gy, const void *w, const float *scale,
                                                             void *gx, int N, int Cin, int Cout) {
    const int chunks = Cin / 8;
    const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (long long)N * chunks) return;
    const int ck = (int)(idx % chunks), n = (int)(idx / chunks);
    float acc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = 0.f;
    const unsigned char *wg = static_cast<const unsigned char *>(w);
    for (int k = 0; k < Cout; ++k) {
        const float g = __uint_as_float((uint32_t)gy[(size_t)n * Cout + k] << 16) * scale[k];
        float v[8];
        unpack8(*reinterpret_cast<const u32x4 *>(wg + ((size_t)k * chunks + ck) * 16), v);
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] += g * v[e];
    }
    *reinterpret_cast<u32x4 *>(static_cast<unsigned char *>(gx) + (size_t)idx * 16) = pack8(acc);
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

hipError_t launch_maxpool_bwd(const PoolArgs &a, const void *gy, void *gx, hipStream_t stream) {
    if (pool_check(a, false) || !a.bf16 || !gy || !gx) return hipErrorInvalidValue;
    const long long total = (long long)a.N * a.H * a.W * (a.C / 8);
    const long long blocks = (total + 255) / 256;
    if (blocks <= 0 || blocks > 0x7FFFFFFFLL) return hipErrorInvalidValue;
    bops::maxpool_bwd_kernel<<<dim3((unsigned)blocks), dim3(256), 0, stream>>>(a, gy, gx, total);
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
        const long long t = (long long)N * (Cin / 8);
        bops::dense_bwd_data_kernel<<<dim3((unsigned)((t + 255) / 256)), dim3(256), 0, stream>>>(
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
