// Operators of the operator-granular graph (the granularity of the paper's cost table, Sec. 5.5:
// ConvForward, BNForward, ... are separate managed tensors) for gfx950, bf16 NHWC:
//   training-mode batch normalisation   y = gamma (x - mu_B) / sqrt(var_B + eps) + beta
//   ReLU                                y = max(x, 0)
//   residual add                        y = x + r
// All three are HBM-bound (16 bytes per lane).  Batch normalisation reads x twice (statistics,
// then normalise) and writes y once:
//   bn_stats_kernel     each workgroup sums (x - K_c) and (x - K_c)^2 over its block of rows, per
//                       channel, fp32, K_c = x[0, c] (shifted data: no cancellation when the mean is
//                       far from 0); lanes own 8 channels, the row-parallel lanes of a workgroup are
//                       combined through LDS in row order (all lanes share that work); partial sums to a
//                       scratch buffer
//   bn_finalize_kernel  one thread per channel adds the partials in block order (double), forms
//                       mean, biased variance and a = gamma / sqrt(var + eps)
//   bn_apply_kernel     y = a_c (x - mean_c) + beta_c   (centred first: no cancellation of two large products)
// No atomics: the result is a fixed function of the input (recomputation is bit-identical).
// Backward of the batch normalisation (chain rule through the three lines above, collapsed):
//   gx = a_c (gy - mean(gy)_c - (x - mu_c) S_c / ((var_c + eps) M)),   S_c = sum gy (x - mu_c)
//   dgamma_c = S_c / sqrt(var_c + eps),   dbeta_c = sum gy
// reads x and gy twice and writes gx once, the floor without stored statistics (x has to be read
// for S_c in any case):
//   bn_bwd_stats_kernel     sums of (x - K_c), (x - K_c)^2, gy, gy (x - K_c) per channel and workgroup
//   bn_bwd_finalize_kernel  adds the partials (double), forms a, mu, mean(gy), S/((var + eps) M) and
//                           the two parameter gradients
//   bn_bwd_apply_kernel     gx from x, gy and the four per-channel factors
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kernels.hpp"

namespace delta {
namespace ops {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

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

// NT = blockDim.x threads (256 or 1024): CH = min(chunks, NT) chunk columns per pass, RS = NT / CH rows
// in parallel.  partial: [gridDim.x][2][C] floats.
__global__ __launch_bounds__(1024) void bn_stats_kernel(const unsigned char *x, float *partial, long long M, int C,
                                                       long long rows_per_block, int CH, int RS) {
    extern __shared__ __align__(16) float red[];                 // [RS][CH][16]
    const int chunks = C / 8;
    const int t = threadIdx.x;
    const int ck0 = t % CH, rsub = t / CH;
    const long long r0 = (long long)blockIdx.x * rows_per_block;
    long long r1 = r0 + rows_per_block;
    if (r1 > M) r1 = M;
    for (int cg = 0; cg < chunks; cg += CH) {
        const int ck = cg + ck0;
        const bool live = ck < chunks && rsub < RS;
        float s1[8], s2[8], k[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) s1[e] = s2[e] = 0.f;
        if (live) {
            unpack8(*reinterpret_cast<const u32x4 *>(x + (size_t)ck * 16), k);      // row 0: the shift
            long long r = r0 + rsub;
            for (; r + 3LL * RS < r1; r += 4LL * RS) {            // four rows in flight per lane
                u32x4 raw[4];
#pragma unroll
                for (int u = 0; u < 4; ++u)
                    raw[u] = *reinterpret_cast<const u32x4 *>(x + ((size_t)(r + (long long)u * RS) * chunks + ck) * 16);
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    float v[8];
                    unpack8(raw[u], v);
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        const float d = v[e] - k[e];
                        s1[e] += d;
                        s2[e] += d * d;
                    }
                }
            }
            for (; r < r1; r += RS) {
                float v[8];
                unpack8(*reinterpret_cast<const u32x4 *>(x + ((size_t)r * chunks + ck) * 16), v);
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const float d = v[e] - k[e];
                    s1[e] += d;
                    s2[e] += d * d;
                }
            }
        }
        if (cg) __syncthreads();                                 // the previous pass's reads are done
        if (rsub < RS) {
            float *p = red + ((size_t)rsub * CH + ck0) * 16;
#pragma unroll
            for (int e = 0; e < 8; ++e) { p[e] = s1[e]; p[8 + e] = s2[e]; }
        }
        __syncthreads();
        // every thread adds the RS row-parallel contributions of some of the CH x 16 sums, in row order
        for (int o = t; o < CH * 16; o += (int)blockDim.x) {
            const int c0 = o >> 4, q = o & 15;
            if (cg + c0 >= chunks) continue;
            float a = 0.f;
            for (int j = 0; j < RS; ++j) a += red[(size_t)j * CH * 16 + o];
            partial[((size_t)blockIdx.x * 2 + (q >> 3)) * C + (cg + c0) * 8 + (q & 7)] = a;
        }
    }
}

// ab: [2][C]: a, then the mean.  A workgroup of 1024 threads takes CL = 1 << cl_bits channels (64, or
// 16 when there are few channels, so that more workgroups and shorter chains share the partials):
// thread (channel lane, group g of G = 1024 / CL) adds the partials of blocks g, g + G, ...
// (coalesced over the channels, eight loads in flight), the G groups are then added in order
// through LDS.
__global__ __launch_bounds__(1024) void bn_finalize_kernel(const unsigned char *x, const float *partial, const float *gamma,
                                                           const float *beta, float *ab, long long M, int C, int blocks,
                                                           float eps, int cl_bits) {
    __shared__ double red[2][1024];                              // [sum][group][channel lane]
    const int CL = 1 << cl_bits, G = 1024 >> cl_bits;
    const int cl = threadIdx.x & (CL - 1), grp = threadIdx.x >> cl_bits;
    const int c = blockIdx.x * CL + cl;
    double s1 = 0.0, s2 = 0.0;
    if (c < C) {
        int b = grp;
        for (; b + 7 * G < blocks; b += 8 * G) {
            float p1[8], p2[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                p1[u] = partial[(size_t)(b + G * u) * 2 * C + c];
                p2[u] = partial[(size_t)(b + G * u) * 2 * C + C + c];
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) { s1 += (double)p1[u]; s2 += (double)p2[u]; }
        }
        for (; b < blocks; b += G) {
            s1 += (double)partial[(size_t)b * 2 * C + c];
            s2 += (double)partial[(size_t)b * 2 * C + C + c];
        }
    }
    red[0][threadIdx.x] = s1;
    red[1][threadIdx.x] = s2;
    __syncthreads();
    if (grp != 0 || c >= C) return;
    s1 = s2 = 0.0;
    for (int g = 0; g < G; ++g) { s1 += red[0][g * CL + cl]; s2 += red[1][g * CL + cl]; }
    const double k = (double)__uint_as_float((uint32_t)reinterpret_cast<const uint16_t *>(x)[c] << 16);
    const double md = s1 / (double)M;
    double var = s2 / (double)M - md * md;
    if (var < 0.0) var = 0.0;
    const double mean = k + md;
    ab[c] = (float)((double)gamma[c] / sqrt(var + (double)eps));
    ab[C + c] = (float)mean;
    (void)beta;
}

__global__ __launch_bounds__(256) void bn_apply_kernel(const u32x4 *__restrict__ x, u32x4 *__restrict__ y,
                                                       const float *__restrict__ ab, const float *__restrict__ beta, int C,
                                                       size_t n16) {
    const int chunks = C / 8;
    const size_t step = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += step) {
        const int ck = (int)(i % chunks);
        float v[8];
        unpack8(x[i], v);
        const f32x4 a0 = *reinterpret_cast<const f32x4 *>(ab + ck * 8), a1 = *reinterpret_cast<const f32x4 *>(ab + ck * 8 + 4);
        const f32x4 m0 = *reinterpret_cast<const f32x4 *>(ab + C + ck * 8), m1 = *reinterpret_cast<const f32x4 *>(ab + C + ck * 8 + 4);
        const f32x4 b0 = *reinterpret_cast<const f32x4 *>(beta + ck * 8), b1 = *reinterpret_cast<const f32x4 *>(beta + ck * 8 + 4);
        u32x4 o;
        o.x = pack2((v[0] - m0.x) * a0.x + b0.x, (v[1] - m0.y) * a0.y + b0.y);
        o.y = pack2((v[2] - m0.z) * a0.z + b0.z, (v[3] - m0.w) * a0.w + b0.w);
        o.z = pack2((v[4] - m1.x) * a1.x + b1.x, (v[5] - m1.y) * a1.y + b1.y);
        o.w = pack2((v[6] - m1.z) * a1.z + b1.z, (v[7] - m1.w) * a1.w + b1.w);
        y[i] = o;
    }
}


// Backward statistics.  Same decomposition as bn_stats_kernel; partial: [gridDim.x][4][C] floats
// (sum d, sum d^2, sum g, sum g d with d = x - K_c).  red: [RS][CH][32].
__global__ __launch_bounds__(1024) void bn_bwd_stats_kernel(const unsigned char *x, const unsigned char *g, float *partial,
                                                           long long M, int C, long long rows_per_block, int CH, int RS) {
    extern __shared__ __align__(16) float red[];
    const int chunks = C / 8;
    const int t = threadIdx.x;
    const int ck0 = t % CH, rsub = t / CH;
    const long long r0 = (long long)blockIdx.x * rows_per_block;
    long long r1 = r0 + rows_per_block;
    if (r1 > M) r1 = M;
    for (int cg = 0; cg < chunks; cg += CH) {
        const int ck = cg + ck0;
        const bool live = ck < chunks && rsub < RS;
        float s1[8], s2[8], s3[8], s4[8], k[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) s1[e] = s2[e] = s3[e] = s4[e] = 0.f;
        if (live) {
            unpack8(*reinterpret_cast<const u32x4 *>(x + (size_t)ck * 16), k);
            long long r = r0 + rsub;
            for (; r + 3LL * RS < r1; r += 4LL * RS) {            // four rows of both tensors in flight per lane
                u32x4 rx[4], rg[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const size_t at = ((size_t)(r + (long long)u * RS) * chunks + ck) * 16;
                    rx[u] = *reinterpret_cast<const u32x4 *>(x + at);
                    rg[u] = *reinterpret_cast<const u32x4 *>(g + at);
                }
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    float v[8], w[8];
                    unpack8(rx[u], v);
                    unpack8(rg[u], w);
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        const float d = v[e] - k[e];
                        s1[e] += d;
                        s2[e] += d * d;
                        s3[e] += w[e];
                        s4[e] += w[e] * d;
                    }
                }
            }
            for (; r < r1; r += RS) {
                const size_t at = ((size_t)r * chunks + ck) * 16;
                float v[8], w[8];
                unpack8(*reinterpret_cast<const u32x4 *>(x + at), v);
                unpack8(*reinterpret_cast<const u32x4 *>(g + at), w);
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const float d = v[e] - k[e];
                    s1[e] += d;
                    s2[e] += d * d;
                    s3[e] += w[e];
                    s4[e] += w[e] * d;
                }
            }
        }
        if (cg) __syncthreads();
        if (rsub < RS) {
            float *p = red + ((size_t)rsub * CH + ck0) * 32;
#pragma unroll
            for (int e = 0; e < 8; ++e) { p[e] = s1[e]; p[8 + e] = s2[e]; p[16 + e] = s3[e]; p[24 + e] = s4[e]; }
        }
        __syncthreads();
        for (int o = t; o < CH * 32; o += (int)blockDim.x) {     // as in bn_stats_kernel
            const int c0 = o >> 5, q = o & 31;
            if (cg + c0 >= chunks) continue;
            float a = 0.f;
            for (int j = 0; j < RS; ++j) a += red[(size_t)j * CH * 32 + o];
            partial[((size_t)blockIdx.x * 4 + (q >> 3)) * C + (cg + c0) * 8 + (q & 7)] = a;
        }
    }
}

// coef: [4][C]: a, mean, mean(gy), S / ((var + eps) M).  gw (may be null): dgamma [C], then dbeta [C].
// Decomposition as in bn_finalize_kernel.
__global__ __launch_bounds__(1024) void bn_bwd_finalize_kernel(const unsigned char *x, const float *partial,
                                                               const float *gamma, float *coef, float *gw, long long M,
                                                               int C, int blocks, float eps, int cl_bits) {
    __shared__ double red[4][1024];
    const int CL = 1 << cl_bits, G = 1024 >> cl_bits;
    const int cl = threadIdx.x & (CL - 1), grp = threadIdx.x >> cl_bits;
    const int c = blockIdx.x * CL + cl;
    double s[4] = {0.0, 0.0, 0.0, 0.0};
    if (c < C) {
        int b = grp;
        for (; b + 3 * G < blocks; b += 4 * G) {
            float p[4][4];
#pragma unroll
            for (int u = 0; u < 4; ++u)
#pragma unroll
                for (int q = 0; q < 4; ++q) p[u][q] = partial[((size_t)(b + G * u) * 4 + q) * C + c];
#pragma unroll
            for (int u = 0; u < 4; ++u)
#pragma unroll
                for (int q = 0; q < 4; ++q) s[q] += (double)p[u][q];
        }
        for (; b < blocks; b += G)
#pragma unroll
            for (int q = 0; q < 4; ++q) s[q] += (double)partial[((size_t)b * 4 + q) * C + c];
    }
#pragma unroll
    for (int q = 0; q < 4; ++q) red[q][threadIdx.x] = s[q];
    __syncthreads();
    if (grp != 0 || c >= C) return;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        s[q] = 0.0;
        for (int g = 0; g < G; ++g) s[q] += red[q][g * CL + cl];
    }
    const double k = (double)__uint_as_float((uint32_t)reinterpret_cast<const uint16_t *>(x)[c] << 16);
    const double md = s[0] / (double)M;
    double var = s[1] / (double)M - md * md;
    if (var < 0.0) var = 0.0;
    const double ve = var + (double)eps;
    const double S = s[3] - md * s[2];                           // sum gy (x - mean)
    coef[c] = (float)((double)gamma[c] / sqrt(ve));
    coef[C + c] = (float)(k + md);
    coef[2 * C + c] = (float)(s[2] / (double)M);
    coef[3 * C + c] = (float)(S / (ve * (double)M));
    if (gw) {
        gw[c] = (float)(S / sqrt(ve));
        gw[C + c] = (float)s[2];
    }
}

__global__ __launch_bounds__(256) void bn_bwd_apply_kernel(const u32x4 *__restrict__ x, const u32x4 *__restrict__ g,
                                                           u32x4 *__restrict__ gx, const float *__restrict__ coef, int C,
                                                           size_t n16) {
    const int chunks = C / 8;
    const size_t step = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += step) {
        const int ck = (int)(i % chunks);
        float v[8], w[8], o[8];
        unpack8(x[i], v);
        unpack8(g[i], w);
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const f32x4 a = *reinterpret_cast<const f32x4 *>(coef + ck * 8 + 4 * h);
            const f32x4 m = *reinterpret_cast<const f32x4 *>(coef + C + ck * 8 + 4 * h);
            const f32x4 c1 = *reinterpret_cast<const f32x4 *>(coef + 2 * C + ck * 8 + 4 * h);
            const f32x4 c2 = *reinterpret_cast<const f32x4 *>(coef + 3 * C + ck * 8 + 4 * h);
#pragma unroll
            for (int e = 0; e < 4; ++e) o[4 * h + e] = a[e] * (w[4 * h + e] - c1[e] - (v[4 * h + e] - m[e]) * c2[e]);
        }
        u32x4 r;
        r.x = pack2(o[0], o[1]); r.y = pack2(o[2], o[3]); r.z = pack2(o[4], o[5]); r.w = pack2(o[6], o[7]);
        gx[i] = r;
    }
}

// y = max(x, 0): a negative bf16 has its sign bit set (NaN passes through, as in the fused epilogue)
__global__ __launch_bounds__(256) void relu_kernel(const u32x4 *__restrict__ x, u32x4 *__restrict__ y, size_t n16) {
    const size_t step = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += step) {
        u32x4 v = x[i];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const uint32_t lo = v[e] & 0xFFFFu, hi = v[e] >> 16;
            const bool nlo = (lo & 0x8000u) && (lo & 0x7FFFu) <= 0x7F80u;    // negative, not NaN
            const bool nhi = (hi & 0x8000u) && (hi & 0x7FFFu) <= 0x7F80u;
            v[e] = (nlo ? 0u : lo) | ((nhi ? 0u : hi) << 16);
        }
        y[i] = v;
    }
}

__global__ __launch_bounds__(256) void add_kernel(const u32x4 *__restrict__ x, const u32x4 *__restrict__ r,
                                                  u32x4 *__restrict__ y, size_t n16) {
    const size_t step = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += step) {
        const u32x4 a = x[i], b = r[i];
        u32x4 o;
#pragma unroll
        for (int e = 0; e < 4; ++e) o[e] = pack2(lo16(a[e]) + lo16(b[e]), hi16(a[e]) + hi16(b[e]));
        y[i] = o;
    }
}

static unsigned stream_blocks(size_t n16) {
    size_t blocks = (n16 + 255) / 256;
    return (unsigned)(blocks > 256 * 16 ? 256 * 16 : blocks);
}

}  // namespace ops

const char *bn_train_check(const void *x, const void *y, const float *gamma, const float *beta, long long M, int C,
                           int bf16) {
    if (!bf16) return "batch normalisation with batch statistics is bf16 only";
    if (M <= 0 || C <= 0 || C % 8 || C > 8192) return "channels must be a multiple of 8, at most 8192";
    if (!x || !y || !gamma || !beta || (((uintptr_t)x | (uintptr_t)y | (uintptr_t)gamma | (uintptr_t)beta) & 15))
        return "pointers must be non-null and 16-byte aligned";
    return nullptr;
}

size_t bn_train_scratch_bytes() { return (size_t)16 << 20; }     // partial sums + the 2 x C factors

// Large tensors take workgroups of 1024 threads, a quarter as many: the same lanes share the rows, and
// the finalize kernel, which runs on a nearly empty chip, reads a quarter of the partial sums.
static void stats_shape(int chunks, long long &blocks, int &NT, int &CH, int &RS) {
    if (blocks < 256) return;
    NT = 1024;
    blocks = (blocks + 3) / 4;
    CH = chunks < NT ? chunks : NT;
    RS = NT / CH;
}

// What the forward needs at most: the 2 x C factors and 64 workgroups' partial sums at C = 8192 (wider
// tensors take fewer workgroups, see the cap below), so that a buffer of this size never changes the
// decomposition - and with it the bits of the result - against a larger one.
size_t bn_train_fwd_scratch_bytes() { return ((size_t)4 << 20) + ((size_t)64 << 10); }

// scratch: device, scratch_bytes (>= bn_train_fwd_scratch_bytes()) bytes, 16-byte aligned.
hipError_t launch_bn_train(const void *x, void *y, const float *gamma, const float *beta, long long M, int C, float eps,
                           int bf16, void *scratch, size_t scratch_bytes, hipStream_t stream) {
    if (bn_train_check(x, y, gamma, beta, M, C, bf16) || !scratch || ((uintptr_t)scratch & 15) ||
        scratch_bytes < bn_train_fwd_scratch_bytes())
        return hipErrorInvalidValue;
    const int chunks = C / 8;
    int NT = 256;
    int CH = chunks < NT ? chunks : NT;
    int RS = NT / CH;
    float *ab = static_cast<float *>(scratch);                   // [2][C]
    float *partial = ab + 2 * (size_t)C;
    const size_t room = (scratch_bytes - 2 * (size_t)C * 4) / ((size_t)2 * C * 4);
    long long blocks = (M + (long long)RS * 4 - 1) / ((long long)RS * 4);    // at least 4 rows per lane
    // fewer partials for wide tensors: the finalize kernel reads blocks x 2 x C floats
    long long cap = 262144 / C;
    cap = cap < 64 ? 64 : (cap > 2048 ? 2048 : cap);
    if (blocks > cap) blocks = cap;
    if (blocks > (long long)room) blocks = (long long)room;
    if (blocks < 1) return hipErrorInvalidValue;
    stats_shape(chunks, blocks, NT, CH, RS);
    const long long rpb = (M + blocks - 1) / blocks;
    blocks = (M + rpb - 1) / rpb;
    const size_t lds = (size_t)RS * CH * 16 * 4;
    static const hipError_t lds_ok = hipFuncSetAttribute(reinterpret_cast<const void *>(ops::bn_stats_kernel),
                                                         hipFuncAttributeMaxDynamicSharedMemorySize, 1024 * 16 * 4);
    if (lds_ok != hipSuccess) return lds_ok;
    ops::bn_stats_kernel<<<dim3((unsigned)blocks), dim3((unsigned)NT), lds, stream>>>(static_cast<const unsigned char *>(x), partial,
                                                                            M, C, rpb, CH, RS);
    const int cl_bits = C <= 512 ? 4 : 6;
    ops::bn_finalize_kernel<<<dim3((unsigned)((C + (1 << cl_bits) - 1) >> cl_bits)), dim3(1024), 0, stream>>>(
        static_cast<const unsigned char *>(x), partial, gamma, beta, ab, M, C, (int)blocks, eps, cl_bits);
    const size_t n16 = (size_t)M * chunks;
    ops::bn_apply_kernel<<<dim3(ops::stream_blocks(n16)), dim3(256), 0, stream>>>(
        static_cast<const ops::u32x4 *>(x), static_cast<ops::u32x4 *>(y), ab, beta, C, n16);
    return hipGetLastError();
}

// Backward of launch_bn_train.  gw: device fp32 [2][C] (dgamma, dbeta) or null.  Same scratch.
hipError_t launch_bn_train_bwd(const void *x, const void *gy, void *gx, const float *gamma, float *gw, long long M, int C,
                               float eps, int bf16, void *scratch, hipStream_t stream) {
    if (bn_train_check(x, gx, gamma, gamma, M, C, bf16) || !gy || ((uintptr_t)gy & 15) || ((uintptr_t)gw & 15) || !scratch ||
        ((uintptr_t)scratch & 15))
        return hipErrorInvalidValue;
    const int chunks = C / 8;
    int NT = 256;
    int CH = chunks < NT ? chunks : NT;
    int RS = NT / CH;
    float *coef = static_cast<float *>(scratch);                 // [4][C]
    float *partial = coef + 4 * (size_t)C;
    const size_t room = (bn_train_scratch_bytes() - 4 * (size_t)C * 4) / ((size_t)4 * C * 4);
    long long blocks = (M + (long long)RS * 4 - 1) / ((long long)RS * 4);
    long long cap = 262144 / C;                                  // 1024 workgroups fill the chip four wavefronts deep
    cap = cap < 64 ? 64 : (cap > 1024 ? 1024 : cap);
    if (blocks > cap) blocks = cap;
    if (blocks > (long long)room) blocks = (long long)room;
    if (blocks < 1) return hipErrorInvalidValue;
    stats_shape(chunks, blocks, NT, CH, RS);
    const long long rpb = (M + blocks - 1) / blocks;
    blocks = (M + rpb - 1) / rpb;
    const size_t lds = (size_t)RS * CH * 32 * 4;
    static const hipError_t lds_ok = hipFuncSetAttribute(reinterpret_cast<const void *>(ops::bn_bwd_stats_kernel),
                                                         hipFuncAttributeMaxDynamicSharedMemorySize, 1024 * 32 * 4);
    if (lds_ok != hipSuccess) return lds_ok;
    ops::bn_bwd_stats_kernel<<<dim3((unsigned)blocks), dim3((unsigned)NT), lds, stream>>>(
        static_cast<const unsigned char *>(x), static_cast<const unsigned char *>(gy), partial, M, C, rpb, CH, RS);
    const int cl_bits = C <= 512 ? 4 : 6;
    ops::bn_bwd_finalize_kernel<<<dim3((unsigned)((C + (1 << cl_bits) - 1) >> cl_bits)), dim3(1024), 0, stream>>>(
        static_cast<const unsigned char *>(x), partial, gamma, coef, gw, M, C, (int)blocks, eps, cl_bits);
    const size_t n16 = (size_t)M * chunks;
    ops::bn_bwd_apply_kernel<<<dim3(ops::stream_blocks(n16)), dim3(256), 0, stream>>>(
        static_cast<const ops::u32x4 *>(x), static_cast<const ops::u32x4 *>(gy), static_cast<ops::u32x4 *>(gx), coef, C, n16);
    return hipGetLastError();
}

hipError_t launch_relu(const void *x, void *y, size_t bytes, int bf16, hipStream_t stream) {
    if (!bf16 || !x || !y || bytes % 16 || (((uintptr_t)x | (uintptr_t)y) & 15)) return hipErrorInvalidValue;
    if (bytes == 0) return hipSuccess;
    ops::relu_kernel<<<dim3(ops::stream_blocks(bytes / 16)), dim3(256), 0, stream>>>(
        static_cast<const ops::u32x4 *>(x), static_cast<ops::u32x4 *>(y), bytes / 16);
    return hipGetLastError();
}

hipError_t launch_add(const void *x, const void *r, void *y, size_t bytes, int bf16, hipStream_t stream) {
    if (!bf16 || !x || !r || !y || bytes % 16 || (((uintptr_t)x | (uintptr_t)r | (uintptr_t)y) & 15)) return hipErrorInvalidValue;
    if (bytes == 0) return hipSuccess;
    ops::add_kernel<<<dim3(ops::stream_blocks(bytes / 16)), dim3(256), 0, stream>>>(
        static_cast<const ops::u32x4 *>(x), static_cast<const ops::u32x4 *>(r), static_cast<ops::u32x4 *>(y), bytes / 16);
    return hipGetLastError();
}

}  // namespace delta
