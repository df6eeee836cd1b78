// Layer normalisation over the channel axis of a [rows, C] bf16 tensor for gfx950:
//   y = (x - mean) / sqrt(var + eps) * gamma + beta     (biased variance, fp32 statistics)
// One operator of a transformer layer's recomputation segment (the paper evaluates BERT-base,
// Sec. 5.2).  HBM-bound: one read and one write of the tensor.  A wavefront owns a row and keeps
// it in registers (16 bytes = 8 channels per lane and round, up to 4 rounds: C <= 2048), so the
// row is read once; mean first, then the variance of the centred values (no cancellation), both
// reduced with a fixed butterfly across the 64 lanes.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kernels.hpp"

namespace delta {
namespace tops {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

static constexpr int kRounds = 4;               // 8 channels x 64 lanes x 4 rounds = 2048 channels
static constexpr int kRowsPerBlock = 4;

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, 64);
    return v;
}

__device__ __forceinline__ uint32_t pack2(float lo, float hi) {
    const f32x2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

__global__ __launch_bounds__(kRowsPerBlock * 64) void layernorm_kernel(const unsigned char *x, unsigned char *y,
                                                                       const float *gamma, const float *beta,
                                                                       long long rows, int C, float eps) {
    const int lane = threadIdx.x & 63;
    const long long row = (long long)blockIdx.x * kRowsPerBlock + (threadIdx.x >> 6);
    if (row >= rows) return;
    const int chunks = C / 8;
    const unsigned char *xr = x + (size_t)row * C * 2;
    float v[kRounds][8];
    float sum = 0.f;
#pragma unroll
    for (int r = 0; r < kRounds; ++r) {
        const int ck = lane + 64 * r;
        u32x4 raw = {0u, 0u, 0u, 0u};
        if (ck < chunks) raw = *reinterpret_cast<const u32x4 *>(xr + (size_t)ck * 16);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            v[r][2 * e] = __uint_as_float(raw[e] << 16);
            v[r][2 * e + 1] = __uint_as_float(raw[e] & 0xFFFF0000u);
            sum += v[r][2 * e] + v[r][2 * e + 1];
        }
    }
    const float mean = wave_sum(sum) / (float)C;
    float sq = 0.f;
#pragma unroll
    for (int r = 0; r < kRounds; ++r) {
        const bool live = lane + 64 * r < chunks;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            v[r][e] -= mean;
            sq += live ? v[r][e] * v[r][e] : 0.f;
        }
    }
    const float rstd = 1.0f / sqrtf(wave_sum(sq) / (float)C + eps);
    unsigned char *yr = y + (size_t)row * C * 2;
#pragma unroll
    for (int r = 0; r < kRounds; ++r) {
        const int ck = lane + 64 * r;
        if (ck >= chunks) continue;
        const f32x4 g0 = *reinterpret_cast<const f32x4 *>(gamma + ck * 8), g1 = *reinterpret_cast<const f32x4 *>(gamma + ck * 8 + 4);
        const f32x4 b0 = *reinterpret_cast<const f32x4 *>(beta + ck * 8), b1 = *reinterpret_cast<const f32x4 *>(beta + ck * 8 + 4);
        u32x4 o;
        o.x = pack2(v[r][0] * rstd * g0.x + b0.x, v[r][1] * rstd * g0.y + b0.y);
        o.y = pack2(v[r][2] * rstd * g0.z + b0.z, v[r][3] * rstd * g0.w + b0.w);
        o.z = pack2(v[r][4] * rstd * g1.x + b1.x, v[r][5] * rstd * g1.y + b1.y);
        o.w = pack2(v[r][6] * rstd * g1.z + b1.z, v[r][7] * rstd * g1.w + b1.w);
        *reinterpret_cast<u32x4 *>(yr + (size_t)ck * 16) = o;
    }
}

}  // namespace tops

const char *layernorm_check(const void *x, const void *y, const float *gamma, const float *beta, long long rows, int C,
                            int bf16) {
    if (!bf16) return "layer normalisation is bf16 only";
    if (rows <= 0 || C <= 0 || C % 8 || C > tops::kRounds * 512) return "channels must be a multiple of 8, at most 2048";
    if (!x || !y || !gamma || !beta || (((uintptr_t)x | (uintptr_t)y | (uintptr_t)gamma | (uintptr_t)beta) & 15))
        return "pointers must be non-null and 16-byte aligned";
    if ((rows + tops::kRowsPerBlock - 1) / tops::kRowsPerBlock > 0x7FFFFFFFLL) return "too many rows";
    return nullptr;
}

hipError_t launch_layernorm(const void *x, void *y, const float *gamma, const float *beta, long long rows, int C,
                            float eps, int bf16, hipStream_t stream) {
    if (layernorm_check(x, y, gamma, beta, rows, C, bf16)) return hipErrorInvalidValue;
    const unsigned blocks = (unsigned)((rows + tops::kRowsPerBlock - 1) / tops::kRowsPerBlock);
    tops::layernorm_kernel<<<dim3(blocks), dim3(tops::kRowsPerBlock * 64), 0, stream>>>(
        static_cast<const unsigned char *>(x), static_cast<unsigned char *>(y), gamma, beta, rows, C, eps);
    return hipGetLastError();
}

}  // namespace delta
