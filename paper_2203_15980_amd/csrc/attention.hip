// Fused multi-head self-attention (forward) for gfx950: ctx = softmax(q k^T / sqrt(d)) v per head,
// the scores and probabilities never leave the chip.
//
// In DELTA's terms this is one operator of a transformer layer's recomputation segment (the paper
// evaluates BERT-base, Sec. 5.2); fusing it removes the two S x S tensors per head that dominate
// an encoder layer's activation memory, which is the same trade DELTA makes at run time
// (regenerate instead of keep), taken at kernel-design time.
//
// Layout.  qkv [N, S, 3H] bf16: q = columns [0,H), k = [H,2H), v = [2H,3H); head h owns columns
// [64h, 64h+64) of each (d = 64).  ctx [N, S, H] bf16.
//
// A workgroup (8 wavefronts) takes one (image, head) and a block of 256 queries; a wavefront owns
// 32 queries.  K and V of the head stream through LDS in blocks of 64 keys, two buffers; block
// b + 1 waits in registers (requested a block earlier) while block b is multiplied, so only the
// first block's latency is exposed (staging all 512 keys up front cost 20 of 68 us at batch 32 x
// 512).  Everything is computed TRANSPOSED so that a lane owns one query:
//   S^T tile (32 keys x 32 queries) = K tile . Q^T        A = K rows from LDS (b128), B = Q from registers
//   lane l holds query l % 32 and keys 8*e4 + 4*(l/32) + e of the tile: the softmax statistics of
//   a query (running maximum, running sum) are per-lane scalars; the two half-waves see disjoint
//   keys and exchange their maxima with one permlane32 swap per block of 64 keys.
//   O^T (64 d x 32 queries) += V^T . P^T                  A = V^T through the LDS transpose read
//   (ds_read_b64_tr_b16: V lies [key][d] in LDS as in memory), B = P straight from the S^T
//   accumulators rounded to bf16: accumulator registers (e4 in {2j, 2j+1}) of a lane are exactly
//   the 8 reduction slots of step j, if the A operand enumerates the keys in the same order
//   (keys 16j + 4*(l/32) + e and 16j + 8 + 4*(l/32) + e) - the order of a reduction is free.
// Online softmax over the 64-key blocks (fp32; the maximum is taken of the raw scores, the scale
// and the subtraction are one fma in front of exp2).  P is rounded to
// bf16 before it multiplies V (the only rounding besides the output's).
// Keys >= S are masked to -inf (their K/V rows in LDS are zeros); query rows >= S are computed on
// a clamped row and not stored.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kernels.hpp"

namespace delta {
namespace attn {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

static constexpr int kD = 64;                    // head dimension
static constexpr int kChunk = 64;                // keys per block (one online-softmax step)
static constexpr int kKT = kChunk / 32;          // 32-key tiles per block
static constexpr int kWaves = 8, kQB = kWaves * 32;   // queries per workgroup (4 wavefronts, two workgroups per CU: 4 % slower)
static constexpr int kPieces = kChunk * 8 / (kWaves * 64);   // 16-byte pieces of K (and of V) per thread and block
static constexpr int kPitch = kD * 2 + 16;       // LDS row pitch in bytes (144: conflict-free b128 rows)
static constexpr int kBufBytes = 2 * kChunk * kPitch;   // K and V of one block: 18 KB

__device__ __forceinline__ uint32_t pack2(float lo, float hi) {
    const f32x2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

struct AttnArgs {
    const unsigned char *qkv;
    unsigned char *ctx;
    int N, S, heads;
    float scale_log2e;                           // log2(e) / sqrt(d)
};

// Two workgroups per CU (<= 128 registers per lane, 36 KB of LDS each): four wavefronts per SIMD, so that
// one wavefront's softmax arithmetic runs under another's MFMAs.  With 128-key blocks (172 registers,
// one workgroup per CU) the same kernel took 54 instead of 45 us at batch 32 x 512.
__global__ __launch_bounds__(kWaves * 64, 2) void attention_kernel(AttnArgs a) {
    extern __shared__ __align__(16) unsigned char smem[];
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int l32 = lane & 31, half = lane >> 5;
    const int qblocks = (a.S + kQB - 1) / kQB;
    int blk = blockIdx.x;
    const int qb = blk % qblocks; blk /= qblocks;
    const int head = blk % a.heads;
    const int n = blk / a.heads;
    const int H = a.heads * kD;
    const size_t row_bytes = (size_t)3 * H * 2;
    const unsigned char *base = a.qkv + (size_t)n * a.S * row_bytes + (size_t)head * kD * 2;

    // this lane's query row, as the B operand of S^T = K Q^T: d 16*ks + 8*half .. +8
    int qrow = qb * kQB + wv * 32 + l32;
    const bool qvalid = qrow < a.S;
    if (!qvalid) qrow = a.S - 1;
    bf16x8 qf[4];
#pragma unroll
    for (int s = 0; s < 4; ++s)
        qf[s] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4 *>(base + (size_t)qrow * row_bytes + (16 * s + 8 * half) * 2));

    f32x16 o[2];
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int e = 0; e < 16; ++e) o[t][e] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;        // l_run: this half-wave's share of the sum

    // transpose-read addressing of V (see the header): within 16 lanes, lane j points at row j / 4
    // and columns 4 * (j % 4) .. +3 of a 4 x 16 block and receives column j of its 4 rows
    const int srow = (lane & 15) >> 2;
    const int scol = 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
    typedef s16x4 __attribute__((address_space(3))) * lds_s16x4_ptr;
    auto tr_read = [&](const unsigned char *p) { return __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(p)); };

    // ---- K/V blocks of 64 keys move global -> registers -> LDS one block ahead of the arithmetic:
    // while block b is multiplied out of buffer b % 2, block b + 1 sits in registers (requested a
    // whole block earlier) and is stored into the other buffer at the start of the next round.
    // 64 rows x 8 pieces x 2 operands / 512 threads = 2 pieces per thread.
    const int nblocks = (a.S + kChunk - 1) / kChunk;
    u32x4 rk[kPieces], rv[kPieces];
    auto fetch = [&](int blk) {                  // rows past S (or blocks past the end): zeros
#pragma unroll
        for (int p = 0; p < kPieces; ++p) {
            const int i = tid + p * (kWaves * 64);
            const int r = blk * kChunk + (i >> 3), seg = i & 7;
            rk[p] = u32x4{0u, 0u, 0u, 0u};
            rv[p] = u32x4{0u, 0u, 0u, 0u};
            if (r < a.S) {
                const unsigned char *src = base + (size_t)r * row_bytes + seg * 16;
                rk[p] = *reinterpret_cast<const u32x4 *>(src + (size_t)H * 2);
                rv[p] = *reinterpret_cast<const u32x4 *>(src + (size_t)H * 4);
            }
        }
    };
    auto stage = [&](int buf) {
        unsigned char *kb = smem + (size_t)buf * kBufBytes, *vb = kb + kChunk * kPitch;
#pragma unroll
        for (int p = 0; p < kPieces; ++p) {
            const int i = tid + p * (kWaves * 64);
            *reinterpret_cast<u32x4 *>(kb + (size_t)(i >> 3) * kPitch + (i & 7) * 16) = rk[p];
            *reinterpret_cast<u32x4 *>(vb + (size_t)(i >> 3) * kPitch + (i & 7) * 16) = rv[p];
        }
    };
    fetch(0);
    stage(0);
    fetch(1);
    __syncthreads();
    for (int blk = 0; blk < nblocks; ++blk) {
        if (blk + 1 < nblocks) stage((blk + 1) & 1);      // that buffer's last readers passed the barrier below
        fetch(blk + 2);
        const unsigned char *ks = smem + (size_t)(blk & 1) * kBufBytes, *vs = ks + kChunk * kPitch;
        const int kend = a.S - blk * kChunk;              // valid keys in this block (>= 1)
        {
            // ---- S^T for the block: tiles of 32 keys x 32 queries
            f32x16 s[kKT];
#pragma unroll
            for (int t = 0; t < kKT; ++t) {
#pragma unroll
                for (int e = 0; e < 16; ++e) s[t][e] = 0.f;
                const unsigned char *krow = ks + (size_t)(32 * t + l32) * kPitch + half * 16;
#pragma unroll
                for (int k4 = 0; k4 < 4; ++k4) {
                    const bf16x8 kf = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4 *>(krow + k4 * 32));
                    s[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[k4], s[t], 0, 0, 0);
                }
            }
            // ---- mask (last block only: a real branch, the selects would otherwise run for every
            // block), running maximum (of the raw scores: the scale is positive)
            float mx = -INFINITY;
            if (__builtin_expect(kend < kChunk, 0)) {
                const int lim = kend - 4 * half;                   // key = 32 t + 8 (e / 4) + (e % 4) + 4 half
#pragma unroll
                for (int t = 0; t < kKT; ++t)
#pragma unroll
                    for (int e = 0; e < 16; ++e)
                        s[t][e] = 32 * t + 8 * (e >> 2) + (e & 3) < lim ? s[t][e] : -INFINITY;
                asm volatile("" ::: "memory");                     // keeps the masked path a separate block
            }
#pragma unroll
            for (int t = 0; t < kKT; ++t)
#pragma unroll
                for (int e = 0; e < 16; ++e) mx = fmaxf(mx, s[t][e]);
            {
                const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(mx), __float_as_uint(mx), false, false);
                mx = fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));   // both half-waves' keys
            }
            const float m_new = fmaxf(m_run, mx * a.scale_log2e);   // finite: every block starts at a valid key
            const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);   // 0 on the first block (m_run = -inf)
            m_run = m_new;
            l_run *= alpha;
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int e = 0; e < 16; ++e) o[t][e] *= alpha;
            // ---- p = exp2(s * scale - m), O^T += V^T P^T
#pragma unroll
            for (int t = 0; t < kKT; ++t) {
                float psum = 0.f;
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    s[t][e] = __builtin_amdgcn_exp2f(__builtin_fmaf(s[t][e], a.scale_log2e, -m_new));
                    psum += s[t][e];
                }
                l_run += psum;
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    u32x4 pb;
                    pb.x = pack2(s[t][8 * j + 0], s[t][8 * j + 1]);
                    pb.y = pack2(s[t][8 * j + 2], s[t][8 * j + 3]);
                    pb.z = pack2(s[t][8 * j + 4], s[t][8 * j + 5]);
                    pb.w = pack2(s[t][8 * j + 6], s[t][8 * j + 7]);
                    const bf16x8 pf = __builtin_bit_cast(bf16x8, pb);
                    const unsigned char *vrow = vs + (size_t)(32 * t + 16 * j + 4 * half + srow) * kPitch + scol * 2;
#pragma unroll
                    for (int dt = 0; dt < 2; ++dt) {
                        const s16x4 v0 = tr_read(vrow + dt * 64);
                        const s16x4 v1 = tr_read(vrow + 8 * kPitch + dt * 64);
                        const s16x8 vf = __builtin_shufflevector(v0, v1, 0, 1, 2, 3, 4, 5, 6, 7);
                        o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, vf), pf, o[dt], 0, 0, 0);
                    }
                }
            }
        }
        __syncthreads();                         // buffer blk % 2 is free; block blk + 1 is visible
    }
    // ---- normalise and store: lane holds query l32, d = 32*dt + 8*e4 + 4*half + e
    {
        const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(l_run), __float_as_uint(l_run), false, false);
        l_run = __uint_as_float(r[0]) + __uint_as_float(r[1]);
    }
    const float inv = 1.0f / l_run;
    if (!qvalid) return;
    unsigned char *out = a.ctx + ((size_t)n * a.S + qrow) * (size_t)H * 2 + (size_t)head * kD * 2;
#pragma unroll
    for (int dt = 0; dt < 2; ++dt)
#pragma unroll
        for (int e4 = 0; e4 < 4; ++e4) {
            uint2 w;
            w.x = pack2(o[dt][4 * e4 + 0] * inv, o[dt][4 * e4 + 1] * inv);
            w.y = pack2(o[dt][4 * e4 + 2] * inv, o[dt][4 * e4 + 3] * inv);
            *reinterpret_cast<uint2 *>(out + (32 * dt + 8 * e4 + 4 * half) * 2) = w;
        }
}

}  // namespace attn

// nullptr when supported, else the reason.  Geometry: N images, S positions, `heads` heads of 64.
const char *attention_check(const void *qkv, const void *ctx, int N, int S, int heads, int bf16) {
    if (!bf16) return "attention is bf16 only";
    if (N <= 0 || S <= 0 || heads <= 0) return "non-positive dimension";
    if (!qkv || !ctx || (((uintptr_t)qkv | (uintptr_t)ctx) & 15)) return "pointers must be non-null and 16-byte aligned";
    if ((long long)N * heads * ((S + attn::kQB - 1) / attn::kQB) > 0x7FFFFFFFLL) return "too many workgroups";
    return nullptr;
}

hipError_t launch_attention(const void *qkv, void *ctx, int N, int S, int heads, int bf16, hipStream_t stream) {
    if (attention_check(qkv, ctx, N, S, heads, bf16)) return hipErrorInvalidValue;
    attn::AttnArgs a;
    a.qkv = static_cast<const unsigned char *>(qkv);
    a.ctx = static_cast<unsigned char *>(ctx);
    a.N = N; a.S = S; a.heads = heads;
    a.scale_log2e = 1.4426950408889634f / 8.0f;          // log2(e) / sqrt(64)
    const size_t lds = (size_t)2 * attn::kBufBytes;      // two buffers of one block: 36 KB
    static bool raised = false;
    if (!raised) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(attn::attention_kernel),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e != hipSuccess) return e;
        raised = true;
    }
    const long long blocks = (long long)N * heads * ((S + attn::kQB - 1) / attn::kQB);
    attn::attention_kernel<<<dim3((unsigned)blocks), dim3(attn::kWaves * 64), lds, stream>>>(a);
    return hipGetLastError();
}

}  // namespace delta
