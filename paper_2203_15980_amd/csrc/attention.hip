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
// 32 queries.  K and V of the head - up to 512 keys at a time - are staged in LDS once per
// workgroup.  Everything is computed TRANSPOSED so that a lane owns one query:
//   S^T tile (32 keys x 32 queries) = K tile . Q^T        A = K rows from LDS (b128), B = Q from registers
//   lane l holds query l % 32 and keys 8*e4 + 4*(l/32) + e of the tile: the softmax statistics of
//   a query (running maximum, running sum) are per-lane scalars; the two half-waves see disjoint
//   keys and exchange their maxima with one permlane32 swap per 128 keys.
//   O^T (64 d x 32 queries) += V^T . P^T                  A = V^T through the LDS transpose read
//   (ds_read_b64_tr_b16: V lies [key][d] in LDS as in memory), B = P straight from the S^T
//   accumulators rounded to bf16: accumulator registers (e4 in {2j, 2j+1}) of a lane are exactly
//   the 8 reduction slots of step j, if the A operand enumerates the keys in the same order
//   (keys 16j + 4*(l/32) + e and 16j + 8 + 4*(l/32) + e) - the order of a reduction is free.
// Online softmax over chunks of 128 keys (fp32; exp2 with the scale folded in).  P is rounded to
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
static constexpr int kWaves = 8, kQB = kWaves * 32;   // queries per workgroup
static constexpr int kChunk = 128;               // keys per online-softmax step
static constexpr int kMaxKeys = 512;             // keys staged at once
static constexpr int kPitch = kD * 2 + 16;       // LDS row pitch in bytes (144: conflict-free b128 rows)

__device__ __forceinline__ uint32_t pack2(float lo, float hi) {
    const f32x2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

struct AttnArgs {
    const unsigned char *qkv;
    unsigned char *ctx;
    int N, S, heads;
    int keys_alloc;                              // LDS rows per operand: multiple of kChunk, <= kMaxKeys
    float scale_log2e;                           // log2(e) / sqrt(d)
};

__global__ __launch_bounds__(kWaves * 64) void attention_kernel(AttnArgs a) {
    extern __shared__ __align__(16) unsigned char smem[];
    unsigned char *ks = smem;
    unsigned char *vs = smem + (size_t)a.keys_alloc * kPitch;
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

    for (int kb0 = 0; kb0 < a.S; kb0 += a.keys_alloc) {
        if (kb0) __syncthreads();                // every wavefront is done with the previous block
        // ---- stage K and V rows kb0 .. kb0 + keys_alloc (zeros past S): 8 lanes per 128-byte row
        for (int i = tid; i < a.keys_alloc * 8; i += kWaves * 64) {
            const int r = i >> 3, seg = i & 7;
            u32x4 kv = {0u, 0u, 0u, 0u}, vv = {0u, 0u, 0u, 0u};
            if (kb0 + r < a.S) {
                const unsigned char *p = base + (size_t)(kb0 + r) * row_bytes + seg * 16;
                kv = *reinterpret_cast<const u32x4 *>(p + (size_t)H * 2);
                vv = *reinterpret_cast<const u32x4 *>(p + (size_t)H * 4);
            }
            *reinterpret_cast<u32x4 *>(ks + (size_t)r * kPitch + seg * 16) = kv;
            *reinterpret_cast<u32x4 *>(vs + (size_t)r * kPitch + seg * 16) = vv;
        }
        __syncthreads();
        const int kend = a.S - kb0 < a.keys_alloc ? a.S - kb0 : a.keys_alloc;   // valid keys in this block
        for (int c0 = 0; c0 < kend; c0 += kChunk) {
            // ---- S^T for 128 keys: 4 tiles of 32 keys x 32 queries
            f32x16 s[4];
#pragma unroll
            for (int t = 0; t < 4; ++t) {
#pragma unroll
                for (int e = 0; e < 16; ++e) s[t][e] = 0.f;
                const unsigned char *krow = ks + (size_t)(c0 + 32 * t + l32) * kPitch + half * 16;
#pragma unroll
                for (int k4 = 0; k4 < 4; ++k4) {
                    const bf16x8 kf = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4 *>(krow + k4 * 32));
                    s[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[k4], s[t], 0, 0, 0);
                }
            }
            // ---- scale, mask, running maximum
            const bool ragged = c0 + kChunk > kend;
            float mx = -INFINITY;
#pragma unroll
            for (int t = 0; t < 4; ++t)
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    float v = s[t][e] * a.scale_log2e;
                    if (ragged) {
                        const int key = c0 + 32 * t + 8 * (e >> 2) + 4 * half + (e & 3);
                        v = key < kend ? v : -INFINITY;
                    }
                    s[t][e] = v;
                    mx = fmaxf(mx, v);
                }
            {
                const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(mx), __float_as_uint(mx), false, false);
                mx = fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));   // both half-waves' keys
            }
            const float m_new = fmaxf(m_run, mx);       // finite: every chunk starts at a valid key
            const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);   // 0 on the first chunk (m_run = -inf)
            m_run = m_new;
            l_run *= alpha;
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int e = 0; e < 16; ++e) o[t][e] *= alpha;
            // ---- p = exp2(s - m), O^T += V^T P^T
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                float psum = 0.f;
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    s[t][e] = __builtin_amdgcn_exp2f(s[t][e] - m_new);
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
                    const unsigned char *vrow = vs + (size_t)(c0 + 32 * t + 16 * j + 4 * half + srow) * kPitch + scol * 2;
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
    const int want = (S + attn::kChunk - 1) / attn::kChunk * attn::kChunk;
    a.keys_alloc = want < attn::kMaxKeys ? want : attn::kMaxKeys;
    a.scale_log2e = 1.4426950408889634f / 8.0f;          // log2(e) / sqrt(64)
    const size_t lds = (size_t)2 * a.keys_alloc * attn::kPitch;
    static bool raised = false;
    if (lds > 64 * 1024 && !raised) {
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
