// Weight gradient of the ResNet stem (7x7, stride 2, pad 3, 3 -> 64 channels, bf16) for gfx950:
//   gw[k][r][s][c] = scale_k * sum over (n, p, q) of gpre[n,p,q,k] * x[n, 2p + r - 3, 2q + s - 3, c]
// the last piece of the training iteration's backward pass (DELTA Sec. 3: the backward pass is what
// reads the stored activations) - the stem has no data gradient to compute.
//
// Same reduction layout as the forward kernel: the input patch of a tile is staged in LDS with its
// pixels padded from 3 to 4 channels, so that for a fixed kernel row r the 8 taps x 4 channels of
// an output pixel (q) are 32 contiguous elements starting at patch column 2q ("j" = 4 s + c; tap 7
// and channel 3 are padding and are dropped at the end).  The reduction runs over output pixels;
// both operands are pixel-major, and the LDS transpose read (ds_read_b64_tr_b16) turns
// "4 pixels x 16 columns" blocks into MFMA operands for both:
//   D[k][j] += A[k][pixel] B[pixel][j]     A from the gpre tile [pixel][64 k], B from the patch:
//   row = pixel (p, q) -> address of patch[2p + r][2q], 32 elements wide (the rows of neighbouring
//   pixels overlap in memory, which a transpose read does not mind).
// A workgroup is 7 wavefronts, one per kernel row r, sharing the staged tiles (8 x 16 output pixels
// per tile, one MFMA k-step per tile row); persistent over tiles (the next tile's pixels and gradient
// rows travel in registers while the current tile is multiplied), accumulators (64 k x 32 j per
// wavefront) in registers, written per workgroup to a partial buffer; a second kernel adds the
// workgroups' partials in a fixed order, applies scale_k and drops the padding.  No atomics.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kernels.hpp"

namespace delta {
namespace stemw {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

static constexpr int kWaves = 7;                         // one per kernel row
static constexpr int kTP = 8, kTQ = 16;                  // output pixels per tile
static constexpr int kPRows = 2 * kTP + 5, kPCols = 2 * kTQ + 6;   // patch: 21 rows x 38 padded pixels
static constexpr int kPPitch = kPCols * 8;               // 304 bytes
static constexpr int kGPitch = 64 * 2 + 16;              // gpre tile row: 64 channels + pad
static constexpr int kPartialFloats = kWaves * 2 * 16 * 64;   // per workgroup: [r][k tile][register][lane]

__global__ __launch_bounds__(kWaves * 64) void stem_wgrad_kernel(ConvArgs a, const unsigned char *g, float *partial,
                                                                 int tiles_p, int tiles_q, int ntiles) {
    __shared__ __align__(16) unsigned char patch[kPRows * kPPitch];
    __shared__ __align__(16) unsigned char gs[kTP * kTQ * kGPitch];
    const int tid = threadIdx.x, lane = tid & 63, r = tid >> 6;
    const uint16_t *xg = static_cast<const uint16_t *>(a.x);
    // transpose-read addressing: within 16 lanes, lane j points at row j / 4, columns 4 (j % 4) .. + 3 of
    // a 4 x 16 block and receives column j of its 4 rows; lanes 32..63 take pixels 8..15 of a step
    const int srow = (lane & 15) >> 2;
    const int scol = 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
    const int half = lane >> 5;
    typedef s16x4 __attribute__((address_space(3))) * lds_s16x4_ptr;
    auto tr_read = [&](const unsigned char *p) { return __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(p)); };

    f32x16 acc[2];
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[u][e] = 0.f;

    // Staging: a thread carries 2 patch pixels (3 channels each) and 3 sixteen-byte pieces of the gpre
    // tile; the next tile's are requested before the current tile's MFMAs and written to LDS after them.
    constexpr int kNT = kWaves * 64;
    constexpr int kPPix = (kPRows * kPCols + kNT - 1) / kNT, kGPieces = (kTP * kTQ * 8 + kNT - 1) / kNT;
    static_assert(kPPix == 2 && kGPieces == 3, "staging registers are sized for these tiles");
    uint16_t px[kPPix][3];
    u32x4 gq[kGPieces];
    uint32_t ok = 0;                              // bit c: patch pixel c is inside the image; bit 8 + c: gpre piece c is
    auto request = [&](int tile) {
        const int n = tile / (tiles_p * tiles_q), t2 = tile - n * tiles_p * tiles_q;
        const int p0 = (t2 / tiles_q) * kTP, q0 = (t2 % tiles_q) * kTQ;
        ok = 0;
#pragma unroll
        for (int c = 0; c < kPPix; ++c) {
            const int e = tid + c * kNT;
            const int i = e / kPCols, j = e - i * kPCols;
            const int h = 2 * p0 - 3 + i, w = 2 * q0 - 3 + j;
            const bool in = e < kPRows * kPCols && (unsigned)h < (unsigned)a.H && (unsigned)w < (unsigned)a.W;
            const uint16_t *src = xg + (in ? ((size_t)((size_t)n * a.H + h) * a.W + w) * 3 : 0);
            px[c][0] = src[0]; px[c][1] = src[1]; px[c][2] = src[2];
            ok |= (uint32_t)in << c;
        }
#pragma unroll
        for (int c = 0; c < kGPieces; ++c) {
            const int e = tid + c * kNT;
            const int pix = e >> 3, seg = e & 7;
            const int p = p0 + pix / kTQ, q = q0 + pix % kTQ;
            const bool in = e < kTP * kTQ * 8 && p < a.P && q < a.Q;
            gq[c] = *reinterpret_cast<const u32x4 *>(g + (in ? (((size_t)n * a.P + p) * a.Q + q) * 128 + seg * 16 : 0));
            ok |= (uint32_t)in << (8 + c);
        }
    };
    auto deposit = [&]() {
#pragma unroll
        for (int c = 0; c < kPPix; ++c) {
            const int e = tid + c * kNT;
            if (e < kPRows * kPCols) {
                const bool in = (ok >> c) & 1u;
                u32x2 v;
                v.x = in ? (uint32_t)px[c][0] | ((uint32_t)px[c][1] << 16) : 0u;
                v.y = in ? (uint32_t)px[c][2] : 0u;
                const int i = e / kPCols, j = e - i * kPCols;
                *reinterpret_cast<u32x2 *>(patch + i * kPPitch + j * 8) = v;
            }
        }
#pragma unroll
        for (int c = 0; c < kGPieces; ++c) {
            const int e = tid + c * kNT;
            if (e < kTP * kTQ * 8) {
                const bool in = (ok >> (8 + c)) & 1u;
                const u32x4 zero = {0u, 0u, 0u, 0u};
                *reinterpret_cast<u32x4 *>(gs + (e >> 3) * kGPitch + (e & 7) * 16) = in ? gq[c] : zero;
            }
        }
    };

    if ((int)blockIdx.x < ntiles) request(blockIdx.x);
    for (int tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
        __syncthreads();                          // the previous tile is no longer read
        deposit();
        if (tile + (int)gridDim.x < ntiles) request(tile + gridDim.x);
        __syncthreads();
#pragma unroll
        for (int pr = 0; pr < kTP; ++pr) {        // one k-step: the 16 pixels of tile row pr
            // B: patch row 2 pr + r, pixels q = 8 half + srow (+ 4), columns j = scol ..
            const unsigned char *brow = patch + (2 * pr + r) * kPPitch + (8 * half + srow) * 16 + scol * 2;
            const s16x4 b0 = tr_read(brow);
            const s16x4 b1 = tr_read(brow + 4 * 16);
            const s16x8 bf = __builtin_shufflevector(b0, b1, 0, 1, 2, 3, 4, 5, 6, 7);
            const unsigned char *arow = gs + (pr * kTQ + 8 * half + srow) * kGPitch + scol * 2;
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const s16x4 a0 = tr_read(arow + u * 64);
                const s16x4 a1 = tr_read(arow + 4 * kGPitch + u * 64);
                const s16x8 af = __builtin_shufflevector(a0, a1, 0, 1, 2, 3, 4, 5, 6, 7);
                acc[u] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, af), __builtin_bit_cast(bf16x8, bf),
                                                                 acc[u], 0, 0, 0);
            }
        }
    }
    float *out = partial + (size_t)blockIdx.x * kPartialFloats + (size_t)r * (2 * 16 * 64);
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
        for (int e = 0; e < 16; ++e) out[(u * 16 + e) * 64 + lane] = acc[u][e];
}

// One workgroup per (r, k tile, register): 64 lanes x 16 groups of workgroup-partials (group g adds
// partials g, g + 16, ..., eight loads in flight), the groups added in order.  Element (r, u, e, lane)
// is k = 32 u + 8 (e / 4) + 4 (lane / 32) + e % 4, j = lane % 32.
__global__ __launch_bounds__(1024) void stem_wgrad_reduce_kernel(const float *partial, const float *scale, float *gw, int nblocks) {
    __shared__ float red[16][64];
    const int lane = threadIdx.x & 63, grp = threadIdx.x >> 6;
    const int idx = blockIdx.x;                   // (r * 2 + u) * 16 + e
    const float *src = partial + (size_t)idx * 64 + lane;
    float s = 0.f;
    int b = grp;
    for (; b + 7 * 16 < nblocks; b += 8 * 16) {
        float v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = src[(size_t)(b + 16 * u) * kPartialFloats];
#pragma unroll
        for (int u = 0; u < 8; ++u) s += v[u];
    }
    for (; b < nblocks; b += 16) s += src[(size_t)b * kPartialFloats];
    red[grp][lane] = s;
    __syncthreads();
    if (grp) return;
    s = 0.f;
#pragma unroll
    for (int g = 0; g < 16; ++g) s += red[g][lane];
    const int e = idx & 15, u = (idx >> 4) & 1, r = idx >> 5;
    const int k = 32 * u + 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3), j = lane & 31;
    const int sx = j >> 2, c = j & 3;
    if (sx < 7 && c < 3) gw[((k * 7 + r) * 7 + sx) * 3 + c] = s * scale[k];
}

static int grid_for(long long ntiles) { return (int)(ntiles < 512 ? ntiles : 512); }

}  // namespace stemw

size_t stem_wgrad_workspace_bytes(const ConvArgs &a) {
    const long long ntiles = (long long)a.N * ((a.P + stemw::kTP - 1) / stemw::kTP) * ((a.Q + stemw::kTQ - 1) / stemw::kTQ);
    return (size_t)stemw::grid_for(ntiles) * stemw::kPartialFloats * sizeof(float);
}

// a: the stem's forward arguments (stem_applies(a)) with a.x = x and a.scale = scale; g = gpre
// [N,P,Q,64] bf16; gw fp32 [64][7][7][3]; workspace of stem_wgrad_workspace_bytes(a), 16-byte aligned.
hipError_t launch_stem_wgrad(const ConvArgs &a, const void *g, float *gw, void *workspace, size_t workspace_bytes,
                             hipStream_t stream) {
    if (!stem_applies(a) || stem_check(a) || !g || !gw || !workspace || workspace_bytes < stem_wgrad_workspace_bytes(a) ||
        (((uintptr_t)g | (uintptr_t)workspace) & 15) || ((uintptr_t)gw & 3))
        return hipErrorInvalidValue;
    const int tiles_p = (a.P + stemw::kTP - 1) / stemw::kTP, tiles_q = (a.Q + stemw::kTQ - 1) / stemw::kTQ;
    const long long ntiles = (long long)a.N * tiles_p * tiles_q;
    if (ntiles <= 0 || ntiles > 0x7FFFFFFFLL) return hipErrorInvalidValue;
    const int grid = stemw::grid_for(ntiles);
    stemw::stem_wgrad_kernel<<<dim3(grid), dim3(stemw::kWaves * 64), 0, stream>>>(
        a, static_cast<const unsigned char *>(g), static_cast<float *>(workspace), tiles_p, tiles_q, (int)ntiles);
    stemw::stem_wgrad_reduce_kernel<<<dim3(stemw::kWaves * 2 * 16), dim3(1024), 0, stream>>>(
        static_cast<const float *>(workspace), a.scale, gw, grid);
    return hipGetLastError();
}

}  // namespace delta
