// Block kernel: one identity bottleneck of ResNet's conv2_x stage in a single launch (bf16, fp32
// accumulate):   a1 = relu(bn1(w1 . x))            1x1, 256 -> 64
//                a2 = relu(bn2(conv3x3(a1, w2)))    3x3, 64 -> 64, stride 1, pad 1
//                out = relu(bn3(w3 . a2) + x)       1x1, 64 -> 256, identity shortcut
// This is the recompute segment DELTA's Recompute action re-runs for a released activation of such
// a block (Sec. 3, Table 1): any subset of {a1, a2, out} is regenerated from the block's input x
// alone, the tensors that are not asked for never reach memory.  Three per-layer launches move
// 2 x (256 + 64 | 64 + 64 | 64 + 256 + 256) bytes per pixel; this kernel reads x once (plus the
// shortcut's re-read, which the caches serve) and writes only what is stored.
//
// A workgroup of 16 wavefronts owns BM consecutive pixels (NHW order) and walks three phases:
//   1. a1 for its pixels and the W + 1 pixels before and after them (the halo the 3x3 needs) is
//      computed by all wavefronts, one 32-pixel tile each: x straight from global memory into
//      registers (64 bytes per lane and 128-byte slice), w1 from LDS; the results go to LDS as
//      bf16 rows of 128 bytes (pitch 144) - exactly the layout the 3x3 reads its operand in;
//   2. a2: every wavefront takes 32 pixels x 64 channels; the nine taps read nine shifted rows of
//      the a1 tile in LDS (taps outside the image are redirected to a row of zeros), w2 is
//      resident in LDS (taps 0-4 staged during phase 1, taps 5-8 into the space w1 leaves);
//      the result stays in registers as bf16, 8 consecutive channels per piece;
//   3. out: those registers are the MFMA's pixel operand as they are (a piece of 8 channels per
//      step; w3's rows are read from LDS in the same channel order), the shortcut is read from x
//      in the same piece layout, and rows of 128 contiguous bytes leave through a
//      wavefront-private LDS tile.
// Orientation as in the per-layer kernels: output channels on the MFMA row axis, pixels on the
// column axis; lane half h owns bytes [64h, 64h + 64) of every 128-byte slice of both operands.
// The order of every sum is fixed and does not depend on which tensors are stored, so whatever
// this kernel produced in the forward pass it reproduces bit for bit in a recomputation.
// Every reduction also runs in the order of the per-layer kernels (slices of the input channels in order,
// the 3x3's taps in order, lane half h supplying bytes [64 h, 64 h + 64) of each 128-byte operand slice),
// so the three tensors carry the bits the three per-layer launches produce: a plan may regenerate a
// tensor with either.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kernels.hpp"

namespace delta {
namespace block {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

static constexpr int kWaves = 16, kThreads = kWaves * 64;
static constexpr int kCin = 256, kMid = 64, kCout = 256;
static constexpr int kPitch = 144;                       // 128-byte rows, 4 banks apart
static constexpr int kW1Pitch = kCin * 2 + 16;           // 528
static constexpr int kMaxHaloTiles = 16;                 // one 32-row tile of phase 1 per wavefront
static constexpr int kTap = kMid * kPitch;               // one 64 x 64 tap of w2 in LDS: 9216 bytes
static constexpr int kRA = (kMaxHaloTiles * 32 + 1) * kPitch;      // a1 rows + the zero row; later the store tiles
static constexpr int kRB = 4 * kTap;                                // w1, then taps 5-8
static constexpr int kRC = 5 * kTap;                                // taps 0-4, then w3
static constexpr int kRD = (2 * kMid + 2 * kMid + 2 * kCout) * 4;   // scale/shift of the three layers
static constexpr int kLds = kRA + kRB + kRC + kRD;
static_assert(kW1Pitch * kMid <= kRB && kCout * kPitch <= kRC && kWaves * 32 * kPitch <= kRA, "LDS regions");
static_assert(kLds <= 160 * 1024, "LDS budget of a CU");

__device__ __forceinline__ uint32_t pack2(float lo, float hi) {
    const f32x2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}
__device__ __forceinline__ float lo16(uint32_t p) { return __uint_as_float(p << 16); }
__device__ __forceinline__ float hi16(uint32_t p) { return __uint_as_float(p & 0xFFFF0000u); }
__device__ __forceinline__ float relu_keep_nan(float v) { return v < 0.f ? 0.f : v; }
__device__ __forceinline__ void wave_fence() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}
__device__ __forceinline__ f32x16 mma(const u32x4 w, const u32x4 x, const f32x16 acc) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, w), __builtin_bit_cast(bf16x8, x), acc, 0, 0, 0);
}

// Two 32-channel accumulator tiles of one 32-pixel column block -> scale/shift, (ReLU), bf16, as four
// pieces of 8 consecutive channels: piece [u][i2] of lane (pixel, half) holds channels
// 32 u + 16 i2 + 8 half .. + 8 of its pixel.  `add` (optional) is added before the ReLU in the same layout.
template <bool HAS_ADD>
__device__ __forceinline__ void finish_tiles(const f32x16 (&acc)[2], const float *scale, const float *shift, int half,
                                             const u32x4 (*add)[2], u32x4 (&piece)[2][2]) {
#pragma unroll
    for (int u = 0; u < 2; ++u) {
        float v[16];
#pragma unroll
        for (int rb = 0; rb < 4; ++rb) {
            const f32x4 sc = *reinterpret_cast<const f32x4 *>(scale + u * 32 + 8 * rb + 4 * half);
            const f32x4 sh = *reinterpret_cast<const f32x4 *>(shift + u * 32 + 8 * rb + 4 * half);
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
            if constexpr (HAS_ADD) {
                const u32x4 r4 = add[u][i2];
                o[0] += lo16(r4.x); o[1] += hi16(r4.x); o[2] += lo16(r4.y); o[3] += hi16(r4.y);
                o[4] += lo16(r4.z); o[5] += hi16(r4.z); o[6] += lo16(r4.w); o[7] += hi16(r4.w);
            }
#pragma unroll
            for (int e = 0; e < 8; ++e) o[e] = relu_keep_nan(o[e]);
            u32x4 out;
            out.x = pack2(o[0], o[1]); out.y = pack2(o[2], o[3]);
            out.z = pack2(o[4], o[5]); out.w = pack2(o[6], o[7]);
            piece[u][i2] = out;
        }
    }
}

// BM: pixels per workgroup; NT1 = ceil((BM + 2W + 2) / 32) <= 16 halo tiles; NT2 = ceil(BM / 32) <= 16.
__global__ __launch_bounds__(kThreads) void bottleneck_block_kernel(BlockArgs a, int BM, int NT1, int NT2) {
    extern __shared__ __align__(16) unsigned char lds[];
    unsigned char *ra = lds;
    unsigned char *rb = lds + kRA;
    unsigned char *rc = rb + kRB;
    float *f1s = reinterpret_cast<float *>(rc + kRC), *f1h = f1s + kMid, *f2s = f1h + kMid, *f2h = f2s + kMid,
          *f3s = f2h + kMid, *f3h = f3s + kCout;

    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int l32 = lane & 31, half = lane >> 5;
    unsigned logical;                                    // neighbouring tiles (shared halo) on one XCD
    {
        const unsigned nb = gridDim.x, per = nb >> 3, rem = nb & 7u;
        const unsigned xcd = blockIdx.x & 7u, idx = blockIdx.x >> 3;
        logical = xcd < rem ? xcd * (per + 1) + idx : rem * (per + 1) + (xcd - rem) * per + idx;
    }
    const int W = a.W, HW = a.H * a.W, M = a.M;
    const long long m0 = (long long)logical * BM;
    const bool need2 = a.a2 != nullptr || a.out != nullptr;
    const bool need3 = a.out != nullptr;
    const int zrow = NT1 * 32;                           // the row of zeros behind the a1 rows

    const unsigned char *xg = static_cast<const unsigned char *>(a.x);

    // ---- phase 1 operand: the x rows of halo tile wv, in flight before anything is staged.
    // Row i of the a1 tile is pixel m0 - (W + 1) + i.  Without the 3x3 only the tile's own pixels count.
    const int own_lo = W + 1, own_hi = W + 1 + BM;       // rows [own_lo, own_hi) are this workgroup's pixels
    const bool p1 = wv < NT1 && (need2 || (wv * 32 < own_hi && wv * 32 + 32 > own_lo));
    u32x4 xf[4][4];
    if (p1) {
        long long q = m0 - (W + 1) + wv * 32 + l32;
        q = q < 0 ? 0 : (q >= M ? (long long)M - 1 : q);                 // clamped rows are never read back
        const unsigned char *xp = xg + (size_t)q * (kCin * 2) + half * 64;
#pragma unroll
        for (int s = 0; s < 4; ++s)
#pragma unroll
            for (int j = 0; j < 4; ++j) xf[s][j] = *reinterpret_cast<const u32x4 *>(xp + s * 128 + j * 16);
    }

    // ---- stage w1, the batch-norm factors, the zero row and (for the 3x3) taps 0-4 of w2
    {
        const unsigned char *w1g = static_cast<const unsigned char *>(a.w1);
        for (int c = tid; c < kMid * 32; c += kThreads) {                 // 32 pieces of 16 bytes per row
            const int row = c >> 5, seg = c & 31;
            *reinterpret_cast<u32x4 *>(rb + row * kW1Pitch + seg * 16) = *reinterpret_cast<const u32x4 *>(w1g + (size_t)c * 16);
        }
        if (tid < kMid) {
            f1s[tid] = a.s1[tid]; f1h[tid] = a.h1[tid];
            f2s[tid] = a.s2[tid]; f2h[tid] = a.h2[tid];
        }
        if (tid < kCout) { f3s[tid] = a.s3[tid]; f3h[tid] = a.h3[tid]; }
        if (tid < 9) *reinterpret_cast<u32x4 *>(ra + zrow * kPitch + tid * 16) = u32x4{0u, 0u, 0u, 0u};
        if (need2) {
            const unsigned char *w2g = static_cast<const unsigned char *>(a.w2);
            for (int c = tid; c < 5 * kMid * 8; c += kThreads) {          // (tap, k, seg)
                const int tap = c / (kMid * 8), rest = c - tap * (kMid * 8), k = rest >> 3, seg = rest & 7;
                *reinterpret_cast<u32x4 *>(rc + tap * kTap + k * kPitch + seg * 16) =
                    *reinterpret_cast<const u32x4 *>(w2g + ((size_t)(k * 9 + tap) * 8 + seg) * 16);
            }
        }
    }
    __syncthreads();

    // ---- phase 1: a1 = relu(bn1(w1 . x)) for one halo tile per wavefront, into LDS
    if (p1) {
        f32x16 acc[2];
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[u][e] = 0.f;
        const unsigned char *wrow = rb + l32 * kW1Pitch + half * 64;
#pragma unroll
        for (int s = 0; s < 4; ++s)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const u32x4 w0 = *reinterpret_cast<const u32x4 *>(wrow + s * 128 + j * 16);
                const u32x4 w1 = *reinterpret_cast<const u32x4 *>(wrow + 32 * kW1Pitch + s * 128 + j * 16);
                acc[0] = mma(w0, xf[s][j], acc[0]);
                acc[1] = mma(w1, xf[s][j], acc[1]);
            }
        u32x4 piece[2][2];
        finish_tiles<false>(acc, f1s, f1h, half, nullptr, piece);
        unsigned char *row = ra + (wv * 32 + l32) * kPitch;
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
            for (int i2 = 0; i2 < 2; ++i2)
                *reinterpret_cast<u32x4 *>(row + (u * 32 + 16 * i2 + 8 * half) * 2) = piece[u][i2];
    }
    __syncthreads();

    // ---- a1 leaves as rows of 128 contiguous bytes (8 lanes per pixel), if it is stored
    if (a.a1) {
        unsigned char *a1g = static_cast<unsigned char *>(a.a1);
        for (int c = tid; c < BM * 8; c += kThreads) {
            const int i = c >> 3, seg = c & 7;
            const long long m = m0 + i;
            if (m < M)
                *reinterpret_cast<u32x4 *>(a1g + (size_t)m * (kMid * 2) + seg * 16) =
                    *reinterpret_cast<const u32x4 *>(ra + (own_lo + i) * kPitch + seg * 16);
        }
    }
    if (!need2) return;

    // ---- phase 2: a2 = relu(bn2(conv3x3(a1))).  Taps 5-8 of w2 travel in registers while taps 0-4
    // are multiplied, and land where w1 was; w3 travels while taps 5-8 are multiplied.
    u32x4 wq[2];
    {
        const unsigned char *w2g = static_cast<const unsigned char *>(a.w2);
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int c = tid + j * kThreads;                             // 4 taps x 64 rows x 8 pieces = 2048
            const int tap = 5 + c / (kMid * 8), rest = c % (kMid * 8), k = rest >> 3, seg = rest & 7;
            wq[j] = *reinterpret_cast<const u32x4 *>(w2g + ((size_t)(k * 9 + tap) * 8 + seg) * 16);
        }
    }
    const bool p2 = wv < NT2;
    const int pi = wv * 32 + l32;                        // this lane's pixel within the tile
    const long long pm = m0 + pi;
    uint32_t valid = 0;                                  // nine bits: tap inside the image
    if (p2 && pi < BM && pm < M) {
        const int hw = (int)(pm % HW), h = hw / W, w_ = hw - h * W;
#pragma unroll
        for (int r = 0; r < 3; ++r)
#pragma unroll
            for (int s = 0; s < 3; ++s)
                if ((unsigned)(h + r - 1) < (unsigned)a.H && (unsigned)(w_ + s - 1) < (unsigned)W) valid |= 1u << (r * 3 + s);
    }
    f32x16 acc2[2];
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc2[u][e] = 0.f;
    auto taps = [&](const unsigned char *wbase, int first, int count) {
#pragma unroll
        for (int t = 0; t < count; ++t) {
            const int tap = first + t, r = tap / 3, s = tap - 3 * r;
            const int row = ((valid >> tap) & 1u) ? pi + r * W + s : zrow;
            const unsigned char *xp = ra + row * kPitch + half * 64;
            const unsigned char *wp = wbase + t * kTap + l32 * kPitch + half * 64;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const u32x4 xv = *reinterpret_cast<const u32x4 *>(xp + q * 16);
                const u32x4 w0 = *reinterpret_cast<const u32x4 *>(wp + q * 16);
                const u32x4 w1 = *reinterpret_cast<const u32x4 *>(wp + 32 * kPitch + q * 16);
                acc2[0] = mma(w0, xv, acc2[0]);
                acc2[1] = mma(w1, xv, acc2[1]);
            }
        }
    };
    if (p2) taps(rc, 0, 5);
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int c = tid + j * kThreads;
        const int t = c / (kMid * 8), rest = c % (kMid * 8), k = rest >> 3, seg = rest & 7;
        *reinterpret_cast<u32x4 *>(rb + t * kTap + k * kPitch + seg * 16) = wq[j];
    }
    if (need3) {
        const unsigned char *w3g = static_cast<const unsigned char *>(a.w3);
#pragma unroll
        for (int j = 0; j < 2; ++j) wq[j] = *reinterpret_cast<const u32x4 *>(w3g + (size_t)(tid + j * kThreads) * 16);
    }
    __syncthreads();
    if (p2) taps(rb, 5, 4);
    u32x4 a2p[2][2];                                     // this lane's pixel of a2: four pieces of 8 channels
    if (p2) finish_tiles<false>(acc2, f2s, f2h, half, nullptr, a2p);
    if (need3) {
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int c = tid + j * kThreads, row = c >> 3, seg = c & 7;  // 256 rows x 8 pieces
            *reinterpret_cast<u32x4 *>(rc + row * kPitch + seg * 16) = wq[j];
        }
    }
    __syncthreads();                                     // a1 and w2 are dead from here on; w3 is in place
    if (!p2) return;

    unsigned char *ttile = ra + wv * (32 * kPitch);      // wavefront-private: pieces in, rows out
    const int trow = lane >> 3, tseg = lane & 7;
    const long long mbase = m0 + wv * 32;
    const int rows_here = BM - wv * 32;                  // rows of this tile that belong to the workgroup
    if (a.a2) {
        unsigned char *a2g = static_cast<unsigned char *>(a.a2);
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
            for (int i2 = 0; i2 < 2; ++i2)
                *reinterpret_cast<u32x4 *>(ttile + l32 * kPitch + (u * 32 + 16 * i2 + 8 * half) * 2) = a2p[u][i2];
        wave_fence();
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const int pr = trow + 8 * t;
            const u32x4 o4 = *reinterpret_cast<const u32x4 *>(ttile + pr * kPitch + tseg * 16);
            if (pr < rows_here && mbase + pr < M)
                *reinterpret_cast<u32x4 *>(a2g + (size_t)(mbase + pr) * (kMid * 2) + tseg * 16) = o4;
        }
        wave_fence();
    }
    if (!need3) return;

    // ---- phase 3: out = relu(bn3(w3 . a2) + x), 64 output channels at a time.
    // The two lanes of a pixel first trade pieces so that lane half h holds channels 32 h .. 32 h + 32 in
    // order (bytes [64 h, 64 h + 64) of the a2 row, as a kernel that reads a2 from memory would): step j of
    // the reduction then multiplies channels 8 j .. + 8 and 32 + 8 j .. + 8, the same sixteen products per
    // MFMA, in the same order, as the per-layer 1x1 kernel - and so the same bits.
    //   before: half 0 holds [0,8) [16,24) [32,40) [48,56), half 1 holds [8,16) [24,32) [40,48) [56,64)
    //   after:  half 0 holds [0,8) [16,24) [8,16) [24,32),  half 1 holds [32,40) [48,56) [40,48) [56,64)
    {
        auto trade = [](u32x4 &lo_keeps, u32x4 &hi_keeps) {   // upper half of the first <-> lower half of the second
            uint32_t *pa = reinterpret_cast<uint32_t *>(&lo_keeps), *pb = reinterpret_cast<uint32_t *>(&hi_keeps);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                auto r = __builtin_amdgcn_permlane32_swap(pa[e], pb[e], false, false);
                pa[e] = r[0];
                pb[e] = r[1];
            }
        };
        trade(a2p[0][0], a2p[1][0]);
        trade(a2p[0][1], a2p[1][1]);
    }
    const bool mine = pi < BM && pm < M;
    const long long rm = mine ? pm : (M - 1);            // clamp: the shortcut loads stay in bounds
    const unsigned char *xres = xg + (size_t)rm * (kCin * 2);
    unsigned char *og = static_cast<unsigned char *>(a.out);
    u32x4 rv[2][2];                                      // one group at a time: the MFMAs of the group cover the latency
    auto load_res = [&](int g, u32x4 (&dst)[2][2]) {
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
            for (int i2 = 0; i2 < 2; ++i2)
                dst[u][i2] = *reinterpret_cast<const u32x4 *>(xres + (size_t)(g * 64 + u * 32 + 16 * i2 + 8 * half) * 2);
    };
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        load_res(g, rv);
        f32x16 acc[2];
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[u][e] = 0.f;
        const unsigned char *wrow = rc + (g * 64 + l32) * kPitch + half * 64;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            // step j: channels 32 half + 8 j .. + 8 - after the trade that is piece [j & 1][j >> 1]
            const u32x4 w0 = *reinterpret_cast<const u32x4 *>(wrow + j * 16);
            const u32x4 w1 = *reinterpret_cast<const u32x4 *>(wrow + 32 * kPitch + j * 16);
            acc[0] = mma(w0, a2p[j & 1][j >> 1], acc[0]);
            acc[1] = mma(w1, a2p[j & 1][j >> 1], acc[1]);
        }
        u32x4 piece[2][2];
        finish_tiles<true>(acc, f3s + g * 64, f3h + g * 64, half, rv, piece);
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
            for (int i2 = 0; i2 < 2; ++i2)
                *reinterpret_cast<u32x4 *>(ttile + l32 * kPitch + (u * 32 + 16 * i2 + 8 * half) * 2) = piece[u][i2];
        wave_fence();
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const int pr = trow + 8 * t;
            const u32x4 o4 = *reinterpret_cast<const u32x4 *>(ttile + pr * kPitch + tseg * 16);
            if (pr < rows_here && mbase + pr < M)
                *reinterpret_cast<u32x4 *>(og + ((size_t)(mbase + pr) * kCout + g * 64) * 2 + tseg * 16) = o4;
        }
        wave_fence();
    }
}

static int max_tile(int W) { return (kMaxHaloTiles * 32 - 2 * W - 2) / 8 * 8; }

}  // namespace block

const char *bottleneck_block_check(const BlockArgs &a) {
    if (a.N <= 0 || a.H <= 0 || a.W <= 0) return "non-positive dimension";
    const long long M = (long long)a.N * a.H * a.W;
    if (M != a.M || M > 0x7FFFFFFFLL / 2) return "pixel count out of range";
    if (block::max_tile(a.W) < 64) return "rows wider than 223 pixels are not supported by the block kernel";
    if (!a.x || !a.w1 || !a.w2 || !a.w3 || !a.s1 || !a.h1 || !a.s2 || !a.h2 || !a.s3 || !a.h3) return "null operand";
    if (!a.a1 && !a.a2 && !a.out) return "nothing to store";
    const uintptr_t all = (uintptr_t)a.x | (uintptr_t)a.a1 | (uintptr_t)a.a2 | (uintptr_t)a.out | (uintptr_t)a.w1 |
                          (uintptr_t)a.w2 | (uintptr_t)a.w3 | (uintptr_t)a.s1 | (uintptr_t)a.h1 | (uintptr_t)a.s2 |
                          (uintptr_t)a.h2 | (uintptr_t)a.s3 | (uintptr_t)a.h3;
    if (all & 15) return "pointers must be 16-byte aligned";
    return nullptr;
}

// Pixels per workgroup: as few rounds of 256 workgroups (one per CU) as the LDS allows, then the
// smallest tile that still gives that many rounds, so that the last round is as full as the others.
int bottleneck_block_tile(const BlockArgs &a) {
    const long long cap = block::max_tile(a.W);
    const long long rounds = (a.M + 256 * cap - 1) / (256 * cap);
    long long bm = (a.M + 256 * rounds - 1) / (256 * rounds);
    bm = (bm + 7) / 8 * 8;
    if (bm < 64) bm = 64;
    if (bm > cap) bm = cap;
    return (int)bm;
}

hipError_t launch_bottleneck_block(const BlockArgs &a, hipStream_t stream) {
    if (bottleneck_block_check(a)) return hipErrorInvalidValue;
    const int BM = bottleneck_block_tile(a);
    const int NT1 = (BM + 2 * a.W + 2 + 31) / 32, NT2 = (BM + 31) / 32;
    if (NT1 > block::kMaxHaloTiles || NT2 > block::kWaves) return hipErrorInvalidValue;
    static const hipError_t raised = hipFuncSetAttribute(reinterpret_cast<const void *>(block::bottleneck_block_kernel),
                                                         hipFuncAttributeMaxDynamicSharedMemorySize, block::kLds);
    if (raised != hipSuccess) return raised;
    const long long blocks = ((long long)a.M + BM - 1) / BM;
    block::bottleneck_block_kernel<<<dim3((unsigned)blocks), dim3(block::kThreads), block::kLds, stream>>>(a, BM, NT1, NT2);
    return hipGetLastError();
}

}  // namespace delta
