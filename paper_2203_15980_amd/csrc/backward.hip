// Backward of the fused layer y = relu?(scale_k * conv(x, w) + shift_k (+ res)) for gfx950, bf16.
//
// DELTA's planner follows the tensor accesses of a whole training iteration (Sec. 3,
// Assumptions 1-3: the backward pass reads the stored forward activations, which is why
// released ones must be regenerated or reloaded).  These kernels are that backward pass for the
// bottleneck layers, with frozen batch-norm statistics:
//
//   gpre = gy * [y > 0]                       relu_mask_kernel (also dL/dres)
//   gx   = conv^T(gpre * scale, w)            the forward kernels, run on gpre with the weights
//                                             transposed, flipped and pre-multiplied by scale
//                                             (bwd_weights_kernel)
//   gw[k,r,s,c] = scale_k * sum_m gpre[m,k] * x[m + (r,s), c]      wgrad_kernel + wgrad_reduce_kernel
//
// wgrad.  The reduction index is the pixel, and both operands are stored pixel-major (NHWC), so
// neither has its reduction axis contiguous per lane the way an MFMA operand wants it.  gfx950's
// LDS transpose read (ds_read_b64_tr_b16) does exactly that turn: 16 lanes each point at 4
// consecutive 16-bit values (four rows of 16 channels) and each lane gets one channel's 4 values
// along the rows.  So tiles are staged in LDS as they lie in memory (position rows x channels) and
// both operands are read with two transpose reads per MFMA.
// Image borders without masks: a chunk is RH image rows, laid out in LDS with the padding columns
// and rows of the convolution made explicit (row length W + 2 for 3x3), zeros there.  A tap is
// then a constant row offset, gpre is zero at the padding positions, and the reduction simply
// runs over all positions of the padded layout (a few percent more MFMAs, no per-element mask).
// One wavefront per (tap, 64 x 64 tile of [k, c]); the wavefronts of a workgroup share the staged
// tiles.  Workgroups are persistent over chunks (split s takes chunks s, s + nsplit, ...) and
// write their accumulators, in accumulator-register order, to a partial buffer; a second kernel
// adds the partials in split order and applies scale_k.  No atomics: the result is a fixed
// function of the inputs.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kernels.hpp"

namespace delta {
namespace bwd {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

static constexpr int kOutOfRange = (int)0x80000000;   // outside every buffer descriptor used here

// ---------------------------------------------------------------- gpre = gy * [y > 0]
// 16 bytes per thread, grid-stride.  bf16: y > 0 <=> sign bit clear and not zero (NaN counts as
// "not greater": the forward's ReLU passes NaN through, its gradient is taken as 0).
template <bool BF16>
__global__ __launch_bounds__(256) void relu_mask_kernel(const u32x4 *__restrict__ y, const u32x4 *__restrict__ gy,
                                                        u32x4 *__restrict__ out, size_t n16) {
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) {
        const u32x4 a = y[i], g = gy[i];
        u32x4 o;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            if constexpr (BF16) o[e] = keep_where_positive_bf16(g[e], a[e]);
            else o[e] = keep_where_positive_f32(g[e], a[e]);
        }
        out[i] = o;
    }
}

// Strided layers: the masked gradient is written at the input's resolution, out[n, s p, s q, :] =
// gy[n, p, q, :] * [y > 0] and zero everywhere else.  With that tensor the data gradient is again a
// stride-1 convolution and the weight gradient the stride-1 reduction (the zeros contribute
// nothing), at the price of stride^2 times the arithmetic.  One 16-byte piece per thread.
template <bool BF16>
__global__ __launch_bounds__(256) void relu_mask_dilate_kernel(const u32x4 *__restrict__ y, const u32x4 *__restrict__ gy,
                                                               u32x4 *__restrict__ out, int H, int W, int P, int Q,
                                                               int vec_per_pixel, int stride, size_t n16) {
    const size_t step = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += step) {
        const size_t pix = i / vec_per_pixel;
        const int v = (int)(i - pix * vec_per_pixel);
        const int w = (int)(pix % W);
        const size_t rest = pix / W;
        const int h = (int)(rest % H);
        const size_t n = rest / H;
        u32x4 o = {0u, 0u, 0u, 0u};
        const int p = h / stride, q = w / stride;
        if (p * stride == h && q * stride == w && p < P && q < Q) {
            const size_t src = ((n * P + p) * Q + q) * vec_per_pixel + v;
            const u32x4 g = gy[src];
            if (y) {
                const u32x4 a = y[src];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    if constexpr (BF16) {
                        const uint32_t lo = a[e] & 0xFFFFu, hi = a[e] >> 16;
                        const bool plo = lo != 0 && lo < 0x7F81u, phi = hi != 0 && hi < 0x7F81u;
                        o[e] = (plo ? (g[e] & 0xFFFFu) : 0u) | (phi ? (g[e] & 0xFFFF0000u) : 0u);
                    } else {
                        o[e] = __uint_as_float(a[e]) > 0.f ? g[e] : 0u;
                    }
                }
            } else {
                o = g;
            }
        }
        out[i] = o;
    }
}

// ---------------------------------------------------------------- strided 1x1 layers, directly
// A 1x1 layer with stride s reads only the pixels (s p, s q) of its input, so both of its
// gradients are stride-1 operations at the OUTPUT's resolution once those pixels are gathered:
//   xs[n,p,q,:] = x[n, s p, s q, :]                          subsample_kernel (for dL/dw)
//   t = 1x1 data gradient of gpre at P x Q
//   gx[n,h,w,:] = (t[n,h/s,w/s,:] on the grid, else 0) + gx_add, optionally * [x > 0]   spread_add_kernel
// One 16-byte piece per thread in both.
// With offsets: xs[n,p,q,:] = x[n, s p + oa, s q + ob, :], zeros where that pixel lies outside the image.
__global__ __launch_bounds__(256) void subsample_kernel(const u32x4 *__restrict__ x, u32x4 *__restrict__ xs, int H, int W,
                                                        int P, int Q, int vec_per_pixel, int stride, int oa, int ob,
                                                        size_t n16) {
    const size_t step = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += step) {
        const size_t pix = i / vec_per_pixel;
        const int v = (int)(i - pix * vec_per_pixel);
        const int q = (int)(pix % Q);
        const size_t rest = pix / Q;
        const int p = (int)(rest % P);
        const size_t n = rest / P;
        const int h = p * stride + oa, w = q * stride + ob;
        u32x4 val = {0u, 0u, 0u, 0u};
        if (h < H && w < W) val = x[((n * H + (size_t)h) * W + (size_t)w) * vec_per_pixel + v];
        xs[i] = val;
    }
}

template <bool BF16>
__global__ __launch_bounds__(256) void spread_add_kernel(const u32x4 *__restrict__ t, const u32x4 *__restrict__ add,
                                                         const u32x4 *__restrict__ mask, u32x4 *__restrict__ out, int H,
                                                         int W, int P, int Q, int vec_per_pixel, int stride, size_t n16) {
    const size_t step = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += step) {
        const size_t pix = i / vec_per_pixel;
        const int v = (int)(i - pix * vec_per_pixel);
        const int w = (int)(pix % W);
        const size_t rest = pix / W;
        const int h = (int)(rest % H);
        const size_t n = rest / H;
        const int p = h / stride, q = w / stride;
        const bool on_grid = p * stride == h && q * stride == w && p < P && q < Q;
        u32x4 o = {0u, 0u, 0u, 0u};
        if (on_grid) o = t[((n * P + p) * Q + q) * vec_per_pixel + v];
        if (add) {
            const u32x4 a = add[i];
            if (!on_grid) {
                o = a;                                   // nothing to add to: the bits pass through
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    if constexpr (BF16) {
                        const float lo = __uint_as_float(o[e] << 16) + __uint_as_float(a[e] << 16);
                        const float hi = __uint_as_float(o[e] & 0xFFFF0000u) + __uint_as_float(a[e] & 0xFFFF0000u);
                        const f32x2 pr = {lo, hi};
                        o[e] = __builtin_bit_cast(uint32_t, __builtin_convertvector(pr, bf16x2));
                    } else {
                        o[e] = __float_as_uint(__uint_as_float(o[e]) + __uint_as_float(a[e]));
                    }
                }
            }
        }
        if (mask) {
            const u32x4 m = mask[i];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                if constexpr (BF16) o[e] = keep_where_positive_bf16(o[e], m[e]);
                else o[e] = keep_where_positive_f32(o[e], m[e]);
            }
        }
        out[i] = o;
    }
}

// ---------------------------------------------------------------- weights for the data gradient
// wt[c][R-1-r][S-1-s][k] = round(w[k][r][s][c] * scale_k): the data gradient is then the forward
// convolution of gpre with wt (stride 1, padding R-1-pad).  One thread per element of wt.
template <bool BF16>
__global__ __launch_bounds__(256) void bwd_weights_kernel(const void *w, const float *scale, void *wt, int K, int R,
                                                          int S, int C) {
    const size_t total = (size_t)K * R * S * C;
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= total) return;
    const int k = (int)(i % K);
    size_t rest = i / K;
    const int s2 = (int)(rest % S); rest /= S;
    const int r2 = (int)(rest % R);
    const int c = (int)(rest / R);
    const size_t src = (((size_t)k * R + (R - 1 - r2)) * S + (S - 1 - s2)) * C + c;
    if constexpr (BF16) {
        const float v = __uint_as_float((uint32_t)static_cast<const uint16_t *>(w)[src] << 16) * scale[k];
        static_cast<__bf16 *>(wt)[i] = (__bf16)v;             // round to nearest even
    } else {
        static_cast<float *>(wt)[i] = static_cast<const float *>(w)[src] * scale[k];
    }
}

// ---------------------------------------------------------------- weight gradient
struct WgradArgs {
    const void *x;       // [N,H,W,C] bf16
    const void *g;       // [N,H,W,K] bf16 (gpre)
    float *partial;      // [nsplit][tiles_y][waves][4 tiles][4][64 lanes] f32x4
    int N, H, W, C, K, R;            // R = S in {1, 3}, stride 1, pad (R-1)/2
    int RH;              // image rows per chunk
    int QN;              // positions per chunk: RH * (W + R - 1), rounded up to 16
    int XN;              // staged activation positions: QN + (R - 1) * (W + R - 1) + (R - 1)
    int nsplit;
    unsigned long long tapwin;   // 4 bits per tap: its position r * R + s in the R x R window (a subset of the
                                 // window's taps when TAPS < R * R)
    int XH, XW, xstep, xoa, xob; // x is [N,XH,XW,C] and position (h, w) reads its pixel (h * xstep + xoa, w * xstep + xob),
                                 // zeros past the image (XH = H, XW = W, xstep = 1, offsets 0: x as it is)
};

// Which way the 64-byte groups of LDS row `row` are permuted (see wgrad_kernel): rows of 128 bytes lie two to
// a 256-byte bank line, so the line's half already separates neighbours and bit 1 of the row number flips
// the group; wider rows start a bank line each and the low two bits of the row number flip it.
template <int TW>
__device__ __forceinline__ int lds_swizzle(int row) { return TW == 1 ? (row >> 1) & 1 : row & 3; }

// KTW x CTW tiles of 64 x 64 [k, c] per workgroup and tap; TAPS = R * R, or fewer: the taps tapwin lists.
// QS wavefronts share each (tap, tile): wavefront qs of them takes the 16-position steps qs, qs + QS, ...
// of every chunk, and when the workgroup has walked all its chunks their sums are added in the order
// of qs (through LDS).  A tile's wavefront alone on its SIMD left the matrix pipe idle whenever it
// waited for its own operand reads or at the two barriers of a chunk.
template <int KTW, int CTW, int TAPS, int QS>
__global__ __launch_bounds__(KTW * CTW * TAPS * QS * 64) void wgrad_kernel(WgradArgs a) {
    constexpr int NB = KTW * CTW * TAPS, NW = NB * QS, NT = NW * 64;
    // LDS rows without padding; the 64-byte groups of a row are permuted by the row number instead
    // (group ^ swizzle(row)), so that the four consecutive rows a transposing read touches at one
    // column lie in four different quarters of the 64 banks (with padded rows of 144 / 272 bytes half
    // of the LDS-active cycles of this kernel were bank conflicts)
    constexpr int GP = KTW * 128, XP = CTW * 128;               // LDS row pitches (bytes)
    constexpr int GSEG = KTW * 8, XSEG = CTW * 8;               // 16-byte segments per row
    constexpr int MAXL = NT >= 512 ? 4 : 8;                      // staged 16-byte pieces per thread, each operand
    extern __shared__ __align__(16) unsigned char smem[];
    unsigned char *gs = smem;                                    // [QN][GP]
    unsigned char *xs = smem + (size_t)a.QN * GP;                // [XN][XP]

    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int base = wv % NB, qs = wv / NB;
    const int tap = base % TAPS, kw = (base / TAPS) % KTW, cw = base / (TAPS * KTW);
    const int B = (a.R - 1) / 2, Wp = a.W + 2 * B;
    const int win = (int)((a.tapwin >> (4 * tap)) & 15);
    const int r = win / a.R, s = win - r * a.R;
    const int tapoff = a.R == 1 ? 0 : r * Wp + s;               // activation row of position q is q + tapoff
    const int ktiles = a.K / (64 * KTW);
    const int ty = blockIdx.y, ct = ty / ktiles, kt = ty - ct * ktiles;   // channel tile groups of this workgroup
    const int HB = (a.H + a.RH - 1) / a.RH;
    const int nchunks = a.N * HB;

    const __amdgpu_buffer_rsrc_t xrsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<void *>(a.x), 0, (int)((size_t)a.N * a.XH * a.XW * a.C * 2), 0x00020000);
    const __amdgpu_buffer_rsrc_t grsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<void *>(a.g), 0, (int)((size_t)a.N * a.H * a.W * a.K * 2), 0x00020000);

    // ---- what this thread stages: piece p covers LDS row (tid + p NT) / SEG, segment % SEG.
    // Per piece: image row relative to the chunk's first row, image column (or -1: a padding
    // position, always zero), and the byte offset of the channel segment.
    int g_row[MAXL], g_col[MAXL], x_row[MAXL], x_col[MAXL];
#pragma unroll
    for (int p = 0; p < MAXL; ++p) {
        const int idx = tid + p * NT;
        {
            const int q = idx / GSEG;                            // position
            const int pr = q / Wp, pc = q - pr * Wp;
            const bool ok = q < a.RH * Wp && pc >= B && pc < B + a.W;
            g_row[p] = q < a.QN ? pr : -2;                       // -2: this thread has no such piece
            g_col[p] = ok ? pc - B : -1;
        }
        {
            const int j = idx / XSEG;                            // staged activation row
            // row j holds padded coordinate f = j - B: padded row f / Wp - B, padded column f % Wp
            const int f = j - B;
            const int pr = f >= 0 ? f / Wp : 0, pc = f >= 0 ? f - pr * Wp : 0;
            const bool ok = f >= 0 && pc >= B && pc < B + a.W;
            x_row[p] = j < a.XN ? pr - B : -1000000;             // relative image row (may be -1 or RH)
            x_col[p] = ok ? pc - B : -1;
        }
    }

    f32x16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    u32x4 rg[MAXL], rx[MAXL];
    auto fetch = [&](int chunk) {                                // chunk >= nchunks: zeros
        const bool live = chunk < nchunks;
        const int n = chunk / HB, h0 = (chunk - n * HB) * a.RH;
#pragma unroll
        for (int p = 0; p < MAXL; ++p) {
            const int idx = tid + p * NT;
            {
                const int h = h0 + g_row[p];
                const bool ok = live && g_row[p] >= 0 && g_col[p] >= 0 && h < a.H;
                const int off = (int)((((size_t)n * a.H + h) * a.W + g_col[p]) * a.K * 2) + kt * (KTW * 128) + (idx % GSEG) * 16;
                rg[p] = __builtin_amdgcn_raw_buffer_load_b128(grsrc, ok ? off : kOutOfRange, 0, 0);
            }
            {
                const int h = h0 + x_row[p];
                const int xh = h * a.xstep + a.xoa, xw = x_col[p] * a.xstep + a.xob;
                const bool ok = live && x_col[p] >= 0 && h >= 0 && h < a.H && x_row[p] > -1000 && xh < a.XH && xw < a.XW;
                const int off = (int)((((size_t)n * a.XH + xh) * a.XW + xw) * a.C * 2) + ct * (CTW * 128) + (idx % XSEG) * 16;
                rx[p] = __builtin_amdgcn_raw_buffer_load_b128(xrsrc, ok ? off : kOutOfRange, 0, 0);
            }
        }
    };
    auto stage = [&]() {
#pragma unroll
        for (int p = 0; p < MAXL; ++p) {
            const int idx = tid + p * NT;
            if (g_row[p] != -2) {
                const int row = idx / GSEG, seg = idx % GSEG;
                *reinterpret_cast<u32x4 *>(gs + row * GP + (((seg >> 2) ^ lds_swizzle<KTW>(row)) << 6) + (seg & 3) * 16) = rg[p];
            }
            if (x_row[p] > -1000) {
                const int row = idx / XSEG, seg = idx % XSEG;
                *reinterpret_cast<u32x4 *>(xs + row * XP + (((seg >> 2) ^ lds_swizzle<CTW>(row)) << 6) + (seg & 3) * 16) = rx[p];
            }
        }
    };

    // transpose-read addressing: lane supplies row (lane % 16) / 4 of a 4-row group and columns
    // 16 * ((lane / 16) % 2) + 4 * (lane % 4) .. +3 of a 32-channel tile; it receives channel
    // lane % 32 of the tile, rows 0..3 of the group.  Lanes 32..63 take positions 8..15 of a step.
    const int srow = (lane & 15) >> 2;
    const int scol = 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
    const int kgrp = lane >> 5;
    // the rows a lane reads are its first row plus multiples of 4 (q0 and the second half of a step), so the
    // swizzle of all of them is that of the first; the two 32-channel halves t of the tile are groups 2 w + t
    const int grow = 8 * kgrp + srow, xrow = 8 * kgrp + srow + tapoff;
    const unsigned char *gbase = gs + (size_t)grow * GP + scol * 2;
    const unsigned char *xbase = xs + (size_t)xrow * XP + scol * 2;
    int goff[2], xoff[2];
#pragma unroll
    for (int t = 0; t < 2; ++t) {
        goff[t] = ((kw * 2 + t) ^ lds_swizzle<KTW>(grow)) << 6;
        xoff[t] = ((cw * 2 + t) ^ lds_swizzle<CTW>(xrow)) << 6;
    }
    typedef s16x4 __attribute__((address_space(3))) * lds_s16x4_ptr;
    auto tr_read = [&](const unsigned char *p) {
        return __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(p));
    };

    int chunk = blockIdx.x;
    fetch(chunk);
    for (; chunk < nchunks; chunk += a.nsplit) {
        __syncthreads();                                         // every wavefront is done with the tiles
        stage();
        fetch(chunk + a.nsplit);                                 // next chunk of this split in flight
        __syncthreads();
        for (int q0 = 16 * qs; q0 < a.QN; q0 += 16 * QS) {
            s16x8 af[2], bf[2];
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                const s16x4 a0 = tr_read(gbase + (size_t)q0 * GP + goff[t]);
                const s16x4 a1 = tr_read(gbase + (size_t)(q0 + 4) * GP + goff[t]);
                af[t] = __builtin_shufflevector(a0, a1, 0, 1, 2, 3, 4, 5, 6, 7);
                const s16x4 b0 = tr_read(xbase + (size_t)q0 * XP + xoff[t]);
                const s16x4 b1 = tr_read(xbase + (size_t)(q0 + 4) * XP + xoff[t]);
                bf[t] = __builtin_shufflevector(b0, b1, 0, 1, 2, 3, 4, 5, 6, 7);
            }
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                        __builtin_bit_cast(bf16x8, af[i]), __builtin_bit_cast(bf16x8, bf[j]), acc[i][j], 0, 0, 0);
        }
    }

    // ---- the QS sums of a tile, added in the order of qs
    if constexpr (QS > 1) {
        __syncthreads();                                         // the staged tiles are dead
        float *red = reinterpret_cast<float *>(smem);            // [QS - 1][NB][i][j][e4][lane] x f32x4
        if (qs > 0) {
            float *dst = red + (size_t)((qs - 1) * NB + base) * 4096;
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
#pragma unroll
                    for (int e4 = 0; e4 < 4; ++e4) {
                        const f32x4 v = {acc[i][j][4 * e4], acc[i][j][4 * e4 + 1], acc[i][j][4 * e4 + 2], acc[i][j][4 * e4 + 3]};
                        *reinterpret_cast<f32x4 *>(dst + ((((i * 2 + j) * 4 + e4) * 64 + lane) * 4)) = v;
                    }
        }
        __syncthreads();
        if (qs > 0) return;
#pragma unroll
        for (int g = 1; g < QS; ++g) {
            const float *src = red + (size_t)((g - 1) * NB + base) * 4096;
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
#pragma unroll
                    for (int e4 = 0; e4 < 4; ++e4) {
                        const f32x4 v = *reinterpret_cast<const f32x4 *>(src + ((((i * 2 + j) * 4 + e4) * 64 + lane) * 4));
                        acc[i][j][4 * e4] += v.x; acc[i][j][4 * e4 + 1] += v.y;
                        acc[i][j][4 * e4 + 2] += v.z; acc[i][j][4 * e4 + 3] += v.w;
                    }
        }
    }
    // ---- partial sums, accumulator-register order: [split][ty][wave][i][j][e4][lane] x f32x4
    float *out = a.partial + ((((size_t)blockIdx.x * gridDim.y + ty) * NB + base) * 4) * (4 * 64 * 4);
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int e4 = 0; e4 < 4; ++e4) {
                const f32x4 v = {acc[i][j][4 * e4], acc[i][j][4 * e4 + 1], acc[i][j][4 * e4 + 2], acc[i][j][4 * e4 + 3]};
                *reinterpret_cast<f32x4 *>(out + ((((i * 2 + j) * 4 + e4) * 64 + lane) * 4)) = v;
            }
}

// gw[k][tap][c] = scale_k * sum over splits of the partial sums, in a fixed order.  A group of
// 64 consecutive f32x4 of the blob (one per lane) is shared by G wavefronts (wavefront g of the
// group adds splits g, g + G, ..., four loads in flight), whose G sums are then added in wavefront
// order; a workgroup of 8 wavefronts takes 8 / G groups.  G follows the number of splits (about
// four loads per lane): with few splits (the wide layers: 4 or 16) every wavefront still has
// loads to issue, with many (256) the loads of a group are spread over the whole workgroup.  (Splitting
// a wavefront's lanes over four splits as well - 256 workgroups instead of 64 for the single-tile layers,
// eight loads in flight - makes this kernel faster alone, 4 us at best, and the backward pass 3 % slower:
// beside the data-gradient stream its time is mostly waiting for free CUs, and more workgroups wait more.)  The
// accumulator layout of a 32x32 tile is: lane l holds column l % 32 and rows 8 e4 + 4 (l / 32) + e
// in register 4 e4 + e, so a thread's four sums go to four k rows of one c, and consecutive lanes
// write consecutive c.
// gw_taps: taps per (k, c) pair in gw; tapout: 4 bits per tap of this launch, its index among them.
template <int G>
__global__ __launch_bounds__(512) void wgrad_reduce_kernel(const float *partial, const float *scale, float *gw, int K,
                                                           int C, int taps, int KTW, int CTW, int nsplit, int gw_taps,
                                                           unsigned long long tapout) {
    __shared__ f32x4 part[8][64];
    const int ktiles = K / (64 * KTW), tiles_y = (C / (64 * CTW)) * ktiles;
    const int NW = KTW * CTW * taps;
    const size_t per_split = (size_t)tiles_y * NW * 1024;      // f32x4 elements per split (a multiple of 512)
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int grp = wave % G, sub = wave / G;
    const size_t idx = ((size_t)blockIdx.x * (8 / G) + sub) * 64 + lane;
    const f32x4 *src = reinterpret_cast<const f32x4 *>(partial) + idx;
    f32x4 sum = {0.f, 0.f, 0.f, 0.f};
    int sp = grp;
    for (; sp + 3 * G < nsplit; sp += 4 * G) {                 // four independent loads in flight
        const f32x4 v0 = src[(size_t)sp * per_split], v1 = src[(size_t)(sp + G) * per_split];
        const f32x4 v2 = src[(size_t)(sp + 2 * G) * per_split], v3 = src[(size_t)(sp + 3 * G) * per_split];
        sum += v0; sum += v1; sum += v2; sum += v3;
    }
    for (; sp < nsplit; sp += G) sum += src[(size_t)sp * per_split];
    if constexpr (G > 1) {
        part[wave][lane] = sum;
        __syncthreads();
        if (grp != 0) return;
#pragma unroll
        for (int g = 1; g < G; ++g) sum += part[wave + g][lane];
    }
    // idx = (((ty * NW + wv) * 4 + tile) * 4 + e4) * 64 + lane
    const int e4 = (int)((idx >> 6) & 3), tile = (int)((idx >> 8) & 3);
    const int wv = (int)((idx >> 10) % NW), ty = (int)((idx >> 10) / NW);
    const int tap = wv % taps, kw = (wv / taps) % KTW, cw = wv / (taps * KTW);
    const int ct = ty / ktiles, kt = ty - ct * ktiles;
    const int i = tile >> 1, j = tile & 1;
    const int c = (ct * CTW + cw) * 64 + j * 32 + (lane & 31);
    const int k0 = (kt * KTW + kw) * 64 + i * 32 + 8 * e4 + 4 * (lane >> 5);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const int k = k0 + e;
        gw[((size_t)k * gw_taps + (int)((tapout >> (4 * tap)) & 15)) * C + c] = sum[e] * scale[k];
    }
}

// fp32 layers (the small correctness configuration): plain fp32 multiply-adds.  One workgroup per
// 16 x 16 tile of (k, c) and tap; thread (kk, cc) walks every position in order, 64 at a time through
// LDS, so there are no partial sums, no workspace and one fixed order of summation.
// g: [N,H,W,K] (dL/d(pre-activation) at the input's resolution), x: [N,H,W,C], gw: [K][R][R][C].
__global__ __launch_bounds__(256) void wgrad_f32_kernel(const float *x, const float *g, const float *scale, float *gw,
                                                        int N, int H, int W, int C, int K, int R, int pad) {
    __shared__ float gs[64][17], xs[64][17];
    const int t = threadIdx.x, kk = t >> 4, cc = t & 15;
    const int k0 = blockIdx.x * 16, c0 = blockIdx.y * 16, tap = blockIdx.z;
    const int r = tap / R, s = tap % R;
    const long long M = (long long)N * H * W;
    float acc = 0.f;
    for (long long m0 = 0; m0 < M; m0 += 64) {
        for (int i = t; i < 1024; i += 256) {
            const int p = i >> 4, ch = i & 15;
            const long long m = m0 + p;
            float gv = 0.f, xv = 0.f;
            if (m < M) {
                gv = g[(size_t)m * K + k0 + ch];
                const int w_ = (int)(m % W), h_ = (int)((m / W) % H);
                const long long n = m / ((long long)W * H);
                const int ih = h_ + r - pad, iw = w_ + s - pad;
                if (ih >= 0 && ih < H && iw >= 0 && iw < W) xv = x[((size_t)(n * H + ih) * W + iw) * C + c0 + ch];
            }
            gs[p][ch] = gv;
            xs[p][ch] = xv;
        }
        __syncthreads();
#pragma unroll 16
        for (int p = 0; p < 64; ++p) acc += gs[p][kk] * xs[p][cc];
        __syncthreads();
    }
    gw[((size_t)(k0 + kk) * R * R + tap) * C + c0 + cc] = acc * scale[k0 + kk];
}

}  // namespace bwd

// ---------------------------------------------------------------- host side

hipError_t launch_relu_mask(const void *y, const void *gy, void *out, size_t bytes, int bf16, hipStream_t stream) {
    if (bytes % 16) return hipErrorInvalidValue;
    const size_t n16 = bytes / 16;
    if (n16 == 0) return hipSuccess;
    size_t blocks = (n16 + 255) / 256;
    if (blocks > 256 * 16) blocks = 256 * 16;
    if (bf16)
        bwd::relu_mask_kernel<true><<<dim3((unsigned)blocks), dim3(256), 0, stream>>>(
            static_cast<const bwd::u32x4 *>(y), static_cast<const bwd::u32x4 *>(gy), static_cast<bwd::u32x4 *>(out), n16);
    else
        bwd::relu_mask_kernel<false><<<dim3((unsigned)blocks), dim3(256), 0, stream>>>(
            static_cast<const bwd::u32x4 *>(y), static_cast<const bwd::u32x4 *>(gy), static_cast<bwd::u32x4 *>(out), n16);
    return hipGetLastError();
}

// y may be null (no ReLU).  out: [N,H,W,K]; gy, y: [N,P,Q,K].
hipError_t launch_relu_mask_dilate(const void *y, const void *gy, void *out, int N, int H, int W, int P, int Q, int K,
                                   int stride, int bf16, hipStream_t stream) {
    const size_t row_bytes = (size_t)K * (bf16 ? 2 : 4);
    if (row_bytes % 16 || stride < 1) return hipErrorInvalidValue;
    const size_t n16 = (size_t)N * H * W * (row_bytes / 16);
    if (n16 == 0) return hipSuccess;
    size_t blocks = (n16 + 255) / 256;
    if (blocks > 256 * 16) blocks = 256 * 16;
    if (bf16)
        bwd::relu_mask_dilate_kernel<true><<<dim3((unsigned)blocks), dim3(256), 0, stream>>>(
            static_cast<const bwd::u32x4 *>(y), static_cast<const bwd::u32x4 *>(gy), static_cast<bwd::u32x4 *>(out), H, W,
            P, Q, (int)(row_bytes / 16), stride, n16);
    else
        bwd::relu_mask_dilate_kernel<false><<<dim3((unsigned)blocks), dim3(256), 0, stream>>>(
            static_cast<const bwd::u32x4 *>(y), static_cast<const bwd::u32x4 *>(gy), static_cast<bwd::u32x4 *>(out), H, W,
            P, Q, (int)(row_bytes / 16), stride, n16);
    return hipGetLastError();
}

// xs: [N,P,Q,C] = x[N,H,W,C] at the pixels (stride p, stride q).
hipError_t launch_subsample(const void *x, void *xs, int N, int H, int W, int P, int Q, int C, int stride, int bf16,
                            hipStream_t stream, int oa, int ob) {
    const size_t row_bytes = (size_t)C * (bf16 ? 2 : 4);
    if (row_bytes % 16 || stride < 1 || oa < 0 || ob < 0 || oa >= stride || ob >= stride) return hipErrorInvalidValue;
    if (oa == 0 && ob == 0 && ((P - 1) * stride >= H || (Q - 1) * stride >= W)) return hipErrorInvalidValue;
    const size_t n16 = (size_t)N * P * Q * (row_bytes / 16);
    if (n16 == 0) return hipSuccess;
    size_t blocks = (n16 + 255) / 256;
    if (blocks > 256 * 16) blocks = 256 * 16;
    bwd::subsample_kernel<<<dim3((unsigned)blocks), dim3(256), 0, stream>>>(
        static_cast<const bwd::u32x4 *>(x), static_cast<bwd::u32x4 *>(xs), H, W, P, Q, (int)(row_bytes / 16), stride, oa, ob,
        n16);
    return hipGetLastError();
}

// out[N,H,W,C] = t[N,P,Q,C] spread to the pixels (stride p, stride q), zero elsewhere, + add (may
// be null), then zero where mask (may be null) is not > 0.
hipError_t launch_spread_add(const void *t, const void *add, const void *mask, void *out, int N, int H, int W, int P,
                             int Q, int C, int stride, int bf16, hipStream_t stream) {
    const size_t row_bytes = (size_t)C * (bf16 ? 2 : 4);
    if (row_bytes % 16 || stride < 1 || (P - 1) * stride >= H || (Q - 1) * stride >= W) return hipErrorInvalidValue;
    const size_t n16 = (size_t)N * H * W * (row_bytes / 16);
    if (n16 == 0) return hipSuccess;
    size_t blocks = (n16 + 255) / 256;
    if (blocks > 256 * 16) blocks = 256 * 16;
    const auto *tp = static_cast<const bwd::u32x4 *>(t);
    const auto *ap = static_cast<const bwd::u32x4 *>(add);
    const auto *mp = static_cast<const bwd::u32x4 *>(mask);
    auto *op = static_cast<bwd::u32x4 *>(out);
    if (bf16)
        bwd::spread_add_kernel<true><<<dim3((unsigned)blocks), dim3(256), 0, stream>>>(tp, ap, mp, op, H, W, P, Q,
                                                                                        (int)(row_bytes / 16), stride, n16);
    else
        bwd::spread_add_kernel<false><<<dim3((unsigned)blocks), dim3(256), 0, stream>>>(tp, ap, mp, op, H, W, P, Q,
                                                                                         (int)(row_bytes / 16), stride, n16);
    return hipGetLastError();
}

hipError_t launch_bwd_weights(const void *w, const float *scale, void *wt, int K, int R, int S, int C, int bf16,
                              hipStream_t stream) {
    const size_t total = (size_t)K * R * S * C;
    if (total == 0 || total > 0x7FFFFFFFull) return hipErrorInvalidValue;
    const unsigned blocks = (unsigned)((total + 255) / 256);
    if (bf16) bwd::bwd_weights_kernel<true><<<dim3(blocks), dim3(256), 0, stream>>>(w, scale, wt, K, R, S, C);
    else bwd::bwd_weights_kernel<false><<<dim3(blocks), dim3(256), 0, stream>>>(w, scale, wt, K, R, S, C);
    return hipGetLastError();
}

namespace {

struct WgradPlan {
    int ktw, ctw, taps, rh, qn, xn, nsplit, tiles_y, waves, qs;   // waves: (tap, tile) pairs; qs wavefronts on each
    size_t lds, partial_bytes;
};

// nullptr and a filled plan, or the reason the weight-gradient kernel does not apply.
// A 1x1 layer has no neighbourhood: its positions are one flat list, which is cut into rows of 64
// (or 32, 16) so that every chunk is full whatever the image size (7 x 7 images gave chunks of 49).
ConvArgs flattened_1x1(const ConvArgs &a) {
    ConvArgs f = a;
    if (a.R != 1 || a.S != 1) return f;
    const long long M = (long long)a.N * a.H * a.W;
    for (int w : {64, 32, 16})
        if (M % w == 0) {
            f.N = 1; f.H = (int)(M / w); f.W = w; f.P = f.H; f.Q = f.W;
            break;
        }
    return f;
}

// Wavefronts per (tap, tile) pair: as many as make a workgroup of 8 (two per SIMD; with 16 the kernel
// spills at 128 registers).  ResNet-50's backward pass at batch 128: 5.76 -> 5.69 ms.
int wgrad_qs(int pairs) {
    int qs = 8 / pairs;
    if (qs < 1) qs = 1;
    if (qs > 8) qs = 8;
    while (qs & (qs - 1)) --qs;                    // 1, 2, 4, 8
    return qs;
}

// ntaps: 0 = all R * S taps; 1, 2 or 4 = a subset of a 3 x 3 window's taps (the strided layers' parity classes)
const char *wgrad_plan(const ConvArgs &a_in, WgradPlan &p, int ntaps = 0) {
    const ConvArgs a = flattened_1x1(a_in);
    if (!a.bf16) return "weight gradient: bf16 only";
    if (a.R != a.S || (a.R != 1 && a.R != 3) || a.stride != 1 || a.pad != (a.R - 1) / 2)
        return "weight gradient: 1x1 or 3x3, stride 1, same padding only";
    if (a.Cin % 64 || a.Cout % 64) return "weight gradient: channel counts must be multiples of 64";
    if ((unsigned long long)a.M * a.Cin * 2ull >= 0x7FFFFFFFull || (unsigned long long)a.M * a.Cout * 2ull >= 0x7FFFFFFFull)
        return "weight gradient: tensors of 2 GiB or more";
    p.taps = ntaps ? ntaps : a.R * a.S;
    if (ntaps && (a.R != 3 || (ntaps != 1 && ntaps != 2 && ntaps != 4) || a.Cin % 128 || a.Cout % 128))
        return "weight gradient: a tap subset needs a 3x3 window and channel counts that are multiples of 128";
    if (p.taps == 9) { p.ktw = 1; p.ctw = 1; }
    else if (ntaps) { p.ktw = 2; p.ctw = ntaps == 4 ? 1 : 2; }        // eight wavefronts either way
    else {
        p.ktw = a.Cout % 256 == 0 ? 4 : (a.Cout % 128 == 0 ? 2 : 1);
        // 128 x 128 tiles where both channel counts allow: the staging registers then hold chunks of
        // 128 positions instead of 64 (twice the MFMAs between barriers; measured 1-2 % of the pass)
        if (p.ktw == 4 && a.Cin % 128 == 0) p.ktw = 2;
        p.ctw = 1;
        // (256 x 128 tiles with 8 wavefronts measured 2-3 % slower on ResNet-50's stage 4/5 layers)
        if (p.ktw == 1) p.ctw = a.Cin % 256 == 0 ? 4 : (a.Cin % 128 == 0 ? 2 : 1);
        else if (p.ktw == 2) p.ctw = a.Cin % 128 == 0 ? 2 : 1;
    }
    p.waves = p.ktw * p.ctw * p.taps;
    p.qs = wgrad_qs(p.waves);
    while ((size_t)(p.qs - 1) * p.waves * 4096 * sizeof(float) > 160 * 1024) p.qs >>= 1;   // their sums meet in LDS
    const int Wp = a.W + (a.R - 1);
    // image rows per chunk: up to about 256 positions, and at most maxl staged pieces per thread
    int rh = (256 + Wp - 1) / Wp;
    if (rh < 1) rh = 1;
    if (rh > a.H) rh = a.H;
    const int nt = p.waves * p.qs * 64;
    const long long maxl = nt >= 512 ? 4 : 8;      // as in the kernel
    const size_t red = (size_t)(p.qs - 1) * p.waves * 4096 * sizeof(float);   // the sums of the extra wavefronts
    for (;; --rh) {
        p.rh = rh;
        p.qn = (rh * Wp + 15) / 16 * 16;
        p.xn = p.qn + (a.R - 1) * Wp + (a.R - 1);
        const long long gpieces = (long long)p.qn * p.ktw * 8, xpieces = (long long)p.xn * p.ctw * 8;
        p.lds = (size_t)p.qn * (p.ktw * 128) + (size_t)p.xn * (p.ctw * 128);
        if (gpieces <= maxl * nt && xpieces <= maxl * nt && p.lds <= 160 * 1024) break;
        if (rh == 1) return "weight gradient: image row too wide for one chunk";
    }
    {
        // chunks of equal height: 14 rows are 7 + 7, not 12 + 2 (the staging cost of a chunk is the
        // same however few rows it holds)
        const int per_image = (a.H + p.rh - 1) / p.rh;
        const int even = (a.H + per_image - 1) / per_image;
        if (even < p.rh) {
            p.rh = even;
            p.qn = (even * Wp + 15) / 16 * 16;
            p.xn = p.qn + (a.R - 1) * Wp + (a.R - 1);
            p.lds = (size_t)p.qn * (p.ktw * 128) + (size_t)p.xn * (p.ctw * 128);
        }
    }
    if (p.lds < red) p.lds = red;
    p.tiles_y = (a.Cin / (64 * p.ctw)) * (a.Cout / (64 * p.ktw));
    const int chunks = a.N * ((a.H + p.rh - 1) / p.rh);
    // one workgroup per CU in all: with two (512) the partial sums double and a ResNet-50 backward pass was
    // 2 % slower, with 384 1 %, with half of the CUs (128) 16 %
    int ns = 256 / p.tiles_y;
    if (ns < 1) ns = 1;
    if (ns > 256) ns = 256;
    if (ns > chunks) ns = chunks;
    p.nsplit = ns;
    p.partial_bytes = (size_t)p.nsplit * p.tiles_y * p.waves * 4 * (4 * 64 * 4) * sizeof(float);
    return nullptr;
}

template <int KTW, int CTW, int TAPS, int QS>
hipError_t launch_wgrad_q(const bwd::WgradArgs &wa, const WgradPlan &p, hipStream_t stream) {
    if constexpr (KTW * CTW * TAPS * QS > 9) {      // wgrad_plan never asks for more (nine taps, or eight wavefronts)
        return hipErrorInvalidValue;
    } else {
        static bool raised = false;
        if (!raised) {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&bwd::wgrad_kernel<KTW, CTW, TAPS, QS>),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
            if (e != hipSuccess) return e;
            raised = true;
        }
        bwd::wgrad_kernel<KTW, CTW, TAPS, QS><<<dim3(p.nsplit, p.tiles_y), dim3(KTW * CTW * TAPS * QS * 64), p.lds, stream>>>(wa);
        return hipGetLastError();
    }
}

template <int KTW, int CTW, int TAPS>
hipError_t launch_wgrad_t(const bwd::WgradArgs &wa, const WgradPlan &p, hipStream_t stream) {
    switch (p.qs) {
    case 1: return launch_wgrad_q<KTW, CTW, TAPS, 1>(wa, p, stream);
    case 2: return launch_wgrad_q<KTW, CTW, TAPS, 2>(wa, p, stream);
    case 4: return launch_wgrad_q<KTW, CTW, TAPS, 4>(wa, p, stream);
    case 8: return launch_wgrad_q<KTW, CTW, TAPS, 8>(wa, p, stream);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace

// fp32: the plain kernel
static const char *wgrad_f32_check(const ConvArgs &a) {
    if (a.R != a.S || (a.R != 1 && a.R != 3) || a.stride != 1 || a.pad != (a.R - 1) / 2)
        return "weight gradient: 1x1 or 3x3, stride 1, same padding only";
    if (a.Cin % 16 || a.Cout % 16) return "weight gradient (fp32): channel counts must be multiples of 16";
    if (a.N < 1 || a.H < 1 || a.W < 1 || a.Cout / 16 > 65535 || a.Cin / 16 > 65535)
        return "weight gradient (fp32): empty or oversized layer";
    return nullptr;
}

const char *wgrad_check(const ConvArgs &a) {
    if (!a.bf16) return wgrad_f32_check(a);
    WgradPlan p;
    return wgrad_plan(a, p);
}

size_t wgrad_workspace_bytes(const ConvArgs &a) {
    WgradPlan p;
    return wgrad_plan(a, p) ? 0 : p.partial_bytes;
}

namespace {

// One weight-gradient launch + its reduction.  ntaps / tapwin: see wgrad_plan and WgradArgs; the
// sums go to taps tapout (4 bits each) of a gw with gw_taps taps per (k, c).
struct XView { int XH, XW, step, oa, ob; };                  // see WgradArgs; XH = 0: x as it is

hipError_t run_wgrad(const ConvArgs &a, const void *g, float *gw, void *workspace, size_t workspace_bytes, int ntaps,
                     unsigned long long tapwin, int gw_taps, unsigned long long tapout, hipStream_t stream,
                     XView xv = XView{0, 0, 1, 0, 0}) {
    WgradPlan p;
    if (wgrad_plan(a, p, ntaps) || !g || !gw || !workspace || workspace_bytes < p.partial_bytes ||
        ((uintptr_t)workspace | (uintptr_t)g | (uintptr_t)a.x) & 15)
        return hipErrorInvalidValue;
    const ConvArgs f = flattened_1x1(a);
    bwd::WgradArgs wa;
    wa.x = a.x; wa.g = g; wa.partial = static_cast<float *>(workspace);
    wa.N = f.N; wa.H = f.H; wa.W = f.W; wa.C = a.Cin; wa.K = a.Cout; wa.R = a.R;
    wa.RH = p.rh; wa.QN = p.qn; wa.XN = p.xn; wa.nsplit = p.nsplit;
    wa.tapwin = tapwin;
    wa.XH = xv.XH ? xv.XH : f.H; wa.XW = xv.XH ? xv.XW : f.W; wa.xstep = xv.step; wa.xoa = xv.oa; wa.xob = xv.ob;
    if ((unsigned long long)f.N * wa.XH * wa.XW * a.Cin * 2ull >= 0x7FFFFFFFull) return hipErrorInvalidValue;
    hipError_t e;
    const int key = p.taps * 100 + p.ktw * 10 + p.ctw;
    switch (key) {
    case 911: e = launch_wgrad_t<1, 1, 9>(wa, p, stream); break;
    case 421: e = launch_wgrad_t<2, 1, 4>(wa, p, stream); break;
    case 222: e = launch_wgrad_t<2, 2, 2>(wa, p, stream); break;
    case 111: e = launch_wgrad_t<1, 1, 1>(wa, p, stream); break;
    case 112: e = launch_wgrad_t<1, 2, 1>(wa, p, stream); break;
    case 114: e = launch_wgrad_t<1, 4, 1>(wa, p, stream); break;
    case 121: e = launch_wgrad_t<2, 1, 1>(wa, p, stream); break;
    case 122: e = launch_wgrad_t<2, 2, 1>(wa, p, stream); break;
    case 141: e = launch_wgrad_t<4, 1, 1>(wa, p, stream); break;
    default: return hipErrorInvalidValue;
    }
    if (e != hipSuccess) return e;
    const size_t quads = (size_t)p.tiles_y * p.waves * 1024;   // f32x4 elements of one split
    // wavefronts per group of 64 sums: about four splits each
    const int G = p.nsplit <= 4 ? 1 : p.nsplit <= 8 ? 2 : p.nsplit <= 16 ? 4 : 8;
    const dim3 grid((unsigned)(quads / 64 / (8 / G)));
#define DELTA_REDUCE(g)                                                                                             \
    bwd::wgrad_reduce_kernel<g><<<grid, dim3(512), 0, stream>>>(wa.partial, a.scale, gw, a.Cout, a.Cin, p.taps,     \
                                                                p.ktw, p.ctw, p.nsplit, gw_taps, tapout)
    switch (G) {
    case 1: DELTA_REDUCE(1); break;
    case 2: DELTA_REDUCE(2); break;
    case 4: DELTA_REDUCE(4); break;
    default: DELTA_REDUCE(8); break;
    }
#undef DELTA_REDUCE
    return hipGetLastError();
}

const unsigned long long kAllTaps = 0x876543210ull;             // tap t of 9 is window position t and output tap t

// The parity classes of a 3x3 stride-2 pad-1 layer.  x[2p + r - 1] is, for r = 1, pixel p of the even
// rows; for r = 0 and r = 2, pixels p - 1 and p of the odd rows.  So against the class tensor
// X_ab[n,i,j,:] = x[n, 2i + a, 2j + b, :] (zeros past the image) the layer's weight gradient is a
// stride-1 weight gradient at the output's resolution that needs, per dimension, window position 1
// (shift 0) for class 0 and window positions 0 and 1 (shifts -1, 0) for class 1 - these feed the
// layer's taps 1, and 0 and 2.
struct S2Class { int a, b, ntaps; unsigned long long tapwin, tapout; };
const S2Class kS2Classes[4] = {
    {0, 0, 1, 0x4ull, 0x4ull},                                   // window (1,1) -> layer tap (1,1)
    {0, 1, 2, 0x43ull, 0x53ull},                                 // window (1,0), (1,1) -> layer taps (1,0), (1,2)
    {1, 0, 2, 0x41ull, 0x71ull},                                 // window (0,1), (1,1) -> layer taps (0,1), (2,1)
    {1, 1, 4, 0x4310ull, 0x8620ull},                             // window (0,0), (0,1), (1,0), (1,1) -> (0,0), (0,2), (2,0), (2,2)
};

ConvArgs s2_class_layer(const ConvArgs &a, const S2Class &, const void *cls) {
    ConvArgs ca = a;
    ca.H = a.P; ca.W = a.Q; ca.stride = 1;
    ca.R = ca.S = 3;
    ca.pad = 1;
    ca.M = a.N * a.P * a.Q;
    ca.x = cls;
    return ca;
}

}  // namespace

// a: the forward layer's geometry with a.x = x, a.scale = scale; g = gpre [N,P,Q,Cout]; gw fp32
// [Cout][R][S][Cin]; workspace of at least wgrad_workspace_bytes(a), 16-byte aligned.
hipError_t launch_wgrad(const ConvArgs &a, const void *g, float *gw, void *workspace, size_t workspace_bytes,
                        hipStream_t stream) {
    const int taps = a.R * a.S;
    if (!a.bf16) {                                               // no workspace
        if (wgrad_f32_check(a) || !a.x || !a.scale || !g || !gw) return hipErrorInvalidValue;
        bwd::wgrad_f32_kernel<<<dim3(a.Cout / 16, a.Cin / 16, taps), dim3(256), 0, stream>>>(
            static_cast<const float *>(a.x), static_cast<const float *>(g), a.scale, gw, a.N, a.H, a.W, a.Cin, a.Cout, a.R,
            a.pad);
        return hipGetLastError();
    }
    return run_wgrad(a, g, gw, workspace, workspace_bytes, 0, taps == 9 ? kAllTaps : 0ull, taps, taps == 9 ? kAllTaps : 0ull,
                     stream);
}

// The weight gradient of a 3x3 stride-2 pad-1 bf16 layer by parity class, from dL/d(pre-activation)
// at the OUTPUT's resolution: four weight gradients at that resolution, each reading its class of
// x's pixels in place (the kernel's staging addresses pixel (2i + a, 2j + b)), each with its reduction.
bool wgrad_s2_applies(const ConvArgs &a) {
    return a.bf16 && a.R == 3 && a.S == 3 && a.stride == 2 && a.pad == 1 && a.Cin % 128 == 0 && a.Cout % 128 == 0 &&
           a.P == (a.H - 1) / 2 + 1 && a.Q == (a.W - 1) / 2 + 1;
}

size_t wgrad_s2_workspace_bytes(const ConvArgs &a) {
    if (!wgrad_s2_applies(a)) return 0;
    size_t most = 0;
    for (const S2Class &c : kS2Classes) {
        WgradPlan p;
        if (wgrad_plan(s2_class_layer(a, c, a.x), p, c.ntaps)) return 0;
        most = p.partial_bytes > most ? p.partial_bytes : most;
    }
    return (most + 255) / 256 * 256;
}

hipError_t launch_wgrad_s2(const ConvArgs &a, const void *g, float *gw, void *workspace, size_t workspace_bytes,
                           hipStream_t stream) {
    const size_t need = wgrad_s2_workspace_bytes(a);
    if (!need || workspace_bytes < need || !g || !gw || !workspace || !a.x || !a.scale || ((uintptr_t)workspace & 255))
        return hipErrorInvalidValue;
    for (const S2Class &c : kS2Classes) {
        const hipError_t e = run_wgrad(s2_class_layer(a, c, a.x), g, gw, workspace, need, c.ntaps, c.tapwin,
                                       9, c.tapout, stream, XView{a.H, a.W, 2, c.a, c.b});
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace delta
