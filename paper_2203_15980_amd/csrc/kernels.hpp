// Internal launchers of the HIP kernels (conv_igemm.hip).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>

namespace delta {

struct ConvArgs {
    const void *x;        // [N,H,W,Cin]
    const void *w;        // [Cout,R,S,Cin]
    const void *res;      // [N,P,Q,Cout] or nullptr
    const void *mask;     // [N,P,Q,Cout] or nullptr: y is stored as 0 where mask is not > 0 (after residual and ReLU)
    void *y;              // [N,P,Q,Cout]
    const float *scale;   // [Cout]
    const float *shift;   // [Cout]
    int N, H, W, Cin, Cout, R, S, stride, pad, P, Q, M;
    int relu;             // 0: none, 1: ReLU, 2: GELU (erf form; tiled kernel only)
    int bf16;             // 1: bf16 storage, fp32 accumulate; 0: fp32
    // Scattered form (launch_conv_scatter only; the data gradient of a strided layer, one parity
    // class of input pixels at a time).  oy_s > 0: output pixel (n, p, q) is stored at pixel
    // (n, p * oy_s + oy_a, q * oy_s + oy_b) of an [N, OH, OW, Cout] tensor; res and mask are read
    // there; P and Q are the caller's (a tap that leaves the input reads zeros); the R x S taps are
    // taps (w_r0 + r * w_step, w_s0 + s * w_step) of a weight tensor [Cout, wR, wS, Cin].
    int oy_s = 0, oy_a = 0, oy_b = 0, OH = 0, OW = 0;
    int wR = 0, wS = 0, w_r0 = 0, w_s0 = 0, w_step = 1;
};

// The test behind every ReLU mask of the backward pass.  bf16: greater than zero <=> sign bit clear,
// not zero and not NaN.  Returns the bits of `v` (two bf16 values) with the halves cleared whose
// half of `m` fails it.
__device__ __forceinline__ uint32_t keep_where_positive_bf16(uint32_t v, uint32_t m) {
    const uint32_t lo = m & 0xFFFFu, hi = m >> 16;
    const bool plo = lo != 0 && lo < 0x7F81u;          // positive, finite or +inf
    const bool phi = hi != 0 && hi < 0x7F81u;
    return (plo ? (v & 0xFFFFu) : 0u) | (phi ? (v & 0xFFFF0000u) : 0u);
}
__device__ __forceinline__ uint32_t keep_where_positive_f32(uint32_t v, uint32_t m) {
    return __uint_as_float(m) > 0.f ? v : 0u;
}

// nullptr when the kernel supports the shape, else the reason.
const char *conv_check(const ConvArgs &a);
const char *conv_kernel_name(const ConvArgs &a);
hipError_t launch_conv(const ConvArgs &a, hipStream_t stream);
const char *conv_scatter_check(const ConvArgs &a);
hipError_t launch_conv_scatter(const ConvArgs &a, hipStream_t stream);
// conv1x1.hip: streaming kernel for bf16 1x1 convolutions whose weights fit LDS
bool conv1x1_stream_applies(const ConvArgs &a);
hipError_t launch_conv1x1_stream(const ConvArgs &a, hipStream_t stream);
// gemm_nt.hip: bf16 1x1 stride-1 layers with a long reduction axis as a 256 x 256-tiled GEMM
bool gemm_nt_applies(const ConvArgs &a);
const char *gemm_nt_kernel_name(const ConvArgs &a);   // with the tile the launch will use
hipError_t launch_gemm_nt(const ConvArgs &a, hipStream_t stream);
// conv3x3_halo.hip: bf16 3x3 stride-1 kernel that keeps the input halo of a pixel tile in LDS
bool conv3x3_halo_applies(const ConvArgs &a);
hipError_t launch_conv3x3_halo(const ConvArgs &a, hipStream_t stream);
// conv3x3_c64.hip: bf16 3x3 stride-1 64 -> 64 channels, persistent workgroups with all nine taps resident in LDS
bool conv3x3_c64_applies(const ConvArgs &a);
hipError_t launch_conv3x3_c64(const ConvArgs &a, hipStream_t stream);
// bottleneck_block.hip: one identity bottleneck of conv2_x (1x1 256 -> 64, 3x3 64 -> 64, 1x1 64 -> 256 + x,
// ReLU after each, bf16) in a single launch; a1 / a2 / out may each be null (not stored)
struct BlockArgs {
    const void *x;                       // [M, 256] block input, also the shortcut ([M, 64] with a projection shortcut)
    void *a1, *a2, *out;                 // [M, 64], [M, 64], [M, 256]
    const void *w1, *w2, *w3;            // [64][256] ([64][64]), [64][3][3][64], [256][64]
    const float *s1, *h1, *s2, *h2, *s3, *h3;   // folded batch-norm scale / shift of the three layers
    int N, H, W, M;
    // projection shortcut (the first block of the stage): sc = ssc * (wsc . x) + hsc, added to the third layer
    int proj;
    const void *wsc;                     // [256][64]
    const float *ssc, *hsc;
    void *sc;                            // [M, 256] or nullptr: not stored
};
const char *bottleneck_block_check(const BlockArgs &a);
hipError_t launch_bottleneck_block(const BlockArgs &a, hipStream_t stream);
// attention.hip: fused multi-head self-attention, head dimension 64, bf16.  qkv [N,S,3*64*heads], ctx [N,S,64*heads]
const char *attention_check(const void *qkv, const void *ctx, int N, int S, int heads, int bf16);
hipError_t launch_attention(const void *qkv, void *ctx, int N, int S, int heads, int bf16, hipStream_t stream);
// transformer_ops.hip: layer normalisation over the last axis of [rows, C], bf16
const char *layernorm_check(const void *x, const void *y, const float *gamma, const float *beta, long long rows, int C,
                            int bf16);
hipError_t launch_layernorm(const void *x, void *y, const float *gamma, const float *beta, long long rows, int C,
                            float eps, int bf16, hipStream_t stream);
// opgranular_ops.hip: training-mode batch normalisation over [M, C] (bf16), ReLU, residual add
const char *bn_train_check(const void *x, const void *y, const float *gamma, const float *beta, long long M, int C,
                           int bf16);
size_t bn_train_scratch_bytes();
size_t bn_train_fwd_scratch_bytes();      // what the forward alone needs of it (any C up to 8192)
hipError_t launch_bn_train(const void *x, void *y, const float *gamma, const float *beta, long long M, int C, float eps,
                           int bf16, void *scratch, size_t scratch_bytes, hipStream_t stream);
hipError_t launch_bn_train_bwd(const void *x, const void *gy, void *gx, const float *gamma, float *gw, long long M, int C,
                               float eps, int bf16, void *scratch, hipStream_t stream);
hipError_t launch_relu(const void *x, void *y, size_t bytes, int bf16, hipStream_t stream);
hipError_t launch_add(const void *x, const void *r, void *y, size_t bytes, int bf16, hipStream_t stream);
// net_ops.hip: ResNet stem (7x7, stride 2, pad 3, 3 -> 64 channels, bf16), pooling, loss
bool stem_applies(const ConvArgs &a);
const char *stem_check(const ConvArgs &a);
hipError_t launch_stem(const ConvArgs &a, hipStream_t stream);
// stem_wgrad.hip: weight gradient of the stem
size_t stem_wgrad_workspace_bytes(const ConvArgs &a);
hipError_t launch_stem_wgrad(const ConvArgs &a, const void *g, float *gw, void *workspace, size_t workspace_bytes,
                             hipStream_t stream);

struct PoolArgs {
    const void *x;   // [N,H,W,C]
    void *y;         // [N,P,Q,C] (max) or [N,C] (global average)
    int N, H, W, C, R, S, stride, pad, P, Q;
    int bf16;
};
const char *pool_check(const PoolArgs &a, bool global_avg);
hipError_t launch_maxpool(const PoolArgs &a, hipStream_t stream);
hipError_t launch_avgpool(const PoolArgs &a, hipStream_t stream);
hipError_t launch_softmax_ce(const void *logits, const void *labels, int N, int classes, int bf16, float *out,
                             hipStream_t stream);

// backward.hip: backward of the fused layer (bf16 weight gradient; data gradient through the
// forward kernels with transformed weights)
hipError_t launch_relu_mask(const void *y, const void *gy, void *out, size_t bytes, int bf16, hipStream_t stream);
hipError_t launch_relu_mask_dilate(const void *y, const void *gy, void *out, int N, int H, int W, int P, int Q, int K,
                                   int stride, int bf16, hipStream_t stream);
hipError_t launch_subsample(const void *x, void *xs, int N, int H, int W, int P, int Q, int C, int stride, int bf16,
                            hipStream_t stream, int oa = 0, int ob = 0);
hipError_t launch_spread_add(const void *t, const void *add, const void *mask, void *out, int N, int H, int W, int P,
                             int Q, int C, int stride, int bf16, hipStream_t stream);
hipError_t launch_bwd_weights(const void *w, const float *scale, void *wt, int K, int R, int S, int C, int bf16,
                              hipStream_t stream);
const char *wgrad_check(const ConvArgs &a);            // nullptr when the weight-gradient kernel applies
size_t wgrad_workspace_bytes(const ConvArgs &a);
// 3x3 stride-2 pad-1 layers by parity class, from the gradient at the output's resolution (a.x = x at the
// input's resolution, a.H, a.W, a.P, a.Q the layer's own)
bool wgrad_s2_applies(const ConvArgs &a);
size_t wgrad_s2_workspace_bytes(const ConvArgs &a);
hipError_t launch_wgrad_s2(const ConvArgs &a, const void *g, float *gw, void *workspace, size_t workspace_bytes,
                           hipStream_t stream);
hipError_t launch_wgrad(const ConvArgs &a, const void *g, float *gw, void *workspace, size_t workspace_bytes,
                        hipStream_t stream);

// backward_ops.hip: backward of pooling, the classifier and the loss (bf16)
// mask_x: gx is also multiplied by [x > 0] (the ReLU mask of the layer that produced the pool's input)
hipError_t launch_maxpool_bwd(const PoolArgs &a, const void *gy, void *gx, int mask_x, hipStream_t stream);
hipError_t launch_avgpool_bwd(const PoolArgs &a, const void *gy, void *gx, hipStream_t stream);
hipError_t launch_softmax_ce_bwd(const void *logits, const void *labels, int N, int classes, void *gz, hipStream_t stream);
hipError_t launch_dense_bwd(const void *x, const void *w, const float *scale, const void *gy, void *gx, float *gw,
                            int N, int Cin, int Cout, hipStream_t stream);

hipError_t launch_bn_fold(const float *gamma, const float *beta, const float *mean, const float *var,
                          float eps, unsigned C, float *scale, float *shift, hipStream_t stream);
hipError_t launch_copy(const void *src, void *dst, size_t bytes, hipStream_t stream);
hipError_t launch_mfma_probe(float *out, int iters, int blocks, hipStream_t stream);

}  // namespace delta
