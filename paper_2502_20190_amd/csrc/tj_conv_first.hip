// First convolution of a pixel Q-network, straight from the replayed u8 frame stacks
// (forward passes of the batched policy update; the x/255 scaling happens here, at the
// network input).  One kernel replaces plane -> channels-last conversion plus GEMM:
//
//   obs, next_obs  u8 [B][4][H][W]   (the minibatch as sampled)
//   out            bf16 [3B * OH*OW][32], channels-last: images s (online net), s' (online),
//                  s' (target net);  relu(conv + bias)
//   act0           bf16 [B][H][W][4]: channels-last copy of the s images, kept for the
//                  weight-gradient pass
//
// The layer is memory bound (32 output channels, patch length 16 k^2), so the design is about
// touching each input byte once: a persistent block per CU loops over images; an image's four
// planes are fetched with 4-byte loads into registers ahead of use, converted to bf16 and
// laid out channels-last in LDS (56 KB for 84 x 84; two such buffers where they fit), and every
// patch operand is then a single 16-byte LDS read (two pixels x four channels are contiguous).  Both networks' weights stay in
// LDS for the block's lifetime; an s' image is multiplied with both while it is resident.
// MFMA: v_mfma_f32_32x32x16_bf16 with a = weights (rows = channels), b = patches (columns), so
// a lane ends up with runs of four consecutive channels of one patch: 8-byte stores.
#include "tj_gemm.h"

namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

constexpr int kThreads = 1024;    // 16 waves: the 13 patch tiles of an 84 x 84 frame in one round
constexpr int kMaxRounds = 4;     // 4-pixel tasks per thread per image: H*W <= 4 * 1024 * 4

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));

// round to nearest even in hardware (v_cvt_pk_bf16_f32); the inputs here are finite
__device__ __forceinline__ uint32_t pack2(float a, float b)
{
    const f32x2_t f = {a, b};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2_t));
}

// DB: two image buffers in LDS.  The next image is converted into the idle buffer at the top of
// an iteration, so one barrier per image suffices and the waves that are done converting start on
// the MFMAs while others still write: conversion (LDS writes, the channels-last copy) and patch
// work (LDS reads, MFMA, output stores) overlap across the block's waves.
template <int KSZ, bool DB>
__global__ __launch_bounds__(kThreads) void conv_first_u8c4(const TjConvFirstArgs a)
{
    extern __shared__ __align__(16) uint8_t smem[];
    const int HW = a.H * a.W;
    const int K = 4 * a.k * a.k;
    const int wpitch = (K + 8) * 2;                  // bytes per weight row in LDS
    const size_t img_bytes = (size_t)HW * 8;          // [H*W][4] bf16
    uint8_t *img0 = smem;
    uint8_t *wl = smem + (DB ? 2 : 1) * img_bytes;    // [2][32][K+8] bf16
    float *bias = (float *)(wl + 2 * 32 * wpitch);    // [2][32]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, h = lane >> 5;

    // weights and biases of both networks, once per block
    for (int v = tid; v < 2 * 32 * (K / 8); v += kThreads) {
        const int net = v / (32 * (K / 8)), r = (v / (K / 8)) % 32, c = v % (K / 8);
        const tj_bf16 *src = (net ? a.W_tg : a.W_on) + (size_t)r * K + c * 8;
        *(u32x4 *)(wl + (net * 32 + r) * wpitch + c * 16) = *(const u32x4 *)src;
    }
    if (tid < 64) bias[tid] = (tid < 32 ? a.b_on : a.b_tg)[tid & 31];

    const int n_task = HW / 4;                        // 4 consecutive pixels, all four planes
    const int n_round = (n_task + kThreads - 1) / kThreads;
    uint32_t px[kMaxRounds][4];
    auto fetch = [&](int g) {                         // image g: s images first, then s'
        const uint8_t *src = (g < a.B ? a.obs + (size_t)g * 4 * HW : a.next_obs + (size_t)(g - a.B) * 4 * HW);
#pragma unroll
        for (int r = 0; r < kMaxRounds; ++r) {
            const int t = tid + r * kThreads;
            if (r < n_round && t < n_task) {
#pragma unroll
                for (int c = 0; c < 4; ++c) px[r][c] = *(const uint32_t *)(src + (size_t)c * HW + 4 * t);
            }
        }
    };
    // registers -> bf16 channels-last in LDS (and in act0 for an s image)
    auto convert = [&](int g, uint8_t *img) {
        tj_bf16 *keep = g < a.B && a.act0 ? a.act0 + (size_t)g * HW * 4 : nullptr;
#pragma unroll
        for (int r = 0; r < kMaxRounds; ++r) {
            const int t = tid + r * kThreads;
            if (r < n_round && t < n_task) {
                u32x4 v[2];
#pragma unroll
                for (int p = 0; p < 4; ++p) {     // pixel 4t + p: channels 0..3
                    float f[4];
#pragma unroll
                    for (int c = 0; c < 4; ++c) f[c] = (float)((px[r][c] >> (8 * p)) & 0xFF) * a.scale;
                    v[p >> 1][2 * (p & 1)] = pack2(f[0], f[1]);
                    v[p >> 1][2 * (p & 1) + 1] = pack2(f[2], f[3]);
                }
                *(u32x4 *)(img + (size_t)t * 32) = v[0];
                *(u32x4 *)(img + (size_t)t * 32 + 16) = v[1];
                if (keep) {
                    *(u32x4 *)(keep + (size_t)t * 16) = v[0];
                    *(u32x4 *)(keep + (size_t)t * 16 + 8) = v[1];
                }
            }
        }
    };

    const int OHW = a.OH * a.OW;
    const int n_tile = (OHW + 31) / 32;
    const int n_img = 2 * a.B;
    // patches x weights of image g in `img`.  Tile = 32 patches; lane l32 owns patch 32*tile + l32.
    auto patches = [&](int g, const uint8_t *img) {
        const int n_net = g < a.B ? 1 : 2;
        for (int tile = wave; tile < n_tile; tile += kThreads / 64) {
            const int m = min(32 * tile + l32, OHW - 1);
            const int oh = m / a.OW, ow = m - oh * a.OW;
            const uint8_t *origin = img + ((size_t)(oh * a.s) * a.W + ow * a.s) * 8;
            f32x16 acc[2];
#pragma unroll
            for (int n = 0; n < 2; ++n)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[n][r] = 0.f;
#pragma unroll 2
            for (int kh = 0; kh < KSZ; ++kh) {
#pragma unroll
                for (int kw0 = 0; kw0 < KSZ; kw0 += 4) {   // 16 contraction values: 4 pixels x 4 channels
                    const u32x4 pv = *(const u32x4 *)(origin + ((size_t)kh * a.W + kw0 + 2 * h) * 8);
                    const int kb = (kh * KSZ + kw0) * 4 + 8 * h;
                    const u32x4 w0 = *(const u32x4 *)(wl + l32 * wpitch + kb * 2);
                    acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, w0),
                                                                     __builtin_bit_cast(bf16x8, pv), acc[0], 0, 0, 0);
                    if (n_net == 2) {
                        const u32x4 w1 = *(const u32x4 *)(wl + (32 + l32) * wpitch + kb * 2);
                        acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, w1),
                                                                         __builtin_bit_cast(bf16x8, pv), acc[1], 0, 0,
                                                                         0);
                    }
                }
            }
            // acc[n][4q + e] = channel 8q + 4h + e of patch 32*tile + l32
            if (32 * tile + l32 < OHW) {
#pragma unroll
                for (int n = 0; n < 2; ++n) {
                    if (n >= n_net) continue;
                    // output image: s -> g, s' online -> g (= B + index), s' target -> g + B
                    tj_bf16 *dst = a.out + ((size_t)(g + n * a.B) * OHW + 32 * tile + l32) * 32;
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const int c0 = 8 * q + 4 * h;
                        float f[4];
#pragma unroll
                        for (int e = 0; e < 4; ++e) f[e] = fmaxf(acc[n][4 * q + e] + bias[n * 32 + c0 + e], 0.f);
                        *(uint2 *)(dst + c0) = make_uint2(pack2(f[0], f[1]), pack2(f[2], f[3]));
                    }
                }
            }
        }
    };

    const int stride = (int)gridDim.x;
    int g = blockIdx.x;
    if (g >= n_img) return;
    fetch(g);
    if constexpr (DB) {
        convert(g, img0);
        if (g + stride < n_img) fetch(g + stride);
        int cur = 0;
        for (; g < n_img; g += stride) {
            // image g is complete in buffer cur (and, first trip, the weights are in); every wave has
            // left the patches of the image before it, which lived in the other buffer
            __syncthreads();
            if (g + stride < n_img) {
                convert(g + stride, img0 + (cur ^ 1) * img_bytes);
                if (g + 2 * stride < n_img) fetch(g + 2 * stride);   // in flight during the MFMAs below
            }
            patches(g, img0 + cur * img_bytes);
            cur ^= 1;
        }
    } else {
        for (; g < n_img; g += stride) {
            __syncthreads();   // the last image's patch reads are done (first trip: the weights are in)
            convert(g, img0);
            __syncthreads();
            if (g + stride < n_img) fetch(g + stride);   // in flight during the MFMAs below
            patches(g, img0);
        }
    }
}

}  // namespace

// LDS bytes with one (buffers = 1) or two image buffers
size_t tj_conv_first_lds_bytes(int H, int W, int k, int buffers)
{
    const int K = 4 * k * k;
    return (size_t)buffers * H * W * 8 + 2 * 32 * (size_t)(K + 8) * 2 + 64 * 4;
}

constexpr size_t kLdsLimit = 150 * 1024;

bool tj_conv_first_fits(int C, int H, int W, int k, int s, int O)
{
    // 16-byte patch reads start on even pixels: even stride and width
    if (C != 4 || O != 32 || (k != 4 && k != 8) || s < 2 || s % 2 || W % 2 || H < k || W < k) return false;
    if ((H * W) % 4 || H * W > 4 * kThreads * kMaxRounds) return false;
    return tj_conv_first_lds_bytes(H, W, k, 1) <= kLdsLimit;
}

int tj_conv_first(const TjConvFirstArgs &a, hipStream_t st)
{
    if (!a.obs || !a.next_obs || !a.W_on || !a.W_tg || !a.b_on || !a.b_tg || !a.out) return TJ_ERR_INVALID_ARG;
    if (a.B < 1 || !tj_conv_first_fits(4, a.H, a.W, a.k, a.s, 32)) return TJ_ERR_SHAPE;
    if (a.OH != (a.H - a.k) / a.s + 1 || a.OW != (a.W - a.k) / a.s + 1) return TJ_ERR_SHAPE;
    if ((((uintptr_t)a.obs | (uintptr_t)a.next_obs) & 3) != 0) return TJ_ERR_INVALID_ARG;
    const bool two = tj_conv_first_lds_bytes(a.H, a.W, a.k, 2) <= kLdsLimit;
    const size_t lds = tj_conv_first_lds_bytes(a.H, a.W, a.k, two ? 2 : 1);
    static bool attr_set = false;
    if (!attr_set) {
        const void *fn[4] = {(const void *)conv_first_u8c4<8, true>, (const void *)conv_first_u8c4<8, false>,
                             (const void *)conv_first_u8c4<4, true>, (const void *)conv_first_u8c4<4, false>};
        for (int i = 0; i < 4; ++i)
            TJ_HIP_TRY(hipFuncSetAttribute(fn[i], hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsLimit));
        attr_set = true;
    }
    int dev = 0, n_cu = 256;
    if (hipGetDevice(&dev) == hipSuccess) {
        int v = 0;
        if (hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0) n_cu = v;
    }
    const int grid = 2 * a.B < n_cu ? 2 * a.B : n_cu;
    if (a.k == 8) {
        if (two) conv_first_u8c4<8, true><<<grid, kThreads, lds, st>>>(a);
        else conv_first_u8c4<8, false><<<grid, kThreads, lds, st>>>(a);
    } else {
        if (two) conv_first_u8c4<4, true><<<grid, kThreads, lds, st>>>(a);
        else conv_first_u8c4<4, false><<<grid, kThreads, lds, st>>>(a);
    }
    return hipGetLastError() == hipSuccess ? TJ_OK : TJ_ERR_DEVICE;
}
