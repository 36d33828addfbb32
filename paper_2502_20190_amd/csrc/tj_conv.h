// Data-movement kernels of the convolutional Q-network path: activations are
// kept channels-last (NHWC), a convolution is a GEMM on a patch matrix whose
// k index runs (kh, kw, c), so that one kernel row of a patch, kw*C + c, is a
// contiguous run of the input.  All kernels here are memory bound.
#pragma once
#include "tj_gemm.h"

namespace tjconv {

struct ConvGeom {
    int C, H, W;        // input channels / height / width
    int OC, OH, OW;     // output
    int k, s;           // square kernel, stride
    int K;              // C * k * k
};

// Observation planes (NCHW, u8 scaled by 1/255 or fp32) -> channels-last T [n][H][W][C].
template <typename T, typename S>
__global__ __launch_bounds__(256) void to_nhwc(const S *__restrict__ src, T *__restrict__ dst, int n, int C,
                                               int H, int W, float scale)
{
    const size_t total = (size_t)n * H * W;
    const size_t p = (size_t)blockIdx.x * 256 + threadIdx.x;   // (img, y, x)
    if (p >= total) return;
    const size_t img = p / ((size_t)H * W), yx = p % ((size_t)H * W);
    const S *sp = src + img * C * H * W + yx;
    T *dp = dst + p * C;
    for (int c = 0; c < C; ++c) dp[c] = TjElem<T>::from_f32((float)sp[(size_t)c * H * W] * scale);
}

// Patch matrix: row m = (img, oh, ow), column (kh*k + kw)*C + c.  One thread copies a
// run of `vec` elements (vec = 8 when the runs are 16-byte aligned, else 1).
template <typename T, int VEC>
__global__ __launch_bounds__(256) void im2col(const T *__restrict__ act, T *__restrict__ patches, ConvGeom g,
                                              size_t n_rows, int ldk)
{
    const int run = g.k * g.C;                 // contiguous elements per kernel row
    const int vpr = run / VEC;                 // vectors per kernel row
    const size_t total = n_rows * g.k * vpr;
    const size_t t = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (t >= total) return;
    const int v = (int)(t % vpr);
    const int kh = (int)((t / vpr) % g.k);
    const size_t m = t / ((size_t)vpr * g.k);
    const int ow = (int)(m % g.OW), oh = (int)((m / g.OW) % g.OH);
    const size_t img = m / ((size_t)g.OW * g.OH);
    const T *sp = act + ((img * g.H + (size_t)(oh * g.s + kh)) * g.W + (size_t)ow * g.s) * g.C + v * VEC;
    T *dp = patches + m * ldk + kh * run + v * VEC;
    if (VEC == 8) {
        *(uint4 *)dp = *(const uint4 *)sp;
    } else {
        dp[0] = sp[0];
    }
}

// Transposed patch matrix of the first n_img images: row k = (kh, kw, c), column m.
template <typename T>
__global__ __launch_bounds__(256) void im2col_t(const T *__restrict__ act, T *__restrict__ pt, ConvGeom g,
                                                size_t n_cols, int ldm)
{
    const size_t m = (size_t)blockIdx.x * 256 + threadIdx.x;
    const int kk = blockIdx.y;                 // (kh*k + kw)*C + c
    if (m >= n_cols) return;
    const int c = kk % g.C, kw = (kk / g.C) % g.k, kh = kk / (g.C * g.k);
    const int ow = (int)(m % g.OW), oh = (int)((m / g.OW) % g.OH);
    const size_t img = m / ((size_t)g.OW * g.OH);
    pt[(size_t)kk * ldm + m] = act[((img * g.H + (size_t)(oh * g.s + kh)) * g.W + (size_t)(ow * g.s + kw)) * g.C + c];
}

// dst[c][r] = src[r][c] for r < R, c < Cc, through a 32 x 32 LDS tile.
template <typename T>
__global__ __launch_bounds__(256) void transpose2d(const T *__restrict__ src, int lds, T *__restrict__ dst,
                                                   int ldd, int R, int Cc)
{
    __shared__ T tile[32][33];
    const int r0 = blockIdx.y * 32, c0 = blockIdx.x * 32;
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int r = r0 + ty + 8 * i, c = c0 + tx;
        tile[ty + 8 * i][tx] = (r < R && c < Cc) ? src[(size_t)r * lds + c] : (T)0;
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int c = c0 + ty + 8 * i, r = r0 + tx;
        if (r < R && c < Cc) dst[(size_t)c * ldd + r] = tile[tx][ty + 8 * i];
    }
}

// Input gradient of a convolution from the patch-gradient matrix (gather form, no atomics):
// dA[img,y,x,c] = sum over the patches (oh, ow) and kernel offsets (kh, kw) with
// oh*s + kh = y, ow*s + kw = x of dpatch[(img,oh,ow)][(kh,kw,c)], then the ReLU derivative of
// the layer below: zero where act <= 0.  Output rows are (img, y, x), C channels each.
template <typename T>
__global__ __launch_bounds__(256) void col2im_mask(const T *__restrict__ dpatch, int ldk,
                                                   const T *__restrict__ act, T *__restrict__ dz, ConvGeom g,
                                                   size_t n_img)
{
    const size_t total = n_img * g.H * g.W * g.C;
    const size_t t = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (t >= total) return;
    const int c = (int)(t % g.C);
    const size_t p = t / g.C;
    const int x = (int)(p % g.W), y = (int)((p / g.W) % g.H);
    const size_t img = p / ((size_t)g.W * g.H);
    float sum = 0.f;
    if (TjElem<T>::to_f32(act[t]) > 0.f) {
        for (int kh = y % g.s; kh < g.k; kh += g.s) {
            const int oh = (y - kh) / g.s;
            if (y < kh || oh >= g.OH) continue;
            for (int kw = x % g.s; kw < g.k; kw += g.s) {
                const int ow = (x - kw) / g.s;
                if (x < kw || ow >= g.OW) continue;
                const size_t m = (img * g.OH + oh) * g.OW + ow;
                sum += TjElem<T>::to_f32(dpatch[m * ldk + (kh * g.k + kw) * g.C + c]);
            }
        }
    }
    dz[t] = TjElem<T>::from_f32(sum);
}

// fp32 master weights [O][C][S] (S = kh*kw of a convolution, or the H*W positions a linear layer
// sees after a convolution; S = 1 for a plain linear layer) -> compute-type copy [O][ldk] with
// k = s*C + c, and optionally its transpose [K][ldo].
template <typename T>
__global__ __launch_bounds__(256) void permute_cast(const float *__restrict__ w, T *__restrict__ wc, int ldk,
                                                    T *__restrict__ wct, int ldo, int O, int C, int S)
{
    const size_t total = (size_t)O * C * S;
    const size_t t = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (t >= total) return;
    const int s = (int)(t % S), c = (int)((t / S) % C), o = (int)(t / ((size_t)S * C));
    const T val = TjElem<T>::from_f32(w[t]);
    const int kk = s * C + c;
    wc[(size_t)o * ldk + kk] = val;
    if (wct) wct[(size_t)kk * ldo + o] = val;
}

// Sums n_part partial weight-gradient slices (kernel order [O][s*C + c], pitch K) and bias
// partials into the flat gradient in parameter order ([O][C][S], then bias [O]).
__global__ __launch_bounds__(256) void reduce_permute(const float *__restrict__ part, size_t zstride, int n_part,
                                                      float *__restrict__ gw, float *__restrict__ gb, int O,
                                                      int C, int S)
{
    const int K = C * S;
    const size_t total = (size_t)O * K + O;
    const size_t t = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (t >= total) return;
    float sum = 0.f;
    if (t < (size_t)O * K) {
        const int s = (int)(t % S), c = (int)((t / S) % C), o = (int)(t / ((size_t)S * C));
        const size_t src = (size_t)o * K + s * C + c;
        for (int z = 0; z < n_part; ++z) sum += part[(size_t)z * zstride + src];
        gw[t] = sum;
    } else {
        const size_t o = t - (size_t)O * K;
        for (int z = 0; z < n_part; ++z) sum += part[(size_t)z * zstride + (size_t)O * K + o];
        gb[o] = sum;
    }
}

}  // namespace tjconv
