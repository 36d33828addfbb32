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
                                               int H, int W, float scale, const uint32_t *__restrict__ rows,
                                               uint32_t n_rows, const uint32_t *__restrict__ planes)
{
    const size_t total = (size_t)n * H * W;
    const size_t p = (size_t)blockIdx.x * 256 + threadIdx.x;   // (img, y, x)
    if (p >= total) return;
    const size_t img = p / ((size_t)H * W), yx = p % ((size_t)H * W);
    T *dp = dst + p * C;
    if (planes) {   // every channel is a plane of its own in the source table: planes[img * 2C + c]
        for (int c = 0; c < C; ++c) {
            const size_t pl = (size_t)min(planes[img * 2 * C + c], n_rows - 1u);
            dp[c] = TjElem<T>::from_f32((float)src[pl * H * W + yx] * scale);
        }
        return;
    }
    const size_t simg = rows ? (size_t)min(rows[img], n_rows - 1u) : img;   // source image, picked by index
    const S *sp = src + simg * C * H * W + yx;
    for (int c = 0; c < C; ++c) dp[c] = TjElem<T>::from_f32((float)sp[(size_t)c * H * W] * scale);
}

// u8 planes with C = 4 -> channels-last bf16, eight pixels per thread: one 8-byte load per plane,
// four 16-byte stores.  H*W must be a multiple of 8.
__global__ __launch_bounds__(256) void to_nhwc_u8c4(const uint8_t *__restrict__ src, tj_bf16 *__restrict__ dst,
                                                    size_t n_img, int HW, float scale,
                                                    const uint32_t *__restrict__ rows, uint32_t n_rows,
                                                    const uint32_t *__restrict__ planes)
{
    const size_t groups = n_img * (size_t)(HW / 8);
    const size_t t = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (t >= groups) return;
    const size_t img = t / (HW / 8), p0 = (t % (HW / 8)) * 8;
    uint64_t pl[4];
    if (planes) {   // planes[img * 8 + c] = the source table's plane that holds channel c
#pragma unroll
        for (int c = 0; c < 4; ++c)
            pl[c] = *(const uint64_t *)(src + (size_t)min(planes[img * 8 + c], n_rows - 1u) * HW + p0);
    } else {
        const size_t simg = rows ? (size_t)min(rows[img], n_rows - 1u) : img;
        const uint8_t *sp = src + simg * 4 * (size_t)HW + p0;
#pragma unroll
        for (int c = 0; c < 4; ++c) pl[c] = *(const uint64_t *)(sp + (size_t)c * HW);
    }
    uint4 *dp = (uint4 *)(dst + (img * HW + p0) * 4);
#pragma unroll
    for (int q = 0; q < 4; ++q) {   // pixels 2q, 2q+1
        uint32_t w[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {   // (pixel 2q + e/2, channels 2(e%2), 2(e%2)+1)
            const int px = 2 * q + (e >> 1), c = 2 * (e & 1);
            const float lo = (float)((pl[c] >> (8 * px)) & 0xFF) * scale;
            const float hi = (float)((pl[c + 1] >> (8 * px)) & 0xFF) * scale;
            w[e] = (uint32_t)tj_f32_to_bf16(lo) | ((uint32_t)tj_f32_to_bf16(hi) << 16);
        }
        dp[q] = make_uint4(w[0], w[1], w[2], w[3]);
    }
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

// The same for 2-byte elements with 16-byte accesses on both sides: a 64 x 64 tile per block, eight
// elements per load and per store.  lds, ldd and Cc are multiples of 8, both bases 16-byte aligned,
// ldd >= R rounded up to 8; rows past R read as zero (so the pad columns of dst are written as zeros).
__global__ __launch_bounds__(256) void transpose2d_v8(const uint16_t *__restrict__ src, int lds,
                                                      uint16_t *__restrict__ dst, int ldd, int R, int Cc)
{
    __shared__ uint16_t tile[64][66];
    const int r0 = blockIdx.y * 64, c0 = blockIdx.x * 64;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int v = threadIdx.x + 256 * i;          // 512 vectors of the tile: row v / 8, columns 8 (v % 8) ..
        const int r = v >> 3, cv = (v & 7) * 8;
        uint4 d = make_uint4(0u, 0u, 0u, 0u);
        if (r0 + r < R && c0 + cv < Cc) d = *(const uint4 *)(src + (size_t)(r0 + r) * lds + c0 + cv);
        const uint32_t w[4] = {d.x, d.y, d.z, d.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            tile[r][cv + 2 * e] = (uint16_t)(w[e] & 0xFFFFu);
            tile[r][cv + 2 * e + 1] = (uint16_t)(w[e] >> 16);
        }
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int v = threadIdx.x + 256 * i;          // output row (source column) v / 8, source rows 8 (v % 8) ..
        const int c = v >> 3, rv = (v & 7) * 8;
        if (c0 + c >= Cc || r0 + rv >= (R + 7) / 8 * 8) continue;
        uint32_t w[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) w[e] = (uint32_t)tile[rv + 2 * e][c] | ((uint32_t)tile[rv + 2 * e + 1][c] << 16);
        *(uint4 *)(dst + (size_t)(c0 + c) * ldd + r0 + rv) = make_uint4(w[0], w[1], w[2], w[3]);
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

// The same for bf16 with C a multiple of 8: one thread owns 8 channels of a pixel (16-byte loads
// of the patch gradients and of the mask, one 16-byte store); same summation order.
__global__ __launch_bounds__(256) void col2im_mask_v8(const tj_bf16 *__restrict__ dpatch, int ldk,
                                                      const tj_bf16 *__restrict__ act, tj_bf16 *__restrict__ dz,
                                                      ConvGeom g, size_t n_img)
{
    const int C8 = g.C / 8;
    const size_t total = n_img * g.H * g.W * C8;
    const size_t t = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (t >= total) return;
    const int c0 = (int)(t % C8) * 8;
    const size_t p = t / C8;
    const int x = (int)(p % g.W), y = (int)((p / g.W) % g.H);
    const size_t img = p / ((size_t)g.W * g.H);
    float sum[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) sum[e] = 0.f;
    for (int kh = y % g.s; kh < g.k; kh += g.s) {
        const int oh = (y - kh) / g.s;
        if (y < kh || oh >= g.OH) continue;
        for (int kw = x % g.s; kw < g.k; kw += g.s) {
            const int ow = (x - kw) / g.s;
            if (x < kw || ow >= g.OW) continue;
            const size_t m = (img * g.OH + oh) * g.OW + ow;
            const uint4 v = *(const uint4 *)(dpatch + m * ldk + (kh * g.k + kw) * g.C + c0);
            const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                sum[2 * e] += tj_bf16_to_f32((tj_bf16)(w[e] & 0xFFFF));
                sum[2 * e + 1] += tj_bf16_to_f32((tj_bf16)(w[e] >> 16));
            }
        }
    }
    const uint4 mv = *(const uint4 *)(act + p * g.C + c0);
    const uint32_t mw[4] = {mv.x, mv.y, mv.z, mv.w};
    uint32_t o[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const float lo = tj_bf16_to_f32((tj_bf16)(mw[e] & 0xFFFF)) > 0.f ? sum[2 * e] : 0.f;
        const float hi = tj_bf16_to_f32((tj_bf16)(mw[e] >> 16)) > 0.f ? sum[2 * e + 1] : 0.f;
        o[e] = (uint32_t)tj_f32_to_bf16(lo) | ((uint32_t)tj_f32_to_bf16(hi) << 16);
    }
    *(uint4 *)(dz + p * g.C + c0) = make_uint4(o[0], o[1], o[2], o[3]);
}

// Copy of a channels-last tensor [n][OH][OW][O] into the interior of a zero-bordered one
// [n][OH + 2 pad][OW + 2 pad][O] (the border is never written).  16 bytes per thread; O % 8 == 0.
__global__ __launch_bounds__(256) void pad_halo(const tj_bf16 *__restrict__ src, tj_bf16 *__restrict__ dst, size_t n,
                                                int OH, int OW, int O, int pad)
{
    const int O8 = O / 8;
    const size_t total = n * OH * OW * O8;
    const size_t t = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (t >= total) return;
    const int c = (int)(t % O8);
    const size_t p = t / O8;
    const int x = (int)(p % OW), y = (int)((p / OW) % OH);
    const size_t img = p / ((size_t)OW * OH);
    const size_t d = ((img * (OH + 2 * pad) + y + pad) * (OW + 2 * pad) + x + pad) * O + c * 8;
    *(uint4 *)(dst + d) = *(const uint4 *)(src + p * O + c * 8);
}

// Weights of the input-gradient GEMM of a convolution (kernel k, stride s, A = ceil(k / s) taps per
// dimension): row j = (py, px, c) over the s x s pixel block and the input channels, column
// (a, b, o) over the taps and the output channels:
//   Wd[j][(a*A + b)*O + o] = W[o][kh][kw][c],  kh = py + (A-1-a) s,  kw = px + (A-1-b) s   (0 if kh or kw >= k)
// with W the fp32 master weights in the kernels' order [o][(kh*k + kw)*C + c].
// All layers in one launch: blocks [block_begin[q], block_begin[q + 1]) build the matrix of job q.
struct DgradWeightJobs {
    int n_job;
    const float *w[TJ_MAX_LAYERS];
    tj_bf16 *wd[TJ_MAX_LAYERS];
    int O[TJ_MAX_LAYERS], C[TJ_MAX_LAYERS], k[TJ_MAX_LAYERS], s[TJ_MAX_LAYERS], A[TJ_MAX_LAYERS];
    unsigned block_begin[TJ_MAX_LAYERS + 1];
};

__global__ __launch_bounds__(256) void dgrad_weights(const DgradWeightJobs jobs)
{
    int q = 0;
    while (q + 1 < jobs.n_job && blockIdx.x >= jobs.block_begin[q + 1]) ++q;
    const float *__restrict__ w = jobs.w[q];
    tj_bf16 *__restrict__ wd = jobs.wd[q];
    const int O = jobs.O[q], C = jobs.C[q], k = jobs.k[q], s = jobs.s[q], A = jobs.A[q];
    const int Kd = A * A * O, N = s * s * C;
    const size_t t = (size_t)(blockIdx.x - jobs.block_begin[q]) * 256 + threadIdx.x;
    if (t >= (size_t)N * Kd) return;
    const int col = (int)(t % Kd), j = (int)(t / Kd);
    const int o = col % O, b = (col / O) % A, a = col / (O * A);
    const int c = j % C, px = (j / C) % s, py = j / (C * s);
    const int kh = py + (A - 1 - a) * s, kw = px + (A - 1 - b) * s;
    float v = 0.f;
    if (kh < k && kw < k) v = w[(size_t)o * (k * k * C) + (kh * k + kw) * C + c];
    wd[t] = tj_f32_to_bf16(v);
}

// Sums the partial gradient slices of every layer into the flat gradient, all layers in one launch.
// Job q: n_part slices of n elements each (slice z at part + z * zstride) -> dst[0, n); blocks
// [block_begin[q], block_begin[q + 1]) work on it, in one of the two forms below; both add in a fixed
// order: deterministic for a given n_part.  Slices start 16-byte aligned and are padded to a multiple
// of 4 elements (zstride % 4 == 0).
struct ReduceJobs {
    int n_job;
    const float *part[TJ_MAX_LAYERS];
    size_t zstride[TJ_MAX_LAYERS];
    int n_part[TJ_MAX_LAYERS];
    float *dst[TJ_MAX_LAYERS];
    size_t n[TJ_MAX_LAYERS];
    unsigned block_begin[TJ_MAX_LAYERS + 1];
};

// Elements one block reduces: 4 * kRedCols, or 1024 where a job has at most kReduceFew slices.
constexpr int kReduceFew = 8;
constexpr int kRedCols = 16, kRedGroups = 256 / kRedCols;
inline unsigned reduce_blocks(size_t n, int n_part)
{
    const size_t per = n_part <= kReduceFew ? 1024 : 4 * kRedCols;
    return (unsigned)((n + per - 1) / per);
}

__global__ __launch_bounds__(256) void reduce_parts(const ReduceJobs jobs)
{
    __shared__ float4 sh[kRedGroups][kRedCols];
    int q = 0;
    while (q + 1 < jobs.n_job && blockIdx.x >= jobs.block_begin[q + 1]) ++q;
    const float *__restrict__ part = jobs.part[q];
    const size_t zstride = jobs.zstride[q], n = jobs.n[q];
    const int n_part = jobs.n_part[q];
    float *__restrict__ dst = jobs.dst[q];
    if (n_part <= kReduceFew) {
        // few slices of a long vector (a linear layer's batch split): one float4 per thread, every slice's
        // load in flight, added in slice order
        const size_t e = ((size_t)(blockIdx.x - jobs.block_begin[q]) * 256 + threadIdx.x) * 4;
        if (e >= n) return;
        float4 p[kReduceFew];
#pragma unroll
        for (int u = 0; u < kReduceFew; ++u)
            p[u] = u < n_part ? *(const float4 *)(part + (size_t)u * zstride + e) : make_float4(0.f, 0.f, 0.f, 0.f);
        float4 sum = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
        for (int u = 0; u < kReduceFew; ++u)
            if (u < n_part) { sum.x += p[u].x; sum.y += p[u].y; sum.z += p[u].z; sum.w += p[u].w; }
        const float out[4] = {sum.x, sum.y, sum.z, sum.w};
#pragma unroll
        for (int k = 0; k < 4; ++k)
            if (e + k < n) dst[e + k] = out[k];
        return;
    }
    // many slices of a short vector (a convolution's row split): a block owns kRedCols float4 columns (256
    // bytes per slice); its kRedGroups thread rows each add every kRedGroups-th slice, eight loads in
    // flight, then the row sums are added in row order
    const int col = threadIdx.x % kRedCols, grp = threadIdx.x / kRedCols;
    const size_t e = ((size_t)(blockIdx.x - jobs.block_begin[q]) * kRedCols + col) * 4;
    float4 sum = make_float4(0.f, 0.f, 0.f, 0.f);
    if (e < n) {
        const float *src = part + e;
        int z = grp;
        for (; z + 7 * kRedGroups < n_part; z += 8 * kRedGroups) {
            float4 p[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) p[u] = *(const float4 *)(src + (size_t)(z + kRedGroups * u) * zstride);
#pragma unroll
            for (int u = 0; u < 8; ++u) { sum.x += p[u].x; sum.y += p[u].y; sum.z += p[u].z; sum.w += p[u].w; }
        }
        for (; z + kRedGroups < n_part; z += 2 * kRedGroups) {
            const float4 p0 = *(const float4 *)(src + (size_t)z * zstride);
            const float4 p1 = *(const float4 *)(src + (size_t)(z + kRedGroups) * zstride);
            sum.x += p0.x; sum.y += p0.y; sum.z += p0.z; sum.w += p0.w;
            sum.x += p1.x; sum.y += p1.y; sum.z += p1.z; sum.w += p1.w;
        }
        for (; z < n_part; z += kRedGroups) {
            const float4 p = *(const float4 *)(src + (size_t)z * zstride);
            sum.x += p.x; sum.y += p.y; sum.z += p.z; sum.w += p.w;
        }
    }
    sh[grp][col] = sum;
    __syncthreads();
    if (grp != 0 || e >= n) return;
#pragma unroll
    for (int g = 1; g < kRedGroups; ++g) {
        const float4 p = sh[g][col];
        sum.x += p.x; sum.y += p.y; sum.z += p.z; sum.w += p.w;
    }
    const float out[4] = {sum.x, sum.y, sum.z, sum.w};
#pragma unroll
    for (int k = 0; k < 4; ++k)
        if (e + k < n) dst[e + k] = out[k];
}

}  // namespace tjconv
