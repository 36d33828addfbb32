// MFMA GEMM used by every dense contraction of the learner step (forward,
// input-gradient and weight-gradient passes of Algorithm 1's policy update).
//
// One kernel shape:   D(i, j) = sum_k P[i][k] * Q[j][k]
// Both operands are contiguous along the contraction index k, which is what the
// MFMA operand registers want (each lane feeds a run of consecutive k).  The
// learner keeps every tensor that is ever contracted along its slow index in a
// second, transposed copy, written by the epilogue of the kernel that produces
// it, so no pass transposes on the fly.
#pragma once
#include "tj_common.h"

typedef uint16_t tj_bf16;  // raw bfloat16 bits

__host__ __device__ inline tj_bf16 tj_f32_to_bf16(float f)
{
    union { float f; uint32_t u; } c;
    c.f = f;
    uint32_t u = c.u;
    if ((u & 0x7F800000u) == 0x7F800000u) return (tj_bf16)((u >> 16) | ((u & 0xFFFFu) ? 0x40u : 0u));
    u += 0x7FFFu + ((u >> 16) & 1u);  // round to nearest, ties to even
    return (tj_bf16)(u >> 16);
}

__host__ __device__ inline float tj_bf16_to_f32(tj_bf16 h)
{
    union { float f; uint32_t u; } c;
    c.u = (uint32_t)h << 16;
    return c.f;
}

template <typename T> struct TjElem;
template <> struct TjElem<float> {
    static constexpr int kVec = 4;  // elements per 16-byte vector
    __host__ __device__ static float from_f32(float x) { return x; }
    __host__ __device__ static float to_f32(float x) { return x; }
};
template <> struct TjElem<tj_bf16> {
    static constexpr int kVec = 8;
    __host__ __device__ static tj_bf16 from_f32(float x) { return tj_f32_to_bf16(x); }
    __host__ __device__ static float to_f32(tj_bf16 x) { return tj_bf16_to_f32(x); }
};

// Gather form of an operand: a convolution as a GEMM without a patch matrix.  Row m of the
// operand is patch m = (img, oh, ow) of a channels-last image batch [img][H][W][C]; its column
// k = (kh, kw, c) lies at  origin(m) + (k / run) * krow_stride + k % run,  run = kw_size * C: one
// kernel row (kw, c) is a contiguous run of the image.  Divisions by ohw and ow are multiplications
// by mg = ceil(2^32 / d) (exact while m * d < 2^32, which tj_gather_make checks).
struct TjGather {
    int on;
    int ohw, ow;
    uint32_t mg_ohw, mg_ow;
    int64_t img_stride;          // elements between images
    int oh_stride, ow_stride;    // elements between patch origins (stride * W * C, stride * C)
    int run, krow_stride;        // elements per kernel row, elements between image rows (W * C)
};

__host__ __device__ inline int64_t tj_gather_origin(const TjGather &g, uint32_t m)
{
#if defined(__HIP_DEVICE_COMPILE__)
    const uint32_t img = __umulhi(m, g.mg_ohw);
#else
    const uint32_t img = (uint32_t)(((uint64_t)m * g.mg_ohw) >> 32);
#endif
    const uint32_t r = m - img * (uint32_t)g.ohw;
#if defined(__HIP_DEVICE_COMPILE__)
    const uint32_t oh = __umulhi(r, g.mg_ow);
#else
    const uint32_t oh = (uint32_t)(((uint64_t)r * g.mg_ow) >> 32);
#endif
    const uint32_t ow = r - oh * (uint32_t)g.ow;
    return (int64_t)img * g.img_stride + (int64_t)oh * g.oh_stride + (int64_t)ow * g.ow_stride;
}

__host__ __device__ inline int tj_gather_koff(const TjGather &g, int k)
{
    const int kh = k / g.run;
    return kh * g.krow_stride + (k - kh * g.run);
}

// Fills g for an image batch [n][H][W][C], square kernel ksz, stride; false if the geometry does
// not fit the 16-byte operand vectors or the exact-division range for max_rows patches.
inline bool tj_gather_make(TjGather &g, int C, int H, int W, int ksz, int stride, int OH, int OW, size_t max_rows)
{
    g.on = 1;
    g.ohw = OH * OW; g.ow = OW;
    g.mg_ohw = (uint32_t)((((uint64_t)1 << 32) + g.ohw - 1) / g.ohw);
    g.mg_ow = (uint32_t)((((uint64_t)1 << 32) + g.ow - 1) / g.ow);
    g.img_stride = (int64_t)H * W * C;
    g.oh_stride = stride * W * C; g.ow_stride = stride * C;
    g.run = ksz * C; g.krow_stride = W * C;
    if (g.ohw < 2 || g.ow < 2) return false;   // ceil(2^32 / 1) does not fit 32 bits
    if (max_rows * (uint64_t)g.ohw >= ((uint64_t)1 << 32)) return false;
    // every 8-element vector of a patch row must be 16-byte aligned and inside one kernel row
    return g.run % 8 == 0 && g.ow_stride % 8 == 0 && g.krow_stride % 8 == 0 && (H * W * C) % 8 == 0;
}

// A run of output columns j that share one P operand (weights) and bias.
template <typename T> struct TjGemmSeg {
    int j_begin, j_end;  // columns [j_begin, j_end) of D
    const T *P;          // [I][ldp]
    const float *bias;   // per i, may be null
    int q_shift;         // Q row of column j is j - q_shift
};

template <typename T> struct TjGemmArgs {
    TjGemmSeg<T> seg[2];
    int n_seg;
    const T *Q;          // [rows][ldq]
    int ldp, ldq;        // row strides in elements (multiples of a 16-byte vector)
    int I, K;            // rows of P; contraction length (rows are zero padded to a vector multiple)
    const float *bias_j; // optional bias per column j (convolutions: j = output channel)
    int relu;            // max(x, 0) after bias
    const T *mask;       // optional: D(i,j) = 0 where mask[j*ldmask + i] <= 0 (ReLU derivative)
    int ldmask;
    T *Ci; int ldci;     // optional: D(i,j) -> Ci[j*ldci + i]   (i contiguous: vector stores)
    T *Cj; int ldcj;     // optional: D(i,j) -> Cj[i*ldcj + j] for j < cj_jmax
    int cj_jmax;
    float *Cf; int ldcf; // optional fp32: D(i,j) -> Cf[z*cf_zstride + j*ldcf + i]
    size_t cf_zstride;
    int k_chunk;         // contraction elements handled per blockIdx.z (multiple of the stage depth)
    int n_split;         // gridDim.z
    float *qsum;         // optional: qsum[z*qsum_zstride + j] = sum over this z's k of Q[j][k]
    size_t qsum_zstride;
    TjGather gather;     // gather.on: P rows are patches of seg[0].P (bf16, one segment of at most 128
                         // columns, whole 64-k stages, no split); ldp is ignored
    TjGather out_map;    // with gather.on and out_map.on: D(i,j) -> Cj[origin(out_map, i) + koff(out_map, j)]
                         // (ldcj ignored): row i is a coarse output position, column j a (pixel, channel) of
                         // the s x s pixel block it owns.  The only output of such a launch; no bias / ReLU.
    const T *mask_cj;    // optional with out_map: the result is zeroed where mask_cj[same offset] <= 0
    int trans;           // bf16 only.  1: both operands are stored contraction-major, P as [k][i] (row pitch ldp)
                         // and Q as [k][j] (row pitch ldq); rows k in [0, K) must exist (K a multiple of 32,
                         // like every split chunk), I and the columns multiples of 8, one segment, no q_shift.
                         // 2: only P is stored that way, Q as usual (no qsum)
};

template <typename T> int tj_gemm(const TjGemmArgs<T> &a, hipStream_t st);

// Two independent bf16 GEMMs as one launch where both fit the direct-to-LDS kernel (they share
// one ramp-up and tail); otherwise the same as two tj_gemm calls.
int tj_gemm_pair(const TjGemmArgs<tj_bf16> &a0, const TjGemmArgs<tj_bf16> &a1, hipStream_t st);
// Sum of the S gradient slices of the flat parameters [begin, end) (multiples of 4): g[i] += g[s*stride + i]
// for s = 1 .. S-1 in that order, the order in which the optimizer kernel adds slices.
struct TjSliceSum {
    float *g;
    int S;
    size_t stride, begin, end;
};
// tj_gemm_pair for two split weight gradients with transposed operands that fill only part of the chip
// (a network's first layer and its head), with that sum as further blocks of the same launch: the
// streaming work runs on the compute units the contractions leave idle.  The range must not overlap
// what the two problems write.  *fused says whether the sum was launched; if not, the call was
// tj_gemm_pair and the optimizer has to add those slices itself.
int tj_gemm_pair_sum(const TjGemmArgs<tj_bf16> &a0, const TjGemmArgs<tj_bf16> &a1, const TjSliceSum &r,
                     hipStream_t st, bool *fused);
// bf16 with gathered operands: the same for two convolutions of equal shape class
int tj_gemm_gather_pair(const TjGemmArgs<tj_bf16> &a0, const TjGemmArgs<tj_bf16> &a1, hipStream_t st);
// fp32: the same for two small problems (falls back to two launches otherwise)
int tj_gemm_pair_f32(const TjGemmArgs<float> &a0, const TjGemmArgs<float> &a1, hipStream_t st);

// Weight and bias gradient of a convolution layer from the channels-last output gradient and the
// channels-last layer input (bf16, 32 or 64 output channels), split over the patch rows:
//   part[z][o*K + k] = sum over slice z of dZ[m][o] * patch[m][k],  part[z][O*K + o] = sum dZ[m][o].
struct TjConvWgradArgs {
    const tj_bf16 *dZ; int O;   // [M rounded up to 64][O]; rows past M must be zero
    const tj_bf16 *act;         // layer input [img][H][W][C]
    TjGather g;                 // patch geometry of this layer
    int M, K;                   // patches, patch length
    float *part; size_t zstride;
    int n_split, m_chunk;       // patch rows per slice, a multiple of 64; n_split * m_chunk >= M
};
int tj_conv_wgrad(const TjConvWgradArgs &a, hipStream_t st);

// First convolution of a pixel network straight from u8 frame stacks [B][4][H][W] (32 output
// channels, square kernel k with k % 4 == 0, even stride): out = relu(conv(x / 255) + b) for the
// images s (online weights), s' (online) and s' (target), channels-last bf16 [3B*OH*OW][32];
// act0 (optional) receives the channels-last bf16 copy of the s images.  Weights are bf16
// [32][16 k^2] with the patch index ordered (kh, kw, c).
struct TjConvFirstArgs {
    const uint8_t *obs, *next_obs;
    int B, H, W, k, s, OH, OW;
    const tj_bf16 *W_on, *W_tg;
    const float *b_on, *b_tg;
    tj_bf16 *act0, *out;
    float scale;
    const uint32_t *rows;   // optional: image b of s / s' is row min(rows[b], n_rows - 1) of obs / next_obs
    uint32_t n_rows;
    const uint32_t *planes; // optional (not with rows): obs = next_obs = a table of n_rows planes of H*W bytes;
                            // channel c of s_b is plane min(planes[8b + c], n_rows - 1), of s'_b planes[8b + 4 + c]
};
bool tj_conv_first_fits(int C, int H, int W, int k, int s, int O);
int tj_conv_first(const TjConvFirstArgs &a, hipStream_t st);

// Weight and bias gradient of that first convolution, also straight from the u8 stacks of the s
// images (no channels-last copy of them is needed then) and the channels-last output gradient
// dZ [B*OH*OW][32].  Block z of n_part (1 <= n_part <= B) sums the images z, z + n_part, ...:
//   part[z*zstride + o*K + k] = sum dZ[m][o] * patch[m][k],   part[z*zstride + 32*K + o] = sum dZ[m][o],
// patch values bf16(x * scale) as in the forward pass, k ordered (kh, kw, c).  Needs the forward
// kernel's geometry and OH, OW multiples of 4.
struct TjConvFirstWgradArgs {
    const uint8_t *obs;
    const tj_bf16 *dZ;
    int B, H, W, k, s, OH, OW;
    float scale;
    float *part; size_t zstride;
    int n_part;
    const uint32_t *rows;   // optional, as in TjConvFirstArgs
    uint32_t n_rows;
    const uint32_t *planes; // optional, as in TjConvFirstArgs (the s planes)
};
bool tj_conv_first_wgrad_fits(int C, int H, int W, int k, int s, int O);
int tj_conv_first_wgrad(const TjConvFirstWgradArgs &a, hipStream_t st);
