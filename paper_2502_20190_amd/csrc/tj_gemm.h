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

};

template <typename T> int tj_gemm(const TjGemmArgs<T> &a, hipStream_t st);
