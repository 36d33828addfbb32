// LDS-staged MFMA GEMM for gfx950:  D(i, j) = sum_k P[i][k] * Q[j][k].
//
// Block = 256 threads = 4 waves in a 2 x 2 arrangement, block tile 128 x 128,
// wave tile 64 x 64 = 2 x 2 MFMA tiles of 32 x 32.  A stage holds 128 bytes of
// k per row (64 bf16 or 32 fp32); rows sit 144 bytes apart in LDS so that the
// 16-byte operand reads of consecutive rows fall on distinct banks.  The next
// stage's global loads are issued before the MFMAs of the current one.
//
// bf16: v_mfma_f32_32x32x16_bf16, lane l feeds row (l % 32) with k = 8*(l / 32)
// + 0..7.  fp32: v_mfma_f32_32x32x2_f32 four times per 16-byte operand; lane
// group g = l / 32 feeds k = 4g + e in the e-th instruction for both operands,
// a permutation of k that the sum does not see.
// Accumulator element r of lane l is D(i, j) with i = 8*(r/4) + 4*(l/32) + r%4
// and j = l % 32, so a lane owns runs of four consecutive i: outputs that are
// contiguous in i get vector stores.
#include "tj_gemm.h"

namespace {

constexpr int BI = 128, BJ = 128;
constexpr int kRowBytes = 128;   // bytes of k per row per stage
constexpr int kLdsRow = 144;     // padded row pitch in LDS
constexpr int kScratchPitch = 144;   // epilogue scratch row pitch: >= 32 fp32, 16-byte aligned

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));   // a 16-byte operand vector in registers
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

template <typename T> __device__ __forceinline__ void mma(f32x16 &acc, const u32x4 &p, const u32x4 &q);

template <> __device__ __forceinline__ void mma<tj_bf16>(f32x16 &acc, const u32x4 &p, const u32x4 &q)
{
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, p),
                                                  __builtin_bit_cast(bf16x8, q), acc, 0, 0, 0);
}

template <> __device__ __forceinline__ void mma<float>(f32x16 &acc, const u32x4 &p, const u32x4 &q)
{
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(p.x), __uint_as_float(q.x), acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(p.y), __uint_as_float(q.y), acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(p.z), __uint_as_float(q.z), acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(p.w), __uint_as_float(q.w), acc, 0, 0, 0);
}

template <typename T> __device__ __forceinline__ float vec_sum(const u32x4 &v);
template <> __device__ __forceinline__ float vec_sum<float>(const u32x4 &v)
{
    return __uint_as_float(v.x) + __uint_as_float(v.y) + __uint_as_float(v.z) + __uint_as_float(v.w);
}
template <> __device__ __forceinline__ float vec_sum<tj_bf16>(const u32x4 &v)
{
    float s = 0.f;
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) s += __uint_as_float(w[e] << 16) + __uint_as_float(w[e] & 0xFFFF0000u);
    return s;
}

// Epilogue of one 32 x 32 accumulator tile in the MFMA layout (i = ibase + 8*(r/4) + 4*(lane/32) + r%4,
// j = jbase + lane%32): bias, ReLU, mask, then the stores into whichever outputs are set.
template <typename T>
__device__ __forceinline__ void pq_epilogue(const TjGemmArgs<T> &a, const TjGemmSeg<T> &seg, const f32x16 &acc,
                                            const int ibase, const int jbase, const int j_end, const int z,
                                            const int lane)
{
    const int l32 = lane & 31, lg = lane >> 5;
    const int j = jbase + l32;
    if (j >= j_end) return;
#pragma unroll
    for (int rq = 0; rq < 4; ++rq) {
        const int ib = ibase + rq * 8 + lg * 4;
        if (ib >= a.I) continue;
        const int nvalid = min(4, a.I - ib);
        float v[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = acc[rq * 4 + e];
        if (seg.bias) {
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (e < nvalid) v[e] += seg.bias[ib + e];
        }
        if (a.bias_j) {
            const float bj = a.bias_j[j];
#pragma unroll
            for (int e = 0; e < 4; ++e) v[e] += bj;
        }
        if (a.relu) {
#pragma unroll
            for (int e = 0; e < 4; ++e) v[e] = fmaxf(v[e], 0.f);
        }
        if (a.mask) {
            const T *mp = a.mask + (size_t)j * a.ldmask + ib;
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (e < nvalid && !(TjElem<T>::to_f32(mp[e]) > 0.f)) v[e] = 0.f;
        }
        if (a.Ci) {
            T *cp = a.Ci + (size_t)j * a.ldci + ib;
            if (nvalid == 4) {
                if constexpr (sizeof(T) == 2) {
                    uint2 o;
                    o.x = (uint32_t)tj_f32_to_bf16(v[0]) | ((uint32_t)tj_f32_to_bf16(v[1]) << 16);
                    o.y = (uint32_t)tj_f32_to_bf16(v[2]) | ((uint32_t)tj_f32_to_bf16(v[3]) << 16);
                    *(uint2 *)cp = o;
                } else {
                    *(float4 *)cp = make_float4(v[0], v[1], v[2], v[3]);
                }
            } else {
                for (int e = 0; e < nvalid; ++e) cp[e] = TjElem<T>::from_f32(v[e]);
            }
        }
        if (a.Cj && j < a.cj_jmax) {
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (e < nvalid) a.Cj[(size_t)(ib + e) * a.ldcj + j] = TjElem<T>::from_f32(v[e]);
        }
        if (a.Cf) {
            float *fp = a.Cf + (size_t)z * a.cf_zstride + (size_t)j * a.ldcf + ib;
            if (nvalid == 4 && ((uintptr_t)fp & 15) == 0) {
                *(float4 *)fp = make_float4(v[0], v[1], v[2], v[3]);
            } else {
                for (int e = 0; e < nvalid; ++e) fp[e] = v[e];
            }
        }
    }
}

// NF = 32-wide fragments per wave and dimension: block tile 64*NF square (four waves, 2 x 2).  NF = 1 gives
// small problems four times as many blocks to spread over the CUs.
template <typename T, int NF>
__global__ __launch_bounds__(256) void gemm_pq(const TjGemmArgs<T> a, const int tiles_seg0)
{
    constexpr int BI = 64 * NF, BJ = 64 * NF;
    constexpr int VE = TjElem<T>::kVec;
    constexpr int KE = kRowBytes / (int)sizeof(T);
    __shared__ __align__(16) uint8_t sP[BI * kLdsRow];
    __shared__ __align__(16) uint8_t sQ[BJ * kLdsRow];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wi = wave & 1, wj = wave >> 1;
    const int l32 = lane & 31, lg = lane >> 5;

    const int sidx = (a.n_seg > 1 && (int)blockIdx.y >= tiles_seg0) ? 1 : 0;
    const TjGemmSeg<T> seg = a.seg[sidx];
    const int j0 = seg.j_begin + ((int)blockIdx.y - (sidx ? tiles_seg0 : 0)) * BJ;
    const int j_end = seg.j_end;
    const int i0 = blockIdx.x * BI;
    const int z = blockIdx.z;
    const int k_begin = z * a.k_chunk;
    const int k_end = min(a.K, k_begin + a.k_chunk);

    // global -> register staging: 2*NF vectors of P and of Q per thread
    const int cv = tid & 7;
    const T *gP[2 * NF];
    const T *gQ[2 * NF];
    bool okP[2 * NF], okQ[2 * NF];
#pragma unroll
    for (int r = 0; r < 2 * NF; ++r) {
        const int row = (tid >> 3) + 32 * r;
        const int i = i0 + row, j = j0 + row;
        okP[r] = i < a.I;
        okQ[r] = j < j_end;
        gP[r] = seg.P + (size_t)(okP[r] ? i : 0) * a.ldp + cv * VE;
        gQ[r] = a.Q + (size_t)(okQ[r] ? j - seg.q_shift : 0) * a.ldq + cv * VE;
    }
    u32x4 rP[2 * NF], rQ[2 * NF];
    const u32x4 zero4 = {0u, 0u, 0u, 0u};
    auto gload = [&](int k0) {
        const bool kin = k0 + cv * VE < k_end;
#pragma unroll
        for (int r = 0; r < 2 * NF; ++r) {
            rP[r] = (okP[r] && kin) ? *(const u32x4 *)(gP[r] + k0) : zero4;
            rQ[r] = (okQ[r] && kin) ? *(const u32x4 *)(gQ[r] + k0) : zero4;
        }
    };
    auto lstore = [&]() {
#pragma unroll
        for (int r = 0; r < 2 * NF; ++r) {
            const int row = (tid >> 3) + 32 * r;
            *(u32x4 *)(sP + row * kLdsRow + cv * 16) = rP[r];
            *(u32x4 *)(sQ + row * kLdsRow + cv * 16) = rQ[r];
        }
    };

    f32x16 acc[NF][NF];
#pragma unroll
    for (int fi = 0; fi < NF; ++fi)
#pragma unroll
        for (int fj = 0; fj < NF; ++fj)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[fi][fj][r] = 0.f;

    const bool do_qsum = a.qsum != nullptr && blockIdx.x == 0 && wi == 0;
    float qs[NF];
#pragma unroll
    for (int f = 0; f < NF; ++f) qs[f] = 0.f;

    gload(k_begin);
    lstore();
    __syncthreads();
    for (int k0 = k_begin; k0 < k_end; k0 += KE) {
        const bool more = k0 + KE < k_end;
        if (more) gload(k0 + KE);
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            u32x4 pf[NF], qf[NF];
#pragma unroll
            for (int f = 0; f < NF; ++f) {
                pf[f] = *(const u32x4 *)(sP + (wi * 32 * NF + f * 32 + l32) * kLdsRow + ks * 32 + lg * 16);
                qf[f] = *(const u32x4 *)(sQ + (wj * 32 * NF + f * 32 + l32) * kLdsRow + ks * 32 + lg * 16);
            }
#pragma unroll
            for (int fi = 0; fi < NF; ++fi)
#pragma unroll
                for (int fj = 0; fj < NF; ++fj) mma<T>(acc[fi][fj], pf[fi], qf[fj]);
            if (do_qsum) {
#pragma unroll
                for (int f = 0; f < NF; ++f) qs[f] += vec_sum<T>(qf[f]);
            }
        }
        __syncthreads();
        if (more) {
            lstore();
            __syncthreads();
        }
    }

    if (do_qsum) {
#pragma unroll
        for (int fj = 0; fj < NF; ++fj) {
            float s = qs[fj] + __shfl_xor(qs[fj], 32, 64);
            const int j = j0 + wj * 32 * NF + fj * 32 + l32;
            if (lg == 0 && j < j_end) a.qsum[(size_t)z * a.qsum_zstride + j] = s;
        }
    }

#pragma unroll
    for (int fi = 0; fi < NF; ++fi)
#pragma unroll
        for (int fj = 0; fj < NF; ++fj)
            pq_epilogue<T>(a, seg, acc[fi][fj], i0 + wi * 32 * NF + fi * 32, j0 + wj * 32 * NF + fj * 32, j_end, z, lane);
}

// Small fp32 problems: a 32 x 32 output tile per block, and the block's four waves split the
// contraction among them (operand fragments straight from global memory in the MFMA layout, eight
// 16-byte loads in flight per lane), so a launch has 16 times the waves of the 64 x 64 tiling and
// each wave a quarter of the dependent MFMA chain.  Waves 1..3 leave their accumulators in LDS,
// wave 0 adds them in wave order (deterministic) and runs the epilogue.
__device__ __forceinline__ void ksplit4_body(const TjGemmArgs<float> &a, const int tiles_seg0, const int bx,
                                             const int by, const int bz)
{
    typedef float T;
    __shared__ float red[3][17][64];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, lg = lane >> 5;
    const int sidx = (a.n_seg > 1 && by >= tiles_seg0) ? 1 : 0;
    const TjGemmSeg<T> seg = a.seg[sidx];
    const int j0 = seg.j_begin + (by - (sidx ? tiles_seg0 : 0)) * 32;
    const int j_end = seg.j_end;
    const int i0 = bx * 32;
    const int z = bz;
    const int k_begin = z * a.k_chunk;
    const int k_end = min(a.K, k_begin + a.k_chunk);

    // k steps of 8 (lane half lg takes k .. k+3 of each step); this wave's share of them
    const int n_step = k_end > k_begin ? (k_end - k_begin + 7) / 8 : 0;
    const int per = (n_step + 3) / 4;
    const int s_begin = min(n_step, wave * per), s_end = min(n_step, s_begin + per);
    const int i = i0 + l32, j = j0 + l32;
    const bool okP = i < a.I, okQ = j < j_end;
    const T *pP = seg.P + (size_t)(okP ? i : 0) * a.ldp + k_begin + lg * 4;
    const T *pQ = a.Q + (size_t)(okQ ? j - seg.q_shift : 0) * a.ldq + k_begin + lg * 4;
    const u32x4 zero4 = {0u, 0u, 0u, 0u};

    f32x16 acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.f;
    const bool do_qsum = a.qsum != nullptr && bx == 0;
    float qs = 0.f;
    for (int s0 = s_begin; s0 < s_end; s0 += 4) {
        u32x4 p[4], q[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int st = s0 + u;
            const bool kin = st < s_end && k_begin + st * 8 + lg * 4 < k_end;   // K and the chunks are multiples of 4
            p[u] = (kin && okP) ? *(const u32x4 *)(pP + st * 8) : zero4;
            q[u] = (kin && okQ) ? *(const u32x4 *)(pQ + st * 8) : zero4;
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            if (s0 + u >= s_end) break;
            mma<T>(acc, p[u], q[u]);
            if (do_qsum) qs += vec_sum<T>(q[u]);
        }
    }
    if (wave > 0) {
#pragma unroll
        for (int r = 0; r < 16; ++r) red[wave - 1][r][lane] = acc[r];
        red[wave - 1][16][lane] = qs;
    }
    __syncthreads();
    if (wave != 0) return;
#pragma unroll
    for (int w = 0; w < 3; ++w) {
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[r] += red[w][r][lane];
        qs += red[w][16][lane];
    }
    if (do_qsum) {
        const float sum = qs + __shfl_xor(qs, 32, 64);
        if (lg == 0 && j < j_end) a.qsum[(size_t)z * a.qsum_zstride + j] = sum;
    }
    pq_epilogue<T>(a, seg, acc, i0, j0, j_end, z, lane);
}

__global__ __launch_bounds__(256) void gemm_f32_ksplit4(const TjGemmArgs<float> a, const int tiles_seg0)
{
    ksplit4_body(a, tiles_seg0, (int)blockIdx.x, (int)blockIdx.y, (int)blockIdx.z);
}

// Two independent small problems in one launch (a layer's weight gradient and input gradient):
// blocks [0, nblk0) work on the first, the rest on the second.
struct PairF32 {
    TjGemmArgs<float> a[2];
    int tiles_seg0[2];
    int gx[2], gy[2];     // tile counts in i and j (the split slices follow)
    int nblk0;
};

__global__ __launch_bounds__(256) void gemm_f32_ksplit4_pair(const PairF32 p)
{
    const int which = (int)blockIdx.x >= p.nblk0 ? 1 : 0;
    const int id = (int)blockIdx.x - which * p.nblk0;
    const int bx = id % p.gx[which], by = (id / p.gx[which]) % p.gy[which], bz = id / (p.gx[which] * p.gy[which]);
    ksplit4_body(p.a[which], p.tiles_seg0[which], bx, by, bz);
}


// Orders this wave's LDS accesses (lane a's write before lane b's read of it) without a block
// barrier: a wave's LDS instructions execute in order, so only the compiler has to be told.
__device__ __forceinline__ void wave_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Bias, ReLU and mask of one 32 x 32 accumulator tile, in place.  v[r] follows the MFMA layout:
// i = ibase + 8*(r/4) + 4*(lane/32) + r%4, j = jbase + lane%32.  Kept apart from the stores: on this
// hardware loads and stores share one counter (vmcnt), so a load issued after a tile's stores would
// wait for those stores to finish.  The kernels run this on every tile first, then store.
__device__ __forceinline__ f32x16 tile_math_edge(const TjGemmArgs<tj_bf16> &a, const TjGemmSeg<tj_bf16> &seg,
                                              f32x16 v, int ibase, int jbase, const int j_end,
                                              const int lane)
{
    typedef tj_bf16 T;
    // Opaque to the optimiser: the per-element addresses and guards below are then formed inside the branch
    // that leads here and do not occupy registers on the interior tiles' path.
    asm volatile("" : "+v"(ibase), "+v"(jbase));
    const int l32 = lane & 31, lg = lane >> 5;
    const int jl = jbase + l32;
    if (seg.bias) {
#pragma unroll
        for (int rq = 0; rq < 4; ++rq)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int i = ibase + rq * 8 + lg * 4 + e;
                if (i < a.I) v[rq * 4 + e] += seg.bias[i];
            }
    }
    if (a.bias_j && jl < j_end) {
        const float bj = a.bias_j[jl];
#pragma unroll
        for (int r = 0; r < 16; ++r) v[r] += bj;
    }
    if (a.relu) {
#pragma unroll
        for (int r = 0; r < 16; ++r) v[r] = fmaxf(v[r], 0.f);
    }
    if (a.mask && jl < j_end) {
#pragma unroll
        for (int rq = 0; rq < 4; ++rq) {
            const int ib = ibase + rq * 8 + lg * 4;
            const T *mp = a.mask + (size_t)jl * a.ldmask + ib;
            if (ib + 3 < a.I) {
                const uint2 mv = *(const uint2 *)mp;   // four bf16
                const uint32_t w[2] = {mv.x, mv.y};
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const uint32_t h = (w[e >> 1] >> ((e & 1) * 16)) & 0xFFFFu;
                    if (!(tj_bf16_to_f32((T)h) > 0.f)) v[rq * 4 + e] = 0.f;
                }
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (ib + e < a.I && !(tj_bf16_to_f32(mp[e]) > 0.f)) v[rq * 4 + e] = 0.f;
            }
        }
    }
    return v;
}

// The stores of one 32 x 32 tile (values already final), staged through a wave-private LDS
// scratch of 32 rows x kScratchPitch bytes so that every lane writes 16 contiguous bytes.  The
// scratch must not be shared with another wave.
enum { kOutCi = 1, kOutCj = 2, kOutCf = 4, kOutAll = 7 };

__device__ __forceinline__ void store_tile_edge(const TjGemmArgs<tj_bf16> &a, const f32x16 v, uint8_t *scr,
                                           int ibase, int jbase, const int j_end, const int z,
                                           const int lane, const int which)
{
    typedef tj_bf16 T;
    asm volatile("" : "+v"(ibase), "+v"(jbase));   // as in tile_math_edge
    const int l32 = lane & 31, lg = lane >> 5;
    if (a.Ci && (which & kOutCi)) {   // rows j, 32 consecutive i (64 bytes) each
        wave_sync();
#pragma unroll
        for (int rq = 0; rq < 4; ++rq) {
            uint2 o;
            o.x = (uint32_t)tj_f32_to_bf16(v[rq * 4]) | ((uint32_t)tj_f32_to_bf16(v[rq * 4 + 1]) << 16);
            o.y = (uint32_t)tj_f32_to_bf16(v[rq * 4 + 2]) | ((uint32_t)tj_f32_to_bf16(v[rq * 4 + 3]) << 16);
            *(uint2 *)(scr + l32 * kScratchPitch + (rq * 8 + lg * 4) * 2) = o;
        }
        wave_sync();
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const int vv = lane + 64 * t, jr = vv >> 2, c = vv & 3;
            const u32x4 d = *(const u32x4 *)(scr + jr * kScratchPitch + c * 16);
            const int j = jbase + jr, i = ibase + c * 8;
            if (j < j_end && i < a.I) {
                T *cp = a.Ci + (size_t)j * a.ldci + i;
                if (i + 8 <= a.I) {
                    *(u32x4 *)cp = d;
                } else {
                    const uint32_t w[4] = {d.x, d.y, d.z, d.w};
#pragma unroll
                    for (int e = 0; e < 8; ++e)
                        if (e < a.I - i) cp[e] = (T)((w[e >> 1] >> ((e & 1) * 16)) & 0xFFFFu);
                }
            }
        }
    }
    if (a.Cj && (which & kOutCj)) {   // rows i, 32 consecutive j (64 bytes) each
        wave_sync();
#pragma unroll
        for (int rq = 0; rq < 4; ++rq)
#pragma unroll
            for (int e = 0; e < 4; ++e)
                *(T *)(scr + (rq * 8 + lg * 4 + e) * kScratchPitch + l32 * 2) = tj_f32_to_bf16(v[rq * 4 + e]);
        wave_sync();
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const int vv = lane + 64 * t, ir = vv >> 2, c = vv & 3;
            const u32x4 d = *(const u32x4 *)(scr + ir * kScratchPitch + c * 16);
            const int i = ibase + ir, j = jbase + c * 8;
            const int jmax = min(j_end, a.cj_jmax);
            if (i < a.I && j < jmax) {
                T *cp = a.Cj + (size_t)i * a.ldcj + j;
                if (j + 8 <= jmax && (((uintptr_t)cp) & 15) == 0) {
                    *(u32x4 *)cp = d;
                } else {
                    const uint32_t w[4] = {d.x, d.y, d.z, d.w};
#pragma unroll
                    for (int e = 0; e < 8; ++e)
                        if (e < jmax - j) cp[e] = (T)((w[e >> 1] >> ((e & 1) * 16)) & 0xFFFFu);
                }
            }
        }
    }
    if (a.Cf && (which & kOutCf)) {   // fp32 rows j, 32 consecutive i (128 bytes) each
        wave_sync();
#pragma unroll
        for (int rq = 0; rq < 4; ++rq)
            *(float4 *)(scr + l32 * kScratchPitch + (rq * 8 + lg * 4) * 4) =
                make_float4(v[rq * 4], v[rq * 4 + 1], v[rq * 4 + 2], v[rq * 4 + 3]);
        wave_sync();
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const int vv = lane + 64 * t, jr = vv >> 3, c = vv & 7;
            const float4 d = *(const float4 *)(scr + jr * kScratchPitch + c * 16);
            const int j = jbase + jr, i = ibase + c * 4;
            if (j < j_end && i < a.I) {
                float *fp = a.Cf + (size_t)z * a.cf_zstride + (size_t)j * a.ldcf + i;
                if (i + 4 <= a.I && (((uintptr_t)fp) & 15) == 0) {
                    *(float4 *)fp = d;
                } else {
                    const float w[4] = {d.x, d.y, d.z, d.w};
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (e < a.I - i) fp[e] = w[e];
                }
            }
        }
    }
}

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));

// Two floats -> packed bf16, round to nearest even (v_cvt_pk_bf16_f32).
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi)
{
    const f32x2_t v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}

// Interior tiles (all 32 x 32 outputs in range, 16-byte aligned bias): the same math and stores
// without per-element guards (the guarded versions above serve the edge tiles).
__device__ __forceinline__ void tile_math(const TjGemmArgs<tj_bf16> &a, const TjGemmSeg<tj_bf16> &seg,
                                          f32x16 &v, const int ibase, const int jbase, const int j_end,
                                          const int lane)
{
    const bool interior = ibase + 32 <= a.I && jbase + 32 <= j_end && (((uintptr_t)seg.bias) & 15) == 0;
    if (!interior) {
        v = tile_math_edge(a, seg, v, ibase, jbase, j_end, lane);
        return;
    }
    const int l32 = lane & 31, lg = lane >> 5;
    if (seg.bias) {
#pragma unroll
        for (int rq = 0; rq < 4; ++rq) {
            const float4 b = *(const float4 *)(seg.bias + ibase + rq * 8 + lg * 4);
            v[rq * 4 + 0] += b.x; v[rq * 4 + 1] += b.y; v[rq * 4 + 2] += b.z; v[rq * 4 + 3] += b.w;
        }
    }
    if (a.bias_j) {
        const float bj = a.bias_j[jbase + l32];
#pragma unroll
        for (int r = 0; r < 16; ++r) v[r] += bj;
    }
    if (a.relu) {
#pragma unroll
        for (int r = 0; r < 16; ++r) v[r] = fmaxf(v[r], 0.f);
    }
    if (a.mask) {
        const tj_bf16 *mp = a.mask + (size_t)(jbase + l32) * a.ldmask + ibase + lg * 4;
#pragma unroll
        for (int rq = 0; rq < 4; ++rq) {
            const uint2 mv = *(const uint2 *)(mp + rq * 8);   // four bf16: positive <=> as int16 > 0
            if (!((int16_t)(mv.x & 0xFFFFu) > 0)) v[rq * 4 + 0] = 0.f;
            if (!((int16_t)(mv.x >> 16) > 0)) v[rq * 4 + 1] = 0.f;
            if (!((int16_t)(mv.y & 0xFFFFu) > 0)) v[rq * 4 + 2] = 0.f;
            if (!((int16_t)(mv.y >> 16) > 0)) v[rq * 4 + 3] = 0.f;
        }
    }
}

__device__ __forceinline__ void store_tile(const TjGemmArgs<tj_bf16> &a, const f32x16 &v, uint8_t *scr,
                                           const int ibase, const int jbase, const int j_end, const int z,
                                           const int lane, const int which = kOutAll)
{
    typedef tj_bf16 T;
    bool interior = ibase + 32 <= a.I && jbase + 32 <= j_end;
    if (a.Cj) interior = interior && jbase + 32 <= a.cj_jmax && ((a.ldcj | jbase) & 7) == 0;
    if (a.Cf) interior = interior && ((((uintptr_t)(a.Cf + (size_t)z * a.cf_zstride)) | (uintptr_t)(a.ldcf * 4)) & 15) == 0;
    if (!interior) {
        if (jbase < j_end && ibase < a.I) store_tile_edge(a, v, scr, ibase, jbase, j_end, z, lane, which);
        return;
    }
    const int l32 = lane & 31, lg = lane >> 5;
    if (a.Ci && (which & kOutCi)) {   // rows j, 32 consecutive i (64 bytes) each
        wave_sync();
#pragma unroll
        for (int rq = 0; rq < 4; ++rq) {
            uint2 o;
            o.x = pack_bf16(v[rq * 4], v[rq * 4 + 1]);
            o.y = pack_bf16(v[rq * 4 + 2], v[rq * 4 + 3]);
            *(uint2 *)(scr + l32 * kScratchPitch + (rq * 8 + lg * 4) * 2) = o;
        }
        wave_sync();
        T *cp = a.Ci + (size_t)(jbase + (lane >> 2)) * a.ldci + ibase + (lane & 3) * 8;
        const uint8_t *sp = scr + (lane >> 2) * kScratchPitch + (lane & 3) * 16;
        *(u32x4 *)cp = *(const u32x4 *)sp;
        *(u32x4 *)(cp + (size_t)16 * a.ldci) = *(const u32x4 *)(sp + 16 * kScratchPitch);
    }
    if (a.Cj && (which & kOutCj)) {   // rows i, 32 consecutive j (64 bytes) each
        wave_sync();
#pragma unroll
        for (int rq = 0; rq < 4; ++rq) {
            const uint32_t p01 = pack_bf16(v[rq * 4], v[rq * 4 + 1]), p23 = pack_bf16(v[rq * 4 + 2], v[rq * 4 + 3]);
            uint8_t *wp = scr + (rq * 8 + lg * 4) * kScratchPitch + l32 * 2;
            *(T *)(wp) = (T)(p01 & 0xFFFFu);
            *(T *)(wp + kScratchPitch) = (T)(p01 >> 16);
            *(T *)(wp + 2 * kScratchPitch) = (T)(p23 & 0xFFFFu);
            *(T *)(wp + 3 * kScratchPitch) = (T)(p23 >> 16);
        }
        wave_sync();
        T *cp = a.Cj + (size_t)(ibase + (lane >> 2)) * a.ldcj + jbase + (lane & 3) * 8;
        const uint8_t *sp = scr + (lane >> 2) * kScratchPitch + (lane & 3) * 16;
        *(u32x4 *)cp = *(const u32x4 *)sp;
        *(u32x4 *)(cp + (size_t)16 * a.ldcj) = *(const u32x4 *)(sp + 16 * kScratchPitch);
    }
    if (a.Cf && (which & kOutCf)) {   // fp32 rows j, 32 consecutive i (128 bytes) each
        wave_sync();
#pragma unroll
        for (int rq = 0; rq < 4; ++rq)
            *(float4 *)(scr + l32 * kScratchPitch + (rq * 8 + lg * 4) * 4) =
                make_float4(v[rq * 4], v[rq * 4 + 1], v[rq * 4 + 2], v[rq * 4 + 3]);
        wave_sync();
        float *fp = a.Cf + (size_t)z * a.cf_zstride + (size_t)(jbase + (lane >> 3)) * a.ldcf + ibase + (lane & 7) * 4;
        const uint8_t *sp = scr + (lane >> 3) * kScratchPitch + (lane & 7) * 16;
#pragma unroll
        for (int t = 0; t < 4; ++t)
            *(u32x4 *)(fp + (size_t)(8 * t) * a.ldcf) = *(const u32x4 *)(sp + 8 * t * kScratchPitch);
    }
}

// Two 32 x 32 tiles that are neighbours along the contiguous index of a bf16 output are stored
// together, so that every store instruction writes whole 128-byte lines (8 lanes per row).
// Ci: tiles v0 | v1 neighbours in i (rows j, 64 consecutive i); the caller has checked that
// both are interior.
__device__ __forceinline__ void store_pair_ci(const TjGemmArgs<tj_bf16> &a, const f32x16 &v0, const f32x16 &v1,
                                              uint8_t *scr, const int ibase, const int jbase, const int lane)
{
    const int l32 = lane & 31, lg = lane >> 5;
    wave_sync();
#pragma unroll
    for (int rq = 0; rq < 4; ++rq) {
        uint2 o0, o1;
        o0.x = pack_bf16(v0[rq * 4], v0[rq * 4 + 1]); o0.y = pack_bf16(v0[rq * 4 + 2], v0[rq * 4 + 3]);
        o1.x = pack_bf16(v1[rq * 4], v1[rq * 4 + 1]); o1.y = pack_bf16(v1[rq * 4 + 2], v1[rq * 4 + 3]);
        *(uint2 *)(scr + l32 * kScratchPitch + (rq * 8 + lg * 4) * 2) = o0;
        *(uint2 *)(scr + l32 * kScratchPitch + 64 + (rq * 8 + lg * 4) * 2) = o1;
    }
    wave_sync();
    tj_bf16 *cp = a.Ci + (size_t)(jbase + (lane >> 3)) * a.ldci + ibase + (lane & 7) * 8;
    const uint8_t *sp = scr + (lane >> 3) * kScratchPitch + (lane & 7) * 16;
#pragma unroll
    for (int t = 0; t < 4; ++t) *(u32x4 *)(cp + (size_t)(8 * t) * a.ldci) = *(const u32x4 *)(sp + 8 * t * kScratchPitch);
}

// The same from values already rounded and packed (p[q] = elements 2q, 2q + 1 of the tile's registers).
__device__ __forceinline__ void store_pair_ci_packed(const TjGemmArgs<tj_bf16> &a, const uint32_t (&p0)[8],
                                                     const uint32_t (&p1)[8], uint8_t *scr, const int ibase,
                                                     const int jbase, const int lane)
{
    const int l32 = lane & 31, lg = lane >> 5;
    wave_sync();
#pragma unroll
    for (int rq = 0; rq < 4; ++rq) {
        *(uint2 *)(scr + l32 * kScratchPitch + (rq * 8 + lg * 4) * 2) = make_uint2(p0[2 * rq], p0[2 * rq + 1]);
        *(uint2 *)(scr + l32 * kScratchPitch + 64 + (rq * 8 + lg * 4) * 2) = make_uint2(p1[2 * rq], p1[2 * rq + 1]);
    }
    wave_sync();
    tj_bf16 *cp = a.Ci + (size_t)(jbase + (lane >> 3)) * a.ldci + ibase + (lane & 7) * 8;
    const uint8_t *sp = scr + (lane >> 3) * kScratchPitch + (lane & 7) * 16;
#pragma unroll
    for (int t = 0; t < 4; ++t) *(u32x4 *)(cp + (size_t)(8 * t) * a.ldci) = *(const u32x4 *)(sp + 8 * t * kScratchPitch);
}

// Cj: tiles v0 | v1 neighbours in j (rows i, 64 consecutive j).
__device__ __forceinline__ void store_pair_cj(const TjGemmArgs<tj_bf16> &a, const f32x16 &v0, const f32x16 &v1,
                                              uint8_t *scr, const int ibase, const int jbase, const int lane)
{
    typedef tj_bf16 T;
    const int l32 = lane & 31, lg = lane >> 5;
    wave_sync();
#pragma unroll
    for (int rq = 0; rq < 4; ++rq) {
        const uint32_t a01 = pack_bf16(v0[rq * 4], v0[rq * 4 + 1]), a23 = pack_bf16(v0[rq * 4 + 2], v0[rq * 4 + 3]);
        const uint32_t b01 = pack_bf16(v1[rq * 4], v1[rq * 4 + 1]), b23 = pack_bf16(v1[rq * 4 + 2], v1[rq * 4 + 3]);
        uint8_t *wp = scr + (rq * 8 + lg * 4) * kScratchPitch + l32 * 2;
        *(T *)(wp) = (T)(a01 & 0xFFFFu);
        *(T *)(wp + kScratchPitch) = (T)(a01 >> 16);
        *(T *)(wp + 2 * kScratchPitch) = (T)(a23 & 0xFFFFu);
        *(T *)(wp + 3 * kScratchPitch) = (T)(a23 >> 16);
        *(T *)(wp + 64) = (T)(b01 & 0xFFFFu);
        *(T *)(wp + 64 + kScratchPitch) = (T)(b01 >> 16);
        *(T *)(wp + 64 + 2 * kScratchPitch) = (T)(b23 & 0xFFFFu);
        *(T *)(wp + 64 + 3 * kScratchPitch) = (T)(b23 >> 16);
    }
    wave_sync();
    T *cp = a.Cj + (size_t)(ibase + (lane >> 3)) * a.ldcj + jbase + (lane & 7) * 8;
    const uint8_t *sp = scr + (lane >> 3) * kScratchPitch + (lane & 7) * 16;
#pragma unroll
    for (int t = 0; t < 4; ++t) *(u32x4 *)(cp + (size_t)(8 * t) * a.ldcj) = *(const u32x4 *)(sp + 8 * t * kScratchPitch);
}

// The same from values already rounded and packed.
__device__ __forceinline__ void store_pair_cj_packed(const TjGemmArgs<tj_bf16> &a, const uint32_t (&p0)[8],
                                                     const uint32_t (&p1)[8], uint8_t *scr, const int ibase,
                                                     const int jbase, const int lane)
{
    typedef tj_bf16 T;
    const int l32 = lane & 31, lg = lane >> 5;
    wave_sync();
#pragma unroll
    for (int rq = 0; rq < 4; ++rq) {
        uint8_t *wp = scr + (rq * 8 + lg * 4) * kScratchPitch + l32 * 2;
        *(T *)(wp) = (T)(p0[2 * rq] & 0xFFFFu);
        *(T *)(wp + kScratchPitch) = (T)(p0[2 * rq] >> 16);
        *(T *)(wp + 2 * kScratchPitch) = (T)(p0[2 * rq + 1] & 0xFFFFu);
        *(T *)(wp + 3 * kScratchPitch) = (T)(p0[2 * rq + 1] >> 16);
        *(T *)(wp + 64) = (T)(p1[2 * rq] & 0xFFFFu);
        *(T *)(wp + 64 + kScratchPitch) = (T)(p1[2 * rq] >> 16);
        *(T *)(wp + 64 + 2 * kScratchPitch) = (T)(p1[2 * rq + 1] & 0xFFFFu);
        *(T *)(wp + 64 + 3 * kScratchPitch) = (T)(p1[2 * rq + 1] >> 16);
    }
    wave_sync();
    T *cp = a.Cj + (size_t)(ibase + (lane >> 3)) * a.ldcj + jbase + (lane & 7) * 8;
    const uint8_t *sp = scr + (lane >> 3) * kScratchPitch + (lane & 7) * 16;
#pragma unroll
    for (int t = 0; t < 4; ++t) *(u32x4 *)(cp + (size_t)(8 * t) * a.ldcj) = *(const u32x4 *)(sp + 8 * t * kScratchPitch);
}

// ---------------------------------------------------------------- bf16 kernel
//
// Block tile 256 (i) x 128 (j), four waves as 2 x 2, wave tile 128 x 64 = 4 x 2
// MFMA tiles (128 accumulator registers), stage depth 64 k.  Two blocks fit a
// CU (55 KB of LDS, < 256 registers), so one block's global-load wait overlaps
// the other's MFMAs.  The 1-D grid is remapped so that the eight XCDs (which
// take workgroups round-robin, each with its own L2) own disjoint runs of j
// tiles and sweep all i tiles of a run: the P operand (weights) stays resident
// in every L2 and each Q row block is fetched from HBM once.
// The epilogue stages each 32 x 32 accumulator tile through a wave-private LDS
// scratch so that global stores are 16 bytes per lane along the contiguous
// index of each output.
constexpr int B2I = 256, B2J = 128;

struct TileMap {
    int tiles_i, tiles_j;   // tile counts (tiles_j over all segments)
    int spread_i;           // 1: the XCDs split the i tiles (few j tiles), 0: they split the j tiles
};

// Tile of a block without a split contraction: id % 8 is the XCD the block lands on.
__device__ __forceinline__ bool xcd_tile(const TileMap &tm, int id, int &ti, int &tj)
{
    const int xcd = id & 7, slot = id >> 3;
    if (tm.spread_i) {
        tj = slot % tm.tiles_j;
        ti = (slot / tm.tiles_j) * 8 + xcd;
    } else {
        ti = slot % tm.tiles_i;
        tj = (slot / tm.tiles_i) * 8 + xcd;
    }
    return ti < tm.tiles_i && tj < tm.tiles_j;
}

inline unsigned xcd_grid(TileMap &tm)
{
    tm.spread_i = tm.tiles_j < 8 && tm.tiles_i > tm.tiles_j;
    return tm.spread_i ? (unsigned)tm.tiles_j * ((tm.tiles_i + 7) / 8) * 8
                       : (unsigned)tm.tiles_i * ((tm.tiles_j + 7) / 8) * 8;
}

__global__ __launch_bounds__(256, 2) void gemm_bf16(const TjGemmArgs<tj_bf16> a, const int tiles_seg0,
                                                    const TileMap tm)
{
    typedef tj_bf16 T;
    constexpr int VE = 8, KE = 64;
    __shared__ __align__(16) uint8_t sP[B2I * kLdsRow];
    __shared__ __align__(16) uint8_t sQ[B2J * kLdsRow];

    // XCD-aware tile order: id % 8 = XCD; an XCD walks i fastest inside its j tiles
    int ti, tj, z;
    {
        const int id = blockIdx.x;
        if (a.n_split > 1) {          // split contraction: slices of one tile land on different XCDs,
            z = id % a.n_split;       // tiles of one slice share the operand columns they stream
            const int t = id / a.n_split;
            ti = t % tm.tiles_i;
            tj = t / tm.tiles_i;
        } else {
            z = 0;
            if (!xcd_tile(tm, id, ti, tj)) return;
        }
        if (tj >= tm.tiles_j) return;
    }

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wi = wave & 1, wj = wave >> 1;
    const int l32 = lane & 31, lg = lane >> 5;

    const int sidx = (a.n_seg > 1 && tj >= tiles_seg0) ? 1 : 0;
    const TjGemmSeg<T> seg = a.seg[sidx];
    const int j0 = seg.j_begin + (tj - (sidx ? tiles_seg0 : 0)) * B2J;
    const int j_end = seg.j_end;
    const int i0 = ti * B2I;
    const int k_begin = z * a.k_chunk;
    const int k_end = min(a.K, k_begin + a.k_chunk);

    const int cv = tid & 7, r0 = tid >> 3;
    const T *gP[8];
    const T *gQ[4];
    uint32_t okmask = 0;
#pragma unroll
    for (int r = 0; r < 8; ++r) {
        const int i = i0 + r0 + 32 * r;
        const bool ok = i < a.I;
        okmask |= (uint32_t)ok << r;
        gP[r] = seg.P + (size_t)(ok ? i : 0) * a.ldp + cv * VE;
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int j = j0 + r0 + 32 * r;
        const bool ok = j < j_end;
        okmask |= (uint32_t)ok << (8 + r);
        gQ[r] = a.Q + (size_t)(ok ? j - seg.q_shift : 0) * a.ldq + cv * VE;
    }
    u32x4 rP[8], rQ[4];
    const u32x4 zero4 = {0u, 0u, 0u, 0u};
    auto gload = [&](int k0) {
        const bool kin = k0 + cv * VE < k_end;
#pragma unroll
        for (int r = 0; r < 8; ++r) rP[r] = (kin && ((okmask >> r) & 1)) ? *(const u32x4 *)(gP[r] + k0) : zero4;
#pragma unroll
        for (int r = 0; r < 4; ++r) rQ[r] = (kin && ((okmask >> (8 + r)) & 1)) ? *(const u32x4 *)(gQ[r] + k0) : zero4;
    };
    auto lstore = [&]() {
#pragma unroll
        for (int r = 0; r < 8; ++r) *(u32x4 *)(sP + (r0 + 32 * r) * kLdsRow + cv * 16) = rP[r];
#pragma unroll
        for (int r = 0; r < 4; ++r) *(u32x4 *)(sQ + (r0 + 32 * r) * kLdsRow + cv * 16) = rQ[r];
    };

    f32x16 acc[4][2];
#pragma unroll
    for (int fi = 0; fi < 4; ++fi)
#pragma unroll
        for (int fj = 0; fj < 2; ++fj)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[fi][fj][r] = 0.f;

    const bool do_qsum = a.qsum != nullptr && ti == 0 && wi == 0;
    float qs[2] = {0.f, 0.f};
    const uint8_t *pbase = sP + (wi * 128 + l32) * kLdsRow + lg * 16;
    const uint8_t *qbase = sQ + (wj * 64 + l32) * kLdsRow + lg * 16;

    gload(k_begin);
    lstore();
    __syncthreads();
    for (int k0 = k_begin; k0 < k_end; k0 += KE) {
        const bool more = k0 + KE < k_end;
        if (more) gload(k0 + KE);
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            u32x4 pf[4], qf[2];
#pragma unroll
            for (int f = 0; f < 4; ++f) pf[f] = *(const u32x4 *)(pbase + f * 32 * kLdsRow + ks * 32);
#pragma unroll
            for (int f = 0; f < 2; ++f) qf[f] = *(const u32x4 *)(qbase + f * 32 * kLdsRow + ks * 32);
#pragma unroll
            for (int fi = 0; fi < 4; ++fi)
#pragma unroll
                for (int fj = 0; fj < 2; ++fj) mma<T>(acc[fi][fj], pf[fi], qf[fj]);
            if (do_qsum) {
                qs[0] += vec_sum<T>(qf[0]);
                qs[1] += vec_sum<T>(qf[1]);
            }
        }
        __syncthreads();
        if (more) {
            lstore();
            __syncthreads();
        }
    }

    if (do_qsum) {
#pragma unroll
        for (int fj = 0; fj < 2; ++fj) {
            float s = qs[fj] + __shfl_xor(qs[fj], 32, 64);
            const int j = j0 + wj * 64 + fj * 32 + l32;
            if (lg == 0 && j < j_end) a.qsum[(size_t)z * a.qsum_zstride + j] = s;
        }
    }

    // ---- epilogue: bias / ReLU / mask on every tile, then the stores, one 32 x 32 tile at a time
    // through wave-private scratch
#pragma unroll
    for (int fi = 0; fi < 4; ++fi)
#pragma unroll
        for (int fj = 0; fj < 2; ++fj)
            tile_math(a, seg, acc[fi][fj], i0 + wi * 128 + fi * 32, j0 + wj * 64 + fj * 32, j_end, lane);
    uint8_t *scr = sP + wave * (32 * kScratchPitch);     // 4.5 KB per wave, inside sP
#pragma unroll
    for (int fi = 0; fi < 4; ++fi) {
#pragma unroll
        for (int fj = 0; fj < 2; ++fj) {
            const int ibase = i0 + wi * 128 + fi * 32;     // first i of this tile
            const int jbase = j0 + wj * 64 + fj * 32;      // first j of this tile
            store_tile(a, acc[fi][fj], scr, ibase, jbase, j_end, z, lane);
        }
    }
}

// ---------------------------------------------------------------- bf16 kernel, direct-to-LDS
//
// Block tile 256 (i) x 64*NFJ (j), eight waves as 4 (i) x 2 (j), wave tile
// 64 x 32*NFJ.  Operands go from global memory straight into LDS
// (global_load_lds, 16 bytes per lane: the 64 lanes of one instruction fill one
// contiguous KiB of a stage buffer), NSTAGE buffers form a ring, and the loads of
// stage s + NSTAGE - 1 are issued before the MFMAs of stage s: nothing is staged
// in registers and HBM latency is covered by NSTAGE - 1 stages of MFMA work.
// A stage holds BKB bytes of k per row (128 or 64).  The LDS serves a 16-byte
// read to 16 lanes per cycle out of 64 four-byte banks, so the operand reads of
// 16 consecutive rows must cover 16 distinct 16-byte columns of a 256-byte
// line.  Without padding this is done by an XOR swizzle applied on the global
// side: the 16-byte vector c of row r is stored at position c ^ ((r >> 1) & 7)
// (128-byte rows) or c ^ ((r >> 2) & 3) (64-byte rows).
// Requires whole stages (K and the split chunk multiples of BKB/2 elements);
// rows past the end are clamped to the last valid row, their results are never
// stored.  vmcnt counts a wave's outstanding loads in issue order, so waiting
// for "at most (stages still in flight) x (loads per stage)" means the oldest
// stage has landed; the barrier that follows extends this to the whole block
// and also says that every wave is done reading the buffer about to be refilled.
template <int N> struct IntC { static constexpr int value = N; };

// LDS bytes of one block: NSTAGE stage buffers of the P tile (256 rows) and of the Q tile.
template <int NFJ, int BKB, int NSTAGE> constexpr int dlds_lds_bytes() { return NSTAGE * (256 + 64 * NFJ) * BKB; }

// TRANS: both operands are stored with the contraction index as their SLOW index, P as [k][i] with
// row pitch ldp and Q as [k][j] with row pitch ldq (the weight gradient dW[j][i] = sum_m dZ[m][j] X[m][i]
// straight from the row-major activations and gradients).  A stage then holds 32 contraction rows
// of 256 (P) and 64*NFJ (Q) columns, fetched as whole rows, and the MFMA operands (8 consecutive
// contraction values per lane) come out of LDS through transposing reads (ds_read_b64_tr_b16:
// lane i of a 16-lane group receives column i of four consecutive rows, whose 8-byte pieces the
// group's lanes 4r .. 4r+3 point at).  The 16-byte vector v of row r is stored at position
// v ^ ((r & 3) << 2), so that the rows one transposing read touches fall into distinct banks.
// Needs BKB = 64, NFJ = 2, one segment, no q_shift, I and the segment's columns multiples of 8.
// TRANS = 2: only P is stored that way (the input gradient dX[j][i] = sum_n dZ[j][n] W[n][i] from
// the row-major weights); Q keeps its contraction-contiguous rows, 32 elements of them per stage.
// OUTS: 0, or the set of outputs (kOutCi | kOutCj | kOutCf) the launch can have: the epilogue of the others
// is not compiled in (shorter code, fewer live registers after the main loop).
template <int NFJ, int BKB, int NSTAGE, bool QSUM, bool GATHER = false, int TRANS = 0, int OUTS = 0>
__device__ __forceinline__ void dlds_body(const TjGemmArgs<tj_bf16> &a_in, const int tiles_seg0, const TileMap &tm,
                                          const int block_id, uint8_t *lds)
{
    TjGemmArgs<tj_bf16> a = a_in;
    if constexpr (OUTS != 0) {
        if (!(OUTS & kOutCi)) a.Ci = nullptr;
        if (!(OUTS & kOutCj)) a.Cj = nullptr;
        if (!(OUTS & kOutCf)) a.Cf = nullptr;
    }
    typedef tj_bf16 T;
    static_assert(TRANS == 0 || (BKB == 64 && NFJ == 2 && !GATHER), "transposed operands: 256 x 128 tiles, 32-row stages");
    constexpr int BJ3 = 64 * NFJ;
    constexpr int KE = BKB / 2;              // k elements per stage
    constexpr int VPR = BKB / 16;            // 16-byte vectors per row
    constexpr int RPI = 1024 / BKB;          // rows filled by one load instruction
    constexpr int CHP = 256 / RPI, CHQ = BJ3 / RPI;
    constexpr int LP = CHP / 8, LQ = (CHQ + 7) / 8;
    constexpr int LPS = LP + LQ;             // load instructions per stage per wave
    constexpr int KS = BKB / 32;             // MFMA k steps per stage
    constexpr int SZA = 256 * BKB, SZB = BJ3 * BKB;
    static_assert(NSTAGE >= 2 && NSTAGE <= 6 && (NSTAGE - 1) * LPS < 64, "ring depth");
    uint8_t *const sA0 = lds;                // stage buffers: P tiles first, then Q tiles
    uint8_t *const sA1 = lds + SZA;
    uint8_t *const sA2 = lds + 2 * SZA;
    uint8_t *const sA3 = lds + 3 * SZA;
    uint8_t *const sB0 = lds + NSTAGE * SZA;
    uint8_t *const sB1 = sB0 + SZB;
    uint8_t *const sB2 = sB0 + 2 * SZB;
    uint8_t *const sB3 = sB0 + 3 * SZB;
    (void)sB0; (void)sB1; (void)sB2; (void)sB3;
    auto bufA = [&](auto u) -> uint8_t * { return lds + decltype(u)::value * SZA; };
    auto bufB = [&](auto u) -> uint8_t * { return lds + NSTAGE * SZA + decltype(u)::value * SZB; };

    int ti, tj, z;
    {
        const int id = block_id;
        if (a.n_split > 1) {
            z = id % a.n_split;
            const int t = id / a.n_split;
            ti = t % tm.tiles_i;
            tj = t / tm.tiles_i;
        } else {
            z = 0;
            if (!xcd_tile(tm, id, ti, tj)) return;
        }
        if (tj >= tm.tiles_j) return;
    }

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wi = wave & 3, wj = wave >> 2;
    const int l32 = lane & 31, lg = lane >> 5;

    const int sidx = (a.n_seg > 1 && tj >= tiles_seg0) ? 1 : 0;
    const TjGemmSeg<T> seg = a.seg[sidx];
    const int j0 = seg.j_begin + (tj - (sidx ? tiles_seg0 : 0)) * BJ3;
    const int j_end = seg.j_end;
    const int i0 = ti * 256;
    const int k_begin = z * a.k_chunk;
    const int k_end = min(a.K, k_begin + a.k_chunk);
    const int n_stage = k_end > k_begin ? (k_end - k_begin) / KE : 0;

    // This wave's load instructions per stage: P chunks wave + 8 t (t < LP) and Q chunks wave + 8 t
    // (t < LQ); a chunk = RPI rows.  Q chunk numbers wrap around CHQ: a chunk past the end repeats an
    // earlier one (same data to the same place) so that every wave issues exactly LPS loads.
    const int lrow = lane / VPR, lpos = lane % VPR;
    auto swizzle = [](int row) { return VPR == 8 ? (row >> 1) & 7 : (row >> 2) & 3; };
    const T *gsrcP[LP];
    const T *gsrcQ[LQ];
    if constexpr (TRANS != 0) {
        // P: load instruction c = wave + 8 t fills rows 2c, 2c+1 (512 bytes each).  Columns past the end
        // repeat the last valid vector.
#pragma unroll
        for (int t = 0; t < LP; ++t) {
            const int row = 2 * (wave + 8 * t) + (lane >> 5);
            const int col = min(i0 + 8 * ((lane & 31) ^ ((row & 3) << 2)), a.I - 8);
            gsrcP[t] = seg.P + (size_t)(k_begin + row) * a.ldp + col;
        }
    } else {
#pragma unroll
        for (int t = 0; t < LP; ++t) {
            const int row = (wave + 8 * t) * RPI + lrow;
            const int i = min(i0 + row, a.I - 1);
            if constexpr (GATHER)
                gsrcP[t] = seg.P + tj_gather_origin(a.gather, (uint32_t)i);
            else
                gsrcP[t] = seg.P + (size_t)i * a.ldp + (lpos ^ swizzle(row)) * 8 + k_begin;
        }
    }
    if constexpr (TRANS == 1) {
        // Q: instruction c = wave fills rows 4c .. 4c+3 (256 bytes each)
        const int rowq = 4 * wave + (lane >> 4);
        const int colq = min(j0 + 8 * ((lane & 15) ^ ((rowq & 3) << 2)), j_end - 8);
        gsrcQ[0] = a.Q + (size_t)(k_begin + rowq) * a.ldq + colq;
    } else {
#pragma unroll
        for (int t = 0; t < LQ; ++t) {
            const int c = (wave + 8 * t) % CHQ;
            const int row = c * RPI + lrow;
            const int j = min(j0 + row, j_end - 1);
            gsrcQ[t] = a.Q + (size_t)(j - seg.q_shift) * a.ldq + (lpos ^ swizzle(row)) * 8 + k_begin;
        }
    }
    // gather form: the k of this lane's vector is the same for all its P rows (the swizzle of a
    // lane's rows does not depend on t), so one offset per stage serves every P load
    const int kposP = (lpos ^ swizzle(wave * RPI + lrow)) * 8 + k_begin;
    // elements a stage advances the sources by
    const size_t stepP = TRANS != 0 ? (size_t)KE * a.ldp : (size_t)KE, stepQ = TRANS == 1 ? (size_t)KE * a.ldq : (size_t)KE;
    // global_load_lds_dwordx4: lane l's 16 bytes go to LDS address M0 + 16 l.  Issued as inline
    // assembly so that the compiler's wait-count pass does not see these loads: it would otherwise
    // put a vmcnt(0) wait (all stages landed) in front of LDS reads it cannot tell apart from the
    // buffers being filled.  Completion is tracked by the explicit vmcnt waits in wait_stage().
    // M0 is written here and by nothing else in this kernel.
    typedef __attribute__((address_space(3))) uint8_t *lds_ptr_t;
    auto dma16 = [](const T *src, uint8_t *dst) {
        const uint32_t lds_addr = (uint32_t)(uintptr_t)(lds_ptr_t)dst;
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_addr), "v"(src)
                     : "memory");
    };
    auto issue = [&](uint8_t *sA, uint8_t *sB, int s) {
        const size_t offP = GATHER ? (size_t)tj_gather_koff(a.gather, kposP + s * KE) : s * stepP;
#pragma unroll
        for (int t = 0; t < LP; ++t) dma16(gsrcP[t] + offP, sA + (wave + 8 * t) * 1024);
#pragma unroll
        for (int t = 0; t < LQ; ++t) {
            const int c = (wave + 8 * t) % CHQ;   // wave-uniform
            dma16(gsrcQ[t] + s * stepQ, sB + c * 1024);
        }
    };

    f32x16 acc[2][NFJ];
#pragma unroll
    for (int fi = 0; fi < 2; ++fi)
#pragma unroll
        for (int fj = 0; fj < NFJ; ++fj)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[fi][fj][r] = 0.f;

    const bool do_qsum = QSUM && a.qsum != nullptr && ti == 0 && wi == 0;
    float qs[NFJ];
#pragma unroll
    for (int fj = 0; fj < NFJ; ++fj) qs[fj] = 0.f;

    const int swz = (swizzle(l32) ^ lg) * 16;   // tile bases are multiples of 32 rows
    const int pa_off = (wi * 64 + l32) * BKB, pb_off = (wj * 32 * NFJ + l32) * BKB;
    // Operand fetch runs one k step ahead of the MFMAs; the scheduling barriers keep the compiler
    // from hoisting every LDS read of a stage to its top (which costs > 256 registers).
    // transposed operands: byte offset of this lane's 8-byte piece in row 8 (lane / 32) + (lane % 16) / 4 of a
    // stage, for the 32 columns starting at the wave's first (fragment f adds 4 vectors before the swizzle)
    const int i16 = lane & 15;
    const int tr_row = 8 * lg + (i16 >> 2), tr_swz = ((i16 >> 2) & 3) << 2;
    const int tr_vec = 2 * ((lane >> 4) & 1) + ((i16 & 3) >> 1), tr_lo = (i16 & 1) * 8;
    auto compute = [&](const uint8_t *sA, const uint8_t *sB) {
        u32x4 pf[2][2], qf[2][NFJ];
        auto fetch = [&](int ks, int set) {
            typedef short s16x4 __attribute__((ext_vector_type(4)));
            typedef __attribute__((address_space(3))) s16x4 *lds_s16x4_ptr;
            auto rd = [&](const uint8_t *base, int pitch, int vec0) {
                const uint8_t *p0 = base + (16 * ks + tr_row) * pitch + (((vec0 + tr_vec) ^ tr_swz) << 4) + tr_lo;
                const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)p0);
                const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(p0 + 4 * pitch));
                const uint2 l2 = __builtin_bit_cast(uint2, lo), h2 = __builtin_bit_cast(uint2, hi);
                const u32x4 v = {l2.x, l2.y, h2.x, h2.y};
                return v;
            };
            const int off = swz ^ (ks * 32);
            if constexpr (TRANS != 0) {
#pragma unroll
                for (int f = 0; f < 2; ++f) pf[set][f] = rd(sA, 512, 8 * wi + 4 * f);
            } else {
#pragma unroll
                for (int f = 0; f < 2; ++f) pf[set][f] = *(const u32x4 *)(sA + pa_off + f * 32 * BKB + off);
            }
            if constexpr (TRANS == 1) {
#pragma unroll
                for (int f = 0; f < NFJ; ++f) qf[set][f] = rd(sB, 2 * BJ3, 4 * NFJ * wj + 4 * f);
            } else {
#pragma unroll
                for (int f = 0; f < NFJ; ++f) qf[set][f] = *(const u32x4 *)(sB + pb_off + f * 32 * BKB + off);
            }
        };
        fetch(0, 0);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const int set = ks & 1;
            if (ks + 1 < KS) fetch(ks + 1, set ^ 1);
#pragma unroll
            for (int fi = 0; fi < 2; ++fi)
#pragma unroll
                for (int fj = 0; fj < NFJ; ++fj) mma<T>(acc[fi][fj], pf[set][fi], qf[set][fj]);
            if constexpr (QSUM) {
                if (do_qsum) {
#pragma unroll
                    for (int fj = 0; fj < NFJ; ++fj) qs[fj] += vec_sum<T>(qf[set][fj]);
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    // s_waitcnt vmcnt(n) only (lgkmcnt and expcnt left alone); n < 64
    auto wait_vm = [&](auto n) {
        constexpr int N = decltype(n)::value;
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
    };
    // stage ss has landed for this wave once at most min(NSTAGE-2, n_stage-1-ss) later stages are pending
    auto wait_stage = [&](int ss) {
        const int later = min(NSTAGE - 2, n_stage - 1 - ss);
        if constexpr (NSTAGE >= 6) { if (later >= 4) { wait_vm(IntC<4 * LPS>{}); return; } }
        if constexpr (NSTAGE >= 5) { if (later >= 3) { wait_vm(IntC<3 * LPS>{}); return; } }
        if constexpr (NSTAGE >= 4) { if (later >= 2) { wait_vm(IntC<2 * LPS>{}); return; } }
        if constexpr (NSTAGE >= 3) { if (later >= 1) { wait_vm(IntC<1 * LPS>{}); return; } }
        wait_vm(IntC<0>{});
    };
    // one ring position: wait for stage ss (in buffer U), refill the buffer freed by stage ss-1, compute
    auto ring_step = [&](auto u, int ss) {
        constexpr int U = decltype(u)::value;
        constexpr int UN = (U + NSTAGE - 1) % NSTAGE;
        wait_stage(ss);
        // A bare barrier: __syncthreads() carries a fence that would wait for every outstanding
        // direct load (vmcnt(0)) and with it the stages meant to stay in flight.  The empty asm
        // statements keep the compiler from moving LDS accesses across the barrier.
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        if (ss + NSTAGE - 1 < n_stage) issue(bufA(IntC<UN>{}), bufB(IntC<UN>{}), ss + NSTAGE - 1);
        compute(bufA(u), bufB(u));
    };

    if (0 < n_stage) issue(bufA(IntC<0>{}), bufB(IntC<0>{}), 0);
    if constexpr (NSTAGE > 2) { if (1 < n_stage) issue(bufA(IntC<1>{}), bufB(IntC<1>{}), 1); }
    if constexpr (NSTAGE > 3) { if (2 < n_stage) issue(bufA(IntC<2>{}), bufB(IntC<2>{}), 2); }
    if constexpr (NSTAGE > 4) { if (3 < n_stage) issue(bufA(IntC<3>{}), bufB(IntC<3>{}), 3); }
    if constexpr (NSTAGE > 5) { if (4 < n_stage) issue(bufA(IntC<4>{}), bufB(IntC<4>{}), 4); }
    for (int s = 0; s < n_stage; s += NSTAGE) {
        ring_step(IntC<0>{}, s);
        if (s + 1 < n_stage) ring_step(IntC<1>{}, s + 1);
        if constexpr (NSTAGE > 2) { if (s + 2 < n_stage) ring_step(IntC<2>{}, s + 2); }
        if constexpr (NSTAGE > 3) { if (s + 3 < n_stage) ring_step(IntC<3>{}, s + 3); }
        if constexpr (NSTAGE > 4) { if (s + 4 < n_stage) ring_step(IntC<4>{}, s + 4); }
        if constexpr (NSTAGE > 5) { if (s + 5 < n_stage) ring_step(IntC<5>{}, s + 5); }
    }
    __syncthreads();   // every wave is done with the operand buffers: the epilogue reuses them

    if constexpr (QSUM) {
        if (do_qsum) {
#pragma unroll
            for (int fj = 0; fj < NFJ; ++fj) {
                float sum = qs[fj] + __shfl_xor(qs[fj], 32, 64);
                const int j = j0 + wj * 32 * NFJ + fj * 32 + l32;
                if (lg == 0 && j < j_end) a.qsum[(size_t)z * a.qsum_zstride + j] = sum;
            }
        }
    }

    if constexpr (GATHER) {
        if (a.out_map.on) {
            // Mapped output (input gradient of a convolution): each 32 x 32 tile is staged in the wave's LDS
            // scratch as bf16 rows of 32 columns; a lane then owns 8 consecutive columns (channels of one
            // pixel) of a row: one 16-byte mask load and one 16-byte store at the mapped address.
            constexpr int WPBm = SZA / (32 * kScratchPitch) >= 4 ? 4 : SZA / (32 * kScratchPitch);
            static_assert(WPBm >= 2 && 7 / WPBm < NSTAGE, "epilogue scratch does not fit the P buffers");
            const int sbm = wave / WPBm;
            uint8_t *scrm = (sbm == 0 ? sA0 : sbm == 1 ? sA1 : sbm == 2 ? sA2 : sA3) + (wave % WPBm) * (32 * kScratchPitch);
#pragma unroll
            for (int fi = 0; fi < 2; ++fi) {
                const int ibase = i0 + wi * 64 + fi * 32;
                int64_t org[2];
#pragma unroll
                for (int t = 0; t < 2; ++t)
                    org[t] = tj_gather_origin(a.out_map, (uint32_t)min(ibase + (lane >> 2) + 16 * t, a.I - 1));
#pragma unroll
                for (int fj = 0; fj < NFJ; ++fj) {
                    const int jbase = j0 + wj * 32 * NFJ + fj * 32;
                    const f32x16 &v = acc[fi][fj];
                    wave_sync();
#pragma unroll
                    for (int rq = 0; rq < 4; ++rq) {
                        const uint32_t p01 = pack_bf16(v[rq * 4], v[rq * 4 + 1]), p23 = pack_bf16(v[rq * 4 + 2], v[rq * 4 + 3]);
                        uint8_t *wp = scrm + (rq * 8 + lg * 4) * kScratchPitch + l32 * 2;
                        *(T *)(wp) = (T)(p01 & 0xFFFFu);
                        *(T *)(wp + kScratchPitch) = (T)(p01 >> 16);
                        *(T *)(wp + 2 * kScratchPitch) = (T)(p23 & 0xFFFFu);
                        *(T *)(wp + 3 * kScratchPitch) = (T)(p23 >> 16);
                    }
                    wave_sync();
                    const int jv = jbase + (lane & 3) * 8;
                    if (jv >= j_end) continue;
                    const int64_t col = tj_gather_koff(a.out_map, jv);
#pragma unroll
                    for (int t = 0; t < 2; ++t) {
                        if (ibase + (lane >> 2) + 16 * t >= a.I) continue;
                        u32x4 d = *(const u32x4 *)(scrm + ((lane >> 2) + 16 * t) * kScratchPitch + (lane & 3) * 16);
                        const int64_t off = org[t] + col;
                        if (a.mask_cj) {
                            const u32x4 m = *(const u32x4 *)(a.mask_cj + off);
#pragma unroll
                            for (int e = 0; e < 4; ++e) {   // keep where the bf16 mask value is > 0
                                const uint32_t lo = m[e] & 0xFFFFu, hi = m[e] >> 16;
                                const uint32_t keep = ((lo & 0x7FFFu) != 0 && !(lo & 0x8000u) ? 0x0000FFFFu : 0u) |
                                                      ((hi & 0x7FFFu) != 0 && !(hi & 0x8000u) ? 0xFFFF0000u : 0u);
                                d[e] &= keep;
                            }
                        }
                        *(u32x4 *)(a.Cj + off) = d;
                    }
                }
            }
            return;
        }
    }

    // ---- epilogue (as in gemm_bf16): math on every tile first, then the stores
    constexpr int WPB = SZA / (32 * kScratchPitch) >= 4 ? 4 : SZA / (32 * kScratchPitch);   // waves per buffer
    static_assert(WPB >= 2 && 7 / WPB < NSTAGE, "epilogue scratch does not fit the P buffers");
    const int sb = wave / WPB;
    uint8_t *scr = (sb == 0 ? sA0 : sb == 1 ? sA1 : sb == 2 ? sA2 : sA3) + (wave % WPB) * (32 * kScratchPitch);
    const int ib0 = i0 + wi * 64, jb0 = j0 + wj * 32 * NFJ;
    if constexpr (OUTS == kOutCi || OUTS == (kOutCi | kOutCj)) {
        // bf16 outputs only: every tile is rounded as soon as its math is done, so the stores start from half
        // as many live registers
        uint32_t pk[2][NFJ][8];
#pragma unroll
        for (int fi = 0; fi < 2; ++fi)
#pragma unroll
            for (int fj = 0; fj < NFJ; ++fj) {
                tile_math(a, seg, acc[fi][fj], ib0 + fi * 32, jb0 + fj * 32, j_end, lane);
#pragma unroll
                for (int q = 0; q < 8; ++q) pk[fi][fj][q] = pack_bf16(acc[fi][fj][2 * q], acc[fi][fj][2 * q + 1]);
            }
        // edge tiles: the guarded stores round again, which leaves a bf16 value as it is
        auto widen = [&](const uint32_t (&p)[8]) {
            f32x16 v;
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                v[2 * q] = __uint_as_float(p[q] << 16);
                v[2 * q + 1] = __uint_as_float(p[q] & 0xFFFF0000u);
            }
            return v;
        };
        if (a.Ci) {
#pragma unroll
            for (int fj = 0; fj < NFJ; ++fj) {
                const int jb = jb0 + fj * 32;
                if (ib0 + 64 <= a.I && jb + 32 <= j_end) {
                    store_pair_ci_packed(a, pk[0][fj], pk[1][fj], scr, ib0, jb, lane);
                } else {
#pragma unroll
                    for (int fi = 0; fi < 2; ++fi)
                        store_tile(a, widen(pk[fi][fj]), scr, ib0 + fi * 32, jb, j_end, z, lane, kOutCi);
                }
            }
        }
        if constexpr ((OUTS & kOutCj) != 0) {
            if (a.Cj) {
                const int jmax = min(j_end, a.cj_jmax);
#pragma unroll
                for (int fi = 0; fi < 2; ++fi) {
#pragma unroll
                    for (int fj = 0; fj + 1 < NFJ; fj += 2) {
                        const int jb = jb0 + fj * 32;
                        if (ib0 + fi * 32 + 32 <= a.I && jb + 64 <= jmax && ((a.ldcj | jb) & 7) == 0) {
                            store_pair_cj_packed(a, pk[fi][fj], pk[fi][fj + 1], scr, ib0 + fi * 32, jb, lane);
                        } else {
                            store_tile(a, widen(pk[fi][fj]), scr, ib0 + fi * 32, jb, j_end, z, lane, kOutCj);
                            store_tile(a, widen(pk[fi][fj + 1]), scr, ib0 + fi * 32, jb + 32, j_end, z, lane, kOutCj);
                        }
                    }
                    if (NFJ & 1)
                        store_tile(a, widen(pk[fi][NFJ - 1]), scr, ib0 + fi * 32, jb0 + (NFJ - 1) * 32, j_end, z, lane, kOutCj);
                }
            }
        }
        return;
    }
#pragma unroll
    for (int fi = 0; fi < 2; ++fi)
#pragma unroll
        for (int fj = 0; fj < NFJ; ++fj)
            tile_math(a, seg, acc[fi][fj], i0 + wi * 64 + fi * 32, j0 + wj * 32 * NFJ + fj * 32, j_end, lane);
    if (a.Ci) {
#pragma unroll
        for (int fj = 0; fj < NFJ; ++fj) {
            const int jb = jb0 + fj * 32;
            if (ib0 + 64 <= a.I && jb + 32 <= j_end) {
                store_pair_ci(a, acc[0][fj], acc[1][fj], scr, ib0, jb, lane);
            } else {
                store_tile(a, acc[0][fj], scr, ib0, jb, j_end, z, lane, kOutCi);
                store_tile(a, acc[1][fj], scr, ib0 + 32, jb, j_end, z, lane, kOutCi);
            }
        }
    }
    if (a.Cj) {
        const int jmax = min(j_end, a.cj_jmax);
#pragma unroll
        for (int fi = 0; fi < 2; ++fi) {
#pragma unroll
            for (int fj = 0; fj + 1 < NFJ; fj += 2) {
                const int jb = jb0 + fj * 32;
                if (ib0 + fi * 32 + 32 <= a.I && jb + 64 <= jmax && ((a.ldcj | jb) & 7) == 0) {
                    store_pair_cj(a, acc[fi][fj], acc[fi][fj + 1], scr, ib0 + fi * 32, jb, lane);
                } else {
                    store_tile(a, acc[fi][fj], scr, ib0 + fi * 32, jb, j_end, z, lane, kOutCj);
                    store_tile(a, acc[fi][fj + 1], scr, ib0 + fi * 32, jb + 32, j_end, z, lane, kOutCj);
                }
            }
            if (NFJ & 1) store_tile(a, acc[fi][NFJ - 1], scr, ib0 + fi * 32, jb0 + (NFJ - 1) * 32, j_end, z, lane, kOutCj);
        }
    }
    if (a.Cf) {
#pragma unroll
        for (int fi = 0; fi < 2; ++fi)
#pragma unroll
            for (int fj = 0; fj < NFJ; ++fj)
                store_tile(a, acc[fi][fj], scr, ib0 + fi * 32, jb0 + fj * 32, j_end, z, lane, kOutCf);
    }
}

#define TJ_DLDS_ATTRS(NFJ, BKB, NSTAGE)                                                             \
    __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(((NFJ) <= 2 && (BKB) * (NSTAGE) <= 192) ? 4 : 2, \
                                                              ((NFJ) <= 2 && (BKB) * (NSTAGE) <= 192) ? 4 : 2)))

template <int NFJ, int BKB, int NSTAGE, bool QSUM, bool GATHER = false, int TRANS = 0, int OUTS = 0>
__global__ TJ_DLDS_ATTRS(NFJ, BKB, NSTAGE) void gemm_bf16_dlds(const TjGemmArgs<tj_bf16> a, const int tiles_seg0,
                                                              const TileMap tm)
{
    __shared__ __align__(1024) uint8_t lds[dlds_lds_bytes<NFJ, BKB, NSTAGE>()];
    dlds_body<NFJ, BKB, NSTAGE, QSUM, GATHER, TRANS, OUTS>(a, tiles_seg0, tm, (int)blockIdx.x, lds);
}

// Two independent GEMMs in one launch (e.g. the weight gradient and the input gradient of a layer,
// which both start from the same dZ): blocks [0, nblk0) work on the first, the rest on the second,
// so the two share one ramp-up and one tail instead of running back to back.  Either may have
// transposed operands (TjGemmArgs::trans); both forms of the body share the stage buffers.
struct GemmPair {
    TjGemmArgs<tj_bf16> a[2];
    int tiles_seg0[2];
    TileMap tm[2];
    int nblk0;
};

// HIDDEN: both members have transposed operands and the outputs of a hidden layer's backward pass (the
// weight gradient only its fp32 slices, the input gradient only its row-major bf16 copy).
template <int NFJ, int BKB, int NSTAGE, int HIDDEN = 0>   // 2: the input gradient also in its transposed layout; 3: see below
__global__ TJ_DLDS_ATTRS(NFJ, BKB, NSTAGE) void gemm_bf16_dlds_pair(const GemmPair p)
{
    __shared__ __align__(1024) uint8_t lds[dlds_lds_bytes<NFJ, BKB, NSTAGE>()];
    const int which = (int)blockIdx.x >= p.nblk0 ? 1 : 0;
    const int id = (int)blockIdx.x - which * p.nblk0;
    if constexpr (HIDDEN == 3) {   // two split weight gradients: fp32 slices only
        dlds_body<NFJ, BKB, NSTAGE, true, false, 0, kOutCf>(p.a[which], p.tiles_seg0[which], p.tm[which], id, lds);
        return;
    }
    if constexpr (HIDDEN == 1 || HIDDEN == 2) {
        static_assert(BKB == 64 && NFJ == 2, "transposed operands: 256 x 128 tiles");
        if (p.a[which].trans == 1)   // block-uniform
            dlds_body<NFJ, BKB, NSTAGE, true, false, 1, kOutCf>(p.a[which], p.tiles_seg0[which], p.tm[which], id, lds);
        else
            dlds_body<NFJ, BKB, NSTAGE, false, false, 2, HIDDEN == 2 ? (kOutCi | kOutCj) : kOutCi>(
                p.a[which], p.tiles_seg0[which], p.tm[which], id, lds);
        return;
    }
    if constexpr (BKB == 64 && NFJ == 2) {
        if (p.a[which].trans == 1) {   // block-uniform
            dlds_body<NFJ, BKB, NSTAGE, true, false, 1>(p.a[which], p.tiles_seg0[which], p.tm[which], id, lds);
            return;
        }
        if (p.a[which].trans == 2) {
            dlds_body<NFJ, BKB, NSTAGE, false, false, 2>(p.a[which], p.tiles_seg0[which], p.tm[which], id, lds);
            return;
        }
    }
    dlds_body<NFJ, BKB, NSTAGE, true>(p.a[which], p.tiles_seg0[which], p.tm[which], id, lds);
}

// Vectors of four per thread in the slice-sum blocks below.  On the 256-1024-1024-1024-32 network at
// batch 8192 the launch takes 29.4 us with one, 26.0 with two, 28.4 - 29.0 with three.
constexpr int kSumVectorsPerThread = 2;

// Two split weight gradients with transposed operands (blocks [0, n_gemm)) and, behind them, the sum of
// the gradient slices of a parameter range whose slices are complete: 512 * kSumVectorsPerThread
// vectors of four per block, slices added in slice order with eight loads per vector in flight,
// exactly as the optimizer kernel adds them.
// Every block of a launch carries the same LDS allocation; it is rounded up here to more than half of a
// CU's 160 KB, so that no two blocks share a CU: a contraction block keeps its CU's load path to itself
// and the streaming blocks run on the CUs that hold none.
__global__ TJ_DLDS_ATTRS(2, 64, 3) void gemm_bf16_dlds_pair_sum(const GemmPair p, const int n_gemm, const TjSliceSum r)
{
    constexpr size_t kAlone = 88 * 1024;
    __shared__ __align__(1024) uint8_t lds[dlds_lds_bytes<2, 64, 3>() > kAlone ? dlds_lds_bytes<2, 64, 3>() : kAlone];
    if ((int)blockIdx.x >= n_gemm) {
        typedef float f32x4_t __attribute__((ext_vector_type(4)));
        constexpr int NV = kSumVectorsPerThread;
        const size_t base = r.begin + ((size_t)((int)blockIdx.x - n_gemm) * (512 * NV) + threadIdx.x) * 4;
        f32x4_t g[NV], q[NV][8];
        bool in[NV];
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            in[v] = base + (size_t)v * 2048 < r.end;
            if (in[v]) g[v] = *(const f32x4_t *)(r.g + base + (size_t)v * 2048);
        }
        for (int s0 = 1; s0 < r.S; s0 += 8) {
#pragma unroll
            for (int u = 0; u < 8; ++u)
#pragma unroll
                for (int v = 0; v < NV; ++v)
                    if (s0 + u < r.S && in[v])
                        q[v][u] = __builtin_nontemporal_load((const f32x4_t *)(r.g + (size_t)(s0 + u) * r.stride + base + (size_t)v * 2048));
#pragma unroll
            for (int u = 0; u < 8; ++u)
#pragma unroll
                for (int v = 0; v < NV; ++v)
                    if (s0 + u < r.S && in[v]) { g[v].x += q[v][u].x; g[v].y += q[v][u].y; g[v].z += q[v][u].z; g[v].w += q[v][u].w; }
        }
#pragma unroll
        for (int v = 0; v < NV; ++v)
            if (in[v]) *(f32x4_t *)(r.g + base + (size_t)v * 2048) = g[v];
        return;
    }
    const int which = (int)blockIdx.x >= p.nblk0 ? 1 : 0;
    dlds_body<2, 64, 3, true, false, 1, kOutCf>(p.a[which], p.tiles_seg0[which], p.tm[which],
                                                (int)blockIdx.x - which * p.nblk0, lds);
}

// The same for two gathered-operand problems (a convolution under the online and under the target
// weights).
template <int NFJ>
__global__ TJ_DLDS_ATTRS(NFJ, 64, 3) void gemm_bf16_dlds_gpair(const GemmPair p)
{
    __shared__ __align__(1024) uint8_t lds[dlds_lds_bytes<NFJ, 64, 3>()];
    const int which = (int)blockIdx.x >= p.nblk0 ? 1 : 0;
    dlds_body<NFJ, 64, 3, false, true>(p.a[which], p.tiles_seg0[which], p.tm[which],
                                       (int)blockIdx.x - which * p.nblk0, lds);
}

// Tile map and grid size of one problem for the 256 x 64*NFJ tiles.
template <int NFJ> unsigned plan_dlds(const TjGemmArgs<tj_bf16> &a, TileMap &tm, int tiles[2])
{
    constexpr int BJ3 = 64 * NFJ;
    tm.tiles_i = (a.I + 255) / 256;
    tiles[0] = tiles[1] = 0;
    for (int s = 0; s < a.n_seg; ++s) tiles[s] = (a.seg[s].j_end - a.seg[s].j_begin + BJ3 - 1) / BJ3;
    tm.tiles_j = tiles[0] + tiles[1];
    tm.spread_i = 0;
    return a.n_split > 1 ? (unsigned)tm.tiles_i * tm.tiles_j * a.n_split : xcd_grid(tm);
}

template <int NFJ, int BKB, int NSTAGE, bool GATHER = false>
int launch_dlds(const TjGemmArgs<tj_bf16> &a, hipStream_t st)
{
    TileMap tm;
    int tiles[2];
    const unsigned nblk = plan_dlds<NFJ>(a, tm, tiles);
    if constexpr (GATHER)
        gemm_bf16_dlds<NFJ, BKB, NSTAGE, false, true><<<nblk, 512, 0, st>>>(a, tiles[0], tm);
    else if (a.qsum)
        gemm_bf16_dlds<NFJ, BKB, NSTAGE, true><<<nblk, 512, 0, st>>>(a, tiles[0], tm);
    else if (a.Ci && !a.Cj && !a.Cf)   // a hidden layer's forward: one bf16 output
        gemm_bf16_dlds<NFJ, BKB, NSTAGE, false, false, 0, kOutCi><<<nblk, 512, 0, st>>>(a, tiles[0], tm);
    else if (a.Ci && a.Cj && !a.Cf)   // ... in both layouts
        gemm_bf16_dlds<NFJ, BKB, NSTAGE, false, false, 0, kOutCi | kOutCj><<<nblk, 512, 0, st>>>(a, tiles[0], tm);
    else
        gemm_bf16_dlds<NFJ, BKB, NSTAGE, false><<<nblk, 512, 0, st>>>(a, tiles[0], tm);
    return hipGetLastError() == hipSuccess ? TJ_OK : TJ_ERR_DEVICE;
}

// The direct-to-LDS kernel needs whole 64-k stages in every split slice and enough rows to fill
// its 256-row tiles; everything else takes the register-staged kernel.  A skinny product (a head
// layer: 32 rows or more) over many columns still streams its column operand faster through the
// direct-to-LDS ring, even though most of a tile's rows repeat the last valid row.
bool uses_dlds(const TjGemmArgs<tj_bf16> &a)
{
    const bool whole_stages = a.K % 64 == 0 && (a.n_split == 1 || a.k_chunk % 64 == 0);
    if (!whole_stages) return false;
    if (a.I >= 128) return true;
    long jtot = 0;
    for (int s = 0; s < a.n_seg; ++s) jtot += a.seg[s].j_end - a.seg[s].j_begin;
    return a.I >= 32 && jtot * (long)a.K >= (1L << 24);
}

// What the transposed-operand form of the direct-to-LDS kernel assumes.
bool trans_ok(const TjGemmArgs<tj_bf16> &a)
{
    if (a.trans < 1 || a.trans > 2 || a.gather.on || a.out_map.on || a.n_seg != 1) return false;
    if (a.I < 8 || a.I % 8) return false;
    if (a.trans == 1) {
        const int cols = a.seg[0].j_end - a.seg[0].j_begin;
        if (a.seg[0].q_shift != 0 || cols < 8 || cols % 8 || a.seg[0].j_begin % 8) return false;
    } else if (a.qsum) {
        return false;
    }
    return a.K % 32 == 0 && (a.n_split == 1 || a.k_chunk % 32 == 0);
}

int launch_bf16(const TjGemmArgs<tj_bf16> &a, const int tiles[2], hipStream_t st)
{
    int jtot = 0;
    for (int s = 0; s < a.n_seg; ++s) jtot += a.seg[s].j_end - a.seg[s].j_begin;
    if (a.trans) {
        if (!trans_ok(a)) return TJ_ERR_SHAPE;
        TileMap tm;
        int t2[2];
        const unsigned nblk = plan_dlds<2>(a, tm, t2);
        if (a.trans == 2)
            gemm_bf16_dlds<2, 64, 3, false, false, 2><<<nblk, 512, 0, st>>>(a, t2[0], tm);
        else if (a.qsum)
            gemm_bf16_dlds<2, 64, 3, true, false, 1><<<nblk, 512, 0, st>>>(a, t2[0], tm);
        else
            gemm_bf16_dlds<2, 64, 3, false, false, 1><<<nblk, 512, 0, st>>>(a, t2[0], tm);
        return hipGetLastError() == hipSuccess ? TJ_OK : TJ_ERR_DEVICE;
    }
    if (a.gather.on) {
        if (a.n_seg != 1 || jtot > 128 || a.K % 64 || a.n_split != 1 || a.qsum || a.I < 1) return TJ_ERR_SHAPE;
        if (a.out_map.on && (!a.Cj || a.Ci || a.Cf || a.relu || a.bias_j || a.seg[0].bias || a.mask))
            return TJ_ERR_SHAPE;
        // short contractions: two blocks per CU overlap their phases
        return jtot > 64 ? launch_dlds<2, 64, 3, true>(a, st) : launch_dlds<1, 64, 3, true>(a, st);
    }
    if (a.out_map.on) return TJ_ERR_SHAPE;
    if (uses_dlds(a)) {
        // pick the j extent of the tile (128 / 192 / 256) that needs the fewest rounds of 256 blocks,
        // weighted by the tile's work; ties go to the larger tile
        if (jtot <= 64) return launch_dlds<1, 128, 3>(a, st);   // narrow outputs (conv channels)
        int best = 2;
        long best_cost = -1;
        for (int nfj = 2; nfj <= 4; ++nfj) {
            long t = 0;
            for (int s = 0; s < a.n_seg; ++s) t += (a.seg[s].j_end - a.seg[s].j_begin + 64 * nfj - 1) / (64 * nfj);
            t *= (long)((a.I + 255) / 256) * a.n_split;
            const long cost = ((t + 255) / 256) * nfj;
            if (best_cost < 0 || cost <= best_cost) { best = nfj; best_cost = cost; }
        }
        if (best == 2) {
            // more tiles than CUs: the shallow-stage variant fits two blocks per CU, so one block's
            // epilogue overlaps the other's main loop; otherwise one block per CU with deep stages
            long t = 0;
            for (int s = 0; s < a.n_seg; ++s) t += (a.seg[s].j_end - a.seg[s].j_begin + 127) / 128;
            t *= (long)((a.I + 255) / 256) * a.n_split;
            if (t > 256) return launch_dlds<2, 64, 3>(a, st);
            // at most half the CUs would get a 128-wide tile: 64-wide tiles give twice the blocks
            return t <= 128 ? launch_dlds<1, 128, 3>(a, st) : launch_dlds<2, 128, 3>(a, st);
        }
        if (best == 3) return launch_dlds<3, 128, 2>(a, st);
        return launch_dlds<4, 128, 2>(a, st);
    }
    TileMap tm;
    tm.tiles_i = (a.I + B2I - 1) / B2I;
    tm.tiles_j = tiles[0] + tiles[1];
    tm.spread_i = 0;
    const unsigned nblk = a.n_split > 1 ? (unsigned)tm.tiles_i * tm.tiles_j * a.n_split : xcd_grid(tm);
    gemm_bf16<<<nblk, 256, 0, st>>>(a, tiles[0], tm);
    return hipGetLastError() == hipSuccess ? TJ_OK : TJ_ERR_DEVICE;
}


// Shapes the kernels' loads and grids assume.
template <typename T> int check_args(const TjGemmArgs<T> &a, int tiles[2])
{
    constexpr int VE = TjElem<T>::kVec;
    constexpr int KE = kRowBytes / (int)sizeof(T);
    if (a.n_seg < 1 || a.n_seg > 2 || a.I <= 0 || a.K <= 0 || a.n_split < 1) return TJ_ERR_SHAPE;
    if (a.gather.on && sizeof(T) != 2) return TJ_ERR_SHAPE;
    if (a.trans) {   // P (and with trans == 1 also Q) as [k][columns]: the pitch bounds the columns, not the contraction
        if (sizeof(T) != 2 || a.ldp % VE || a.ldq % VE || a.I > a.ldp || a.K % VE) return TJ_ERR_SHAPE;
        for (int s = 0; s < a.n_seg; ++s)
            if (a.trans == 1 ? a.seg[s].j_end > a.ldq : a.K > a.ldq) return TJ_ERR_SHAPE;
    } else if ((!a.gather.on && (a.ldp % VE || a.K > a.ldp)) || a.ldq % VE || a.K % VE || a.K > a.ldq) {
        return TJ_ERR_SHAPE;
    }
    if (a.n_split > 1 && (a.k_chunk % KE || (size_t)a.k_chunk * a.n_split < (size_t)a.K)) return TJ_ERR_SHAPE;
    if (a.n_split == 1 && a.k_chunk < a.K) return TJ_ERR_SHAPE;
    if ((a.Ci && a.ldci % VE) || (a.mask && a.ldmask % 4)) return TJ_ERR_SHAPE;
    tiles[0] = tiles[1] = 0;
    for (int s = 0; s < a.n_seg; ++s) {
        if (a.seg[s].j_end <= a.seg[s].j_begin || !a.seg[s].P) return TJ_ERR_SHAPE;
        tiles[s] = (a.seg[s].j_end - a.seg[s].j_begin + BJ - 1) / BJ;
    }
    return TJ_OK;
}

}  // namespace

int tj_gemm_pair(const TjGemmArgs<tj_bf16> &a0, const TjGemmArgs<tj_bf16> &a1, hipStream_t st)
{
    int tiles[2], rc;
    if ((rc = check_args(a0, tiles)) != TJ_OK || (rc = check_args(a1, tiles)) != TJ_OK) return rc;
    auto fits = [](const TjGemmArgs<tj_bf16> &a) { return a.trans ? trans_ok(a) : uses_dlds(a); };
    if (a0.gather.on || a1.gather.on || !fits(a0) || !fits(a1)) {   // no common kernel: one after the other
        if ((rc = tj_gemm<tj_bf16>(a0, st)) != TJ_OK) return rc;
        return tj_gemm<tj_bf16>(a1, st);
    }
    GemmPair p;
    p.a[0] = a0; p.a[1] = a1;
    if (!a0.trans && !a1.trans) {   // two or more rounds of 256 x 256 tiles (one block per CU): a third less operand traffic
        // per flop than 256 x 128; with fewer tiles the two-blocks-per-CU variant below is as fast
        const unsigned m0 = plan_dlds<4>(a0, p.tm[0], tiles);
        p.tiles_seg0[0] = tiles[0];
        const unsigned m1 = plan_dlds<4>(a1, p.tm[1], tiles);
        p.tiles_seg0[1] = tiles[0];
        if (m0 + m1 >= 512) {
            p.nblk0 = (int)m0;
            gemm_bf16_dlds_pair<4, 128, 2><<<m0 + m1, 512, 0, st>>>(p);
            return hipGetLastError() == hipSuccess ? TJ_OK : TJ_ERR_DEVICE;
        }
    }
    if (!a0.trans && !a1.trans) {   // few tiles (skinny problems): 256 x 64 tiles with deep stages, one block per CU
        const unsigned s0 = plan_dlds<1>(a0, p.tm[0], tiles);
        p.tiles_seg0[0] = tiles[0];
        const unsigned s1 = plan_dlds<1>(a1, p.tm[1], tiles);
        p.tiles_seg0[1] = tiles[0];
        if (s0 + s1 <= 256) {
            p.nblk0 = (int)s0;
            if (a0.Cf && !a0.Ci && !a0.Cj && a1.Cf && !a1.Ci && !a1.Cj)
                gemm_bf16_dlds_pair<1, 128, 3, 3><<<s0 + s1, 512, 0, st>>>(p);
            else
                gemm_bf16_dlds_pair<1, 128, 3><<<s0 + s1, 512, 0, st>>>(p);
            return hipGetLastError() == hipSuccess ? TJ_OK : TJ_ERR_DEVICE;
        }
    }
    const unsigned n0 = plan_dlds<2>(a0, p.tm[0], tiles);
    p.tiles_seg0[0] = tiles[0];
    const unsigned n1 = plan_dlds<2>(a1, p.tm[1], tiles);
    p.tiles_seg0[1] = tiles[0];
    p.nblk0 = (int)n0;
    auto hidden = [](const TjGemmArgs<tj_bf16> &a) {
        return a.trans == 1 ? (a.Cf && !a.Ci && !a.Cj) : (a.trans == 2 && a.Ci && !a.Cf);
    };
    if (hidden(a0) && hidden(a1) && !(a0.trans == 2 && a0.Cj) && !(a1.trans == 2 && a1.Cj))
        gemm_bf16_dlds_pair<2, 64, 3, 1><<<n0 + n1, 512, 0, st>>>(p);
    else if (hidden(a0) && hidden(a1))
        gemm_bf16_dlds_pair<2, 64, 3, 2><<<n0 + n1, 512, 0, st>>>(p);
    else
        gemm_bf16_dlds_pair<2, 64, 3><<<n0 + n1, 512, 0, st>>>(p);
    return hipGetLastError() == hipSuccess ? TJ_OK : TJ_ERR_DEVICE;
}

int tj_gemm_pair_sum(const TjGemmArgs<tj_bf16> &a0, const TjGemmArgs<tj_bf16> &a1, const TjSliceSum &r,
                     hipStream_t st, bool *fused)
{
    *fused = false;
    int tiles[2], rc;
    if ((rc = check_args(a0, tiles)) != TJ_OK || (rc = check_args(a1, tiles)) != TJ_OK) return rc;
    auto slices_only = [](const TjGemmArgs<tj_bf16> &a) {
        return a.trans == 1 && trans_ok(a) && !a.gather.on && a.Cf && !a.Ci && !a.Cj;
    };
    const bool range_ok = r.g && r.S > 1 && r.begin % 4 == 0 && r.end % 4 == 0 && r.begin < r.end && r.end <= r.stride;
    if (!slices_only(a0) || !slices_only(a1) || !range_ok) return tj_gemm_pair(a0, a1, st);
    GemmPair p;
    p.a[0] = a0; p.a[1] = a1;
    const unsigned n0 = plan_dlds<2>(a0, p.tm[0], tiles);
    p.tiles_seg0[0] = tiles[0];
    const unsigned n1 = plan_dlds<2>(a1, p.tm[1], tiles);
    p.tiles_seg0[1] = tiles[0];
    p.nblk0 = (int)n0;
    const size_t per_block = 512 * (size_t)kSumVectorsPerThread;
    const size_t n_sum = ((r.end - r.begin) / 4 + per_block - 1) / per_block;
    // worth it only where the contractions leave compute units idle
    if (n0 + n1 >= 256 || n_sum >= (1u << 24)) return tj_gemm_pair(a0, a1, st);
    gemm_bf16_dlds_pair_sum<<<n0 + n1 + (unsigned)n_sum, 512, 0, st>>>(p, (int)(n0 + n1), r);
    if (hipGetLastError() != hipSuccess) return TJ_ERR_DEVICE;
    *fused = true;
    return TJ_OK;
}

int tj_gemm_gather_pair(const TjGemmArgs<tj_bf16> &a0, const TjGemmArgs<tj_bf16> &a1, hipStream_t st)
{
    int tiles[2], rc;
    if ((rc = check_args(a0, tiles)) != TJ_OK || (rc = check_args(a1, tiles)) != TJ_OK) return rc;
    auto fits = [](const TjGemmArgs<tj_bf16> &a, int &jtot) {   // what the gathered launch of launch_bf16 takes
        jtot = a.n_seg == 1 ? a.seg[0].j_end - a.seg[0].j_begin : 0;
        return a.gather.on && !a.out_map.on && a.n_seg == 1 && jtot <= 128 && a.K % 64 == 0 && a.n_split == 1 &&
               !a.qsum && a.I >= 1;
    };
    int j0 = 0, j1 = 0;
    if (!fits(a0, j0) || !fits(a1, j1) || (j0 > 64) != (j1 > 64)) {   // no common kernel: one after the other
        if ((rc = tj_gemm<tj_bf16>(a0, st)) != TJ_OK) return rc;
        return tj_gemm<tj_bf16>(a1, st);
    }
    GemmPair p;
    p.a[0] = a0; p.a[1] = a1;
    if (j0 > 64) {
        const unsigned n0 = plan_dlds<2>(a0, p.tm[0], tiles);
        p.tiles_seg0[0] = tiles[0];
        const unsigned n1 = plan_dlds<2>(a1, p.tm[1], tiles);
        p.tiles_seg0[1] = tiles[0];
        p.nblk0 = (int)n0;
        gemm_bf16_dlds_gpair<2><<<n0 + n1, 512, 0, st>>>(p);
    } else {
        const unsigned n0 = plan_dlds<1>(a0, p.tm[0], tiles);
        p.tiles_seg0[0] = tiles[0];
        const unsigned n1 = plan_dlds<1>(a1, p.tm[1], tiles);
        p.tiles_seg0[1] = tiles[0];
        p.nblk0 = (int)n0;
        gemm_bf16_dlds_gpair<1><<<n0 + n1, 512, 0, st>>>(p);
    }
    return hipGetLastError() == hipSuccess ? TJ_OK : TJ_ERR_DEVICE;
}

// Tile counts of the 32 x 32 tiling, and whether the problem is small enough for it
static bool ksplit4_plan(const TjGemmArgs<float> &a, int t32[2], long &blocks)
{
    long t64 = 0, t128 = 0;
    t32[0] = t32[1] = 0;
    for (int s = 0; s < a.n_seg; ++s) {
        const int len = a.seg[s].j_end - a.seg[s].j_begin;
        t128 += (len + BJ - 1) / BJ;
        t64 += (len + 63) / 64;
        t32[s] = (len + 31) / 32;
    }
    blocks = (long)((a.I + 31) / 32) * (t32[0] + t32[1]) * a.n_split;
    // the same thresholds as tj_gemm<float>
    return (long)((a.I + BI - 1) / BI) * t128 * a.n_split < 128 && (long)((a.I + 63) / 64) * t64 * a.n_split < 256;
}

int tj_gemm_pair_f32(const TjGemmArgs<float> &a0, const TjGemmArgs<float> &a1, hipStream_t st)
{
    int tiles[2], rc;
    if ((rc = check_args(a0, tiles)) != TJ_OK || (rc = check_args(a1, tiles)) != TJ_OK) return rc;
    PairF32 p;
    long n0 = 0, n1 = 0;
    int t0[2], t1[2];
    if (!ksplit4_plan(a0, t0, n0) || !ksplit4_plan(a1, t1, n1) || n0 + n1 > 0x7fffffff) {   // one after the other
        if ((rc = tj_gemm<float>(a0, st)) != TJ_OK) return rc;
        return tj_gemm<float>(a1, st);
    }
    p.a[0] = a0; p.a[1] = a1;
    p.tiles_seg0[0] = t0[0]; p.tiles_seg0[1] = t1[0];
    p.gx[0] = (a0.I + 31) / 32; p.gy[0] = t0[0] + t0[1];
    p.gx[1] = (a1.I + 31) / 32; p.gy[1] = t1[0] + t1[1];
    p.nblk0 = (int)n0;
    gemm_f32_ksplit4_pair<<<(unsigned)(n0 + n1), 256, 0, st>>>(p);
    return hipGetLastError() == hipSuccess ? TJ_OK : TJ_ERR_DEVICE;
}

template <typename T> int tj_gemm(const TjGemmArgs<T> &a, hipStream_t st)
{
    int tiles[2], rc;
    if ((rc = check_args(a, tiles)) != TJ_OK) return rc;
    if constexpr (sizeof(T) == 2) return launch_bf16(a, tiles, st);
    dim3 grid((a.I + BI - 1) / BI, tiles[0] + tiles[1], a.n_split);
    if ((long)grid.x * grid.y * grid.z < 128) {   // too few 128 x 128 tiles to fill the chip: 64 x 64 tiles
        int t64[2] = {0, 0};
        for (int s = 0; s < a.n_seg; ++s) t64[s] = (a.seg[s].j_end - a.seg[s].j_begin + 63) / 64;
        dim3 g64((a.I + 63) / 64, t64[0] + t64[1], a.n_split);
        if constexpr (sizeof(T) == 4) {
            if ((long)g64.x * g64.y * g64.z < 256) {   // and too few of those: 32 x 32 tiles, waves split k
                int t32[2] = {0, 0};
                for (int s = 0; s < a.n_seg; ++s) t32[s] = (a.seg[s].j_end - a.seg[s].j_begin + 31) / 32;
                dim3 g32((a.I + 31) / 32, t32[0] + t32[1], a.n_split);
                gemm_f32_ksplit4<<<g32, 256, 0, st>>>(a, t32[0]);
                return hipGetLastError() == hipSuccess ? TJ_OK : TJ_ERR_DEVICE;
            }
        }
        gemm_pq<T, 1><<<g64, 256, 0, st>>>(a, t64[0]);
    } else {
        gemm_pq<T, 2><<<grid, 256, 0, st>>>(a, tiles[0]);
    }
    return hipGetLastError() == hipSuccess ? TJ_OK : TJ_ERR_DEVICE;
}

template int tj_gemm<float>(const TjGemmArgs<float> &, hipStream_t);
template int tj_gemm<tj_bf16>(const TjGemmArgs<tj_bf16> &, hipStream_t);
