// Weight gradient of a convolution layer (backward of Algorithm 1's policy update through a
// convolutional Q-network) without a patch matrix:
//
//   dW[o][k] = sum_m dZ[m][o] * patch[m][k],   db[o] = sum_m dZ[m][o]
//
// m runs over the patches (img, oh, ow), k = (kh, kw, c) over a patch, which is gathered from the
// channels-last layer input on the fly.  Both operands are stored with the contraction index m as
// their SLOW index (dZ is [m][o], a patch row is contiguous in k), the opposite of what MFMA
// operand registers want (8 consecutive contraction values per lane).  The transposition happens
// on the way out of LDS: ds_read_b64_tr_b16 (gfx950) hands each lane of a 16-lane group four
// values taken from four consecutive LDS rows, i.e. lane i, element j = row j, column i of a
// 4 x 16 block whose rows the group's lanes 4j .. 4j+3 point at (8 bytes each).
//
// Block: all O (32 or 64) output channels x 128 patch columns, 8 waves = 4 column waves of 32 columns x 2
// row groups; the patch rows are split over blockIdx (deterministic partial sums, reduced by the
// caller).  Stages of 64 patch rows go global -> LDS directly (global_load_lds_dwordx4) through a ring
// of 3 buffers with explicit vmcnt accounting, as in the GEMM kernels; row group g contracts rows
// 32 g .. 32 g + 31 of every stage, and the two groups' accumulators are added through LDS at the end
// (group 0 + group 1).  Two row groups per block instead of twice as many row slices: the same number
// of blocks and resident waves writes half as many partial results.  LDS rows are XOR-swizzled on the
// global side so that the rows one transposing read touches fall into distinct bank groups.
#include "tj_gemm.h"

namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __attribute__((address_space(3))) s16x4 *lds_s16x4_ptr;
typedef __attribute__((address_space(3))) uint8_t *lds_u8_ptr;

constexpr int kBM = 64;          // patch rows per stage (32 per row group)
constexpr int kNST = 3;          // ring depth
constexpr int kBJ = 128;         // patch columns per block
constexpr int kLPS = 3;          // direct loads per stage per wave: 2 of the patch tile, 1 of dZ

__device__ __forceinline__ bf16x8 read_tr8(const uint8_t *p0, const uint8_t *p1)
{
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)p0);
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)p1);
    const s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, v);
}

__device__ __forceinline__ float sum8(bf16x8 v)
{
    float s = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) s += (float)v[e];
    return s;
}

template <int NFI>
__global__ __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(4, 4)))
void conv_wgrad_bf16(const TjConvWgradArgs a, const int njb)
{
    constexpr int O = 32 * NFI;
    constexpr int SZB = kBM * kBJ * 2;   // 16 KiB: 64 rows of 256 bytes
    constexpr int SZA = kBM * O * 2;     // 4 or 8 KiB
    constexpr int NA = SZA / 1024;       // dZ load instructions per stage
    __shared__ __align__(1024) uint8_t sB[kNST * SZB];
    __shared__ __align__(1024) uint8_t sA[kNST * SZA];
    static_assert(kNST * SZB >= (4 * NFI * 16 + NFI) * 64 * 4, "the ring doubles as the row groups' reduction scratch");

    // id % 8 is the XCD a block lands on: the column blocks of one row slice share an XCD (and
    // with it the L2 that holds the slice's image rows)
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int jb = slot % njb, z = (slot / njb) * 8 + xcd;
    if (z >= a.n_split) return;
    const int j0 = jb * kBJ;
    const int Mpad = (a.M + kBM - 1) / kBM * kBM;
    const int m_begin = z * a.m_chunk;
    const int m_end = min(Mpad, m_begin + a.m_chunk);
    const int n_stage = m_end > m_begin ? (m_end - m_begin) / kBM : 0;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int cw = wave & 3, rg = wave >> 2;   // column wave, row group

    // ---- loader roles
    // patch tile: instruction c = wave + 8 t covers rows 4c .. 4c+3 (256 bytes each); this lane
    // fetches the 16-byte vector stored at position (lane & 15) of row 4c + (lane >> 4)
    const int bsw = (lane >> 4) << 2;                           // swizzle of the lane's row: (row & 3) << 2
    int kkB = j0 + 8 * ((lane & 15) ^ bsw);
    if (kkB >= a.K) kkB = 0;                                    // columns past the patch: loaded, never stored
    const int koffB = tj_gather_koff(a.g, kkB);
    const int browB[2] = {4 * wave + (lane >> 4), 4 * (wave + 8) + (lane >> 4)};
    // dZ tile: instruction ia = wave % NA (with 32 channels the upper four waves repeat the lower four's loads)
    const int ia = wave % NA;
    int arow, acol;
    if (NFI == 2) {   // 128-byte rows, 8 per instruction
        arow = 8 * ia + (lane >> 3);
        acol = ((lane & 7) ^ (((arow >> 1) & 1) << 2)) * 8;
    } else {          // 64-byte rows, 16 per instruction
        arow = 16 * ia + (lane >> 2);
        acol = (lane & 3) * 8;
    }
    auto dma16 = [](const tj_bf16 *src, uint8_t *dst) {
        const uint32_t lds_addr = (uint32_t)(uintptr_t)(lds_u8_ptr)dst;
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_addr), "v"(src)
                     : "memory");
    };
    auto issue = [&](int s) {
        const int u = s % kNST;
        const int m0 = m_begin + s * kBM;
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const int m = min(m0 + browB[t], a.M - 1);   // rows past M meet zero rows of dZ
            dma16(a.act + tj_gather_origin(a.g, (uint32_t)m) + koffB, sB + u * SZB + (wave + 8 * t) * 1024);
        }
        dma16(a.dZ + (size_t)(m0 + arow) * O + acol, sA + u * SZA + ia * 1024);
    };

    // ---- consumer roles: lane (n = lane % 32, h = lane / 32) of a wave feeds column n of the MFMA
    // operand with contraction values 8h .. 8h+7 of each 16-row step, as two transposing reads
    const int i16 = lane & 15, g2 = (lane >> 4) & 1, h = lane >> 5;
    const int rowl = 32 * rg + 8 * h + (i16 >> 2);
    const int b_off = rowl * 256 + (((4 * cw + 2 * g2 + ((i16 & 3) >> 1)) ^ (((i16 >> 2) & 3) << 2)) << 4) + (i16 & 1) * 8;
    int a_off[NFI];
#pragma unroll
    for (int fi = 0; fi < NFI; ++fi) {
        if (NFI == 2)
            a_off[fi] = rowl * 128 + (((4 * fi + 2 * g2 + ((i16 & 3) >> 1)) ^ (((i16 >> 3) & 1) << 2)) << 4) + (i16 & 1) * 8;
        else
            a_off[fi] = rowl * 64 + ((2 * g2 + ((i16 & 3) >> 1)) << 4) + (i16 & 1) * 8;
    }

    f32x16 acc[NFI];
#pragma unroll
    for (int fi = 0; fi < NFI; ++fi)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[fi][r] = 0.f;
    const bool do_bias = jb == 0 && cw == 0;
    float bs[NFI];
#pragma unroll
    for (int fi = 0; fi < NFI; ++fi) bs[fi] = 0.f;

    if (0 < n_stage) issue(0);
    if (1 < n_stage) issue(1);
    for (int s = 0; s < n_stage; ++s) {
        // stage s has landed for this wave once at most min(1, n_stage-1-s) later stages are pending
        if (s + 1 < n_stage)
            asm volatile("s_waitcnt vmcnt(%0)" ::"n"(kLPS) : "memory");
        else
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_barrier();   // bare barrier: no fence, the stages in flight stay in flight
        asm volatile("" ::: "memory");
        if (s + kNST - 1 < n_stage) issue(s + kNST - 1);   // into the buffer stage s-1 has left
        const uint8_t *pB = sB + (s % kNST) * SZB + b_off;
        const uint8_t *pA = sA + (s % kNST) * SZA;
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {   // the row group's 32 rows, 16 per step
            const bf16x8 bq = read_tr8(pB + (16 * ks) * 256, pB + (16 * ks + 4) * 256);
#pragma unroll
            for (int fi = 0; fi < NFI; ++fi) {
                const int rb = O * 2;
                const bf16x8 ap = read_tr8(pA + a_off[fi] + (16 * ks) * rb, pA + a_off[fi] + (16 * ks + 4) * rb);
                acc[fi] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ap, bq, acc[fi], 0, 0, 0);
                if (do_bias) bs[fi] += sum8(ap);
            }
        }
    }

    // ---- the two row groups' sums: group 1 hands its accumulators over through the (now idle) ring
    float *red = (float *)sB;   // [cw][fi][r][lane], then the bias sums [fi][lane]
    __syncthreads();            // every wave has left the last stage
    if (rg == 1) {
#pragma unroll
        for (int fi = 0; fi < NFI; ++fi) {
#pragma unroll
            for (int r = 0; r < 16; ++r) red[((cw * NFI + fi) * 16 + r) * 64 + lane] = acc[fi][r];
            if (do_bias) red[(4 * NFI * 16 + fi) * 64 + lane] = bs[fi];
        }
    }
    __syncthreads();
    if (rg == 1) return;
#pragma unroll
    for (int fi = 0; fi < NFI; ++fi) {
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[fi][r] += red[((cw * NFI + fi) * 16 + r) * 64 + lane];
        if (do_bias) bs[fi] += red[(4 * NFI * 16 + fi) * 64 + lane];
    }

    // ---- partial results: acc[fi][r] = dW(o = 32 fi + 8 (r/4) + 4 h + r%4, k = j0 + 32 cw + lane%32)
    float *out = a.part + (size_t)z * a.zstride;
    const int kk = j0 + 32 * cw + (lane & 31);
    if (kk < a.K) {
#pragma unroll
        for (int fi = 0; fi < NFI; ++fi)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int o = 32 * fi + 8 * (r >> 2) + 4 * h + (r & 3);
                out[(size_t)o * a.K + kk] = acc[fi][r];
            }
    }
    if (do_bias) {
#pragma unroll
        for (int fi = 0; fi < NFI; ++fi) {
            const float sum = bs[fi] + __shfl_xor(bs[fi], 32, 64);
            if (h == 0) out[(size_t)O * a.K + 32 * fi + (lane & 31)] = sum;
        }
    }
}

}  // namespace

int tj_conv_wgrad(const TjConvWgradArgs &a, hipStream_t st)
{
    // what the kernel's loads and its grid assume
    if (!a.dZ || !a.act || !a.part || !a.g.on) return TJ_ERR_INVALID_ARG;
    if ((a.O != 32 && a.O != 64) || a.M < 1 || a.K < 8 || a.K % 8) return TJ_ERR_SHAPE;
    if (a.n_split < 1 || a.m_chunk < kBM || a.m_chunk % kBM) return TJ_ERR_SHAPE;
    if ((size_t)a.m_chunk * a.n_split < (size_t)a.M) return TJ_ERR_SHAPE;
    if (a.zstride < (size_t)a.O * a.K + a.O) return TJ_ERR_SHAPE;
    const int njb = (a.K + kBJ - 1) / kBJ;
    const unsigned nblk = 8u * njb * ((a.n_split + 7) / 8);
    if (a.O == 64)
        conv_wgrad_bf16<2><<<nblk, 512, 0, st>>>(a, njb);
    else
        conv_wgrad_bf16<1><<<nblk, 512, 0, st>>>(a, njb);
    return hipGetLastError() == hipSuccess ? TJ_OK : TJ_ERR_DEVICE;
}
