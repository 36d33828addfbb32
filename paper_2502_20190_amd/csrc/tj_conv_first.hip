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

// The four planes of an image as 4-byte pieces (task t = pixels 4t .. 4t+3 of every plane), up to
// kMaxRounds tasks per thread.
struct PlaneRegs {
    uint32_t px[kMaxRounds][4];
};

// Byte offsets of an image's four planes inside its source table: the planes of batch position b, of the
// table row an index names for it, or four planes named one by one (a frame ring's frames).  Indices
// are clamped to the table.
struct PlaneOff {
    size_t o[4];
};

__device__ __forceinline__ PlaneOff plane_offsets(const uint32_t *rows, const uint32_t *planes, const uint32_t n_rows,
                                                  const int b, const bool next, const int HW)
{
    PlaneOff p;
    if (planes) {
        const uint32_t *q = planes + (size_t)b * 8 + (next ? 4 : 0);
#pragma unroll
        for (int c = 0; c < 4; ++c) p.o[c] = (size_t)min(q[c], n_rows - 1u) * HW;
    } else {
        const uint32_t r = rows ? min(rows[b], n_rows - 1u) : (uint32_t)b;
#pragma unroll
        for (int c = 0; c < 4; ++c) p.o[c] = ((size_t)r * 4 + c) * HW;
    }
    return p;
}

__device__ __forceinline__ void fetch_planes(PlaneRegs &p, const uint8_t *src, const PlaneOff &off, const int n_task,
                                             const int n_round, const int tid)
{
#pragma unroll
    for (int r = 0; r < kMaxRounds; ++r) {
        const int t = tid + r * kThreads;
        if (r < n_round && t < n_task) {
#pragma unroll
            for (int c = 0; c < 4; ++c) p.px[r][c] = *(const uint32_t *)(src + off.o[c] + 4 * t);
        }
    }
}

// registers -> bf16(x * scale), channels-last, in LDS (and in `keep` where given)
__device__ __forceinline__ void convert_planes(const PlaneRegs &p, uint8_t *img, tj_bf16 *keep, const float scale,
                                               const int n_task, const int n_round, const int tid)
{
#pragma unroll
    for (int r = 0; r < kMaxRounds; ++r) {
        const int t = tid + r * kThreads;
        if (r < n_round && t < n_task) {
            u32x4 v[2];
#pragma unroll
            for (int q = 0; q < 4; ++q) {     // pixel 4t + q: channels 0..3
                float f[4];
#pragma unroll
                for (int c = 0; c < 4; ++c) f[c] = (float)((p.px[r][c] >> (8 * q)) & 0xFF) * scale;
                v[q >> 1][2 * (q & 1)] = pack2(f[0], f[1]);
                v[q >> 1][2 * (q & 1) + 1] = pack2(f[2], f[3]);
            }
            *(u32x4 *)(img + (size_t)t * 32) = v[0];
            *(u32x4 *)(img + (size_t)t * 32 + 16) = v[1];
            if (keep) {
                *(u32x4 *)(keep + (size_t)t * 16) = v[0];
                *(u32x4 *)(keep + (size_t)t * 16 + 8) = v[1];
            }
        }
    }
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
    PlaneRegs px;
    const int n_img = 2 * a.B;
    const int stride = (int)gridDim.x;
    // Image g (s images first, then s') lies in its table at the batch position itself or where the
    // caller's indices put it.  Fetches go through the block's images in order, so the place of the
    // next fetch is looked up right after the current one was issued, off the critical path.
    auto where = [&](int g) -> PlaneOff {
        return plane_offsets(a.rows, a.planes, a.n_rows, g < a.B ? g : g - a.B, g >= a.B, HW);
    };
    PlaneOff off_next = where((int)blockIdx.x < n_img ? (int)blockIdx.x : 0);
    auto fetch = [&](int g) {
        fetch_planes(px, g < a.B ? a.obs : a.next_obs, off_next, n_task, n_round, tid);
        if (g + stride < n_img) off_next = where(g + stride);
    };
    auto convert = [&](int g, uint8_t *img) {         // ... and the channels-last copy of an s image
        tj_bf16 *keep = g < a.B && a.act0 ? a.act0 + (size_t)g * HW * 4 : nullptr;
        convert_planes(px, img, keep, a.scale, n_task, n_round, tid);
    };

    const int OHW = a.OH * a.OW;
    const int n_tile = (OHW + 31) / 32;
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

// ---------------------------------------------------------------- weight gradient of the same layer
//
//   dW[o][k] = sum_m dZ[m][o] * patch[m][k],   db[o] = sum_m dZ[m][o],   m = (image, oh, ow)
//
// again from the u8 stacks: a persistent block per CU loops over s images, converts an image into
// LDS exactly as the forward kernel does (so the values are those the forward pass multiplied) and
// brings the image's OH*OW rows of dZ in beside it (direct-to-LDS loads, two buffers).  Both MFMA
// operands want 8 consecutive contraction values (patches m) per lane, and both tensors have m as
// their slow index; ds_read_b64_tr_b16 does the transposition on the way out of LDS: lane i of a
// 16-lane group receives element i of four rows whose 8-byte pieces the group's lanes 4r .. 4r+3 point
// at.  A piece of a patch row is one pixel (four channels), and consecutive patches of an output row
// are s pixels apart, so the rows are simply addressed inside the resident image.
// The 16 waves are K/32 column tiles (32 patch elements) x 16/(K/32) groups that split an image's
// patches; accumulators persist over the block's images, the groups are summed through LDS at the
// end in a fixed order.
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef __attribute__((address_space(3))) s16x4 *lds_s16x4_ptr;
typedef __attribute__((address_space(3))) uint8_t *lds_u8_ptr;

__device__ __forceinline__ bf16x8 read_tr8(const uint8_t *p0, const uint8_t *p1)
{
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)p0);
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)p1);
    const s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, v);
}

template <int KSZ, int CT>
__global__ __launch_bounds__(kThreads) void conv_first_wgrad_u8c4(const TjConvFirstWgradArgs a)
{
    extern __shared__ __align__(16) uint8_t smem[];
    constexpr int K = 4 * KSZ * KSZ;
    constexpr int NW = kThreads / 64;
    constexpr int NCT = K / 32;          // column tiles of 32 patch elements
    constexpr int NWC = NCT / CT;        // wave columns: a wave owns CT neighbouring tiles, which share its dZ operand
    constexpr int NMG = NW / NWC;        // wave groups over an image's patches
    static_assert(NWC * CT == NCT && NWC * NMG == NW, "column tiles must divide the waves");
    constexpr int kTileRows = 32 / (4 * KSZ);   // kernel rows (kw, c) a column tile spans
    static_assert(kTileRows * 4 * KSZ == 32, "column tiles of whole kernel rows");
    const int HW = a.H * a.W, OHW = a.OH * a.OW;
    const size_t img_bytes = (size_t)HW * 8;
    const int dz_bytes = OHW * 64;       // a multiple of 1 KiB
    uint8_t *img = smem;
    uint8_t *dzb = smem + img_bytes;     // two buffers of dz_bytes

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int h = lane >> 5, i16 = lane & 15, g2 = (lane >> 4) & 1;
    const int ct = (wave % NWC) * CT, mg = wave / NWC;   // first column tile of this wave, its group
    const int n_step = OHW / 16;         // 16 patches per MFMA (OH and OW are multiples of 4)
    const int per = (n_step + NMG - 1) / NMG;
    const int s_begin = min(mg * per, n_step), s_end = min(s_begin + per, n_step);

    // A step contracts over 16 patches: four consecutive output columns (4 owq .. 4 owq + 3) of four
    // consecutive output rows (4 ob .. 4 ob + 3); step t = ob (OW/4) + owq.  Slot 4r + j of a step is the patch
    // (4 ob + r, 4 owq + j), so every address below is a per-lane constant plus a per-step scalar.
    // This lane's piece of a transposing read: slot 8h + i16/4 (and + 4: the next output row), elements
    // 16 g2 + 4 (i16 % 4) .. +3 of the tile's 32 columns (one pixel's four channels).
    const int slot = 8 * h + (i16 >> 2), r = slot >> 2, j = slot & 3;
    const int kk = 32 * ct + 16 * g2 + 4 * (i16 & 3);       // patch element = (kh, kw, c = 0)
    const int kh = kk / (4 * KSZ);
    const int b_lane = ((r * a.s + kh) * a.W + j * a.s) * 8 + (kk - kh * 4 * KSZ) * 2, b_next = a.s * a.W * 8;
    const int a_lane = (r * a.OW + j) * 64 + (16 * g2 + 4 * (i16 & 3)) * 2, a_next = a.OW * 64;
    const int nq = a.OW / 4;
    const int b_ob = 4 * a.s * a.W * 8, b_owq = 4 * a.s * 8;   // bytes per step of ob, of owq: patches
    const int a_ob = 4 * a.OW * 64, a_owq = 4 * 64;            // ... rows of dZ
    const int ob_begin = s_begin / nq, owq_begin = s_begin - ob_begin * nq;

    const int n_task = HW / 4;
    const int n_round = (n_task + kThreads - 1) / kThreads;
    PlaneRegs px;
    auto dma_dz = [&](int g, uint8_t *dst) {
        const tj_bf16 *src = a.dZ + (size_t)g * OHW * 32 + lane * 8;
        for (int c = wave; c * 1024 < dz_bytes; c += NW) {
            const uint32_t lds_addr = (uint32_t)(uintptr_t)(lds_u8_ptr)(dst + c * 1024);
            asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_addr),
                         "v"(src + c * 512)
                         : "memory");
        }
    };

    f32x16 acc[CT];
#pragma unroll
    for (int c = 0; c < CT; ++c)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[c][r] = 0.f;
    float bs = 0.f;
    const bool do_bias = ct == 0;
    const int b_tile = kTileRows * a.W * 8;   // bytes from a column tile's pixels to the next tile's

    const int stride = (int)gridDim.x;
    int g = blockIdx.x;
    if (g >= a.B) return;                // the host launches at most B blocks
    // place of an s image in its table, as in the forward kernel; the next fetch's is looked up one image ahead
    PlaneOff off_next = plane_offsets(a.rows, a.planes, a.n_rows, g, false, HW);
    fetch_planes(px, a.obs, off_next, n_task, n_round, tid);
    if (g + stride < a.B) off_next = plane_offsets(a.rows, a.planes, a.n_rows, g + stride, false, HW);
    dma_dz(g, dzb);
    int cur = 0;
    for (; g < a.B; g += stride) {
        __syncthreads();                 // every wave has left the image before this one
        convert_planes(px, img, nullptr, a.scale, n_task, n_round, tid);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // this wave's share of dZ(g) has landed
        __syncthreads();                 // image and dZ rows complete
        if (g + stride < a.B) {          // in flight during the MFMAs below
            fetch_planes(px, a.obs, off_next, n_task, n_round, tid);
            if (g + 2 * stride < a.B) off_next = plane_offsets(a.rows, a.planes, a.n_rows, g + 2 * stride, false, HW);
            dma_dz(g + stride, dzb + (cur ^ 1) * dz_bytes);
        }
        const uint8_t *dz = dzb + cur * dz_bytes + a_lane, *pim = img + b_lane;
        int ob = ob_begin, owq = owq_begin;
        for (int st = s_begin; st < s_end; ++st) {
            const uint8_t *pb = pim + ob * b_ob + owq * b_owq, *pa = dz + ob * a_ob + owq * a_owq;
            const bf16x8 ap = read_tr8(pa, pa + a_next);
            bf16x8 bq[CT];
#pragma unroll
            for (int c = 0; c < CT; ++c) bq[c] = read_tr8(pb + c * b_tile, pb + c * b_tile + b_next);
#pragma unroll
            for (int c = 0; c < CT; ++c) acc[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ap, bq[c], acc[c], 0, 0, 0);
            if (do_bias) {
#pragma unroll
                for (int e = 0; e < 8; ++e) bs += (float)ap[e];
            }
            if (++owq == nq) { owq = 0; ++ob; }
        }
        cur ^= 1;
    }

    // ---- sum the wave groups (group 0 adds groups 1 .. NMG-1 in order) and write the block's slice
    // acc[c][r] = dW(o = 8 (r/4) + 4h + r%4, k = 32 (ct + c) + lane%32);  bs (after the half-wave sum) = db(lane%32)
    __syncthreads();                     // the image buffer is free: it becomes the scratch
    float *scr = (float *)smem;          // [NMG-1][NCT][16][64], then [NMG-1][32]
    float *scr_b = scr + (size_t)(NMG - 1) * NCT * 16 * 64;
    bs += __shfl_xor(bs, 32, 64);
    if (mg > 0) {
#pragma unroll
        for (int c = 0; c < CT; ++c)
#pragma unroll
            for (int r = 0; r < 16; ++r) scr[(((size_t)(mg - 1) * NCT + ct + c) * 16 + r) * 64 + lane] = acc[c][r];
        if (do_bias && h == 0) scr_b[(mg - 1) * 32 + lane] = bs;
    }
    __syncthreads();
    if (mg == 0) {
#pragma unroll 1
        for (int q = 1; q < NMG; ++q) {
#pragma unroll
            for (int c = 0; c < CT; ++c)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[c][r] += scr[(((size_t)(q - 1) * NCT + ct + c) * 16 + r) * 64 + lane];
            if (do_bias && h == 0) bs += scr_b[(q - 1) * 32 + lane];
        }
        float *out = a.part + (size_t)blockIdx.x * a.zstride;
#pragma unroll
        for (int c = 0; c < CT; ++c)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int o = 8 * (r >> 2) + 4 * h + (r & 3);
                out[(size_t)o * K + 32 * (ct + c) + (lane & 31)] = acc[c][r];
            }
        if (do_bias && h == 0) out[(size_t)32 * K + lane] = bs;
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
    if ((a.rows || a.planes) && a.n_rows == 0) return TJ_ERR_INVALID_ARG;
    if (a.rows && a.planes) return TJ_ERR_INVALID_ARG;
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

constexpr int kWgradTiles8 = 2;   // column tiles per wave of the 8 x 8 kernel's weight gradient

// LDS bytes of the weight-gradient kernel: one image, two dZ buffers; the final sum of the wave groups
// reuses them
static size_t conv_first_wgrad_lds_bytes(int H, int W, int k, int OHW)
{
    const int K = 4 * k * k, nct = K / 32, nmg = (kThreads / 64) / (nct / (k == 8 ? kWgradTiles8 : 1));
    const size_t work = (size_t)H * W * 8 + 2 * (size_t)OHW * 64;
    const size_t scratch = (size_t)(nmg - 1) * nct * 16 * 64 * 4 + (size_t)(nmg - 1) * 32 * 4;
    return work > scratch ? work : scratch;
}

bool tj_conv_first_wgrad_fits(int C, int H, int W, int k, int s, int O)
{
    if (!tj_conv_first_fits(C, H, W, k, s, O)) return false;
    const int OH = (H - k) / s + 1, OW = (W - k) / s + 1;
    if (OW % 4 || OH % 4) return false;             // 4 x 4 blocks of patches per MFMA step, whole 1 KiB loads of dZ
    return conv_first_wgrad_lds_bytes(H, W, k, OH * OW) <= kLdsLimit;
}

int tj_conv_first_wgrad(const TjConvFirstWgradArgs &a, hipStream_t st)
{
    if (!a.obs || !a.dZ || !a.part) return TJ_ERR_INVALID_ARG;
    if (a.B < 1 || a.n_part < 1 || a.n_part > a.B) return TJ_ERR_SHAPE;
    if (!tj_conv_first_wgrad_fits(4, a.H, a.W, a.k, a.s, 32)) return TJ_ERR_SHAPE;
    if (a.OH != (a.H - a.k) / a.s + 1 || a.OW != (a.W - a.k) / a.s + 1) return TJ_ERR_SHAPE;
    if (a.zstride < (size_t)32 * 4 * a.k * a.k + 32) return TJ_ERR_SHAPE;
    if ((((uintptr_t)a.obs) & 3) != 0 || (((uintptr_t)a.dZ) & 15) != 0) return TJ_ERR_INVALID_ARG;
    if ((a.rows || a.planes) && a.n_rows == 0) return TJ_ERR_INVALID_ARG;
    if (a.rows && a.planes) return TJ_ERR_INVALID_ARG;
    const size_t lds = conv_first_wgrad_lds_bytes(a.H, a.W, a.k, a.OH * a.OW);
    static bool attr_set = false;
    if (!attr_set) {
        TJ_HIP_TRY(hipFuncSetAttribute((const void *)conv_first_wgrad_u8c4<8, kWgradTiles8>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                       (int)kLdsLimit));
        TJ_HIP_TRY(hipFuncSetAttribute((const void *)conv_first_wgrad_u8c4<4, 1>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                       (int)kLdsLimit));
        attr_set = true;
    }
    if (a.k == 8)
        conv_first_wgrad_u8c4<8, kWgradTiles8><<<a.n_part, kThreads, lds, st>>>(a);
    else
        conv_first_wgrad_u8c4<4, 1><<<a.n_part, kThreads, lds, st>>>(a);
    return hipGetLastError() == hipSuccess ? TJ_OK : TJ_ERR_DEVICE;
}
