// The Learner's policy update (Algorithm 1 of the paper, batched as a double-DQN
// step): forward of the online network on [s ; s'] and of the target network on
// s' as one grouped GEMM per layer, fused TD-target / Huber / loss kernel,
// backward through Q_online(s), fused Adam, periodic hard target update.
//
// Device layout inside the caller's arena (T = fp32 or bf16 compute type, every
// 2-D buffer has its row pitch padded to a 16-byte multiple, pads stay zero):
//   theta_on, theta_tg, m, v      fp32 [P]      master state, flat order
//   gpart                         fp32 [S_ends][Ppad] split-K partial gradients, summed into slice 0 (S slices for the hidden layers)
//   Wc_on[l]  T [out][ld(in)]     WcT_on[l] T [in][ld(out)]   Wc_tg[l]
//   X[l]   T [3B][ld(d_l)]   rows: s | s' (online) | s' (target); X[0] has 2B rows
//   XT[l]  T [d_l][ld(B)]    transposed copy of the s rows (written only for weight gradients that
//                            contract over transposed operands: ragged batches or widths)
//   Qout   fp32 [3B][ld4(A)]
//   dZ[l]  T [B][ld(d_l)]    dZT[l] T [d_l][ld(B)]
#include "tj_gemm.h"
#include "tj_conv.h"
#include <math.h>
#include <string.h>
#include <algorithm>
#include <vector>

namespace {

// ---------------------------------------------------------------- small kernels

// Cast fp32 [R][C] to T with a padded pitch, and optionally to its transpose,
// through an LDS tile.  blockIdx.z selects the job.
template <typename T> struct CastJob {
    const float *src;   // [R][C], pitch C
    T *dst;             // [R][ldd]   (may be null)
    T *dstT;            // [C][lddT]  (may be null)
    int R, C, ldd, lddT;
    const uint32_t *rows = nullptr;   // optional: source row r is row min(rows[r], n_rows - 1) of src
    uint32_t n_rows = 0;
};
template <typename T> struct CastJobs {
    CastJob<T> job[TJ_MAX_LAYERS];
};

template <typename T> struct CastPack;
template <> struct CastPack<float> {
    typedef float4 Vec;   // 16 bytes of T
    __device__ static void store4(float *p, float a, float b, float c, float d) { *(float4 *)p = make_float4(a, b, c, d); }
    __device__ static Vec pack(const float *x) { return make_float4(x[0], x[1], x[2], x[3]); }
};
template <> struct CastPack<tj_bf16> {
    typedef uint4 Vec;
    __device__ static uint32_t two(float a, float b) { return (uint32_t)tj_f32_to_bf16(a) | ((uint32_t)tj_f32_to_bf16(b) << 16); }
    __device__ static void store4(tj_bf16 *p, float a, float b, float c, float d) { *(uint2 *)p = make_uint2(two(a, b), two(c, d)); }
    __device__ static Vec pack(const float *x)
    {
        return make_uint4(two(x[0], x[1]), two(x[2], x[3]), two(x[4], x[5]), two(x[6], x[7]));
    }
};

// 64 x 64 tiles: float4 loads, 8- or 16-byte stores of the straight copy, and 16-byte stores of the
// transposed copy out of an LDS tile (a vector of the transpose covers consecutive source rows).
// Vector stores may run into the pad elements of a row (inside the pitch): those are written as
// zero, which is what they hold anyway.  `vec` = the source is 16-byte aligned with C % 4 == 0.
template <typename T>
__global__ __launch_bounds__(256) void cast_transpose(const CastJobs<T> jobs)
{
    constexpr int VE = TjElem<T>::kVec;
    __shared__ float tile[64][65];
    const CastJob<T> jb = jobs.job[blockIdx.z];
    const int r0 = blockIdx.y * 64, c0 = blockIdx.x * 64;
    if (r0 >= jb.R || c0 >= jb.C) return;
    const bool vec = (((uintptr_t)jb.src & 15) == 0) && (jb.C % 4 == 0);
    const int tc = (threadIdx.x & 15) * 4, tr = threadIdx.x >> 4;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int r = r0 + tr + 16 * i, c = c0 + tc;
        float x[4] = {0.f, 0.f, 0.f, 0.f};
        if (r < jb.R && c < jb.C) {
            const size_t rs = jb.rows ? (size_t)min(jb.rows[r], jb.n_rows - 1u) : (size_t)r;
            const float *sp = jb.src + rs * jb.C + c;
            if (vec) {
                const float4 v = *(const float4 *)sp;
                x[0] = v.x; x[1] = v.y; x[2] = v.z; x[3] = v.w;
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (c + e < jb.C) x[e] = sp[e];
            }
            if (jb.dst) {
                T *dp = jb.dst + (size_t)r * jb.ldd + c;
                if (c + 4 <= jb.ldd) {
                    CastPack<T>::store4(dp, x[0], x[1], x[2], x[3]);
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (c + e < jb.C) dp[e] = TjElem<T>::from_f32(x[e]);
                }
            }
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) tile[tr + 16 * i][tc + e] = x[e];
    }
    if (!jb.dstT) return;
    __syncthreads();
    constexpr int VPC = 64 / VE;   // vectors per tile column
    for (int v = threadIdx.x; v < 64 * VPC; v += 256) {
        const int c = c0 + v / VPC, rq = (v % VPC) * VE, r = r0 + rq;
        if (c >= jb.C || r >= jb.R) continue;
        float x[VE];
#pragma unroll
        for (int u = 0; u < VE; ++u) x[u] = tile[rq + u][v / VPC];
        T *dp = jb.dstT + (size_t)c * jb.lddT + r;
        if (r + VE <= jb.lddT) {
            *(typename CastPack<T>::Vec *)dp = CastPack<T>::pack(x);
        } else {
#pragma unroll
            for (int u = 0; u < VE; ++u)
                if (r + u < jb.R) dp[u] = TjElem<T>::from_f32(x[u]);
        }
    }
}

template <typename T> int launch_cast(const CastJobs<T> &jobs, int n_jobs, hipStream_t st)
{
    int maxR = 0, maxC = 0;
    for (int i = 0; i < n_jobs; ++i) {
        maxR = jobs.job[i].R > maxR ? jobs.job[i].R : maxR;
        maxC = jobs.job[i].C > maxC ? jobs.job[i].C : maxC;
    }
    if (n_jobs == 0 || maxR == 0 || maxC == 0) return TJ_OK;
    dim3 grid((maxC + 63) / 64, (maxR + 63) / 64, n_jobs);
    cast_transpose<T><<<grid, 256, 0, st>>>(jobs);
    return hipGetLastError() == hipSuccess ? TJ_OK : TJ_ERR_DEVICE;
}

// Zero fill of a 16-byte aligned region (a kernel rather than a memset node, so that a caller may
// capture the step into a HIP graph).
__global__ __launch_bounds__(256) void zero_fill16(uint4 *__restrict__ p, size_t n16)
{
    const size_t stride = (size_t)gridDim.x * 256;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += stride) p[i] = make_uint4(0u, 0u, 0u, 0u);
}

inline int launch_zero(void *p, size_t bytes, hipStream_t st)   // bytes: a multiple of 256 (arena pieces)
{
    const size_t n16 = bytes / 16;
    if (n16 == 0) return TJ_OK;
    const unsigned blocks = (unsigned)((n16 + 255) / 256 < 4096 ? (n16 + 255) / 256 : 4096);
    zero_fill16<<<blocks, 256, 0, st>>>((uint4 *)p, n16);
    return hipGetLastError() == hipSuccess ? TJ_OK : TJ_ERR_DEVICE;
}

// TD target, Huber loss and its gradient, one thread per transition, one wave per block (many
// small blocks: the kernel is latency bound).
//   a* = argmax_a Q_on(s',a) (lowest index on ties); y = r + gamma (1-done) Q_tg(s',a*)
//   d = Q_on(s,a) - y; loss = mean Huber_kappa(d); dL/dQ_on(s,a) = clip(d,-k,k)/B
// Q rows: [0,B) Q_on(s), [B,2B) Q_on(s'), [2B,3B) Q_tg(s'); ldq is a multiple of 4 floats.  Each
// block leaves the sum of its losses in loss_part; the optimizer kernel adds them up.
constexpr int kTdBlock = 64;

__device__ __forceinline__ float huber_and_grad(float d, float kappa, int B, float *g)
{
    const float ad = fabsf(d);
    *g = fminf(fmaxf(d, -kappa), kappa) / (float)B;
    return ad <= kappa ? 0.5f * d * d : kappa * (ad - 0.5f * kappa);
}

template <typename T>
__global__ __launch_bounds__(kTdBlock) void td_huber(const float *__restrict__ Q, int ldq, int B, int A,
                                                     const int32_t *__restrict__ action,
                                                     const float *__restrict__ reward,
                                                     const uint8_t *__restrict__ done, float gamma, float kappa,
                                                     T *__restrict__ dZ, int lddz, T *__restrict__ dZT, int lddzt,
                                                     int32_t *__restrict__ astar, float *__restrict__ loss_part)
{
    const int j = blockIdx.x * kTdBlock + threadIdx.x;
    float loss = 0.f;
    if (j < B) {
        const float4 *qn = (const float4 *)(Q + (size_t)(B + j) * ldq);
        int best = 0;
        float bv = -INFINITY;
        for (int a4 = 0; a4 < (A + 3) / 4; ++a4) {   // pad columns of Q are never written: guard by A
            const float4 x = qn[a4];
            const float xs[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (a4 * 4 + e < A && (xs[e] > bv || (a4 == 0 && e == 0))) { bv = xs[e]; best = a4 * 4 + e; }
        }
        astar[j] = best;
        int aj = action[j];
        aj = aj < 0 ? 0 : (aj >= A ? A - 1 : aj);
        const float not_done = done[j] ? 0.f : 1.f;
        const float y = reward[j] + gamma * not_done * Q[(size_t)(2 * B + j) * ldq + best];
        float g;
        loss = huber_and_grad(Q[(size_t)j * ldq + aj] - y, kappa, B, &g);
        const T gz = TjElem<T>::from_f32(g), z0 = TjElem<T>::from_f32(0.f);
        for (int a = 0; a < A; ++a) {
            const T val = a == aj ? gz : z0;
            dZ[(size_t)j * lddz + a] = val;
            if (dZT) dZT[(size_t)a * lddzt + j] = val;   // null where the head's weight gradient reads dZ row-major
        }
    }
    // wave reduction in a fixed order
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) loss += __shfl_down(loss, off, 64);
    if (threadIdx.x == 0) loss_part[blockIdx.x] = loss;
}

// Epsilon-greedy action per observation from its Q row (Algorithm 1, step 1).  Two draws of the
// sampler's generator per observation: the top 24 bits of draw 2j against the threshold decide,
// draw 2j+1 scaled by mul-high picks the uniform action.
__global__ __launch_bounds__(256) void egreedy(const float *__restrict__ Q, int ldq, uint32_t n, int A,
                                               uint32_t threshold, uint64_t seed, int32_t version,
                                               int32_t *__restrict__ action, int32_t *__restrict__ version_out,
                                               float *__restrict__ q_out)
{
    const uint32_t j = blockIdx.x * 256 + threadIdx.x;
    if (j >= n) return;
    const float *q = Q + (size_t)j * ldq;
    int best = 0;
    float bv = q[0];
    if (q_out) q_out[(size_t)j * A] = bv;
    for (int a = 1; a < A; ++a) {
        const float x = q[a];
        if (q_out) q_out[(size_t)j * A + a] = x;
        if (x > bv) { bv = x; best = a; }
    }
    const uint64_t u = tj_splitmix64(seed, 2 * (uint64_t)j), v = tj_splitmix64(seed, 2 * (uint64_t)j + 1);
    action[j] = (uint32_t)(u >> 40) < threshold ? (int32_t)__umul64hi(v, (uint64_t)A) : best;
    version_out[j] = version;
}

inline uint32_t egreedy_threshold(float epsilon)
{
    const double scaled = (double)epsilon * 16777216.0;
    return scaled <= 0.0 ? 0u : (scaled >= 16777216.0 ? 16777216u : (uint32_t)scaled);
}

// Head layer and TD step in one kernel (bf16 compute type, at most 32 actions).  The head's
// forward is bound by reading its input rows once, so the three Q tiles of 32 transitions are
// computed by one block and consumed in place:
//   Q_on(s), Q_on(s'), Q_tg(s') = X W^T + b  for the block's rows  ->  Q (kept for inspection),
//   then the TD target, Huber loss and dL/dQ exactly as td_huber.
// 12 waves: 3 Q tiles x 4 interleaved quarters of the contraction.  Each wave streams its own
// 32 x 64-element operand pieces: whole 128-byte lines from global memory (8 lanes per row),
// through a wave-private, XOR-swizzled LDS slab, into the MFMA operand layout (lane (r, h)
// holds 8 consecutive k of row r); no block barrier in the loop.
typedef float headf32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 headbf16x8 __attribute__((ext_vector_type(8)));
typedef uint32_t headu32x4 __attribute__((ext_vector_type(4)));

constexpr int kHeadRows = 32;    // transitions per block
constexpr int kHeadSplit = 4;    // waves sharing one tile's contraction
constexpr int kHeadWaves = 3 * kHeadSplit;
constexpr int kHeadThreads = 64 * kHeadWaves;

struct HeadTdArgs {
    const tj_bf16 *X; int ldx;             // head input, rows row0[g] + j for tile g
    int row0[3];
    const tj_bf16 *W_on, *W_tg; int ldw;   // [A][ldw]
    const float *b_on, *b_tg;
    int B, A, K;
    float *Q; int ldq;                     // [3B][ldq]
    const int32_t *action; const float *reward; const uint8_t *done;
    float gamma, kappa;
    tj_bf16 *dZ; int lddz;                 // [B][lddz]
    tj_bf16 *dZT; int lddzt;               // [A][lddzt]; may be null (the head's weight gradient reads dZ row-major)
    int32_t *astar;
    float *loss_part;                      // one per block
    // optional: gradient wrt the head's input rows of s, dX[j][k] = relu'(X[j][k]) g_j W_on[a_j][k]
    // (dL/dQ has one non-zero per row, so this product needs no contraction)
    tj_bf16 *dX; int lddx;                 // [B][lddx]
    tj_bf16 *dXT; int lddxt;               // [Kin][lddxt]
    int Kin;                               // real (unpadded) width of the head's input
};

__device__ __forceinline__ void head_wave_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

__global__ __launch_bounds__(kHeadThreads) void head_td(const HeadTdArgs a)
{
    // per wave: 256 16-byte slots of X and 256 of W (32 rows x 8 pieces, piece p of row r in slot
    // 8 r + (p ^ (r & 7))); afterwards the same memory holds the waves' partial tiles
    __shared__ headu32x4 stage[kHeadWaves][2][256];
    __shared__ float qs[3][kHeadRows][33];
    __shared__ int s_aj[kHeadRows];
    __shared__ float s_g[kHeadRows];
    typedef float PartTile[kHeadRows][36];   // [transition][action]
    static_assert(sizeof(PartTile) * kHeadWaves <= sizeof(stage), "partial tiles must fit the staging slabs");
    PartTile *part = (PartTile *)&stage[0][0][0];

    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int grp = w / kHeadSplit, kq = w % kHeadSplit;
    const int r = lane & 31, h = lane >> 5;
    const int j0 = blockIdx.x * kHeadRows;
    const tj_bf16 *xbase = a.X + ((size_t)a.row0[grp] + j0) * a.ldx;
    const tj_bf16 *wbase = grp == 2 ? a.W_tg : a.W_on;
    const headu32x4 zero = {0u, 0u, 0u, 0u};
    const int lrow = lane >> 3, lpiece = lane & 7;   // loader role: row 8 t + lrow, 16-byte piece lpiece
    const int n_trip = (a.K + 63) / 64;
    headf32x16 acc = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    // two trips of loads stay in flight per wave (register sets 0 and 1)
    headu32x4 xr[2][4], wr[2][4];
    auto fetch = [&](int set, int trip) {
        const int k = trip * 64 + lpiece * 8;
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const int row = 8 * t + lrow;
            xr[set][t] = (k < a.K && j0 + row < a.B) ? *(const headu32x4 *)(xbase + (size_t)row * a.ldx + k) : zero;
            wr[set][t] = (k < a.K && row < a.A) ? *(const headu32x4 *)(wbase + (size_t)row * a.ldw + k) : zero;
        }
    };
    auto consume = [&](int set) {
        head_wave_sync();   // the last trip's operand reads precede these writes
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const int row = 8 * t + lrow, slot = 8 * row + (lpiece ^ (row & 7));
            stage[w][0][slot] = xr[set][t];
            stage[w][1][slot] = wr[set][t];
        }
        head_wave_sync();
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const int slot = 8 * r + ((2 * s + h) ^ (r & 7));
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(headbf16x8, stage[w][1][slot]),
                                                          __builtin_bit_cast(headbf16x8, stage[w][0][slot]), acc,
                                                          0, 0, 0);
        }
    };
    // fetches past the end of the contraction load nothing and contribute zeros
    fetch(0, kq);
    fetch(1, kq + kHeadSplit);
    for (int trip = kq; trip < n_trip; trip += 2 * kHeadSplit) {
        consume(0);
        fetch(0, trip + 2 * kHeadSplit);
        consume(1);
        fetch(1, trip + 3 * kHeadSplit);
    }
    __syncthreads();   // every wave is done with its slab before the partial tiles overwrite them
    // acc[4*q + e] = partial Q(transition r, action 8*q + 4*h + e)
#pragma unroll
    for (int q = 0; q < 4; ++q)
        *(float4 *)&part[w][r][8 * q + 4 * h] = make_float4(acc[4 * q], acc[4 * q + 1], acc[4 * q + 2], acc[4 * q + 3]);
    __syncthreads();
    for (int e = threadIdx.x; e < 3 * kHeadRows * 32; e += kHeadThreads) {
        const int g = e >> 10, j = (e >> 5) & 31, i = e & 31;
        float q = part[g * kHeadSplit][j][i];
#pragma unroll
        for (int s = 1; s < kHeadSplit; ++s) q += part[g * kHeadSplit + s][j][i];
        if (i < a.A) q += (g == 2 ? a.b_tg : a.b_on)[i];
        qs[g][j][i] = q;
        if (i < a.A && j0 + j < a.B) a.Q[((size_t)g * a.B + j0 + j) * a.ldq + i] = q;
    }
    __syncthreads();
    if (w == 0) {
        float loss = 0.f, g = 0.f;
        int aj = -1;
        const int j = j0 + lane;
        if (lane < kHeadRows && j < a.B) {
            int best = 0;
            float qrow[32];   // all 32 reads issue before the first comparison
#pragma unroll
            for (int i = 0; i < 32; ++i) qrow[i] = qs[1][lane][i];
            float bv = qrow[0];
#pragma unroll
            for (int i = 1; i < 32; ++i)
                if (i < a.A && qrow[i] > bv) { bv = qrow[i]; best = i; }
            a.astar[j] = best;
            aj = a.action[j];
            aj = aj < 0 ? 0 : (aj >= a.A ? a.A - 1 : aj);
            const float not_done = a.done[j] ? 0.f : 1.f;
            const float y = a.reward[j] + a.gamma * not_done * qs[2][lane][best];
            loss = huber_and_grad(qs[0][lane][aj] - y, a.kappa, a.B, &g);
        }
        if (lane < kHeadRows) { s_aj[lane] = aj; s_g[lane] = g; }
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) loss += __shfl_down(loss, off, 64);
        if (lane == 0) a.loss_part[blockIdx.x] = loss;
    }
    __syncthreads();
    // dL/dQ as whole 16-byte vectors: rows of dZ (pad columns up to the vector are zero), and the
    // block's 32 columns of dZ^T (columns past the batch, inside the pitch, are zero)
    const int nva = (a.A + 7) / 8;
    for (int e = threadIdx.x; e < kHeadRows * nva; e += kHeadThreads) {
        const int j = e / nva, vc = e % nva;
        if (j0 + j >= a.B) continue;
        const int aj = s_aj[j];
        const uint32_t gz = tj_f32_to_bf16(s_g[j]);
        headu32x4 o = zero;
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (aj == 8 * vc + 2 * u || aj == 8 * vc + 2 * u + 1) o[u] = gz << (16 * (aj & 1));
        *(headu32x4 *)(a.dZ + (size_t)(j0 + j) * a.lddz + 8 * vc) = o;
    }
    for (int e = threadIdx.x; a.dZT && e < a.A * (kHeadRows / 8); e += kHeadThreads) {
        const int arow = e >> 2, vc = e & 3;
        if (j0 + 8 * vc >= a.lddzt) continue;
        headu32x4 o = zero;
#pragma unroll
        for (int u = 0; u < 8; ++u)
            if (s_aj[8 * vc + u] == arow) o[u >> 1] |= (uint32_t)tj_f32_to_bf16(s_g[8 * vc + u]) << (16 * (u & 1));
        *(headu32x4 *)(a.dZT + (size_t)arow * a.lddzt + j0 + 8 * vc) = o;
    }
    if (!a.dX) return;
    // Input gradient of the head layer for the block's 32 transitions, in chunks of 256 columns:
    // product of the bf16 gradient and the bf16 weight in fp32 (exact), ReLU mask from the
    // activation, rounded to bf16: what the contraction over the actions would give.  Rows go out
    // as 16-byte vectors; the transposed copy leaves through an LDS tile [column][transition].
    constexpr int kChunk = 256, kPitch = kHeadRows + 8;   // 80-byte rows: 16-byte aligned, spread over the banks
    tj_bf16 *tile = (tj_bf16 *)&stage[0][0][0];
    static_assert(kChunk * kPitch * 2 <= (int)sizeof(stage), "transpose tile must fit the staging slabs");
    const bool want_t = a.dXT != nullptr;   // block-uniform
    if (!want_t) {
        // rows only: every thread takes up to kInFlight vectors of the 32 x K block and issues all their
        // loads before the first product, so the block makes one round trip to memory per pass
        constexpr int kInFlight = 6;
        const int nvec = a.K / 8, total = kHeadRows * nvec;
        for (int base = threadIdx.x; base < total; base += kInFlight * kHeadThreads) {
            headu32x4 x[kInFlight], wv[kInFlight];
#pragma unroll
            for (int u = 0; u < kInFlight; ++u) {
                const int e = base + u * kHeadThreads, j = e / nvec, k = (e % nvec) * 8;
                const int aj = e < total ? s_aj[j] : -1;
                x[u] = wv[u] = zero;
                if (aj >= 0) {
                    x[u] = *(const headu32x4 *)(a.X + ((size_t)a.row0[0] + j0 + j) * a.ldx + k);
                    wv[u] = *(const headu32x4 *)(a.W_on + (size_t)aj * a.ldw + k);
                }
            }
#pragma unroll
            for (int u = 0; u < kInFlight; ++u) {
                const int e = base + u * kHeadThreads, j = e / nvec, k = (e % nvec) * 8;
                if (e >= total || j0 + j >= a.B) continue;
                const float g = tj_bf16_to_f32(tj_f32_to_bf16(s_g[j]));
                headu32x4 o;
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    const uint32_t xl = x[u][c] & 0xFFFFu, xh = x[u][c] >> 16;
                    const float pl = g * __uint_as_float(wv[u][c] << 16), ph = g * __uint_as_float(wv[u][c] & 0xFFFF0000u);
                    const uint32_t lo = (int16_t)xl > 0 ? tj_f32_to_bf16(pl) : 0u;
                    const uint32_t hi = (int16_t)xh > 0 ? tj_f32_to_bf16(ph) : 0u;
                    o[c] = lo | (hi << 16);
                }
                *(headu32x4 *)(a.dX + (size_t)(j0 + j) * a.lddx + k) = o;
            }
        }
        return;
    }
    for (int k0 = 0; k0 < a.K; k0 += kChunk) {
        if (want_t) __syncthreads();   // the partial tiles (first pass) or the previous chunk's tile have been read
        for (int e = threadIdx.x; e < kHeadRows * (kChunk / 8); e += kHeadThreads) {
            const int j = e / (kChunk / 8), k = k0 + (e % (kChunk / 8)) * 8;
            headu32x4 o = zero;
            const int aj = s_aj[j];
            if (k < a.K && aj >= 0) {
                const headu32x4 x = *(const headu32x4 *)(a.X + ((size_t)a.row0[0] + j0 + j) * a.ldx + k);
                const headu32x4 w = *(const headu32x4 *)(a.W_on + (size_t)aj * a.ldw + k);
                const float g = tj_bf16_to_f32(tj_f32_to_bf16(s_g[j]));
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const uint32_t xl = x[u] & 0xFFFFu, xh = x[u] >> 16;
                    const float pl = g * __uint_as_float(w[u] << 16), ph = g * __uint_as_float(w[u] & 0xFFFF0000u);
                    const uint32_t lo = (int16_t)xl > 0 ? tj_f32_to_bf16(pl) : 0u;
                    const uint32_t hi = (int16_t)xh > 0 ? tj_f32_to_bf16(ph) : 0u;
                    o[u] = lo | (hi << 16);
                }
            }
            if (k < a.K && j0 + j < a.B) *(headu32x4 *)(a.dX + (size_t)(j0 + j) * a.lddx + k) = o;
            if (want_t) {
#pragma unroll
                for (int u = 0; u < 8; ++u)
                    tile[(k - k0 + u) * kPitch + j] = (tj_bf16)((o[u >> 1] >> (16 * (u & 1))) & 0xFFFFu);
            }
        }
        if (!want_t) continue;
        __syncthreads();
        for (int e = threadIdx.x; e < kChunk * (kHeadRows / 8); e += kHeadThreads) {
            const int k = k0 + (e >> 2), vc = e & 3;
            if (k >= a.Kin || j0 + 8 * vc >= a.lddxt) continue;   // columns past the batch, inside the pitch, are zero
            *(headu32x4 *)(a.dXT + (size_t)k * a.lddxt + j0 + 8 * vc) = *(const headu32x4 *)(tile + (k - k0) * kPitch + 8 * vc);
        }
    }
}

// Streaming (nontemporal) 16-byte accesses: optimizer state and gradient slices are touched once
// per step and are larger than L2, so they should not displace the GEMM operands there.
typedef float f32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ float4 ld4_stream(const float *p)
{
    const f32x4_t v = __builtin_nontemporal_load((const f32x4_t *)p);
    return make_float4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void st4_stream(float *p, float a, float b, float c, float d)
{
    const f32x4_t v = {a, b, c, d};
    __builtin_nontemporal_store(v, (f32x4_t *)p);
}

// Where Adam also writes the compute-type copy of a weight block: flat parameters [begin, end)
// go to dst[0 .. end-begin) (only blocks whose copy has no row padding).
template <typename T> struct EmitTable {
    int n;
    size_t begin[TJ_MAX_LAYERS], end[TJ_MAX_LAYERS];
    T *dst[TJ_MAX_LAYERS];
    // optional transposed copy of a small layer ([C][ldT], element (o, k) of the [O][C] block at k * ldT + o)
    T *dstT[TJ_MAX_LAYERS];
    int C[TJ_MAX_LAYERS], ldT[TJ_MAX_LAYERS];
};

template <typename T>
__device__ __forceinline__ void emit_transposed(const EmitTable<T> &tab, int k, size_t e, float th)
{
    if (!tab.dstT[k] || e < tab.begin[k] || e >= tab.end[k]) return;
    const size_t idx = e - tab.begin[k];
    const int o = (int)(idx / (size_t)tab.C[k]), kk = (int)(idx % (size_t)tab.C[k]);
    tab.dstT[k][(size_t)kk * tab.ldT[k] + o] = TjElem<T>::from_f32(th);
}

// Convolution weights whose input-gradient matrix the optimizer refreshes as it updates them:
// Wd[(py, px, c)][(a, b, o)] = W[o][kh][kw][c] with kh = py + (A-1-a) s, kw = px + (A-1-b) s (the layout
// tjconv::dgrad_weights builds; entries with kh or kw beyond the kernel are zero and never written here).
struct DgradEmit {
    int n;
    size_t begin[TJ_MAX_LAYERS], end[TJ_MAX_LAYERS];   // flat parameter range of the layer's weights
    tj_bf16 *wd[TJ_MAX_LAYERS];
    int O[TJ_MAX_LAYERS], C[TJ_MAX_LAYERS], k[TJ_MAX_LAYERS], s[TJ_MAX_LAYERS], A[TJ_MAX_LAYERS];
};

__device__ __forceinline__ void emit_dgrad(const DgradEmit &dg, size_t e, float th)
{
    for (int q = 0; q < dg.n; ++q) {
        if (e < dg.begin[q] || e >= dg.end[q]) continue;
        const int O = dg.O[q], C = dg.C[q], k = dg.k[q], s = dg.s[q], A = dg.A[q];
        const int idx = (int)(e - dg.begin[q]), kkc = k * k * C;
        const int o = idx / kkc, r = idx - o * kkc;
        const int kh = r / (k * C), kw = (r / C) % k, c = r % C;
        const int py = kh % s, a = A - 1 - kh / s, px = kw % s, b = A - 1 - kw / s;
        const size_t j = (size_t)(py * s + px) * C + c, col = (size_t)(a * A + b) * O + o;
        dg.wd[q][j * ((size_t)A * A * O) + col] = tj_f32_to_bf16(th);
    }
}

template <typename T> __device__ __forceinline__ void emit4(T *dst, const float (&x)[4]);
template <> __device__ __forceinline__ void emit4<float>(float *dst, const float (&x)[4])
{
    *(float4 *)dst = make_float4(x[0], x[1], x[2], x[3]);
}
template <> __device__ __forceinline__ void emit4<tj_bf16>(tj_bf16 *dst, const float (&x)[4])
{
    uint2 o;
    o.x = (uint32_t)tj_f32_to_bf16(x[0]) | ((uint32_t)tj_f32_to_bf16(x[1]) << 16);
    o.y = (uint32_t)tj_f32_to_bf16(x[2]) | ((uint32_t)tj_f32_to_bf16(x[3]) << 16);
    *(uint2 *)dst = o;
}

// The step's loss: the TD kernel's per-block sums, added in a fixed order (strided per lane,
// then one shuffle tree) by the first wave of the optimizer kernel, which runs after every
// TD block has finished.
struct LossFinal {
    const float *part;
    int n_part, B;
    uint32_t t_next;
    tj_step_stats *out, *internal;   // out: caller's (may be null)
    // on-policy update: per-block sums of the three terms (four floats per block) instead, finalised the same way
    const float *ppo_part = nullptr;
    int ppo_n_part = 0;
    float c_v = 0.f, c_e = 0.f;
    tj_ppo_stats *ppo_out = nullptr, *ppo_internal = nullptr;
};

// Adam on the flat fp32 master state (bias-corrected, eps outside the square root); the gradient
// is the sum of S slices (split batch contraction of the weight-gradient GEMMs), added in slice
// order and written back to slice 0.  The parameters [mid_begin, mid_end) (multiples of 4; a
// network's hidden layers) have S_mid slices instead: 1 where an earlier launch has done that sum
// already and slice 0 is the gradient.  Also emits the compute-type copy of the weights: with one
// slice 16 B read and 12 B + sizeof(T) written per parameter.
template <typename T>
__global__ __launch_bounds__(256) void adam_update(float *__restrict__ theta, float *__restrict__ m,
                                                   float *__restrict__ v, float *__restrict__ gpart,
                                                   int S, size_t gstride, size_t P, float lr, float b1,
                                                   float b2, float eps, float c1, float c2,
                                                   const EmitTable<T> tab, const LossFinal lf, const DgradEmit dg,
                                                   const size_t mid_begin, const size_t mid_end, const int S_mid)
{
    if (blockIdx.x == 0 && threadIdx.x < 64 && lf.ppo_part) {
        // means of the three terms and the objective, from the per-block sums (fixed order)
        float s[3] = {0.f, 0.f, 0.f};
        for (int b = threadIdx.x; b < lf.ppo_n_part; b += 64)
            for (int q = 0; q < 3; ++q) s[q] += lf.ppo_part[(size_t)b * 4 + q];
#pragma unroll
        for (int q = 0; q < 3; ++q)
#pragma unroll
            for (int off = 32; off > 0; off >>= 1) s[q] += __shfl_down(s[q], off, 64);
        if (threadIdx.x == 0) {
            tj_ppo_stats o;
            o.loss_pi = s[0] / (float)lf.B;
            o.loss_v = s[1] / (float)lf.B;
            o.entropy = s[2] / (float)lf.B;
            o.loss = o.loss_pi + lf.c_v * o.loss_v - lf.c_e * o.entropy;
            o.step = lf.t_next;
            *lf.ppo_internal = o;
            if (lf.ppo_out) *lf.ppo_out = o;
        }
    } else if (blockIdx.x == 0 && threadIdx.x < 64) {
        float s = 0.f;
        for (int b = threadIdx.x; b < lf.n_part; b += 64) s += lf.part[b];
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) s += __shfl_down(s, off, 64);
        if (threadIdx.x == 0) {
            tj_step_stats o;
            o.loss = s / (float)lf.B;
            o.step = lf.t_next;
            *lf.internal = o;
            if (lf.out) *lf.out = o;
        }
    }
    const size_t i = ((size_t)blockIdx.x * 256 + threadIdx.x) * 4;
    if (i >= P) return;
    if (i + 4 <= P) {
        float4 g = ld4_stream(gpart + i);
        float4 mm = ld4_stream(m + i), vv = ld4_stream(v + i), th = ld4_stream(theta + i);
        const int Sv = (i >= mid_begin && i < mid_end) ? S_mid : S;
        if (Sv > 1) {   // slices are added in slice order, eight loads in flight at a time
            float4 p[8];
            for (int s0 = 1; s0 < Sv; s0 += 8) {
#pragma unroll
                for (int u = 0; u < 8; ++u)
                    if (s0 + u < Sv) p[u] = ld4_stream(gpart + (size_t)(s0 + u) * gstride + i);
#pragma unroll
                for (int u = 0; u < 8; ++u)
                    if (s0 + u < Sv) { g.x += p[u].x; g.y += p[u].y; g.z += p[u].z; g.w += p[u].w; }
            }
            *(float4 *)(gpart + i) = g;   // slice 0 keeps the step's gradient
        }
        float ga[4] = {g.x, g.y, g.z, g.w}, ma[4] = {mm.x, mm.y, mm.z, mm.w};
        float va[4] = {vv.x, vv.y, vv.z, vv.w}, ta[4] = {th.x, th.y, th.z, th.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            ma[e] = b1 * ma[e] + (1.f - b1) * ga[e];
            va[e] = b2 * va[e] + (1.f - b2) * ga[e] * ga[e];
            ta[e] -= lr * (ma[e] / c1) / (sqrtf(va[e] / c2) + eps);
        }
        st4_stream(m + i, ma[0], ma[1], ma[2], ma[3]);
        st4_stream(v + i, va[0], va[1], va[2], va[3]);
        st4_stream(theta + i, ta[0], ta[1], ta[2], ta[3]);
        for (int k = 0; k < tab.n; ++k) {
            if (i + 4 <= tab.begin[k] || i >= tab.end[k]) continue;
            if (i >= tab.begin[k] && i + 4 <= tab.end[k] && ((i - tab.begin[k]) & 3) == 0) {
                emit4<T>(tab.dst[k] + (i - tab.begin[k]), ta);
            } else {
                for (int e = 0; e < 4; ++e)
                    if (i + e >= tab.begin[k] && i + e < tab.end[k])
                        tab.dst[k][i + e - tab.begin[k]] = TjElem<T>::from_f32(ta[e]);
            }
#pragma unroll
            for (int e = 0; e < 4; ++e) emit_transposed<T>(tab, k, i + e, ta[e]);
        }
        if (dg.n > 0) {
#pragma unroll
            for (int e = 0; e < 4; ++e) emit_dgrad(dg, i + e, ta[e]);
        }
    } else {
        for (size_t e = i; e < P; ++e) {
            float g = gpart[e];
            const int Se = (e >= mid_begin && e < mid_end) ? S_mid : S;
            for (int s = 1; s < Se; ++s) g += gpart[(size_t)s * gstride + e];
            if (Se > 1) gpart[e] = g;
            const float mm = b1 * m[e] + (1.f - b1) * g;
            const float vv = b2 * v[e] + (1.f - b2) * g * g;
            m[e] = mm;
            v[e] = vv;
            const float th = theta[e] - lr * (mm / c1) / (sqrtf(vv / c2) + eps);
            theta[e] = th;
            for (int k = 0; k < tab.n; ++k) {
                if (e >= tab.begin[k] && e < tab.end[k]) tab.dst[k][e - tab.begin[k]] = TjElem<T>::from_f32(th);
                emit_transposed<T>(tab, k, e, th);
            }
            emit_dgrad(dg, e, th);
        }
    }
}

// ---------------------------------------------------------------- on-policy workload
//
// The PPO column of the paper's hyperparameter table (gamma 0.99, GAE 0.95, rollouts of 512
// steps, batch = buffer, Adam eps 1e-5).  The estimator is GAE (Schulman et al. 2016, Eq. 16),
// the objective the clipped surrogate with value and entropy terms (Schulman et al. 2017,
// Eq. 7 and 9).

// Advantages of one rollout per wave.  A_t = delta_t + c_t A_{t+1} is a chain of affine maps
// x -> D + C x, which compose associatively: a lane folds its 8 consecutive steps into one map,
// a suffix scan over the lanes (shuffles) gives every lane the advantage that enters its run, and
// the lane then replays its 8 steps.  Chunks of 512 steps, last chunk first, carry A across.
__global__ __launch_bounds__(256) void gae_scan(uint32_t n_env, uint32_t T, const float *__restrict__ reward,
                                                const float *__restrict__ value,
                                                const uint8_t *__restrict__ done, float gamma, float lam,
                                                float *__restrict__ adv, float *__restrict__ ret)
{
    const uint32_t env = blockIdx.x * 4 + (threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    if (env >= n_env) return;
    const float *r = reward + (size_t)env * T, *v = value + (size_t)env * ((size_t)T + 1);
    const uint8_t *dn = done + (size_t)env * T;
    float *ao = adv + (size_t)env * T, *ro = ret + (size_t)env * T;
    float carry = 0.f;   // A at the first step of the chunk after this one (A_T = 0)
    for (int64_t end = T; end > 0; end -= 512) {
        const int64_t t0 = end - 512 + 8 * lane;
        float dl[8], c[8], v0[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int64_t t = t0 + e;
            if (t >= 0) {
                const float nd = dn[t] ? 0.f : 1.f;
                v0[e] = v[t];
                dl[e] = r[t] + gamma * v[t + 1] * nd - v0[e];
                c[e] = gamma * lam * nd;
            } else {   // before the rollout: the identity map
                v0[e] = 0.f; dl[e] = 0.f; c[e] = 1.f;
            }
        }
        float C = 1.f, D = 0.f;
#pragma unroll
        for (int e = 7; e >= 0; --e) { D = dl[e] + c[e] * D; C = c[e] * C; }
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {   // (C, D) of lanes [lane, lane + 2 off)
            const float C2 = __shfl_down(C, off, 64), D2 = __shfl_down(D, off, 64);
            if (lane + off < 64) { D = D + C * D2; C = C * C2; }
        }
        const float a_first = D + C * carry;       // A at this lane's first step
        float a = __shfl_down(a_first, 1, 64);     // A entering from the lane above
        if (lane == 63) a = carry;
#pragma unroll
        for (int e = 7; e >= 0; --e) {
            a = dl[e] + c[e] * a;
            const int64_t t = t0 + e;
            if (t >= 0) { ao[t] = a; ro[t] = a + v0[e]; }
        }
        carry = __shfl(a_first, 0, 64);
    }
}

// Clipped actor-critic objective on the head's output Z[j] = (logits z_0..z_{A-1}, value):
//   p = softmax(z), rho = p[a_j] / exp(old_logp_j), H = -sum p log p
//   loss_j = -min(rho Adv, clip(rho, 1-c, 1+c) Adv) + c_v (V - ret)^2 - c_e H
// Writes d(mean loss)/dZ in compute type, row-major and transposed (the two operand layouts of
// the backward GEMMs), and per-block sums of the three terms.  Eight lanes per sample; both
// copies of the gradient leave through an LDS tile (whole 16-byte vectors row-major, 32
// consecutive samples per head output transposed).
template <typename T> struct PpoHeadArgs {
    const float *Z; int ldz; int B, A;
    const int32_t *action; const float *old_logp, *adv, *ret;
    float clip, c_v, c_e;
    T *dZ; int lddz; T *dZT; int lddzt;   // dZT may be null (the head's weight gradient reads dZ row-major)
    float *part;   // [blocks][4]: sum L_pi, sum L_v, sum H, unused
};

constexpr int kPpoRows = 32;    // samples per block of ppo_head
constexpr int kPpoLanes = 8;    // lanes per sample: lane g owns head outputs g, g + 8, ...

// The objective for the block's 32 samples; `z` = this thread's sample's head outputs (global memory
// or LDS), read only where the sample exists.
constexpr int kPpoTileElems = kPpoRows * (64 + 8);   // A + 1 <= 64 columns, plus one 16-byte vector per row (bf16: 8 elements)
template <typename T> __device__ __forceinline__ int ppo_tile_cols(int A) { return (A + 1 + 16 / (int)sizeof(T) - 1) / (16 / (int)sizeof(T)) * (16 / (int)sizeof(T)); }

// `tile` ([kPpoRows][cols + one vector], kPpoTileElems elements) receives the block's gradient rows, zero
// in the pad columns (bf16: up to the next multiple of 16); `red` is scratch for the block sums.
template <typename T>
__device__ __forceinline__ void ppo_objective(const PpoHeadArgs<T> &a, const float *z, T *tile,
                                              float (*red)[3])
{
    constexpr int VEC = 16 / (int)sizeof(T);
    constexpr int NI = 64 / kPpoLanes;               // head outputs per lane, at most
    const int cols = ppo_tile_cols<T>(a.A);            // row-major columns written per sample (<= lddz)
    const int pitch = cols + VEC;                      // odd number of vectors: rows spread over the banks
    // bf16: the fused head kernel contracts over the columns in steps of 16 (cols + 8 >= the next multiple of 16)
    const int cols16 = sizeof(T) == 2 ? (cols + 15) / 16 * 16 : cols;
    const int row0 = blockIdx.x * kPpoRows;
    const int r = threadIdx.x / kPpoLanes, g = threadIdx.x % kPpoLanes;
    const int j = row0 + r;
    // sums over the lanes of one sample (8 consecutive lanes of a wave)
    auto group_sum = [](float v) {
        v += __shfl_xor(v, 1, 64); v += __shfl_xor(v, 2, 64); v += __shfl_xor(v, 4, 64);
        return v;
    };
    float l_pi = 0.f, l_v = 0.f, H = 0.f;
    if (j < a.B) {   // uniform over a sample's lanes
        float zv[NI];
        float mx = -INFINITY;
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            const int k = g + kPpoLanes * i;
            zv[i] = k < a.A ? z[k] : -INFINITY;
            mx = fmaxf(mx, zv[i]);
        }
        mx = fmaxf(mx, __shfl_xor(mx, 1, 64)); mx = fmaxf(mx, __shfl_xor(mx, 2, 64)); mx = fmaxf(mx, __shfl_xor(mx, 4, 64));
        float se = 0.f;
#pragma unroll
        for (int i = 0; i < NI; ++i)
            if (g + kPpoLanes * i < a.A) se += expf(zv[i] - mx);
        const float lse = mx + logf(group_sum(se));
        float h = 0.f;
#pragma unroll
        for (int i = 0; i < NI; ++i)
            if (g + kPpoLanes * i < a.A) h -= expf(zv[i] - lse) * (zv[i] - lse);
        H = group_sum(h);
        const int act = min(max(a.action[j], 0), a.A - 1);
        const float adv = a.adv[j];
        const float rho = expf(z[act] - lse - a.old_logp[j]);
        const float rc = fminf(fmaxf(rho, 1.f - a.clip), 1.f + a.clip);
        const float s1 = rho * adv, s2 = rc * adv;
        const bool unclipped = s1 <= s2;   // the minimum is the unclipped term: it carries the gradient
        const float verr = z[a.A] - a.ret[j];
        l_pi = -(unclipped ? s1 : s2);
        l_v = verr * verr;
        const float inv_b = 1.f / (float)a.B;
        T *row = tile + r * pitch;
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            const int k = g + kPpoLanes * i;
            if (k < a.A) {
                const float lp = zv[i] - lse, pk = expf(lp);
                float gr = a.c_e * pk * (lp + H);
                if (unclipped) gr -= adv * rho * ((k == act ? 1.f : 0.f) - pk);
                row[k] = TjElem<T>::from_f32(gr * inv_b);
            } else if (k == a.A) {
                row[k] = TjElem<T>::from_f32(2.f * a.c_v * verr * inv_b);
            } else if (k < cols16) {
                row[k] = TjElem<T>::from_f32(0.f);
            }
        }
        if (g != 0) { l_pi = 0.f; l_v = 0.f; H = 0.f; }   // one lane per sample carries its terms
    }
    // block sums in a fixed order: shuffle tree per wave, then the waves in turn
    float s[3] = {l_pi, l_v, H};
#pragma unroll
    for (int q = 0; q < 3; ++q)
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) s[q] += __shfl_down(s[q], off, 64);
    if ((threadIdx.x & 63) == 0)
        for (int q = 0; q < 3; ++q) red[threadIdx.x >> 6][q] = s[q];
    __syncthreads();
    if (threadIdx.x < 3) {
        float t = red[0][threadIdx.x];
        for (int w = 1; w < kPpoRows * kPpoLanes / 64; ++w) t += red[w][threadIdx.x];
        a.part[(size_t)blockIdx.x * 4 + threadIdx.x] = t;
    }
    const int n_rows = min(kPpoRows, a.B - row0);
    // row-major gradient: whole 16-byte vectors, consecutive lanes on consecutive vectors of a row
    const int vpr = cols / VEC;
    for (int v = threadIdx.x; v < n_rows * vpr; v += kPpoRows * kPpoLanes) {
        const int rr = v / vpr, c = v - rr * vpr;
        *(uint4 *)(a.dZ + (size_t)(row0 + rr) * a.lddz + c * VEC) = *(const uint4 *)(tile + rr * pitch + c * VEC);
    }
    // transposed gradient: 32 consecutive samples of one head output per 32 lanes
    for (int e = threadIdx.x; a.dZT && e < (a.A + 1) * kPpoRows; e += kPpoRows * kPpoLanes) {
        const int k = e / kPpoRows, rr = e % kPpoRows;
        if (rr < n_rows) a.dZT[(size_t)k * a.lddzt + row0 + rr] = tile[rr * pitch + k];
    }
}

template <typename T>
__global__ __launch_bounds__(kPpoRows * kPpoLanes) void ppo_head(const PpoHeadArgs<T> a)
{
    __shared__ __align__(16) T tile[kPpoTileElems];
    __shared__ float red[kPpoRows * kPpoLanes / 64][3];
    const size_t j = (size_t)blockIdx.x * kPpoRows + threadIdx.x / kPpoLanes;
    ppo_objective<T>(a, a.Z + j * a.ldz, tile, red);
}

// The head layer's forward and the objective in one kernel (bf16, at most 32 head outputs): the
// contraction of the Q-learner's fused head kernel for one tile of 32 samples (4 waves split it, each
// streaming its own operand pieces through a wave-private swizzled LDS slab), then the objective on
// the head outputs where they lie in LDS.  The outputs are also written to Z (fp32), as the head GEMM
// would have left them.
constexpr int kPpoFusedMaxK = 1024;   // widest head input whose input gradient the fused kernel takes
struct PpoFusedArgs {
    PpoHeadArgs<tj_bf16> h;            // h.Z: destination of the head outputs
    const tj_bf16 *X; int ldx;         // head input [B][ldx]
    const tj_bf16 *W; int ldw;         // [A + 1][ldw]
    const float *bias;
    int K;
    // optional: the head's input gradient dX[j][k] = relu'(X[j][k]) sum_o dZ[j][o] W[o][k], from the
    // transposed weight copy WT [K][ldwt] (pad columns zero, ldwt >= the head outputs rounded up to 16);
    // needs K % 32 == 0
    const tj_bf16 *WT; int ldwt;
    tj_bf16 *dX; int lddx;
};

__global__ __launch_bounds__(kPpoRows * kPpoLanes) __attribute__((amdgpu_waves_per_eu(4, 4)))
void ppo_head_fused(const PpoFusedArgs a)
{
    // at most 32 head outputs: gradient rows of 32 columns plus one vector
    __shared__ __align__(16) tj_bf16 tile[kPpoRows * 40];
    __shared__ float red[kPpoRows * kPpoLanes / 64][3];
    constexpr int NW = kPpoRows * kPpoLanes / 64;   // 4 waves
    // 32 KiB of slabs, 35 KB per block in all: four blocks per CU, so that 32768 samples are one round.
    // During the contraction: per wave 256 16-byte slots of X and 256 of W.  Afterwards: the waves' partial
    // tiles [0, 18 K), the summed head outputs behind them, the sign bits of the head's input (one byte
    // per 8 columns, the input gradient's ReLU mask) at 24 K; last, per wave 4 KiB of gradient rows at 0.
    __shared__ headu32x4 stage[NW][2][256];
    typedef float PartTile[kPpoRows][36];
    typedef float OutTile[kPpoRows][33];
    constexpr int kMaskAt = 24576, kMaskPitch = kPpoFusedMaxK / 8;
    static_assert(sizeof(PartTile) * NW + sizeof(OutTile) <= kMaskAt, "partial and output tiles end before the mask bytes");
    static_assert(kMaskAt + kPpoRows * kMaskPitch <= (int)sizeof(stage) && NW * 4096 <= kMaskAt, "mask bytes and row slabs fit");
    PartTile *part = (PartTile *)&stage[0][0][0];
    OutTile &zs = *(OutTile *)((uint8_t *)&stage[0][0][0] + sizeof(PartTile) * NW);
    uint8_t *xmask = (uint8_t *)&stage[0][0][0] + kMaskAt;
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int r = lane & 31, h = lane >> 5;
    const int j0 = blockIdx.x * kPpoRows, n_out = a.h.A + 1;
    const tj_bf16 *xbase = a.X + (size_t)j0 * a.ldx;
    const headu32x4 zero = {0u, 0u, 0u, 0u};
    const int lrow = lane >> 3, lpiece = lane & 7;   // loader role: row 8 t + lrow, 16-byte piece lpiece
    const int n_trip = (a.K + 63) / 64;
    const bool keep_mask = a.dX != nullptr;           // then K <= kPpoFusedMaxK: at most 4 trips per wave
    uint32_t mreg[4] = {0u, 0u, 0u, 0u};              // sign bits of this lane's operand pieces: byte s of word (trip - w) / NW
    headf32x16 acc = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    headu32x4 xr[2][4], wr[2][4];   // two trips of loads stay in flight per wave
    // block-uniform bases + 32-bit byte offsets per lane (a tile's rows span well under 4 GiB)
    const uint8_t *xb = (const uint8_t *)xbase, *wb = (const uint8_t *)a.W;
    auto fetch = [&](int set, int trip) {
        const int k = trip * 64 + lpiece * 8;
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const int row = 8 * t + lrow;
            const uint32_t xo = (uint32_t)(row * a.ldx + k) * 2u, wo = (uint32_t)(row * a.ldw + k) * 2u;
            xr[set][t] = (k < a.K && j0 + row < a.h.B) ? *(const headu32x4 *)(xb + xo) : zero;
            wr[set][t] = (k < a.K && row < n_out) ? *(const headu32x4 *)(wb + wo) : zero;
        }
    };
    auto consume = [&](int set, int trip) {
        head_wave_sync();   // the last trip's operand reads precede these writes
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const int row = 8 * t + lrow, slot = 8 * row + (lpiece ^ (row & 7));
            stage[w][0][slot] = xr[set][t];
            stage[w][1][slot] = wr[set][t];
        }
        head_wave_sync();
        uint32_t word = 0;
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const int slot = 8 * r + ((2 * s + h) ^ (r & 7));
            const headu32x4 xv = stage[w][0][slot];   // columns 64 trip + 8 (2s + h) .. + 7 of sample r
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(headbf16x8, stage[w][1][slot]),
                                                          __builtin_bit_cast(headbf16x8, xv), acc, 0, 0, 0);
            if (keep_mask) {   // bit e of byte s: element e of this piece is positive
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    word |= ((int16_t)(xv[u] & 0xFFFFu) > 0 ? 1u : 0u) << (8 * s + 2 * u);
                    word |= ((int16_t)(xv[u] >> 16) > 0 ? 1u : 0u) << (8 * s + 2 * u + 1);
                }
            }
        }
        if (keep_mask) {
            const int i = (trip - w) / NW;
#pragma unroll
            for (int q = 0; q < 4; ++q) mreg[q] = i == q ? word : mreg[q];
        }
    };
    fetch(0, w);
    fetch(1, w + NW);
    for (int trip = w; trip < n_trip; trip += 2 * NW) {
        consume(0, trip);
        fetch(0, trip + 2 * NW);
        consume(1, trip + NW);
        fetch(1, trip + 3 * NW);
    }
    __syncthreads();   // every wave is done with its slab before the partial tiles overwrite them
    // acc[4*q + e] = partial output 8*q + 4*h + e of sample r
#pragma unroll
    for (int q = 0; q < 4; ++q)
        *(float4 *)&part[w][r][8 * q + 4 * h] = make_float4(acc[4 * q], acc[4 * q + 1], acc[4 * q + 2], acc[4 * q + 3]);
    if (keep_mask) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int trip = w + NW * i;
            if (trip >= n_trip) continue;
#pragma unroll
            for (int sp = 0; sp < 4; ++sp) xmask[r * kMaskPitch + trip * 8 + 2 * sp + h] = (uint8_t)(mreg[i] >> (8 * sp));
        }
    }
    __syncthreads();
    for (int e = threadIdx.x; e < kPpoRows * 32; e += kPpoRows * kPpoLanes) {
        const int j = e >> 5, i = e & 31;
        float z = part[0][j][i];
#pragma unroll
        for (int s = 1; s < NW; ++s) z += part[s][j][i];
        if (i < n_out) z += a.bias[i];
        zs[j][i] = z;
        if (i < n_out && j0 + j < a.h.B) const_cast<float *>(a.h.Z)[(size_t)(j0 + j) * a.h.ldz + i] = z;
    }
    __syncthreads();
    ppo_objective<tj_bf16>(a.h, &zs[threadIdx.x / kPpoLanes][0], tile, red);
    if (!a.dX) return;   // block-uniform

    // ---- input gradient of the head layer for the block's 32 samples.  Per 32 columns k one MFMA tile
    // D(k, sample) = sum_o WT[k][o] dZ[sample][o] (one or two 16-wide steps over the head outputs); a
    // wave takes pairs of such tiles, stages them as [sample][64 columns] in its slab (vector v of row r
    // at v ^ (r & 7)) and writes rows of 128 bytes, masked with the sign bits kept from the contraction.
    __syncthreads();     // the partial tiles and head outputs have been read: the slabs are free again
    const int cols = ppo_tile_cols<tj_bf16>(a.h.A), pitch = cols + 8, nks = (cols + 15) / 16;
    headu32x4 dz[2];
#pragma unroll
    for (int ks = 0; ks < 2; ++ks)
        dz[ks] = ks < nks ? *(const headu32x4 *)(tile + r * pitch + 8 * h + 16 * ks) : zero;
    uint8_t *slab = (uint8_t *)&stage[0][0][0] + w * 4096;
    const int n_chunk = a.K / 32, n_group = (n_chunk + 1) / 2;
    for (int gi = w; gi < n_group; gi += NW) {
        const int c_begin = 2 * gi, c_n = min(2, n_chunk - c_begin);
        // the group's weight pieces first, all loads in flight together (a tile past the end repeats the last one)
        headu32x4 wv[2][2];
#pragma unroll
        for (int c = 0; c < 2; ++c) {
            const int k0 = min(c_begin + c, n_chunk - 1) * 32;
#pragma unroll
            for (int ks = 0; ks < 2; ++ks)
                wv[c][ks] = ks < nks ? *(const headu32x4 *)((const uint8_t *)a.WT +
                                                             (uint32_t)((k0 + r) * a.ldwt + 8 * h + 16 * ks) * 2u)
                                     : zero;
        }
        head_wave_sync();   // the last group's rows have been read out of the slab
#pragma unroll
        for (int c = 0; c < 2; ++c) {
            if (c >= c_n) break;
            headf32x16 d = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < 2; ++ks) {
                if (ks < nks)
                    d = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(headbf16x8, wv[c][ks]),
                                                                __builtin_bit_cast(headbf16x8, dz[ks]), d, 0, 0, 0);
            }
            // d[4q + e] = dX(sample r, column 32 (c_begin + c) + 8q + 4h + e), before the mask
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const uint32_t lo = (uint32_t)tj_f32_to_bf16(d[4 * q]) | ((uint32_t)tj_f32_to_bf16(d[4 * q + 1]) << 16);
                const uint32_t hi = (uint32_t)tj_f32_to_bf16(d[4 * q + 2]) | ((uint32_t)tj_f32_to_bf16(d[4 * q + 3]) << 16);
                const int v = 4 * c + q;
                *(uint2 *)(slab + r * 128 + ((v ^ (r & 7)) << 4) + 8 * h) = make_uint2(lo, hi);
            }
        }
        head_wave_sync();
#pragma unroll
        for (int pass = 0; pass < 4; ++pass) {
            const int row = 8 * pass + (lane >> 3), v = lane & 7;
            if (v < 4 * c_n && j0 + row < a.h.B) {
                const int k = 32 * c_begin + 8 * v;
                const headu32x4 g = *(const headu32x4 *)(slab + row * 128 + ((v ^ (row & 7)) << 4));
                const uint32_t bits = xmask[row * kMaskPitch + (k >> 3)];
                headu32x4 o;
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const uint32_t lo = (bits >> (2 * u)) & 1u ? (g[u] & 0xFFFFu) : 0u;
                    const uint32_t hi = (bits >> (2 * u + 1)) & 1u ? (g[u] & 0xFFFF0000u) : 0u;
                    o[u] = lo | hi;
                }
                *(headu32x4 *)((uint8_t *)(a.dX + (size_t)j0 * a.lddx) + (uint32_t)(row * a.lddx + k) * 2u) = o;
            }
        }
    }
}

// Splits head rows [n][ldz] into logits [n][A] and values [n].
__global__ __launch_bounds__(256) void split_head(const float *__restrict__ Z, int ldz, uint32_t n, int A,
                                                  float *__restrict__ logits, float *__restrict__ value)
{
    const uint32_t j = blockIdx.x * 256 + threadIdx.x;
    if (j >= n) return;
    const float *z = Z + (size_t)j * ldz;
    if (logits)
        for (int k = 0; k < A; ++k) logits[(size_t)j * A + k] = z[k];
    if (value) value[j] = z[A];
}

// Acting under the stochastic policy: row j of Z = (logits, value); u_j = top 24 bits of
// SplitMix64(seed, j) / 2^24; the action is the first whose cumulative softmax probability exceeds
// u_j (the last action if rounding leaves none).  One thread per observation.
__global__ __launch_bounds__(256) void ppo_sample(const float *__restrict__ Z, int ldz, uint32_t n, int A,
                                                  uint64_t seed, int32_t *__restrict__ action,
                                                  float *__restrict__ logp, float *__restrict__ value)
{
    const uint32_t j = blockIdx.x * 256 + threadIdx.x;
    if (j >= n) return;
    const float *z = Z + (size_t)j * ldz;
    float mx = z[0];
    for (int k = 1; k < A; ++k) mx = fmaxf(mx, z[k]);
    float se = 0.f;
    for (int k = 0; k < A; ++k) se += expf(z[k] - mx);
    const float lse = mx + logf(se);
    const float u = (float)(tj_splitmix64(seed, j) >> 40) * (1.f / 16777216.f);   // exact: 24 bits
    float cdf = 0.f;
    int pick = A - 1;
    for (int k = 0; k < A; ++k) {
        cdf += expf(z[k] - lse);
        if (cdf > u) { pick = k; break; }
    }
    action[j] = pick;
    logp[j] = z[pick] - lse;
    if (value) value[j] = z[A];
}

// Sum of S fp32 partial outputs [j][i] of a split forward contraction (slice order), plus the bias
// of row j's network (rows >= j_target use the second), ReLU, cast; writes the activation rows
// Y[j][i] and, for j < jt_max, the transposed copy YT[i][j].  Four consecutive i per thread.
template <typename T>
__global__ __launch_bounds__(256) void sum_bias_relu(const float *__restrict__ part, size_t zstride, int S, int J,
                                                     int I, const float *__restrict__ bias0,
                                                     const float *__restrict__ bias1, int j_target,
                                                     T *__restrict__ Y, int ldy, T *__restrict__ YT, int ldyt,
                                                     int jt_max)
{
    const size_t v = (size_t)blockIdx.x * 256 + threadIdx.x;
    const int vpr = I / 4;
    if (v >= (size_t)J * vpr) return;
    const int j = (int)(v / vpr), i = (int)(v - (size_t)j * vpr) * 4;
    const float *src = part + (size_t)j * I + i;
    float4 acc = *(const float4 *)src;
    for (int z = 1; z < S; ++z) {
        const float4 p = *(const float4 *)(src + (size_t)z * zstride);
        acc.x += p.x; acc.y += p.y; acc.z += p.z; acc.w += p.w;
    }
    const float *b = (j >= j_target ? bias1 : bias0) + i;
    const float o[4] = {fmaxf(acc.x + b[0], 0.f), fmaxf(acc.y + b[1], 0.f), fmaxf(acc.z + b[2], 0.f),
                        fmaxf(acc.w + b[3], 0.f)};
    T *y = Y + (size_t)j * ldy + i;
#pragma unroll
    for (int e = 0; e < 4; ++e) y[e] = TjElem<T>::from_f32(o[e]);
    if (j < jt_max)
#pragma unroll
        for (int e = 0; e < 4; ++e) YT[(size_t)(i + e) * ldyt + j] = TjElem<T>::from_f32(o[e]);
}

struct LayerPlan {
    int in, out;           // features
    int ld_in, ld_out;     // padded pitches (elements of T)
    size_t w_off, b_off;   // offsets into the flat parameter vector
};

int round_up(int x, int a) { return (x + a - 1) / a * a; }

bool desc_ok(const tj_learner_desc *d)
{
    if (!d || d->n_layers < 1 || d->n_layers > TJ_MAX_LAYERS) return false;
    if (!d->in_c || !d->in_h || !d->in_w || !d->max_batch) return false;
    if (d->precision != TJ_PRECISION_FP32 && d->precision != TJ_PRECISION_BF16) return false;
    if (d->obs_dtype != TJ_OBS_F32 && d->obs_dtype != TJ_OBS_U8) return false;
    for (uint32_t i = 0; i < d->n_layers; ++i) {
        if (d->layers[i].out == 0) return false;
        if (d->layers[i].kind != TJ_LAYER_LINEAR && d->layers[i].kind != TJ_LAYER_CONV2D) return false;
        if (d->layers[i].kind == TJ_LAYER_CONV2D && (!d->layers[i].kernel || !d->layers[i].stride)) return false;
    }
    return d->layers[d->n_layers - 1].kind == TJ_LAYER_LINEAR;
}

bool all_linear(const tj_learner_desc *d)
{
    for (uint32_t i = 0; i < d->n_layers; ++i)
        if (d->layers[i].kind != TJ_LAYER_LINEAR) return false;
    return d->obs_dtype == TJ_OBS_F32;
}

// Reads n elements of compute type from the device and widens them to float (host side).
template <typename T> int fetch_as_float(const T *d_src, size_t n, std::vector<float> &out, hipStream_t st)
{
    std::vector<T> raw(n);
    out.resize(n);
    if (hipMemcpyAsync(raw.data(), d_src, n * sizeof(T), hipMemcpyDeviceToHost, st) != hipSuccess ||
        hipStreamSynchronize(st) != hipSuccess) {
        (void)hipGetLastError();
        return TJ_ERR_DEVICE;
    }
    for (size_t i = 0; i < n; ++i) out[i] = TjElem<T>::to_f32(raw[i]);
    return TJ_OK;
}

}  // namespace

struct tj_learner {
    virtual ~tj_learner() {}
    virtual int step(const tj_minibatch *mb, tj_step_stats *d_stats, hipStream_t st) = 0;
    virtual int get_state(int which, float *h_out, size_t n, hipStream_t st) = 0;
    virtual int set_state(int which, const float *h_in, size_t n, hipStream_t st) = 0;
    virtual int infer(uint32_t n, const void *d_obs, float epsilon, uint64_t seed, int32_t *d_action,
                    int32_t *d_version, float *d_q, hipStream_t st) = 0;
    // on-policy learners only
    virtual int ppo_step(const tj_ppo_batch *, tj_ppo_stats *, hipStream_t) { return TJ_ERR_INVALID_ARG; }
    virtual int ppo_evaluate(uint32_t, const float *, float *, float *, hipStream_t) { return TJ_ERR_INVALID_ARG; }
    virtual int ppo_act(uint32_t, const float *, uint64_t, int32_t *, float *, float *, hipStream_t)
    {
        return TJ_ERR_INVALID_ARG;
    }
    uint64_t t = 0;
    hipEvent_t ev[5];
    bool timed = false;
    int mark(int i, hipStream_t st)
    {
        if (timed && hipEventRecord(ev[i], st) != hipSuccess) return TJ_ERR_DEVICE;
        return TJ_OK;
    }
};

namespace {

// The head layer's forward and the TD step, between phase marks 1 and 2.  bf16 with at most 32
// actions: the fused kernel (mark 1 before it); otherwise a GEMM into Q, mark 1, td_huber.
// X rows row0[0] + j, row0[1] + j, row0[2] + j hold the head's input for s, s' (online), s' (target).
template <typename T> struct HeadTd {
    const T *X; int ldx; int row0[3];
    const T *W_on, *W_tg; int ldw;
    const float *b_on, *b_tg;
    int B, A, K;
    float *Q; int ldq;
    T *dZ; int lddz; T *dZT; int lddzt;
    int32_t *astar; float *loss_part;
    // where the fused kernel runs it also writes the gradient wrt the head's input (rows of s) and
    // its transpose, if dX is set
    T *dX; int lddx; T *dXT; int lddxt; int Kin;
};

template <typename T> constexpr bool head_fused(int A) { return sizeof(T) == 2 && A <= 32; }
template <typename T> int td_blocks(int B, int A)
{
    return head_fused<T>(A) ? (B + kHeadRows - 1) / kHeadRows : (B + kTdBlock - 1) / kTdBlock;
}

template <typename T>
int run_head_td(tj_learner *self, const HeadTd<T> &h, const tj_minibatch *mb, float gamma, float kappa,
                hipStream_t st)
{
    int rc;
    if constexpr (sizeof(T) == 2) {
        if (head_fused<T>(h.A)) {
            if ((rc = self->mark(1, st)) != TJ_OK) return rc;
            HeadTdArgs a;
            a.X = h.X; a.ldx = h.ldx;
            for (int g = 0; g < 3; ++g) a.row0[g] = h.row0[g];
            a.W_on = h.W_on; a.W_tg = h.W_tg; a.ldw = h.ldw; a.b_on = h.b_on; a.b_tg = h.b_tg;
            a.B = h.B; a.A = h.A; a.K = h.K; a.Q = h.Q; a.ldq = h.ldq;
            a.action = mb->action; a.reward = mb->reward; a.done = mb->done;
            a.gamma = gamma; a.kappa = kappa;
            a.dZ = h.dZ; a.lddz = h.lddz; a.dZT = h.dZT; a.lddzt = h.lddzt;
            a.astar = h.astar; a.loss_part = h.loss_part;
            a.dX = h.dX; a.lddx = h.lddx; a.dXT = h.dXT; a.lddxt = h.lddxt; a.Kin = h.Kin;
            head_td<<<td_blocks<T>(h.B, h.A), kHeadThreads, 0, st>>>(a);
            return hipGetLastError() == hipSuccess ? TJ_OK : TJ_ERR_DEVICE;
        }
    }
    TjGemmArgs<T> g;
    memset(&g, 0, sizeof(g));
    g.n_seg = 2;
    g.seg[0] = {0, 2 * h.B, h.W_on, h.b_on, 0};
    g.seg[1] = {2 * h.B, 3 * h.B, h.W_tg, h.b_tg, 2 * h.B - h.row0[2]};
    g.Q = h.X;
    g.ldp = h.ldw; g.ldq = h.ldx;
    g.I = h.A; g.K = h.K;
    g.k_chunk = g.K; g.n_split = 1;
    g.Cf = h.Q; g.ldcf = h.ldq;
    if ((rc = tj_gemm<T>(g, st)) != TJ_OK) return rc;
    if ((rc = self->mark(1, st)) != TJ_OK) return rc;
    td_huber<T><<<td_blocks<T>(h.B, h.A), kTdBlock, 0, st>>>(h.Q, h.ldq, h.B, h.A, mb->action, mb->reward, mb->done,
                                                             gamma, kappa, h.dZ, h.lddz, h.dZT, h.lddzt, h.astar,
                                                             h.loss_part);
    return hipGetLastError() == hipSuccess ? TJ_OK : TJ_ERR_DEVICE;
}

template <typename T> struct MlpLearner : tj_learner {
    static constexpr int VE = TjElem<T>::kVec;
    tj_learner_desc d;
    int L = 0, A = 0, Bmax = 0, ldB = 0, ldA = 0, S = 1;
    int S_ends = 1;   // slices of the first and the last layer's weight gradients (>= S)
    int n_pass = 3;                        // stacked forward passes: s, s' (online), s' (target); 1 = on-policy
    size_t P = 0, Ppad = 0;
    std::vector<LayerPlan> lay;
    float *theta_on = nullptr, *theta_tg = nullptr, *m = nullptr, *v = nullptr, *gpart = nullptr;
    T *Wc_on[TJ_MAX_LAYERS], *WcT_on[TJ_MAX_LAYERS], *Wc_tg[TJ_MAX_LAYERS];
    T *X[TJ_MAX_LAYERS], *XT[TJ_MAX_LAYERS], *dZ[TJ_MAX_LAYERS + 1], *dZT[TJ_MAX_LAYERS + 1];
    size_t wc_bytes = 0;                   // contiguous block of all Wc_on (and of all Wc_tg)
    uint8_t *act_begin = nullptr;          // activation block, re-zeroed when the batch changes
    size_t act_bytes = 0;
    float *Qout = nullptr, *loss_part = nullptr;
    int32_t *astar = nullptr;
    tj_step_stats *stats_internal = nullptr;
    int last_batch = -1;

    // Lays the arena out; with a null base it only measures.
    size_t plan(void *base)
    {
        TjArena a(base);
        L = (int)d.n_layers;
        Bmax = (int)d.max_batch;
        ldB = round_up(Bmax, VE);
        lay.resize(L);
        int in = (int)(d.in_c * d.in_h * d.in_w);
        size_t off = 0;
        for (int l = 0; l < L; ++l) {
            lay[l].in = in;
            lay[l].out = (int)d.layers[l].out;
            lay[l].ld_in = round_up(in, VE);
            // (bf16) a narrow head is padded to one whole 64-k stage, so that the input-gradient
            // GEMM that contracts over it can use the direct-to-LDS kernel; the pads stay zero
            lay[l].ld_out = round_up(lay[l].out, (sizeof(T) == 2 && l == L - 1 && in >= 128) ? 64 : VE);
            lay[l].w_off = off; off += (size_t)in * lay[l].out;
            lay[l].b_off = off; off += lay[l].out;
            in = lay[l].out;
        }
        P = off;
        Ppad = tj_align_up(P, 64);
        A = lay[L - 1].out;
        ldA = round_up(A, 4);
        // split the batch contraction of the weight-gradient GEMMs so that each
        // slice still runs a long k loop
        // (fp32 nets here are small: more slices give the few output tiles enough blocks)
        S = Bmax / (sizeof(T) == 4 ? 64 : 1024);
        S = S < 1 ? 1 : (S > 8 ? 8 : S);
        theta_on = (float *)a.take(P * 4);
        theta_tg = (float *)a.take(P * 4);
        m = (float *)a.take(P * 4);
        v = (float *)a.take(P * 4);
        // The first layer's and the head's weight gradients share one launch of few 256 x 128 tiles; on a
        // large batch more slices than S let that launch reach every CU (bf16 nets of three layers or more,
        // where those two layers are apart in the flat gradient and their ranges start at whole vectors).
        S_ends = S;
        if (sizeof(T) == 2 && L >= 3 && lay[1].w_off % 4 == 0 && lay[L - 1].w_off % 4 == 0) {
            const int tiles = ((lay[0].in + 255) / 256) * ((lay[0].out + 127) / 128) +
                              ((lay[L - 1].in + 255) / 256) * ((lay[L - 1].out + 127) / 128);
            const int want = Bmax / 1024, fit = 256 / tiles;
            S_ends = std::max(S, std::min(want, fit));
        }
        gpart = (float *)a.take((size_t)S_ends * Ppad * 4);
        size_t wc0 = a.off;
        for (int l = 0; l < L; ++l) Wc_on[l] = (T *)a.take((size_t)lay[l].out * lay[l].ld_in * sizeof(T));
        wc_bytes = a.off - wc0;
        for (int l = 0; l < L; ++l) Wc_tg[l] = (T *)a.take((size_t)lay[l].out * lay[l].ld_in * sizeof(T));
        for (int l = 0; l < L; ++l) WcT_on[l] = (T *)a.take((size_t)lay[l].in * lay[l].ld_out * sizeof(T));
        size_t act0 = a.off;
        act_begin = base ? (uint8_t *)base + act0 : nullptr;
        for (int l = 0; l < L; ++l) {
            const size_t rows = (size_t)(n_pass == 1 ? 1 : (l == 0 ? 2 : 3)) * Bmax;
            X[l] = (T *)a.take(rows * lay[l].ld_in * sizeof(T));
            XT[l] = (T *)a.take((size_t)lay[l].in * ldB * sizeof(T));
        }
        for (int l = 1; l <= L; ++l) {
            dZ[l] = (T *)a.take((size_t)Bmax * lay[l - 1].ld_out * sizeof(T));
            dZT[l] = (T *)a.take((size_t)lay[l - 1].out * ldB * sizeof(T));
        }
        act_bytes = a.off - act0;
        Qout = (float *)a.take((size_t)n_pass * Bmax * ldA * 4);
        astar = (int32_t *)a.take((size_t)Bmax * 4);
        loss_part = (float *)a.take((size_t)((Bmax + kHeadRows - 1) / kHeadRows) * 4);
        stats_internal = (tj_step_stats *)a.take(sizeof(tj_step_stats));
        plan_more(a);
        return a.off;
    }

    virtual void plan_more(TjArena &) {}   // further pieces of a derived learner

    // statistics of an on-policy update that the optimizer kernel finalises (part == nullptr: none)
    struct PpoFinal {
        const float *part = nullptr;
        int n_part = 0;
        float c_v = 0.f, c_e = 0.f;
        tj_ppo_stats *out = nullptr, *internal = nullptr;
    } ppo_fin;

    // fp32 master -> compute-type copies (and transposes for the online net)
    // Adam writes the straight copy of every weight block whose rows need no padding
    bool adam_emits(int l) const { return lay[l].ld_in == lay[l].in; }
    // ... and the transposed copy of a small block with it (scattered element stores: only worth it where the
    // copy kernel's launch costs more than they do)
    bool adam_emits_t(int l) const
    {
        return adam_emits(l) && keeps_wct(l) && (size_t)lay[l].in * lay[l].out <= ((size_t)1 << 18);
    }

    // Weight gradient of layer l (1-based) straight from the row-major X_{l-1} and dZ_l (transposing LDS
    // reads) instead of their transposed copies: bf16, whole 32-row stages of the batch, widths that are
    // whole 16-byte vectors.  The first and the last layer too, although their narrow sides fill few of the
    // 256 x 128 tiles that form takes (their pair is 96 blocks on the 256-1024-1024-1024-32 net): what
    // counts is that no transposed copy of X_{l-1} and of dZ_l is written at all where it applies, which
    // makes the forward pass of the last hidden layer and the input-gradient pass of the second layer
    // one-layout launches like the others.
    bool wgrad_trans(int l, int B) const
    {
        if (sizeof(T) != 2 || B % 32 != 0 || l < 1 || l > L) return false;
        return lay[l - 1].in % 8 == 0 && lay[l - 1].out % 8 == 0;
    }

    // Input gradient of layer l (1-based, l >= 2) with the row-major weight copy as its first operand
    // (transposing LDS reads): bf16, a contraction over whole 32-row stages of the weight matrix.  Such a
    // layer keeps no transposed weight copy.
    bool dgrad_trans(int l) const
    {
        return sizeof(T) == 2 && lay[l - 1].in % 8 == 0 && lay[l - 1].out % 32 == 0;
    }
    // Layer index l (0-based) keeps a transposed weight copy: its input gradient exists, is a contraction
    // (the head's is not where the TD kernel writes it) and does not read the straight copy.
    virtual bool head_input_gradient_fused() const { return false; }   // a derived learner's head kernel reads WcT
    bool keeps_wct(int l) const
    {
        if (l == 0) return false;
        if (l == L - 1 && head_input_gradient_fused()) return true;
        if (l == L - 1 && n_pass == 3 && head_fused<T>(A)) return false;
        return !dgrad_trans(l + 1);
    }

    int recast(bool online, hipStream_t st, bool after_adam = false)
    {
        CastJobs<T> jobs;
        int n = 0;
        for (int l = 0; l < L; ++l) {
            CastJob<T> j;
            j.src = (online ? theta_on : theta_tg) + lay[l].w_off;
            j.dst = online ? Wc_on[l] : Wc_tg[l];
            if (after_adam && adam_emits(l)) j.dst = nullptr;
            j.dstT = online && keeps_wct(l) && !(after_adam && adam_emits_t(l)) ? WcT_on[l] : nullptr;
            j.R = lay[l].out; j.C = lay[l].in;
            j.ldd = lay[l].ld_in; j.lddT = lay[l].ld_out;
            if (j.dst || j.dstT) jobs.job[n++] = j;
        }
        return launch_cast<T>(jobs, n, st);
    }

    int step(const tj_minibatch *mb, tj_step_stats *d_stats, hipStream_t st) override
    {
        const int B = (int)mb->batch;
        if (B < 1 || B > Bmax) return TJ_ERR_SHAPE;
        if (!mb->obs || !mb->next_obs || !mb->action || !mb->reward || !mb->done) return TJ_ERR_INVALID_ARG;
        if (mb->row_index && (mb->n_rows == 0 || mb->n_rows > 0xFFFFFFFFull)) return TJ_ERR_INVALID_ARG;
        if (mb->plane_index) return TJ_ERR_INVALID_ARG;   // planes are channels of an image: pixel networks only
        int rc;
        if (last_batch != B) {
            // pad columns beyond the batch must read as zero in the batch contraction
            // (the arena starts zeroed; only a shrinking batch leaves stale columns behind)
            if (last_batch > B && (rc = launch_zero(act_begin, act_bytes, st)) != TJ_OK) return rc;
            last_batch = B;
        }

        // network input: [s ; s'] in compute type (and the transpose of s where the first layer's weight
        // gradient still contracts over transposed operands)
        {
            CastJobs<T> jobs;
            jobs.job[0] = {(const float *)mb->obs, X[0], wgrad_trans(1, B) ? nullptr : XT[0], B, lay[0].in, lay[0].ld_in, ldB};
            jobs.job[1] = {(const float *)mb->next_obs, X[0] + (size_t)B * lay[0].ld_in, nullptr, B,
                           lay[0].in, lay[0].ld_in, ldB};
            if (mb->row_index) {   // rows of the caller's tables (the ring itself), picked by index
                jobs.job[0].rows = jobs.job[1].rows = mb->row_index;
                jobs.job[0].n_rows = jobs.job[1].n_rows = (uint32_t)mb->n_rows;
            }
            if ((rc = launch_cast<T>(jobs, 2, st)) != TJ_OK) return rc;
        }
        if ((rc = mark(0, st)) != TJ_OK) return rc;

        // forward: columns j = rows of the stacked batch; [0,2B) online, [2B,3B) target
        for (int l = 0; l + 1 < L; ++l) {
            TjGemmArgs<T> g;
            memset(&g, 0, sizeof(g));
            g.n_seg = 2;
            g.seg[0] = {0, 2 * B, Wc_on[l], theta_on + lay[l].b_off, 0};
            g.seg[1] = {2 * B, 3 * B, Wc_tg[l], theta_tg + lay[l].b_off, l == 0 ? B : 0};
            g.Q = X[l];
            g.ldp = lay[l].ld_in; g.ldq = lay[l].ld_in;
            g.I = lay[l].out; g.K = lay[l].ld_in;
            g.k_chunk = g.K; g.n_split = 1;
            g.relu = 1;
            g.Ci = X[l + 1]; g.ldci = lay[l].ld_out;
            if (!wgrad_trans(l + 2, B)) { g.Cj = XT[l + 1]; g.ldcj = ldB; g.cj_jmax = B; }
            if ((rc = tj_gemm<T>(g, st)) != TJ_OK) return rc;
        }
        {   // head layer and TD step
            const LayerPlan &lh = lay[L - 1];
            HeadTd<T> h;
            h.X = X[L - 1]; h.ldx = lh.ld_in;
            h.row0[0] = 0; h.row0[1] = B; h.row0[2] = L == 1 ? B : 2 * B;
            h.W_on = Wc_on[L - 1]; h.W_tg = Wc_tg[L - 1]; h.ldw = lh.ld_in;
            h.b_on = theta_on + lh.b_off; h.b_tg = theta_tg + lh.b_off;
            h.B = B; h.A = A; h.K = lh.ld_in;
            h.Q = Qout; h.ldq = ldA;
            h.dZ = dZ[L]; h.lddz = lh.ld_out; h.dZT = wgrad_trans(L, B) ? nullptr : dZT[L]; h.lddzt = ldB;
            h.astar = astar; h.loss_part = loss_part;
            h.dX = nullptr; h.lddx = 0; h.dXT = nullptr; h.lddxt = 0; h.Kin = lh.in;
            if (head_fused<T>(A) && L >= 2) {   // the fused kernel also writes the head's input gradient
                h.dX = dZ[L - 1]; h.lddx = lh.ld_in;
                if (!wgrad_trans(L - 1, B)) { h.dXT = dZT[L - 1]; h.lddxt = ldB; }
            }
            if ((rc = run_head_td<T>(this, h, mb, d.gamma, d.huber_delta, st)) != TJ_OK) return rc;
        }
        if ((rc = mark(2, st)) != TJ_OK) return rc;
        return backward_update(B, td_blocks<T>(B, A), d_stats, st, head_fused<T>(A) && L >= 2);
    }

    // From dZ[L] / dZT[L] (gradient wrt the head's output, and its transpose) to the updated
    // parameters: backward GEMMs, slice reduction, Adam, refreshed weight copies, target sync.
    // n_loss_part per-block loss sums in loss_part are folded into the step's statistics.
    int backward_update(int B, int n_loss_part, tj_step_stats *d_stats, hipStream_t st, bool head_dx_done = false)
    {
        int rc;
        const int Kb = round_up(B, VE);
        // backward through the online network on s.  The weight gradient and the input gradient of a layer both
        // start from dZ_l and are independent: one paired launch where the kernels allow it.  The head's weight
        // gradient shares the launch of the first layer's weight gradient instead (neither is a problem that
        // fills the chip); its input gradient runs alone unless the TD kernel has already written it.
        TjGemmArgs<T> gw_head;
        bool head_pending = false;
        bool slices_summed = false;   // the hidden layers' gradient slices are summed before the optimizer launch
        for (int l = L; l >= 1; --l) {
            const LayerPlan &lp = lay[l - 1];
            TjGemmArgs<T> gw, gd;
            {   // dW_l[n][k] = sum_m dZ_l[m][n] X_{l-1}[m][k]; db_l[n] = sum_m dZ_l[m][n]
                TjGemmArgs<T> &g = gw;
                memset(&g, 0, sizeof(g));
                g.n_seg = 1;
                if (wgrad_trans(l, B)) {   // row-major operands, contraction over their rows
                    g.seg[0] = {0, lp.out, X[l - 1], nullptr, 0};
                    g.Q = dZ[l];
                    g.ldp = lp.ld_in; g.ldq = lp.ld_out;
                    g.trans = 1;
                } else {
                    g.seg[0] = {0, lp.out, XT[l - 1], nullptr, 0};
                    g.Q = dZT[l];
                    g.ldp = ldB; g.ldq = ldB;
                }
                g.I = lp.in; g.K = Kb;
                const int Sl = (l == 1 || l == L) ? S_ends : S;
                g.n_split = Sl;
                const int ke = 128 / (int)sizeof(T);
                g.k_chunk = round_up((Kb + Sl - 1) / Sl, ke);
                g.Cf = gpart + lp.w_off; g.ldcf = lp.in; g.cf_zstride = Ppad;
                g.qsum = gpart + lp.b_off; g.qsum_zstride = Ppad;
            }
            // the head's weight gradient waits for the first layer's (bf16, two layers or more): both are
            // narrow split contractions, neither of which fills the chip alone
            const bool defer_head = l == L && L >= 2 && sizeof(T) == 2;
            if (defer_head && head_dx_done) {
                gw_head = gw;
                head_pending = true;
                continue;
            }
            if (l >= 2) {   // dX_{l-1}[m][k] = relu'(X_{l-1}) * sum_n dZ_l[m][n] W_l[n][k]
                TjGemmArgs<T> &g = gd;
                memset(&g, 0, sizeof(g));
                g.n_seg = 1;
                g.Q = dZ[l];
                g.ldq = lp.ld_out;
                g.I = lp.in;
                if (dgrad_trans(l)) {   // the weights as stored, [n][k]: the contraction runs over their rows
                    g.seg[0] = {0, B, Wc_on[l - 1], nullptr, 0};
                    g.ldp = lp.ld_in; g.K = lp.out;
                    g.trans = 2;
                } else {
                    g.seg[0] = {0, B, WcT_on[l - 1], nullptr, 0};
                    g.ldp = lp.ld_out; g.K = lp.ld_out;   // pad columns are zero in both operands
                }
                g.k_chunk = g.K; g.n_split = 1;
                g.mask = X[l - 1]; g.ldmask = lp.ld_in;
                g.Ci = dZ[l - 1]; g.ldci = lp.ld_in;
                if (!wgrad_trans(l - 1, B)) { g.Cj = dZT[l - 1]; g.ldcj = ldB; g.cj_jmax = B; }
            }
            if (defer_head) {   // the input gradient alone now
                if ((rc = tj_gemm<T>(gd, st)) != TJ_OK) return rc;
                gw_head = gw;
                head_pending = true;
                continue;
            }
            if (l >= 2) {
                if constexpr (sizeof(T) == 2) rc = tj_gemm_pair(gw, gd, st);
                else rc = tj_gemm_pair_f32(gw, gd, st);
                if (rc != TJ_OK) return rc;
                continue;
            }
            if (head_pending) {   // l == 1
                if constexpr (sizeof(T) == 2) {
                    // The first layer's and the head's weight gradients fill less than half of the chip, and the
                    // slices of the layers between them (a contiguous range of the flat gradient) are complete
                    // by now: their sum rides in this launch, and the optimizer reads one slice for them.
                    const TjSliceSum r = {gpart, S, Ppad, lay[1].w_off, lay[L - 1].w_off};
                    if (L >= 3 && S > 1) rc = tj_gemm_pair_sum(gw, gw_head, r, st, &slices_summed);
                    else rc = tj_gemm_pair(gw, gw_head, st);
                } else {
                    rc = TJ_ERR_SHAPE;   // the fused head kernel exists for bf16 only
                }
                if (rc != TJ_OK) return rc;
                head_pending = false;
                continue;
            }
            if ((rc = tj_gemm<T>(gw, st)) != TJ_OK) return rc;
        }

        if ((rc = mark(3, st)) != TJ_OK) return rc;   // the gradient slices not summed yet are summed by the Adam kernel
        t += 1;
        const float c1 = (float)(1.0 - pow((double)d.beta1, (double)t));
        const float c2 = (float)(1.0 - pow((double)d.beta2, (double)t));
        EmitTable<T> tab;
        tab.n = 0;
        for (int l = 0; l < L; ++l) {
            if (!adam_emits(l)) continue;
            tab.begin[tab.n] = lay[l].w_off;
            tab.end[tab.n] = lay[l].w_off + (size_t)lay[l].in * lay[l].out;
            tab.dstT[tab.n] = adam_emits_t(l) ? WcT_on[l] : nullptr;
            tab.C[tab.n] = lay[l].in; tab.ldT[tab.n] = lay[l].ld_out;
            tab.dst[tab.n++] = Wc_on[l];
        }
        LossFinal lf = {loss_part, n_loss_part, B, (uint32_t)t, d_stats, stats_internal};
        if (ppo_fin.part) {   // set by the on-policy learner for this call
            lf.ppo_part = ppo_fin.part; lf.ppo_n_part = ppo_fin.n_part;
            lf.c_v = ppo_fin.c_v; lf.c_e = ppo_fin.c_e;
            lf.ppo_out = ppo_fin.out; lf.ppo_internal = ppo_fin.internal;
        }
        DgradEmit no_dgrad;
        no_dgrad.n = 0;
        // hidden layers: S slices, or one where the last launch has summed them; first and last layer: S_ends
        const bool mid = L >= 3 && (slices_summed || S_ends != S);
        const size_t mid_begin = mid ? lay[1].w_off : 0, mid_end = mid ? lay[L - 1].w_off : 0;
        adam_update<T><<<(unsigned)((P + 1023) / 1024), 256, 0, st>>>(theta_on, m, v, gpart, S_ends, Ppad, P, d.lr,
                                                                      d.beta1, d.beta2, d.eps, c1, c2, tab, lf, no_dgrad,
                                                                      mid_begin, mid_end, slices_summed ? 1 : S);
        if (hipGetLastError() != hipSuccess) return TJ_ERR_DEVICE;
        if ((rc = mark(4, st)) != TJ_OK) return rc;
        if ((rc = recast(true, st, true)) != TJ_OK) return rc;   // transposed copies (and padded blocks)
        if (d.target_interval && t % d.target_interval == 0) {
            TJ_HIP_TRY(hipMemcpyAsync(theta_tg, theta_on, P * 4, hipMemcpyDeviceToDevice, st));
            TJ_HIP_TRY(hipMemcpyAsync(Wc_tg[0], Wc_on[0], wc_bytes, hipMemcpyDeviceToDevice, st));
        }
        return TJ_OK;
    }

    // Policy inference on n <= 2*Bmax observations: online forward in the step's own buffers
    // (rows [0, n) of every X_l), then the epsilon-greedy kernel on the Q rows.
    int infer(uint32_t n_, const void *d_obs, float epsilon, uint64_t seed, int32_t *d_action, int32_t *d_version,
            float *d_q, hipStream_t st) override
    {
        const int n = (int)n_;
        if (n < 1 || n > (n_pass == 1 ? 1 : 2) * Bmax) return TJ_ERR_SHAPE;
        if (!d_obs || !d_action || !d_version || !(epsilon >= 0.f && epsilon <= 1.f)) return TJ_ERR_INVALID_ARG;
        int rc;
        CastJobs<T> jobs;
        jobs.job[0] = {(const float *)d_obs, X[0], nullptr, n, lay[0].in, lay[0].ld_in, ldB};
        if ((rc = launch_cast<T>(jobs, 1, st)) != TJ_OK) return rc;
        for (int l = 0; l < L; ++l) {
            TjGemmArgs<T> g;
            memset(&g, 0, sizeof(g));
            g.n_seg = 1;
            g.seg[0] = {0, n, Wc_on[l], theta_on + lay[l].b_off, 0};
            g.Q = X[l];
            g.ldp = lay[l].ld_in; g.ldq = lay[l].ld_in;
            g.I = lay[l].out; g.K = lay[l].ld_in;
            g.k_chunk = g.K; g.n_split = 1;
            if (l + 1 < L) {
                g.relu = 1;
                g.Ci = X[l + 1]; g.ldci = lay[l].ld_out;
            } else {
                g.Cf = Qout; g.ldcf = ldA;
            }
            if ((rc = tj_gemm<T>(g, st)) != TJ_OK) return rc;
        }
        egreedy<<<(n + 255) / 256, 256, 0, st>>>(Qout, ldA, (uint32_t)n, A, egreedy_threshold(epsilon), seed,
                                                 (int32_t)t, d_action, d_version, d_q);
        return hipGetLastError() == hipSuccess ? TJ_OK : TJ_ERR_DEVICE;
    }

    int get_state(int which, float *h_out, size_t n, hipStream_t st) override
    {
        const float *src = nullptr;
        switch (which) {
        case TJ_STATE_PARAMS: src = theta_on; break;
        case TJ_STATE_TARGET: src = theta_tg; break;
        case TJ_STATE_ADAM_M: src = m; break;
        case TJ_STATE_ADAM_V: src = v; break;
        default: break;
        }
        if (src) {
            if (n != P) return TJ_ERR_INVALID_ARG;
            TJ_HIP_TRY(hipMemcpyAsync(h_out, src, P * 4, hipMemcpyDeviceToHost, st));
            TJ_HIP_TRY(hipStreamSynchronize(st));
            return TJ_OK;
        }
        if (which == TJ_STATE_GRADS) {   // slice 0 holds the sum over the split slices
            if (n != P) return TJ_ERR_INVALID_ARG;
            TJ_HIP_TRY(hipMemcpyAsync(h_out, gpart, P * 4, hipMemcpyDeviceToHost, st));
            TJ_HIP_TRY(hipStreamSynchronize(st));
            return TJ_OK;
        }
        if (which == TJ_STATE_WEIGHTS_COMPUTE || which == TJ_STATE_WEIGHTS_COMPUTE_T ||
            which == TJ_STATE_WEIGHTS_COMPUTE_TARGET) {
            if (n != P) return TJ_ERR_INVALID_ARG;
            const bool tg = which == TJ_STATE_WEIGHTS_COMPUTE_TARGET, tr = which == TJ_STATE_WEIGHTS_COMPUTE_T;
            TJ_HIP_TRY(hipMemcpyAsync(h_out, tg ? theta_tg : theta_on, P * 4, hipMemcpyDeviceToHost, st));   // biases
            TJ_HIP_TRY(hipStreamSynchronize(st));
            std::vector<float> w;
            for (int l = 0; l < L; ++l) {
                const LayerPlan &lp = lay[l];
                float *dst = h_out + lp.w_off;
                int rc;
                if (tr && keeps_wct(l)) {
                    if ((rc = fetch_as_float<T>(WcT_on[l], (size_t)lp.in * lp.ld_out, w, st)) != TJ_OK) return rc;
                    for (int o = 0; o < lp.out; ++o)
                        for (int k = 0; k < lp.in; ++k) dst[(size_t)o * lp.in + k] = w[(size_t)k * lp.ld_out + o];
                } else {
                    if ((rc = fetch_as_float<T>(tg ? Wc_tg[l] : Wc_on[l], (size_t)lp.out * lp.ld_in, w, st)) != TJ_OK)
                        return rc;
                    for (int o = 0; o < lp.out; ++o)
                        for (int k = 0; k < lp.in; ++k) dst[(size_t)o * lp.in + k] = w[(size_t)o * lp.ld_in + k];
                }
            }
            return TJ_OK;
        }
        if (which == TJ_STATE_QVALS) {
            if (last_batch < 1 || n != 3 * (size_t)last_batch * A) return TJ_ERR_INVALID_ARG;
            std::vector<float> tmp(3 * (size_t)last_batch * ldA);
            TJ_HIP_TRY(hipMemcpyAsync(tmp.data(), Qout, tmp.size() * 4, hipMemcpyDeviceToHost, st));
            TJ_HIP_TRY(hipStreamSynchronize(st));
            for (size_t r = 0; r < 3 * (size_t)last_batch; ++r)
                for (int a = 0; a < A; ++a) h_out[r * A + a] = tmp[r * ldA + a];
            return TJ_OK;
        }
        if (which == TJ_STATE_ASTAR) {
            if (last_batch < 1 || n != (size_t)last_batch) return TJ_ERR_INVALID_ARG;
            std::vector<int32_t> tmp(last_batch);
            TJ_HIP_TRY(hipMemcpyAsync(tmp.data(), astar, tmp.size() * 4, hipMemcpyDeviceToHost, st));
            TJ_HIP_TRY(hipStreamSynchronize(st));
            for (int j = 0; j < last_batch; ++j) h_out[j] = (float)tmp[j];
            return TJ_OK;
        }
        return TJ_ERR_INVALID_ARG;
    }

    int set_state(int which, const float *h_in, size_t n, hipStream_t st) override
    {
        if (n != P) return TJ_ERR_INVALID_ARG;
        float *dst = nullptr;
        switch (which) {
        case TJ_STATE_PARAMS: dst = theta_on; break;
        case TJ_STATE_TARGET: dst = theta_tg; break;
        case TJ_STATE_ADAM_M: dst = m; break;
        case TJ_STATE_ADAM_V: dst = v; break;
        default: return TJ_ERR_INVALID_ARG;
        }
        TJ_HIP_TRY(hipMemcpyAsync(dst, h_in, P * 4, hipMemcpyHostToDevice, st));
        int rc = TJ_OK;
        if (which == TJ_STATE_PARAMS) rc = recast(true, st);
        if (which == TJ_STATE_TARGET) rc = recast(false, st);
        TJ_HIP_TRY(hipStreamSynchronize(st));
        return rc;
    }
};

// Actor-critic MLP (shared trunk; head = A logits + 1 value) updated with the clipped objective on
// the whole batch.  One forward pass (no target network, no s'), so the activation buffers hold
// max_batch rows; backward, slice reduction, Adam and the weight copies are the Q-learner's.
template <typename T> struct PpoLearner : MlpLearner<T> {
    // The objective kernel can also produce the head's input gradient (bf16, at most 32 head outputs, a head
    // input of whole 32-column tiles without row padding, a transposed weight copy wide enough for its
    // 16-wide contraction steps); the transposed copy of the head's weights is kept for it.
    bool head_input_gradient_fused() const override
    {
        if (sizeof(T) != 2 || this->L < 3 || this->A > 32) return false;
        const auto &lh = this->lay[this->L - 1];
        const int cols16 = (round_up(this->A, 8) + 15) / 16 * 16;
        return lh.in % 32 == 0 && lh.in <= kPpoFusedMaxK && lh.ld_in == lh.in && lh.ld_out >= cols16;
    }
    using Base = MlpLearner<T>;
    tj_ppo_desc pd;
    float *ppo_part = nullptr;
    tj_ppo_stats *ppo_stats = nullptr;

    void plan_more(TjArena &a) override
    {
        ppo_part = (float *)a.take((size_t)((this->Bmax + kPpoRows - 1) / kPpoRows) * 4 * 4);
        ppo_stats = (tj_ppo_stats *)a.take(sizeof(tj_ppo_stats));
    }

    int step(const tj_minibatch *, tj_step_stats *, hipStream_t) override { return TJ_ERR_INVALID_ARG; }
    int infer(uint32_t, const void *, float, uint64_t, int32_t *, int32_t *, float *, hipStream_t) override
    {
        return TJ_ERR_INVALID_ARG;
    }

    // forward of n rows of fp32 observations through the trunk and the head; head rows in Qout
    int forward(int n, const float *d_obs, bool keep_transposes, hipStream_t st, bool trunk_only = false)
    {
        int rc;
        const auto &lay = this->lay;
        CastJobs<T> jobs;
        jobs.job[0] = {d_obs, this->X[0], keep_transposes && !this->wgrad_trans(1, n) ? this->XT[0] : nullptr, n,
                       lay[0].in, lay[0].ld_in, this->ldB};
        if ((rc = launch_cast<T>(jobs, 1, st)) != TJ_OK) return rc;
        if (keep_transposes && (rc = this->mark(0, st)) != TJ_OK) return rc;
        for (int l = 0; l < this->L - (trunk_only ? 1 : 0); ++l) {
            TjGemmArgs<T> g;
            memset(&g, 0, sizeof(g));
            g.n_seg = 1;
            g.seg[0] = {0, n, this->Wc_on[l], this->theta_on + lay[l].b_off, 0};
            g.Q = this->X[l];
            g.ldp = lay[l].ld_in; g.ldq = lay[l].ld_in;
            g.I = lay[l].out; g.K = lay[l].ld_in;
            g.k_chunk = g.K; g.n_split = 1;
            if (l + 1 < this->L) {
                g.relu = 1;
                g.Ci = this->X[l + 1]; g.ldci = lay[l].ld_out;
                if (keep_transposes && !this->wgrad_trans(l + 2, n)) { g.Cj = this->XT[l + 1]; g.ldcj = this->ldB; g.cj_jmax = n; }
            } else {
                g.Cf = this->Qout; g.ldcf = this->ldA;
            }
            if ((rc = tj_gemm<T>(g, st)) != TJ_OK) return rc;
        }
        return TJ_OK;
    }

    int ppo_step(const tj_ppo_batch *pb, tj_ppo_stats *d_stats, hipStream_t st) override
    {
        const int B = (int)pb->batch;
        if (B < 1 || B > this->Bmax) return TJ_ERR_SHAPE;
        if (!pb->obs || !pb->action || !pb->old_logp || !pb->adv || !pb->ret) return TJ_ERR_INVALID_ARG;
        int rc;
        if (this->last_batch != B) {
            // pad columns beyond the batch must read as zero in the batch contraction
            if (this->last_batch > B && (rc = launch_zero(this->act_begin, this->act_bytes, st)) != TJ_OK) return rc;
            this->last_batch = B;
        }
        // bf16 with at most 32 head outputs: the head layer's forward runs inside the objective kernel
        const bool fused = sizeof(T) == 2 && this->A <= 32 && this->L >= 2;
        // the same kernel writes the head's input gradient where the layer below takes it row-major
        const bool fused_dx = fused && head_input_gradient_fused() && this->wgrad_trans(this->L - 1, B);
        if ((rc = forward(B, pb->obs, true, st, fused)) != TJ_OK) return rc;
        if ((rc = this->mark(1, st)) != TJ_OK) return rc;
        const auto &lh = this->lay[this->L - 1];
        PpoHeadArgs<T> a;
        a.Z = this->Qout; a.ldz = this->ldA; a.B = B; a.A = this->A - 1;
        a.action = pb->action; a.old_logp = pb->old_logp; a.adv = pb->adv; a.ret = pb->ret;
        a.clip = pd.clip; a.c_v = pd.c_v; a.c_e = pd.c_e;
        a.dZ = this->dZ[this->L]; a.lddz = lh.ld_out; a.lddzt = this->ldB;
        a.dZT = this->wgrad_trans(this->L, B) ? nullptr : this->dZT[this->L];
        a.part = ppo_part;
        const int nblk = (B + kPpoRows - 1) / kPpoRows;
        if constexpr (sizeof(T) == 2) {
            if (fused) {
                PpoFusedArgs f;
                f.h = a;
                f.X = this->X[this->L - 1]; f.ldx = lh.ld_in;
                f.W = this->Wc_on[this->L - 1]; f.ldw = lh.ld_in;
                f.bias = this->theta_on + lh.b_off;
                f.K = lh.ld_in;
                f.WT = nullptr; f.ldwt = 0; f.dX = nullptr; f.lddx = 0;
                if (fused_dx) {   // ... and the head's input gradient, row-major only
                    f.WT = this->WcT_on[this->L - 1]; f.ldwt = lh.ld_out;
                    f.dX = this->dZ[this->L - 1]; f.lddx = lh.ld_in;
                }
                ppo_head_fused<<<nblk, kPpoRows * kPpoLanes, 0, st>>>(f);
            }
        }
        if (!fused) ppo_head<T><<<nblk, kPpoRows * kPpoLanes, 0, st>>>(a);
        if (hipGetLastError() != hipSuccess) return TJ_ERR_DEVICE;
        if ((rc = this->mark(2, st)) != TJ_OK) return rc;
        // the optimizer kernel's first wave turns the per-block sums into the step's statistics
        this->ppo_fin.part = ppo_part; this->ppo_fin.n_part = nblk;
        this->ppo_fin.c_v = pd.c_v; this->ppo_fin.c_e = pd.c_e;
        this->ppo_fin.out = d_stats; this->ppo_fin.internal = ppo_stats;
        rc = this->backward_update(B, 0, nullptr, st, fused_dx);
        this->ppo_fin.part = nullptr;
        return rc;
    }

    int ppo_evaluate(uint32_t n_, const float *d_obs, float *d_logits, float *d_value, hipStream_t st) override
    {
        const int n = (int)n_;
        if (n < 1 || n > this->Bmax) return TJ_ERR_SHAPE;
        if (!d_obs || (!d_logits && !d_value)) return TJ_ERR_INVALID_ARG;
        int rc;
        if ((rc = forward(n, d_obs, false, st)) != TJ_OK) return rc;
        split_head<<<(n + 255) / 256, 256, 0, st>>>(this->Qout, this->ldA, n_, this->A - 1, d_logits, d_value);
        return hipGetLastError() == hipSuccess ? TJ_OK : TJ_ERR_DEVICE;
    }

    int ppo_act(uint32_t n_, const float *d_obs, uint64_t seed, int32_t *d_action, float *d_logp, float *d_value,
                hipStream_t st) override
    {
        const int n = (int)n_;
        if (n < 1 || n > this->Bmax) return TJ_ERR_SHAPE;
        if (!d_obs || !d_action || !d_logp) return TJ_ERR_INVALID_ARG;
        int rc;
        if ((rc = forward(n, d_obs, false, st)) != TJ_OK) return rc;
        ppo_sample<<<(n + 255) / 256, 256, 0, st>>>(this->Qout, this->ldA, n_, this->A - 1, seed, d_action, d_logp,
                                                     d_value);
        return hipGetLastError() == hipSuccess ? TJ_OK : TJ_ERR_DEVICE;
    }
};

// ---------------------------------------------------------------- convolutional Q-networks
//
// Convolutions first, then linear layers.  Activations are channels-last; a convolution is the
// GEMM  act_out[m][oc] = relu(sum_k patch[m][k] W[oc][k] + b[oc])  on an explicit patch matrix
// (rows m = (image, oh, ow), k = (kh, kw, c)), its weight gradient contracts the transposed
// patch matrix with dZ^T over m (split many ways, reduced and un-permuted afterwards), its input
// gradient is a GEMM to a patch-gradient matrix followed by a gather (col2im) with the ReLU mask.
// Images are ordered s | s' | s'(target copy from layer 1 on).
//   act[l]      input of layer l: conv [n_img][H][W][C]; linear [3B][ldK]
//   patches[l]  [n_img*OH*OW][ldK]      patchesT[l] [K][ld(B*OH*OW)]   (conv)
//   XT[l]       [K][ld(B)]                                               (linear)
//   dZ[l]       gradient wrt the output of layer l: conv [B*OH*OW][OC], linear [B][ldO]; dZT[l]
//   dpatch[l]   [B*OH*OW][ldK] (conv, l > 0)   part[l]  fp32 [n_split][O*K + O (padded)]
template <typename T> struct ConvLearner : tj_learner {
    static constexpr int VE = TjElem<T>::kVec;
    struct NLayer {
        int kind;
        tjconv::ConvGeom g;
        int O, C, S, K, ldK, ldO;       // weight [O][C][S]; K = C*S
        int OHW;                        // conv: OH*OW
        size_t w_off, b_off;
        int n_split;
        size_t part_stride;
        bool implicit;                  // conv without patch matrices: operand gathers (bf16, 32/64 channels)
        TjGather gth;
        // input gradient as one gathered GEMM over the zero-bordered output gradient (see backward)
        bool dgrad_gather;
        TjGather dg_in, dg_out;
        int A, Kd, Nd, pad;             // taps per dimension, A*A*O, s*s*C, A-1
        T *dZh, *Wd;
        T *Wc_on, *WcT_on, *Wc_tg, *patches, *patchesT, *XT, *dZ, *dZT, *dpatch;
        float *part;
        // linear layer whose forward fills too few tiles: the contraction is split f_split ways into
        // fp32 partial outputs, summed with bias and ReLU by sum_bias_relu
        int f_split, f_chunk;
        float *f_part;
    };
    tj_learner_desc d;
    int L = 0, A = 0, Bmax = 0, ldB = 0, ldA = 0;
    size_t P = 0, Ppad = 0;
    std::vector<NLayer> lay;
    T *act[TJ_MAX_LAYERS + 1];
    float *theta_on = nullptr, *theta_tg = nullptr, *m = nullptr, *v = nullptr, *grad = nullptr;
    T *wc_on_begin = nullptr, *wc_tg_begin = nullptr;
    size_t wc_bytes = 0;
    uint8_t *act_begin = nullptr;
    size_t act_bytes = 0;
    float *Qout = nullptr, *loss_part = nullptr;
    int32_t *astar = nullptr;
    tj_step_stats *stats_internal = nullptr;
    int last_batch = -1;
    bool shape_ok = true;
    bool first_fused = false;   // layer 0 runs straight from the u8 frames (tj_conv_first)
    bool first_wgrad_u8 = false;   // ... and so does its weight gradient: no channels-last copy of the s images
    int n_cu = 0;                  // compute units of the device (asked once)

    size_t plan(void *base)
    {
        TjArena a(base);
        L = (int)d.n_layers;
        Bmax = (int)d.max_batch;
        ldB = round_up(Bmax, VE);
        lay.assign(L, NLayer());
        int c = (int)d.in_c, h = (int)d.in_h, w = (int)d.in_w;
        bool seen_linear = false, prev_conv = false;
        size_t off = 0;
        shape_ok = d.layers[0].kind == TJ_LAYER_CONV2D;
        for (int l = 0; l < L; ++l) {
            NLayer &y = lay[l];
            y.kind = (int)d.layers[l].kind;
            if (y.kind == TJ_LAYER_CONV2D) {
                if (seen_linear) shape_ok = false;
                tjconv::ConvGeom &g = y.g;
                g.C = c; g.H = h; g.W = w; g.k = (int)d.layers[l].kernel; g.s = (int)d.layers[l].stride;
                if (h < g.k || w < g.k) { shape_ok = false; g.k = 1; g.s = 1; }
                g.OC = (int)d.layers[l].out;
                g.OH = (h - g.k) / g.s + 1; g.OW = (w - g.k) / g.s + 1;
                g.K = c * g.k * g.k;
                y.O = g.OC; y.C = c; y.S = g.k * g.k; y.K = g.K; y.OHW = g.OH * g.OW;
                y.ldK = round_up(y.K, VE);
                y.ldO = y.O;
                if (y.O % VE) shape_ok = false;            // channels-last rows must be whole vectors
                y.implicit = false;
                if (sizeof(T) == 2 && (y.O == 32 || y.O == 64) && y.K % 64 == 0)
                    y.implicit = tj_gather_make(y.gth, g.C, g.H, g.W, g.k, g.s, g.OH, g.OW,
                                                3 * (size_t)Bmax * y.OHW);
                y.dgrad_gather = false;
                if (l > 0 && y.implicit && g.k % g.s == 0 && g.H % g.s == 0 && g.W % g.s == 0 && g.C % 8 == 0) {
                    y.A = g.k / g.s; y.pad = y.A - 1;
                    y.Kd = y.A * y.A * y.O; y.Nd = g.s * g.s * g.C;
                    const int Hc = g.H / g.s, Wc = g.W / g.s;
                    if (y.Kd % 64 == 0 && y.Nd <= 128)
                        y.dgrad_gather =
                            tj_gather_make(y.dg_in, y.O, g.OH + 2 * y.pad, g.OW + 2 * y.pad, y.A, 1, Hc, Wc,
                                           (size_t)Bmax * Hc * Wc) &&
                            tj_gather_make(y.dg_out, g.C, g.H, g.W, g.s, g.s, Hc, Wc, (size_t)Bmax * Hc * Wc);
                }
                c = g.OC; h = g.OH; w = g.OW;
                prev_conv = true;
            } else {
                y.implicit = false;
                y.dgrad_gather = false;
                seen_linear = true;
                y.O = (int)d.layers[l].out;
                if (prev_conv) { y.C = c; y.S = h * w; } else { y.C = c * h * w; y.S = 1; }
                y.K = y.C * y.S; y.OHW = 1;
                y.ldK = round_up(y.K, VE);
                if (prev_conv && y.K % VE) shape_ok = false;
                y.ldO = round_up(y.O, (sizeof(T) == 2 && l == L - 1 && y.K >= 128) ? 64 : VE);
                c = y.O; h = 1; w = 1;
                prev_conv = false;
            }
            y.w_off = off; off += (size_t)y.O * y.K;
            y.b_off = off; off += y.O;
            // weight-gradient contraction length and its split
            const size_t Ms = (size_t)Bmax * y.OHW;
            size_t ns = Ms / 4096;
            y.n_split = (int)(ns < 1 ? 1 : (ns > 128 ? 128 : ns));
            if (y.kind == TJ_LAYER_LINEAR) {   // enough slices to fill the chip with 256 x 128 tiles
                const size_t tiles = (((size_t)y.K + 255) / 256) * (((size_t)y.O + 127) / 128);
                ns = tiles >= 256 ? 1 : 256 / tiles;
                if (ns > (size_t)Bmax / 256) ns = (size_t)Bmax / 256;
                y.n_split = (int)(ns < 1 ? 1 : (ns > 8 ? 8 : ns));
            }
            if (y.implicit) {   // about 512 blocks (128 patch columns each), each with at least four 64-row stages
                const size_t njb = ((size_t)y.K + 127) / 128, stages = (Ms + 63) / 64;
                ns = 512 / njb;
                if (ns > stages / 4) ns = stages / 4;
                y.n_split = (int)(ns < 1 ? 1 : ns);
            }
            y.part_stride = tj_align_up((size_t)y.O * y.K + y.O, 64);
        }
        if (lay[L - 1].kind != TJ_LAYER_LINEAR) shape_ok = false;
        first_fused = sizeof(T) == 2 && d.obs_dtype == TJ_OBS_U8 && lay[0].kind == TJ_LAYER_CONV2D &&
                      lay[0].implicit && lay[0].ldK == lay[0].K &&
                      tj_conv_first_fits(lay[0].g.C, lay[0].g.H, lay[0].g.W, lay[0].g.k, lay[0].g.s, lay[0].O);
        first_wgrad_u8 = first_fused && tj_conv_first_wgrad_fits(lay[0].g.C, lay[0].g.H, lay[0].g.W, lay[0].g.k,
                                                                 lay[0].g.s, lay[0].O);
        P = off;
        Ppad = tj_align_up(P, 64);
        A = lay[L - 1].O;
        ldA = round_up(A, 4);
        theta_on = (float *)a.take(P * 4);
        theta_tg = (float *)a.take(P * 4);
        m = (float *)a.take(P * 4);
        v = (float *)a.take(P * 4);
        grad = (float *)a.take(Ppad * 4);
        size_t wc0 = a.off;
        for (int l = 0; l < L; ++l) lay[l].Wc_on = (T *)a.take((size_t)lay[l].O * lay[l].ldK * sizeof(T));
        wc_bytes = a.off - wc0;
        wc_on_begin = lay[0].Wc_on;
        for (int l = 0; l < L; ++l) lay[l].Wc_tg = (T *)a.take((size_t)lay[l].O * lay[l].ldK * sizeof(T));
        wc_tg_begin = lay[0].Wc_tg;
        for (int l = 0; l < L; ++l) lay[l].WcT_on = (T *)a.take((size_t)lay[l].K * lay[l].ldO * sizeof(T));
        for (int l = 0; l < L; ++l) lay[l].part = (float *)a.take((size_t)lay[l].n_split * lay[l].part_stride * 4);
        for (int l = 0; l < L; ++l)
            lay[l].Wd = lay[l].dgrad_gather ? (T *)a.take((size_t)lay[l].Nd * lay[l].Kd * sizeof(T)) : nullptr;
        size_t act0 = a.off;
        act_begin = base ? (uint8_t *)base + act0 : nullptr;
        const size_t B = (size_t)Bmax;
        for (int l = 0; l < L; ++l) {
            NLayer &y = lay[l];
            if (y.kind == TJ_LAYER_CONV2D) {
                const size_t n_img = l == 0 ? 2 * B : 3 * B;
                act[l] = (T *)a.take(n_img * y.g.H * y.g.W * y.g.C * sizeof(T));
                y.XT = nullptr;
                if (y.implicit) {   // no patch matrices; dZ rows padded (zero) to whole 64-row stages
                    y.patches = y.patchesT = y.dZT = nullptr;
                    y.dZ = (T *)a.take((B * y.OHW + 64) * y.O * sizeof(T));
                } else {
                    y.patches = (T *)a.take(n_img * y.OHW * y.ldK * sizeof(T));
                    y.patchesT = (T *)a.take((size_t)y.K * round_up((int)(B * y.OHW), VE) * sizeof(T));
                    y.dZ = (T *)a.take(B * y.OHW * y.O * sizeof(T));
                    y.dZT = (T *)a.take((size_t)y.O * round_up((int)(B * y.OHW), VE) * sizeof(T));
                }
                y.f_split = 1; y.f_chunk = 0; y.f_part = nullptr;
                y.dpatch = (l > 0 && !y.dgrad_gather) ? (T *)a.take(B * y.OHW * y.ldK * sizeof(T)) : nullptr;
                y.dZh = y.dgrad_gather ? (T *)a.take(B * (y.g.OH + 2 * y.pad) * (y.g.OW + 2 * y.pad) * y.O * sizeof(T))
                                       : nullptr;
            } else {
                act[l] = (T *)a.take(3 * B * y.ldK * sizeof(T));
                y.patches = y.patchesT = y.dpatch = nullptr;
                y.f_split = 1; y.f_chunk = y.ldK; y.f_part = nullptr;
                if (sizeof(T) == 2 && l + 1 < L && y.ldK % 64 == 0 && y.O >= 128 && y.O % 4 == 0) {
                    const long tiles = (long)((y.O + 255) / 256) * ((3 * B + 63) / 64);
                    const int stages = y.ldK / 64;
                    if (tiles < 64 && stages >= 16) {   // a long contraction on a few blocks
                        int fs = (int)(256 / tiles);
                        if (fs > 8) fs = 8;
                        if (fs > stages / 4) fs = stages / 4;
                        y.f_chunk = (stages + fs - 1) / fs * 64;
                        y.f_split = (y.ldK + y.f_chunk - 1) / y.f_chunk;
                        y.f_part = (float *)a.take((size_t)y.f_split * 3 * B * y.O * 4);
                    }
                }
                y.XT = (T *)a.take((size_t)y.K * ldB * sizeof(T));
                y.dZ = (T *)a.take(B * y.ldO * sizeof(T));
                y.dZT = (T *)a.take((size_t)y.O * ldB * sizeof(T));
            }
        }
        act_bytes = a.off - act0;
        Qout = (float *)a.take(3 * B * ldA * 4);
        astar = (int32_t *)a.take(B * 4);
        loss_part = (float *)a.take((size_t)((Bmax + kHeadRows - 1) / kHeadRows) * 4);
        stats_internal = (tj_step_stats *)a.take(sizeof(tj_step_stats));
        return a.off;
    }

    // Master state (theta, m, v, grad) is kept in the kernels' own order: per layer W[O][k] with
    // k = s*C + c (s = kernel position or, for a linear layer after a convolution, pixel), then the
    // bias.  The caller's order W[O][C][S] appears only in get_state / set_state.
    void permute_host(const float *src, float *dst, bool to_internal) const
    {
        for (int l = 0; l < L; ++l) {
            const NLayer &y = lay[l];
            for (int o = 0; o < y.O; ++o)
                for (int c = 0; c < y.C; ++c)
                    for (int s = 0; s < y.S; ++s) {
                        const size_t user = y.w_off + ((size_t)o * y.C + c) * y.S + s;
                        const size_t mine = y.w_off + (size_t)o * y.K + (size_t)s * y.C + c;
                        if (to_internal) dst[mine] = src[user]; else dst[user] = src[mine];
                    }
            for (int o = 0; o < y.O; ++o) dst[y.b_off + o] = src[y.b_off + o];
        }
    }

    // Adam writes the straight copy of every weight block whose rows need no padding
    bool adam_emits(int l) const { return lay[l].ldK == lay[l].K; }

    // fp32 master -> compute-type copies (and the transposes the input-gradient GEMMs contract over)
    int recast(bool online, hipStream_t st, bool after_adam = false)
    {
        CastJobs<T> jobs;
        int n = 0;
        for (int l = 0; l < L; ++l) {
            NLayer &y = lay[l];
            CastJob<T> j;
            j.src = (online ? theta_on : theta_tg) + y.w_off;
            j.dst = online ? y.Wc_on : y.Wc_tg;
            if (after_adam && adam_emits(l)) j.dst = nullptr;
            j.dstT = (online && keeps_wct(l)) ? y.WcT_on : nullptr;
            j.R = y.O; j.C = y.K; j.ldd = y.ldK; j.lddT = y.ldO;
            if (j.dst || j.dstT) jobs.job[n++] = j;
        }
        if constexpr (sizeof(T) == 2) {
            if (online && !after_adam) {   // after an update the optimizer kernel has refreshed them
                tjconv::DgradWeightJobs dj;
                dj.n_job = 0;
                dj.block_begin[0] = 0;
                for (int l = 0; l < L; ++l) {
                    NLayer &y = lay[l];
                    if (!y.dgrad_gather) continue;
                    const int q = dj.n_job++;
                    dj.w[q] = theta_on + y.w_off; dj.wd[q] = y.Wd;
                    dj.O[q] = y.O; dj.C[q] = y.g.C; dj.k[q] = y.g.k; dj.s[q] = y.g.s; dj.A[q] = y.A;
                    dj.block_begin[q + 1] = dj.block_begin[q] + (unsigned)(((size_t)y.Nd * y.Kd + 255) / 256);
                }
                if (dj.n_job > 0) {
                    tjconv::dgrad_weights<<<dj.block_begin[dj.n_job], 256, 0, st>>>(dj);
                    if (hipGetLastError() != hipSuccess) return TJ_ERR_DEVICE;
                }
            }
        }
        return launch_cast<T>(jobs, n, st);
    }

    static dim3 grid1(size_t n) { return dim3((unsigned)((n + 255) / 256)); }

    // A hidden linear layer's weight gradient straight from the row-major input rows and dZ (transposing LDS
    // reads, as in the MLP learner): bf16, whole 32-row stages of the batch, widths that are whole 16-byte
    // vectors and fill 256 x 128 tiles.  Such a layer needs neither the transposed input nor dZ^T.
    bool lin_wgrad_trans(int l, int B) const
    {
        if (sizeof(T) != 2 || l < 1 || l >= L - 1 || lay[l].kind != TJ_LAYER_LINEAR) return false;
        return B % 32 == 0 && B >= 1024 && lay[l].K % 8 == 0 && lay[l].O % 8 == 0 && lay[l].K >= 256 && lay[l].O >= 128;
    }

    // A linear layer's input gradient with the row-major weight copy as its first operand (transposing LDS
    // reads): bf16, a contraction over whole 32-row stages of the weight matrix, batches large enough for the
    // 256 x 128 tiles that form takes.  Decided by the largest batch, so that the set of weight copies is fixed.
    bool lin_dgrad_trans(int l) const
    {
        if (sizeof(T) != 2 || l < 1 || lay[l].kind != TJ_LAYER_LINEAR || Bmax < 1024) return false;
        return lay[l].K % 8 == 0 && lay[l].O % 32 == 0;
    }
    // Layer l keeps a transposed weight copy: its input gradient exists and is a contraction over that copy (a
    // convolution's is one only on the explicit patch path; the head's is not where the TD kernel writes it).
    virtual bool head_input_gradient_fused() const { return false; }   // a derived learner's head kernel reads WcT
    bool keeps_wct(int l) const
    {
        if (l == 0) return false;
        if (l == L - 1 && head_input_gradient_fused()) return true;
        const NLayer &y = lay[l];
        if (y.kind == TJ_LAYER_CONV2D) return !y.dgrad_gather;
        if (l == L - 1 && head_fused<T>(A) && L >= 2 && lay[L - 2].kind == TJ_LAYER_LINEAR) return false;
        return !lin_dgrad_trans(l);
    }

    int transpose(const T *src, int lds, T *dst, int ldd, int R, int Cc, hipStream_t st)
    {
        if constexpr (sizeof(T) == 2) {
            if (lds % 8 == 0 && ldd % 8 == 0 && Cc % 8 == 0 && ldd >= round_up(R, 8) &&
                (((uintptr_t)src | (uintptr_t)dst) & 15) == 0) {
                dim3 g64((Cc + 63) / 64, (R + 63) / 64);
                tjconv::transpose2d_v8<<<g64, 256, 0, st>>>((const uint16_t *)src, lds, (uint16_t *)dst, ldd, R, Cc);
                return hipGetLastError() == hipSuccess ? TJ_OK : TJ_ERR_DEVICE;
            }
        }
        dim3 grid((Cc + 31) / 32, (R + 31) / 32);
        tjconv::transpose2d<T><<<grid, 256, 0, st>>>(src, lds, dst, ldd, R, Cc);
        return hipGetLastError() == hipSuccess ? TJ_OK : TJ_ERR_DEVICE;
    }

    int step(const tj_minibatch *mb, tj_step_stats *d_stats, hipStream_t st) override
    {
        const int B = (int)mb->batch;
        if (B < 1 || B > Bmax) return TJ_ERR_SHAPE;
        if (!mb->obs || !mb->next_obs || !mb->action || !mb->reward || !mb->done) return TJ_ERR_INVALID_ARG;
        if ((mb->row_index || mb->plane_index) && (mb->n_rows == 0 || mb->n_rows > 0xFFFFFFFFull))
            return TJ_ERR_INVALID_ARG;
        if (mb->row_index && mb->plane_index) return TJ_ERR_INVALID_ARG;
        int rc;
        if (last_batch != B) {
            if (last_batch > B && (rc = launch_zero(act_begin, act_bytes, st)) != TJ_OK) return rc;
            last_batch = B;
        }
        const int Kb = round_up(B, VE);

        bool first_done = false;
        if constexpr (sizeof(T) == 2) {
            if (first_fused && (((uintptr_t)mb->obs | (uintptr_t)mb->next_obs) & 3) == 0) {
                const tjconv::ConvGeom &g = lay[0].g;
                TjConvFirstArgs fa;
                fa.obs = (const uint8_t *)mb->obs; fa.next_obs = (const uint8_t *)mb->next_obs;
                fa.B = B; fa.H = g.H; fa.W = g.W; fa.k = g.k; fa.s = g.s; fa.OH = g.OH; fa.OW = g.OW;
                fa.W_on = lay[0].Wc_on; fa.W_tg = lay[0].Wc_tg;
                fa.b_on = theta_on + lay[0].b_off; fa.b_tg = theta_tg + lay[0].b_off;
                fa.act0 = first_wgrad_u8 ? nullptr : act[0]; fa.out = act[1];
                fa.scale = 1.0f / 255.0f;
                fa.rows = mb->row_index; fa.n_rows = (uint32_t)mb->n_rows; fa.planes = mb->plane_index;
                if ((rc = mark(0, st)) != TJ_OK) return rc;
                if ((rc = tj_conv_first(fa, st)) != TJ_OK) return rc;
                first_done = true;
            }
        }
        if (!first_done) {   // observations -> channels-last compute type, images s | s'
            const tjconv::ConvGeom &g = lay[0].g;
            const size_t px = (size_t)B * g.H * g.W, img = (size_t)g.H * g.W * g.C;
            const uint32_t *rows = mb->row_index;
            const uint32_t n_rows = (uint32_t)mb->n_rows;
            // by planes: channel c of s_j is plane_index[2C j + c], of s'_j plane_index[2C j + C + c]
            const uint32_t *pl_s = mb->plane_index, *pl_n = mb->plane_index ? mb->plane_index + g.C : nullptr;
            bool fast = false;
            if constexpr (sizeof(T) == 2) {
                fast = d.obs_dtype == TJ_OBS_U8 && g.C == 4 && (g.H * g.W) % 8 == 0 &&
                       (((uintptr_t)mb->obs | (uintptr_t)mb->next_obs) & 7) == 0;
                if (fast) {
                    const size_t groups = (size_t)B * (g.H * g.W / 8);
                    tjconv::to_nhwc_u8c4<<<grid1(groups), 256, 0, st>>>((const uint8_t *)mb->obs, act[0], (size_t)B,
                                                                        g.H * g.W, 1.0f / 255.0f, rows, n_rows, pl_s);
                    tjconv::to_nhwc_u8c4<<<grid1(groups), 256, 0, st>>>((const uint8_t *)mb->next_obs,
                                                                        act[0] + (size_t)B * img, (size_t)B,
                                                                        g.H * g.W, 1.0f / 255.0f, rows, n_rows, pl_n);
                }
            }
            if (fast) {
            } else if (d.obs_dtype == TJ_OBS_U8) {
                tjconv::to_nhwc<T, uint8_t><<<grid1(px), 256, 0, st>>>((const uint8_t *)mb->obs, act[0], B, g.C, g.H,
                                                                       g.W, 1.0f / 255.0f, rows, n_rows, pl_s);
                tjconv::to_nhwc<T, uint8_t><<<grid1(px), 256, 0, st>>>((const uint8_t *)mb->next_obs,
                                                                       act[0] + (size_t)B * img, B, g.C, g.H, g.W,
                                                                       1.0f / 255.0f, rows, n_rows, pl_n);
            } else {
                tjconv::to_nhwc<T, float><<<grid1(px), 256, 0, st>>>((const float *)mb->obs, act[0], B, g.C, g.H, g.W,
                                                                     1.0f, rows, n_rows, pl_s);
                tjconv::to_nhwc<T, float><<<grid1(px), 256, 0, st>>>((const float *)mb->next_obs,
                                                                     act[0] + (size_t)B * img, B, g.C, g.H, g.W, 1.0f,
                                                                     rows, n_rows, pl_n);
            }
            if (hipGetLastError() != hipSuccess) return TJ_ERR_DEVICE;
            if ((rc = mark(0, st)) != TJ_OK) return rc;
        }

        // ---- forward
        for (int l = first_done ? 1 : 0; l < L; ++l) {
            NLayer &y = lay[l];
            if (y.kind == TJ_LAYER_CONV2D) {
                const tjconv::ConvGeom &g = y.g;
                const size_t n_img = l == 0 ? 2 * (size_t)B : 3 * (size_t)B;
                const size_t rows = n_img * y.OHW, Ms = (size_t)B * y.OHW;
                const int run = g.k * g.C;
                if (!y.implicit) {
                    const bool vec = sizeof(T) == 2 && run % 8 == 0 && (g.s * g.C) % 8 == 0 &&
                                     (g.W * g.C) % 8 == 0 && y.ldK % 8 == 0;
                    if (vec)
                        tjconv::im2col<T, 8><<<grid1(rows * g.k * (run / 8)), 256, 0, st>>>(act[l], y.patches, g, rows, y.ldK);
                    else
                        tjconv::im2col<T, 1><<<grid1(rows * g.k * run), 256, 0, st>>>(act[l], y.patches, g, rows, y.ldK);
                    dim3 grid((unsigned)((Ms + 255) / 256), (unsigned)y.K);
                    tjconv::im2col_t<T><<<grid, 256, 0, st>>>(act[l], y.patchesT, g, Ms,
                                                              round_up((int)((size_t)Bmax * y.OHW), VE));
                    if (hipGetLastError() != hipSuccess) return TJ_ERR_DEVICE;
                }
                TjGemmArgs<T> both[2];
                for (int net = 0; net < 2; ++net) {   // online on s and s', target on s'
                    const size_t row0 = net == 0 ? 0 : (l == 0 ? Ms : 2 * Ms);
                    const size_t nrow = net == 0 ? 2 * Ms : Ms;
                    TjGemmArgs<T> &gm = both[net];
                    memset(&gm, 0, sizeof(gm));
                    gm.n_seg = 1;
                    if (y.implicit) {   // patches gathered from the images themselves
                        const size_t img0 = row0 / y.OHW;
                        gm.seg[0] = {0, y.O, act[l] + img0 * (size_t)g.H * g.W * g.C, nullptr, 0};
                        gm.gather = y.gth;
                    } else {
                        gm.seg[0] = {0, y.O, y.patches + row0 * y.ldK, nullptr, 0};
                    }
                    gm.Q = net == 0 ? y.Wc_on : y.Wc_tg;
                    gm.ldp = y.ldK; gm.ldq = y.ldK;
                    gm.I = (int)nrow; gm.K = y.ldK; gm.k_chunk = gm.K; gm.n_split = 1;
                    gm.bias_j = (net == 0 ? theta_on : theta_tg) + y.b_off;
                    gm.relu = 1;
                    gm.Cj = act[l + 1] + (net == 0 ? 0 : 2 * Ms * y.O); gm.ldcj = y.O; gm.cj_jmax = y.O;
                }
                bool paired = false;
                if constexpr (sizeof(T) == 2) {
                    if (y.implicit) {   // the two networks' passes share one launch
                        if ((rc = tj_gemm_gather_pair(both[0], both[1], st)) != TJ_OK) return rc;
                        paired = true;
                    }
                }
                if (!paired)
                    for (int net = 0; net < 2; ++net)
                        if ((rc = tj_gemm<T>(both[net], st)) != TJ_OK) return rc;
            } else {
                if (l > 0 && lay[l - 1].kind == TJ_LAYER_CONV2D && !lin_wgrad_trans(l, B))   // transposed input of the s rows
                    if ((rc = transpose(act[l], y.ldK, y.XT, ldB, B, y.K, st)) != TJ_OK) return rc;
                TjGemmArgs<T> gm;
                memset(&gm, 0, sizeof(gm));
                gm.n_seg = 2;
                gm.seg[0] = {0, 2 * B, y.Wc_on, theta_on + y.b_off, 0};
                gm.seg[1] = {2 * B, 3 * B, y.Wc_tg, theta_tg + y.b_off, 0};
                gm.Q = act[l];
                gm.ldp = y.ldK; gm.ldq = y.ldK;
                gm.I = y.O; gm.K = y.ldK; gm.k_chunk = gm.K; gm.n_split = 1;
                if (l + 1 == L) break;   // the head layer runs with the TD step below
                if (y.f_split > 1) {   // split contraction: partial sums, then bias + ReLU + both layouts
                    gm.seg[0].bias = nullptr; gm.seg[1].bias = nullptr;
                    gm.n_split = y.f_split; gm.k_chunk = y.f_chunk;
                    gm.Cf = y.f_part; gm.ldcf = y.O; gm.cf_zstride = (size_t)3 * B * y.O;
                    if ((rc = tj_gemm<T>(gm, st)) != TJ_OK) return rc;
                    const size_t nvec = (size_t)3 * B * (y.O / 4);
                    sum_bias_relu<T><<<grid1(nvec), 256, 0, st>>>(y.f_part, gm.cf_zstride, y.f_split, 3 * B, y.O,
                                                               theta_on + y.b_off, theta_tg + y.b_off, 2 * B,
                                                               act[l + 1], lay[l + 1].ldK, lay[l + 1].XT, ldB, B);
                    if (hipGetLastError() != hipSuccess) return TJ_ERR_DEVICE;
                    continue;
                }
                gm.relu = 1;
                gm.Ci = act[l + 1]; gm.ldci = lay[l + 1].ldK;
                if (!lin_wgrad_trans(l + 1, B)) { gm.Cj = lay[l + 1].XT; gm.ldcj = ldB; gm.cj_jmax = B; }
                if ((rc = tj_gemm<T>(gm, st)) != TJ_OK) return rc;
            }
        }
        bool head_dx_done = false;
        {   // head layer and TD step
            NLayer &y = lay[L - 1];
            HeadTd<T> h;
            h.X = act[L - 1]; h.ldx = y.ldK;
            h.row0[0] = 0; h.row0[1] = B; h.row0[2] = 2 * B;
            h.W_on = y.Wc_on; h.W_tg = y.Wc_tg; h.ldw = y.ldK;
            h.b_on = theta_on + y.b_off; h.b_tg = theta_tg + y.b_off;
            h.B = B; h.A = A; h.K = y.ldK;
            h.Q = Qout; h.ldq = ldA;
            h.dZ = y.dZ; h.lddz = y.ldO; h.dZT = y.dZT; h.lddzt = ldB;
            h.astar = astar; h.loss_part = loss_part;
            h.dX = nullptr; h.lddx = 0; h.dXT = nullptr; h.lddxt = 0; h.Kin = y.K;
            head_dx_done = head_fused<T>(A) && L >= 2 && lay[L - 2].kind == TJ_LAYER_LINEAR;
            if (head_dx_done) {   // the fused kernel also writes the head's input gradient
                h.dX = lay[L - 2].dZ; h.lddx = y.ldK;
                if (!lin_wgrad_trans(L - 2, B)) { h.dXT = lay[L - 2].dZT; h.lddxt = ldB; }
            }
            if ((rc = run_head_td<T>(this, h, mb, d.gamma, d.huber_delta, st)) != TJ_OK) return rc;
        }
        if ((rc = mark(2, st)) != TJ_OK) return rc;

        // ---- backward through Q_online(s)
        // the partial weight gradients of all layers are summed by one launch after the loop
        tjconv::ReduceJobs jobs;
        jobs.n_job = 0;
        jobs.block_begin[0] = 0;
        auto add_reduce_job = [&](const float *part, size_t zstride, int n_part, float *dst, size_t n) {
            const int q = jobs.n_job++;
            jobs.part[q] = part; jobs.zstride[q] = zstride; jobs.n_part[q] = n_part; jobs.dst[q] = dst; jobs.n[q] = n;
            jobs.block_begin[q + 1] = jobs.block_begin[q] + tjconv::reduce_blocks(n, n_part);
        };
        for (int l = L - 1; l >= 0; --l) {
            NLayer &y = lay[l];
            const bool conv = y.kind == TJ_LAYER_CONV2D;
            const size_t Ms = (size_t)B * y.OHW;
            const int Kc = conv ? round_up((int)Ms, VE) : Kb;      // contraction of the weight gradient
            const int ldm = conv ? round_up((int)((size_t)Bmax * y.OHW), VE) : ldB;
            bool wgrad_done = false;
            if constexpr (sizeof(T) == 2) {
                if (l == 0 && first_done && first_wgrad_u8) {   // from the u8 stacks, one slice per block
                    if (n_cu == 0) {
                        int dev = 0, v = 0;
                        n_cu = 256;
                        if (hipGetDevice(&dev) == hipSuccess &&
                            hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0)
                            n_cu = v;
                    }
                    const tjconv::ConvGeom &g = y.g;
                    TjConvFirstWgradArgs wa;
                    wa.obs = (const uint8_t *)mb->obs; wa.dZ = y.dZ;
                    wa.B = B; wa.H = g.H; wa.W = g.W; wa.k = g.k; wa.s = g.s; wa.OH = g.OH; wa.OW = g.OW;
                    wa.scale = 1.0f / 255.0f;
                    wa.rows = mb->row_index; wa.n_rows = (uint32_t)mb->n_rows; wa.planes = mb->plane_index;
                    wa.part = y.part; wa.zstride = y.part_stride;
                    wa.n_part = std::min(B, std::min(n_cu, y.n_split));
                    if ((rc = tj_conv_first_wgrad(wa, st)) != TJ_OK) return rc;
                    add_reduce_job(y.part, y.part_stride, wa.n_part, grad + y.w_off, (size_t)y.O * y.K + y.O);
                    wgrad_done = true;
                }
                if (!wgrad_done && conv && y.implicit) {   // straight from dZ and the layer input
                    TjConvWgradArgs wa;
                    wa.dZ = y.dZ; wa.O = y.O; wa.act = act[l]; wa.g = y.gth;
                    wa.M = (int)Ms; wa.K = y.K;
                    wa.part = y.part; wa.zstride = y.part_stride;
                    wa.n_split = y.n_split;
                    wa.m_chunk = round_up((int)((Ms + y.n_split - 1) / y.n_split), 64);
                    if ((rc = tj_conv_wgrad(wa, st)) != TJ_OK) return rc;
                    add_reduce_job(y.part, y.part_stride, y.n_split, grad + y.w_off, (size_t)y.O * y.K + y.O);
                    wgrad_done = true;
                }
            }
            TjGemmArgs<T> gw;            // a linear layer's weight gradient waits for its input gradient:
            bool gw_pending = false;     // the two share one launch (bf16)
            if (!wgrad_done) {   // dW[o][k] = sum_m dZ[m][o] X[m][k] (k in kernel order), db[o] = sum_m dZ[m][o]
                TjGemmArgs<T> &gm = gw;
                memset(&gm, 0, sizeof(gm));
                gm.n_seg = 1;
                if (lin_wgrad_trans(l, B)) {   // row-major operands, contraction over their rows
                    gm.seg[0] = {0, y.O, act[l], nullptr, 0};
                    gm.Q = y.dZ;
                    gm.ldp = y.ldK; gm.ldq = y.ldO;
                    gm.trans = 1;
                } else {
                    gm.seg[0] = {0, y.O, conv ? y.patchesT : y.XT, nullptr, 0};
                    gm.Q = y.dZT;
                    gm.ldp = ldm;   // pitches follow the largest batch, so pad columns are never written
                    gm.ldq = ldm;
                }
                gm.I = y.K; gm.K = Kc;
                int ns = y.n_split;
                const int ke = 128 / (int)sizeof(T);
                gm.k_chunk = round_up((Kc + ns - 1) / ns, ke);
                gm.n_split = ns;
                gm.Cf = y.part; gm.ldcf = y.K; gm.cf_zstride = y.part_stride;
                gm.qsum = y.part + (size_t)y.O * y.K; gm.qsum_zstride = y.part_stride;
                gw_pending = sizeof(T) == 2 && !conv && l > 0 && !(l == L - 1 && head_dx_done);
                if (!gw_pending && (rc = tj_gemm<T>(gm, st)) != TJ_OK) return rc;
                add_reduce_job(y.part, y.part_stride, ns, grad + y.w_off, (size_t)y.O * y.K + y.O);
            }
            if (l == 0) break;
            NLayer &below = lay[l - 1];
            if (l == L - 1 && head_dx_done) continue;   // written by the TD kernel
            if (!conv) {   // dX[m][k] = relu'(X) * sum_o dZ[m][o] W[o][k]
                TjGemmArgs<T> gm;
                memset(&gm, 0, sizeof(gm));
                gm.n_seg = 1;
                gm.Q = y.dZ;
                gm.ldq = y.ldO;
                gm.I = y.K;
                if (lin_dgrad_trans(l)) {   // the weights as stored, [o][k]: the contraction runs over their rows
                    gm.seg[0] = {0, B, y.Wc_on, nullptr, 0};
                    gm.ldp = y.ldK; gm.K = y.O;
                    gm.trans = 2;
                } else {
                    gm.seg[0] = {0, B, y.WcT_on, nullptr, 0};
                    gm.ldp = y.ldO; gm.K = y.ldO;
                }
                gm.k_chunk = gm.K; gm.n_split = 1;
                gm.mask = act[l]; gm.ldmask = y.ldK;
                gm.Ci = below.dZ; gm.ldci = y.ldK;
                if (below.kind == TJ_LAYER_LINEAR && !lin_wgrad_trans(l - 1, B)) {
                    gm.Cj = below.dZT; gm.ldcj = ldB; gm.cj_jmax = B;
                }
                if constexpr (sizeof(T) == 2) {
                    if (gw_pending) {
                        if ((rc = tj_gemm_pair(gw, gm, st)) != TJ_OK) return rc;
                        gw_pending = false;
                    } else if ((rc = tj_gemm<T>(gm, st)) != TJ_OK) {
                        return rc;
                    }
                } else {
                    if ((rc = tj_gemm<T>(gm, st)) != TJ_OK) return rc;
                }
            } else if (y.dgrad_gather) {
                // dX[img, s yy + py, s xx + px, c] = sum_{a,b,o} dZ0[img, yy + a, xx + b, o] * Wd[(py,px,c)][(a,b,o)],
                // dZ0 = the output gradient with a zero border of A-1: a stride-1 gathered GEMM whose row is a
                // coarse position (yy, xx) and whose columns are the s x s pixel block times the channels
                if constexpr (sizeof(T) == 2) {
                    const tjconv::ConvGeom &g = y.g;
                    const size_t np = (size_t)B * g.OH * g.OW * (y.O / 8);
                    tjconv::pad_halo<<<grid1(np), 256, 0, st>>>(y.dZ, y.dZh, (size_t)B, g.OH, g.OW, y.O, y.pad);
                    if (hipGetLastError() != hipSuccess) return TJ_ERR_DEVICE;
                    TjGemmArgs<T> gm;
                    memset(&gm, 0, sizeof(gm));
                    gm.n_seg = 1;
                    gm.seg[0] = {0, y.Nd, y.dZh, nullptr, 0};
                    gm.gather = y.dg_in;
                    gm.Q = y.Wd;
                    gm.ldp = y.Kd; gm.ldq = y.Kd;
                    gm.I = B * (g.H / g.s) * (g.W / g.s); gm.K = y.Kd; gm.k_chunk = gm.K; gm.n_split = 1;
                    gm.out_map = y.dg_out;
                    gm.Cj = below.dZ; gm.cj_jmax = y.Nd;
                    gm.mask_cj = act[l];
                    if ((rc = tj_gemm<T>(gm, st)) != TJ_OK) return rc;
                }
            } else {       // patch gradients, then the gather back onto the input pixels with the ReLU mask
                TjGemmArgs<T> gm;
                memset(&gm, 0, sizeof(gm));
                gm.n_seg = 1;
                gm.seg[0] = {0, y.K, y.dZ, nullptr, 0};
                gm.Q = y.WcT_on;
                gm.ldp = y.O; gm.ldq = y.ldO;
                gm.I = (int)Ms; gm.K = y.O; gm.k_chunk = gm.K; gm.n_split = 1;
                gm.Cj = y.dpatch; gm.ldcj = y.ldK; gm.cj_jmax = y.K;
                if ((rc = tj_gemm<T>(gm, st)) != TJ_OK) return rc;
                const size_t n = (size_t)B * y.g.H * y.g.W * y.g.C;
                bool v8 = false;
                if constexpr (sizeof(T) == 2) {
                    v8 = y.g.C % 8 == 0 && y.ldK % 8 == 0;
                    if (v8)
                        tjconv::col2im_mask_v8<<<grid1(n / 8), 256, 0, st>>>(y.dpatch, y.ldK, act[l], below.dZ, y.g,
                                                                            (size_t)B);
                }
                if (!v8)
                    tjconv::col2im_mask<T><<<grid1(n), 256, 0, st>>>(y.dpatch, y.ldK, act[l], below.dZ, y.g, (size_t)B);
                if (hipGetLastError() != hipSuccess) return TJ_ERR_DEVICE;
            }
            if (below.kind == TJ_LAYER_CONV2D && !below.implicit) {   // dZ^T of a conv layer: [OC][B*OH*OW]
                const int Mb = (int)((size_t)B * below.OHW);
                if ((rc = transpose(below.dZ, below.O, below.dZT, round_up((int)((size_t)Bmax * below.OHW), VE), Mb,
                                    below.O, st)) != TJ_OK)
                    return rc;
            }
        }
        tjconv::reduce_parts<<<jobs.block_begin[jobs.n_job], 256, 0, st>>>(jobs);
        if (hipGetLastError() != hipSuccess) return TJ_ERR_DEVICE;
        if ((rc = mark(3, st)) != TJ_OK) return rc;

        t += 1;
        const float c1 = (float)(1.0 - pow((double)d.beta1, (double)t));
        const float c2 = (float)(1.0 - pow((double)d.beta2, (double)t));
        EmitTable<T> tab;
        tab.n = 0;
        for (int l = 0; l < L; ++l) {
            if (!adam_emits(l)) continue;
            tab.begin[tab.n] = lay[l].w_off;
            tab.end[tab.n] = lay[l].w_off + (size_t)lay[l].O * lay[l].K;
            tab.dstT[tab.n] = nullptr; tab.C[tab.n] = 0; tab.ldT[tab.n] = 0;
            tab.dst[tab.n++] = lay[l].Wc_on;
        }
        const LossFinal lf = {loss_part, td_blocks<T>(B, A), B, (uint32_t)t, d_stats, stats_internal};
        DgradEmit dg;   // the convolutions' input-gradient weights follow their master weights in the same kernel
        dg.n = 0;
        if constexpr (sizeof(T) == 2) {
            for (int l = 0; l < L; ++l) {
                const NLayer &y = lay[l];
                if (!y.dgrad_gather) continue;
                const int q = dg.n++;
                dg.begin[q] = y.w_off; dg.end[q] = y.w_off + (size_t)y.O * y.K;
                dg.wd[q] = y.Wd;
                dg.O[q] = y.O; dg.C[q] = y.g.C; dg.k[q] = y.g.k; dg.s[q] = y.g.s; dg.A[q] = y.A;
            }
        }
        adam_update<T><<<(unsigned)((P + 1023) / 1024), 256, 0, st>>>(theta_on, m, v, grad, 1, Ppad, P, d.lr, d.beta1,
                                                                      d.beta2, d.eps, c1, c2, tab, lf, dg, 0, 0, 1);
        if (hipGetLastError() != hipSuccess) return TJ_ERR_DEVICE;
        if ((rc = mark(4, st)) != TJ_OK) return rc;
        if ((rc = recast(true, st, true)) != TJ_OK) return rc;
        if (d.target_interval && t % d.target_interval == 0) {
            TJ_HIP_TRY(hipMemcpyAsync(theta_tg, theta_on, P * 4, hipMemcpyDeviceToDevice, st));
            TJ_HIP_TRY(hipMemcpyAsync(wc_tg_begin, wc_on_begin, wc_bytes, hipMemcpyDeviceToDevice, st));
        }
        return TJ_OK;
    }

    // Policy inference on n <= 2*Bmax observations with the online network, in the step's buffers.
    int infer(uint32_t n_, const void *d_obs, float epsilon, uint64_t seed, int32_t *d_action, int32_t *d_version,
            float *d_q, hipStream_t st) override
    {
        const int n = (int)n_;
        if (n < 1 || n > 2 * Bmax) return TJ_ERR_SHAPE;
        if (!d_obs || !d_action || !d_version || !(epsilon >= 0.f && epsilon <= 1.f)) return TJ_ERR_INVALID_ARG;
        int rc;
        {
            const tjconv::ConvGeom &g = lay[0].g;
            const size_t px = (size_t)n * g.H * g.W;
            bool fast = false;
            if constexpr (sizeof(T) == 2) {
                fast = d.obs_dtype == TJ_OBS_U8 && g.C == 4 && (g.H * g.W) % 8 == 0 && ((uintptr_t)d_obs & 7) == 0;
                if (fast)
                    tjconv::to_nhwc_u8c4<<<grid1((size_t)n * (g.H * g.W / 8)), 256, 0, st>>>(
                        (const uint8_t *)d_obs, act[0], (size_t)n, g.H * g.W, 1.0f / 255.0f, nullptr, 0u, nullptr);
            }
            if (!fast) {
                if (d.obs_dtype == TJ_OBS_U8)
                    tjconv::to_nhwc<T, uint8_t><<<grid1(px), 256, 0, st>>>((const uint8_t *)d_obs, act[0], n, g.C, g.H,
                                                                           g.W, 1.0f / 255.0f, nullptr, 0u, nullptr);
                else
                    tjconv::to_nhwc<T, float><<<grid1(px), 256, 0, st>>>((const float *)d_obs, act[0], n, g.C, g.H, g.W,
                                                                         1.0f, nullptr, 0u, nullptr);
            }
            if (hipGetLastError() != hipSuccess) return TJ_ERR_DEVICE;
        }
        for (int l = 0; l < L; ++l) {
            NLayer &y = lay[l];
            TjGemmArgs<T> gm;
            memset(&gm, 0, sizeof(gm));
            gm.n_seg = 1;
            gm.ldp = y.ldK; gm.ldq = y.ldK;
            gm.K = y.ldK; gm.k_chunk = gm.K; gm.n_split = 1;
            if (y.kind == TJ_LAYER_CONV2D) {
                const tjconv::ConvGeom &g = y.g;
                const size_t rows = (size_t)n * y.OHW;
                if (y.implicit) {
                    gm.seg[0] = {0, y.O, act[l], nullptr, 0};
                    gm.gather = y.gth;
                } else {
                    const int run = g.k * g.C;
                    const bool vec = sizeof(T) == 2 && run % 8 == 0 && (g.s * g.C) % 8 == 0 &&
                                     (g.W * g.C) % 8 == 0 && y.ldK % 8 == 0;
                    if (vec)
                        tjconv::im2col<T, 8><<<grid1(rows * g.k * (run / 8)), 256, 0, st>>>(act[l], y.patches, g, rows, y.ldK);
                    else
                        tjconv::im2col<T, 1><<<grid1(rows * g.k * run), 256, 0, st>>>(act[l], y.patches, g, rows, y.ldK);
                    if (hipGetLastError() != hipSuccess) return TJ_ERR_DEVICE;
                    gm.seg[0] = {0, y.O, y.patches, nullptr, 0};
                }
                gm.Q = y.Wc_on;
                gm.I = (int)rows;
                gm.bias_j = theta_on + y.b_off;
                gm.relu = 1;
                gm.Cj = act[l + 1]; gm.ldcj = y.O; gm.cj_jmax = y.O;
            } else {
                gm.seg[0] = {0, n, y.Wc_on, theta_on + y.b_off, 0};
                gm.Q = act[l];
                gm.I = y.O;
                if (l + 1 < L) {
                    gm.relu = 1;
                    gm.Ci = act[l + 1]; gm.ldci = lay[l + 1].ldK;
                } else {
                    gm.Cf = Qout; gm.ldcf = ldA;
                }
            }
            if ((rc = tj_gemm<T>(gm, st)) != TJ_OK) return rc;
        }
        egreedy<<<(n + 255) / 256, 256, 0, st>>>(Qout, ldA, (uint32_t)n, A, egreedy_threshold(epsilon), seed,
                                                 (int32_t)t, d_action, d_version, d_q);
        return hipGetLastError() == hipSuccess ? TJ_OK : TJ_ERR_DEVICE;
    }

    int get_state(int which, float *h_out, size_t n, hipStream_t st) override
    {
        const float *src = nullptr;
        switch (which) {
        case TJ_STATE_PARAMS: src = theta_on; break;
        case TJ_STATE_TARGET: src = theta_tg; break;
        case TJ_STATE_ADAM_M: src = m; break;
        case TJ_STATE_ADAM_V: src = v; break;
        case TJ_STATE_GRADS: src = grad; break;
        default: break;
        }
        if (src) {
            if (n != P) return TJ_ERR_INVALID_ARG;
            std::vector<float> tmp(P);
            TJ_HIP_TRY(hipMemcpyAsync(tmp.data(), src, P * 4, hipMemcpyDeviceToHost, st));
            TJ_HIP_TRY(hipStreamSynchronize(st));
            permute_host(tmp.data(), h_out, false);
            return TJ_OK;
        }
        if (which == TJ_STATE_WEIGHTS_COMPUTE || which == TJ_STATE_WEIGHTS_COMPUTE_T ||
            which == TJ_STATE_WEIGHTS_COMPUTE_TARGET) {
            if (n != P) return TJ_ERR_INVALID_ARG;
            const bool tg = which == TJ_STATE_WEIGHTS_COMPUTE_TARGET, tr = which == TJ_STATE_WEIGHTS_COMPUTE_T;
            std::vector<float> tmp(P), w;
            TJ_HIP_TRY(hipMemcpyAsync(tmp.data(), tg ? theta_tg : theta_on, P * 4, hipMemcpyDeviceToHost, st));   // biases
            TJ_HIP_TRY(hipStreamSynchronize(st));
            for (int l = 0; l < L; ++l) {
                const NLayer &y = lay[l];
                float *dst = tmp.data() + y.w_off;   // the kernels' order [O][k]
                int rc;
                if (tr && keeps_wct(l)) {
                    if ((rc = fetch_as_float<T>(y.WcT_on, (size_t)y.K * y.ldO, w, st)) != TJ_OK) return rc;
                    for (int o = 0; o < y.O; ++o)
                        for (int k = 0; k < y.K; ++k) dst[(size_t)o * y.K + k] = w[(size_t)k * y.ldO + o];
                } else {
                    if ((rc = fetch_as_float<T>(tg ? y.Wc_tg : y.Wc_on, (size_t)y.O * y.ldK, w, st)) != TJ_OK) return rc;
                    for (int o = 0; o < y.O; ++o)
                        for (int k = 0; k < y.K; ++k) dst[(size_t)o * y.K + k] = w[(size_t)o * y.ldK + k];
                }
            }
            permute_host(tmp.data(), h_out, false);
            return TJ_OK;
        }
        if (which == TJ_STATE_QVALS) {
            if (last_batch < 1 || n != 3 * (size_t)last_batch * A) return TJ_ERR_INVALID_ARG;
            std::vector<float> tmp(3 * (size_t)last_batch * ldA);
            TJ_HIP_TRY(hipMemcpyAsync(tmp.data(), Qout, tmp.size() * 4, hipMemcpyDeviceToHost, st));
            TJ_HIP_TRY(hipStreamSynchronize(st));
            for (size_t r = 0; r < 3 * (size_t)last_batch; ++r)
                for (int a = 0; a < A; ++a) h_out[r * A + a] = tmp[r * ldA + a];
            return TJ_OK;
        }
        if (which == TJ_STATE_ASTAR) {
            if (last_batch < 1 || n != (size_t)last_batch) return TJ_ERR_INVALID_ARG;
            std::vector<int32_t> tmp(last_batch);
            TJ_HIP_TRY(hipMemcpyAsync(tmp.data(), astar, tmp.size() * 4, hipMemcpyDeviceToHost, st));
            TJ_HIP_TRY(hipStreamSynchronize(st));
            for (int j = 0; j < last_batch; ++j) h_out[j] = (float)tmp[j];
            return TJ_OK;
        }
        return TJ_ERR_INVALID_ARG;
    }

    int set_state(int which, const float *h_in, size_t n, hipStream_t st) override
    {
        if (n != P) return TJ_ERR_INVALID_ARG;
        float *dst = nullptr;
        switch (which) {
        case TJ_STATE_PARAMS: dst = theta_on; break;
        case TJ_STATE_TARGET: dst = theta_tg; break;
        case TJ_STATE_ADAM_M: dst = m; break;
        case TJ_STATE_ADAM_V: dst = v; break;
        default: return TJ_ERR_INVALID_ARG;
        }
        std::vector<float> tmp(P);
        permute_host(h_in, tmp.data(), true);
        TJ_HIP_TRY(hipMemcpyAsync(dst, tmp.data(), P * 4, hipMemcpyHostToDevice, st));
        int rc = TJ_OK;
        if (which == TJ_STATE_PARAMS) rc = recast(true, st);
        if (which == TJ_STATE_TARGET) rc = recast(false, st);
        TJ_HIP_TRY(hipStreamSynchronize(st));   // tmp lives until the copy is done
        return rc;
    }
};

template <typename L>
int create_learner(const tj_learner_desc *desc, void *arena, size_t bytes, const float *h_on, const float *h_tg,
                   hipStream_t st, tj_learner **out)
{
    L *l = new L();
    l->d = *desc;
    size_t need = l->plan(nullptr);
    if (bytes < need) { delete l; return TJ_ERR_ARENA_TOO_SMALL; }
    l->plan(arena);
    int rc = TJ_OK;
    if (hipMemsetAsync(arena, 0, need, st) != hipSuccess) rc = TJ_ERR_DEVICE;
    if (rc == TJ_OK) rc = l->set_state(TJ_STATE_PARAMS, h_on, l->P, st);
    if (rc == TJ_OK) rc = l->set_state(TJ_STATE_TARGET, h_tg, l->P, st);
    if (rc != TJ_OK) { delete l; return rc; }
    *out = l;
    return TJ_OK;
}

template <typename T> size_t measure_conv(const tj_learner_desc *desc)
{
    ConvLearner<T> l;
    l.d = *desc;
    size_t n = l.plan(nullptr);
    return l.shape_ok ? n : 0;
}

template <typename T>
int create_mlp(const tj_learner_desc *desc, void *arena, size_t bytes, const float *h_on, const float *h_tg,
               hipStream_t st, tj_learner **out)
{
    MlpLearner<T> *l = new MlpLearner<T>();
    l->d = *desc;
    size_t need = l->plan(nullptr);
    if (bytes < need) { delete l; return TJ_ERR_ARENA_TOO_SMALL; }
    l->plan(arena);
    int rc = TJ_OK;
    if (hipMemsetAsync(arena, 0, need, st) != hipSuccess) rc = TJ_ERR_DEVICE;
    if (rc == TJ_OK) rc = l->set_state(TJ_STATE_PARAMS, h_on, l->P, st);
    if (rc == TJ_OK) rc = l->set_state(TJ_STATE_TARGET, h_tg, l->P, st);
    if (rc != TJ_OK) { delete l; return rc; }
    *out = l;
    return TJ_OK;
}

template <typename T> size_t measure_mlp(const tj_learner_desc *desc)
{
    MlpLearner<T> l;
    l.d = *desc;
    return l.plan(nullptr);
}

}  // namespace

extern "C" {

size_t tj_learner_num_params(const tj_learner_desc *d)
{
    if (!desc_ok(d)) return 0;
    size_t c = d->in_c, h = d->in_h, w = d->in_w, p = 0;
    for (uint32_t i = 0; i < d->n_layers; ++i) {
        const tj_layer &L = d->layers[i];
        if (L.kind == TJ_LAYER_CONV2D) {
            if (h < L.kernel || w < L.kernel) return 0;
            p += (size_t)L.out * c * L.kernel * L.kernel + L.out;
            h = (h - L.kernel) / L.stride + 1;
            w = (w - L.kernel) / L.stride + 1;
            c = L.out;
        } else {
            p += (size_t)L.out * c * h * w + L.out;
            c = L.out; h = 1; w = 1;
        }
    }
    return p;
}

size_t tj_learner_arena_bytes(const tj_learner_desc *d)
{
    if (!desc_ok(d)) return 0;
    if (!all_linear(d)) return d->precision == TJ_PRECISION_BF16 ? measure_conv<tj_bf16>(d) : measure_conv<float>(d);
    return d->precision == TJ_PRECISION_BF16 ? measure_mlp<tj_bf16>(d) : measure_mlp<float>(d);
}

int tj_learner_create(const tj_learner_desc *d, void *dev_arena, size_t arena_bytes, const float *h_on,
                      const float *h_tg, void *hip_stream, tj_learner **out)
{
    if (!out) return TJ_ERR_INVALID_ARG;
    *out = nullptr;
    if (!desc_ok(d) || !dev_arena || ((uintptr_t)dev_arena & 255) || !h_on || !h_tg) return TJ_ERR_INVALID_ARG;
    hipStream_t st = (hipStream_t)hip_stream;
    if (!all_linear(d)) {
        if (tj_learner_arena_bytes(d) == 0) return TJ_ERR_SHAPE;
        return d->precision == TJ_PRECISION_BF16
                   ? create_learner<ConvLearner<tj_bf16>>(d, dev_arena, arena_bytes, h_on, h_tg, st, out)
                   : create_learner<ConvLearner<float>>(d, dev_arena, arena_bytes, h_on, h_tg, st, out);
    }
    return d->precision == TJ_PRECISION_BF16 ? create_mlp<tj_bf16>(d, dev_arena, arena_bytes, h_on, h_tg, st, out)
                                             : create_mlp<float>(d, dev_arena, arena_bytes, h_on, h_tg, st, out);
}

int tj_learner_destroy(tj_learner *l)
{
    if (!l) return TJ_ERR_INVALID_ARG;
    delete l;
    return TJ_OK;
}

int tj_learner_step(tj_learner *l, const tj_minibatch *mb, tj_step_stats *d_stats, void *hip_stream)
{
    if (!l || !mb) return TJ_ERR_INVALID_ARG;
    return l->step(mb, d_stats, (hipStream_t)hip_stream);
}

int tj_actor_act(tj_learner *l, uint32_t n, const void *d_obs, float epsilon, uint64_t seed, int32_t *d_action,
                 int32_t *d_version, float *d_q, void *hip_stream)
{
    if (!l) return TJ_ERR_INVALID_ARG;
    return l->infer(n, d_obs, epsilon, seed, d_action, d_version, d_q, (hipStream_t)hip_stream);
}

int tj_learner_get_state(tj_learner *l, int which, float *h_out, size_t n, void *hip_stream)
{
    if (!l || !h_out) return TJ_ERR_INVALID_ARG;
    return l->get_state(which, h_out, n, (hipStream_t)hip_stream);
}

int tj_learner_set_state(tj_learner *l, int which, const float *h_in, size_t n, void *hip_stream)
{
    if (!l || !h_in) return TJ_ERR_INVALID_ARG;
    return l->set_state(which, h_in, n, (hipStream_t)hip_stream);
}

int tj_learner_set_phase_events(tj_learner *l, void *const *hip_events, uint32_t n)
{
    if (!l) return TJ_ERR_INVALID_ARG;
    if (!hip_events || n == 0) {
        l->timed = false;
        return TJ_OK;
    }
    if (n != 5) return TJ_ERR_INVALID_ARG;
    for (int i = 0; i < 5; ++i) {
        if (!hip_events[i]) return TJ_ERR_INVALID_ARG;
        l->ev[i] = (hipEvent_t)hip_events[i];
    }
    l->timed = true;
    return TJ_OK;
}

int tj_learner_get_step(tj_learner *l, uint64_t *h_t)
{
    if (!l || !h_t) return TJ_ERR_INVALID_ARG;
    *h_t = l->t;
    return TJ_OK;
}

int tj_learner_set_step(tj_learner *l, uint64_t t)
{
    if (!l) return TJ_ERR_INVALID_ARG;
    l->t = t;
    return TJ_OK;
}

}  // extern "C"

// ---- on-policy workload

namespace {

bool ppo_desc_ok(const tj_ppo_desc *d)
{
    if (!d || !d->obs_dim || !d->max_batch || d->n_actions < 1 || d->n_actions > 63) return false;
    if (d->n_hidden + 1 > TJ_MAX_LAYERS) return false;
    if (d->precision != TJ_PRECISION_FP32 && d->precision != TJ_PRECISION_BF16) return false;
    for (uint32_t i = 0; i < d->n_hidden; ++i)
        if (!d->hidden[i]) return false;
    return d->clip > 0.f && d->clip < 1.f && d->c_v >= 0.f && d->c_e >= 0.f;
}

// the network as a layer chain: hidden layers, then n_actions logits + 1 value
tj_learner_desc ppo_network(const tj_ppo_desc *d)
{
    tj_learner_desc n;
    memset(&n, 0, sizeof(n));
    n.n_layers = d->n_hidden + 1;
    for (uint32_t i = 0; i < d->n_hidden; ++i) n.layers[i] = {TJ_LAYER_LINEAR, d->hidden[i], 0, 0};
    n.layers[d->n_hidden] = {TJ_LAYER_LINEAR, d->n_actions + 1, 0, 0};
    n.in_c = d->obs_dim; n.in_h = 1; n.in_w = 1;
    n.obs_dtype = TJ_OBS_F32;
    n.precision = d->precision;
    n.max_batch = d->max_batch;
    n.lr = d->lr; n.beta1 = d->beta1; n.beta2 = d->beta2; n.eps = d->eps;
    n.target_interval = 0;
    return n;
}

template <typename T> size_t measure_ppo(const tj_ppo_desc *d)
{
    PpoLearner<T> l;
    l.d = ppo_network(d);
    l.n_pass = 1;
    return l.plan(nullptr);
}

template <typename T>
int create_ppo(const tj_ppo_desc *d, void *arena, size_t bytes, const float *h_theta, hipStream_t st, tj_learner **out)
{
    PpoLearner<T> *l = new PpoLearner<T>();
    l->pd = *d;
    l->d = ppo_network(d);
    l->n_pass = 1;
    const size_t need = l->plan(nullptr);
    if (bytes < need) { delete l; return TJ_ERR_ARENA_TOO_SMALL; }
    l->plan(arena);
    int rc = TJ_OK;
    if (hipMemsetAsync(arena, 0, need, st) != hipSuccess) rc = TJ_ERR_DEVICE;
    if (rc == TJ_OK) rc = l->set_state(TJ_STATE_PARAMS, h_theta, l->P, st);
    if (rc != TJ_OK) { delete l; return rc; }
    *out = l;
    return TJ_OK;
}

}  // namespace

extern "C" {

int tj_gae(uint32_t n_env, uint32_t T, const float *d_reward, const float *d_value, const uint8_t *d_done, float gamma,
           float lambda, float *d_adv, float *d_ret, void *hip_stream)
{
    if (!d_reward || !d_value || !d_done || !d_adv || !d_ret) return TJ_ERR_INVALID_ARG;
    if (!(gamma >= 0.f && gamma <= 1.f) || !(lambda >= 0.f && lambda <= 1.f)) return TJ_ERR_INVALID_ARG;
    if (n_env == 0 || T == 0) return TJ_OK;
    gae_scan<<<(n_env + 3) / 4, 256, 0, (hipStream_t)hip_stream>>>(n_env, T, d_reward, d_value, d_done, gamma, lambda,
                                                                    d_adv, d_ret);
    return hipGetLastError() == hipSuccess ? TJ_OK : TJ_ERR_DEVICE;
}

size_t tj_ppo_num_params(const tj_ppo_desc *d)
{
    if (!ppo_desc_ok(d)) return 0;
    const tj_learner_desc n = ppo_network(d);
    return tj_learner_num_params(&n);
}

size_t tj_ppo_arena_bytes(const tj_ppo_desc *d)
{
    if (!ppo_desc_ok(d)) return 0;
    return d->precision == TJ_PRECISION_BF16 ? measure_ppo<tj_bf16>(d) : measure_ppo<float>(d);
}

int tj_ppo_create(const tj_ppo_desc *d, void *dev_arena, size_t arena_bytes, const float *h_init, void *hip_stream,
                  tj_learner **out)
{
    if (!out) return TJ_ERR_INVALID_ARG;
    *out = nullptr;
    if (!ppo_desc_ok(d) || !dev_arena || ((uintptr_t)dev_arena & 255) || !h_init) return TJ_ERR_INVALID_ARG;
    hipStream_t st = (hipStream_t)hip_stream;
    return d->precision == TJ_PRECISION_BF16 ? create_ppo<tj_bf16>(d, dev_arena, arena_bytes, h_init, st, out)
                                             : create_ppo<float>(d, dev_arena, arena_bytes, h_init, st, out);
}

int tj_ppo_step(tj_learner *l, const tj_ppo_batch *batch, tj_ppo_stats *d_stats, void *hip_stream)
{
    if (!l || !batch) return TJ_ERR_INVALID_ARG;
    return l->ppo_step(batch, d_stats, (hipStream_t)hip_stream);
}

int tj_ppo_evaluate(tj_learner *l, uint32_t n, const float *d_obs, float *d_logits, float *d_value, void *hip_stream)
{
    if (!l) return TJ_ERR_INVALID_ARG;
    return l->ppo_evaluate(n, d_obs, d_logits, d_value, (hipStream_t)hip_stream);
}

int tj_ppo_act(tj_learner *l, uint32_t n, const float *d_obs, uint64_t seed, int32_t *d_action, float *d_logp,
               float *d_value, void *hip_stream)
{
    if (!l) return TJ_ERR_INVALID_ARG;
    return l->ppo_act(n, d_obs, seed, d_action, d_logp, d_value, (hipStream_t)hip_stream);
}

}  // extern "C"
