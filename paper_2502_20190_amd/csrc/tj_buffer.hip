// Replay ring buffer with policy-version tags and the staleness-gated uniform
// sampler (Buffer component and learner load of Section 3.1 of the paper).
//
// Device layout (structure of arrays inside the caller's arena):
//   obs, next_obs  [N][row_bytes]      action i32 [N]   reward f32 [N]
//   done u8 [N]    version i32 [N]
//   mask  u64 [ceil(N/64)]  bit b of word w = slot 64w+b is eligible
//   tile_count / tile_off u32 [ceil(N/1024)]
//   state u32 [8] {sticky, K, arc begin, arc length, rows inserted so far (u64), -, -}
//
// tj_sample = three kernels on one stream:
//   1 mask_count   : one wave per tile of 1024 slots reads the tags (16 bytes per lane), ballots ->
//                    mask words, popcount -> per-tile counts              (HBM bound, 4N B)
//   2 select_rows  : every block repeats the exclusive prefix sum of the tile counts in LDS, then
//                    per draw: SplitMix64, mul-high range reduction, binary search over the tile
//                    offsets, popcount walk over the tile's mask words, k-th set bit; copies the
//                    scalar fields
//   3 copy_rows    : gathers obs / next_obs rows with 16-byte lanes
//                    (HBM bound, 2*B*row_bytes read + written)
// Rings of more than 8192 tiles (8.4 M slots) scan in a kernel of their own (tile_scan, select_slots).
#include "tj_common.h"
#include <mutex>

namespace {

constexpr int kTile = 1024;        // slots per tile
constexpr int kWordsPerTile = kTile / 64;
constexpr uint32_t kInvalid = 0xFFFFFFFFu;

struct RingPtrs {
    uint8_t *obs, *next_obs;
    int32_t *action;
    float *reward;
    uint8_t *done;
    int32_t *version;
};

// ---------------------------------------------------------------- sampler

// Bit i of a 16-bit value to bit 4 i.
__device__ __forceinline__ unsigned long long spread4(unsigned long long x)
{
    x = (x | (x << 24)) & 0x000000FF000000FFull;
    x = (x | (x << 12)) & 0x000F000F000F000Full;
    x = (x | (x << 6)) & 0x0303030303030303ull;
    x = (x | (x << 3)) & 0x1111111111111111ull;
    return x;
}

// One wave per tile of 1024 slots (four tiles per block): the wave reads the tile's tags as four
// 1 KiB runs (16 bytes per lane, all four loads in flight), so lane l of run r holds slots
// 256 r + 4 l .. + 3.  Sixteen ballots (one per run and element) give the eligibility bits; mask
// word 4 r + q collects, for the lanes 16 q + i, bit e of lane i at position 4 i + e.  Lanes 0..15
// write the tile's 16 mask words (one 128-byte line), lane 0 its count.
// Slots of the arc [ex_begin, ex_begin + ex_len) (mod cap), which an unfinished concurrent insert
// is overwriting, are not eligible.  FRAME adds the frame ring's rule: not the newest row (no
// successor), and once the ring has wrapped the look-back (age) must not reach past the oldest slot.
template <bool FRAME>
__global__ __launch_bounds__(256) void mask_count(const int32_t *__restrict__ version,
                                                  const uint8_t *__restrict__ age, uint32_t count, uint32_t head,
                                                  uint32_t cap, int64_t cur, int64_t max_st,
                                                  unsigned long long *__restrict__ mask,
                                                  uint32_t *__restrict__ tile_count,
                                                  const uint32_t *__restrict__ state, uint32_t n_tiles)
{
    const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint32_t tile = blockIdx.x * 4 + wave;
    if (tile >= n_tiles) return;
    const uint32_t ex_begin = FRAME ? 0u : state[2], ex_len = FRAME ? 0u : state[3];
    const uint32_t newest = head == 0 ? cap - 1 : head - 1;
    const uint32_t base = tile * kTile;
    int4 v[4];
    uint32_t ag[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {   // the tag array is padded to whole 256-byte pieces: a vector that starts inside it ends inside it
        const uint32_t s0 = base + 256 * r + 4 * lane;
        v[r] = s0 < count ? *(const int4 *)(version + s0) : make_int4(0, 0, 0, 0);
        if (FRAME) ag[r] = (s0 < count && count == cap) ? *(const uint32_t *)(age + s0) : 0u;
    }
    unsigned long long b[4][4];
    uint32_t cnt = 0;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int32_t ve[4] = {v[r].x, v[r].y, v[r].z, v[r].w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const uint32_t s = base + 256 * r + 4 * lane + e;
            const int64_t st = cur - (int64_t)ve[e];
            bool ok = s < count && st >= 0 && st <= max_st;
            if (FRAME) {
                const uint32_t from_oldest = s >= head ? s - head : s + (cap - head);
                ok = ok && s != newest && (count != cap || from_oldest >= ((ag[r] >> (8 * e)) & 0xFFu));
            } else {
                const uint32_t d = s >= ex_begin ? s - ex_begin : s + (cap - ex_begin);
                ok = ok && d >= ex_len;
            }
            b[r][e] = __ballot(ok);
            cnt += __popcll(b[r][e]);
        }
    }
    const uint32_t q = lane & 3;
    unsigned long long word = 0;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        unsigned long long wr = 0;
#pragma unroll
        for (int e = 0; e < 4; ++e) wr |= spread4((b[r][e] >> (16 * q)) & 0xFFFFull) << e;
        if ((lane >> 2) == (uint32_t)r) word = wr;
    }
    if (lane < 16) mask[(size_t)tile * kWordsPerTile + lane] = word;   // the mask array is padded to whole tiles
    if (lane == 0) tile_count[tile] = cnt;
}

// Exclusive scan of the tile counts by one block of 1024 threads, four counts per thread and
// pass (one pass covers 4096 tiles = 4M slots); K to state[1]; K == 0 raises the sticky status.
// A ticket shared by all mask blocks would save this launch but costs more: thousands of atomics
// on one address serialise at about 25 ns each.
__global__ __launch_bounds__(1024) void tile_scan(const uint32_t *__restrict__ tile_count,
                                                  uint32_t n_tiles, uint32_t *__restrict__ tile_off,
                                                  uint32_t *__restrict__ state)
{
    __shared__ uint32_t wave_sum[16];
    __shared__ uint32_t carry;
    const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (threadIdx.x == 0) carry = 0;
    __syncthreads();
    for (uint32_t base = 0; base < n_tiles; base += 4096) {
        const uint32_t t = base + threadIdx.x * 4;
        uint32_t c[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) c[e] = t + e < n_tiles ? tile_count[t + e] : 0;
        const uint32_t mine = c[0] + c[1] + c[2] + c[3];
        uint32_t incl = mine;                      // inclusive scan inside the wave
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            uint32_t up = __shfl_up(incl, d, 64);
            if (lane >= (uint32_t)d) incl += up;
        }
        if (lane == 63) wave_sum[wave] = incl;
        __syncthreads();
        uint32_t before = carry;
        for (uint32_t w = 0; w < wave; ++w) before += wave_sum[w];
        uint32_t run = before + incl - mine;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            if (t + e < n_tiles) tile_off[t + e] = run;
            run += c[e];
        }
        __syncthreads();
        if (threadIdx.x == 1023) carry = before + incl;
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        state[1] = carry;
        if (carry == 0) state[0] = (uint32_t)TJ_ERR_NO_ELIGIBLE;
    }
}

// One thread per draw, one wave per block (the kernel is a chain of dependent loads).
__global__ __launch_bounds__(64) void select_slots(
    const unsigned long long *__restrict__ mask, const uint32_t *__restrict__ tile_off,
    uint32_t n_tiles, const uint32_t *__restrict__ state, uint64_t seed, uint32_t batch,
    RingPtrs ring, uint32_t *__restrict__ idx, int32_t *__restrict__ action,
    float *__restrict__ reward, uint8_t *__restrict__ done)
{
    const uint32_t j = blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= batch) return;
    const uint32_t K = state[1];
    if (K == 0) {
        idx[j] = kInvalid;
        return;
    }
    uint32_t k = (uint32_t)__umul64hi(tj_splitmix64(seed, j), (uint64_t)K);
    // last tile t with tile_off[t] <= k
    uint32_t lo = 0, hi = n_tiles;
    while (hi - lo > 1) {
        uint32_t mid = (lo + hi) >> 1;
        if (tile_off[mid] <= k) lo = mid; else hi = mid;
    }
    uint32_t rem = k - tile_off[lo];
    uint32_t w = lo * kWordsPerTile;
    unsigned long long m = mask[w];
    uint32_t c = __popcll(m);
    // K > 0 guarantees the walk ends inside this tile
    for (int i = 1; i < kWordsPerTile && rem >= c; ++i) {
        rem -= c;
        ++w;
        m = mask[w];
        c = __popcll(m);
    }
    for (uint32_t i = 0; i < rem; ++i) m &= m - 1;   // drop the rem lowest set bits
    uint32_t slot = w * 64 + (uint32_t)(__ffsll((long long)m) - 1);
    idx[j] = slot;
    action[j] = ring.action[slot];
    reward[j] = ring.reward[slot];
    done[j] = ring.done[slot];
}

// ---------------------------------------------------------------- row copies

// Streaming copies: rows are touched once, so loads and stores bypass the caches' LRU
// (nontemporal) and leave L2 to the tag array and the learner's operands.
template <typename V> __device__ __forceinline__ V ld_stream(const V *p) { return __builtin_nontemporal_load(p); }
template <typename V> __device__ __forceinline__ void st_stream(V *p, V v) { __builtin_nontemporal_store(v, p); }
template <> __device__ __forceinline__ uint4 ld_stream<uint4>(const uint4 *p)
{
    typedef uint32_t u4 __attribute__((ext_vector_type(4)));
    const u4 v = __builtin_nontemporal_load((const u4 *)p);
    return make_uint4(v.x, v.y, v.z, v.w);
}
template <> __device__ __forceinline__ void st_stream<uint4>(uint4 *p, uint4 v)
{
    typedef uint32_t u4 __attribute__((ext_vector_type(4)));
    const u4 w = {v.x, v.y, v.z, v.w};
    __builtin_nontemporal_store(w, (u4 *)p);
}

// Scan and select in one kernel, R draws per block.  Every block first repeats the exclusive prefix
// sum of the tile counts (at most kScanTiles of them, read from L2) and keeps it in LDS, which
// replaces a scan launch of its own: thread t loads counts 32 t .. 32 t + 31 as eight 16-byte
// vectors (all in flight), sums them, one shuffle scan over the wave and the wave totals give its
// base, and it writes its 32 running sums back as vectors.  Block 0 publishes K.  Threads j < R then
// take their draws as select_slots does, with the binary search in LDS and the tile's 16 mask words
// fetched as one 128-byte line.
constexpr int kScanTiles = 8192;
constexpr int kMaxDrawsPerBlock = 64;

__global__ __launch_bounds__(256) void select_rows(
    const unsigned long long *__restrict__ mask, const uint32_t *__restrict__ tile_count, uint32_t n_tiles,
    uint32_t *__restrict__ state, uint64_t seed, uint32_t batch, uint32_t R, RingPtrs ring,
    uint32_t *__restrict__ idx, int32_t *__restrict__ action, float *__restrict__ reward,
    uint8_t *__restrict__ done)
{
    constexpr int E = kScanTiles / 256;      // counts per thread
    __shared__ __align__(16) uint32_t off[kScanTiles];
    __shared__ uint32_t wave_sum[4];
    const uint32_t tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    uint32_t c[E];
#pragma unroll
    for (int v = 0; v < E / 4; ++v) {   // the array is padded to whole 256-byte pieces: a vector that starts inside it ends inside it
        const uint32_t i = tid * E + 4 * v;
        const uint4 x = i < n_tiles ? *(const uint4 *)(tile_count + i) : make_uint4(0u, 0u, 0u, 0u);
        c[4 * v] = x.x; c[4 * v + 1] = i + 1 < n_tiles ? x.y : 0u;
        c[4 * v + 2] = i + 2 < n_tiles ? x.z : 0u; c[4 * v + 3] = i + 3 < n_tiles ? x.w : 0u;
    }
    uint32_t mine = 0;
#pragma unroll
    for (int e = 0; e < E; ++e) mine += c[e];
    uint32_t incl = mine;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const uint32_t up = __shfl_up(incl, d, 64);
        if (lane >= (uint32_t)d) incl += up;
    }
    if (lane == 63) wave_sum[wave] = incl;
    __syncthreads();
    uint32_t run = incl - mine;
    for (uint32_t w = 0; w < wave; ++w) run += wave_sum[w];
    const uint32_t K = wave_sum[0] + wave_sum[1] + wave_sum[2] + wave_sum[3];
#pragma unroll
    for (int v = 0; v < E / 4; ++v) {
        uint4 o;
        o.x = run; run += c[4 * v];
        o.y = run; run += c[4 * v + 1];
        o.z = run; run += c[4 * v + 2];
        o.w = run; run += c[4 * v + 3];
        *(uint4 *)(off + tid * E + 4 * v) = o;
    }
    if (blockIdx.x == 0 && tid == 0) {
        state[1] = K;
        if (K == 0) state[0] = (uint32_t)TJ_ERR_NO_ELIGIBLE;
    }
    __syncthreads();
    const uint32_t j = blockIdx.x * R + tid;
    if (tid >= R || j >= batch) return;
    uint32_t slot = kInvalid;
    if (K != 0) {
        const uint32_t k = (uint32_t)__umul64hi(tj_splitmix64(seed, j), (uint64_t)K);
        uint32_t a = 0, b = n_tiles;             // last tile t with off[t] <= k
        while (b - a > 1) {
            const uint32_t mid = (a + b) >> 1;
            if (off[mid] <= k) a = mid; else b = mid;
        }
        uint32_t rem = k - off[a];
        const ulonglong2 *mw = (const ulonglong2 *)(mask + (size_t)a * kWordsPerTile);
        unsigned long long m[kWordsPerTile];
#pragma unroll
        for (int i = 0; i < kWordsPerTile / 2; ++i) {
            const ulonglong2 t = mw[i];
            m[2 * i] = t.x; m[2 * i + 1] = t.y;
        }
        uint32_t w = 0;
        unsigned long long mm = m[0];
#pragma unroll
        for (int i = 0; i < kWordsPerTile - 1; ++i) {   // K > 0 guarantees the walk ends inside this tile
            const uint32_t cw = __popcll(mm);
            if (w == (uint32_t)i && rem >= cw) { rem -= cw; w = i + 1; mm = m[i + 1]; }
        }
        for (uint32_t i = 0; i < rem; ++i) mm &= mm - 1;   // drop the rem lowest set bits
        slot = (a * kWordsPerTile + w) * 64 + (uint32_t)(__ffsll((long long)mm) - 1);
        action[j] = ring.action[slot];
        reward[j] = ring.reward[slot];
        done[j] = ring.done[slot];
    }
    idx[j] = slot;
}

// mode 0 (gather): dst row r <- src row idx[r];  mode 1 (insert): dst row
// (head + r) mod cap <- src row r.  Rows are `vpr` vectors of type V.
// blockIdx.x = row, blockIdx.y = chunk of 256*U vectors inside the row,
// blockIdx.z selects the field (obs / next_obs).
template <typename V, int U>
__global__ __launch_bounds__(256) void copy_rows_wide(const V *__restrict__ src0, V *__restrict__ dst0,
                                                      const V *__restrict__ src1, V *__restrict__ dst1,
                                                      uint32_t vpr, const uint32_t *__restrict__ idx,
                                                      int mode, uint64_t head, uint64_t cap)
{
    const uint32_t r = blockIdx.x;
    const V *src = blockIdx.z ? src1 : src0;
    V *dst = blockIdx.z ? dst1 : dst0;
    uint64_t srow, drow;
    if (mode == 0) {
        uint32_t s = idx[r];
        if (s == kInvalid) return;
        srow = s; drow = r;
    } else {
        srow = r; drow = head + r; if (drow >= cap) drow -= cap;
    }
    const V *sp = src + srow * vpr;
    V *dp = dst + drow * vpr;
    const uint32_t c0 = blockIdx.y * (256 * U) + threadIdx.x;
    V tmp[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        uint32_t c = c0 + u * 256;
        if (c < vpr) tmp[u] = ld_stream(sp + c);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
        uint32_t c = c0 + u * 256;
        if (c < vpr) st_stream(dp + c, tmp[u]);
    }
}

// Narrow rows (vpr < 256): flat index over rows*vpr vectors, several rows per block.
template <typename V, int U>
__global__ __launch_bounds__(256) void copy_rows_narrow(const V *__restrict__ src0, V *__restrict__ dst0,
                                                        const V *__restrict__ src1, V *__restrict__ dst1,
                                                        uint32_t vpr, uint32_t rows,
                                                        const uint32_t *__restrict__ idx, int mode,
                                                        uint64_t head, uint64_t cap)
{
    const V *src = blockIdx.z ? src1 : src0;
    V *dst = blockIdx.z ? dst1 : dst0;
    const uint32_t total = rows * vpr;
    const uint32_t f0 = blockIdx.x * (256 * U) + threadIdx.x;
    V tmp[U];
    uint64_t daddr[U];
    bool live[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        uint32_t f = f0 + u * 256;
        live[u] = f < total;
        if (!live[u]) continue;
        uint32_t r = f / vpr, c = f - r * vpr;
        uint64_t srow, drow;
        if (mode == 0) {
            uint32_t s = idx[r];
            if (s == kInvalid) { live[u] = false; continue; }
            srow = s; drow = r;
        } else {
            srow = r; drow = head + r; if (drow >= cap) drow -= cap;
        }
        tmp[u] = ld_stream(src + srow * vpr + c);
        daddr[u] = drow * vpr + c;
    }
#pragma unroll
    for (int u = 0; u < U; ++u)
        if (live[u]) st_stream(dst + daddr[u], tmp[u]);
}

// The four scalar fields of an insert: slot (head + i) mod cap <- row i.
__global__ __launch_bounds__(256) void insert_scalars(RingPtrs ring, uint32_t n,
                                                      const int32_t *__restrict__ action,
                                                      const float *__restrict__ reward,
                                                      const uint8_t *__restrict__ done,
                                                      const int32_t *__restrict__ version,
                                                      uint64_t head, uint64_t cap)
{
    uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    uint64_t s = head + i;
    if (s >= cap) s -= cap;
    ring.action[s] = action[i];
    ring.reward[s] = reward[i];
    ring.done[s] = done[i];
    ring.version[s] = version[i];
}

// Last kernel of an insert on its stream: every kernel that wrote the rows has finished, so the
// running total of inserted rows may advance.
__global__ void publish_rows(uint32_t *state, unsigned long long total)
{
    if (threadIdx.x == 0 && blockIdx.x == 0)
        __hip_atomic_store((unsigned long long *)(state + 4), total, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Before a sample that may overlap concurrent inserts: the arc of slots whose insert had been
// issued (rows_issued, host count at the call) but had not finished when this kernel ran.  One
// snapshot serves all blocks of the mask kernel, and tj_buffer_status reports it.
__global__ void snapshot_arc(uint32_t *state, unsigned long long rows_issued, unsigned long long cap)
{
    if (threadIdx.x != 0 || blockIdx.x != 0) return;
    const unsigned long long done =
        __hip_atomic_load((unsigned long long *)(state + 4), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    unsigned long long len = rows_issued > done ? rows_issued - done : 0;
    if (len > cap) len = cap;
    state[2] = (uint32_t)(done % cap);
    state[3] = (uint32_t)len;
}

__global__ void zero_words(uint32_t *p, uint32_t n)
{
    uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0;
}

template <typename V>
int launch_copy_rows(const void *s0, void *d0, const void *s1, void *d1, uint32_t row_bytes,
                     uint32_t rows, const uint32_t *idx, int mode, uint64_t head, uint64_t cap,
                     hipStream_t st, uint32_t nz)
{
    const uint32_t vpr = row_bytes / sizeof(V);
    if (vpr >= 256) {
        // U vectors per thread: one block covers up to 256*U vectors of a row
        if (vpr <= 256 * 2) {
            dim3 g2(rows, (vpr + 511) / 512, nz);
            copy_rows_wide<V, 2><<<g2, 256, 0, st>>>((const V *)s0, (V *)d0, (const V *)s1, (V *)d1, vpr,
                                                     idx, mode, head, cap);
        } else if (vpr <= 256 * 4) {
            dim3 g4(rows, (vpr + 1023) / 1024, nz);
            copy_rows_wide<V, 4><<<g4, 256, 0, st>>>((const V *)s0, (V *)d0, (const V *)s1, (V *)d1, vpr,
                                                     idx, mode, head, cap);
        } else {
            dim3 g8(rows, (vpr + 2047) / 2048, nz);
            copy_rows_wide<V, 8><<<g8, 256, 0, st>>>((const V *)s0, (V *)d0, (const V *)s1, (V *)d1, vpr,
                                                     idx, mode, head, cap);
        }
    } else {
        constexpr int U = 2;
        // rows * vpr must fit 32 bits: callers split larger jobs
        uint64_t total = (uint64_t)rows * vpr;
        dim3 grid((uint32_t)((total + 256 * U - 1) / (256 * U)), 1, nz);
        copy_rows_narrow<V, U><<<grid, 256, 0, st>>>((const V *)s0, (V *)d0, (const V *)s1, (V *)d1, vpr,
                                                     rows, idx, mode, head, cap);
    }
    return hipGetLastError() == hipSuccess ? TJ_OK : TJ_ERR_DEVICE;
}

// nz = 2: both tensor pairs (s0 -> d0, s1 -> d1); nz = 1: only the first
int copy_rows(const void *s0, void *d0, const void *s1, void *d1, uint32_t row_bytes, uint32_t rows,
              const uint32_t *idx, int mode, uint64_t head, uint64_t cap, hipStream_t st, uint32_t nz = 2)
{
    if (rows == 0) return TJ_OK;
    auto aligned = [&](size_t a) {
        return row_bytes % a == 0 && ((uintptr_t)s0 | (uintptr_t)d0 | (uintptr_t)s1 | (uintptr_t)d1) % a == 0;
    };
    if (aligned(16)) return launch_copy_rows<uint4>(s0, d0, s1, d1, row_bytes, rows, idx, mode, head, cap, st, nz);
    if (aligned(4)) return launch_copy_rows<uint32_t>(s0, d0, s1, d1, row_bytes, rows, idx, mode, head, cap, st, nz);
    return launch_copy_rows<uint8_t>(s0, d0, s1, d1, row_bytes, rows, idx, mode, head, cap, st, nz);
}

size_t layout(const tj_buffer_desc *d, TjArena &a, RingPtrs *ring, unsigned long long **mask,
              uint32_t **tile_count, uint32_t **tile_off, uint32_t **state)
{
    const uint64_t n = d->capacity;
    const size_t row = (size_t)d->obs_elems * (d->obs_dtype == TJ_OBS_F32 ? 4 : 1);
    const uint64_t n_tiles = (n + kTile - 1) / kTile;
    RingPtrs r;
    r.obs = (uint8_t *)a.take(n * row);
    r.next_obs = (uint8_t *)a.take(n * row);
    r.action = (int32_t *)a.take(n * 4);
    r.reward = (float *)a.take(n * 4);
    r.done = (uint8_t *)a.take(n);
    r.version = (int32_t *)a.take(n * 4);
    unsigned long long *m = (unsigned long long *)a.take(n_tiles * kWordsPerTile * 8);
    uint32_t *tc = (uint32_t *)a.take(n_tiles * 4);
    uint32_t *to = (uint32_t *)a.take(n_tiles * 4);
    uint32_t *s = (uint32_t *)a.take(32);
    if (ring) *ring = r;
    if (mask) *mask = m;
    if (tile_count) *tile_count = tc;
    if (tile_off) *tile_off = to;
    if (state) *state = s;
    return a.off;
}

bool desc_ok(const tj_buffer_desc *d)
{
    return d && d->capacity >= 1 && d->capacity < 0xFFFFFFFFull && d->obs_elems >= 1 &&
           (d->obs_dtype == TJ_OBS_F32 || d->obs_dtype == TJ_OBS_U8);
}


// ---------------------------------------------------------------- frame ring
//
// One u8 frame per slot; an observation is the stack of the last k frames of its episode (early in
// an episode the first frame is repeated), rebuilt when a minibatch is gathered.  age[t] = rows
// since the start of row t's episode, capped at k-1.

// Ages of the n rows being inserted (row i goes to slot head + i).  A row starts an episode if it is
// the first row ever or follows a row with done = 1; the look-back of at most k-1 rows reads the
// incoming done flags and, before the chunk, the ring's (written by earlier inserts).
__global__ __launch_bounds__(256) void frame_ages(uint8_t *__restrict__ age, const uint8_t *__restrict__ ring_done,
                                                  const uint8_t *__restrict__ done_in, uint32_t n, uint64_t head,
                                                  uint64_t cap, uint64_t rows_before, uint32_t k)
{
    const uint32_t i = blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    uint32_t a = k - 1;
    for (uint32_t d = 0; d + 1 < k; ++d) {
        const int64_t r = (int64_t)i - d;                       // row of this chunk, may be negative
        const uint64_t g = rows_before + i - d;                  // the same row counted from the first ever
        bool start;
        if (g == 0) {
            start = true;
        } else if (r >= 1) {
            start = done_in[r - 1] != 0;
        } else {
            const uint64_t back = (uint64_t)(1 - r);             // slots before head
            start = ring_done[(head + cap - back % cap) % cap] != 0;
        }
        if (start) { a = d; break; }
        if (g == 0) break;
    }
    uint64_t s = head + i;
    if (s >= cap) s -= cap;
    age[s] = (uint8_t)a;
}

// Minibatch row r, plane q of 2k: q < k is position q of the stack of slot idx[r], q >= k position
// q - k of the stack of its successor.  Position p of the stack of slot t is the frame in slot
// t - min(k-1-p, age[t]).  U vectors of V per thread, streaming accesses.
template <typename V, int U>
__global__ __launch_bounds__(256) void gather_stacks(const V *__restrict__ frame, const uint8_t *__restrict__ age,
                                                     const uint32_t *__restrict__ idx, V *__restrict__ obs,
                                                     V *__restrict__ next_obs, uint32_t vpf, uint32_t k,
                                                     uint32_t cap)
{
    const uint32_t r = blockIdx.x, q = blockIdx.z;
    uint32_t t = idx[r];
    if (t == kInvalid) return;
    const uint32_t p = q < k ? q : q - k;
    if (q >= k) t = t + 1 == cap ? 0 : t + 1;
    uint32_t back = k - 1 - p;
    const uint32_t a = age[t];
    if (back > a) back = a;
    const uint32_t src = t >= back ? t - back : t + cap - back;
    const V *sp = frame + (size_t)src * vpf;
    V *dp = (q < k ? obs : next_obs) + ((size_t)r * k + p) * vpf;
    const uint32_t c0 = blockIdx.y * (256 * U) + threadIdx.x;
    V tmp[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const uint32_t c = c0 + u * 256;
        if (c < vpf) tmp[u] = sp[c];        // up to 8 planes of neighbouring rows read the same frame: cached
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const uint32_t c = c0 + u * 256;
        if (c < vpf) st_stream(dp + c, tmp[u]);
    }
}

// The same addressing without the copy: out[r][q] = the slot whose frame is plane q of minibatch row r
// (all ones where the draw found nothing).
__global__ __launch_bounds__(256) void stack_plane_slots(const uint8_t *__restrict__ age, const uint32_t *__restrict__ idx,
                                                         uint32_t *__restrict__ out, uint32_t batch, uint32_t k,
                                                         uint32_t cap)
{
    const uint32_t i = blockIdx.x * 256 + threadIdx.x;
    if (i >= batch * 2 * k) return;
    const uint32_t r = i / (2 * k), q = i % (2 * k);
    uint32_t t = idx[r];
    if (t == kInvalid) { out[i] = kInvalid; return; }
    const uint32_t p = q < k ? q : q - k;
    if (q >= k) t = t + 1 == cap ? 0 : t + 1;
    uint32_t back = k - 1 - p;
    const uint32_t a = age[t];
    if (back > a) back = a;
    out[i] = t >= back ? t - back : t + cap - back;
}

template <typename V>
int launch_gather_stacks(const void *frame, const uint8_t *age, const uint32_t *idx, void *obs, void *next_obs,
                         uint32_t frame_bytes, uint32_t k, uint32_t cap, uint32_t batch, hipStream_t st)
{
    const uint32_t vpf = frame_bytes / sizeof(V);
    constexpr int U = 2;
    dim3 grid(batch, (vpf + 256 * U - 1) / (256 * U), 2 * k);
    gather_stacks<V, U><<<grid, 256, 0, st>>>((const V *)frame, age, idx, (V *)obs, (V *)next_obs, vpf, k, cap);
    return hipGetLastError() == hipSuccess ? TJ_OK : TJ_ERR_DEVICE;
}

bool frame_desc_ok(const tj_frame_buffer_desc *d)
{
    return d && d->stack >= 1 && d->stack <= 16 && d->frame_elems >= 1 && d->capacity >= 2ull * d->stack &&
           d->capacity < 0xFFFFFFFFull;
}

struct FrameLayout {
    uint8_t *frame, *age;
    RingPtrs ring;
    unsigned long long *mask;
    uint32_t *tile_count, *tile_off, *state;
};

size_t frame_layout(const tj_frame_buffer_desc *d, TjArena &a, FrameLayout *out)
{
    const uint64_t n = d->capacity, n_tiles = (n + kTile - 1) / kTile;
    FrameLayout l;
    l.frame = (uint8_t *)a.take(n * d->frame_elems);
    l.age = (uint8_t *)a.take(n);
    l.ring.obs = l.ring.next_obs = nullptr;
    l.ring.action = (int32_t *)a.take(n * 4);
    l.ring.reward = (float *)a.take(n * 4);
    l.ring.done = (uint8_t *)a.take(n);
    l.ring.version = (int32_t *)a.take(n * 4);
    l.mask = (unsigned long long *)a.take(n_tiles * kWordsPerTile * 8);
    l.tile_count = (uint32_t *)a.take(n_tiles * 4);
    l.tile_off = (uint32_t *)a.take(n_tiles * 4);
    l.state = (uint32_t *)a.take(32);
    if (out) *out = l;
    return a.off;
}

}  // namespace

struct tj_frame_buffer {
    tj_frame_buffer_desc desc;
    FrameLayout l;
    uint64_t head = 0, count = 0, rows_total = 0;
    hipEvent_t ev[3];
    bool timed = false;
};

namespace {
}  // namespace

struct tj_buffer {
    tj_buffer_desc desc;
    RingPtrs ring;
    unsigned long long *mask;
    uint32_t *tile_count, *tile_off, *state;
    uint32_t row_bytes, n_tiles;
    uint64_t head, count;
    hipEvent_t ev[3];
    bool timed;
    // Concurrent inserts: rows_issued counts every row ever passed to an insert call (host side, at
    // the call); its device twin in state[4..5] advances when an insert's kernels have run.  The
    // difference, taken on the device just before a sample's mask kernel, is the arc that sample
    // leaves out.  sample_done marks the end of the latest tj_sample.
    uint64_t rows_issued = 0;
    bool concurrent_used = false;
    hipEvent_t sample_done = nullptr;
    hipStream_t last_sample_stream = nullptr;
    bool sampled = false;
};

extern "C" {

size_t tj_buffer_arena_bytes(const tj_buffer_desc *desc)
{
    if (!desc_ok(desc)) return 0;
    TjArena a(nullptr);
    return layout(desc, a, nullptr, nullptr, nullptr, nullptr, nullptr);
}

int tj_buffer_create(const tj_buffer_desc *desc, void *dev_arena, size_t arena_bytes, void *hip_stream,
                     tj_buffer **out)
{
    if (!out) return TJ_ERR_INVALID_ARG;
    *out = nullptr;
    if (!desc_ok(desc) || !dev_arena || ((uintptr_t)dev_arena & 255)) return TJ_ERR_INVALID_ARG;
    if (arena_bytes < tj_buffer_arena_bytes(desc)) return TJ_ERR_ARENA_TOO_SMALL;
    tj_buffer *b = new tj_buffer();
    b->desc = *desc;
    TjArena a(dev_arena);
    layout(desc, a, &b->ring, &b->mask, &b->tile_count, &b->tile_off, &b->state);
    b->row_bytes = desc->obs_elems * (desc->obs_dtype == TJ_OBS_F32 ? 4u : 1u);
    b->n_tiles = (uint32_t)((desc->capacity + kTile - 1) / kTile);
    b->head = b->count = 0;
    b->timed = false;
    zero_words<<<1, 64, 0, (hipStream_t)hip_stream>>>(b->state, 8);
    if (hipGetLastError() != hipSuccess) {
        delete b;
        return TJ_ERR_DEVICE;
    }
    *out = b;
    return TJ_OK;
}

int tj_buffer_destroy(tj_buffer *buf)
{
    if (!buf) return TJ_ERR_INVALID_ARG;
    if (buf->sample_done) (void)hipEventDestroy(buf->sample_done);
    delete buf;
    return TJ_OK;
}

static int insert_rows(tj_buffer *buf, uint32_t n, const void *d_obs, const void *d_next_obs,
                       const int32_t *d_action, const float *d_reward, const uint8_t *d_done,
                       const int32_t *d_version, hipStream_t st)
{
    const uint64_t cap = buf->desc.capacity;
    // narrow rows use a flat 32-bit vector index: split very large inserts
    const uint32_t max_rows = 1u << 20;
    for (uint32_t done_rows = 0; done_rows < n; done_rows += max_rows) {
        uint32_t rows = n - done_rows < max_rows ? n - done_rows : max_rows;
        uint64_t head = (buf->head + done_rows) % cap;
        size_t off = (size_t)done_rows * buf->row_bytes;
        int rc = copy_rows((const uint8_t *)d_obs + off, buf->ring.obs, (const uint8_t *)d_next_obs + off,
                           buf->ring.next_obs, buf->row_bytes, rows, nullptr, 1, head, cap, st);
        if (rc != TJ_OK) return rc;
    }
    insert_scalars<<<(n + 255) / 256, 256, 0, st>>>(buf->ring, n, d_action, d_reward, d_done, d_version,
                                                    buf->head, cap);
    publish_rows<<<1, 64, 0, st>>>(buf->state, (unsigned long long)(buf->rows_issued + n));
    if (hipGetLastError() != hipSuccess) return TJ_ERR_DEVICE;
    buf->rows_issued += n;
    buf->head = (buf->head + n) % cap;
    buf->count = buf->count + n < cap ? buf->count + n : cap;
    return TJ_OK;
}

int tj_buffer_insert(tj_buffer *buf, uint32_t n, const void *d_obs, const void *d_next_obs,
                     const int32_t *d_action, const float *d_reward, const uint8_t *d_done,
                     const int32_t *d_version, void *hip_stream)
{
    if (!buf) return TJ_ERR_INVALID_ARG;
    if (n == 0) return TJ_OK;
    if (!d_obs || !d_next_obs || !d_action || !d_reward || !d_done || !d_version) return TJ_ERR_INVALID_ARG;
    if ((uint64_t)n > buf->desc.capacity) return TJ_ERR_CAPACITY;
    return insert_rows(buf, n, d_obs, d_next_obs, d_action, d_reward, d_done, d_version, (hipStream_t)hip_stream);
}

int tj_buffer_insert_concurrent(tj_buffer *buf, uint32_t n, const void *d_obs, const void *d_next_obs,
                                const int32_t *d_action, const float *d_reward, const uint8_t *d_done,
                                const int32_t *d_version, void *insert_stream)
{
    if (!buf) return TJ_ERR_INVALID_ARG;
    if (n == 0) return TJ_OK;
    if (!d_obs || !d_next_obs || !d_action || !d_reward || !d_done || !d_version) return TJ_ERR_INVALID_ARG;
    if ((uint64_t)n > buf->desc.capacity) return TJ_ERR_CAPACITY;
    hipStream_t st = (hipStream_t)insert_stream;
    // Samples issued so far may still be reading the slots about to be overwritten.  Once concurrent
    // inserts are in use every tj_sample records sample_done at its end; the first concurrent insert
    // records it here, behind whatever the sampling stream has been given so far.
    if (!buf->concurrent_used && buf->sampled) {
        if (!buf->sample_done) TJ_HIP_TRY(hipEventCreateWithFlags(&buf->sample_done, hipEventDisableTiming));
        TJ_HIP_TRY(hipEventRecord(buf->sample_done, buf->last_sample_stream));
    }
    if (buf->sample_done) TJ_HIP_TRY(hipStreamWaitEvent(st, buf->sample_done, 0));
    buf->concurrent_used = true;
    return insert_rows(buf, n, d_obs, d_next_obs, d_action, d_reward, d_done, d_version, st);
}

// The sampler's kernels on `st`, with the eligibility mask, the tile counts and the tile offsets in
// the given scratch (the ring arena's own, or the library's built-in one).
static int sample_into(tj_buffer *buf, uint32_t batch, int64_t current_version, int64_t max_staleness,
                       uint64_t seed, const tj_minibatch *out, hipStream_t st, unsigned long long *mask,
                       uint32_t *tile_count, uint32_t *tile_off, bool may_create_event)
{
    if (!buf || !out || batch == 0 || out->batch != batch) return TJ_ERR_INVALID_ARG;
    if (!out->action || !out->reward || !out->done || !out->idx) return TJ_ERR_INVALID_ARG;
    // observations: both destinations, or neither (indices and scalar fields only)
    if ((out->obs == nullptr) != (out->next_obs == nullptr)) return TJ_ERR_INVALID_ARG;
    if (batch > (1u << 20)) return TJ_ERR_SHAPE;
    // later concurrent inserts wait for the end of this sample: the event must exist
    if (buf->concurrent_used && !buf->sample_done) {
        if (!may_create_event) return TJ_ERR_INVALID_ARG;
        TJ_HIP_TRY(hipEventCreateWithFlags(&buf->sample_done, hipEventDisableTiming));
    }
    const uint32_t count = (uint32_t)buf->count;
    // only the tiles that hold valid slots take part (at least one, so K is always written)
    uint32_t n_tiles = (count + kTile - 1) / kTile;
    if (n_tiles == 0) n_tiles = 1;
    // With concurrent inserts in play, the arc to leave out is taken on the device, in stream order
    // just before the mask kernel; otherwise it stays empty (state[2..3] = 0).
    if (buf->concurrent_used) {
        snapshot_arc<<<1, 64, 0, st>>>(buf->state, (unsigned long long)buf->rows_issued,
                                       (unsigned long long)buf->desc.capacity);
        if (hipGetLastError() != hipSuccess) return TJ_ERR_DEVICE;
    }
    if (buf->timed) TJ_HIP_TRY(hipEventRecord(buf->ev[0], st));
    mask_count<false><<<(n_tiles + 3) / 4, 256, 0, st>>>(buf->ring.version, nullptr, count, 0u,
                                                         (uint32_t)buf->desc.capacity, current_version, max_staleness,
                                                         mask, tile_count, buf->state, n_tiles);
    if (n_tiles <= (uint32_t)kScanTiles) {
        uint32_t R = batch / 256;   // draws per block: a few hundred blocks at most repeat the prefix sum
        R = R < 1 ? 1 : (R > (uint32_t)kMaxDrawsPerBlock ? (uint32_t)kMaxDrawsPerBlock : R);
        select_rows<<<(batch + R - 1) / R, 256, 0, st>>>(mask, tile_count, n_tiles, buf->state, seed, batch, R, buf->ring,
                                                         out->idx, out->action, out->reward, out->done);
    } else {
        tile_scan<<<1, 1024, 0, st>>>(tile_count, n_tiles, tile_off, buf->state);
        select_slots<<<(batch + 63) / 64, 64, 0, st>>>(mask, tile_off, n_tiles, buf->state, seed, batch, buf->ring,
                                                       out->idx, out->action, out->reward, out->done);
    }
    if (hipGetLastError() != hipSuccess) return TJ_ERR_DEVICE;
    if (buf->timed) TJ_HIP_TRY(hipEventRecord(buf->ev[1], st));
    int rc = TJ_OK;
    if (out->obs)
        rc = copy_rows(buf->ring.obs, out->obs, buf->ring.next_obs, out->next_obs, buf->row_bytes, batch, out->idx, 0,
                       0, buf->desc.capacity, st);
    if (rc == TJ_OK && buf->timed) TJ_HIP_TRY(hipEventRecord(buf->ev[2], st));
    buf->last_sample_stream = st;
    buf->sampled = true;
    if (rc == TJ_OK && buf->concurrent_used) TJ_HIP_TRY(hipEventRecord(buf->sample_done, st));
    return rc;
}

int tj_sample(tj_buffer *buf, uint32_t batch, int64_t current_version, int64_t max_staleness,
              uint64_t seed, const tj_minibatch *out, void *hip_stream)
{
    if (!buf) return TJ_ERR_INVALID_ARG;
    return sample_into(buf, batch, current_version, max_staleness, seed, out, (hipStream_t)hip_stream, buf->mask,
                       buf->tile_count, buf->tile_off, true);
}

// ---- the allocation-free variant: the sampler's scratch lives in the library's own image
constexpr uint64_t kNoAllocMaxSlots = TJ_SAMPLE_NOALLOC_MAX_CAPACITY;
constexpr size_t kNoAllocTiles = (size_t)(kNoAllocMaxSlots / kTile);
constexpr size_t kNoAllocMaskBytes = kNoAllocTiles * kWordsPerTile * 8;
constexpr size_t kNoAllocBytes = kNoAllocMaskBytes + 2 * kNoAllocTiles * 4;
static __device__ __align__(256) unsigned char scratch[kNoAllocBytes];

// Device address of `scratch` on the current device (every device holds its own copy of the array
// at its own address): looked up once per device, with that device current.
constexpr int kMaxDevices = 64;
static void *g_scratch_ptr[kMaxDevices];
static std::mutex g_scratch_lock;

static int scratch_on_current_device(unsigned char **out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
        (void)hipGetLastError();
        return TJ_ERR_DEVICE;
    }
    std::lock_guard<std::mutex> hold(g_scratch_lock);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
            (void)hipGetLastError();
            return TJ_ERR_DEVICE;
        }
        g_scratch_ptr[dev] = p;
    }
    *out = (unsigned char *)g_scratch_ptr[dev];
    return TJ_OK;
}

int tj_sample_noalloc(tj_buffer *buf, uint32_t batch, int64_t current_version, int64_t max_staleness,
                      uint64_t seed, const tj_minibatch *out, void *hip_stream)
{
    if (!buf) return TJ_ERR_INVALID_ARG;
    if (buf->desc.capacity > kNoAllocMaxSlots) return TJ_ERR_SCRATCH_LIMIT;
    unsigned char *base = nullptr;
    int rc = scratch_on_current_device(&base);
    if (rc != TJ_OK) return rc;
    // every tile the kernels read is written by this call first: nothing has to start at zero
    unsigned long long *mask = (unsigned long long *)base;
    uint32_t *tile_count = (uint32_t *)(base + kNoAllocMaskBytes);
    uint32_t *tile_off = tile_count + kNoAllocTiles;
    return sample_into(buf, batch, current_version, max_staleness, seed, out, (hipStream_t)hip_stream, mask,
                       tile_count, tile_off, false);
}

int tj_buffer_reads_done(tj_buffer *buf, void *hip_stream)
{
    if (!buf) return TJ_ERR_INVALID_ARG;
    hipStream_t st = (hipStream_t)hip_stream;
    // the same marker a sample leaves at its end, moved behind the work that read the ring after it
    if (!buf->sample_done) TJ_HIP_TRY(hipEventCreateWithFlags(&buf->sample_done, hipEventDisableTiming));
    TJ_HIP_TRY(hipEventRecord(buf->sample_done, st));
    buf->last_sample_stream = st;
    buf->sampled = true;
    return TJ_OK;
}

int tj_buffer_set_phase_events(tj_buffer *buf, void *const *hip_events, uint32_t n)
{
    if (!buf) return TJ_ERR_INVALID_ARG;
    if (!hip_events || n == 0) {
        buf->timed = false;
        return TJ_OK;
    }
    if (n != 3) return TJ_ERR_INVALID_ARG;
    for (int i = 0; i < 3; ++i) {
        if (!hip_events[i]) return TJ_ERR_INVALID_ARG;
        buf->ev[i] = (hipEvent_t)hip_events[i];
    }
    buf->timed = true;
    return TJ_OK;
}

int tj_buffer_status(tj_buffer *buf, tj_buffer_info *h_out, void *hip_stream)
{
    if (!buf || !h_out) return TJ_ERR_INVALID_ARG;
    hipStream_t st = (hipStream_t)hip_stream;
    uint32_t h[4] = {0, 0, 0, 0};   // sticky, K, arc begin, arc length of the last sample
    TJ_HIP_TRY(hipMemcpyAsync(h, buf->state, sizeof(h), hipMemcpyDeviceToHost, st));
    TJ_HIP_TRY(hipStreamSynchronize(st));
    h_out->capacity = buf->desc.capacity;
    h_out->head = buf->head;
    h_out->count = buf->count;
    h_out->last_n_eligible = h[1];
    h_out->sticky_error = (int32_t)h[0];
    h_out->last_excluded_begin = h[3] ? h[2] : 0;
    h_out->last_excluded_len = h[3];
    if (h[0] != 0) {
        zero_words<<<1, 64, 0, st>>>(buf->state, 1);
        TJ_HIP_TRY(hipStreamSynchronize(st));
    }
    return (int32_t)h[0];
}

void *tj_buffer_field_ptr(tj_buffer *buf, int field)
{
    if (!buf) return nullptr;
    switch (field) {
    case 0: return buf->ring.obs;
    case 1: return buf->ring.next_obs;
    case 2: return buf->ring.action;
    case 3: return buf->ring.reward;
    case 4: return buf->ring.done;
    case 5: return buf->ring.version;
    default: return nullptr;
    }
}

size_t tj_frame_buffer_arena_bytes(const tj_frame_buffer_desc *desc)
{
    if (!frame_desc_ok(desc)) return 0;
    TjArena a(nullptr);
    return frame_layout(desc, a, nullptr);
}

int tj_frame_buffer_create(const tj_frame_buffer_desc *desc, void *dev_arena, size_t arena_bytes, void *hip_stream,
                           tj_frame_buffer **out)
{
    if (!out) return TJ_ERR_INVALID_ARG;
    *out = nullptr;
    if (!frame_desc_ok(desc) || !dev_arena || ((uintptr_t)dev_arena & 255)) return TJ_ERR_INVALID_ARG;
    if (arena_bytes < tj_frame_buffer_arena_bytes(desc)) return TJ_ERR_ARENA_TOO_SMALL;
    tj_frame_buffer *b = new tj_frame_buffer();
    b->desc = *desc;
    TjArena a(dev_arena);
    frame_layout(desc, a, &b->l);
    zero_words<<<1, 64, 0, (hipStream_t)hip_stream>>>(b->l.state, 8);
    if (hipGetLastError() != hipSuccess) {
        delete b;
        return TJ_ERR_DEVICE;
    }
    *out = b;
    return TJ_OK;
}

int tj_frame_buffer_destroy(tj_frame_buffer *buf)
{
    if (!buf) return TJ_ERR_INVALID_ARG;
    delete buf;
    return TJ_OK;
}

int tj_frame_buffer_insert(tj_frame_buffer *buf, uint32_t n, const uint8_t *d_frame, const int32_t *d_action,
                           const float *d_reward, const uint8_t *d_done, const int32_t *d_version, void *hip_stream)
{
    if (!buf) return TJ_ERR_INVALID_ARG;
    if (n == 0) return TJ_OK;
    if (!d_frame || !d_action || !d_reward || !d_done || !d_version) return TJ_ERR_INVALID_ARG;
    const uint64_t cap = buf->desc.capacity;
    if ((uint64_t)n > cap) return TJ_ERR_CAPACITY;
    hipStream_t st = (hipStream_t)hip_stream;
    // ages first: they read the ring's done flags of earlier rows, which the scalar copy below may overwrite
    frame_ages<<<(n + 255) / 256, 256, 0, st>>>(buf->l.age, buf->l.ring.done, d_done, n, buf->head, cap,
                                                buf->rows_total, buf->desc.stack);
    if (hipGetLastError() != hipSuccess) return TJ_ERR_DEVICE;
    const uint32_t max_rows = 1u << 20;
    for (uint32_t done_rows = 0; done_rows < n; done_rows += max_rows) {
        const uint32_t rows = n - done_rows < max_rows ? n - done_rows : max_rows;
        const uint64_t head = (buf->head + done_rows) % cap;
        const uint8_t *src = d_frame + (size_t)done_rows * buf->desc.frame_elems;
        int rc = copy_rows(src, buf->l.frame, src, buf->l.frame, buf->desc.frame_elems, rows, nullptr, 1, head, cap,
                           st, 1);
        if (rc != TJ_OK) return rc;
    }
    insert_scalars<<<(n + 255) / 256, 256, 0, st>>>(buf->l.ring, n, d_action, d_reward, d_done, d_version, buf->head,
                                                    cap);
    if (hipGetLastError() != hipSuccess) return TJ_ERR_DEVICE;
    buf->rows_total += n;
    buf->head = (buf->head + n) % cap;
    buf->count = buf->count + n < cap ? buf->count + n : cap;
    return TJ_OK;
}

int tj_frame_sample(tj_frame_buffer *buf, uint32_t batch, int64_t current_version, int64_t max_staleness,
                    uint64_t seed, const tj_minibatch *out, void *hip_stream)
{
    if (!buf || !out || batch == 0 || out->batch != batch) return TJ_ERR_INVALID_ARG;
    if (!out->action || !out->reward || !out->done || !out->idx) return TJ_ERR_INVALID_ARG;
    // observations: both destinations, or neither (indices and scalar fields only)
    if ((out->obs == nullptr) != (out->next_obs == nullptr)) return TJ_ERR_INVALID_ARG;
    if (batch > (1u << 20)) return TJ_ERR_SHAPE;
    hipStream_t st = (hipStream_t)hip_stream;
    const uint32_t count = (uint32_t)buf->count, cap = (uint32_t)buf->desc.capacity;
    uint32_t n_tiles = (count + kTile - 1) / kTile;
    if (n_tiles == 0) n_tiles = 1;
    if (buf->timed) TJ_HIP_TRY(hipEventRecord(buf->ev[0], st));
    mask_count<true><<<(n_tiles + 3) / 4, 256, 0, st>>>(buf->l.ring.version, buf->l.age, count, (uint32_t)buf->head, cap,
                                                        current_version, max_staleness, buf->l.mask, buf->l.tile_count,
                                                        buf->l.state, n_tiles);
    if (n_tiles <= (uint32_t)kScanTiles) {
        uint32_t R = batch / 256;
        R = R < 1 ? 1 : (R > (uint32_t)kMaxDrawsPerBlock ? (uint32_t)kMaxDrawsPerBlock : R);
        select_rows<<<(batch + R - 1) / R, 256, 0, st>>>(buf->l.mask, buf->l.tile_count, n_tiles, buf->l.state, seed,
                                                         batch, R, buf->l.ring, out->idx, out->action, out->reward,
                                                         out->done);
    } else {
        tile_scan<<<1, 1024, 0, st>>>(buf->l.tile_count, n_tiles, buf->l.tile_off, buf->l.state);
        select_slots<<<(batch + 63) / 64, 64, 0, st>>>(buf->l.mask, buf->l.tile_off, n_tiles, buf->l.state, seed, batch,
                                                       buf->l.ring, out->idx, out->action, out->reward, out->done);
    }
    if (hipGetLastError() != hipSuccess) return TJ_ERR_DEVICE;
    if (buf->timed) TJ_HIP_TRY(hipEventRecord(buf->ev[1], st));
    const uint32_t fb = buf->desc.frame_elems, k = buf->desc.stack;
    if (!out->obs) {   // no stacks: the slots of their frames instead
        if (!out->plane_index) return TJ_ERR_INVALID_ARG;
        stack_plane_slots<<<(batch * 2 * k + 255) / 256, 256, 0, st>>>(buf->l.age, out->idx, out->plane_index, batch, k, cap);
        if (hipGetLastError() != hipSuccess) return TJ_ERR_DEVICE;
        if (buf->timed) TJ_HIP_TRY(hipEventRecord(buf->ev[2], st));
        return TJ_OK;
    }
    auto aligned = [&](size_t a) {
        return fb % a == 0 && ((uintptr_t)buf->l.frame | (uintptr_t)out->obs | (uintptr_t)out->next_obs) % a == 0;
    };
    int rc;
    if (aligned(16))
        rc = launch_gather_stacks<uint4>(buf->l.frame, buf->l.age, out->idx, out->obs, out->next_obs, fb, k, cap,
                                         batch, st);
    else if (aligned(4))
        rc = launch_gather_stacks<uint32_t>(buf->l.frame, buf->l.age, out->idx, out->obs, out->next_obs, fb, k, cap,
                                            batch, st);
    else
        rc = launch_gather_stacks<uint8_t>(buf->l.frame, buf->l.age, out->idx, out->obs, out->next_obs, fb, k, cap,
                                           batch, st);
    if (rc == TJ_OK && buf->timed) TJ_HIP_TRY(hipEventRecord(buf->ev[2], st));
    return rc;
}

int tj_frame_buffer_set_phase_events(tj_frame_buffer *buf, void *const *hip_events, uint32_t n)
{
    if (!buf) return TJ_ERR_INVALID_ARG;
    if (!hip_events || n == 0) {
        buf->timed = false;
        return TJ_OK;
    }
    if (n != 3) return TJ_ERR_INVALID_ARG;
    for (int i = 0; i < 3; ++i) {
        if (!hip_events[i]) return TJ_ERR_INVALID_ARG;
        buf->ev[i] = (hipEvent_t)hip_events[i];
    }
    buf->timed = true;
    return TJ_OK;
}

int tj_frame_buffer_status(tj_frame_buffer *buf, tj_buffer_info *h_out, void *hip_stream)
{
    if (!buf || !h_out) return TJ_ERR_INVALID_ARG;
    hipStream_t st = (hipStream_t)hip_stream;
    uint32_t h[4] = {0, 0, 0, 0};
    TJ_HIP_TRY(hipMemcpyAsync(h, buf->l.state, sizeof(h), hipMemcpyDeviceToHost, st));
    TJ_HIP_TRY(hipStreamSynchronize(st));
    h_out->capacity = buf->desc.capacity;
    h_out->head = buf->head;
    h_out->count = buf->count;
    h_out->last_n_eligible = h[1];
    h_out->sticky_error = (int32_t)h[0];
    h_out->last_excluded_begin = h_out->last_excluded_len = 0;
    if (h[0] != 0) {
        zero_words<<<1, 64, 0, st>>>(buf->l.state, 1);
        TJ_HIP_TRY(hipStreamSynchronize(st));
    }
    return (int32_t)h[0];
}

void *tj_frame_buffer_field_ptr(tj_frame_buffer *buf, int field)
{
    if (!buf) return nullptr;
    switch (field) {
    case 0: return buf->l.frame;
    case 1: return buf->l.age;
    case 2: return buf->l.ring.action;
    case 3: return buf->l.ring.reward;
    case 4: return buf->l.ring.done;
    case 5: return buf->l.ring.version;
    default: return nullptr;
    }
}

const char *tj_strerror(int status)
{
    switch (status) {
    case TJ_OK: return "ok";
    case TJ_ERR_INVALID_ARG: return "invalid argument";
    case TJ_ERR_SHAPE: return "unsupported shape";
    case TJ_ERR_ARENA_TOO_SMALL: return "arena too small";
    case TJ_ERR_NO_ELIGIBLE: return "no eligible transition inside the staleness gate";
    case TJ_ERR_CAPACITY: return "more rows than the ring holds";
    case TJ_ERR_DEVICE: return "HIP call failed";
    case TJ_ERR_SCRATCH_LIMIT: return "ring larger than the built-in scratch of the allocation-free call";
    default: return "unknown status";
    }
}

}  // extern "C"
