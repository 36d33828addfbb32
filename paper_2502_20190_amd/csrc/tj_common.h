// Internal helpers shared by the HIP sources of the library (not part of the ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include "../../include/tianji.h"

#define TJ_HIP_TRY(expr)                                   \
    do {                                                   \
        hipError_t e_ = (expr);                            \
        if (e_ != hipSuccess) {                            \
            (void)hipGetLastError();                       \
            return TJ_ERR_DEVICE;                          \
        }                                                  \
    } while (0)

static inline size_t tj_align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Carves 256-byte aligned pieces out of a caller-owned arena.
struct TjArena {
    uint8_t *base;
    size_t off;
    explicit TjArena(void *p) : base((uint8_t *)p), off(0) {}
    void *take(size_t bytes)
    {
        void *p = base ? base + off : nullptr;
        off += tj_align_up(bytes ? bytes : 1, 256);
        return p;
    }
};

// SplitMix64 (Steele, Lea, Flood 2014) as a counter-based generator: output j of stream `seed`.
__device__ __forceinline__ uint64_t tj_splitmix64(uint64_t seed, uint64_t j)
{
    uint64_t z = seed + (j + 1) * 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}
