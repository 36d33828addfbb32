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
