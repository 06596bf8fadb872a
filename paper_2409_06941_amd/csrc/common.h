// Internal declarations shared by the library's translation units (not part of the C ABI).
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>
#include <vector>

#include "freeride.h"

// Accounting allocator handed to a task's init() (memory limit, Section 4.5 of the paper).
struct fr_alloc {
    uint64_t limit = 0;
    uint64_t used = 0;
    bool oom = false;
    bool host_only = false;
    int device = 0;
    int hip_error = 0;
    uint64_t peak = 0;
    struct Block { void* ptr; uint64_t bytes; };
    std::vector<Block> blocks;
};

void fr_alloc_reset(fr_alloc* a, uint64_t limit, bool host_only, int device);
void fr_alloc_release(fr_alloc* a);   // frees every block handed out

// Stage-load kernels (gemm.hip).
int fr_busywait_launch(uint64_t ns, int wall_clock_khz, hipStream_t stream);
int fr_alufill_launch(uint64_t ns, int wall_clock_khz, uint32_t workgroups, hipStream_t stream);

#define FR_HIP_TRY(expr, errslot)                      \
    do {                                               \
        hipError_t e__ = (expr);                       \
        if (e__ != hipSuccess) {                       \
            (errslot) = (int)e__;                      \
            return FR_ERR_HIP;                         \
        }                                              \
    } while (0)
