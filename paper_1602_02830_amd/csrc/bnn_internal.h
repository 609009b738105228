// Internal helpers shared by the HIP translation units of libbnn_hip.
// Written for gfx950 (CDNA4, 64-wide wavefronts) only.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "bnn.h"

// v_writelane_b32 through its LLVM intrinsic (this compiler exposes no __builtin for it):
// returns `old` with lane `lane` replaced by the wavefront-uniform `value`.
extern "C" __device__ int bnn_llvm_writelane(int value, int lane, int old) __asm("llvm.amdgcn.writelane.i32");

namespace bnn {

constexpr int kWave = 64;
constexpr int64_t kMaxDim = (int64_t(1) << 31) - 1;
// Largest K of a product: the kernels hold K and ceil(K / 32) = (K + 31) >> 5 in 32-bit integers.
constexpr int64_t kMaxK = (int64_t(1) << 31) - 32;

inline bool aligned_to(const void* p, size_t a) {
    return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0;
}

inline int check_launch() {
    return hipGetLastError() == hipSuccess ? BNN_OK : BNN_ERR_LAUNCH;
}

inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// Store of an int32 result with agent scope (global_store_dword ... sc1: written through the die's L2).
// Measured against plain and non-temporal stores on whole int32 products, it is the fastest policy while the
// output is not much larger than the last-level cache, and by far the fastest where rows of the output are
// not whole 128-byte lines (3000 x 3000 x 784: 13.6 vs 20.0 us).
__device__ inline void store_result(int32_t* p, int32_t v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Mask of the valid bits of the last word of a K-bit row (all ones if K % 32 == 0).
__host__ __device__ inline uint32_t tail_mask(int64_t K) {
    const int r = int(K & 31);
    return r ? ((1u << r) - 1u) : 0xFFFFFFFFu;
}

// OR over each aligned group of 8 lanes, result in every lane of the group.
// Data-parallel-primitive (DPP) lane permutes: xor-1 and xor-2 inside a quad,
// then a mirror of the 8-lane half row, which swaps the two quads.
// Every lane of the wavefront must be active.
__device__ inline uint32_t or_reduce8(uint32_t v) {
    v |= uint32_t(__builtin_amdgcn_update_dpp(0, int(v), 0xB1, 0xF, 0xF, true));   // quad_perm [1,0,3,2]
    v |= uint32_t(__builtin_amdgcn_update_dpp(0, int(v), 0x4E, 0xF, 0xF, true));   // quad_perm [2,3,0,1]
    v |= uint32_t(__builtin_amdgcn_update_dpp(0, int(v), 0x141, 0xF, 0xF, true));  // row_half_mirror
    return v;
}

// Work split of the streaming kernels' fast path (rows that are whole numbers of 128-element units,
// 16-byte aligned): a unit is 4 consecutive output words = 128 consecutive elements of one row, taken by
// an aligned group of 8 lanes; a 256-thread workgroup takes 32 units per step - one 16 KB stretch of a
// row (units_per_row % 32 == 0) or 32 / units_per_row whole rows (32 % units_per_row == 0) - and
// `steps` such steps on consecutive rows, so a thread's columns never change.
struct UnitSplit {
    int units_per_row;     // cols / 128
    int slices_per_row;    // workgroups side by side on one row (1 if a workgroup covers whole rows)
    int rows_per_step;     // rows a workgroup covers per step (1 if a row needs several workgroups)
    int steps;             // steps per workgroup
};

// False if the shape does not fit the split.
inline bool unit_split(int64_t cols, int steps, UnitSplit& us) {
    if (cols <= 0 || cols % 128 != 0 || cols / 128 > (int64_t(1) << 24)) return false;
    const int upr = int(cols / 128);
    if (upr % 32 == 0) {
        us = UnitSplit{upr, upr / 32, 1, steps};
        return true;
    }
    if (32 % upr == 0) {
        us = UnitSplit{upr, 1, 32 / upr, steps};
        return true;
    }
    return false;
}

}  // namespace bnn
