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

}  // namespace bnn
