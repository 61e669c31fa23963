// Device-side helpers shared by the kernels (included by .hip files only).
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

namespace lsh {

// Workgroup barrier that orders LDS traffic only, for kernels that hand tiles from wave to wave
// through LDS and never through global memory: a wave's global loads (tiles for stages to come,
// the next list block) and its stores stay in flight across the barrier, where __syncthreads()
// would wait for all of them.
__device__ __forceinline__ void lds_barrier() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// 4 x 4 transpose across the four lanes of a quad: on entry lane u holds x[t] = value of
// (function u of the quad, vector t); on exit x[t] = value of (function t, vector u).
// Two butterfly stages of quad-permute DPP moves (no LDS traffic).
__device__ __forceinline__ void quad_transpose(uint32_t (&x)[4]) {
    const bool odd = threadIdx.x & 1, hi = threadIdx.x & 2;
    constexpr int kXor1 = 0xB1, kXor2 = 0x4E;  // quad_perm [1,0,3,2] and [2,3,0,1]
    uint32_t t0 = odd ? x[0] : x[1], t1 = odd ? x[2] : x[3];
    t0 = (uint32_t)__builtin_amdgcn_mov_dpp((int)t0, kXor1, 0xf, 0xf, true);
    t1 = (uint32_t)__builtin_amdgcn_mov_dpp((int)t1, kXor1, 0xf, 0xf, true);
    if (odd) { x[0] = t0; x[2] = t1; } else { x[1] = t0; x[3] = t1; }
    t0 = hi ? x[0] : x[2];
    t1 = hi ? x[1] : x[3];
    t0 = (uint32_t)__builtin_amdgcn_mov_dpp((int)t0, kXor2, 0xf, 0xf, true);
    t1 = (uint32_t)__builtin_amdgcn_mov_dpp((int)t1, kXor2, 0xf, 0xf, true);
    if (hi) { x[0] = t0; x[1] = t1; } else { x[2] = t0; x[3] = t1; }
}

}  // namespace lsh
