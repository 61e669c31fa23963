// Compound keys (Sec. 3.2): the ids of the g = k/L functions of one table are folded into
// one 64-bit key, key = sum_t uint32(h_t) * C^(g-1-t) mod 2^64 (Horner form).
// One thread per (vector, table); a wave reads one contiguous run of ids.
#include <hip/hip_runtime.h>

#include "lsh_internal.h"

namespace lsh {
namespace {

__global__ __launch_bounds__(256) void pack_kernel(const int32_t *__restrict__ ids, uint64_t total_keys,
                                                   uint32_t g, uint64_t *__restrict__ keys) {
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    for (uint64_t e = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; e < total_keys; e += stride) {
        const int32_t *src = ids + e * g;  // key e = (vector e / L, table e % L); ids are [N][L][g]
        uint64_t key = 0;
        if ((g & 3) == 0) {
            for (uint32_t t = 0; t < g; t += 4) {
                const int4 q = *reinterpret_cast<const int4 *>(src + t);
                key = key * kKeyMultiplier + (uint32_t)q.x;
                key = key * kKeyMultiplier + (uint32_t)q.y;
                key = key * kKeyMultiplier + (uint32_t)q.z;
                key = key * kKeyMultiplier + (uint32_t)q.w;
            }
        } else {
            for (uint32_t t = 0; t < g; ++t) key = key * kKeyMultiplier + (uint32_t)src[t];
        }
        keys[e] = key;
    }
}

}  // namespace

int launch_pack(const lsh_params *p, const int32_t *d_ids, uint64_t N, uint32_t L, uint64_t *d_keys,
                void *stream) {
    const uint32_t g = p->k / L;
    const uint64_t total = N * L;
    uint64_t blocks = (total + 255) / 256;
    const uint64_t cap = (uint64_t)(p->num_cus > 0 ? p->num_cus : 256) * 32;
    if (blocks > cap) blocks = cap;
    hipLaunchKernelGGL(pack_kernel, dim3((uint32_t)blocks), dim3(256), 0,
                       reinterpret_cast<hipStream_t>(stream), d_ids, total, g, d_keys);
    return hipGetLastError() == hipSuccess ? LSH_OK : LSH_ERR_HIP;
}

}  // namespace lsh
