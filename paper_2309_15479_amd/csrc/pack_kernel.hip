// Compound keys (Sec. 3.2): the ids of the g = k/L functions of one table are folded into
// one 64-bit key, key = sum_t uint32(h_t) * C^(g-1-t) mod 2^64 (Horner form).
//
// HBM-bound: 4k bytes read and 8L written per vector.  The fast kernel reads the id array as
// one flat stream of 16-byte quads, a wave per contiguous kilobyte (a key's g ids sit in
// g/4 neighbouring lanes); every lane folds its four ids, scales the partial by the power of
// C that belongs to its position, and the partials of a key are summed with xor-shuffles.
// The generic kernel (one thread per key) covers the other group sizes.
#include <hip/hip_runtime.h>

#include "lsh_internal.h"

namespace lsh {
namespace {

typedef int intx4 __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(256) void pack_quads_kernel(const int32_t *__restrict__ ids, uint64_t total_quads,
                                                        uint32_t lanes_per_key, uint64_t *__restrict__ keys) {
    // weight of this lane's partial: C^(4 * (lanes_per_key - 1 - position))
    const uint32_t pos = threadIdx.x % lanes_per_key;
    uint64_t c4 = kKeyMultiplier * kKeyMultiplier;
    c4 *= c4;
    uint64_t weight = 1;
    for (uint32_t e = pos + 1; e < lanes_per_key; ++e) weight *= c4;
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    // total_quads is a multiple of lanes_per_key and the stride of 64: whole keys stay in a wave.
    // Four loads are in flight per lane (measured: 2 % faster with 1024 ids per vector, nothing with
    // 512).
    constexpr int kInFlight = 4;
    const uint64_t padded = (total_quads + 63) / 64 * 64;
    for (uint64_t q0 = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; q0 < padded; q0 += kInFlight * stride) {
        int4 h[kInFlight];
#pragma unroll
        for (int u = 0; u < kInFlight; ++u) {
            const uint64_t q = q0 + u * stride;
            // every id is read once and every key written once: non-temporal both ways (the loads
            // 10 %, the stores another 2 % on the 512-id shape)
            if (q < total_quads) {
                const intx4 t = __builtin_nontemporal_load(reinterpret_cast<const intx4 *>(ids) + q);
                h[u] = make_int4(t[0], t[1], t[2], t[3]);
            } else {
                h[u] = make_int4(0, 0, 0, 0);
            }
        }
#pragma unroll
        for (int u = 0; u < kInFlight; ++u) {
            const uint64_t q = q0 + u * stride;
            if (q >= padded) break;  // uniform: q0 and the stride are multiples of 64 apart from the lane number
            uint64_t part = (uint32_t)h[u].x;
            part = part * kKeyMultiplier + (uint32_t)h[u].y;
            part = part * kKeyMultiplier + (uint32_t)h[u].z;
            part = part * kKeyMultiplier + (uint32_t)h[u].w;
            part *= weight;
            for (uint32_t d = lanes_per_key >> 1; d >= 1; d >>= 1) part += __shfl_xor(part, (int)d);
            if (pos == 0 && q < total_quads) __builtin_nontemporal_store(part, &keys[q / lanes_per_key]);
        }
    }
}

__global__ __launch_bounds__(256) void pack_kernel(const int32_t *__restrict__ ids, uint64_t total_keys,
                                                   uint32_t g, uint64_t *__restrict__ keys) {
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    for (uint64_t e = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; e < total_keys; e += stride) {
        const int32_t *src = ids + e * g;  // key e = (vector e / L, table e % L); ids are [N][L][g]
        uint64_t key = 0;
        for (uint32_t t = 0; t < g; ++t) key = key * kKeyMultiplier + (uint32_t)src[t];
        keys[e] = key;
    }
}

}  // namespace

int launch_pack(const lsh_params *p, const int32_t *d_ids, uint64_t N, uint32_t L, uint64_t *d_keys,
                void *stream) {
    const uint32_t g = p->k / L;
    const uint64_t total = N * L;
    const uint64_t cap = (uint64_t)(p->num_cus > 0 ? p->num_cus : 256) * 16;
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    const uint32_t lanes = g / 4;
    const bool quads = g % 4 == 0 && lanes >= 1 && lanes <= 64 && (lanes & (lanes - 1)) == 0 &&
                       (reinterpret_cast<uintptr_t>(d_ids) & 15) == 0;
    if (quads) {
        const uint64_t total_quads = total * lanes;
        uint64_t blocks = (total_quads + 255) / 256;
        if (blocks > cap) blocks = cap;
        hipLaunchKernelGGL(pack_quads_kernel, dim3((uint32_t)blocks), dim3(256), 0, s, d_ids, total_quads, lanes,
                           d_keys);
    } else {
        uint64_t blocks = (total + 255) / 256;
        if (blocks > cap) blocks = cap;
        hipLaunchKernelGGL(pack_kernel, dim3((uint32_t)blocks), dim3(256), 0, s, d_ids, total, g, d_keys);
    }
    return hipGetLastError() == hipSuccess ? LSH_OK : LSH_ERR_HIP;
}

}  // namespace lsh
