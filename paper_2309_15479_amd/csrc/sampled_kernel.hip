// Sampled-projection kernel (FastLSH, Sec. 3.1, Eq. 5) for gfx950.
//
//   p_j(v) = sum_{i<m} a~_j[i] * v[S_j[i]],   h_j(v) = floor((p_j(v) + b~_j) / w)
//
// Mapping: one lane = one hash function j; one workgroup = a tile of SUB*RT vectors times
// `blockDim.x` functions.  The vector tile is read from HBM once (coalesced along the
// coordinate axis) and kept in LDS with RT vectors interleaved per coordinate slot
// ([sub-tile][coordinate][RT]), so that one 4*RT-byte LDS read fetches the sampled
// coordinate of RT vectors and feeds RT FMAs.  Each lane walks its own (LDS offset,
// coefficient) list; there is no cross-lane reduction.  The lists are stored
// sample-major ([i][j]) so that a wave reads them coalesced; when m equals the register
// chunk they are loaded once per workgroup and stay in VGPRs while the workgroup loops
// over its tiles.
#include <hip/hip_runtime.h>

#include "lsh_internal.h"

namespace lsh {
namespace {

constexpr int kChunk = 32;             // samples held in registers at a time
constexpr uint32_t kLdsBudget = 144u * 1024u;  // of the CU's 160 KB

template <int RT>
struct VecOf;
template <>
struct VecOf<1> { using type = float; };
template <>
struct VecOf<2> { using type = float2; };
template <>
struct VecOf<4> { using type = float4; };

template <int RT>
__device__ __forceinline__ void lds_read_slot(const char *slot, float (&x)[RT]) {
    if constexpr (RT == 8) {
        const float4 lo = *reinterpret_cast<const float4 *>(slot);
        const float4 hi = *reinterpret_cast<const float4 *>(slot + 16);
        x[0] = lo.x; x[1] = lo.y; x[2] = lo.z; x[3] = lo.w;
        x[4] = hi.x; x[5] = hi.y; x[6] = hi.z; x[7] = hi.w;
    } else if constexpr (RT == 4) {
        const float4 q = *reinterpret_cast<const float4 *>(slot);
        x[0] = q.x; x[1] = q.y; x[2] = q.z; x[3] = q.w;
    } else if constexpr (RT == 2) {
        const float2 q = *reinterpret_cast<const float2 *>(slot);
        x[0] = q.x; x[1] = q.y;
    } else {
        x[0] = *reinterpret_cast<const float *>(slot);
    }
}

template <int RT>
__device__ __forceinline__ void lds_write_slot(float *slot, const float (&x)[RT]) {
    if constexpr (RT == 8) {
        *reinterpret_cast<float4 *>(slot) = make_float4(x[0], x[1], x[2], x[3]);
        *reinterpret_cast<float4 *>(slot + 4) = make_float4(x[4], x[5], x[6], x[7]);
    } else if constexpr (RT == 4) {
        *reinterpret_cast<float4 *>(slot) = make_float4(x[0], x[1], x[2], x[3]);
    } else if constexpr (RT == 2) {
        *reinterpret_cast<float2 *>(slot) = make_float2(x[0], x[1]);
    } else {
        *slot = x[0];
    }
}

struct SampledArgs {
    const float *data;   // [N][n]
    uint64_t N;
    uint32_t n, k, m_pad, kpad;
    const Sample *tab;   // [m_pad][kpad]
    const float *off;    // [kpad]
    float w, inv_w;
    int w_is_pow2;
    int epilogue;        // Epilogue
    void *out;
    uint32_t L, g;       // key groups (Epilogue::Keys)
};

// Epilogue for one (vector, function): `row` is uniform in the workgroup, so the wave-wide
// ballot and shuffles below are executed by whole waves.
__device__ __forceinline__ void finish(const SampledArgs &a, uint64_t row, uint32_t j, float p, float b,
                                       uint64_t key_pow) {
    if (row >= a.N) return;
    if (a.epilogue == (int)Epilogue::Proj) {
        if (j < a.k) reinterpret_cast<float *>(a.out)[row * a.k + j] = p;
        return;
    }
    if (a.epilogue == (int)Epilogue::Signs) {
        const uint64_t word = __ballot(j < a.k && p >= 0.f);
        const uint32_t words = (a.k + 63) / 64;
        if ((threadIdx.x & 63) == 0 && j < a.k)
            reinterpret_cast<uint64_t *>(a.out)[row * words + (j >> 6)] = word;
        return;
    }
    const float q = a.w_is_pow2 ? (p + b) * a.inv_w : (p + b) / a.w;
    const int h = (int)floorf(q);
    if (a.epilogue == (int)Epilogue::Ids) {
        if (j < a.k) reinterpret_cast<int32_t *>(a.out)[row * a.k + j] = h;
    } else {  // Keys: g consecutive lanes fold their ids; g is a power of two <= 64
        uint64_t term = (uint64_t)(uint32_t)h * key_pow;
        for (uint32_t d = a.g >> 1; d >= 1; d >>= 1) term += __shfl_xor(term, (int)d);
        if (j < a.k && (j % a.g) == 0) reinterpret_cast<uint64_t *>(a.out)[row * a.L + j / a.g] = term;
    }
}

// REG: m_pad == kChunk, the lane's whole list stays in registers across tiles.
template <int RT, int SUB, bool REG>
__global__ __launch_bounds__(REG ? 512 : 1024) void sampled_kernel(const SampledArgs a) {
    extern __shared__ __align__(16) float tile[];  // [SUB][n + 1][RT]; slot n holds zeros
    const uint32_t n = a.n;
    const uint32_t j = blockIdx.y * blockDim.x + threadIdx.x;  // < kpad
    const uint32_t slots = n + 1;
    constexpr uint32_t kTileRows = RT * SUB;
    const uint64_t ntiles = (a.N + kTileRows - 1) / kTileRows;

    Sample s[kChunk];
    if constexpr (REG) {
#pragma unroll
        for (int i = 0; i < kChunk; ++i) s[i] = a.tab[(size_t)i * a.kpad + j];
    }
    const float b = a.off[j];

    // the zero slot of every sub-tile (target of padding samples)
    if (threadIdx.x < SUB * RT) {
        const uint32_t st = threadIdx.x / RT, r = threadIdx.x % RT;
        tile[((size_t)st * slots + n) * RT + r] = 0.f;
    }

    uint64_t key_pow = 1;  // C^(g-1-t) for this lane's position t in its key group
    if (a.epilogue == (int)Epilogue::Keys) {
        const uint32_t t = j % a.g;
        for (uint32_t e = 0; e + 1 + t < a.g; ++e) key_pow *= kKeyMultiplier;
    }

    for (uint64_t t = blockIdx.x; t < ntiles; t += gridDim.x) {
        const uint64_t row0 = t * kTileRows;
        __syncthreads();  // every lane is done reading the previous tile
        for (uint32_t e = threadIdx.x; e < SUB * n; e += blockDim.x) {
            const uint32_t st = e / n, c = e - st * n;
            float x[RT];
#pragma unroll
            for (int r = 0; r < RT; ++r) {
                const uint64_t row = row0 + (uint64_t)st * RT + r;
                x[r] = row < a.N ? a.data[row * n + c] : 0.f;
            }
            lds_write_slot<RT>(tile + ((size_t)st * slots + c) * RT, x);
        }
        __syncthreads();

        if constexpr (REG) {
            // lists already in registers: finish one sub-tile (RT vectors) at a time
#pragma unroll 1
            for (int st = 0; st < SUB; ++st) {
                const char *base = reinterpret_cast<const char *>(tile + (size_t)st * slots * RT);
                float acc[RT];
#pragma unroll
                for (int r = 0; r < RT; ++r) acc[r] = 0.f;
#pragma unroll
                for (int i = 0; i < kChunk; ++i) {
                    float x[RT];
                    lds_read_slot<RT>(base + s[i].lds_byte_offset, x);
#pragma unroll
                    for (int r = 0; r < RT; ++r) acc[r] = fmaf(s[i].coef, x[r], acc[r]);
                    // keep the scheduler from hoisting every LDS read of the sub-tile to the
                    // front (which would need more registers than a lane has)
                    if ((i & 7) == 7) __builtin_amdgcn_sched_barrier(0);
                }
#pragma unroll
                for (int r = 0; r < RT; ++r)
                    finish(a, row0 + (uint64_t)st * RT + r, j, acc[r], b, key_pow);
            }
        } else {
            // lists streamed through registers one chunk at a time, each chunk applied to
            // every sub-tile before the next is fetched
            float acc[SUB][RT];
#pragma unroll
            for (int st = 0; st < SUB; ++st)
#pragma unroll
                for (int r = 0; r < RT; ++r) acc[st][r] = 0.f;
            for (uint32_t i0 = 0; i0 < a.m_pad; i0 += kChunk) {
#pragma unroll
                for (int i = 0; i < kChunk; ++i) s[i] = a.tab[(size_t)(i0 + i) * a.kpad + j];
#pragma unroll
                for (int st = 0; st < SUB; ++st) {
                    const char *base = reinterpret_cast<const char *>(tile + (size_t)st * slots * RT);
#pragma unroll
                    for (int i = 0; i < kChunk; ++i) {
                        float x[RT];
                        lds_read_slot<RT>(base + s[i].lds_byte_offset, x);
#pragma unroll
                        for (int r = 0; r < RT; ++r) acc[st][r] = fmaf(s[i].coef, x[r], acc[st][r]);
                    }
                }
            }
#pragma unroll
            for (int st = 0; st < SUB; ++st)
#pragma unroll
                for (int r = 0; r < RT; ++r)
                    finish(a, row0 + (uint64_t)st * RT + r, j, acc[st][r], b, key_pow);
        }
    }
}

template <int RT, int SUB>
int launch_variant(const lsh_params *p, const SampledArgs &args, dim3 grid, dim3 block,
                   hipStream_t stream) {
    const SampledPlan &pl = p->plan;
    auto fn = pl.reg_table ? &sampled_kernel<RT, SUB, true> : &sampled_kernel<RT, SUB, false>;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(fn),
                                       hipFuncAttributeMaxDynamicSharedMemorySize,
                                       (int)pl.lds_bytes);
    if (e != hipSuccess) return LSH_ERR_HIP;
    hipLaunchKernelGGL(fn, grid, block, pl.lds_bytes, stream, args);
    return hipGetLastError() == hipSuccess ? LSH_OK : LSH_ERR_HIP;
}

}  // namespace

// Tile shape by dimension: as many interleaved vectors as fit the LDS budget.
SampledPlan plan_sampled(uint32_t n, uint32_t k, uint32_t m) {
    SampledPlan pl;
    const uint64_t slot_bytes = 4ull * (n + 1ull);
    if (slot_bytes * 32 <= kLdsBudget) { pl.rt = 8; pl.sub = 4; }
    else if (slot_bytes * 8 <= kLdsBudget) { pl.rt = 8; pl.sub = 1; }
    else if (slot_bytes * 4 <= kLdsBudget) { pl.rt = 4; pl.sub = 1; }
    else if (slot_bytes * 2 <= kLdsBudget) { pl.rt = 2; pl.sub = 1; }
    else if (slot_bytes <= kLdsBudget) { pl.rt = 1; pl.sub = 1; }
    else return pl;  // unsupported: one vector does not fit in LDS
    pl.lds_bytes = (uint32_t)(slot_bytes * pl.rt * pl.sub);
    const uint32_t k64 = (k + 63) / 64 * 64;
    pl.reg_table = (m <= (uint32_t)kChunk);
    // register-resident lists need up to 256 VGPRs per lane: at most 512 lanes per workgroup
    const uint32_t max_block = pl.reg_table ? 512 : 1024;
    pl.block = k64 >= max_block ? max_block : (k64 >= 512 ? 512 : (k64 >= 256 ? 256 : k64));
    pl.kblocks = (k64 + pl.block - 1) / pl.block;
    pl.kpad = pl.block * pl.kblocks;
    pl.supported = true;
    return pl;
}

uint32_t sampled_chunk() { return kChunk; }

int launch_sampled(const lsh_params *p, Epilogue ep, const float *d_data, uint64_t N, void *d_out,
                   uint32_t L, void *stream) {
    const SampledPlan &pl = p->plan;
    if (!pl.supported) return LSH_ERR_UNSUPPORTED;
    SampledArgs a;
    a.data = d_data;
    a.N = N;
    a.n = p->n;
    a.k = p->k;
    a.m_pad = (p->m + kChunk - 1) / kChunk * kChunk;
    a.kpad = pl.kpad;
    a.tab = p->d_samples;
    a.off = p->d_off;
    a.w = p->w;
    a.inv_w = 1.0f / p->w;
    int exp2 = 0;
    a.w_is_pow2 = (std::frexp(p->w, &exp2) == 0.5f) ? 1 : 0;
    a.epilogue = (int)ep;
    a.out = d_out;
    a.L = L;
    a.g = L ? p->k / L : 1;
    const uint64_t tile_rows = (uint64_t)pl.rt * pl.sub;
    const uint64_t ntiles = (N + tile_rows - 1) / tile_rows;
    // persistent workgroups: a few per CU, count a multiple of 8 so that the kblocks
    // workgroups that share a vector tile land on the same XCD (and its L2)
    const uint32_t per_cu = pl.lds_bytes > 72 * 1024 ? 1 : (pl.lds_bytes > 36 * 1024 ? 2 : 4);
    uint64_t gx = (uint64_t)p->num_cus * per_cu / pl.kblocks;
    gx = gx < 8 ? 8 : gx / 8 * 8;
    if (gx > ntiles) gx = ntiles;
    dim3 grid((uint32_t)gx, pl.kblocks), block(pl.block);
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    if (pl.rt == 8 && pl.sub == 4) return launch_variant<8, 4>(p, a, grid, block, s);
    if (pl.rt == 8) return launch_variant<8, 1>(p, a, grid, block, s);
    if (pl.rt == 4) return launch_variant<4, 1>(p, a, grid, block, s);
    if (pl.rt == 2) return launch_variant<2, 1>(p, a, grid, block, s);
    return launch_variant<1, 1>(p, a, grid, block, s);
}

}  // namespace lsh
