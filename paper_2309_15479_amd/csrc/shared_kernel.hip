// FastLSH with one sample per table (Sec. 3.1 read literally: one multiset S; Sec. 3.2: tables
// of g = k / L functions) for gfx950:
//
//   p_j(v) = sum_{i<m} a~_j[i] * v[S_l[i]],   l = j / g,   h_j(v) = floor((p_j(v) + b~_j) / w)
//
// When the g functions of a table share S_l, the table's projections are a small dense
// product [g x m] . [m x vectors] of the coefficient vectors with the gathered sub-vectors
// S_l(v): the gather is done once per (vector, table) instead of once per (vector, function),
// and the multiply-adds move from the vector ALU to the matrix cores.
//
// Mapping.  A workgroup of 16 waves walks tiles of `rows` vectors (persistent, double-buffered
// in LDS as [vector][n + 4] floats, next tile prefetched HBM -> registers during the
// contraction).  A wave owns RB blocks of 16 consecutive functions (a block lies inside one
// table) and keeps their coefficients in registers for the whole launch.  Per block and 16
// vectors it issues KS = ceil(m / 4) `v_mfma_f32_16x16x4_f32`:
//   row operand    A[i][kq] = a~_{block*16 + i}[4*kk + kq]        lane = i + 16*kq   (registers)
//   column operand B[kq][c] = v_{vector c}[S_l[4*kk + kq]]         lane = c + 16*kq   (one 4-byte LDS read)
//   result         D[4*q + r][c] in register r of lane c + 16*q: four consecutive functions
//                  of one vector per lane, so ids leave as 16-byte stores.
// The tile's row stride n + 4 puts the 16 vectors of a read 4 banks apart when n is a multiple
// of 64 (conflict-free for one coordinate; two coordinates of a step collide when they are
// equal modulo 4, which the host avoids by choosing which samples share a step).  The 4 pad
// floats of a row are kept zero: samples beyond m read them.
//
// Maximum inner product search (appendix): the transformed vectors are
// P~(v) = (sqrt(kappa~^2 - ||S(v)||^2), S(v)) for data and Q~(u) = (0, S(u) / ||S(u)||) for
// queries, hashed with the l2 hash whose coefficient vector is (a0_j, a~_j).  The lanes
// already hold the sampled coordinates as column operands, so ||S_l(v)||^2 is their sum of
// squares over the steps and over the four lanes of a vector; the data hash adds
// a0_j * sqrt(kappa~_l^2 - ||S_l(v)||^2) to the projection, the query hash divides it by
// ||S_l(u)||, and a first pass takes kappa~_l^2 = max_v ||S_l(v)||^2 with the same arithmetic
// (so the difference is exactly 0 for the vector that attains it).  The extra component and
// the offset enter as one more MFMA step, row operand (a0_j, b~_j, 0, 0), column operand
// (sqrt(kappa~^2 - ||S(v)||^2), 1, 0, 0): one register per block instead of eight.
#include <hip/hip_runtime.h>

#include <cmath>

#include "lsh_internal.h"

namespace lsh {
namespace {

constexpr uint32_t kLdsBudget = 158u * 1024u;
constexpr int kPre = 5;           // float4 prefetch registers per lane: rows * n / 4 <= kPre * lanes

typedef float float4v __attribute__((ext_vector_type(4)));

struct SharedArgs {
    const float *data;  // [N][n]
    uint64_t N;
    uint32_t n, k, g;
    uint32_t rows;               // vectors per tile, a multiple of 32 (of 16 for the 32-step kernel)
    uint32_t stride;             // floats per tile row in LDS
    uint32_t n4_magic;           // floor(2^32 / (n / 4)) + 1: e / (n / 4) = mulhi(e, n4_magic) for e * n / 4 < 2^32
    uint32_t blocks_per_table;   // ceil(g / 16)
    uint32_t nblocks;            // L * blocks_per_table
    const float *coef;           // [blocks][KS][64]   row operands, one float per lane
    const uint32_t *sample_off;  // [blocks][KS][4]    4 * S_l[4*kk + kq]: byte offset inside a tile row
    const float *offset;         // [blocks][16]       b~ of the block's functions
    const float *extra;          // [blocks][64]       row operand (a0, b~, 0, 0) of the extra step (maximum inner product)
    const float *kappa2;         // [L]                kappa~_l^2, input of the data hash
    int raw;                     // maximum inner product hashes: write the projections, not the ids
    float w, inv_w;
    int w_is_pow2;
    int staged;                  // two-block waves pair up their pieces into whole 128-byte lines (needs g % 16 == 0)
    void *out;
};

// EP: 0 bucket ids, 1 raw projections, 2 one 64-bit key per table (Sec. 3.2; the fold of pack_kernel.hip),
//     3 kappa~_l^2 (atomic max into out, float [L]), 4 maximum-inner-product data hash, 5 query hash
// GEOM: the tile geometry of n = 128 (128-vector tiles, row stride 132) as compile-time
// constants: the loop over the tile's vector blocks is then unrolled and a block's LDS offset is
// an immediate of the read instead of a vector add per read (a sixth of the kernel's
// vector-ALU instructions, which do not overlap with its MFMAs).
template <int KS, int RB, int WAVES, int EP, bool GEOM>
__global__ __launch_bounds__(WAVES * 64, 4) void shared_kernel(const SharedArgs a) {
    constexpr uint32_t kWaves = WAVES, kLanes = WAVES * 64;
    // blocks of 16 vectors in flight: VB * RB independent accumulators (one with 32 steps of
    // coefficients in registers, and so that 16-vector tiles are possible)
    constexpr int VB = (RB >= 4 || KS >= 32) ? 1 : 2;
    extern __shared__ __align__(16) float tile[];  // 2 x [rows][stride]
    const uint32_t n = GEOM ? 128u : a.n, n4 = n >> 2, rows = GEOM ? 128u : a.rows, stride = GEOM ? 132u : a.stride;
    const uint32_t lane = threadIdx.x & 63, c16 = lane & 15, q = lane >> 4;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint32_t block0 = (blockIdx.y * kWaves + wave) * RB;
    const uint64_t ntiles = (a.N + rows - 1) / rows;
    const uint32_t buf_floats = rows * stride;

    // this wave's blocks: coefficients, per-lane LDS offsets of the sampled coordinates, b~
    float cf[RB][KS];
    // per-lane LDS byte offsets of the sampled coordinates: one register per step, or (32 steps:
    // the registers are needed for the coefficients) the offsets inside a tile row packed two to
    // a register, with the lane's row offset added at each read
    constexpr bool kPacked = KS >= 32;
    uint32_t xo[RB][kPacked ? KS / 2 : KS];
    const uint32_t lane_row = c16 * stride * 4;
    constexpr bool PROJ = EP == 1, KEYS = EP == 2, KAPPA = EP == 3, MDATA = EP == 4, MQUERY = EP == 5;
    constexpr bool NORMS = EP >= 3;
    constexpr bool kEarlyStash = EP < 3;
    float bq[RB][4];
    uint32_t fn0[RB];  // first of the lane's four functions, or >= k when it has none
    uint64_t pw[KEYS ? RB : 1];  // keys: C^(g - 4 - position in the table of the lane's first function), 0 for none
    float cfx[MDATA || MQUERY ? RB : 1];  // row operand of the extra step
    float kap[MDATA ? RB : 1];            // kappa~^2 of the block's table
    float kmax[KAPPA ? RB : 1];    // running max of ||S_l(v)||^2 over the vectors this lane has seen
#pragma unroll
    for (int e = 0; e < RB; ++e) {
        const uint32_t blk = block0 + e;
        const bool have = blk < a.nblocks;
        const uint32_t table = blk / a.blocks_per_table, in_table = (blk % a.blocks_per_table) * 16 + q * 4;
        fn0[e] = have && in_table < a.g ? table * a.g + in_table : a.k;
#pragma unroll
        for (int kk = 0; kk < KS; ++kk) {
            cf[e][kk] = have ? a.coef[((size_t)blk * KS + kk) * 64 + lane] : 0.f;
            const uint32_t off = have ? a.sample_off[((size_t)blk * KS + kk) * 4 + q] : 0u;  // < 4 n + 16 < 65536
            if constexpr (kPacked) {
                if (kk & 1) xo[e][kk / 2] |= off << 16; else xo[e][kk / 2] = off;
            } else {
                xo[e][kk] = off + lane_row;
            }
        }
        if constexpr (EP < 3) {
#pragma unroll
            for (int r = 0; r < 4; ++r) bq[e][r] = a.offset[(size_t)blk * 16 + q * 4 + r];  // padded to every wave's blocks
        }
        if constexpr (KEYS) {
            uint64_t c = have && in_table < a.g ? 1 : 0;  // g % 4 == 0: a lane has four functions or none
            for (uint32_t i = in_table + 4; i < a.g; ++i) c *= kKeyMultiplier;
            pw[e] = c;
        }
        if constexpr (MDATA || MQUERY) cfx[e] = a.extra[(size_t)blk * 64 + lane];
        if constexpr (MDATA) kap[e] = have ? a.kappa2[table] : 0.f;
        if constexpr (KAPPA) kmax[e] = 0.f;
    }
    // the pad floats of every tile row (both buffers) stay zero for the whole launch
    for (uint32_t i = threadIdx.x; i < 2 * rows * 4; i += kLanes) tile[(i >> 2) * stride + n + (i & 3)] = 0.f;

    // tile transfer: element e of the tile's float4 sequence = (vector e / n4, coordinates
    // 4 * (e % n4) ..); the slot arithmetic is redone at every use (it is cheap, and kept in
    // registers across the contraction it would push the coefficient registers out)
    float4 pre[kPre];
    auto opaque = [](uint32_t v) {
        asm volatile("" : "+v"(v));
        return v;
    };
    auto fetch = [&](uint64_t row0) {
        const uint32_t tid = opaque(threadIdx.x);
#pragma unroll
        for (int f = 0; f < kPre; ++f) {
            const uint32_t e = tid + f * kLanes;
            const uint32_t r = __umulhi(e, a.n4_magic), c4 = e - r * n4;
            const bool ok = r < rows && row0 + r < a.N;
            pre[f] = ok ? *reinterpret_cast<const float4 *>(a.data + (row0 + r) * n + c4 * 4)
                        : make_float4(0.f, 0.f, 0.f, 0.f);
        }
    };
    auto stash = [&](float *buf) {
        const uint32_t tid = opaque(threadIdx.x);
#pragma unroll
        for (int f = 0; f < kPre; ++f) {
            const uint32_t e = tid + f * kLanes;
            const uint32_t r = __umulhi(e, a.n4_magic), c4 = e - r * n4;
            if (r < rows) *reinterpret_cast<float4 *>(buf + r * stride + c4 * 4) = pre[f];
        }
    };

    uint64_t t = blockIdx.x;
    if (t >= ntiles) return;
    fetch(t * rows);
    stash(tile);
    __syncthreads();
    uint32_t cur = 0;
    for (; t < ntiles; t += gridDim.x) {
        const uint64_t row0 = t * rows;
        const uint64_t t_next = t + gridDim.x;
        if (t_next < ntiles) fetch(t_next * rows);

        const char *base = reinterpret_cast<const char *>(tile + cur * buf_floats);
        if constexpr (kPacked) {
            // or the compiler would unpack them once, outside the tile loop, into twice the registers
#pragma unroll
            for (int e = 0; e < RB; ++e)
#pragma unroll
                for (int h = 0; h < KS / 2; ++h) asm volatile("" : "+v"(xo[e][h]));
        }
#pragma unroll(GEOM ? 8 : 1)
        for (uint32_t vb = 0; vb < rows / 16; vb += VB) {
            float4v acc[VB][RB];
#pragma unroll
            for (int u = 0; u < VB; ++u)
#pragma unroll
                for (int e = 0; e < RB; ++e) acc[u][e] = float4v{0.f, 0.f, 0.f, 0.f};
            // byte offsets of the vector blocks (wave-uniform; opaque so that the compiler
            // adds them at each read instead of keeping xo + offset for both blocks in registers)
            uint32_t voff[VB];
#pragma unroll
            for (int u = 0; u < VB; ++u) {
                voff[u] = (vb + u) * 16 * stride * 4;
                if constexpr (!GEOM) asm volatile("" : "+s"(voff[u]));
            }
            // software pipeline: the LDS reads of step kk + kAhead are issued before the MFMAs of
            // step kk (scheduling barriers keep the compiler from batching reads and MFMAs apart)
            constexpr int kAhead = 2;
            float x[kAhead + 1][VB][RB];
            auto read_step = [&](int kk) {
#pragma unroll
                for (int u = 0; u < VB; ++u)
#pragma unroll
                    for (int e = 0; e < RB; ++e)
                    {
                        uint32_t off;
                        if constexpr (kPacked) {
                            off = lane_row + ((kk & 1) ? xo[e][kk / 2] >> 16 : xo[e][kk / 2] & 0xffffu);
                        } else {
                            off = xo[e][kk];
                        }
                        x[kk % (kAhead + 1)][u][e] = *reinterpret_cast<const float *>(base + (voff[u] + off));
                    }
            };
#pragma unroll
            for (int kk = 0; kk < kAhead; ++kk) read_step(kk);
            float nrm[NORMS ? VB : 1][NORMS ? RB : 1];  // ||S_l(v)||^2: this lane's coordinates, then the vector's
            if constexpr (NORMS) {
#pragma unroll
                for (int u = 0; u < VB; ++u)
#pragma unroll
                    for (int e = 0; e < RB; ++e) nrm[u][e] = 0.f;
            }
#pragma unroll
            for (int kk = 0; kk < KS; ++kk) {
                __builtin_amdgcn_sched_barrier(0);
                if (kk + kAhead < KS) read_step(kk + kAhead);
#pragma unroll
                for (int u = 0; u < VB; ++u)
#pragma unroll
                    for (int e = 0; e < RB; ++e) {
                        const float xv = x[kk % (kAhead + 1)][u][e];
                        if constexpr (!KAPPA) acc[u][e] = __builtin_amdgcn_mfma_f32_16x16x4f32(cf[e][kk], xv, acc[u][e], 0, 0, 0);
                        if constexpr (NORMS) nrm[u][e] = fmaf(xv, xv, nrm[u][e]);
                    }
            }
            __builtin_amdgcn_sched_barrier(0);
            // The prefetched tile goes to the other LDS buffer after the first block's MFMAs and
            // before any of this tile's stores: the counter of outstanding memory operations is
            // in order, so a wait for the prefetch registers issued after stores would wait for
            // those stores too (a trip to HBM per tile).  By now the loads have had a quarter
            // of the tile's time to arrive.  (The maximum-inner-product hashes have no registers
            // left for it at this point and keep the hand-over at the end of the tile.)
            if constexpr (kEarlyStash) {
                if (vb == 0 && t_next < ntiles) stash(tile + (cur ^ 1) * buf_floats);
            }
            if constexpr (NORMS) {
                // lanes c, c + 16, c + 32, c + 48 hold the partial sums of vector c: one more MFMA
                // with an all-ones row operand adds them, D[i][c] = sum_kq partial[kq][c] in every
                // row i, so every lane of the vector gets the same bits (the same instruction on
                // the same operands in the kappa~ pass and in the data hash)
#pragma unroll
                for (int u = 0; u < VB; ++u)
#pragma unroll
                    for (int e = 0; e < RB; ++e) {
                        const float4v sum = __builtin_amdgcn_mfma_f32_16x16x4f32(1.0f, nrm[u][e], float4v{0.f, 0.f, 0.f, 0.f}, 0, 0, 0);
                        nrm[u][e] = sum[0];
                        if constexpr (KAPPA) kmax[e] = fmaxf(kmax[e], nrm[u][e]);  // vectors beyond N are zero rows
                    }
            }
            if constexpr (KAPPA) continue;
#pragma unroll
            for (int u = 0; u < VB; ++u) {
                uint4 v[RB];
#pragma unroll
                for (int e = 0; e < RB; ++e) {
                    uint32_t w4[4];
                    if constexpr (MDATA || MQUERY) {
                        // data: sqrt(kappa~^2 - ||S(v)||^2) (0 when the norm exceeds kappa~); query: 1 / ||S(u)||
                        float scale;
                        if constexpr (MDATA) {
                            scale = __builtin_amdgcn_sqrtf(fmaxf(kap[e] - nrm[u][e], 0.f));  // 1 ulp; sqrt(0) = 0
                        } else {
                            scale = nrm[u][e] > 0.f ? __builtin_amdgcn_rsqf(nrm[u][e]) : 0.f;
                            acc[u][e] *= scale;
                        }
                        // extra step: + a0_j * scale (data) + b~_j (ids)
                        const float one = a.raw ? 0.f : 1.f;
                        const float colx = q == 0 ? (MDATA ? scale : 0.f) : (q == 1 ? one : 0.f);
                        acc[u][e] = __builtin_amdgcn_mfma_f32_16x16x4f32(cfx[e], colx, acc[u][e], 0, 0, 0);
                    }
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const float p = acc[u][e][r];
                        if (PROJ || (NORMS && a.raw)) {
                            w4[r] = __float_as_uint(p);
                        } else if constexpr (NORMS) {
                            w4[r] = (uint32_t)(int)floorf(a.w_is_pow2 ? p * a.inv_w : p / a.w);  // b~ is in p already
                        } else {
                            const float s = a.w_is_pow2 ? fmaf(p, a.inv_w, bq[e][r] * a.inv_w) : (p + bq[e][r]) / a.w;
                            w4[r] = (uint32_t)(int)floorf(s);
                        }
                    }
                    v[e] = make_uint4(w4[0], w4[1], w4[2], w4[3]);
                }
                if constexpr (KEYS) {
                    // Horner fold of the lane's four ids of each block, times the lane's power of
                    // C, summed over the four lanes (c, q = 0..3) that hold a block; a table of 32
                    // functions is the wave's two blocks
                    uint64_t part[RB];
#pragma unroll
                    for (int e = 0; e < RB; ++e) {
                        uint64_t h = v[e].x;
                        h = h * kKeyMultiplier + v[e].y;
                        h = h * kKeyMultiplier + v[e].z;
                        h = h * kKeyMultiplier + v[e].w;
                        part[e] = h * pw[e];
                    }
                    if (RB == 2 && a.blocks_per_table == 2) part[0] += part[1];
#pragma unroll
                    for (int e = 0; e < RB; ++e) {
                        part[e] += __shfl_xor(part[e], 16);
                        part[e] += __shfl_xor(part[e], 32);
                    }
                    const uint64_t row = row0 + (vb + u) * 16 + opaque(c16);
                    uint64_t *keys = reinterpret_cast<uint64_t *>(a.out) + row * (a.nblocks / a.blocks_per_table);
                    if (opaque(q) == 0 && row < a.N && block0 < a.nblocks) {
                        if (RB == 2 && a.blocks_per_table == 1) {
                            if (block0 + 1 < a.nblocks) {
                                *reinterpret_cast<ulonglong2 *>(keys + block0) = make_ulonglong2(part[0], part[1]);
                            } else {
                                keys[block0] = part[0];
                            }
                        } else {
                            keys[block0 / a.blocks_per_table] = part[0];
                        }
                    }
                    continue;
                }
                if constexpr (RB == 2) {
                    if (a.staged) {  // uniform
                        // The wave's two blocks are 32 consecutive functions = 128 bytes of a
                        // vector's ids, held as 16-byte pieces by 8 lanes: lanes (c, q), q = 0..3,
                        // hold piece q (block 0) and piece 4 + q (block 1) of vector c.  Lanes c
                        // and c ^ 8 swap one piece each (a rotation by 8 inside the row of 16
                        // lanes, DPP), after which one store covers vectors 0..7 and another
                        // vectors 8..15 with whole 128-byte lines (a store that leaves 64-byte
                        // halves of 16 lines is a fifth slower on this memory system).
                        const uint32_t lane_o = opaque(lane);
                        const bool upper = lane_o & 8;
                        const uint4 give = upper ? v[0] : v[1];
                        uint4 got;
                        got.x = (uint32_t)__builtin_amdgcn_mov_dpp((int)give.x, 0x128, 0xf, 0xf, true);  // row_ror:8
                        got.y = (uint32_t)__builtin_amdgcn_mov_dpp((int)give.y, 0x128, 0xf, 0xf, true);
                        got.z = (uint32_t)__builtin_amdgcn_mov_dpp((int)give.z, 0x128, 0xf, 0xf, true);
                        got.w = (uint32_t)__builtin_amdgcn_mov_dpp((int)give.w, 0x128, 0xf, 0xf, true);
                        // lane (c, q): piece q of vector c % 8 (+ 8 for the second store) when c < 8,
                        // piece 4 + q when c >= 8
                        const uint4 first = upper ? got : v[0], second = upper ? v[1] : got;
                        const uint64_t row = row0 + (vb + u) * 16 + (lane_o & 7);
                        uint32_t *dst = reinterpret_cast<uint32_t *>(a.out) + row * a.k + block0 * 16 +
                                        ((upper ? 4u : 0u) + (lane_o >> 4)) * 4;
                        if (block0 < a.nblocks) {
                            if (row < a.N) *reinterpret_cast<uint4 *>(dst) = first;
                            if (row + 8 < a.N) *reinterpret_cast<uint4 *>(dst + 8 * (size_t)a.k) = second;
                        }
                        continue;
                    }
                }
                const uint64_t row = row0 + (vb + u) * 16 + opaque(c16);
#pragma unroll
                for (int e = 0; e < RB; ++e)
                    if (fn0[e] < a.k && row < a.N)
                        *reinterpret_cast<uint4 *>(reinterpret_cast<uint32_t *>(a.out) + row * a.k + fn0[e]) = v[e];
            }
        }

        if constexpr (!kEarlyStash) {
            if (t_next < ntiles) stash(tile + (cur ^ 1) * buf_floats);
        }
        __syncthreads();  // next buffer complete; everyone is done with the current one
        cur ^= 1;
    }
    if constexpr (KAPPA) {
        // max over the wave's 16 vector columns, then one atomic per block; norms are >= 0, so
        // their bit patterns order like the values
#pragma unroll
        for (int e = 0; e < RB; ++e) {
            float v = kmax[e];
#pragma unroll
            for (int s = 1; s < 16; s *= 2) v = fmaxf(v, __shfl_xor(v, s));
            if (lane == 0 && block0 + e < a.nblocks)
                atomicMax(reinterpret_cast<unsigned int *>(a.out) + (block0 + e) / a.blocks_per_table, __float_as_uint(v));
        }
    }
}

__global__ void clear_kernel(float *d, uint32_t count) {
    const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) d[i] = 0.f;
}

template <typename Kernel>
int launch(Kernel fn, uint32_t lds_bytes, const SharedArgs &args, dim3 grid, uint32_t lanes, hipStream_t stream) {
    if (ensure_lds_limit(reinterpret_cast<const void *>(fn), lds_bytes) != LSH_OK) return LSH_ERR_HIP;
    hipLaunchKernelGGL(fn, grid, dim3(lanes), lds_bytes, stream, args);
    return hipGetLastError() == hipSuccess ? LSH_OK : LSH_ERR_HIP;
}

}  // namespace

// Shapes the kernel takes: n a multiple of 4 whose tile of >= 32 vectors (>= 16 for lists of more
// than 64 samples) fits LDS twice, lists of at most 128 samples, tables of a multiple of 4 functions.
SharedPlan plan_shared(uint32_t n, uint32_t k, uint32_t m, uint32_t L) {
    SharedPlan pl;
    if (!L || k % L || (n & 3) || m > 128 || m == n) return pl;
    const uint32_t g = k / L;
    if (g & 3) return pl;
    pl.stride = n + 4;
    pl.g = g;
    pl.ksteps = m <= 32 ? 8 : m <= 64 ? 16 : 32;
    pl.blocks_per_table = (g + 15) / 16;
    pl.nblocks = L * pl.blocks_per_table;
    // One workgroup of 16 waves per CU with the largest tile that fits LDS twice (two
    // workgroups of 8 waves on 64-vector tiles measured slower).  A wave keeps 2 * rb * ksteps
    // coefficient and offset registers: at most 32 of a lane's 128.
    struct Shape { uint32_t waves, rows, per_cu; };
    for (const Shape sh : {Shape{16, 128, 1}, Shape{16, 64, 1}, Shape{16, 32, 1}, Shape{16, 16, 1}}) {
        if (sh.rows == 16 && pl.ksteps != 32) continue;  // only the 32-step kernel walks single 16-vector blocks
        if (2ull * sh.rows * pl.stride * 4 * sh.per_cu > kLdsBudget) continue;
        if ((uint64_t)sh.rows * (n / 4) > (uint64_t)kPre * sh.waves * 64) continue;
        pl.waves = sh.waves;
        pl.rows = sh.rows;
        pl.per_cu = sh.per_cu;
        break;
    }
    if (!pl.rows) return pl;
    const uint32_t rb_max = pl.ksteps >= 32 ? 1 : (pl.waves == 8 ? 32 : 16) / pl.ksteps;
    pl.rb = 1;
    while (pl.rb < rb_max && pl.waves * pl.rb < pl.nblocks) pl.rb *= 2;
    pl.kblocks = (pl.nblocks + pl.waves * pl.rb - 1) / (pl.waves * pl.rb);
    pl.lds_bytes = 2 * pl.rows * pl.stride * 4;
    // whole-line stores when a wave's two blocks are 32 consecutive functions and every block is full
    pl.staged = pl.rb == 2 && g % 16 == 0 && pl.nblocks % 2 == 0;
    pl.supported = true;
    return pl;
}

// Device tables in the kernel's operand layout (see the file comment).
void build_shared_tables(const lsh_params *p, std::vector<float> &coef, std::vector<uint32_t> &sample_off,
                         std::vector<float> &offset, std::vector<float> &extra) {
    const SharedPlan &pl = p->shared_plan;
    const uint32_t ks = pl.ksteps, blocks = pl.kblocks * pl.waves * pl.rb;
    coef.assign((size_t)blocks * ks * 64, 0.f);
    sample_off.assign((size_t)blocks * ks * 4, 4u * p->n);  // default: the row's zero pad
    offset.assign((size_t)blocks * 16, 0.f);
    extra.assign((size_t)blocks * 64, 0.f);
    // Which sample sits in which slot (step kk, lane group kq) is free: a projection is a sum.
    // The 64 lanes of a column-operand read address banks 4 * vector + coordinate (mod 64), so
    // the four coordinates of a step hit distinct banks iff they differ modulo 4.  Per table,
    // deal the samples (and the pads, which read coordinate n = 0 mod 4) to the steps from the
    // residue classes with the most left, one per class where four classes are left.
    constexpr uint32_t kPad = 0xFFFFFFFFu;
    std::vector<uint32_t> slot_sample((size_t)(pl.nblocks / pl.blocks_per_table) * ks * 4, kPad);
    for (uint32_t table = 0; table < pl.nblocks / pl.blocks_per_table; ++table) {
        std::vector<uint32_t> cls[4];
        for (uint32_t smp = p->m; smp-- > 0;) cls[p->idx[(size_t)table * pl.g * p->m + smp] & 3].push_back(smp);
        for (uint32_t pad = p->m; pad < ks * 4; ++pad) cls[0].insert(cls[0].begin(), kPad);  // pads leave last
        for (uint32_t kk = 0; kk < ks; ++kk) {
            uint32_t taken[4] = {0, 0, 0, 0};
            for (uint32_t kq = 0; kq < 4; ++kq) {
                // the class with the most left among those not used in this step, else the fullest
                int best = -1;
                for (int pass = 0; pass < 2 && best < 0; ++pass)
                    for (int c = 0; c < 4; ++c)
                        if (!cls[c].empty() && (pass == 1 || !taken[c]) &&
                            (best < 0 || cls[c].size() > cls[best].size()))
                            best = c;
                slot_sample[((size_t)table * ks + kk) * 4 + kq] = cls[best].back();
                cls[best].pop_back();
                taken[best] = 1;
            }
        }
    }
    for (uint32_t blk = 0; blk < pl.nblocks; ++blk) {
        const uint32_t table = blk / pl.blocks_per_table, first = (blk % pl.blocks_per_table) * 16;
        for (uint32_t kk = 0; kk < ks; ++kk)
            for (uint32_t kq = 0; kq < 4; ++kq) {
                // sample number; a pad slot keeps coefficient 0 and reads the row's zero pad
                const uint32_t s = slot_sample[((size_t)table * ks + kk) * 4 + kq];
                if (s < p->m)
                    sample_off[((size_t)blk * ks + kk) * 4 + kq] = 4u * p->idx[(size_t)table * pl.g * p->m + s];
                for (uint32_t i = 0; i < 16; ++i) {
                    const uint32_t in_table = first + i;
                    if (s < p->m && in_table < pl.g)
                        coef[((size_t)blk * ks + kk) * 64 + kq * 16 + i] =
                            p->coef[(size_t)(table * pl.g + in_table) * p->m + s];
                }
            }
        for (uint32_t i = 0; i < 16; ++i)
            if (first + i < pl.g) {
                offset[(size_t)blk * 16 + i] = p->off[table * pl.g + first + i];
                extra[(size_t)blk * 64 + i] = p->extra[table * pl.g + first + i];       // row operand, sample lane 0
                extra[(size_t)blk * 64 + 16 + i] = p->off[table * pl.g + first + i];    // sample lane 1
            }
    }
}

// Keys come out of the kernel when the key groups are the tables and a table is one block or
// the two blocks of one wave.
bool shared_keys_ok(const lsh_params *p, uint32_t L) {
    const SharedPlan &pl = p->shared_plan;
    return pl.supported && L == p->shared_tables && (pl.blocks_per_table == 1 || (pl.blocks_per_table == 2 && pl.rb == 2));
}

int clear_floats(float *d, uint32_t count, void *stream) {
    if (!count) return LSH_OK;
    hipLaunchKernelGGL(clear_kernel, dim3((count + 255) / 256), dim3(256), 0, reinterpret_cast<hipStream_t>(stream), d, count);
    return hipGetLastError() == hipSuccess ? LSH_OK : LSH_ERR_HIP;
}

int launch_shared(const lsh_params *p, int ep, const float *d_data, uint64_t N, void *d_out, void *stream,
                  const float *d_kappa2, int raw) {
    const SharedPlan &pl = p->shared_plan;
    if (!pl.supported) return LSH_ERR_UNSUPPORTED;
    SharedArgs a;
    a.data = d_data;
    a.N = N;
    a.n = p->n;
    a.k = p->k;
    a.g = pl.g;
    a.rows = pl.rows;
    a.stride = pl.stride;
    a.n4_magic = (uint32_t)((1ull << 32) / (p->n / 4)) + 1;
    a.blocks_per_table = pl.blocks_per_table;
    a.nblocks = pl.nblocks;
    a.coef = p->d_shared_coef;
    a.sample_off = p->d_shared_sample_off;
    a.offset = p->d_shared_offset;
    a.extra = p->d_shared_extra;
    a.kappa2 = d_kappa2;
    a.raw = raw;
    a.w = p->w;
    a.inv_w = 1.0f / p->w;
    int exp2 = 0;
    a.w_is_pow2 = (std::frexp(p->w, &exp2) == 0.5f) ? 1 : 0;
    a.out = d_out;
    a.staged = pl.staged ? 1 : 0;
    const uint64_t ntiles = (N + pl.rows - 1) / pl.rows;
    // persistent workgroups, as many as fit the CUs; a multiple of 8 along x, so that the
    // kblocks workgroups sharing a vector tile land on one XCD
    uint64_t gx = (uint64_t)p->num_cus * pl.per_cu / pl.kblocks;
    gx = gx < 8 ? 8 : gx / 8 * 8;
    if (gx > ntiles) gx = ntiles;
    dim3 grid((uint32_t)gx, pl.kblocks);
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    const bool geom = p->n == 128 && pl.rows == 128 && pl.stride == 132;
#define LSH_SHARED_EP(KS_, RB_, WAVES_, G_, EP_) \
    if (ep == EP_) return launch(&shared_kernel<KS_, RB_, WAVES_, EP_, G_>, pl.lds_bytes, a, grid, WAVES_ * 64, s);
#define LSH_SHARED_CASE(KS_, RB_, WAVES_, G_) \
    if (pl.ksteps == KS_ && pl.rb == RB_ && pl.waves == WAVES_ && geom == G_) { \
        LSH_SHARED_EP(KS_, RB_, WAVES_, G_, 0) LSH_SHARED_EP(KS_, RB_, WAVES_, G_, 1) LSH_SHARED_EP(KS_, RB_, WAVES_, G_, 2) \
        LSH_SHARED_EP(KS_, RB_, WAVES_, G_, 3) LSH_SHARED_EP(KS_, RB_, WAVES_, G_, 4) LSH_SHARED_EP(KS_, RB_, WAVES_, G_, 5) \
        return LSH_ERR_INVALID_ARG; \
    }
    LSH_SHARED_CASE(8, 1, 16, false) LSH_SHARED_CASE(8, 2, 16, false) LSH_SHARED_CASE(16, 1, 16, false)
    LSH_SHARED_CASE(32, 1, 16, false)
    LSH_SHARED_CASE(8, 1, 16, true) LSH_SHARED_CASE(8, 2, 16, true) LSH_SHARED_CASE(16, 1, 16, true)
#undef LSH_SHARED_CASE
#undef LSH_SHARED_EP
    return LSH_ERR_UNSUPPORTED;
}

}  // namespace lsh
