// FastLSH with ONE sample S per table (Sec. 3.1 read literally; Sec. 4.1: given S, a table's
// functions are E2LSH functions on the sub-vector S(v)) for large dimensions on gfx950: the
// shapes whose vectors do not fit LDS whole (the 4096- and 16384-dimensional workloads).
//
//   p_j(v) = sum_{i<m} a~_j[i] * v[S_l[i]],  l = table of function j;  h_j = floor((p_j + b~_j) / w)
//
// Per (vector, table) the m sampled coordinates are gathered once and contracted with the
// table's g coefficient vectors on the matrix cores: k * m / g gathers per vector instead of
// k * m, and the multiply-adds leave the vector ALU.  The launch is then bound by reading the
// data.
//
// A tile is 16 vectors x a range of 1024 coordinates, kept row-major in LDS ([vector][1024 + 4]
// floats, two buffers); as in ranged_kernel.hip a workgroup is 8 contracting waves plus 4
// loading waves that fetch the next (tile, range) behind the contraction, one barrier per step.
// A contracting wave owns up to 16 blocks of 16 consecutive functions of one table (the MFMA
// rows of v_mfma_f32_16x16x4_f32, the 16 vectors being its columns).  The host buckets every
// table's samples by range and deals them to MFMA steps of four samples; per step a lane reads
// one coefficient (row l % 16, sample l / 16 of the step) and one LDS offset from its list,
// reads the sampled coordinate of vector l % 16 from the tile (the four coordinates of a step
// differ modulo 4 where the table allows it, so that the 64 lanes hit 64 banks), and issues
// one MFMA.  A wave's lists form one stream of list blocks (six steps each) in consumption order
// (range after range, block of functions after block), prefetched three list blocks ahead
// through a ring of four register sets; accumulators persist across ranges.  A table's list
// for one range is padded to whole list blocks with coefficient 0 (the matrix pipe has time to
// spare: the launch is bound by memory).
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstring>
#include <vector>

#include "lsh_internal.h"

namespace lsh {
namespace {

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef uint32_t uintx4 __attribute__((ext_vector_type(4)));

constexpr int kCWs = (int)kRangeComputeWaves;  // contracting waves
constexpr int kLWs = 4;                        // loading waves: wave kCWs + s loads vectors 4s .. 4s + 3
constexpr int kThreadsSR = (kCWs + kLWs) * 64;
constexpr int kCs = (int)kRangeCoords;
constexpr int kRowFloats = kCs + 4;            // row stride: 4 floats of padding spread the vectors over the banks
constexpr int kBufBytesSR = 16 * kRowFloats * 4;
constexpr int kUs = (int)kSharedRangeBlockSteps;  // MFMA steps per lane in a list block

// Returns v through an empty asm: values derived from it are recomputed where they are used
// instead of being kept in registers across the contraction loops.
__device__ __forceinline__ uint32_t fresh(uint32_t v) {
    asm volatile("" : "+v"(v));
    return v;
}

struct SharedRangedArgs {
    const float *data;  // [N][n]
    uint64_t N;
    uint32_t n, k, g, blocks_per_table, nblocks, R;
    const float *off;   // [>= k]
    float w, inv_w;
    int w_is_pow2, proj;
    void *out;
    const uint2 *lists;  // list blocks: kUs x 64 lanes x {coefficient bits, LDS byte offset}
};

template <int BPW>
__global__ __launch_bounds__(kThreadsSR) void shared_ranged_kernel(const SharedRangedArgs a,
                                                                   const uint32_t *__restrict__ list_len,
                                                                   const uint2 *__restrict__ streams) {
    extern __shared__ __align__(16) char lds_sr[];  // 2 buffers x [16 vectors][1028 floats]
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint32_t lane = threadIdx.x & 63;
    const uint32_t n = a.n, R = a.R;
    const uint64_t ntiles = (a.N + 15) / 16;
    const uint64_t first_tile = blockIdx.x;  // the host launches at most ntiles workgroups along x

    if (wave >= (uint32_t)kCWs) {
        // ---- loading waves: four vectors each, a vector's range as four pieces of 256 coordinates
        // (a wave instruction moves 1 KB of one vector), two vectors at a time
        const uint32_t v0 = (wave - kCWs) * 4;
        uint64_t t_next = first_tile;
        uint32_t r_next = 0, b = 1;
        for (;;) {
            const bool more = t_next < ntiles;
            if (more) {
                const uint32_t c0 = r_next * kCs;
                char *dst = lds_sr + (b ^ 1) * kBufBytesSR + lane * 16;
#pragma unroll
                for (int half = 0; half < 2; ++half) {
                    floatx4 pre[2][4];
#pragma unroll
                    for (int v = 0; v < 2; ++v) {
                        uint64_t row = t_next * 16 + v0 + 2 * half + v;
                        row = row < a.N ? row : a.N - 1;  // rows beyond the data repeat the last vector (never stored)
                        const float *src = a.data + row * n;
#pragma unroll
                        for (int piece = 0; piece < 4; ++piece) {
                            const uint32_t c = c0 + piece * 256 + lane * 4;
                            // coordinates beyond n read the row's first ones; zeros are stored for them
                            pre[v][piece] = *reinterpret_cast<const floatx4 *>(src + (c < n ? c : 0u));
                        }
                    }
#pragma unroll
                    for (int v = 0; v < 2; ++v)
#pragma unroll
                        for (int piece = 0; piece < 4; ++piece) {
                            const bool inside = c0 + piece * 256 + lane * 4 < n;
                            const floatx4 x = pre[v][piece];
                            const floatx4 z = {inside ? x[0] : 0.f, inside ? x[1] : 0.f, inside ? x[2] : 0.f, inside ? x[3] : 0.f};
                            *reinterpret_cast<floatx4 *>(dst + (v0 + 2 * half + v) * kRowFloats * 4 + piece * 1024) = z;
                        }
                }
            }
            __syncthreads();
            if (!more) break;
            b ^= 1;
            if (++r_next == R) {
                r_next = 0;
                t_next += gridDim.x;
            }
        }
        return;
    }

    // ---- contracting waves
    const uint32_t stream_id = blockIdx.y * kCWs + wave;
    const uint2 si = streams[stream_id];  // {first list block, list blocks}
    const uint2 *sbase = a.lists + (size_t)si.x * (kUs * 64) + lane;
    const uint32_t sblocks = si.y;
    const uint32_t *len_base = list_len + (size_t)stream_id * R * BPW;
    // List registers: a ring of four blocks.  Block i of the stream lives in ring[i % 4]; when
    // block i is about to be used, block i + 3 is asked for (into the set used just before), so
    // a block has the time of three others to arrive: a table's list for one range is rarely
    // longer than one block, far shorter than a trip to L2.  The ring position is static in the
    // code: the loop over a list's blocks is entered at the position where the last list ended.
    uint2 ring[4][kUs];
    uint32_t next_block = 0;
    auto load_block = [&](uint2 (&blk)[kUs]) __attribute__((always_inline)) {
        const uint2 *src = sbase + (size_t)next_block * (kUs * 64);
#pragma unroll
        for (int i = 0; i < kUs; ++i) blk[i] = src[i * 64];
        next_block = next_block + 1 == sblocks ? 0 : next_block + 1;
    };
    if (sblocks) {
        load_block(ring[0]);
        load_block(ring[1]);
        load_block(ring[2]);
    }
    uint32_t phase = 0;  // ring set of the next block to use
    const uint32_t row_off = (lane & 15) * kRowFloats * 4;  // this lane's vector in the tile

    __syncthreads();  // first buffer written
    uint32_t b = 0;
    for (uint64_t t = first_tile; t < ntiles; t += gridDim.x) {
        floatx4 acc[BPW];
#pragma unroll
        for (int f = 0; f < BPW; ++f) acc[f] = floatx4{0.f, 0.f, 0.f, 0.f};
        for (uint32_t r = 0; r < R; ++r) {
            const char *buf = lds_sr + b * kBufBytesSR + row_off;
#pragma unroll
            for (int f = 0; f < BPW; ++f) {
                uint32_t left = len_base[r * BPW + f];  // list blocks of kUs steps (the last one padded with zero steps)
                // one block: all reads, then the MFMAs (padding steps multiply zeros: the matrix pipe has time to spare)
                auto run = [&](const uint2 (&blk)[kUs]) __attribute__((always_inline)) {
                    float x[kUs];
#pragma unroll
                    for (int s = 0; s < kUs; ++s) x[s] = *reinterpret_cast<const float *>(buf + blk[s].y);
#pragma unroll
                    for (int s = 0; s < kUs; ++s)
                        acc[f] = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(blk[s].x), x[s], acc[f], 0, 0, 0);
                };
                while (left) {
                    switch (phase) {
                        case 0:
                            load_block(ring[3]);
                            run(ring[0]);
                            if (--left == 0) { phase = 1; break; }
                            [[fallthrough]];
                        case 1:
                            load_block(ring[0]);
                            run(ring[1]);
                            if (--left == 0) { phase = 2; break; }
                            [[fallthrough]];
                        case 2:
                            load_block(ring[1]);
                            run(ring[2]);
                            if (--left == 0) { phase = 3; break; }
                            [[fallthrough]];
                        default:
                            load_block(ring[2]);
                            run(ring[3]);
                            --left;
                            phase = 0;
                    }
                }
            }
            if (r + 1 == R) {
                // register e of a block's accumulator: function 4 (l / 16) + e of the block, vector l % 16
                const uint32_t ln = fresh(lane);
                const uint64_t vec = t * 16 + (ln & 15);
#pragma unroll
                for (int f = 0; f < BPW; ++f) {
                    const uint32_t blk = (blockIdx.y * BPW + f) * kCWs + wave;  // global block number
                    const uint32_t in_table = (blk % a.blocks_per_table) * 16 + 4 * (ln >> 4);
                    const uint32_t j = (blk / a.blocks_per_table) * a.g + in_table;
                    if (blk < a.nblocks && in_table < a.g && vec < a.N) {  // g is a multiple of 4: whole quads
                        uintx4 v;
                        if (a.proj) {
#pragma unroll
                            for (int e = 0; e < 4; ++e) v[e] = __float_as_uint(acc[f][e]);
                        } else {
                            const floatx4 bq = *reinterpret_cast<const floatx4 *>(a.off + j);
#pragma unroll
                            for (int e = 0; e < 4; ++e) {
                                const float h = a.w_is_pow2 ? fmaf(acc[f][e], a.inv_w, bq[e] * a.inv_w) : (acc[f][e] + bq[e]) / a.w;
                                v[e] = (uint32_t)(int)floorf(h);
                            }
                        }
                        *reinterpret_cast<uintx4 *>(reinterpret_cast<uint32_t *>(a.out) + vec * a.k + j) = v;
                    }
                }
            }
            __syncthreads();  // the other buffer is complete, everyone is done with this one
            b ^= 1;
        }
    }
}

}  // namespace

// Shapes the kernel takes: one sample per table, n a multiple of 4, tables of a multiple of 4
// functions, offsets aligned for 16-byte reads (k a multiple of 4 follows).
SharedRangedPlan plan_shared_ranged(uint32_t n, uint32_t k, uint32_t m, uint32_t L) {
    SharedRangedPlan pl;
    if (!L || k % L || (n & 3) || m >= n) return pl;
    const uint32_t g = k / L;
    if (g & 3) return pl;
    pl.g = g;
    pl.blocks_per_table = (g + 15) / 16;
    pl.nblocks = L * pl.blocks_per_table;
    const uint32_t per_wg_max = kRangeComputeWaves * kSharedRangeBlocksPerWave;
    pl.kblocks = (pl.nblocks + per_wg_max - 1) / per_wg_max;
    const uint32_t per_wg = (pl.nblocks + pl.kblocks - 1) / pl.kblocks;
    pl.bpw = (per_wg + kRangeComputeWaves - 1) / kRangeComputeWaves;
    // instantiated: 1, 2, 4, 8, 16 blocks per wave
    uint32_t inst = 1;
    while (inst < pl.bpw) inst *= 2;
    pl.bpw = inst;
    pl.R = (n + kRangeCoords - 1) / kRangeCoords;
    pl.supported = true;
    return pl;
}

// Host tables: per contracting wave one stream of list blocks in consumption order (range after
// range, within a range the wave's blocks one after the other); per step and lane the
// coefficient of (row l % 16, sample l / 16) and the LDS byte offset of that sample's coordinate
// inside the range.
void build_shared_ranged_tables(const lsh_params *p, std::vector<uint32_t> &lists, std::vector<uint32_t> &list_len,
                                std::vector<uint32_t> &stream_info) {
    const SharedRangedPlan &pl = p->shared_ranged_plan;
    const uint32_t R = pl.R, CW = kRangeComputeWaves, U = kSharedRangeBlockSteps, bpw = pl.bpw, m = p->m;
    const uint32_t tables = pl.nblocks / pl.blocks_per_table, streams = pl.kblocks * CW;
    // per table and range: the samples dealt to steps of four, coordinates of a step distinct
    // modulo 4 where the classes allow it; 0xFFFFFFFF marks a padding slot
    constexpr uint32_t kPad = 0xFFFFFFFFu;
    std::vector<std::vector<uint32_t>> slots((size_t)tables * R);
    for (uint32_t table = 0; table < tables; ++table) {
        const uint32_t *S = &p->idx[(size_t)table * pl.g * m];
        std::vector<std::vector<uint32_t>> cls((size_t)R * 4);
        for (uint32_t smp = m; smp-- > 0;) cls[(size_t)(S[smp] / kRangeCoords) * 4 + (S[smp] & 3)].push_back(smp);
        for (uint32_t r = 0; r < R; ++r) {
            std::vector<uint32_t> *c = &cls[(size_t)r * 4];
            size_t left = c[0].size() + c[1].size() + c[2].size() + c[3].size();
            std::vector<uint32_t> &out = slots[(size_t)table * R + r];
            while (left) {
                bool taken[4] = {false, false, false, false};
                for (uint32_t kq = 0; kq < 4; ++kq) {
                    int best = -1;
                    for (int pass = 0; pass < 2 && best < 0; ++pass)
                        for (int q = 0; q < 4; ++q)
                            if (!c[q].empty() && (pass == 1 || !taken[q]) && (best < 0 || c[q].size() > c[best].size()))
                                best = q;
                    if (best < 0) {
                        out.push_back(kPad);
                    } else {
                        out.push_back(c[best].back());
                        c[best].pop_back();
                        taken[best] = true;
                        --left;
                    }
                }
            }
        }
    }
    list_len.assign((size_t)streams * R * bpw, 0);
    stream_info.assign((size_t)streams * 2, 0);
    lists.clear();
    uint32_t blocks = 0;
    for (uint32_t y = 0; y < pl.kblocks; ++y)
        for (uint32_t cw = 0; cw < CW; ++cw) {
            const uint32_t start = blocks;
            for (uint32_t r = 0; r < R; ++r)
                for (uint32_t f = 0; f < bpw; ++f) {
                    const uint32_t blk = (y * bpw + f) * CW + cw;
                    if (blk >= pl.nblocks) continue;
                    const uint32_t table = blk / pl.blocks_per_table, first = (blk % pl.blocks_per_table) * 16;
                    const std::vector<uint32_t> &sl = slots[(size_t)table * R + r];
                    const uint32_t steps = (uint32_t)sl.size() / 4;
                    const uint32_t nb = (steps + U - 1) / U;  // the steps that pad the last block multiply by zero
                    list_len[((size_t)(y * CW + cw) * R + r) * bpw + f] = nb;
                    lists.resize((size_t)(blocks + nb) * U * 64 * 2, 0u);
                    for (uint32_t s = 0; s < steps; ++s)
                        for (uint32_t kq = 0; kq < 4; ++kq) {
                            const uint32_t smp = sl[(size_t)s * 4 + kq];
                            const uint32_t coord = smp == kPad ? 0 : p->idx[(size_t)table * pl.g * m + smp] - r * kRangeCoords;
                            for (uint32_t i = 0; i < 16; ++i) {
                                float c = 0.f;
                                if (smp != kPad && first + i < pl.g) c = p->coef[(size_t)(table * pl.g + first + i) * m + smp];
                                uint32_t bits;
                                std::memcpy(&bits, &c, 4);
                                const size_t at = (((size_t)blocks + s / U) * U + s % U) * 64 + kq * 16 + i;
                                lists[at * 2] = bits;
                                lists[at * 2 + 1] = coord * 4;
                            }
                        }
                    blocks += nb;
                }
            stream_info[(size_t)(y * CW + cw) * 2] = start;
            stream_info[(size_t)(y * CW + cw) * 2 + 1] = blocks - start;
        }
    if (lists.empty()) lists.assign(2, 0u);
}

// proj != 0: raw projections instead of bucket ids
int launch_shared_ranged(const lsh_params *p, int proj, const float *d_data, uint64_t N, void *d_out, void *stream) {
    const SharedRangedPlan &pl = p->shared_ranged_plan;
    if (!pl.supported || !p->d_sr_lists) return LSH_ERR_UNSUPPORTED;
    SharedRangedArgs a;
    a.data = d_data;
    a.N = N;
    a.n = p->n;
    a.k = p->k;
    a.g = pl.g;
    a.blocks_per_table = pl.blocks_per_table;
    a.nblocks = pl.nblocks;
    a.R = pl.R;
    a.off = p->d_off;
    a.w = p->w;
    a.inv_w = 1.0f / p->w;
    int exp2 = 0;
    a.w_is_pow2 = (std::frexp(p->w, &exp2) == 0.5f) ? 1 : 0;
    a.proj = proj;
    a.out = d_out;
    a.lists = static_cast<const uint2 *>(p->d_sr_lists);
    const uint32_t *len = static_cast<const uint32_t *>(p->d_sr_list_len);
    const uint2 *streams = static_cast<const uint2 *>(p->d_sr_stream);
    const uint64_t ntiles = (N + 15) / 16;
    // one workgroup per CU (two 64 KB buffers); the kblocks workgroups of a tile run on one XCD
    uint64_t gx = (uint64_t)p->num_cus / pl.kblocks;
    gx = gx < 8 ? 8 : gx / 8 * 8;
    if (gx > ntiles) gx = ntiles;
    const dim3 grid((uint32_t)gx, pl.kblocks);
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
#define LSH_SR_CASE(B_) \
    case B_: { \
        auto fn = &shared_ranged_kernel<B_>; \
        if (ensure_lds_limit(reinterpret_cast<const void *>(fn), 2 * kBufBytesSR) != LSH_OK) return LSH_ERR_HIP; \
        hipLaunchKernelGGL(fn, grid, dim3(kThreadsSR), 2 * kBufBytesSR, s, a, len, streams); \
        break; \
    }
    switch (pl.bpw) {
        LSH_SR_CASE(1) LSH_SR_CASE(2) LSH_SR_CASE(4) LSH_SR_CASE(8) LSH_SR_CASE(16)
        default: return LSH_ERR_UNSUPPORTED;
    }
#undef LSH_SR_CASE
    return hipGetLastError() == hipSuccess ? LSH_OK : LSH_ERR_HIP;
}

}  // namespace lsh
