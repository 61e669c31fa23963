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
// one MFMA.
//
// With the samples gathered once per table, what is left to stream per tile is the lists: they
// come from L2, many times the bytes of the tile itself, and set the pace of the launch.  So
// they are kept small and cheap to fetch: a list block of U steps holds U x 64 coefficients (one
// per lane and step, a lane's four consecutive steps side by side so that one 16-byte load
// brings them) and, apart from them, one record of U 16-bit offsets per sample slot l / 16,
// which the sixteen lanes of a slot all read from the same address (a few bytes per block out
// of L2 instead of a word per lane and step).  A vector memory instruction costs the CU's
// memory pipeline 9 to 14 clocks whatever it hits, so their number per MFMA is what counts.
//
// The lists are also what a wave waits for if they arrive late, so they are asked for well ahead: a
// wave's list blocks (U steps each) form one stream in consumption order (range after range,
// block of functions after block) that runs through a ring of four register sets, a block
// being requested while the block three places before it is used.  The position in the ring
// must be the same on every path through the code (the compiler counts outstanding loads per
// path and otherwise waits for the newest), so list lengths are uniform: all lists of a range
// are padded with zero coefficients to the longest one, which is either one block for every
// range (short lists: the 16 blocks of a wave go round the ring) or a multiple of four blocks
// (a list goes round the ring whole turns).  The matrix pipe has time to spare for the padding
// steps: with the lists on time the launch is bound by reading the data.
//
// Maximum inner product search (appendix; one sample per table): as in shared_kernel.hip the
// lanes hold the sampled coordinates, so ||S_l(v)||^2 costs one multiply-add per LDS read
// (padding steps read a zero) and one MFMA with an all-ones row operand per block and tile to
// add the four partial sums of a vector.  Modes: 3 kappa~_l^2 = max_v ||S_l(v)||^2 (atomic
// maximum per table), 4 data hash, the projection plus a0_j sqrt(kappa~_l^2 - ||S_l(v)||^2),
// 5 query hash, the projection divided by ||S_l(u)||; the extra component and the offset enter
// as one more MFMA step with the row operand (a0_j, b~_j, 0, 0).
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstring>
#include <vector>

#include "lsh_internal.h"

namespace lsh {
namespace {

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef float floatx2 __attribute__((ext_vector_type(2)));
typedef uint32_t uintx4 __attribute__((ext_vector_type(4)));

constexpr int kCWs = (int)kRangeComputeWaves;  // contracting waves
constexpr int kLWs = 4;                        // loading waves: wave kCWs + s loads vectors 4s .. 4s + 3
constexpr int kThreadsSR = (kCWs + kLWs) * 64;
constexpr int kLongRing = 4;                   // ring sets for long lists (short lists: four)
constexpr int kCs = (int)kRangeCoords;
constexpr int kRowFloats = kCs + 4;            // row stride: 4 floats of padding spread the vectors over the banks
constexpr int kBufBytesSR = 16 * kRowFloats * 4;

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
    const float *extra;     // [nblocks][64] row operand (a0, b~, 0, 0) of the extra step (maximum inner product)
    const float *kappa2;    // [tables] kappa~_l^2, input of the data hash
    int raw;                // maximum-inner-product modes: projections instead of ids
    const float *coefs;     // list blocks: U steps x 64 lanes
    const uint32_t *offs;   // per list block: 4 sample slots x (U + 1) / 2 words of two 16-bit LDS byte offsets
};

// BPW: blocks of 16 functions per contracting wave; U: steps per list block; SHORT: every list is one block;
// MODE: 0 ids or projections, 3 kappa~^2, 4 maximum-inner-product data hash, 5 query hash
template <int BPW, int U, bool SHORT, int MODE>
__global__ __launch_bounds__(kThreadsSR) void shared_ranged_kernel(const SharedRangedArgs a,
                                                                   const uint32_t *__restrict__ range_groups,
                                                                   const uint2 *__restrict__ streams) {
    static_assert(!SHORT || BPW % 4 == 0, "short lists go round the ring of four by blocks");
    static_assert(U % 2 == 0, "a lane loads the coefficients of four or two steps at a time");
    constexpr int NR = SHORT ? 4 : kLongRing;  // ring sets
    constexpr bool KAPPA = MODE == 3, MDATA = MODE == 4, MQUERY = MODE == 5, NORMS = MODE >= 3;
    extern __shared__ __align__(16) char lds_sr[];  // 2 buffers x [16 vectors][1028 floats]
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint32_t lane = threadIdx.x & 63;
    const uint32_t n = a.n, R = a.R;
    const uint64_t ntiles = (a.N + 15) / 16;
    const uint64_t first_tile = blockIdx.x;  // the host launches at most ntiles workgroups along x

    if (wave >= (uint32_t)kCWs) {
        // ---- loading waves: four vectors each, a vector's range as four pieces of 256 coordinates
        // (a wave instruction moves 1 KB of one vector), all sixteen pieces in flight at once
        const uint32_t v0 = (wave - kCWs) * 4;
        uint64_t t_next = first_tile;
        uint32_t r_next = 0, b = 1;
        for (;;) {
            const bool more = t_next < ntiles;
            if (more) {
                const uint32_t c0 = r_next * kCs;
                char *dst = lds_sr + (b ^ 1) * kBufBytesSR + lane * 16;
                floatx4 pre[4][4];
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    uint64_t row = t_next * 16 + v0 + v;
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
                for (int v = 0; v < 4; ++v)
#pragma unroll
                    for (int piece = 0; piece < 4; ++piece) {
                        const bool inside = c0 + piece * 256 + lane * 4 < n;
                        const floatx4 x = pre[v][piece];
                        const floatx4 z = {inside ? x[0] : 0.f, inside ? x[1] : 0.f, inside ? x[2] : 0.f, inside ? x[3] : 0.f};
                        *reinterpret_cast<floatx4 *>(dst + (v0 + v) * kRowFloats * 4 + piece * 1024) = z;
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
    constexpr int OW = (U + 1) / 2;  // words of offsets per sample slot and block
    // uniform block pointers plus a per-lane index: the loads take a scalar base and a 32-bit lane offset
    const float *cbase = a.coefs + (size_t)si.x * (U * 64);
    const uint32_t *obase = a.offs + (size_t)si.x * (4 * OW);
    const uint32_t oslot = (lane >> 4) * OW;
    const uint32_t sblocks = si.y;  // at least the ring
    // Block i of the stream lives in ring set i % NR; when block i is about to be used, block
    // i + NR - 1 is requested into the set used just before.
    float ring_c[NR][U];
    uint32_t ring_o[NR][OW];
    uint32_t next_block = 0;
    auto load_block = [&](int set) __attribute__((always_inline)) {
        const float *cs = cbase + (size_t)next_block * (U * 64);
        const uint32_t *os = obase + (size_t)next_block * (4 * OW);
        // coefficients of four steps per load, [steps / 4][lane][4], then of the last two, [lane][2]
#pragma unroll
        for (int i = 0; i < U / 4; ++i) {
            const floatx4 c4 = *reinterpret_cast<const floatx4 *>(cs + i * 256 + lane * 4);
#pragma unroll
            for (int e = 0; e < 4; ++e) ring_c[set][4 * i + e] = c4[e];
        }
        if constexpr (U % 4 == 2) {
            const floatx2 c2 = *reinterpret_cast<const floatx2 *>(cs + (U / 4) * 256 + lane * 2);
            ring_c[set][U - 2] = c2[0];
            ring_c[set][U - 1] = c2[1];
        }
#pragma unroll
        for (int i = 0; i < OW; ++i) ring_o[set][i] = os[oslot + i];
        next_block = next_block + 1 == sblocks ? 0 : next_block + 1;
        __builtin_amdgcn_sched_barrier(0);  // the request stays here, three blocks ahead of its use
    };
#pragma unroll
    for (int i = 0; i < NR - 1; ++i) load_block(i);
    const uint32_t row_off = (lane & 15) * kRowFloats * 4;  // this lane's vector in the tile
    // the four floats after a row's 1024 coordinates stay zero: what padding steps read
    if (wave == 0) {
        const uint32_t buffer = lane >> 5, row = (lane >> 1) & 15, half = lane & 1;
        *reinterpret_cast<uint2 *>(lds_sr + buffer * kBufBytesSR + row * kRowFloats * 4 + kCs * 4 + half * 8) = make_uint2(0u, 0u);
    }
    [[maybe_unused]] float kmax[KAPPA ? BPW : 1];  // kappa~^2 pass: largest ||S(v)||^2 seen per block
#pragma unroll
    for (int f = 0; f < (KAPPA ? BPW : 1); ++f) kmax[f] = 0.f;

    __syncthreads();  // first buffer written
    uint32_t b = 0;
    for (uint64_t t = first_tile; t < ntiles; t += gridDim.x) {
        floatx4 acc[BPW];
        [[maybe_unused]] float nrm[NORMS ? BPW : 1];  // this lane's share of ||S(v)||^2 per block
#pragma unroll
        for (int f = 0; f < BPW; ++f) acc[f] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int f = 0; f < (NORMS ? BPW : 1); ++f) nrm[f] = 0.f;
        for (uint32_t r = 0; r < R; ++r) {
            const char *buf = lds_sr + b * kBufBytesSR + row_off;
            // one block: all reads, then the MFMAs
            auto run = [&](int set, floatx4 &c, [[maybe_unused]] float &n2) __attribute__((always_inline)) {
                float x[U];
                // the offsets are taken apart here, not where they were requested (which would wait for them there)
#pragma unroll
                for (int i = 0; i < OW; ++i) asm volatile("" : "+v"(ring_o[set][i]));
#pragma unroll
                for (int s = 0; s < U; ++s) {
                    const uint32_t off = (ring_o[set][s >> 1] >> (16 * (s & 1))) & 0xFFFFu;
                    x[s] = *reinterpret_cast<const float *>(buf + off);
                }
                __builtin_amdgcn_sched_barrier(0);  // all reads of the block go out before its first MFMA
#pragma unroll
                for (int s = 0; s < U; ++s) {
                    if constexpr (!KAPPA) c = __builtin_amdgcn_mfma_f32_16x16x4f32(ring_c[set][s], x[s], c, 0, 0, 0);
                    if constexpr (NORMS) n2 = fmaf(x[s], x[s], n2);
                }
                __builtin_amdgcn_sched_barrier(0);
            };
            if constexpr (SHORT) {
#pragma unroll
                for (int f = 0; f < BPW; ++f) {
                    load_block((f + 3) & 3);
                    run(f & 3, acc[f], nrm[NORMS ? f : 0]);
                }
            } else {
                const uint32_t groups = range_groups[r];  // turns of the ring per list in this range, at least one
#pragma unroll
                for (int f = 0; f < BPW; ++f) {
                    uint32_t left = groups;
                    do {
#pragma unroll
                        for (int q = 0; q < NR; ++q) {
                            load_block((q + NR - 1) % NR);
                            run(q, acc[f], nrm[NORMS ? f : 0]);
                        }
                    } while (--left);
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
                    [[maybe_unused]] float norm2 = 0.f;
                    if constexpr (NORMS) {
                        // lanes c, c + 16, c + 32, c + 48 hold the partial sums of vector c: an MFMA with an
                        // all-ones row operand adds them and leaves the sum in every lane of the vector (the
                        // same instruction on the same operands in the kappa~ pass and in the data hash)
                        const floatx4 sum = __builtin_amdgcn_mfma_f32_16x16x4f32(1.0f, nrm[f], floatx4{0.f, 0.f, 0.f, 0.f}, 0, 0, 0);
                        norm2 = sum[0];
                    }
                    if constexpr (KAPPA) {
                        kmax[f] = fmaxf(kmax[f], norm2);  // rows beyond N repeat the last vector
                        continue;
                    }
                    if constexpr (MDATA || MQUERY) {
                        if (blk < a.nblocks) {  // uniform
                            // data: sqrt(kappa~^2 - ||S(v)||^2) (0 when the norm exceeds kappa~); query: 1 / ||S(u)||
                            float scale;
                            if constexpr (MDATA) {
                                scale = __builtin_amdgcn_sqrtf(fmaxf(a.kappa2[blk / a.blocks_per_table] - norm2, 0.f));  // 1 ulp; sqrt(0) = 0
                            } else {
                                scale = norm2 > 0.f ? __builtin_amdgcn_rsqf(norm2) : 0.f;
                                acc[f] *= scale;
                            }
                            // the extra step: + a0_j * scale (data) + b~_j (ids)
                            const uint32_t slot = ln >> 4;
                            const float one = a.raw ? 0.f : 1.f;
                            const float colx = slot == 0 ? (MDATA ? scale : 0.f) : (slot == 1 ? one : 0.f);
                            acc[f] = __builtin_amdgcn_mfma_f32_16x16x4f32(a.extra[(size_t)blk * 64 + ln], colx, acc[f], 0, 0, 0);
                        }
                    }
                    if (blk < a.nblocks && in_table < a.g && vec < a.N) {  // g is a multiple of 4: whole quads
                        uintx4 v;
                        if (NORMS ? a.raw : a.proj) {
#pragma unroll
                            for (int e = 0; e < 4; ++e) v[e] = __float_as_uint(acc[f][e]);
                        } else if constexpr (NORMS) {
#pragma unroll
                            for (int e = 0; e < 4; ++e)  // b~ is in the accumulator already
                                v[e] = (uint32_t)(int)floorf(a.w_is_pow2 ? acc[f][e] * a.inv_w : acc[f][e] / a.w);
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
    if constexpr (KAPPA) {
        // max over the wave's 16 vector columns, then one atomic per block; norms are >= 0, so
        // their bit patterns order like the values
#pragma unroll
        for (int f = 0; f < BPW; ++f) {
            float v = kmax[f];
#pragma unroll
            for (int s = 1; s < 16; s *= 2) v = fmaxf(v, __shfl_xor(v, s));
            const uint32_t blk = (blockIdx.y * BPW + f) * kCWs + wave;
            if (lane == 0 && blk < a.nblocks)
                atomicMax(reinterpret_cast<unsigned int *>(a.out) + blk / a.blocks_per_table, __float_as_uint(v));
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
    // instantiated: 4, 8, 16 blocks per wave (blocks beyond the last one hold zero lists)
    uint32_t inst = 4;
    while (inst < pl.bpw) inst *= 2;
    pl.bpw = inst;
    pl.R = (n + kRangeCoords - 1) / kRangeCoords;
    pl.supported = true;
    return pl;
}

// Host tables: per contracting wave one stream of list blocks in consumption order (range after
// range, within a range the wave's blocks one after the other); per step and lane the
// coefficient of (row l % 16, sample l / 16) and the LDS byte offset of that sample's coordinate
// inside the range.  Chooses the list layout (steps per block, short or long lists) and notes
// it in the plan; range_groups holds, per range, the turns of the ring a list takes (long lists).
void build_shared_ranged_tables(const lsh_params *p, SharedRangedPlan &pl, std::vector<float> &coefs,
                                std::vector<uint32_t> &offs, std::vector<uint32_t> &range_groups,
                                std::vector<uint32_t> &stream_info, std::vector<float> *extra) {
    if (extra) {  // row operand of the extra step: sample slot 0 holds a0_j, slot 1 the offset b~_j
        extra->assign((size_t)pl.nblocks * 64, 0.f);
        for (uint32_t blk = 0; blk < pl.nblocks; ++blk) {
            const uint32_t table = blk / pl.blocks_per_table, first = (blk % pl.blocks_per_table) * 16;
            for (uint32_t i = 0; i < 16 && first + i < pl.g; ++i) {
                if (!p->extra.empty()) (*extra)[(size_t)blk * 64 + i] = p->extra[table * pl.g + first + i];
                (*extra)[(size_t)blk * 64 + 16 + i] = p->off[table * pl.g + first + i];
            }
        }
    }
    const uint32_t R = pl.R, CW = kRangeComputeWaves, bpw = pl.bpw, m = p->m;
    const uint32_t tables = pl.nblocks / pl.blocks_per_table, streams = pl.kblocks * CW;
    // per table and range: the samples dealt to steps of four, coordinates of a step distinct
    // modulo 4 where the classes allow it; 0xFFFFFFFF marks a padding slot
    constexpr uint32_t kPad = 0xFFFFFFFFu;
    std::vector<std::vector<uint32_t>> slots((size_t)tables * R);
    std::vector<uint32_t> longest(R, 0);  // steps of the longest list of a range
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
            longest[r] = std::max(longest[r], (uint32_t)out.size() / 4);
        }
    }
    // layout: short lists (one block of 4, 6 or 8 steps per list) if every list fits, else whole
    // turns of the long-list ring (4 blocks of 4, 6 or 8 steps), whichever pads least
    const uint32_t top = *std::max_element(longest.begin(), longest.end());
    range_groups.assign(R, 1);
    if (top <= 8) {
        pl.short_lists = true;
        pl.block_steps = top <= 4 ? 4 : top <= 6 ? 6 : 8;
    } else {
        pl.short_lists = false;
        uint64_t best = ~0ull;
        for (uint32_t u = 4; u <= 8; u += 2) {
            uint64_t cost = 0;
            for (uint32_t r = 0; r < R; ++r) cost += std::max(1u, (longest[r] + kLongRing * u - 1) / (kLongRing * u)) * kLongRing * u;
            if (cost <= best) {  // ties: the larger block (requests reach further ahead)
                best = cost;
                pl.block_steps = u;
            }
        }
        for (uint32_t r = 0; r < R; ++r)
            range_groups[r] = std::max(1u, (longest[r] + kLongRing * pl.block_steps - 1) / (kLongRing * pl.block_steps));
    }
    const uint32_t U = pl.block_steps, OW = (U + 1) / 2;
    std::vector<uint32_t> list_blocks(R);
    uint32_t per_stream = 0;
    for (uint32_t r = 0; r < R; ++r) {
        list_blocks[r] = pl.short_lists ? 1 : kLongRing * range_groups[r];
        per_stream += list_blocks[r] * bpw;
    }
    stream_info.assign((size_t)streams * 2, 0);
    coefs.assign((size_t)streams * per_stream * U * 64, 0.f);
    // steps and slots that only pad (coefficient zero) read one of the four zero floats that follow a
    // row's 1024 coordinates: four different banks per vector, like a step of real samples, and
    // nothing for the squared norms of the maximum-inner-product modes
    offs.assign((size_t)streams * per_stream * 4 * OW, 0u);
    for (size_t rec = 0; rec < offs.size() / OW; ++rec)
        for (uint32_t s = 0; s < U; ++s)
            offs[rec * OW + s / 2] |= ((kRangeCoords + (uint32_t)(rec & 3)) * 4u) << (16 * (s & 1));
    for (uint32_t y = 0; y < pl.kblocks; ++y)
        for (uint32_t cw = 0; cw < CW; ++cw) {
            const uint32_t stream = y * CW + cw;
            uint32_t blocks = stream * per_stream;
            stream_info[(size_t)stream * 2] = blocks;
            stream_info[(size_t)stream * 2 + 1] = per_stream;
            for (uint32_t r = 0; r < R; ++r)
                for (uint32_t f = 0; f < bpw; ++f, blocks += list_blocks[r]) {
                    const uint32_t blk = (y * bpw + f) * CW + cw;
                    if (blk >= pl.nblocks) continue;  // a list of zeros
                    const uint32_t table = blk / pl.blocks_per_table, first = (blk % pl.blocks_per_table) * 16;
                    const std::vector<uint32_t> &sl = slots[(size_t)table * R + r];
                    const uint32_t steps = (uint32_t)sl.size() / 4;
                    for (uint32_t s = 0; s < steps; ++s)
                        for (uint32_t kq = 0; kq < 4; ++kq) {
                            const uint32_t smp = sl[(size_t)s * 4 + kq];
                            if (smp == kPad) continue;
                            const size_t block = (size_t)blocks + s / U;
                            const uint32_t in_block = s % U;
                            const uint32_t coord = p->idx[(size_t)table * pl.g * m + smp] - r * kRangeCoords;
                            uint32_t &word = offs[(block * 4 + kq) * OW + in_block / 2];
                            word = (word & ~(0xFFFFu << (16 * (in_block & 1)))) | (coord * 4) << (16 * (in_block & 1));
                            // steps in fours [lane][4]; the last two of a block of six [lane][2]
                            const uint32_t four = in_block / 4 * 4, width = U - four >= 4 ? 4 : 2;
                            for (uint32_t i = 0; i < 16 && first + i < pl.g; ++i)  // rows beyond the table keep zero
                                coefs[(block * U + four) * 64 + (kq * 16 + i) * width + in_block % 4] =
                                    p->coef[(size_t)(table * pl.g + first + i) * m + smp];
                        }
                }
        }
}

// mode: 0 bucket ids, 1 raw projections, 3 kappa~^2 per table (atomic maximum into d_out), 4 and 5
// the maximum-inner-product data and query hashes (raw != 0: their projections)
int launch_shared_ranged(const lsh_params *p, int mode, const float *d_data, uint64_t N, void *d_out, void *stream,
                         const float *d_kappa2, int raw) {
    const SharedRangedPlan &pl = p->shared_ranged_plan;
    if (!pl.supported || !p->d_sr_lists || !p->d_sr_offs) return LSH_ERR_UNSUPPORTED;
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
    a.proj = mode == 1;
    a.extra = static_cast<const float *>(p->d_sr_extra);
    a.kappa2 = d_kappa2;
    a.raw = raw;
    if (mode >= 3 && !p->d_sr_extra) return LSH_ERR_UNSUPPORTED;
    a.out = d_out;
    a.coefs = static_cast<const float *>(p->d_sr_lists);
    a.offs = static_cast<const uint32_t *>(p->d_sr_offs);
    const uint32_t *groups = static_cast<const uint32_t *>(p->d_sr_list_len);
    const uint2 *streams = static_cast<const uint2 *>(p->d_sr_stream);
    const uint64_t ntiles = (N + 15) / 16;
    // one workgroup per CU (two 64 KB buffers); the kblocks workgroups of a tile run on one XCD
    uint64_t gx = (uint64_t)p->num_cus / pl.kblocks;
    gx = gx < 8 ? 8 : gx / 8 * 8;
    if (gx > ntiles) gx = ntiles;
    const dim3 grid((uint32_t)gx, pl.kblocks);
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
#define LSH_SR_LAUNCH(B_, U_, S_, M_) \
    { \
        auto fn = &shared_ranged_kernel<B_, U_, S_, M_>; \
        if (ensure_lds_limit(reinterpret_cast<const void *>(fn), 2 * kBufBytesSR) != LSH_OK) return LSH_ERR_HIP; \
        hipLaunchKernelGGL(fn, grid, dim3(kThreadsSR), 2 * kBufBytesSR, s, a, groups, streams); \
    }
#define LSH_SR_MODES(B_, U_, S_) \
    { \
        if (mode <= 1) LSH_SR_LAUNCH(B_, U_, S_, 0) \
        else if (mode == 3) LSH_SR_LAUNCH(B_, U_, S_, 3) \
        else if (mode == 4) LSH_SR_LAUNCH(B_, U_, S_, 4) \
        else if (mode == 5) LSH_SR_LAUNCH(B_, U_, S_, 5) \
        else return LSH_ERR_INVALID_ARG; \
    }
#define LSH_SR_STEPS(B_, U_) \
    case U_: \
        if (pl.short_lists) LSH_SR_MODES(B_, U_, true) else LSH_SR_MODES(B_, U_, false) \
        break;
#define LSH_SR_CASE(B_) \
    case B_: \
        switch (pl.block_steps) { \
            LSH_SR_STEPS(B_, 4) LSH_SR_STEPS(B_, 6) LSH_SR_STEPS(B_, 8) \
            default: return LSH_ERR_UNSUPPORTED; \
        } \
        break;
    switch (pl.bpw) {
        LSH_SR_CASE(4) LSH_SR_CASE(8) LSH_SR_CASE(16)
        default: return LSH_ERR_UNSUPPORTED;
    }
#undef LSH_SR_CASE
#undef LSH_SR_STEPS
#undef LSH_SR_MODES
#undef LSH_SR_LAUNCH
    return hipGetLastError() == hipSuccess ? LSH_OK : LSH_ERR_HIP;
}

}  // namespace lsh
