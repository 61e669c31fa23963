// FastLSH with ONE sample S per table (Sec. 3.1 read literally; Sec. 4.1: given S, a table's
// functions are E2LSH functions on the sub-vector S(v)) for large dimensions on gfx950: the
// shapes whose vectors do not fit LDS whole (the 4096- and 16384-dimensional workloads).
//
//   p_j(v) = sum_{i<m} a~_j[i] * v[S_l[i]],  l = table of function j;  h_j = floor((p_j + b~_j) / w)
//
// Per (vector, table) the m sampled coordinates are gathered once and contracted with the
// table's g coefficient vectors on the matrix cores: k * m / g gathers per vector instead of
// k * m, and the multiply-adds leave the vector ALU.
//
// A tile is 16 vectors.  LDS holds a ring of eight ranges of 256 coordinates of every vector,
// row-major ([vector][8 x 256 + 4] floats: coordinate c of a vector always sits at float
// c % 2048 of its row); as in ranged_kernel.hip a workgroup is 8 contracting waves plus 4
// loading waves, and a tile passes in stages: in stage s the loading waves write range s + 7
// while the contracting waves may read the ranges s .. s + 6.  A sample of range r can therefore
// be contracted in any of the stages r - 6 .. r, and the host uses that freedom to give every
// table the same number of MFMA steps in a stage (next paragraph) with next to no padding.
//
// A contracting wave owns up to 16 blocks of 16 consecutive functions of one table (the MFMA
// rows of v_mfma_f32_16x16x4_f32, the 16 vectors being its columns); their accumulators persist
// over the stages of a tile.  Per MFMA step of four samples a lane reads one coefficient (row
// l % 16, sample l / 16 of the step) and one LDS offset from its list, reads the sampled
// coordinate of vector l % 16 from the ring (the four coordinates of a step differ modulo 4
// where the table allows it, so that the 64 lanes hit 64 banks), and issues one MFMA.
//
// With the samples gathered once per table, what is left to stream per tile is the lists: they
// come from L2, many times the bytes of the tile itself.  So they are kept small and cheap to
// fetch: a list block of 8 steps holds 8 x 64 coefficients (one per lane and step, a lane's four
// consecutive steps side by side so that one 16-byte load brings them) and, apart from them, one
// record of eight 16-bit offsets per sample slot l / 16, which the sixteen lanes of a slot all
// read from the same address.  A vector memory instruction costs the CU's memory pipeline 9 to
// 14 clocks whatever it hits, so their number per MFMA is what counts.
//
// The lists are also what a wave waits for if they arrive late, so they are asked for well
// ahead: a wave's list blocks form one stream in consumption order that runs through a ring of
// four register sets, a block being requested while the block three places before it is used.
// The position in that ring must be the same on every path through the code (the compiler
// counts outstanding loads per path and otherwise waits for the newest), so the unit of work is
// a turn of the ring: 32 steps, 32 / B for each of the wave's B blocks in turn (the accumulator of
// a step is then fixed by its place in the turn), and a stage is a whole number of turns, the
// same for every wave (the host's table of turns per stage).  The barriers between stages order
// LDS traffic only, so list requests and id stores stay in flight across them.
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

#include "device_utils.h"
#include "lsh_internal.h"

namespace lsh {
namespace {

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef uint32_t uintx4 __attribute__((ext_vector_type(4)));

constexpr int kCWs = (int)kRangeComputeWaves;  // contracting waves
constexpr int kLWs = 4;                        // loading waves: wave kCWs + s loads vectors 4s .. 4s + 3
constexpr int kThreadsSR = (kCWs + kLWs) * 64;
constexpr int kRing = 4;                       // register sets of the list ring
constexpr int kU = 8;                          // MFMA steps per list block
constexpr int kTurnSteps = kRing * kU;         // steps of one turn of the list ring
constexpr int kOW = kU / 2;                    // words of 16-bit offsets per sample slot and block
constexpr int kCs = (int)kWindowCoords;        // coordinates per range
constexpr int kSlotsSR = (int)kWindowSlots;    // ranges in the LDS ring
constexpr int kLookSR = (int)kWindowLook;      // a stage reads its own range and this many after it
constexpr int kRowFloats = kSlotsSR * kCs + 4; // row stride: the 4 floats of padding spread the vectors over the banks
constexpr int kRingBytesSR = 16 * kRowFloats * 4;
// after the ring: the offsets b~ of the workgroup's functions (maximum inner product: the row operand of the
// extra step, a0 and b~), [wave][block][32], then the turns of every stage
constexpr int kLdsLimitSR = 160 * 1024;
constexpr int kAhead = 4;                      // register sets of a loading wave: a range is requested three stages before it is written
static_assert(kRowFloats * 4 + 16 <= 65536, "list offsets are 16 bits");
static_assert(kSlotsSR == kLookSR + 2 && kSlotsSR % kAhead == 0, "ring geometry");

// Returns v through an empty asm: values derived from it are recomputed where they are used
// instead of being kept in registers across the contraction loops.
__device__ __forceinline__ uint32_t fresh(uint32_t v) {
    asm volatile("" : "+v"(v));
    return v;
}

struct SharedRangedArgs {
    const float *data;  // [N][n]
    uint64_t N;
    uint32_t n, k, g, blocks_per_table, nblocks;
    uint32_t nchunks, stages;  // ranges that hold data; stages per tile (a multiple of the ring slots)
    const float *off;   // [>= k]
    float w, inv_w;
    int w_is_pow2, proj;
    void *out;
    const float *extra;     // [nblocks][64] row operand (a0, b~, 0, 0) of the extra step (maximum inner product)
    const float *kappa2;    // [tables] kappa~_l^2, input of the data hash
    int raw;                // maximum-inner-product modes: projections instead of ids
    uint64_t *keys;         // key mode: [N][tables]; out is then the ids' array or null
    const float *coefs;     // list blocks: 8 steps x 64 lanes
    const uint32_t *offs;   // per list block: 4 sample slots x 4 words of two 16-bit byte offsets into a row of the ring
};

// BPW: blocks of 16 functions per contracting wave (a turn of the list ring gives each of them 32 / BPW steps);
// MODE: 0 ids or projections, 3 kappa~^2, 4 maximum-inner-product data hash, 5 query hash,
// 6 one 64-bit key per table (tables of at most 16 functions: one block each), and the ids too if asked for
template <int BPW, int MODE>
__global__ __launch_bounds__(kThreadsSR) void shared_ranged_kernel(const SharedRangedArgs a,
                                                                   const uint32_t *__restrict__ stage_turns,
                                                                   const uint2 *__restrict__ streams) {
    static_assert(kTurnSteps % BPW == 0, "a turn deals the same number of steps to every block");
    constexpr int Q = kTurnSteps / BPW;  // consecutive steps of one block within a turn
    constexpr bool KAPPA = MODE == 3, MDATA = MODE == 4, MQUERY = MODE == 5, NORMS = MODE >= 3 && MODE <= 5;
    constexpr bool KEYS = MODE == 6;
    extern __shared__ __align__(16) char lds_sr[];  // [16 vectors][8 ranges x 256 + 4 floats], offsets, turns
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint32_t lane = threadIdx.x & 63;
    const uint32_t n = a.n, S = a.stages;
    float *lds_off = reinterpret_cast<float *>(lds_sr + kRingBytesSR) + wave * (BPW * 32);  // this wave's [BPW][32]
    uint32_t *lds_turns = reinterpret_cast<uint32_t *>(lds_sr + kRingBytesSR + kCWs * BPW * 128);
    const uint64_t ntiles = (a.N + 15) / 16;
    const uint64_t first_tile = blockIdx.x;  // the host launches at most ntiles workgroups along x
    const uint64_t my_tiles = (ntiles - first_tile + gridDim.x - 1) / gridDim.x;
    // Barriers, counted from the first: barrier b ends stage b - 1 (barrier 0 opens stage 0).  The
    // loading waves write item x (range x % S of the workgroup's tile x / S) after barrier x - 7,
    // when the range that lived in its slot has had its last stage, and before barrier x - 6,
    // which opens the first stage that may read it.

    if (wave >= (uint32_t)kCWs) {
        // ---- loading waves: four vectors each, one 1 KB instruction per vector and range; a
        // range is requested three stages before it is written to LDS
        // the loading waves' few instructions go first: a range requested late is bandwidth lost
        __builtin_amdgcn_s_setprio(3);
        const uint32_t v0 = (wave - kCWs) * 4;
        const uint64_t total = my_tiles * S;  // a multiple of 8
        uint64_t f_tile = first_tile, s_tile = first_tile;
        uint32_t f_r = 0, s_r = 0;
        auto fetch = [&](floatx4 (&pre)[4]) __attribute__((always_inline)) {
            // items past the data (ranges beyond n, tiles beyond the last) load the first tile's
            // first range: the number of requests in flight is the same on every path
            const bool real = f_tile < ntiles && f_r < a.nchunks;
            const uint64_t tile = real ? f_tile : first_tile;
            const uint32_t c = (real ? f_r : 0u) * kCs + lane * 4;
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                uint64_t row = tile * 16 + v0 + v;
                row = row < a.N ? row : a.N - 1;  // rows beyond the data repeat the last vector (never stored)
                // coordinates beyond n read the row's first ones; zeros are stored for them
                pre[v] = *reinterpret_cast<const floatx4 *>(a.data + row * n + (c < n ? c : 0u));
            }
            if (++f_r == S) {
                f_r = 0;
                f_tile += gridDim.x;
            }
        };
        auto stash = [&](const floatx4 (&pre)[4]) __attribute__((always_inline)) {
            if (s_tile < ntiles && s_r < a.nchunks) {
                const bool inside = s_r * kCs + lane * 4 < n;
                char *dst = lds_sr + ((s_r % kSlotsSR) * kCs + lane * 4) * 4;
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const floatx4 x = pre[v];
                    const floatx4 z = {inside ? x[0] : 0.f, inside ? x[1] : 0.f, inside ? x[2] : 0.f, inside ? x[3] : 0.f};
                    *reinterpret_cast<floatx4 *>(dst + (v0 + v) * kRowFloats * 4) = z;
                }
            }
            if (++s_r == S) {
                s_r = 0;
                s_tile += gridDim.x;
            }
        };
        floatx4 pre[kAhead][4];
#pragma unroll
        for (int d = 0; d < kAhead - 1; ++d) fetch(pre[d]);
        for (uint64_t x = 0; x < total; x += kAhead) {
#pragma unroll
            for (int d = 0; d < kAhead; ++d) {
                if (x + d > (uint64_t)kLookSR) lds_barrier();  // barrier x + d - 7
                fetch(pre[(d + kAhead - 1) % kAhead]);
                stash(pre[d]);
            }
        }
        // barriers total - 7 .. total of the contracting waves
#pragma unroll
        for (int i = 0; i < kLookSR + 2; ++i) lds_barrier();
        return;
    }

    // ---- contracting waves
    const uint32_t stream_id = blockIdx.y * kCWs + wave;
    const uint2 si = streams[stream_id];  // {first list block, list blocks per tile}
    // uniform block pointers plus a per-lane index: the loads take a scalar base and a 32-bit lane offset
    const float *cbase = a.coefs + (size_t)si.x * (kU * 64);
    const uint32_t *obase = a.offs + (size_t)si.x * (4 * kOW);
    const uint32_t oslot = (lane >> 4) * kOW;
    const uint32_t sblocks = si.y;  // a multiple of the ring, at least one turn
    // Block i of the stream lives in ring set i % 4; when block i is about to be used, block
    // i + 3 is requested into the set used just before.
    float ring_c[kRing][kU];
    uint32_t ring_o[kRing][kOW];
    uint32_t next_block = 0;
    auto load_block = [&](int set) __attribute__((always_inline)) {
        const float *cs = cbase + (size_t)next_block * (kU * 64);
        const uint32_t *os = obase + (size_t)next_block * (4 * kOW);
        // coefficients of four steps per load: [steps / 4][lane][4]
#pragma unroll
        for (int i = 0; i < kU / 4; ++i) {
            const floatx4 c4 = *reinterpret_cast<const floatx4 *>(cs + i * 256 + lane * 4);
#pragma unroll
            for (int e = 0; e < 4; ++e) ring_c[set][4 * i + e] = c4[e];
        }
#pragma unroll
        for (int i = 0; i < kOW; ++i) ring_o[set][i] = os[oslot + i];
        next_block = next_block + 1 == sblocks ? 0 : next_block + 1;
        __builtin_amdgcn_sched_barrier(0);  // the request stays here, three blocks ahead of its use
    };
#pragma unroll
    for (int i = 0; i < kRing - 1; ++i) load_block(i);
    const char *row = lds_sr + (lane & 15) * kRowFloats * 4;  // this lane's vector in the ring
    // the four floats after a row's coordinates stay zero: what padding steps read
    if (wave == 0 && lane < 16) *reinterpret_cast<floatx4 *>(lds_sr + (lane * kRowFloats + kSlotsSR * kCs) * 4) = floatx4{0.f, 0.f, 0.f, 0.f};
    // The offsets b~ of the wave's functions and the table of turns are read from LDS where they
    // are needed: a vector memory load there would make the wave wait for everything it has in
    // flight, the id stores of the block before included.
    if (wave == 1)
        for (uint32_t i = lane; i < S; i += 64) lds_turns[i] = stage_turns[i];
    {
        // lanes 0 .. 15: the offsets of the 16 functions of every block; maximum inner product: lanes
        // 0 .. 31, the first two sample slots of the extra step's row operand (a0_j, then b~_j)
        float own[BPW];
#pragma unroll
        for (int f = 0; f < BPW; ++f) {
            const uint32_t blk = (blockIdx.y * BPW + f) * kCWs + wave;
            if constexpr (NORMS) {
                const bool live = blk < a.nblocks && lane < 32;
                own[f] = a.extra[live ? (size_t)blk * 64 + lane : 0];
                own[f] = live ? own[f] : 0.f;
            } else {
                const uint32_t in_table = (blk % a.blocks_per_table) * 16 + (lane & 15);
                const bool live = blk < a.nblocks && in_table < a.g;
                own[f] = a.off[live ? (blk / a.blocks_per_table) * a.g + in_table : 0u];
                own[f] = live ? own[f] : 0.f;
            }
        }
        if (lane < (NORMS ? 32 : 16)) {
#pragma unroll
            for (int f = 0; f < BPW; ++f) lds_off[f * 32 + lane] = own[f];
        }
    }
    // key mode (Sec. 3.2): a lane folds its four ids, weighs the fold by the power of the multiplier that
    // belongs to the last of them, C^(g - 1 - t), and the four lanes of a vector add up
    [[maybe_unused]] uint64_t key_pow = 1;
    if constexpr (KEYS) {
        const uint32_t t_last = 4 * (lane >> 4) + 3;
        for (uint32_t e = 0; e + 1 + t_last < a.g; ++e) key_pow *= kKeyMultiplier;
        if (t_last >= a.g) key_pow = 0;  // rows beyond the table
    }
    [[maybe_unused]] float kmax[KAPPA ? BPW : 1];  // kappa~^2 pass: largest ||S(v)||^2 seen per block
#pragma unroll
    for (int f = 0; f < (KAPPA ? BPW : 1); ++f) kmax[f] = 0.f;

    lds_barrier();  // barrier 0: the ranges 0 .. 6 of the first tile are written
    uint32_t turns_next = lds_turns[0];
    for (uint64_t t = first_tile; t < ntiles; t += gridDim.x) {
        floatx4 acc[BPW];
        [[maybe_unused]] float nrm[NORMS ? BPW : 1];  // this lane's share of ||S(v)||^2 per block
#pragma unroll
        for (int f = 0; f < BPW; ++f) acc[f] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int f = 0; f < (NORMS ? BPW : 1); ++f) nrm[f] = 0.f;
        for (uint32_t s = 0; s < S; ++s) {
            uint32_t turns = __builtin_amdgcn_readfirstlane(turns_next);
            turns_next = lds_turns[s + 1 == S ? 0 : s + 1];  // arrives behind the stage's own LDS reads
            for (; turns; --turns) {
#pragma unroll
                for (int q = 0; q < kRing; ++q) {
                    load_block((q + kRing - 1) % kRing);
                    // one block: all reads, then the MFMAs; step 8 q + e of the turn belongs to block (8 q + e) / Q
                    float x[kU];
                    // the offsets are taken apart here, not where they were requested (which would wait for them there)
#pragma unroll
                    for (int i = 0; i < kOW; ++i) asm volatile("" : "+v"(ring_o[q][i]));
#pragma unroll
                    for (int e = 0; e < kU; ++e) {
                        const uint32_t off = (ring_o[q][e >> 1] >> (16 * (e & 1))) & 0xFFFFu;
                        x[e] = *reinterpret_cast<const float *>(row + off);
                    }
                    __builtin_amdgcn_sched_barrier(0);  // all reads of the block go out before its first MFMA
#pragma unroll
                    for (int e = 0; e < kU; ++e) {
                        const int f = (kU * q + e) / Q;
                        if constexpr (!KAPPA) acc[f] = __builtin_amdgcn_mfma_f32_16x16x4f32(ring_c[q][e], x[e], acc[f], 0, 0, 0);
                        if constexpr (NORMS) nrm[f] = fmaf(x[e], x[e], nrm[f]);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            if (s + 1 == S) {
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
                            const float rowx = lds_off[f * 32 + (ln & 31)];  // the last two sample slots multiply zeros
                            acc[f] = __builtin_amdgcn_mfma_f32_16x16x4f32(rowx, colx, acc[f], 0, 0, 0);
                        }
                    }
                    if constexpr (KEYS) {
                        // every lane takes part in the exchange; blocks and rows beyond the data fold zeros or
                        // values nobody stores
                        const floatx4 bq = *reinterpret_cast<const floatx4 *>(lds_off + f * 32 + 4 * (ln >> 4));
                        uintx4 v;
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const float h = a.w_is_pow2 ? fmaf(acc[f][e], a.inv_w, bq[e] * a.inv_w) : (acc[f][e] + bq[e]) / a.w;
                            v[e] = (uint32_t)(int)floorf(h);
                        }
                        uint64_t part = v[0];
#pragma unroll
                        for (int e = 1; e < 4; ++e) part = part * kKeyMultiplier + v[e];
                        part *= key_pow;
                        part += __shfl_xor(part, 16);
                        part += __shfl_xor(part, 32);
                        if (blk < a.nblocks && vec < a.N) {  // one block per table: the block number is the table
                            if (ln < 16) a.keys[vec * a.nblocks + blk] = part;
                            if (a.out && in_table < a.g)
                                *reinterpret_cast<uintx4 *>(reinterpret_cast<uint32_t *>(a.out) + vec * a.k + j) = v;
                        }
                        continue;
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
                            const floatx4 bq = *reinterpret_cast<const floatx4 *>(lds_off + f * 32 + 4 * (ln >> 4));
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
            lds_barrier();  // ends stage s: the next range is written, everyone is done with the oldest one
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
    pl.nchunks = (n + kWindowCoords - 1) / kWindowCoords;
    pl.stages = (pl.nchunks + kWindowSlots - 1) / kWindowSlots * kWindowSlots;
    if (kRingBytesSR + kCWs * pl.bpw * 128 + (size_t)pl.stages * 4 > (size_t)kLdsLimitSR) return pl;  // the table of turns no longer fits LDS
    pl.supported = true;
    return pl;
}

// Host tables.  First the schedule: every table's samples are dealt to the stages of a tile, a
// sample of range r to one of the stages r - 6 .. r (what the ring holds), every table getting
// the same number of MFMA steps in a stage, a multiple of the 32 / bpw steps a turn of the list
// ring gives a block.  Stage after stage the length is the smallest that takes the samples whose
// last stage this is, for the table that has most of them; a table fills the rest of its steps
// with the samples that are due soonest, so later stages find less left to do.  Then the lists:
// per contracting wave one stream of list blocks in consumption order (stage after stage, turn
// after turn, within a turn the wave's blocks one after the other); per step and lane the
// coefficient of (row l % 16, sample l / 16) and the byte offset of that sample's coordinate in a
// row of the ring.  stage_turns holds the turns of the list ring per stage.
void build_shared_ranged_tables(const lsh_params *p, SharedRangedPlan &pl, std::vector<float> &coefs,
                                std::vector<uint32_t> &offs, std::vector<uint32_t> &stage_turns,
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
    const uint32_t S = pl.stages, CW = kRangeComputeWaves, bpw = pl.bpw, m = p->m;
    const uint32_t Q = kTurnSteps / bpw;  // steps of a block per turn
    const uint32_t tables = pl.nblocks / pl.blocks_per_table, streams = pl.kblocks * CW;
    constexpr uint32_t kPad = 0xFFFFFFFFu;
    // samples of every table by range, then stage after stage
    std::vector<std::vector<uint32_t>> by_range((size_t)tables * S);
    for (uint32_t table = 0; table < tables; ++table) {
        const uint32_t *smp_coord = &p->idx[(size_t)table * pl.g * m];
        for (uint32_t smp = m; smp-- > 0;) by_range[(size_t)table * S + smp_coord[smp] / kWindowCoords].push_back(smp);
    }
    // slots[table * S + s]: the stage's samples dealt to steps of four, 0xFFFFFFFF marks a padding slot
    std::vector<std::vector<uint32_t>> slots((size_t)tables * S);
    stage_turns.assign(S, 0);
    for (uint32_t s = 0; s < S; ++s) {
        size_t due = 0;
        for (uint32_t table = 0; table < tables; ++table) due = std::max(due, by_range[(size_t)table * S + s].size());
        const uint32_t turns = (uint32_t)((due + 4 * Q - 1) / (4 * Q));
        stage_turns[s] = turns;
        const uint32_t steps = turns * Q;
        for (uint32_t table = 0; table < tables; ++table) {
            const uint32_t *smp_coord = &p->idx[(size_t)table * pl.g * m];
            // the stage's samples: those due now, then the soonest due, by coordinate class modulo 4
            std::vector<uint32_t> cls[4];
            uint32_t room = 4 * steps;
            for (uint32_t r = s; r < S && r <= s + kWindowLook && room; ++r) {
                std::vector<uint32_t> &have = by_range[(size_t)table * S + r];
                while (!have.empty() && room) {
                    cls[smp_coord[have.back()] & 3].push_back(have.back());
                    have.pop_back();
                    --room;
                }
            }
            // steps of four samples whose coordinates differ modulo 4 where the classes allow it
            std::vector<uint32_t> &out = slots[(size_t)table * S + s];
            size_t left = cls[0].size() + cls[1].size() + cls[2].size() + cls[3].size();
            while (left) {
                bool taken[4] = {false, false, false, false};
                for (uint32_t kq = 0; kq < 4; ++kq) {
                    int best = -1;
                    for (int pass = 0; pass < 2 && best < 0; ++pass)
                        for (int q = 0; q < 4; ++q)
                            if (!cls[q].empty() && (pass == 1 || !taken[q]) && (best < 0 || cls[q].size() > cls[best].size()))
                                best = q;
                    if (best < 0) {
                        out.push_back(kPad);
                    } else {
                        out.push_back(cls[best].back());
                        cls[best].pop_back();
                        taken[best] = true;
                        --left;
                    }
                }
            }
            out.resize((size_t)4 * steps, kPad);
        }
    }
    uint32_t per_stream = 0;  // list blocks of a stream per tile
    std::vector<uint32_t> stage_first(S);
    for (uint32_t s = 0; s < S; ++s) {
        stage_first[s] = per_stream;
        per_stream += stage_turns[s] * kRing;
    }
    stream_info.assign((size_t)streams * 2, 0);
    coefs.assign((size_t)streams * per_stream * kU * 64, 0.f);
    // steps and slots that only pad (coefficient zero) read one of the four zero floats that follow a
    // row's coordinates: four different banks per vector, like a step of real samples, and
    // nothing for the squared norms of the maximum-inner-product modes
    offs.assign((size_t)streams * per_stream * 4 * kOW, 0u);
    for (size_t rec = 0; rec < offs.size() / kOW; ++rec)
        for (uint32_t e = 0; e < (uint32_t)kU; ++e)
            offs[rec * kOW + e / 2] |= ((kWindowSlots * kWindowCoords + (uint32_t)(rec & 3)) * 4u) << (16 * (e & 1));
    for (uint32_t y = 0; y < pl.kblocks; ++y)
        for (uint32_t cw = 0; cw < CW; ++cw) {
            const uint32_t stream = y * CW + cw;
            stream_info[(size_t)stream * 2] = stream * per_stream;
            stream_info[(size_t)stream * 2 + 1] = per_stream;
            for (uint32_t s = 0; s < S; ++s)
                for (uint32_t turn = 0; turn < stage_turns[s]; ++turn)
                    for (uint32_t i = 0; i < (uint32_t)kTurnSteps; ++i) {
                        const uint32_t f = i / Q, blk = (y * bpw + f) * CW + cw;
                        if (blk >= pl.nblocks) continue;  // a list of zeros
                        const uint32_t table = blk / pl.blocks_per_table, first = (blk % pl.blocks_per_table) * 16;
                        const uint32_t step = turn * Q + i % Q;  // of this block's table in the stage
                        const size_t block = (size_t)stream * per_stream + stage_first[s] + turn * kRing + i / kU;
                        const uint32_t in_block = i % kU;
                        for (uint32_t kq = 0; kq < 4; ++kq) {
                            const uint32_t smp = slots[(size_t)table * S + s][(size_t)step * 4 + kq];
                            if (smp == kPad) continue;
                            const uint32_t in_row = p->idx[(size_t)table * pl.g * m + smp] % (kWindowSlots * kWindowCoords);
                            uint32_t &word = offs[(block * 4 + kq) * kOW + in_block / 2];
                            word = (word & ~(0xFFFFu << (16 * (in_block & 1)))) | (in_row * 4) << (16 * (in_block & 1));
                            // a lane's four consecutive steps side by side: [steps / 4][lane][4]
                            for (uint32_t r16 = 0; r16 < 16 && first + r16 < pl.g; ++r16)  // rows beyond the table keep zero
                                coefs[(block * kU + in_block / 4 * 4) * 64 + (kq * 16 + r16) * 4 + in_block % 4] =
                                    p->coef[(size_t)(table * pl.g + first + r16) * m + smp];
                        }
                    }
        }
}

// Keys come out of the kernel when the key groups are the tables and a table is one block.
bool shared_ranged_keys_ok(const lsh_params *p, uint32_t L) {
    const SharedRangedPlan &pl = p->shared_ranged_plan;
    return pl.supported && p->d_sr_lists && L == p->shared_tables && pl.blocks_per_table == 1;
}

// mode: 0 bucket ids, 1 raw projections, 3 kappa~^2 per table (atomic maximum into d_out), 4 and 5
// the maximum-inner-product data and query hashes (raw != 0: their projections), 6 the tables'
// keys into d_keys (tables of at most 16 functions) and, if d_out is not null, the ids as well
int launch_shared_ranged(const lsh_params *p, int mode, const float *d_data, uint64_t N, void *d_out, void *stream,
                         const float *d_kappa2, int raw, uint64_t *d_keys) {
    const SharedRangedPlan &pl = p->shared_ranged_plan;
    if (!pl.supported || !p->d_sr_lists || !p->d_sr_offs) return LSH_ERR_UNSUPPORTED;
    if (!N) return LSH_OK;
    SharedRangedArgs a;
    a.data = d_data;
    a.N = N;
    a.n = p->n;
    a.k = p->k;
    a.g = pl.g;
    a.blocks_per_table = pl.blocks_per_table;
    a.nblocks = pl.nblocks;
    a.nchunks = pl.nchunks;
    a.stages = pl.stages;
    a.off = p->d_off;
    a.w = p->w;
    a.inv_w = 1.0f / p->w;
    int exp2 = 0;
    a.w_is_pow2 = (std::frexp(p->w, &exp2) == 0.5f) ? 1 : 0;
    a.proj = mode == 1;
    a.extra = static_cast<const float *>(p->d_sr_extra);
    a.kappa2 = d_kappa2;
    a.raw = raw;
    a.keys = d_keys;
    if (mode >= 3 && mode <= 5 && !p->d_sr_extra) return LSH_ERR_UNSUPPORTED;
    if (mode == 6 && (pl.blocks_per_table != 1 || !d_keys)) return LSH_ERR_UNSUPPORTED;
    a.out = d_out;
    a.coefs = static_cast<const float *>(p->d_sr_lists);
    a.offs = static_cast<const uint32_t *>(p->d_sr_offs);
    const uint32_t *turns = static_cast<const uint32_t *>(p->d_sr_list_len);
    const uint2 *streams = static_cast<const uint2 *>(p->d_sr_stream);
    const uint64_t ntiles = (N + 15) / 16;
    // one workgroup per CU (the ring takes 128 KB of LDS); the kblocks workgroups of a tile run on one XCD
    uint64_t gx = (uint64_t)p->num_cus / pl.kblocks;
    gx = gx < 8 ? 8 : gx / 8 * 8;
    if (gx > ntiles) gx = ntiles;
    const dim3 grid((uint32_t)gx, pl.kblocks);
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    const uint32_t lds_bytes = kRingBytesSR + kCWs * pl.bpw * 128 + pl.stages * 4;
#define LSH_SR_LAUNCH(B_, M_) \
    { \
        auto fn = &shared_ranged_kernel<B_, M_>; \
        if (ensure_lds_limit(reinterpret_cast<const void *>(fn), lds_bytes) != LSH_OK) return LSH_ERR_HIP; \
        hipLaunchKernelGGL(fn, grid, dim3(kThreadsSR), lds_bytes, s, a, turns, streams); \
    }
#define LSH_SR_CASE(B_) \
    case B_: \
        if (mode <= 1) LSH_SR_LAUNCH(B_, 0) \
        else if (mode == 3) LSH_SR_LAUNCH(B_, 3) \
        else if (mode == 4) LSH_SR_LAUNCH(B_, 4) \
        else if (mode == 5) LSH_SR_LAUNCH(B_, 5) \
        else if (mode == 6) LSH_SR_LAUNCH(B_, 6) \
        else return LSH_ERR_INVALID_ARG; \
        break;
    switch (pl.bpw) {
        LSH_SR_CASE(4) LSH_SR_CASE(8) LSH_SR_CASE(16)
        default: return LSH_ERR_UNSUPPORTED;
    }
#undef LSH_SR_CASE
#undef LSH_SR_LAUNCH
    return hipGetLastError() == hipSuccess ? LSH_OK : LSH_ERR_HIP;
}

}  // namespace lsh
