// Projections a_j . v for n = 128 as a dense product on the bf16 matrix cores, with fp32 accuracy,
// and the epilogues on them: bucket ids (Eq. 1, Eq. 5), raw projections, compound keys (Sec. 3.2)
// and sign hashes (Sec. 5).  The coefficient matrix is an E2LSH object's (Sec. 2.2) or a FastLSH
// object's written out over all coordinates (Sec. 3.1: zeros at the coordinates a function does
// not sample): at n = 128 the matrix cores do the whole row in less time than the vector ALU
// gathers and multiplies a quarter of it.
//
// The fp32 MFMA of this part runs at a sixteenth of the bf16 rate, so the product is computed
// from three-way bf16 splits instead: an fp32 value x is EXACTLY x1 + x2 + x3 with
// x1 = bf16(x), x2 = bf16(x - x1), x3 = bf16(x - x1 - x2) under round-to-nearest (each step
// leaves at most the bits below the previous term's last place: 8 + 8 + 8 significant bits),
// and a . v = sum over splits of a_p v_q.  The six products with p + q <= 4 are formed (exact in
// the fp32 accumulator's inputs: an 8 x 8 bit product); the three left out are below
// 2^-23 |a v| together, the size of one fp32 rounding.  Six bf16 MFMAs do the work of one fp32
// product at 16 / 6 of its speed.
//
// Sign hashes (Sec. 5, angular similarity) need the sign of the projection only, and are
// compared away from zero: with two-way splits and the three products a1 v1 + a1 v2 + a2 v1 the
// terms left out are below 3 * 2^-16 |a v| per coordinate, under half of the 1e-4 |a| |S(v)|
// inside which a sign may differ from the exact one.
//
//   V [N][128] row-major (vectors), A [kpad][128] row-major (row j = a_j, fp32).
//
// Terms that are zero are skipped by tile.  Data whose values fit a bf16 (8 significant bits:
// byte-valued descriptors, small integers) have v2 = v3 = 0, and values of at most 16
// significant bits have v3 = 0; the waves that split a tile note the highest non-zero term
// they saw ("level" 1, 2 or 3), and the tile then takes 3, 5 or all 6 products (signs: 2 or 3).
// A product with an all-zero operand adds exactly nothing, so the results are the same bits.
//
// Workgroup = 512 threads (8 waves), persistent, one per CU.  A wave owns 32 functions and keeps
// their coefficients, already split, in 96 registers for the whole launch (the row operand of
// v_mfma_f32_32x32x16_bf16: lane l holds row l % 32, contraction indices 16 s + 8 (l / 32) ...
// + 7 of step s).  A workgroup therefore covers 256 functions; a tile is 64 vectors, split on
// the way into LDS (three planes of bf16, rows padded to 272 bytes so that the 16-byte operand
// reads of 16 consecutive rows cover all banks once) and shared by the 8 waves.  The column
// operand uses the same contraction indices per lane, so any lane layout of them that is the
// same for both operands gives the same sums.  As in the fp32 kernels a lane ends up with runs
// of four consecutive functions of one vector (accumulator register i = function
// 8 (i / 4) + 4 (l / 32) + i % 4, vector l % 32); ids and projections then change lanes through
// LDS so that 8 lanes store a whole 128-byte line, keys are folded from the runs where they
// are, sign bits are gathered into half a word per vector and wave.
#include <hip/hip_runtime.h>

#include <cmath>
#include <type_traits>

#include "lsh_internal.h"

namespace lsh {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef uint32_t uintx4 __attribute__((ext_vector_type(4)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr int SN = 128;            // contraction length
constexpr int KSTEPS = SN / 16;    // MFMA steps
constexpr int TV = 64;             // vectors per tile (two column blocks of 32)
constexpr int ROWB = SN * 2 + 16;  // bytes per vector and plane in LDS
constexpr int PLANE = TV * ROWB;
constexpr int BUF = 3 * PLANE;     // one tile: 52224 bytes
constexpr int kThreadsS = 512;
constexpr int kFuncsPerWave = 32, kFuncsPerBlock = 8 * kFuncsPerWave;
constexpr int kQuads = TV * (SN / 4) / kThreadsS;  // 16-byte pieces of a tile per thread: 4
// per wave: 32 vectors x 32 results of a column block, rows padded to 144 bytes (conflict-free
// 16-byte writes by vector), through which the results change lanes before they are stored
constexpr int STAGE_ROWB = 32 * 4 + 16;
constexpr int STAGE = 32 * STAGE_ROWB;
constexpr int kLevelOffset = 2 * BUF, kStageOffset = 2 * BUF + 16;
constexpr int kOffsetsOffset = kStageOffset + 8 * STAGE;  // the waves' 32 offsets b~ each
constexpr int kLdsBytes = kOffsetsOffset + 8 * 128;       // 142 352

struct SplitArgs {
    const float *data;  // [N][128]
    const float *a;     // [>= k rows][128]
    const float *off;   // [>= k]; not read for signs
    uint64_t N;
    uint32_t k;         // multiple of 32 (signs: of 64)
    uint32_t g;         // keys: functions per table, 4, 8, 16 or 32
    float w, inv_w;
    void *out;          // [N][k]; signs [N][k / 64]; keys [N][k / g]
    void *out2;         // ids and keys in one launch: the keys [N][k / g] (the ids go to out)
};

__device__ __forceinline__ void split3(float x, __bf16 &x1, __bf16 &x2, __bf16 &x3) {
    x1 = (__bf16)x;
    const float r1 = x - (float)x1;
    x2 = (__bf16)r1;
    x3 = (__bf16)(r1 - (float)x2);
}

enum : int { kIds = 0, kProj = 1, kSigns = 2, kKeys = 3, kIdsKeys = 4 };

// EP: bucket ids, raw projections (both [N][k], 4 bytes each), sign words ([N][k / 64] of 64
// bits), the compound keys of Sec. 3.2 folded from the ids ([N][k / g] of 64 bits), or ids and
// keys together (the ids are in registers when the keys are folded: one pass over the data
// instead of a hashing launch and a packing launch that reads the ids back)
template <int EP, bool POW2>
__global__ __launch_bounds__(kThreadsS, 2) void dense_split_kernel(const SplitArgs a) {
    constexpr bool PROJ = EP == kProj, SIGNS = EP == kSigns, KEYS = EP == kKeys, BOTH = EP == kIdsKeys;
    constexpr int NSPLIT = SIGNS ? 2 : 3;
    // blocks of 32 functions per wave.  Signs: two (their two-way splits leave the registers), so
    // that a workgroup covers 512 functions and a tile is split once where two workgroups of 256
    // would each split it; a wave then owns whole 64-bit sign words.
    constexpr int FB = SIGNS ? 2 : 1;
    constexpr uint32_t kWaveFuncs = kFuncsPerWave * FB, kBlockFuncs = kFuncsPerBlock * FB;
    extern __shared__ __align__(16) char lds_s[];  // 2 x [3 planes][64 vectors][272 bytes], then 2 level words
    // level word of a buffer: 4 * (number of the tile in this workgroup's sequence + 1) + level,
    // raised by atomic maximum, so that it never has to be cleared between tiles
    uint32_t *const level_word = reinterpret_cast<uint32_t *>(lds_s + kLevelOffset);

    const uint32_t slices = (a.k + kBlockFuncs - 1) / kBlockFuncs;
    const uint64_t ntiles = (a.N + TV - 1) / TV;
    // workgroups i, i + 8, ... share an XCD (and its L2): the slices of one row tile run there
    // side by side
    const uint32_t slot = blockIdx.x / 8, slots = gridDim.x / 8;
    const uint32_t slice = slot % slices;
    const uint64_t stream = (uint64_t)(slot / slices) * 8 + blockIdx.x % 8, streams = (uint64_t)(slots / slices) * 8;
    if (slot / slices >= slots / slices) return;

    const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint32_t lr = lane & 31, lh = lane >> 5;
    const uint32_t wf = slice * kBlockFuncs + wave * kWaveFuncs;  // first function of the wave
    const bool active = wf < a.k;                                     // whole wave

    // coefficients of the wave's blocks of 32 functions, split, resident: c[block][step][term]
    bf16x8 c[FB][KSTEPS][NSPLIT];
    if (active) {
#pragma unroll
        for (int fb = 0; fb < FB; ++fb) {
            const float *row = a.a + (size_t)(wf + 32 * fb + lr) * SN + 8 * lh;
#pragma unroll
            for (int s = 0; s < KSTEPS; ++s) {
                const float4 u0 = *reinterpret_cast<const float4 *>(row + 16 * s);
                const float4 u1 = *reinterpret_cast<const float4 *>(row + 16 * s + 4);
                const float u[8] = {u0.x, u0.y, u0.z, u0.w, u1.x, u1.y, u1.z, u1.w};
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    __bf16 x1, x2, x3;
                    split3(u[e], x1, x2, x3);
                    c[fb][s][0][e] = x1;
                    c[fb][s][1][e] = x2;
                    if constexpr (NSPLIT == 3) c[fb][s][2][e] = x3;
                }
            }
        }
    } else {
#pragma unroll
        for (int fb = 0; fb < FB; ++fb)
#pragma unroll
            for (int s = 0; s < KSTEPS; ++s)
#pragma unroll
                for (int p = 0; p < NSPLIT; ++p)
#pragma unroll
                    for (int e = 0; e < 8; ++e) c[fb][s][p][e] = (__bf16)0.f;
    }

    // loader: thread t takes the 16-byte pieces t, t + 512, ... of the tile (32 pieces per vector);
    // rows beyond the last vector read the last vector (computed, never stored), so a fetch is in
    // bounds for any tile number
    const uint32_t ld_vec = threadIdx.x >> 5, ld_piece = threadIdx.x & 31;
    float4 raw[kQuads];
    auto fetch = [&](uint64_t tile) {
#pragma unroll
        for (int q = 0; q < kQuads; ++q) {
            uint64_t vec = tile * TV + ld_vec + 16 * q;
            vec = vec < a.N ? vec : a.N - 1;
            // streamed once (the workgroup that shares the tile finds it in L2 all the same)
            const floatx4 v = __builtin_nontemporal_load(reinterpret_cast<const floatx4 *>(a.data + vec * SN + ld_piece * 4));
            raw[q] = make_float4(v[0], v[1], v[2], v[3]);
        }
    };
    uint32_t seen2 = 0, seen3 = 0;  // bits of the second and third terms this lane has produced for the tile
    auto stash_quad = [&](char *buf, int q) {
        {
            const float u[4] = {raw[q].x, raw[q].y, raw[q].z, raw[q].w};
            bf16x4 h[3];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                __bf16 x1, x2, x3;
                split3(u[e], x1, x2, x3);
                h[0][e] = x1;
                h[1][e] = x2;
                h[2][e] = x3;
            }
            char *dst = buf + (ld_vec + 16 * q) * ROWB + ld_piece * 8;
#pragma unroll
            for (int p = 0; p < NSPLIT; ++p) *reinterpret_cast<bf16x4 *>(dst + p * PLANE) = h[p];
            const uint2 t2 = *reinterpret_cast<const uint2 *>(&h[1]);
            seen2 |= (t2.x | t2.y) & 0x7fff7fffu;
            if constexpr (NSPLIT == 3) {
                const uint2 t3 = *reinterpret_cast<const uint2 *>(&h[2]);
                seen3 |= (t3.x | t3.y) & 0x7fff7fffu;
            }
        }
    };
    // after the last piece of a tile: one lane per wave raises the buffer's level word
    auto publish_level = [&](uint32_t buf_index, uint32_t seq) {
        const bool any3 = __any(seen3 != 0), any2 = __any(seen2 != 0);  // a non-zero third term implies a non-zero second
        if ((any2 || any3) && lane == 0) atomicMax(&level_word[buf_index], 4 * (seq + 1) + (any3 ? 3u : 2u));
        seen2 = 0;
        seen3 = 0;
    };
    auto stash = [&](char *buf) {
#pragma unroll
        for (int q = 0; q < kQuads; ++q) stash_quad(buf, q);
    };

    if (threadIdx.x < 2) level_word[threadIdx.x] = 0;
    __syncthreads();
    uint64_t t = stream;
    uint32_t seq = 0;  // number of the tile in this workgroup's sequence
    fetch(t);
    stash(lds_s);
    publish_level(0, 0);
    __syncthreads();
    fetch(t + streams);
    uint32_t cur = 0;

    if (!active) {
        // waves beyond the last function only help to load: same barriers as the others
        for (; t < ntiles; t += streams) {
            stash(lds_s + (cur ^ 1) * BUF);
            publish_level(cur ^ 1, seq + 1);
            fetch(t + 2 * streams);
            __syncthreads();
            cur ^= 1;
            ++seq;
        }
        return;
    }

    const uint32_t rd_off = lr * ROWB + lh * 16;  // + column block * 32 rows + plane + 32 bytes per step
    // one contraction step (16 indices) for both column blocks of 32 vectors: 12 MFMAs
    // (for the column blocks vb0 <= vb < vb1 of 32 vectors)
    auto step = [&](auto level_tag, const char *base, int s, floatx16 (&acc)[FB][2], int vb0, int vb1) {
        constexpr int LEVEL = decltype(level_tag)::value;  // highest non-zero term of the tile's vectors
        constexpr int NREAD = LEVEL < NSPLIT ? LEVEL : NSPLIT;
        bf16x8 d[2][NREAD];
#pragma unroll
        for (int vb = 0; vb < 2; ++vb)
#pragma unroll
            for (int p = 0; p < NREAD; ++p)
                if (vb >= vb0 && vb < vb1)
                    d[vb][p] = *reinterpret_cast<const bf16x8 *>(base + vb * 32 * ROWB + s * 32 + p * PLANE);
        // one product of terms for all accumulator tiles at a time, smallest terms first: the
        // tiles alternate, so that an MFMA never waits for the one just issued
        auto product = [&](auto pc_tag, auto pd_tag) {
            constexpr int PC = decltype(pc_tag)::value, PD = decltype(pd_tag)::value;
#pragma unroll
            for (int fb = 0; fb < FB; ++fb)
#pragma unroll
                for (int vb = 0; vb < 2; ++vb)
                    if (vb >= vb0 && vb < vb1)
                        acc[fb][vb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(c[fb][s][PC], d[vb][PD], acc[fb][vb], 0, 0, 0);
        };
        using T0 = std::integral_constant<int, 0>;
        using T1 = std::integral_constant<int, 1>;
        using T2 = std::integral_constant<int, 2>;
        if constexpr (NSPLIT == 3) {
            product(T2{}, T0{});
            if constexpr (LEVEL >= 2) product(T1{}, T1{});
            if constexpr (LEVEL >= 3) product(T0{}, T2{});
        }
        product(T1{}, T0{});
        if constexpr (LEVEL >= 2) product(T0{}, T1{});
        product(T0{}, T0{});
    };
    // Epilogue in two parts.  `settle` turns the accumulators of a tile into the 2 x 16 results
    // a lane keeps (bucket ids or raw projections); `store_piece` writes one 16-byte piece of
    // them.  The 8 pieces of a tile leave one per contraction step of the NEXT tile: a burst of
    // 64 store instructions per workgroup at the end of a tile holds the waves (and with them the
    // matrix pipe) until the memory pipeline has taken them.
    // An accumulator lane holds 16-byte pieces of 32 different vectors; stored like that, an
    // instruction writes 32-byte runs (two lanes per vector).  The pieces go through a
    // wave-private LDS block instead and come back with 8 consecutive lanes holding the 128 bytes
    // of one vector's 32 results: whole lines, 8 vectors per store instruction (measured on a
    // work copy with the stores moved to such addresses: 0.60 -> 0.48 ms for the SIFT shape).
    char *const stage = lds_s + kStageOffset + wave * STAGE;
    const uint32_t stage_wr = lr * STAGE_ROWB + 16 * lh;                // + 32 q
    const uint32_t stage_rd = (lane >> 3) * STAGE_ROWB + (lane & 7) * 16;  // + 8 j rows
    const uint32_t st_off = ((lane >> 3) * a.k + wf) * 4 + (lane & 7) * 16;  // in a block of 32 x k outputs; below 2^32 (host)
    // The wave's 32 offsets b~ wait in LDS and are read back four at a time at the tile's end:
    // held in registers through the contraction they cost 16 per lane (the ids epilogue then
    // needs 252 registers instead of 238 and runs 5 % slower; ids and keys together spill).
    constexpr bool OFFSETS = EP == kIds || EP == kKeys || EP == kIdsKeys;
    float *const wave_offsets = reinterpret_cast<float *>(lds_s + kOffsetsOffset + wave * 128);
    if constexpr (OFFSETS) {
        if (lane < 32) {
            const float b = a.off[wf + lane];
            wave_offsets[lane] = POW2 ? b * a.inv_w : b;
        }
    }
    uintx4 res[2][(SIGNS || KEYS || BOTH) ? 1 : 4];  // ids or the bits of the projections
    uint32_t sign_word[2][2] = {{0, 0}, {0, 0}};  // [column block][low, high half of the wave's sign word]
    // keys: a lane's four ids of accumulator group q are consecutive functions 8q + 4 (l / 32) ...
    // + 3 of the wave's 32; they are folded by Horner's rule and weighted with the power of C of
    // their place in the table, C^(g - 4 - (8q + 4 (l / 32)) % g)
    uint64_t key_weight[4] = {1, 1, 1, 1};
    if constexpr (KEYS) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const uint32_t expo = a.g - 4 - ((8 * q + 4 * lh) % a.g);
            for (uint32_t e = 0; e < expo; ++e) key_weight[q] *= kKeyMultiplier;
        }
    }
    // the four weighted partial keys of a lane (one per accumulator group) of column block vb:
    // summed per table inside the lane and across the two lanes that share a vector, and stored
    // ids and keys: the keys are folded from the staged pieces: lane l then holds the ids of
    // functions 4 (l % 8) .. + 3 of the wave's 32 for one vector, folds them by Horner's rule,
    // weights them with the power of C of their place in the table, and the g / 4 neighbouring
    // lanes of a table add up.  This epilogue stores ids and keys at the end of the tile instead of
    // spreading the ids over the next tile's steps: the 32 registers that would hold them are
    // what the fold needs.
    uint64_t piece_weight = 1;
    if constexpr (BOTH) {
        const uint32_t expo = a.g - 4 - ((4 * (lane & 7)) % a.g);
        for (uint32_t e = 0; e < expo; ++e) piece_weight *= kKeyMultiplier;
    }
    uint64_t t_settle = 0;  // the tile whose accumulators settle() is given (keys are stored from there)
    auto store_keys = [&](const uint64_t (&part)[4], int vb) {
        const uint64_t vec = t_settle * TV + vb * 32 + lr;
        uint64_t *row = reinterpret_cast<uint64_t *>(a.out) + vec * (a.k / a.g) + wf / a.g;
        // tables of the wave: 32 / g; a table's parts lie in one or both lanes of the vector
        if (a.g == 4) {  // uniform; table 2q + l / 32, one part each
            if (vec < a.N) {
#pragma unroll
                for (int q = 0; q < 4; ++q) row[2 * q + lh] = part[q];
            }
        } else {
            uint64_t key[4];
            int tables = 0;
            if (a.g == 8) {
                tables = 4;
#pragma unroll
                for (int q = 0; q < 4; ++q) key[q] = part[q];
            } else if (a.g == 16) {
                tables = 2;
                key[0] = part[0] + part[1];
                key[1] = part[2] + part[3];
                key[2] = key[3] = 0;
            } else {
                tables = 1;
                key[0] = part[0] + part[1] + part[2] + part[3];
                key[1] = key[2] = key[3] = 0;
            }
#pragma unroll
            for (int tb = 0; tb < 4; ++tb) {
                if (tb < tables) {  // uniform
                    const uint64_t sum = key[tb] + __shfl_xor(key[tb], 32);
                    if (lh == 0 && vec < a.N) row[tb] = sum;
                }
            }
        }
    };
    auto settle = [&](const floatx16 (&acc)[FB][2], int vb0, int vb1) {
#pragma unroll
        for (int vb = 0; vb < 2; ++vb) {
            if (vb < vb0 || vb >= vb1) continue;
            if constexpr (KEYS) {
                uint64_t part[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    uint64_t fold = 0;
                    const floatx4 b4 = *reinterpret_cast<const floatx4 *>(wave_offsets + 8 * q + 4 * lh);
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float p = acc[0][vb][4 * q + e];
                        const float h = POW2 ? fmaf(p, a.inv_w, b4[e]) : (p + b4[e]) / a.w;
                        fold = fold * kKeyMultiplier + (uint32_t)(int)floorf(h);
                    }
                    part[q] = fold * key_weight[q];
                }
                store_keys(part, vb);
            } else if constexpr (SIGNS) {
                // bit 8q + 4 (l / 32) + e of a block of 32 functions from accumulator 4q + e; the
                // two lanes that share a vector then join their halves
#pragma unroll
                for (int fb = 0; fb < FB; ++fb) {
                    uint32_t bits = 0;
#pragma unroll
                    for (int i = 0; i < 16; ++i) bits |= (acc[fb][vb][i] >= 0.f ? 1u : 0u) << (8 * (i / 4) + (i % 4));
                    bits <<= 4 * lh;
                    sign_word[vb][fb] = bits | (uint32_t)__shfl_xor((int)bits, 32);
                }
            } else {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    uintx4 v;
                    [[maybe_unused]] floatx4 b4;
                    if constexpr (OFFSETS) b4 = *reinterpret_cast<const floatx4 *>(wave_offsets + 8 * q + 4 * lh);
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float p = acc[0][vb][4 * q + e];
                        if constexpr (PROJ) {
                            v[e] = __float_as_uint(p);
                        } else {
                            const float h = POW2 ? fmaf(p, a.inv_w, b4[e]) : (p + b4[e]) / a.w;
                            v[e] = (uint32_t)(int)floorf(h);
                        }
                    }
                    *reinterpret_cast<uintx4 *>(stage + stage_wr + 32 * q) = v;
                }
                if constexpr (BOTH) {
                    const uint64_t vec0 = t_settle * TV + vb * 32;
                    const uint32_t first = 4 * (lane & 7);  // of the wave's 32 functions
#pragma unroll
                    for (int j = 0; j < 4; ++j) {  // piece j: vectors 8j .. 8j + 7, 8 lanes each
                        const uintx4 v = *reinterpret_cast<const uintx4 *>(stage + stage_rd + 8 * j * STAGE_ROWB);
                        const uint64_t vec = vec0 + 8 * j + (lane >> 3);
                        uint64_t fold = v[0];
#pragma unroll
                        for (int e = 1; e < 4; ++e) fold = fold * kKeyMultiplier + v[e];
                        fold *= piece_weight;
                        if (a.g >= 8) fold += __shfl_xor(fold, 1);  // uniform
                        if (a.g >= 16) fold += __shfl_xor(fold, 2);
                        if (a.g >= 32) fold += __shfl_xor(fold, 4);
                        if (vec < a.N) {
                            char *dst = reinterpret_cast<char *>(a.out) + (vec0 + 8 * j) * a.k * 4 + st_off;
                            __builtin_nontemporal_store(v, reinterpret_cast<uintx4 *>(dst));
                            if (first % a.g == 0)
                                reinterpret_cast<uint64_t *>(a.out2)[vec * (a.k / a.g) + (wf + first) / a.g] = fold;
                        }
                        __builtin_amdgcn_sched_barrier(0);  // one piece at a time: no registers for four
                    }
                    continue;
                }
                // the wave's own LDS accesses execute in order: no wait between writes and reads
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    res[vb][j] = *reinterpret_cast<const uintx4 *>(stage + stage_rd + 8 * j * STAGE_ROWB);
            }
        }
    };
    // signs: the wave's 64 functions are the 64-bit word wf / 64 of each vector
    const uint32_t sign_off = (lr * (a.k / 64) + wf / 64) * 8;  // in a block of 32 vectors
    auto store_piece = [&](auto full_tag, uint64_t tile, int piece) {
        const int vb = piece / 4, q = piece % 4;
        const uint64_t vec0 = tile * TV + vb * 32;
        if constexpr (KEYS || BOTH) {
            return;  // stored by settle()
        } else if constexpr (SIGNS) {
            if (q != 0 || lh != 0) return;
            if constexpr (!decltype(full_tag)::value) {
                if (vec0 + lr >= a.N) return;
            }
            char *dst = reinterpret_cast<char *>(a.out) + vec0 * (a.k / 64) * 8 + sign_off;
            *reinterpret_cast<uint2 *>(dst) = make_uint2(sign_word[vb][0], sign_word[vb][1]);
        } else {
            // piece q of a column block: vectors 8q .. 8q + 7, 8 lanes each
            if constexpr (!decltype(full_tag)::value) {
                if (vec0 + 8 * q + (lane >> 3) >= a.N) return;
            }
            char *dst = reinterpret_cast<char *>(a.out) + (vec0 + 8 * q) * a.k * 4 + st_off;
            // whole lines that nothing reads back soon: non-temporal (2-3 % on the SIFT shape; on
            // partial lines such stores lose, as they no longer combine in L2)
            __builtin_nontemporal_store(res[vb][q], reinterpret_cast<uintx4 *>(dst));
        }
    };
    // One tile.  The vector-ALU and memory work shares the scheduling regions of the contraction
    // steps, so that the matrix pipe runs in its background (and in that of the other wave of the
    // SIMD): step s stores piece s of the previous tile, and the last four steps each split one
    // 16-byte piece of the next tile on its way to LDS.  The loads these consume were issued a
    // tile earlier and have the first steps to arrive; the loads of the tile after the next are
    // issued last.
    uint64_t t_prev = 0;
    auto contract_tile = [&](auto have_prev, auto level_tag) {
        const char *base = lds_s + cur * BUF + rd_off;
        char *next = lds_s + (cur ^ 1) * BUF;
        floatx16 acc[FB][2];
#pragma unroll
        for (int fb = 0; fb < FB; ++fb)
#pragma unroll
            for (int vb = 0; vb < 2; ++vb)
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[fb][vb][i] = 0.f;
        if constexpr (SIGNS) {
            // two function blocks per wave: the column blocks take turns, so that only half of the
            // accumulators are live at a time; the second pass carries the split of the next tile
#pragma unroll
            for (int vb = 0; vb < 2; ++vb) {
#pragma unroll
                for (int s = 0; s < KSTEPS; ++s) {
                    step(level_tag, base, s, acc, vb, vb + 1);
                    if constexpr (decltype(have_prev)::value) {
                        if (s == 0) store_piece(std::true_type{}, t_prev, 4 * vb);
                    }
                    if (vb == 1 && s >= KSTEPS - kQuads) stash_quad(next, s - (KSTEPS - kQuads));
                    __builtin_amdgcn_sched_barrier(0);
                }
                t_settle = t;
                settle(acc, vb, vb + 1);
            }
        } else {
#pragma unroll
            for (int s = 0; s < KSTEPS; ++s) {
                step(level_tag, base, s, acc, 0, 2);
                if constexpr (decltype(have_prev)::value) store_piece(std::true_type{}, t_prev, s);  // a tile with a successor is whole
                if (s >= KSTEPS - kQuads) stash_quad(next, s - (KSTEPS - kQuads));
                __builtin_amdgcn_sched_barrier(0);
            }
            t_settle = t;
            settle(acc, 0, 2);
        }
    };
    auto run_tile = [&](auto have_prev) {
        // the level of the tile in the current buffer: stale words belong to earlier tiles
        const uint32_t word = __builtin_amdgcn_readfirstlane(level_word[cur]);
        const uint32_t level = (word >> 2) == seq + 1 ? (word & 3u) : 1u;
        if (level == 1) contract_tile(have_prev, std::integral_constant<int, 1>{});
        else if (level == 2) contract_tile(have_prev, std::integral_constant<int, 2>{});
        else contract_tile(have_prev, std::integral_constant<int, 3>{});
        // the loads go out after the variants have joined: none is in flight where registers
        // might have to be copied
        publish_level(cur ^ 1, seq + 1);
        t_prev = t;
        fetch(t + 2 * streams);
        __syncthreads();  // next buffer complete; everyone is done with the current one
        cur ^= 1;
        ++seq;
    };
    static_assert(KSTEPS == 8, "one stored piece per contraction step");
    if (t >= ntiles) return;
    run_tile(std::false_type{});
    for (t += streams; t < ntiles; t += streams) run_tile(std::true_type{});
#pragma unroll
    for (int piece = 0; piece < 8; ++piece) store_piece(std::false_type{}, t_prev, piece);
}

}  // namespace

bool dense_split_supported(const lsh_params *p) {
    return p->n == (uint32_t)SN && p->k % kFuncsPerWave == 0 && p->k <= (1u << 24) && p->d_dense != nullptr;
}

bool dense_split_keys_supported(const lsh_params *p, uint32_t L) {
    if (!dense_split_supported(p) || !L || p->k % L) return false;
    const uint32_t g = p->k / L;
    return g == 4 || g == 8 || g == 16 || g == 32;
}

bool dense_split_signs_supported(const lsh_params *p) {
    return p->n == (uint32_t)SN && p->k % 64 == 0 && p->k <= (1u << 24) && p->d_dense != nullptr;
}

// ep: 0 bucket ids, 1 raw projections, 2 sign words, 3 keys of L tables, 4 ids (d_out) and keys (d_out2)
int launch_dense_split(const lsh_params *p, int ep, const float *d_data, uint64_t N, void *d_out,
                       void *stream, uint32_t L, void *d_out2) {
    SplitArgs a;
    a.data = d_data;
    a.a = p->d_dense;
    a.off = p->d_off;
    a.N = N;
    a.k = p->k;
    a.g = L ? p->k / L : 0;
    a.w = p->w;
    a.inv_w = 1.0f / p->w;
    a.out = d_out;
    a.out2 = d_out2;
    int exp2 = 0;
    const bool pw = (ep != kIds && ep != kKeys && ep != kIdsKeys) || std::frexp(p->w, &exp2) == 0.5f;  // only ids and keys divide
    const uint32_t block_funcs = kFuncsPerBlock * (ep == kSigns ? 2 : 1);
    const uint32_t slices = (p->k + block_funcs - 1) / block_funcs;
    // one workgroup per CU (102 KB of LDS); every XCD needs a workgroup per slice of functions
    uint32_t wgs = (uint32_t)(p->num_cus > 0 ? p->num_cus : 256) / 8 * 8;
    if (wgs < 8) wgs = 8;
    while (wgs / 8 < slices) wgs += 8;
    const uint32_t lds_bytes = kLdsBytes;  // two tiles, their level words, the waves' staging blocks
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
#define LSH_SPLIT_CASE(E_, W_) \
    if (ep == E_ && pw == W_) { \
        auto fn = &dense_split_kernel<E_, W_>; \
        if (ensure_lds_limit(reinterpret_cast<const void *>(fn), lds_bytes) != LSH_OK) return LSH_ERR_HIP; \
        hipLaunchKernelGGL(fn, dim3(wgs), dim3(kThreadsS), lds_bytes, s, a); \
    }
    LSH_SPLIT_CASE(kIds, true) LSH_SPLIT_CASE(kIds, false) LSH_SPLIT_CASE(kProj, true) LSH_SPLIT_CASE(kSigns, true)
    LSH_SPLIT_CASE(kKeys, true) LSH_SPLIT_CASE(kKeys, false) LSH_SPLIT_CASE(kIdsKeys, true) LSH_SPLIT_CASE(kIdsKeys, false)
#undef LSH_SPLIT_CASE
    return hipGetLastError() == hipSuccess ? LSH_OK : LSH_ERR_HIP;
}

}  // namespace lsh
