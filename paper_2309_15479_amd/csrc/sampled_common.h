// Device-side pieces shared by the sampled-projection kernels (sampled_kernel.hip,
// ranged_kernel.hip): the kernel argument block, the tile loads and their transposition, and
// the epilogues (bucket ids, raw projections, sign words, keys).  Included by .hip files only.
#pragma once
#include <hip/hip_runtime.h>

#include "device_utils.h"
#include "lsh_internal.h"

namespace lsh {
namespace {

template <int RT>
__device__ __forceinline__ void lds_read_slot(const char *slot, float (&x)[RT]) {
    if constexpr (RT == 4) {
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
    if constexpr (RT == 4) {
        *reinterpret_cast<float4 *>(slot) = make_float4(x[0], x[1], x[2], x[3]);
    } else if constexpr (RT == 2) {
        *reinterpret_cast<float2 *>(slot) = make_float2(x[0], x[1]);
    } else {
        *slot = x[0];
    }
}

// Empty volatile asm through which four accumulators flow: it emits nothing, but the FMAs
// that produce its inputs cannot be sunk below it (nor the next ones hoisted above), which
// keeps them inside the scheduling region they were written in.
__device__ __forceinline__ void pin(float (&v)[4]) {
    asm volatile("" : "+v"(v[0]), "+v"(v[1]), "+v"(v[2]), "+v"(v[3]));
}

// Returns v through an empty asm: the compiler can no longer treat values derived from it as
// loop invariants, so it recomputes cheap per-lane addresses where they are used instead of
// keeping dozens of them (and spilling) across the gather loops.
__device__ __forceinline__ uint32_t fresh(uint32_t v) {
    asm volatile("" : "+v"(v));
    return v;
}

struct SampledArgs {
    const float *data;   // [N][n]
    uint64_t N;
    uint32_t n, k, m_pad, kpad, classes;
    const Sample *tab;   // [m_pad][kpad]
    const float *off;    // [kpad]
    float w, inv_w;
    int w_is_pow2;
    int epilogue;        // Epilogue
    void *out;
    void *out2;          // Epilogue::IdsKeys: the keys (the ids go to out)
    uint32_t L, g;       // key groups (Epilogue::Keys, Epilogue::IdsKeys)
    // register-list kernel only: floats per tile buffer; float offset of the second,
    // class-rotated tile copy inside a buffer (0: single copy)
    uint32_t buf_floats, copy_b_floats;
    // ranged kernel only (ranged_kernel.hip)
    uint32_t chunk, nchunks;     // coordinates per range, number of ranges
    uint32_t stages, bar_stride; // stages per tile (a multiple of the ring's slots); words per workgroup in list_len
    const uint4 *triples;        // list blocks (quads of entries: coefficients, then 16-bit LDS slot numbers), stream after stream
    const uint32_t *list_len;    // [workgroup along the function axis][bar_stride] barriers before the first block of a tile and after each block
    const uint2 *stream;         // [stream] {first block, blocks per tile}
    uint32_t fpt;                // functions per lane
};

// The LDS slot (one coordinate of four vectors) that lane `lane` of a wave contributes to a
// 64-coordinate piece: coordinate c_first + lane of vectors row_first .. row_first + 3.
// With n a multiple of 4 each lane loads 16 contiguous bytes instead of four separate
// words (coordinates c_first + 4*(lane/4) .. + 3 of vector row_first + lane % 4: a quad of
// lanes covers 4 vectors x 4 coordinates, a wave reads 256 contiguous bytes of each vector):
// a quarter of the vector-memory instructions.  The registers then hold the transpose of
// the slot; slot_from_raw() turns them into the slot just before it is written to LDS.
// `limit` bounds the coordinates of the piece (exclusive); it is a multiple of 4 when vec4.
template <bool vec4>
__device__ __forceinline__ void load_raw(const float *__restrict__ tile_rows, uint32_t rows_valid, uint32_t n,
                                         uint32_t row_first, uint32_t c_first, uint32_t limit, uint32_t lane,
                                         float (&x)[4]) {
    // tile_rows = first vector of the tile (wave-uniform pointer); rows and coordinates are
    // 32-bit offsets from it.  Rows past the end of the data and coordinates past `limit`
    // read element 0 of the tile instead (always valid memory): their values are never used.
    if (vec4) {
        const uint32_t row = row_first + (lane & 3);
        const uint32_t c = c_first + (lane & ~3u);
        const uint32_t off = (c < limit && row < rows_valid) ? row * n + c : 0u;
        // a tile is read once: non-temporal, which leaves L2 to the sample lists (2 % at n = 4096,
        // m = 64; nothing elsewhere)
        typedef float floatx4 __attribute__((ext_vector_type(4)));
        const floatx4 q = __builtin_nontemporal_load(reinterpret_cast<const floatx4 *>(tile_rows + off));
        x[0] = q[0]; x[1] = q[1]; x[2] = q[2]; x[3] = q[3];
    } else {
        const uint32_t c = c_first + lane;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const uint32_t off = (c < limit && row_first + r < rows_valid) ? (row_first + r) * n + c : 0u;
            x[r] = __builtin_nontemporal_load(tile_rows + off);
        }
    }
}

template <bool vec4>
__device__ __forceinline__ void slot_from_raw(float (&x)[4]) {
    if (vec4) {
        uint32_t v[4] = {__float_as_uint(x[0]), __float_as_uint(x[1]), __float_as_uint(x[2]), __float_as_uint(x[3])};
        quad_transpose(v);
#pragma unroll
        for (int r = 0; r < 4; ++r) x[r] = __uint_as_float(v[r]);
    }
}

// Sum of a 64-bit value over each aligned group of g consecutive lanes (g a power of two
// <= 64); every lane of the group gets the sum.  Steps inside a row of 16 lanes are DPP moves
// (quad permutes, half-row and row mirrors: no LDS traffic, the resource the gather is short
// of); only the steps across rows use the LDS crossbar.
template <int CTRL>
__device__ __forceinline__ uint64_t dpp_u64(uint64_t v) {
    const uint32_t lo = (uint32_t)__builtin_amdgcn_mov_dpp((int)(uint32_t)v, CTRL, 0xf, 0xf, true);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_mov_dpp((int)(uint32_t)(v >> 32), CTRL, 0xf, 0xf, true);
    return ((uint64_t)hi << 32) | lo;
}

__device__ __forceinline__ uint64_t group_sum(uint64_t v, uint32_t g) {
    if (g >= 2) v += dpp_u64<0xB1>(v);    // quad_perm [1,0,3,2]
    if (g >= 4) v += dpp_u64<0x4E>(v);    // quad_perm [2,3,0,1]
    if (g >= 8) v += dpp_u64<0x141>(v);   // row_half_mirror: the other quad of the half row
    if (g >= 16) v += dpp_u64<0x140>(v);  // row_mirror: the other half of the row
    if (g >= 32) v += __shfl_xor(v, 16);
    if (g >= 64) v += __shfl_xor(v, 32);
    return v;
}

// The same transpose for fp32 values, on the matrix pipe instead of the vector ALU (which is
// what bounds the sampled kernels): the 4x4x1 MFMA computes, in every quad of lanes,
// D[i][u] += A[i] * B[u] with A[i], B[u] taken from lanes i, u of the quad and D[i][u] landing in
// register i of lane u.  Four of them, with A = x[t] and B = [u == t], leave x[u] of lane i in
// register i of lane u.  Multiplying by 1 and adding zeros is exact for finite values;
// callers clamp first, so that a non-finite value cannot leak into its quad neighbours.
typedef float float4v __attribute__((ext_vector_type(4)));
__device__ __forceinline__ void quad_transpose_mfma(float (&x)[4], const float (&unit)[4]) {
    float4v d = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int t = 0; t < 4; ++t) d = __builtin_amdgcn_mfma_f32_4x4x1f32(x[t], unit[t], d, 0, 0, 0);
#pragma unroll
    for (int t = 0; t < 4; ++t) x[t] = d[t];
}

// v_writelane_b32 as a compiler intrinsic (this compiler has no builtin of that name); written
// as inline assembly instead it would miss the wait states the hardware needs between a
// vector compare that writes the scalar value and the lane write that reads it.
extern "C" __device__ int write_lane(int value, int lane, int old) __asm("llvm.amdgcn.writelane.i32");

// One tile's results of one lane: acc[s][r] belongs to vector row0 + s*RT + r.  A vector
// memory instruction costs the memory pipeline about the same whether a lane moves 4 or 16
// bytes, and this kernel issues one store per (wave, vector): so with 4-vector slots the ids
// of a quad of lanes are transposed in registers first and leave as 16-byte stores (four
// consecutive functions of one vector per lane), and sign words leave one store per tile.
// For a power-of-two w, (p + b) / w is computed as fma(p, 1/w, b/w): scaling by a power of two
// commutes with the rounding of the sum, so the result is the same float.
// FULL: every vector of the tile exists; the stores then go to a wave-uniform base (scalar
// arithmetic) plus the per-lane byte offset full_off the caller keeps in a register:
// ((lane % 4) * k + (j & ~3)) * 4 for ids, (lane % 64 * ceil(k / 64) + j / 64) * 8 for sign words.
template <int RT, int SUB, int EP, bool FULL = false>
__device__ __forceinline__ void finish(const SampledArgs &a, uint64_t row0, uint32_t j,
                                       const float (&acc)[SUB][RT], float b, uint64_t key_pow,
                                       uint32_t full_off = 0) {
    const bool live = j < a.k;
    switch (EP) {
        case (int)Epilogue::Ids:
        case (int)Epilogue::Proj: {
            constexpr bool ids = EP == (int)Epilogue::Ids;
            uint32_t *out = reinterpret_cast<uint32_t *>(a.out);
            const bool wide = RT == 4 && (a.k & 3) == 0;
            const float b_scaled = b * a.inv_w;
            float unit[4];
#pragma unroll
            for (int t = 0; t < 4; ++t) unit[t] = (threadIdx.x & 3) == (uint32_t)t ? 1.f : 0.f;
#pragma unroll
            for (int s = 0; s < SUB; ++s) {
                float q[RT];
#pragma unroll
                for (int r = 0; r < RT; ++r) {
                    const float p = acc[s][r];
                    q[r] = !ids ? p : a.w_is_pow2 ? fmaf(p, a.inv_w, b_scaled) : (p + b) / a.w;
                }
                if constexpr (RT == 4) {
                    if (wide) {  // uniform
                        // beyond +-2^31 the conversion saturates anyway
                        const float bound = ids ? 2147483648.f : 3.4028234664e38f;
#pragma unroll
                        for (int r = 0; r < RT; ++r) q[r] = __builtin_amdgcn_fmed3f(q[r], -bound, bound);
                        quad_transpose_mfma(q, unit);
                        const uint64_t row = row0 + s * RT + (threadIdx.x & 3);
                        const uint32_t j4 = j & ~3u;
                        uint32_t v[4];
#pragma unroll
                        for (int r = 0; r < RT; ++r) v[r] = ids ? (uint32_t)(int)floorf(q[r]) : __float_as_uint(q[r]);
                        if constexpr (FULL) {
                            char *base = reinterpret_cast<char *>(out + (row0 + s * RT) * a.k);  // uniform
                            if (j4 < a.k) *reinterpret_cast<uint4 *>(base + full_off) = make_uint4(v[0], v[1], v[2], v[3]);
                        } else if (j4 < a.k && row < a.N) {
                            *reinterpret_cast<uint4 *>(out + row * a.k + j4) = make_uint4(v[0], v[1], v[2], v[3]);
                        }
                        continue;
                    }
                }
#pragma unroll
                for (int r = 0; r < RT; ++r) {
                    const uint64_t row = row0 + s * RT + r;
                    if (live && row < a.N) out[row * a.k + j] = ids ? (uint32_t)(int)floorf(q[r]) : __float_as_uint(q[r]);
                }
            }
            break;
        }
        case (int)Epilogue::Signs: {
            uint64_t *out = reinterpret_cast<uint64_t *>(a.out);
            const uint32_t words = (a.k + 63) / 64;
            const uint32_t lane = threadIdx.x & 63;
            uint32_t lo = 0, hi = 0;  // lane v of the wave keeps the word of the tile's vector v
#pragma unroll
            for (int s = 0; s < SUB; ++s)
#pragma unroll
                for (int r = 0; r < RT; ++r) {
                    const uint64_t word = __ballot(live && acc[s][r] >= 0.f);  // whole waves get here
                    // the wave-uniform word goes into lane s * RT + r only
                    lo = (uint32_t)write_lane((int)(uint32_t)word, s * RT + r, (int)lo);
                    hi = (uint32_t)write_lane((int)(uint32_t)(word >> 32), s * RT + r, (int)hi);
                }
            const uint64_t mine = ((uint64_t)hi << 32) | lo;
            const uint64_t row = row0 + lane;
            if constexpr (FULL) {
                char *base = reinterpret_cast<char *>(out + row0 * words);  // uniform
                if (lane < (uint32_t)(SUB * RT) && (j & ~63u) < a.k) *reinterpret_cast<uint64_t *>(base + full_off) = mine;
            } else if (lane < (uint32_t)(SUB * RT) && (j & ~63u) < a.k && row < a.N) {
                out[row * words + (j >> 6)] = mine;
            }
            break;
        }
        default: {  // Keys: g consecutive lanes fold their ids; g is a power of two <= 64
            // IdsKeys (launched only with 4-vector sub-tiles, g >= 4 and k a multiple of 4): the
            // transposed path below, which also stores the four ids a lane holds after the transpose
            constexpr bool both = EP == (int)Epilogue::IdsKeys;
            uint64_t *out = reinterpret_cast<uint64_t *>(both ? a.out2 : a.out);
            if constexpr (RT == 4) {
                if (both || a.g >= 4) {  // uniform
                    // As for ids, the quads are transposed first: a lane then holds the ids of the
                    // quad's four consecutive functions for ONE vector, folds them by Horner's rule
                    // (three multiplications by C and one by its power of C, instead of one 64-bit
                    // multiplication per id and vector), and only the g / 4 partials of a vector are
                    // left to add across lanes: those of the lanes i, i + 4, i + 8, ... of the key
                    // group, by DPP shifts inside a row of 16 lanes and exchanges across rows.
                    // (for g >= 4 the kernels pass key_pow = C^(g-1-(t|3)), the power of the quad's last function)
                    // everything per lane is derived from j, which the register-list kernels pass
                    // through an empty asm every tile: derived from threadIdx.x it would be hoisted
                    // out of the tile loop and held in registers across the gather
                    const uint32_t g_log2 = 31 - __builtin_clz(a.g), t = j & (a.g - 1), u_mine = j & 3;  // workgroup sizes are multiples of 4
                    float unit[4];
#pragma unroll
                    for (int u = 0; u < 4; ++u) unit[u] = u_mine == (uint32_t)u ? 1.f : 0.f;
                    const float b_scaled = b * a.inv_w;
#pragma unroll
                    for (int s = 0; s < SUB; ++s) {
                        float q[RT];
#pragma unroll
                        for (int r = 0; r < RT; ++r) {
                            const float v = a.w_is_pow2 ? fmaf(acc[s][r], a.inv_w, b_scaled) : (acc[s][r] + b) / a.w;
                            q[r] = __builtin_amdgcn_fmed3f(v, -2147483648.f, 2147483648.f);
                        }
                        quad_transpose_mfma(q, unit);
                        uint32_t id[4];
#pragma unroll
                        for (int r = 0; r < RT; ++r) id[r] = (uint32_t)(int)floorf(q[r]);
                        if constexpr (both) {
                            // functions j & ~3 .. + 3 of vector row0 + s * RT + u_mine, as in the ids epilogue
                            const uint64_t id_row = row0 + s * RT + u_mine;
                            if ((j & ~3u) < a.k && id_row < a.N)
                                *reinterpret_cast<uint4 *>(reinterpret_cast<uint32_t *>(a.out) + id_row * a.k + (j & ~3u)) =
                                    make_uint4(id[0], id[1], id[2], id[3]);
                        }
                        uint64_t part = id[0];
                        part = part * kKeyMultiplier + id[1];
                        part = part * kKeyMultiplier + id[2];
                        part = part * kKeyMultiplier + id[3];
                        part *= key_pow;
                        if (a.g >= 8) part += dpp_u64<0x104>(part);   // row_shl:4: lane i takes lane i + 4 (0 past the row)
                        if (a.g >= 16) part += dpp_u64<0x108>(part);  // row_shl:8
                        if (a.g >= 32) part += __shfl_down(part, 16);
                        if (a.g >= 64) part += __shfl_down(part, 32);
                        const uint64_t row = row0 + s * RT + u_mine;
                        if (live && row < a.N && t < 4) out[row * a.L + (j >> g_log2)] = part;
                    }
                    break;
                }
            }
#pragma unroll
            for (int s = 0; s < SUB; ++s)
#pragma unroll
                for (int r = 0; r < RT; ++r) {
                    const uint64_t row = row0 + s * RT + r;
                    const float q = a.w_is_pow2 ? (acc[s][r] + b) * a.inv_w : (acc[s][r] + b) / a.w;
                    const uint64_t key = group_sum((uint64_t)(uint32_t)(int)floorf(q) * key_pow, a.g);
                    if (live && row < a.N && (j % a.g) == 0) out[row * a.L + j / a.g] = key;
                }
        }
    }
}

}  // namespace
}  // namespace lsh
