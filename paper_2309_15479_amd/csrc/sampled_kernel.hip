// Sampled-projection kernel (FastLSH, Sec. 3.1, Eq. 5) for gfx950.
//
//   p_j(v) = sum_{i<m} a~_j[i] * v[S_j[i]],   h_j(v) = floor((p_j(v) + b~_j) / w)
//
// Mapping: one lane = one hash function j; one workgroup = a tile of SUB*RT vectors times
// blockDim.x functions.  The vector tile is read from HBM once (coalesced along the
// coordinate axis) and kept in LDS as [coordinate][sub-tile][RT vectors], so that one
// 4*RT-byte LDS read fetches a sampled coordinate of RT vectors, and the SUB reads of one
// sample differ only in their immediate offset.  Each lane walks its own list of
// (LDS offset, coefficient) pairs; there is no cross-lane reduction.
//
// Every gather-FMA costs one 64-lane vector-ALU slot (4 cycles of a SIMD: the library is
// compiled without packed fp32) and 4 bytes of LDS bandwidth, and the two ceilings are close, so both are
// kept lean.  LDS: the order in which a lane visits its samples is chosen on the host
// (schedule.cpp) such that the lanes served together by one pass of an LDS read (four quads
// of lanes for 16-byte reads) hit distinct bank classes; with more than one sub-tile the
// coordinate stride is padded to an odd number of 16-byte slots, which keeps "distinct
// coordinates mod 16" equivalent to "distinct bank classes" for every sub-tile.  Vector ALU:
// 16-vector tiles share each address computation among 16 FMAs, and the epilogues move what
// they can to the matrix pipe, the scalar ALU and single instructions (see finish()).  The
// lists are stored step-major ([step][function]) so that a wave reads them coalesced.
//
// Three kernels: sampled_reg_kernel keeps lists of up to 64 samples in registers for the whole
// launch (small n); sampled_kernel streams longer lists through registers for every
// full-dimension tile; sampled_chunked_kernel cuts large vectors into coordinate ranges that
// fill LDS and walks per-range lists.
#include <hip/hip_runtime.h>

#include <mutex>
#include <type_traits>
#include <unordered_map>

#include "device_utils.h"
#include "lsh_internal.h"

namespace lsh {
namespace {

constexpr int kChunk = 32;                     // samples held in registers at a time
constexpr uint32_t kLdsBudget = 158u * 1024u;  // of the CU's 160 KB
// chunked kernel: 64-coordinate pieces of the next chunk a wave prefetches into registers
// (6 x 16 waves cover the 1376 coordinates x 4 sub-tiles that fill LDS)
constexpr int kChunkPre = 6;

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
    uint32_t L, g;       // key groups (Epilogue::Keys)
    // register-list kernel only: floats per tile buffer; float offset of the second,
    // class-rotated tile copy inside a buffer (0: single copy)
    uint32_t buf_floats, copy_b_floats;
    // chunked kernel only
    uint32_t chunk, nchunks;     // coordinates per LDS chunk, number of chunks
    const uint2 *chunk_info;     // [waves][nchunks] {first table entry, steps}
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
            uint64_t *out = reinterpret_cast<uint64_t *>(a.out);
            if constexpr (RT == 4) {
                if (a.g >= 4) {  // uniform
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
                        uint64_t part = (uint32_t)(int)floorf(q[0]);
                        part = part * kKeyMultiplier + (uint32_t)(int)floorf(q[1]);
                        part = part * kKeyMultiplier + (uint32_t)(int)floorf(q[2]);
                        part = part * kKeyMultiplier + (uint32_t)(int)floorf(q[3]);
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

// Streamed-list kernel: every tile, each lane streams its (offset, coefficient) list through
// registers one chunk at a time and applies the chunk to all SUB sub-tiles.
template <int RT, int SUB, int EP>
__global__ __launch_bounds__(1024) void sampled_kernel(const SampledArgs a) {
    extern __shared__ __align__(16) float tile[];  // [n + classes][SP][RT]
    constexpr uint32_t SP = SUB == 1 ? 1 : SUB + 1;
    constexpr uint32_t kTileRows = RT * SUB;
    const uint32_t n = a.n;
    const uint32_t j = blockIdx.y * blockDim.x + threadIdx.x;  // < kpad
    const uint64_t ntiles = (a.N + kTileRows - 1) / kTileRows;
    const float b = a.off[j];

    // zero slots: the targets of padding samples
    for (uint32_t e = threadIdx.x; e < a.classes * SP * RT; e += blockDim.x)
        tile[(size_t)n * SP * RT + e] = 0.f;

    uint64_t key_pow = 1;  // C^(g-1-t) for this lane's position t in its key group
    if (EP == (int)Epilogue::Keys) {
        uint32_t t = j % a.g;
        if (RT == 4 && a.g >= 4) t |= 3;  // the transposed fold multiplies by the power of the quad's last function
        for (uint32_t e = 0; e + 1 + t < a.g; ++e) key_pow *= kKeyMultiplier;
    }

    // wave w loads the 64-coordinate chunks q = w, w + nwaves, ... of the tile; chunk q is
    // coordinates (q / SUB) * 64 .. + 63 of sub-tile q % SUB
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint32_t lane = threadIdx.x & 63;
    const uint32_t nwaves = blockDim.x >> 6;
    const uint32_t nchunks = SUB * ((n + 63) / 64);

    const char *base = reinterpret_cast<const char *>(tile);
    for (uint64_t t = blockIdx.x; t < ntiles; t += gridDim.x) {
        const uint64_t row0 = t * kTileRows;
        __syncthreads();  // every lane is done reading the previous tile
        for (uint32_t q = wave; q < nchunks; q += nwaves) {
            const uint32_t st = q % SUB, c = (q / SUB) * 64 + lane;
            if (c < n) {
                float x[RT];
#pragma unroll
                for (int r = 0; r < RT; ++r) {
                    const uint64_t row = row0 + (uint64_t)st * RT + r;
                    x[r] = row < a.N ? a.data[row * n + c] : 0.f;
                }
                lds_write_slot<RT>(tile + ((size_t)c * SP + st) * RT, x);
            }
        }
        __syncthreads();

        float acc[SUB][RT];
#pragma unroll
        for (int st = 0; st < SUB; ++st)
#pragma unroll
            for (int r = 0; r < RT; ++r) acc[st][r] = 0.f;

        for (uint32_t i0 = 0; i0 < a.m_pad; i0 += kChunk) {
            Sample s[kChunk];
#pragma unroll
            for (int i = 0; i < kChunk; ++i) s[i] = a.tab[(size_t)(i0 + i) * a.kpad + j];
#pragma unroll
            for (int i = 0; i < kChunk; ++i) {
                const char *slot = base + s[i].lds_byte_offset;
#pragma unroll
                for (int st = 0; st < SUB; ++st) {
                    float x[RT];
                    lds_read_slot<RT>(slot + st * RT * 4, x);
#pragma unroll
                    for (int r = 0; r < RT; ++r) acc[st][r] = fmaf(s[i].coef, x[r], acc[st][r]);
                }
            }
        }
        finish<RT, SUB, EP>(a, row0, j, acc, b, key_pow);
    }
}

// Register-list kernel for m_pad == MCH * kChunk (MCH = 1 or 2): a lane's whole list stays in VGPRs while the
// workgroup walks its tiles.  The LDS tile is double buffered: the next tile's vectors are
// fetched from HBM into registers before the current tile is processed and written to the
// other buffer afterwards, so one barrier per tile suffices and HBM latency hides behind the
// gather.  The gather itself is software pipelined by hand (reads of sample i+1 are issued
// with the FMAs of sample i); scheduling barriers keep the compiler from hoisting every LDS
// read of the tile to the front, which would need more registers than a lane has.
// PF = 64-coordinate chunks each wave fetches per tile (see launch_sampled).
// REGULAR: the launch covers whole tiles only, n is a multiple of 64 and every wave has PF
// pieces inside the vector: loads, LDS writes and stores then need no predicates and their
// addresses are a wave-uniform base plus per-lane constants (the host sends the vectors
// beyond the last whole tile through the general instantiation).
template <int SUB, int PF, int MCH, int EP, bool REGULAR>
__global__ __launch_bounds__(512, MCH == 1 ? 4 : 2) void sampled_reg_kernel(const SampledArgs a) {
    constexpr int RT = 4;
    extern __shared__ __align__(16) float tile[];  // 2 x [n + classes][SP][RT]
    constexpr uint32_t SP = SUB == 1 ? 1 : SUB + 1;
    constexpr uint32_t kTileRows = RT * SUB;
    const uint32_t n = a.n;
    const uint32_t j = blockIdx.y * blockDim.x + threadIdx.x;  // < kpad
    const uint64_t ntiles = (a.N + kTileRows - 1) / kTileRows;
    const uint32_t buf_floats = a.buf_floats;

    // list entries kept in registers: coefficients, and LDS byte offsets (below 64 KB for
    // the tiles this kernel takes) two to a register
    constexpr int kList = kChunk * MCH;
    constexpr int kDepth = 2;  // samples whose LDS reads are in flight or being consumed
    uint32_t po[kList / 2];
    float cf[kList];
#pragma unroll
    for (int i = 0; i < kList; i += 2) {
        const Sample s0 = a.tab[(size_t)i * a.kpad + j], s1 = a.tab[(size_t)(i + 1) * a.kpad + j];
        po[i / 2] = s0.lds_byte_offset | (s1.lds_byte_offset << 16);
        cf[i] = s0.coef;
        cf[i + 1] = s1.coef;
    }
    const float b = a.off[j];

    for (uint32_t e = threadIdx.x; e < a.classes * SP * RT; e += blockDim.x) {
        tile[(size_t)n * SP * RT + e] = 0.f;
        tile[buf_floats + (size_t)n * SP * RT + e] = 0.f;
    }

    uint64_t key_pow = 1;
    if (EP == (int)Epilogue::Keys) {
        uint32_t t = j % a.g;
        if (RT == 4 && a.g >= 4) t |= 3;  // the transposed fold multiplies by the power of the quad's last function
        for (uint32_t e = 0; e + 1 + t < a.g; ++e) key_pow *= kKeyMultiplier;
    }

    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint32_t lane = threadIdx.x & 63;
    const uint32_t nwaves = blockDim.x >> 6;
    const uint32_t nchunks = SUB * ((n + 63) / 64);
    const bool vec4 = (n & 3) == 0;

    float pre[PF][RT];
    auto fetch_as = [&](uint64_t row0, auto vec) {
        constexpr bool V = decltype(vec)::value;
        const float *rows = a.data + row0 * n;
        const uint32_t rows_valid = (uint32_t)min((uint64_t)kTileRows, a.N - row0);
        const uint32_t ln = fresh(lane);
#pragma unroll
        for (int f = 0; f < PF; ++f) {
            const uint32_t q = wave + f * nwaves;
            load_raw<V>(rows, rows_valid, n, (q % SUB) * RT, (q / SUB) * 64, q < nchunks ? n : 0, ln, pre[f]);
        }
    };
    auto stash_as = [&](float *buf, auto vec) {
        constexpr bool V = decltype(vec)::value;
        const uint32_t ln = fresh(lane);
#pragma unroll
        for (int f = 0; f < PF; ++f) {
            const uint32_t q = wave + f * nwaves;
            const uint32_t st = q % SUB, c = (q / SUB) * 64 + ln;
            slot_from_raw<V>(pre[f]);
            if (q < nchunks && c < n) {
                lds_write_slot<RT>(buf + ((size_t)c * SP + st) * RT, pre[f]);
                if (a.copy_b_floats)  // second copy: slots rotated inside every run of 16 coordinates
                    lds_write_slot<RT>(buf + a.copy_b_floats + ((size_t)((c & ~15u) | ((c + (c >> 4)) & 15u)) * SP + st) * RT,
                                       pre[f]);
            }
        }
    };
    const uint32_t ld_off = (lane & 3) * n + (lane & ~3u);
    auto fetch_full = [&](uint64_t row0) {
#pragma unroll
        for (int f = 0; f < PF; ++f) {
            const uint32_t q = wave + f * nwaves;
            const float *src = a.data + (row0 + (q % SUB) * RT) * n + (q / SUB) * 64;  // uniform
            const float4 v = *reinterpret_cast<const float4 *>(src + ld_off);
            pre[f][0] = v.x; pre[f][1] = v.y; pre[f][2] = v.z; pre[f][3] = v.w;
        }
    };
    auto stash_full = [&](float *buf) {
#pragma unroll
        for (int f = 0; f < PF; ++f) {
            const uint32_t q = wave + f * nwaves;
            const uint32_t st = q % SUB, c = (q / SUB) * 64 + lane;
            slot_from_raw<true>(pre[f]);
            lds_write_slot<RT>(buf + ((size_t)c * SP + st) * RT, pre[f]);
            if (a.copy_b_floats)
                lds_write_slot<RT>(buf + a.copy_b_floats + ((size_t)((c & ~15u) | ((c + (c >> 4)) & 15u)) * SP + st) * RT,
                                   pre[f]);
        }
    };
    // the vectorised and the word-by-word variants are separate straight-line code
    auto fetch = [&](uint64_t row0) {
        if constexpr (REGULAR) fetch_full(row0);
        else if (vec4) fetch_as(row0, std::true_type{});
        else fetch_as(row0, std::false_type{});
    };
    auto stash = [&](float *buf) {
        if constexpr (REGULAR) stash_full(buf);
        else if (vec4) stash_as(buf, std::true_type{});
        else stash_as(buf, std::false_type{});
    };
    const uint32_t full_off = EP == (int)Epilogue::Signs ? (lane * ((a.k + 63) / 64) + (j >> 6)) * 8
                                                        : ((lane & 3) * a.k + (j & ~3u)) * 4;

    uint64_t t = blockIdx.x;
    if (t < ntiles) {
        fetch(t * kTileRows);
        stash(tile);
    }
    __syncthreads();
    uint32_t cur = 0;
    for (; t < ntiles; t += gridDim.x) {
        const uint64_t row0 = t * kTileRows;
        const uint64_t t_next = t + gridDim.x;
        if (t_next < ntiles) fetch(t_next * kTileRows);

        const char *base = reinterpret_cast<const char *>(tile + cur * buf_floats);
        float acc[SUB][RT];
#pragma unroll
        for (int st = 0; st < SUB; ++st)
#pragma unroll
            for (int r = 0; r < RT; ++r) acc[st][r] = 0.f;

        // the packed offsets pass through an empty asm every tile, or the compiler would unpack
        // them once, outside the tile loop, into twice the registers
#pragma unroll
        for (int h = 0; h < kList / 2; ++h) asm volatile("" : "+v"(po[h]));
        auto read_sample = [&](int i, float4 (&x)[SUB]) {
            const uint32_t off = (i & 1) ? po[i / 2] >> 16 : po[i / 2] & 0xffffu;
#pragma unroll
            for (int st = 0; st < SUB; ++st) x[st] = *reinterpret_cast<const float4 *>(base + off + st * 16);
        };
        float4 x[kDepth][SUB];
#pragma unroll
        for (int i = 0; i < kDepth - 1; ++i) read_sample(i, x[i]);
#pragma unroll
        for (int i = 0; i < kList; ++i) {
            // region: the reads of sample i + kDepth - 1 may interleave with the FMAs of sample i,
            // nothing else
            __builtin_amdgcn_sched_barrier(0);
            if (i + kDepth - 1 < kList) read_sample(i + kDepth - 1, x[(i + kDepth - 1) % kDepth]);
#pragma unroll
            for (int st = 0; st < SUB; ++st) {
                const float4 &v = x[i % kDepth][st];
                acc[st][0] = fmaf(cf[i], v.x, acc[st][0]);
                acc[st][1] = fmaf(cf[i], v.y, acc[st][1]);
                acc[st][2] = fmaf(cf[i], v.z, acc[st][2]);
                acc[st][3] = fmaf(cf[i], v.w, acc[st][3]);
                pin(acc[st]);
            }
        }
        __builtin_amdgcn_sched_barrier(0);
        // The next tile goes to LDS before this tile's results are stored: the counter of
        // outstanding memory operations is in order, so a wait for the prefetched registers that
        // came after the stores would also wait for them, a trip to HBM per tile.
        if (t_next < ntiles) stash(tile + (cur ^ 1) * buf_floats);
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (EP == (int)Epilogue::Keys) {
            // the key fold needs a few registers more than the other epilogues: the offset is read
            // again every tile (an L2 hit, issued after the wait for the prefetched tile) rather
            // than held across the gather
            const uint32_t jt = fresh(j);
            finish<RT, SUB, EP, REGULAR>(a, row0, jt, acc, a.off[jt], key_pow, full_off);
        } else {
            finish<RT, SUB, EP, REGULAR>(a, row0, fresh(j), acc, b, key_pow, full_off);
        }
        __syncthreads();  // next buffer complete; everyone is done with the current one
        cur ^= 1;
    }
}

// Chunked kernel for large n (or long lists at large n): the tile holds 4*SUB vectors times a
// range of `chunk` coordinates (one workgroup per CU with nearly all of its LDS), so that enough vectors share one pass over the lists to keep
// list traffic (L2 -> registers) well below the LDS gather traffic.  Every function's samples
// are bucketed by coordinate range on the host; the 64 lists of a wave for one range are
// padded to a common length (wave-uniform trip count) and bank-scheduled like the flat lists.
// Accumulators persist across the ranges of a tile.
template <int SUB, int FPT, int EP>
__global__ __launch_bounds__(1024) void sampled_chunked_kernel(const SampledArgs a) {
    constexpr int RT = 4;
    constexpr int kStep = 8;   // list entries fetched at a time; list lengths are multiples of it
    constexpr int kPre = kChunkPre;  // 64-coordinate pieces of the next chunk a wave holds in registers
    extern __shared__ __align__(16) float tile[];  // [chunk + classes][SP][RT]
    constexpr uint32_t SP = SUB == 1 ? 1 : SUB + 1;
    constexpr uint32_t kTileRows = RT * SUB;
    const uint32_t n = a.n;
    // a lane owns FPT functions, blockDim.x apart: j0 + f * blockDim.x
    const uint32_t j0 = blockIdx.y * blockDim.x * FPT + threadIdx.x;
    const uint64_t ntiles = (a.N + kTileRows - 1) / kTileRows;
    float b[FPT];
    uint64_t key_pow[FPT];
#pragma unroll
    for (int f = 0; f < FPT; ++f) {
        const uint32_t j = j0 + f * blockDim.x;  // < kpad
        b[f] = a.off[j];
        key_pow[f] = 1;
        if (EP == (int)Epilogue::Keys) {
            uint32_t t = j % a.g;
            if (RT == 4 && a.g >= 4) t |= 3;  // the transposed fold multiplies by the power of the quad's last function
            for (uint32_t e = 0; e + 1 + t < a.g; ++e) key_pow[f] *= kKeyMultiplier;
        }
    }

    for (uint32_t e = threadIdx.x; e < a.classes * SP * RT; e += blockDim.x)
        tile[(size_t)a.chunk * SP * RT + e] = 0.f;

    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint32_t lane = threadIdx.x & 63;
    const uint32_t nwaves = blockDim.x >> 6;
    const uint32_t wave_global = __builtin_amdgcn_readfirstlane(j0 >> 6);
    const uint32_t pieces = SUB * ((a.chunk + 63) / 64);  // 64-coordinate pieces of one chunk (<= kPre * nwaves)
    const bool vec4 = (n & 3) == 0;
    const char *base = reinterpret_cast<const char *>(tile);

    // The next chunk (of this tile, or the first of the next tile) travels HBM -> registers
    // while the current one is gathered from LDS, and is written to LDS between two barriers.
    float pre[kPre][RT];
    auto fetch_as = [&](uint64_t row0, uint32_t q, auto vec) {
        constexpr bool V = decltype(vec)::value;
        const uint32_t c0 = q * a.chunk;
        const float *rows = a.data + row0 * n;
        const uint32_t rows_valid = (uint32_t)min((uint64_t)kTileRows, a.N - row0);
        const uint32_t end = c0 + a.chunk < n ? c0 + a.chunk : n;  // chunk % 16 == 0
        const uint32_t ln = fresh(lane);
#pragma unroll
        for (int f = 0; f < kPre; ++f) {
            const uint32_t pc = wave + f * nwaves;
            load_raw<V>(rows, rows_valid, n, (pc % SUB) * RT, c0 + (pc / SUB) * 64, pc < pieces ? end : 0, ln,
                        pre[f]);
        }
    };
    auto stash_as = [&](auto vec) {
        constexpr bool V = decltype(vec)::value;
        const uint32_t ln = fresh(lane);
#pragma unroll
        for (int f = 0; f < kPre; ++f) {
            const uint32_t pc = wave + f * nwaves;
            const uint32_t st = pc % SUB, cc = (pc / SUB) * 64 + ln;
            slot_from_raw<V>(pre[f]);
            if (pc < pieces && cc < a.chunk) lds_write_slot<RT>(tile + ((size_t)cc * SP + st) * RT, pre[f]);
        }
    };
    auto fetch = [&](uint64_t row0, uint32_t q) {
        if (vec4) fetch_as(row0, q, std::true_type{});
        else fetch_as(row0, q, std::false_type{});
    };
    auto stash = [&]() {
        if (vec4) stash_as(std::true_type{});
        else stash_as(std::false_type{});
    };

    uint64_t t = blockIdx.x;
    if (t >= ntiles) return;
    fetch(t * kTileRows, 0);
    stash();
    __syncthreads();
    for (; t < ntiles; t += gridDim.x) {
        const uint64_t row0 = t * kTileRows;
        float acc[FPT][SUB][RT];
#pragma unroll
        for (int f = 0; f < FPT; ++f)
#pragma unroll
            for (int st = 0; st < SUB; ++st)
#pragma unroll
                for (int r = 0; r < RT; ++r) acc[f][st][r] = 0.f;

        for (uint32_t q = 0; q < a.nchunks; ++q) {
            const bool last = q + 1 == a.nchunks;
            const uint64_t t_next = t + gridDim.x;
            const bool more = !last || t_next < ntiles;
            if (more) fetch((last ? t_next : t) * kTileRows, last ? 0 : q + 1);

#pragma unroll
            for (int f = 0; f < FPT; ++f) {
                const uint2 info = a.chunk_info[(size_t)(wave_global + f * nwaves) * a.nchunks + q];
                const Sample *list = a.tab + info.x + lane;
                for (uint32_t s0 = 0; s0 < info.y; s0 += kStep) {
                    Sample e[kStep];
#pragma unroll
                    for (int i = 0; i < kStep; ++i) e[i] = list[(size_t)(s0 + i) * 64];
#pragma unroll
                    for (int i = 0; i < kStep; ++i) {
                        __builtin_amdgcn_sched_barrier(0);
                        float4 x[SUB];
#pragma unroll
                        for (int st = 0; st < SUB; ++st)
                            x[st] = *reinterpret_cast<const float4 *>(base + e[i].lds_byte_offset + st * 16);
#pragma unroll
                        for (int st = 0; st < SUB; ++st) {
                            acc[f][st][0] = fmaf(e[i].coef, x[st].x, acc[f][st][0]);
                            acc[f][st][1] = fmaf(e[i].coef, x[st].y, acc[f][st][1]);
                            acc[f][st][2] = fmaf(e[i].coef, x[st].z, acc[f][st][2]);
                            acc[f][st][3] = fmaf(e[i].coef, x[st].w, acc[f][st][3]);
                            pin(acc[f][st]);
                        }
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
                if (last) finish<RT, SUB, EP>(a, row0, fresh(j0) + f * blockDim.x, acc[f], b[f], key_pow[f]);
            }
            __syncthreads();  // every lane is done reading this chunk
            if (more) stash();
            __syncthreads();
        }
    }
}

template <typename Kernel>
int launch_kernel(Kernel fn, uint32_t lds_bytes, const SampledArgs &args, dim3 grid, dim3 block,
                  hipStream_t stream) {
    if (ensure_lds_limit(reinterpret_cast<const void *>(fn), lds_bytes) != LSH_OK) return LSH_ERR_HIP;
    hipLaunchKernelGGL(fn, grid, block, lds_bytes, stream, args);
    return hipGetLastError() == hipSuccess ? LSH_OK : LSH_ERR_HIP;
}

}  // namespace

// hipFuncSetAttribute costs about a millisecond of host time: raise a kernel's dynamic LDS
// limit once (per kernel and size), not per launch.
int ensure_lds_limit(const void *fn, uint32_t lds_bytes) {
    static std::mutex mu;
    static std::unordered_map<const void *, uint32_t> granted;
    std::lock_guard<std::mutex> lock(mu);
    auto it = granted.find(fn);
    if (it != granted.end() && it->second >= lds_bytes) return LSH_OK;
    if (hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes) != hipSuccess)
        return LSH_ERR_HIP;
    granted[fn] = lds_bytes;
    return LSH_OK;
}

uint32_t sampled_chunk() { return kChunk; }

// Tile shape by dimension: as many vectors as fit the LDS budget.
SampledPlan plan_sampled(uint32_t n, uint32_t k, uint32_t m) {
    SampledPlan pl;
    auto fits = [&](uint32_t rt, uint32_t sub, uint32_t classes) {
        const uint64_t sp = sub == 1 ? 1 : sub + 1;
        const uint64_t bytes = (uint64_t)(n + classes) * sp * rt * 4;
        if (bytes > kLdsBudget) return false;
        pl.rt = rt; pl.sub = sub; pl.sp = (uint32_t)sp; pl.classes = classes;
        pl.group = rt == 4 ? 16 : 32;
        pl.lds_bytes = (uint32_t)bytes;
        return true;
    };
    // 16-byte reads: 16 lanes per pass over 16 classes; 8-byte: 32 lanes over 32; 4-byte:
    // 32 lanes over 64 banks
    if (!(fits(4, 8, 16) || fits(4, 4, 16) || fits(4, 2, 16) || fits(4, 1, 16) || fits(2, 1, 32) ||
          fits(1, 1, 64)))
        return pl;  // unsupported: one vector does not fit in LDS
    pl.m_pad = (m + kChunk - 1) / kChunk * kChunk;
    const uint32_t k64 = (k + 63) / 64 * 64;
    // Register-list kernel: lists of at most two chunks, 16-byte slots, two tile buffers in LDS.
    // The kernel is bound by vector-ALU issue (a 64-lane FMA takes a SIMD four cycles), so the
    // tile is the largest whose accumulators and in-flight reads still fit the 128 registers of
    // a lane (16 vectors): the per-sample address arithmetic and the per-tile load and barrier
    // code are then shared by the most FMAs.  Only while a tile stays small (at most 2 prefetch
    // pieces per wave): with large n one tile's gather is shorter than the latency of the next
    // tile's loads, and the chunked kernel, which shares a bigger tile among more functions, wins.
    pl.reg_table = false;
    if (pl.m_pad <= 2u * kChunk && pl.rt == 4) {
        const uint32_t block = k64 >= 512 ? 512 : k64;
        for (uint32_t sub : {4u, 2u, 1u}) {
            const uint64_t sp = sub == 1 ? 1 : sub + 1;
            const uint64_t bytes = (uint64_t)(n + 16) * sp * 16;
            const uint32_t chunks = sub * ((n + 63) / 64);
            const uint32_t pf = (chunks + block / 64 - 1) / (block / 64);
            if (2 * bytes > kLdsBudget || pf > 2) continue;
            fits(4, sub, 16);
            pl.reg_table = true;
            pl.prefetch = pf <= 1 ? 1 : 2;
            // a second, class-rotated copy of the tile (see schedule.cpp) where it costs no
            // occupancy and LDS offsets still fit the kernel's 16 bits
            const uint64_t bytes2 = bytes + (uint64_t)((n + 15) / 16 * 16) * sp * 16;
            const uint32_t lanes = pl.m_pad == kChunk ? 1024 : 512;
            const uint32_t wgs = lanes / block < 2 ? lanes / block : 2;
            if (bytes2 <= 65536 && 2 * bytes2 * wgs <= kLdsBudget) {
                pl.copies = 2;
                pl.lds_bytes = (uint32_t)bytes2;
            }
            break;
        }
    }
    // Chunked kernel: when a full-dimension tile would hold fewer than 16 vectors and the lists
    // do not stay in registers.  16 vectors x `chunk` coordinates, two workgroups per CU.
    pl.chunked = false;
    if (!pl.reg_table && (pl.rt != 4 || pl.sub < 4) && k64 >= 512) {  // enough waves to prefetch a chunk
        const uint32_t slot = 5 * 16;  // SUB = 4: 5 slots of 16 bytes per coordinate
        const uint32_t block = k64 >= 1024 ? 1024 : k64;
        // the chunk must fit in LDS and its pieces in the waves' prefetch registers (kChunkPre pieces
        // of 64 coordinates x 4 sub-tiles per wave)
        uint32_t cmax = (kLdsBudget / slot - 16) / 16 * 16;
        const uint32_t by_regs = (uint32_t)kChunkPre * (block / 64) / 4 * 64;
        if (cmax > by_regs) cmax = by_regs;
        pl.nchunks = (n + cmax - 1) / cmax;
        pl.chunk = ((n + pl.nchunks - 1) / pl.nchunks + 15) / 16 * 16;
        pl.nchunks = (n + pl.chunk - 1) / pl.chunk;
        pl.rt = 4; pl.sub = 4; pl.sp = 5; pl.classes = 16; pl.group = 16;
        pl.lds_bytes = (pl.chunk + 16) * slot;
        pl.chunked = true;
        // with more than 1024 functions a lane takes two (1024 apart), so that a chunk is
        // loaded once for 2048 functions
        pl.fpt = k64 > 1024 ? 2 : 1;
    }
    const uint32_t max_block = pl.reg_table ? 512 : 1024;
    pl.block = k64 >= max_block ? max_block : k64;
    const uint32_t per_wg = pl.block * (pl.chunked ? pl.fpt : 1);
    pl.kblocks = (k64 + per_wg - 1) / per_wg;
    pl.kpad = per_wg * pl.kblocks;
    pl.supported = true;
    return pl;
}

int launch_sampled(const lsh_params *p, Epilogue ep, const float *d_data, uint64_t N, void *d_out,
                   uint32_t L, void *stream) {
    const SampledPlan &pl = p->plan;
    if (!pl.supported) return LSH_ERR_UNSUPPORTED;
    SampledArgs a;
    a.data = d_data;
    a.N = N;
    a.n = p->n;
    a.k = p->k;
    a.m_pad = pl.m_pad;
    a.kpad = pl.kpad;
    a.classes = pl.classes;
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
    a.buf_floats = pl.lds_bytes / 4;
    a.copy_b_floats = pl.copies == 2 ? (p->n + pl.classes) * pl.sp * pl.rt : 0;
    a.chunk = pl.chunk;
    a.nchunks = pl.nchunks;
    a.chunk_info = static_cast<const uint2 *>(p->d_chunk_info);
    const uint64_t tile_rows = (uint64_t)pl.rt * pl.sub;
    const uint64_t ntiles = (N + tile_rows - 1) / tile_rows;
    // persistent workgroups: as many per CU as LDS and waves allow (at most 2048 lanes), count
    // a multiple of 8 so that the kblocks workgroups sharing a vector tile land on one XCD
    const uint32_t lds_bytes = pl.reg_table ? 2 * pl.lds_bytes : pl.lds_bytes;
    uint32_t per_cu = kLdsBudget / lds_bytes;
    // register-list kernel: 4 waves per SIMD (128 VGPRs per lane; 2 and 256 with two list
    // chunks), else 8
    const uint32_t by_lanes =
        (pl.reg_table ? (pl.m_pad == (uint32_t)kChunk ? 1024 : 512) : 2048) / pl.block;
    if (per_cu > by_lanes) per_cu = by_lanes;
    if (per_cu < 1) per_cu = 1;
    uint64_t gx = (uint64_t)p->num_cus * per_cu / pl.kblocks;
    gx = gx < 8 ? 8 : gx / 8 * 8;
    if (gx > ntiles) gx = ntiles;
    dim3 grid((uint32_t)gx, pl.kblocks), block(pl.block);
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    // one instantiation per epilogue: a run-time switch inside the kernels costs registers
    // (spills) in the gather loop
#define LSH_EP_CASES(CALL) \
    switch (ep) { \
        case Epilogue::Ids: CALL((int)Epilogue::Ids) break; \
        case Epilogue::Proj: CALL((int)Epilogue::Proj) break; \
        case Epilogue::Signs: CALL((int)Epilogue::Signs) break; \
        default: CALL((int)Epilogue::Keys) break; \
    }
    if (pl.reg_table) {
        // whole tiles of a regular shape go through the predicate-free instantiation, the
        // vectors after them (fewer than one tile) through the general one
        const bool regular = pl.sub == 4 && (p->n & 63) == 0 && pl.sub * (p->n / 64) == pl.prefetch * (pl.block / 64) &&
                             (ep == Epilogue::Signs || ep == Epilogue::Keys || (p->k & 3) == 0);
        const uint64_t n_whole = regular ? N / tile_rows * tile_rows : 0;
        SampledArgs tail = a;
        tail.data = d_data + n_whole * p->n;
        tail.N = N - n_whole;
        const uint64_t out_bytes_per_vector = ep == Epilogue::Signs  ? 8ull * ((p->k + 63) / 64)
                                              : ep == Epilogue::Keys ? 8ull * L
                                                                     : 4ull * p->k;
        tail.out = static_cast<char *>(d_out) + n_whole * out_bytes_per_vector;
        a.N = n_whole;
        const uint64_t tail_tiles = (tail.N + tile_rows - 1) / tile_rows;
        dim3 tail_grid((uint32_t)(tail_tiles < gx ? tail_tiles : gx), pl.kblocks);
        if (n_whole && grid.x > n_whole / tile_rows) grid.x = (uint32_t)(n_whole / tile_rows);
#define LSH_REG_LAUNCH(SUB_, PF_, MCH_, EP_, REG_, ARGS_, GRID_) \
    launch_kernel(&sampled_reg_kernel<SUB_, PF_, MCH_, EP_, REG_>, lds_bytes, ARGS_, GRID_, block, s)
#define LSH_REG_CASE(SUB_, PF_, EP_) \
    if (pl.sub == SUB_ && pl.prefetch == PF_) { \
        int rc = LSH_OK; \
        if constexpr (SUB_ == 4) { \
            if (n_whole) \
                rc = pl.m_pad == (uint32_t)kChunk ? LSH_REG_LAUNCH(SUB_, PF_, 1, EP_, true, a, grid) \
                                                  : LSH_REG_LAUNCH(SUB_, PF_, 2, EP_, true, a, grid); \
        } \
        if (rc == LSH_OK && tail.N) \
            rc = pl.m_pad == (uint32_t)kChunk ? LSH_REG_LAUNCH(SUB_, PF_, 1, EP_, false, tail, tail_grid) \
                                              : LSH_REG_LAUNCH(SUB_, PF_, 2, EP_, false, tail, tail_grid); \
        return rc; \
    }
#define LSH_REG_ALL(EP_) \
    LSH_REG_CASE(4, 1, EP_) LSH_REG_CASE(4, 2, EP_) LSH_REG_CASE(2, 1, EP_) LSH_REG_CASE(2, 2, EP_) \
    LSH_REG_CASE(1, 1, EP_) LSH_REG_CASE(1, 2, EP_)
        LSH_EP_CASES(LSH_REG_ALL)
#undef LSH_REG_ALL
#undef LSH_REG_CASE
#undef LSH_REG_LAUNCH
        return LSH_ERR_UNSUPPORTED;
    }
#define LSH_GEN_ALL(EP_) \
    if (pl.chunked && pl.fpt == 2) return launch_kernel(&sampled_chunked_kernel<4, 2, EP_>, lds_bytes, a, grid, block, s); \
    if (pl.chunked) return launch_kernel(&sampled_chunked_kernel<4, 1, EP_>, lds_bytes, a, grid, block, s); \
    if (pl.rt == 4 && pl.sub == 8) return launch_kernel(&sampled_kernel<4, 8, EP_>, lds_bytes, a, grid, block, s); \
    if (pl.rt == 4 && pl.sub == 4) return launch_kernel(&sampled_kernel<4, 4, EP_>, lds_bytes, a, grid, block, s); \
    if (pl.rt == 4 && pl.sub == 2) return launch_kernel(&sampled_kernel<4, 2, EP_>, lds_bytes, a, grid, block, s); \
    if (pl.rt == 4) return launch_kernel(&sampled_kernel<4, 1, EP_>, lds_bytes, a, grid, block, s); \
    if (pl.rt == 2) return launch_kernel(&sampled_kernel<2, 1, EP_>, lds_bytes, a, grid, block, s); \
    return launch_kernel(&sampled_kernel<1, 1, EP_>, lds_bytes, a, grid, block, s);
    LSH_EP_CASES(LSH_GEN_ALL)
#undef LSH_GEN_ALL
#undef LSH_EP_CASES
    return LSH_ERR_UNSUPPORTED;
}

}  // namespace lsh
