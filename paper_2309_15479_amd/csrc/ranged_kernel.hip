// Sampled-projection kernel (FastLSH, Sec. 3.1, Eq. 5) for long lists and large dimensions on
// gfx950: the 960-, 4096- and 16384-dimensional shapes.
//
//   p_j(v) = sum_{i<m} a~_j[i] * v[S_j[i]],   h_j(v) = floor((p_j(v) + b~_j) / w)
//
// Mapping as in sampled_kernel.hip: one lane = one hash function, a tile = 16 vectors kept in LDS
// as 16-byte slots (one coordinate of four vectors), one 16-byte LDS read feeds four
// multiply-adds.  What differs:
//
//  * Coordinate ranges.  A tile is 16 vectors x a range of 1024 coordinates (64 KB), laid out
//    [sub-tile of 4 vectors][coordinate], so the four reads of a sample differ only in their
//    immediate offset and a slot's bank class is its coordinate modulo 16 without any padding.
//    LDS holds two such buffers.  Every function's samples are bucketed by range on the host;
//    accumulators persist across the ranges of a tile.
//
//  * Loader waves.  A workgroup is 8 gathering waves plus 4 loading waves.  While the gatherers
//    walk their lists over buffer s, the loaders fetch the next (tile, range) from HBM and write
//    it, transposed, to buffer s ^ 1; one barrier per step.  The two kinds of wave have their
//    own counters of outstanding memory operations, so a gatherer's wait for list entries never
//    waits for tile data.
//
//  * Packed lists.  The kernel is bound by vector-ALU issue (sixteen multiply-adds per list
//    entry), so everything else an entry costs is kept small: a lane's list is stored in quads
//    of entries, 16 bytes of coefficients and 8 bytes holding four 16-bit LDS byte offsets, which
//    one add with a sub-word operand turns into the entry's address (one instruction per entry;
//    a vector memory instruction per 2.7 entries).  Lists are cut into blocks of three quads; the
//    blocks of one gathering wave form one contiguous stream in the order the wave consumes
//    them (range after range, and within a range function after function), so the next block
//    is always prefetched, across list boundaries and around the end of the stream to the next
//    tile.
//
//  * A lane owns up to four functions (sets of 64 functions, 8 sets apart), so that a
//    workgroup covers up to 2048 functions per tile load.
//
// Padding entries (a wave's 64 lists of one range are padded to a common length, a multiple of
// four) carry coefficient 0 and read one of the first 16 slots of the range, whichever bank
// class the schedule wants; the loaders write zeros to the slots beyond the last coordinate,
// so such an entry always multiplies a finite value of the same vector by zero.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstring>
#include <vector>
#include <type_traits>

#include "sampled_common.h"

namespace lsh {
namespace {

constexpr int kCW = (int)kRangeComputeWaves;  // gathering waves
constexpr int kLW = 4;                        // loading waves: wave kCW + s loads sub-tile s
constexpr int kThreads = (kCW + kLW) * 64;
constexpr int kC = (int)kRangeCoords;
constexpr int kSubBytes = kC * 16;            // one sub-tile of one buffer
constexpr int kBufBytes = 4 * kSubBytes;      // 64 KB
constexpr int kU = (int)kRangeBlockQuads;     // quads of entries per lane in a list block
constexpr int kPieces = kC / 64;              // 64-coordinate pieces of a sub-tile

typedef float floatx4 __attribute__((ext_vector_type(4)));

// one block of a lane's list: kU quads of entries
struct ListBlock {
    uint4 coef[kU];  // four coefficients (float bits)
    uint2 off[kU];   // four 16-bit LDS byte offsets of the entries' slots in sub-tile 0
};

// the four 16-byte slots of one entry: the same coordinate in the four sub-tiles
__device__ __forceinline__ void read_entry(const char *p, float4 (&x)[4]) {
#pragma unroll
    for (int st = 0; st < 4; ++st) x[st] = *reinterpret_cast<const float4 *>(p + st * kSubBytes);
}

__device__ __forceinline__ void fma_entry(float c, const float4 (&x)[4], float (&acc)[4][4]) {
#pragma unroll
    for (int st = 0; st < 4; ++st) {
        acc[st][0] = fmaf(c, x[st].x, acc[st][0]);
        acc[st][1] = fmaf(c, x[st].y, acc[st][1]);
        acc[st][2] = fmaf(c, x[st].z, acc[st][2]);
        acc[st][3] = fmaf(c, x[st].w, acc[st][3]);
        pin(acc[st]);
    }
}

// Four entries of a lane's list against the 16 vectors of the tile; the LDS reads of an entry go
// out before the multiply-adds of the entry before it.  (Deeper read-ahead, tried with a ring of
// three register sets and with all reads of a group up front, changes nothing but the register
// count: the vector ALU is busy in 96 % of the cycles.)
__device__ __forceinline__ void gather_quad(const char *buf, const uint4 c, const uint2 o, float (&acc)[4][4]) {
    float4 x[2][4];
    __builtin_amdgcn_sched_barrier(0);
    read_entry(buf + (o.x & 0xFFFFu), x[0]);
    __builtin_amdgcn_sched_barrier(0);
    read_entry(buf + (o.x >> 16), x[1]);
    fma_entry(__uint_as_float(c.x), x[0], acc);
    __builtin_amdgcn_sched_barrier(0);
    read_entry(buf + (o.y & 0xFFFFu), x[0]);
    fma_entry(__uint_as_float(c.y), x[1], acc);
    __builtin_amdgcn_sched_barrier(0);
    read_entry(buf + (o.y >> 16), x[1]);
    fma_entry(__uint_as_float(c.z), x[0], acc);
    __builtin_amdgcn_sched_barrier(0);
    fma_entry(__uint_as_float(c.w), x[1], acc);
    __builtin_amdgcn_sched_barrier(0);
}

// the first `quads` (1..kU) quads of a block
__device__ __forceinline__ void gather_block(const char *buf, const ListBlock &blk, uint32_t quads,
                                             float (&acc)[4][4]) {
#pragma unroll
    for (int t = 0; t < kU; ++t)
        if ((uint32_t)t < quads) gather_quad(buf, blk.coef[t], blk.off[t], acc);  // uniform
}

template <int FPT, int EP>
__global__ __launch_bounds__(kThreads) void sampled_ranged_kernel(const SampledArgs a,
                                                                  const uint32_t *__restrict__ list_len,
                                                                  const uint2 *__restrict__ streams) {
    extern __shared__ __align__(16) char lds[];  // 2 buffers x [4 sub-tiles][1024 slots] x 16 bytes
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint32_t lane = threadIdx.x & 63;
    const uint32_t n = a.n, R = a.nchunks;
    const uint64_t ntiles = (a.N + 15) / 16;
    const uint64_t first_tile = blockIdx.x;  // the host launches at most ntiles workgroups along x

    if (wave >= (uint32_t)kCW) {
        // ---- loading waves: wave kCW + s fetches sub-tile s (vectors 4s .. 4s + 3) of every step
        const uint32_t st = wave - kCW;
        const bool vec4 = (n & 3) == 0;
        float pre[kPieces][4];
        char *mine = lds + st * kSubBytes + lane * 16;
        auto fetch = [&](uint64_t tile, uint32_t r, auto vec) __attribute__((always_inline)) {
            constexpr bool V = decltype(vec)::value;
            const uint64_t row0 = tile * 16;
            const float *rows = a.data + row0 * n;
            const uint32_t rows_valid = (uint32_t)min((uint64_t)16, a.N - row0);
            const uint32_t c0 = r * kC;
            const uint32_t end = c0 + kC < n ? c0 + kC : n;
#pragma unroll
            for (int f = 0; f < kPieces; ++f)
                load_raw<V>(rows, rows_valid, n, st * 4, c0 + f * 64, end, lane, pre[f]);
        };
        auto stash = [&](uint32_t b, uint32_t r, auto vec) __attribute__((always_inline)) {
            constexpr bool V = decltype(vec)::value;
            const uint32_t len = n - r * kC;  // coordinates of this range (>= kC: all of them)
#pragma unroll
            for (int f = 0; f < kPieces; ++f) {
                slot_from_raw<V>(pre[f]);
                const bool inside = (uint32_t)(f * 64) + lane < len;
                floatx4 v = {inside ? pre[f][0] : 0.f, inside ? pre[f][1] : 0.f, inside ? pre[f][2] : 0.f,
                             inside ? pre[f][3] : 0.f};
                *reinterpret_cast<floatx4 *>(mine + b * kBufBytes + f * 64 * 16) = v;
            }
        };
        // one iteration per step plus one: iteration i fetches step i (the first one fills buffer
        // 0 before anybody reads), then meets the gathering waves at the barrier that ends step i - 1
        uint64_t t_next = first_tile;
        uint32_t r_next = 0, b = 1;
        for (;;) {
            const bool more = t_next < ntiles;
            if (more) {
                if (vec4) {
                    fetch(t_next, r_next, std::true_type{});
                    stash(b ^ 1, r_next, std::true_type{});
                } else {
                    fetch(t_next, r_next, std::false_type{});
                    stash(b ^ 1, r_next, std::false_type{});
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

    // ---- gathering waves
    const uint32_t stream_id = blockIdx.y * kCW + wave;
    const uint2 si = streams[stream_id];  // {first block, blocks}
    // a block in memory: kU x 64 lanes x 16 bytes of coefficients, then kU x 64 x 8 bytes of offsets
    constexpr uint32_t kBlockWords = kU * 64 * 6;
    const uint32_t *sbase = reinterpret_cast<const uint32_t *>(a.triples) + (size_t)si.x * kBlockWords;
    const uint32_t sblocks = si.y;
    const uint32_t *len_base = list_len + (size_t)stream_id * R * FPT;
    // list registers: the block in use and the one after it (always on its way)
    ListBlock P, Q;
    uint32_t next_block = 0;
    auto load_block = [&](ListBlock &blk) __attribute__((always_inline)) {
        const uint32_t *src = sbase + (size_t)next_block * kBlockWords;
#pragma unroll
        for (int i = 0; i < kU; ++i) {
            blk.coef[i] = *reinterpret_cast<const uint4 *>(src + (i * 64 + lane) * 4);
            blk.off[i] = *reinterpret_cast<const uint2 *>(src + kU * 64 * 4 + (i * 64 + lane) * 2);
        }
        next_block = next_block + 1 == sblocks ? 0 : next_block + 1;
    };
    if (sblocks) load_block(P);

    // function of this lane in set f: sets are kCW apart
    const uint32_t j0 = (blockIdx.y * kCW * FPT + wave) * 64 + lane;
    float bias[FPT];
    uint64_t key_pow[FPT];
#pragma unroll
    for (int f = 0; f < FPT; ++f) {
        const uint32_t j = j0 + f * kCW * 64;  // < kpad
        bias[f] = a.off[j];
        key_pow[f] = 1;
        if (EP == (int)Epilogue::Keys || EP == (int)Epilogue::IdsKeys) {
            uint32_t t = j % a.g;
            if (a.g >= 4) t |= 3;  // the transposed fold multiplies by the power of the quad's last function
            for (uint32_t e = 0; e + 1 + t < a.g; ++e) key_pow[f] *= kKeyMultiplier;
        }
    }

    __syncthreads();  // first buffer written
    uint32_t b = 0;
    for (uint64_t t = first_tile; t < ntiles; t += gridDim.x) {
        float acc[FPT][4][4];
#pragma unroll
        for (int f = 0; f < FPT; ++f)
#pragma unroll
            for (int st = 0; st < 4; ++st)
#pragma unroll
                for (int r = 0; r < 4; ++r) acc[f][st][r] = 0.f;

        for (uint32_t r = 0; r < R; ++r) {
            const char *buf = lds + b * kBufBytes;
#pragma unroll
            for (int f = 0; f < FPT; ++f) {
                const uint32_t quads = len_base[r * FPT + f] / 4;  // list lengths are multiples of four
                // blocks two at a time, the registers of one being refilled while the other is used
                for (uint32_t done = 0; done < quads; done += 2 * kU) {
                    load_block(Q);
                    const uint32_t left = quads - done;
                    gather_block(buf, P, left < (uint32_t)kU ? left : kU, acc[f]);
                    if (left > (uint32_t)kU) {
                        load_block(P);
                        gather_block(buf, Q, left - kU < (uint32_t)kU ? left - kU : kU, acc[f]);
                    } else {
                        P = Q;
                    }
                }
            }
            if (r + 1 == R) {
#pragma unroll
                for (int f = 0; f < FPT; ++f)
                    finish<4, 4, EP>(a, t * 16, fresh(j0) + f * kCW * 64, acc[f], bias[f], key_pow[f]);
            }
            __syncthreads();  // the other buffer is complete, everyone is done with this one
            b ^= 1;
        }
    }
}

template <typename Kernel>
int launch(Kernel fn, const SampledArgs &args, dim3 grid, hipStream_t stream) {
    if (ensure_lds_limit(reinterpret_cast<const void *>(fn), 2 * kBufBytes) != LSH_OK) return LSH_ERR_HIP;
    hipLaunchKernelGGL(fn, grid, dim3(kThreads), 2 * kBufBytes, stream, args, args.list_len, args.stream);
    return hipGetLastError() == hipSuccess ? LSH_OK : LSH_ERR_HIP;
}

}  // namespace

// Host tables of the ranged kernel (stream_info: {first block, blocks} per gathering wave).
void build_ranged_tables(const lsh_params *p, std::vector<uint32_t> &words, std::vector<uint32_t> &list_len,
                         std::vector<uint32_t> &stream_info) {
    // one stream of list blocks per gathering wave, in the order the wave consumes them:
    // range after range, within a range the wave's functions-per-lane sets one after the
    // other.  A block is kRangeBlockQuads quads of entries x 64 lanes: 16 bytes of
    // coefficients per quad and lane, then 8 bytes of 16-bit LDS byte offsets
    // (16 x (coordinate minus the range's first)).
    const SampledPlan &pl = p->plan;
    const uint32_t R = pl.nchunks, CW = kRangeComputeWaves, U = kRangeBlockQuads, fpt = pl.fpt;
    const uint32_t real_sets = (p->k + 63) / 64, streams = pl.kblocks * CW;
    const size_t block_words = (size_t)U * 64 * 6, off_base = (size_t)U * 64 * 4;
    std::vector<size_t> first_entry((size_t)real_sets * R);  // of each (set, range) in p->order
    size_t at = 0;
    for (uint32_t s = 0; s < real_sets; ++s)
        for (uint32_t q = 0; q < R; ++q) {
            first_entry[(size_t)s * R + q] = at;
            at += (size_t)p->chunk_steps[(size_t)s * R + q] * 64;
        }
    list_len.assign((size_t)streams * R * fpt, 0);
    stream_info.assign((size_t)streams * 2, 0);
    words.clear();
    uint32_t blocks = 0;
    for (uint32_t y = 0; y < pl.kblocks; ++y)
        for (uint32_t cw = 0; cw < CW; ++cw) {
            const uint32_t start = blocks;
            for (uint32_t q = 0; q < R; ++q)
                for (uint32_t f = 0; f < fpt; ++f) {
                    const uint32_t s = (y * fpt + f) * CW + cw;
                    const uint32_t T = s < real_sets ? p->chunk_steps[(size_t)s * R + q] : 0;  // multiple of 4
                    list_len[((size_t)(y * CW + cw) * R + q) * fpt + f] = T;
                    const uint32_t nb = (T / 4 + U - 1) / U;
                    words.resize((size_t)(blocks + nb) * block_words, 0u);
                    for (uint32_t e = 0; e < T; ++e)
                        for (uint32_t l = 0; l < 64; ++l) {
                            const uint32_t ent = p->order[first_entry[(size_t)s * R + q] + (size_t)e * 64 + l];
                            const uint32_t j = s * 64 + l;
                            uint32_t slot;
                            float c = 0.f;
                            if ((ent & kPadSample) || j >= p->k) {
                                slot = (ent & ~kPadSample) % pl.classes;  // a slot of the wanted bank class
                            } else {
                                slot = p->idx[(size_t)j * p->m + ent] - q * pl.chunk;
                                c = p->coef[(size_t)j * p->m + ent];
                            }
                            const size_t blk = (size_t)(blocks + e / (4 * U)) * block_words;
                            const uint32_t quad = e / 4 % U, pos = e % 4;
                            std::memcpy(&words[blk + ((size_t)quad * 64 + l) * 4 + pos], &c, 4);
                            words[blk + off_base + ((size_t)quad * 64 + l) * 2 + pos / 2] |= (slot * 16u) << (16 * (pos % 2));
                        }
                    blocks += nb;
                }
            stream_info[(size_t)(y * CW + cw) * 2] = start;
            stream_info[(size_t)(y * CW + cw) * 2 + 1] = blocks - start;
        }
    if (words.empty()) words.assign(4, 0u);
}

int launch_ranged(const lsh_params *p, Epilogue ep, const float *d_data, uint64_t N, void *d_out, uint32_t L,
                  void *stream, void *d_out2) {
    const SampledPlan &pl = p->plan;
    if (!pl.ranged || !p->d_triples) return LSH_ERR_UNSUPPORTED;
    SampledArgs a = {};
    a.data = d_data;
    a.N = N;
    a.n = p->n;
    a.k = p->k;
    a.kpad = pl.kpad;
    a.classes = pl.classes;
    a.off = p->d_off;
    a.w = p->w;
    a.inv_w = 1.0f / p->w;
    int exp2 = 0;
    a.w_is_pow2 = (std::frexp(p->w, &exp2) == 0.5f) ? 1 : 0;
    a.epilogue = (int)ep;
    a.out = d_out;
    a.out2 = d_out2;
    a.L = L;
    a.g = L ? p->k / L : 1;
    a.chunk = pl.chunk;
    a.nchunks = pl.nchunks;
    a.triples = static_cast<const uint4 *>(p->d_triples);
    a.list_len = static_cast<const uint32_t *>(p->d_list_len);
    a.stream = static_cast<const uint2 *>(p->d_stream);
    a.fpt = pl.fpt;
    const uint64_t ntiles = (N + 15) / 16;
    // one workgroup per CU (two 64 KB buffers), persistent over the tiles; the kblocks workgroups
    // that share a tile differ by a multiple of 8 in their linear number and so run on one XCD
    uint64_t gx = (uint64_t)p->num_cus / pl.kblocks;
    gx = gx < 8 ? 8 : gx / 8 * 8;
    if (gx > ntiles) gx = ntiles;
    const dim3 grid((uint32_t)gx, pl.kblocks);
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
#define LSH_RANGED_FPT(EP_) \
    switch (pl.fpt) { \
        case 1: return launch(&sampled_ranged_kernel<1, EP_>, a, grid, s); \
        case 2: return launch(&sampled_ranged_kernel<2, EP_>, a, grid, s); \
        case 3: return launch(&sampled_ranged_kernel<3, EP_>, a, grid, s); \
        case 4: return launch(&sampled_ranged_kernel<4, EP_>, a, grid, s); \
        default: return LSH_ERR_UNSUPPORTED; \
    }
    switch (ep) {
        case Epilogue::Ids: LSH_RANGED_FPT((int)Epilogue::Ids)
        case Epilogue::Proj: LSH_RANGED_FPT((int)Epilogue::Proj)
        case Epilogue::Signs: LSH_RANGED_FPT((int)Epilogue::Signs)
        case Epilogue::IdsKeys: LSH_RANGED_FPT((int)Epilogue::IdsKeys)
        default: LSH_RANGED_FPT((int)Epilogue::Keys)
    }
#undef LSH_RANGED_FPT
}

}  // namespace lsh
