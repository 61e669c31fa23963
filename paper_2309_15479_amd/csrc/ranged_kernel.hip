// Sampled-projection kernel (FastLSH, Sec. 3.1, Eq. 5) for long lists and large dimensions on
// gfx950: the 4096- and 16384-dimensional shapes.
//
//   p_j(v) = sum_{i<m} a~_j[i] * v[S_j[i]],   h_j(v) = floor((p_j(v) + b~_j) / w)
//
// Mapping as in sampled_kernel.hip: one lane = one hash function, a tile = 16 vectors kept in LDS
// as 16-byte slots (one coordinate of four vectors), one 16-byte LDS read feeds four
// multiply-adds.  What differs:
//
//  * A ring of coordinate ranges.  LDS holds 16 vectors x 2048 coordinates (128 KB) as a ring of
//    eight slots of 256 coordinates, laid out [ring slot][sub-tile of 4 vectors][coordinate], so
//    the four reads of a sample differ only in their immediate offset and a slot's bank class
//    is its coordinate modulo 16.  A tile passes through in stages (a multiple of eight per
//    tile, so that a range has the same slot in every tile): stage s brings range s into the
//    ring, and during stage s the ranges s .. s + 6 are readable while the slot of range s - 1
//    is being refilled with range s + 7 (of this tile or the first ranges of the next).
//    Accumulators persist across the stages of a tile.
//
//  * Lists that work ahead.  Every function's samples are ordered by range on the host.  All
//    gathering waves of a workgroup run the same number of entries per stage, but a lane may
//    spend a stage's entries on any readable range, so a function with few samples in the
//    current range works ahead on the next six: since all functions have m samples, almost no
//    entry is padding (schedule.cpp; with one fixed stage per range, 1.63 / 1.28 entries per
//    sample were visited at m = 64 / 256, n = 4096, now 1.13 / 1.03).
//
//  * Loader waves.  A workgroup is 8 gathering waves plus 4 loading waves, which meet at one
//    barrier per stage.  A loading wave keeps the loads of three stages in flight (the stages
//    are short: 2 us at m = 64) and writes each, transposed, into its slot one barrier before
//    the first list may read it.  The two kinds of wave have their own counters of outstanding
//    memory operations, so a gatherer's wait for list entries never waits for tile data; the
//    barrier orders LDS traffic only, so neither waits there for what it has in flight.
//
//  * Packed lists.  The kernel is bound by vector-ALU issue (sixteen multiply-adds per list
//    entry), so everything else an entry costs is kept small: a lane's list is stored in quads
//    of entries, 16 bytes of coefficients and 8 bytes holding four 16-bit LDS slot numbers, which
//    one shift with a sub-word operand turns into the entry's address (one instruction per entry;
//    a vector memory instruction per two entries).  A lane owns up to four functions (sets of 64
//    functions, 8 sets apart, so that a workgroup covers up to 2048 functions per tile load)
//    and a list block holds the next quad of each of them (two or four quads with two or one
//    functions per lane, unless a range holds fewer samples than that), an even number of
//    blocks per tile.  The blocks of one gathering wave form one contiguous stream that wraps
//    around at the end of a tile; the block after the one in use is always on its way, across
//    stages and tiles.  Where the stages end is a table of barrier counts per block, read with
//    scalar loads.
//
// Padding entries (where a lane has nothing readable left, to fill a stage up to a whole
// block, and the spare steps that let the bank schedule move samples) carry coefficient 0 and read one of the first 16 slots of the stage's own range,
// whichever bank class the schedule wants; the loaders write zeros to the slots beyond the
// last coordinate, so such an entry always multiplies a finite value of the same vector by
// zero.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstring>
#include <map>
#include <mutex>
#include <vector>
#include <type_traits>

#include "sampled_common.h"

namespace lsh {
namespace {

constexpr int kCW = (int)kRangeComputeWaves;  // gathering waves
constexpr int kLW = 4;                        // loading waves: wave kCW + s loads sub-tile s
constexpr int kThreads = (kCW + kLW) * 64;
constexpr int kC = (int)kWindowCoords;
constexpr int kSlots = (int)kWindowSlots;
constexpr int kSubBytes = kC * 16;             // one sub-tile of one ring slot
constexpr int kSlotBytes = 4 * kSubBytes;      // one ring slot: 16 KB
constexpr int kLdsBytes = kSlots * kSlotBytes; // 128 KB
constexpr int kPieces = kC / 64;               // 64-coordinate pieces of a slot
constexpr int kDepth = 4;                      // register sets of a loading wave: loads of kDepth - 1 stages in flight
static_assert(kWindowSlots % kDepth == 0, "the stages of a workgroup are a multiple of the loaders' register sets");
static_assert(kWindowLook + 2 == kWindowSlots, "one slot is being filled, the others are readable");

typedef float floatx4 __attribute__((ext_vector_type(4)));

// one block of a lane's lists: U quads of entries
template <int U>
struct ListBlock {
    uint4 coef[U];  // four coefficients (float bits)
    uint2 off[U];   // four 16-bit numbers of the entries' 16-byte slots in sub-tile 0 (LDS byte address / 16)
};

// The four 16-byte slots of one entry: the same coordinate in the four sub-tiles.  `address` is
// the LDS byte address itself (the kernel's only LDS is the dynamic array, which starts at 0:
// checked at launch), so no base is added per entry.
__device__ __forceinline__ void read_entry(uint32_t address, floatx4 (&x)[4]) {
    typedef const __attribute__((address_space(3))) floatx4 *SlotPointer;
#pragma unroll
    for (int st = 0; st < 4; ++st) x[st] = *(SlotPointer)(uintptr_t)(address + st * kSubBytes);
}

__device__ __forceinline__ void fma_entry(float c, const floatx4 (&x)[4], float (&acc)[4][4]) {
#pragma unroll
    for (int st = 0; st < 4; ++st) {
        acc[st][0] = fmaf(c, x[st][0], acc[st][0]);
        acc[st][1] = fmaf(c, x[st][1], acc[st][1]);
        acc[st][2] = fmaf(c, x[st][2], acc[st][2]);
        acc[st][3] = fmaf(c, x[st][3], acc[st][3]);
        pin(acc[st]);
    }
}

// LDS byte address of the slot whose number is the low (HI = 0) or high half of `pair`: one
// shift whose operand is the half-word.  (Written out because the compiler, given the shift
// and the mask or the two shifts, emits two instructions.)
template <int HI>
__device__ __forceinline__ uint32_t slot_address(uint32_t pair) {
    uint32_t r;
    if (HI)
        asm("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:WORD_1"
            : "=v"(r) : "s"(4u), "v"(pair));
    else
        asm("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:WORD_0"
            : "=v"(r) : "s"(4u), "v"(pair));
    return r;
}

// Four entries of a lane's list against the 16 vectors of the tile; the LDS reads of an entry go
// out before the multiply-adds of the entry before it.  (Deeper read-ahead, tried with a ring of
// three register sets and with all reads of a group up front, changes nothing but the register
// count: the vector ALU is the busy unit either way.)
__device__ __forceinline__ void gather_quad(const uint4 c, const uint2 o, float (&acc)[4][4]) {
    floatx4 x[2][4];
    __builtin_amdgcn_sched_barrier(0);
    read_entry(slot_address<0>(o.x), x[0]);
    __builtin_amdgcn_sched_barrier(0);
    read_entry(slot_address<1>(o.x), x[1]);
    fma_entry(__uint_as_float(c.x), x[0], acc);
    __builtin_amdgcn_sched_barrier(0);
    read_entry(slot_address<0>(o.y), x[0]);
    fma_entry(__uint_as_float(c.y), x[1], acc);
    __builtin_amdgcn_sched_barrier(0);
    read_entry(slot_address<1>(o.y), x[1]);
    fma_entry(__uint_as_float(c.z), x[0], acc);
    __builtin_amdgcn_sched_barrier(0);
    fma_entry(__uint_as_float(c.w), x[1], acc);
    __builtin_amdgcn_sched_barrier(0);
}

// FPT functions per lane, QPF quads of each per list block
template <int FPT, int QPF, int EP>
__global__ __launch_bounds__(kThreads) void sampled_ranged_kernel(const SampledArgs a,
                                                                  const uint32_t *__restrict__ barriers,
                                                                  const uint2 *__restrict__ streams) {
    extern __shared__ __align__(16) char lds[];  // [8 ring slots][4 sub-tiles][256 coordinates] x 16 bytes
    constexpr int U = FPT * QPF;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint32_t lane = threadIdx.x & 63;
    const uint32_t n = a.n, R = a.nchunks, stages = a.stages;
    const uint64_t ntiles = (a.N + 15) / 16;
    const uint64_t first_tile = blockIdx.x;  // the host launches at most ntiles workgroups along x
    const uint64_t my_tiles = (ntiles - first_tile + gridDim.x - 1) / gridDim.x;
    const uint64_t total = my_tiles * stages;  // stages of this workgroup, numbered x = 0 .. total - 1:
                                               // stage x owns ring slot x % 8 = its range % 8

    if (wave >= (uint32_t)kCW) {
        // ---- loading waves: wave kCW + st fetches sub-tile st (vectors 4 st .. 4 st + 3) of every stage
        const uint32_t st = wave - kCW;
        char *mine = lds + st * kSubBytes + lane * 16;
        // the whole loop once for rows of a multiple of four floats (16-byte loads) and once for
        // the others: one path through it keeps the count of loads in flight exact
        auto loader = [&](auto vec) __attribute__((always_inline)) {
            constexpr bool V = decltype(vec)::value;
            float pre[kDepth][kPieces][4];
            // the stage fetched next and the stage written next, each as (number, tile, range)
            uint64_t xf = 0, tf = first_tile, xs = 0;
            uint32_t rf = 0, rs = 0;
            auto fetch = [&](float (&set)[kPieces][4]) __attribute__((always_inline)) {
                // stages past the last one and stages without a range of their own fetch the
                // tile's first coordinates again: the values are never written to LDS
                const bool real = xf < total && rf < R;
                const uint64_t row0 = (real ? tf : first_tile) * 16;
                const float *rows = a.data + row0 * n;
                const uint32_t rows_valid = (uint32_t)min((uint64_t)16, a.N - row0);
                const uint32_t c0 = real ? rf * kC : 0;
                const uint32_t end = c0 + kC < n ? c0 + kC : n;
#pragma unroll
                for (int f = 0; f < kPieces; ++f) load_raw<V>(rows, rows_valid, n, st * 4, c0 + f * 64, end, lane, set[f]);
                ++xf;
                if (++rf == stages) {
                    rf = 0;
                    tf += gridDim.x;
                }
            };
            auto stash = [&](float (&set)[kPieces][4]) __attribute__((always_inline)) {
                if (rs < R) {
                    const uint32_t len = n - rs * kC;  // coordinates of this range (>= kC: all of them)
                    char *dst = mine + (uint32_t)(xs & (kSlots - 1)) * kSlotBytes;
#pragma unroll
                    for (int f = 0; f < kPieces; ++f) {
                        slot_from_raw<V>(set[f]);
                        const bool inside = (uint32_t)(f * 64) + lane < len;
                        floatx4 v = {inside ? set[f][0] : 0.f, inside ? set[f][1] : 0.f, inside ? set[f][2] : 0.f,
                                     inside ? set[f][3] : 0.f};
                        *reinterpret_cast<floatx4 *>(dst + f * 64 * 16) = v;
                    }
                }
                ++xs;
                if (++rs == stages) rs = 0;
            };
            // Barrier b (b = 0 before the first stage, then one at the end of every stage) lets the
            // gatherers into stage b, which reads the stages b .. b + 6: stage x is written after
            // barrier x - 8 (its slot's previous owner, stage x - 8, is no longer read) and before
            // barrier x - 6.
#pragma unroll
            for (int d = 0; d + 1 < kDepth; ++d) fetch(pre[d]);
            // (a tile has a multiple of eight stages, so `total` is a multiple of kDepth: no
            // test inside the unrolled body, which keeps the count of loads in flight exact)
            for (uint64_t x = 0; x < total; x += kDepth) {
#pragma unroll
                for (int d = 0; d < kDepth; ++d) {
                    if (x + d > (uint64_t)kWindowLook) lds_barrier();
                    fetch(pre[(d + kDepth - 1) % kDepth]);
                    stash(pre[d]);
                }
            }
        };
        if ((n & 3) == 0) loader(std::true_type{});
        else loader(std::false_type{});
        // the barriers the gatherers still pass: total + 1 in all
        const uint64_t passed = total > (uint64_t)kWindowLook + 1 ? total - (kWindowLook + 1) : 0;
        for (uint64_t b = passed; b < total + 1; ++b) lds_barrier();
        return;
    }

    // ---- gathering waves
    const uint32_t stream_id = blockIdx.y * kCW + wave;
    const uint2 si = streams[stream_id];  // {first block, blocks per tile}
    // a block in memory: U x 64 lanes x 16 bytes of coefficients, then U x 64 x 8 bytes of offsets
    constexpr uint32_t kBlockWords = U * 64 * 6;
    const uint32_t *sbase = reinterpret_cast<const uint32_t *>(a.triples) + (size_t)si.x * kBlockWords;
    const uint32_t sblocks = si.y;
    // barriers to pass before the first block of a tile and after each of its blocks
    const uint32_t *bar = barriers + (size_t)blockIdx.y * a.bar_stride;
    // list registers: the block in use and the one after it (always on its way)
    ListBlock<U> P, Q;
    uint32_t next_block = 0;
    auto load_block = [&](ListBlock<U> &blk) __attribute__((always_inline)) {
        const uint32_t *src = sbase + (size_t)next_block * kBlockWords;
#pragma unroll
        for (int i = 0; i < U; ++i) {
            blk.coef[i] = *reinterpret_cast<const uint4 *>(src + (i * 64 + lane) * 4);
            blk.off[i] = *reinterpret_cast<const uint2 *>(src + U * 64 * 4 + (i * 64 + lane) * 2);
        }
        next_block = next_block + 1 == sblocks ? 0 : next_block + 1;
    };
    load_block(P);

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

    auto gather_block = [&](const ListBlock<U> &blk, float (&acc)[FPT][4][4]) __attribute__((always_inline)) {
#pragma unroll
        for (int f = 0; f < FPT; ++f)
#pragma unroll
            for (int q = 0; q < QPF; ++q) gather_quad(blk.coef[f * QPF + q], blk.off[f * QPF + q], acc[f]);
    };
    auto pass = [&](uint32_t count) __attribute__((always_inline)) {
        for (uint32_t i = 0; i < count; ++i) lds_barrier();
    };

    lds_barrier();  // the first seven stages are in the ring
    for (uint64_t t = first_tile; t < ntiles; t += gridDim.x) {
        float acc[FPT][4][4];
#pragma unroll
        for (int f = 0; f < FPT; ++f)
#pragma unroll
            for (int st = 0; st < 4; ++st)
#pragma unroll
                for (int r = 0; r < 4; ++r) acc[f][st][r] = 0.f;
        pass(bar[0]);
        // blocks two at a time (the host makes their number even), the registers of one being
        // refilled while the other is used: no block is ever copied from register to register
        for (uint32_t q = 0; q < sblocks; q += 2) {
            load_block(Q);
            gather_block(P, acc);
            pass(bar[q + 1]);
            load_block(P);
            gather_block(Q, acc);
            if (q + 2 < sblocks) pass(bar[q + 2]);
        }
#pragma unroll
        for (int f = 0; f < FPT; ++f)
            finish<4, 4, EP>(a, t * 16, fresh(j0) + f * kCW * 64, acc[f], bias[f], key_pow[f]);
        pass(bar[sblocks]);  // the tile's last stages
    }
}

template <typename Kernel>
int launch(Kernel fn, const SampledArgs &args, dim3 grid, hipStream_t stream) {
    if (ensure_lds_limit(reinterpret_cast<const void *>(fn), kLdsBytes) != LSH_OK) return LSH_ERR_HIP;
    // the gatherers use LDS byte addresses counted from 0: the dynamic array must be all the LDS
    // there is (asked once per kernel)
    static std::mutex mu;
    static std::map<const void *, bool> starts_at_zero;
    {
        std::lock_guard<std::mutex> lock(mu);
        auto it = starts_at_zero.find(reinterpret_cast<const void *>(fn));
        if (it == starts_at_zero.end()) {
            hipFuncAttributes attr;
            if (hipFuncGetAttributes(&attr, reinterpret_cast<const void *>(fn)) != hipSuccess) return LSH_ERR_HIP;
            it = starts_at_zero.emplace(reinterpret_cast<const void *>(fn), attr.sharedSizeBytes == 0).first;
        }
        if (!it->second) return LSH_ERR_UNSUPPORTED;
    }
    hipLaunchKernelGGL(fn, grid, dim3(kThreads), kLdsBytes, stream, args, args.list_len, args.stream);
    return hipGetLastError() == hipSuccess ? LSH_OK : LSH_ERR_HIP;
}

}  // namespace

// Host tables of the ranged kernel: the list blocks, the barrier counts [kblocks][blocks + 1]
// (before the first block of a tile and after each block), and {first block, blocks per tile}
// per gathering wave.
void build_ranged_tables(const lsh_params *p, std::vector<uint32_t> &words, std::vector<uint32_t> &barriers,
                         std::vector<uint32_t> &stream_info) {
    // One stream of list blocks per gathering wave, in the order the wave consumes them.  A
    // block is, for each of the lane's fpt functions, its next qpf quads of entries x 64
    // lanes: 16 bytes of coefficients per quad and lane, then 8 bytes of 16-bit slot numbers:
    // 1024 x (range modulo 8) + coordinate minus the range's first (LDS byte address / 16 of
    // the coordinate's slot in sub-tile 0).
    const SampledPlan &pl = p->plan;
    const uint32_t CW = kRangeComputeWaves, fpt = pl.fpt, qpf = pl.qpf, U = fpt * qpf, S = pl.stages;
    const uint32_t real_sets = (p->k + 63) / 64, streams = pl.kblocks * CW;
    const size_t block_words = (size_t)U * 64 * 6, off_base = (size_t)U * 64 * 4;
    // every workgroup's blocks per tile; the sets of a workgroup are consecutive in p->order
    uint32_t max_blocks = 0;
    std::vector<uint32_t> wg_entries(pl.kblocks, 0);
    for (uint32_t y = 0; y < pl.kblocks; ++y) {
        for (uint32_t s = 0; s < S; ++s) wg_entries[y] += p->chunk_steps[(size_t)y * S + s];
        max_blocks = std::max(max_blocks, wg_entries[y] / (4 * qpf));
    }
    const uint32_t bar_stride = max_blocks + 1;  // the same for every workgroup
    barriers.assign((size_t)pl.kblocks * bar_stride, 0);
    stream_info.assign((size_t)streams * 2, 0);
    words.clear();
    uint32_t blocks = 0;
    size_t set_base = 0;  // first entry in p->order of the workgroup's first set
    for (uint32_t y = 0; y < pl.kblocks; ++y) {
        const uint32_t E = wg_entries[y], nb = E / (4 * qpf);
        const uint32_t *len = &p->chunk_steps[(size_t)y * S];
        // the stage each entry position belongs to
        std::vector<uint32_t> stage_of(E);
        {
            uint32_t at = 0;
            for (uint32_t s = 0; s < S; ++s)
                for (uint32_t e = 0; e < len[s]; ++e) stage_of[at++] = s;
        }
        // barrier counts: every stage ends with one, after its last block (stages without
        // entries end right after the stage before them)
        const size_t bar0 = (size_t)y * bar_stride;
        {
            uint32_t at = 0;
            for (uint32_t s = 0; s < S; ++s) {
                at += len[s];
                ++barriers[bar0 + at / (4 * qpf)];
            }
        }
        const uint32_t sets_here = std::min(real_sets - std::min(real_sets, y * fpt * CW), fpt * CW);
        for (uint32_t cw = 0; cw < CW; ++cw) {
            const uint32_t start = blocks;
            words.resize((size_t)(blocks + nb) * block_words, 0u);
            for (uint32_t f = 0; f < fpt; ++f) {
                const uint32_t in_wg = f * CW + cw, s = y * fpt * CW + in_wg;
                // a set's entries in p->order: stage after stage, steps x 64
                const size_t first = set_base + (size_t)in_wg * E * 64;
                for (uint32_t e = 0; e < E; ++e) {
                    const uint32_t stage = stage_of[e];
                    for (uint32_t l = 0; l < 64; ++l) {
                        const uint32_t j = s * 64 + l;
                        uint32_t slot;
                        float c = 0.f;
                        const uint32_t ent = in_wg < sets_here ? p->order[first + (size_t)e * 64 + l] : kPadSample;
                        if ((ent & kPadSample) || j >= p->k) {
                            // a slot of the wanted bank class in the stage's own range
                            slot = (stage % kWindowSlots) * 4 * kWindowCoords + (ent & ~kPadSample) % pl.classes;
                        } else {
                            const uint32_t coord = p->idx[(size_t)j * p->m + ent];
                            slot = (coord / kWindowCoords % kWindowSlots) * 4 * kWindowCoords + coord % kWindowCoords;
                            c = p->coef[(size_t)j * p->m + ent];
                        }
                        const size_t blk = (size_t)(start + e / (4 * qpf)) * block_words;
                        const uint32_t quad = f * qpf + e / 4 % qpf, pos = e % 4;
                        std::memcpy(&words[blk + ((size_t)quad * 64 + l) * 4 + pos], &c, 4);
                        words[blk + off_base + ((size_t)quad * 64 + l) * 2 + pos / 2] |= slot << (16 * (pos % 2));
                    }
                }
            }
            blocks += nb;
            stream_info[(size_t)(y * CW + cw) * 2] = start;
            stream_info[(size_t)(y * CW + cw) * 2 + 1] = nb;
        }
        set_base += (size_t)sets_here * E * 64;
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
    a.stages = pl.stages;
    a.bar_stride = p->ranged_bar_stride;
    a.triples = static_cast<const uint4 *>(p->d_triples);
    a.list_len = static_cast<const uint32_t *>(p->d_list_len);
    a.stream = static_cast<const uint2 *>(p->d_stream);
    a.fpt = pl.fpt;
    const uint64_t ntiles = (N + 15) / 16;
    // one workgroup per CU (128 KB of LDS), persistent over the tiles; the kblocks workgroups
    // that share a tile differ by a multiple of 8 in their linear number and so run on one XCD
    uint64_t gx = (uint64_t)p->num_cus / pl.kblocks;
    gx = gx < 8 ? 8 : gx / 8 * 8;
    if (gx > ntiles) gx = ntiles;
    const dim3 grid((uint32_t)gx, pl.kblocks);
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
#define LSH_RANGED_FPT(EP_) \
    switch (pl.fpt * 8 + pl.qpf) { \
        case 1 * 8 + 1: return launch(&sampled_ranged_kernel<1, 1, EP_>, a, grid, s); \
        case 1 * 8 + 2: return launch(&sampled_ranged_kernel<1, 2, EP_>, a, grid, s); \
        case 1 * 8 + 4: return launch(&sampled_ranged_kernel<1, 4, EP_>, a, grid, s); \
        case 2 * 8 + 1: return launch(&sampled_ranged_kernel<2, 1, EP_>, a, grid, s); \
        case 2 * 8 + 2: return launch(&sampled_ranged_kernel<2, 2, EP_>, a, grid, s); \
        case 3 * 8 + 1: return launch(&sampled_ranged_kernel<3, 1, EP_>, a, grid, s); \
        case 4 * 8 + 1: return launch(&sampled_ranged_kernel<4, 1, EP_>, a, grid, s); \
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
