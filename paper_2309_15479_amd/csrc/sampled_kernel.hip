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
// Two kernels here: sampled_reg_kernel keeps lists of up to 64 samples in registers for the
// whole launch (small n); sampled_kernel streams longer lists through registers for every
// full-dimension tile.  Large vectors are cut into coordinate ranges by the kernel of
// ranged_kernel.hip.
#include <hip/hip_runtime.h>

#include <map>
#include <mutex>
#include <type_traits>

#include "sampled_common.h"

namespace lsh {
namespace {

constexpr int kChunk = 32;                     // samples held in registers at a time
constexpr uint32_t kLdsBudget = 158u * 1024u;  // of the CU's 160 KB

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
    if (EP == (int)Epilogue::Keys || EP == (int)Epilogue::IdsKeys) {
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

template <typename Kernel>
int launch_kernel(Kernel fn, uint32_t lds_bytes, const SampledArgs &args, dim3 grid, dim3 block,
                  hipStream_t stream) {
    if (ensure_lds_limit(reinterpret_cast<const void *>(fn), lds_bytes) != LSH_OK) return LSH_ERR_HIP;
    hipLaunchKernelGGL(fn, grid, block, lds_bytes, stream, args);
    return hipGetLastError() == hipSuccess ? LSH_OK : LSH_ERR_HIP;
}

}  // namespace

// hipFuncSetAttribute costs about a millisecond of host time: raise a kernel's dynamic LDS
// limit once per kernel, size and device (the attribute belongs to the kernel as loaded on the
// current device), not per launch.
int ensure_lds_limit(const void *fn, uint32_t lds_bytes) {
    static std::mutex mu;
    static std::map<std::pair<int, const void *>, uint32_t> granted;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return LSH_ERR_HIP;
    std::lock_guard<std::mutex> lock(mu);
    auto it = granted.find({dev, fn});
    if (it != granted.end() && it->second >= lds_bytes) return LSH_OK;
    if (hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes) != hipSuccess)
        return LSH_ERR_HIP;
    granted[{dev, fn}] = lds_bytes;
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
    const uint32_t k64 = (k + 63) / 64 * 64;
    const bool whole_vector_fits = fits(4, 8, 16) || fits(4, 4, 16) || fits(4, 2, 16) || fits(4, 1, 16) ||
                                   fits(2, 1, 32) || fits(1, 1, 64);
    pl.m_pad = (m + kChunk - 1) / kChunk * kChunk;
    // Register-list kernel: lists of at most two chunks, 16-byte slots, two tile buffers in LDS.
    // The kernel is bound by vector-ALU issue (a 64-lane FMA takes a SIMD four cycles), so the
    // tile is the largest whose accumulators and in-flight reads still fit the 128 registers of
    // a lane (16 vectors): the per-sample address arithmetic and the per-tile load and barrier
    // code are then shared by the most FMAs.  Only while a tile stays small (at most 2 prefetch
    // pieces per wave): with large n one tile's gather is shorter than the latency of the next
    // tile's loads, and the ranged kernel, which shares a bigger tile among more functions, wins.
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
    // Ranged kernel (ranged_kernel.hip): when a full-dimension tile would hold fewer than 16
    // vectors (or none) and the lists do not stay in registers, given enough functions for its 8
    // gathering waves.  A lane owns up to 4 functions (sets of 64 functions, 8 sets apart).
    pl.ranged = false;
    if (!pl.reg_table && (!whole_vector_fits || pl.rt != 4 || pl.sub < 4) && k64 >= 64 * kRangeComputeWaves) {
        const uint32_t nsets = k64 / 64;
        const uint32_t per_wg_max = kRangeComputeWaves * 4;
        pl.kblocks = (nsets + per_wg_max - 1) / per_wg_max;
        const uint32_t per_wg = (nsets + pl.kblocks - 1) / pl.kblocks;
        pl.fpt = (per_wg + kRangeComputeWaves - 1) / kRangeComputeWaves;
        pl.kpad = pl.kblocks * kRangeComputeWaves * pl.fpt * 64;
        pl.block = 64 * kRangeComputeWaves;
        pl.chunk = kWindowCoords;
        pl.nchunks = (n + kWindowCoords - 1) / kWindowCoords;
        // quads of a function per list block: blocks of 4 quads (3 with three functions per
        // lane) keep the next block's loads far enough ahead, but a stage is a whole number of
        // blocks, so no more quads than a function has samples per range
        pl.qpf = 4 / pl.fpt;
        while (pl.qpf > 1 && (uint64_t)pl.qpf * 4 * pl.nchunks > m) pl.qpf /= 2;
        pl.stages = (pl.nchunks + kWindowSlots - 1) / kWindowSlots * kWindowSlots;
        pl.rt = 4; pl.sub = 4; pl.sp = 4; pl.classes = 16; pl.group = 16;
        pl.lds_bytes = kWindowSlots * 4 * kWindowCoords * 16;
        pl.copies = 1;
        pl.ranged = true;
        pl.supported = true;
        return pl;
    }
    if (!whole_vector_fits) return pl;  // unsupported: too few functions for the ranged kernel
    const uint32_t max_block = pl.reg_table ? 512 : 1024;
    pl.block = k64 >= max_block ? max_block : k64;
    pl.kblocks = (k64 + pl.block - 1) / pl.block;
    pl.kpad = pl.block * pl.kblocks;
    pl.supported = true;
    return pl;
}

// Shapes whose gather kernel has the epilogue that writes ids and keys: tiles of 4-vector
// sub-tiles (the ids of a quad of lanes are transposed), tables of a power of two >= 4 functions,
// k a multiple of 4; not the register-list kernels.
bool sampled_ids_keys_supported(const lsh_params *p, uint32_t L) {
    const SampledPlan &pl = p->plan;
    if (!pl.supported || !L || p->k % L || (p->k & 3)) return false;
    const uint32_t g = p->k / L;
    if (g < 4 || g > 64 || (g & (g - 1))) return false;
    return pl.ranged || (!pl.reg_table && pl.rt == 4);
}

int launch_sampled(const lsh_params *p, Epilogue ep, const float *d_data, uint64_t N, void *d_out,
                   uint32_t L, void *stream, void *d_out2) {
    const SampledPlan &pl = p->plan;
    if (!pl.supported) return LSH_ERR_UNSUPPORTED;
    if (ep == Epilogue::IdsKeys && !sampled_ids_keys_supported(p, L)) return LSH_ERR_UNSUPPORTED;
    if (pl.ranged) return launch_ranged(p, ep, d_data, N, d_out, L, stream, d_out2);
    SampledArgs a = {};
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
    a.out2 = d_out2;
    a.L = L;
    a.g = L ? p->k / L : 1;
    a.buf_floats = pl.lds_bytes / 4;
    a.copy_b_floats = pl.copies == 2 ? (p->n + pl.classes) * pl.sp * pl.rt : 0;
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
    if (ep == Epilogue::IdsKeys) {  // 4-vector sub-tiles only (checked above)
        constexpr int EK = (int)Epilogue::IdsKeys;
        if (pl.sub == 8) return launch_kernel(&sampled_kernel<4, 8, EK>, lds_bytes, a, grid, block, s);
        if (pl.sub == 4) return launch_kernel(&sampled_kernel<4, 4, EK>, lds_bytes, a, grid, block, s);
        if (pl.sub == 2) return launch_kernel(&sampled_kernel<4, 2, EK>, lds_bytes, a, grid, block, s);
        return launch_kernel(&sampled_kernel<4, 1, EK>, lds_bytes, a, grid, block, s);
    }
#define LSH_GEN_ALL(EP_) \
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
