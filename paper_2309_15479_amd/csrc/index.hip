// LSH index (Sec. 3.2): L hash tables of <key, id> pairs and the lookup of a query's L
// buckets, for gfx950.
//
// The paper fixes what a table holds (every vector's id under its key H_l(v)) and how a query
// uses it (fetch the L buckets H_1(u) .. H_L(u), evaluate the candidates), not a layout.  Here a
// table is the vector ids sorted by key (a stable radix sort of N <key, id> pairs, ids
// ascending inside a bucket; all tables are sorted together by the kernels below): a bucket is a contiguous run of the sorted ids, found by binary
// search of the sorted keys.  No chains, no resizing, 12 bytes per vector and table.
//
//   build      keys [N][L] -> per table: sorted keys [N], ids in key order [N]
//   probe      query keys [Q][L] -> per (query, table): first position and length of the bucket
//   candidates concatenation of a query's L buckets, all queries, at given offsets
//   nearest    processing of the candidates (Sec. 3.2, last paragraph): the candidate closest to
//              the query in l2, distances in fp32 over the full vectors; all candidates (the
//              exact version) or only the first max_candidates of the combined list (the
//              approximate version evaluates no more than 3L points)
#include <hip/hip_runtime.h>

#include <mutex>
#include <new>

#include "lsh.h"

struct lsh_index {
    uint64_t N = 0;
    uint32_t L = 0;
    int device = -1;
    uint64_t *d_keys = nullptr;  // [L][N] ascending per table
    uint32_t *d_ids = nullptr;   // [L][N] vector ids in key order (ascending within equal keys)
};

namespace {

// one thread per (query, table): lower and upper bound of the query's key in the table
__global__ void probe_kernel(const uint64_t *__restrict__ sorted_keys, uint64_t N, uint32_t L,
                             const uint64_t *__restrict__ qkeys, uint64_t items, uint32_t *__restrict__ start,
                             uint32_t *__restrict__ count) {
    const uint64_t item = blockIdx.x * (uint64_t)blockDim.x + threadIdx.x;
    if (item >= items) return;
    const uint32_t l = (uint32_t)(item % L);
    const uint64_t key = qkeys[item];
    const uint64_t *table = sorted_keys + (uint64_t)l * N;
    uint64_t lo = 0, hi = N;  // first position with table[pos] >= key
    while (lo < hi) {
        const uint64_t mid = (lo + hi) / 2;
        if (table[mid] < key) lo = mid + 1;
        else hi = mid;
    }
    const uint64_t first = lo;
    hi = N;  // first position with table[pos] > key
    while (lo < hi) {
        const uint64_t mid = (lo + hi) / 2;
        if (table[mid] <= key) lo = mid + 1;
        else hi = mid;
    }
    start[item] = (uint32_t)first;
    count[item] = (uint32_t)(lo - first);
}

// Exclusive prefix sum of 32-bit counts into 64-bit offsets, three small launches: (1) every
// block of kScanBlock counts adds up its own, (2) one block turns the block sums into block
// offsets in place, (3) every block scans its counts again on top of its offset.  `partial`
// holds one 64-bit word per block; every word is written by (1) before it is read, so the
// buffer needs no clearing between calls.
constexpr uint32_t kScanThreads = 256, kScanPerThread = 8, kScanBlock = kScanThreads * kScanPerThread;

// sum over the workgroup; every thread gets the total, `before` = sum over the threads below it
__device__ __forceinline__ uint64_t block_scan(uint64_t mine, uint64_t *wave_sums, uint64_t &before) {
    const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint64_t incl = mine;
    for (int d = 1; d < 64; d <<= 1) {
        const uint64_t up = __shfl_up(incl, d);
        if (lane >= (uint32_t)d) incl += up;
    }
    __syncthreads();  // wave_sums may still be read from an earlier call in the same kernel
    if (lane == 63) wave_sums[wave] = incl;
    __syncthreads();
    uint64_t below = 0, total = 0;
    for (uint32_t w = 0; w < kScanThreads / 64; ++w) {
        if (w < wave) below += wave_sums[w];
        total += wave_sums[w];
    }
    before = below + incl - mine;
    return total;
}

__global__ __launch_bounds__(kScanThreads) void scan_block_sums(const uint32_t *__restrict__ count, uint64_t items,
                                                                 uint64_t *__restrict__ partial) {
    __shared__ uint64_t wave_sums[kScanThreads / 64];
    const uint64_t first = (uint64_t)blockIdx.x * kScanBlock + (uint64_t)threadIdx.x * kScanPerThread;
    uint64_t mine = 0;
    for (uint32_t e = 0; e < kScanPerThread; ++e)
        if (first + e < items) mine += count[first + e];
    uint64_t before;
    const uint64_t total = block_scan(mine, wave_sums, before);
    if (threadIdx.x == 0) partial[blockIdx.x] = total;
}

// one workgroup: partial[b] <- sum of partial[0 .. b), for b < blocks, chunk after chunk
__global__ __launch_bounds__(kScanThreads) void scan_partials(uint64_t *__restrict__ partial, uint64_t blocks) {
    __shared__ uint64_t wave_sums[kScanThreads / 64];
    uint64_t carry = 0;
    for (uint64_t base = 0; base < blocks; base += kScanBlock) {
        const uint64_t first = base + (uint64_t)threadIdx.x * kScanPerThread;
        uint64_t v[kScanPerThread], mine = 0;
        for (uint32_t e = 0; e < kScanPerThread; ++e) {
            v[e] = first + e < blocks ? partial[first + e] : 0;
            mine += v[e];
        }
        uint64_t before;
        const uint64_t total = block_scan(mine, wave_sums, before);
        uint64_t run = carry + before;
        for (uint32_t e = 0; e < kScanPerThread; ++e) {
            if (first + e < blocks) partial[first + e] = run;
            run += v[e];
        }
        carry += total;
    }
}

// offsets[i] = sum of count[0 .. i) for i <= items (the last entry is the total)
__global__ __launch_bounds__(kScanThreads) void scan_offsets(const uint32_t *__restrict__ count, uint64_t items,
                                                              const uint64_t *__restrict__ partial,
                                                              uint64_t *__restrict__ offsets) {
    __shared__ uint64_t wave_sums[kScanThreads / 64];
    const uint64_t first = (uint64_t)blockIdx.x * kScanBlock + (uint64_t)threadIdx.x * kScanPerThread;
    uint32_t v[kScanPerThread];
    uint64_t mine = 0;
    for (uint32_t e = 0; e < kScanPerThread; ++e) {
        v[e] = first + e < items ? count[first + e] : 0;
        mine += v[e];
    }
    uint64_t before;
    block_scan(mine, wave_sums, before);
    uint64_t run = partial[blockIdx.x] + before;
    for (uint32_t e = 0; e < kScanPerThread; ++e) {
        if (first + e <= items) offsets[first + e] = run;  // element `items` receives the total
        run += v[e];
    }
}

// the three launches; partial must hold (items / kScanBlock + 1) words
int launch_offsets_scan(const uint32_t *d_count, uint64_t items, uint64_t *d_partial, uint64_t *d_offsets,
                        hipStream_t s) {
    const uint64_t blocks = items / kScanBlock + 1;  // covers element `items` too
    hipLaunchKernelGGL(scan_block_sums, dim3((uint32_t)blocks), dim3(kScanThreads), 0, s, d_count, items, d_partial);
    hipLaunchKernelGGL(scan_partials, dim3(1), dim3(kScanThreads), 0, s, d_partial, blocks);
    hipLaunchKernelGGL(scan_offsets, dim3((uint32_t)blocks), dim3(kScanThreads), 0, s, d_count, items, d_partial,
                       d_offsets);
    return hipGetLastError() == hipSuccess ? LSH_OK : LSH_ERR_HIP;
}

// Stable least-significant-digit radix sort of all L key columns at once (one grid row per
// table): eight passes of 8 bits.  A pass is three launches: per-tile digit histograms, an
// exclusive scan of the (digit, tile) counts of every table, and the scatter.  A tile is 4096
// consecutive pairs; wave w of the workgroup owns pairs 1024 w ... 1024 w + 1023 of it, slot i
// of lane l being pair 64 i + l, so (wave, slot, lane) order is memory order and the ranks
// below keep equal keys in their original order (ids ascending inside a bucket).  The first
// pass reads the keys in place from the caller's [N][L] array and numbers the pairs itself.
constexpr uint32_t kSortThreads = 256, kSortSlots = 16, kSortTile = kSortThreads * kSortSlots;
constexpr uint32_t kSortWaves = kSortThreads / 64;

template <bool FIRST>
__device__ __forceinline__ uint64_t sort_key(const uint64_t *__restrict__ keys, uint64_t N, uint32_t L, uint32_t l,
                                             uint64_t i) {
    return FIRST ? keys[i * L + l] : keys[(uint64_t)l * N + i];
}

// hist[(l * 256 + digit) * tiles + tile] = pairs of the tile with that digit
template <bool FIRST>
__global__ __launch_bounds__(kSortThreads) void sort_histogram(const uint64_t *__restrict__ keys, uint64_t N, uint32_t L,
                                                                uint32_t shift, uint32_t tiles,
                                                                uint32_t *__restrict__ hist) {
    __shared__ uint32_t bins[256];
    // first pass: the L workgroups that read one tile of the caller's [N][L] rows are neighbours
    // in launch order and find it in L2 (else every table would fetch the whole array again)
    const uint32_t l = FIRST ? blockIdx.x % L : blockIdx.y, tile = FIRST ? blockIdx.x / L : blockIdx.x;
    bins[threadIdx.x] = 0;
    __syncthreads();
    const uint64_t first = (uint64_t)tile * kSortTile;
    for (uint32_t e = threadIdx.x; e < kSortTile; e += kSortThreads) {
        const uint64_t i = first + e;
        if (i < N) atomicAdd(&bins[(uint32_t)(sort_key<FIRST>(keys, N, L, l, i) >> shift) & 255u], 1u);
    }
    __syncthreads();
    hist[((size_t)l * 256 + threadIdx.x) * tiles + tile] = bins[threadIdx.x];
}

// one workgroup per table: hist <- exclusive prefix sum over its 256 * tiles counts, in place
__global__ __launch_bounds__(kScanThreads) void sort_scan(uint32_t *__restrict__ hist, uint32_t tiles) {
    __shared__ uint64_t wave_sums[kScanThreads / 64];
    uint32_t *mine = hist + (size_t)blockIdx.x * 256 * tiles;
    const uint64_t count = (uint64_t)256 * tiles;
    uint64_t carry = 0;
    for (uint64_t base = 0; base < count; base += kScanBlock) {
        const uint64_t first = base + (uint64_t)threadIdx.x * kScanPerThread;
        uint32_t v[kScanPerThread];
        uint64_t sum = 0;
        for (uint32_t e = 0; e < kScanPerThread; ++e) {
            v[e] = first + e < count ? mine[first + e] : 0;
            sum += v[e];
        }
        uint64_t before;
        const uint64_t total = block_scan(sum, wave_sums, before);
        uint64_t run = carry + before;
        for (uint32_t e = 0; e < kScanPerThread; ++e) {
            if (first + e < count) mine[first + e] = (uint32_t)run;  // below N < 2^31
            run += v[e];
        }
        carry += total;
    }
}

// The scatter of a pass.  A pair's place in the output is (pairs of smaller digits in its
// table) + (pairs of its digit in earlier tiles) + (pairs of its digit before it in its tile);
// the first two come scanned from the histograms, the third from wave ballots in memory order.
// The tile is first put in that order in LDS and then written out by consecutive threads:
// pairs of one digit are then neighbours in LDS and in memory, so the stores of a wave are a
// few runs instead of 64 separate 8-byte writes (about three times faster than scattering from the
// registers on this part).
template <bool FIRST>
__global__ __launch_bounds__(kSortThreads) void sort_scatter(const uint64_t *__restrict__ keys,
                                                              const uint32_t *__restrict__ ids, uint64_t N, uint32_t L,
                                                              uint32_t shift, uint32_t tiles,
                                                              const uint32_t *__restrict__ offsets,
                                                              uint64_t *__restrict__ out_keys,
                                                              uint32_t *__restrict__ out_ids) {
    __shared__ uint32_t counter[kSortWaves][256];  // per wave: pairs seen so far per digit, then its first place in the tile's order
    __shared__ uint32_t delta[256];                // per digit: first output position minus first place in the tile's order
    __shared__ uint32_t wave_total[kSortWaves];
    __shared__ uint64_t tile_keys[kSortTile];
    __shared__ uint32_t tile_ids[kSortTile];
    const uint32_t l = FIRST ? blockIdx.x % L : blockIdx.y, tile = FIRST ? blockIdx.x / L : blockIdx.x;  // as in sort_histogram
    const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (uint32_t w = 0; w < kSortWaves; ++w) counter[w][threadIdx.x] = 0;
    __syncthreads();
    const uint64_t tile_first = (uint64_t)tile * kSortTile;
    const uint64_t first = tile_first + (uint64_t)wave * (kSortSlots * 64) + lane;
    const uint64_t below = (1ull << lane) - 1;
    uint64_t key[kSortSlots];
    uint32_t id[kSortSlots];
    uint32_t rank[kSortSlots];
    volatile uint32_t *mine = counter[wave];
#pragma unroll
    for (uint32_t i = 0; i < kSortSlots; ++i) {
        const uint64_t at = first + (uint64_t)i * 64;
        const bool valid = at < N;
        key[i] = valid ? sort_key<FIRST>(keys, N, L, l, at) : 0;
        id[i] = FIRST ? (uint32_t)at : valid ? ids[(uint64_t)l * N + at] : 0u;
        const uint32_t digit = (uint32_t)(key[i] >> shift) & 255u;
        // lanes of the wave that hold the same digit in this slot
        uint64_t peers = __ballot(valid);
#pragma unroll
        for (uint32_t bit = 0; bit < 8; ++bit) {
            const uint64_t set = __ballot((digit >> bit) & 1u);
            peers &= ((digit >> bit) & 1u) ? set : ~set;
        }
        const uint32_t seen = mine[digit];
        rank[i] = seen + (uint32_t)__popcll(peers & below);
        __builtin_amdgcn_wave_barrier();
        if (valid && (peers & below) == 0) mine[digit] = seen + (uint32_t)__popcll(peers);  // the first of the peers
        __builtin_amdgcn_wave_barrier();
    }
    __syncthreads();
    {   // thread d: the tile's pairs of digit d, their first place in the tile's order (an exclusive
        // scan over the digits) and, per wave, the first place of that wave's pairs of the digit
        uint32_t per_wave[kSortWaves], total = 0;
        for (uint32_t w = 0; w < kSortWaves; ++w) {
            per_wave[w] = counter[w][threadIdx.x];
            total += per_wave[w];
        }
        uint32_t incl = total;  // inclusive scan over the 64 digits of this wave, then over the waves
#pragma unroll
        for (uint32_t step = 1; step < 64; step <<= 1) {
            const uint32_t up = __shfl_up(incl, step);
            if (lane >= step) incl += up;
        }
        if (lane == 63) wave_total[wave] = incl;
        __syncthreads();
        uint32_t start = incl - total;
        for (uint32_t w = 0; w < wave; ++w) start += wave_total[w];
        delta[threadIdx.x] = offsets[((size_t)l * 256 + threadIdx.x) * tiles + tile] - start;
        for (uint32_t w = 0; w < kSortWaves; ++w) {
            counter[w][threadIdx.x] = start;
            start += per_wave[w];
        }
    }
    __syncthreads();
#pragma unroll
    for (uint32_t i = 0; i < kSortSlots; ++i) {
        const uint64_t at = first + (uint64_t)i * 64;
        if (at >= N) continue;
        const uint32_t digit = (uint32_t)(key[i] >> shift) & 255u;
        const uint32_t place = counter[wave][digit] + rank[i];
        tile_keys[place] = key[i];
        tile_ids[place] = id[i];
    }
    __syncthreads();
    const uint32_t pairs = (uint32_t)(N - tile_first < kSortTile ? N - tile_first : kSortTile);
    for (uint32_t place = threadIdx.x; place < pairs; place += kSortThreads) {
        const uint64_t k64 = tile_keys[place];
        const uint64_t pos = (uint64_t)l * N + (uint32_t)(delta[(uint32_t)(k64 >> shift) & 255u] + place);
        out_keys[pos] = k64;
        out_ids[pos] = tile_ids[place];
    }
}

// Scratch of lsh_index_candidate_offsets_static: the block sums of the scan, for callers that
// must not allocate.  One copy per GPU, held until the process ends; its device address is
// looked up once per device (the name below is only a host-side handle of the symbol).
constexpr uint64_t kStaticScanItems = 1ull << 22;
constexpr uint64_t kStaticScanWords = kStaticScanItems / kScanBlock + 1;
static __device__ __align__(256) uint64_t scratch[kStaticScanWords];

constexpr int kMaxDevices = 64;
std::mutex scratch_mutex;
uint64_t *scratch_of_device[kMaxDevices] = {};

// device address of `scratch` on the current device (null on failure)
uint64_t *static_scratch() {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(scratch_mutex);
    if (!scratch_of_device[dev]) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess) {
            (void)hipGetLastError();
            return nullptr;
        }
        scratch_of_device[dev] = static_cast<uint64_t *>(ptr);
    }
    return scratch_of_device[dev];
}

// one wave per (query, table): copies the bucket's ids to the output run of that item
__global__ void candidates_kernel(const uint32_t *__restrict__ sorted_ids, uint64_t N, uint32_t L,
                                  const uint32_t *__restrict__ start, const uint32_t *__restrict__ count,
                                  const uint64_t *__restrict__ offsets, uint64_t items, uint32_t *__restrict__ out) {
    const uint32_t lane = threadIdx.x & 63;
    const uint64_t waves = ((uint64_t)gridDim.x * blockDim.x) >> 6;
    for (uint64_t item = (blockIdx.x * (uint64_t)blockDim.x + threadIdx.x) >> 6; item < items; item += waves) {
        const uint32_t l = (uint32_t)(item % L);
        const uint32_t *src = sorted_ids + (uint64_t)l * N + start[item];
        uint32_t *dst = out + offsets[item];
        for (uint32_t i = lane; i < count[item]; i += 64) dst[i] = src[i];
    }
}

// one workgroup per query: squared l2 distance of every candidate of its L buckets (a candidate
// met in several tables is simply evaluated again), minimum with ties to the smaller id.
// INNER: the score is the inner product with the query instead and the largest one wins
// (maximum inner product search; internally the negated product is minimised).
template <bool INNER>
__global__ __launch_bounds__(256) void nearest_kernel(const uint32_t *__restrict__ sorted_ids, uint64_t N, uint32_t L,
                                                      const float *__restrict__ data, const float *__restrict__ queries,
                                                      uint32_t n, const uint32_t *__restrict__ start,
                                                      const uint32_t *__restrict__ count, uint32_t max_candidates,
                                                      uint32_t *__restrict__ best_id, float *__restrict__ best_dist) {
    extern __shared__ float query[];  // [n], then per-wave results
    const uint64_t q = blockIdx.x;
    const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6, waves = blockDim.x >> 6;
    for (uint32_t c = threadIdx.x; c < n; c += blockDim.x) query[c] = queries[q * n + c];
    __syncthreads();
    float mine_d = INFINITY;
    uint32_t mine_id = 0xFFFFFFFFu;
    uint32_t seen = 0;  // candidates are dealt to the waves round-robin over all L buckets
    for (uint32_t l = 0; l < L && seen < max_candidates; ++l) {
        const uint32_t first = start[q * L + l];
        uint32_t len = count[q * L + l];
        if (len > max_candidates - seen) len = max_candidates - seen;  // only the first max_candidates of the list
        const uint32_t *bucket = sorted_ids + (uint64_t)l * N + first;
        for (uint32_t i = (wave + waves - seen % waves) % waves; i < len; i += waves) {
            const uint32_t id = bucket[i];
            const float *v = data + (uint64_t)id * n;
            float acc = 0.f;
            for (uint32_t c = lane; c < n; c += 64) {
                if constexpr (INNER) {
                    acc = fmaf(-v[c], query[c], acc);
                } else {
                    const float d = v[c] - query[c];
                    acc = fmaf(d, d, acc);
                }
            }
            for (int s = 32; s > 0; s >>= 1) acc += __shfl_xor(acc, s);
            if (acc < mine_d || (acc == mine_d && id < mine_id)) {
                mine_d = acc;
                mine_id = id;
            }
        }
        seen += len;
    }
    float *wave_d = query + n;
    uint32_t *wave_id = reinterpret_cast<uint32_t *>(wave_d + waves);
    if (lane == 0) {
        wave_d[wave] = mine_d;
        wave_id[wave] = mine_id;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (uint32_t w = 1; w < waves; ++w)
            if (wave_d[w] < mine_d || (wave_d[w] == mine_d && wave_id[w] < mine_id)) {
                mine_d = wave_d[w];
                mine_id = wave_id[w];
            }
        best_id[q] = mine_id;
        best_dist[q] = INNER ? -mine_d : mine_d;  // no candidate: +inf distance, -inf inner product
    }
}

int on_index_device(const lsh_index *ix) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return LSH_ERR_HIP;
    return dev == ix->device ? LSH_OK : LSH_ERR_INVALID_ARG;
}

}  // namespace

extern "C" {

int lsh_index_build(const uint64_t *d_keys, uint64_t N, uint32_t L, void *stream, lsh_index_t **out) {
    if (!out) return LSH_ERR_INVALID_ARG;
    *out = nullptr;
    if (!d_keys || !N || !L || N >= (1ull << 31) || L > 65535) return LSH_ERR_INVALID_ARG;  // positions are 32-bit, tables a grid row
    int count = 0;
    if (hipGetDeviceCount(&count) != hipSuccess || count <= 0) {
        (void)hipGetLastError();
        return LSH_ERR_NO_DEVICE;
    }
    // the first pass launches one workgroup per (tile, table) in a row
    if (((N + kSortTile - 1) / kSortTile) * L >= (1ull << 31)) return LSH_ERR_UNSUPPORTED;
    lsh_index *ix = new (std::nothrow) lsh_index;
    if (!ix) return LSH_ERR_ALLOC;
    ix->N = N;
    ix->L = L;
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    const uint32_t tiles = (uint32_t)((N + kSortTile - 1) / kSortTile);
    // the other half of the ping-pong, and the (digit, tile) counts of every table
    uint64_t *tmp_keys = nullptr;
    uint32_t *tmp_ids = nullptr, *hist = nullptr;
    int rc = LSH_OK;
    if (hipGetDevice(&ix->device) != hipSuccess) rc = LSH_ERR_HIP;
    if (rc == LSH_OK && hipMalloc(&ix->d_keys, (size_t)L * N * sizeof(uint64_t)) != hipSuccess) rc = LSH_ERR_ALLOC;
    if (rc == LSH_OK && hipMalloc(&ix->d_ids, (size_t)L * N * sizeof(uint32_t)) != hipSuccess) rc = LSH_ERR_ALLOC;
    // temporaries are allocated and released in stream order: the host does not wait for the sort
    if (rc == LSH_OK && hipMallocAsync(reinterpret_cast<void **>(&tmp_keys), (size_t)L * N * sizeof(uint64_t), s) != hipSuccess)
        rc = LSH_ERR_ALLOC;
    if (rc == LSH_OK && hipMallocAsync(reinterpret_cast<void **>(&tmp_ids), (size_t)L * N * sizeof(uint32_t), s) != hipSuccess)
        rc = LSH_ERR_ALLOC;
    if (rc == LSH_OK && hipMallocAsync(reinterpret_cast<void **>(&hist), (size_t)L * 256 * tiles * sizeof(uint32_t), s) != hipSuccess)
        rc = LSH_ERR_ALLOC;
    if (rc == LSH_OK) {
        const dim3 grid(tiles, L), block(kSortThreads);
        // eight passes; odd passes write the index's own arrays, so the last one ends there
        for (uint32_t pass = 0; pass < 8; ++pass) {
            const uint32_t shift = 8 * pass;
            const uint64_t *src_keys = pass == 0 ? d_keys : (pass & 1) ? tmp_keys : ix->d_keys;
            const uint32_t *src_ids = (pass & 1) ? tmp_ids : ix->d_ids;
            uint64_t *dst_keys = (pass & 1) ? ix->d_keys : tmp_keys;
            uint32_t *dst_ids = (pass & 1) ? ix->d_ids : tmp_ids;
            if (pass == 0) {
                const dim3 linear(tiles * L);  // below 2^31 (checked above)
                hipLaunchKernelGGL(sort_histogram<true>, linear, block, 0, s, src_keys, N, L, shift, tiles, hist);
                hipLaunchKernelGGL(sort_scan, dim3(L), dim3(kScanThreads), 0, s, hist, tiles);
                hipLaunchKernelGGL(sort_scatter<true>, linear, block, 0, s, src_keys, src_ids, N, L, shift, tiles, hist,
                                   dst_keys, dst_ids);
            } else {
                hipLaunchKernelGGL(sort_histogram<false>, grid, block, 0, s, src_keys, N, L, shift, tiles, hist);
                hipLaunchKernelGGL(sort_scan, dim3(L), dim3(kScanThreads), 0, s, hist, tiles);
                hipLaunchKernelGGL(sort_scatter<false>, grid, block, 0, s, src_keys, src_ids, N, L, shift, tiles, hist,
                                   dst_keys, dst_ids);
            }
        }
        if (hipGetLastError() != hipSuccess) rc = LSH_ERR_HIP;
    }
    if (tmp_keys) (void)hipFreeAsync(tmp_keys, s);
    if (tmp_ids) (void)hipFreeAsync(tmp_ids, s);
    if (hist) (void)hipFreeAsync(hist, s);
    if (rc != LSH_OK) {
        (void)hipStreamSynchronize(s);
        (void)hipGetLastError();
        lsh_index_destroy(ix);
        return rc;
    }
    *out = ix;
    return LSH_OK;
}

void lsh_index_destroy(lsh_index_t *ix) {
    if (!ix) return;
    int prev = -1;  // the tables live on the device the index was built on
    const bool switched = ix->device >= 0 && hipGetDevice(&prev) == hipSuccess && prev != ix->device &&
                          hipSetDevice(ix->device) == hipSuccess;
    if (ix->d_keys) (void)hipFree(ix->d_keys);
    if (ix->d_ids) (void)hipFree(ix->d_ids);
    if (switched) (void)hipSetDevice(prev);
    delete ix;
}

int lsh_index_tables(const lsh_index_t *ix, uint64_t *N, uint32_t *L, const uint64_t **d_sorted_keys,
                     const uint32_t **d_sorted_ids) {
    if (!ix) return LSH_ERR_INVALID_ARG;
    if (N) *N = ix->N;
    if (L) *L = ix->L;
    if (d_sorted_keys) *d_sorted_keys = ix->d_keys;
    if (d_sorted_ids) *d_sorted_ids = ix->d_ids;
    return LSH_OK;
}

int lsh_index_probe(const lsh_index_t *ix, const uint64_t *d_qkeys, uint64_t Q, uint32_t *d_start, uint32_t *d_count,
                    void *stream) {
    if (!ix) return LSH_ERR_INVALID_ARG;
    if (Q == 0) return LSH_OK;
    if (!d_qkeys || !d_start || !d_count) return LSH_ERR_INVALID_ARG;
    int rc = on_index_device(ix);
    if (rc != LSH_OK) return rc;
    const uint64_t items = Q * ix->L;
    hipLaunchKernelGGL(probe_kernel, dim3((uint32_t)((items + 255) / 256)), dim3(256), 0,
                       reinterpret_cast<hipStream_t>(stream), ix->d_keys, ix->N, ix->L, d_qkeys, items, d_start, d_count);
    return hipGetLastError() == hipSuccess ? LSH_OK : LSH_ERR_HIP;
}

int lsh_index_candidate_offsets(const uint32_t *d_count, uint64_t items, uint64_t *d_offsets, void *stream) {
    if (!d_offsets || (items && !d_count) || items >= (1ull << 31)) return LSH_ERR_INVALID_ARG;
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    uint64_t *partial = nullptr;
    int rc = LSH_OK;
    if (hipMalloc(&partial, (items / kScanBlock + 1) * sizeof(uint64_t)) != hipSuccess) rc = LSH_ERR_ALLOC;
    if (rc == LSH_OK) rc = launch_offsets_scan(d_count, items, partial, d_offsets, s);
    if (rc == LSH_OK && hipStreamSynchronize(s) != hipSuccess) rc = LSH_ERR_HIP;
    if (partial) (void)hipFree(partial);
    if (rc != LSH_OK) (void)hipGetLastError();
    return rc;
}

int lsh_index_candidate_offsets_static(const uint32_t *d_count, uint64_t items, uint64_t *d_offsets, void *stream) {
    if (!d_offsets || (items && !d_count)) return LSH_ERR_INVALID_ARG;
    if (items > kStaticScanItems) return LSH_ERR_UNSUPPORTED;
    uint64_t *partial = static_scratch();
    if (!partial) return LSH_ERR_HIP;
    return launch_offsets_scan(d_count, items, partial, d_offsets, reinterpret_cast<hipStream_t>(stream));
}

int lsh_index_candidates(const lsh_index_t *ix, const uint32_t *d_start, const uint32_t *d_count,
                         const uint64_t *d_offsets, uint64_t Q, uint32_t *d_out, void *stream) {
    if (!ix) return LSH_ERR_INVALID_ARG;
    if (Q == 0) return LSH_OK;
    if (!d_start || !d_count || !d_offsets || !d_out) return LSH_ERR_INVALID_ARG;
    int rc = on_index_device(ix);
    if (rc != LSH_OK) return rc;
    const uint64_t items = Q * ix->L;
    const uint64_t wanted = (items * 64 + 255) / 256;  // one wave per item, up to 2^20 workgroups
    hipLaunchKernelGGL(candidates_kernel, dim3((uint32_t)(wanted < (1u << 20) ? wanted : (1u << 20))), dim3(256), 0,
                       reinterpret_cast<hipStream_t>(stream), ix->d_ids, ix->N, ix->L, d_start, d_count, d_offsets, items,
                       d_out);
    return hipGetLastError() == hipSuccess ? LSH_OK : LSH_ERR_HIP;
}

static int best_candidate(bool inner, const lsh_index_t *ix, const float *d_data, const float *d_queries, uint32_t n,
                          const uint32_t *d_start, const uint32_t *d_count, uint64_t Q, uint32_t max_candidates,
                          uint32_t *d_best_id, float *d_best_score, void *stream) {
    if (!ix || !n) return LSH_ERR_INVALID_ARG;
    if (Q == 0) return LSH_OK;
    if (!d_data || !d_queries || !d_start || !d_count || !d_best_id || !d_best_score) return LSH_ERR_INVALID_ARG;
    if (Q >= (1ull << 31)) return LSH_ERR_INVALID_ARG;
    if ((uint64_t)n * 4 + 64 > 64 * 1024) return LSH_ERR_UNSUPPORTED;  // the query is kept in LDS
    int rc = on_index_device(ix);
    if (rc != LSH_OK) return rc;
    const uint32_t lds = n * 4 + 4 * 8;
    const uint32_t limit = max_candidates ? max_candidates : 0xFFFFFFFFu;
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    if (inner)
        hipLaunchKernelGGL(nearest_kernel<true>, dim3((uint32_t)Q), dim3(256), lds, s, ix->d_ids, ix->N, ix->L, d_data,
                           d_queries, n, d_start, d_count, limit, d_best_id, d_best_score);
    else
        hipLaunchKernelGGL(nearest_kernel<false>, dim3((uint32_t)Q), dim3(256), lds, s, ix->d_ids, ix->N, ix->L, d_data,
                           d_queries, n, d_start, d_count, limit, d_best_id, d_best_score);
    return hipGetLastError() == hipSuccess ? LSH_OK : LSH_ERR_HIP;
}

int lsh_index_nearest(const lsh_index_t *ix, const float *d_data, const float *d_queries, uint32_t n,
                      const uint32_t *d_start, const uint32_t *d_count, uint64_t Q, uint32_t max_candidates,
                      uint32_t *d_best_id, float *d_best_dist, void *stream) {
    return best_candidate(false, ix, d_data, d_queries, n, d_start, d_count, Q, max_candidates, d_best_id, d_best_dist,
                          stream);
}

int lsh_index_best_inner_product(const lsh_index_t *ix, const float *d_data, const float *d_queries, uint32_t n,
                                 const uint32_t *d_start, const uint32_t *d_count, uint64_t Q,
                                 uint32_t max_candidates, uint32_t *d_best_id, float *d_best_ip, void *stream) {
    return best_candidate(true, ix, d_data, d_queries, n, d_start, d_count, Q, max_candidates, d_best_id, d_best_ip,
                          stream);
}

}  // extern "C"
