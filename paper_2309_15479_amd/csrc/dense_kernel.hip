// Dense E2LSH kernel (Sec. 2.2, Eq. 1) for gfx950: P = V . A^T on the fp32 matrix cores,
// with h = floor((P + b) / w) applied to the accumulators before they leave registers.
//
//   V [N][n] row-major (vectors), A [k][n] row-major (row j = a_j): both operands are
//   contiguous along the contraction axis n.
//
// Workgroup = 256 threads (4 waves, 2 x 2), persistent; block tile 128 vectors x 128
// functions, contraction step 32.  Each wave owns 64 x 64 outputs as 2 x 2 tiles of
// v_mfma_f32_32x32x2_f32 (16 accumulator registers per tile).  Operand tiles go
// HBM/L2 -> registers -> LDS (double buffered, one barrier per step) -> registers.
//
// MFMA operand layout (32x32x2): lane l supplies A[row = l % 32][kk = l / 32] and
// B[kk = l / 32][col = l % 32]; it receives D[8*(i/4) + 4*(l/32) + i%4][l % 32] in
// accumulator register i.  The coefficients are the row operand and the vectors the column
// operand, so a lane ends up with runs of four consecutive functions of one vector: the ids
// leave as 16-byte stores (a 4-byte store per lane costs the memory pipeline as much as a
// 16-byte one, and with n = 128 the stores weigh as much as the MFMAs).  The order in which contraction indices are fed is free, so
// within a group of 8 indices lanes 0-31 take indices 0..3 and lanes 32-63 take 4..7:
// every lane then reads 4 consecutive floats (one 16-byte LDS read) per group.
#include <hip/hip_runtime.h>

#include <type_traits>

#include "lsh_internal.h"

namespace lsh {
namespace {

constexpr int BM = 128, BN = 128, BK = 32;
constexpr int LDS_STRIDE = BK + 4;  // floats; 144 B keeps 16-byte alignment, spreads banks
constexpr int kThreads = 256;

typedef float floatx16 __attribute__((ext_vector_type(16)));

struct DenseArgs {
    const float *data;  // [N][n]
    const float *a;     // [kpad][n], rows >= k are zero
    const float *off;   // [>= kpad]
    uint64_t N;
    uint32_t n, k;
    float w, inv_w;
    int w_is_pow2;
    int proj;           // 1: write raw projections (float), 0: bucket ids (int32)
    void *out;          // [N][k]
};

// 128 x 32 operand tile = 1024 float4; thread t loads float4 #t, #t+T, ... (T threads):
// row = f / 8, column group = f % 8 (8 consecutive lanes read 128 contiguous bytes).
template <bool VEC4, int T>
__device__ __forceinline__ void load_tile(const float *__restrict__ base, uint64_t row0,
                                          uint64_t row_limit, uint32_t n, uint32_t k0,
                                          float4 (&reg)[1024 / T]) {
#pragma unroll
    for (int q = 0; q < 1024 / T; ++q) {
        const int f = threadIdx.x + q * T;
        const uint64_t row = row0 + (f >> 3);
        const uint32_t col = k0 + ((f & 7) << 2);
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (row < row_limit) {
            const float *src = base + row * n + col;
            if (VEC4) {
                if (col < n) v = *reinterpret_cast<const float4 *>(src);  // n % 4 == 0
            } else {
                if (col + 0 < n) v.x = src[0];
                if (col + 1 < n) v.y = src[1];
                if (col + 2 < n) v.z = src[2];
                if (col + 3 < n) v.w = src[3];
            }
        }
        reg[q] = v;
    }
}

template <int T>
__device__ __forceinline__ void store_tile(float *lds, const float4 (&reg)[1024 / T]) {
#pragma unroll
    for (int q = 0; q < 1024 / T; ++q) {
        const int f = threadIdx.x + q * T;
        *reinterpret_cast<float4 *>(lds + (f >> 3) * LDS_STRIDE + ((f & 7) << 2)) = reg[q];
    }
}

// Persistent workgroups walk a list of (row tile, column tile) pairs.  The list is laid out
// per XCD (workgroup g runs on XCD g % 8 under round-robin dispatch): row tile r belongs to
// XCD r % 8, and the workgroups of one XCD take that XCD's pairs in order, column tile
// fastest, so the column tiles of a row tile are in flight together and share it in that
// XCD's L2.  The first contraction step of the next pair is fetched during the last step of
// the current one, so its latency hides behind the MFMAs and the epilogue.
// MI = 32-row MFMA tiles per wave along the vector axis: 2 -> 4 waves of 64 x 64 outputs,
// 1 -> 8 waves of 32 x 64 (twice the waves per CU; used for short contractions, where the
// epilogue and its stores weigh as much as the MFMAs and need other waves to hide behind).
template <bool VEC4, bool PROJ, bool POW2, int MI>
__global__ __launch_bounds__(512 / MI, MI == 1 ? 4 : 2) void dense_kernel(const DenseArgs a) {
    using OutT = typename std::conditional<PROJ, float, int32_t>::type;
    constexpr int T = 512 / MI;
    __shared__ __align__(16) float lds_a[2][BM * LDS_STRIDE];
    __shared__ __align__(16) float lds_b[2][BN * LDS_STRIDE];

    const uint32_t ntile_n = (a.k + BN - 1) / BN;
    const uint64_t ntile_m = (a.N + BM - 1) / BM;
    const uint32_t xcd = blockIdx.x % 8, slot = blockIdx.x / 8, slots = gridDim.x / 8;
    const uint64_t rows_here = ntile_m > xcd ? (ntile_m - xcd + 7) / 8 : 0;  // row tiles of this XCD
    const uint64_t items = rows_here * ntile_n;
    const uint64_t b_rows = (uint64_t)ntile_n * BN;
    const uint32_t nsteps = (a.n + BK - 1) / BK;

    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int wm = (wave >> 1) * (32 * MI), wn = (wave & 1) * 64;
    const int lr = lane & 31, lh = lane >> 5;

    floatx16 acc[MI][2];
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < 2; ++ni)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[mi][ni][i] = 0.f;

    float4 ra[1024 / T], rb[1024 / T];
    uint64_t item = slot;
    if (item >= items) return;
    uint64_t row0 = ((item / ntile_n) * 8 + xcd) * BM;
    uint32_t col0 = (uint32_t)(item % ntile_n) * BN;
    load_tile<VEC4, T>(a.data, row0, a.N, a.n, 0, ra);
    load_tile<VEC4, T>(a.a, col0, b_rows, a.n, 0, rb);
    store_tile<T>(lds_a[0], ra);
    store_tile<T>(lds_b[0], rb);
    __syncthreads();
    int cur = 0;

    while (true) {
        const uint64_t next_item = item + slots;
        const bool has_next = next_item < items;
        const uint64_t next_row0 = has_next ? ((next_item / ntile_n) * 8 + xcd) * BM : 0;
        const uint32_t next_col0 = has_next ? (uint32_t)(next_item % ntile_n) * BN : 0;
        for (uint32_t step = 0; step < nsteps; ++step) {
            const bool last = step + 1 == nsteps;
            const bool fetch = !last || has_next;
            if (fetch) {
                load_tile<VEC4, T>(a.data, last ? next_row0 : row0, a.N, a.n, last ? 0 : (step + 1) * BK, ra);
                load_tile<VEC4, T>(a.a, last ? next_col0 : col0, b_rows, a.n, last ? 0 : (step + 1) * BK, rb);
            }
            const float *la = lds_a[cur] + (wm + lr) * LDS_STRIDE + lh * 4;
            const float *lb = lds_b[cur] + (wn + lr) * LDS_STRIDE + lh * 4;
#pragma unroll
            for (int kg = 0; kg < BK / 8; ++kg) {
                float4 fa[MI], fb[2];
#pragma unroll
                for (int mi = 0; mi < MI; ++mi)
                    fa[mi] = *reinterpret_cast<const float4 *>(la + mi * 32 * LDS_STRIDE + kg * 8);
#pragma unroll
                for (int ni = 0; ni < 2; ++ni)
                    fb[ni] = *reinterpret_cast<const float4 *>(lb + ni * 32 * LDS_STRIDE + kg * 8);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
#pragma unroll
                    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                        for (int ni = 0; ni < 2; ++ni) {
                            const float av = e == 0 ? fa[mi].x : e == 1 ? fa[mi].y : e == 2 ? fa[mi].z : fa[mi].w;
                            const float bv = e == 0 ? fb[ni].x : e == 1 ? fb[ni].y : e == 2 ? fb[ni].z : fb[ni].w;
                            acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x2f32(bv, av, acc[mi][ni], 0, 0, 0);
                        }
                }
            }
            if (fetch) {
                store_tile<T>(lds_a[cur ^ 1], ra);  // the other buffer: last read before the previous barrier
                store_tile<T>(lds_b[cur ^ 1], rb);
            }
            __syncthreads();
            cur ^= 1;
            if (last) {
                // epilogue, after the barrier: the stores drain while the next pair's first step
                // computes.  The coefficient tile is the row operand of the MFMA, so register
                // 4q + t of tile (mi, ni) is function 8q + 4*lh + t of the tile for vector lr:
                // four consecutive functions per lane and one 16-byte store per register quad.
                const bool interior = row0 + BM <= a.N && col0 + BN <= a.k && (a.k & 3) == 0;
#pragma unroll
                for (int mi = 0; mi < MI; ++mi) {
                    const uint64_t row = row0 + wm + mi * 32 + lr;
                    OutT *dst_row = reinterpret_cast<OutT *>(a.out) + row * a.k;
#pragma unroll
                    for (int ni = 0; ni < 2; ++ni) {
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            const uint32_t col = col0 + wn + ni * 32 + 8 * q + 4 * lh;
                            const float4 b = *reinterpret_cast<const float4 *>(a.off + col);  // padded
                            const float bb[4] = {b.x, b.y, b.z, b.w};
                            OutT v[4];
#pragma unroll
                            for (int t = 0; t < 4; ++t) {
                                const float p = acc[mi][ni][4 * q + t];
                                acc[mi][ni][4 * q + t] = 0.f;
                                if constexpr (PROJ) {
                                    v[t] = p;
                                } else {
                                    v[t] = (int)floorf(POW2 ? (p + bb[t]) * a.inv_w : (p + bb[t]) / a.w);
                                }
                            }
                            if (interior) {
                                using Vec4 = typename std::conditional<PROJ, float4, int4>::type;
                                Vec4 w4;
                                w4.x = v[0]; w4.y = v[1]; w4.z = v[2]; w4.w = v[3];
                                *reinterpret_cast<Vec4 *>(dst_row + col) = w4;
                            } else if (row < a.N) {
#pragma unroll
                                for (int t = 0; t < 4; ++t)
                                    if (col + t < a.k) dst_row[col + t] = v[t];
                            }
                        }
                    }
                }
            }
        }
        if (!has_next) break;
        item = next_item;
        row0 = next_row0;
        col0 = next_col0;
    }
}

// Short contractions (n <= 128): with only n/32 steps per output tile the kernel above spends
// as much on operand traffic (every 16-byte load or store instruction occupies the vector
// memory pipeline for tens of cycles), LDS staging and barriers as on MFMAs.  Here a
// persistent workgroup of 8 waves owns ONE tile of 128 functions, keeps its coefficients in
// LDS for the whole launch, and walks row tiles: per row tile it loads only the 128 x n
// block of vectors (whole contraction at once; the next block is prefetched into registers
// while the current one is multiplied), so there are two barriers per 128 x 128 outputs and
// half the load instructions.  Wave tile 32 vectors x 64 functions.
constexpr int SK = 128;            // largest contraction length
constexpr int SSTRIDE = SK + 4;    // floats; 528 B: 16-byte aligned, conflict-free operand reads
constexpr int kShortNI = 1;                        // 32-function MFMA tiles per wave
constexpr int kSmallThreads = 1024 / kShortNI;      // 16 waves of 32 x 32 outputs (or 8 of 32 x 64)
constexpr int kBlockRegs = 4096 / kSmallThreads;   // float4 per thread of a 128 x 128 block

template <bool VEC4>
__device__ __forceinline__ void load_block(const float *__restrict__ base, uint64_t row0, uint64_t row_limit,
                                           uint32_t n, float4 (&reg)[kBlockRegs]) {
#pragma unroll
    for (int q = 0; q < kBlockRegs; ++q) {
        const int f = threadIdx.x + q * kSmallThreads;  // 128 rows x 32 chunks of 4 floats
        const uint64_t row = row0 + (f >> 5);
        const uint32_t col = (f & 31) << 2;
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (row < row_limit) {
            const float *src = base + row * n + col;
            if (VEC4) {
                if (col < n) v = *reinterpret_cast<const float4 *>(src);
            } else {
                if (col + 0 < n) v.x = src[0];
                if (col + 1 < n) v.y = src[1];
                if (col + 2 < n) v.z = src[2];
                if (col + 3 < n) v.w = src[3];
            }
        }
        reg[q] = v;
    }
}

template <bool VEC4>
__device__ __forceinline__ void load_block_part(const float *__restrict__ base, uint64_t row0, uint64_t row_limit,
                                                uint32_t n, float4 (&reg)[kBlockRegs], int q) {
    const int f = threadIdx.x + q * kSmallThreads;
    const uint64_t row = row0 + (f >> 5);
    const uint32_t col = (f & 31) << 2;
    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
    if (row < row_limit) {
        const float *src = base + row * n + col;
        if (VEC4) {
            if (col < n) v = *reinterpret_cast<const float4 *>(src);
        } else {
            if (col + 0 < n) v.x = src[0];
            if (col + 1 < n) v.y = src[1];
            if (col + 2 < n) v.z = src[2];
            if (col + 3 < n) v.w = src[3];
        }
    }
    reg[q] = v;
}

__device__ __forceinline__ void store_block(float *lds, const float4 (&reg)[kBlockRegs]) {
#pragma unroll
    for (int q = 0; q < kBlockRegs; ++q) {
        const int f = threadIdx.x + q * kSmallThreads;
        *reinterpret_cast<float4 *>(lds + (f >> 5) * SSTRIDE + ((f & 31) << 2)) = reg[q];
    }
}

template <bool VEC4, bool PROJ, bool POW2>
__global__ __launch_bounds__(kSmallThreads) void dense_short_kernel(const DenseArgs a) {
    using OutT = typename std::conditional<PROJ, float, int32_t>::type;
    static_assert(kShortNI == 1, "one 32 x 32 MFMA tile per wave");
    extern __shared__ __align__(16) float lds[];
    float *lds_b = lds;                   // [128 functions][SSTRIDE]
    float *lds_a = lds + BN * SSTRIDE;    // [128 vectors][SSTRIDE]

    const uint32_t ntile_n = (a.k + BN - 1) / BN;
    const uint64_t ntile_m = (a.N + BM - 1) / BM;
    const uint32_t xcd = blockIdx.x % 8, slot = blockIdx.x / 8, slots = gridDim.x / 8;
    const uint32_t ct = slot % ntile_n;                       // this workgroup's function tile
    const uint64_t stream = slot / ntile_n, streams = slots / ntile_n;
    if (stream >= streams) return;
    const uint32_t col0 = ct * BN;
    const uint32_t groups = (a.n + 7) / 8;                    // groups of 8 contraction indices

    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    constexpr int WN = BN / 32;
    const int wm = (wave / WN) * 32, wn = (wave % WN) * 32;
    const int lr = lane & 31, lh = lane >> 5;

    float4 r[kBlockRegs];
    load_block<VEC4>(a.a, col0, (uint64_t)ntile_n * BN, a.n, r);   // coefficient rows are padded
    store_block(lds_b, r);

    // row tiles of this stream: xcd + 8 * (stream + t * streams)
    const uint64_t stride = 8 * streams;
    uint64_t rt = xcd + 8 * stream;
    if (rt < ntile_m) load_block<VEC4>(a.data, rt * BM, a.N, a.n, r);

    // One quad of the epilogue: registers 4q..4q+3 of the accumulator are functions
    // 8q + 4*lh .. + 3 of the wave's 32, for vector lr; one 16-byte store.
    const bool k_vec = (a.k & 3) == 0 && col0 + BN <= a.k;
    // The offsets of the lane's 16 functions stay in registers: a load inside the tile loop
    // would have to be waited for with vmcnt(0), which also waits for the id stores issued
    // just before it, i.e. for a full trip to HBM, four times per tile.
    float4 bq[4];
#pragma unroll
    for (int q = 0; q < 4; ++q)
        bq[q] = *reinterpret_cast<const float4 *>(a.off + col0 + wn + 8 * q + 4 * lh);  // padded
    auto finish_quad = [&](const floatx16 &acc, int q, uint64_t tile) {
        const uint64_t row0 = tile * BM;
        const uint64_t row = row0 + wm + lr;
        OutT *dst_row = reinterpret_cast<OutT *>(a.out) + row * a.k;
        const uint32_t col = col0 + wn + 8 * q + 4 * lh;
        const float bb[4] = {bq[q].x, bq[q].y, bq[q].z, bq[q].w};
        OutT v[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const float p = acc[4 * q + t];
            if constexpr (PROJ) {
                v[t] = p;
            } else {
                v[t] = (int)floorf(POW2 ? (p + bb[t]) * a.inv_w : (p + bb[t]) / a.w);
            }
        }
        if (k_vec && row0 + BM <= a.N) {
            using Vec4 = typename std::conditional<PROJ, float4, int4>::type;
            Vec4 w4;
            w4.x = v[0]; w4.y = v[1]; w4.z = v[2]; w4.w = v[3];
            *reinterpret_cast<Vec4 *>(dst_row + col) = w4;
        } else if (row < a.N) {
#pragma unroll
            for (int t = 0; t < 4; ++t)
                if (col + t < a.k) dst_row[col + t] = v[t];
        }
    };

    floatx16 acc, done;
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = done[i] = 0.f;
    bool have_done = false;
    uint64_t done_tile = 0;

    for (; rt < ntile_m; rt += stride) {
        __syncthreads();  // everyone is done with the previous block of vectors
        store_block(lds_a, r);
        __syncthreads();
        const bool more = rt + stride < ntile_m;
        const float *la = lds_a + (wm + lr) * SSTRIDE + lh * 4;
        const float *lb = lds_b + (wn + lr) * SSTRIDE + lh * 4;
        // The memory work of a tile is spread over its contraction steps instead of coming in
        // bursts: the previous tile's four stores go out during steps 0..3, the next block's
        // loads during the later steps.  All CUs run the same program on equal tiles and stay
        // in step, so bursts would leave HBM idle during the MFMA phases and the MFMAs idle
        // during the bursts.
#pragma unroll
        for (int kg = 0; kg < SK / 8; ++kg) {
            if (kg < (int)groups) {
                const float4 fa = *reinterpret_cast<const float4 *>(la + kg * 8);
                const float4 fb = *reinterpret_cast<const float4 *>(lb + kg * 8);
                acc = __builtin_amdgcn_mfma_f32_32x32x2f32(fb.x, fa.x, acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_32x32x2f32(fb.y, fa.y, acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_32x32x2f32(fb.z, fa.z, acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_32x32x2f32(fb.w, fa.w, acc, 0, 0, 0);
            }
            if (kg < 4 && have_done) finish_quad(done, kg, done_tile);
            constexpr int kFirstLoad = 5, kLoadEvery = (SK / 8 - kFirstLoad) / kBlockRegs;
            if (more && kg >= kFirstLoad && (kg - kFirstLoad) % kLoadEvery == 0 &&
                (kg - kFirstLoad) / kLoadEvery < kBlockRegs)
                load_block_part<VEC4>(a.data, (rt + stride) * BM, a.N, a.n, r, (kg - kFirstLoad) / kLoadEvery);
        }
        done = acc;
        done_tile = rt;
        have_done = true;
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[i] = 0.f;
    }
    if (have_done) {
#pragma unroll
        for (int q = 0; q < 4; ++q) finish_quad(done, q, done_tile);
    }
}


// The same persistent scheme for the plain case n == 128, k a multiple of 128, stripped of
// per-tile vector-ALU work.  On this part a vector-ALU instruction and an MFMA of the same SIMD
// do not overlap (the co-execution counter reads 0), so every address computation, predicate
// or register copy in the tile loop is taken from the matrix pipe: the 120 such instructions
// per wave and tile of the general kernel cost it a tenth of its time.  Here the loads and
// stores use a uniform tile pointer (scalar registers) plus a per-lane byte offset that never
// changes, LDS accesses use immediate offsets, and the epilogue is one FMA and one
// floor-convert per output (b~ / w is folded into the FMA's addend).  Only the last, partial
// row tile takes predicated accesses.
template <bool PROJ, bool POW2>
__global__ __launch_bounds__(kSmallThreads) void dense_lean_kernel(const DenseArgs a) {
    using OutT = typename std::conditional<PROJ, float, int32_t>::type;
    using Vec4 = typename std::conditional<PROJ, float4, int4>::type;
    static_assert(sizeof(OutT) == 4, "ids and projections are 4 bytes");
    extern __shared__ __align__(16) float lds[];
    float *lds_b = lds;                 // [128 functions][SSTRIDE]
    float *lds_a = lds + BN * SSTRIDE;  // [128 vectors][SSTRIDE]

    const uint32_t ntile_n = a.k / BN;
    const uint64_t ntile_m = (a.N + BM - 1) / BM, full_m = a.N / BM;
    const uint32_t xcd = blockIdx.x % 8, slot = blockIdx.x / 8, slots = gridDim.x / 8;
    const uint32_t ct = slot % ntile_n;
    const uint64_t stream = slot / ntile_n, streams = slots / ntile_n;
    if (stream >= streams) return;
    const uint32_t col0 = ct * BN;

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = (wave / (BN / 32)) * 32, wn = (wave % (BN / 32)) * 32;
    const int lr = lane & 31, lh = lane >> 5;

    // per-lane byte offsets, constant for the whole launch
    const uint32_t ld_off = (threadIdx.x >> 5) * (SK * 4) + (threadIdx.x & 31) * 16;   // in a 128 x 128 block of floats
    float *const lw = lds_a + (threadIdx.x >> 5) * SSTRIDE + (threadIdx.x & 31) * 4;     // + q * 32 rows
    const uint32_t st_off = ((uint32_t)(wm + lr) * a.k + col0 + wn + 4 * lh) * 4;        // in a 128 x k block of outputs; + 32 q
    const float *la = lds_a + (wm + lr) * SSTRIDE + lh * 4;
    const float *lb = lds_b + (wn + lr) * SSTRIDE + lh * 4;
    const char *const data = reinterpret_cast<const char *>(a.data);
    char *const out = reinterpret_cast<char *>(a.out);

    float4 r[kBlockRegs];
    // One 16-byte piece of a block of vectors.  FULL: the tile has all its 128 rows, the address
    // is the uniform tile pointer plus the lane's constant offset; otherwise rows beyond N read
    // row N - 1 (computed, never stored).
    auto fetch = [&](auto full_tag, uint64_t tile, int q) -> float4 {
        if constexpr (decltype(full_tag)::value) {
            return *reinterpret_cast<const float4 *>(data + tile * (uint64_t)(BM * SK * 4) + (ld_off + q * 32 * SK * 4));
        } else {
            uint64_t row = tile * BM + (threadIdx.x >> 5) + q * 32;
            row = row < a.N ? row : a.N - 1;
            return *reinterpret_cast<const float4 *>(data + row * (SK * 4) + (threadIdx.x & 31) * 16);
        }
    };

    // coefficient tile, resident for the whole launch (rows padded to the tile grid)
#pragma unroll
    for (int q = 0; q < kBlockRegs; ++q)
        r[q] = *reinterpret_cast<const float4 *>(reinterpret_cast<const char *>(a.a) + (uint64_t)col0 * (SK * 4) +
                                                 (ld_off + q * 32 * SK * 4));
#pragma unroll
    for (int q = 0; q < kBlockRegs; ++q)
        *reinterpret_cast<float4 *>(lds_b + (threadIdx.x >> 5) * SSTRIDE + (threadIdx.x & 31) * 4 + q * 32 * SSTRIDE) = r[q];

    // epilogue constants: accumulator register 4q + t is function col0 + wn + 8q + 4 lh + t
    float bs[16];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const float4 b = *reinterpret_cast<const float4 *>(a.off + col0 + wn + 8 * q + 4 * lh);
        bs[4 * q + 0] = POW2 ? b.x * a.inv_w : b.x;
        bs[4 * q + 1] = POW2 ? b.y * a.inv_w : b.y;
        bs[4 * q + 2] = POW2 ? b.z * a.inv_w : b.z;
        bs[4 * q + 3] = POW2 ? b.w * a.inv_w : b.w;
    }
#pragma unroll
    for (int i = 0; i < 16; ++i) asm volatile("" : "+v"(bs[i]));  // held in registers, not recomputed per tile

    const uint64_t stride = 8 * streams;
    uint64_t rt = xcd + 8 * stream;
    if (rt < full_m) {
#pragma unroll
        for (int q = 0; q < kBlockRegs; ++q) r[q] = fetch(std::true_type{}, rt, q);
    }

    OutT res[16];  // finished outputs of the previous tile; their stores go out during the next tile
    uint64_t done_tile = 0;
    auto store_quad = [&](auto full_tag, int q) {
        Vec4 w4;
        w4.x = res[4 * q + 0]; w4.y = res[4 * q + 1]; w4.z = res[4 * q + 2]; w4.w = res[4 * q + 3];
        char *dst = out + done_tile * ((uint64_t)BM * 4) * a.k + (st_off + 32 * q);
        if (decltype(full_tag)::value || done_tile * BM + wm + lr < a.N) *reinterpret_cast<Vec4 *>(dst) = w4;
    };

    // LDS hand-over: the block of vectors in `r` replaces the one in LDS.
    auto hand_over = [&]() {
        __syncthreads();  // everyone is done with the previous block of vectors
#pragma unroll
        for (int q = 0; q < kBlockRegs; ++q) *reinterpret_cast<float4 *>(lw + q * 32 * SSTRIDE) = r[q];
        __syncthreads();
    };

    // One tile: 16 contraction steps with the memory work spread between them, then the epilogue
    // arithmetic into `res`.  The next block's four loads go out during steps 0..3 (they have the
    // rest of the tile to arrive), the previous tile's four stores during steps 5, 7, 9, 11; the
    // hand-over that follows waits for the loads only (the counter of outstanding memory
    // operations is in order, and the stores were issued after them).  FULL: a tile of the main
    // loop, which has all its rows and prefetches full tiles only; the partial last tile runs
    // the other instantiation once, after the loop.  STORE: there is a previous tile to store.
    auto run_tile = [&](auto full_tag, auto store_tag) {
        constexpr bool FULL = decltype(full_tag)::value, STORE = decltype(store_tag)::value;
        const uint64_t next = rt + stride;
        const bool more = FULL && next < full_m;
        floatx16 acc;
        // The operands of step kg + 1 are read from LDS before the MFMAs of step kg are issued:
        // the four waves of a SIMD run in step, so a read issued only after a wave's MFMAs
        // would find all of them waiting for LDS at the same time, with the matrix pipe idle.
        float4 fa[2], fb[2];
        fa[0] = *reinterpret_cast<const float4 *>(la);
        fb[0] = *reinterpret_cast<const float4 *>(lb);
#pragma unroll
        for (int kg = 0; kg < SK / 8; ++kg) {
            if (kg + 1 < SK / 8) {
                fa[(kg + 1) & 1] = *reinterpret_cast<const float4 *>(la + (kg + 1) * 8);
                fb[(kg + 1) & 1] = *reinterpret_cast<const float4 *>(lb + (kg + 1) * 8);
            }
            __builtin_amdgcn_sched_barrier(0);
            const float4 xa = fa[kg & 1], xb = fb[kg & 1];
            if (kg == 0) {
                const floatx16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
                acc = __builtin_amdgcn_mfma_f32_32x32x2f32(xb.x, xa.x, zero, 0, 0, 0);
            } else {
                acc = __builtin_amdgcn_mfma_f32_32x32x2f32(xb.x, xa.x, acc, 0, 0, 0);
            }
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(xb.y, xa.y, acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(xb.z, xa.z, acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(xb.w, xa.w, acc, 0, 0, 0);
            if constexpr (FULL) {
                if (more && kg == 0) r[0] = fetch(full_tag, next, 0);
                if (more && kg == 1) r[1] = fetch(full_tag, next, 1);
                if (more && kg == 2) r[2] = fetch(full_tag, next, 2);
                if (more && kg == 3) r[3] = fetch(full_tag, next, 3);
            }
            if constexpr (STORE) {
                if (kg >= 5 && kg <= 11 && (kg & 1)) store_quad(full_tag, (kg - 5) >> 1);  // in a FULL pass the previous tile was a full one
            }
            __builtin_amdgcn_sched_barrier(0);  // keeps the memory instructions at their steps
        }
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            if constexpr (PROJ) {
                res[i] = acc[i];
            } else if constexpr (POW2) {
                res[i] = (int)floorf(fmaf(acc[i], a.inv_w, bs[i]));
            } else {
                res[i] = (int)floorf((acc[i] + bs[i]) / a.w);
            }
        }
        done_tile = rt;
    };

    bool have_done = false;
    if (rt < full_m) {
        hand_over();
        run_tile(std::true_type{}, std::false_type{});  // first tile: nothing to store yet
        have_done = true;
        rt += stride;
        if (rt < full_m) {
            hand_over();
            // the hand-over sits at the end of the loop body, after the body's loads and stores in
            // straight-line code: at the top of the loop it would also be reached from the first
            // tile, which has no stores after its loads, and would have to wait for everything
            while (true) {
                run_tile(std::true_type{}, std::true_type{});
                rt += stride;
                if (rt >= full_m) break;
                hand_over();
            }
        }
    }
    if (rt < ntile_m) {  // the partial tile, if it is this workgroup's
#pragma unroll
        for (int q = 0; q < kBlockRegs; ++q) r[q] = fetch(std::false_type{}, rt, q);
        hand_over();
        if (have_done) run_tile(std::false_type{}, std::true_type{}); else run_tile(std::false_type{}, std::false_type{});
        have_done = true;
    }
    if (have_done) {
#pragma unroll
        for (int q = 0; q < 4; ++q) store_quad(std::false_type{}, q);
    }
}

}  // namespace

uint32_t dense_col_tile() { return BN; }

int launch_dense(const lsh_params *p, bool proj, const float *d_data, uint64_t N, void *d_out,
                 void *stream) {
    DenseArgs a;
    a.data = d_data;
    a.a = p->d_dense;
    a.off = p->d_off;
    a.N = N;
    a.n = p->n;
    a.k = p->k;
    a.w = p->w;
    a.inv_w = 1.0f / p->w;
    int exp2 = 0;
    a.w_is_pow2 = (std::frexp(p->w, &exp2) == 0.5f) ? 1 : 0;
    a.proj = proj ? 1 : 0;
    a.out = d_out;
    const uint64_t tiles_m = (N + BM - 1) / BM;
    const uint64_t tiles_n = (p->k + BN - 1) / BN;
    // persistent grid: two workgroups per CU (LDS and registers allow two), a multiple of 8
    uint64_t blocks = (uint64_t)(p->num_cus > 0 ? p->num_cus : 256) * 2 / 8 * 8;
    const uint64_t most = (tiles_m + 7) / 8 * tiles_n * 8;  // no XCD has more pairs than this / 8
    if (blocks > most) blocks = most;
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    const bool vec4 = p->n % 4 == 0;
    if (p->n <= (uint32_t)SK) {
        // one workgroup per CU (135 KB of LDS); every XCD needs at least one workgroup per
        // function tile
        const uint32_t lds_bytes = 2 * BN * SSTRIDE * sizeof(float);
        uint32_t wgs = (uint32_t)(p->num_cus > 0 ? p->num_cus : 256) / 8 * 8;
        while (wgs / 8 < tiles_n) wgs += 8;
        const dim3 g2(wgs), b2(kSmallThreads);
        const bool pw = a.w_is_pow2 != 0;
        if (p->n == (uint32_t)SK && p->k % BN == 0 && (uint64_t)p->k * BM * 4 < (1ull << 32)) {
#define LSH_LEAN_CASE(P_, W_) \
    if (proj == P_ && pw == W_) { \
        auto fn = &dense_lean_kernel<P_, W_>; \
        if (ensure_lds_limit(reinterpret_cast<const void *>(fn), lds_bytes) != LSH_OK) return LSH_ERR_HIP; \
        hipLaunchKernelGGL(fn, g2, b2, lds_bytes, s, a); \
    }
            LSH_LEAN_CASE(false, true) LSH_LEAN_CASE(false, false) LSH_LEAN_CASE(true, true) LSH_LEAN_CASE(true, false)
#undef LSH_LEAN_CASE
            return hipGetLastError() == hipSuccess ? LSH_OK : LSH_ERR_HIP;
        }
#define LSH_SHORT_CASE(V_, P_, W_) \
    if (vec4 == V_ && proj == P_ && pw == W_) { \
        auto fn = &dense_short_kernel<V_, P_, W_>; \
        if (ensure_lds_limit(reinterpret_cast<const void *>(fn), lds_bytes) != LSH_OK) return LSH_ERR_HIP; \
        hipLaunchKernelGGL(fn, g2, b2, lds_bytes, s, a); \
    }
        LSH_SHORT_CASE(true, false, true) LSH_SHORT_CASE(true, false, false)
        LSH_SHORT_CASE(false, false, true) LSH_SHORT_CASE(false, false, false)
        LSH_SHORT_CASE(true, true, true) LSH_SHORT_CASE(false, true, true)
        LSH_SHORT_CASE(true, true, false) LSH_SHORT_CASE(false, true, false)
#undef LSH_SHORT_CASE
        return hipGetLastError() == hipSuccess ? LSH_OK : LSH_ERR_HIP;
    }
    const int mi = 2;
    const dim3 grid((uint32_t)blocks), block(512 / mi);
#define LSH_DENSE_CASE(V_, P_, W_) \
    if (vec4 == V_ && proj == P_ && (a.w_is_pow2 != 0) == W_) { \
        if (mi == 1) hipLaunchKernelGGL((dense_kernel<V_, P_, W_, 1>), grid, block, 0, s, a); \
        else hipLaunchKernelGGL((dense_kernel<V_, P_, W_, 2>), grid, block, 0, s, a); \
    }
    LSH_DENSE_CASE(true, false, true) LSH_DENSE_CASE(true, false, false)
    LSH_DENSE_CASE(false, false, true) LSH_DENSE_CASE(false, false, false)
    LSH_DENSE_CASE(true, true, true) LSH_DENSE_CASE(false, true, true)
    LSH_DENSE_CASE(true, true, false) LSH_DENSE_CASE(false, true, false)
#undef LSH_DENSE_CASE
    return hipGetLastError() == hipSuccess ? LSH_OK : LSH_ERR_HIP;
}

}  // namespace lsh
