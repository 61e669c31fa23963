// Dense E2LSH kernel (Sec. 2.2, Eq. 1) for gfx950: P = V . A^T on the fp32 matrix cores,
// with h = floor((P + b) / w) applied to the accumulators before they leave registers.
//
//   V [N][n] row-major (vectors), A [k][n] row-major (row j = a_j): both operands are
//   contiguous along the contraction axis n.
//
// Workgroup = 256 threads (4 waves, 2 x 2), block tile 128 vectors x 128 functions,
// contraction step 32.  Each wave owns 64 x 64 outputs as 2 x 2 tiles of
// v_mfma_f32_32x32x2_f32 (16 accumulator registers per tile).  Operand tiles go
// HBM/L2 -> registers -> LDS (double buffered, one barrier per step) -> registers.
//
// MFMA operand layout (32x32x2): lane l supplies A[row = l % 32][kk = l / 32] and
// B[kk = l / 32][col = l % 32]; it receives D[8*(i/4) + 4*(l/32) + i%4][l % 32] in
// accumulator register i.  The order in which contraction indices are fed is free, so
// within a group of 8 indices lanes 0-31 take indices 0..3 and lanes 32-63 take 4..7:
// every lane then reads 4 consecutive floats (one 16-byte LDS read) per group.
#include <hip/hip_runtime.h>

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

// 128 x 32 operand tile = 1024 float4; thread t loads float4 #t, #t+256, #t+512, #t+768:
// row = f / 8, column group = f % 8 (8 consecutive lanes read 128 contiguous bytes).
template <bool VEC4>
__device__ __forceinline__ void load_tile(const float *__restrict__ base, uint64_t row0,
                                          uint64_t row_limit, uint32_t n, uint32_t k0,
                                          float4 (&reg)[4]) {
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int f = threadIdx.x + q * kThreads;
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

__device__ __forceinline__ void store_tile(float *lds, const float4 (&reg)[4]) {
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int f = threadIdx.x + q * kThreads;
        *reinterpret_cast<float4 *>(lds + (f >> 3) * LDS_STRIDE + ((f & 7) << 2)) = reg[q];
    }
}

template <bool VEC4>
__global__ __launch_bounds__(kThreads) void dense_kernel(const DenseArgs a) {
    __shared__ __align__(16) float lds_a[2][BM * LDS_STRIDE];
    __shared__ __align__(16) float lds_b[2][BN * LDS_STRIDE];

    // blockIdx.x walks the function tiles fastest: consecutive workgroups share the
    // vector tile (and the whole coefficient matrix stays in L2)
    const uint32_t ntile_n = (a.k + BN - 1) / BN;
    const uint64_t tile_m = blockIdx.x / ntile_n;
    const uint32_t tile_n = blockIdx.x % ntile_n;
    const uint64_t row0 = tile_m * BM;
    const uint32_t col0 = tile_n * BN;

    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int wm = (wave >> 1) * 64, wn = (wave & 1) * 64;
    const int lr = lane & 31, lh = lane >> 5;

    floatx16 acc[2][2];
#pragma unroll
    for (int mi = 0; mi < 2; ++mi)
#pragma unroll
        for (int ni = 0; ni < 2; ++ni)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[mi][ni][i] = 0.f;

    float4 ra[4], rb[4];
    const uint32_t nsteps = (a.n + BK - 1) / BK;
    const uint64_t b_rows = (uint64_t)ntile_n * BN;
    load_tile<VEC4>(a.data, row0, a.N, a.n, 0, ra);
    load_tile<VEC4>(a.a, col0, b_rows, a.n, 0, rb);
    store_tile(lds_a[0], ra);
    store_tile(lds_b[0], rb);
    __syncthreads();

    for (uint32_t step = 0; step < nsteps; ++step) {
        const int cur = step & 1;
        if (step + 1 < nsteps) {
            load_tile<VEC4>(a.data, row0, a.N, a.n, (step + 1) * BK, ra);
            load_tile<VEC4>(a.a, col0, b_rows, a.n, (step + 1) * BK, rb);
        }
        const float *la = lds_a[cur] + (wm + lr) * LDS_STRIDE + lh * 4;
        const float *lb = lds_b[cur] + (wn + lr) * LDS_STRIDE + lh * 4;
#pragma unroll
        for (int kg = 0; kg < BK / 8; ++kg) {
            float4 fa[2], fb[2];
#pragma unroll
            for (int mi = 0; mi < 2; ++mi)
                fa[mi] = *reinterpret_cast<const float4 *>(la + mi * 32 * LDS_STRIDE + kg * 8);
#pragma unroll
            for (int ni = 0; ni < 2; ++ni)
                fb[ni] = *reinterpret_cast<const float4 *>(lb + ni * 32 * LDS_STRIDE + kg * 8);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
#pragma unroll
                for (int mi = 0; mi < 2; ++mi)
#pragma unroll
                    for (int ni = 0; ni < 2; ++ni) {
                        const float av = e == 0 ? fa[mi].x : e == 1 ? fa[mi].y : e == 2 ? fa[mi].z : fa[mi].w;
                        const float bv = e == 0 ? fb[ni].x : e == 1 ? fb[ni].y : e == 2 ? fb[ni].z : fb[ni].w;
                        acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x2f32(av, bv, acc[mi][ni], 0, 0, 0);
                    }
            }
        }
        if (step + 1 < nsteps) {
            store_tile(lds_a[cur ^ 1], ra);  // the other buffer: last read before the previous barrier
            store_tile(lds_b[cur ^ 1], rb);
        }
        __syncthreads();
    }

    // epilogue: accumulator i of tile (mi, ni) is output row 8*(i/4) + 4*lh + i%4, column lr
#pragma unroll
    for (int ni = 0; ni < 2; ++ni) {
        const uint32_t col = col0 + wn + ni * 32 + lr;
        const bool col_ok = col < a.k;
        const float b = a.off[col];  // padded to the tile grid
#pragma unroll
        for (int mi = 0; mi < 2; ++mi) {
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const uint64_t row = row0 + wm + mi * 32 + 8 * (i >> 2) + 4 * lh + (i & 3);
                if (!col_ok || row >= a.N) continue;
                const float p = acc[mi][ni][i];
                if (a.proj) {
                    reinterpret_cast<float *>(a.out)[row * a.k + col] = p;
                } else {
                    const float q = a.w_is_pow2 ? (p + b) * a.inv_w : (p + b) / a.w;
                    reinterpret_cast<int32_t *>(a.out)[row * a.k + col] = (int)floorf(q);
                }
            }
        }
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
    const uint64_t blocks = tiles_m * tiles_n;
    if (blocks > 0x7fffffffull) return LSH_ERR_UNSUPPORTED;
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    if (p->n % 4 == 0)
        hipLaunchKernelGGL(dense_kernel<true>, dim3((uint32_t)blocks), dim3(kThreads), 0, s, a);
    else
        hipLaunchKernelGGL(dense_kernel<false>, dim3((uint32_t)blocks), dim3(kThreads), 0, s, a);
    return hipGetLastError() == hipSuccess ? LSH_OK : LSH_ERR_HIP;
}

}  // namespace lsh
