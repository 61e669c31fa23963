// Dense E2LSH projections (Sec. 2.2, Eq. 1) for any dimension n on the bf16 matrix cores of
// gfx950, with fp32 accuracy: P = V A^T from exact three-way bf16 splits of both operands and
// the six products of weight >= 2^-16 (see dense_split_kernel.hip for the arithmetic and its
// error: what is left out is below 2^-23 of each term |a_i v_i|).  The fp32 MFMA runs at a
// sixteenth of the bf16 rate, so six bf16 products are 16/6 of its speed at best.
//
//   V [N][n] fp32 row-major; A already split on the host into three bf16 planes, stored in the
//   order of use: [function tile of 256][stage of 16 coordinates][plane][row][coordinate]
//   (zero rows up to a multiple of 256, zero columns up to a multiple of 16).
//
// Workgroup = 4 waves, one per SIMD; tile = 256 functions x 256 vectors, contraction in stages
// of 16 coordinates.  A wave owns 128 functions x 128 vectors: 4 x 4 blocks of
// v_mfma_f32_32x32x16_bf16, 256 accumulator registers (functions are the row operand, so an
// accumulator lane holds runs of four consecutive functions of one vector).  The large tile is
// what counts: the time of this kernel follows the instructions that bring operands in (global
// loads, LDS writes, LDS reads) per multiply-add, and a 128 x 128 wave tile needs half as many
// as a 64 x 64 one.  Per stage a thread brings 16 bytes of four vector rows (4 fp32 each,
// split here on their way to LDS) and 16 bytes of each plane of two coefficient rows (8 bf16);
// LDS holds three stages, [plane][row][32 bytes], the two 16-byte halves of a row swapped in
// rows whose number has bit 3 set, which makes the 16-byte operand reads of 32 consecutive rows
// (and the writes) conflict-free without padding.  While stage s is contracted, the operand
// registers it has finished with are refilled from stage s + 1, stage s + 2 is written to LDS
// and the loads of stage s + 3 go out into the registers just stored (one set: a stage is 96
// MFMAs per wave, about 1.8 us).  With one wave per SIMD nothing else hides what a wave
// issues between two MFMAs, so the stage is written out MFMA by MFMA with at most one memory
// instruction or the split of one vector element after each (scheduling barriers keep that
// order); one LDS-only barrier per stage.
//
// Placement: workgroup g runs on XCD g % 8.  XCD x takes the vector tiles x, x + 8, ...; the
// F function tiles of a vector tile go to F workgroups of that XCD, which walk the stages in
// step, so a vector stage is fetched into the XCD's L2 once and the other F - 1 workgroups hit
// there; a workgroup keeps its function tile for all its vector tiles, and the workgroups of
// an XCD that have the same one (workgroups per XCD / F of them) share its stages in L2, too.
// (With a number of function tiles that does not divide the workgroups of an XCD: function
// tiles dealt to the XCDs, every XCD walking all vectors.)
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstring>
#include <type_traits>
#include <utility>
#include <vector>

#include "device_utils.h"
#include "lsh_internal.h"

namespace lsh {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef uint32_t uintx4 __attribute__((ext_vector_type(4)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr int TF = 256;    // functions per tile
constexpr int TVW = 256;   // vectors per tile
constexpr int NB = 4;      // 32 x 32 blocks of a wave along either axis: a wave owns 128 functions x 128 vectors
constexpr int KB = 16;     // coordinates per stage = one MFMA step
constexpr int ROWB = 32;   // bytes per row and plane in a stage: two 16-byte halves, swapped in rows with bit 3 set
constexpr int A_PLANE = TF * ROWB, V_PLANE = TVW * ROWB;
constexpr int STAGE = 3 * (A_PLANE + V_PLANE);  // 49152 bytes
constexpr int kThreadsW = 256;
constexpr int kStagePlanes = 3 * TF * KB;  // bf16 elements of one function tile's three planes in one stage
constexpr int kLdsBytesW = 3 * STAGE;

struct WideArgs {
    const float *data;       // [N][n]
    const uint16_t *planes;  // [kpad / 256][npad / 16][3][256][16] bf16 bit patterns
    const float *off;        // [>= kpad]
    uint64_t N;
    uint32_t n, npad, k, kpad;
    float w, inv_w;
    void *out;               // [N][k]
};

// x = x1 + x2 + x3 exactly, each a bf16 (round to nearest even)
__device__ __forceinline__ void split3(float x, __bf16 &x1, __bf16 &x2, __bf16 &x3) {
    x1 = (__bf16)x;
    const float r1 = x - (float)x1;
    x2 = (__bf16)r1;
    x3 = (__bf16)(r1 - (float)x2);
}

// PROJ: raw projections instead of bucket ids.  POW2: w is a power of two (fma(p, 1/w, b/w) is
// then the same float as (p + b) / w).  VEC: k is a multiple of 4 (16-byte stores).
template <bool PROJ, bool POW2, bool VEC>
__global__ __launch_bounds__(kThreadsW) void dense_split_wide_kernel(const WideArgs a) {
    extern __shared__ __align__(16) char lds_w[];  // 3 stages x ([3][256][32] coefficients, [3][256][32] vectors)
    const uint32_t lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint32_t lr = lane & 31, lh = lane >> 5;
    const uint32_t fw = wave & 1, vw = wave >> 1;  // the wave's half of the functions, half of the vectors

    // which (function tile, vector tile) pairs this workgroup takes
    const uint32_t F = a.kpad / TF;
    const uint64_t Vt = (a.N + TVW - 1) / TVW;
    const uint32_t x = blockIdx.x & 7, i = blockIdx.x >> 3, per_xcd = gridDim.x >> 3;
    uint32_t ft_first, ft_step, reps, rep;
    if (F >= 8) {
        ft_first = x; ft_step = 8; reps = 1; rep = 0;
    } else {
        ft_first = x % F; ft_step = F;  // one function tile per XCD
        reps = (8 - ft_first + F - 1) / F;  // XCDs that share it
        rep = x / F;
    }

    // loading roles: 16 bytes of the vector tile and of each coefficient plane per stage
    const uint32_t vr = threadIdx.x >> 2, vq = threadIdx.x & 3;  // vector rows vr + 64 h (h < 4), 4-coordinate piece
    const uint32_t ar = threadIdx.x >> 1, ah = threadIdx.x & 1;  // coefficient rows ar and ar + 128, 8-coordinate half
    const uint32_t stages = a.npad / KB;

    // operand read and write offsets inside a stage (half h of row r sits at 16 * (h ^ bit 3 of r))
    const uint32_t rd_a = (fw * 32 * NB + lr) * ROWB + ((lh ^ ((lr >> 3) & 1)) << 4);                // + rb * 32 rows + plane
    const uint32_t rd_v = 3 * A_PLANE + (vw * 32 * NB + lr) * ROWB + ((lh ^ ((lr >> 3) & 1)) << 4);  // + cb * 32 rows + plane
    const uint32_t wr_a = ar * ROWB + ((ah ^ ((ar >> 3) & 1)) << 4);
    const uint32_t wr_v = 3 * A_PLANE + vr * ROWB + (((vq >> 1) ^ ((vr >> 3) & 1)) << 4) + ((vq & 1) << 3);

    // When the number of function tiles divides an XCD's workgroups (the usual case), XCD x
    // takes the vector tiles x, x + 8, ... and F of its workgroups contract one of them at the
    // same time, each with its own function tile: the vector tile is then fetched into that
    // XCD's L2 once instead of once per XCD.
    const bool by_vector = per_xcd % F == 0 && F <= per_xcd;
    uint64_t vt_first = (uint64_t)i * reps + rep, vt_step = (uint64_t)per_xcd * reps;
    if (by_vector) {
        ft_first = i % F;
        ft_step = F;  // one function tile per workgroup
        const uint32_t groups = per_xcd / F;
        vt_first = x + 8ull * (i / F);
        vt_step = 8ull * groups;
    }
    for (uint32_t ft = ft_first; ft < F; ft += ft_step) {
        // the planes are stored stage by stage: [function tile][stage][plane][256 rows][16 coordinates],
        // so the 64 lanes of a load read 1 KB in one piece (thread t: 16 bytes at 16 t of rows 0-127)
        const uint16_t *arow = a.planes + (size_t)ft * stages * kStagePlanes + threadIdx.x * 8;
        for (uint64_t vt = vt_first; vt < Vt; vt += vt_step) {
            const float *vrow[4];
#pragma unroll
            for (int h = 0; h < 4; ++h) {
                uint64_t row = vt * TVW + vr + h * 64;
                row = row < a.N ? row : a.N - 1;  // rows beyond the data repeat the last vector (never stored)
                vrow[h] = a.data + row * a.n + vq * 4;
            }

            // the registers of the global loads: the stage on its way to LDS
            floatx4 gv[4];
            uintx4 ga[2][3];
            // Every load is issued unconditionally (the compiler can then count the loads in flight
            // exactly and wait for the oldest only): stages beyond the last read the last stage's
            // coefficients against zeros.
            auto gload = [&](uint32_t s, floatx4 (&v)[4], uintx4 (&c)[2][3]) __attribute__((always_inline)) {
                const uint32_t k0 = s * KB;
                // coordinates beyond n read the row's first ones instead; lstore() replaces them by zeros
#pragma unroll
                for (int h = 0; h < 4; ++h) v[h] = *reinterpret_cast<const floatx4 *>(vrow[h] + (k0 + vq * 4 < a.n ? k0 : 0u));
                const uint32_t ka = s < stages ? s : stages - 1;  // stage
#pragma unroll
                for (int h = 0; h < 2; ++h)
#pragma unroll
                    for (int p = 0; p < 3; ++p)
                        c[h][p] = *reinterpret_cast<const uintx4 *>(arow + (size_t)ka * kStagePlanes + p * (TF * KB) + h * 128 * KB);
            };
            auto lstore = [&](char *stage, uint32_t s, const floatx4 (&v)[4], const uintx4 (&c)[2][3]) __attribute__((always_inline)) {
                const bool inside = s * KB + vq * 4 < a.n;
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    bf16x4 h[3];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        __bf16 x1, x2, x3;
                        split3(inside ? v[r][e] : 0.f, x1, x2, x3);
                        h[0][e] = x1;
                        h[1][e] = x2;
                        h[2][e] = x3;
                    }
#pragma unroll
                    for (int p = 0; p < 3; ++p) *reinterpret_cast<bf16x4 *>(stage + wr_v + r * 64 * ROWB + p * V_PLANE) = h[p];
                }
#pragma unroll
                for (int r = 0; r < 2; ++r)
#pragma unroll
                    for (int p = 0; p < 3; ++p) *reinterpret_cast<uintx4 *>(stage + wr_a + r * 128 * ROWB + p * A_PLANE) = c[r][p];
            };

            floatx16 acc[NB][NB];
#pragma unroll
            for (int rb = 0; rb < NB; ++rb)
#pragma unroll
                for (int cb = 0; cb < NB; ++cb)
#pragma unroll
                    for (int e = 0; e < 16; ++e) acc[rb][cb][e] = 0.f;

            // Operand registers of the stage being contracted: fa[block][plane], fv[block][plane].
            // A plane's registers are read again, for the next stage, as soon as the last product
            // that uses them has been issued.
            bf16x8 fa[NB][3], fv[NB][3];
            auto read_a = [&](const char *stage, int p) __attribute__((always_inline)) {
#pragma unroll
                for (int b = 0; b < NB; ++b)
                    fa[b][p] = *reinterpret_cast<const bf16x8 *>(stage + rd_a + b * 32 * ROWB + p * A_PLANE);
            };
            auto read_v = [&](const char *stage, int p) __attribute__((always_inline)) {
#pragma unroll
                for (int b = 0; b < NB; ++b)
                    fv[b][p] = *reinterpret_cast<const bf16x8 *>(stage + rd_v + b * 32 * ROWB + p * V_PLANE);
            };
            auto read_a1 = [&](const char *stage, int b, int p) __attribute__((always_inline)) {
                fa[b][p] = *reinterpret_cast<const bf16x8 *>(stage + rd_a + b * 32 * ROWB + p * A_PLANE);
            };
            auto read_v1 = [&](const char *stage, int b, int p) __attribute__((always_inline)) {
                fv[b][p] = *reinterpret_cast<const bf16x8 *>(stage + rd_v + b * 32 * ROWB + p * V_PLANE);
            };
            // single loads of the next stage's operands, small enough to go out in the shadow of one MFMA
            auto load_v_row = [&](uint32_t s, int h, floatx4 (&v)[4]) __attribute__((always_inline)) {
                const uint32_t k0 = s * KB;
                v[h] = *reinterpret_cast<const floatx4 *>(vrow[h] + (k0 + vq * 4 < a.n ? k0 : 0u));
            };
            auto load_a_piece = [&](uint32_t s, int h, int p, uintx4 (&c)[2][3]) __attribute__((always_inline)) {
                const uint32_t ka = s < stages ? s : stages - 1;  // stage
                c[h][p] = *reinterpret_cast<const uintx4 *>(arow + (size_t)ka * kStagePlanes + p * (TF * KB) + h * 128 * KB);
            };

            // One stage.  LDS holds three stages: s (in the operand registers by now), s + 1 (written
            // during the previous iteration, read into the freed operand registers during this one)
            // and s + 2 (written during this one from the load registers, which then take the loads
            // of stage s + 3).  A wave is alone on its SIMD, so everything that is not an MFMA is cut
            // into pieces that go out one after each MFMA: an operand register is refilled right
            // after the last MFMA that reads it, the stores to LDS and the global loads ride along.
            auto iteration = [&](uint32_t s, floatx4 (&v_set)[4], uintx4 (&c_set)[2][3]) __attribute__((always_inline)) {
                const char *cur = lds_w + (s % 3) * STAGE;
                const char *nxt = lds_w + ((s + 1) % 3) * STAGE;
                char *far = lds_w + ((s + 2) % 3) * STAGE;  // last read two iterations ago: free since the barrier before this one
                const bool inside = (s + 2) * KB + vq * 4 < a.n;
                bf16x4 h[3];  // a vector row on its way: split in one product, written during the next
                auto split_element = [&](int r, int e) __attribute__((always_inline)) {
                    __bf16 x1, x2, x3;
                    split3(inside ? v_set[r][e] : 0.f, x1, x2, x3);
                    h[0][e] = x1;
                    h[1][e] = x2;
                    h[2][e] = x3;
                };
                auto write_plane = [&](int r, int pl) __attribute__((always_inline)) {
                    *reinterpret_cast<bf16x4 *>(far + wr_v + r * 64 * ROWB + pl * V_PLANE) = h[pl];
                };
                auto store_a = [&](int r, int pl) __attribute__((always_inline)) {
                    *reinterpret_cast<uintx4 *>(far + wr_a + r * 128 * ROWB + pl * A_PLANE) = c_set[r][pl];
                };
                // What goes out after MFMA i (0..15) of product k (0..5) of the stage: at most one
                // memory instruction, or the split of one vector element.  Products 0, 1, 2 and 5 run
                // row by row, 3 and 4 column by column, so that after every fourth MFMA one operand
                // register has been read for the last time and is refilled from the next stage.
                auto after = [&](auto K_, auto I_) __attribute__((always_inline)) {
                    constexpr int k = decltype(K_)::value, i = decltype(I_)::value;
                    if constexpr (i % 4 == 3) {
                        constexpr int q = i / 4;
                        if constexpr (k == 0) read_v1(cur, q, 2);  // read in every row of the stage before's last product
                        if constexpr (k == 1) read_a1(nxt, q, 1);
                        if constexpr (k == 2) read_a1(nxt, q, 2);
                        if constexpr (k == 3) read_v1(nxt, q, 1);
                        if constexpr (k == 4) read_v1(nxt, q, 0);
                        if constexpr (k == 5) read_a1(nxt, q, 0);
                    } else if constexpr (k == 0 || k == 5) {  // the two coefficient rows: store, then load again
                        constexpr int r = k == 0 ? 0 : 1;
                        if constexpr (i < 3) store_a(r, i);
                        if constexpr (i >= 4 && i < 7) load_a_piece(s + 3, r, i - 4, c_set);
                        if constexpr (k == 0 && i >= 8 && i < 13) split_element(0, i < 11 ? i - 8 : 3);
                    } else {  // products 1..4: write vector row k - 1, load it again, split row k
                        if constexpr (i < 3) write_plane(k - 1, i);
                        if constexpr (i == 4) load_v_row(s + 3, k - 1, v_set);
                        if constexpr (k < 4 && (i == 5 || i == 6 || i == 8 || i == 9)) split_element(k, i < 7 ? i - 5 : i - 6);
                    }
                };
                auto product = [&](auto K_, auto PA_, auto PV_, auto BY_ROW_) __attribute__((always_inline)) {
                    constexpr int pa = decltype(PA_)::value, pv = decltype(PV_)::value;
                    constexpr bool by_row = decltype(BY_ROW_)::value;
                    [&]<int... I>(std::integer_sequence<int, I...>) __attribute__((always_inline)) {
                        (([&] {
                            constexpr int rb = by_row ? I / 4 : I % 4, cb = by_row ? I % 4 : I / 4;
                            acc[rb][cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[rb][pa], fv[cb][pv], acc[rb][cb], 0, 0, 0);
                            __builtin_amdgcn_sched_barrier(0);
                            after(K_, std::integral_constant<int, I>{});
                            __builtin_amdgcn_sched_barrier(0);
                        }()), ...);
                    }(std::make_integer_sequence<int, 16>{});
                };
                using std::integral_constant;
                __builtin_amdgcn_sched_barrier(0);
                product(integral_constant<int, 0>{}, integral_constant<int, 1>{}, integral_constant<int, 1>{}, std::true_type{});
                lds_barrier();  // stage s + 1 is complete in LDS (the product before touched stage s and the free slot only)
                __builtin_amdgcn_sched_barrier(0);
                product(integral_constant<int, 1>{}, integral_constant<int, 1>{}, integral_constant<int, 0>{}, std::true_type{});
                product(integral_constant<int, 2>{}, integral_constant<int, 2>{}, integral_constant<int, 0>{}, std::true_type{});
                product(integral_constant<int, 3>{}, integral_constant<int, 0>{}, integral_constant<int, 1>{}, std::false_type{});
                product(integral_constant<int, 4>{}, integral_constant<int, 0>{}, integral_constant<int, 0>{}, std::false_type{});
                product(integral_constant<int, 5>{}, integral_constant<int, 0>{}, integral_constant<int, 2>{}, std::true_type{});
            };

            // prologue: stages 0 and 1 to LDS, stage 2 on its way
            gload(0, gv, ga);
            lstore(lds_w, 0, gv, ga);
            gload(1, gv, ga);
            lstore(lds_w + STAGE, 1, gv, ga);
            gload(2, gv, ga);
            __syncthreads();
            read_a(lds_w, 1);  // in the order of the refills
            read_a(lds_w, 2);
            read_v(lds_w, 1);
            read_v(lds_w, 0);
            read_a(lds_w, 0);
            read_v(lds_w, 2);
            for (uint32_t s = 0; s < stages; ++s) iteration(s, gv, ga);
            __syncthreads();  // the next tile's prologue writes stages that the last iterations read

            // epilogue: register 4q + e of block (rb, cb) is function 8q + 4 (l / 32) + e of the
            // block's 32, vector l % 32
#pragma unroll
            for (int rb = 0; rb < NB; ++rb)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const uint32_t j = ft * TF + fw * 32 * NB + rb * 32 + 8 * q + 4 * lh;  // < kpad
                    float b4[4] = {0.f, 0.f, 0.f, 0.f};
                    if constexpr (!PROJ) {
                        const floatx4 t = *reinterpret_cast<const floatx4 *>(a.off + j);
#pragma unroll
                        for (int e = 0; e < 4; ++e) b4[e] = POW2 ? t[e] * a.inv_w : t[e];
                    }
#pragma unroll
                    for (int cb = 0; cb < NB; ++cb) {
                        const uint64_t vec = vt * TVW + vw * 32 * NB + cb * 32 + lr;
                        uintx4 v;
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const float p = acc[rb][cb][4 * q + e];
                            if constexpr (PROJ) {
                                v[e] = __float_as_uint(p);
                            } else {
                                const float h = POW2 ? fmaf(p, a.inv_w, b4[e]) : (p + b4[e]) / a.w;
                                v[e] = (uint32_t)(int)floorf(h);
                            }
                        }
                        if (vec < a.N) {
                            uint32_t *dst = reinterpret_cast<uint32_t *>(a.out) + vec * a.k + j;
                            if constexpr (VEC) {
                                if (j < a.k) *reinterpret_cast<uintx4 *>(dst) = v;
                            } else {
#pragma unroll
                                for (int e = 0; e < 4; ++e)
                                    if (j + e < a.k) dst[e] = v[e];
                            }
                        }
                    }
                }
        }
    }
}

uint16_t to_bf16(float x) {  // round to nearest even; NaN stays NaN
    uint32_t u;
    std::memcpy(&u, &x, 4);
    if ((u & 0x7F800000u) == 0x7F800000u) return (uint16_t)((u >> 16) | ((u & 0xFFFFu) ? 0x40u : 0u));
    return (uint16_t)((u + 0x7FFFu + ((u >> 16) & 1u)) >> 16);
}

float from_bf16(uint16_t h) {
    const uint32_t u = (uint32_t)h << 16;
    float x;
    std::memcpy(&x, &u, 4);
    return x;
}

}  // namespace

uint32_t dense_wide_row_tile() { return TF; }
uint32_t dense_wide_col_step() { return KB; }

// The three bf16 planes of a coefficient matrix [k][n] in the order the kernel reads them:
// [function tile of 256][stage of 16 coordinates][plane][row][coordinate], zeros beyond k and n.
void build_dense_planes(const float *a, uint32_t k, uint32_t n, uint32_t kpad, uint32_t npad,
                        std::vector<uint16_t> &planes) {
    planes.assign((size_t)3 * kpad * npad, 0);
    const uint32_t stages = npad / KB;
    for (uint32_t j = 0; j < k; ++j)
        for (uint32_t c = 0; c < n; ++c) {
            const float x = a[(size_t)j * n + c];
            const uint16_t h1 = to_bf16(x);
            const float r1 = x - from_bf16(h1);
            const uint16_t h2 = to_bf16(r1);
            const uint16_t h3 = to_bf16(r1 - from_bf16(h2));
            const size_t at = ((size_t)(j / TF) * stages + c / KB) * kStagePlanes + (size_t)(j % TF) * KB + c % KB;
            planes[at] = h1;
            planes[at + TF * KB] = h2;
            planes[at + 2 * TF * KB] = h3;
        }
}

bool dense_wide_supported(const lsh_params *p) {
    return p->m == p->n && p->d_dense_planes != nullptr && p->n % 4 == 0 && (uint64_t)p->k * 4 < (1ull << 32);
}

int launch_dense_wide(const lsh_params *p, bool proj, const float *d_data, uint64_t N, void *d_out, void *stream) {
    WideArgs a;
    a.data = d_data;
    a.planes = static_cast<const uint16_t *>(p->d_dense_planes);
    a.off = p->d_off;
    a.N = N;
    a.n = p->n;
    a.npad = (p->n + KB - 1) / KB * KB;
    a.k = p->k;
    a.kpad = (p->k + TF - 1) / TF * TF;
    a.w = p->w;
    a.inv_w = 1.0f / p->w;
    a.out = d_out;
    int exp2 = 0;
    const bool pw = proj || std::frexp(p->w, &exp2) == 0.5f;
    const bool vec = p->k % 4 == 0;
    // one workgroup per CU (144 KB of LDS), a multiple of 8 so that every XCD gets the same number
    uint32_t wgs = (uint32_t)(p->num_cus > 0 ? p->num_cus : 256) / 8 * 8;
    if (wgs < 8) wgs = 8;
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
#define LSH_WIDE_CASE(P_, W_, V_) \
    if (proj == P_ && pw == W_ && vec == V_) { \
        auto fn = &dense_split_wide_kernel<P_, W_, V_>; \
        if (ensure_lds_limit(reinterpret_cast<const void *>(fn), kLdsBytesW) != LSH_OK) return LSH_ERR_HIP; \
        hipLaunchKernelGGL(fn, dim3(wgs), dim3(kThreadsW), kLdsBytesW, s, a); \
    }
    LSH_WIDE_CASE(false, true, true) LSH_WIDE_CASE(false, false, true) LSH_WIDE_CASE(true, true, true)
    LSH_WIDE_CASE(false, true, false) LSH_WIDE_CASE(false, false, false) LSH_WIDE_CASE(true, true, false)
#undef LSH_WIDE_CASE
    return hipGetLastError() == hipSuccess ? LSH_OK : LSH_ERR_HIP;
}

}  // namespace lsh
