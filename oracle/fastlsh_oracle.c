/*
 * CPU oracle for batched l2 LSH hash evaluation (E2LSH and FastLSH).
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a plain, slow, fp64
 * restatement of the paper's definitions, used only to check the GPU library
 * and as a timed CPU baseline.  It shares no source, header, table or constant
 * generator with the GPU library and must never be called from the product
 * path.
 *
 * What follows the paper:
 *   - E2LSH hash        h_{a,b}(v) = floor((a^T v + b) / w)          (Sec. 2.2, Eq. 1)
 *   - sampling operator S(v): m coordinates of v, in draw order,
 *     duplicates kept                                                 (Sec. 3.1, first step)
 *   - FastLSH hash      h(v) = floor((a~^T S(v) + b~) / w~)           (Sec. 3.1, Eq. 5)
 *   - compound code     H(v) = (h_1(v), ..., h_k(v)), L groups        (Sec. 3.2)
 *   - angular use: sign of the sampled projection (the paper, Sec. 5,
 *     only says "normalise, then use FastLSH"; the sign form is the
 *     sign-random-projection hash it cites in Sec. 1)
 *
 * What the paper leaves open and this file fixes (each listed in the design
 * notes of the repository):
 *   - the random number generator: Philox4x64-10 (Salmon, Moraes, Dror, Shaw,
 *     "Parallel random numbers: as easy as 1, 2, 3", SC'11) used as a pure
 *     function of (seed, stream, function j, sample i, attempt t);
 *   - N(0,1) by the Box-Muller transform (cosine branch) on two 53-bit
 *     uniforms, rounded once to fp32; b~ = fp32(u * w), u in [0,1);
 *   - sampling without replacement (partial Fisher-Yates shuffle, draw order
 *     kept) as the default, with replacement (the paper's i.i.d. multiset) as
 *     the alternative; m == n means "no sampling": S_j = (0, 1, ..., n-1);
 *   - 64-bit key of a group of g bucket ids: Horner polynomial in a fixed odd
 *     multiplier, arithmetic mod 2^64;
 *   - whether the k functions share their sample S: Sec. 3.1 draws "a multiset S" once,
 *     Sec. 3.2 draws k functions independently from the family.  Default: every function its
 *     own S_j.  Alternative (oracle_params_shared): the g = k/L functions of one table share
 *     one S (that of the table's first function), with their own a~_j and b~_j.
 *
 * Parity status: the arithmetic (gather, projection, floor, signs, keys) is
 * pinned by the tests under tests/ (paper's worked sampling example, exact
 * rational brute force, dense-matrix reduction, closed-form collision law).
 * The parameter tables are "parity unpinned" by the paper, which names no
 * generator; Philox itself is pinned by its published known-answer vectors and
 * by numpy's independent implementation, the table construction by
 * statistical tests.
 *
 * Build: gcc -O2 -ffp-contract=off -fopenmp -shared -fPIC fastlsh_oracle.c -lm
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_OK 0
#define ORACLE_ERR_ARG (-1)
#define ORACLE_ERR_ALLOC (-2)
#define ORACLE_ERR_RANGE (-3) /* a bucket id does not fit int32 */

/* ------------------------------------------------------------------------ */
/* Philox4x64-10, from its published definition (SC'11, Sec. 3.3 + Table 2). */
/* ------------------------------------------------------------------------ */

static void mulhilo64(uint64_t a, uint64_t b, uint64_t *hi, uint64_t *lo)
{
    unsigned __int128 p = (unsigned __int128)a * (unsigned __int128)b;
    *hi = (uint64_t)(p >> 64);
    *lo = (uint64_t)p;
}

void oracle_philox4x64_10(const uint64_t ctr[4], const uint64_t key[2], uint64_t out[4])
{
    const uint64_t MUL0 = 0xD2E7470EE14C6C93ULL, MUL1 = 0xCA5A826395121157ULL;
    const uint64_t WEYL0 = 0x9E3779B97F4A7C15ULL, WEYL1 = 0xBB67AE8584CAA73BULL;
    uint64_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint64_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        uint64_t hi0, lo0, hi1, lo1;
        if (round > 0) { k0 += WEYL0; k1 += WEYL1; }
        mulhilo64(MUL0, c0, &hi0, &lo0);
        mulhilo64(MUL1, c2, &hi1, &lo1);
        uint64_t n0 = hi1 ^ c1 ^ k0, n1 = lo1, n2 = hi0 ^ c3 ^ k1, n3 = lo0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* One block of random words for table element (stream, j, i), attempt t. */
enum { STREAM_INDEX = 0, STREAM_COEF = 1, STREAM_OFFSET = 2 };

static void draw_block(uint64_t seed, uint64_t stream, uint64_t j, uint64_t i, uint64_t t,
                       uint64_t out[4])
{
    uint64_t ctr[4] = { i, j, stream, t };
    uint64_t key[2] = { seed, 0 };
    oracle_philox4x64_10(ctr, key, out);
}

/* Unbiased integer in [0, bound): rejection of the incomplete top interval. */
static uint64_t draw_below(uint64_t seed, uint64_t j, uint64_t i, uint64_t bound)
{
    uint64_t reject_from_top = (0 - bound) % bound; /* 2^64 mod bound */
    for (uint64_t t = 0;; ++t) {
        uint64_t r[4];
        draw_block(seed, STREAM_INDEX, j, i, t, r);
        /* accept r[0] iff r[0] < 2^64 - (2^64 mod bound) */
        if (r[0] <= UINT64_MAX - reject_from_top) return r[0] % bound;
    }
}

static double uniform53(uint64_t word) { return (double)(word >> 11) * 0x1.0p-53; }

/*
 * Parameter tables of the k hash functions (Sec. 3.1: S, a~, b~; Sec. 2.2: a, b).
 *   idx  [k*m]  0-based sampled coordinates, draw order
 *   coef [k*m]  a~_j[i] ~ N(0,1), fp32
 *   off  [k]    b~_j ~ U[0,w), fp32
 */
static int params_tables(uint32_t n, uint32_t k, uint32_t m, float w, uint64_t seed,
                         uint32_t with_replacement, uint32_t group, uint32_t *idx, float *coef,
                         float *off)
{
    if (!n || !k || !m || m > n || !(w > 0.0f) || !isfinite(w) || !idx || !coef || !off)
        return ORACLE_ERR_ARG;
    uint32_t *perm = NULL;
    if (m < n && !with_replacement) {
        perm = (uint32_t *)malloc((size_t)n * sizeof(uint32_t));
        if (!perm) return ORACLE_ERR_ALLOC;
    }
    for (uint32_t j = 0; j < k; ++j) {
        uint32_t *S = idx + (size_t)j * m;
        /* the function whose draws give S: j itself, or the first function of j's table */
        const uint32_t js = j - j % group;
        if (m == n) {
            for (uint32_t i = 0; i < m; ++i) S[i] = i;              /* no sampling */
        } else if (with_replacement) {
            for (uint32_t i = 0; i < m; ++i)                          /* i.i.d. multiset */
                S[i] = (uint32_t)draw_below(seed, js, i, n);
        } else {
            for (uint32_t c = 0; c < n; ++c) perm[c] = c;             /* Fisher-Yates, m steps */
            for (uint32_t i = 0; i < m; ++i) {
                uint32_t r = i + (uint32_t)draw_below(seed, js, i, n - i);
                uint32_t tmp = perm[i]; perm[i] = perm[r]; perm[r] = tmp;
                S[i] = perm[i];
            }
        }
        for (uint32_t i = 0; i < m; ++i) {
            uint64_t r[4];
            draw_block(seed, STREAM_COEF, j, i, 0, r);
            double u1 = ((double)(r[0] >> 11) + 1.0) * 0x1.0p-53;     /* (0,1] */
            double u2 = uniform53(r[1]);                               /* [0,1) */
            double z = sqrt(-2.0 * log(u1)) * cos(6.283185307179586476925286766559 * u2);
            coef[(size_t)j * m + i] = (float)z;
        }
        {
            uint64_t r[4];
            draw_block(seed, STREAM_OFFSET, j, 0, 0, r);
            float b = (float)(uniform53(r[0]) * (double)w);
            if (b >= w) b = nextafterf(w, 0.0f);
            off[j] = b;
        }
    }
    free(perm);
    return ORACLE_OK;
}

int oracle_params(uint32_t n, uint32_t k, uint32_t m, float w, uint64_t seed,
                  uint32_t with_replacement, uint32_t *idx, float *coef, float *off)
{
    return params_tables(n, k, m, w, seed, with_replacement, 1, idx, coef, off);
}

/*
 * The same tables with one sample S per table of g = k / L functions (Sec. 3.1 read
 * literally: one multiset S, then the projection vectors): functions l*g .. l*g + g - 1 all
 * get the S that function l*g has in oracle_params; a~ and b~ stay per function.
 */
int oracle_params_shared(uint32_t n, uint32_t k, uint32_t m, float w, uint64_t seed,
                         uint32_t with_replacement, uint32_t L, uint32_t *idx, float *coef,
                         float *off)
{
    if (!L || !k || k % L) return ORACLE_ERR_ARG;
    return params_tables(n, k, m, w, seed, with_replacement, k / L, idx, coef, off);
}

/* ------------------------------------------------------------------------ */
/* The hash functions.                                                      */
/* ------------------------------------------------------------------------ */

/* S(v): the m sampled coordinates of v, in draw order (Sec. 3.1, first step). */
static void sample_vector(const float *v, const uint32_t *S, uint32_t m, double *v_tilde)
{
    for (uint32_t i = 0; i < m; ++i) v_tilde[i] = (double)v[S[i]];
}

/* a^T x in fp64, terms added in index order; also sum of |a_i x_i|. */
static double dot(const float *a, const double *x, uint32_t len, double *abs_sum)
{
    double s = 0.0, t = 0.0;
    for (uint32_t i = 0; i < len; ++i) {
        double term = (double)a[i] * x[i];
        s += term;
        t += fabs(term);
    }
    if (abs_sum) *abs_sum = t;
    return s;
}

/* floor((p + b) / w) as a real number (Eq. 1 / Eq. 5). */
static double bucket_real(double p, float b, float w) { return floor((p + (double)b) / (double)w); }

static int store_bucket(double h, int32_t *out)
{
    if (!(h >= -2147483648.0 && h <= 2147483647.0)) return ORACLE_ERR_RANGE;
    *out = (int32_t)h;
    return ORACLE_OK;
}

/*
 * FastLSH (Eq. 5) for N row-major vectors.  Any of proj, abs_sum, ids, frac may
 * be NULL.  proj[N*k] = a~_j^T S_j(v); abs_sum[N*k] = sum_i |a~_j[i] S_j(v)_i|;
 * ids[N*k] = bucket; frac[N*k] = (p+b)/w - floor((p+b)/w), the position inside
 * the bucket in units of w.
 */
int oracle_fastlsh(const float *data, uint64_t N, uint32_t n, uint32_t k, uint32_t m,
                   const uint32_t *idx, const float *coef, const float *off, float w,
                   double *proj, double *abs_sum, int32_t *ids, double *frac, int nthreads)
{
    if (!data || !idx || !coef || !n || !k || !m) return ORACLE_ERR_ARG;
    if ((ids || frac) && (!off || !(w > 0.0f))) return ORACLE_ERR_ARG;
    for (size_t e = 0; e < (size_t)k * m; ++e)
        if (idx[e] >= n) return ORACLE_ERR_ARG;
    int status = ORACLE_OK;
#ifdef _OPENMP
    if (nthreads < 1) nthreads = 1;
#pragma omp parallel for num_threads(nthreads) schedule(static) reduction(min : status)
#endif
    for (int64_t r = 0; r < (int64_t)N; ++r) {
        const float *v = data + (size_t)r * n;
        double *v_tilde = (double *)malloc((size_t)m * sizeof(double));
        if (!v_tilde) { status = ORACLE_ERR_ALLOC; continue; }
        for (uint32_t j = 0; j < k; ++j) {
            size_t o = (size_t)r * k + j;
            double t;
            sample_vector(v, idx + (size_t)j * m, m, v_tilde);
            double p = dot(coef + (size_t)j * m, v_tilde, m, &t);
            if (proj) proj[o] = p;
            if (abs_sum) abs_sum[o] = t;
            if (ids || frac) {
                double h = bucket_real(p, off[j], w);
                if (ids && store_bucket(h, &ids[o]) != ORACLE_OK) status = ORACLE_ERR_RANGE;
                if (frac) frac[o] = (p + (double)off[j]) / (double)w - h;
            }
        }
        free(v_tilde);
    }
    return status;
}

/*
 * E2LSH (Eq. 1): a is the dense k x n coefficient matrix, row j = a_j.
 * Written from Eq. 1 alone; it does not go through the sampling code.
 */
int oracle_e2lsh(const float *data, uint64_t N, uint32_t n, uint32_t k, const float *a,
                 const float *off, float w, double *proj, double *abs_sum, int32_t *ids,
                 double *frac, int nthreads)
{
    if (!data || !a || !n || !k) return ORACLE_ERR_ARG;
    if ((ids || frac) && (!off || !(w > 0.0f))) return ORACLE_ERR_ARG;
    int status = ORACLE_OK;
#ifdef _OPENMP
    if (nthreads < 1) nthreads = 1;
#pragma omp parallel for num_threads(nthreads) schedule(static) reduction(min : status)
#endif
    for (int64_t r = 0; r < (int64_t)N; ++r) {
        const float *v = data + (size_t)r * n;
        for (uint32_t j = 0; j < k; ++j) {
            size_t o = (size_t)r * k + j;
            const float *aj = a + (size_t)j * n;
            double p = 0.0, t = 0.0;
            for (uint32_t c = 0; c < n; ++c) {
                double term = (double)aj[c] * (double)v[c];
                p += term;
                t += fabs(term);
            }
            if (proj) proj[o] = p;
            if (abs_sum) abs_sum[o] = t;
            if (ids || frac) {
                double h = bucket_real(p, off[j], w);
                if (ids && store_bucket(h, &ids[o]) != ORACLE_OK) status = ORACLE_ERR_RANGE;
                if (frac) frac[o] = (p + (double)off[j]) / (double)w - h;
            }
        }
    }
    return status;
}

/*
 * Sign hashes: bit j of a vector = [a~_j^T S_j(v) >= 0], packed 64 functions
 * per word, function j in word j / 64 at bit j % 64 (bit 0 = least
 * significant).  words[N * ceil(k/64)]; unused high bits of the last word are 0.
 * proj / norm_prod may be NULL; norm_prod = ||a~_j||_2 * ||S_j(v)||_2.
 */
int oracle_signs(const float *data, uint64_t N, uint32_t n, uint32_t k, uint32_t m,
                 const uint32_t *idx, const float *coef, uint64_t *words, double *proj,
                 double *norm_prod, int nthreads)
{
    if (!data || !idx || !coef || !words || !n || !k || !m) return ORACLE_ERR_ARG;
    for (size_t e = 0; e < (size_t)k * m; ++e)
        if (idx[e] >= n) return ORACLE_ERR_ARG;
    uint32_t W = (k + 63) / 64;
    int status = ORACLE_OK;
#ifdef _OPENMP
    if (nthreads < 1) nthreads = 1;
#pragma omp parallel for num_threads(nthreads) schedule(static) reduction(min : status)
#endif
    for (int64_t r = 0; r < (int64_t)N; ++r) {
        const float *v = data + (size_t)r * n;
        double *v_tilde = (double *)malloc((size_t)m * sizeof(double));
        if (!v_tilde) { status = ORACLE_ERR_ALLOC; continue; }
        for (uint32_t q = 0; q < W; ++q) words[(size_t)r * W + q] = 0;
        for (uint32_t j = 0; j < k; ++j) {
            sample_vector(v, idx + (size_t)j * m, m, v_tilde);
            double p = dot(coef + (size_t)j * m, v_tilde, m, NULL);
            if (p >= 0.0) words[(size_t)r * W + j / 64] |= (uint64_t)1 << (j % 64);
            if (proj) proj[(size_t)r * k + j] = p;
            if (norm_prod) {
                double na = 0.0, nv = 0.0;
                for (uint32_t i = 0; i < m; ++i) {
                    double ai = (double)coef[(size_t)j * m + i];
                    na += ai * ai;
                    nv += v_tilde[i] * v_tilde[i];
                }
                norm_prod[(size_t)r * k + j] = sqrt(na) * sqrt(nv);
            }
        }
        free(v_tilde);
    }
    return status;
}

/*
 * Compound keys (Sec. 3.2): the k functions form L groups of g = k / L
 * consecutive functions; group l holds functions l*g .. l*g+g-1.  The 64-bit
 * key of a group is sum_t uint32(h_{l*g+t}) * MULT^(g-1-t) mod 2^64.
 */
int oracle_pack_keys(const int32_t *ids, uint64_t N, uint32_t k, uint32_t L, uint64_t *keys)
{
    const uint64_t MULT = 0x9E3779B97F4A7C15ULL;
    if (!ids || !keys || !k || !L || k % L) return ORACLE_ERR_ARG;
    uint32_t g = k / L;
    for (uint64_t r = 0; r < N; ++r)
        for (uint32_t l = 0; l < L; ++l) {
            uint64_t key = 0;
            for (uint32_t t = 0; t < g; ++t)
                key = key * MULT + (uint64_t)(uint32_t)ids[r * k + (uint64_t)l * g + t];
            keys[r * L + l] = key;
        }
    return ORACLE_OK;
}

int oracle_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
