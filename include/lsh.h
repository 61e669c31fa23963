/*
 * lsh.h -- C ABI of the MI355X (gfx950) library for batched l2 LSH hash evaluation.
 *
 * The operation (paper: "Fast Locality Sensitive Hashing with Theoretical
 * Guarantee", FastLSH):
 *
 *   E2LSH   (Sec. 2.2, Eq. 1):  h_{a,b}(v)   = floor((a^T v + b) / w),   a in R^n
 *   FastLSH (Sec. 3.1, Eq. 5):  h_{a~,b~}(v) = floor((a~^T S(v) + b~) / w~), a~ in R^m
 *
 * where S(.) keeps m sampled coordinates of v in draw order (Sec. 3.1, first
 * step), a / a~ have i.i.d. N(0,1) entries and b / b~ is uniform on [0, w).
 * All k hash functions are evaluated for all N vectors; here k is the TOTAL
 * number of functions (the paper's k functions per table times L tables,
 * Sec. 3.2), function j belonging to table j / (k/L).
 *
 * Conventions
 *   - Every function returns an int status: LSH_OK (0) or a negative LSH_ERR_*.
 *     Nothing throws or aborts.  lsh_status_string() names a status.
 *   - "d_" arguments are DEVICE pointers owned by the caller; they must be valid
 *     on the device that was current when the params object was created.  All
 *     other pointers are HOST pointers.
 *   - data is row-major fp32 [N][n], 16-byte-aligned base; outputs are row-major.
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream).  Hash
 *     calls only enqueue work on it and never synchronise; the caller keeps
 *     data/outputs alive until the stream has drained.
 *   - N = 0 is LSH_OK and launches nothing (data/output pointers may then be NULL).
 *   - The params object and its device tables belong to the library and are
 *     freed by lsh_params_destroy().  One object may be used from several host
 *     threads for hashing; create/destroy are not thread-safe against its use.
 */
#ifndef LSH_H
#define LSH_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define LSH_OK 0
#define LSH_ERR_INVALID_ARG (-1) /* null pointer, zero size, m > n, bad w, k % L != 0 ... */
#define LSH_ERR_ALLOC (-2)       /* host or device allocation failed */
#define LSH_ERR_HIP (-3)         /* a HIP runtime call or kernel launch failed */
#define LSH_ERR_UNSUPPORTED (-4) /* no kernel covers this shape (see each call) */
#define LSH_ERR_NO_DEVICE (-5)   /* params object has no device tables (no GPU at create) */

/* flags of lsh_params_create_ex */
#define LSH_SAMPLE_WITHOUT_REPLACEMENT 0u /* m distinct coordinates per function (default) */
#define LSH_SAMPLE_WITH_REPLACEMENT 1u    /* m i.i.d. draws: the multiset of Sec. 3.1 */

typedef struct lsh_params lsh_params_t; /* opaque */

/*
 * Draw the k hash functions (Sec. 3.1: S_j, a~_j, b~_j for j < k; Sec. 2.2 when
 * m == n) and, if a GPU is present, upload their tables to the current device.
 *   n     vector dimension (>= 1)
 *   k     number of hash functions (>= 1)
 *   m     sampled dimensions per function, 1 <= m <= n; m == n means no
 *         sampling: S_j = (0..n-1) and the functions are E2LSH functions
 *   w     bucket width, finite and > 0
 *   seed  the tables are a pure function of (n, k, m, w, seed, flags): each
 *         element is one Philox4x64-10 block keyed by seed and indexed by
 *         (table, j, i); N(0,1) by Box-Muller; without replacement = the first
 *         m steps of a Fisher-Yates shuffle
 *   out   receives the object (host pointer to a pointer)
 * Errors: INVALID_ARG, ALLOC, HIP.  Without a GPU the object is still created
 * (getters work) and hash calls return LSH_ERR_NO_DEVICE.
 */
int lsh_params_create(uint32_t n, uint32_t k, uint32_t m, float w, uint64_t seed,
                      lsh_params_t **out);
int lsh_params_create_ex(uint32_t n, uint32_t k, uint32_t m, float w, uint64_t seed,
                         uint32_t flags, lsh_params_t **out);
/*
 * The same with ONE sample per table (Sec. 3.1 read literally: a single multiset S is drawn,
 * then the projection vectors): with L > 0 (k % L == 0) the g = k / L functions of table l,
 * j = l*g .. l*g + g - 1, all use the sample S that function l*g gets from
 * lsh_params_create_ex; a~_j and b~_j stay per function.  Given S, the functions of a table
 * are independent E2LSH functions on the same sub-vector (Sec. 4.1), so a table's key collides
 * with probability p_w(s~)^g given S instead of the product over g independent samples.
 * Every hash call accepts such an object; lsh_hash_fastlsh, lsh_project_fastlsh and (called
 * with the same L, g <= 32) lsh_hash_fastlsh_keys then gather each table's sub-vector once and
 * contract it with the g coefficient vectors on the matrix cores when the shape allows
 * (n % 4 == 0 and g % 4 == 0; with m <= 64 and n <= 612 or 64 < m <= 128 and n <= 1260 whole
 * vectors stay in LDS and lsh_hash_fastlsh_keys takes g <= 32; at any larger n or m < n the
 * kernel works by coordinate ranges, up to n of about 10^6, and lsh_hash_fastlsh_keys and
 * lsh_hash_fastlsh_ids_keys take g <= 16 in one launch), and fall back to the per-function
 * gather kernels otherwise.  L == 0 is lsh_params_create_ex.
 * Errors: as lsh_params_create, and INVALID_ARG when k % L != 0.
 */
int lsh_params_create_shared(uint32_t n, uint32_t k, uint32_t m, float w, uint64_t seed,
                             uint32_t flags, uint32_t L, lsh_params_t **out);
void lsh_params_destroy(lsh_params_t *params);

/*
 * Host copies of the canonical tables (for inspection and bit-exact checks).
 *   indices [k*m]  S_j[i], 0-based coordinate numbers, draw order (row j = function j)
 *   coeffs  [k*m]  a~_j[i]
 *   offsets [k]    b~_j
 * Caller provides the arrays.  Errors: INVALID_ARG.
 */
int lsh_params_get_indices(const lsh_params_t *params, uint32_t *out);
int lsh_params_get_coeffs(const lsh_params_t *params, float *out);
int lsh_params_get_offsets(const lsh_params_t *params, float *out);
/* the six scalars: n, k, m, flags as uint32; w; seed.  Any out pointer may be NULL. */
int lsh_params_get_shape(const lsh_params_t *params, uint32_t *n, uint32_t *k, uint32_t *m,
                         uint32_t *flags, float *w, uint64_t *seed);

/* L of lsh_params_create_shared (0: every function has its own sample). */
int lsh_params_get_tables(const lsh_params_t *params, uint32_t *shared_tables);
/* a0 [k] of the maximum-inner-product transform (see lsh_hash_mips_data); host array of the
 * caller.  Errors: INVALID_ARG, UNSUPPORTED (the object was not made by lsh_params_create_shared
 * with L > 0). */
int lsh_params_get_mips_coeffs(const lsh_params_t *params, float *out);

/*
 * The order in which the sampled kernel visits each function's samples.  A projection is a
 * sum, so the kernel is free to reorder; it uses an order in which the `group` lanes
 * (functions) that one pass of an LDS read serves touch distinct bank classes
 * (coordinate % classes), and pads every list to `steps` entries.  Within each run of 64
 * functions the passes are: group == 32: functions 0-31 and 32-63; group == 16: the runs of
 * four functions numbered {0,3,5,6}, {1,2,4,7}, {8,11,13,14}, {9,10,12,15} (run q = functions
 * 4q..4q+3), as measured for 16-byte LDS reads on gfx950.
 *   order [k*steps]  entry (j, i) = position in function j's canonical list (0..m-1), plus
 *                    0x40000000 when the sample is read from the second copy of the tile
 *                    (small n: the tile is kept twice in LDS, the second time with
 *                    coordinate c in class (c + c / classes) % classes, and every sample is
 *                    read from the copy that evens out the classes' loads), or
 *                    0x80000000 | class for a padding sample (coefficient 0), or 0xFFFFFFFF
 *                    (unused tail: for large n the samples are visited range by range, a
 *                    sample of the r-th range of 256 coordinates in one of the stages
 *                    r - 6 .. r of a tile, with all functions of a workgroup of up to 2048
 *                    in lockstep; rows of different workgroups may differ in length and
 *                    steps is then the longest row)
 *   modelled_passes  sum over lane groups and steps of the largest number of lanes sharing a
 *                    class (k/group * steps when the schedule is conflict-free)
 * Any out pointer may be NULL.  Errors: INVALID_ARG, UNSUPPORTED (n too large for the kernel).
 */
int lsh_params_get_schedule(const lsh_params_t *params, uint32_t *order, uint32_t *steps,
                            uint32_t *group, uint32_t *classes, uint64_t *modelled_passes);

/*
 * Host-side check of the list tables of the kernels that work by coordinate ranges (the
 * sampled projection, Eq. 5, at large n; with one sample per table the matrix-core kernel for
 * large n): the tables are built as for the device and walked as the kernels walk them on a
 * pseudo-random vector derived from seed, in double precision; *worst receives the largest
 * |walked - direct| / sum_i |a~_j[i] v[S_j[i]]| over the functions, direct being the sum of
 * Eq. 5 taken from the canonical tables (about 1e-16 when the tables are right, infinity when a
 * stream is inconsistent).  Needs no GPU.
 * Errors: INVALID_ARG (null), UNSUPPORTED (the object's kernels use no such lists), ALLOC.
 */
int lsh_params_check_lists(const lsh_params_t *params, uint64_t seed, double *worst);

/*
 * One sample per table (Sec. 3.1, 4.1) at large n: how the matrix-core kernel that works by
 * coordinate ranges deals a table's m samples to its stages.  *stages receives the stages of a
 * tile of 16 vectors and *steps the MFMA steps of four samples that every block of 16
 * functions takes per tile (all tables get the same number; steps * 4 - m of the sample slots
 * are padding).  Needs no GPU.
 * Errors: INVALID_ARG (null), UNSUPPORTED (the object does not run on that kernel), ALLOC.
 */
int lsh_params_get_shared_schedule(const lsh_params_t *params, uint32_t *stages, uint32_t *steps);

/*
 * FastLSH bucket ids (Eq. 5): d_out_buckets[v*k + j] = floor((a~_j^T S_j(v) + b~_j) / w)
 * as int32 (saturating), for v < N, j < k.  Sampled-projection kernel: each vector
 * tile is read from HBM once, kept in LDS, and every function gathers its m
 * coordinates from there.  fp32 accumulation.  (n == 128 with k a multiple of 32: by default
 * the matrix-core kernel of lsh_params_set_dense_arithmetic instead, over the coefficients
 * written out over all n coordinates.)
 * Errors: INVALID_ARG (null pointers), NO_DEVICE, UNSUPPORTED (n > 40384: one vector must
 * fit in LDS), HIP.
 */
int lsh_hash_fastlsh(const lsh_params_t *params, const float *d_data, uint64_t N,
                     int32_t *d_out_buckets, void *stream);

/*
 * E2LSH bucket ids (Eq. 1) by a dense [N x n] . [n x k] matrix-core contraction (arithmetic:
 * see lsh_params_set_dense_arithmetic) with the floor((. + b) / w) epilogue fused.  Requires params created with m == n
 * (INVALID_ARG otherwise).  Same output layout as lsh_hash_fastlsh, and the two agree
 * on such params up to fp32 summation order.
 */
int lsh_hash_e2lsh(const lsh_params_t *params, const float *d_data, uint64_t N,
                   int32_t *d_out_buckets, void *stream);

/*
 * Arithmetic of the matrix-core kernels of this object: lsh_hash_e2lsh and lsh_project_e2lsh,
 * and at n == 128 also lsh_hash_fastlsh, lsh_project_fastlsh, lsh_hash_fastlsh_keys (4 to 32
 * functions per table; objects with one sample per function) and lsh_hash_signs, which then
 * run as a dense product over the coefficients written
 * out over all n coordinates: zeros where a function does not sample, sums where it samples a
 * coordinate more than once.
 * LSH_DENSE_AUTO (the default): for n == 128 and k a multiple of 32 every fp32 operand is
 * split exactly into three bf16 terms and the product is formed from the six bf16 MFMA
 * products of weight >= 2^-16, accumulated in fp32; what is left out is below 2^-23 of each
 * term |a_i v_i|, one fp32 rounding, and the projections stay within the same
 * 1e-5 * sum_i |a_i v_i| of the exact value as the fp32 path.  (Operands whose bf16 rounding
 * overflows, |x| > 3.39e38, give NaN there.)  Products of terms that are zero for a whole tile
 * of 64 vectors are skipped, which changes no bit of the result: byte-valued data take half of
 * the products.  With n == 128 and k a multiple of 64,
 * lsh_hash_signs runs on the matrix cores too, with two-way splits and three products: what
 * they leave out is below 3 * 2^-16 * sum_i |a_i v_i|, under half of the 1e-4 * |a| * |S(v)| around
 * zero inside which a sign bit is unspecified.  Objects with m == n and another n that is a
 * multiple of 4 take the same six products in lsh_hash_e2lsh and lsh_project_e2lsh (no
 * products skipped); any other shape uses fp32 MFMA.
 * LSH_DENSE_FP32: fp32 MFMA for every dense product, and the gathered fp32 kernels for FastLSH
 * ids, projections, keys and signs at every n.
 * LSH_DENSE_MATRIX: as LSH_DENSE_AUTO, and lsh_hash_fastlsh and lsh_project_fastlsh of an object
 * with m < n and any n that is a multiple of 4 also run as that bf16 x 3 product over the
 * coefficients written out over all n coordinates (same error bound).  It costs n multiply-adds
 * per function where the gather costs m, on matrix cores that are several times faster per
 * multiply-add: on the 4096-dimensional shape it is the faster route from about m = n / 5 on.
 * The first call with this mode builds the object's bf16 planes (6 bytes x k x n of device
 * memory, freed with the object; call it with the object's device current).
 * The mode is a plain field of the object, read by every hash call when it launches: set it
 * while no other thread is calling into the same object (calls already enqueued keep the mode
 * they were launched with).
 * Errors: INVALID_ARG (null, unknown mode, another device current); for LSH_DENSE_MATRIX also
 * UNSUPPORTED (n not a multiple of 4), NO_DEVICE, ALLOC, HIP.
 */
#define LSH_DENSE_AUTO 0
#define LSH_DENSE_FP32 1
#define LSH_DENSE_MATRIX 2
int lsh_params_set_dense_arithmetic(lsh_params_t *params, int mode);

/*
 * Sign hashes for angular similarity (Sec. 5: FastLSH on normalised data; the sign form
 * of the sampled projection): bit j = [a~_j^T S_j(v) >= 0]; function j is bit j % 64
 * (bit 0 least significant) of d_out_words[v * ceil(k/64) + j / 64]; unused high bits of
 * the last word are 0.  b~ and w are not used.  A bit whose projection lies within
 * 1e-4 * |a~_j| * |S_j(v)| of zero is unspecified (see lsh_params_set_dense_arithmetic).
 */
int lsh_hash_signs(const lsh_params_t *params, const float *d_data, uint64_t N,
                   uint64_t *d_out_words, void *stream);

/*
 * Compound keys (Sec. 3.2: H(v) is the concatenation of the codes of one table).  The k
 * ids of a vector form L groups of g = k/L consecutive ids; d_out_keys[v*L + l] =
 * sum_t uint32(h_{l*g+t}) * C^(g-1-t) mod 2^64 with C = 0x9E3779B97F4A7C15.  (The lossless
 * concatenation itself is d_buckets viewed as [N][L][g].)
 * Errors: INVALID_ARG (L == 0 or k % L != 0).
 */
int lsh_pack_keys(const lsh_params_t *params, const int32_t *d_buckets, uint64_t N, uint32_t L,
                  uint64_t *d_out_keys, void *stream);

/*
 * lsh_hash_fastlsh followed by lsh_pack_keys in one kernel: the ids never reach HBM.
 * UNSUPPORTED unless g = k/L is a power of two <= 64 (use the two calls otherwise).
 */
int lsh_hash_fastlsh_keys(const lsh_params_t *params, const float *d_data, uint64_t N, uint32_t L,
                          uint64_t *d_out_keys, void *stream);

/*
 * Bucket ids AND compound keys (Sec. 3.2) in one pass over the data, for callers that want
 * both (ids for exact verification or re-ranking, keys for the tables): d_out_buckets as
 * lsh_hash_fastlsh writes them, d_out_keys as lsh_pack_keys would fold them from exactly those
 * ids.  One kernel launch, the ids being in registers when the keys are folded, for objects
 * with one sample per function when g = k/L is 4, 8, 16 or 32 at n == 128 (k a multiple of 32,
 * default arithmetic), or a power of two from 4 to 64 with k a multiple of 4 on the shapes of
 * the streamed-list gather kernels (lists too long for registers: the 960-, 4096- and
 * 16384-dimensional workloads); any other object or L runs the two launches inside the call.
 * Errors: INVALID_ARG (null pointers, L == 0, k % L != 0), and those of lsh_hash_fastlsh.
 */
int lsh_hash_fastlsh_ids_keys(const lsh_params_t *params, const float *d_data, uint64_t N, uint32_t L,
                              int32_t *d_out_buckets, uint64_t *d_out_keys, void *stream);

/*
 * Raw fp32 projections a~_j^T S_j(v) (before + b, / w, floor), d_out_proj[v*k + j]; for
 * accuracy checks.  lsh_project_e2lsh requires m == n and uses the MFMA path.
 */
int lsh_project_fastlsh(const lsh_params_t *params, const float *d_data, uint64_t N,
                        float *d_out_proj, void *stream);
int lsh_project_e2lsh(const lsh_params_t *params, const float *d_data, uint64_t N,
                      float *d_out_proj, void *stream);

/*
 * Timing aid for callers without HIP bindings: records two events around `reps`
 * back-to-back launches of one hash call on `stream`, waits for them, and returns the
 * mean milliseconds per launch in *ms_per_launch.  `which`: 0 fastlsh ids, 1 e2lsh ids,
 * 2 signs, 3 pack_keys (d_in = ids), 4 fastlsh_keys.  L is used by 3 and 4.  This call
 * DOES synchronise (on its own events only).
 */
int lsh_time_launches(const lsh_params_t *params, int which, const void *d_in, uint64_t N,
                      uint32_t L, void *d_out, void *stream, int reps, float *ms_per_launch);

/*
 * LSH index (Sec. 3.2): L hash tables of <key, id> pairs and the lookup of a query's L buckets.
 * A table is the vector ids sorted by key (stable: ids ascending inside a bucket), a bucket a
 * contiguous run of them found by binary search; 12 bytes per vector and table of device
 * memory, owned by the index object.
 *
 * lsh_index_build: d_keys [N][L] (device, as written by lsh_pack_keys or
 *   lsh_hash_fastlsh_keys), N < 2^31, L <= 65535.  Sorts all L columns together on `stream`
 *   (a stable radix sort of this library, eight passes of 8 bits, the keys read in place) and
 *   does not wait: d_keys must stay alive until the stream has passed the build, and the index
 *   may be used by later work on the same stream (or after synchronising).  A second buffer of
 *   12 bytes per pair is allocated and released in stream order.
 * lsh_index_tables: N, L and the device arrays sorted keys [L][N], ids in key order [L][N]
 *   (owned by the index; any out pointer may be NULL).
 * lsh_index_probe: d_qkeys [Q][L] -> d_start [Q][L], d_count [Q][L]: the bucket of query q in
 *   table l is ids[l][start .. start + count).  count 0 = empty bucket.  Asynchronous.
 * lsh_index_candidate_offsets: exclusive prefix sum of `items` counts into d_offsets
 *   [items + 1] (the last entry is the total; items = 0 writes the single 0 and d_count may
 *   then be NULL); waits for the stream.
 * lsh_index_candidates: the buckets of every (query, table) item copied to
 *   d_out[offsets[item] ..): a query's combined candidate list is its L runs one after the
 *   other (an id met in several tables appears once per table).  Asynchronous.
 * lsh_index_nearest: processing of the candidates (Sec. 3.2, last paragraph): for every
 *   query the candidate with the smallest squared l2 distance over the full n-dimensional
 *   vectors (fp32; ties to the smaller id) -> d_best_id [Q] (0xFFFFFFFF when all L buckets
 *   are empty), d_best_dist [Q] (squared distance, +inf when none).  max_candidates = 0
 *   evaluates every candidate (the exact version); otherwise only the first max_candidates
 *   entries of the query's combined list are evaluated (the approximate version of the paper
 *   uses 3L).  d_data [N][n] must be the indexed vectors, d_queries [Q][n].  Asynchronous.
 * lsh_index_best_inner_product: the same walk for maximum inner product search (appendix): the
 *   candidate with the largest inner product v . u with the query (fp32; ties to the smaller
 *   id) -> d_best_id, d_best_ip [Q] (-inf when there is no candidate).  The index is then built
 *   from the keys of lsh_hash_mips_data and probed with those of lsh_hash_mips_query.
 * Errors: INVALID_ARG (null pointers, N = 0, N >= 2^31, L > 65535, called on another device than the one
 * the index was built on), ALLOC, HIP, NO_DEVICE, UNSUPPORTED (lsh_index_nearest and
 * lsh_index_best_inner_product: n > 16368).
 */
typedef struct lsh_index lsh_index_t; /* opaque */
int lsh_index_build(const uint64_t *d_keys, uint64_t N, uint32_t L, void *stream, lsh_index_t **out);
void lsh_index_destroy(lsh_index_t *index);
int lsh_index_tables(const lsh_index_t *index, uint64_t *N, uint32_t *L, const uint64_t **d_sorted_keys,
                     const uint32_t **d_sorted_ids);
int lsh_index_probe(const lsh_index_t *index, const uint64_t *d_qkeys, uint64_t Q, uint32_t *d_start,
                    uint32_t *d_count, void *stream);
int lsh_index_candidate_offsets(const uint32_t *d_count, uint64_t items, uint64_t *d_offsets, void *stream);
/*
 * lsh_index_candidate_offsets for callers that cannot allocate device memory or wait (code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): the same three
 * launches, with the scan's block sums in a 16 KB device array that the library holds on every
 * GPU it has run on until the process ends, instead of a temporary allocation.  Calls no
 * allocator, does not wait for the stream, and records no memset.  items <= 4,194,304 (2^22);
 * more returns UNSUPPORTED.  All calls on one GPU share that array: two calls whose kernels may
 * overlap in time (different streams, or a graph replayed while another call runs) race; calls
 * on one stream are ordered and safe.  Same outputs as lsh_index_candidate_offsets, bit for bit.
 * Errors: INVALID_ARG (null pointers), UNSUPPORTED (items above the limit), HIP.
 */
int lsh_index_candidate_offsets_static(const uint32_t *d_count, uint64_t items, uint64_t *d_offsets, void *stream);
int lsh_index_candidates(const lsh_index_t *index, const uint32_t *d_start, const uint32_t *d_count,
                         const uint64_t *d_offsets, uint64_t Q, uint32_t *d_out, void *stream);
int lsh_index_nearest(const lsh_index_t *index, const float *d_data, const float *d_queries, uint32_t n,
                      const uint32_t *d_start, const uint32_t *d_count, uint64_t Q, uint32_t max_candidates,
                      uint32_t *d_best_id, float *d_best_dist, void *stream);
int lsh_index_best_inner_product(const lsh_index_t *index, const float *d_data, const float *d_queries, uint32_t n,
                                 const uint32_t *d_start, const uint32_t *d_count, uint64_t Q,
                                 uint32_t max_candidates, uint32_t *d_best_id, float *d_best_ip, void *stream);

/*
 * Maximum inner product search (appendix "Extension to Maximum Inner Product Search").  With one
 * sample S_l per table (lsh_params_create_shared, L > 0; the appendix' "sample operator S" and
 * its constant kappa~ are per table here), data and queries are transformed as
 *     P~_l(v) = ( sqrt(kappa~_l^2 - ||S_l(v)||^2), S_l(v) ),   kappa~_l = max_i ||S_l(v_i)||
 *     Q~_l(u) = ( 0, S_l(u) / ||S_l(u)|| )            (the appendix asks for ||S(u)|| = 1)
 * and hashed with the l2 hash (Eq. 1) whose coefficient vector is (a0_j, a~_j), a0_j ~ N(0,1)
 * one more draw per function (generator table 3):
 *     data   h_j(v) = floor((a0_j sqrt(kappa~_l^2 - ||S_l(v)||^2) + a~_j . S_l(v) + b~_j) / w)
 *     query  h_j(u) = floor((a~_j . S_l(u) / ||S_l(u)|| + b~_j) / w),        l = j div (k / L)
 * The nearest transformed data vector of a transformed query is the data vector with the
 * largest inner product with the query on the sampled coordinates.
 *
 * lsh_mips_kappa      d_kappa2 [L] float (device) <- max over the N vectors of ||S_l(v)||^2;
 *                     accumulate != 0 keeps what d_kappa2 holds and only raises it (data that
 *                     arrives in batches), 0 starts from zero.  NaN coordinates are ignored.
 * lsh_hash_mips_data  d_out [N][k] int32 bucket ids of the data; d_kappa2 from lsh_mips_kappa
 *                     over ALL data vectors (a vector whose norm exceeds kappa~_l is hashed as
 *                     if it attained it).
 * lsh_hash_mips_query d_out [Q][k] int32 bucket ids of the queries (a query whose sub-vector is
 *                     all zero projects to 0).
 * lsh_project_mips_*  the value before "+ b~_j) / w" as float, for parity checks.
 * All arithmetic is fp32; a norm is the sum of four partial sums, each taken in the order the
 * kernel walks the sample (the kappa~ pass and the data hash walk it alike, so the vector that
 * attains kappa~_l gets exactly 0 under the root).  The ids feed
 * lsh_pack_keys and the index like any others.  Pointers are device pointers, outputs are the
 * caller's; asynchronous on `stream`.
 * Errors: as lsh_hash_fastlsh; UNSUPPORTED when the object has no shared samples or its shape
 * is outside the matrix-core kernels' (n % 4 == 0 and g % 4 == 0 at any n, see
 * lsh_params_create_shared; there is no per-function gather fallback for these calls).
 */
int lsh_mips_kappa(const lsh_params_t *params, const float *d_data, uint64_t N, int accumulate,
                   float *d_kappa2, void *stream);
int lsh_hash_mips_data(const lsh_params_t *params, const float *d_data, uint64_t N,
                       const float *d_kappa2, int32_t *d_out, void *stream);
int lsh_hash_mips_query(const lsh_params_t *params, const float *d_queries, uint64_t Q,
                        int32_t *d_out, void *stream);
int lsh_project_mips_data(const lsh_params_t *params, const float *d_data, uint64_t N,
                          const float *d_kappa2, float *d_out, void *stream);
int lsh_project_mips_query(const lsh_params_t *params, const float *d_queries, uint64_t Q,
                           float *d_out, void *stream);

/*
 * Collision probabilities (host functions, no GPU involved): what one needs to choose m and
 * the bucket width.  All pointers are host pointers.
 *
 * lsh_e2lsh_collision_probability: p_w(s) of Eq. 2 (Sec. 2.2) for two vectors at distance
 *   s >= 0 under bucket width w, in closed form.
 * lsh_pair_statistics: for a vector pair (v, u) of dimension n and sample size m, mu~ = m * mean
 *   and sigma~ = sqrt(m * variance) of the n squared coordinate differences (v_i - u_i)^2
 *   (Sec. 4.1, first paragraph).
 * lsh_fastlsh_collision_probability: p(s, sigma) of Eq. 9 (Sec. 4.1) under the paper's model
 *   s~^2 ~ N(mu~, sigma~^2) truncated to [0, inf), computed as the mixture of Eq. 2 over that
 *   distribution (absolute error below 1e-10).
 * lsh_fastlsh_moment_factors: epsilon and lambda of the moment lemma of Sec. 4.2:
 *   E[(s~X)^2] = mu~ (1 + epsilon), E[(s~X)^4] = 3 mu~^2 (1 + lambda).
 * lsh_equivalent_width: the FastLSH width w * sqrt(m / n) under which, for large m, the
 *   collision law equals E2LSH's with width w (corollary of Sec. 4.2; the variance of the
 *   sampled projection difference is m s^2 / n).
 * lsh_mips_collision_probability: the last equation of the appendix on maximum inner product
 *   search: the transformed pair's squared distance is s~^2 + delta with
 *   delta = kappa~^2 - ||S(v)||^2 >= 0, so the law of Eq. 9 applies with mean mu~ + delta.
 * Errors: INVALID_ARG (null pointer, non-positive or non-finite mu~ or w, negative sigma~ or delta).
 */
int lsh_e2lsh_collision_probability(double s, double w, double *p);
int lsh_pair_statistics(const float *v, const float *u, uint32_t n, uint32_t m, double *mu_tilde,
                        double *sigma_tilde);
int lsh_fastlsh_collision_probability(double mu_tilde, double sigma_tilde, double w, double *p);
int lsh_fastlsh_moment_factors(double mu_tilde, double sigma_tilde, double *epsilon, double *lambda);
double lsh_equivalent_width(uint32_t n, uint32_t m, double w);
int lsh_mips_collision_probability(double mu_tilde, double sigma_tilde, double delta, double w, double *p);

const char *lsh_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* LSH_H */
