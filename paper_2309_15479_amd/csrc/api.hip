// C ABI of liblsh (see include/lsh.h): argument checks, table upload, dispatch.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstring>
#include <new>

#include "lsh_internal.h"

namespace lsh {

uint32_t dense_col_tile();

void free_tables(lsh_params *p) {
    if (p->device < 0) return;
    int prev = -1;
    if (hipGetDevice(&prev) == hipSuccess && prev != p->device) (void)hipSetDevice(p->device);
    if (p->d_samples) (void)hipFree(p->d_samples);
    if (p->d_off) (void)hipFree(p->d_off);
    if (p->d_dense) (void)hipFree(p->d_dense);
    if (p->d_dense_planes) (void)hipFree(p->d_dense_planes);
    p->d_dense_planes = nullptr;
    if (p->d_triples) (void)hipFree(p->d_triples);
    if (p->d_list_len) (void)hipFree(p->d_list_len);
    if (p->d_stream) (void)hipFree(p->d_stream);
    p->d_triples = p->d_list_len = p->d_stream = nullptr;
    if (p->d_shared_coef) (void)hipFree(p->d_shared_coef);
    if (p->d_shared_sample_off) (void)hipFree(p->d_shared_sample_off);
    if (p->d_shared_offset) (void)hipFree(p->d_shared_offset);
    if (p->d_shared_extra) (void)hipFree(p->d_shared_extra);
    if (p->d_sr_lists) (void)hipFree(p->d_sr_lists);
    if (p->d_sr_offs) (void)hipFree(p->d_sr_offs);
    if (p->d_sr_extra) (void)hipFree(p->d_sr_extra);
    if (p->d_sr_list_len) (void)hipFree(p->d_sr_list_len);
    if (p->d_sr_stream) (void)hipFree(p->d_sr_stream);
    p->d_sr_lists = p->d_sr_offs = p->d_sr_list_len = p->d_sr_stream = p->d_sr_extra = nullptr;
    p->d_shared_extra = nullptr;
    p->d_shared_coef = nullptr;
    p->d_shared_sample_off = nullptr;
    p->d_shared_offset = nullptr;
    p->d_samples = nullptr;
    p->d_off = nullptr;
    p->d_dense = nullptr;
    if (prev >= 0 && prev != p->device) (void)hipSetDevice(prev);
    p->device = -1;
}

// Builds the kernel-side layouts from the canonical tables and copies them to the
// current device.  Returns LSH_OK with p->device == -1 when there is no GPU.
int upload_tables(lsh_params *p) {
    int count = 0;
    if (hipGetDeviceCount(&count) != hipSuccess || count <= 0) {
        (void)hipGetLastError();
        return LSH_OK;
    }
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return LSH_ERR_HIP;
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, dev) != hipSuccess) return LSH_ERR_HIP;
    p->num_cus = prop.multiProcessorCount;
    p->device = dev;

    const uint32_t m_pad = p->plan.m_pad;
    const uint32_t kpad = p->plan.supported ? p->plan.kpad : (p->k + 63) / 64 * 64;
    p->kpad_dense = 0;
    // n == 128: the matrix-core sign kernel takes any object's coefficients written out densely
    if (p->m == p->n || p->n == 128) p->kpad_dense = (p->k + dense_col_tile() - 1) / dense_col_tile() * dense_col_tile();
    // the wide matrix-core kernel reads offsets up to its function tiles
    // (every object with n a multiple of 4 may be switched to that kernel later, see
    // lsh_params_set_dense_arithmetic; the planes themselves are built here only for m == n)
    const bool wide = p->m == p->n && p->n != 128 && p->n % 4 == 0;
    const uint32_t kpad_wide = p->n % 4 == 0 ? (p->k + dense_wide_row_tile() - 1) / dense_wide_row_tile() * dense_wide_row_tile() : 0;
    uint32_t off_len = kpad > p->kpad_dense ? kpad : p->kpad_dense;
    if (off_len < kpad_wide) off_len = kpad_wide;

    int rc = LSH_OK;
    try {
        std::vector<float> off(off_len, 0.f);
        for (uint32_t j = 0; j < p->k; ++j) off[j] = p->off[j];
        if (hipMalloc(&p->d_off, off.size() * sizeof(float)) != hipSuccess) rc = LSH_ERR_ALLOC;
        if (rc == LSH_OK &&
            hipMemcpy(p->d_off, off.data(), off.size() * sizeof(float), hipMemcpyHostToDevice) != hipSuccess)
            rc = LSH_ERR_HIP;

        if (rc == LSH_OK && p->plan.supported && p->plan.ranged) {
            std::vector<uint32_t> words, list_len, stream_info;
            build_ranged_tables(p, words, list_len, stream_info);
            p->ranged_bar_stride = (uint32_t)(list_len.size() / p->plan.kblocks);
            for (size_t i = 1; i < stream_info.size(); i += 2)
                if (stream_info[i] % 2) rc = LSH_ERR_UNSUPPORTED;  // the kernel takes a tile's blocks two at a time
            auto upload = [&](void **dst, const void *src, size_t bytes) {
                if (rc == LSH_OK && hipMalloc(dst, bytes) != hipSuccess) rc = LSH_ERR_ALLOC;
                if (rc == LSH_OK && hipMemcpy(*dst, src, bytes, hipMemcpyHostToDevice) != hipSuccess) rc = LSH_ERR_HIP;
            };
            upload(&p->d_triples, words.data(), words.size() * sizeof(uint32_t));
            upload(&p->d_list_len, list_len.data(), list_len.size() * sizeof(uint32_t));
            upload(&p->d_stream, stream_info.data(), stream_info.size() * sizeof(uint32_t));
        }
        if (rc == LSH_OK && p->plan.supported && !p->plan.ranged) {
            // step-major [m_pad][kpad] in scheduled order; padding samples (and the lanes
            // beyond k) read a zero slot with coefficient 0
            const SampledPlan &pl = p->plan;
            const uint32_t slot_bytes = pl.sp * pl.rt * 4u;
            std::vector<Sample> tab((size_t)m_pad * kpad, Sample{p->n * slot_bytes, 0.f});
            for (uint32_t j = 0; j < p->k; ++j)
                for (uint32_t i = 0; i < m_pad; ++i) {
                    Sample &s = tab[(size_t)i * kpad + j];
                    const uint32_t e = p->order[(size_t)j * m_pad + i];
                    if (e & kPadSample) {
                        s.lds_byte_offset = (p->n + (e & ~kPadSample)) * slot_bytes;
                        // the zero slot whose class equals the requested one
                        const uint32_t want = e & ~kPadSample;
                        for (uint32_t z = p->n; z < p->n + pl.classes; ++z)
                            if (z % pl.classes == want) s.lds_byte_offset = z * slot_bytes;
                        s.coef = 0.f;
                    } else {
                        const uint32_t pos = e & ~kCopyB;
                        const uint32_t c = p->idx[(size_t)j * p->m + pos];
                        // second copy: after the first copy and its zero slots
                        s.lds_byte_offset = (e & kCopyB)
                                                ? (p->n + pl.classes + copy_b_slot(c, pl.classes)) * slot_bytes
                                                : c * slot_bytes;
                        s.coef = p->coef[(size_t)j * p->m + pos];
                    }
                }
            if (hipMalloc(&p->d_samples, tab.size() * sizeof(Sample)) != hipSuccess) rc = LSH_ERR_ALLOC;
            if (rc == LSH_OK && hipMemcpy(p->d_samples, tab.data(), tab.size() * sizeof(Sample),
                                          hipMemcpyHostToDevice) != hipSuccess)
                rc = LSH_ERR_HIP;
        }
        if (rc == LSH_OK && p->shared_plan.supported) {
            std::vector<float> coef, offset, extra;
            std::vector<uint32_t> sample_off;
            build_shared_tables(p, coef, sample_off, offset, extra);
            auto upload = [&](void **dst, const void *src, size_t bytes) {
                if (rc == LSH_OK && hipMalloc(dst, bytes) != hipSuccess) rc = LSH_ERR_ALLOC;
                if (rc == LSH_OK && hipMemcpy(*dst, src, bytes, hipMemcpyHostToDevice) != hipSuccess) rc = LSH_ERR_HIP;
            };
            upload(reinterpret_cast<void **>(&p->d_shared_coef), coef.data(), coef.size() * sizeof(float));
            upload(reinterpret_cast<void **>(&p->d_shared_sample_off), sample_off.data(),
                   sample_off.size() * sizeof(uint32_t));
            upload(reinterpret_cast<void **>(&p->d_shared_offset), offset.data(), offset.size() * sizeof(float));
            upload(reinterpret_cast<void **>(&p->d_shared_extra), extra.data(), extra.size() * sizeof(float));
        }
        if (rc == LSH_OK && p->shared_ranged_plan.supported) {
            std::vector<float> lists;
            std::vector<uint32_t> offs, stage_turns, stream_info;
            std::vector<float> extra;
            build_shared_ranged_tables(p, p->shared_ranged_plan, lists, offs, stage_turns, stream_info, &extra);
            auto upload = [&](void **dst, const void *src, size_t bytes) {
                if (rc == LSH_OK && hipMalloc(dst, bytes) != hipSuccess) rc = LSH_ERR_ALLOC;
                if (rc == LSH_OK && hipMemcpy(*dst, src, bytes, hipMemcpyHostToDevice) != hipSuccess) rc = LSH_ERR_HIP;
            };
            upload(&p->d_sr_lists, lists.data(), lists.size() * sizeof(float));
            upload(&p->d_sr_offs, offs.data(), offs.size() * sizeof(uint32_t));
            upload(&p->d_sr_extra, extra.data(), extra.size() * sizeof(float));
            upload(&p->d_sr_list_len, stage_turns.data(), stage_turns.size() * sizeof(uint32_t));
            upload(&p->d_sr_stream, stream_info.data(), stream_info.size() * sizeof(uint32_t));
        }
        if (rc == LSH_OK && p->kpad_dense) {
            // m == n: S_j is the identity, so the canonical coefficient table IS the dense
            // matrix A [k][n]; rows up to the tile grid are zero.  m < n: zeros at the coordinates
            // a function does not sample; a coordinate drawn more than once gets the sum
            std::vector<float> dense((size_t)p->kpad_dense * p->n, 0.f);
            if (p->m == p->n) {
                std::copy(p->coef.begin(), p->coef.end(), dense.begin());
            } else {
                for (uint32_t j = 0; j < p->k; ++j)
                    for (uint32_t i = 0; i < p->m; ++i)
                        dense[(size_t)j * p->n + p->idx[(size_t)j * p->m + i]] += p->coef[(size_t)j * p->m + i];
            }
            if (hipMalloc(&p->d_dense, dense.size() * sizeof(float)) != hipSuccess) rc = LSH_ERR_ALLOC;
            if (rc == LSH_OK && hipMemcpy(p->d_dense, dense.data(), dense.size() * sizeof(float),
                                          hipMemcpyHostToDevice) != hipSuccess)
                rc = LSH_ERR_HIP;
            if (rc == LSH_OK && wide) {
                // the same matrix as exact three-way bf16 splits, for the wide matrix-core kernel
                const uint32_t npad = (p->n + dense_wide_col_step() - 1) / dense_wide_col_step() * dense_wide_col_step();
                std::vector<uint16_t> planes;
                build_dense_planes(p->coef.data(), p->k, p->n, kpad_wide, npad, planes);
                if (hipMalloc(&p->d_dense_planes, planes.size() * sizeof(uint16_t)) != hipSuccess) rc = LSH_ERR_ALLOC;
                if (rc == LSH_OK && hipMemcpy(p->d_dense_planes, planes.data(), planes.size() * sizeof(uint16_t),
                                              hipMemcpyHostToDevice) != hipSuccess)
                    rc = LSH_ERR_HIP;
            }
        }
    } catch (const std::bad_alloc &) {
        rc = LSH_ERR_ALLOC;
    }
    if (rc != LSH_OK) {
        (void)hipGetLastError();
        free_tables(p);
    }
    return rc;
}

namespace {

// N == 0 is valid with any data/out pointers (an empty tensor has no storage)
int check_hash_args(const lsh_params *p, const void *d_in, const void *d_out, uint64_t N) {
    if (!p) return LSH_ERR_INVALID_ARG;
    if (N && (!d_in || !d_out)) return LSH_ERR_INVALID_ARG;
    if (p->device < 0) return LSH_ERR_NO_DEVICE;
    int dev = -1;  // the tables live on the device that was current at create time
    if (hipGetDevice(&dev) != hipSuccess) return LSH_ERR_HIP;
    if (dev != p->device) return LSH_ERR_INVALID_ARG;
    return LSH_OK;
}

bool is_pow2(uint32_t x) { return x && !(x & (x - 1)); }

}  // namespace
}  // namespace lsh

using namespace lsh;

extern "C" {

int lsh_params_create_shared(uint32_t n, uint32_t k, uint32_t m, float w, uint64_t seed, uint32_t flags,
                             uint32_t L, lsh_params_t **out) {
    if (!out) return LSH_ERR_INVALID_ARG;
    *out = nullptr;
    if (!n || !k || !m || m > n || !(w > 0.f) || !std::isfinite(w)) return LSH_ERR_INVALID_ARG;
    if (flags & ~LSH_SAMPLE_WITH_REPLACEMENT) return LSH_ERR_INVALID_ARG;
    if ((uint64_t)k * m > (1ull << 31)) return LSH_ERR_INVALID_ARG;
    if (L && k % L) return LSH_ERR_INVALID_ARG;
    lsh_params *p = new (std::nothrow) lsh_params;
    if (!p) return LSH_ERR_ALLOC;
    p->n = n; p->k = k; p->m = m; p->w = w; p->seed = seed; p->flags = flags;
    p->shared_tables = L;
    int rc = generate_tables(n, k, m, w, seed, flags, L ? k / L : 1, p->idx, p->coef, p->off);
    if (rc == LSH_OK && L) rc = generate_extra_coefficients(k, seed, p->extra);
    if (rc == LSH_OK) {
        p->plan = plan_sampled(n, k, m);
        p->shared_plan = plan_shared(n, k, m, L);
        if (!p->shared_plan.supported) p->shared_ranged_plan = plan_shared_ranged(n, k, m, L);
        if (p->plan.supported) {
            try {
                const SampledPlan &pl = p->plan;
                p->schedule_cost =
                    pl.ranged ? schedule_windowed(p->idx, k, m, pl.chunk, pl.nchunks, pl.stages, kWindowLook,
                                                  pl.fpt * kRangeComputeWaves, 4 * pl.qpf,
                                                  m + (uint32_t)(0.5 * std::sqrt((double)m)),  // spare steps: see schedule_windowed
                                                  pl.group, pl.classes,
                                                  p->chunk_steps, p->order)
                              : schedule_samples(p->idx, k, m, pl.m_pad, pl.group, pl.classes, pl.copies,
                                                  p->order);
            } catch (const std::bad_alloc &) {
                rc = LSH_ERR_ALLOC;
            }
            // a schedule the kernel could not follow must never reach the device
            try {
                if (rc == LSH_OK && p->plan.ranged && !ranged_schedule_valid(p)) rc = LSH_ERR_UNSUPPORTED;
            } catch (const std::bad_alloc &) {
                rc = LSH_ERR_ALLOC;
            }
        }
    }
    if (rc == LSH_OK) rc = upload_tables(p);
    if (rc != LSH_OK) {
        delete p;
        return rc;
    }
    *out = p;
    return LSH_OK;
}

int lsh_params_create_ex(uint32_t n, uint32_t k, uint32_t m, float w, uint64_t seed, uint32_t flags,
                         lsh_params_t **out) {
    return lsh_params_create_shared(n, k, m, w, seed, flags, 0, out);
}

int lsh_params_create(uint32_t n, uint32_t k, uint32_t m, float w, uint64_t seed, lsh_params_t **out) {
    return lsh_params_create_ex(n, k, m, w, seed, LSH_SAMPLE_WITHOUT_REPLACEMENT, out);
}

void lsh_params_destroy(lsh_params_t *p) {
    if (!p) return;
    free_tables(p);
    delete p;
}

int lsh_params_get_indices(const lsh_params_t *p, uint32_t *out) {
    if (!p || !out) return LSH_ERR_INVALID_ARG;
    std::copy(p->idx.begin(), p->idx.end(), out);
    return LSH_OK;
}

int lsh_params_get_coeffs(const lsh_params_t *p, float *out) {
    if (!p || !out) return LSH_ERR_INVALID_ARG;
    std::copy(p->coef.begin(), p->coef.end(), out);
    return LSH_OK;
}

int lsh_params_get_offsets(const lsh_params_t *p, float *out) {
    if (!p || !out) return LSH_ERR_INVALID_ARG;
    std::copy(p->off.begin(), p->off.end(), out);
    return LSH_OK;
}

int lsh_params_get_shape(const lsh_params_t *p, uint32_t *n, uint32_t *k, uint32_t *m, uint32_t *flags,
                         float *w, uint64_t *seed) {
    if (!p) return LSH_ERR_INVALID_ARG;
    if (n) *n = p->n;
    if (k) *k = p->k;
    if (m) *m = p->m;
    if (flags) *flags = p->flags;
    if (w) *w = p->w;
    if (seed) *seed = p->seed;
    return LSH_OK;
}

int lsh_params_get_tables(const lsh_params_t *p, uint32_t *shared_tables) {
    if (!p || !shared_tables) return LSH_ERR_INVALID_ARG;
    *shared_tables = p->shared_tables;
    return LSH_OK;
}

int lsh_params_get_mips_coeffs(const lsh_params_t *p, float *out) {
    if (!p || !out) return LSH_ERR_INVALID_ARG;
    if (p->extra.empty()) return LSH_ERR_UNSUPPORTED;
    std::copy(p->extra.begin(), p->extra.end(), out);
    return LSH_OK;
}

int lsh_params_get_schedule(const lsh_params_t *p, uint32_t *order, uint32_t *steps, uint32_t *group,
                            uint32_t *classes, uint64_t *modelled_passes) {
    if (!p) return LSH_ERR_INVALID_ARG;
    const SampledPlan &pl = p->plan;
    if (!pl.supported) return LSH_ERR_UNSUPPORTED;
    uint32_t nsteps = pl.m_pad;
    const bool by_range = pl.ranged;
    const uint32_t sets_per_wg = pl.fpt * kRangeComputeWaves;
    std::vector<uint32_t> wg_steps;
    if (by_range) {  // the longest list of any workgroup (all lists of a workgroup are equally long)
        nsteps = 0;
        wg_steps.assign(pl.kblocks, 0);
        for (uint32_t y = 0; y < pl.kblocks; ++y) {
            for (uint32_t q = 0; q < pl.stages; ++q) wg_steps[y] += p->chunk_steps[(size_t)y * pl.stages + q];
            nsteps = std::max(nsteps, wg_steps[y]);
        }
    }
    if (steps) *steps = nsteps;
    if (group) *group = pl.group;
    if (classes) *classes = pl.classes;
    if (modelled_passes) *modelled_passes = p->schedule_cost;
    if (!order) return LSH_OK;
    if (!by_range) {
        std::copy(p->order.begin(), p->order.end(), order);
        return LSH_OK;
    }
    std::fill(order, order + (size_t)p->k * nsteps, 0xFFFFFFFFu);
    size_t base = 0;  // p->order: set after set, each stage after stage, steps x 64
    for (uint32_t w = 0; w < (p->k + 63) / 64; ++w) {
        const uint32_t len = wg_steps[w / sets_per_wg];
        for (uint32_t st = 0; st < len; ++st)
            for (uint32_t l = 0; l < 64 && w * 64 + l < p->k; ++l)
                order[(size_t)(w * 64 + l) * nsteps + st] = p->order[base + (size_t)st * 64 + l];
        base += (size_t)len * 64;
    }
    return LSH_OK;
}

int lsh_hash_fastlsh(const lsh_params_t *p, const float *d_data, uint64_t N, int32_t *d_out, void *stream) {
    int rc = check_hash_args(p, d_data, d_out, N);
    if (rc != LSH_OK || N == 0) return rc;
    if (p->shared_plan.supported) return launch_shared(p, 0, d_data, N, d_out, stream);
    if (p->shared_ranged_plan.supported) return launch_shared_ranged(p, 0, d_data, N, d_out, stream);
    if (p->dense_arithmetic != LSH_DENSE_FP32 && dense_split_supported(p))
        return launch_dense_split(p, 0, d_data, N, d_out, stream);
    if (p->dense_arithmetic == LSH_DENSE_MATRIX && p->d_dense_planes)
        return launch_dense_wide(p, false, d_data, N, d_out, stream);
    return launch_sampled(p, Epilogue::Ids, d_data, N, d_out, 0, stream);
}

int lsh_project_fastlsh(const lsh_params_t *p, const float *d_data, uint64_t N, float *d_out, void *stream) {
    int rc = check_hash_args(p, d_data, d_out, N);
    if (rc != LSH_OK || N == 0) return rc;
    if (p->shared_plan.supported) return launch_shared(p, 1, d_data, N, d_out, stream);
    if (p->shared_ranged_plan.supported) return launch_shared_ranged(p, 1, d_data, N, d_out, stream);
    if (p->dense_arithmetic != LSH_DENSE_FP32 && dense_split_supported(p))
        return launch_dense_split(p, 1, d_data, N, d_out, stream);
    if (p->dense_arithmetic == LSH_DENSE_MATRIX && p->d_dense_planes)
        return launch_dense_wide(p, true, d_data, N, d_out, stream);
    return launch_sampled(p, Epilogue::Proj, d_data, N, d_out, 0, stream);
}

int lsh_hash_signs(const lsh_params_t *p, const float *d_data, uint64_t N, uint64_t *d_out, void *stream) {
    int rc = check_hash_args(p, d_data, d_out, N);
    if (rc != LSH_OK || N == 0) return rc;
    if (p->dense_arithmetic != LSH_DENSE_FP32 && dense_split_signs_supported(p))
        return launch_dense_split(p, 2, d_data, N, d_out, stream);
    return launch_sampled(p, Epilogue::Signs, d_data, N, d_out, 0, stream);
}

int lsh_hash_fastlsh_keys(const lsh_params_t *p, const float *d_data, uint64_t N, uint32_t L,
                          uint64_t *d_out, void *stream) {
    int rc = check_hash_args(p, d_data, d_out, N);
    if (rc != LSH_OK) return rc;
    if (!L || p->k % L) return LSH_ERR_INVALID_ARG;
    const uint32_t g = p->k / L;
    if (!is_pow2(g) || g > 64) return LSH_ERR_UNSUPPORTED;
    if (N == 0) return LSH_OK;
    if (shared_keys_ok(p, L)) return launch_shared(p, 2, d_data, N, d_out, stream);
    if (shared_ranged_keys_ok(p, L)) return launch_shared_ranged(p, 6, d_data, N, nullptr, stream, nullptr, 0, d_out);
    if (p->dense_arithmetic != LSH_DENSE_FP32 && !p->shared_plan.supported && dense_split_keys_supported(p, L))
        return launch_dense_split(p, 3, d_data, N, d_out, stream, L);
    return launch_sampled(p, Epilogue::Keys, d_data, N, d_out, L, stream);
}

int lsh_hash_fastlsh_ids_keys(const lsh_params_t *p, const float *d_data, uint64_t N, uint32_t L,
                              int32_t *d_ids, uint64_t *d_keys, void *stream) {
    int rc = check_hash_args(p, d_data, d_ids, N);
    if (rc != LSH_OK) return rc;
    if (!L || p->k % L || (N && !d_keys)) return LSH_ERR_INVALID_ARG;
    if (N == 0) return LSH_OK;
    // one launch where a kernel has the epilogue for it; the results are those of the two calls
    // either way (the keys are folded from the very ids that are stored)
    if (shared_ranged_keys_ok(p, L)) return launch_shared_ranged(p, 6, d_data, N, d_ids, stream, nullptr, 0, d_keys);
    const bool per_function = !p->shared_plan.supported && !p->shared_ranged_plan.supported;
    if (per_function && p->dense_arithmetic != LSH_DENSE_FP32 && dense_split_keys_supported(p, L))
        return launch_dense_split(p, 4, d_data, N, d_ids, stream, L, d_keys);
    if (per_function && !(p->dense_arithmetic != LSH_DENSE_FP32 && dense_split_supported(p)) &&
        sampled_ids_keys_supported(p, L))
        return launch_sampled(p, Epilogue::IdsKeys, d_data, N, d_ids, L, stream, d_keys);
    rc = lsh_hash_fastlsh(p, d_data, N, d_ids, stream);
    if (rc != LSH_OK) return rc;
    return launch_pack(p, d_ids, N, L, d_keys, stream);
}

int lsh_mips_kappa(const lsh_params_t *p, const float *d_data, uint64_t N, int accumulate, float *d_kappa2,
                   void *stream) {
    if (!d_kappa2) return LSH_ERR_INVALID_ARG;
    int rc = check_hash_args(p, d_data, d_kappa2, N);
    if (rc != LSH_OK) return rc;
    if (!p->shared_plan.supported && !p->shared_ranged_plan.supported) return LSH_ERR_UNSUPPORTED;
    if (!accumulate) rc = clear_floats(d_kappa2, p->shared_tables, stream);
    if (rc != LSH_OK || N == 0) return rc;
    if (p->shared_ranged_plan.supported) return launch_shared_ranged(p, 3, d_data, N, d_kappa2, stream);
    return launch_shared(p, 3, d_data, N, d_kappa2, stream);
}

static int mips_data(const lsh_params_t *p, const float *d_data, uint64_t N, const float *d_kappa2, void *d_out,
                     void *stream, int raw) {
    int rc = check_hash_args(p, d_data, d_out, N);
    if (rc != LSH_OK) return rc;
    if (N && !d_kappa2) return LSH_ERR_INVALID_ARG;
    if (!p->shared_plan.supported && !p->shared_ranged_plan.supported) return LSH_ERR_UNSUPPORTED;
    if (N == 0) return LSH_OK;
    if (p->shared_ranged_plan.supported) return launch_shared_ranged(p, 4, d_data, N, d_out, stream, d_kappa2, raw);
    return launch_shared(p, 4, d_data, N, d_out, stream, d_kappa2, raw);
}

static int mips_query(const lsh_params_t *p, const float *d_queries, uint64_t Q, void *d_out, void *stream, int raw) {
    int rc = check_hash_args(p, d_queries, d_out, Q);
    if (rc != LSH_OK) return rc;
    if (!p->shared_plan.supported && !p->shared_ranged_plan.supported) return LSH_ERR_UNSUPPORTED;
    if (Q == 0) return LSH_OK;
    if (p->shared_ranged_plan.supported) return launch_shared_ranged(p, 5, d_queries, Q, d_out, stream, nullptr, raw);
    return launch_shared(p, 5, d_queries, Q, d_out, stream, nullptr, raw);
}

int lsh_hash_mips_data(const lsh_params_t *p, const float *d_data, uint64_t N, const float *d_kappa2,
                       int32_t *d_out, void *stream) {
    return mips_data(p, d_data, N, d_kappa2, d_out, stream, 0);
}

int lsh_project_mips_data(const lsh_params_t *p, const float *d_data, uint64_t N, const float *d_kappa2,
                          float *d_out, void *stream) {
    return mips_data(p, d_data, N, d_kappa2, d_out, stream, 1);
}

int lsh_hash_mips_query(const lsh_params_t *p, const float *d_queries, uint64_t Q, int32_t *d_out, void *stream) {
    return mips_query(p, d_queries, Q, d_out, stream, 0);
}

int lsh_project_mips_query(const lsh_params_t *p, const float *d_queries, uint64_t Q, float *d_out,
                           void *stream) {
    return mips_query(p, d_queries, Q, d_out, stream, 1);
}

int lsh_hash_e2lsh(const lsh_params_t *p, const float *d_data, uint64_t N, int32_t *d_out, void *stream) {
    int rc = check_hash_args(p, d_data, d_out, N);
    if (rc != LSH_OK) return rc;
    if (p->m != p->n) return LSH_ERR_INVALID_ARG;
    if (N == 0) return LSH_OK;
    if (p->dense_arithmetic != LSH_DENSE_FP32 && dense_split_supported(p))
        return launch_dense_split(p, 0, d_data, N, d_out, stream);
    if (p->dense_arithmetic != LSH_DENSE_FP32 && dense_wide_supported(p))
        return launch_dense_wide(p, false, d_data, N, d_out, stream);
    return launch_dense(p, false, d_data, N, d_out, stream);
}

int lsh_project_e2lsh(const lsh_params_t *p, const float *d_data, uint64_t N, float *d_out, void *stream) {
    int rc = check_hash_args(p, d_data, d_out, N);
    if (rc != LSH_OK) return rc;
    if (p->m != p->n) return LSH_ERR_INVALID_ARG;
    if (N == 0) return LSH_OK;
    if (p->dense_arithmetic != LSH_DENSE_FP32 && dense_split_supported(p))
        return launch_dense_split(p, 1, d_data, N, d_out, stream);
    if (p->dense_arithmetic != LSH_DENSE_FP32 && dense_wide_supported(p))
        return launch_dense_wide(p, true, d_data, N, d_out, stream);
    return launch_dense(p, true, d_data, N, d_out, stream);
}

int lsh_params_set_dense_arithmetic(lsh_params_t *p, int mode) {
    if (!p || (mode != LSH_DENSE_AUTO && mode != LSH_DENSE_FP32 && mode != LSH_DENSE_MATRIX)) return LSH_ERR_INVALID_ARG;
    if (mode == LSH_DENSE_MATRIX && p->n != 128 && !p->d_dense_planes) {
        // the sampled coefficients written out over all n coordinates (zeros where a function does
        // not sample, sums where it samples a coordinate more than once), as the bf16 planes of
        // the matrix-core kernel for any n: built on first use
        if (p->n % 4 != 0 || (uint64_t)p->k * 4 >= (1ull << 32)) return LSH_ERR_UNSUPPORTED;
        if (p->device < 0) return LSH_ERR_NO_DEVICE;
        int dev = -1;
        if (hipGetDevice(&dev) != hipSuccess) return LSH_ERR_HIP;
        if (dev != p->device) return LSH_ERR_INVALID_ARG;
        try {
            std::vector<float> dense((size_t)p->k * p->n, 0.f);
            for (uint32_t j = 0; j < p->k; ++j)
                for (uint32_t i = 0; i < p->m; ++i)
                    dense[(size_t)j * p->n + p->idx[(size_t)j * p->m + i]] += p->coef[(size_t)j * p->m + i];
            const uint32_t kpad_wide = (p->k + dense_wide_row_tile() - 1) / dense_wide_row_tile() * dense_wide_row_tile();
            const uint32_t npad = (p->n + dense_wide_col_step() - 1) / dense_wide_col_step() * dense_wide_col_step();
            std::vector<uint16_t> planes;
            build_dense_planes(dense.data(), p->k, p->n, kpad_wide, npad, planes);
            void *d = nullptr;
            if (hipMalloc(&d, planes.size() * sizeof(uint16_t)) != hipSuccess) {
                (void)hipGetLastError();
                return LSH_ERR_ALLOC;
            }
            if (hipMemcpy(d, planes.data(), planes.size() * sizeof(uint16_t), hipMemcpyHostToDevice) != hipSuccess) {
                (void)hipFree(d);
                (void)hipGetLastError();
                return LSH_ERR_HIP;
            }
            p->d_dense_planes = d;
        } catch (const std::bad_alloc &) {
            return LSH_ERR_ALLOC;
        }
    }
    p->dense_arithmetic = mode;
    return LSH_OK;
}

int lsh_pack_keys(const lsh_params_t *p, const int32_t *d_ids, uint64_t N, uint32_t L, uint64_t *d_keys,
                  void *stream) {
    int rc = check_hash_args(p, d_ids, d_keys, N);
    if (rc != LSH_OK) return rc;
    if (!L || p->k % L) return LSH_ERR_INVALID_ARG;
    if (N == 0) return LSH_OK;
    return launch_pack(p, d_ids, N, L, d_keys, stream);
}

int lsh_time_launches(const lsh_params_t *p, int which, const void *d_in, uint64_t N, uint32_t L,
                      void *d_out, void *stream, int reps, float *ms_per_launch) {
    if (!ms_per_launch || reps <= 0 || which < 0 || which > 4) return LSH_ERR_INVALID_ARG;
    int rc = check_hash_args(p, d_in, d_out, N);
    if (rc != LSH_OK) return rc;
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    hipEvent_t t0 = nullptr, t1 = nullptr;
    if (hipEventCreate(&t0) != hipSuccess) return LSH_ERR_HIP;
    if (hipEventCreate(&t1) != hipSuccess) {
        (void)hipEventDestroy(t0);
        return LSH_ERR_HIP;
    }
    rc = hipEventRecord(t0, s) == hipSuccess ? LSH_OK : LSH_ERR_HIP;
    for (int r = 0; r < reps && rc == LSH_OK; ++r) {
        switch (which) {
            case 0: rc = lsh_hash_fastlsh(p, (const float *)d_in, N, (int32_t *)d_out, stream); break;
            case 1: rc = lsh_hash_e2lsh(p, (const float *)d_in, N, (int32_t *)d_out, stream); break;
            case 2: rc = lsh_hash_signs(p, (const float *)d_in, N, (uint64_t *)d_out, stream); break;
            case 3: rc = lsh_pack_keys(p, (const int32_t *)d_in, N, L, (uint64_t *)d_out, stream); break;
            default: rc = lsh_hash_fastlsh_keys(p, (const float *)d_in, N, L, (uint64_t *)d_out, stream);
        }
    }
    if (rc == LSH_OK && hipEventRecord(t1, s) != hipSuccess) rc = LSH_ERR_HIP;
    if (rc == LSH_OK && hipEventSynchronize(t1) != hipSuccess) rc = LSH_ERR_HIP;
    float ms = 0.f;
    if (rc == LSH_OK && hipEventElapsedTime(&ms, t0, t1) != hipSuccess) rc = LSH_ERR_HIP;
    (void)hipEventDestroy(t0);
    (void)hipEventDestroy(t1);
    if (rc == LSH_OK) *ms_per_launch = ms / (float)reps;
    return rc;
}

const char *lsh_status_string(int status) {
    switch (status) {
        case LSH_OK: return "ok";
        case LSH_ERR_INVALID_ARG: return "invalid argument";
        case LSH_ERR_ALLOC: return "allocation failed";
        case LSH_ERR_HIP: return "HIP runtime error";
        case LSH_ERR_UNSUPPORTED: return "unsupported shape";
        case LSH_ERR_NO_DEVICE: return "params object has no device tables";
        default: return "unknown status";
    }
}

}  // extern "C"
