// Internal declarations shared by the host and device translation units of liblsh.
#pragma once
#include <cstddef>
#include <cstdint>
#include <vector>

#include "lsh.h"

namespace lsh {

// One entry of the device table of the sampled-projection kernel: where to read in the
// LDS tile (byte offset of the sampled coordinate's slot) and the coefficient.
struct Sample {
    uint32_t lds_byte_offset;
    float coef;
};

// How the sampled kernel is launched for one params object; fixed at create time.
// LDS tile layout: [coordinate slot][sub-tile (+1 pad slot when sub > 1)][rt vectors],
// n coordinate slots followed by `classes` zero slots (one per bank class).
struct SampledPlan {
    uint32_t rt = 0;         // vectors per LDS read (4: 16-byte reads, 2: 8-byte, 1: 4-byte)
    uint32_t sub = 0;        // sub-tiles of rt vectors per workgroup tile (8, 4, 2 or 1)
    uint32_t sp = 0;         // sub-tile slots per coordinate: sub + 1 (odd) or 1
    uint32_t group = 0;      // lanes served together by one pass of an LDS read
    uint32_t classes = 0;    // bank classes: slots c, c' collide iff c % classes == c' % classes
    uint32_t m_pad = 0;      // samples per function, padded to the register chunk
    uint32_t block = 0;      // threads per workgroup = functions per workgroup
    uint32_t kblocks = 0;    // workgroups along the function axis
    uint32_t kpad = 0;       // block * kblocks >= k
    uint32_t lds_bytes = 0;  // LDS bytes of one tile buffer (both copies when copies == 2)
    uint32_t copies = 1;     // 2: the tile is kept twice, the second copy with rotated bank classes
    bool reg_table = false;  // register-list kernel: (offset, coef) lists live in VGPRs
    bool ranged = false;     // ranged kernel (ranged_kernel.hip): lists cut by coordinate range, packed quads of entries
    uint32_t chunk = 0, nchunks = 0;  // ranged kernel: coordinates per range, number of ranges
    uint32_t stages = 0;     // ranged kernel: steps of the range ring per tile (>= nchunks; divides or is a multiple of the ring)
    uint32_t fpt = 1;        // ranged kernel: functions per lane
    uint32_t qpf = 1;        // ranged kernel: quads of entries per function in one list block
    uint32_t prefetch = 0;   // register-list kernel: 64-coordinate chunks fetched per wave and tile
    bool supported = false;
};

// Plan of the shared-sample kernel (shared_kernel.hip): one sample S per table of g functions.
struct SharedPlan {
    uint32_t g = 0;                 // functions per table
    uint32_t rows = 0;              // vectors per LDS tile
    uint32_t waves = 0;             // waves per workgroup (16 or 8)
    uint32_t per_cu = 0;            // workgroups per CU
    uint32_t stride = 0;            // floats per tile row
    uint32_t ksteps = 0;            // MFMA steps of 4 samples: 8 (m <= 32) or 16 (m <= 64)
    uint32_t blocks_per_table = 0;  // blocks of 16 functions per table
    uint32_t nblocks = 0;           // L * blocks_per_table
    uint32_t rb = 0;                // blocks per wave
    uint32_t kblocks = 0;           // workgroups along the function axis
    uint32_t lds_bytes = 0;
    bool staged = false;            // ids leave as whole 128-byte lines (lanes pair up their 16-byte pieces)
    bool supported = false;
};

// Plan of the shared-sample kernel for large dimensions (shared_ranged_kernel.hip).
struct SharedRangedPlan {
    uint32_t g = 0;                 // functions per table
    uint32_t blocks_per_table = 0;  // blocks of 16 functions per table
    uint32_t nblocks = 0;           // L * blocks_per_table
    uint32_t kblocks = 0;           // workgroups along the function axis
    uint32_t bpw = 0;               // blocks per contracting wave (4, 8 or 16)
    uint32_t nchunks = 0;           // coordinate ranges of kWindowCoords that hold data
    uint32_t stages = 0;            // stages per tile: nchunks rounded up to a multiple of the ring slots
    bool supported = false;
};

constexpr uint32_t kPadSample = 0x80000000u;  // schedule entry: padding sample | bank class
constexpr uint32_t kCopyB = 0x40000000u;      // schedule entry: read the sample from the second tile copy

// Slot of coordinate c in the second tile copy: inside every run of `classes` coordinates the
// slots are rotated by the run's number, so coordinates that share a bank class in the first
// copy (equal c % classes) fall into different classes in the second.
inline uint32_t copy_b_slot(uint32_t c, uint32_t classes) {
    return c / classes * classes + (c + c / classes) % classes;
}

}  // namespace lsh

struct lsh_params {
    uint32_t n = 0, k = 0, m = 0, flags = 0;
    uint32_t shared_tables = 0;  // L when the k/L functions of a table share one sample S, else 0
    float w = 0.f;
    uint64_t seed = 0;
    // canonical host tables
    std::vector<uint32_t> idx;  // [k][m]
    std::vector<float> coef;    // [k][m]
    std::vector<float> off;     // [k]
    std::vector<float> extra;   // [k] a0 of the maximum-inner-product transform (one sample per table only)
    // device side
    int device = -1;  // -1: no device tables
    int num_cus = 0;
    lsh::SampledPlan plan;
    std::vector<uint32_t> order;       // [k][m_pad] visiting order of each function's samples
    uint64_t schedule_cost = 0;        // modelled LDS passes (see schedule.cpp)
    std::vector<uint32_t> chunk_steps; // ranged plan: [workgroups along the function axis][stages] entries per function and stage
    lsh::Sample *d_samples = nullptr;  // flat plans: [m_pad][kpad] step-major
    // ranged plan: packed list blocks (quads of entries), barriers after each block [kblocks][blocks + 1], streams {first block, blocks}
    void *d_triples = nullptr, *d_list_len = nullptr, *d_stream = nullptr;
    uint32_t ranged_bar_stride = 0;    // barrier counts per workgroup in d_list_len
    float *d_off = nullptr;            // [kpad]
    float *d_dense = nullptr;          // [kpad_dense][n]: row j = a_j written out over all n coordinates; m == n or n == 128, else null
    uint32_t kpad_dense = 0;
    void *d_dense_planes = nullptr;    // m == n, n != 128: the same matrix as three bf16 planes, [kpad / 256][npad / 16][3][256][16]
    int dense_arithmetic = LSH_DENSE_AUTO;  // see lsh_params_set_dense_arithmetic
    // one sample per table: operand tables of the shared-sample kernel (null when unsupported)
    lsh::SharedPlan shared_plan;
    float *d_shared_coef = nullptr;
    uint32_t *d_shared_sample_off = nullptr;
    float *d_shared_offset = nullptr;
    float *d_shared_extra = nullptr;
    // one sample per table, large n: lists of the shared-sample ranged kernel (null when unused)
    lsh::SharedRangedPlan shared_ranged_plan;
    void *d_sr_lists = nullptr, *d_sr_offs = nullptr, *d_sr_list_len = nullptr, *d_sr_stream = nullptr, *d_sr_extra = nullptr;
};

namespace lsh {

// host: draws the canonical tables (returns LSH_OK / LSH_ERR_*)
// (sample_group consecutive functions share the sample S of the first of them; 1 = every
// function its own)
int generate_tables(uint32_t n, uint32_t k, uint32_t m, float w, uint64_t seed, uint32_t flags,
                    uint32_t sample_group, std::vector<uint32_t> &idx, std::vector<float> &coef,
                    std::vector<float> &off);
int generate_extra_coefficients(uint32_t k, uint64_t seed, std::vector<float> &extra);

// host: bank-conflict-free visiting order of every function's samples (schedule.cpp)
uint64_t schedule_samples(const std::vector<uint32_t> &idx, uint32_t k, uint32_t m, uint32_t m_pad,
                          uint32_t group, uint32_t classes, uint32_t copies, std::vector<uint32_t> &order_out);

uint64_t schedule_windowed(const std::vector<uint32_t> &idx, uint32_t k, uint32_t m, uint32_t chunk,
                           uint32_t nchunks, uint32_t stages, uint32_t look, uint32_t sets_per_workgroup,
                           uint32_t step_quantum, uint32_t min_steps, uint32_t group, uint32_t classes,
                           std::vector<uint32_t> &steps_out, std::vector<uint32_t> &order_out);

// device: plan + upload + launches (defined in the .hip files)
SampledPlan plan_sampled(uint32_t n, uint32_t k, uint32_t m);
int upload_tables(lsh_params *p);
void free_tables(lsh_params *p);

enum class Epilogue : int { Ids = 0, Proj = 1, Signs = 2, Keys = 3, IdsKeys = 4 };  // IdsKeys: ids to d_out, keys to d_out2
int launch_sampled(const lsh_params *p, Epilogue ep, const float *d_data, uint64_t N, void *d_out,
                   uint32_t L, void *stream, void *d_out2 = nullptr);
bool sampled_ids_keys_supported(const lsh_params *p, uint32_t L);
// ranged kernel (ranged_kernel.hip): geometry constants the host tables are built for
constexpr uint32_t kRangeComputeWaves = 8;   // waves of a workgroup that gather or contract (the others load tiles)
constexpr uint32_t kWindowCoords = 256;      // coordinates per range (one ring slot holds 16 vectors of them)
constexpr uint32_t kWindowSlots = 8;         // ring slots in LDS
constexpr uint32_t kWindowLook = 6;          // a stage may read its own range and this many after it (the last slot is being filled)
int launch_ranged(const lsh_params *p, Epilogue ep, const float *d_data, uint64_t N, void *d_out,
                  uint32_t L, void *stream, void *d_out2 = nullptr);
bool ranged_schedule_valid(const lsh_params *p);  // selfcheck.cpp: run at create time
void build_ranged_tables(const lsh_params *p, std::vector<uint32_t> &words, std::vector<uint32_t> &list_len,
                         std::vector<uint32_t> &stream_info);
constexpr uint32_t kSharedRangeBlocksPerWave = 16;  // blocks of 16 functions a contracting wave owns at most
SharedRangedPlan plan_shared_ranged(uint32_t n, uint32_t k, uint32_t m, uint32_t L);
void build_shared_ranged_tables(const lsh_params *p, SharedRangedPlan &pl, std::vector<float> &coefs,
                                std::vector<uint32_t> &offs, std::vector<uint32_t> &stage_turns,
                                std::vector<uint32_t> &stream_info, std::vector<float> *extra = nullptr);
int launch_shared_ranged(const lsh_params *p, int mode, const float *d_data, uint64_t N, void *d_out, void *stream,
                         const float *d_kappa2 = nullptr, int raw = 0, uint64_t *d_keys = nullptr);
SharedPlan plan_shared(uint32_t n, uint32_t k, uint32_t m, uint32_t L);
void build_shared_tables(const lsh_params *p, std::vector<float> &coef, std::vector<uint32_t> &sample_off,
                         std::vector<float> &offset, std::vector<float> &extra);
// ep: 0 bucket ids, 1 raw projections, 2 one key per table (needs shared_keys_ok);
// maximum-inner-product transform: 3 max of ||S_l(v)||^2 per table into d_out (float [L], atomic
// max: cleared by the caller), 4 data hash (needs d_kappa2, float [L]), 5 query hash; raw != 0
// makes 4 and 5 write the projections instead of the ids
int launch_shared(const lsh_params *p, int ep, const float *d_data, uint64_t N, void *d_out, void *stream,
                  const float *d_kappa2 = nullptr, int raw = 0);
int clear_floats(float *d, uint32_t count, void *stream);
// the shared-sample kernel can fold keys when a table lies inside one wave's blocks
bool shared_keys_ok(const lsh_params *p, uint32_t L);
bool shared_ranged_keys_ok(const lsh_params *p, uint32_t L);
// raises a kernel's dynamic LDS limit once (per kernel and size)
int ensure_lds_limit(const void *fn, uint32_t lds_bytes);
int launch_dense(const lsh_params *p, bool proj, const float *d_data, uint64_t N, void *d_out,
                 void *stream);
// bf16 x 3 matrix-core version of the dense product (n = 128, k a multiple of 32) over the
// coefficient rows written out densely: E2LSH objects, and FastLSH objects as a dense product with
// zeros at the coordinates a function does not sample
bool dense_split_supported(const lsh_params *p);
// ... and of the sign hashes of any object with n = 128 and k a multiple of 64 (dense coefficient rows)
bool dense_split_signs_supported(const lsh_params *p);
// ... and of the keys of L tables of 4, 8, 16 or 32 functions
bool dense_split_keys_supported(const lsh_params *p, uint32_t L);
// ep: 0 bucket ids, 1 raw projections, 2 sign words, 3 keys (L tables)
int launch_dense_split(const lsh_params *p, int ep, const float *d_data, uint64_t N, void *d_out,
                       void *stream, uint32_t L = 0, void *d_out2 = nullptr);
// bf16 x 3 matrix-core version of the dense product for any n that is a multiple of 4
// (dense_split_wide_kernel.hip), over the coefficient planes split on the host
bool dense_wide_supported(const lsh_params *p);
uint32_t dense_wide_row_tile();
uint32_t dense_wide_col_step();
void build_dense_planes(const float *a, uint32_t k, uint32_t n, uint32_t kpad, uint32_t npad,
                        std::vector<uint16_t> &planes);
int launch_dense_wide(const lsh_params *p, bool proj, const float *d_data, uint64_t N, void *d_out, void *stream);
int launch_pack(const lsh_params *p, const int32_t *d_ids, uint64_t N, uint32_t L,
                uint64_t *d_keys, void *stream);

constexpr uint64_t kKeyMultiplier = 0x9E3779B97F4A7C15ull;

}  // namespace lsh
