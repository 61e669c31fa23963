// Host-side check of the list tables that the ranged kernels consume (ranged_kernel.hip,
// shared_ranged_kernel.hip): the tables are built exactly as for the device and walked the way
// the kernels walk them (stream after stream, range after range, block after block, the same
// index arithmetic) on a pseudo-random vector, in double precision; the result must be the
// projection of Eq. 5, p_j = sum_i a~_j[i] v[S_j[i]], computed straight from the canonical
// tables.  Needs no GPU: the most intricate host code of the library is testable where it is
// written.  ranged_schedule_valid() is the part of it that runs whenever an object for the gather
// kernel by coordinate ranges is created: a schedule the kernel could not follow is refused there.
#include <algorithm>
#include <cmath>
#include <cstring>
#include <vector>

#include "lsh_internal.h"

namespace lsh {
namespace {

// a deterministic vector with entries in [-1, 1) (SplitMix64; nothing of the hashing path)
std::vector<double> test_vector(uint32_t n, uint64_t seed) {
    std::vector<double> v(n);
    uint64_t x = seed;
    for (uint32_t c = 0; c < n; ++c) {
        x += 0x9E3779B97F4A7C15ull;
        uint64_t z = x;
        z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
        z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
        z ^= z >> 31;
        v[c] = (double)(z >> 11) * (2.0 / 9007199254740992.0) - 1.0;
    }
    return v;
}

// worst |walked - direct| / sum_i |a v| over the functions
double compare(const lsh_params *p, const std::vector<double> &v, const std::vector<double> &walked) {
    double worst = 0.0;
    for (uint32_t j = 0; j < p->k; ++j) {
        double direct = 0.0, scale = 0.0;
        for (uint32_t i = 0; i < p->m; ++i) {
            const double t = (double)p->coef[(size_t)j * p->m + i] * v[p->idx[(size_t)j * p->m + i]];
            direct += t;
            scale += std::fabs(t);
        }
        const double err = std::fabs(walked[j] - direct) / (scale > 0.0 ? scale : 1.0);
        if (!(err <= worst)) worst = err;  // NaN counts as the worst
    }
    return worst;
}

}  // namespace

// Cheap check of the ranged kernel's schedule, run whenever such an object is created: every
// function's samples appear exactly once, each in a stage whose ring holds its range (stage <=
// range <= stage + look), and a tile is an even number of list blocks.
bool ranged_schedule_valid(const lsh_params *p) {
    const SampledPlan &pl = p->plan;
    const uint32_t sets_per_wg = pl.fpt * kRangeComputeWaves, nsets = (p->k + 63) / 64, S = pl.stages;
    if (p->chunk_steps.size() != (size_t)pl.kblocks * S) return false;
    std::vector<uint8_t> seen(p->m);
    size_t base = 0;
    for (uint32_t set = 0; set < nsets; ++set) {
        const uint32_t *len = &p->chunk_steps[(size_t)(set / sets_per_wg) * S];
        uint32_t steps = 0;
        for (uint32_t s = 0; s < S; ++s) steps += len[s];
        if (steps % (4 * pl.qpf) || steps / (4 * pl.qpf) % 2) return false;
        if (base + (size_t)steps * 64 > p->order.size()) return false;
        for (uint32_t l = 0; l < 64; ++l) {
            const uint32_t j = set * 64 + l;
            std::fill(seen.begin(), seen.end(), 0);
            uint32_t found = 0, at = 0;
            for (uint32_t s = 0; s < S; ++s)
                for (uint32_t e = 0; e < len[s]; ++e, ++at) {
                    const uint32_t ent = p->order[base + (size_t)at * 64 + l];
                    if (ent & kPadSample) continue;
                    if (j >= p->k || ent >= p->m || seen[ent]) return false;
                    const uint32_t range = p->idx[(size_t)j * p->m + ent] / pl.chunk;
                    if (range < s || range > s + kWindowLook) return false;
                    seen[ent] = 1;
                    ++found;
                }
            if (found != (j < p->k ? p->m : 0u)) return false;
        }
        base += (size_t)steps * 64;
    }
    return base == p->order.size();
}

namespace {

double walk_ranged(const lsh_params *p, const std::vector<double> &v) {
    // Follows every gathering wave through one tile as the kernel does: block after block, the
    // stage advancing by the barrier counts, every entry's slot number resolved against what
    // the ring holds at that stage (slot x holds the range r in stage .. stage + 6 with
    // r % 8 == x; the eighth slot is being refilled and must not be read).
    const SampledPlan &pl = p->plan;
    std::vector<uint32_t> words, barriers, info;
    build_ranged_tables(p, words, barriers, info);
    const uint32_t CW = kRangeComputeWaves, fpt = pl.fpt, qpf = pl.qpf, U = fpt * qpf;
    const uint32_t bar_stride = (uint32_t)(barriers.size() / pl.kblocks);
    const size_t block_words = (size_t)U * 64 * 6, off_base = (size_t)U * 64 * 4;
    std::vector<double> walked(p->k, 0.0);
    for (uint32_t y = 0; y < pl.kblocks; ++y)
        for (uint32_t cw = 0; cw < CW; ++cw) {
            const uint32_t stream = y * CW + cw, first = info[(size_t)stream * 2], blocks = info[(size_t)stream * 2 + 1];
            if (blocks + 1 > bar_stride || blocks % 2) return INFINITY;  // the kernel takes the blocks two at a time
            const uint32_t *bar = &barriers[(size_t)y * bar_stride];
            uint32_t stage = bar[0];
            for (uint32_t b = 0; b < blocks; ++b) {
                if (stage >= pl.stages) return INFINITY;  // entries after the tile's last barrier
                const uint32_t *blk = &words[(size_t)(first + b) * block_words];
                for (uint32_t u = 0; u < U; ++u)
                    for (uint32_t pos = 0; pos < 4; ++pos)
                        for (uint32_t l = 0; l < 64; ++l) {
                            float c;
                            std::memcpy(&c, &blk[((size_t)u * 64 + l) * 4 + pos], 4);
                            const uint32_t pair = blk[off_base + ((size_t)u * 64 + l) * 2 + pos / 2];
                            const uint32_t slot = (pair >> (16 * (pos % 2))) & 0xFFFFu;
                            const uint32_t ring = slot / (4 * kWindowCoords), in_range = slot % (4 * kWindowCoords);
                            if (ring >= kWindowSlots || in_range >= kWindowCoords) return INFINITY;
                            const uint32_t r = stage + (ring + kWindowSlots - stage % kWindowSlots) % kWindowSlots;
                            if (r > stage + kWindowLook || r >= pl.nchunks) return INFINITY;  // not (yet) in the ring
                            const uint32_t coord = r * kWindowCoords + in_range;
                            const uint32_t j = ((y * fpt + u / qpf) * CW + cw) * 64 + l;
                            if (j < p->k) walked[j] += (double)c * (coord < p->n ? v[coord] : 0.0);
                            else if (c != 0.f) return INFINITY;  // a lane beyond k must not contribute
                        }
                stage += bar[b + 1];
            }
            if (stage != pl.stages) return INFINITY;  // one barrier per stage of the tile
        }
    return compare(p, v, walked);
}

double walk_shared_ranged(const lsh_params *p, const std::vector<double> &v) {
    // Follows every contracting wave through one tile: stage after stage, turn after turn of the
    // list ring, step i of a turn on block i / (32 / bpw) of the wave; every offset is resolved
    // against what the ring holds at that stage, as in walk_ranged.
    SharedRangedPlan pl = p->shared_ranged_plan;
    std::vector<float> coefs;
    std::vector<uint32_t> offs, turns, info;
    build_shared_ranged_tables(p, pl, coefs, offs, turns, info);
    const uint32_t U = 8, OW = 4, ring = 4, CW = kRangeComputeWaves, Q = ring * U / pl.bpw;
    const uint32_t row = kWindowSlots * kWindowCoords;
    if (turns.size() != pl.stages || pl.stages % kWindowSlots) return INFINITY;
    std::vector<double> walked(p->k, 0.0);
    for (uint32_t y = 0; y < pl.kblocks; ++y)
        for (uint32_t cw = 0; cw < CW; ++cw) {
            const uint32_t stream = y * CW + cw, first = info[(size_t)stream * 2], blocks = info[(size_t)stream * 2 + 1];
            uint32_t next = 0;
            for (uint32_t s = 0; s < pl.stages; ++s)
                for (uint32_t turn = 0; turn < turns[s]; ++turn)
                    for (uint32_t b = 0; b < ring; ++b, ++next) {
                        if (next >= blocks) return INFINITY;
                        const float *cb = &coefs[(size_t)(first + next) * U * 64];
                        const uint32_t *ob = &offs[(size_t)(first + next) * 4 * OW];
                        for (uint32_t e = 0; e < U; ++e) {
                            const uint32_t f = (b * U + e) / Q;
                            const uint32_t blk = (y * pl.bpw + f) * CW + cw;  // global block number
                            for (uint32_t l = 0; l < 64; ++l) {
                                const float c = cb[(size_t)(e / 4 * 4) * 64 + l * 4 + e % 4];
                                const uint32_t off = (ob[(l / 16) * OW + e / 2] >> (16 * (e & 1))) & 0xFFFFu;
                                uint32_t coord = p->n;  // beyond the row: a zero float
                                if (off % 4 || off / 4 >= row + 4) return INFINITY;
                                if (off / 4 < row) {
                                    const uint32_t slot = off / 4 / kWindowCoords;
                                    const uint32_t r = s + (slot + kWindowSlots - s % kWindowSlots) % kWindowSlots;
                                    if (r > s + kWindowLook || r >= pl.nchunks) return INFINITY;  // not (yet) in the ring
                                    coord = r * kWindowCoords + off / 4 % kWindowCoords;
                                }
                                const uint32_t in_table = (blk % pl.blocks_per_table) * 16 + l % 16;
                                const uint32_t j = (blk / pl.blocks_per_table) * pl.g + in_table;
                                if (blk < pl.nblocks && in_table < pl.g) walked[j] += (double)c * (coord < p->n ? v[coord] : 0.0);
                                else if (c != 0.f) return INFINITY;
                            }
                        }
                    }
            if (next != blocks || blocks < ring) return INFINITY;
        }
    return compare(p, v, walked);
}

}  // namespace
}  // namespace lsh

int lsh_params_check_lists(const lsh_params_t *p, uint64_t seed, double *worst) {
    if (!p || !worst) return LSH_ERR_INVALID_ARG;
    const bool shared = p->shared_ranged_plan.supported;
    const bool ranged = !shared && !p->shared_plan.supported && p->plan.supported && p->plan.ranged;
    if (!shared && !ranged) return LSH_ERR_UNSUPPORTED;
    try {
        const std::vector<double> v = lsh::test_vector(p->n, seed);
        *worst = shared ? lsh::walk_shared_ranged(p, v) : lsh::walk_ranged(p, v);
    } catch (const std::bad_alloc &) {
        return LSH_ERR_ALLOC;
    }
    return LSH_OK;
}

int lsh_params_get_shared_schedule(const lsh_params_t *p, uint32_t *stages, uint32_t *steps) {
    if (!p || !stages || !steps) return LSH_ERR_INVALID_ARG;
    if (!p->shared_ranged_plan.supported) return LSH_ERR_UNSUPPORTED;
    try {
        lsh::SharedRangedPlan pl = p->shared_ranged_plan;
        std::vector<float> coefs;
        std::vector<uint32_t> offs, turns, info;
        lsh::build_shared_ranged_tables(p, pl, coefs, offs, turns, info);
        uint32_t total = 0;
        for (uint32_t t : turns) total += t;
        *stages = pl.stages;
        *steps = total * (4 * 8 / pl.bpw);  // a turn of the list ring: four blocks of eight steps, dealt to the wave's blocks
    } catch (const std::bad_alloc &) {
        return LSH_ERR_ALLOC;
    }
    return LSH_OK;
}
