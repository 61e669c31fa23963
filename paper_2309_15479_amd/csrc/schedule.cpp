// Bank-conflict-free gather schedule for the sampled-projection kernels.
//
// In the kernels one lane owns one hash function and, at step i, reads the LDS slot of its
// i-th sampled coordinate.  The hardware serves a wave's LDS read in passes of `group`
// lanes, and inside a pass two lanes collide when their slots fall in the same bank class
// (slot index modulo 16 / 32 / 64 for 16- / 8- / 4-byte slots: 64 banks of 4 bytes).
// Measured on gfx950 (lane-pair conflict matrix with fixed addresses): 8- and 4-byte reads
// are served in two passes, lanes 0-31 and 32-63; 16-byte reads in four passes of four lane
// quads each (quad q = lanes 4q..4q+3): {0,3,5,6}, {1,2,4,7}, {8,11,13,14}, {9,10,12,15}.
// A projection is a sum, so each function's samples may be visited in any order: this file
// picks, per group of lanes, an order in which the lanes of a pass hit distinct classes at
// (almost) every step.
//
// Per group this is the decomposition of a bipartite multigraph (lanes x classes, one edge
// per sample) into `steps` sets holding one edge of every lane.  Each step is built as a
// maximum matching found with augmenting paths, classes visited in order of remaining
// degree so that the heaviest classes are always served; lanes left without a free class
// double up on the least-loaded class they still need (a two-way conflict at that step).
// Padding samples (coefficient 0) are wildcards: they read one of the tile's zero slots,
// of whichever class is free.
//
// A perfect schedule needs every class to be wanted by at most `steps` samples of a group,
// which random samples do not grant (with 16 lanes x 32 samples over 16 classes the busiest
// class is wanted about 42 times).  Where LDS has room the kernel therefore keeps a second
// copy of the tile whose slots are rotated (copy_b_slot): every sample then has two classes
// to choose from, the choice is made per group so that the classes are evenly loaded
// (balance_copies), and the decomposition above comes out conflict-free or nearly so.
//
// Two table shapes are built from it: the flat one (every function's m samples, padded to
// m_pad) and the chunked one (samples bucketed by coordinate range, every wave's bucket
// padded to the longest list among its 64 lanes).
#include <algorithm>
#include <numeric>

#include "lsh_internal.h"

namespace lsh {
namespace {

// Schedules one pass group.  cls[l] = bank class of each sample of lane l (in list order).
// out[l][step] = position in lane l's list, or kPadSample | class.  Returns the cost.
struct GroupScheduler {
    int lanes = 0, classes = 0;
    std::vector<std::vector<int>> cnt;                      // [lane][class] samples not yet placed
    std::vector<std::vector<std::vector<uint32_t>>> where;  // [lane][class] -> list positions
    std::vector<int> pad, deg, match_class_of_lane, visited, class_order, load;

    bool augment(int c) {  // give class c a lane (Kuhn's algorithm from the class side)
        for (int l = 0; l < lanes; ++l) {
            if (!cnt[l][c] || visited[l]) continue;
            visited[l] = 1;
            const int other = match_class_of_lane[l];
            if (other < 0 || augment(other)) {
                match_class_of_lane[l] = c;
                return true;
            }
        }
        return false;
    }

    uint64_t run(const std::vector<std::vector<uint32_t>> &cls, int nclasses, int steps,
                 std::vector<std::vector<uint32_t>> &out) {
        lanes = (int)cls.size();
        classes = nclasses;
        cnt.assign(lanes, std::vector<int>(classes, 0));
        where.assign(lanes, std::vector<std::vector<uint32_t>>(classes));
        pad.assign(lanes, 0);
        deg.assign(classes, 0);
        class_order.resize(classes);
        load.resize(classes);
        out.assign(lanes, std::vector<uint32_t>(steps, 0));
        for (int l = 0; l < lanes; ++l) {
            pad[l] = steps - (int)cls[l].size();
            for (uint32_t i = (uint32_t)cls[l].size(); i-- > 0;) {  // reversed: pop_back yields list order
                const uint32_t c = cls[l][i];
                ++cnt[l][c];
                ++deg[c];
                where[l][c].push_back(i);
            }
        }
        uint64_t cost = 0;
        for (int step = 0; step < steps; ++step) {
            std::iota(class_order.begin(), class_order.end(), 0);
            std::stable_sort(class_order.begin(), class_order.end(),
                             [&](int a, int b) { return deg[a] > deg[b]; });
            match_class_of_lane.assign(lanes, -1);
            for (int c : class_order) {
                if (!deg[c]) break;
                visited.assign(lanes, 0);
                augment(c);
            }
            std::fill(load.begin(), load.end(), 0);
            for (int l = 0; l < lanes; ++l)
                if (match_class_of_lane[l] >= 0) ++load[match_class_of_lane[l]];
            const int steps_left = steps - step;
            for (int l = 0; l < lanes; ++l) {
                int c = match_class_of_lane[l];
                const bool must_use_real = pad[l] == 0;
                const bool only_pads_left = pad[l] == steps_left;
                if (c >= 0 && only_pads_left) {
                    --load[c];
                    c = -1;
                }
                if (c < 0 && !must_use_real) {  // a wildcard on the least-loaded class
                    int best = 0;
                    for (int q = 1; q < classes; ++q)
                        if (load[q] < load[best]) best = q;
                    ++load[best];
                    --pad[l];
                    out[l][step] = kPadSample | (uint32_t)best;
                    continue;
                }
                if (c < 0) {  // double up on the least-loaded class the lane still needs
                    for (int q = 0; q < classes; ++q)
                        if (cnt[l][q] &&
                            (c < 0 || load[q] < load[c] || (load[q] == load[c] && deg[q] > deg[c])))
                            c = q;
                    ++load[c];
                }
                --cnt[l][c];
                --deg[c];
                out[l][step] = where[l][c].back();
                where[l][c].pop_back();
            }
            cost += (uint64_t)*std::max_element(load.begin(), load.end());
        }
        return cost;
    }
};

// Chooses, for every sample of a group, the tile copy to read it from: a[e] / b[e] are the
// sample's classes in the first / second copy; returns the chosen class per sample with the
// largest class load as small as possible.  Local search by augmenting paths: while some
// chain of single-sample moves x0 -> x1 -> ... -> xt leads from a class to one holding at
// least two samples fewer, shift one sample along every link (only the ends change load).
std::vector<uint32_t> balance_copies(const std::vector<uint32_t> &a, const std::vector<uint32_t> &b,
                                     uint32_t classes) {
    std::vector<uint32_t> cur(a);
    std::vector<int> load(classes, 0), from_sample(classes), seen(classes);
    for (uint32_t c : cur) ++load[c];
    std::vector<uint32_t> by_load(classes), frontier;
    for (bool moved = true; moved;) {
        moved = false;
        std::iota(by_load.begin(), by_load.end(), 0u);
        std::stable_sort(by_load.begin(), by_load.end(), [&](uint32_t x, uint32_t y) { return load[x] > load[y]; });
        for (uint32_t src : by_load) {
            std::fill(seen.begin(), seen.end(), 0);
            std::fill(from_sample.begin(), from_sample.end(), -1);
            seen[src] = 1;
            frontier.assign(1, src);
            int target = -1;
            for (size_t f = 0; f < frontier.size() && target < 0; ++f) {
                const uint32_t x = frontier[f];
                for (size_t e = 0; e < cur.size() && target < 0; ++e) {
                    if (cur[e] != x) continue;
                    const uint32_t y = a[e] == x ? b[e] : a[e];
                    if (y == x || seen[y]) continue;
                    seen[y] = 1;
                    from_sample[y] = (int)e;
                    if (load[y] + 2 <= load[src]) target = (int)y;
                    else frontier.push_back(y);
                }
            }
            if (target < 0) continue;
            for (uint32_t y = (uint32_t)target; y != src;) {  // walk the chain back to src
                const int e = from_sample[y];
                const uint32_t x = cur[e];
                cur[e] = y;
                y = x;
            }
            --load[src];
            ++load[target];
            moved = true;
            break;
        }
    }
    return cur;
}

// lanes of a wave in pass order: `group` consecutive entries are served together
void pass_order_of(uint32_t group, uint32_t (&order)[64]) {
    for (uint32_t l = 0; l < 64; ++l) order[l] = l;
    if (group == 16) {
        const uint32_t quads[16] = {0, 3, 5, 6, 1, 2, 4, 7, 8, 11, 13, 14, 9, 10, 12, 15};
        for (uint32_t l = 0; l < 64; ++l) order[l] = quads[l / 4] * 4 + l % 4;
    }
}

}  // namespace

// Flat schedule.  idx: canonical [k][m] coordinates.  order_out: [k][m_pad], entry = position
// in the canonical list (0..m-1), with kCopyB set when the sample is to be read from the
// second tile copy (copies == 2), or kPadSample | class for a padding sample that should read
// the zero slot of that class.  Returns the modelled cost: sum over pass groups and steps of
// the largest number of lanes sharing a class (groups * steps when conflict-free).
uint64_t schedule_samples(const std::vector<uint32_t> &idx, uint32_t k, uint32_t m, uint32_t m_pad,
                          uint32_t group, uint32_t classes, uint32_t copies, std::vector<uint32_t> &order_out) {
    order_out.assign((size_t)k * m_pad, 0);
    uint32_t pass_order[64];
    pass_order_of(group, pass_order);
    uint64_t cost = 0;
    GroupScheduler g;
    std::vector<uint32_t> fn, class_a, class_b;
    std::vector<std::vector<uint32_t>> cls, out;
    for (uint32_t g0 = 0; g0 < (k + 63) / 64 * 64; g0 += group) {
        fn.clear();
        for (uint32_t e = 0; e < group; ++e) {
            const uint32_t j = g0 / 64 * 64 + pass_order[g0 % 64 + e];
            if (j < k) fn.push_back(j);
        }
        if (fn.empty()) continue;
        cls.assign(fn.size(), std::vector<uint32_t>(m));
        class_a.clear();
        class_b.clear();
        for (size_t l = 0; l < fn.size(); ++l)
            for (uint32_t i = 0; i < m; ++i) {
                const uint32_t c = idx[(size_t)fn[l] * m + i];
                class_a.push_back(c % classes);
                class_b.push_back(copies == 2 ? copy_b_slot(c, classes) % classes : c % classes);
            }
        const std::vector<uint32_t> chosen = copies == 2 ? balance_copies(class_a, class_b, classes) : class_a;
        for (size_t l = 0; l < fn.size(); ++l)
            for (uint32_t i = 0; i < m; ++i) cls[l][i] = chosen[l * m + i];
        cost += g.run(cls, (int)classes, (int)m_pad, out);
        for (size_t l = 0; l < fn.size(); ++l)
            for (uint32_t s = 0; s < m_pad; ++s) {
                uint32_t e = out[l][s];
                if (!(e & kPadSample) && chosen[l * m + e] != class_a[l * m + e]) e |= kCopyB;
                order_out[(size_t)fn[l] * m_pad + s] = e;
            }
    }
    return cost;
}

// Chunked schedule: coordinates are cut into nchunks ranges of `chunk` coordinates; the
// samples of a function are bucketed by range, and for every wave (64 consecutive functions)
// and range the 64 buckets are padded to a common length (a multiple of `step_quantum`) and
// scheduled per pass group.  steps_out[wave * nchunks + q] = that length; order_out holds, wave
// after wave and range after range, steps x 64 entries (step-major, lane-minor), each a
// position in the function's canonical list or kPadSample | class.
uint64_t schedule_chunked(const std::vector<uint32_t> &idx, uint32_t k, uint32_t m, uint32_t chunk,
                          uint32_t nchunks, uint32_t step_quantum, uint32_t group, uint32_t classes,
                          std::vector<uint32_t> &steps_out, std::vector<uint32_t> &order_out) {
    const uint32_t nwaves = (k + 63) / 64;
    steps_out.assign((size_t)nwaves * nchunks, 0);
    order_out.clear();
    uint32_t pass_order[64];
    pass_order_of(group, pass_order);
    uint64_t cost = 0;
    GroupScheduler g;
    std::vector<std::vector<std::vector<uint32_t>>> bucket(64);  // [lane][range] -> canonical positions
    std::vector<std::vector<uint32_t>> cls, out;
    std::vector<uint32_t> lanes_of_group;
    for (uint32_t w = 0; w < nwaves; ++w) {
        for (uint32_t l = 0; l < 64; ++l) {
            bucket[l].assign(nchunks, {});
            const uint32_t j = w * 64 + l;
            if (j >= k) continue;
            for (uint32_t i = 0; i < m; ++i) bucket[l][idx[(size_t)j * m + i] / chunk].push_back(i);
        }
        for (uint32_t q = 0; q < nchunks; ++q) {
            uint32_t longest = 0;
            for (uint32_t l = 0; l < 64; ++l)
                longest = std::max<uint32_t>(longest, (uint32_t)bucket[l][q].size());
            const uint32_t steps = (longest + step_quantum - 1) / step_quantum * step_quantum;
            steps_out[(size_t)w * nchunks + q] = steps;
            const size_t base = order_out.size();
            order_out.resize(base + (size_t)steps * 64, kPadSample);
            for (uint32_t g0 = 0; g0 < 64 && steps; g0 += group) {
                lanes_of_group.clear();
                for (uint32_t e = 0; e < group; ++e) lanes_of_group.push_back(pass_order[g0 + e]);
                cls.assign(lanes_of_group.size(), {});
                for (size_t t = 0; t < lanes_of_group.size(); ++t) {
                    const uint32_t l = lanes_of_group[t];
                    const uint32_t j = w * 64 + l;
                    for (uint32_t pos : bucket[l][q]) cls[t].push_back(idx[(size_t)j * m + pos] % classes);
                }
                cost += g.run(cls, (int)classes, (int)steps, out);
                for (size_t t = 0; t < lanes_of_group.size(); ++t) {
                    const uint32_t l = lanes_of_group[t];
                    for (uint32_t s = 0; s < steps; ++s) {
                        const uint32_t e = out[t][s];
                        order_out[base + (size_t)s * 64 + l] = (e & kPadSample) ? e : bucket[l][q][e];
                    }
                }
            }
        }
    }
    return cost;
}

}  // namespace lsh
