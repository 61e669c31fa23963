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
// m_pad) and the windowed one for large n (samples visited range by range with a window of
// ranges to work ahead in; see schedule_windowed).
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

// Orders one stage of a pass group: every lane has at most `steps` samples (cls[l][i] = bank
// class); out[l][step] = i or kPadSample | class.  A class wanted at most `steps` times gets
// one vertex, a class wanted more often one vertex per `steps` samples; padding entries fill
// every lane up to `steps` edges on vertices that still have room.  Lanes and vertices then
// have at most `steps` edges each, so the edges can be coloured with `steps` colours with no
// colour twice at a lane or a vertex (Koenig's edge-colouring theorem; alternating-path
// recolouring), and colour = step: two lanes collide in a step only through a class's second
// vertex, that is once per sample beyond `steps` at most.
struct StageColoring {
    struct Edge { int lane, vertex; uint32_t payload; int colour; };
    std::vector<Edge> edges;
    std::vector<std::vector<int>> at_lane, at_vertex;  // [lane or vertex][colour] -> edge or -1
    std::vector<int> degree, load;

    int free_colour(const std::vector<int> &row) const {
        for (size_t c = 0; c < row.size(); ++c)
            if (row[c] < 0) return (int)c;
        return -1;
    }

    uint64_t run(const std::vector<std::vector<uint32_t>> &cls, int classes, int steps,
                 std::vector<std::vector<uint32_t>> &out) {
        const int lanes = (int)cls.size();
        edges.clear();
        std::vector<int> wanted(classes, 0);
        int vertices = classes;
        for (int l = 0; l < lanes; ++l)
            for (uint32_t i = 0; i < cls[l].size(); ++i) {
                const int c = (int)cls[l][i], copy = wanted[c]++ / steps;
                edges.push_back({l, c + copy * classes, i, -1});
                vertices = std::max(vertices, c + (copy + 1) * classes);
            }
        degree.assign(vertices, 0);
        for (const Edge &e : edges) ++degree[e.vertex];
        for (int l = 0; l < lanes; ++l)
            for (int pad = (int)cls[l].size(); pad < steps; ++pad) {
                int best = 0;  // the emptiest class: its first vertex has room, since all edges together are lanes x steps
                for (int c = 1; c < classes; ++c)
                    if (degree[c] < degree[best]) best = c;
                ++degree[best];
                edges.push_back({l, best, kPadSample | (uint32_t)best, -1});
            }
        at_lane.assign(lanes, std::vector<int>(steps, -1));
        at_vertex.assign(vertices, std::vector<int>(steps, -1));
        std::vector<int> path;
        for (int e = 0; e < (int)edges.size(); ++e) {
            const int l = edges[e].lane, v = edges[e].vertex;
            const int a = free_colour(at_lane[l]);
            int b = free_colour(at_vertex[v]);
            if (at_vertex[v][a] >= 0) {
                // colour a is taken at v: swap a and b along the path of edges coloured a, b, a, ...
                // that starts at v (it cannot come back to l, which has no edge of colour a)
                path.clear();
                int x = at_vertex[v][a];
                bool on_vertex_side = true;  // x was found from its vertex end; continue from its lane end
                while (x >= 0) {
                    path.push_back(x);
                    const int want = edges[x].colour == a ? b : a;
                    x = on_vertex_side ? at_lane[edges[x].lane][want] : at_vertex[edges[x].vertex][want];
                    on_vertex_side = !on_vertex_side;
                }
                for (int y : path) {
                    at_lane[edges[y].lane][edges[y].colour] = -1;
                    at_vertex[edges[y].vertex][edges[y].colour] = -1;
                }
                for (int y : path) {
                    edges[y].colour = edges[y].colour == a ? b : a;
                    at_lane[edges[y].lane][edges[y].colour] = y;
                    at_vertex[edges[y].vertex][edges[y].colour] = y;
                }
            }
            edges[e].colour = a;
            at_lane[l][a] = e;
            at_vertex[v][a] = e;
        }
        out.assign(lanes, std::vector<uint32_t>(steps, kPadSample));
        uint64_t cost = 0;
        for (int st = 0; st < steps; ++st) {
            load.assign(classes, 0);
            for (int l = 0; l < lanes; ++l) {
                const Edge &e = edges[at_lane[l][st]];
                out[l][st] = e.payload;
                ++load[e.vertex % classes];
            }
            cost += (uint64_t)*std::max_element(load.begin(), load.end());
        }
        return cost;
    }
};

// Schedules one pass group over the stages of a tile (see schedule_windowed): stage by stage it
// picks the samples every lane visits in that stage so that no bank class is wanted more often
// than the stage has steps, then leaves the order inside the stage to StageColoring.
struct WindowScheduler {
    int lanes = 0, classes = 0;
    std::vector<std::vector<uint32_t>> by;            // [lane] list positions bucketed by (range, class)
    std::vector<std::vector<uint32_t>> bucket_first;  // [lane][range * classes + class] first entry of the bucket in `by`
    std::vector<std::vector<uint32_t>> bucket_left;   // [lane][range * classes + class] entries not yet visited
    std::vector<std::vector<int>> left_in;            // [lane][range] samples not yet visited
    std::vector<int> total_left;
    std::vector<std::vector<int>> avail, flow;        // [lane][class] optional samples on offer / taken
    std::vector<int> room, cap, from_lane, from_class, seen_lane, seen_class, want, class_order;
    StageColoring inner;

    // takes one sample of class c from the earliest of lane l's ranges first .. last that has one
    uint32_t take(int l, int c, int first, int last) {
        for (int r = first; r <= last; ++r) {
            uint32_t &left = bucket_left[l][(size_t)r * classes + c];
            if (!left) continue;
            --left;
            --left_in[l][r];
            --total_left[l];
            return by[l][bucket_first[l][(size_t)r * classes + c] + left];
        }
        return kPadSample;  // not reached: the caller counted the class in
    }

    // One more optional sample for lane l0 (a lane with room): an augmenting path lane -> class
    // with spare capacity, re-routing what other lanes have taken.
    bool augment(int l0) {
        std::fill(seen_lane.begin(), seen_lane.end(), 0);
        std::fill(seen_class.begin(), seen_class.end(), 0);
        std::vector<int> queue_l(1, l0);
        seen_lane[l0] = 1;
        from_lane.assign(lanes, -1);  // class through which a lane was reached (giving one up)
        for (size_t q = 0; q < queue_l.size(); ++q) {
            const int l = queue_l[q];
            for (int c : class_order) {  // the classes the group still wants most first
                if (seen_class[c] || flow[l][c] >= avail[l][c]) continue;
                seen_class[c] = 1;
                from_class[c] = l;
                if (cap[c] > 0) {  // spare capacity: push one unit along the path
                    --cap[c];
                    int cc = c;
                    for (;;) {
                        const int ll = from_class[cc];
                        ++flow[ll][cc];
                        if (ll == l0) return true;
                        cc = from_lane[ll];
                        --flow[ll][cc];
                    }
                }
                for (int l2 = 0; l2 < lanes; ++l2)  // a lane that holds a sample of c could take another class instead
                    if (!seen_lane[l2] && flow[l2][c] > 0) {
                        seen_lane[l2] = 1;
                        from_lane[l2] = c;
                        queue_l.push_back(l2);
                    }
            }
        }
        return false;
    }

    // range_of[l][i], cls[l][i]: range and bank class of lane l's i-th sample (ranges ascending).
    // out[l][step] = i or kPadSample | class, over the sum of len[] steps.
    uint64_t run(const std::vector<std::vector<uint32_t>> &range_of, const std::vector<std::vector<uint32_t>> &cls,
                 int nclasses, int nranges, int look, const uint32_t *len, int stages,
                 std::vector<std::vector<uint32_t>> &out) {
        lanes = (int)cls.size();
        classes = nclasses;
        uint32_t steps_total = 0;
        for (int s = 0; s < stages; ++s) steps_total += len[s];
        by.resize(lanes);
        bucket_first.resize(lanes);
        bucket_left.resize(lanes);
        left_in.assign(lanes, std::vector<int>(nranges, 0));
        total_left.assign(lanes, 0);
        avail.assign(lanes, std::vector<int>(classes, 0));
        flow.assign(lanes, std::vector<int>(classes, 0));
        room.assign(lanes, 0);
        cap.assign(classes, 0);
        from_class.assign(classes, -1);
        seen_lane.assign(lanes, 0);
        seen_class.assign(classes, 0);
        out.assign(lanes, std::vector<uint32_t>(steps_total, 0));
        for (int l = 0; l < lanes; ++l) {
            by[l].clear();
            // bucket the positions by (range, class), last first so that taking from the back yields list order
            std::vector<std::vector<uint32_t>> tmp((size_t)nranges * classes);
            for (uint32_t i = (uint32_t)cls[l].size(); i-- > 0;) tmp[(size_t)range_of[l][i] * classes + cls[l][i]].push_back(i);
            bucket_first[l].assign((size_t)nranges * classes + 1, 0);
            bucket_left[l].assign((size_t)nranges * classes, 0);
            for (size_t b = 0; b < tmp.size(); ++b) {
                bucket_first[l][b + 1] = bucket_first[l][b] + (uint32_t)tmp[b].size();
                bucket_left[l][b] = (uint32_t)tmp[b].size();
                by[l].insert(by[l].end(), tmp[b].begin(), tmp[b].end());
            }
            for (uint32_t i = 0; i < cls[l].size(); ++i) ++left_in[l][range_of[l][i]];
            total_left[l] = (int)cls[l].size();
        }
        std::vector<uint32_t> after(nranges);  // steps between the end of this stage and the end of stage r
        std::vector<std::vector<uint32_t>> picked(lanes), picked_cls(lanes), order;
        uint64_t cost = 0;
        uint32_t at = 0;
        for (int s = 0; s < stages; at += len[s], ++s) {
            const int T = (int)len[s];
            if (!T) continue;
            {
                uint32_t u = 0;
                for (int r = s; r < nranges; ++r) {
                    if (r > s) u += len[r];
                    after[r] = u;
                }
            }
            const int last_readable = std::min(nranges - 1, s + look);
            std::fill(cap.begin(), cap.end(), T);
            // what every lane has to visit now to keep its deadlines: with unvisited(r) samples of
            // ranges <= r and after[r] steps left for them later, the earliest
            // max_r (unvisited(r) - after[r]) samples (earliest range first)
            for (int l = 0; l < lanes; ++l) {
                picked[l].clear();
                picked_cls[l].clear();
                int unvisited = 0, due = 0;
                for (int r = s; r < nranges && unvisited < total_left[l]; ++r) {
                    unvisited += left_in[l][r];
                    due = std::max(due, unvisited - (int)after[r]);
                }
                for (int r = s; r <= last_readable && due > 0; ++r) {
                    while (due > 0 && left_in[l][r] > 0) {
                        // of a range that is only partly due, the classes with the most capacity left
                        int best = -1;
                        for (int c = 0; c < classes; ++c)
                            if (bucket_left[l][(size_t)r * classes + c] && (best < 0 || cap[c] > cap[best])) best = c;
                        picked[l].push_back(take(l, best, r, r));
                        picked_cls[l].push_back((uint32_t)best);
                        --cap[best];
                        --due;
                    }
                }
                room[l] = T - (int)picked[l].size();
            }
            // optional samples: as many as fit without pushing a class beyond T, the ranges that
            // are due soonest offered first (what is visited now will not crowd their own stage)
            for (int l = 0; l < lanes; ++l) {
                std::fill(flow[l].begin(), flow[l].end(), 0);
                std::fill(avail[l].begin(), avail[l].end(), 0);
            }
            for (int c = 0; c < classes; ++c) cap[c] = std::max(cap[c], 0);
            class_order.resize(classes);
            for (int r = s; r <= last_readable; ++r) {
                want.assign(classes, 0);
                for (int l = 0; l < lanes; ++l) {
                    if (!left_in[l][r]) continue;
                    for (int c = 0; c < classes; ++c) {
                        avail[l][c] += (int)bucket_left[l][(size_t)r * classes + c];
                        want[c] += (int)bucket_left[l][(size_t)r * classes + c];
                    }
                }
                std::iota(class_order.begin(), class_order.end(), 0);
                std::stable_sort(class_order.begin(), class_order.end(), [&](int a, int b) { return want[a] > want[b]; });
                for (bool more = true; more;) {  // one unit per lane and round, so that the lanes share the capacity evenly
                    more = false;
                    for (int l = 0; l < lanes; ++l) {
                        int taken = 0;
                        for (int c = 0; c < classes; ++c) taken += flow[l][c];
                        if (taken < room[l] && augment(l)) more = true;
                    }
                }
            }
            for (int l = 0; l < lanes; ++l)
                for (int c = 0; c < classes; ++c)
                    for (int f = 0; f < flow[l][c]; ++f) {
                        picked[l].push_back(take(l, c, s, last_readable));
                        picked_cls[l].push_back((uint32_t)c);
                    }
            // the order inside the stage
            cost += inner.run(picked_cls, classes, T, order);
            for (int l = 0; l < lanes; ++l)
                for (int st = 0; st < T; ++st) {
                    const uint32_t v = order[l][st];
                    out[l][at + st] = (v & kPadSample) ? v : picked[l][v];
                }
        }
        return cost;
    }
};

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

// Windowed schedule for large n.  Coordinates are cut into `nchunks` ranges of `chunk`
// coordinates that pass through a ring of LDS slots: at stage s of a tile (stage s < nchunks
// brings in range s, later stages nothing) the ranges s .. s + look are readable.  All lanes
// of a workgroup (sets_per_workgroup sets of 64 consecutive functions) walk every stage in
// lockstep, so a stage has one length for all of them; but a sample of range r may be visited
// in any of the stages r - look .. r, which lets a lane whose ranges are unevenly filled work
// ahead instead of waiting: since every function has the same m samples, the lists then
// need hardly any padding (with one fixed stage per range the 64 lists of a wave had to be
// padded to the longest of them, range by range: 1.6 entries per sample at m = 64, n = 4096).
//
// Stage lengths: stage after stage, the shortest length (a multiple of step_quantum) in which
// every lane can still visit all samples whose last stage this is, given that each lane has
// visited, earliest range first, as many readable samples as the stages so far had room for.
// Earliest-deadline-first is optimal for unit tasks whose windows are ordered like their
// deadlines, so these are the pointwise smallest cumulative lengths of any valid schedule.
// Given the stage lengths, each pass group is scheduled step by step like a flat list, except
// that a lane's choice at a step is limited to what keeps its own deadlines: with slack(r) =
// steps left until the end of stage r minus the lane's unvisited samples of ranges <= r, it
// may take a sample of range q (readable: q <= stage + look) only if slack(r) >= 1 for all
// r < q, and a padding entry only if slack(r) >= 1 for all r.  Inside these limits the step
// is a maximum matching of lanes to bank classes as above.
//
// steps_out[workgroup * stages + s] = entries per function in stage s; order_out holds,
// workgroup after workgroup, set after set and stage after stage, steps x 64 entries
// (step-major, lane-minor), each a position in the function's canonical list or
// kPadSample | class.
uint64_t schedule_windowed(const std::vector<uint32_t> &idx, uint32_t k, uint32_t m, uint32_t chunk,
                           uint32_t nchunks, uint32_t stages, uint32_t look, uint32_t sets_per_workgroup,
                           uint32_t step_quantum, uint32_t min_steps, uint32_t group, uint32_t classes,
                           std::vector<uint32_t> &steps_out, std::vector<uint32_t> &order_out) {
    const uint32_t nsets = (k + 63) / 64;
    const uint32_t nwg = (nsets + sets_per_workgroup - 1) / sets_per_workgroup;
    steps_out.assign((size_t)nwg * stages, 0);
    order_out.clear();
    uint32_t pass_order[64];
    pass_order_of(group, pass_order);
    uint64_t cost = 0;
    WindowScheduler ws;
    std::vector<std::vector<uint32_t>> cls, rng, out;
    std::vector<uint32_t> sorted, first_of_range, done;
    for (uint32_t y = 0; y < nwg; ++y) {
        const uint32_t set0 = y * sets_per_workgroup, set1 = std::min(nsets, set0 + sets_per_workgroup);
        const uint32_t lanes = (set1 - set0) * 64;
        // every lane's canonical positions sorted by range (stable), and where each range starts
        sorted.assign((size_t)lanes * m, 0);
        first_of_range.assign((size_t)lanes * (nchunks + 1), 0);
        for (uint32_t t = 0; t < lanes; ++t) {
            const uint32_t j = set0 * 64 + t;
            uint32_t *first = &first_of_range[(size_t)t * (nchunks + 1)];
            if (j >= k) continue;  // no samples: all zeros
            for (uint32_t i = 0; i < m; ++i) ++first[idx[(size_t)j * m + i] / chunk + 1];
            for (uint32_t q = 0; q < nchunks; ++q) first[q + 1] += first[q];
            std::vector<uint32_t> at(first, first + nchunks);
            for (uint32_t i = 0; i < m; ++i) sorted[(size_t)t * m + at[idx[(size_t)j * m + i] / chunk]++] = i;
        }
        // stage lengths (done[t] = samples lane t has visited when it takes the earliest range first)
        done.assign(lanes, 0);
        uint32_t *len = &steps_out[(size_t)y * stages];
        for (uint32_t s = 0; s < stages && s < nchunks; ++s) {
            uint32_t must = 0;
            for (uint32_t t = 0; t < lanes; ++t) {
                const uint32_t due = first_of_range[(size_t)t * (nchunks + 1) + s + 1];
                if (due > done[t]) must = std::max(must, due - done[t]);
            }
            len[s] = (must + step_quantum - 1) / step_quantum * step_quantum;
            const uint32_t last = std::min(nchunks - 1, s + look);
            for (uint32_t t = 0; t < lanes; ++t) {
                const uint32_t readable = first_of_range[(size_t)t * (nchunks + 1) + last + 1] - done[t];
                done[t] += std::min(len[s], readable);
            }
        }
        // Spare steps.  Without padding the busiest bank class of a pass group is wanted more
        // often than there are steps, and every such sample costs an extra pass of the LDS
        // read; a padding entry costs one pass, too, but it is a wildcard that lets the
        // matching shift the load.  Lengthen the stages in proportion until a tile has
        // min_steps steps.
        size_t wg_steps = 0;
        for (uint32_t s = 0; s < stages; ++s) wg_steps += len[s];
        if (wg_steps && wg_steps < min_steps) {
            const uint64_t extra = min_steps - wg_steps;
            uint64_t before = 0, given = 0;
            for (uint32_t s = 0; s < stages; ++s) {
                before += len[s];
                const uint64_t upto = extra * before / wg_steps / step_quantum * step_quantum;
                len[s] += (uint32_t)(upto - given);
                given = upto;
            }
            wg_steps += given;
        }
        // an even number of list blocks (of step_quantum steps) per tile: the kernel keeps two
        // blocks in registers and alternates between them without ever copying one
        if (wg_steps / step_quantum % 2) {
            uint32_t last = 0;
            for (uint32_t s = 0; s < stages; ++s)
                if (len[s]) last = s;
            len[last] += step_quantum;
            wg_steps += step_quantum;
        }
        for (uint32_t set = set0; set < set1; ++set) {
            const size_t base = order_out.size();
            order_out.resize(base + wg_steps * 64, kPadSample);
            for (uint32_t g0 = 0; g0 < 64; g0 += group) {
                cls.assign(group, {});
                rng.assign(group, {});
                for (uint32_t e = 0; e < group; ++e) {
                    const uint32_t l = pass_order[g0 + e], t = (set - set0) * 64 + l, j = set * 64 + l;
                    if (j >= k) continue;
                    for (uint32_t i = 0; i < m; ++i) {
                        const uint32_t c = idx[(size_t)j * m + sorted[(size_t)t * m + i]];
                        cls[e].push_back(c % classes);
                        rng[e].push_back(c / chunk);
                    }
                }
                cost += ws.run(rng, cls, (int)classes, (int)nchunks, (int)look, len, (int)stages, out);
                for (uint32_t e = 0; e < group; ++e) {
                    const uint32_t l = pass_order[g0 + e], t = (set - set0) * 64 + l;
                    for (size_t st = 0; st < wg_steps; ++st) {
                        const uint32_t v = out[e][st];
                        order_out[base + st * 64 + l] = (v & kPadSample) ? v : sorted[(size_t)t * m + v];
                    }
                }
            }
        }
    }
    return cost;
}

}  // namespace lsh
