// Host-side construction of the hash-function tables (Sec. 3.1: the multiset S, the
// projection vector a~ and the offset b~ of every function; Sec. 2.2 when m == n).
//
// The paper names no random number generator.  Every table element here is one block of
// Philox4x64-10 (Salmon et al., SC'11), keyed by the seed and indexed by
// (sample i, function j, table id, attempt), so any element can be produced on its own.
#include <cmath>
#include <cstring>
#include <limits>
#include <new>

#include "lsh_internal.h"

namespace lsh {
namespace {

struct Block {
    uint64_t v[4];
};

// Philox4x64 with 10 rounds: two 64x64->128 multiplies per round, the high halves are
// xored with the neighbouring counter words and the (Weyl-bumped) key.
struct Philox4x64 {
    static constexpr uint64_t kMulA = 0xD2E7470EE14C6C93ull;
    static constexpr uint64_t kMulB = 0xCA5A826395121157ull;
    static constexpr uint64_t kBumpA = 0x9E3779B97F4A7C15ull;
    static constexpr uint64_t kBumpB = 0xBB67AE8584CAA73Bull;

    static Block run(Block x, uint64_t key_a, uint64_t key_b) {
        for (int r = 0; r < 10; ++r) {
            const unsigned __int128 pa = static_cast<unsigned __int128>(kMulA) * x.v[0];
            const unsigned __int128 pb = static_cast<unsigned __int128>(kMulB) * x.v[2];
            Block y;
            y.v[0] = static_cast<uint64_t>(pb >> 64) ^ x.v[1] ^ key_a;
            y.v[1] = static_cast<uint64_t>(pb);
            y.v[2] = static_cast<uint64_t>(pa >> 64) ^ x.v[3] ^ key_b;
            y.v[3] = static_cast<uint64_t>(pa);
            x = y;
            key_a += kBumpA;
            key_b += kBumpB;
        }
        return x;
    }
};

enum TableId : uint64_t { kIndexTable = 0, kCoefTable = 1, kOffsetTable = 2, kExtraTable = 3 };

inline Block element_block(uint64_t seed, TableId table, uint64_t j, uint64_t i, uint64_t attempt) {
    return Philox4x64::run(Block{{i, j, static_cast<uint64_t>(table), attempt}}, seed, 0);
}

// uniform integer in [0, range): words from the part of 2^64 that range does not divide
// evenly are discarded and the next attempt's block is used.
inline uint32_t uniform_below(uint64_t seed, uint64_t j, uint64_t i, uint64_t range) {
    const uint64_t leftover = (~uint64_t{0} % range + 1) % range;  // 2^64 mod range
    const uint64_t last_ok = ~uint64_t{0} - leftover;
    for (uint64_t attempt = 0;; ++attempt) {
        const uint64_t word = element_block(seed, kIndexTable, j, i, attempt).v[0];
        if (word <= last_ok) return static_cast<uint32_t>(word % range);
    }
}

inline double top53(uint64_t word) { return std::ldexp(static_cast<double>(word >> 11), -53); }

}  // namespace

int generate_tables(uint32_t n, uint32_t k, uint32_t m, float w, uint64_t seed, uint32_t flags,
                    uint32_t sample_group, std::vector<uint32_t> &idx, std::vector<float> &coef,
                    std::vector<float> &off) {
    try {
        idx.assign(static_cast<size_t>(k) * m, 0);
        coef.assign(static_cast<size_t>(k) * m, 0.f);
        off.assign(k, 0.f);
    } catch (const std::bad_alloc &) {
        return LSH_ERR_ALLOC;
    }
    const bool replace = (flags & LSH_SAMPLE_WITH_REPLACEMENT) != 0;
    std::vector<uint32_t> deck;  // Fisher-Yates deck, restored after every function
    std::vector<uint32_t> swapped_with;
    if (m < n && !replace) {
        try {
            deck.resize(n);
            swapped_with.resize(m);
        } catch (const std::bad_alloc &) {
            return LSH_ERR_ALLOC;
        }
        for (uint32_t c = 0; c < n; ++c) deck[c] = c;
    }
    const double two_pi = 6.283185307179586476925286766559;
    for (uint32_t j = 0; j < k; ++j) {
        uint32_t *S = &idx[static_cast<size_t>(j) * m];
        float *a = &coef[static_cast<size_t>(j) * m];
        // sample_group consecutive functions use the draws of the first of them for S
        const uint32_t owner = j / sample_group * sample_group;
        if (m == n) {
            for (uint32_t i = 0; i < m; ++i) S[i] = i;
        } else if (replace) {
            for (uint32_t i = 0; i < m; ++i) S[i] = uniform_below(seed, owner, i, n);
        } else {
            for (uint32_t i = 0; i < m; ++i) {
                const uint32_t pick = i + uniform_below(seed, owner, i, n - i);
                swapped_with[i] = pick;
                std::swap(deck[i], deck[pick]);
                S[i] = deck[i];
            }
            for (uint32_t i = m; i-- > 0;) std::swap(deck[i], deck[swapped_with[i]]);  // undo
        }
        for (uint32_t i = 0; i < m; ++i) {
            const Block r = element_block(seed, kCoefTable, j, i, 0);
            const double radius_u = std::ldexp(static_cast<double>(r.v[0] >> 11) + 1.0, -53);  // (0,1]
            const double angle_u = top53(r.v[1]);                                               // [0,1)
            const double z = std::sqrt(-2.0 * std::log(radius_u)) * std::cos(two_pi * angle_u);
            a[i] = static_cast<float>(z);
        }
        const Block r = element_block(seed, kOffsetTable, j, 0, 0);
        float b = static_cast<float>(top53(r.v[0]) * static_cast<double>(w));
        if (b >= w) b = std::nextafterf(w, 0.f);
        off[j] = b;
    }
    return LSH_OK;
}

// a0_j of the maximum-inner-product transform (appendix on maximum inner product search): one
// more N(0,1) coefficient per function, for the extra leading component of the transformed
// vectors.  Table 3 of the generator, element 0 of function j, drawn like the coefficients.
int generate_extra_coefficients(uint32_t k, uint64_t seed, std::vector<float> &extra) {
    try {
        extra.assign(k, 0.f);
    } catch (const std::bad_alloc &) {
        return LSH_ERR_ALLOC;
    }
    const double two_pi = 6.283185307179586476925286766559;
    for (uint32_t j = 0; j < k; ++j) {
        const Block r = element_block(seed, kExtraTable, j, 0, 0);
        const double radius_u = std::ldexp(static_cast<double>(r.v[0] >> 11) + 1.0, -53);
        extra[j] = static_cast<float>(std::sqrt(-2.0 * std::log(radius_u)) * std::cos(two_pi * top53(r.v[1])));
    }
    return LSH_OK;
}

}  // namespace lsh
