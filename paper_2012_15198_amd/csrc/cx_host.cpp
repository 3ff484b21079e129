// Host half of the gossip-mixing library: topology generation (Algorithm 2 of the
// Crossover-SGD paper), host-side table checks, status strings and tuning state.
// Integer arithmetic only; no device code and no HIP calls in this file.
#include "cx_mix.h"

#include <algorithm>
#include <atomic>
#include <vector>

namespace {

// SplitMix64 output function: a bijective 64-bit bit mixer.
inline uint64_t scramble(uint64_t v)
{
    v ^= v >> 30; v *= 0xBF58476D1CE4E5B9ULL;
    v ^= v >> 27; v *= 0x94D049BB133111EBULL;
    v ^= v >> 31;
    return v;
}

// Counter-based draw stream of one (round, segment) topology.
struct DrawStream {
    uint64_t base;
    DrawStream(uint64_t seed, uint32_t round, uint32_t segment)
    {
        base = scramble(seed + 0x9E3779B97F4A7C15ULL);
        base = scramble(base + round);
        base = scramble(base + segment);
    }
    // index-th draw reduced to [0, bound): high word of the 64x64-bit product
    uint32_t below(uint32_t index, uint32_t bound) const
    {
        const uint64_t raw = scramble(base + index);
        return static_cast<uint32_t>((static_cast<unsigned __int128>(raw) * bound) >> 64);
    }
};

// One fair table.  `pool` holds the rows nobody has chosen yet, ascending; row i draws
// a position among the pool entries other than itself (the roulette row with the taken
// entries and the diagonal zeroed, renormalised -> uniform over what is left).
void fair_table(const DrawStream &rng, int32_t n, int32_t *recv_from, std::vector<int32_t> &pool)
{
    pool.resize(n);
    for (int32_t j = 0; j < n; ++j) pool[j] = j;
    for (int32_t i = 0; i < n; ++i) {
        // rows below i that are still free stay in the pool, so look i up by value
        const auto self = std::lower_bound(pool.begin(), pool.end(), i);
        const bool self_free = self != pool.end() && *self == i;
        const uint32_t choices = static_cast<uint32_t>(pool.size()) - (self_free ? 1u : 0u);
        if (choices == 0) {
            // only i itself is left (can only happen for the last row): trade with a
            // uniformly chosen earlier row, which keeps the table a derangement
            const uint32_t k = rng.below(static_cast<uint32_t>(n), static_cast<uint32_t>(n - 1));
            recv_from[i] = recv_from[k];
            recv_from[k] = i;
            pool.clear();
            continue;
        }
        uint32_t pos = rng.below(static_cast<uint32_t>(i), choices);
        if (self_free && pos >= static_cast<uint32_t>(self - pool.begin())) ++pos;  // skip i
        recv_from[i] = pool[pos];
        pool.erase(pool.begin() + pos);
    }
}

constexpr int kTuningKeys = 11;
// Random topology WITHOUT fair peer selection: every row draws independently among the
// other n-1 rows, so rows may be picked twice or never (the paper's comparison case).
void unfair_table(const DrawStream &rng, int32_t n, int32_t *recv_from)
{
    for (int32_t i = 0; i < n; ++i) {
        const int32_t pick = static_cast<int32_t>(rng.below(static_cast<uint32_t>(i), static_cast<uint32_t>(n - 1)));
        recv_from[i] = pick + (pick >= i ? 1 : 0);      // skip the row itself
    }
}

std::atomic<int32_t> g_tuning[kTuningKeys] = {{-1}, {-1}, {-1}, {-1}, {-1}, {-1}, {-1}, {-1}, {-1}, {-1}, {-1}};

}  // namespace

extern "C" {

const char *cx_status_string(int status)
{
    switch (status) {
    case CX_OK: return "CX_OK";
    case CX_ERR_NULL: return "CX_ERR_NULL";
    case CX_ERR_SHAPE: return "CX_ERR_SHAPE";
    case CX_ERR_SEGMENTS: return "CX_ERR_SEGMENTS";
    case CX_ERR_PEERS: return "CX_ERR_PEERS";
    case CX_ERR_ALIGN: return "CX_ERR_ALIGN";
    case CX_ERR_ALIAS: return "CX_ERR_ALIAS";
    case CX_ERR_HIP: return "CX_ERR_HIP";
    case CX_ERR_UNSUPPORTED: return "CX_ERR_UNSUPPORTED";
    case CX_ERR_MEMORY: return "CX_ERR_MEMORY";
    default: return "CX_ERR_UNKNOWN";
    }
}

int cx_abi_version(void) { return 4; }

int cx_topology_gen(uint64_t seed, int32_t n, int32_t S, int32_t round0, int32_t R,
                    int32_t mode, int32_t *peers_host)
{
    if (!peers_host) return CX_ERR_NULL;
    if (n < 2 || n > CX_MAX_ROWS || S < 1 || R < 0 || round0 < 0) return CX_ERR_SHAPE;
    if (static_cast<int64_t>(round0) + R > INT32_MAX) return CX_ERR_SHAPE;
    const bool same_for_all_segments = (mode & CX_TOPO_SAME_ALL_SEGMENTS) != 0;
    mode &= ~CX_TOPO_SAME_ALL_SEGMENTS;
    if (mode != CX_TOPO_FAIR && mode != CX_TOPO_DIRECTED_EXP && mode != CX_TOPO_UNFAIR) return CX_ERR_UNSUPPORTED;

    int32_t hops = 0;                       // number of distinct exponential hops
    while ((int64_t{1} << hops) < n) ++hops;

    std::vector<int32_t> pool;
    pool.reserve(n);
    for (int32_t r = 0; r < R; ++r) {
        const int32_t t = round0 + r;
        for (int32_t s = 0; s < S; ++s) {
            int32_t *row = peers_host + (static_cast<int64_t>(r) * S + s) * n;
            if (same_for_all_segments && s > 0) {
                std::copy_n(peers_host + static_cast<int64_t>(r) * S * n, n, row);
            } else if (mode == CX_TOPO_FAIR) {
                fair_table(DrawStream(seed, static_cast<uint32_t>(t), static_cast<uint32_t>(s)),
                           n, row, pool);
            } else if (mode == CX_TOPO_UNFAIR) {
                unfair_table(DrawStream(seed, static_cast<uint32_t>(t), static_cast<uint32_t>(s)), n, row);
            } else {
                const int32_t hop = static_cast<int32_t>((int64_t{1} << (t % hops)) % n);
                for (int32_t i = 0; i < n; ++i) row[i] = i >= hop ? i - hop : i - hop + n;
            }
        }
    }
    return CX_OK;
}

int cx_check_segments(const int64_t *seg_off_host, int32_t S, int64_t P)
{
    if (!seg_off_host) return CX_ERR_NULL;
    if (S < 1 || P < 1) return CX_ERR_SHAPE;
    if (seg_off_host[0] != 0 || seg_off_host[S] != P) return CX_ERR_SEGMENTS;
    for (int32_t s = 0; s < S; ++s)
        if (seg_off_host[s + 1] < seg_off_host[s]) return CX_ERR_SEGMENTS;
    return CX_OK;
}

int cx_check_peers(const int32_t *peers_host, int32_t S, int32_t n, int32_t mode)
{
    if (!peers_host) return CX_ERR_NULL;
    if (S < 1 || n < 2 || n > CX_MAX_ROWS) return CX_ERR_SHAPE;
    const bool same_for_all_segments = (mode & CX_TOPO_SAME_ALL_SEGMENTS) != 0;
    mode &= ~CX_TOPO_SAME_ALL_SEGMENTS;
    if (mode != CX_TOPO_FAIR && mode != CX_TOPO_DIRECTED_EXP && mode != CX_TOPO_UNFAIR) return CX_ERR_UNSUPPORTED;
    const bool duplicates_allowed = mode == CX_TOPO_UNFAIR;
    std::vector<uint8_t> seen(n);
    for (int32_t s = 0; s < S; ++s) {
        std::fill(seen.begin(), seen.end(), 0);
        const int32_t *row = peers_host + static_cast<int64_t>(s) * n;
        for (int32_t i = 0; i < n; ++i) {
            const int32_t j = row[i];
            if (j < 0 || j >= n || j == i) return CX_ERR_PEERS;
            if (seen[j] && !duplicates_allowed) return CX_ERR_PEERS;
            seen[j] = 1;
        }
        if (same_for_all_segments && s > 0 && !std::equal(row, row + n, peers_host)) return CX_ERR_PEERS;
    }
    return CX_OK;
}

int cx_set_tuning(int32_t key, int32_t value)
{
    if (key < 0 || key >= kTuningKeys) return CX_ERR_SHAPE;
    if (value != -1) {
        if (key == 0 && value != 1 && value != 2 && value != 4) return CX_ERR_SHAPE;
        if (key == 1 && (value < 1 || value > 8)) return CX_ERR_SHAPE;
        if (key == 2 && value != 0 && value != 1) return CX_ERR_SHAPE;
        if (key == 3 && value != 2 && value != 4 && value != 8) return CX_ERR_SHAPE;
        if ((key == 4 || key == 5 || key == 7 || key == 8 || key == 10) && value != 0 && value != 1) return CX_ERR_SHAPE;
        if (key == 6 && (value < 1 || value > 4096)) return CX_ERR_SHAPE;
        if (key == 9 && (value < 0 || value > 16)) return CX_ERR_SHAPE;
    }
    g_tuning[key].store(value);
    return CX_OK;
}

int cx_get_tuning(int32_t key)
{
    if (key < 0 || key >= kTuningKeys) return CX_ERR_SHAPE;
    return g_tuning[key].load();
}

}  // extern "C"
