// Sanitizer run of the library's host half (csrc/cx_host.cpp) next to the CPU oracle
// (oracle/cx_oracle.c): built with -fsanitize=address,undefined by tests/test_host_sanitizers.py.
// It generates topologies with both for many shapes and modes and compares them entry by entry,
// runs the two table checkers on good and bad tables, and drives every oracle mixing function on
// heap buffers of exactly the stated sizes, so that any read or write past them is reported.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "cx_mix.h"

extern "C" {
int oracle_topology(uint64_t seed, int32_t n, int32_t S, int32_t round0, int32_t R, int32_t mode, int32_t *out);
int oracle_gossip_mix(const float *, float *, int64_t, int32_t, int64_t, int32_t, const int64_t *, const int32_t *);
int oracle_gossip_mix_bf16(const uint16_t *, uint16_t *, int64_t, int32_t, int64_t, int32_t, const int64_t *, const int32_t *);
int oracle_gossip_mix_f16(const uint16_t *, uint16_t *, int64_t, int32_t, int64_t, int32_t, const int64_t *, const int32_t *);
int oracle_hier_mix_f64(const float *, double *, int64_t, int32_t, int64_t, int32_t, int32_t, const int64_t *, const int32_t *);
int oracle_hier_mix_f32(const float *, float *, int64_t, int32_t, int64_t, int32_t, int32_t, const int64_t *, const int32_t *);
int oracle_hier_mix16_f64(int, const uint16_t *, double *, int64_t, int32_t, int64_t, int32_t, int32_t, const int64_t *, const int32_t *);
int oracle_hier_mix16_f32(int, const uint16_t *, uint16_t *, int64_t, int32_t, int64_t, int32_t, int32_t, const int64_t *, const int32_t *);
int oracle_sgd_fused_mix_f64(const float *, const float *, const float *, double *, double *, float, float, float,
                             int64_t, int32_t, int64_t, int32_t, const int64_t *, const int32_t *);
int oracle_sgd_fused_mix_f32(const float *, const float *, const float *, float *, float *, float, float, float,
                             int64_t, int32_t, int64_t, int32_t, const int64_t *, const int32_t *);
int oracle_hier_sgd_fused_mix_f64(const float *, const float *, const float *, double *, double *, float, float, float,
                                  int64_t, int32_t, int64_t, int32_t, int32_t, const int64_t *, const int32_t *);
int oracle_hier_sgd_fused_mix_f32(const float *, const float *, const float *, float *, float *, float, float, float,
                                  int64_t, int32_t, int64_t, int32_t, int32_t, const int64_t *, const int32_t *);
int oracle_pushsum_mix_f64(const float *, const float *, double *, double *, double *, int64_t, int32_t, int64_t, int32_t);
int oracle_pushsum_mix_f32(const float *, const float *, float *, float *, float *, int64_t, int32_t, int64_t, int32_t);
}

#define CHECK(cond)                                                              \
    do {                                                                         \
        if (!(cond)) { std::printf("FAILED line %d: %s\n", __LINE__, #cond); return 1; } \
    } while (0)

int main()
{
    // --- topology: library against oracle, all modes, sizes up to the maximum
    const int shapes[][4] = {{2, 1, 0, 4}, {3, 5, 2, 40}, {8, 4, 0, 10}, {33, 3, 7, 5}, {128, 8, 0, 3}, {1024, 2, 1, 2}};
    const int modes[] = {CX_TOPO_FAIR, CX_TOPO_DIRECTED_EXP, CX_TOPO_UNFAIR, CX_TOPO_FAIR | CX_TOPO_SAME_ALL_SEGMENTS,
                         CX_TOPO_UNFAIR | CX_TOPO_SAME_ALL_SEGMENTS};
    for (const auto &sh : shapes)
        for (int mode : modes)
            for (uint64_t seed : {uint64_t{0}, uint64_t{2}, ~uint64_t{0}}) {
                const int n = sh[0], S = sh[1], r0 = sh[2], R = sh[3];
                const size_t words = static_cast<size_t>(R) * S * n;
                std::vector<int32_t> a(words, -5), b(words, -7);           // exact size: overruns are caught
                CHECK(cx_topology_gen(seed, n, S, r0, R, mode, a.data()) == CX_OK);
                CHECK(oracle_topology(seed, n, S, r0, R, mode, b.data()) == 0);
                CHECK(std::memcmp(a.data(), b.data(), words * sizeof(int32_t)) == 0);
                for (int r = 0; r < R; ++r)
                    CHECK(cx_check_peers(a.data() + static_cast<size_t>(r) * S * n, S, n, mode) == CX_OK);
            }
    std::vector<int32_t> one(8);
    CHECK(cx_topology_gen(1, 8, 1, 0, 0, 0, one.data()) == CX_OK);        // R = 0 writes nothing
    CHECK(cx_topology_gen(1, 1, 1, 0, 1, 0, one.data()) == CX_ERR_SHAPE);
    CHECK(cx_topology_gen(1, 8, 1, INT32_MAX, 1, 0, one.data()) == CX_ERR_SHAPE);
    CHECK(cx_topology_gen(1, 8, 1, 0, 1, 7, one.data()) == CX_ERR_UNSUPPORTED);

    // --- checkers on bad tables
    const int32_t fixed_point[] = {0, 2, 1}, duplicate[] = {1, 0, 0}, too_large[] = {1, 2, 3}, negative[] = {-1, 2, 0};
    CHECK(cx_check_peers(fixed_point, 1, 3, CX_TOPO_FAIR) == CX_ERR_PEERS);
    CHECK(cx_check_peers(duplicate, 1, 3, CX_TOPO_FAIR) == CX_ERR_PEERS);
    CHECK(cx_check_peers(duplicate, 1, 3, CX_TOPO_UNFAIR) == CX_OK);
    CHECK(cx_check_peers(too_large, 1, 3, CX_TOPO_UNFAIR) == CX_ERR_PEERS);
    CHECK(cx_check_peers(negative, 1, 3, CX_TOPO_FAIR) == CX_ERR_PEERS);
    CHECK(cx_check_peers(nullptr, 1, 3, CX_TOPO_FAIR) == CX_ERR_NULL);
    const int64_t good[] = {0, 0, 5, 9}, bad_end[] = {0, 4, 8}, bad_order[] = {0, 6, 5, 9};
    CHECK(cx_check_segments(good, 3, 9) == CX_OK);
    CHECK(cx_check_segments(bad_end, 2, 9) == CX_ERR_SEGMENTS);
    CHECK(cx_check_segments(bad_order, 3, 9) == CX_ERR_SEGMENTS);
    for (int k = -1; k < 12; ++k) (void)cx_get_tuning(k);
    CHECK(cx_set_tuning(99, 1) == CX_ERR_SHAPE);
    CHECK(std::strcmp(cx_status_string(CX_ERR_ALIAS), "CX_ERR_ALIAS") == 0);

    // --- every oracle mixing function on buffers of exactly [W][ld] (ld == P: no slack at all)
    const int W = 12, G = 4, L = W / G, S = 3;
    const int64_t P = 37, ld = 37;
    const int64_t so[] = {0, 11, 11, 37};                                  // one empty segment
    std::vector<int32_t> peers(static_cast<size_t>(S) * W), lpeers(static_cast<size_t>(S) * L);
    CHECK(cx_topology_gen(3, W, S, 0, 1, CX_TOPO_FAIR, peers.data()) == CX_OK);
    CHECK(cx_topology_gen(3, L, S, 0, 1, CX_TOPO_FAIR, lpeers.data()) == CX_OK);
    const size_t n = static_cast<size_t>(W) * ld, nl = static_cast<size_t>(L) * ld;
    std::vector<float> x(n), v(n), g(n), vl(nl), xo(n), vo(n), vlo(nl), w(W, 1.0f), wo(W), z(n);
    std::vector<double> xd(n), vd(n), vld(nl), wd(W), zd(n);
    std::vector<uint16_t> h(n), ho(n);
    unsigned rng = 7u;
    for (size_t i = 0; i < n; ++i) {
        rng = rng * 1664525u + 1013904223u;
        x[i] = static_cast<float>(static_cast<int>(rng >> 8) % 2001 - 1000) * 1e-3f;
        v[i] = x[i] * 0.1f;
        g[i] = -x[i] * 0.01f;
        h[i] = static_cast<uint16_t>(rng >> 12);                           // any bit pattern, NaNs included
    }
    for (size_t i = 0; i < nl; ++i) vl[i] = v[i];
    CHECK(oracle_gossip_mix(x.data(), xo.data(), ld, W, P, S, so, peers.data()) == 0);
    CHECK(oracle_gossip_mix_bf16(h.data(), ho.data(), ld, W, P, S, so, peers.data()) == 0);
    CHECK(oracle_gossip_mix_f16(h.data(), ho.data(), ld, W, P, S, so, peers.data()) == 0);
    CHECK(oracle_hier_mix_f64(x.data(), xd.data(), ld, W, P, G, S, so, lpeers.data()) == 0);
    CHECK(oracle_hier_mix_f32(x.data(), xo.data(), ld, W, P, G, S, so, lpeers.data()) == 0);
    CHECK(oracle_hier_mix_f32(x.data(), xo.data(), ld, W, P, W, S, so, nullptr) == 0);   // one group
    for (int fmt = 0; fmt < 2; ++fmt) {
        CHECK(oracle_hier_mix16_f64(fmt, h.data(), xd.data(), ld, W, P, G, S, so, lpeers.data()) == 0);
        CHECK(oracle_hier_mix16_f32(fmt, h.data(), ho.data(), ld, W, P, G, S, so, lpeers.data()) == 0);
    }
    CHECK(oracle_sgd_fused_mix_f64(x.data(), v.data(), g.data(), xd.data(), vd.data(), 0.1f, 0.9f, 1e-4f, ld, W, P, S, so, peers.data()) == 0);
    CHECK(oracle_sgd_fused_mix_f32(x.data(), v.data(), g.data(), xo.data(), vo.data(), 0.1f, 0.9f, 1e-4f, ld, W, P, S, so, peers.data()) == 0);
    CHECK(oracle_hier_sgd_fused_mix_f64(x.data(), vl.data(), g.data(), xd.data(), vld.data(), 0.1f, 0.9f, 1e-4f, ld, W, P, G, S, so, lpeers.data()) == 0);
    CHECK(oracle_hier_sgd_fused_mix_f32(x.data(), vl.data(), g.data(), xo.data(), vlo.data(), 0.1f, 0.9f, 1e-4f, ld, W, P, G, S, so, lpeers.data()) == 0);
    CHECK(oracle_pushsum_mix_f64(x.data(), w.data(), xd.data(), wd.data(), zd.data(), ld, W, P, 4) == 0);
    CHECK(oracle_pushsum_mix_f32(x.data(), w.data(), xo.data(), wo.data(), z.data(), ld, W, P, 4) == 0);
    CHECK(oracle_pushsum_mix_f32(x.data(), w.data(), xo.data(), wo.data(), nullptr, ld, W, P, 11) == 0);
    for (int i = 0; i < W; ++i) CHECK(wo[i] == 1.0f);
    std::printf("ok\n");
    return 0;
}
