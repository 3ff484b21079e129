// Host check of build_schedule (csrc/cx_schedule.hpp): the cycle order the kernels derive from
// a peer table, run by a group of real threads (a barrier for group.sync(), an atomic add) and
// compared with a plain serial cycle walk.  Built by tests/test_host_schedule.py, optionally
// with -fsanitize=thread so that a missing sync shows up as a data race.
#include <pthread.h>

#include <algorithm>
#include <atomic>
#include <cstdio>
#include <cstdlib>
#include <thread>
#include <vector>

#include "cx_schedule.hpp"

struct ThreadGroup {
    pthread_barrier_t *barrier;
    void sync() const { pthread_barrier_wait(barrier); }
    void add(int *p, int v) const { __atomic_fetch_add(p, v, __ATOMIC_RELAXED); }
};

// rows in cycle order, cycles by ascending first row, the last row of each cycle flagged;
// a table that is not a permutation of 0..n-1 counts as the identity
static std::vector<int> serial_schedule(std::vector<int> tab)
{
    const int n = static_cast<int>(tab.size());
    std::vector<int> indeg(n, 0), out;
    bool ok = true;
    for (int i = 0; i < n; ++i)
        if (tab[i] < 0 || tab[i] >= n) { ok = false; tab[i] = i; }
    for (int i = 0; i < n; ++i) ++indeg[tab[i]];
    for (int i = 0; i < n; ++i) ok = ok && indeg[i] == 1;
    if (!ok) for (int i = 0; i < n; ++i) tab[i] = i;
    std::vector<char> seen(n, 0);
    for (int start = 0; start < n; ++start) {
        if (seen[start]) continue;
        for (int cur = start; !seen[cur]; cur = tab[cur]) { seen[cur] = 1; out.push_back(cur); }
        out.back() |= kLastBit;
    }
    return out;
}

int main(int argc, char **argv)
{
    const int nthreads = argc > 1 ? std::atoi(argv[1]) : 4;
    const int max_n = argc > 2 ? std::atoi(argv[2]) : 1024;
    unsigned rng = 12345u;
    auto next = [&rng]() { rng = rng * 1664525u + 1013904223u; return rng >> 8; };
    long cases = 0;
    for (int n = 1; n <= max_n; n = n < 40 ? n + 1 : n * 2 - 7) {
        for (int rep = 0; rep < (n < 40 ? 24 : 6); ++rep) {
            const int S = 2, seg = rep & 1;
            std::vector<int32_t> peers(static_cast<size_t>(S) * n, 0);
            int32_t *t = peers.data() + static_cast<size_t>(seg) * n;
            for (int i = 0; i < n; ++i) t[i] = i;
            int shift = 0;
            switch (rep % 6) {
            case 0: case 1: case 2:                       // random permutation
                for (int i = n - 1; i > 0; --i) std::swap(t[i], t[next() % (i + 1)]);
                break;
            case 3:                                       // duplicates: not a permutation
                for (int i = 0; i < n; ++i) t[i] = static_cast<int32_t>(next() % n);
                break;
            case 4:                                       // the push-sum shift, table unused
                shift = n > 1 ? 1 + static_cast<int>(next() % (n - 1)) : 0;
                break;
            default:                                      // an entry out of range
                for (int i = n - 1; i > 0; --i) std::swap(t[i], t[next() % (i + 1)]);
                t[next() % n] = n + 3;
            }
            std::vector<int> as_table(n);
            for (int i = 0; i < n; ++i) as_table[i] = shift > 0 ? ((i - shift) % n + n) % n : t[i];
            const std::vector<int> want = serial_schedule(as_table);

            std::vector<int> work(kScheduleWords(n), -77);
            pthread_barrier_t barrier;
            pthread_barrier_init(&barrier, nullptr, nthreads);
            std::vector<std::thread> pool;
            for (int tid = 0; tid < nthreads; ++tid)
                pool.emplace_back([&, tid]() {
                    build_schedule(work.data(), n, tid, nthreads, shift > 0 ? nullptr : peers.data(), seg, shift,
                                   ThreadGroup{&barrier});
                });
            for (auto &th : pool) th.join();
            pthread_barrier_destroy(&barrier);
            for (int i = 0; i < n; ++i)
                if (work[n + i] != want[i]) {
                    std::printf("MISMATCH n=%d rep=%d position %d: got %x want %x\n", n, rep, i, work[n + i], want[i]);
                    return 1;
                }
            ++cases;
        }
    }
    std::printf("ok %ld tables, %d threads\n", cases, nthreads);
    return 0;
}
