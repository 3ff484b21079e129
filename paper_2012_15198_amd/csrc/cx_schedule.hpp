// Cycle schedule of a peer table: the order in which the mixing kernels visit the rows.
// Plain C++ with no device intrinsics, so that the same text runs inside the kernels (the
// including file defines CX_SCHED_FN as __device__ __forceinline__) and in a host test.
#ifndef CX_SCHEDULE_HPP
#define CX_SCHEDULE_HPP
#include <cstddef>
#include <cstdint>

#ifndef CX_SCHED_FN
#define CX_SCHED_FN inline
#endif

constexpr int kLastBit = 1 << 30;          // schedule entry flag: last row of its cycle
constexpr int kRowMask = kLastBit - 1;

// ---------------------------------------------------------------------------------
// Cycle schedule of one segment, built in LDS by a group of threads (one wavefront in its
// private region, or a whole workgroup): `work` holds kScheduleWords(n) ints,
//   work[0..n)   : the table as used (a table that is not a permutation -> the identity)
//   work[n..2n)  : the schedule: rows in cycle order, cycles by ascending smallest row, each
//                  starting at its smallest row; kLastBit marks the last row of a cycle
// Source of the table: shift > 0 -> row i receives from (i - shift) mod n;
// peers == null -> identity; else peers[seg*n + i].
// No serial walk: every row finds the smallest row of its cycle and its distance to it by
// pointer doubling (log2 n rounds over words that pack successor, minimum and distance), a
// prefix sum over the cycle lengths places the cycles, and every row writes its own entry.
// `group.sync()` orders the group's traffic on `work`; `group.add(p, v)` is an atomic *p += v.
// ---------------------------------------------------------------------------------
constexpr int kRowBits = 10;                          // CX_MAX_ROWS == 1 << kRowBits
constexpr int kRowField = (1 << kRowBits) - 1;
constexpr size_t kScheduleWords(int n) { return 4 * static_cast<size_t>(n) + 4; }

template <class Group>
CX_SCHED_FN void build_schedule(int *work, int n, int tid, int nthreads, const int32_t *peers, int seg,
                                int shift, Group group)
{
    int *tab = work, *sched = work + n, *a = work + 2 * n, *b = work + 3 * n;
    int *bad = work + 4 * n;
    if (tid == 0) *bad = 0;
    bool ok = true;
    for (int i = tid; i < n; i += nthreads) {
        int v = i;
        if (shift > 0) v = i >= shift ? i - shift : i - shift + n;
        else if (peers) v = peers[static_cast<int64_t>(seg) * n + i];
        if (static_cast<unsigned>(v) >= static_cast<unsigned>(n)) { ok = false; v = i; }
        tab[i] = v;
        sched[i] = 0;
    }
    group.sync();
    for (int i = tid; i < n; i += nthreads) group.add(&sched[tab[i]], 1);   // in-degree
    group.sync();
    for (int i = tid; i < n; i += nthreads) ok = ok && (sched[i] == 1);
    if (!ok) group.add(bad, 1);
    group.sync();
    const bool valid = *bad == 0;
    // word i: successor after `span` steps | smallest row among the next `span` rows of the
    // cycle, i included | distance from i to that row
    for (int i = tid; i < n; i += nthreads) {
        if (!valid) tab[i] = i;
        a[i] = (valid ? tab[i] : i) | (i << kRowBits);
    }
    group.sync();
    for (int span = 1; span < n; span <<= 1) {
        for (int i = tid; i < n; i += nthreads) {
            const int w = a[i];
            const int wj = a[w & kRowField];
            int mn = (w >> kRowBits) & kRowField, d = w >> (2 * kRowBits);
            const int mj = (wj >> kRowBits) & kRowField;
            if (mj < mn) { mn = mj; d = span + (wj >> (2 * kRowBits)); }
            b[i] = (wj & kRowField) | (mn << kRowBits) | (d << (2 * kRowBits));
        }
        group.sync();
        int *t = a; a = b; b = t;
    }
    // a[i] now names the smallest row of i's cycle and i's distance to it.  Cycle lengths at
    // the smallest rows, then an inclusive prefix sum that ends in `b`.
    int rounds = 0;
    for (int span = 1; span < n; span <<= 1) ++rounds;
    int *p = (rounds & 1) ? sched : b, *q = (rounds & 1) ? b : sched;
    for (int i = tid; i < n; i += nthreads) {
        const bool leader = ((a[i] >> kRowBits) & kRowField) == i;
        p[i] = leader ? (a[tab[i]] >> (2 * kRowBits)) + 1 : 0;
    }
    group.sync();
    for (int span = 1; span < n; span <<= 1) {
        for (int i = tid; i < n; i += nthreads) q[i] = p[i] + (i >= span ? p[i - span] : 0);
        group.sync();
        int *t = p; p = q; q = t;
    }
    // p == b: cycles end at p[smallest row]; place every row
    for (int i = tid; i < n; i += nthreads) {
        const int w = a[i];
        const int mn = (w >> kRowBits) & kRowField, d = w >> (2 * kRowBits);
        const int len = (a[tab[mn]] >> (2 * kRowBits)) + 1;
        const int pos = d == 0 ? 0 : len - d;
        sched[p[mn] - len + pos] = i | (pos == len - 1 ? kLastBit : 0);
    }
    group.sync();
}

#endif  // CX_SCHEDULE_HPP
