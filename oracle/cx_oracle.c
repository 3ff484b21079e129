/*
 * CPU oracle for the segment-wise gossip parameter-mixing step of Crossover-SGD.
 *
 * TEST INFRASTRUCTURE ONLY.  Plain, single-threaded, scalar C, written from the
 * paper's Algorithm 1 (overlapped segment-wise communication), Algorithm 2
 * (random topology with fair peer selection) and Section 3.3 (hierarchical
 * variant).  It shares no code, header, table or constant generator with the
 * HIP library; only tests, the smoke check and the benchmark's cpu_baseline leg
 * may call it.  The product path never does.
 *
 * Conventions (all matrices row-major, row i = worker i's flat parameter vector):
 *   x        float [W][ld], columns [0,P) used, [P,ld) never touched
 *   seg_off  int64 [S+1], non-decreasing, seg_off[0]=0, seg_off[S]=P;
 *            segment s = columns [seg_off[s], seg_off[s+1])
 *   peers    int32 [S][n]; peers[s][i] = the row whose segment s row i RECEIVES
 *            (Algorithm 1: receive_from = destinations[my_rank])
 * Every function reads only its inputs' round-start values ("snapshot"): in
 * Algorithm 1 all sends are posted before any averaging happens.
 * Output buffers must not overlap input buffers.
 *
 * Pins (tests/test_oracle_*.py): SplitMix64 published vectors for the bit mixer;
 * exact draw-tree probabilities for n<=6 (3/8 : 5/8 at n=3); derangement and
 * double-stochasticity on every table; W=2 / W=3 hand cases; column-mean
 * conservation; the halving of the deviation norm at W=3; G=W equals the plain
 * column mean; log2(W) exponential hops equal the exact mean; the fused update
 * with mixing off equals torch.optim.SGD; the gradient-reducing hierarchical step
 * with one group equals SGD on the averaged gradient; the bfloat16 and binary16
 * conversions against torch's and numpy's on every bit pattern, their rounding
 * ties, underflow and overflow by hand; the double -> 16-bit rounding against an exact
 * rational nearest-value search (every tie, the overflow point, the subnormal range) and
 * numpy; the optimizer steps on 16-bit rows by hand (one case that tells one rounding from
 * rounding through fp32), against the fp32-row steps on widened rows and against
 * torch.optim.SGD; the push-sum round on 16-bit rows by hand on exact values, its
 * invariants (column sums, weight sum, z * w' = x'), the exponential graph reaching the
 * mean in log2 W rounds, its rounding against the double reference, and against the
 * fp32-row round between the pinned conversions.  No function here is "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------------- */
/* Counter-based random draws (the paper only says "seed = rseed, shared by   */
/* every process"; a generator keyed by (seed, round, segment, draw index)    */
/* gives every process the same table and every segment a different one,      */
/* which Section 3 requires).  The bit mixer is the SplitMix64 output function.*/
/* ------------------------------------------------------------------------- */
uint64_t oracle_mix64(uint64_t z)
{
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ULL;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBULL;
    return z ^ (z >> 31);
}

/* key of one (round, segment) topology */
uint64_t oracle_key(uint64_t seed, int32_t round, int32_t segment)
{
    uint64_t h = oracle_mix64(seed + 0x9E3779B97F4A7C15ULL);
    h = oracle_mix64(h + (uint64_t)(uint32_t)round);
    h = oracle_mix64(h + (uint64_t)(uint32_t)segment);
    return h;
}

/* k-th raw 64-bit draw of that topology */
uint64_t oracle_draw(uint64_t key, uint32_t k)
{
    return oracle_mix64(key + (uint64_t)k);
}

/* uniform integer in [0,m): floor(v * m / 2^64) */
uint32_t oracle_uniform(uint64_t v, uint32_t m)
{
    return (uint32_t)(((unsigned __int128)v * (unsigned __int128)m) >> 64);
}

/*
 * Algorithm 2 for one (round, segment): sequential roulette draw.
 * Row i of the roulette starts uniform over all ranks but i (zero diagonal);
 * ranks already chosen are zeroed and the row renormalised, so the draw is
 * uniform over the remaining ranks other than i, taken in ascending rank order.
 * If the last rank finds only itself left (the printed algorithm would divide
 * by zero), it swaps with a uniformly drawn earlier rank k: d[n-1]=d[k],
 * d[k]=n-1, using draw index n.
 * Returns 0, or -1 if n < 2.
 */
int oracle_fair_draw(uint64_t key, int32_t n, int32_t *d)
{
    if (n < 2) return -1;
    unsigned char *taken = (unsigned char *)calloc((size_t)n, 1);
    if (!taken) return -2;
    for (int32_t i = 0; i < n; ++i) {
        uint32_t m = 0;                       /* ranks with non-zero roulette */
        for (int32_t j = 0; j < n; ++j)
            if (j != i && !taken[j]) ++m;
        if (m == 0) {                         /* dead end: only i itself is left */
            uint32_t k = oracle_uniform(oracle_draw(key, (uint32_t)n), (uint32_t)(n - 1));
            d[i] = d[k];
            d[k] = i;
            taken[i] = 1;
            continue;
        }
        uint32_t t = oracle_uniform(oracle_draw(key, (uint32_t)i), m);
        for (int32_t j = 0; j < n; ++j) {
            if (j == i || taken[j]) continue;
            if (t == 0) { d[i] = j; taken[j] = 1; break; }
            --t;
        }
    }
    free(taken);
    return 0;
}

/*
 * The "conventional" random topology the paper compares with (Sections 3.2, 4.3):
 * every rank draws its peer uniformly among the other n-1 ranks, independently, so
 * a rank may be chosen several times or not at all (row-stochastic mixing matrix).
 */
int oracle_unfair_draw(uint64_t key, int32_t n, int32_t *d)
{
    if (n < 2) return -1;
    for (int32_t i = 0; i < n; ++i) {
        uint32_t t = oracle_uniform(oracle_draw(key, (uint32_t)i), (uint32_t)(n - 1));
        d[i] = (int32_t)t < i ? (int32_t)t : (int32_t)t + 1;   /* t-th rank other than i */
    }
    return 0;
}

/*
 * Peer tables for rounds [round0, round0+R), S segments, n gossiping rows.
 * mode 0: fair random topology (Algorithm 2), a fresh one per (round, segment).
 * mode 1: time-varying directed exponential graph (the SGP comparison):
 *         in round t every row i receives from (i - 2^(t mod ceil(log2 n))) mod n,
 *         the same shift for every segment.
 * mode 2: random topology without fair peer selection (duplicates allowed).
 * mode + 16: the table of segment 0 is used for every segment of the round, which
 *         Section 3 says equals model-wise communication.
 * out: int32 [R][S][n].
 */
int oracle_topology(uint64_t seed, int32_t n, int32_t S, int32_t round0, int32_t R,
                    int32_t mode, int32_t *out)
{
    if (n < 2 || S < 1 || R < 0 || round0 < 0) return -1;
    int same = (mode & 16) != 0;
    mode &= ~16;
    int32_t nlog = 0;
    while (((int64_t)1 << nlog) < (int64_t)n) ++nlog;     /* ceil(log2 n) */
    for (int32_t r = 0; r < R; ++r) {
        for (int32_t s = 0; s < S; ++s) {
            int32_t *d = out + ((int64_t)r * S + s) * n;
            if (same && s > 0) {
                memcpy(d, out + (int64_t)r * S * n, sizeof(int32_t) * (size_t)n);
            } else if (mode == 0) {
                int rc = oracle_fair_draw(oracle_key(seed, round0 + r, s), n, d);
                if (rc) return rc;
            } else if (mode == 2) {
                int rc = oracle_unfair_draw(oracle_key(seed, round0 + r, s), n, d);
                if (rc) return rc;
            } else if (mode == 1) {
                int64_t hop = (int64_t)1 << ((round0 + r) % nlog);
                for (int32_t i = 0; i < n; ++i)
                    d[i] = (int32_t)((((int64_t)i - hop) % n + n) % n);
            } else {
                return -1;
            }
        }
    }
    return 0;
}

/* ------------------------------------------------------------------------- */
/* Algorithm 1, averaging line: layer = (layer + received_layer) / 2, fp32.  */
/* ------------------------------------------------------------------------- */
int oracle_gossip_mix(const float *x_in, float *x_out, int64_t ld, int32_t W, int64_t P,
                      int32_t S, const int64_t *seg_off, const int32_t *peers)
{
    (void)P;
    for (int32_t s = 0; s < S; ++s)
        for (int32_t i = 0; i < W; ++i) {
            int32_t j = peers[(int64_t)s * W + i];       /* receive_from */
            for (int64_t c = seg_off[s]; c < seg_off[s + 1]; ++c)
                x_out[i * ld + c] = (x_in[i * ld + c] + x_in[j * ld + c]) * 0.5f;
        }
    return 0;
}

/* ------------------------------------------------------------------------- */
/* The same averaging on bfloat16 rows (the paper trains in mixed precision): */
/* widen both values to fp32, add, halve, round once to bfloat16 (nearest,    */
/* ties to even).  x holds bfloat16 bit patterns.                             */
/* ------------------------------------------------------------------------- */
float oracle_bf16_to_f32(uint16_t h)
{
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return f;
}

uint16_t oracle_f32_to_bf16(float f)
{
    uint32_t u;
    memcpy(&u, &f, sizeof u);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);   /* NaN stays NaN */
    uint32_t kept_lsb = (u >> 16) & 1u;
    u += 0x7fffu + kept_lsb;          /* below half rounds down, above up, a tie to the even */
    return (uint16_t)(u >> 16);
}

int oracle_gossip_mix_bf16(const uint16_t *x_in, uint16_t *x_out, int64_t ld, int32_t W, int64_t P,
                           int32_t S, const int64_t *seg_off, const int32_t *peers)
{
    (void)P;
    for (int32_t s = 0; s < S; ++s)
        for (int32_t i = 0; i < W; ++i) {
            int32_t j = peers[(int64_t)s * W + i];
            for (int64_t c = seg_off[s]; c < seg_off[s + 1]; ++c) {
                float a = oracle_bf16_to_f32(x_in[i * ld + c]);
                float b = oracle_bf16_to_f32(x_in[j * ld + c]);
                x_out[i * ld + c] = oracle_f32_to_bf16((a + b) * 0.5f);
            }
        }
    return 0;
}

/* ------------------------------------------------------------------------- */
/* The same averaging on IEEE binary16 rows (1 sign, 5 exponent, 10 fraction  */
/* bits, bias 15): widen, add and halve in fp32, round once to binary16       */
/* (nearest, ties to even; gradual underflow; overflow to infinity).          */
/* ------------------------------------------------------------------------- */
float oracle_f16_to_f32(uint16_t h)
{
    uint32_t sign = (uint32_t)(h & 0x8000u) << 16;
    uint32_t e = (h >> 10) & 31u, m = h & 1023u;
    float f;
    if (e == 0) {                                   /* zero or subnormal: m * 2^-24 */
        f = ldexpf((float)m, -24);
        return sign ? -f : f;
    }
    uint32_t u = (e == 31) ? (sign | 0x7f800000u | (m << 13))      /* infinity, NaN */
                           : (sign | ((e + 112u) << 23) | (m << 13));
    memcpy(&f, &u, sizeof f);
    return f;
}

uint16_t oracle_f32_to_f16(float f)
{
    uint32_t u;
    memcpy(&u, &f, sizeof u);
    uint16_t sign = (uint16_t)((u >> 16) & 0x8000u);
    uint32_t a = u & 0x7fffffffu;
    if (a > 0x7f800000u) return (uint16_t)(sign | 0x7e00u | ((a >> 13) & 0x3ffu));   /* NaN stays NaN */
    if (a >= 0x47800000u) return (uint16_t)(sign | 0x7c00u);       /* 2^16 and above, infinity */
    if (a < 0x38800000u) {                          /* below 2^-14: a multiple of 2^-24 */
        float mag;
        memcpy(&mag, &a, sizeof mag);
        uint32_t q = (uint32_t)nearbyintf(ldexpf(mag, 24));        /* 0..1024, ties to even */
        return (uint16_t)(sign | q);
    }
    uint32_t kept_lsb = (a >> 13) & 1u;
    a += 0xfffu + kept_lsb;                         /* round the 13 dropped bits, ties to even */
    uint32_t h = (a >> 13) - (112u << 10);          /* may carry up to 0x7c00 = infinity */
    return (uint16_t)(sign | h);
}

int oracle_gossip_mix_f16(const uint16_t *x_in, uint16_t *x_out, int64_t ld, int32_t W, int64_t P,
                          int32_t S, const int64_t *seg_off, const int32_t *peers)
{
    (void)P;
    for (int32_t s = 0; s < S; ++s)
        for (int32_t i = 0; i < W; ++i) {
            int32_t j = peers[(int64_t)s * W + i];
            for (int64_t c = seg_off[s]; c < seg_off[s + 1]; ++c) {
                float a = oracle_f16_to_f32(x_in[i * ld + c]);
                float b = oracle_f16_to_f32(x_in[j * ld + c]);
                x_out[i * ld + c] = oracle_f32_to_f16((a + b) * 0.5f);
            }
        }
    return 0;
}

/* ------------------------------------------------------------------------- */
/* Hierarchical variant (Section 3.3): (1) reduce inside each group of G      */
/* consecutive rows to the group mean held by the leader, (2) the L = W/G     */
/* leaders gossip segment-wise, (3) the leader's result is broadcast to its   */
/* group.  With L == 1 step (2) is empty and every row gets the global mean.  */
/* Reference mode: all arithmetic in double, result returned as double.       */
/* ------------------------------------------------------------------------- */
int oracle_hier_mix_f64(const float *x_in, double *y_out, int64_t ld, int32_t W, int64_t P,
                        int32_t G, int32_t S, const int64_t *seg_off,
                        const int32_t *leader_peers)
{
    (void)P;
    int32_t L = W / G;
    double *m = (double *)malloc(sizeof(double) * (size_t)L);
    if (!m) return -2;
    for (int32_t s = 0; s < S; ++s)
        for (int64_t c = seg_off[s]; c < seg_off[s + 1]; ++c) {
            for (int32_t g = 0; g < L; ++g) {
                double acc = 0.0;
                for (int32_t j = 0; j < G; ++j)
                    acc += (double)x_in[((int64_t)g * G + j) * ld + c];
                m[g] = acc / (double)G;
            }
            for (int32_t g = 0; g < L; ++g) {
                double y = m[g];
                if (L > 1) y = (m[g] + m[leader_peers[(int64_t)s * L + g]]) * 0.5;
                for (int32_t j = 0; j < G; ++j)
                    y_out[((int64_t)g * G + j) * ld + c] = y;
            }
        }
    free(m);
    return 0;
}

/* fp32 pairwise sum of n values spaced `stride` apart: split at the largest
 * power of two below n, sum each part the same way, add the two parts. */
static float tree_sum_f32(const float *x, int64_t stride, int32_t n)
{
    if (n == 1) return x[0];
    int32_t h = 1;
    while (h * 2 < n) h *= 2;
    float a = tree_sum_f32(x, stride, h);
    float b = tree_sum_f32(x + (int64_t)h * stride, stride, n - h);
    return a + b;
}

/* Same steps in fp32 with a fixed order: pairwise-tree group sum, times the
 * fp32 reciprocal of G, then the fp32 pairwise average between leaders. */
int oracle_hier_mix_f32(const float *x_in, float *x_out, int64_t ld, int32_t W, int64_t P,
                        int32_t G, int32_t S, const int64_t *seg_off,
                        const int32_t *leader_peers)
{
    (void)P;
    int32_t L = W / G;
    float inv_g = 1.0f / (float)G;
    float *m = (float *)malloc(sizeof(float) * (size_t)L);
    if (!m) return -2;
    for (int32_t s = 0; s < S; ++s)
        for (int64_t c = seg_off[s]; c < seg_off[s + 1]; ++c) {
            for (int32_t g = 0; g < L; ++g)
                m[g] = tree_sum_f32(x_in + (int64_t)g * G * ld + c, ld, G) * inv_g;
            for (int32_t g = 0; g < L; ++g) {
                float y = m[g];
                if (L > 1) y = (m[g] + m[leader_peers[(int64_t)s * L + g]]) * 0.5f;
                for (int32_t j = 0; j < G; ++j)
                    x_out[((int64_t)g * G + j) * ld + c] = y;
            }
        }
    free(m);
    return 0;
}

/* ------------------------------------------------------------------------- */
/* The hierarchical step on 16-bit rows (fmt 0 = bfloat16, 1 = binary16): every */
/* value is widened exactly, the step runs as above, and each result is rounded */
/* ONCE to the 16-bit format.  Reference mode returns the unrounded doubles.    */
/* ------------------------------------------------------------------------- */
static float widen16(int fmt, uint16_t h) { return fmt ? oracle_f16_to_f32(h) : oracle_bf16_to_f32(h); }
static uint16_t narrow16(int fmt, float f) { return fmt ? oracle_f32_to_f16(f) : oracle_f32_to_bf16(f); }

int oracle_hier_mix16_f64(int fmt, const uint16_t *x_in, double *y_out, int64_t ld, int32_t W,
                          int64_t P, int32_t G, int32_t S, const int64_t *seg_off,
                          const int32_t *leader_peers)
{
    (void)P;
    int32_t L = W / G;
    double *m = (double *)malloc(sizeof(double) * (size_t)L);
    if (!m) return -2;
    for (int32_t s = 0; s < S; ++s)
        for (int64_t c = seg_off[s]; c < seg_off[s + 1]; ++c) {
            for (int32_t g = 0; g < L; ++g) {
                double sum = 0.0;
                for (int32_t j = 0; j < G; ++j)
                    sum += (double)widen16(fmt, x_in[((int64_t)g * G + j) * ld + c]);
                m[g] = sum / (double)G;
            }
            for (int32_t g = 0; g < L; ++g) {
                double y = m[g];
                if (L > 1) y = (m[g] + m[leader_peers[(int64_t)s * L + g]]) * 0.5;
                for (int32_t j = 0; j < G; ++j)
                    y_out[((int64_t)g * G + j) * ld + c] = y;
            }
        }
    free(m);
    return 0;
}

int oracle_hier_mix16_f32(int fmt, const uint16_t *x_in, uint16_t *x_out, int64_t ld, int32_t W,
                          int64_t P, int32_t G, int32_t S, const int64_t *seg_off,
                          const int32_t *leader_peers)
{
    (void)P;
    int32_t L = W / G;
    float inv_g = 1.0f / (float)G;
    float *m = (float *)malloc(sizeof(float) * (size_t)L);
    float *col = (float *)malloc(sizeof(float) * (size_t)W);
    if (!m || !col) { free(m); free(col); return -2; }
    for (int32_t s = 0; s < S; ++s)
        for (int64_t c = seg_off[s]; c < seg_off[s + 1]; ++c) {
            for (int32_t i = 0; i < W; ++i) col[i] = widen16(fmt, x_in[(int64_t)i * ld + c]);
            for (int32_t g = 0; g < L; ++g)
                m[g] = tree_sum_f32(col + (int64_t)g * G, 1, G) * inv_g;
            for (int32_t g = 0; g < L; ++g) {
                float y = m[g];
                if (L > 1) y = (m[g] + m[leader_peers[(int64_t)s * L + g]]) * 0.5f;
                uint16_t r = narrow16(fmt, y);
                for (int32_t j = 0; j < G; ++j)
                    x_out[((int64_t)g * G + j) * ld + c] = r;
            }
        }
    free(m);
    free(col);
    return 0;
}

/* ------------------------------------------------------------------------- */
/* Local momentum-SGD step, then Algorithm 1's averaging on the updated       */
/* parameters (Section 3.1: averaging happens after the gradient is applied): */
/*     g' = g + wd*x ;  v' = mu*v + g' ;  x_half = x - lr*v'                  */
/*     x'_i = (x_half_i + x_half_peer) / 2                                    */
/* lr, mu, wd are the fp32 hyper-parameter values.  Reference mode: double.   */
/* ------------------------------------------------------------------------- */
int oracle_sgd_fused_mix_f64(const float *x_in, const float *v_in, const float *g,
                             double *x_out, double *v_out, float lr, float mu, float wd,
                             int64_t ld, int32_t W, int64_t P, int32_t S,
                             const int64_t *seg_off, const int32_t *peers)
{
    (void)P;
    double *xh = (double *)malloc(sizeof(double) * (size_t)W);
    if (!xh) return -2;
    for (int32_t s = 0; s < S; ++s)
        for (int64_t c = seg_off[s]; c < seg_off[s + 1]; ++c) {
            for (int32_t i = 0; i < W; ++i) {
                int64_t e = i * ld + c;
                double gp = (double)g[e] + (double)wd * (double)x_in[e];
                double vn = (double)mu * (double)v_in[e] + gp;
                v_out[e] = vn;
                xh[i] = (double)x_in[e] - (double)lr * vn;
            }
            for (int32_t i = 0; i < W; ++i)
                x_out[i * ld + c] = (xh[i] + xh[peers[(int64_t)s * W + i]]) * 0.5;
        }
    free(xh);
    return 0;
}

/* Same steps, every operation rounded to fp32, no fused multiply-add
 * (build with -ffp-contract=off). */
int oracle_sgd_fused_mix_f32(const float *x_in, const float *v_in, const float *g,
                             float *x_out, float *v_out, float lr, float mu, float wd,
                             int64_t ld, int32_t W, int64_t P, int32_t S,
                             const int64_t *seg_off, const int32_t *peers)
{
    (void)P;
    float *xh = (float *)malloc(sizeof(float) * (size_t)W);
    if (!xh) return -2;
    for (int32_t s = 0; s < S; ++s)
        for (int64_t c = seg_off[s]; c < seg_off[s + 1]; ++c) {
            for (int32_t i = 0; i < W; ++i) {
                int64_t e = i * ld + c;
                float t0 = wd * x_in[e];
                float gp = g[e] + t0;
                float t1 = mu * v_in[e];
                float vn = t1 + gp;
                float t2 = lr * vn;
                v_out[e] = vn;
                xh[i] = x_in[e] - t2;
            }
            for (int32_t i = 0; i < W; ++i)
                x_out[i * ld + c] = (xh[i] + xh[peers[(int64_t)s * W + i]]) * 0.5f;
        }
    free(xh);
    return 0;
}

/* ------------------------------------------------------------------------- */
/* Hierarchical Crossover-SGD as Section 3.3 states it: (1) the gradients of  */
/* the G workers of a group are reduced (averaged) at the group's leader,     */
/* which applies them to its model with the momentum-SGD step above; (2) the  */
/* L = W/G leaders gossip segment-wise on the updated parameters; (3) every   */
/* leader's result is broadcast to its group.                                 */
/*   x  float [W][ld]  only leader rows (row g*G) are read; all rows written  */
/*   v  float [L][ld]  the leaders' momentum                                  */
/*   g  float [W][ld]  every worker's gradient                                */
/* With L == 1 step (2) is empty: this is AllReduce-SGD.                      */
/* ------------------------------------------------------------------------- */
int oracle_hier_sgd_fused_mix_f64(const float *x_in, const float *v_in, const float *g,
                                  double *x_out, double *v_out, float lr, float mu, float wd,
                                  int64_t ld, int32_t W, int64_t P, int32_t G, int32_t S,
                                  const int64_t *seg_off, const int32_t *leader_peers)
{
    (void)P;
    int32_t L = W / G;
    double *h = (double *)malloc(sizeof(double) * (size_t)L);
    if (!h) return -2;
    for (int32_t s = 0; s < S; ++s)
        for (int64_t c = seg_off[s]; c < seg_off[s + 1]; ++c) {
            for (int32_t q = 0; q < L; ++q) {
                double gbar = 0.0;
                for (int32_t j = 0; j < G; ++j)
                    gbar += (double)g[((int64_t)q * G + j) * ld + c];
                gbar /= (double)G;
                double xl = (double)x_in[(int64_t)q * G * ld + c];
                double gp = gbar + (double)wd * xl;
                double vn = (double)mu * (double)v_in[(int64_t)q * ld + c] + gp;
                v_out[(int64_t)q * ld + c] = vn;
                h[q] = xl - (double)lr * vn;
            }
            for (int32_t q = 0; q < L; ++q) {
                double y = h[q];
                if (L > 1) y = (h[q] + h[leader_peers[(int64_t)s * L + q]]) * 0.5;
                for (int32_t j = 0; j < G; ++j)
                    x_out[((int64_t)q * G + j) * ld + c] = y;
            }
        }
    free(h);
    return 0;
}

/* Same steps in fp32 with the fixed order: pairwise-tree gradient sum times the
 * fp32 reciprocal of G, then the unfused fp32 optimizer step and average. */
int oracle_hier_sgd_fused_mix_f32(const float *x_in, const float *v_in, const float *g,
                                  float *x_out, float *v_out, float lr, float mu, float wd,
                                  int64_t ld, int32_t W, int64_t P, int32_t G, int32_t S,
                                  const int64_t *seg_off, const int32_t *leader_peers)
{
    (void)P;
    int32_t L = W / G;
    float inv_g = 1.0f / (float)G;
    float *h = (float *)malloc(sizeof(float) * (size_t)L);
    if (!h) return -2;
    for (int32_t s = 0; s < S; ++s)
        for (int64_t c = seg_off[s]; c < seg_off[s + 1]; ++c) {
            for (int32_t q = 0; q < L; ++q) {
                float gbar = tree_sum_f32(g + (int64_t)q * G * ld + c, ld, G) * inv_g;
                float xl = x_in[(int64_t)q * G * ld + c];
                float t0 = wd * xl;
                float gp = gbar + t0;
                float t1 = mu * v_in[(int64_t)q * ld + c];
                float vn = t1 + gp;
                float t2 = lr * vn;
                v_out[(int64_t)q * ld + c] = vn;
                h[q] = xl - t2;
            }
            for (int32_t q = 0; q < L; ++q) {
                float y = h[q];
                if (L > 1) y = (h[q] + h[leader_peers[(int64_t)s * L + q]]) * 0.5f;
                for (int32_t j = 0; j < G; ++j)
                    x_out[((int64_t)q * G + j) * ld + c] = y;
            }
        }
    free(h);
    return 0;
}

/* ------------------------------------------------------------------------- */
/* The optimizer steps on 16-bit rows (Section 4.1 / Table 1: the paper trains  */
/* in mixed precision).  Reading: the parameters x and the gradients g are held */
/* in the 16-bit format (fmt 0 = bfloat16, 1 = binary16), the momentum v stays  */
/* fp32, as mixed-precision optimizers keep their state.  Every input is        */
/* widened exactly, the step runs in double exactly as above, v' is rounded     */
/* once to fp32 and x' ONCE to the 16-bit format, straight from the double (not */
/* through fp32: rounding twice can land on the wrong side of a tie).           */
/* ------------------------------------------------------------------------- */
/* double -> 16-bit pattern, nearest, ties to even, straight from the double's own bits.
 * keep = fraction bits of the target (7 or 10), emin = its smallest normal exponent. */
static uint16_t round_double_to_16(double d, int keep, int emin, int emax, int bias)
{
    uint64_t u;
    memcpy(&u, &d, sizeof u);
    uint16_t sign = (uint16_t)((u >> 48) & 0x8000u);
    uint64_t a = u & 0x7fffffffffffffffULL;
    uint16_t inf = (uint16_t)(((1u << (15 - keep)) - 1u) << keep);
    if (a > 0x7ff0000000000000ULL) return (uint16_t)(sign | inf | (1u << (keep - 1)));   /* NaN stays a quiet NaN */
    if (a == 0x7ff0000000000000ULL) return (uint16_t)(sign | inf);
    if (a == 0) return sign;
    int e = (int)(a >> 52) - 1023;                     /* widened 16- and 32-bit values are normal doubles */
    uint64_t m = (a & 0xfffffffffffffULL) | (1ULL << 52);   /* 53-bit significand, value = m * 2^(e-52) */
    if ((a >> 52) == 0) { e = -1022; m = a; }          /* a subnormal double: far below both formats */
    /* the unit of the result: 2^(e-keep) for a normal result, 2^(emin-keep) in the subnormal range */
    int drop = 52 - keep + (e < emin ? emin - e : 0);   /* low bits of m that fall below that unit */
    uint64_t q, rest, half;
    if (drop >= 64) { q = 0; rest = 1; half = 2; }      /* far below half a unit */
    else {
        q = m >> drop;
        rest = m & ((1ULL << drop) - 1ULL);
        half = 1ULL << (drop - 1);
    }
    if (rest > half || (rest == half && (q & 1ULL))) ++q;
    /* q counts units; turn it into exponent and fraction fields (a carry moves up by itself) */
    uint32_t bits;
    if (e < emin) bits = (uint32_t)q;                   /* subnormal, or exactly the smallest normal */
    else bits = (uint32_t)(((uint64_t)(e + bias - 1) << keep) + q);   /* q includes the hidden one */
    if (bits >= inf || e > emax) return (uint16_t)(sign | inf);       /* overflow to infinity */
    return (uint16_t)(sign | bits);
}

uint16_t oracle_f64_to_bf16(double d) { return round_double_to_16(d, 7, -126, 127, 127); }
uint16_t oracle_f64_to_f16(double d) { return round_double_to_16(d, 10, -14, 15, 15); }

static uint16_t narrow16_from_double(int fmt, double d) { return fmt ? oracle_f64_to_f16(d) : oracle_f64_to_bf16(d); }

/* n doubles -> n 16-bit patterns, each rounded once (the loop over the function above). */
void oracle_narrow16_array(int fmt, const double *in, uint16_t *out, int64_t n)
{
    for (int64_t i = 0; i < n; ++i) out[i] = narrow16_from_double(fmt, in[i]);
}

/* The hierarchical step on 16-bit rows with ONE rounding: oracle_hier_mix16_f64's doubles, each
 * rounded straight to the 16-bit format (the variant above rounds an fp32 tree sum instead). */
int oracle_hier_mix16(int fmt, const uint16_t *x_in, uint16_t *x_out, int64_t ld, int32_t W,
                      int64_t P, int32_t G, int32_t S, const int64_t *seg_off,
                      const int32_t *leader_peers)
{
    size_t n = (size_t)W * (size_t)ld;
    double *y = (double *)calloc(n, sizeof(double));
    if (!y) return -2;
    int rc = oracle_hier_mix16_f64(fmt, x_in, y, ld, W, P, G, S, seg_off, leader_peers);
    for (int32_t s = 0; rc == 0 && s < S; ++s)
        for (int64_t c = seg_off[s]; c < seg_off[s + 1]; ++c)
            for (int32_t i = 0; i < W; ++i) x_out[i * ld + c] = narrow16_from_double(fmt, y[i * ld + c]);
    free(y);
    return rc;
}

/* Reference mode: the unrounded doubles.  x, g: uint16 [W][ld]; v: float [W][ld]. */
int oracle_sgd_fused_mix16_f64(int fmt, const uint16_t *x_in, const float *v_in, const uint16_t *g,
                               double *x_out, double *v_out, float lr, float mu, float wd,
                               int64_t ld, int32_t W, int64_t P, int32_t S,
                               const int64_t *seg_off, const int32_t *peers)
{
    (void)P;
    double *xh = (double *)malloc(sizeof(double) * (size_t)W);
    if (!xh) return -2;
    for (int32_t s = 0; s < S; ++s)
        for (int64_t c = seg_off[s]; c < seg_off[s + 1]; ++c) {
            for (int32_t i = 0; i < W; ++i) {
                int64_t e = i * ld + c;
                double x = (double)widen16(fmt, x_in[e]);
                double gp = (double)widen16(fmt, g[e]) + (double)wd * x;
                double vn = (double)mu * (double)v_in[e] + gp;
                v_out[e] = vn;
                xh[i] = x - (double)lr * vn;
            }
            for (int32_t i = 0; i < W; ++i)
                x_out[i * ld + c] = (xh[i] + xh[peers[(int64_t)s * W + i]]) * 0.5;
        }
    free(xh);
    return 0;
}

/* The step as the 16-bit entry points return it: x' in the 16-bit format, v' in fp32, each
 * rounded once from the reference's double. */
int oracle_sgd_fused_mix16(int fmt, const uint16_t *x_in, const float *v_in, const uint16_t *g,
                           uint16_t *x_out, float *v_out, float lr, float mu, float wd,
                           int64_t ld, int32_t W, int64_t P, int32_t S,
                           const int64_t *seg_off, const int32_t *peers)
{
    size_t n = (size_t)W * (size_t)ld;
    double *x64 = (double *)calloc(n, sizeof(double)), *v64 = (double *)calloc(n, sizeof(double));
    if (!x64 || !v64) { free(x64); free(v64); return -2; }
    int rc = oracle_sgd_fused_mix16_f64(fmt, x_in, v_in, g, x64, v64, lr, mu, wd, ld, W, P, S, seg_off, peers);
    for (int32_t s = 0; rc == 0 && s < S; ++s)
        for (int64_t c = seg_off[s]; c < seg_off[s + 1]; ++c)
            for (int32_t i = 0; i < W; ++i) {
                x_out[i * ld + c] = narrow16_from_double(fmt, x64[i * ld + c]);
                v_out[i * ld + c] = (float)v64[i * ld + c];
            }
    free(x64);
    free(v64);
    return rc;
}

/* Section 3.3 with gradients on 16-bit rows: g uint16 [W][ld], x uint16 [W][ld] (leader rows
 * read, all rows written), v float [L][ld]. */
int oracle_hier_sgd_fused_mix16_f64(int fmt, const uint16_t *x_in, const float *v_in, const uint16_t *g,
                                    double *x_out, double *v_out, float lr, float mu, float wd,
                                    int64_t ld, int32_t W, int64_t P, int32_t G, int32_t S,
                                    const int64_t *seg_off, const int32_t *leader_peers)
{
    (void)P;
    int32_t L = W / G;
    double *h = (double *)malloc(sizeof(double) * (size_t)L);
    if (!h) return -2;
    for (int32_t s = 0; s < S; ++s)
        for (int64_t c = seg_off[s]; c < seg_off[s + 1]; ++c) {
            for (int32_t q = 0; q < L; ++q) {
                double gbar = 0.0;
                for (int32_t j = 0; j < G; ++j)
                    gbar += (double)widen16(fmt, g[((int64_t)q * G + j) * ld + c]);
                gbar /= (double)G;
                double xl = (double)widen16(fmt, x_in[(int64_t)q * G * ld + c]);
                double gp = gbar + (double)wd * xl;
                double vn = (double)mu * (double)v_in[(int64_t)q * ld + c] + gp;
                v_out[(int64_t)q * ld + c] = vn;
                h[q] = xl - (double)lr * vn;
            }
            for (int32_t q = 0; q < L; ++q) {
                double y = h[q];
                if (L > 1) y = (h[q] + h[leader_peers[(int64_t)s * L + q]]) * 0.5;
                for (int32_t j = 0; j < G; ++j)
                    x_out[((int64_t)q * G + j) * ld + c] = y;
            }
        }
    free(h);
    return 0;
}

int oracle_hier_sgd_fused_mix16(int fmt, const uint16_t *x_in, const float *v_in, const uint16_t *g,
                                uint16_t *x_out, float *v_out, float lr, float mu, float wd,
                                int64_t ld, int32_t W, int64_t P, int32_t G, int32_t S,
                                const int64_t *seg_off, const int32_t *leader_peers)
{
    int32_t L = W / G;
    size_t n = (size_t)W * (size_t)ld, nl = (size_t)L * (size_t)ld;
    double *x64 = (double *)calloc(n, sizeof(double)), *v64 = (double *)calloc(nl, sizeof(double));
    if (!x64 || !v64) { free(x64); free(v64); return -2; }
    int rc = oracle_hier_sgd_fused_mix16_f64(fmt, x_in, v_in, g, x64, v64, lr, mu, wd, ld, W, P, G, S, seg_off, leader_peers);
    for (int32_t s = 0; rc == 0 && s < S; ++s)
        for (int64_t c = seg_off[s]; c < seg_off[s + 1]; ++c) {
            for (int32_t i = 0; i < W; ++i) x_out[i * ld + c] = narrow16_from_double(fmt, x64[i * ld + c]);
            for (int32_t q = 0; q < L; ++q) v_out[q * ld + c] = (float)v64[q * ld + c];
        }
    free(x64);
    free(v64);
    return rc;
}

/* ------------------------------------------------------------------------- */
/* SGP-style push-sum comparison: every row keeps half of its (x, w) and      */
/* pushes half to row (i + hop) mod W, i.e. row i receives from (i - hop):    */
/*     x'_i = (x_i + x_{i-hop}) / 2 ;  w'_i = (w_i + w_{i-hop}) / 2 ;         */
/*     z_i = x'_i / w'_i  (de-biased parameters, optional).                   */
/* Whole vector at once (model-wise, S = 1).                                  */
/* ------------------------------------------------------------------------- */
int oracle_pushsum_mix_f64(const float *x_in, const float *w_in, double *x_out,
                           double *w_out, double *z_out /* may be NULL */,
                           int64_t ld, int32_t W, int64_t P, int32_t hop)
{
    for (int32_t i = 0; i < W; ++i) {
        int32_t j = ((i - hop) % W + W) % W;
        double wn = ((double)w_in[i] + (double)w_in[j]) * 0.5;
        w_out[i] = wn;
        for (int64_t c = 0; c < P; ++c) {
            double xn = ((double)x_in[i * ld + c] + (double)x_in[j * ld + c]) * 0.5;
            x_out[i * ld + c] = xn;
            if (z_out) z_out[i * ld + c] = xn / wn;
        }
    }
    return 0;
}

int oracle_pushsum_mix_f32(const float *x_in, const float *w_in, float *x_out,
                           float *w_out, float *z_out /* may be NULL */,
                           int64_t ld, int32_t W, int64_t P, int32_t hop)
{
    for (int32_t i = 0; i < W; ++i) {
        int32_t j = ((i - hop) % W + W) % W;
        float wn = (w_in[i] + w_in[j]) * 0.5f;
        w_out[i] = wn;
        for (int64_t c = 0; c < P; ++c) {
            float xn = (x_in[i * ld + c] + x_in[j * ld + c]) * 0.5f;
            x_out[i * ld + c] = xn;
            if (z_out) z_out[i * ld + c] = xn / wn;
        }
    }
    return 0;
}

/* Push-sum on 16-bit rows (Section 4.1's mixed precision applied to the SGP comparison of Sections 2.1 and 3):
 * the parameter rows are bfloat16 (fmt 0) or binary16 (fmt 1), the push-sum weights stay fp32.  The rows are
 * widened exactly and the round is the fp32 one above, value for value:
 *     xn = (float(x_i) + float(x_{i-hop})) * 0.5f ;  wn = (w_i + w_{i-hop}) * 0.5f ;
 *     x'_i = round16(xn) ;  z_i = round16(xn / wn)        (z from the unrounded fp32 average)
 * with round16 = round to nearest even into the row format.  The _f64 variant returns the same quantities
 * in double arithmetic, unrounded, as the reference the 16-bit results are measured against. */
int oracle_pushsum_mix16(int fmt, const uint16_t *x_in, const float *w_in, uint16_t *x_out, float *w_out,
                         uint16_t *z_out /* may be NULL */, int64_t ld, int32_t W, int64_t P, int32_t hop)
{
    if (fmt != 0 && fmt != 1) return -1;
    for (int32_t i = 0; i < W; ++i) {
        int32_t j = ((i - hop) % W + W) % W;
        float wn = (w_in[i] + w_in[j]) * 0.5f;
        w_out[i] = wn;
        for (int64_t c = 0; c < P; ++c) {
            float xn = (widen16(fmt, x_in[i * ld + c]) + widen16(fmt, x_in[j * ld + c])) * 0.5f;
            x_out[i * ld + c] = narrow16(fmt, xn);
            if (z_out) z_out[i * ld + c] = narrow16(fmt, xn / wn);
        }
    }
    return 0;
}

int oracle_pushsum_mix16_f64(int fmt, const uint16_t *x_in, const float *w_in, double *x_out, double *w_out,
                             double *z_out /* may be NULL */, int64_t ld, int32_t W, int64_t P, int32_t hop)
{
    if (fmt != 0 && fmt != 1) return -1;
    for (int32_t i = 0; i < W; ++i) {
        int32_t j = ((i - hop) % W + W) % W;
        double wn = ((double)w_in[i] + (double)w_in[j]) * 0.5;
        w_out[i] = wn;
        for (int64_t c = 0; c < P; ++c) {
            double xn = ((double)widen16(fmt, x_in[i * ld + c]) + (double)widen16(fmt, x_in[j * ld + c])) * 0.5;
            x_out[i * ld + c] = xn;
            if (z_out) z_out[i * ld + c] = xn / wn;
        }
    }
    return 0;
}
