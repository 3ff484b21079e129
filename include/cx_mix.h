/*
 * cx_mix.h -- C ABI of the MI355X (gfx950) segment-wise gossip parameter-mixing library.
 *
 * The library implements the data-parallel hot path of Crossover-SGD
 * (arXiv 2012.15198): W simulated workers' flat fp32 parameter vectors are the rows
 * of one HBM-resident matrix, every vector is cut into S segments, and in every
 * round each segment of each row is averaged with the same segment of a peer row
 * taken from a per-(round, segment) peer table (Algorithm 1); the tables come from
 * the random topology with fair peer selection (Algorithm 2).
 *
 * Common conventions
 *   x          float32 [W][ld] row-major DEVICE memory, row i = worker i; columns
 *              [0,P) are used, [P,ld) are never read or written.  ld % 4 == 0 and
 *              16-byte aligned base pointers are required (CX_ERR_ALIGN otherwise).
 *   seg_off    int64 [S+1] DEVICE memory, non-decreasing, seg_off[0] = 0,
 *              seg_off[S] = P; segment s = columns [seg_off[s], seg_off[s+1]).
 *              Segment starts need not be multiples of 4.  Empty segments are fine.
 *   peers      int32 [S][n] DEVICE memory for ONE round; peers[s][i] is the row
 *              whose segment s row i RECEIVES and averages with (Algorithm 1:
 *              receive_from = destinations[my_rank]).  Each peers[s] must be a
 *              permutation of 0..n-1; the method's tables also have no fixed point.
 *   stream     a hipStream_t passed as void* (NULL = the default stream).  Mixing
 *              calls only enqueue work: they never synchronise, never allocate and
 *              never free device memory.  The caller owns every buffer and must keep
 *              it alive until the stream has passed the call.  A call enqueues one
 *              mixing kernel (out of place: preceded by a few-microsecond kernel that
 *              derives the row order from the peer table).
 *   buffers    x_out may be the same pointer as x_in (in place) or a second matrix that
 *              does not overlap it (out of place, e.g. two buffers used in turn round
 *              after round); partial overlap is CX_ERR_ALIAS.  Either way every value is
 *              computed from the round's input rows (Algorithm 1 posts every send before
 *              any averaging), every element is read from HBM once and written once, and
 *              for peer tables that are permutations the results are bit-identical (a table
 *              that is not a permutation is honoured out of place only: see "peer table").
 *              The two cases run different kernels:
 *              in place, one wavefront owns a column tile and walks the rows along the
 *              cycles of the peer permutation; out of place, one short workgroup per
 *              (row, column chunk) reads the row and its peer and writes the result --
 *              the faster of the two on MI355X (about 75 % against about 71 % of the HBM
 *              peak on a 32 x 25.6M matrix).
 *   peer table in place, each peers[s] must be a permutation of 0..n-1: a segment whose
 *              table is not one is left unmixed (treated as the identity).  Out of place,
 *              any table with entries in [0, n) is served as written (a table with
 *              duplicates, i.e. a random topology without fair peer selection, included);
 *              an entry outside [0, n) stands for the row itself.  Segment offsets are
 *              clamped to [0, P].  No table content can make a kernel index out of bounds.
 *              Device tables are NOT read by the host: check their host mirrors with
 *              cx_check_segments / cx_check_peers before uploading.
 *   scratch    the out-of-place kernels keep a row-order table in library-owned device
 *              memory (static, per entry point 4 slots of 1 MiB per GPU), so no call
 *              allocates.  A slot serves one stream at a time; calls on one stream run in
 *              order, so a table is never rewritten while it is read.  A stream keeps its slot
 *              while it has work in flight; when all slots are taken, the slot of a stream that
 *              has drained or been destroyed changes hands, and a stream that finds none runs
 *              without the table: same results, lower speed.  Calls recorded under stream
 *              capture get a slot apart from the one their stream uses for eager calls and keep
 *              it, so a captured graph may be replayed on any stream while eager calls go on;
 *              graphs captured on ONE stream share that slot: replay them in one stream's order.
 *              Matrices under 64 MiB run without the table (nothing to gain: they stay cached).
 *              Host threads may call concurrently; the two launches of a call stay together.
 *   limits     at most CX_MAX_ROWS gossiping rows (W, or W/G in hierarchical mode).
 *   return     CX_OK (0) or a negative cx_status.  Argument errors are detected on the host
 *              before anything is enqueued.
 */
#ifndef CX_MIX_H
#define CX_MIX_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define CX_MAX_ROWS 1024

enum cx_status {
    CX_OK = 0,
    CX_ERR_NULL = -1,        /* a required pointer is NULL */
    CX_ERR_SHAPE = -2,       /* W, P, S, G, ld, hop, R ... out of range */
    CX_ERR_SEGMENTS = -3,    /* seg_off is not 0 = o[0] <= o[1] <= ... <= o[S] = P */
    CX_ERR_PEERS = -4,       /* a peer row is not a fixed-point-free permutation */
    CX_ERR_ALIGN = -5,       /* pointer not 16-byte aligned or ld % 4 != 0 */
    CX_ERR_ALIAS = -6,       /* buffers overlap in an unsupported way */
    CX_ERR_HIP = -7,         /* the HIP runtime reported an error at launch */
    CX_ERR_UNSUPPORTED = -8, /* valid request this build cannot serve (see each call) */
    CX_ERR_MEMORY = -9       /* cx_hbm_alloc: not enough free device memory */
};

/* Topology modes of cx_topology_gen. */
enum cx_topology_mode {
    CX_TOPO_FAIR = 0,                /* Algorithm 2: random topology with fair peer selection */
    CX_TOPO_DIRECTED_EXP = 1,        /* SGP's time-varying directed exponential graph */
    CX_TOPO_UNFAIR = 2,              /* random topology without fair selection (duplicates) */
    CX_TOPO_SAME_ALL_SEGMENTS = 16   /* OR-ed in: segment 0's table for every segment */
};

/* Human-readable name of a status code (static storage). */
const char *cx_status_string(int status);

/* ABI version of this header (bumped on any signature change): 4. */
int cx_abi_version(void);

/* ------------------------------------------------------------------------------------
 * cx_topology_gen -- Algorithm 2, "random topology with fair peer selection", for
 * rounds [round0, round0+R), S segments and n gossiping rows.  HOST call, host memory.
 *   mode 0  fair random topology: for i = 0..n-1 draw uniformly among the rows that are
 *           neither i (zero diagonal of the roulette) nor already chosen, candidates in
 *           ascending order.  If the last row finds only itself left, it swaps with a
 *           uniformly drawn earlier row k (d[n-1] = d[k], d[k] = n-1).  Draws come from
 *           a counter-based generator keyed by (seed, round, segment, draw index), so a
 *           table is a pure function of its coordinates: every worker derives the same
 *           one from the shared seed, every segment gets a different one (Section 3),
 *           and a run can be resumed at any round.
 *   mode 1  time-varying directed exponential graph of the SGP comparison: in round t
 *           row i receives from (i - 2^(t mod ceil(log2 n))) mod n, for every segment.
 *   mode 2  the conventional random topology the paper compares with (Sections 3.2, 4.3):
 *           row i draws uniformly among the other n-1 rows (draw index i), independently of
 *           the other rows, so a row may be chosen several times or never.  Such a table is
 *           not a permutation: mix with it OUT OF PLACE only (in place it would leave every
 *           segment unmixed; see cx_check_peers).
 *   | 16    every segment of a round gets segment 0's table, which equals model-wise
 *           communication (Section 3; the "without segment-wise" ablation of Section 4.3).
 *   peers_host  int32 [R][S][n], caller-allocated, written completely on success.
 * Errors: CX_ERR_NULL; CX_ERR_SHAPE if n < 2, n > CX_MAX_ROWS, S < 1, R < 0, round0 < 0
 * or round0 + R overflows; CX_ERR_UNSUPPORTED for an unknown mode.
 */
int cx_topology_gen(uint64_t seed, int32_t n, int32_t S, int32_t round0, int32_t R,
                    int32_t mode, int32_t *peers_host);

/* Host-side checks of the host mirrors of the device tables.  The mixing calls never read a
 * device table on the host (that would need a synchronisation), so a caller validates the
 * host copy before uploading it.
 * cx_check_segments: 0 = seg_off[0] <= seg_off[1] <= ... <= seg_off[S] = P, else CX_ERR_SEGMENTS.
 * cx_check_peers: peers_host is int32 [S][n]; `mode` names the kind of table, which is also what
 * the two kernels accept:
 *   CX_TOPO_FAIR, CX_TOPO_DIRECTED_EXP  every peers[s] is a permutation of 0..n-1 without a fixed
 *       point (Section 3.2: every row is chosen exactly once and nobody chooses itself).  This is
 *       what a call that updates its matrix IN PLACE needs: in place, a segment whose table is not
 *       a permutation is left unmixed (the call still returns CX_OK: it cannot look).
 *   CX_TOPO_UNFAIR  entries in [0, n), no row names itself, duplicates allowed (the random
 *       topology without fair peer selection of Sections 3.2 / 4.3).  Such a table is served as
 *       written by calls whose output buffers differ from their input buffers, and ONLY by them.
 * OR-ing CX_TOPO_SAME_ALL_SEGMENTS into mode additionally requires all S tables to be equal.
 * Returns CX_ERR_PEERS for a table that fails its mode's test, CX_ERR_UNSUPPORTED for an unknown
 * mode, CX_ERR_NULL / CX_ERR_SHAPE (S < 1, n < 2, n > CX_MAX_ROWS) as usual. */
int cx_check_segments(const int64_t *seg_off_host, int32_t S, int64_t P);
int cx_check_peers(const int32_t *peers_host, int32_t S, int32_t n, int32_t mode);

/* ------------------------------------------------------------------------------------
 * cx_gossip_mix -- Algorithm 1, averaging step, for all W rows at once:
 *     x_out[i][c] = (x_in[i][c] + x_in[peers[s][i]][c]) * 0.5f   for c in segment s,
 * one fp32 add and one fp32 multiply per element (round-to-nearest-even, subnormals
 * kept), so results are bit-identical to that formula evaluated in any language.
 * Errors: CX_ERR_NULL; CX_ERR_SHAPE if W < 2, W > CX_MAX_ROWS, S < 1, P < 1, ld < P;
 * CX_ERR_ALIGN; CX_ERR_ALIAS; CX_ERR_UNSUPPORTED if flags != 0; CX_ERR_HIP.
 */
int cx_gossip_mix(const float *x_in, float *x_out, int64_t ld, int32_t W, int64_t P,
                  int32_t S, const int64_t *seg_off_dev, const int32_t *peers_dev,
                  uint32_t flags, void *stream);

/* ------------------------------------------------------------------------------------
 * cx_gossip_mix_noalloc -- cx_gossip_mix, out of place, for callers that cannot allocate device
 * memory or call anything that might: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same arguments, same kernels and bit-identical results; the
 * difference is where the kernels' scratch (the row-order table) lives: in ONE static device
 * array of CX_NOALLOC_ORDER_WORDS 32-bit words (1 MiB) per GPU, held until the process ends, whose
 * address the library asks the runtime for once per device.  The call makes no hipMalloc /
 * hipFree and no allocating library call; it enqueues two kernels on `stream`.
 *   x_out must differ from x_in (CX_ERR_ALIAS otherwise: the in-place kernel has no scratch).
 *   The table needs W words per cluster of 65,536 columns (8 clusters side by side):
 *   CX_ERR_SHAPE if ceil(P / 1024) > 64 * (CX_NOALLOC_ORDER_WORDS / W - 8), e.g. P > 133 M columns
 *   at W = 128 or P > 16 M at W = 1024 -- the call never falls back to a slower path silently.
 *   (Launch parameters changed through cx_set_tuning move this limit.)
 *   Every call on a GPU uses that GPU's one table, on whatever stream: calls that overlap in time
 *   on one GPU race on it and give wrong results -- run them in one stream's order.  Nothing
 *   has to be cleared between calls: a call rewrites every word it reads.
 * Errors otherwise as cx_gossip_mix; CX_ERR_HIP also if the runtime cannot name the array.
 */
#define CX_NOALLOC_ORDER_WORDS (1 << 18)
int cx_gossip_mix_noalloc(const float *x_in, float *x_out, int64_t ld, int32_t W, int64_t P,
                          int32_t S, const int64_t *seg_off_dev, const int32_t *peers_dev,
                          uint32_t flags, void *stream);

/* ------------------------------------------------------------------------------------
 * cx_hier_mix -- hierarchical Crossover-SGD (Section 3.3) on parameters: groups are G
 * consecutive rows, the first row of a group is its leader, L = W / G.
 *     m_g  = (x_{gG} + x_{gG+1} + ... + x_{gG+G-1}) / G        (rows summed in order)
 *     y_g  = (m_g + m_{leader_peers[s][g]}) * 0.5              (skipped when L == 1)
 *     every row of group g  <-  fp32(y_g)
 * evaluated in fp64 (inputs widened exactly) and rounded ONCE to fp32, nearest even: the result is
 * the correctly rounded value of the formula, within 2^-24 relative of it however much cancels
 * inside a group.  G == 1 is cx_gossip_mix (its fp32 formula, bit for bit).
 * leader_peers_dev is int32 [S][L] (may be NULL when L == 1: the result is then the
 * global mean, i.e. the AllReduce mixing matrix).
 * Errors: as cx_gossip_mix, plus CX_ERR_SHAPE if G < 1, W % G != 0 or L > CX_MAX_ROWS;
 * CX_ERR_UNSUPPORTED if G is not one of 1 ... 8, 16.
 */
int cx_hier_mix(const float *x_in, float *x_out, int64_t ld, int32_t W, int64_t P,
                int32_t G, int32_t S, const int64_t *seg_off_dev,
                const int32_t *leader_peers_dev, uint32_t flags, void *stream);

/* ------------------------------------------------------------------------------------
 * cx_pushsum_mix -- SGP-style push-sum comparison (Sections 2.1 and 3): every row keeps
 * half of (x, w) and pushes half to row (i + hop) mod W, model-wise (one segment):
 *     j = (i - hop) mod W
 *     x_out[i] = (x_in[i] + x_in[j]) * 0.5f ;  w_out[i] = (w_in[i] + w_in[j]) * 0.5f
 *     z_out[i] = x_out[i] / w_out[i]            (only if z_out != NULL)
 * w_in / w_out are float32 [W] DEVICE vectors and must not overlap each other.
 * z_out (float32 [W][ld]) must not overlap x_in or x_out.
 * Errors: as cx_gossip_mix, plus CX_ERR_SHAPE if hop is outside [1, W).
 */
int cx_pushsum_mix(const float *x_in, float *x_out, const float *w_in, float *w_out,
                   float *z_out, int64_t ld, int32_t W, int64_t P, int32_t hop,
                   uint32_t flags, void *stream);

/* ------------------------------------------------------------------------------------
 * cx_sgd_fused_mix -- local momentum-SGD step fused in front of Algorithm 1's averaging
 * (Section 3.1: parameters are averaged after the gradient has been applied):
 *     t = g + wd * x ;  v' = mu * v + t ;  h = x - lr * v'                       (per row)
 *     x_out[i][c] = fp32((h[i][c] + h[peers[s][i]][c]) * 0.5) ;  v_out = fp32(v')
 * The whole chain, the average included, is evaluated in fp64 (inputs widened exactly, lr, mu,
 * wd as the doubles of their fp32 values, operations in the order written, no fused
 * multiply-add); v' and x_out are each rounded ONCE to fp32 (nearest even).  Results are
 * therefore the correctly rounded values of that fp64 formula: within 2^-24 relative of it,
 * however large lr * v' is against x.
 * v_out may equal v_in (in place) and x_out may equal x_in; g is only read.
 * x, v and g share shape and ld.  Each of x, v, g is read once, x and v written once.
 * Errors: as cx_gossip_mix.
 */
int cx_sgd_fused_mix(const float *x_in, float *x_out, const float *v_in, float *v_out,
                     const float *g, float lr, float mu, float wd, int64_t ld, int32_t W,
                     int64_t P, int32_t S, const int64_t *seg_off_dev,
                     const int32_t *peers_dev, uint32_t flags, void *stream);

/* ------------------------------------------------------------------------------------
 * cx_hier_sgd_fused_mix -- hierarchical Crossover-SGD exactly as Section 3.3 states it:
 * (1) the gradients of the G workers of a group are reduced at the group's leader, which
 * applies them to its model; (2) the L = W / G leaders gossip segment-wise (Algorithm 1);
 * (3) each leader's result is broadcast to its group.
 *     gbar_q = (g_{qG} + g_{qG+1} + ... + g_{qG+G-1}) / G              (summed in row order)
 *     t = gbar_q + wd * x_q ;  v'_q = mu * v_q + t ;  h_q = x_q - lr * v'_q     (x_q = leader row)
 *     y_q = (h_q + h_{leader_peers[s][q]}) * 0.5                         (skipped when L == 1)
 *     every row of group q  <-  fp32(y_q) ;  v_out[q] = fp32(v'_q)
 * evaluated in fp64 and rounded once, as in cx_sgd_fused_mix.
 *   x_in, x_out, g   float32 [W][ld]; of x_in only the leader rows (q * G) are read
 *   v_in, v_out      float32 [L][ld]: the leaders' momentum
 * x_out may equal x_in and v_out may equal v_in (then both must); with L == 1 this is
 * AllReduce-SGD.  Per worker-parameter it moves 8 + 12/G bytes (read g, write x; the leader
 * also reads x, v and writes v).
 * Errors: as cx_hier_mix (group sizes 1 ... 8, 16); CX_ERR_ALIAS also if exactly one of x, v is
 * updated in place, or v overlaps x or g.
 */
int cx_hier_sgd_fused_mix(const float *x_in, float *x_out, const float *v_in, float *v_out,
                          const float *g, float lr, float mu, float wd, int64_t ld, int32_t W,
                          int64_t P, int32_t G, int32_t S, const int64_t *seg_off_dev,
                          const int32_t *leader_peers_dev, uint32_t flags, void *stream);

/* ------------------------------------------------------------------------------------
 * cx_gossip_mix_bf16 -- cx_gossip_mix on bfloat16 rows (the paper trains in mixed precision,
 * Section 4.1 / Table 1): x is uint16 [W][ld] holding bfloat16 bit patterns, ld % 8 == 0,
 *     x_out[i][c] = bf16_rne((float(x_in[i][c]) + float(x_in[peers[s][i]][c])) * 0.5f),
 * fp32 arithmetic, one rounding to bfloat16 (nearest even; NaN stays a quiet NaN).  Moves
 * 4 bytes per worker-parameter.  Everything else as cx_gossip_mix.
 */
int cx_gossip_mix_bf16(const uint16_t *x_in, uint16_t *x_out, int64_t ld, int32_t W, int64_t P,
                       int32_t S, const int64_t *seg_off_dev, const int32_t *peers_dev,
                       uint32_t flags, void *stream);

/* ------------------------------------------------------------------------------------
 * cx_gossip_mix_f16 -- the same on IEEE binary16 rows (the other 16-bit format of mixed
 * precision training, Section 4.1): x is uint16 [W][ld] holding binary16 bit patterns,
 * ld % 8 == 0,
 *     x_out[i][c] = f16_rne((float(x_in[i][c]) + float(x_in[peers[s][i]][c])) * 0.5f),
 * fp32 arithmetic, one rounding to binary16 (nearest even, gradual underflow, overflow to
 * infinity; NaN stays a quiet NaN).  Everything else as cx_gossip_mix_bf16.
 */
int cx_gossip_mix_f16(const uint16_t *x_in, uint16_t *x_out, int64_t ld, int32_t W, int64_t P,
                      int32_t S, const int64_t *seg_off_dev, const int32_t *peers_dev,
                      uint32_t flags, void *stream);

/* ------------------------------------------------------------------------------------
 * cx_hier_mix_bf16 / cx_hier_mix_f16 -- cx_hier_mix (Section 3.3) on 16-bit rows: x is uint16
 * [W][ld] of bfloat16 / binary16 bit patterns, ld % 8 == 0.  Every value is widened exactly, the
 * group sum, the division by G and the leader average run in fp64 as in cx_hier_mix, and the result
 * is rounded ONCE (nearest even, straight from the fp64 value) before it is written to the G rows of
 * the group.  G = 1 ... 8 (CX_ERR_UNSUPPORTED otherwise); G = 1 is cx_gossip_mix_bf16 / _f16 (and
 * needs W >= 2).  Everything else as cx_hier_mix.
 */
int cx_hier_mix_bf16(const uint16_t *x_in, uint16_t *x_out, int64_t ld, int32_t W, int64_t P,
                     int32_t G, int32_t S, const int64_t *seg_off_dev,
                     const int32_t *leader_peers_dev, uint32_t flags, void *stream);
int cx_hier_mix_f16(const uint16_t *x_in, uint16_t *x_out, int64_t ld, int32_t W, int64_t P,
                    int32_t G, int32_t S, const int64_t *seg_off_dev,
                    const int32_t *leader_peers_dev, uint32_t flags, void *stream);

/* ------------------------------------------------------------------------------------
 * cx_sgd_fused_mix_bf16 / _f16 and cx_hier_sgd_fused_mix_bf16 / _f16 -- the two optimizer steps on
 * mixed-precision state (Section 4.1 / Table 1: the paper trains in mixed precision): parameters x and
 * gradients g are uint16 [W][ld] of bfloat16 / binary16 bit patterns, the momentum v stays float32
 * ([W][ld], or [L][ld] in the hierarchical step), all with the same ld, ld % 8 == 0.
 * Every input is widened exactly and the step runs in fp64 exactly as in cx_sgd_fused_mix /
 * cx_hier_sgd_fused_mix; v' is rounded once to fp32 and x' ONCE to the 16-bit format (nearest even,
 * straight from the fp64 value: not through fp32, which could land on the wrong side of a tie).
 * Bytes per worker-parameter: 14 (flat: read x, g, v; write x, v) and 4 + 10/G (hierarchical).
 * x and v are updated either both in place or both out of place (CX_ERR_ALIAS otherwise, and
 * for any other overlap between x, v and g).  Hierarchical group sizes: 1 ... 8.
 * Everything else as cx_sgd_fused_mix and cx_hier_sgd_fused_mix.
 */
int cx_sgd_fused_mix_bf16(const uint16_t *x_in, uint16_t *x_out, const float *v_in, float *v_out,
                          const uint16_t *g, float lr, float mu, float wd, int64_t ld, int32_t W,
                          int64_t P, int32_t S, const int64_t *seg_off_dev, const int32_t *peers_dev,
                          uint32_t flags, void *stream);
int cx_sgd_fused_mix_f16(const uint16_t *x_in, uint16_t *x_out, const float *v_in, float *v_out,
                         const uint16_t *g, float lr, float mu, float wd, int64_t ld, int32_t W,
                         int64_t P, int32_t S, const int64_t *seg_off_dev, const int32_t *peers_dev,
                         uint32_t flags, void *stream);
int cx_hier_sgd_fused_mix_bf16(const uint16_t *x_in, uint16_t *x_out, const float *v_in, float *v_out,
                               const uint16_t *g, float lr, float mu, float wd, int64_t ld, int32_t W,
                               int64_t P, int32_t G, int32_t S, const int64_t *seg_off_dev,
                               const int32_t *leader_peers_dev, uint32_t flags, void *stream);
int cx_hier_sgd_fused_mix_f16(const uint16_t *x_in, uint16_t *x_out, const float *v_in, float *v_out,
                              const uint16_t *g, float lr, float mu, float wd, int64_t ld, int32_t W,
                              int64_t P, int32_t G, int32_t S, const int64_t *seg_off_dev,
                              const int32_t *leader_peers_dev, uint32_t flags, void *stream);

/* ------------------------------------------------------------------------------------
 * cx_pushsum_mix_bf16 / cx_pushsum_mix_f16 -- the push-sum comparison (Sections 2.1 and 3) on
 * 16-bit parameter rows (Section 4.1's mixed precision): x_in, x_out and z_out are bit patterns,
 * uint16 [W][ld] with ld % 8 == 0; the weights stay float32.  Rows are widened exactly and the
 * round is cx_pushsum_mix's, value for value, each output narrowed once (nearest even):
 *     j = (i - hop) mod W ;  a = (float(x_in[i]) + float(x_in[j])) * 0.5f
 *     x_out[i] = round16(a) ;  w_out[i] = (w_in[i] + w_in[j]) * 0.5f
 *     z_out[i] = round16(a / w_out[i])       (only if z_out != NULL; from the unrounded a)
 * Errors and overlap rules as cx_pushsum_mix; CX_ERR_ALIGN if ld % 8 != 0.
 */
int cx_pushsum_mix_bf16(const uint16_t *x_in, uint16_t *x_out, const float *w_in, float *w_out,
                        uint16_t *z_out, int64_t ld, int32_t W, int64_t P, int32_t hop,
                        uint32_t flags, void *stream);
int cx_pushsum_mix_f16(const uint16_t *x_in, uint16_t *x_out, const float *w_in, float *w_out,
                       uint16_t *z_out, int64_t ld, int32_t W, int64_t P, int32_t hop,
                       uint32_t flags, void *stream);

/* ------------------------------------------------------------------------------------
 * cx_hbm_alloc / cx_hbm_free -- device memory for the worker matrices, placed for the kernels
 * above.  Not an operation of the paper: it exists because WHERE a matrix lies in physical
 * memory sets the rate of the kernels that write many rows at once (the hierarchical mix of
 * Section 3.3, the in-place walk), and a caller cannot place memory with hipMalloc.  Measured
 * on MI355X (not on every machine alike): the 288 GiB act as three zones of 96 GiB of physical addresses; the hierarchical
 * mix at W = 256 runs at 67-69 % of the HBM peak when the buffer it writes lies in the zone of
 * the buffer it reads, at 73 % into another zone, at 77-78 % when both are spread over two
 * or three zones.  Buffers that hipMalloc returns one after the other mostly share a zone.
 *   cx_hbm_alloc places `count` blocks of bytes[k] (each rounded up to 2 MiB) TOGETHER on the
 *   current device: every block is assembled from 256 MiB pieces of physical memory that lie
 *   evenly over all the memory that is free when the call starts, mapped to one virtual range
 *   (2 MiB aligned), readable and writable by that device only.  Contents are unspecified.
 *   (CX_HBM_PIECE_MIB in the environment, an even number from 2 to 1024, sets another piece
 *   size: a knob for measurements; 16, 64 and 256 MiB measured alike.)
 *   ptrs_out[k] (host array of `count` pointers) receives the device addresses; on any error
 *   every entry is NULL and nothing stays allocated.  Blocks of one call interleave, so ask
 *   for the buffers of one job (x, x', v, v', g) in one call.
 *   While the call runs it holds all free memory of the device but 8 GiB (other allocations
 *   in that window may fail); it takes a few seconds, most of it the driver clearing what is
 *   given back.  Meant for start-up, not for a loop.  Thread-safe.
 *   The pointers are ordinary device pointers for every call of this header, for kernels and
 *   hipMemcpy; they are NOT hipMalloc pointers: release each with cx_hbm_free, never hipFree.
 *   cx_hbm_free waits for the block's device to go idle (hipDeviceSynchronize: not while a
 *   stream of that device is capturing a graph), then unmaps the block.
 * Errors: CX_ERR_NULL; CX_ERR_SHAPE if count < 1, count > 64 or a size < 1; CX_ERR_UNSUPPORTED
 * if flags != 0, and from cx_hbm_free for a pointer that is not a live block of cx_hbm_alloc;
 * CX_ERR_MEMORY if the device has less free memory than asked for; CX_ERR_HIP if the runtime
 * refuses a reservation or a mapping.
 */
int cx_hbm_alloc(void **ptrs_out, const int64_t *bytes, int32_t count, uint32_t flags);
int cx_hbm_free(void *ptr);

/* ------------------------------------------------------------------------------------
 * Measurement helpers (not part of the method).
 * cx_copy_baseline: dst[i] = src[i] for n floats (n % 4 == 0, 16-byte aligned) with the
 * same load/store instructions as the mixing kernels; the practical HBM ceiling and the
 * calibration kernel for the profiler's byte counters.
 * cx_set_tuning / cx_get_tuning: process-global launch parameters for sweeps and tests.
 *   key 0: 16-byte slices per lane per row (1, 2, 4)      key 1: waves per workgroup (1..8)
 *   key 2: non-temporal stores (and in-place loads) (0/1) key 3: in place: rows in flight per lane (2, 4, 8)
 *   key 4: in place: workgroup walks rows in lock-step (0/1)
 *   key 5: 1 = use the in-place kernel for out-of-place calls too
 *   key 6: out of place: chunks per cluster (1..4096)     key 7: out of place: XCD-aware block order (0/1)
 *   key 8: out of place: rows ordered along the permutation cycles (0 never, 1 always; default: from 64 MiB)
 *   key 9: resident workgroups per CU, both kernels (1..16; 0 = as many as fit)
 *   key 10: cx_hier_mix, G = 8, out of place: 1 = reduce the group through LDS, one row per wavefront
 *           (same results as the default sum in registers; kept for side-by-side measurement)
 * A (key 0, key 3) pair that an operator was not built with falls back to its default.
 * cx_set_tuning returns CX_ERR_SHAPE for an unknown key or value; a value of -1 restores
 * the default.
 */
int cx_copy_baseline(const float *src, float *dst, int64_t n, void *stream);
int cx_set_tuning(int32_t key, int32_t value);
int cx_get_tuning(int32_t key);

#ifdef __cplusplus
}
#endif
#endif /* CX_MIX_H */
