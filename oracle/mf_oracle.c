/*
 * mf_oracle.c -- plain, slow, single-threaded CPU reference for SGD matrix factorization.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  Only the tests, the smoke check and the
 * cpu_baseline leg of the benchmark may load it.  It shares no code, header, table or
 * helper with the HIP library; the two are written independently from the paper.
 *
 * What it follows (sections / equations / algorithms of the paper):
 *   - prediction  r_uv ~ p_u . q_v                          : Eq. 1
 *   - per-rating loss (r - p.q)^2 + lP |p|^2 + lQ |q|^2     : Eq. 3
 *   - per-rating step  e = r - p.q ; p += g(e q - l p) ; q += g(e p - l q)
 *                                                            : Algorithm 1 (training phase),
 *                                                              Eq. 4-6 up to the factor 2
 *   - block grid, independent / conflicting blocks          : Section 3.1 (FPSGD), Example 2
 *   - RMSE as the quality metric                            : Section 7 (experiment setup)
 *
 * Readings where the paper is silent (each also listed in the design notes):
 *   - both right-hand sides of the step use the values read BEFORE the step (the two
 *     gradients of Eq. 4-5 are taken at the same point);
 *   - Algorithm 1 governs the scale: step = -(gamma/2) * gradient of Eq. 3;
 *   - one lambda for P and Q; regularisation is applied per rating;
 *   - visiting order = the canonical order the block partition defines (below), the same
 *     every epoch; every rating exactly once per epoch;
 *   - indices are 0-based; Q is held transposed (Qt[v] is the paper's column q_v).
 *
 * Arithmetic: `arith` selects the number system of the factor state.
 *   MFO_ARITH_F64 : state, dot product and step all in double.  This is the definition.
 *   MFO_ARITH_F32 : state on the fp32 grid; dot in double rounded once to fp32; the
 *                   element-wise step in fp32, written as  x + ((g*e)*y - (g*lambda)*x)
 *                   with the inner multiply-subtract fused (fmaf) and every other operation
 *                   rounded separately.
 *   MFO_ARITH_F16 : as F32, then every stored value is rounded to IEEE binary16
 *                   (round-to-nearest-even) after every step ("stored fp16, updated in
 *                   fp32").  The rounding to binary16 is a decision taken from an fp32 value;
 *                   the grouping above is Algorithm 1's line regrouped so that this value is
 *                   defined operation by operation and does not depend on the order in which
 *                   the dot product is summed (the dot is exact to double precision).
 * The state arrays are always `double` so one interface serves the three.
 *
 * Parity pins live in tests/test_oracle_pins.py (worked example of the paper, finite
 * differences of Eq. 3, a hand-computed k=1 step, fixed points, noiseless planted data,
 * exactly-once counters, brute-force partition, numpy RMSE, numpy binary16 rounding).
 * The in-block visiting order, the stratum order, the split rules and the initialiser's
 * hash are conventions of this build with nothing in the paper to pin them to.
 *
 * Build: gcc -O2 -ffp-contract=off -fopenmp -shared -fPIC (see oracle/build.py).
 */
#include <math.h>
#ifdef _OPENMP
#include <omp.h>
#endif
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define MFO_ARITH_F64 0
#define MFO_ARITH_F32 1
#define MFO_ARITH_F16 2

#define MFO_SPLIT_EQUAL_WIDTH 0
#define MFO_SPLIT_NNZ_BALANCED 1
#define MFO_SPLIT_NNZ_WIDTH_BALANCED 2

/* ------------------------------------------------------------------------------------ */
/* binary16 rounding (round to nearest, ties to even), written from the IEEE-754 format: */
/* 1 sign, 5 exponent (bias 15), 10 fraction bits; subnormal step 2^-24; max 65504.      */
/* ------------------------------------------------------------------------------------ */
double mfo_round_f16(double x)
{
    if (x != x || x == 0.0 || isinf(x)) return x;
    double ax = fabs(x);
    int e;
    (void)frexp(ax, &e);          /* ax = f * 2^e, f in [0.5, 1)  => ax in [2^(e-1), 2^e) */
    int exp2 = e - 1;             /* exponent of the leading bit                         */
    if (exp2 < -14) exp2 = -14;   /* subnormal range shares the spacing of 2^-14         */
    double ulp = ldexp(1.0, exp2 - 10);
    double q = ax / ulp;          /* exact: division by a power of two                   */
    double r = nearbyint(q);      /* default rounding mode = ties to even                */
    double y = r * ulp;
    if (y > 65504.0) y = INFINITY;
    return x < 0 ? -y : y;
}

/* ------------------------------------------------------------------------------------ */
/* Initialiser ("init_model" of Algorithm 1; the paper only says "generated randomly"). */
/* Counter-based: value(i) = scale * U01(mix(seed, stream, i)) with U01 = top 24 bits.   */
/* The mixer is the published SplitMix64 output function.  Both sides of the parity test  */
/* implement this same generator on their own.                                           */
/* ------------------------------------------------------------------------------------ */
static uint64_t mix64(uint64_t z)
{
    z += 0x9E3779B97F4A7C15ULL;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ULL;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBULL;
    return z ^ (z >> 31);
}

void mfo_init_factors(double* x, int64_t count, uint64_t seed, uint64_t stream, float scale, int arith)
{
    uint64_t key = mix64(seed ^ (stream * 0xD1B54A32D192ED03ULL));
    for (int64_t i = 0; i < count; ++i) {
        uint64_t h = mix64(key + (uint64_t)i);
        float u01 = (float)(h >> 40) * (1.0f / 16777216.0f);   /* exact: 24 bits * 2^-24 */
        float val = u01 * scale;                                /* one fp32 rounding      */
        x[i] = (arith == MFO_ARITH_F16) ? mfo_round_f16((double)val) : (double)val;
    }
}

/* ------------------------------------------------------------------------------------ */
/* Partition: grid of G_r x G_c blocks (Section 3.1: R is divided into blocks; blocks     */
/* that share neither a row nor a column range are independent).                          */
/* ------------------------------------------------------------------------------------ */

/* bounds[a] = ceil(a*size/G): the uniform division. */
void mfo_bounds_equal_width(int64_t size, int32_t G, int32_t* bounds)
{
    for (int32_t a = 0; a <= G; ++a) {
        int64_t num = (int64_t)a * size;
        bounds[a] = (int32_t)((num + G - 1) / G);
    }
}

/* bounds[a] = smallest id x whose exclusive degree prefix S[x] >= ceil(a*nnz/G);
 * bounds[0]=0, bounds[G]=size.  Splits the axis so each strip holds about nnz/G ratings. */
int mfo_bounds_nnz_balanced(const int32_t* idx, int64_t nnz, int64_t size, int32_t G, int32_t* bounds)
{
    int64_t* S = (int64_t*)calloc((size_t)size + 1, sizeof(int64_t));
    if (!S) return -3;
    for (int64_t t = 0; t < nnz; ++t) S[idx[t] + 1] += 1;
    for (int64_t x = 0; x < size; ++x) S[x + 1] += S[x];      /* S[x] = #ratings with id < x */
    bounds[0] = 0;
    int64_t x = 0;                       /* targets grow with a, so the scan never restarts */
    for (int32_t a = 1; a < G; ++a) {
        int64_t target = ((int64_t)a * nnz + G - 1) / G;
        while (x < size && S[x] < target) ++x;
        bounds[a] = (int32_t)x;
    }
    bounds[G] = (int32_t)size;
    free(S);
    return 0;
}

/* Every id x carries the weight deg(x)*size + nnz (its share of the ratings plus its share of
 * the axis, both scaled to the common denominator nnz*size); with the exclusive prefix
 * W[x] = S[x]*size + x*nnz (W[size] = 2*nnz*size), bounds[a] = smallest x with
 * W[x] >= ceil(a*W[size]/G).  A strip then holds at most about twice its fair share of the
 * ratings AND spans at most about twice its fair share of the ids.  nnz = 0 counts as 1. */
int mfo_bounds_nnz_width_balanced(const int32_t* idx, int64_t nnz, int64_t size, int32_t G, int32_t* bounds)
{
    int64_t* S = (int64_t*)calloc((size_t)size + 1, sizeof(int64_t));
    if (!S) return -3;
    for (int64_t t = 0; t < nnz; ++t) S[idx[t] + 1] += 1;
    for (int64_t x = 0; x < size; ++x) S[x + 1] += S[x];
    int64_t unit = nnz > 0 ? nnz : 1;
    int64_t total = S[size] * size + size * unit;
    bounds[0] = 0;
    int64_t x = 0;
    for (int32_t a = 1; a < G; ++a) {
        int64_t target = (int64_t)(((__int128)a * total + G - 1) / G);
        while (x < size && S[x] * size + x * unit < target) ++x;
        bounds[a] = (int32_t)x;
    }
    bounds[G] = (int32_t)size;
    free(S);
    return 0;
}

static int32_t strip_of(const int32_t* bounds, int32_t G, int32_t id)
{
    /* the strip a with bounds[a] <= id < bounds[a+1] = the largest a in [0,G) with
     * bounds[a] <= id (bounds is non-decreasing, bounds[0] = 0; empty strips are skipped) */
    int32_t lo = 0, hi = G - 1;
    while (lo < hi) {
        int32_t mid = lo + (hi - lo + 1) / 2;
        if (bounds[mid] <= id) lo = mid; else hi = mid - 1;
    }
    return lo;
}

/* Two blocks (a1,b1), (a2,b2) are independent iff they share neither the row strip nor
 * the column strip (Section 3.1 and Example 2). */
int mfo_blocks_independent(int32_t a1, int32_t b1, int32_t a2, int32_t b2)
{
    return (a1 != a2) && (b1 != b2);
}

typedef struct {
    int64_t L;       /* linear block id = stratum * G_r + a */
    int64_t rank;    /* place of the row inside its strip (the row index itself for row_seed 0) */
    int32_t v;
    int64_t t;       /* original position: total order even for duplicate (u,v) */
} sort_key;

static int cmp_key(const void* pa, const void* pb)
{
    const sort_key* x = (const sort_key*)pa;
    const sort_key* y = (const sort_key*)pb;
    if (x->L != y->L) return x->L < y->L ? -1 : 1;
    if (x->rank != y->rank) return x->rank < y->rank ? -1 : 1;
    if (x->v != y->v) return x->v < y->v ? -1 : 1;
    if (x->t != y->t) return x->t < y->t ? -1 : 1;
    return 0;
}

static uint64_t mix64(uint64_t z);

/* Randomised order of the rows inside a block (the paper's scheduler visits "randomly"; it fixes
 * no generator).  Convention of this build: the rows of row strip a (first row `first`, `width`
 * rows) are visited in the order of ((u - first) * 2147483647 + offset_a) mod width with
 * offset_a = mix64(row_seed + a) mod width -- an affine map with a prime multiplier larger than
 * any width, hence a permutation of the strip's rows.  row_seed = 0 keeps ascending row order.
 * All ratings of one row stay together, ordered by column and original position. */
int64_t mfo_row_rank(int32_t u, int32_t first, int32_t width, uint64_t row_seed, int32_t a)
{
    if (row_seed == 0) return (int64_t)u;
    uint64_t offset = mix64(row_seed + (uint64_t)a) % (uint64_t)width;
    return (int64_t)((((uint64_t)(u - first)) * 2147483647ULL + offset) % (uint64_t)width);
}

/* Stratum of block (a,b): s = (b - a) mod G_c.  For fixed s the G_r blocks (a, (a+s) mod G_c)
 * have pairwise different a and (because G_r <= G_c) pairwise different b: they are mutually
 * independent.  Linear id L = s*G_r + a.  perm lists the original positions in ascending
 * (L, u, v, t); block_ptr[L] is where block L starts in perm. */
int mfo_partition_seeded(const int32_t* rows, const int32_t* cols, int64_t nnz, int64_t m, int64_t n,
                         int32_t G_r, int32_t G_c, int32_t split, uint64_t row_seed,
                         int64_t* perm, int64_t* block_ptr, int32_t* row_bounds, int32_t* col_bounds);

int mfo_partition(const int32_t* rows, const int32_t* cols, int64_t nnz, int64_t m, int64_t n,
                  int32_t G_r, int32_t G_c, int32_t split,
                  int64_t* perm, int64_t* block_ptr, int32_t* row_bounds, int32_t* col_bounds)
{
    return mfo_partition_seeded(rows, cols, nnz, m, n, G_r, G_c, split, 0, perm, block_ptr, row_bounds, col_bounds);
}

/* The same with the rows of every block in the order of mfo_row_rank (row_seed 0: ascending). */
int mfo_partition_seeded(const int32_t* rows, const int32_t* cols, int64_t nnz, int64_t m, int64_t n,
                         int32_t G_r, int32_t G_c, int32_t split, uint64_t row_seed,
                         int64_t* perm, int64_t* block_ptr, int32_t* row_bounds, int32_t* col_bounds)
{
    if (G_r < 1 || G_c < G_r || G_r > m || G_c > n) return -1;
    for (int64_t t = 0; t < nnz; ++t)
        if (rows[t] < 0 || rows[t] >= m || cols[t] < 0 || cols[t] >= n) return -5;
    if (split == MFO_SPLIT_EQUAL_WIDTH) {
        mfo_bounds_equal_width(m, G_r, row_bounds);
        mfo_bounds_equal_width(n, G_c, col_bounds);
    } else if (split == MFO_SPLIT_NNZ_BALANCED) {
        if (mfo_bounds_nnz_balanced(rows, nnz, m, G_r, row_bounds)) return -3;
        if (mfo_bounds_nnz_balanced(cols, nnz, n, G_c, col_bounds)) return -3;
    } else if (split == MFO_SPLIT_NNZ_WIDTH_BALANCED) {
        if (mfo_bounds_nnz_width_balanced(rows, nnz, m, G_r, row_bounds)) return -3;
        if (mfo_bounds_nnz_width_balanced(cols, nnz, n, G_c, col_bounds)) return -3;
    } else return -1;

    sort_key* keys = (sort_key*)malloc((size_t)(nnz > 0 ? nnz : 1) * sizeof(sort_key));
    if (!keys) return -3;
    for (int64_t t = 0; t < nnz; ++t) {
        int32_t a = strip_of(row_bounds, G_r, rows[t]);
        int32_t b = strip_of(col_bounds, G_c, cols[t]);
        int32_t s = (b - a) % G_c;
        if (s < 0) s += G_c;
        keys[t].L = (int64_t)s * G_r + a;
        keys[t].rank = mfo_row_rank(rows[t], row_bounds[a], row_bounds[a + 1] - row_bounds[a], row_seed, a);
        keys[t].v = cols[t];
        keys[t].t = t;
    }
    qsort(keys, (size_t)nnz, sizeof(sort_key), cmp_key);
    int64_t nblocks = (int64_t)G_r * G_c;
    for (int64_t L = 0; L <= nblocks; ++L) block_ptr[L] = 0;
    for (int64_t pos = 0; pos < nnz; ++pos) {
        perm[pos] = keys[pos].t;
        block_ptr[keys[pos].L + 1] += 1;
    }
    for (int64_t L = 0; L < nblocks; ++L) block_ptr[L + 1] += block_ptr[L];
    free(keys);
    return 0;
}

/* ------------------------------------------------------------------------------------ */
/* One SGD step on one rating (Algorithm 1, body of the inner loop).                     */
/* ------------------------------------------------------------------------------------ */
static void step_f64(double* p, double* q, int32_t k, double r, double g, double lam)
{
    double dot = 0.0;
    for (int32_t f = 0; f < k; ++f) dot += p[f] * q[f];
    double e = r - dot;
    for (int32_t f = 0; f < k; ++f) {
        double pf = p[f], qf = q[f];                 /* both sides use the old values */
        p[f] = pf + g * (e * qf - lam * pf);
        q[f] = qf + g * (e * pf - lam * qf);
    }
}

static void step_f32(double* p, double* q, int32_t k, float r, float g, float lam, int to_f16)
{
    double dot = 0.0;
    for (int32_t f = 0; f < k; ++f) dot += p[f] * q[f];   /* state is on the fp32 grid   */
    float e = r - (float)dot;
    float step = g * e;                                    /* gamma * e                   */
    float shrink = g * lam;                                /* gamma * lambda              */
    for (int32_t f = 0; f < k; ++f) {
        float pf = (float)p[f], qf = (float)q[f];
        float sp = shrink * pf, sq = shrink * qf;          /* -ffp-contract=off: only the */
        float pn = pf + fmaf(step, qf, -sp);               /* explicit fmaf is fused      */
        float qn = qf + fmaf(step, pf, -sq);
        p[f] = to_f16 ? mfo_round_f16((double)pn) : (double)pn;
        q[f] = to_f16 ? mfo_round_f16((double)qn) : (double)qn;
    }
}

void mfo_sgd_step(double* p, double* q, int32_t k, float r, float lr, float lambda, int arith)
{
    if (arith == MFO_ARITH_F64) step_f64(p, q, k, (double)r, (double)lr, (double)lambda);
    else step_f32(p, q, k, r, lr, lambda, arith == MFO_ARITH_F16);
}

static void run_block(double* P, double* Qt, int32_t k, const int32_t* rows, const int32_t* cols,
                      const float* vals, const int64_t* perm, int64_t begin, int64_t end,
                      float lr, float lambda, int arith, int32_t* visits)
{
    for (int64_t pos = begin; pos < end; ++pos) {
        int64_t t = perm[pos];
        mfo_sgd_step(P + (int64_t)rows[t] * k, Qt + (int64_t)cols[t] * k, k, vals[t], lr, lambda, arith);
        if (visits) visits[t] += 1;
    }
}

/* One epoch in the canonical order: strata 0..G_c-1; inside a stratum blocks a=0..G_r-1;
 * inside a block the stored (row-major) order.  `block_order`, if given, holds for every
 * stratum a permutation of 0..G_r-1 (G_c*G_r entries) and replaces the a=0..G_r-1 order:
 * because the blocks of a stratum are independent the result must not change by one bit. */
int mfo_sgd_epoch(double* P, double* Qt, int32_t k, const int32_t* rows, const int32_t* cols,
                  const float* vals, const int64_t* perm, const int64_t* block_ptr,
                  int32_t G_r, int32_t G_c, float lr, float lambda, int arith,
                  const int32_t* block_order, int32_t* visits)
{
    if (arith < 0 || arith > 2 || k < 1) return -1;
    for (int32_t s = 0; s < G_c; ++s)
        for (int32_t i = 0; i < G_r; ++i) {
            int32_t a = block_order ? block_order[(int64_t)s * G_r + i] : i;
            int64_t L = (int64_t)s * G_r + a;
            run_block(P, Qt, k, rows, cols, vals, perm, block_ptr[L], block_ptr[L + 1], lr, lambda, arith, visits);
        }
    return 0;
}

/* The same epoch with the independent blocks of each stratum run by OpenMP threads.  The
 * result is bit-identical to mfo_sgd_epoch (tested); it exists only so that multi-epoch
 * runs on the large configurations finish in reasonable time. */
int mfo_sgd_epoch_omp(double* P, double* Qt, int32_t k, const int32_t* rows, const int32_t* cols,
                      const float* vals, const int64_t* perm, const int64_t* block_ptr,
                      int32_t G_r, int32_t G_c, float lr, float lambda, int arith)
{
    if (arith < 0 || arith > 2 || k < 1) return -1;
    for (int32_t s = 0; s < G_c; ++s) {
#pragma omp parallel for schedule(dynamic, 1)
        for (int32_t a = 0; a < G_r; ++a) {
            int64_t L = (int64_t)s * G_r + a;
            run_block(P, Qt, k, rows, cols, vals, perm, block_ptr[L], block_ptr[L + 1], lr, lambda, arith, 0);
        }
    }
    return 0;
}

/* Randomised visiting order (the paper's scheduler hands out blocks "randomly", Section 3.1
 * and Example 3; it fixes no generator).  Convention of this build: per epoch a permutation
 * of the strata, still exactly once per epoch and still deterministic -- stratum s gets the key
 * mix64(mix64(seed ^ epoch * 0xD1B54A32D192ED03) + s) and the strata are visited in ascending
 * (key, s).  order[t] = stratum visited at step t. */
uint64_t mfo_mix64(uint64_t z) { return mix64(z); }

void mfo_stratum_order(uint64_t seed, uint64_t epoch, int32_t G_c, int32_t* order)
{
    uint64_t base = mix64(seed ^ (epoch * 0xD1B54A32D192ED03ULL));
    uint64_t* key = (uint64_t*)malloc((size_t)G_c * sizeof(uint64_t));
    for (int32_t s = 0; s < G_c; ++s) key[s] = mix64(base + (uint64_t)s);
    /* selection by repeated minimum: quadratic, obviously a sort by (key, s) */
    char* used = (char*)calloc((size_t)G_c, 1);
    for (int32_t t = 0; t < G_c; ++t) {
        int32_t best = -1;
        for (int32_t s = 0; s < G_c; ++s)
            if (!used[s] && (best < 0 || key[s] < key[best])) best = s;   /* ties: the smaller s stays */
        used[best] = 1;
        order[t] = best;
    }
    free(used);
    free(key);
}

/* One epoch with the strata visited in the given order (a permutation of 0..G_c-1); inside a
 * stratum and inside a block as mfo_sgd_epoch.  parallel != 0 runs the independent blocks of a
 * stratum on OpenMP threads (bit-identical, as for mfo_sgd_epoch_omp). */
int mfo_sgd_epoch_ordered(double* P, double* Qt, int32_t k, const int32_t* rows, const int32_t* cols,
                          const float* vals, const int64_t* perm, const int64_t* block_ptr,
                          int32_t G_r, int32_t G_c, float lr, float lambda, int arith,
                          const int32_t* stratum_order, int parallel, int32_t* visits)
{
    if (arith < 0 || arith > 2 || k < 1 || !stratum_order) return -1;
    for (int32_t t = 0; t < G_c; ++t) {
        int32_t s = stratum_order[t];
        if (s < 0 || s >= G_c) return -2;
        if (parallel && !visits) {
#pragma omp parallel for schedule(dynamic, 1)
            for (int32_t a = 0; a < G_r; ++a) {
                int64_t L = (int64_t)s * G_r + a;
                run_block(P, Qt, k, rows, cols, vals, perm, block_ptr[L], block_ptr[L + 1], lr, lambda, arith, 0);
            }
        } else {
            for (int32_t a = 0; a < G_r; ++a) {
                int64_t L = (int64_t)s * G_r + a;
                run_block(P, Qt, k, rows, cols, vals, perm, block_ptr[L], block_ptr[L + 1], lr, lambda, arith, visits);
            }
        }
    }
    return 0;
}

/* Plain Algorithm 1 over the ratings in the order given (no grid): used by pins. */
void mfo_sgd_sweep(double* P, double* Qt, int32_t k, const int32_t* rows, const int32_t* cols,
                   const float* vals, int64_t nnz, float lr, float lambda, int arith)
{
    for (int64_t t = 0; t < nnz; ++t)
        mfo_sgd_step(P + (int64_t)rows[t] * k, Qt + (int64_t)cols[t] * k, k, vals[t], lr, lambda, arith);
}

/* Prediction of one entry (Eq. 1). */
double mfo_predict(const double* P, const double* Qt, int32_t k, int64_t u, int64_t v)
{
    double dot = 0.0;
    for (int32_t f = 0; f < k; ++f) dot += P[u * k + f] * Qt[v * k + f];
    return dot;
}

/* Per-rating loss of Eq. 3. */
double mfo_rating_loss(const double* p, const double* q, int32_t k, double r, double lamP, double lamQ)
{
    double dot = 0.0, pp = 0.0, qq = 0.0;
    for (int32_t f = 0; f < k; ++f) { dot += p[f] * q[f]; pp += p[f] * p[f]; qq += q[f] * q[f]; }
    return (r - dot) * (r - dot) + lamP * pp + lamQ * qq;
}

/* RMSE = sqrt( mean_t (r_t - p_u.q_v)^2 ), double throughout, no clipping. */
double mfo_rmse(const double* P, const double* Qt, int32_t k, const int32_t* rows, const int32_t* cols,
                const float* vals, int64_t count)
{
    double acc = 0.0;
    for (int64_t t = 0; t < count; ++t) {
        double d = (double)vals[t] - mfo_predict(P, Qt, k, rows[t], cols[t]);
        acc += d * d;
    }
    return sqrt(acc / (double)count);
}

int mfo_num_threads(void)
{
    int n = 1;
#ifdef _OPENMP
#pragma omp parallel
    {
#pragma omp master
        n = omp_get_num_threads();
    }
#endif
    return n;
}
