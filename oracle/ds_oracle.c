/*
 * DS-Sync reference oracle (plain C, fp64 arithmetic) -- TEST INFRASTRUCTURE ONLY.
 *
 * This file is the slow, obviously-correct CPU statement of what one DS-Sync
 * synchronisation step computes.  It exists to check the GPU library and to
 * be timed as a reported CPU baseline.  Only the test-suite, the smoke check
 * and the benchmark's cpu_baseline leg may call it.  It shares no code,
 * header, table or helper with the GPU library.
 *
 * What is implemented, and where the paper defines it:
 *   orc_partition  -- the per-iteration division of the N workers into
 *                     non-overlapping groups (Listing 1, the lookup of worker
 *                     i's group for iteration t; Sec. IV-B2, W_k = disjoint fully
 *                     connected sub-graphs covering all nodes).  The paper's own
 *                     list is topology derived; here the list entry for
 *                     iteration t is drawn by a counter-based shuffle whose
 *                     specification is restated below.
 *   orc_step       -- Listing 1, optimizer.step() followed by
 *                     DS_Sync.Average(model, group); Sec. III-A step 4
 *                     (parameters are averaged inside the group AFTER the local
 *                     update); Sec. IV-B2, X_{k+1} = W_k X_k with
 *                     w_ij = 1/|group| inside a group and 0 elsewhere.
 *   orc_consensus  -- the left-hand quantity of Lemma 1 (Sec. IV-B2), per
 *                     worker and un-squared: || x_i - mean_j x_j ||_2.
 *
 * Pins (see tests, "not gpu"): dense mixing-matrix products (Sec. IV-B2), the
 * closed-form trajectory of Sec. III-A step 4, group size N == single-machine
 * SGD on the mean gradient (Sec. I), group size 1 == independent SGD, mean
 * preservation by a doubly stochastic W_k, Lemma 1's bound, published
 * splitmix64 outputs and golden permutations.  No function here is unpinned.
 *
 * Precision: every replica element is stored as fp32 (the replica dtype);
 * all arithmetic inside a step is fp64 with a single final rounding to fp32.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* number of host threads the column loops below run on */
int orc_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ------------------------------------------------------------------------- */
/* Partition: counter-based shuffle.  All arithmetic is modulo 2^64.         */
/*   gamma = 0x9E3779B97F4A7C15                                              */
/*   mix(z): z ^= z>>30; z *= 0xBF58476D1CE4E5B9; z ^= z>>27;                */
/*           z *= 0x94D049BB133111EB; z ^= z>>31   (splitmix64 finaliser)    */
/*   key(seed,t) = mix( mix(seed) + (t+1)*gamma )   -- nothing carried over  */
/*   draw: s += gamma; r = mix(s)                                            */
/*   perm = identity; for i = W-1 down to 1: j = floor(r*(i+1) / 2^64);      */
/*          swap perm[i], perm[j]                                            */
/*   group k = perm[off[k]] .. perm[off[k+1]-1], off = prefix sums of sizes  */
/* ------------------------------------------------------------------------- */

uint64_t orc_mix64(uint64_t z)
{
    z ^= z >> 30;
    z *= 0xBF58476D1CE4E5B9ULL;
    z ^= z >> 27;
    z *= 0x94D049BB133111EBULL;
    z ^= z >> 31;
    return z;
}

uint64_t orc_key(uint64_t seed, uint64_t t)
{
    const uint64_t gamma = 0x9E3779B97F4A7C15ULL;
    return orc_mix64(orc_mix64(seed) + (t + 1) * gamma);
}

/* returns 0, or -1 when the sizes are not a division of W workers */
int orc_partition(uint64_t seed, uint64_t t, int32_t W, const int32_t *sizes,
                  int32_t n_groups, int32_t *perm, int32_t *off)
{
    const uint64_t gamma = 0x9E3779B97F4A7C15ULL;
    if (W < 1 || n_groups < 1) return -1;
    int64_t total = 0;
    for (int32_t k = 0; k < n_groups; ++k) {
        if (sizes[k] < 1) return -1;
        total += sizes[k];
    }
    if (total != W) return -1;

    uint64_t s = orc_key(seed, t);
    for (int32_t i = 0; i < W; ++i) perm[i] = i;
    for (int32_t i = W - 1; i >= 1; --i) {
        s += gamma;
        uint64_t r = orc_mix64(s);
        unsigned __int128 wide = (unsigned __int128)r * (unsigned __int128)(uint64_t)(i + 1);
        int32_t j = (int32_t)(uint64_t)(wide >> 64);
        int32_t tmp = perm[i];
        perm[i] = perm[j];
        perm[j] = tmp;
    }
    off[0] = 0;
    for (int32_t k = 0; k < n_groups; ++k) off[k + 1] = off[k] + sizes[k];
    return 0;
}

/* ------------------------------------------------------------------------- */
/* One synchronisation step.                                                 */
/* ------------------------------------------------------------------------- */

/* bf16 -> fp64 is exact: the 16 bits are the top half of an fp32 pattern */
static double bf16_bits_to_double(uint16_t b)
{
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

static int cmp_i32(const void *a, const void *b)
{
    int32_t x = *(const int32_t *)a, y = *(const int32_t *)b;
    return (x > y) - (x < y);
}

/*
 * X  [W, ldx] fp32, in/out.   G [W, ldg], fp32 (g_is_bf16 == 0) or raw bf16
 * bits (g_is_bf16 == 1).  Columns col0 .. col0+ncols-1 of every row are
 * processed; other columns are untouched.
 *
 * For every group k and column p (Listing 1; Sec. IV-B2):
 *     y_i   = X[i,p] - lr * G[i,p]                (the worker's local update)
 *     m     = (1/|g_k|) * sum_{i in g_k} y_i      (members in ascending index)
 *     X[i,p] = (float) m   for every i in g_k
 */
int orc_step(float *X, const void *G, int g_is_bf16, int64_t col0, int64_t ncols,
             int64_t ldx, int64_t ldg, int32_t W, const int32_t *perm,
             const int32_t *off, int32_t n_groups, float lr)
{
    const double lrd = (double)lr;
    const float *Gf = (const float *)G;
    const uint16_t *Gh = (const uint16_t *)G;
    int32_t *members = (int32_t *)malloc(sizeof(int32_t) * (size_t)W);
    if (!members) return -2;

    for (int32_t k = 0; k < n_groups; ++k) {
        const int32_t n = off[k + 1] - off[k];
        for (int32_t q = 0; q < n; ++q) members[q] = perm[off[k] + q];
        qsort(members, (size_t)n, sizeof(int32_t), cmp_i32);

#pragma omp parallel for schedule(static)
        for (int64_t p = col0; p < col0 + ncols; ++p) {
            double acc = 0.0;
            for (int32_t q = 0; q < n; ++q) {
                const int64_t i = members[q];
                const double x = (double)X[i * ldx + p];
                const double g = g_is_bf16 ? bf16_bits_to_double(Gh[i * ldg + p])
                                           : (double)Gf[i * ldg + p];
                acc += x - lrd * g;
            }
            const float m = (float)(acc / (double)n);
            for (int32_t q = 0; q < n; ++q) X[(int64_t)members[q] * ldx + p] = m;
        }
    }
    free(members);
    return 0;
}

/* ------------------------------------------------------------------------- */
/* One step with the fuller local optimizer and the SWA ensemble of           */
/* Listing 1.  Sec. V-A3 keeps the hyper-parameters of the original model     */
/* papers (SGD with momentum and weight decay for the WideResNets); Listing 1 */
/* hands only the model to Average(), so the momentum buffer stays local.     */
/* For every worker i and column p:                                           */
/*     d   = g + weight_decay * x                                             */
/*     v'  = momentum * v + d            (V absent: v' = d)                    */
/*     y_i = x - lr * v'                                                       */
/* then the group mean m of the y_i replaces x for every member, and          */
/*     s'  = factor * s + (1 - factor) * m      (Listing 1: SWA_model update)  */
/* V and S are fp32 state, one row per worker, and may each be NULL.          */
/* ------------------------------------------------------------------------- */
int orc_step_opt(float *X, const void *G, int g_is_bf16, float *V, float *S, int64_t col0, int64_t ncols,
                 int64_t ldx, int64_t ldg, int64_t ldv, int64_t lds, int32_t W, const int32_t *perm,
                 const int32_t *off, int32_t n_groups, float lr, float momentum, float weight_decay,
                 float factor)
{
    const double lrd = (double)lr, mud = (double)momentum, wdd = (double)weight_decay, fd = (double)factor;
    const float *Gf = (const float *)G;
    const uint16_t *Gh = (const uint16_t *)G;
    int32_t *members = (int32_t *)malloc(sizeof(int32_t) * (size_t)W);
    if (!members) return -2;

    for (int32_t k = 0; k < n_groups; ++k) {
        const int32_t n = off[k + 1] - off[k];
        for (int32_t q = 0; q < n; ++q) members[q] = perm[off[k] + q];
        qsort(members, (size_t)n, sizeof(int32_t), cmp_i32);

#pragma omp parallel for schedule(static)
        for (int64_t p = col0; p < col0 + ncols; ++p) {
            double acc = 0.0;
            for (int32_t q = 0; q < n; ++q) {
                const int64_t i = members[q];
                const double x = (double)X[i * ldx + p];
                const double g = g_is_bf16 ? bf16_bits_to_double(Gh[i * ldg + p])
                                           : (double)Gf[i * ldg + p];
                const double d = g + wdd * x;
                double v = d;
                if (V) {
                    v = mud * (double)V[i * ldv + p] + d;
                    V[i * ldv + p] = (float)v;
                }
                acc += x - lrd * v;
            }
            const float m = (float)(acc / (double)n);
            for (int32_t q = 0; q < n; ++q) {
                const int64_t i = members[q];
                X[i * ldx + p] = m;
                if (S) S[i * lds + p] = (float)(fd * (double)S[i * lds + p] + (1.0 - fd) * (double)m);
            }
        }
    }
    free(members);
    return 0;
}

/* ------------------------------------------------------------------------- */
/* Consensus deviation (Lemma 1's left side, un-squared, per worker):        */
/*     xbar[p] = (1/W) sum_i X[i,p];  d_i = sqrt( sum_p (X[i,p]-xbar[p])^2 ) */
/* ------------------------------------------------------------------------- */
int orc_consensus(const float *X, int64_t P, int64_t ld, int32_t W, double *d_out)
{
    double *xbar = (double *)malloc(sizeof(double) * (size_t)(P > 0 ? P : 1));
    if (!xbar) return -2;

#pragma omp parallel for schedule(static)
    for (int64_t p = 0; p < P; ++p) {
        double s = 0.0;
        for (int32_t i = 0; i < W; ++i) s += (double)X[(int64_t)i * ld + p];
        xbar[p] = s / (double)W;
    }
    /* one worker per loop trip: each d_i is one sequential fp64 sum over p */
#pragma omp parallel for schedule(dynamic, 1)
    for (int32_t i = 0; i < W; ++i) {
        double s = 0.0;
        for (int64_t p = 0; p < P; ++p) {
            const double e = (double)X[(int64_t)i * ld + p] - xbar[p];
            s += e * e;
        }
        d_out[i] = sqrt(s);
    }
    free(xbar);
    return 0;
}

/* ------------------------------------------------------------------------- */
/* Yardstick of the parity tests (not a step of the method): the largest      */
/*     |got - want| / max(|want|, rms of want's row)                          */
/* over columns col0 .. col0+ncols-1 of two fp32 [W, ld] blocks, the rms taken */
/* over those same columns.  The denominator keeps "relative error" meaningful */
/* for parameters near zero.  A NaN anywhere makes the result NaN.             */
/* ------------------------------------------------------------------------- */
double orc_scaled_error(const float *got, const float *want, int64_t col0, int64_t ncols,
                        int64_t ld_got, int64_t ld_want, int32_t W)
{
    double worst = 0.0;
    int bad = 0;
    for (int32_t i = 0; i < W; ++i) {
        const float *g = got + (int64_t)i * ld_got + col0;
        const float *w = want + (int64_t)i * ld_want + col0;
        double sq = 0.0;
#pragma omp parallel for schedule(static) reduction(+ : sq)
        for (int64_t p = 0; p < ncols; ++p) sq += (double)w[p] * (double)w[p];
        double rms = ncols > 0 ? sqrt(sq / (double)ncols) : 0.0;
        if (rms < 1e-30) rms = 1e-30;
        double row_worst = 0.0;
#pragma omp parallel for schedule(static) reduction(max : row_worst) reduction(| : bad)
        for (int64_t p = 0; p < ncols; ++p) {
            const double a = (double)g[p], b = (double)w[p];
            const double den = fabs(b) > rms ? fabs(b) : rms;
            const double e = fabs(a - b) / den;
            if (e != e) bad |= 1;
            if (e > row_worst) row_worst = e;
        }
        if (row_worst > worst) worst = row_worst;
    }
    return bad ? NAN : worst;
}

/* Number of host threads the column loops use from now on (the benchmark's
 * single-thread leg sets 1 and restores the previous value). */
void orc_set_num_threads(int n)
{
#ifdef _OPENMP
    if (n >= 1) omp_set_num_threads(n);
#else
    (void)n;
#endif
}
