/* Drives the CPU oracle (oracle/ds_oracle.c) with random shapes, windows and
 * pitches under AddressSanitizer and UndefinedBehaviorSanitizer.  Every buffer
 * is allocated at exactly the size the call may touch, so an access one
 * element too far is an error.  Prints "ok <cases>" on success. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

uint64_t orc_key(uint64_t seed, uint64_t t);
int orc_partition(uint64_t seed, uint64_t t, int32_t W, const int32_t *sizes, int32_t n_groups, int32_t *perm,
                  int32_t *off);
int orc_step(float *X, const void *G, int g_is_bf16, int64_t col0, int64_t ncols, int64_t ldx, int64_t ldg, int32_t W,
             const int32_t *perm, const int32_t *off, int32_t n_groups, float lr);
int orc_step_opt(float *X, const void *G, int g_is_bf16, float *V, float *S, int64_t col0, int64_t ncols, int64_t ldx,
                 int64_t ldg, int64_t ldv, int64_t lds, int32_t W, const int32_t *perm, const int32_t *off,
                 int32_t n_groups, float lr, float momentum, float weight_decay, float factor);
int orc_consensus(const float *X, int64_t P, int64_t ld, int32_t W, double *d_out);
double orc_scaled_error(const float *got, const float *want, int64_t col0, int64_t ncols, int64_t ld_got,
                        int64_t ld_want, int32_t W);
void orc_set_num_threads(int n);

static uint64_t state = 0x1234567ULL;
static uint64_t rnd(void) { state = state * 6364136223846793005ULL + 1442695040888963407ULL; return state >> 33; }
static int64_t between(int64_t lo, int64_t hi) { return lo + (int64_t)(rnd() % (uint64_t)(hi - lo + 1)); }
static float small(void) { return (float)((double)(rnd() % 2001) / 1000.0 - 1.0); }

/* a stack of W rows whose last row ends right after the window: rows * ld would be too generous */
static size_t stack_elems(int32_t W, int64_t ld, int64_t col0, int64_t ncols) {
    const int64_t n = (int64_t)(W - 1) * ld + col0 + ncols;
    return n > 0 ? (size_t)n : 1;
}

int main(void) {
    int cases = 0;
    for (int it = 0; it < 400; ++it) {
        const int32_t W = (int32_t)between(1, 64);
        int32_t sizes[64], n_groups = 0, left = W;
        while (left > 0) { int32_t s = (int32_t)between(1, left); sizes[n_groups++] = s; left -= s; }
        int32_t *perm = malloc(sizeof(int32_t) * (size_t)W), *off = malloc(sizeof(int32_t) * (size_t)(n_groups + 1));
        if (orc_partition(rnd(), rnd(), W, sizes, n_groups, perm, off) != 0) { printf("partition failed\n"); return 1; }
        char seen[64]; memset(seen, 0, sizeof seen);
        for (int32_t i = 0; i < W; ++i) { if (perm[i] < 0 || perm[i] >= W || seen[perm[i]]) { printf("not a permutation\n"); return 1; } seen[perm[i]] = 1; }
        if (off[0] != 0 || off[n_groups] != W) { printf("offsets\n"); return 1; }
        /* arguments the oracle must refuse without touching anything */
        if (orc_partition(1, 1, 0, sizes, n_groups, perm, off) == 0) { printf("W = 0 accepted\n"); return 1; }

        const int64_t col0 = between(0, 40), ncols = between(0, 300);
        const int64_t ldx = col0 + ncols + between(0, 9), ldg = col0 + ncols + between(0, 9);
        const int64_t ldv = col0 + ncols + between(0, 9), lds = col0 + ncols + between(0, 9);
        const int bf16 = (int)(rnd() & 1);
        orc_set_num_threads((int)between(1, 4));
        float *X = malloc(sizeof(float) * stack_elems(W, ldx, col0, ncols));
        float *V = malloc(sizeof(float) * stack_elems(W, ldv, col0, ncols));
        float *S = malloc(sizeof(float) * stack_elems(W, lds, col0, ncols));
        void *G = malloc((bf16 ? 2 : 4) * stack_elems(W, ldg, col0, ncols));
        for (size_t i = 0; i < stack_elems(W, ldx, col0, ncols); ++i) X[i] = small();
        for (size_t i = 0; i < stack_elems(W, ldv, col0, ncols); ++i) V[i] = small();
        for (size_t i = 0; i < stack_elems(W, lds, col0, ncols); ++i) S[i] = small();
        for (size_t i = 0; i < stack_elems(W, ldg, col0, ncols); ++i) {
            if (bf16) ((uint16_t *)G)[i] = (uint16_t)(0x3c00 + rnd() % 0x400); else ((float *)G)[i] = small();
        }
        if (orc_step(X, G, bf16, col0, ncols, ldx, ldg, W, perm, off, n_groups, 0.01f) != 0) { printf("step failed\n"); return 1; }
        const int use_v = (int)(rnd() & 1), use_s = (int)(rnd() & 1);
        if (orc_step_opt(X, G, bf16, use_v ? V : NULL, use_s ? S : NULL, col0, ncols, ldx, ldg, ldv, lds, W, perm, off,
                         n_groups, 0.01f, 0.9f, 1e-3f, 0.8f) != 0) { printf("step_opt failed\n"); return 1; }
        /* members of a group hold the same values afterwards */
        for (int32_t k = 0; k < n_groups; ++k)
            for (int32_t q = off[k] + 1; q < off[k + 1]; ++q)
                for (int64_t c = col0; c < col0 + ncols; ++c)
                    if (X[(int64_t)perm[q] * ldx + c] != X[(int64_t)perm[off[k]] * ldx + c]) { printf("members differ\n"); return 1; }
        /* consensus and the parity yardstick on exactly sized windows */
        const int64_t P = col0 + ncols;
        double *d = malloc(sizeof(double) * (size_t)W);
        if (orc_consensus(X, P, ldx, W, d) != 0) { printf("consensus failed\n"); return 1; }
        for (int32_t i = 0; i < W; ++i) if (!(d[i] >= 0.0)) { printf("bad norm\n"); return 1; }
        const double e = orc_scaled_error(X, X, col0, ncols, ldx, ldx, W);
        if (e != 0.0) { printf("a stack differs from itself: %g\n", e); return 1; }
        free(d); free(G); free(S); free(V); free(X); free(off); free(perm);
        ++cases;
    }
    printf("ok %d\n", cases);
    return 0;
}
