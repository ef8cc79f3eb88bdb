/*
 * Host sanitizer target of the fp64 oracle -- TEST INFRASTRUCTURE ONLY.
 *
 * Built together with slicemoe_oracle.c under -fsanitize=address,undefined and run by the CPU test suite: it calls
 * every entry point of the oracle on small layers whose buffers have exactly the documented sizes, so that an index
 * past the end of any input or output, a signed overflow or a misaligned access inside the oracle ends the run with a
 * sanitizer report.  The values are checked only through invariants that hold for any input (counts sum to T*S*k,
 * probabilities in (0, 1], perm/inv are inverse to each other); the numeric pins live in the Python tests.
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int oracle_route(const double *, int64_t, int, int, int, int, const double *, const double *, const double *, const double *,
                 int32_t *, double *, double *, double *);
int oracle_route_train(const double *, int64_t, int, int, int, int, const double *, const double *, const double *,
                       const double *, double, double, const double *, double, const double *, int32_t *, double *,
                       double *, double *);
int oracle_dispatch(const int32_t *, int64_t, int, int, int64_t, int32_t *, int32_t *, int32_t *, int32_t *, int32_t *);
int oracle_expert_rows(const double *, int, int, int, const int32_t *, const double *, const int32_t *, int64_t,
                       const double *, const double *, const double *, const double *, int, double *);
int oracle_combine(const double *, const int32_t *, int64_t, int, int, double *);
int oracle_slices(const double *, int64_t, int, int, int, const int32_t *, const double *, const int32_t *, const double *,
                  const double *, const double *, const double *, int, double *);
int oracle_forward(const double *, int64_t, int, int, int, int, int, int, int64_t, const double *, const double *,
                   const double *, const double *, const double *, const double *, const double *, const double *, int,
                   double *, int32_t *, double *, double *, int32_t *, int32_t *, int32_t *, int32_t *, int32_t *);
int oracle_backward(const double *, int64_t, int, int, int, int, int, const double *, const double *, const double *,
                    const double *, const double *, const double *, const double *, const double *, double, double,
                    const double *, double, const double *, const int32_t *, const int32_t *, const double *,
                    const double *, double *, double *, double *, double *, double *, double *, double *, double *, double *);
int oracle_load_stats(const int32_t *, int, double *, double *, double *);
double oracle_gelu(double);

static uint64_t state = 0x1234567u;
static double draw(void) /* uniform in (-1, 1), a fixed sequence */
{
    state = state * 6364136223846793005ull + 1442695040888963407ull;
    return (double)(state >> 11) / 9007199254740992.0 * 2.0 - 1.0;
}

/* exactly n elements (at least one byte, so that the pointer is valid) filled from the sequence */
static double *rand_f64(size_t n, double scale)
{
    double *p = (double *)malloc(n ? n * sizeof(double) : 1);
    if (!p) abort();
    for (size_t i = 0; i < n; ++i) p[i] = scale * draw();
    return p;
}
static double *new_f64(size_t n)
{
    double *p = (double *)malloc(n ? n * sizeof(double) : 1);
    if (!p) abort();
    return p;
}
static int32_t *new_i32(size_t n)
{
    int32_t *p = (int32_t *)malloc(n ? n * sizeof(int32_t) : 1);
    if (!p) abort();
    return p;
}

#define CHECK(cond)                                                              \
    do {                                                                         \
        if (!(cond)) {                                                           \
            fprintf(stderr, "sanitize_main: check failed at line %d: %s\n", __LINE__, #cond); \
            exit(2);                                                             \
        }                                                                        \
    } while (0)

static void one_layer(int64_t T, int d, int S, int Hr, int E, int k, int He, int64_t capacity, double rate, double sigma)
{
    const int ds = d / S;
    const int64_t Ns = T * S, Na = Ns * k;
    double *h = rand_f64((size_t)(T * d), 1.0);
    double *Wr1 = rand_f64((size_t)ds * Hr, 0.5), *br1 = rand_f64((size_t)Hr, 0.5);
    double *Wr2 = rand_f64((size_t)Hr * E, 0.5), *br2 = rand_f64((size_t)E, 0.5);
    double *W1 = rand_f64((size_t)E * ds * He, 0.5), *b1 = rand_f64((size_t)E * He, 0.5);
    double *W2 = rand_f64((size_t)E * He * ds, 0.5), *b2 = rand_f64((size_t)E * ds, 0.5);
    double *G = rand_f64((size_t)(T * d), 1.0);
    double *noise = rand_f64((size_t)(Ns * E), 1.0);
    double *drop_u = rand_f64((size_t)Na, 0.5);
    for (int64_t a = 0; a < Na; ++a) drop_u[a] += 0.5; /* (0, 1) */

    /* whole layer */
    double *h_out = new_f64((size_t)(T * d)), *pk = new_f64((size_t)Na), *margin = new_f64((size_t)Ns);
    int32_t *idx = new_i32((size_t)Na), *counts_raw = new_i32((size_t)E), *counts = new_i32((size_t)E);
    int32_t *offsets = new_i32((size_t)E + 1), *perm = new_i32((size_t)Na), *inv = new_i32((size_t)Na);
    CHECK(oracle_forward(h, T, d, S, Hr, E, k, He, capacity, Wr1, br1, Wr2, br2, W1, b1, W2, b2, 0, h_out, idx, pk, margin,
                         counts_raw, counts, offsets, perm, inv) == 0);
    int64_t sum_raw = 0;
    for (int e = 0; e < E; ++e) sum_raw += counts_raw[e];
    CHECK(sum_raw == Na);
    CHECK(offsets[0] == 0);
    for (int64_t r = 0; r < offsets[E]; ++r) CHECK(perm[r] >= 0 && perm[r] < Na && inv[perm[r]] == r);
    for (int64_t a = 0; a < Na; ++a) CHECK(pk[a] > 0.0 && pk[a] <= 1.0 && idx[a] >= 0 && idx[a] < E);

    /* stage functions on the same routing */
    double *logits = new_f64((size_t)(Ns * E));
    int32_t *idx2 = new_i32((size_t)Na);
    double *pk2 = new_f64((size_t)Na);
    CHECK(oracle_route(h, Ns, ds, Hr, E, k, Wr1, br1, Wr2, br2, idx2, pk2, logits, margin) == 0);
    CHECK(memcmp(idx, idx2, (size_t)Na * sizeof(int32_t)) == 0);
    CHECK(oracle_route(h, Ns, ds, Hr, E, k, Wr1, br1, Wr2, br2, idx2, pk2, NULL, NULL) == 0);
    CHECK(oracle_dispatch(idx, Ns, k, E, capacity, counts_raw, counts, offsets, perm, inv) == 0);
    const int64_t kept = offsets[E];
    double *y = new_f64((size_t)(kept * ds)), *out = new_f64((size_t)(Ns * ds)), *out2 = new_f64((size_t)(Ns * ds));
    CHECK(oracle_expert_rows(h, ds, He, k, idx, pk, perm, kept, W1, b1, W2, b2, 0, y) == 0);
    CHECK(oracle_combine(y, inv, Ns, k, ds, out) == 0);
    CHECK(oracle_slices(h, Ns, ds, He, k, idx, pk, inv, W1, b1, W2, b2, 0, out2) == 0);
    CHECK(oracle_slices(h, Ns, ds, He, k, idx, pk, NULL, W1, b1, W2, b2, 1, out2) == 0);

    /* training-time router and the backward through it */
    CHECK(oracle_route_train(h, Ns, ds, Hr, E, k, Wr1, br1, Wr2, br2, 0.7, sigma, noise, rate, drop_u, idx2, pk2, logits,
                             margin) == 0);
    CHECK(oracle_dispatch(idx2, Ns, k, E, capacity, counts_raw, counts, offsets, perm, inv) == 0);
    double *dx = new_f64((size_t)(Ns * ds));
    double *dWr1 = new_f64((size_t)ds * Hr), *dbr1 = new_f64((size_t)Hr), *dWr2 = new_f64((size_t)Hr * E);
    double *dbr2 = new_f64((size_t)E), *dW1 = new_f64((size_t)E * ds * He), *db1 = new_f64((size_t)E * He);
    double *dW2 = new_f64((size_t)E * He * ds), *db2 = new_f64((size_t)E * ds);
    CHECK(oracle_backward(h, Ns, ds, Hr, E, k, He, Wr1, br1, Wr2, br2, W1, b1, W2, b2, 0.7, sigma, noise, rate, drop_u, idx2,
                          inv, G, NULL, dx, dWr1, dbr1, dWr2, dbr2, dW1, db1, dW2, db2) == 0);
    double *capg = new_f64((size_t)E);
    CHECK(oracle_backward(h, Ns, ds, Hr, E, k, He, Wr1, br1, Wr2, br2, W1, b1, W2, b2, 0.7, sigma, noise, rate, drop_u, idx2,
                          inv, G, capg, dx, dWr1, dbr1, dWr2, dbr2, dW1, db1, dW2, db2) == 0);
    free(capg);
    double cv_pop, cv_sample, ele;
    CHECK(oracle_load_stats(counts_raw, E, &cv_pop, &cv_sample, &ele) == 0);
    CHECK(ele >= -1e-12 && ele <= 1.0 + 1e-12 && cv_pop >= 0.0);

    free(h); free(Wr1); free(br1); free(Wr2); free(br2); free(W1); free(b1); free(W2); free(b2); free(G); free(noise);
    free(drop_u); free(h_out); free(pk); free(margin); free(idx); free(counts_raw); free(counts); free(offsets); free(perm);
    free(inv); free(logits); free(idx2); free(pk2); free(y); free(out); free(out2); free(dx); free(dWr1); free(dbr1);
    free(dWr2); free(dbr2); free(dW1); free(db1); free(dW2); free(db2);
}

int main(void)
{
    CHECK(oracle_gelu(0.0) == 0.0);
    one_layer(5, 12, 3, 7, 4, 2, 5, -1, 0.0, 0.0);    /* odd sizes, dropless */
    one_layer(9, 12, 3, 7, 4, 2, 5, 5, 0.3, 0.2);     /* capacity drops, dropout, noise */
    one_layer(6, 8, 2, 3, 3, 3, 2, 4, 0.5, 0.0);      /* k == E, capacity below the load */
    one_layer(4, 6, 1, 5, 1, 1, 3, -1, 0.0, 0.1);     /* one expert, one slice per token */
    one_layer(0, 8, 2, 4, 4, 2, 4, -1, 0.2, 0.1);     /* empty batch */
    one_layer(70, 32, 4, 16, 8, 2, 12, 30, 0.2, 0.0); /* more slices than threads */
    /* bad arguments are refused, not acted on */
    int32_t bad_idx[2] = {0, 9}, c[4], o[5], p[2], iv[2];
    CHECK(oracle_dispatch(bad_idx, 1, 2, 4, -1, c, c, o, p, iv) == -1);
    CHECK(oracle_route(NULL, 1, 1, 1, 1, 1, NULL, NULL, NULL, NULL, NULL, NULL, NULL, NULL) == -1);
    puts("sanitize_main: ok");
    return 0;
}
