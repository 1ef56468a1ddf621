/*
 * Memory- and undefined-behaviour check of the CPU oracle (test infrastructure, like the
 * oracle itself).  Built together with castling_oracle.c under
 *   gcc -O1 -g -fsanitize=address,undefined -fno-sanitize-recover=all -fopenmp
 * and run by tests/test_oracle_sanitized.py: every exported function is called on small shapes
 * chosen for their edges (one token, one row, one column, filters wider than the grid, class
 * tokens, pooled grids with odd sides, rows under the norm floor), each in tightly sized heap
 * buffers so that any access past an end is caught, and the two forms the oracle has of each
 * quantity (explicit definition / reassociated state / sampled rows) are compared.
 * Exit status 0 = clean; the sanitizers abort otherwise, a disagreement returns 1.
 */
#include "castling_oracle.c"

#include <stdio.h>

static uint64_t rng_state = 0x9E3779B97F4A7C15ull;
static double rnd(void)  /* uniform in (-1, 1), xorshift */
{
    rng_state ^= rng_state << 13;
    rng_state ^= rng_state >> 7;
    rng_state ^= rng_state << 17;
    return (double)(rng_state >> 11) / 4503599627370496.0 - 1.0;
}
static double* fill(size_t n)
{
    double* p = (double*)malloc(sizeof(double) * (n ? n : 1));
    for (size_t i = 0; i < n; ++i) p[i] = rnd();
    return p;
}
/* max |a - b| relative to max(1, max |a|): a zero row under the norm floor has gradients of the
 * order 1 / eps */
static double maxdiff(const double* a, const double* b, size_t n)
{
    double m = 0.0, scale = 1.0;
    for (size_t i = 0; i < n; ++i) {
        const double e = fabs(a[i] - b[i]);
        if (!(e <= m)) m = e;  /* NaN propagates */
        if (fabs(a[i]) > scale) scale = fabs(a[i]);
    }
    return m / scale;
}

static int failures = 0;
static void expect(int ok, const char* what, int B, int heads, int H, int W, int d, int ks, int extra)
{
    if (!ok) {
        fprintf(stderr, "MISMATCH %s at B=%d heads=%d H=%d W=%d d=%d ks=%d extra=%d\n", what, B, heads,
                H, W, d, ks, extra);
        ++failures;
    }
}

static void layer_case(int B, int heads, int H, int W, int d, int ks, int extra, double eps)
{
    const int N = extra + H * W;
    const size_t total = (size_t)B * heads * N * d, nw = (size_t)heads * d * ks * ks;
    double *q = fill(total), *k = fill(total), *v = fill(total), *g = fill(total);
    double *w = fill(nw), *bias = fill((size_t)heads * d);
    for (int c = 0; c < d; ++c) q[c] = 0.0;                       /* a zero query row */
    for (int c = 0; c < d; ++c) k[(size_t)(N - 1) * d + c] = 0.0;  /* a zero key row */
    for (int norm = 0; norm < 2; ++norm)
        for (unsigned br = 1; br <= 3; ++br) {
            double *a = fill(total), *b = fill(total);
            oracle_forward_explicit(q, k, v, w, bias, B, heads, H, W, d, ks, norm, br, eps, extra, a);
            oracle_forward(q, k, v, w, bias, B, heads, H, W, d, ks, norm, br, eps, extra, b);
            expect(maxdiff(a, b, total) < 1e-9, "forward", B, heads, H, W, d, ks, extra);
            /* every row through the sampled form, last unit first */
            const int64_t nrows = (int64_t)B * heads * N;
            int64_t* us = (int64_t*)malloc(sizeof(int64_t) * nrows);
            int64_t* ts = (int64_t*)malloc(sizeof(int64_t) * nrows);
            for (int64_t i = 0; i < nrows; ++i) {
                us[i] = (int64_t)B * heads - 1 - i / N;
                ts[i] = N - 1 - i % N;
            }
            double* rows = fill((size_t)nrows * d);
            oracle_forward_explicit_rows(q, k, v, w, NULL, B, heads, H, W, d, ks, norm, br, eps, extra,
                                         us, ts, nrows, rows);
            oracle_forward_explicit(q, k, v, w, NULL, B, heads, H, W, d, ks, norm, br, eps, extra, a);
            int ok = 1;
            for (int64_t i = 0; i < nrows && ok; ++i)
                ok = maxdiff(rows + (size_t)i * d, a + ((size_t)us[i] * N + ts[i]) * d, d) < 1e-10;
            expect(ok, "forward rows", B, heads, H, W, d, ks, extra);
            /* gradients: definition, reassociated, sampled rows */
            double *dq = fill(total), *dk = fill(total), *dv = fill(total), *dw = fill(nw);
            double *db = fill((size_t)heads * d);
            double *eq = fill(total), *ek = fill(total), *ev = fill(total), *ew = fill(nw);
            const int residual = (br & 1u) ? norm : 0;
            oracle_backward_explicit(q, k, v, w, g, B, heads, H, W, d, ks, norm, br, eps, extra, residual,
                                     dq, dk, dv, dw, db);
            oracle_backward(q, k, v, w, g, B, heads, H, W, d, ks, norm, br, eps, extra, residual, eq, ek,
                            ev, ew, NULL);
            expect(maxdiff(dq, eq, total) < 1e-8 && maxdiff(dk, ek, total) < 1e-8 &&
                       maxdiff(dv, ev, total) < 1e-8 && maxdiff(dw, ew, nw) < 1e-8,
                   "backward", B, heads, H, W, d, ks, extra);
            double *rq = fill((size_t)nrows * d), *rk = fill((size_t)nrows * d), *rv = fill((size_t)nrows * d);
            oracle_backward_explicit_rows(q, k, v, w, g, B, heads, H, W, d, ks, norm, br, eps, extra,
                                          residual, us, ts, nrows, rq, rk, rv);
            ok = 1;
            for (int64_t i = 0; i < nrows && ok; ++i) {
                const size_t o = ((size_t)us[i] * N + ts[i]) * d;
                ok = maxdiff(rq + (size_t)i * d, dq + o, d) < 1e-8 && maxdiff(rk + (size_t)i * d, dk + o, d) < 1e-8 &&
                     maxdiff(rv + (size_t)i * d, dv + o, d) < 1e-8;
            }
            expect(ok, "backward rows", B, heads, H, W, d, ks, extra);
            free(a); free(b); free(us); free(ts); free(rows); free(dq); free(dk); free(dv); free(dw);
            free(db); free(eq); free(ek); free(ev); free(ew); free(rq); free(rk); free(rv);
        }
    /* state and the DWConv alone */
    double* st = fill((size_t)B * heads * (d + 1) * (d + 1));
    oracle_state(k, v, B, heads, N, d, eps, st);
    expect(fabs(st[(size_t)(d + 1) * (d + 1) - 1] - N) < 1e-12, "state corner", B, heads, H, W, d, ks, extra);
    free(st);
    if (extra == 0) {
        double* o = fill(total);
        oracle_dwconv(v, w, bias, B, heads, H, W, d, ks, o);
        free(o);
    }
    free(q); free(k); free(v); free(g); free(w); free(bias);
}

static void pooled_case(int B, int heads, int H, int W, int d, int ks, int residual)
{
    const int s = 2, N = H * W, Nq = ((H + 1) / 2) * ((W + 1) / 2);
    const size_t tk = (size_t)B * heads * N * d, tq = (size_t)B * heads * Nq * d;
    const size_t nw = (size_t)heads * d * ks * ks;
    double *q = fill(tq), *k = fill(tk), *v = fill(tk), *g = fill(tq), *w = fill(nw);
    double* bias = fill((size_t)heads * d);
    for (int norm = 0; norm < 2; ++norm)
        for (unsigned br = 1; br <= 3; ++br) {
            if (residual && !(br & 1u)) continue;
            double *a = fill(tq), *b = fill(tq);
            oracle_forward_pooled_explicit(q, k, v, w, bias, B, heads, H, W, d, ks, s, residual, norm, br,
                                           1e-12, a);
            oracle_forward_pooled(q, k, v, w, bias, B, heads, H, W, d, ks, s, residual, norm, br, 1e-12, b);
            expect(maxdiff(a, b, tq) < 1e-9, "pooled forward", B, heads, H, W, d, ks, 0);
            double *dq = fill(tq), *dk = fill(tk), *dv = fill(tk), *dw = fill(nw), *db = fill((size_t)heads * d);
            oracle_backward_pooled_explicit(q, k, v, w, g, B, heads, H, W, d, ks, s, residual, norm, br,
                                            1e-12, dq, dk, dv, dw, db);
            free(a); free(b); free(dq); free(dk); free(dv); free(dw); free(db);
        }
    free(q); free(k); free(v); free(g); free(w); free(bias);
}

static void pairwise_case(int B, int heads, int N, int d)
{
    const size_t total = (size_t)B * heads * N * d;
    double *q = fill(total), *k = fill(total), *v = fill(total), *o = fill(total);
    double *A = fill((size_t)N * N), *L = fill((size_t)N * N), *P = fill((size_t)N * N);
    int64_t* nnz = (int64_t*)malloc(sizeof(int64_t) * (size_t)B * heads);
    oracle_sim_angular(q, k, N, d, 1e-12, A);
    oracle_sim_linear(q, k, N, d, 1e-12, L);
    int ok = 1;
    for (int i = 0; i < N * N; ++i) ok = ok && A[i] >= -1e-12 && A[i] <= 1.0 + 1e-12 && fabs(L[i] - 0.5) <= 1.0 / ORACLE_PI + 1e-12;
    expect(ok, "similarity ranges", B, heads, N, 1, d, 0, 0);
    for (int normalize = 0; normalize < 2; ++normalize) {
        oracle_softmax_probs(q, k, N, d, normalize, 0.7, 1e-12, P);
        double rs = 0.0;
        for (int j = 0; j < N; ++j) rs += P[j];
        expect(fabs(rs - 1.0) < 1e-12, "softmax row sum", B, heads, N, 1, d, 0, 0);
        oracle_sparse_attn(q, k, v, B, heads, N, d, normalize, 0.7, 0.02, 1e-12, o, nnz);
        oracle_sparse_attn(q, k, v, B, heads, N, d, normalize, 0.7, 2.0, 1e-12, o, nnz);  /* nothing kept */
        expect(nnz[0] == 0, "sparse threshold above 1 keeps nothing", B, heads, N, 1, d, 0, 0);
    }
    oracle_angular_attn(q, k, v, B, heads, N, d, 0, 1e-12, o);
    oracle_angular_attn(q, k, v, B, heads, N, d, 1, 1e-12, o);
    expect(fabs(oracle_sim_series(0.0, 6) - 0.5) < 1e-15 && oracle_series_coeff(1) > 0.0, "series", 0, 0, 0, 0, 0, 0, 0);
    free(q); free(k); free(v); free(o); free(A); free(L); free(P); free(nnz);
}

int main(void)
{
    oracle_set_num_threads(4);
    /*         B  h  H   W  d  ks extra eps */
    layer_case(1, 1, 1,  1, 1, 1, 0, 1e-12);   /* one token, one feature */
    layer_case(1, 2, 1,  1, 3, 9, 0, 1e-12);   /* filter far wider than the grid */
    layer_case(2, 1, 1,  7, 2, 5, 0, 1e-12);   /* one row */
    layer_case(1, 1, 6,  1, 2, 7, 3, 1e-12);   /* one column, class tokens */
    layer_case(2, 3, 4,  5, 6, 3, 0, 2.0);     /* rows under the norm floor */
    layer_case(1, 2, 3,  3, 5, 9, 2, 1e-12);
    layer_case(1, 1, 9, 11, 8, 5, 1, 1e-12);
    pooled_case(1, 1, 1, 1, 2, 3, 1);
    pooled_case(2, 2, 5, 7, 3, 5, 1);          /* odd sides: the last pooled row and column */
    pooled_case(1, 2, 6, 4, 4, 3, 0);
    pooled_case(1, 1, 1, 6, 2, 9, 1);
    pairwise_case(1, 1, 1, 1);
    pairwise_case(2, 2, 9, 5);
    if (failures) return 1;
    printf("oracle self-check clean (%d threads)\n", oracle_num_threads());
    return 0;
}
