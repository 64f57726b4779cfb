/*
 * Memory-safety check of the oracle (test infrastructure of test infrastructure): every function of gas_oracle.c is
 * called on seeded random batch subgraphs (empty rows, repeated neighbours, a row that names every column, zero-size
 * cases), both storage types, with every buffer allocated at exactly the size the interface states and row strides
 * larger than the width, so that the address and undefined-behaviour sanitizers see any access outside them.
 * Built and run by tests/test_oracle_sanitizers.py:
 *     gcc -O1 -g -fopenmp -fsanitize=address,undefined -fno-sanitize-recover=undefined sanitize_check.c -lm
 * Values are not checked here (the pins do that); finite outputs are.
 */
#include "gas_oracle.c"

#include <stdio.h>

static uint64_t state = 0x9E3779B97F4A7C15ull;
static uint32_t rnd(void) {
    state = state * 6364136223846793005ull + 1442695040888963407ull;
    return (uint32_t)(state >> 33);
}
static double unit(void) { return (double)rnd() / 2147483648.0 - 0.5; }

static void* rows(int64_t n, int64_t ld, int dt) {          /* [n, ld] filled with values in (-0.5, 0.5) */
    size_t count = (size_t)(n * ld);
    void* p = malloc(count * (dt == OR_F32 ? 4 : 2) + 1);   /* + 1: n == 0 still gives a distinct pointer */
    for (size_t i = 0; i < count; ++i) store_elem(p, (int64_t)i, dt, unit());
    return p;
}

static int64_t failures = 0;
static void all_finite(const char* what, const void* p, int64_t n, int64_t ld, int32_t F, int dt) {
    for (int64_t i = 0; i < n; ++i)
        for (int32_t f = 0; f < F; ++f)
            if (!isfinite(load_elem(p, i * ld + f, dt))) {
                printf("non-finite value from %s at (%lld, %d)\n", what, (long long)i, f);
                ++failures;
                return;
            }
}

static void one_case(int64_t nb, int64_t nh, int32_t F, int32_t F2, int dt, int kind) {
    const int64_t nv = nb + nh, N = nv + 5;
    /* pattern: kind 0 random sparse, 1 with empty rows, 2 first row names every column, 3 repeated neighbours */
    int32_t* rowptr = (int32_t*)malloc((size_t)(nb + 1) * 4);
    int64_t cap = nb * 12 + nv + 1, nnz = 0;
    int32_t* col = (int32_t*)malloc((size_t)cap * 4);
    rowptr[0] = 0;
    for (int64_t v = 0; v < nb; ++v) {
        int64_t d = rnd() % 12;
        if (kind == 1 && (v % 3) == 0) d = 0;
        if (kind == 2 && v == 0) d = nv;
        for (int64_t k = 0; k < d; ++k) {
            int32_t c = (kind == 2 && v == 0) ? (int32_t)k : (int32_t)(rnd() % (uint32_t)nv);
            if (kind == 3 && k > 0 && (k & 1)) c = col[nnz - 1];
            col[nnz++] = c;
        }
        rowptr[v + 1] = (int32_t)nnz;
    }
    int32_t* n_id = (int32_t*)malloc((size_t)nv * 4 + 1);
    for (int64_t i = 0; i < nv; ++i) n_id[i] = (int32_t)(N - 1 - i);              /* distinct ids: the last nv, reversed */
    int32_t* deg = (int32_t*)malloc((size_t)N * 4);
    for (int64_t i = 0; i < N; ++i) deg[i] = (int32_t)(rnd() % 50);
    const int64_t ld = F + 3, ld2 = F2 + 1;

    /* pull, push */
    void* hist = rows(N, ld, dt);
    void* x = rows(nv, ld, dt);
    oracle_pull(hist, ld, n_id + nb, nh, F, dt == OR_F32 ? 4 : 2, (char*)x + nb * ld * (dt == OR_F32 ? 4 : 2), ld);
    oracle_push(x, ld, n_id, nb, F, dt == OR_F32 ? 4 : 2, hist, ld);
    all_finite("pull/push", x, nv, ld, F, dt);

    /* coefficients, aggregation and its adjoint */
    float* val = (float*)malloc((size_t)nnz * 4 + 1);
    oracle_gcn_norm(rowptr, col, nb, n_id, deg, val);
    void* r = rows(nb, ld, dt);
    void* z = rows(nb, ld, dt);
    oracle_spmm(rowptr, col, val, 0.0, x, ld, dt, F, 0.9, r, ld, 0.1, z, ld, dt, nb);
    oracle_spmm(rowptr, col, NULL, 1.1, x, ld, dt, F, 1.0, NULL, 0, 0.0, z, ld, OR_F32 == dt ? OR_F32 : OR_BF16, nb);
    all_finite("spmm", z, nb, ld, F, dt);
    void* gx = rows(nv, ld, dt);
    oracle_spmm_t(rowptr, col, val, 0.0, 0.9, z, ld, dt, F, nb, nv, gx, ld, dt);
    oracle_spmm_t(rowptr, col, NULL, 1.1, 1.0, z, ld, dt, F, nb, nb, gx, ld, dt);
    all_finite("spmm_t", gx, nb, ld, F, dt);

    /* transforms and their backward */
    void* w = rows(F, F2, dt);
    void* w2 = rows(F2, F, dt);
    void* bias = rows(1, F2, dt);
    void* bias2 = rows(1, F, dt);
    void* y = rows(nb, ld2, dt);
    oracle_linear(z, ld, nb, F, w, F2, bias, dt, 0.0, 1.0, 1, y, ld2, dt);
    if (F == F2) oracle_linear(z, ld, nb, F, w, F2, NULL, dt, 0.6, 0.4, 0, y, ld2, dt);
    all_finite("linear", y, nb, ld2, F2, dt);
    void* y2 = rows(nb, ld, dt);
    oracle_mlp2(z, ld, nb, F, w, F2, bias, w2, F, bias2, dt, 1, y2, ld, dt);
    all_finite("mlp2", y2, nb, ld, F, dt);
    void* gp = rows(nb, ld2, dt);
    oracle_relu_bwd(gp, ld2, y, ld2, nb, F2, dt, gp, ld2);
    void* gz = rows(nb, ld, dt);
    oracle_linear_bwd_input(gp, ld2, nb, F2, w, F, dt, 0.0, 1.0, NULL, 0, gz, ld);
    oracle_linear_bwd_input(gp, ld2, nb, F2, w, F, dt, 0.0, 1.0, z, ld, gz, ld);
    all_finite("linear_bwd_input", gz, nb, ld, F, dt);
    float* dw = (float*)malloc((size_t)F * F2 * 4);
    oracle_linear_bwd_weight(z, ld, gp, ld2, nb, F, F2, dt, 0.5, dw);
    all_finite("linear_bwd_weight", dw, F, F2, F2, OR_F32);
    oracle_sgd_step(w, (int64_t)F * F2, dt, dw, 0.01, 1e-4);

    /* loss */
    int32_t* labels = (int32_t*)malloc((size_t)nb * 4 + 1);
    for (int64_t i = 0; i < nb; ++i) labels[i] = (i % 5 == 0) ? -1 : (int32_t)(rnd() % (uint32_t)F2);
    float* loss_rows = (float*)malloc((size_t)nb * 4 + 1);
    double loss_sum = 0.0;
    oracle_softmax_xent(y, ld2, nb, F2, dt, labels, 1.0 / (double)(nb > 0 ? nb : 1), loss_rows, &loss_sum, gp, ld2);
    all_finite("softmax_xent", gp, nb, ld2, F2, dt);
    if (!isfinite(loss_sum)) { printf("non-finite loss\n"); ++failures; }

    /* PNA and GAT aggregations and their backward */
    void* add = rows(nb, ld, dt);
    const int64_t ld9 = 9 * (int64_t)F + 2;
    void* out9 = rows(nb, ld9, dt);
    oracle_pna_aggregate(rowptr, col, nb, x, ld, dt, F, add, ld, 1.7, out9, ld9);
    oracle_pna_aggregate(rowptr, col, nb, x, ld, dt, F, NULL, 0, 1.7, out9, ld9);
    all_finite("pna_aggregate", out9, nb, ld9, 9 * F, dt);
    void* gadd = rows(nb, ld, dt);
    oracle_pna_aggregate_bwd(rowptr, col, nb, nv, x, ld, dt, F, 1.7, out9, ld9, gx, ld, gadd, ld);
    oracle_pna_aggregate_bwd(rowptr, col, nb, nb, x, ld, dt, F, 1.7, out9, ld9, gx, ld, NULL, 0);
    all_finite("pna_aggregate_bwd", gx, nb, ld, F, dt);
    void* a_dst = rows(1, F, dt);
    void* a_src = rows(1, F, dt);
    oracle_gat_aggregate(rowptr, col, nb, x, ld, dt, F, a_dst, a_src, 0.2, 1, z, ld);
    all_finite("gat_aggregate", z, nb, ld, F, dt);
    float* ga = (float*)malloc((size_t)F * 8);
    oracle_gat_aggregate_bwd(rowptr, col, nb, nv, x, ld, dt, F, a_dst, a_src, 0.2, z, ld, gx, ld, ga, ga + F);
    oracle_gat_aggregate_bwd(rowptr, col, nb, nb, x, ld, dt, F, a_dst, a_src, 0.2, z, ld, gx, ld, ga, ga + F);
    all_finite("gat_aggregate_bwd", gx, nb, ld, F, dt);
    all_finite("gat attention gradients", ga, 2, F, F, OR_F32);

    /* regulariser pieces */
    oracle_axpy(x, ld, gx, ld, nb, F, dt, 0.3, z, ld);
    float* dist = (float*)malloc((size_t)nb * 4 + 1);
    double dist_sum = 0.0;
    oracle_row_distance(x, ld, z, ld, nb, F, dt, dist, &dist_sum);
    oracle_row_distance_bwd(x, ld, z, ld, nb, F, dt, 0.5, gz, ld);
    all_finite("row_distance_bwd", gz, nb, ld, F, dt);

    free(rowptr); free(col); free(n_id); free(deg); free(hist); free(x); free(val); free(r); free(z); free(gx);
    free(w); free(w2); free(bias); free(bias2); free(y); free(y2); free(gp); free(gz); free(dw); free(labels);
    free(loss_rows); free(add); free(out9); free(gadd); free(a_dst); free(a_src); free(ga); free(dist);
}

int main(void) {
    int cases = 0;
    const int64_t sizes[][2] = {{0, 0}, {1, 0}, {1, 1}, {7, 0}, {40, 25}, {130, 300}, {257, 64}};
    const int32_t widths[][2] = {{1, 1}, {7, 5}, {16, 16}, {33, 9}};
    for (int dt = 0; dt < 2; ++dt)
        for (size_t s = 0; s < sizeof(sizes) / sizeof(sizes[0]); ++s)
            for (size_t w = 0; w < sizeof(widths) / sizeof(widths[0]); ++w)
                for (int kind = 0; kind < 4; ++kind) {
                    if (sizes[s][0] + sizes[s][1] == 0 && kind == 2) continue;
                    one_case(sizes[s][0], sizes[s][1], widths[w][0], widths[w][1], dt, kind);
                    ++cases;
                }
    uint16_t edge = oracle_round_bf16(3.3895313892515355e38);       /* rounds to infinity, must not trap */
    (void)edge;
    printf("%d cases, %d threads, %lld failures\n", cases, oracle_num_threads(), (long long)failures);
    return failures != 0;
}
