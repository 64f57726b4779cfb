/*
 * Plain CPU oracle for the GAS layer step.  TEST INFRASTRUCTURE ONLY: the
 * tests, the smoke check and the benchmark's cpu_baseline leg call it; the
 * product never does, and it shares no code with the HIP library.
 *
 * Every function is the written-out definition of one operation of the
 * mini-batch message-passing step with historical embeddings:
 *   - pull / push: the Pull and Push operations of the paper's Algorithm 1
 *     (row gather from, and row scatter into, a history table);
 *   - spmm: the neighbourhood sum of the paper's Eq. (1)/(2) over the rows of
 *     the batch subgraph, with the edge weights of the GCN, GCNII and GIN
 *     operators of its operator appendix;
 *   - spmm_t: the adjoint of that sum (backward aggregation);
 *   - linear: the dense transform of the same operators;
 *   - gcn_norm: the coefficient 1/c_{w,v} of the GCN operator.
 * Arithmetic is double precision; a value is rounded once, at the store into
 * a buffer whose type the interface fixes (fp32, or bf16 with round-to-
 * nearest-even).  No blocking, fusion or reordering: loops run in the order
 * the definitions state.
 */
#include <stdint.h>
#include <string.h>
#include <math.h>
#include <stdlib.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { OR_F32 = 0, OR_BF16 = 1 };

/* bf16 = upper 16 bits of an IEEE fp32 */
static double bf16_to_double(uint16_t h) {
    uint32_t u = ((uint32_t)h) << 16;
    float f;
    memcpy(&f, &u, 4);
    return (double)f;
}

/* double -> bf16, round to nearest even, decided on the exact double value */
static uint16_t double_to_bf16(double x) {
    if (isnan(x)) return 0x7FC0;
    float f = (float)x;               /* candidate; may itself have rounded */
    uint32_t u;
    memcpy(&u, &f, 4);
    /* bracket x between two neighbouring bf16 values (truncate fp32 toward zero) */
    uint32_t lo_bits = u & 0xFFFF0000u;
    float lo_f;
    memcpy(&lo_f, &lo_bits, 4);
    if (isinf(f)) return (uint16_t)(u >> 16);
    /* (float)x may have rounded across a bf16 boundary away from zero */
    if (fabs((double)lo_f) > fabs(x)) {
        lo_bits -= 0x10000u;
        memcpy(&lo_f, &lo_bits, 4);
    }
    uint32_t hi_bits = lo_bits + 0x10000u;
    float hi_f;
    memcpy(&hi_f, &hi_bits, 4);
    double dl = fabs(x - (double)lo_f), dh = fabs((double)hi_f - x);
    if (isinf(hi_f)) dh = fabs(ldexp(1.0, 128) * (x < 0 ? -1.0 : 1.0) - x);
    uint32_t pick;
    if (dl < dh) pick = lo_bits;
    else if (dh < dl) pick = hi_bits;
    else pick = ((lo_bits >> 16) & 1u) ? hi_bits : lo_bits;   /* tie: even mantissa */
    return (uint16_t)(pick >> 16);
}

static double load_elem(const void* p, int64_t i, int dt) {
    return dt == OR_F32 ? (double)((const float*)p)[i] : bf16_to_double(((const uint16_t*)p)[i]);
}

static void store_elem(void* p, int64_t i, int dt, double v) {
    if (dt == OR_F32) ((float*)p)[i] = (float)v;
    else ((uint16_t*)p)[i] = double_to_bf16(v);
}

uint16_t oracle_round_bf16(double x) { return double_to_bf16(x); }

/* Pull: dst[i, :] = hist[idx[i], :]  (Algorithm 1, Pull^(l) for w in V_b \ B_b) */
void oracle_pull(const void* hist, int64_t ld_hist, const int32_t* idx, int64_t n,
                 int32_t F, int32_t elem_bytes, void* dst, int64_t ld_dst) {
    for (int64_t i = 0; i < n; ++i)
        memcpy((char*)dst + i * ld_dst * elem_bytes,
               (const char*)hist + (int64_t)idx[i] * ld_hist * elem_bytes, (size_t)F * elem_bytes);
}

/* Push: hist[idx[i], :] = src[i, :]  (Algorithm 1, Push^(l) for v in B_b) */
void oracle_push(const void* src, int64_t ld_src, const int32_t* idx, int64_t n,
                 int32_t F, int32_t elem_bytes, void* hist, int64_t ld_hist) {
    for (int64_t i = 0; i < n; ++i)
        memcpy((char*)hist + (int64_t)idx[i] * ld_hist * elem_bytes,
               (const char*)src + i * ld_src * elem_bytes, (size_t)F * elem_bytes);
}

/* 1/c_{w,v} = 1 / (sqrt(deg(w)+1) * sqrt(deg(v)+1)) for every stored entry
 * (v = row, w = column), degrees taken on the full graph (GCN operator). */
void oracle_gcn_norm(const int32_t* ptr, const int32_t* ind, int64_t n_rows,
                     const int32_t* n_id, const int32_t* deg, float* val) {
    for (int64_t v = 0; v < n_rows; ++v)
        for (int64_t k = ptr[v]; k < ptr[v + 1]; ++k) {
            double dv = (double)deg[n_id[v]] + 1.0, dw = (double)deg[n_id[ind[k]]] + 1.0;
            val[k] = (float)(1.0 / (sqrt(dw) * sqrt(dv)));
        }
}

/* Z[v,:] = s_agg * sum_{k in row v} val[k] * X[col[k],:] + diag * X[v,:] + s_res * R[v,:]
 * GCN: val = 1/c, diag = 0 (the self-loop is a stored entry).  GIN: val = 1
 * (NULL), diag = 1+eps.  GCNII: s_agg = 1-alpha, R = initial embedding, s_res = alpha. */
void oracle_spmm(const int32_t* rowptr, const int32_t* col, const float* val, double diag,
                 const void* X, int64_t ldx, int dtx, int32_t F, double s_agg,
                 const void* R, int64_t ldr, double s_res,
                 void* Z, int64_t ldz, int dtz, int64_t n_rows) {
#pragma omp parallel for schedule(dynamic, 64)
    for (int64_t v = 0; v < n_rows; ++v) {
        double* acc = (double*)calloc((size_t)F, sizeof(double));
        for (int64_t k = rowptr[v]; k < rowptr[v + 1]; ++k) {
            double a = val ? (double)val[k] : 1.0;
            int64_t w = col[k];
            for (int32_t j = 0; j < F; ++j) acc[j] += a * load_elem(X, w * ldx + j, dtx);
        }
        for (int32_t j = 0; j < F; ++j) {
            double z = s_agg * acc[j];
            if (diag != 0.0) z += diag * load_elem(X, v * ldx + j, dtx);
            if (R) z += s_res * load_elem(R, v * ldr + j, dtx);
            store_elem(Z, v * ldz + j, dtz, z);
        }
        free(acc);
    }
}

/* Adjoint of the aggregation, written from the SAME row-major entries as the
 * forward: GX[col[k],:] += s_agg * val[k] * G[v,:] for every stored (v, col[k]),
 * plus diag * G[u,:] for u < n_rows.  Rows u >= n_out of GX are not produced. */
void oracle_spmm_t(const int32_t* rowptr, const int32_t* col, const float* val, double diag, double s_agg,
                   const void* G, int64_t ldg, int dtg, int32_t F, int64_t n_rows,
                   int64_t n_out, void* GX, int64_t ldgx, int dtgx) {
    double* acc = (double*)calloc((size_t)n_out * F, sizeof(double));
    for (int64_t v = 0; v < n_rows; ++v)
        for (int64_t k = rowptr[v]; k < rowptr[v + 1]; ++k) {
            int64_t u = col[k];
            if (u >= n_out) continue;
            double a = val ? (double)val[k] : 1.0;
            for (int32_t j = 0; j < F; ++j) acc[u * F + j] += a * load_elem(G, v * ldg + j, dtg);
        }
    for (int64_t u = 0; u < n_out; ++u)
        for (int32_t j = 0; j < F; ++j) {
            double g = s_agg * acc[u * F + j];
            if (diag != 0.0 && u < n_rows) g += diag * load_elem(G, u * ldg + j, dtg);
            store_elem(GX, u * ldgx + j, dtgx, g);
        }
    free(acc);
}

/* Y = act( c_identity * Z + c_weight * (Z W) + bias ),  W row-major [F_in, F_out].
 * GCN: c_identity = 0, c_weight = 1.  GCNII: the identity map W <- (1-beta) I + beta W
 * gives c_identity = 1-beta, c_weight = beta (needs F_in == F_out). */
void oracle_linear(const void* Z, int64_t ldz, int64_t n_rows, int32_t F_in,
                   const void* W, int32_t F_out, const void* bias, int dt,
                   double c_identity, double c_weight, int relu,
                   void* Y, int64_t ldy, int dty) {
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n_rows; ++i)
        for (int32_t j = 0; j < F_out; ++j) {
            double s = 0.0;
            for (int32_t k = 0; k < F_in; ++k)
                s += load_elem(Z, i * ldz + k, dt) * load_elem(W, (int64_t)k * F_out + j, dt);
            double y = c_weight * s;
            if (c_identity != 0.0) y += c_identity * load_elem(Z, i * ldz + j, dt);
            if (bias) y += load_elem(bias, j, dt);
            if (relu && y < 0.0) y = 0.0;
            store_elem(Y, i * ldy + j, dty, y);
        }
}

/* GIN update: Y = act( relu(Z W1 + b1) W2 + b2 ); the hidden activation stays
 * in double (it is not a buffer of the interface). */
void oracle_mlp2(const void* Z, int64_t ldz, int64_t n_rows, int32_t F_in,
                 const void* W1, int32_t F_hid, const void* b1,
                 const void* W2, int32_t F_out, const void* b2, int dt, int relu_out,
                 void* Y, int64_t ldy, int dty) {
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n_rows; ++i) {
        double* h = (double*)calloc((size_t)F_hid, sizeof(double));
        for (int32_t j = 0; j < F_hid; ++j) {
            double s = 0.0;
            for (int32_t k = 0; k < F_in; ++k)
                s += load_elem(Z, i * ldz + k, dt) * load_elem(W1, (int64_t)k * F_hid + j, dt);
            if (b1) s += load_elem(b1, j, dt);
            h[j] = s > 0.0 ? s : 0.0;
        }
        for (int32_t j = 0; j < F_out; ++j) {
            double s = 0.0;
            for (int32_t k = 0; k < F_hid; ++k) s += h[k] * load_elem(W2, (int64_t)k * F_out + j, dt);
            if (b2) s += load_elem(b2, j, dt);
            if (relu_out && s < 0.0) s = 0.0;
            store_elem(Y, i * ldy + j, dty, s);
        }
        free(h);
    }
}

int oracle_num_threads(void) {
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

/* ------------------------------------------------------------------------
 * Backward pass of the transform (chain rule on the operator equations of the
 * paper's operator appendix; the paper itself only states that gradients are
 * taken through the layers, Section 2 advantage (1)).
 * ------------------------------------------------------------------------ */

/* ReLU backward: GP = GY where Y > 0, else 0. */
void oracle_relu_bwd(const void* GY, int64_t ldgy, const void* Y, int64_t ldy, int64_t n_rows, int32_t F,
                     int dt, void* GP, int64_t ldgp) {
    for (int64_t i = 0; i < n_rows; ++i)
        for (int32_t j = 0; j < F; ++j) {
            double y = load_elem(Y, i * ldy + j, dt);
            store_elem(GP, i * ldgp + j, dt, y > 0.0 ? load_elem(GY, i * ldgy + j, dt) : 0.0);
        }
}

/* Input gradient of Y = c_identity * Z + c_weight * (Z W):
 *   GZ = c_identity * GP + c_weight * (GP W^T),  then GZ *= [mask > 0] if a mask is given
 * (the mask is the hidden activation of a GIN MLP).  W is [F_in, F_out]. */
void oracle_linear_bwd_input(const void* GP, int64_t ldgp, int64_t n_rows, int32_t F_out,
                             const void* W, int32_t F_in, int dt, double c_identity, double c_weight,
                             const void* mask, int64_t ldmask, void* GZ, int64_t ldgz) {
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n_rows; ++i)
        for (int32_t k = 0; k < F_in; ++k) {
            double s = 0.0;
            for (int32_t j = 0; j < F_out; ++j)
                s += load_elem(GP, i * ldgp + j, dt) * load_elem(W, (int64_t)k * F_out + j, dt);
            double g = c_weight * s;
            if (c_identity != 0.0) g += c_identity * load_elem(GP, i * ldgp + k, dt);
            if (mask && !(load_elem(mask, i * ldmask + k, dt) > 0.0)) g = 0.0;
            store_elem(GZ, i * ldgz + k, dt, g);
        }
}

/* Weight gradient of the same transform: dW[k, j] = c_weight * sum_i Z[i, k] * GP[i, j], kept in fp32. */
void oracle_linear_bwd_weight(const void* Z, int64_t ldz, const void* GP, int64_t ldgp, int64_t n_rows,
                              int32_t F_in, int32_t F_out, int dt, double c_weight, float* dW) {
#pragma omp parallel for schedule(static)
    for (int32_t k = 0; k < F_in; ++k)
        for (int32_t j = 0; j < F_out; ++j) {
            double s = 0.0;
            for (int64_t i = 0; i < n_rows; ++i)
                s += load_elem(Z, i * ldz + k, dt) * load_elem(GP, i * ldgp + j, dt);
            dW[(int64_t)k * F_out + j] = (float)(c_weight * s);
        }
}

/*
 * Loss on the mini-batch and the optimisation step that closes Algorithm 1's
 * loop body.  The paper computes the loss on the in-batch nodes only (Section 1,
 * mini-batch training) and evaluates on node classification; it names neither
 * the loss nor the optimiser.  Taken here: softmax cross-entropy over the
 * labelled in-batch rows and plain gradient descent with L2 weight decay
 * (Section 3, "L2 regularization is usually sufficient" for GCN).
 *
 *   p_ic       = exp(a_ic) / sum_c' exp(a_ic')
 *   loss_i     = -log p_{i, label_i}                (0 where label_i < 0)
 *   grad_ic    = scale * (p_ic - [c == label_i])    (0 where label_i < 0)
 * loss_sum = sum_i loss_i in double.
 */
void oracle_softmax_xent(const void* A, int64_t lda, int64_t n_rows, int32_t n_classes, int dt,
                         const int32_t* labels, double scale, float* loss_rows, double* loss_sum,
                         void* G, int64_t ldg) {
    double total = 0.0;
    for (int64_t i = 0; i < n_rows; ++i) {
        int32_t y = labels[i];
        if (y < 0) {
            loss_rows[i] = 0.f;
            for (int32_t c = 0; c < n_classes; ++c) store_elem(G, i * ldg + c, dt, 0.0);
            continue;
        }
        double amax = -INFINITY;
        for (int32_t c = 0; c < n_classes; ++c) {
            double a = load_elem(A, i * lda + c, dt);
            if (a > amax) amax = a;
        }
        double denom = 0.0;
        for (int32_t c = 0; c < n_classes; ++c) denom += exp(load_elem(A, i * lda + c, dt) - amax);
        double li = -(load_elem(A, i * lda + y, dt) - amax - log(denom));
        loss_rows[i] = (float)li;
        total += li;
        for (int32_t c = 0; c < n_classes; ++c) {
            double p = exp(load_elem(A, i * lda + c, dt) - amax) / denom;
            store_elem(G, i * ldg + c, dt, scale * (p - (c == y ? 1.0 : 0.0)));
        }
    }
    if (loss_sum) *loss_sum = total;
}

/* W <- W - lr * (dW + weight_decay * W), element-wise; dW is fp32, W is stored in dt. */
void oracle_sgd_step(void* W, int64_t n, int dt, const float* dW, double lr, double weight_decay) {
    for (int64_t i = 0; i < n; ++i) {
        double w = load_elem(W, i, dt);
        store_elem(W, i, dt, w - lr * ((double)dW[i] + weight_decay * w));
    }
}

/*
 * PNA's neighbourhood aggregation (paper, operator appendix): the tensor product of the scalers
 * [1, s(deg(v), 1), s(deg(v), -1)] with the aggregators [mean, min, max] over the neighbours of v, where
 * s(d, a) = (log(d + 1) / delta)^a and delta is the mean of log(deg + 1) over the graph (passed in).
 *
 *   agg_j[v] = add[v] + (mean | min | max)_{w in N(v)} X[w]      j = 0, 1, 2, element-wise
 *   out[v]   = [ agg_0, agg_1, agg_2,  s agg_0, s agg_1, s agg_2,  agg_0 / s, agg_1 / s, agg_2 / s ]
 *
 * with s = log(d_v + 1) / delta and d_v the number of entries of row v (all neighbours of an in-batch node are
 * in the batch subgraph, so this is its degree in the full graph).  `add` (optional) is the part of a message
 * that depends on the receiving node only and therefore commutes with all three aggregators.  A node without
 * neighbours receives no message: its nine blocks are zero.
 */
void oracle_pna_aggregate(const int32_t* rowptr, const int32_t* col, int64_t n_rows, const void* X, int64_t ldx,
                          int dt, int32_t F, const void* add, int64_t ldadd, double delta, void* out,
                          int64_t ldout) {
    #pragma omp parallel for schedule(dynamic, 64)
    for (int64_t v = 0; v < n_rows; ++v) {
        int64_t b = rowptr[v], e = rowptr[v + 1];
        double d = (double)(e - b);
        double s = log(d + 1.0) / delta;
        for (int32_t f = 0; f < F; ++f) {
            double agg[3] = {0.0, 0.0, 0.0};
            if (e > b) {
                double sum = 0.0, mn = INFINITY, mx = -INFINITY;
                for (int64_t k = b; k < e; ++k) {
                    double x = load_elem(X, (int64_t)col[k] * ldx + f, dt);
                    sum += x;
                    if (x < mn) mn = x;
                    if (x > mx) mx = x;
                }
                double q = add ? load_elem(add, v * ldadd + f, dt) : 0.0;
                agg[0] = sum / d + q;
                agg[1] = mn + q;
                agg[2] = mx + q;
            }
            for (int j = 0; j < 3; ++j) {
                store_elem(out, v * ldout + (int64_t)j * F + f, dt, agg[j]);
                store_elem(out, v * ldout + (int64_t)(3 + j) * F + f, dt, e > b ? s * agg[j] : 0.0);
                store_elem(out, v * ldout + (int64_t)(6 + j) * F + f, dt, e > b ? agg[j] / s : 0.0);
            }
        }
    }
}

/*
 * GAT's anisotropic aggregation (paper, operator appendix), one head: for every row v of the batch subgraph,
 * whose entries list N(v) and v itself,
 *     e_k      = LeakyReLU(a_dst . P[v] + a_src . P[col[k]])          (negative slope given)
 *     alpha_k  = exp(e_k) / sum_k' exp(e_k')                          (softmax over the row's entries)
 *     Z[v]     = sum_k alpha_k P[col[k]]          (followed by ReLU if asked: the activation between layers)
 * with P = H W computed beforehand for every node of V_b.  a = [a_dst, a_src] is the attention vector split into
 * the part that meets the receiving node and the part that meets the neighbour.  A row without entries gives
 * zeros.  Written as the definition: scores, their maximum, the normalised weights, the weighted sum.
 */
void oracle_gat_aggregate(const int32_t* rowptr, const int32_t* col, int64_t n_rows, const void* P, int64_t ldp,
                          int dt, int32_t F, const void* a_dst, const void* a_src, double negative_slope,
                          int relu, void* Z, int64_t ldz) {
    #pragma omp parallel for schedule(dynamic, 64)
    for (int64_t v = 0; v < n_rows; ++v) {
        int64_t b = rowptr[v], e = rowptr[v + 1];
        if (e == b) {
            for (int32_t f = 0; f < F; ++f) store_elem(Z, v * ldz + f, dt, 0.0);
            continue;
        }
        double sv = 0.0;
        for (int32_t f = 0; f < F; ++f) sv += load_elem(a_dst, f, dt) * load_elem(P, v * ldp + f, dt);
        double* score = (double*)malloc(sizeof(double) * (size_t)(e - b));
        double mx = -INFINITY;
        for (int64_t k = b; k < e; ++k) {
            double sw = 0.0;
            for (int32_t f = 0; f < F; ++f) sw += load_elem(a_src, f, dt) * load_elem(P, (int64_t)col[k] * ldp + f, dt);
            double x = sv + sw;
            x = x > 0.0 ? x : negative_slope * x;
            score[k - b] = x;
            if (x > mx) mx = x;
        }
        double den = 0.0;
        for (int64_t k = b; k < e; ++k) den += exp(score[k - b] - mx);
        for (int32_t f = 0; f < F; ++f) {
            double acc = 0.0;
            for (int64_t k = b; k < e; ++k)
                acc += exp(score[k - b] - mx) / den * load_elem(P, (int64_t)col[k] * ldp + f, dt);
            store_elem(Z, v * ldz + f, dt, (relu && acc < 0.0) ? 0.0 : acc);
        }
        free(score);
    }
}

/*
 * Backward of PNA's aggregation (chain rule on the aggregators of the operator appendix).  With, for a row v of d > 0
 * entries and s = log(d + 1) / delta,
 *     c_i[v, f] = G[v, i F + f] + s G[v, (3 + i) F + f] + G[v, (6 + i) F + f] / s     (i = mean, min, max),
 * the gradient of the added term is c_0 + c_1 + c_2, and the gradient of X receives, from every entry k of row v,
 * c_0 / d, plus c_1 where k is the FIRST entry of the row (in stored order) that attains the minimum of feature f,
 * plus c_2 where it is the first that attains the maximum (the subgradient that follows the aggregator's own choice).
 * GX has n_out rows (columns u < n_out of the pattern; entries into other columns are dropped, as for the sum
 * aggregation's adjoint); Gadd [n_rows, F] may be NULL.  Written as a scatter over the rows in double.
 */
void oracle_pna_aggregate_bwd(const int32_t* rowptr, const int32_t* col, int64_t n_rows, int64_t n_out, const void* X,
                              int64_t ldx, int dt, int32_t F, double delta, const void* G, int64_t ldg, void* GX,
                              int64_t ldgx, void* Gadd, int64_t ldga) {
    double* acc = (double*)calloc((size_t)(n_out > 0 ? n_out : 1) * (size_t)F, sizeof(double));
    for (int64_t v = 0; v < n_rows; ++v) {
        int64_t b = rowptr[v], e = rowptr[v + 1];
        double d = (double)(e - b);
        double s = log(d + 1.0) / delta;
        for (int32_t f = 0; f < F; ++f) {
            if (e == b) {
                if (Gadd) store_elem(Gadd, v * ldga + f, dt, 0.0);
                continue;
            }
            double c[3];
            for (int i = 0; i < 3; ++i)
                c[i] = load_elem(G, v * ldg + (int64_t)i * F + f, dt) + s * load_elem(G, v * ldg + (int64_t)(3 + i) * F + f, dt) +
                       load_elem(G, v * ldg + (int64_t)(6 + i) * F + f, dt) / s;
            int64_t kmin = b, kmax = b;
            double mn = INFINITY, mx = -INFINITY;
            for (int64_t k = b; k < e; ++k) {
                double x = load_elem(X, (int64_t)col[k] * ldx + f, dt);
                if (x < mn) { mn = x; kmin = k; }
                if (x > mx) { mx = x; kmax = k; }
            }
            for (int64_t k = b; k < e; ++k)
                if (col[k] < n_out) acc[(int64_t)col[k] * F + f] += c[0] / d;
            if (col[kmin] < n_out) acc[(int64_t)col[kmin] * F + f] += c[1];
            if (col[kmax] < n_out) acc[(int64_t)col[kmax] * F + f] += c[2];
            if (Gadd) store_elem(Gadd, v * ldga + f, dt, c[0] + c[1] + c[2]);
        }
    }
    for (int64_t u = 0; u < n_out; ++u)
        for (int32_t f = 0; f < F; ++f) store_elem(GX, u * ldgx + f, dt, acc[u * F + f]);
    free(acc);
}

/*
 * Backward of GAT's aggregation (chain rule on the operator appendix's equations; GZ is the gradient at the weighted
 * sum BEFORE any activation).  Per row v with scores t_k = a_dst . P[v] + a_src . P[col k], e_k = LeakyReLU(t_k),
 * alpha = softmax(e):
 *     dalpha_k = GZ[v] . P[col k],   de_k = alpha_k (dalpha_k - sum_j alpha_j dalpha_j),   dt_k = de_k * LeakyReLU'(t_k),
 *     GP[col k] += alpha_k GZ[v] + dt_k a_src,    GP[v] += (sum_k dt_k) a_dst,
 *     Ga_dst += (sum_k dt_k) P[v],                Ga_src += sum_k dt_k P[col k].
 * GP has n_out rows (rows u < n_out of P); Ga_dst, Ga_src: fp32 [F], over ALL entries.
 */
void oracle_gat_aggregate_bwd(const int32_t* rowptr, const int32_t* col, int64_t n_rows, int64_t n_out, const void* P,
                              int64_t ldp, int dt, int32_t F, const void* a_dst, const void* a_src,
                              double negative_slope, const void* GZ, int64_t ldgz, void* GP, int64_t ldgp,
                              float* Ga_dst, float* Ga_src) {
    double* acc = (double*)calloc((size_t)(n_out > 0 ? n_out : 1) * (size_t)F, sizeof(double));
    double* gd = (double*)calloc((size_t)F, sizeof(double));
    double* gs = (double*)calloc((size_t)F, sizeof(double));
    for (int64_t v = 0; v < n_rows; ++v) {
        int64_t b = rowptr[v], e = rowptr[v + 1], n = e - b;
        if (n == 0) continue;
        double* t = (double*)malloc(sizeof(double) * (size_t)n * 3);
        double *alpha = t + n, *dal = t + 2 * n;
        double sv = 0.0, mx = -INFINITY;
        for (int32_t f = 0; f < F; ++f) sv += load_elem(a_dst, f, dt) * load_elem(P, v * ldp + f, dt);
        for (int64_t k = 0; k < n; ++k) {
            double sw = 0.0, da = 0.0;
            for (int32_t f = 0; f < F; ++f) {
                double p = load_elem(P, (int64_t)col[b + k] * ldp + f, dt);
                sw += load_elem(a_src, f, dt) * p;
                da += load_elem(GZ, v * ldgz + f, dt) * p;
            }
            t[k] = sv + sw;
            dal[k] = da;
            double ek = t[k] > 0.0 ? t[k] : negative_slope * t[k];
            if (ek > mx) mx = ek;
        }
        double den = 0.0;
        for (int64_t k = 0; k < n; ++k) {
            double ek = t[k] > 0.0 ? t[k] : negative_slope * t[k];
            alpha[k] = exp(ek - mx);
            den += alpha[k];
        }
        double mean_da = 0.0;
        for (int64_t k = 0; k < n; ++k) { alpha[k] /= den; mean_da += alpha[k] * dal[k]; }
        double sum_dt = 0.0;
        for (int64_t k = 0; k < n; ++k) {
            double dtk = alpha[k] * (dal[k] - mean_da) * (t[k] > 0.0 ? 1.0 : negative_slope);
            sum_dt += dtk;
            int64_t c = col[b + k];
            for (int32_t f = 0; f < F; ++f) {
                double p = load_elem(P, c * ldp + f, dt);
                gs[f] += dtk * p;
                if (c < n_out) acc[c * F + f] += alpha[k] * load_elem(GZ, v * ldgz + f, dt) + dtk * load_elem(a_src, f, dt);
            }
        }
        for (int32_t f = 0; f < F; ++f) {
            gd[f] += sum_dt * load_elem(P, v * ldp + f, dt);
            if (v < n_out) acc[v * F + f] += sum_dt * load_elem(a_dst, f, dt);
        }
        free(t);
    }
    for (int64_t u = 0; u < n_out; ++u)
        for (int32_t f = 0; f < F; ++f) store_elem(GP, u * ldgp + f, dt, acc[u * F + f]);
    for (int32_t f = 0; f < F; ++f) { Ga_dst[f] = (float)gd[f]; Ga_src[f] = (float)gs[f]; }
    free(acc); free(gd); free(gs);
}

/*
 * Pieces of the auxiliary loss of the paper's Eq. (3), L_reg = || f(h) - f(h + eps) ||: the perturbed input
 * Y = X + alpha E (E holds the drawn perturbations, one row per node) and the Euclidean distance between the
 * rows of two layer outputs, dist[i] = || A[i, :] - B[i, :] ||_2, with its sum over the rows in double.
 */
void oracle_axpy(const void* X, int64_t ldx, const void* E, int64_t lde, int64_t n_rows, int32_t F, int dt,
                 double alpha, void* Y, int64_t ldy) {
    for (int64_t i = 0; i < n_rows; ++i)
        for (int32_t f = 0; f < F; ++f)
            store_elem(Y, i * ldy + f, dt, load_elem(X, i * ldx + f, dt) + alpha * load_elem(E, i * lde + f, dt));
}

void oracle_row_distance(const void* A, int64_t lda, const void* B, int64_t ldb, int64_t n_rows, int32_t F, int dt,
                         float* dist, double* dist_sum) {
    double total = 0.0;
    for (int64_t i = 0; i < n_rows; ++i) {
        double s = 0.0;
        for (int32_t f = 0; f < F; ++f) {
            double d = load_elem(A, i * lda + f, dt) - load_elem(B, i * ldb + f, dt);
            s += d * d;
        }
        s = sqrt(s);
        dist[i] = (float)s;
        total += s;
    }
    if (dist_sum) *dist_sum = total;
}

/*
 * Gradient of scale * sum_i ||A[i] - B[i]||_2 with respect to A (Eq. 3's distance; the gradient with respect to
 * B is its negative): row i is scale * (A[i] - B[i]) / ||A[i] - B[i]||_2, zero where the rows are equal.
 */
void oracle_row_distance_bwd(const void* A, int64_t lda, const void* B, int64_t ldb, int64_t n_rows, int32_t F, int dt,
                             double scale, void* G, int64_t ldg) {
    for (int64_t i = 0; i < n_rows; ++i) {
        double s = 0.0;
        for (int32_t f = 0; f < F; ++f) {
            double d = load_elem(A, i * lda + f, dt) - load_elem(B, i * ldb + f, dt);
            s += d * d;
        }
        s = sqrt(s);
        for (int32_t f = 0; f < F; ++f) {
            double d = load_elem(A, i * lda + f, dt) - load_elem(B, i * ldb + f, dt);
            store_elem(G, i * ldg + f, dt, s > 0.0 ? scale * d / s : 0.0);
        }
    }
}

