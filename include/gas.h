/*
 * gas.h - C ABI of the MI355X (gfx950) library for the GNNAutoScale (GAS)
 * mini-batch message-passing step with historical embeddings.
 *
 * One layer of the step, for a mini-batch B with halo V_b \ B (paper,
 * Algorithm 1 and Eq. 2):
 *     gas_pull    halo rows of the mini-batch tensor  <- history table rows
 *     gas_spmm    Z = aggregation over the rows of the batch subgraph G_b
 *     gas_linear  Y = dense transform of Z          (gas_mlp2 for GIN's MLP)
 *     gas_push    history table rows                <- fresh in-batch rows
 * and gas_spmm_t, the adjoint of the aggregation, for the backward pass.
 *
 * Conventions
 *   - Every data pointer is a DEVICE pointer owned by the caller.  The library
 *     neither frees nor keeps them.  The only library-owned memory is inside a
 *     gas_plan.
 *   - Matrices are row-major; "ld" is the row stride in ELEMENTS (ld >= F).
 *   - Indices are int32; byte offsets are computed in 64 bits, so tables
 *     larger than 4 GiB are fine.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Calls are asynchronous on it and never synchronise, with one exception:
 *     gas_plan_create and gas_validate_indices copy a little data to the host
 *     and wait for it.
 *   - Every call returns a gas_status; gas_last_error() gives a message for
 *     the last failure on the calling thread.  Arguments are checked on the
 *     host before anything is launched; a failed call launches nothing.
 *   - Index VALUES are not range-checked on the hot path (an out-of-range
 *     index is undefined behaviour); gas_validate_indices checks them.
 *   - Rows whose base address and byte stride are multiples of 16 take the
 *     128-bit path; anything else falls back to an element-wise path with
 *     identical results.
 *   - Reductions use no atomics and a fixed order: results are bit-identical
 *     from run to run for the same inputs and the same plan.
 */
#ifndef GAS_H
#define GAS_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Exported symbol (the library is built with hidden default visibility). */
#define GAS_API __attribute__((visibility("default")))

typedef enum { GAS_F32 = 0, GAS_BF16 = 1 } gas_dtype;

typedef enum {
    GAS_OK = 0,
    GAS_ERR_ARG = -1,    /* null pointer, negative size, ld < F, ... */
    GAS_ERR_DTYPE = -2,  /* unknown or unsupported dtype combination */
    GAS_ERR_RANGE = -4,  /* gas_validate_indices found an index out of range */
    GAS_ERR_HIP = -5,    /* a HIP runtime call failed */
    GAS_ERR_NOMEM = -6,  /* device allocation for a plan failed */
    GAS_ERR_IO = -7      /* a file of a history table on disk could not be opened, sized, read or written */
} gas_status;

/* Message of the last failure on this thread (static storage, never NULL). */
GAS_API const char* gas_last_error(void);

/* Library version, major*10000 + minor*100 + patch. */
GAS_API int gas_version(void);

/*
 * Pull (Algorithm 1: h_w <- Pull(w) for all w in V_b \ B_b).
 *     dst[i, 0:F] = hist[r(i), 0:F],  i in [0, n),
 *     r(i) = idx[i] if idx != NULL else base + i.
 * hist:  [n_hist_rows, F] table, row stride ld_hist.  dst: [n, F], stride ld_dst.
 * idx:   int32[n] global node ids (duplicates allowed), or NULL for the
 *        contiguous range starting at `base` (`base` is ignored otherwise).
 * The first layer's input is the same call on the feature table.
 * Pure data movement: the result is bit-exact.  n == 0 is a no-op.
 */
GAS_API gas_status gas_pull(const void* hist, int64_t n_hist_rows, int64_t ld_hist,
                    const int32_t* idx, int64_t base, int64_t n, int32_t F, gas_dtype dt,
                    void* dst, int64_t ld_dst, void* stream);

/*
 * Push (Algorithm 1: Push(h_v) for all v in B_b).
 *     hist[r(i), 0:F] = src[i, 0:F],  i in [0, n),  r(i) as in gas_pull.
 * idx must hold DISTINCT ids (a mini-batch is a set of nodes); duplicates
 * are undefined behaviour.  Rows of hist not named by idx are not touched.
 */
GAS_API gas_status gas_push(const void* src, int64_t ld_src,
                    const int32_t* idx, int64_t base, int64_t n, int32_t F, gas_dtype dt,
                    void* hist, int64_t n_hist_rows, int64_t ld_hist, void* stream);

/*
 * Edge coefficients of the GCN operator (operator appendix, GCN):
 *     val[k] = 1 / ( sqrt(deg[n_id[ind[k]]] + 1) * sqrt(deg[n_id[r]] + 1) )
 * for every stored entry k of row r of a compressed sparse pattern (ptr, ind)
 * with n_rows rows.  deg holds the degrees of the FULL graph, indexed by
 * global id; n_id maps local ids to global ids.  Evaluated in fp64 and rounded
 * once to fp32.  The formula is symmetric, so the same call serves the CSR and
 * the CSC copy of a batch subgraph.
 */
GAS_API gas_status gas_gcn_norm(const int32_t* ptr, const int32_t* ind, int64_t n_rows,
                        const int32_t* n_id, const int32_t* deg, float* val, void* stream);

/*
 * Schedule for one compressed sparse pattern (groups of light rows, chunk
 * lists of the heavy rows, partial-sum workspace).  Built once per batch
 * subgraph (Algorithm 1 builds G_b once per batch) and reused by every layer
 * and every epoch; one plan for the CSR, one for the CSC copy.  ptr is a device
 * pointer (int32[n_rows+1]); ind (device, int32[nnz], each row ascending) may
 * be NULL; when given it is used to cut and order the chunks of heavy rows by
 * L2-sized windows of the rows they gather, and to see whether the pattern is clustered (most entries of a row
 * name rows near it, as in a batch of partition clusters): then each of the
 * eight XCDs is given one contiguous range of light rows, so a cluster is
 * gathered into one L2 instead of eight.  Either the local column ids or the
 * source indices of gas_fuse_sources may be passed.  The plan is built by
 * kernels on `stream`; a few counters are read back, so the call waits for the
 * stream (twice); ptr is validated
 * (0 = ptr[0] <= ptr[r] <= ptr[r+1] <= ptr[n_rows] = nnz, else GAS_ERR_ARG).
 * max_F is the widest feature dimension the plan will be used with (sizes the
 * workspace and the windows).  A plan must not be used by two streams at the
 * same time.
 *
 * gas_plan_create_opt takes the schedule's parameters explicitly (NULL or a
 * zero field = the default): rows with more than heavy_threshold entries
 * (512) are cut into chunks of at most `chunk` entries (256) that end at a
 * window boundary once they hold min_chunk entries (32); window_rows = rows of
 * the gathered table per window (default: 2 MiB worth of rows of max_F floats,
 * rounded down to a power of two; -1 = no windows); xcd_ranges: 0 = decide
 * from the pattern, 1 = always, 2 = never.  The parameters change which
 * wavefront sums what, never the set of terms: results agree to rounding
 * between parameter sets and are bit-identical for one set.
 */
typedef struct gas_plan gas_plan;
typedef struct {
    int32_t heavy_threshold;
    int32_t chunk;
    int32_t min_chunk;
    int32_t window_rows;
    int32_t xcd_ranges;
    int32_t host_builder;   /* 1: build the plan on the host from copies of ptr and ind (slow; the reference the
                               device builder is tested against: both give the same lists) */
} gas_plan_options;
GAS_API gas_status gas_plan_create(const int32_t* ptr, const int32_t* ind, int64_t n_rows, int64_t nnz,
                           int32_t max_F, void* stream, gas_plan** out);
GAS_API gas_status gas_plan_create_opt(const int32_t* ptr, const int32_t* ind, int64_t n_rows, int64_t nnz,
                               int32_t max_F, const gas_plan_options* opt, void* stream, gas_plan** out);
GAS_API void gas_plan_destroy(gas_plan* plan);

/*
 * Inspection of a plan (tests, tools).  gas_plan_describe: info[0..15] = n_rows, nnz, number of groups of light
 * rows, of heavy rows, of chunks, whether the XCD ranges are used, max_F, then the nine range boundaries (in
 * groups).  gas_plan_copy_lists copies the plan's lists to HOST buffers (any may be NULL): group int32[2 * groups]
 * (first and end row), heavy int32[2 * heavy + 1] (row ids, then the first chunk slot of each and the end), chunk
 * int32[3 * chunks] (slot, first entry, end entry, in processing order); waits for `stream`.
 */
GAS_API gas_status gas_plan_describe(const gas_plan* plan, int64_t info[16]);
GAS_API gas_status gas_plan_copy_lists(const gas_plan* plan, int32_t* group, int32_t* heavy, int32_t* chunk,
                               void* stream);

/*
 * Aggregation over the batch subgraph (Eq. 1 / Eq. 2 with the operators of the
 * operator appendix), rows = in-batch nodes, columns = in-batch nodes followed
 * by halo nodes:
 *     Z[v, :] = s_agg * sum_{k in row v} val[k] * X[col[k], :]
 *               + diag * X[v, :] + s_res * R[v, :],          v in [0, n_rows)
 * where n_rows is the row count the plan was created with.
 * GCN:   val = 1/c (self-loop stored as an entry), diag = 0, s_agg = 1, R = NULL.
 * GIN:   val = NULL (all ones), diag = 1 + eps.
 * GCNII: s_agg = 1 - alpha, R = initial embedding of the in-batch nodes, s_res = alpha.
 * rowptr int32[n_rows+1], col int32[nnz] (local ids), val fp32[nnz] or NULL.
 * X: [>= max(col)+1, F] of type dt_x; R (optional): [n_rows, F] of type dt_x;
 * Z: [n_rows, F] of type dt_z.  Accumulation is fp32 in a fixed order; bf16
 * outputs are rounded to nearest even.  `plan` must have been created from
 * this rowptr.  Z must not alias X or R.
 */
GAS_API gas_status gas_spmm(const gas_plan* plan, const int32_t* rowptr, const int32_t* col,
                    const float* val, float diag,
                    const void* X, int64_t ldx, gas_dtype dt_x, int32_t F,
                    float s_agg, const void* R, int64_t ldr, float s_res,
                    void* Z, int64_t ldz, gas_dtype dt_z, void* stream);

/*
 * Aggregation with the historical embeddings read in place (Eq. 2, line 3:
 * in-batch neighbours contribute their fresh embeddings, out-of-batch
 * neighbours their stored ones).  Same sum, same order and bit-identical
 * result as gas_pull of the halo rows followed by gas_spmm, without writing
 * and re-reading the halo rows of the mini-batch tensor.
 * src int32[nnz] replaces col: src[k] >= 0 is a row of X (an in-batch node,
 * X is [n_rows, F]); src[k] < 0 names row -1-src[k] of the history table
 * hist [n_hist_rows, F] (same dtype as X).  gas_fuse_sources builds src.
 * diag, s_agg, R, s_res, Z, plan as in gas_spmm.
 */
GAS_API gas_status gas_spmm_hist(const gas_plan* plan, const int32_t* rowptr, const int32_t* src,
                         const float* val, float diag,
                         const void* X, int64_t ldx,
                         const void* hist, int64_t n_hist_rows, int64_t ld_hist, gas_dtype dt_x, int32_t F,
                         float s_agg, const void* R, int64_t ldr, float s_res,
                         void* Z, int64_t ldz, gas_dtype dt_z, void* stream);

/*
 * Source indices for gas_spmm_hist from the local column ids of a batch
 * subgraph: src[k] = col[k] if col[k] < nb (in-batch), else -1 - n_id[col[k]]
 * (global id of the halo node, i.e. its row in every history table).  Done
 * once per batch; the result serves every layer.  src is caller-owned, int32[nnz].
 */
GAS_API gas_status gas_fuse_sources(const int32_t* col, int64_t nnz, int64_t nb, const int32_t* n_id,
                            int32_t* src, void* stream);

/*
 * Backward aggregation: the adjoint of gas_spmm's sum, computed as a
 * row-parallel product over the CSC copy of the same pattern (no atomics):
 *     GX[u, :] = s_agg * sum_{k in column u} val[k] * G[row[k], :] + [u < n_diag] diag * G[u, :]
 * for u in [0, n_out), n_out being the row count of the plan.  colptr
 * int32[n_out+1], row int32[nnz], val in CSC order.  n_out = number of
 * in-batch nodes when gradients into halo rows are not needed (histories are
 * constants), or all of V_b.  n_diag = number of
 * rows of G (the diagonal term exists for in-batch nodes only).
 * `plan` must have been created from colptr[0 .. n_out].
 */
GAS_API gas_status gas_spmm_t(const gas_plan* plan, const int32_t* colptr, const int32_t* row,
                      const float* val, float diag, float s_agg, int64_t n_diag,
                      const void* G, int64_t ldg, gas_dtype dt_g, int32_t F,
                      void* GX, int64_t ldgx, gas_dtype dt_gx, void* stream);

/*
 * Dense transform of the GCN / GCNII operators:
 *     Y = act( c_identity * Z + c_weight * (Z W) + bias )
 * Z [n_rows, F_in], W [F_in, F_out] row-major contiguous, bias [F_out] or NULL,
 * all of type dt; Y [n_rows, F_out] of type dt.  GCN: c_identity = 0,
 * c_weight = 1.  GCNII's identity map W <- (1-beta) I + beta W: c_identity =
 * 1 - beta, c_weight = beta (then F_in must equal F_out).  relu != 0 applies
 * max(0, .).  Runs on the matrix cores: fp32 MFMA for GAS_F32; bf16 MFMA with
 * fp32 accumulation for GAS_BF16.  Y must not alias Z.
 */
GAS_API gas_status gas_linear(const void* Z, int64_t ldz, int64_t n_rows, int32_t F_in,
                      const void* W, int32_t F_out, const void* bias, gas_dtype dt,
                      float c_identity, float c_weight, int relu,
                      void* Y, int64_t ldy, void* stream);

/*
 * GIN update (operator appendix, GIN): Y = act( relu(Z W1 + b1) W2 + b2 ),
 * both products in one kernel; the hidden activation never leaves the chip
 * (kept in fp32 for GAS_F32, rounded to bf16 for GAS_BF16).
 * W1 [F_in, F_hid], W2 [F_hid, F_out]; F_hid <= 256.
 */
GAS_API gas_status gas_mlp2(const void* Z, int64_t ldz, int64_t n_rows, int32_t F_in,
                    const void* W1, int32_t F_hid, const void* b1,
                    const void* W2, int32_t F_out, const void* b2, gas_dtype dt,
                    int relu_out, void* Y, int64_t ldy, void* stream);

/*
 * Transform with the Push fused into its epilogue (Algorithm 1: compute the
 * layer for the in-batch nodes, Push the result): same as gas_linear /
 * gas_mlp2, and every output row i is also stored to hist[idx[i], 0:F_out]
 * (idx int32[n_rows], distinct; hist [n_hist_rows, F_out] of type dt, row stride
 * ld_hist).  Y is written as well (it is the next layer's input).  Same bits as
 * the unfused call followed by gas_push; the output is not re-read.
 */
GAS_API gas_status gas_linear_push(const void* Z, int64_t ldz, int64_t n_rows, int32_t F_in,
                           const void* W, int32_t F_out, const void* bias, gas_dtype dt,
                           float c_identity, float c_weight, int relu, void* Y, int64_t ldy,
                           const int32_t* idx, void* hist, int64_t n_hist_rows, int64_t ld_hist, void* stream);
GAS_API gas_status gas_mlp2_push(const void* Z, int64_t ldz, int64_t n_rows, int32_t F_in,
                         const void* W1, int32_t F_hid, const void* b1,
                         const void* W2, int32_t F_out, const void* b2, gas_dtype dt,
                         int relu_out, void* Y, int64_t ldy,
                         const int32_t* idx, void* hist, int64_t n_hist_rows, int64_t ld_hist, void* stream);

/*
 * The GIN update for a training pass: gas_mlp2_push (idx == NULL and hist == NULL: no Push) which also stores the
 * hidden activation relu(Z W1 + b1) to H_out [n_rows, F_hid] (type dt, row stride ldh_out): the backward pass reads
 * it (weight gradient of W2, ReLU mask).  Where the fused kernel applies (bf16, widths up to 256, 16-byte aligned
 * rows, at least 4096 rows) the hidden tile is stored from LDS on its way; elsewhere the call runs as two stored
 * linears.  H_out must not alias Z or Y.
 */
GAS_API gas_status gas_mlp2_keep(const void* Z, int64_t ldz, int64_t n_rows, int32_t F_in,
                         const void* W1, int32_t F_hid, const void* b1,
                         const void* W2, int32_t F_out, const void* b2, gas_dtype dt,
                         int relu_out, void* Y, int64_t ldy, void* H_out, int64_t ldh_out,
                         const int32_t* idx, void* hist, int64_t n_hist_rows, int64_t ld_hist, void* stream);

/*
 * One whole layer in one launch, for narrow layers (Algorithm 1's loop body
 * for the in-batch nodes: aggregate over G_b with both sources of Eq. 2,
 * transform, Push):
 *     Z[v, :] = s_agg * sum_k val[k] * S(src[k]) + diag * X[v, :] + s_res * R[v, :]
 *     Y[v, :] = act( c_identity * Z[v, :] + c_weight * (Z W)[v, :] + bias )
 *     push_hist[push_idx[v], :] = Y[v, :]                (if push_idx != NULL)
 * with S(s) = X[s, :] for s >= 0 and hist[-1-s, :] for s < 0, exactly as in
 * gas_spmm_hist (hist may be NULL when no index is negative: then src is the
 * plain column array and X the whole mini-batch tensor) and the transform of
 * gas_linear.  The aggregated tile stays on the chip; Z is written only if
 * Z_out != NULL ([n_rows, F_in], row stride ldz_out: a training pass reads it
 * again for the weight gradient).
 * Needs no plan.  Meant for deep narrow models (the 64-layer GCNII of the
 * paper's experiments), which are bound by launches: rows of any length are
 * handled, but long rows are not split, so wide or heavy-tailed layers should
 * use gas_spmm_hist + gas_linear_push.
 * Restrictions: GAS_F32 only (GAS_ERR_DTYPE otherwise); F_in and F_out
 * multiples of 4, at most 128; X, hist, R, W, Z_out 16-byte aligned with row strides
 * that are multiples of 4 elements (GAS_ERR_ARG otherwise, nothing is
 * launched).  val may be NULL (all ones), R and bias may be NULL.  Results are
 * deterministic (fixed summation order) and agree with the two-call form to
 * rounding (the order of the row sum differs).
 */
GAS_API gas_status gas_spmm_linear(const int32_t* rowptr, const int32_t* src, const float* val, int64_t n_rows,
                           const void* X, int64_t ldx, const void* hist, int64_t n_hist_rows, int64_t ld_hist,
                           gas_dtype dt, int32_t F_in, float diag, float s_agg,
                           const void* R, int64_t ldr, float s_res,
                           const void* W, int32_t F_out, const void* bias,
                           float c_identity, float c_weight, int relu, void* Y, int64_t ldy,
                           void* Z_out, int64_t ldz_out,
                           const int32_t* push_idx, void* push_hist, int64_t n_push_rows, int64_t ld_push,
                           void* stream);

/*
 * Backward pass of the transform (chain rule on the operator equations; the
 * paper takes gradients through its layers, Section 2 advantage (1), without
 * spelling them out).  With P = c_identity * Z + c_weight * (Z W) and Y = relu(P):
 *
 * gas_relu_bwd:            GP = GY where Y > 0, else 0 (element-wise; GP may alias GY).
 * gas_linear_bwd_input:    GZ = c_identity * GP + c_weight * (GP W^T), then, if mask != NULL,
 *                          GZ = 0 where mask <= 0 (mask [n_rows, F_in] is the hidden
 *                          activation of a GIN MLP: the ReLU between its two linears).
 *                          GP [n_rows, F_out], W [F_in, F_out] as in gas_linear, GZ [n_rows, F_in].
 * gas_linear_bwd_weight:   dW [F_in, F_out] fp32 = c_weight * Z^T GP.  The sum over the rows
 *                          is formed in slabs of rows whose partial results go to
 *                          `workspace` (device memory, at least
 *                          gas_linear_bwd_weight_workspace(n_rows, F_in, F_out) bytes, caller-
 *                          owned, contents undefined afterwards) and are added in slab order:
 *                          no atomics, bit-identical from run to run.
 * All matrices have type dt except dW (fp32).  Products run on the matrix cores.
 */
GAS_API gas_status gas_relu_bwd(const void* GY, int64_t ldgy, const void* Y, int64_t ldy, int64_t n_rows,
                        int32_t F, gas_dtype dt, void* GP, int64_t ldgp, void* stream);
GAS_API gas_status gas_linear_bwd_input(const void* GP, int64_t ldgp, int64_t n_rows, int32_t F_out,
                                const void* W, int32_t F_in, gas_dtype dt, float c_identity, float c_weight,
                                const void* mask, int64_t ldmask, void* GZ, int64_t ldgz, void* stream);
GAS_API int64_t gas_linear_bwd_weight_workspace(int64_t n_rows, int32_t F_in, int32_t F_out);
GAS_API gas_status gas_linear_bwd_weight(const void* Z, int64_t ldz, const void* GP, int64_t ldgp,
                                 int64_t n_rows, int32_t F_in, int32_t F_out, gas_dtype dt, float c_weight,
                                 float* dW, void* workspace, int64_t workspace_bytes, void* stream);

/*
 * gas_linear_bwd_weight for callers that cannot allocate or pass a workspace:
 * code under HIP graph capture, tight serving or training loops, harnesses that
 * forbid hipMalloc.  Same kernels, same slabs and the same bits as
 * gas_linear_bwd_weight, with the slab partials kept in a static device array of
 * the library (64 MiB on every GPU the library runs on, held until the process
 * ends) instead of a caller's workspace.  Calls no hipMalloc, hipFree or other
 * allocating routine.  Shapes whose partials exceed the array
 * (gas_linear_bwd_weight_workspace(n_rows, F_in, F_out) > 64 MiB; at widths
 * 256 x 256 that is above 1,048,576 rows) are rejected with GAS_ERR_ARG and
 * nothing is launched.  All calls on one GPU share that GPU's array: calls that
 * overlap in time on one GPU (two streams, two threads) race; calls on one
 * stream are ordered and safe.  Every partial a call reads it has written
 * itself, so nothing needs clearing between calls.
 */
GAS_API gas_status gas_linear_bwd_weight_static(const void* Z, int64_t ldz, const void* GP, int64_t ldgp,
                                        int64_t n_rows, int32_t F_in, int32_t F_out, gas_dtype dt, float c_weight,
                                        float* dW, void* stream);

/*
 * Loss of a mini-batch and the parameter update that close the loop body of
 * Algorithm 1 (the loss is taken over the in-batch nodes only, Section 1; the
 * paper's tasks are node classification; Section 3 names L2 regularisation).
 *
 * gas_softmax_xent: for every row i with 0 <= labels[i] < n_classes
 *     p_ic = softmax(A[i, :])_c,  loss_rows[i] = -log p_{i, labels[i]},
 *     G[i, c] = scale * (p_ic - [c == labels[i]]);
 * rows with a label outside that range (-1 = unlabelled) get loss 0 and a zero
 * gradient row.  A, G: [n_rows, n_classes] of type dt (device), G != A;
 * labels int32[n_rows]; loss_rows fp32[n_rows]; loss_sum: optional fp32[1],
 * receives the sum of loss_rows added in a fixed order (double accumulation).
 * Arithmetic in fp32.
 *
 * gas_sgd_step: W[i] <- W[i] - lr * (dW[i] + weight_decay * W[i]) for the n
 * contiguous elements of W (type dt, device); dW fp32[n] (as written by
 * gas_linear_bwd_weight).
 */
GAS_API gas_status gas_softmax_xent(const void* A, int64_t lda, int64_t n_rows, int32_t n_classes, gas_dtype dt,
                            const int32_t* labels, float scale, float* loss_rows, float* loss_sum,
                            void* G, int64_t ldg, void* stream);
GAS_API gas_status gas_sgd_step(void* W, int64_t n, gas_dtype dt, const float* dW, float lr, float weight_decay,
                        void* stream);

/*
 * Gradient clipping by the global norm (Section 3 of the paper: clipping keeps
 * the parameters, and so the histories, from changing too fast).
 * gas_sq_norm: out[0] = sum of x[i]^2, i in [0, n) (fp64 accumulation in a
 * fixed order, one fp32 result); called once per gradient of the step, the
 * results side by side in one float array.
 * gas_sgd_step_clipped: gas_sgd_step with every gradient multiplied by
 *     c = min(1, max_norm / (sqrt(sum_k sq_norms[k]) + 1e-6)),
 * sq_norms (device, float[n_norms]) holding the squared norms of ALL gradients
 * of the step, so that the same c is applied to every weight matrix; c is
 * formed on the device (nothing is read back).  max_norm > 0.
 */
GAS_API gas_status gas_sq_norm(const float* x, int64_t n, float* out, void* stream);
GAS_API gas_status gas_sgd_step_clipped(void* W, int64_t n, gas_dtype dt, const float* dW, float lr,
                                float weight_decay, const float* sq_norms, int32_t n_norms, float max_norm,
                                void* stream);

/*
 * PNA's neighbourhood aggregation (operator appendix): for every row v of the
 * batch subgraph, in one pass over the gathered rows,
 *     agg_0 = mean, agg_1 = min, agg_2 = max  over X[col[k], 0:F], k in row v,
 *     each plus add[v, 0:F] if add is given (the part of a message that depends
 *     on the receiving node only),
 * and out[v] = [agg_0 agg_1 agg_2 | s agg_0 .. | agg_0 / s ..] (9 F columns),
 * s = log(d_v + 1) / delta, d_v = rowptr[v+1] - rowptr[v]; delta > 0 is the
 * mean of log(deg + 1) over the graph.  Rows without entries give zeros.
 * rowptr int32[n_rows+1], col int32[nnz] in range of X's rows; X, add, out of
 * type dt (device), out must not alias them.  Deterministic: which lane folds
 * which entry depends on the row's length and on F alone (rows of at most 64
 * pieces of 16 bytes are shared by teams of lanes, rows above 2,048 entries by
 * the wavefronts of a workgroup, folded in a fixed order).
 */
GAS_API gas_status gas_pna_aggregate(const int32_t* rowptr, const int32_t* col, int64_t n_rows,
                             const void* X, int64_t ldx, gas_dtype dt, int32_t F,
                             const void* add, int64_t ldadd, float delta,
                             void* out, int64_t ldout, void* stream);

/*
 * GAT's anisotropic aggregation (operator appendix), one head: for every row
 * v of the batch subgraph (its entries list N(v) and v itself),
 *     e_k = LeakyReLU(a_dst . P[v] + a_src . P[col[k]])  (negative_slope),
 *     Z[v] = act(sum_k softmax_k(e)_k P[col[k]]),  act = ReLU if relu != 0,
 * P = H W [n_cols, F] computed beforehand (rows 0..n_rows-1 are the in-batch
 * nodes); a_dst, a_src: the two halves of the attention vector, [F] of type
 * dt.  Scores, softmax and the weighted sum take one pass over the gathered
 * rows (fp32 arithmetic; running maxima and sums kept per team of lanes, and
 * per wavefront for rows above 2,048 entries, merged in a fixed order that
 * depends on the row's length and on F alone: deterministic).
 * Rows without entries give zeros.  F <= 1024.  Z must not alias P.
 */
GAS_API gas_status gas_gat_aggregate(const int32_t* rowptr, const int32_t* col, int64_t n_rows,
                             const void* P, int64_t ldp, gas_dtype dt, int32_t F,
                             const void* a_dst, const void* a_src, float negative_slope, int relu,
                             void* Z, int64_t ldz, void* stream);

/*
 * Backward passes of the two aggregations above (chain rule on the equations of the operator appendix), without
 * floating-point atomics: a pass over the rows of the pattern leaves per-row / per-entry factors in `workspace`, a pass over the
 * columns (the CSC copy: colptr int32[n_cols+1], row int32[nnz], and csc_pos int32[nnz] = the position of every CSC
 * entry in the CSR arrays) sums each column's contributions in stored order.  n_out <= n_cols output rows are
 * written (the in-batch nodes when histories are constants, or all of V_b).  workspace: device memory of at least
 * gas_*_bwd_workspace(...) bytes, caller-owned, contents undefined afterwards.
 * plan_t: a plan of the CSC copy for exactly the n_out output rows, gas_plan_create(colptr, colptr[n_out], max_F >= F,
 * n_out, row), or NULL.  With it, and rows of at most 64 pieces of 16 bytes that are 16-byte aligned, the row pass
 * gathers like the forward call and the sum of whole rows over a column's entries is taken by gas_spmm_t's kernels
 * (which rounds it to the storage type before the remaining terms are added: one more rounding for bf16).  Without
 * it, or for other shapes, plain kernels run: one wavefront per row and per column, one entry at a time; slow, and
 * the definition the fast path is tested against.  Fixed summation order either way (not the same order: the two
 * paths agree to rounding).  The plan's partial-sum workspace is in use during the call, as in gas_spmm_t.
 *
 * gas_pna_aggregate_bwd: G [n_rows, 9 F] is the gradient of gas_pna_aggregate's output.  With s and d as there and
 *     c_i = G[v, i F + f] + s G[v, (3+i) F + f] + G[v, (6+i) F + f] / s   (i = mean, min, max; rows with entries),
 * Gadd[v] = c_0 + c_1 + c_2 (optional, [n_rows, F]) and GX[u] receives from every entry (v, u): c_0 / d, plus c_1
 * where the entry is the FIRST of row v (in stored order) attaining the minimum of that feature, plus c_2 for the
 * maximum.  colptr needs n_out + 1 entries.
 *
 * gas_gat_aggregate_bwd: GZ [n_rows, F] is the gradient at the weighted sum BEFORE any activation (apply
 * gas_relu_bwd first when the forward call had relu set).  Per row v, with t_k, alpha_k as in gas_gat_aggregate:
 *     dalpha_k = GZ[v] . P[col k],  dt_k = alpha_k (dalpha_k - sum_j alpha_j dalpha_j) LeakyReLU'(t_k),
 *     GP[col k] += alpha_k GZ[v] + dt_k a_src,   GP[v] += (sum_k dt_k) a_dst,
 *     Ga_dst = sum_v (sum_k dt_k) P[v],          Ga_src = sum over all entries of dt_k P[col k]   (fp32 [F]).
 * n_cols = rows of P = columns of the pattern (the column pass runs over all of them: Ga_src needs every entry).
 */
GAS_API int64_t gas_pna_aggregate_bwd_workspace(int64_t n_rows, int64_t nnz, int32_t F);
GAS_API gas_status gas_pna_aggregate_bwd(const gas_plan* plan_t, const int32_t* rowptr, const int32_t* col, int64_t n_rows,
                                 int64_t nnz, const int32_t* colptr, const int32_t* row, const int32_t* csc_pos, int64_t n_out,
                                 const void* X, int64_t ldx, gas_dtype dt, int32_t F, float delta,
                                 const void* G, int64_t ldg, void* GX, int64_t ldgx, void* Gadd, int64_t ldga,
                                 void* workspace, int64_t workspace_bytes, void* stream);
GAS_API int64_t gas_gat_aggregate_bwd_workspace(int64_t n_rows, int64_t n_cols, int64_t nnz, int32_t F);
GAS_API gas_status gas_gat_aggregate_bwd(const gas_plan* plan_t, const int32_t* rowptr, const int32_t* col, int64_t n_rows,
                                 const int32_t* colptr, const int32_t* row, const int32_t* csc_pos, int64_t n_cols,
                                 int64_t n_out, int64_t nnz, const void* P, int64_t ldp, gas_dtype dt, int32_t F,
                                 const void* a_dst, const void* a_src, float negative_slope,
                                 const void* GZ, int64_t ldgz, void* GP, int64_t ldgp, float* Ga_dst, float* Ga_src,
                                 void* workspace, int64_t workspace_bytes, void* stream);

/*
 * Pieces of the auxiliary loss of Eq. (3), || f(h) - f(h + eps) ||, which is
 * a second forward pass of a layer on a perturbed input:
 * gas_axpy:          Y = X + alpha E, element-wise over [n_rows, F] of type dt
 *                    (E: the drawn perturbations, one row per node; Y may be X);
 * gas_row_distance:  dist[i] = || A[i, :] - B[i, :] ||_2 (fp32[n_rows]), and,
 *                    if dist_sum is given (fp32[1]), their sum in a fixed order.
 */
GAS_API gas_status gas_axpy(const void* X, int64_t ldx, const void* E, int64_t lde, int64_t n_rows, int32_t F,
                    gas_dtype dt, float alpha, void* Y, int64_t ldy, void* stream);
GAS_API gas_status gas_row_distance(const void* A, int64_t lda, const void* B, int64_t ldb, int64_t n_rows,
                            int32_t F, gas_dtype dt, float* dist, float* dist_sum, void* stream);

/*
 * Row-wise inner products: dot[i] = sum_f A[i, f] * B[i, f] (fp32[n_rows], fp32 accumulation), and, if dot_sum is
 * given (fp32[1]), their sum in a fixed order (double accumulation).  With A the gradient at a GIN layer's
 * aggregated rows and B the layer's in-batch input rows, dot_sum is the gradient of that layer's eps (operator
 * appendix, GIN: the self term is (1 + eps) h_v and eps is trainable, so dL/d eps = sum_v <dL/dZ_v, h_v>).
 * A, B: [n_rows, F] of type dt.
 */
GAS_API gas_status gas_row_dot(const void* A, int64_t lda, const void* B, int64_t ldb, int64_t n_rows,
                       int32_t F, gas_dtype dt, float* dot, float* dot_sum, void* stream);

/*
 * Gradient of the distance of Eq. (3): G[i, :] = scale * (A[i, :] - B[i, :]) / ||A[i, :] - B[i, :]||_2, zero where
 * the two rows are equal; this is d/dA of scale * sum_i ||A[i] - B[i]||_2, and d/dB is its negative.  A, B, G:
 * [n_rows, F] of type dt.  With it the regulariser's gradient with respect to a layer's weights is two passes of
 * the layer's backward calls (one per evaluation, output gradients G and -G).
 */
GAS_API gas_status gas_row_distance_bwd(const void* A, int64_t lda, const void* B, int64_t ldb, int64_t n_rows,
                                int32_t F, gas_dtype dt, float scale, void* G, int64_t ldg, void* stream);

/*
 * Histories outside HBM (the paper keeps them in host memory and overlaps
 * the transfers with computation, Section 5 "PyGAS"): gas_pull and gas_push accept a
 * table in pinned host memory once its device-side address is known; the
 * copy kernel then moves the rows over the host link itself, with no staging
 * copy and no host thread, and overlaps with other work when launched on a
 * stream of its own.  gas_host_table_pointer returns that address for memory
 * allocated with hipHostMalloc (torch's pin_memory), or GAS_ERR_ARG if the
 * device cannot address it (never pass such a pointer to a kernel).
 * gas_pull_host / gas_push_host: gas_pull / gas_push with `hist` such an
 * address; same arguments and result, launched on a small grid (the host
 * link needs few requests in flight) so that kernels of other streams keep
 * the compute units.
 */
GAS_API gas_status gas_host_table_pointer(const void* host_ptr, void** device_ptr);
GAS_API gas_status gas_pull_host(const void* hist, int64_t n_hist_rows, int64_t ld_hist,
                         const int32_t* idx, int64_t base, int64_t n, int32_t F, gas_dtype dt,
                         void* dst, int64_t ld_dst, void* stream);
GAS_API gas_status gas_push_host(const void* src, int64_t ld_src, const int32_t* idx, int64_t base,
                         int64_t n, int32_t F, gas_dtype dt,
                         void* hist, int64_t n_hist_rows, int64_t ld_hist, void* stream);

/*
 * Histories on disk (the paper's "Conclusion and Future Work" names disk
 * storage as the tier behind host memory; the transfers follow the scheme of
 * its Section 5 "PyGAS": rows are gathered into pinned buffers by host
 * threads, copied beside the computation, and a layer waits only for its
 * own rows).  A gas_disk_table is a file of n_rows x F elements of type dt,
 * row after row, nothing else in it (rows never written read as zeros), with
 * I/O threads, two pinned staging buffers, a copy stream at the default
 * priority and one worker thread that runs the table's transfers in the
 * order they were queued.
 *
 * gas_disk_open:  flags: GAS_DISK_CREATE makes (or empties) the file and
 *                 sizes it; without it the file must exist with exactly the
 *                 table's size.  The host threads reach the file through a
 *                 shared mapping (copies into and out of the page cache, no
 *                 system call per row); then nobody may shrink the file
 *                 while the table is open, and a failing storage device
 *                 ends the process with a signal.  GAS_DISK_CALLS uses
 *                 pread / pwrite instead: slower for scattered rows, every
 *                 failure a GAS_ERR_IO.  io_threads (at most 16, 0 = 8): how
 *                 many of the process's I/O threads a transfer of this table
 *                 uses (one pool serves all tables); staging_bytes 0 =
 *                 32 MiB per buffer (allocated at the first transfer).
 *                 HOST pointers.
 * gas_disk_pull:  dst[i, 0:F] = table[r(i), 0:F] with r(i) as in gas_pull;
 *                 idx is a HOST array (copied before the call returns), dst
 *                 DEVICE memory [n, F], row stride ld_dst.  Returns at once
 *                 with a ticket; the transfer starts after the work queued
 *                 on `stream` so far has finished (so it may overwrite rows
 *                 that work still reads) and is complete, rows in dst, when
 *                 gas_disk_wait(ticket) returns.
 * gas_disk_push:  table[r(i), 0:F] = src[i, 0:F], src DEVICE memory, read
 *                 after the work queued on `stream` so far; src must stay
 *                 unchanged until gas_disk_wait(ticket) returns.  Duplicate
 *                 rows in idx: one of the values is kept.
 * gas_disk_wait:  blocks the calling thread until the transfer with that
 *                 ticket (and all queued before it) has finished; ticket 0 =
 *                 everything queued so far.  Returns the first failure of
 *                 any transfer of the table (GAS_ERR_IO, GAS_ERR_HIP), which
 *                 is kept: later calls report it too and later transfers are
 *                 dropped.
 * gas_disk_read_rows / gas_disk_write_rows: the same row moves between the
 *                 file and HOST memory, done by the calling thread after
 *                 everything queued has finished (initialising a table,
 *                 reading results back).
 * gas_disk_sync:  waits like gas_disk_wait(0) and flushes the file's data to
 *                 the storage device.
 * gas_disk_close: finishes queued transfers, frees everything; the file
 *                 stays.  A NULL table is allowed.
 * Indices and ranges are checked before anything is queued (GAS_ERR_RANGE).
 * One thread at a time may call into a given table; different tables are
 * independent.  All of a table's device transfers use the device that was
 * current at its first pull or push.  Pure data movement: bit-exact.
 */
typedef struct gas_disk_table gas_disk_table;
enum { GAS_DISK_CREATE = 1, GAS_DISK_CALLS = 2 };
GAS_API gas_status gas_disk_open(const char* path, int64_t n_rows, int32_t F, gas_dtype dt, int32_t flags,
                         int32_t io_threads, int64_t staging_bytes, gas_disk_table** table);
GAS_API gas_status gas_disk_close(gas_disk_table* table);
GAS_API gas_status gas_disk_pull(gas_disk_table* table, const int32_t* idx, int64_t base, int64_t n,
                         void* dst, int64_t ld_dst, void* stream, int64_t* ticket);
GAS_API gas_status gas_disk_push(gas_disk_table* table, const int32_t* idx, int64_t base, int64_t n,
                         const void* src, int64_t ld_src, void* stream, int64_t* ticket);
GAS_API gas_status gas_disk_wait(gas_disk_table* table, int64_t ticket);
GAS_API gas_status gas_disk_read_rows(gas_disk_table* table, const int32_t* idx, int64_t base, int64_t n,
                              void* dst, int64_t ld_dst);
GAS_API gas_status gas_disk_write_rows(gas_disk_table* table, const int32_t* idx, int64_t base, int64_t n,
                               const void* src, int64_t ld_src);
GAS_API gas_status gas_disk_sync(gas_disk_table* table);

/*
 * Debug helper: GAS_ERR_RANGE if any idx[i] is outside [0, limit).  Copies a
 * flag back and waits for `stream`.
 */
GAS_API gas_status gas_validate_indices(const int32_t* idx, int64_t n, int64_t limit, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* GAS_H */
