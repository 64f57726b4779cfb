// Backward passes of the PNA and GAT aggregations (paper, operator appendix; the chain rule on their equations).
//
// Both aggregations gather rows by column index, so their adjoint scatters to those rows.  To stay free of
// atomics and keep a fixed summation order the scatter is turned around, as for the sum aggregation: a first kernel
// walks the rows of the pattern (CSR) and leaves, per row or per entry, the factors the adjoint needs; a second
// kernel walks the columns (the CSC copy, with the position of every entry in the CSR arrays) and sums, for each
// column, the contributions of its entries in stored order.  One wavefront per row / column, lanes over the
// features: these are correctness-first kernels of a widening row, not tuned ones.
#include "common.h"

namespace gas {
namespace {

template <bool BF>
__device__ __forceinline__ float ld(const char* p, int64_t i) {
    if constexpr (BF) return __uint_as_float((uint32_t)reinterpret_cast<const uint16_t*>(p)[i] << 16);
    else return reinterpret_cast<const float*>(p)[i];
}
template <bool BF>
__device__ __forceinline__ void st(char* p, int64_t i, float x) {
    if constexpr (BF) reinterpret_cast<uint16_t*>(p)[i] = (uint16_t)f32_to_bf16(x);
    else reinterpret_cast<float*>(p)[i] = x;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
}

// ------------------------------------------------------------------------------------------------ PNA
struct PnaBwdArgs {
    const int32_t* rowptr; const int32_t* col; int64_t n_rows;
    const int32_t* colptr; const int32_t* row; const int32_t* csc_pos; int64_t n_out;
    const char* X; int64_t ldx;
    const char* G; int64_t ldg;
    char* GX; int64_t ldgx;
    char* Gadd; int64_t ldga;
    float* C;          // [n_rows][3][F]: c_mean / d, c_min, c_max
    int32_t* K;        // [n_rows][2][F]: entry position of the first minimum and of the first maximum
    int F;
    float inv_delta;
};

// Row v: the three block gradients folded with their scalers, and which entry holds each feature's extremes.
template <bool BF>
__global__ __launch_bounds__(64) void pna_bwd_rows_kernel(PnaBwdArgs a) {
    const int64_t v = blockIdx.x;
    const int lane = threadIdx.x;
    const int b = a.rowptr[v], e = a.rowptr[v + 1];
    const float d = (float)(e - b);
    const float s = logf(d + 1.f) * a.inv_delta;
    for (int f = lane; f < a.F; f += 64) {
        float* c = a.C + (v * 3) * a.F + f;
        int32_t* kk = a.K + (v * 2) * a.F + f;
        if (e == b) {
            c[0] = 0.f; c[a.F] = 0.f; c[2 * a.F] = 0.f;
            kk[0] = -1; kk[a.F] = -1;
            if (a.Gadd) st<BF>(a.Gadd, v * a.ldga + f, 0.f);
            continue;
        }
        float mn = INFINITY, mx = -INFINITY;
        int kmin = b, kmax = b;
        for (int k = b; k < e; ++k) {
            const float x = ld<BF>(a.X, (int64_t)a.col[k] * a.ldx + f);
            if (x < mn) { mn = x; kmin = k; }            // strict: the first entry that attains it keeps it
            if (x > mx) { mx = x; kmax = k; }
        }
        float cc[3];
#pragma unroll
        for (int i = 0; i < 3; ++i)
            cc[i] = ld<BF>(a.G, v * a.ldg + (int64_t)i * a.F + f) + s * ld<BF>(a.G, v * a.ldg + (int64_t)(3 + i) * a.F + f) +
                    ld<BF>(a.G, v * a.ldg + (int64_t)(6 + i) * a.F + f) / s;
        c[0] = cc[0] / d; c[a.F] = cc[1]; c[2 * a.F] = cc[2];
        kk[0] = kmin; kk[a.F] = kmax;
        if (a.Gadd) st<BF>(a.Gadd, v * a.ldga + f, cc[0] + cc[1] + cc[2]);
    }
}

// Column u: the sum over its entries (v, u), in stored order, of what row v owes this entry.
template <bool BF>
__global__ __launch_bounds__(64) void pna_bwd_cols_kernel(PnaBwdArgs a) {
    const int64_t u = blockIdx.x;
    const int lane = threadIdx.x;
    const int b = a.colptr[u], e = a.colptr[u + 1];
    for (int f = lane; f < a.F; f += 64) {
        float acc = 0.f;
        for (int q = b; q < e; ++q) {
            const int64_t v = a.row[q];
            const int k = a.csc_pos[q];
            const float* c = a.C + (v * 3) * a.F + f;
            const int32_t* kk = a.K + (v * 2) * a.F + f;
            acc += c[0];
            if (kk[0] == k) acc += c[a.F];
            if (kk[a.F] == k) acc += c[2 * a.F];
        }
        st<BF>(a.GX, u * a.ldgx + f, acc);
    }
}

// ------------------------------------------------------------------------------------------------ GAT
constexpr int kMaxPerLane = 16;                      // features per lane: F <= 1024, as in the forward kernel

struct GatBwdArgs {
    const int32_t* rowptr; const int32_t* col; int64_t n_rows;
    const int32_t* colptr; const int32_t* row; const int32_t* csc_pos; int64_t n_cols, n_out;
    const char* P; int64_t ldp;
    const char* a_dst; const char* a_src;
    const char* GZ; int64_t ldgz;
    char* GP; int64_t ldgp;
    float* alpha;      // [nnz]: scores, then attention weights
    float* dt;         // [nnz]: dalpha, then the gradient at the raw scores
    float* csum;       // [n_rows]: sum of dt over the row
    float* tsum;       // [n_cols]: sum of dt over the column
    int F;
    float slope;
};

// Row v: scores and softmax again, then per entry the attention weight and the gradient at its raw score.
template <bool BF>
__global__ __launch_bounds__(64) void gat_bwd_rows_kernel(GatBwdArgs a) {
    const int64_t v = blockIdx.x;
    const int lane = threadIdx.x;
    const int b = a.rowptr[v], e = a.rowptr[v + 1];
    if (e == b) {
        if (lane == 0) a.csum[v] = 0.f;
        return;
    }
    const int nf = (a.F + 63) / 64;
    float asrc[kMaxPerLane], gz[kMaxPerLane];
    float sv = 0.f;
#pragma unroll
    for (int j = 0; j < kMaxPerLane; ++j) {
        const int f = lane + 64 * j;
        const bool on = j < nf && f < a.F;
        asrc[j] = on ? ld<BF>(a.a_src, f) : 0.f;
        gz[j] = on ? ld<BF>(a.GZ, v * a.ldgz + f) : 0.f;
        if (on) sv = fmaf(ld<BF>(a.a_dst, f), ld<BF>(a.P, v * a.ldp + f), sv);
    }
    sv = wave_sum(sv);
    float mx = -INFINITY;
    for (int k = b; k < e; ++k) {
        const int64_t c = a.col[k];
        float sw = 0.f, da = 0.f;
#pragma unroll
        for (int j = 0; j < kMaxPerLane; ++j) {
            const int f = lane + 64 * j;
            if (j < nf && f < a.F) {
                const float p = ld<BF>(a.P, c * a.ldp + f);
                sw = fmaf(asrc[j], p, sw);
                da = fmaf(gz[j], p, da);
            }
        }
        sw = wave_sum(sw);
        da = wave_sum(da);
        const float t = sv + sw;
        mx = fmaxf(mx, t > 0.f ? t : a.slope * t);
        // t and da are the same in every lane: the lane that will read entry k below is the one that stores it,
        // so no lane ever reads another lane's store
        if (lane == ((k - b) & 63)) { a.alpha[k] = t; a.dt[k] = da; }
    }
    float den = 0.f;
    for (int k = b + lane; k < e; k += 64) {
        const float t = a.alpha[k];
        den += expf((t > 0.f ? t : a.slope * t) - mx);
    }
    den = wave_sum(den);
    float mean_da = 0.f;
    for (int k = b + lane; k < e; k += 64) {
        const float t = a.alpha[k];
        mean_da += expf((t > 0.f ? t : a.slope * t) - mx) / den * a.dt[k];
    }
    mean_da = wave_sum(mean_da);
    float sum_dt = 0.f;
    for (int k = b + lane; k < e; k += 64) {
        const float t = a.alpha[k];
        const float al = expf((t > 0.f ? t : a.slope * t) - mx) / den;
        const float dtk = al * (a.dt[k] - mean_da) * (t > 0.f ? 1.f : a.slope);
        a.alpha[k] = al;
        a.dt[k] = dtk;
        sum_dt += dtk;
    }
    sum_dt = wave_sum(sum_dt);
    if (lane == 0) a.csum[v] = sum_dt;
}

// Column u of the pattern = row u of P: sum over its entries (v, u) of alpha GZ[v] + dt a_src, plus, for an
// in-batch node, its own row's total times a_dst.
template <bool BF>
__global__ __launch_bounds__(64) void gat_bwd_cols_kernel(GatBwdArgs a) {
    const int64_t u = blockIdx.x;
    const int lane = threadIdx.x;
    const int b = a.colptr[u], e = a.colptr[u + 1];
    const int nf = (a.F + 63) / 64;
    float acc[kMaxPerLane];
#pragma unroll
    for (int j = 0; j < kMaxPerLane; ++j) acc[j] = 0.f;
    float ts = 0.f;
    const bool keep = u < a.n_out;
    for (int q = b; q < e; ++q) {
        const int k = a.csc_pos[q];
        ts += a.dt[k];
        if (keep) {
            const int64_t v = a.row[q];
            const float al = a.alpha[k];
#pragma unroll
            for (int j = 0; j < kMaxPerLane; ++j) {
                const int f = lane + 64 * j;
                if (j < nf && f < a.F) acc[j] = fmaf(al, ld<BF>(a.GZ, v * a.ldgz + f), acc[j]);
            }
        }
    }
    if (lane == 0) a.tsum[u] = ts;
    if (!keep) return;
    const float cs = u < a.n_rows ? a.csum[u] : 0.f;
#pragma unroll
    for (int j = 0; j < kMaxPerLane; ++j) {
        const int f = lane + 64 * j;
        if (j < nf && f < a.F)
            st<BF>(a.GP, u * a.ldgp + f, acc[j] + ts * ld<BF>(a.a_src, f) + cs * ld<BF>(a.a_dst, f));
    }
}

// out[f] = sum_i w[i] M[i, f] in a fixed order: slabs of 1024 rows, one partial row per slab, then the slabs in order.
constexpr int kSlab = 1024;
template <bool BF>
__global__ __launch_bounds__(256) void wcolsum_partial_kernel(const char* M, int64_t ldm, const float* w, int64_t n, int F,
                                                              float* partial) {
    const int64_t r0 = (int64_t)blockIdx.x * kSlab, r1 = min(n, r0 + kSlab);
    for (int f = threadIdx.x; f < F; f += 256) {
        float acc = 0.f;
        for (int64_t i = r0; i < r1; ++i) acc = fmaf(w[i], ld<BF>(M, i * ldm + f), acc);
        partial[(int64_t)blockIdx.x * F + f] = acc;
    }
}
__global__ __launch_bounds__(256) void wcolsum_reduce_kernel(const float* partial, int64_t n_slabs, int F, float* out) {
    const int f = blockIdx.x * 256 + threadIdx.x;
    if (f >= F) return;
    double acc = 0.0;
    for (int64_t sidx = 0; sidx < n_slabs; ++sidx) acc += (double)partial[sidx * F + f];
    out[f] = (float)acc;
}

int64_t align_up(int64_t x) { return (x + 255) / 256 * 256; }

}  // namespace
}  // namespace gas

using namespace gas;

extern "C" {

int64_t gas_pna_aggregate_bwd_workspace(int64_t n_rows, int32_t F) {
    if (n_rows <= 0 || F <= 0) return 0;
    return align_up(n_rows * 3 * (int64_t)F * 4) + align_up(n_rows * 2 * (int64_t)F * 4);
}

gas_status gas_pna_aggregate_bwd(const int32_t* rowptr, const int32_t* col, int64_t n_rows, const int32_t* colptr,
                                 const int32_t* row, const int32_t* csc_pos, int64_t n_out, const void* X, int64_t ldx,
                                 gas_dtype dt, int32_t F, float delta, const void* G, int64_t ldg, void* GX,
                                 int64_t ldgx, void* Gadd, int64_t ldga, void* workspace, int64_t workspace_bytes,
                                 void* stream) {
    if (!valid_dtype(dt)) return fail(GAS_ERR_DTYPE, "gas_pna_aggregate_bwd: unknown dtype %d", (int)dt);
    GAS_REQUIRE(n_rows >= 0 && n_out >= 0 && F > 0, "gas_pna_aggregate_bwd: n_rows=%lld n_out=%lld F=%d",
                (long long)n_rows, (long long)n_out, F);
    GAS_REQUIRE(delta > 0.f, "gas_pna_aggregate_bwd: delta must be positive");
    GAS_REQUIRE(n_rows <= 0x7FFFFFFFLL && n_out <= 0x7FFFFFFFLL, "gas_pna_aggregate_bwd: too many rows for one launch");
    if (n_rows == 0 && n_out == 0) return GAS_OK;
    GAS_REQUIRE(n_out == 0 || (colptr && GX && ldgx >= F), "gas_pna_aggregate_bwd: null column pointers or output");
    GAS_REQUIRE(n_rows == 0 || (rowptr && col && row && csc_pos && X && G && ldx >= F && ldg >= 9 * (int64_t)F),
                "gas_pna_aggregate_bwd: null pointer or row stride smaller than the row");
    GAS_REQUIRE(!Gadd || ldga >= F, "gas_pna_aggregate_bwd: row stride of Gadd smaller than F");
    GAS_REQUIRE(n_rows == 0 || (workspace && workspace_bytes >= gas_pna_aggregate_bwd_workspace(n_rows, F)),
                "gas_pna_aggregate_bwd: workspace of %lld bytes needed, %lld given",
                (long long)gas_pna_aggregate_bwd_workspace(n_rows, F), (long long)workspace_bytes);
    PnaBwdArgs a;
    a.rowptr = rowptr; a.col = col; a.n_rows = n_rows;
    a.colptr = colptr; a.row = row; a.csc_pos = csc_pos; a.n_out = n_out;
    a.X = static_cast<const char*>(X); a.ldx = ldx;
    a.G = static_cast<const char*>(G); a.ldg = ldg;
    a.GX = static_cast<char*>(GX); a.ldgx = ldgx;
    a.Gadd = static_cast<char*>(Gadd); a.ldga = ldga;
    a.C = static_cast<float*>(workspace);
    a.K = reinterpret_cast<int32_t*>(static_cast<char*>(workspace) + align_up(n_rows * 3 * (int64_t)F * 4));
    a.F = F; a.inv_delta = 1.f / delta;
    hipStream_t s = (hipStream_t)stream;
    if (n_rows > 0) {
        if (dt == GAS_BF16) hipLaunchKernelGGL(pna_bwd_rows_kernel<true>, dim3((unsigned)n_rows), dim3(64), 0, s, a);
        else hipLaunchKernelGGL(pna_bwd_rows_kernel<false>, dim3((unsigned)n_rows), dim3(64), 0, s, a);
    }
    if (n_out > 0) {
        if (dt == GAS_BF16) hipLaunchKernelGGL(pna_bwd_cols_kernel<true>, dim3((unsigned)n_out), dim3(64), 0, s, a);
        else hipLaunchKernelGGL(pna_bwd_cols_kernel<false>, dim3((unsigned)n_out), dim3(64), 0, s, a);
    }
    GAS_CHECK_HIP(hipGetLastError());
    return GAS_OK;
}

int64_t gas_gat_aggregate_bwd_workspace(int64_t n_rows, int64_t n_cols, int64_t nnz, int32_t F) {
    if (n_rows < 0 || n_cols <= 0 || nnz < 0 || F <= 0) return 0;
    const int64_t slabs = (n_cols + kSlab - 1) / kSlab;
    return 2 * align_up(nnz * 4) + align_up(n_rows * 4) + align_up(n_cols * 4) + 2 * align_up(slabs * (int64_t)F * 4);
}

gas_status gas_gat_aggregate_bwd(const int32_t* rowptr, const int32_t* col, int64_t n_rows, const int32_t* colptr,
                                 const int32_t* row, const int32_t* csc_pos, int64_t n_cols, int64_t n_out,
                                 int64_t nnz, const void* P, int64_t ldp, gas_dtype dt, int32_t F, const void* a_dst,
                                 const void* a_src, float negative_slope, const void* GZ, int64_t ldgz, void* GP,
                                 int64_t ldgp, float* Ga_dst, float* Ga_src, void* workspace, int64_t workspace_bytes,
                                 void* stream) {
    if (!valid_dtype(dt)) return fail(GAS_ERR_DTYPE, "gas_gat_aggregate_bwd: unknown dtype %d", (int)dt);
    GAS_REQUIRE(n_rows >= 0 && n_cols >= n_rows && n_out >= 0 && n_out <= n_cols && nnz >= 0 && F > 0 &&
                F <= 64 * kMaxPerLane, "gas_gat_aggregate_bwd: n_rows=%lld n_cols=%lld n_out=%lld nnz=%lld F=%d (F <= %d)",
                (long long)n_rows, (long long)n_cols, (long long)n_out, (long long)nnz, F, 64 * kMaxPerLane);
    GAS_REQUIRE(n_cols <= 0x7FFFFFFFLL, "gas_gat_aggregate_bwd: too many rows for one launch");
    if (n_cols == 0) return GAS_OK;
    GAS_REQUIRE(rowptr && colptr && P && a_dst && a_src && GZ && Ga_dst && Ga_src && (nnz == 0 || (col && row && csc_pos)),
                "gas_gat_aggregate_bwd: null pointer");
    GAS_REQUIRE(ldp >= F && ldgz >= F && (n_out == 0 || (GP && ldgp >= F)), "gas_gat_aggregate_bwd: null output or row stride smaller than F");
    GAS_REQUIRE(workspace && workspace_bytes >= gas_gat_aggregate_bwd_workspace(n_rows, n_cols, nnz, F),
                "gas_gat_aggregate_bwd: workspace of %lld bytes needed, %lld given",
                (long long)gas_gat_aggregate_bwd_workspace(n_rows, n_cols, nnz, F), (long long)workspace_bytes);
    char* w = static_cast<char*>(workspace);
    GatBwdArgs a;
    a.rowptr = rowptr; a.col = col; a.n_rows = n_rows;
    a.colptr = colptr; a.row = row; a.csc_pos = csc_pos; a.n_cols = n_cols; a.n_out = n_out;
    a.P = static_cast<const char*>(P); a.ldp = ldp;
    a.a_dst = static_cast<const char*>(a_dst); a.a_src = static_cast<const char*>(a_src);
    a.GZ = static_cast<const char*>(GZ); a.ldgz = ldgz;
    a.GP = static_cast<char*>(GP); a.ldgp = ldgp;
    a.alpha = reinterpret_cast<float*>(w); w += align_up(nnz * 4);
    a.dt = reinterpret_cast<float*>(w); w += align_up(nnz * 4);
    a.csum = reinterpret_cast<float*>(w); w += align_up(n_rows * 4);
    a.tsum = reinterpret_cast<float*>(w); w += align_up(n_cols * 4);
    const int64_t slabs = (n_cols + kSlab - 1) / kSlab;
    float* part_dst = reinterpret_cast<float*>(w); w += align_up(slabs * (int64_t)F * 4);
    float* part_src = reinterpret_cast<float*>(w);
    a.F = F; a.slope = negative_slope;
    hipStream_t s = (hipStream_t)stream;
    const bool bf = dt == GAS_BF16;
    if (n_rows > 0) {
        if (bf) hipLaunchKernelGGL(gat_bwd_rows_kernel<true>, dim3((unsigned)n_rows), dim3(64), 0, s, a);
        else hipLaunchKernelGGL(gat_bwd_rows_kernel<false>, dim3((unsigned)n_rows), dim3(64), 0, s, a);
    }
    if (bf) hipLaunchKernelGGL(gat_bwd_cols_kernel<true>, dim3((unsigned)n_cols), dim3(64), 0, s, a);
    else hipLaunchKernelGGL(gat_bwd_cols_kernel<false>, dim3((unsigned)n_cols), dim3(64), 0, s, a);
    // Ga_dst = sum over the in-batch nodes of (row total of dt) P[v];  Ga_src = sum over all nodes of (column total) P[u]
    const int64_t slabs_rows = (n_rows + kSlab - 1) / kSlab;
    const unsigned fblocks = (unsigned)((F + 255) / 256);
    if (bf) {
        if (slabs_rows > 0) hipLaunchKernelGGL(wcolsum_partial_kernel<true>, dim3((unsigned)slabs_rows), dim3(256), 0, s, a.P, ldp, a.csum, n_rows, F, part_dst);
        hipLaunchKernelGGL(wcolsum_partial_kernel<true>, dim3((unsigned)slabs), dim3(256), 0, s, a.P, ldp, a.tsum, n_cols, F, part_src);
    } else {
        if (slabs_rows > 0) hipLaunchKernelGGL(wcolsum_partial_kernel<false>, dim3((unsigned)slabs_rows), dim3(256), 0, s, a.P, ldp, a.csum, n_rows, F, part_dst);
        hipLaunchKernelGGL(wcolsum_partial_kernel<false>, dim3((unsigned)slabs), dim3(256), 0, s, a.P, ldp, a.tsum, n_cols, F, part_src);
    }
    hipLaunchKernelGGL(wcolsum_reduce_kernel, dim3(fblocks), dim3(256), 0, s, part_dst, slabs_rows, F, Ga_dst);
    hipLaunchKernelGGL(wcolsum_reduce_kernel, dim3(fblocks), dim3(256), 0, s, part_src, slabs, F, Ga_src);
    GAS_CHECK_HIP(hipGetLastError());
    return GAS_OK;
}

}  // extern "C"
