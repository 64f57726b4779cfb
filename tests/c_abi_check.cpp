// A consumer of the C ABI without Python or PyTorch: plain pointers from hipMalloc, the calls of include/gas.h on the
// default stream, results copied back and compared with the CPU oracle's C functions (oracle/gas_oracle.c, linked as
// the checker).  One layer step on a small random batch: pull, aggregate (sum with a self term, as GIN), transform,
// push, backward aggregate; fp32.  Built and run by tests/test_gpu_c_abi.py.  Exit status 0 = all within 1e-5.
#include <hip/hip_runtime_api.h>
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <vector>

#include "gas.h"

extern "C" {
void oracle_pull(const void* hist, int64_t ld_hist, const int32_t* idx, int64_t n, int32_t F, int32_t elem_bytes, void* dst,
                 int64_t ld_dst);
void oracle_push(const void* src, int64_t ld_src, const int32_t* idx, int64_t n, int32_t F, int32_t elem_bytes, void* hist,
                 int64_t ld_hist);
void oracle_spmm(const int32_t* rowptr, const int32_t* col, const float* val, double diag, const void* X, int64_t ldx, int dtx,
                 int32_t F, double s_agg, const void* R, int64_t ldr, double s_res, void* Z, int64_t ldz, int dtz,
                 int64_t n_rows);
void oracle_spmm_t(const int32_t* rowptr, const int32_t* col, const float* val, double diag, double s_agg, const void* G,
                   int64_t ldg, int dtg, int32_t F, int64_t n_rows, int64_t n_out, void* GX, int64_t ldgx, int dtgx);
void oracle_linear(const void* Z, int64_t ldz, int64_t n_rows, int32_t F_in, const void* W, int32_t F_out, const void* bias,
                   int dt, double c_identity, double c_weight, int relu, void* Y, int64_t ldy, int dty);
}

#define HIP(expr)                                                                          \
    do {                                                                                   \
        hipError_t e_ = (expr);                                                            \
        if (e_ != hipSuccess) { printf("%s: %s\n", #expr, hipGetErrorString(e_)); return 2; } \
    } while (0)
#define GAS(expr)                                                                   \
    do {                                                                            \
        if ((expr) != GAS_OK) { printf("%s: %s\n", #expr, gas_last_error()); return 2; } \
    } while (0)

static uint64_t state = 2106;
static uint32_t rnd() {
    state = state * 6364136223846793005ull + 1442695040888963407ull;
    return (uint32_t)(state >> 33);
}
static float unit() { return (float)rnd() / 2147483648.0f - 0.5f; }

template <typename T>
static T* to_device(const std::vector<T>& h) {
    T* d = nullptr;
    if (hipMalloc((void**)&d, h.size() * sizeof(T) + 16) != hipSuccess) return nullptr;
    if (hipMemcpy(d, h.data(), h.size() * sizeof(T), hipMemcpyHostToDevice) != hipSuccess) return nullptr;
    return d;
}

static double worst(const std::vector<float>& got, const std::vector<float>& want, int64_t rows, int F) {
    double top = 0;
    for (float v : want) top = fmax(top, fabs((double)v));
    double w = 0;
    for (int64_t r = 0; r < rows; ++r) {                    // every row on its own scale, floor 1e-3 of the tensor's
        double rmax = 0, err = 0;
        for (int f = 0; f < F; ++f) {
            rmax = fmax(rmax, fabs((double)want[r * F + f]));
            err = fmax(err, fabs((double)got[r * F + f] - (double)want[r * F + f]));
        }
        w = fmax(w, err / fmax(rmax, 1e-3 * top));
    }
    return w;
}

int main() {
    const int64_t nb = 3000, nh = 2000, nv = nb + nh, N = 8000;
    const int F = 64, Fo = 48;
    // the batch subgraph: about 20 entries per row, one row of 900, one empty row; columns ascending per row
    std::vector<int32_t> rowptr(nb + 1, 0), col;
    for (int64_t v = 0; v < nb; ++v) {
        const int d = v == 7 ? 900 : (v == 11 ? 0 : 4 + (int)(rnd() % 32));
        std::vector<char> pick((size_t)nv, 0);
        for (int k = 0; k < d; ++k) pick[rnd() % nv] = 1;
        for (int64_t u = 0; u < nv; ++u)
            if (pick[(size_t)u]) col.push_back((int32_t)u);
        rowptr[v + 1] = (int32_t)col.size();
    }
    const int64_t nnz = (int64_t)col.size();
    std::vector<int32_t> colptr(nv + 1, 0), row((size_t)nnz);
    for (int32_t c : col) ++colptr[c + 1];
    for (int64_t u = 0; u < nv; ++u) colptr[u + 1] += colptr[u];
    {
        std::vector<int32_t> fill(colptr.begin(), colptr.end() - 1);
        for (int64_t v = 0; v < nb; ++v)
            for (int32_t k = rowptr[v]; k < rowptr[v + 1]; ++k) row[(size_t)fill[col[k]]++] = (int32_t)v;
    }
    std::vector<int32_t> n_id((size_t)nv);
    {                                                       // distinct node ids: the head of a random permutation
        std::vector<int32_t> perm((size_t)N);
        for (int64_t i = 0; i < N; ++i) perm[(size_t)i] = (int32_t)i;
        for (int64_t i = N - 1; i > 0; --i) { const int64_t j = rnd() % (i + 1); std::swap(perm[(size_t)i], perm[(size_t)j]); }
        for (int64_t i = 0; i < nv; ++i) n_id[(size_t)i] = perm[(size_t)i];
    }
    std::vector<float> hist((size_t)(N * F)), x((size_t)(nv * F)), w((size_t)(F * Fo)), g((size_t)(nb * F));
    for (auto& v : hist) v = unit();
    for (auto& v : x) v = unit();
    for (auto& v : w) v = unit() * 0.3f;
    for (auto& v : g) v = unit();

    // ---- device side, through the C ABI only
    int32_t *d_rowptr = to_device(rowptr), *d_col = to_device(col), *d_colptr = to_device(colptr), *d_row = to_device(row),
            *d_nid = to_device(n_id);
    float *d_hist = to_device(hist), *d_x = to_device(x), *d_w = to_device(w), *d_g = to_device(g);
    float *d_z = nullptr, *d_y = nullptr, *d_hist_out = nullptr, *d_gx = nullptr;
    HIP(hipMalloc((void**)&d_z, nb * F * 4));
    HIP(hipMalloc((void**)&d_y, nb * Fo * 4));
    HIP(hipMalloc((void**)&d_hist_out, N * Fo * 4));
    HIP(hipMalloc((void**)&d_gx, nb * F * 4));
    HIP(hipMemset(d_hist_out, 0, N * Fo * 4));
    if (!d_rowptr || !d_col || !d_colptr || !d_row || !d_nid || !d_hist || !d_x || !d_w || !d_g) { printf("allocation failed\n"); return 2; }
    gas_plan *plan = nullptr, *plan_t = nullptr;
    GAS(gas_pull(d_hist, N, F, d_nid + nb, 0, nh, F, GAS_F32, d_x + nb * F, F, nullptr));
    GAS(gas_plan_create(d_rowptr, d_col, nb, nnz, F, nullptr, &plan));
    GAS(gas_spmm(plan, d_rowptr, d_col, nullptr, 1.1f, d_x, F, GAS_F32, F, 1.f, nullptr, 0, 0.f, d_z, F, GAS_F32, nullptr));
    GAS(gas_linear(d_z, F, nb, F, d_w, Fo, nullptr, GAS_F32, 0.f, 1.f, 1, d_y, Fo, nullptr));
    GAS(gas_push(d_y, Fo, d_nid, 0, nb, Fo, GAS_F32, d_hist_out, N, Fo, nullptr));
    GAS(gas_plan_create(d_colptr, d_row, nb, colptr[nb], F, nullptr, &plan_t));
    GAS(gas_spmm_t(plan_t, d_colptr, d_row, nullptr, 1.1f, 1.f, nb, d_g, F, GAS_F32, F, d_gx, F, GAS_F32, nullptr));
    HIP(hipDeviceSynchronize());
    std::vector<float> got_z((size_t)(nb * F)), got_y((size_t)(nb * Fo)), got_hist((size_t)(N * Fo)), got_gx((size_t)(nb * F)),
        got_x((size_t)(nv * F));
    HIP(hipMemcpy(got_x.data(), d_x, got_x.size() * 4, hipMemcpyDeviceToHost));
    HIP(hipMemcpy(got_z.data(), d_z, got_z.size() * 4, hipMemcpyDeviceToHost));
    HIP(hipMemcpy(got_y.data(), d_y, got_y.size() * 4, hipMemcpyDeviceToHost));
    HIP(hipMemcpy(got_hist.data(), d_hist_out, got_hist.size() * 4, hipMemcpyDeviceToHost));
    HIP(hipMemcpy(got_gx.data(), d_gx, got_gx.size() * 4, hipMemcpyDeviceToHost));
    gas_plan_destroy(plan);
    gas_plan_destroy(plan_t);

    // ---- the oracle, on the host
    oracle_pull(hist.data(), F, n_id.data() + nb, nh, F, 4, x.data() + nb * F, F);
    std::vector<float> z((size_t)(nb * F)), y((size_t)(nb * Fo)), hist_out((size_t)(N * Fo), 0.f), gx((size_t)(nb * F));
    oracle_spmm(rowptr.data(), col.data(), nullptr, 1.1, x.data(), F, 0, F, 1.0, nullptr, 0, 0.0, z.data(), F, 0, nb);
    oracle_linear(z.data(), F, nb, F, w.data(), Fo, nullptr, 0, 0.0, 1.0, 1, y.data(), Fo, 0);
    oracle_push(y.data(), Fo, n_id.data(), nb, Fo, 4, hist_out.data(), Fo);
    oracle_spmm_t(rowptr.data(), col.data(), nullptr, 1.1, 1.0, g.data(), F, 0, F, nb, nb, gx.data(), F, 0);

    int bad = 0;
    if (memcmp(got_x.data(), x.data(), x.size() * 4) != 0) { printf("pull: not bit-exact\n"); ++bad; }
    const double ez = worst(got_z, z, nb, F), ey = worst(got_y, y, nb, Fo), eh = worst(got_hist, hist_out, N, Fo),
                 eg = worst(got_gx, gx, nb, F);
    printf("worst per-row relative error: spmm %.2e, linear %.2e, push %.2e, spmm_t %.2e (nnz %lld)\n", ez, ey, eh, eg,
           (long long)nnz);
    if (ez > 1e-5 || ey > 1e-5 || eh > 1e-5 || eg > 1e-5) ++bad;
    int touched = 0;                                        // rows the push did not name stay zero
    for (int64_t r = 0; r < N; ++r) {
        bool any = false;
        for (int f = 0; f < Fo; ++f) any = any || got_hist[(size_t)(r * Fo + f)] != 0.f;
        touched += any;
    }
    if (touched > nb) { printf("push touched %d rows, the batch has %lld\n", touched, (long long)nb); ++bad; }
    printf(bad ? "FAILED\n" : "ok\n");
    return bad ? 1 : 0;
}
