// PNA's neighbourhood aggregation (paper, operator appendix): mean, min and max over the neighbours of every
// in-batch node in ONE pass over the gathered rows, times the degree scalers 1, s and 1/s.  HBM-bound like the
// sum aggregation; three aggregators from one gather cost a third of three separate calls.
#include "wave.h"

namespace gas {
namespace {

struct PnaArgs {
    const int32_t* rowptr; const int32_t* col;
    int64_t n_rows;
    const char* X; int64_t ldx;
    const char* add; int64_t ldadd;
    char* out; int64_t ldout;
    int F;
    float inv_delta;
};

// One wavefront per row of the batch subgraph; lane l owns the 16-byte piece l (+64, +128, ...) of the feature
// row.  Neighbour indices are read 64 at a time and broadcast; gathers are issued sixteen at a time and folded in
// index order, so the result does not depend on timing.
template <bool BF>
__global__ __launch_bounds__(64) void pna_rows_kernel(PnaArgs a) {
    constexpr int E = Elems<BF>::E, EB = BF ? 2 : 4;
    constexpr int U = 16;                             // gathers in flight per lane
    const int64_t v = blockIdx.x;
    const int lane = threadIdx.x;
    const int b = a.rowptr[v], e = a.rowptr[v + 1];
    const int pieces = a.F / E;                       // 16-byte pieces per row
    const float d = (float)(e - b);
    const float s = logf(d + 1.f) * a.inv_delta;
    for (int p0 = 0; p0 < pieces; p0 += 64) {
        const int piece = p0 + lane;
        const bool on = piece < pieces;
        float sum[E], mn[E], mx[E];
#pragma unroll
        for (int i = 0; i < E; ++i) { sum[i] = 0.f; mn[i] = INFINITY; mx[i] = -INFINITY; }
        for (int k0 = b; k0 < e; k0 += 64) {
            const int cnt = min(64, e - k0);
            const int mine = lane < cnt ? a.col[k0 + lane] : 0;
            for (int j0 = 0; j0 < cnt; j0 += U) {
                u32x4 r[U];
#pragma unroll
                for (int j = 0; j < U; ++j) {
                    const int c = __builtin_amdgcn_readlane(mine, (j0 + j) & 63);
                    r[j] = u32x4{0u, 0u, 0u, 0u};
                    if (on && j0 + j < cnt)
                        r[j] = *reinterpret_cast<const u32x4*>(a.X + ((int64_t)c * a.ldx + (int64_t)piece * E) * EB);
                }
#pragma unroll
                for (int j = 0; j < U; ++j) {
                    if (j0 + j < cnt) {
                        float x[E];
                        unpack<BF>(r[j], x);
#pragma unroll
                        for (int i = 0; i < E; ++i) {
                            sum[i] += x[i];
                            mn[i] = fminf(mn[i], x[i]);
                            mx[i] = fmaxf(mx[i], x[i]);
                        }
                    }
                }
            }
        }
        if (!on) continue;
        float q[E];
#pragma unroll
        for (int i = 0; i < E; ++i) q[i] = 0.f;
        if (a.add && e > b) {
            const u32x4 r = *reinterpret_cast<const u32x4*>(a.add + (v * a.ldadd + (int64_t)piece * E) * EB);
            unpack<BF>(r, q);
        }
        float agg[3][E];
        const float inv_d = e > b ? 1.f / d : 0.f;
#pragma unroll
        for (int i = 0; i < E; ++i) {
            agg[0][i] = e > b ? sum[i] * inv_d + q[i] : 0.f;
            agg[1][i] = e > b ? mn[i] + q[i] : 0.f;
            agg[2][i] = e > b ? mx[i] + q[i] : 0.f;
        }
        const float inv_s = e > b ? 1.f / s : 0.f;
        char* o = a.out + (v * a.ldout + (int64_t)piece * E) * EB;
#pragma unroll
        for (int j = 0; j < 3; ++j) {
            float t1[E], t2[E];
#pragma unroll
            for (int i = 0; i < E; ++i) { t1[i] = s * agg[j][i]; t2[i] = agg[j][i] * inv_s; }
            __builtin_nontemporal_store(pack<BF>(agg[j]), reinterpret_cast<u32x4*>(o + (int64_t)j * a.F * EB));
            __builtin_nontemporal_store(pack<BF>(t1), reinterpret_cast<u32x4*>(o + (int64_t)(3 + j) * a.F * EB));
            __builtin_nontemporal_store(pack<BF>(t2), reinterpret_cast<u32x4*>(o + (int64_t)(6 + j) * a.F * EB));
        }
    }
}

// any width and alignment: one thread per (row, feature)
template <bool BF>
__global__ __launch_bounds__(256) void pna_generic_kernel(PnaArgs a) {
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= a.n_rows * a.F) return;
    const int64_t v = idx / a.F;
    const int f = (int)(idx % a.F);
    auto ld = [&](const char* p, int64_t i) -> float {
        if constexpr (BF) return __uint_as_float((uint32_t)reinterpret_cast<const uint16_t*>(p)[i] << 16);
        else return reinterpret_cast<const float*>(p)[i];
    };
    auto st = [&](int64_t i, float x) {
        if constexpr (BF) reinterpret_cast<uint16_t*>(a.out)[i] = (uint16_t)f32_to_bf16(x);
        else reinterpret_cast<float*>(a.out)[i] = x;
    };
    const int b = a.rowptr[v], e = a.rowptr[v + 1];
    float sum = 0.f, mn = INFINITY, mx = -INFINITY;
    for (int k = b; k < e; ++k) {
        const float x = ld(a.X, (int64_t)a.col[k] * a.ldx + f);
        sum += x; mn = fminf(mn, x); mx = fmaxf(mx, x);
    }
    const float d = (float)(e - b), s = logf(d + 1.f) * a.inv_delta;
    const float q = (a.add && e > b) ? ld(a.add, v * a.ldadd + f) : 0.f;
    const float agg[3] = {e > b ? sum / d + q : 0.f, e > b ? mn + q : 0.f, e > b ? mx + q : 0.f};
    const float inv_s = e > b ? 1.f / s : 0.f;
    for (int j = 0; j < 3; ++j) {
        st(v * a.ldout + (int64_t)j * a.F + f, agg[j]);
        st(v * a.ldout + (int64_t)(3 + j) * a.F + f, s * agg[j]);
        st(v * a.ldout + (int64_t)(6 + j) * a.F + f, agg[j] * inv_s);
    }
}

}  // namespace
}  // namespace gas

using namespace gas;

extern "C" gas_status gas_pna_aggregate(const int32_t* rowptr, const int32_t* col, int64_t n_rows, const void* X,
                                        int64_t ldx, gas_dtype dt, int32_t F, const void* add, int64_t ldadd,
                                        float delta, void* out, int64_t ldout, void* stream) {
    if (!valid_dtype(dt)) return fail(GAS_ERR_DTYPE, "gas_pna_aggregate: unknown dtype %d", (int)dt);
    GAS_REQUIRE(n_rows >= 0 && F > 0, "gas_pna_aggregate: n_rows=%lld F=%d", (long long)n_rows, F);
    GAS_REQUIRE(delta > 0.f, "gas_pna_aggregate: delta must be positive");
    if (n_rows == 0) return GAS_OK;
    GAS_REQUIRE(rowptr && col && X && out, "gas_pna_aggregate: null pointer");
    GAS_REQUIRE(ldx >= F && ldout >= 9 * (int64_t)F && (!add || ldadd >= F), "gas_pna_aggregate: row stride smaller than the row");
    GAS_REQUIRE(out != X && out != add, "gas_pna_aggregate: the output must not alias an input");
    GAS_REQUIRE(n_rows <= 0x7FFFFFFFLL, "gas_pna_aggregate: too many rows for one launch");
    PnaArgs a;
    a.rowptr = rowptr; a.col = col; a.n_rows = n_rows;
    a.X = static_cast<const char*>(X); a.ldx = ldx;
    a.add = static_cast<const char*>(add); a.ldadd = ldadd;
    a.out = static_cast<char*>(out); a.ldout = ldout;
    a.F = F; a.inv_delta = 1.f / delta;
    const int e = dt == GAS_BF16 ? 8 : 4;
    hipStream_t s = (hipStream_t)stream;
    const bool vec = F % e == 0 && ldx % e == 0 && ldout % e == 0 && (!add || ldadd % e == 0) && aligned16(X) &&
                     aligned16(out) && (!add || aligned16(add));
    if (vec) {
        if (dt == GAS_BF16) hipLaunchKernelGGL(pna_rows_kernel<true>, dim3((unsigned)n_rows), dim3(64), 0, s, a);
        else hipLaunchKernelGGL(pna_rows_kernel<false>, dim3((unsigned)n_rows), dim3(64), 0, s, a);
    } else {
        const int64_t blocks = (n_rows * F + 255) / 256;
        GAS_REQUIRE(blocks <= 0x7FFFFFFFLL, "gas_pna_aggregate: problem too large for the element-wise path");
        if (dt == GAS_BF16) hipLaunchKernelGGL(pna_generic_kernel<true>, dim3((unsigned)blocks), dim3(256), 0, s, a);
        else hipLaunchKernelGGL(pna_generic_kernel<false>, dim3((unsigned)blocks), dim3(256), 0, s, a);
    }
    GAS_CHECK_HIP(hipGetLastError());
    return GAS_OK;
}
