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

// Rows of at most 64 pieces of 16 bytes, G = 16, 32 or 64 lanes per row (at least the number of pieces).  A
// wavefront's S = 64 / G teams of G lanes each hold the whole row and take the entries in turn (team t the entries
// t, t + S, ... of every block of 64), 16 or 32 gathers in flight per wavefront step; the teams' sums, minima and
// maxima are folded pair by pair afterwards.  A row of more than kLongRow entries is shared by the kLongWaves
// wavefronts of a workgroup in the same way, block of 64 entries by block, and their results are folded in
// wavefront order.  Which lane adds which entry depends on the row's length and the width alone, so the order of
// every sum is fixed.

template <bool BF, int G>
__device__ __forceinline__ void pna_gather(const PnaArgs& a, int b, int e, int first, int stride,
                                           float (&sum)[Elems<BF>::E], float (&mn)[Elems<BF>::E], float (&mx)[Elems<BF>::E]) {
    constexpr int E = Elems<BF>::E, EB = BF ? 2 : 4, S = 64 / G, U = S == 1 ? 16 : 32 / S;
    const int lane = threadIdx.x & 63, team = lane / G, tl = lane % G;
    const bool on = tl * E < a.F;
#pragma unroll
    for (int i = 0; i < E; ++i) { sum[i] = 0.f; mn[i] = INFINITY; mx[i] = -INFINITY; }
    for (int k0 = b + 64 * first; k0 < e; k0 += 64 * stride) {
        const int cnt = min(64, e - k0);
        const int mine = lane < cnt ? a.col[k0 + lane] : 0;
        for (int j0 = 0; j0 < cnt; j0 += U * S) {
            u32x4 r[U];
#pragma unroll
            for (int j = 0; j < U; ++j) {
                const int kk = j0 + j * S + team;
                int c;
                if constexpr (S == 1) c = __builtin_amdgcn_readlane(mine, kk & 63);
                else c = __shfl(mine, kk & 63);
                r[j] = u32x4{0u, 0u, 0u, 0u};
                if (on && kk < cnt)
                    r[j] = *reinterpret_cast<const u32x4*>(a.X + ((int64_t)c * a.ldx + (int64_t)tl * E) * EB);
            }
#pragma unroll
            for (int j = 0; j < U; ++j) {
                if (j0 + j * S + team < cnt) {
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
#pragma unroll
    for (int o = G; o < 64; o <<= 1) {
#pragma unroll
        for (int i = 0; i < E; ++i) {
            sum[i] += __shfl_xor(sum[i], o);
            mn[i] = fminf(mn[i], __shfl_xor(mn[i], o));
            mx[i] = fmaxf(mx[i], __shfl_xor(mx[i], o));
        }
    }
}

// The nine output blocks of row v from its folded sums; every team of the wavefront holds them, and team t stores
// the blocks of the aggregators j with j % S == t.
template <bool BF, int G>
__device__ __forceinline__ void pna_finish(const PnaArgs& a, int64_t v, int n_entries, const float (&sum)[Elems<BF>::E],
                                           const float (&mn)[Elems<BF>::E], const float (&mx)[Elems<BF>::E]) {
    constexpr int E = Elems<BF>::E, EB = BF ? 2 : 4, S = 64 / G;
    const int lane = threadIdx.x & 63, team = lane / G, tl = lane % G;
    if (tl * E >= a.F) return;
    const bool any = n_entries > 0;
    const float d = (float)n_entries;
    const float s = logf(d + 1.f) * a.inv_delta;
    float q[E];
#pragma unroll
    for (int i = 0; i < E; ++i) q[i] = 0.f;
    if (a.add && any) unpack<BF>(*reinterpret_cast<const u32x4*>(a.add + (v * a.ldadd + (int64_t)tl * E) * EB), q);
    float agg[3][E];
    const float inv_d = any ? 1.f / d : 0.f;
#pragma unroll
    for (int i = 0; i < E; ++i) {
        agg[0][i] = any ? sum[i] * inv_d + q[i] : 0.f;
        agg[1][i] = any ? mn[i] + q[i] : 0.f;
        agg[2][i] = any ? mx[i] + q[i] : 0.f;
    }
    const float inv_s = any ? 1.f / s : 0.f;
    char* o = a.out + (v * a.ldout + (int64_t)tl * E) * EB;
#pragma unroll
    for (int j = 0; j < 3; ++j) {
        if (j % S != team) continue;
        float t1[E], t2[E];
#pragma unroll
        for (int i = 0; i < E; ++i) { t1[i] = s * agg[j][i]; t2[i] = agg[j][i] * inv_s; }
        __builtin_nontemporal_store(pack<BF>(agg[j]), reinterpret_cast<u32x4*>(o + (int64_t)j * a.F * EB));
        __builtin_nontemporal_store(pack<BF>(t1), reinterpret_cast<u32x4*>(o + (int64_t)(3 + j) * a.F * EB));
        __builtin_nontemporal_store(pack<BF>(t2), reinterpret_cast<u32x4*>(o + (int64_t)(6 + j) * a.F * EB));
    }
}

// one wavefront per row; long rows are left to pna_long_rows_kernel
template <bool BF, int G>
__global__ __launch_bounds__(64) void pna_rows_kernel(PnaArgs a) {
    constexpr int E = Elems<BF>::E;
    const int64_t v = blockIdx.x;
    const int b = a.rowptr[v], e = a.rowptr[v + 1];
    if (e - b > kLongRow) return;
    float sum[E], mn[E], mx[E];
    pna_gather<BF, G>(a, b, e, 0, 1, sum, mn, mx);
    pna_finish<BF, G>(a, v, e - b, sum, mn, mx);
}

// Workgroup w looks at the rows w, w + gridDim.x, ... (512 of them at a time), and every row of more than kLongRow
// entries among them is gathered by all its wavefronts together.
template <bool BF, int G>
__global__ __launch_bounds__(64 * kLongWaves) void pna_long_rows_kernel(PnaArgs a) {
    constexpr int E = Elems<BF>::E, T = 64 * kLongWaves;
    __shared__ int queue[T];
    __shared__ int n_queued;
    __shared__ float red[kLongWaves][3][E][64];
    const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
    for (int64_t r0 = blockIdx.x; r0 < a.n_rows; r0 += (int64_t)T * gridDim.x) {
        const int nq = queue_long_rows(a.rowptr, a.n_rows, r0, queue, &n_queued);
        for (int q = 0; q < nq; ++q) {
            const int64_t v = queue[q];
            const int b = a.rowptr[v], e = a.rowptr[v + 1];
            float sum[E], mn[E], mx[E];
            pna_gather<BF, G>(a, b, e, w, kLongWaves, sum, mn, mx);
            if (w > 0) {
#pragma unroll
                for (int i = 0; i < E; ++i) { red[w][0][i][lane] = sum[i]; red[w][1][i][lane] = mn[i]; red[w][2][i][lane] = mx[i]; }
            }
            __syncthreads();
            if (w == 0) {
                for (int o = 1; o < kLongWaves; ++o) {
#pragma unroll
                    for (int i = 0; i < E; ++i) {
                        sum[i] += red[o][0][i][lane];
                        mn[i] = fminf(mn[i], red[o][1][i][lane]);
                        mx[i] = fmaxf(mx[i], red[o][2][i][lane]);
                    }
                }
                pna_finish<BF, G>(a, v, e - b, sum, mn, mx);
            }
            __syncthreads();
        }
    }
}

// rows of more than 64 pieces: one wavefront per row; lane l owns the pieces l, l + 64, ... and the row's entries
// are walked once per 64 pieces
template <bool BF>
__global__ __launch_bounds__(64) void pna_wide_rows_kernel(PnaArgs a) {
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

template <bool BF, int G>
void launch_rows(const PnaArgs& a, hipStream_t s) {
    hipLaunchKernelGGL((pna_rows_kernel<BF, G>), dim3((unsigned)a.n_rows), dim3(64), 0, s, a);
    const unsigned blocks = long_row_blocks(a.n_rows);
    hipLaunchKernelGGL((pna_long_rows_kernel<BF, G>), dim3(blocks), dim3(64 * kLongWaves), 0, s, a);
}

template <bool BF>
void launch_vec(const PnaArgs& a, hipStream_t s) {
    const int pieces = a.F / Elems<BF>::E;
    if (pieces <= 16) launch_rows<BF, 16>(a, s);
    else if (pieces <= 32) launch_rows<BF, 32>(a, s);
    else if (pieces <= 64) launch_rows<BF, 64>(a, s);
    else hipLaunchKernelGGL(pna_wide_rows_kernel<BF>, dim3((unsigned)a.n_rows), dim3(64), 0, s, a);
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
        if (dt == GAS_BF16) launch_vec<true>(a, s);
        else launch_vec<false>(a, s);
    } else {
        const int64_t blocks = (n_rows * F + 255) / 256;
        GAS_REQUIRE(blocks <= 0x7FFFFFFFLL, "gas_pna_aggregate: problem too large for the element-wise path");
        if (dt == GAS_BF16) hipLaunchKernelGGL(pna_generic_kernel<true>, dim3((unsigned)blocks), dim3(256), 0, s, a);
        else hipLaunchKernelGGL(pna_generic_kernel<false>, dim3((unsigned)blocks), dim3(256), 0, s, a);
    }
    GAS_CHECK_HIP(hipGetLastError());
    return GAS_OK;
}
