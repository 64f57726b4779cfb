// Backward passes of the PNA and GAT aggregations (paper, operator appendix; the chain rule on their equations).
//
// Both aggregations gather rows by column index, so their adjoint scatters to those rows.  To stay free of
// atomics and keep a fixed summation order the scatter is turned around, as for the sum aggregation: a first kernel
// walks the rows of the pattern (CSR) and leaves, per row or per entry, the factors the adjoint needs; a second
// kernel walks the columns (the CSC copy, with the position of every entry in the CSR arrays) and sums, for each
// column, the contributions of its entries in stored order.
//
// Two sets of kernels.  The plain ones (one wavefront per row / column, one entry at a time, any width and
// alignment) are the definition and the fallback.  The fast ones take rows of at most 64 pieces of 16 bytes: the
// row pass gathers as the forward kernels do (a whole neighbour row per wavefront-wide load, several in flight),
// and the dense part of the column pass -- a sum of whole rows weighted per entry -- is the backward aggregation
// gas_spmm_t itself, with its plan for the CSC copy; what is left for kernels of this file is per-entry scalars
// and short lists.
#include <initializer_list>

#include "plan.h"
#include "wave.h"

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

// ---- fast path: rows of at most 64 pieces of 16 bytes
//
// The mean's share of the gradient is a sum of whole rows (C0[v] = c_mean / d for every entry of column u): that is
// the backward aggregation gas_spmm_t on C0.  Minimum and maximum pass their gradient to ONE entry per row and
// feature, so over all rows there are only 2 F n_rows such contributions, against F nnz for the mean.  The row pass
// therefore leaves them as short lists: for every row two lists of F (feature, value) items, one for the minima and
// one for the maxima, sorted by the entry that won them, and for every entry of the pattern where its items start
// in its row's lists and how many they are.  The column pass walks a column's entries in stored order and adds each
// entry's few items to the column's sums (kept in LDS, since an item names any feature): minima first, then maxima,
// entry after entry, so the order of every sum is fixed.
constexpr int kPnaChunk = 512;          // entries of a row whose items are counted and placed in one go

struct PnaFastArgs {
    const int32_t* rowptr; const int32_t* col; int64_t n_rows;
    const int32_t* colptr; const int32_t* row; const int32_t* csc_pos; int64_t n_out;
    const char* X; int64_t ldx;
    const char* G; int64_t ldg;
    char* GX; int64_t ldgx;
    char* Gadd; int64_t ldga;
    char* C0;              // [n_rows, F] in the storage type: c_mean / d
    uint16_t* items_f;     // [n_rows][2][F]: features, minima then maxima, each sorted by the winning entry
    float* items_v;        // [n_rows][2][F]: their values c_min / c_max
    uint2* ent;            // [nnz]: x = start | count << 16 in the row's minima list, y = the same for the maxima
    int F;
    float inv_delta;
};

// Row v = [b, e), b < e.  G: lanes that hold a row (at least its number of pieces).  With G < 64 the wavefront's
// S = 64 / G teams each hold the row and take the entries in turn while gathering (team t the entries t, t + S, ...);
// their winners are merged before the rest, which the lanes of team 0 do as lanes 0 .. G - 1 of the wavefront.
// W = 1: one wavefront has the whole row.  W = kLongWaves: the wavefronts of a workgroup gather the row's blocks of
// 64 entries in turn (wavefront w the blocks w, w + W, ...), their winners are merged through LDS (redv, redk:
// W x E x 64 values each), and wavefront 0 does the rest while the others wait at its barriers.
template <bool BF, int G, int W>
__device__ __forceinline__ void pna_bwd_row(const PnaFastArgs& a, int64_t v, int b, int e, uint32_t (*cnt)[kPnaChunk],
                                            float* redv, int* redk) {
    constexpr int E = Elems<BF>::E, EB = BF ? 2 : 4, S = 64 / G, U = 16 / (S > 2 ? 2 : 1);
    const int lane = threadIdx.x & 63, team = lane / G, tl = lane % G;
    const int w = W == 1 ? 0 : (int)(threadIdx.x >> 6);
    const int d = e - b;
    float mn[E], mx[E];
    int kmn[E], kmx[E];
#pragma unroll
    for (int i = 0; i < E; ++i) { mn[i] = INFINITY; mx[i] = -INFINITY; kmn[i] = b; kmx[i] = b; }
    const bool gon = tl * E < a.F;
    for (int k0 = b + 64 * w; k0 < e; k0 += 64 * W) {
        const int n64 = min(64, e - k0);
        const int mine = lane < n64 ? a.col[k0 + lane] : 0;
        for (int j0 = 0; j0 < n64; j0 += U * S) {
            u32x4 r[U];
#pragma unroll
            for (int j = 0; j < U; ++j) {
                const int kk = j0 + j * S + team;
                int c;
                if constexpr (S == 1) c = __builtin_amdgcn_readlane(mine, kk & 63);
                else c = __shfl(mine, kk & 63);
                r[j] = u32x4{0u, 0u, 0u, 0u};
                if (gon && kk < n64)
                    r[j] = *reinterpret_cast<const u32x4*>(a.X + ((int64_t)c * a.ldx + (int64_t)tl * E) * EB);
            }
#pragma unroll
            for (int j = 0; j < U; ++j) {
                const int kk = j0 + j * S + team;
                if (kk < n64) {
                    float x[E];
                    unpack<BF>(r[j], x);
                    const int k = k0 + kk;
#pragma unroll
                    for (int i = 0; i < E; ++i) {
                        if (x[i] < mn[i]) { mn[i] = x[i]; kmn[i] = k; }      // strict: the first entry that attains it
                        if (x[i] > mx[i]) { mx[i] = x[i]; kmx[i] = k; }
                    }
                }
            }
        }
    }
    // the teams' winners merged: the smaller (larger) value, and of equal values the earlier entry
#pragma unroll
    for (int o = G; o < 64; o <<= 1) {
#pragma unroll
        for (int i = 0; i < E; ++i) {
            const float xn = __shfl_xor(mn[i], o), xx = __shfl_xor(mx[i], o);
            const int kn = __shfl_xor(kmn[i], o), kx = __shfl_xor(kmx[i], o);
            if (xn < mn[i] || (xn == mn[i] && kn < kmn[i])) { mn[i] = xn; kmn[i] = kn; }
            if (xx > mx[i] || (xx == mx[i] && kx < kmx[i])) { mx[i] = xx; kmx[i] = kx; }
        }
    }
    if constexpr (W > 1) {                            // the wavefronts' winners, by the same rule: minima, then maxima
        if (w > 0) {
#pragma unroll
            for (int i = 0; i < E; ++i) { redv[(w * E + i) * 64 + lane] = mn[i]; redk[(w * E + i) * 64 + lane] = kmn[i]; }
        }
        __syncthreads();
        if (w == 0) {
            for (int o = 1; o < W; ++o) {
#pragma unroll
                for (int i = 0; i < E; ++i) {
                    const float xn = redv[(o * E + i) * 64 + lane];
                    const int kn = redk[(o * E + i) * 64 + lane];
                    if (xn < mn[i] || (xn == mn[i] && kn < kmn[i])) { mn[i] = xn; kmn[i] = kn; }
                }
            }
        }
        __syncthreads();
        if (w > 0) {
#pragma unroll
            for (int i = 0; i < E; ++i) { redv[(w * E + i) * 64 + lane] = mx[i]; redk[(w * E + i) * 64 + lane] = kmx[i]; }
        }
        __syncthreads();
        if (w == 0) {
            for (int o = 1; o < W; ++o) {
#pragma unroll
                for (int i = 0; i < E; ++i) {
                    const float xx = redv[(o * E + i) * 64 + lane];
                    const int kx = redk[(o * E + i) * 64 + lane];
                    if (xx > mx[i] || (xx == mx[i] && kx < kmx[i])) { mx[i] = xx; kmx[i] = kx; }
                }
            }
        }
        __syncthreads();
    }
    const bool active = w == 0;                       // from here on the other wavefronts only keep the barriers
    const bool on = active && lane * E < a.F;
    // the three block gradients folded with their scalers
    const float df = (float)d;
    const float s = logf(df + 1.f) * a.inv_delta;
    float cc[3][E];
    if (on) {
        const char* grow = a.G + (v * a.ldg + (int64_t)lane * E) * EB;
#pragma unroll
        for (int j = 0; j < 3; ++j) {
            float g0[E], g1[E], g2[E];
            unpack<BF>(*reinterpret_cast<const u32x4*>(grow + (int64_t)j * a.F * EB), g0);
            unpack<BF>(*reinterpret_cast<const u32x4*>(grow + (int64_t)(3 + j) * a.F * EB), g1);
            unpack<BF>(*reinterpret_cast<const u32x4*>(grow + (int64_t)(6 + j) * a.F * EB), g2);
#pragma unroll
            for (int i = 0; i < E; ++i) cc[j][i] = g0[i] + s * g1[i] + g2[i] / s;
        }
        float t[E];
#pragma unroll
        for (int i = 0; i < E; ++i) t[i] = cc[0][i] / df;
        *reinterpret_cast<u32x4*>(a.C0 + (v * a.F + (int64_t)lane * E) * EB) = pack<BF>(t);
        if (a.Gadd) {
#pragma unroll
            for (int i = 0; i < E; ++i) t[i] = cc[0][i] + cc[1][i] + cc[2][i];
            *reinterpret_cast<u32x4*>(a.Gadd + (v * a.ldga + (int64_t)lane * E) * EB) = pack<BF>(t);
        }
    } else {
#pragma unroll
        for (int j = 0; j < 3; ++j)
#pragma unroll
            for (int i = 0; i < E; ++i) cc[j][i] = 0.f;
    }
    // the items, sorted by winning entry: count per entry (integer adds in LDS), exclusive scan, place
    uint16_t* itf = a.items_f + v * 2 * a.F;
    float* itv = a.items_v + v * 2 * a.F;
    uint32_t base0 = 0, base1 = 0;
    for (int c0 = 0; c0 < d; c0 += kPnaChunk) {
        const int n = min(kPnaChunk, d - c0);
        if (active)
            for (int t = lane; t < 2 * kPnaChunk; t += 64) (&cnt[0][0])[t] = 0u;
        __syncthreads();
        int r0[E], r1[E];
#pragma unroll
        for (int i = 0; i < E; ++i) {
            const int p0 = kmn[i] - b - c0, p1 = kmx[i] - b - c0;
            r0[i] = (on && p0 >= 0 && p0 < n) ? (int)atomicAdd(&cnt[0][p0], 1u) : -1;
            r1[i] = (on && p1 >= 0 && p1 < n) ? (int)atomicAdd(&cnt[1][p1], 1u) : -1;
        }
        __syncthreads();
        if (active) {
            uint32_t c[2][8], tot0 = 0, tot1 = 0;
#pragma unroll
            for (int t = 0; t < 8; ++t) {
                c[0][t] = cnt[0][lane * 8 + t];
                c[1][t] = cnt[1][lane * 8 + t];
                tot0 += c[0][t];
                tot1 += c[1][t];
            }
            uint32_t inc0 = tot0, inc1 = tot1;
#pragma unroll
            for (int o = 1; o < 64; o <<= 1) {
                const uint32_t t0 = __shfl_up(inc0, o), t1 = __shfl_up(inc1, o);
                if (lane >= o) { inc0 += t0; inc1 += t1; }
            }
            uint32_t ex0 = base0 + inc0 - tot0, ex1 = base1 + inc1 - tot1;
#pragma unroll
            for (int t = 0; t < 8; ++t) {
                const int slot = lane * 8 + t;
                if (slot < n) a.ent[(int64_t)b + c0 + slot] = uint2{ex0 | (c[0][t] << 16), ex1 | (c[1][t] << 16)};
                cnt[0][slot] = ex0;
                cnt[1][slot] = ex1;
                ex0 += c[0][t];
                ex1 += c[1][t];
            }
            base0 += __shfl(inc0, 63);
            base1 += __shfl(inc1, 63);
        }
        __syncthreads();
#pragma unroll
        for (int i = 0; i < E; ++i) {
            if (r0[i] >= 0) {
                const uint32_t pos = cnt[0][kmn[i] - b - c0] + (uint32_t)r0[i];
                itf[pos] = (uint16_t)(lane * E + i);
                itv[pos] = cc[1][i];
            }
            if (r1[i] >= 0) {
                const uint32_t pos = cnt[1][kmx[i] - b - c0] + (uint32_t)r1[i];
                itf[a.F + pos] = (uint16_t)(lane * E + i);
                itv[a.F + pos] = cc[2][i];
            }
        }
        __syncthreads();
    }
}

// one wavefront per row; long rows are left to pna_bwd_long_rows_kernel
template <bool BF, int G>
__global__ __launch_bounds__(64) void pna_bwd_rows_vec_kernel(PnaFastArgs a) {
    constexpr int E = Elems<BF>::E, EB = BF ? 2 : 4;
    __shared__ uint32_t cnt[2][kPnaChunk];
    const int64_t v = blockIdx.x;
    const int lane = threadIdx.x;
    const int b = a.rowptr[v], e = a.rowptr[v + 1];
    if (e == b) {
        if (lane * E < a.F) {
            *reinterpret_cast<u32x4*>(a.C0 + (v * a.F + (int64_t)lane * E) * EB) = u32x4{0u, 0u, 0u, 0u};
            if (a.Gadd) *reinterpret_cast<u32x4*>(a.Gadd + (v * a.ldga + (int64_t)lane * E) * EB) = u32x4{0u, 0u, 0u, 0u};
        }
        return;
    }
    if (e - b > kLongRow) return;
    pna_bwd_row<BF, G, 1>(a, v, b, e, cnt, nullptr, nullptr);
}

template <bool BF, int G>
__global__ __launch_bounds__(64 * kLongWaves) void pna_bwd_long_rows_kernel(PnaFastArgs a) {
    constexpr int E = Elems<BF>::E, T = 64 * kLongWaves;
    __shared__ int queue[T];
    __shared__ int n_queued;
    __shared__ uint32_t cnt[2][kPnaChunk];
    __shared__ float redv[kLongWaves * E * 64];
    __shared__ int redk[kLongWaves * E * 64];
    for (int64_t r0 = blockIdx.x; r0 < a.n_rows; r0 += (int64_t)T * gridDim.x) {
        const int nq = queue_long_rows(a.rowptr, a.n_rows, r0, queue, &n_queued);
        for (int q = 0; q < nq; ++q) {
            const int64_t v = queue[q];
            pna_bwd_row<BF, G, kLongWaves>(a, v, a.rowptr[v], a.rowptr[v + 1], cnt, redv, redk);   // ends with a barrier
        }
    }
}

template <bool BF, int G>
void launch_pna_bwd_rows(const PnaFastArgs& a, hipStream_t s) {
    hipLaunchKernelGGL((pna_bwd_rows_vec_kernel<BF, G>), dim3((unsigned)a.n_rows), dim3(64), 0, s, a);
    const unsigned blocks = long_row_blocks(a.n_rows);
    hipLaunchKernelGGL((pna_bwd_long_rows_kernel<BF, G>), dim3(blocks), dim3(64 * kLongWaves), 0, s, a);
}

// The items of the entries [b, e) of one column (of its blocks of 64 entries first, first + stride, ...), added to
// the sums `acc` by the wavefront: the records of 64 entries are read at once, the items of eight entries are in
// flight at a time, and they are added entry after entry, minima before maxima.
__device__ __forceinline__ void add_items_of_column(const PnaFastArgs& a, int b, int e, float* acc, int first = 0,
                                                    int stride = 1) {
    constexpr int U = 8;
    const int lane = threadIdx.x & 63;
    const int64_t F2 = 2 * (int64_t)a.F;
    for (int q0 = b + 64 * first; q0 < e; q0 += 64 * stride) {
        const int n64 = min(64, e - q0);
        int myv = 0;
        uint32_t rx = 0u, ry = 0u;
        if (lane < n64) {
            myv = a.row[q0 + lane];
            const uint2 rec = a.ent[a.csc_pos[q0 + lane]];
            rx = rec.x;
            ry = rec.y;
        }
        if (__ballot(((rx | ry) >> 16) != 0u) == 0ull) continue;
        for (int j0 = 0; j0 < n64; j0 += U) {
            uint32_t itf[2][U];
            float itv[2][U];
#pragma unroll
            for (int j = 0; j < U; ++j) {
                const int64_t vj = __builtin_amdgcn_readlane(myv, (j0 + j) & 63);
                const uint32_t r[2] = {(uint32_t)__builtin_amdgcn_readlane((int)rx, (j0 + j) & 63),
                                       (uint32_t)__builtin_amdgcn_readlane((int)ry, (j0 + j) & 63)};
#pragma unroll
                for (int w = 0; w < 2; ++w) {
                    itf[w][j] = 0u;
                    itv[w][j] = 0.f;
                    if ((uint32_t)lane < (r[w] >> 16)) {
                        const int64_t idx = vj * F2 + (int64_t)w * a.F + (r[w] & 0xFFFFu) + lane;
                        itf[w][j] = a.items_f[idx];
                        itv[w][j] = a.items_v[idx];
                    }
                }
            }
#pragma unroll
            for (int j = 0; j < U; ++j) {
                const int64_t vj = __builtin_amdgcn_readlane(myv, (j0 + j) & 63);
                const uint32_t r[2] = {(uint32_t)__builtin_amdgcn_readlane((int)rx, (j0 + j) & 63),
                                       (uint32_t)__builtin_amdgcn_readlane((int)ry, (j0 + j) & 63)};
#pragma unroll
                for (int w = 0; w < 2; ++w) {
                    const uint32_t count = r[w] >> 16;
                    if (count == 0u) continue;
                    if ((uint32_t)lane < count) acc[itf[w][j]] += itv[w][j];
                    for (uint32_t t0 = 64u; t0 < count; t0 += 64u) {      // an entry that won more than 64 features
                        if (t0 + lane < count) {
                            const int64_t idx = vj * F2 + (int64_t)w * a.F + (r[w] & 0xFFFFu) + t0 + lane;
                            acc[a.items_f[idx]] += a.items_v[idx];
                        }
                    }
                }
            }
        }
    }
}

// A column of more than kLongWinners entries is shared by the wavefronts of a workgroup (a hub column of 17,000
// entries is 2,000 dependent steps for one wavefront).
constexpr int kLongWinners = 512;

// Column u, after the backward aggregation has left the mean's share in GX[u]: one wavefront per column.  (Four
// columns per wavefront, sixteen lanes each walking its column's entries one by one, was measured slower on both
// benchmark batches: the eight entries in flight per column matter more than the idle lanes.  So was one wavefront
// walking the contiguous entries of 2, 3, 4 or 8 consecutive columns as one list with one set of sums per column:
// fewer wavefronts, each with a longer chain of dependent steps.)
template <bool BF>
__global__ __launch_bounds__(64) void pna_bwd_winners_kernel(PnaFastArgs a) {
    constexpr int E = Elems<BF>::E, EB = BF ? 2 : 4;
    __shared__ float acc[64 * E];
    const int64_t u = blockIdx.x;
    const int lane = threadIdx.x;
    const int b = a.colptr[u], e = a.colptr[u + 1];
    if (b == e) return;                              // the aggregation wrote zeros and nothing is added
    if (e - b > kLongWinners) return;                // pna_bwd_winners_long_kernel
    const bool on = lane * E < a.F;
    char* gx = a.GX + (u * a.ldgx + (int64_t)lane * E) * EB;
    if (on) {
        float g[E];
        unpack<BF>(*reinterpret_cast<const u32x4*>(gx), g);
#pragma unroll
        for (int i = 0; i < E; ++i) acc[lane * E + i] = g[i];
    }
    __syncthreads();
    add_items_of_column(a, b, e, acc);
    __syncthreads();
    if (on) {
        float g[E];
#pragma unroll
        for (int i = 0; i < E; ++i) g[i] = acc[lane * E + i];
        *reinterpret_cast<u32x4*>(gx) = pack<BF>(g);
    }
}

// Columns of more than kLongWinners entries, found as the long rows are: the wavefronts of the workgroup take the
// column's blocks of 64 entries in turn, each with sums of its own in LDS (F floats per wavefront), which are then
// added to the column's row of GX in wavefront order.
template <bool BF>
__global__ __launch_bounds__(64 * kLongWaves) void pna_bwd_winners_long_kernel(PnaFastArgs a) {
    constexpr int E = Elems<BF>::E, EB = BF ? 2 : 4, T = 64 * kLongWaves;
    __shared__ int queue[T];
    __shared__ int n_queued;
    extern __shared__ float sums[];                  // [kLongWaves][F]
    const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
    float* mine = sums + w * a.F;
    for (int64_t r0 = blockIdx.x; r0 < a.n_out; r0 += (int64_t)T * gridDim.x) {
        const int nq = queue_long_rows(a.colptr, a.n_out, r0, queue, &n_queued, kLongWinners);
        for (int q = 0; q < nq; ++q) {
            const int64_t u = queue[q];
            for (int t = lane; t < a.F; t += 64) mine[t] = 0.f;
            add_items_of_column(a, a.colptr[u], a.colptr[u + 1], mine, w, kLongWaves);
            __syncthreads();
            if (w == 0 && lane * E < a.F) {
                char* gx = a.GX + (u * a.ldgx + (int64_t)lane * E) * EB;
                float g[E];
                unpack<BF>(*reinterpret_cast<const u32x4*>(gx), g);
                for (int o = 0; o < kLongWaves; ++o)
#pragma unroll
                    for (int i = 0; i < E; ++i) g[i] += sums[o * a.F + lane * E + i];
                *reinterpret_cast<u32x4*>(gx) = pack<BF>(g);
            }
            __syncthreads();
        }
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

// ---- fast path: rows of at most 64 pieces of 16 bytes
// Row v = [b, e), b < e, as gat_bwd_rows_kernel, with the gathers of the forward kernel: eight neighbour rows in
// flight per lane, both dot products of an entry (with a_src for the score, with GZ[v] for the gradient of its
// attention weight) reduced over the lanes eight entries at a time.  A row of at most G < 64 pieces is held by each
// of the wavefront's S = 64 / G teams of G lanes, which take the entries in turn (team t the entries t, t + S, ...).
// W = 1: one wavefront has the whole row.  W = kLongWaves: the wavefronts of a workgroup take the row's blocks of 64
// entries in turn (wavefront w the blocks w, w + W, ...) and meet for the row's maximum and its three sums, which
// are added in wavefront order; `red` is their W floats of LDS.  Either way entry k is stored and read again by
// one and the same lane, so no lane ever reads another lane's store.
template <bool BF, int G, int W>
__device__ __forceinline__ void gat_bwd_row(const GatBwdArgs& a, int64_t v, int b, int e, float* red) {
    constexpr int E = Elems<BF>::E, EB = BF ? 2 : 4, U = 8, S = 64 / G;
    const int lane = threadIdx.x & 63, team = lane / G, tl = lane % G;
    const int first = W == 1 ? 0 : (int)(threadIdx.x >> 6);
    const bool on = tl * E < a.F;
    auto piece = [&](const char* base, int64_t row_elems) {
        u32x4 t = {0u, 0u, 0u, 0u};
        if (on) t = *reinterpret_cast<const u32x4*>(base + (row_elems + (int64_t)tl * E) * EB);
        return t;
    };
    float ar[E], gz[E], x[E], ad[E];
    unpack<BF>(piece(a.a_src, 0), ar);
    unpack<BF>(piece(a.a_dst, 0), ad);
    unpack<BF>(piece(a.GZ, v * a.ldgz), gz);
    unpack<BF>(piece(a.P, v * a.ldp), x);
    float sv = 0.f;
#pragma unroll
    for (int i = 0; i < E; ++i) sv += ad[i] * x[i];
    sv = team_sum<G>(sv);
    float mx = -INFINITY;
    for (int k0 = b + 64 * first; k0 < e; k0 += 64 * W) {
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
                    r[j] = *reinterpret_cast<const u32x4*>(a.P + ((int64_t)c * a.ldp + (int64_t)tl * E) * EB);
            }
            float sw[U], da[U];
#pragma unroll
            for (int j = 0; j < U; ++j) {
                unpack<BF>(r[j], x);
                sw[j] = 0.f;
                da[j] = 0.f;
#pragma unroll
                for (int i = 0; i < E; ++i) {
                    sw[j] = fmaf(ar[i], x[i], sw[j]);
                    da[j] = fmaf(gz[i], x[i], da[j]);
                }
            }
            team_sum8<G>(sw);
            team_sum8<G>(da);
            // entry j0 + i of the block is stored by lane j0 + i; its two sums are with team i % S, in slot i / S
            const int mine_i = lane - j0;
            float my_t = 0.f, my_da = 0.f;
#pragma unroll
            for (int j = 0; j < U; ++j) {
                float tj = sv + sw[j], dj = da[j];
                if (j * S + team < cnt - j0) mx = fmaxf(mx, tj > 0.f ? tj : a.slope * tj);
                if constexpr (S > 1) {
                    const int src = (mine_i & (S - 1)) * G;
                    tj = __shfl(tj, src);
                    dj = __shfl(dj, src);
                }
                if (mine_i >= j * S && mine_i < (j + 1) * S) { my_t = tj; my_da = dj; }
            }
            if (mine_i >= 0 && mine_i < U * S && lane < cnt) { a.alpha[k0 + lane] = my_t; a.dt[k0 + lane] = my_da; }
        }
    }
#pragma unroll
    for (int o = G; o < 64; o <<= 1) mx = fmaxf(mx, __shfl_xor(mx, o));
    mx = across_waves<W, true>(mx, red);
    float den = 0.f;
    for (int k = b + 64 * first + lane; k < e; k += 64 * W) {
        const float t = a.alpha[k];
        den += expf((t > 0.f ? t : a.slope * t) - mx);
    }
    den = across_waves<W, false>(wave_sum(den), red);
    float mean_da = 0.f;
    for (int k = b + 64 * first + lane; k < e; k += 64 * W) {
        const float t = a.alpha[k];
        mean_da += expf((t > 0.f ? t : a.slope * t) - mx) / den * a.dt[k];
    }
    mean_da = across_waves<W, false>(wave_sum(mean_da), red);
    float sum_dt = 0.f;
    for (int k = b + 64 * first + lane; k < e; k += 64 * W) {
        const float t = a.alpha[k];
        const float al = expf((t > 0.f ? t : a.slope * t) - mx) / den;
        const float dtk = al * (a.dt[k] - mean_da) * (t > 0.f ? 1.f : a.slope);
        a.alpha[k] = al;
        a.dt[k] = dtk;
        sum_dt += dtk;
    }
    sum_dt = across_waves<W, false>(wave_sum(sum_dt), red);
    if (threadIdx.x == 0) a.csum[v] = sum_dt;
}

// one wavefront per row; long rows are left to gat_bwd_long_rows_kernel
template <bool BF, int G>
__global__ __launch_bounds__(64) void gat_bwd_rows_vec_kernel(GatBwdArgs a) {
    const int64_t v = blockIdx.x;
    const int b = a.rowptr[v], e = a.rowptr[v + 1];
    if (e == b) {
        if (threadIdx.x == 0) a.csum[v] = 0.f;
        return;
    }
    if (e - b > kLongRow) return;
    gat_bwd_row<BF, G, 1>(a, v, b, e, nullptr);
}

template <bool BF, int G>
__global__ __launch_bounds__(64 * kLongWaves) void gat_bwd_long_rows_kernel(GatBwdArgs a) {
    constexpr int T = 64 * kLongWaves;
    __shared__ int queue[T];
    __shared__ int n_queued;
    __shared__ float red[kLongWaves];
    for (int64_t r0 = blockIdx.x; r0 < a.n_rows; r0 += (int64_t)T * gridDim.x) {
        const int nq = queue_long_rows(a.rowptr, a.n_rows, r0, queue, &n_queued);
        for (int q = 0; q < nq; ++q) {
            const int64_t v = queue[q];
            gat_bwd_row<BF, G, kLongWaves>(a, v, a.rowptr[v], a.rowptr[v + 1], red);   // ends with a barrier
        }
    }
}

template <bool BF, int G>
void launch_gat_bwd_rows(const GatBwdArgs& a, hipStream_t s) {
    hipLaunchKernelGGL((gat_bwd_rows_vec_kernel<BF, G>), dim3((unsigned)a.n_rows), dim3(64), 0, s, a);
    const unsigned blocks = long_row_blocks(a.n_rows);
    hipLaunchKernelGGL((gat_bwd_long_rows_kernel<BF, G>), dim3(blocks), dim3(64 * kLongWaves), 0, s, a);
}

// The attention weights and the score gradients in the order of the CSC copy: the coefficients of the backward
// aggregation, and the terms of the column totals.
__global__ __launch_bounds__(256) void permute_entries_kernel(const float* __restrict__ alpha, const float* __restrict__ dt,
                                                              const int32_t* __restrict__ pos, int64_t n,
                                                              float* __restrict__ val_t, float* __restrict__ dt_t) {
    const int64_t q = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (q >= n) return;
    const int k = pos[q];
    val_t[q] = alpha[k];
    dt_t[q] = dt[k];
}

// tsum[u] = the column's total of dt.  A wavefront takes 64 consecutive columns, whose terms are contiguous: a lane
// adds the terms of its own column in stored order when there are at most 64 of them.  Longer columns are left to
// column_totals_long_kernel: hub columns sit next to each other, and sixty-four of them in one wavefront's share,
// summed one after the other, were most of this step's time.
constexpr int kLongColumn = 64;

__global__ __launch_bounds__(256) void column_totals_kernel(const int32_t* __restrict__ colptr, const float* __restrict__ dt_t,
                                                            int64_t n_cols, float* __restrict__ tsum) {
    const int64_t u = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (u >= n_cols) return;
    const int b = colptr[u], e = colptr[u + 1];
    if (e - b > kLongColumn) return;
    float ts = 0.f;
    for (int q = b; q < e; q += 8) {                  // eight loads in flight, added in stored order
        float x[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) x[j] = q + j < e ? dt_t[q + j] : 0.f;
#pragma unroll
        for (int j = 0; j < 8; ++j) ts += x[j];
    }
    tsum[u] = ts;
}

// The columns of more than kLongColumn terms, found as the long rows are: one wavefront per column, lanes stride over
// its terms, then a fixed reduction over the lanes.
__global__ __launch_bounds__(64 * kLongWaves) void column_totals_long_kernel(const int32_t* __restrict__ colptr,
                                                                             const float* __restrict__ dt_t, int64_t n_cols,
                                                                             float* __restrict__ tsum) {
    constexpr int T = 64 * kLongWaves;
    __shared__ int queue[T];
    __shared__ int n_queued;
    const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
    for (int64_t r0 = blockIdx.x; r0 < n_cols; r0 += (int64_t)T * gridDim.x) {
        const int nq = queue_long_rows(colptr, n_cols, r0, queue, &n_queued, kLongColumn);
        for (int q = w; q < nq; q += kLongWaves) {
            const int64_t u = queue[q];
            const int b = colptr[u], e = colptr[u + 1];
            float p = 0.f;
            for (int t = b + lane; t < e; t += 64) p += dt_t[t];
            p = wave_sum(p);
            if (lane == 0) tsum[u] = p;
        }
        __syncthreads();
    }
}

// GP[u] += tsum[u] a_src + csum[u] a_dst after the backward aggregation has left sum_k alpha_k GZ[row k] in GP[u]:
// one thread per 16-byte piece.
template <bool BF>
__global__ __launch_bounds__(256) void gat_bwd_rank_one_kernel(GatBwdArgs a) {
    constexpr int E = Elems<BF>::E, EB = BF ? 2 : 4;
    const int pieces = a.F / E;
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= a.n_out * pieces) return;
    const int64_t u = idx / pieces;
    const int p = (int)(idx - u * pieces);
    const float ts = a.tsum[u], cs = u < a.n_rows ? a.csum[u] : 0.f;
    float g[E], ar[E], ad[E];
    char* gp = a.GP + (u * a.ldgp + (int64_t)p * E) * EB;
    unpack<BF>(*reinterpret_cast<const u32x4*>(gp), g);
    unpack<BF>(*reinterpret_cast<const u32x4*>(a.a_src + (int64_t)p * E * EB), ar);
    unpack<BF>(*reinterpret_cast<const u32x4*>(a.a_dst + (int64_t)p * E * EB), ad);
#pragma unroll
    for (int i = 0; i < E; ++i) g[i] = g[i] + ts * ar[i] + cs * ad[i];
    *reinterpret_cast<u32x4*>(gp) = pack<BF>(g);
}

// out[f] = sum_i w[i] M[i, f] in a fixed order: slabs of 1024 rows, one partial row per slab, then groups of 256
// partial rows at a time until one is left.
constexpr int kSlab = 1024;
constexpr int kGroup = 256;
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
// The same for rows of at most 64 pieces of 16 bytes: each of the four wavefronts takes a quarter of the slab, a
// whole row per load, eight rows in flight; the four partial rows are added in wavefront order.
template <bool BF>
__global__ __launch_bounds__(256) void wcolsum_partial_vec_kernel(const char* M, int64_t ldm, const float* w, int64_t n, int F,
                                                                  float* partial) {
    constexpr int E = Elems<BF>::E, EB = BF ? 2 : 4, U = 8;
    __shared__ float part[4][64 * E];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int64_t r0 = (int64_t)blockIdx.x * kSlab + wave * (kSlab / 4), r1 = min(n, r0 + kSlab / 4);
    const bool on = lane * E < F;
    float acc[E];
#pragma unroll
    for (int i = 0; i < E; ++i) acc[i] = 0.f;
    for (int64_t i0 = r0; i0 < r1; i0 += 64) {
        const int cnt = (int)min<int64_t>(64, r1 - i0);
        const float mine = lane < cnt ? w[i0 + lane] : 0.f;
        for (int j0 = 0; j0 < cnt; j0 += U) {
            u32x4 r[U];
#pragma unroll
            for (int j = 0; j < U; ++j) {
                r[j] = u32x4{0u, 0u, 0u, 0u};
                if (on && j0 + j < cnt)
                    r[j] = *reinterpret_cast<const u32x4*>(M + ((i0 + j0 + j) * ldm + (int64_t)lane * E) * EB);
            }
#pragma unroll
            for (int j = 0; j < U; ++j) {
                const float wj = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, mine), (j0 + j) & 63));
                float x[E];
                unpack<BF>(r[j], x);
#pragma unroll
                for (int i = 0; i < E; ++i) acc[i] = fmaf(wj, x[i], acc[i]);     // rows beyond cnt: weight 0, row 0
            }
        }
    }
#pragma unroll
    for (int i = 0; i < E; ++i) part[wave][lane * E + i] = acc[i];
    __syncthreads();
    for (int f = threadIdx.x; f < F; f += 256)
        partial[(int64_t)blockIdx.x * F + f] = ((part[0][f] + part[1][f]) + part[2][f]) + part[3][f];
}
// out[g, f] = sum of the partial rows of group g (kGroup of them), added in order
__global__ __launch_bounds__(256) void wcolsum_reduce_kernel(const float* partial, int64_t n, int F, float* out) {
    const int f = blockIdx.y * 256 + threadIdx.x;
    if (f >= F) return;
    const int64_t i0 = (int64_t)blockIdx.x * kGroup, i1 = min(n, i0 + kGroup);
    double acc = 0.0;
    for (int64_t i = i0; i < i1; ++i) acc += (double)partial[i * F + f];
    out[(int64_t)blockIdx.x * F + f] = (float)acc;
}

int64_t align_up(int64_t x);
int64_t wcolsum_scratch_floats(int64_t n, int F) {
    const int64_t slabs = (n + kSlab - 1) / kSlab;
    return (slabs + (slabs + kGroup - 1) / kGroup + 2) * (int64_t)F;
}
// scratch: wcolsum_scratch_floats(n, F) floats.  n == 0 gives zeros.
void weighted_column_sum(const char* M, int64_t ldm, const float* w, int64_t n, int F, bool bf, bool vec, float* scratch,
                         float* out, hipStream_t s) {
    const int64_t slabs = (n + kSlab - 1) / kSlab;
    const unsigned fblocks = (unsigned)((F + 255) / 256);
    if (slabs > 0) {
        if (vec) {
            if (bf) hipLaunchKernelGGL(wcolsum_partial_vec_kernel<true>, dim3((unsigned)slabs), dim3(256), 0, s, M, ldm, w, n, F, scratch);
            else hipLaunchKernelGGL(wcolsum_partial_vec_kernel<false>, dim3((unsigned)slabs), dim3(256), 0, s, M, ldm, w, n, F, scratch);
        } else {
            if (bf) hipLaunchKernelGGL(wcolsum_partial_kernel<true>, dim3((unsigned)slabs), dim3(256), 0, s, M, ldm, w, n, F, scratch);
            else hipLaunchKernelGGL(wcolsum_partial_kernel<false>, dim3((unsigned)slabs), dim3(256), 0, s, M, ldm, w, n, F, scratch);
        }
    }
    float* cur = scratch;
    float* other = scratch + slabs * (int64_t)F;
    int64_t count = slabs;
    for (;;) {
        const int64_t groups = (count + kGroup - 1) / kGroup;
        if (groups <= 1) {                      // also count == 0: one block whose empty sum writes zeros
            hipLaunchKernelGGL(wcolsum_reduce_kernel, dim3(1, fblocks), dim3(256), 0, s, cur, count, F, out);
            return;
        }
        hipLaunchKernelGGL(wcolsum_reduce_kernel, dim3((unsigned)groups, fblocks), dim3(256), 0, s, cur, count, F, other);
        float* t = cur;
        cur = other;
        other = t;                              // the groups of one level always fit in front of the level before
        count = groups;
    }
}

int64_t align_up(int64_t x) { return (x + 255) / 256 * 256; }

// rows of at most 64 pieces of 16 bytes, every row 16-byte aligned
bool vec_rows(gas_dtype dt, int32_t F, std::initializer_list<const void*> ptrs, std::initializer_list<int64_t> lds) {
    const int e = dt == GAS_BF16 ? 8 : 4;
    if (F % e != 0 || F / e > 64) return false;
    for (const void* p : ptrs)
        if (p && !aligned16(p)) return false;
    for (int64_t ld : lds)
        if (ld % e != 0) return false;
    return true;
}

}  // namespace
}  // namespace gas

using namespace gas;

extern "C" {

int64_t gas_pna_aggregate_bwd_workspace(int64_t n_rows, int64_t nnz, int32_t F) {
    if (n_rows <= 0 || nnz < 0 || F <= 0) return 0;
    const int64_t plain = align_up(n_rows * 3 * (int64_t)F * 4) + align_up(n_rows * 2 * (int64_t)F * 4);
    const int64_t fast = align_up(n_rows * (int64_t)F * 4) + align_up(n_rows * 2 * (int64_t)F * 2) +
                         align_up(n_rows * 2 * (int64_t)F * 4) + align_up(nnz * 8);
    return plain > fast ? plain : fast;
}

gas_status gas_pna_aggregate_bwd(const gas_plan* plan_t, const int32_t* rowptr, const int32_t* col, int64_t n_rows,
                                 int64_t nnz, const int32_t* colptr, const int32_t* row, const int32_t* csc_pos,
                                 int64_t n_out, const void* X, int64_t ldx, gas_dtype dt, int32_t F, float delta,
                                 const void* G, int64_t ldg, void* GX, int64_t ldgx, void* Gadd, int64_t ldga,
                                 void* workspace, int64_t workspace_bytes, void* stream) {
    if (!valid_dtype(dt)) return fail(GAS_ERR_DTYPE, "gas_pna_aggregate_bwd: unknown dtype %d", (int)dt);
    GAS_REQUIRE(n_rows >= 0 && n_out >= 0 && nnz >= 0 && F > 0, "gas_pna_aggregate_bwd: n_rows=%lld n_out=%lld nnz=%lld F=%d",
                (long long)n_rows, (long long)n_out, (long long)nnz, F);
    GAS_REQUIRE(delta > 0.f, "gas_pna_aggregate_bwd: delta must be positive");
    GAS_REQUIRE(n_rows <= 0x7FFFFFFFLL && n_out <= 0x7FFFFFFFLL, "gas_pna_aggregate_bwd: too many rows for one launch");
    if (n_rows == 0 && n_out == 0) return GAS_OK;
    GAS_REQUIRE(n_out == 0 || (colptr && GX && ldgx >= F), "gas_pna_aggregate_bwd: null column pointers or output");
    GAS_REQUIRE(n_rows == 0 || (rowptr && col && row && csc_pos && X && G && ldx >= F && ldg >= 9 * (int64_t)F),
                "gas_pna_aggregate_bwd: null pointer or row stride smaller than the row");
    GAS_REQUIRE(!Gadd || ldga >= F, "gas_pna_aggregate_bwd: row stride of Gadd smaller than F");
    GAS_REQUIRE(n_rows == 0 || (workspace && workspace_bytes >= gas_pna_aggregate_bwd_workspace(n_rows, nnz, F)),
                "gas_pna_aggregate_bwd: workspace of %lld bytes needed, %lld given",
                (long long)gas_pna_aggregate_bwd_workspace(n_rows, nnz, F), (long long)workspace_bytes);
    GAS_REQUIRE(!plan_t || plan_t->n_rows == n_out, "gas_pna_aggregate_bwd: the plan is for %lld columns, n_out is %lld",
                plan_t ? (long long)plan_t->n_rows : 0ll, (long long)n_out);
    hipStream_t s = (hipStream_t)stream;
    const bool bf = dt == GAS_BF16;
    if (plan_t && n_rows > 0 && n_out > 0 && F <= 0xFFFF &&
        vec_rows(dt, F, {X, G, GX, Gadd, workspace}, {ldx, ldg, ldgx, Gadd ? ldga : 0})) {
        char* w = static_cast<char*>(workspace);
        PnaFastArgs a;
        a.rowptr = rowptr; a.col = col; a.n_rows = n_rows;
        a.colptr = colptr; a.row = row; a.csc_pos = csc_pos; a.n_out = n_out;
        a.X = static_cast<const char*>(X); a.ldx = ldx;
        a.G = static_cast<const char*>(G); a.ldg = ldg;
        a.GX = static_cast<char*>(GX); a.ldgx = ldgx;
        a.Gadd = static_cast<char*>(Gadd); a.ldga = ldga;
        a.C0 = w; w += align_up(n_rows * (int64_t)F * 4);
        a.items_f = reinterpret_cast<uint16_t*>(w); w += align_up(n_rows * 2 * (int64_t)F * 2);
        a.items_v = reinterpret_cast<float*>(w); w += align_up(n_rows * 2 * (int64_t)F * 4);
        a.ent = reinterpret_cast<uint2*>(w);
        a.F = F; a.inv_delta = 1.f / delta;
        const int pieces = F / (bf ? 8 : 4);
        if (bf) {
            if (pieces <= 16) launch_pna_bwd_rows<true, 16>(a, s);
            else if (pieces <= 32) launch_pna_bwd_rows<true, 32>(a, s);
            else launch_pna_bwd_rows<true, 64>(a, s);
        } else {
            if (pieces <= 16) launch_pna_bwd_rows<false, 16>(a, s);
            else if (pieces <= 32) launch_pna_bwd_rows<false, 32>(a, s);
            else launch_pna_bwd_rows<false, 64>(a, s);
        }
        GAS_CHECK_HIP(hipGetLastError());
        // the mean's share: GX[u] = sum over the entries (v, u) of C0[v]
        const gas_status st = gas_spmm_t(plan_t, colptr, row, nullptr, 0.f, 1.f, 0, a.C0, F, dt, F, GX, ldgx, dt, stream);
        if (st != GAS_OK) return st;
        if (bf) hipLaunchKernelGGL(pna_bwd_winners_kernel<true>, dim3((unsigned)n_out), dim3(64), 0, s, a);
        else hipLaunchKernelGGL(pna_bwd_winners_kernel<false>, dim3((unsigned)n_out), dim3(64), 0, s, a);
        const size_t sums_bytes = (size_t)kLongWaves * F * 4;
        if (bf) hipLaunchKernelGGL(pna_bwd_winners_long_kernel<true>, dim3(long_row_blocks(n_out)), dim3(64 * kLongWaves), sums_bytes, s, a);
        else hipLaunchKernelGGL(pna_bwd_winners_long_kernel<false>, dim3(long_row_blocks(n_out)), dim3(64 * kLongWaves), sums_bytes, s, a);
        GAS_CHECK_HIP(hipGetLastError());
        return GAS_OK;
    }
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
    if (n_rows > 0) {
        if (bf) hipLaunchKernelGGL(pna_bwd_rows_kernel<true>, dim3((unsigned)n_rows), dim3(64), 0, s, a);
        else hipLaunchKernelGGL(pna_bwd_rows_kernel<false>, dim3((unsigned)n_rows), dim3(64), 0, s, a);
    }
    if (n_out > 0) {
        if (bf) hipLaunchKernelGGL(pna_bwd_cols_kernel<true>, dim3((unsigned)n_out), dim3(64), 0, s, a);
        else hipLaunchKernelGGL(pna_bwd_cols_kernel<false>, dim3((unsigned)n_out), dim3(64), 0, s, a);
    }
    GAS_CHECK_HIP(hipGetLastError());
    return GAS_OK;
}

int64_t gas_gat_aggregate_bwd_workspace(int64_t n_rows, int64_t n_cols, int64_t nnz, int32_t F) {
    if (n_rows < 0 || n_cols <= 0 || nnz < 0 || F <= 0) return 0;
    return 4 * align_up(nnz * 4) + align_up(n_rows * 4) + align_up(n_cols * 4) +
           2 * align_up(wcolsum_scratch_floats(n_cols, F) * 4);
}

gas_status gas_gat_aggregate_bwd(const gas_plan* plan_t, const int32_t* rowptr, const int32_t* col, int64_t n_rows,
                                 const int32_t* colptr, const int32_t* row, const int32_t* csc_pos, int64_t n_cols,
                                 int64_t n_out, int64_t nnz, const void* P, int64_t ldp, gas_dtype dt, int32_t F,
                                 const void* a_dst, const void* a_src, float negative_slope, const void* GZ,
                                 int64_t ldgz, void* GP, int64_t ldgp, float* Ga_dst, float* Ga_src, void* workspace,
                                 int64_t workspace_bytes, void* stream) {
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
    GAS_REQUIRE(!plan_t || plan_t->n_rows == n_out, "gas_gat_aggregate_bwd: the plan is for %lld columns, n_out is %lld",
                plan_t ? (long long)plan_t->n_rows : 0ll, (long long)n_out);
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
    float* val_t = reinterpret_cast<float*>(w); w += align_up(nnz * 4);
    float* dt_t = reinterpret_cast<float*>(w); w += align_up(nnz * 4);
    a.csum = reinterpret_cast<float*>(w); w += align_up(n_rows * 4);
    a.tsum = reinterpret_cast<float*>(w); w += align_up(n_cols * 4);
    float* part_dst = reinterpret_cast<float*>(w); w += align_up(wcolsum_scratch_floats(n_cols, F) * 4);
    float* part_src = reinterpret_cast<float*>(w);
    a.F = F; a.slope = negative_slope;
    hipStream_t s = (hipStream_t)stream;
    const bool bf = dt == GAS_BF16;
    const bool vec = vec_rows(dt, F, {P, GZ, GP, a_dst, a_src}, {ldp, ldgz, ldgp});
    if (plan_t && n_out > 0 && vec) {
        if (n_rows > 0) {
            const int pieces = F / (bf ? 8 : 4);
            if (bf) {
                if (pieces <= 16) launch_gat_bwd_rows<true, 16>(a, s);
                else if (pieces <= 32) launch_gat_bwd_rows<true, 32>(a, s);
                else launch_gat_bwd_rows<true, 64>(a, s);
            } else {
                if (pieces <= 16) launch_gat_bwd_rows<false, 16>(a, s);
                else if (pieces <= 32) launch_gat_bwd_rows<false, 32>(a, s);
                else launch_gat_bwd_rows<false, 64>(a, s);
            }
        }
        GAS_REQUIRE(plan_t->nnz <= nnz, "gas_gat_aggregate_bwd: the plan has %lld entries, the pattern %lld",
                    (long long)plan_t->nnz, (long long)nnz);
        if (nnz > 0)
            hipLaunchKernelGGL(permute_entries_kernel, dim3((unsigned)((nnz + 255) / 256)), dim3(256), 0, s, a.alpha, a.dt,
                               csc_pos, nnz, val_t, dt_t);
        hipLaunchKernelGGL(column_totals_kernel, dim3((unsigned)((n_cols + 255) / 256)), dim3(256), 0, s, colptr, dt_t, n_cols,
                           a.tsum);
        hipLaunchKernelGGL(column_totals_long_kernel, dim3(long_row_blocks(n_cols)), dim3(64 * kLongWaves), 0, s, colptr, dt_t,
                           n_cols, a.tsum);
        GAS_CHECK_HIP(hipGetLastError());
        // GP[u] = sum over the entries (v, u) of alpha GZ[v]: the backward aggregation with the attention weights
        // as coefficients, in the order of the CSC copy; then the two rank-one terms
        const gas_status st = gas_spmm_t(plan_t, colptr, row, val_t, 0.f, 1.f, 0, GZ, ldgz, dt, F, GP, ldgp, dt, stream);
        if (st != GAS_OK) return st;
        const int64_t pieces = n_out * (F / (bf ? 8 : 4));
        GAS_REQUIRE((pieces + 255) / 256 <= 0x7FFFFFFFLL, "gas_gat_aggregate_bwd: output too large for one launch");
        if (bf) hipLaunchKernelGGL(gat_bwd_rank_one_kernel<true>, dim3((unsigned)((pieces + 255) / 256)), dim3(256), 0, s, a);
        else hipLaunchKernelGGL(gat_bwd_rank_one_kernel<false>, dim3((unsigned)((pieces + 255) / 256)), dim3(256), 0, s, a);
    } else {
        if (n_rows > 0) {
            if (bf) hipLaunchKernelGGL(gat_bwd_rows_kernel<true>, dim3((unsigned)n_rows), dim3(64), 0, s, a);
            else hipLaunchKernelGGL(gat_bwd_rows_kernel<false>, dim3((unsigned)n_rows), dim3(64), 0, s, a);
        }
        if (bf) hipLaunchKernelGGL(gat_bwd_cols_kernel<true>, dim3((unsigned)n_cols), dim3(64), 0, s, a);
        else hipLaunchKernelGGL(gat_bwd_cols_kernel<false>, dim3((unsigned)n_cols), dim3(64), 0, s, a);
    }
    // Ga_dst = sum over the in-batch nodes of (row total of dt) P[v];  Ga_src = sum over all nodes of (column total) P[u]
    weighted_column_sum(a.P, ldp, a.csum, n_rows, F, bf, vec, part_dst, Ga_dst, s);
    weighted_column_sum(a.P, ldp, a.tsum, n_cols, F, bf, vec, part_src, Ga_src, s);
    GAS_CHECK_HIP(hipGetLastError());
    return GAS_OK;
}

}  // extern "C"
