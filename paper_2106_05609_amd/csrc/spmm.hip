// Neighbourhood aggregation over the batch subgraph (gas_spmm) and its adjoint
// (gas_spmm_t): row-parallel compressed-sparse-row products without atomics.
//
// What is computed is the sum of the paper's Eq. (1)/(2) for the in-batch
// rows, with the edge weights of the GCN / GCNII / GIN operators folded into
// `val`, `diag`, `s_agg` and the residual term.
//
// Mapping to the machine.  A feature row is cut into 16-byte units; a "team" of
// G = 2^k lanes (G >= units per row, at most 64) owns one row, so one wavefront
// works on 64/G neighbours at a time and a wavefront-wide load instruction
// always fetches whole contiguous rows.  The wavefront stages 64 column
// indices and weights at a time in registers (one coalesced load) and
// broadcasts them with lane permutes; U independent row loads are in flight
// per lane.  Rows with at most `threshold` entries take one wavefront each.
// Heavier rows (power-law hubs) are cut into chunks of at most `chunk` entries,
// one wavefront per chunk (spmm_chunk_kernel), whose fp32 partial sums go to a
// workspace and are added in a fixed order by spmm_heavy_reduce_kernel; the
// light rows follow in spmm_rows_kernel.  The chunks are cut and ordered by
// L2-sized windows of the source rows (plan_host.h states the rules), so that
// wavefronts running together gather from rows that fit the L2 of every XCD.
// The summation order is a
// function of the plan alone, so results are bit-identical from run to run.
#include "common.h"
#include "plan.h"

#include <algorithm>
#include <string.h>
#include <vector>

namespace gas {
namespace {

struct SpmmArgs {
    const int32_t* ptr;
    const int32_t* ind;
    const float* val;
    const char* X;
    int64_t x_stride;     // bytes
    const char* H;        // history table for entries with a negative index (row -1-index), or null
    int64_t h_stride;
    const char* R;
    int64_t r_stride;
    char* Z;
    int64_t z_stride;
    float diag, s_agg, s_res;
    int64_t n_rows, n_diag;
    int units;            // 16-byte units per row of X
    int F;
    int threshold;
    const int32_t* chunk;       // plan lists
    int64_t n_chunks;
    const int32_t* heavy;
    int64_t n_heavy;
    float* partial;
    const int32_t* group;       // row groups of the light rows (wave-per-row path)
    int64_t n_groups;
    int xcd_ranges;       // grouped light rows: one contiguous range of groups per XCD, [xcd_start[x], xcd_start[x+1])
    int64_t xcd_start[9];
};

template <bool XBF>
struct Unit {
    static constexpr int E = XBF ? 8 : 4;   // elements per 16-byte unit
    static __device__ __forceinline__ void fma(float (&acc)[E], float w, const u32x4& v) {
        if constexpr (XBF) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                acc[2 * i] = fmaf(w, bf16_lo(v[i]), acc[2 * i]);
                acc[2 * i + 1] = fmaf(w, bf16_hi(v[i]), acc[2 * i + 1]);
            }
        } else {
#pragma unroll
            for (int i = 0; i < 4; ++i) acc[i] = fmaf(w, __uint_as_float(v[i]), acc[i]);
        }
    }
};

template <int G>
__device__ __forceinline__ int bcast_i(int v, int k) {
    if constexpr (G == 64) return __builtin_amdgcn_readlane(v, k);
    else return __shfl(v, k, 64);
}
template <int G>
__device__ __forceinline__ float bcast_f(float v, int k) {
    if constexpr (G == 64) return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), k));
    else return __shfl(v, k, 64);
}

// Sum of val[k] * X[ind[k], :] over k in [begin, end) for this lane's units.
// Afterwards every team of the wavefront holds the full sum.
template <int G, int UPT, int U, bool XBF>
__device__ __forceinline__ void accumulate(const SpmmArgs& a, int begin, int end,
                                           float (&acc)[UPT][Unit<XBF>::E]) {
    constexpr int S = kWave / G;
    constexpr int E = Unit<XBF>::E;
    const int lane = threadIdx.x & 63;
    const int team = lane / G, tl = lane % G;
#pragma unroll
    for (int p = 0; p < UPT; ++p)
#pragma unroll
        for (int e = 0; e < E; ++e) acc[p][e] = 0.f;
    const char* xb = a.X + (int64_t)tl * 16;
    const char* hb = a.H + (int64_t)tl * 16;
    const int nunits = a.units;
    for (int t = begin; t < end; t += kWave) {
        const int cnt = min(kWave, end - t);
        int my_c = 0;
        float my_w = 0.f;
        if (lane < cnt) {
            my_c = __builtin_nontemporal_load(a.ind + t + lane);     // streamed once: keep it out of the way of X in L2
            my_w = a.val ? __builtin_nontemporal_load(a.val + t + lane) : 1.f;
        }
        for (int j = 0; j < cnt; j += S * U) {
            u32x4 v[U][UPT];
            float w[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int k = j + u * S + team;
                const bool ok = k < cnt;
                const int c = bcast_i<G>(my_c, k & 63);
                const float ww = bcast_f<G>(my_w, k & 63);
                w[u] = ok ? ww : 0.f;
#pragma unroll
                for (int p = 0; p < UPT; ++p) {
                    v[u][p] = u32x4{0u, 0u, 0u, 0u};
                    // index >= 0: row of the mini-batch tensor; index < 0: row -1-index of the history table
                    const bool in_batch = c >= 0;
                    const char* src = (in_batch ? xb : hb) +
                                      (int64_t)(in_batch ? c : -1 - c) * (in_batch ? a.x_stride : a.h_stride);
                    if (ok && tl + p * G < nunits)
                        v[u][p] = *reinterpret_cast<const u32x4*>(src + (int64_t)p * G * 16);
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u)
#pragma unroll
                for (int p = 0; p < UPT; ++p) Unit<XBF>::fma(acc[p], w[u], v[u][p]);
        }
    }
    if constexpr (S > 1) {
#pragma unroll
        for (int off = G; off < kWave; off <<= 1)
#pragma unroll
            for (int p = 0; p < UPT; ++p)
#pragma unroll
                for (int e = 0; e < E; ++e) acc[p][e] += __shfl_xor(acc[p][e], off, 64);
    }
}

// Z[row, unit] = s_agg * acc + diag * X[row, unit] + s_res * R[row, unit]
template <bool XBF, bool ZBF>
__device__ __forceinline__ void epilogue(const SpmmArgs& a, int64_t row, int unit, float (&acc)[Unit<XBF>::E]) {
    constexpr int E = Unit<XBF>::E;
    float z[E];
#pragma unroll
    for (int e = 0; e < E; ++e) z[e] = a.s_agg * acc[e];
    if (a.diag != 0.f && row < a.n_diag) {
        float t[E];
#pragma unroll
        for (int e = 0; e < E; ++e) t[e] = 0.f;
        Unit<XBF>::fma(t, a.diag, *reinterpret_cast<const u32x4*>(a.X + row * a.x_stride + (int64_t)unit * 16));
#pragma unroll
        for (int e = 0; e < E; ++e) z[e] += t[e];
    }
    if (a.R) {
        float t[E];
#pragma unroll
        for (int e = 0; e < E; ++e) t[e] = 0.f;
        Unit<XBF>::fma(t, a.s_res, *reinterpret_cast<const u32x4*>(a.R + row * a.r_stride + (int64_t)unit * 16));
#pragma unroll
        for (int e = 0; e < E; ++e) z[e] += t[e];
    }
    char* zp = a.Z + row * a.z_stride;
    if constexpr (ZBF) {
        static_assert(!ZBF || XBF, "bf16 output needs bf16 input");
        u32x4 o;
#pragma unroll
        for (int i = 0; i < 4; ++i) o[i] = pack_bf16(z[2 * i], z[2 * i + 1]);
        __builtin_nontemporal_store(o, reinterpret_cast<u32x4*>(zp + (int64_t)unit * 16));
    } else {
#pragma unroll
        for (int q = 0; q < E / 4; ++q) {
            f32x4 o = {z[4 * q], z[4 * q + 1], z[4 * q + 2], z[4 * q + 3]};
            __builtin_nontemporal_store(o, reinterpret_cast<f32x4*>(zp + ((int64_t)unit * E + 4 * q) * 4));
        }
    }
}

// ---- wave-per-row path for rows of exactly 64 vectors of VB bytes (1 KiB, 512 B or 256 B)
// Short rows are the common case on power-law graphs, and one wavefront per row
// pays three dependent memory latencies (row pointers, indices, feature rows)
// for a handful of gathers.  Here consecutive light rows are bundled at plan
// time into groups of at most 64 entries and 63 rows: the wavefront loads the
// group's row pointers with one load and all its indices and weights with
// another, then streams the gathers of the whole group, 8 in flight per lane,
// flushing a row (epilogue + store) whenever the entry cursor crosses a row
// boundary.  Every lane works on every row (lane l owns bytes [l*VB, (l+1)*VB) of
// the row), all control flow is wavefront-uniform, and the order of summation
// within a row is the stored order.
template <int VB> struct VecOf;
template <> struct VecOf<16> { typedef u32x4 type; };
template <> struct VecOf<8> { typedef u32x2 type; };
typedef uint32_t u32x1 __attribute__((ext_vector_type(1)));
template <> struct VecOf<4> { typedef u32x1 type; };

template <int VB, bool XBF>
struct LaneAcc {
    static constexpr int NW = VB / 4;                 // dwords per lane and row
    static constexpr int E = XBF ? 2 * NW : NW;       // elements per lane and row
    typedef typename VecOf<VB>::type V;
    float v[E];
    __device__ __forceinline__ void clear() {
#pragma unroll
        for (int e = 0; e < E; ++e) v[e] = 0.f;
    }
    __device__ __forceinline__ void fma(float w, const V& x) {
#pragma unroll
        for (int i = 0; i < NW; ++i) {
            if constexpr (XBF) {
                v[2 * i] = fmaf(w, bf16_lo(x[i]), v[2 * i]);
                v[2 * i + 1] = fmaf(w, bf16_hi(x[i]), v[2 * i + 1]);
            } else {
                v[i] = fmaf(w, __uint_as_float(x[i]), v[i]);
            }
        }
    }
};

template <int VB, bool XBF, bool ZBF>
__device__ __forceinline__ void flush_row(const SpmmArgs& a, int64_t row, int lane, LaneAcc<VB, XBF>& acc,
                                          const typename VecOf<VB>::type& own) {
    // `own` = this lane's piece of X[row, :], loaded ahead of time by the caller (only read when diag != 0)
    typedef typename VecOf<VB>::type V;
    constexpr int E = LaneAcc<VB, XBF>::E, NW = VB / 4;
    float z[E];
#pragma unroll
    for (int e = 0; e < E; ++e) z[e] = a.s_agg * acc.v[e];
    if (a.diag != 0.f && row < a.n_diag) {
        LaneAcc<VB, XBF> t;
        t.clear();
        t.fma(a.diag, own);
#pragma unroll
        for (int e = 0; e < E; ++e) z[e] += t.v[e];
    }
    if (a.R) {
        LaneAcc<VB, XBF> t;
        t.clear();
        t.fma(a.s_res, *reinterpret_cast<const V*>(a.R + row * a.r_stride + (int64_t)lane * VB));
#pragma unroll
        for (int e = 0; e < E; ++e) z[e] += t.v[e];
    }
    char* zp = a.Z + row * a.z_stride;
    if constexpr (ZBF) {
        V o;
#pragma unroll
        for (int i = 0; i < NW; ++i) o[i] = pack_bf16(z[2 * i], z[2 * i + 1]);
        __builtin_nontemporal_store(o, reinterpret_cast<V*>(zp + (int64_t)lane * VB));
    } else if constexpr (XBF) {      // bf16 in, fp32 out: twice the bytes
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            V o;
#pragma unroll
            for (int i = 0; i < NW; ++i) o[i] = __float_as_uint(z[q * NW + i]);
            __builtin_nontemporal_store(o, reinterpret_cast<V*>(zp + (int64_t)lane * 2 * VB + q * VB));
        }
    } else {
        V o;
#pragma unroll
        for (int i = 0; i < NW; ++i) o[i] = __float_as_uint(z[i]);
        __builtin_nontemporal_store(o, reinterpret_cast<V*>(zp + (int64_t)lane * VB));
    }
    acc.clear();
}

template <int VB, bool XBF, bool ZBF>
__device__ __forceinline__ void light_group(const SpmmArgs& a, int64_t g) {
    typedef typename VecOf<VB>::type V;
    constexpr int U = 8;
    const int lane = threadIdx.x & 63;
    const int r0 = a.group[2 * g], nrows = a.group[2 * g + 1] - r0;   // 1 <= nrows <= 63
    const int my_ptr = lane <= nrows ? a.ptr[r0 + lane] : 0;
    const int e0 = __builtin_amdgcn_readlane(my_ptr, 0);
    const int e1 = __builtin_amdgcn_readlane(my_ptr, nrows);
    const char* xb = a.X + (int64_t)lane * VB;
    const char* hb = a.H + (int64_t)lane * VB;
    LaneAcc<VB, XBF> acc;
    acc.clear();
    int r = 0;                                                     // row being accumulated (relative to r0)
    int row_end = __builtin_amdgcn_readlane(my_ptr, 1);            // first entry after row r
    // The diagonal term needs X[row, :] at every flush.  Its address depends on the row number alone, so the
    // pieces of the next four rows are kept in flight in a small ring instead of being loaded (and waited for)
    // at the flush itself: rows of 0-1 entries would otherwise pay a full memory latency each.
    constexpr int D = 4;
    V own[D];
    const bool use_diag = a.diag != 0.f;
    auto load_own = [&](int rr) -> V {
        V v{};
        const int64_t row = (int64_t)r0 + rr;
        if (use_diag && rr < nrows && row < a.n_diag) v = *reinterpret_cast<const V*>(xb + row * a.x_stride);
        return v;
    };
#pragma unroll
    for (int d = 0; d < D; ++d) own[d] = load_own(d);
    auto flush = [&]() {
        flush_row<VB, XBF, ZBF>(a, r0 + r, lane, acc, own[0]);
#pragma unroll
        for (int d = 0; d + 1 < D; ++d) own[d] = own[d + 1];
        own[D - 1] = load_own(r + D);
        ++r;
    };
    // a single row longer than 64 entries makes its own group: walk it 64 entries at a time
    for (int t = e0; t < e1; t += kWave) {
        const int cnt = min(kWave, e1 - t);
        int my_c = 0;
        float my_w = 0.f;
        if (lane < cnt) {
            my_c = __builtin_nontemporal_load(a.ind + t + lane);
            my_w = a.val ? __builtin_nontemporal_load(a.val + t + lane) : 1.f;
        }
        for (int j = 0; j < cnt; j += U) {
            V v[U];
            float w[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int k = j + u;
                const int c = __builtin_amdgcn_readlane(my_c, k & 63);
                w[u] = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(my_w), k & 63));
                const bool in_batch = c >= 0;
                const char* src = (in_batch ? xb : hb) +
                                  (int64_t)(in_batch ? c : -1 - c) * (in_batch ? a.x_stride : a.h_stride);
                if (k < cnt) v[u] = *reinterpret_cast<const V*>(src);
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int k = j + u;
                if (k < cnt) {
                    while (t + k >= row_end) {                     // crossed into the next row (or over empty rows)
                        flush();
                        row_end = __builtin_amdgcn_readlane(my_ptr, (r + 1) & 63);
                    }
                    acc.fma(w[u], v[u]);
                }
            }
        }
    }
    while (r < nrows) flush();                                     // last row and trailing empty rows
}

// One chunk of a heavy row on the wave-per-row layout (rows of 64 vectors of VB bytes): every lane owns VB bytes
// of the row, 8 gathers in flight per lane, the fp32 partial sum goes to the chunk's slot of the workspace.
template <int VB, bool XBF, int U>
__device__ __forceinline__ void chunk_wave_per_row(const SpmmArgs& a, int64_t c) {
    typedef typename VecOf<VB>::type V;
    constexpr int E = LaneAcc<VB, XBF>::E;
    const int lane = threadIdx.x & 63;
    const int begin = a.chunk[3 * c + 1], end = a.chunk[3 * c + 2];
    const char* xb = a.X + (int64_t)lane * VB;
    const char* hb = a.H + (int64_t)lane * VB;
    LaneAcc<VB, XBF> acc;
    acc.clear();
    for (int t = begin; t < end; t += kWave) {
        const int cnt = min(kWave, end - t);
        int my_c = 0;
        float my_w = 0.f;
        if (lane < cnt) {
            my_c = __builtin_nontemporal_load(a.ind + t + lane);
            my_w = a.val ? __builtin_nontemporal_load(a.val + t + lane) : 1.f;
        }
        for (int j = 0; j < cnt; j += U) {
            V v[U];
            float w[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int k = j + u;
                const int ci = __builtin_amdgcn_readlane(my_c, k & 63);
                w[u] = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(my_w), k & 63));
                const bool in_batch = ci >= 0;
                const char* src = (in_batch ? xb : hb) +
                                  (int64_t)(in_batch ? ci : -1 - ci) * (in_batch ? a.x_stride : a.h_stride);
                if (k < cnt) v[u] = *reinterpret_cast<const V*>(src);
            }
#pragma unroll
            for (int u = 0; u < U; ++u)
                if (j + u < cnt) acc.fma(w[u], v[u]);
        }
    }
    float* dst = a.partial + (int64_t)a.chunk[3 * c] * a.F + (int64_t)lane * E;
    if constexpr (E == 8) {
        *reinterpret_cast<f32x4*>(dst) = f32x4{acc.v[0], acc.v[1], acc.v[2], acc.v[3]};
        *reinterpret_cast<f32x4*>(dst + 4) = f32x4{acc.v[4], acc.v[5], acc.v[6], acc.v[7]};
    } else if constexpr (E == 4) {
        *reinterpret_cast<f32x4*>(dst) = f32x4{acc.v[0], acc.v[1], acc.v[2], acc.v[3]};
    } else if constexpr (E == 2) {
        *reinterpret_cast<u32x2*>(dst) = u32x2{__float_as_uint(acc.v[0]), __float_as_uint(acc.v[1])};
    } else {
        *dst = acc.v[0];
    }
}

// Chunks of heavy rows: one wavefront per chunk, partial sums to the workspace.
// Workgroups take the window-ordered list four chunks at a time.  At most
// four wavefronts per SIMD: fewer chunks in flight keep the gathers of the
// running chunks inside a narrower range of rows (measured: 2-4 % faster than
// 5 or 8, 3 and fewer are slower).
template <int G, int UPT, int U, bool XBF, int VB>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(4, 4))) void spmm_chunk_kernel(SpmmArgs a) {
    constexpr int E = Unit<XBF>::E;
    const int lane = threadIdx.x & 63;
    const int64_t c = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (c >= a.n_chunks) return;
    if constexpr (VB > 0) {                 // rows of 64 vectors
        chunk_wave_per_row<VB, XBF, U>(a, c);
        return;
    }
    float acc[UPT][E];
    accumulate<G, UPT, U, XBF>(a, a.chunk[3 * c + 1], a.chunk[3 * c + 2], acc);
    if (lane < G) {
#pragma unroll
        for (int p = 0; p < UPT; ++p) {
            const int unit = lane + p * G;
            if (unit < a.units) {
                float* dst = a.partial + (int64_t)a.chunk[3 * c] * a.F + (int64_t)unit * E;
#pragma unroll
                for (int q = 0; q < E / 4; ++q)
                    *reinterpret_cast<f32x4*>(dst + 4 * q) =
                        f32x4{acc[p][4 * q], acc[p][4 * q + 1], acc[p][4 * q + 2], acc[p][4 * q + 3]};
            }
        }
    }
}

// Light rows, finished in one go (epilogue and store).  VB > 0: bundled into
// groups, one wavefront per row (rows of exactly 64 vectors of VB bytes);
// VB == 0: one wavefront per row, teams of G lanes per neighbour.
template <int G, int UPT, int U, bool XBF, bool ZBF, int VB>
__global__ __launch_bounds__(256) void spmm_rows_kernel(SpmmArgs a) {
    if constexpr (VB > 0) {
        // Workgroups go to the eight XCDs in turn and each XCD has its own L2: with xcd_ranges every XCD takes one
        // contiguous range of the groups (equal cost per range), so rows of one cluster of the partition gather
        // into one L2, not eight.  The plan turns this on where the pattern is clustered.
        int64_t g = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6), g_end = a.n_groups;
        if (a.xcd_ranges) {
            const int x = blockIdx.x & 7;
            g = a.xcd_start[x] + (int64_t)(blockIdx.x >> 3) * 4 + (threadIdx.x >> 6);
            g_end = a.xcd_start[x + 1];
        }
        if (g < g_end) light_group<VB, XBF, ZBF>(a, g);
    } else {
        constexpr int E = Unit<XBF>::E;
        const int lane = threadIdx.x & 63;
        const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
        if (row >= a.n_rows) return;
        const int begin = a.ptr[row], end = a.ptr[row + 1];
        if (end - begin > a.threshold) return;       // heavy row: done by the chunk kernel
        float acc[UPT][E];
        accumulate<G, UPT, U, XBF>(a, begin, end, acc);
        if (lane < G) {
#pragma unroll
            for (int p = 0; p < UPT; ++p)
                if (lane + p * G < a.units) epilogue<XBF, ZBF>(a, row, lane + p * G, acc[p]);
        }
    }
}

// One wavefront per heavy row: add the chunk partials in chunk order.
template <bool XBF, bool ZBF>
__global__ __launch_bounds__(256) void spmm_heavy_reduce_kernel(SpmmArgs a) {
    const int64_t h = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (h >= a.n_heavy) return;
    constexpr int E = Unit<XBF>::E;
    const int64_t row = a.heavy[h];
    const int first = a.heavy[a.n_heavy + h], last = a.heavy[a.n_heavy + h + 1];
    for (int unit = threadIdx.x & 63; unit < a.units; unit += kWave) {
        float acc[E];
#pragma unroll
        for (int e = 0; e < E; ++e) acc[e] = 0.f;
        for (int c = first; c < last; ++c) {
            const float* src = a.partial + (int64_t)c * a.F + (int64_t)unit * E;
#pragma unroll
            for (int q = 0; q < E / 4; ++q) {
                const f32x4 v = *reinterpret_cast<const f32x4*>(src + 4 * q);
#pragma unroll
                for (int i = 0; i < 4; ++i) acc[4 * q + i] += v[i];
            }
        }
        epilogue<XBF, ZBF>(a, row, unit, acc);
    }
}

// Element-wise path for rows that are not 16-byte aligned or not a whole
// number of 16-byte units: one wavefront per row, one lane per feature.
template <bool XBF, bool ZBF>
__global__ __launch_bounds__(256) void spmm_generic_kernel(SpmmArgs a) {
    const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= a.n_rows) return;
    const int begin = a.ptr[row], end = a.ptr[row + 1];
    auto ld = [](const char* base, int64_t stride, int64_t r, int f) -> float {
        if constexpr (XBF) return __uint_as_float((uint32_t) * reinterpret_cast<const uint16_t*>(base + r * stride + 2 * f) << 16);
        else return *reinterpret_cast<const float*>(base + r * stride + 4 * (int64_t)f);
    };
    for (int f = threadIdx.x & 63; f < a.F; f += kWave) {
        float acc = 0.f;
        for (int k = begin; k < end; ++k) {
            const int c = a.ind[k];
            const float x = c >= 0 ? ld(a.X, a.x_stride, c, f) : ld(a.H, a.h_stride, -1 - c, f);
            acc = fmaf(a.val ? a.val[k] : 1.f, x, acc);
        }
        float z = a.s_agg * acc;
        if (a.diag != 0.f && row < a.n_diag) z += a.diag * ld(a.X, a.x_stride, row, f);
        if (a.R) z += a.s_res * ld(a.R, a.r_stride, row, f);
        if constexpr (ZBF) *reinterpret_cast<uint16_t*>(a.Z + row * a.z_stride + 2 * f) = (uint16_t)f32_to_bf16(z);
        else *reinterpret_cast<float*>(a.Z + row * a.z_stride + 4 * (int64_t)f) = z;
    }
}

template <int G, int UPT, int U, bool XBF, int VB = 0>
gas_status launch_chunks(const SpmmArgs& a, hipStream_t s) {
    const int64_t blocks = (a.n_chunks + 3) / 4;
    if (blocks > 0x7FFFFFFFLL) return fail(GAS_ERR_ARG, "gas_spmm: too many workgroups for one launch");
    hipLaunchKernelGGL((spmm_chunk_kernel<G, UPT, U, XBF, VB>), dim3((unsigned)blocks), dim3(256), 0, s, a);
    return GAS_OK;
}

template <bool XBF>
gas_status dispatch_chunks(const SpmmArgs& a, hipStream_t s) {
    const int u = a.units;
    if (u == 64) return launch_chunks<64, 1, 8, XBF, 16>(a, s);
    if (u == 32) return launch_chunks<32, 1, 8, XBF, 8>(a, s);
    if (u == 16) return launch_chunks<16, 1, 8, XBF, 4>(a, s);
    if (u <= 8) return launch_chunks<8, 1, 8, XBF>(a, s);
    if (u <= 16) return launch_chunks<16, 1, 8, XBF>(a, s);
    if (u <= 32) return launch_chunks<32, 1, 8, XBF>(a, s);
    if (u <= 64) return launch_chunks<64, 1, 8, XBF>(a, s);
    if (u <= 128) return launch_chunks<64, 2, 4, XBF>(a, s);
    return launch_chunks<64, 4, 2, XBF>(a, s);
}

template <int G, int UPT, int U, bool XBF, bool ZBF, int VB = 0>
gas_status launch_rows(const SpmmArgs& a, hipStream_t s) {
    const int64_t items = VB > 0 ? a.n_groups : a.n_rows;
    int64_t blocks = (items + 3) / 4;
    if (VB > 0 && a.xcd_ranges) {
        int64_t longest = 0;
        for (int x = 0; x < 8; ++x) longest = std::max(longest, a.xcd_start[x + 1] - a.xcd_start[x]);
        blocks = 8 * ((longest + 3) / 4);
    }
    if (blocks > 0x7FFFFFFFLL) return fail(GAS_ERR_ARG, "gas_spmm: too many workgroups for one launch");
    if (blocks > 0)
        hipLaunchKernelGGL((spmm_rows_kernel<G, UPT, U, XBF, ZBF, VB>), dim3((unsigned)blocks), dim3(256), 0, s, a);
    return GAS_OK;
}

template <bool XBF, bool ZBF>
gas_status dispatch_units(const SpmmArgs& a, hipStream_t s) {
    const int u = a.units;
    if (u > 256) return fail(GAS_ERR_ARG, "feature rows longer than 4096 bytes are not supported (F*size = %d)", u * 16);
    // heavy rows first: chunk partials, then their reduction; the light rows follow on the same stream
    if (a.n_chunks > 0) {
        const gas_status st = dispatch_chunks<XBF>(a, s);
        if (st != GAS_OK) return st;
        hipLaunchKernelGGL((spmm_heavy_reduce_kernel<XBF, ZBF>), dim3((unsigned)((a.n_heavy + 3) / 4)), dim3(256),
                           0, s, a);
    }
    gas_status st;
    // rows of exactly 1 KiB, 512 B or 256 B: grouped wave-per-row path
    if (a.group && u == 64) st = launch_rows<64, 1, 8, XBF, ZBF, 16>(a, s);
    else if (a.group && u == 32) st = launch_rows<32, 1, 4, XBF, ZBF, 8>(a, s);
    else if (a.group && u == 16) st = launch_rows<16, 1, 4, XBF, ZBF, 4>(a, s);
    else if (u <= 8) st = launch_rows<8, 1, 2, XBF, ZBF>(a, s);
    else if (u <= 16) st = launch_rows<16, 1, 4, XBF, ZBF>(a, s);
    else if (u <= 32) st = launch_rows<32, 1, 4, XBF, ZBF>(a, s);
    else if (u <= 64) st = launch_rows<64, 1, 8, XBF, ZBF>(a, s);
    else if (u <= 128) st = launch_rows<64, 2, 4, XBF, ZBF>(a, s);
    else st = launch_rows<64, 4, 2, XBF, ZBF>(a, s);
    if (st != GAS_OK) return st;
    GAS_CHECK_HIP(hipGetLastError());
    return GAS_OK;
}

gas_status run_spmm(const char* who, const gas_plan* plan, const int32_t* ptr, const int32_t* ind, const float* val,
                    float diag, int64_t n_diag, const void* X, int64_t ldx, const void* H, int64_t ldh,
                    gas_dtype dt_x, int32_t F, float s_agg,
                    const void* R, int64_t ldr, float s_res, void* Z, int64_t ldz, gas_dtype dt_z, hipStream_t s) {
    if (!valid_dtype(dt_x) || !valid_dtype(dt_z)) return fail(GAS_ERR_DTYPE, "%s: unknown dtype", who);
    if (dt_x == GAS_F32 && dt_z == GAS_BF16)
        return fail(GAS_ERR_DTYPE, "%s: fp32 input with bf16 output is not supported", who);
    GAS_REQUIRE(plan, "%s: null plan", who);
    if (plan->n_rows == 0) return GAS_OK;
    GAS_REQUIRE(ptr && X && Z, "%s: null pointer", who);
    GAS_REQUIRE(plan->nnz == 0 || ind, "%s: null index array", who);
    GAS_REQUIRE(F > 0 && F <= plan->max_F, "%s: F=%d outside (0, plan max_F=%d]", who, F, plan->max_F);
    GAS_REQUIRE(ldx >= F && ldz >= F && (!R || ldr >= F) && (!H || ldh >= F), "%s: row stride smaller than F", who);
    GAS_REQUIRE(Z != X && Z != R, "%s: output aliases an input", who);
    const int xb = elem_bytes(dt_x), zb = elem_bytes(dt_z);
    // Rows longer than 4096 bytes (a wide input layer) are aggregated panel by panel: the sum is separate for
    // every feature column, so a panel of columns is an aggregation of its own over the same pattern.
    const int64_t panel = 4096 / xb;
    if ((int64_t)F > panel) {
        for (int64_t f0 = 0; f0 < F; f0 += panel) {
            const int32_t fw = (int32_t)std::min<int64_t>(panel, F - f0);
            const gas_status st = run_spmm(who, plan, ptr, ind, val, diag, n_diag, static_cast<const char*>(X) + f0 * xb,
                                           ldx, H ? static_cast<const char*>(H) + f0 * xb : nullptr, ldh, dt_x, fw, s_agg,
                                           R ? static_cast<const char*>(R) + f0 * xb : nullptr, ldr, s_res,
                                           static_cast<char*>(Z) + f0 * zb, ldz, dt_z, s);
            if (st != GAS_OK) return st;
        }
        return GAS_OK;
    }
    SpmmArgs a;
    a.ptr = ptr; a.ind = ind; a.val = val;
    a.X = static_cast<const char*>(X); a.x_stride = ldx * xb;
    a.H = static_cast<const char*>(H); a.h_stride = ldh * xb;
    a.R = static_cast<const char*>(R); a.r_stride = ldr * xb;
    a.Z = static_cast<char*>(Z); a.z_stride = ldz * zb;
    a.diag = diag; a.s_agg = s_agg; a.s_res = s_res;
    a.n_rows = plan->n_rows; a.n_diag = n_diag;
    a.units = (F * xb) / 16; a.F = F;
    a.threshold = plan->threshold;
    a.chunk = plan->d_chunk; a.n_chunks = plan->n_chunks;
    a.heavy = plan->d_heavy; a.n_heavy = plan->n_heavy;
    a.partial = plan->d_partial;
    a.group = plan->d_group; a.n_groups = plan->n_groups;
    a.xcd_ranges = plan->xcd_ranges;
    for (int x = 0; x < 9; ++x) a.xcd_start[x] = plan->xcd_start[x];
    const bool vec = (F * xb) % 16 == 0 && aligned16(X) && a.x_stride % 16 == 0 && aligned16(Z) &&
                     a.z_stride % 16 == 0 && (!R || (aligned16(R) && a.r_stride % 16 == 0)) &&
                     (!H || (aligned16(H) && a.h_stride % 16 == 0));
    const bool xbf = dt_x == GAS_BF16, zbf = dt_z == GAS_BF16;
    if (vec) {
        if (!xbf) return dispatch_units<false, false>(a, s);
        return zbf ? dispatch_units<true, true>(a, s) : dispatch_units<true, false>(a, s);
    }
    const unsigned blocks = (unsigned)((a.n_rows + 3) / 4);
    if (!xbf) hipLaunchKernelGGL((spmm_generic_kernel<false, false>), dim3(blocks), dim3(256), 0, s, a);
    else if (zbf) hipLaunchKernelGGL((spmm_generic_kernel<true, true>), dim3(blocks), dim3(256), 0, s, a);
    else hipLaunchKernelGGL((spmm_generic_kernel<true, false>), dim3(blocks), dim3(256), 0, s, a);
    GAS_CHECK_HIP(hipGetLastError());
    return GAS_OK;
}

__global__ __launch_bounds__(256) void fuse_sources_kernel(const int32_t* __restrict__ col, int64_t nnz, int64_t nb,
                                                           const int32_t* __restrict__ n_id,
                                                           int32_t* __restrict__ src) {
    const int64_t k = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (k >= nnz) return;
    const int32_t c = col[k];
    src[k] = c < nb ? c : -1 - n_id[c];
}

}  // namespace
}  // namespace gas

using namespace gas;

extern "C" {

gas_status gas_spmm(const gas_plan* plan, const int32_t* rowptr, const int32_t* col, const float* val, float diag,
                    const void* X, int64_t ldx, gas_dtype dt_x, int32_t F, float s_agg, const void* R, int64_t ldr,
                    float s_res, void* Z, int64_t ldz, gas_dtype dt_z, void* stream) {
    return run_spmm("gas_spmm", plan, rowptr, col, val, diag, plan ? plan->n_rows : 0, X, ldx, nullptr, 0, dt_x, F,
                    s_agg, R, ldr, s_res, Z, ldz, dt_z, (hipStream_t)stream);
}

gas_status gas_spmm_t(const gas_plan* plan, const int32_t* colptr, const int32_t* row, const float* val, float diag,
                      float s_agg, int64_t n_diag, const void* G, int64_t ldg, gas_dtype dt_g, int32_t F, void* GX,
                      int64_t ldgx, gas_dtype dt_gx, void* stream) {
    GAS_REQUIRE(n_diag >= 0, "gas_spmm_t: n_diag=%lld", (long long)n_diag);
    return run_spmm("gas_spmm_t", plan, colptr, row, val, diag, n_diag, G, ldg, nullptr, 0, dt_g, F, s_agg, nullptr,
                    0, 0.f, GX, ldgx, dt_gx, (hipStream_t)stream);
}

gas_status gas_spmm_hist(const gas_plan* plan, const int32_t* rowptr, const int32_t* src, const float* val,
                         float diag, const void* X, int64_t ldx, const void* hist, int64_t n_hist_rows,
                         int64_t ld_hist, gas_dtype dt_x, int32_t F, float s_agg, const void* R, int64_t ldr,
                         float s_res, void* Z, int64_t ldz, gas_dtype dt_z, void* stream) {
    GAS_REQUIRE(hist && n_hist_rows > 0, "gas_spmm_hist: null or empty history table");
    GAS_REQUIRE(Z != hist, "gas_spmm_hist: output aliases the history table");
    return run_spmm("gas_spmm_hist", plan, rowptr, src, val, diag, plan ? plan->n_rows : 0, X, ldx, hist, ld_hist,
                    dt_x, F, s_agg, R, ldr, s_res, Z, ldz, dt_z, (hipStream_t)stream);
}

gas_status gas_fuse_sources(const int32_t* col, int64_t nnz, int64_t nb, const int32_t* n_id, int32_t* src,
                            void* stream) {
    GAS_REQUIRE(nnz >= 0 && nb >= 0, "gas_fuse_sources: nnz=%lld nb=%lld", (long long)nnz, (long long)nb);
    if (nnz == 0) return GAS_OK;
    GAS_REQUIRE(col && n_id && src, "gas_fuse_sources: null pointer");
    const int64_t blocks = (nnz + 255) / 256;
    GAS_REQUIRE(blocks <= 0x7FFFFFFFLL, "gas_fuse_sources: too many entries");
    hipLaunchKernelGGL(fuse_sources_kernel, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream, col, nnz, nb,
                       n_id, src);
    GAS_CHECK_HIP(hipGetLastError());
    return GAS_OK;
}

}  // extern "C"
