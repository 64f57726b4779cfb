// GAT's anisotropic aggregation (paper, operator appendix), one head: attention scores, their softmax over the
// entries of a row and the weighted sum of the gathered rows in ONE pass (running maximum and running sum,
// rescaled block by block), so every neighbour row is gathered once.  The score of an entry needs the whole
// gathered row, which a wavefront holds across its lanes: the dot product with the attention vector is a
// reduction over the lanes.  HBM-bound like the other aggregations.
#include "wave.h"

namespace gas {
namespace {

struct GatArgs {
    const int32_t* rowptr; const int32_t* col;
    int64_t n_rows;
    const char* P; int64_t ldp;
    const char* a_dst; const char* a_src;
    char* Z; int64_t ldz;
    int F;
    float slope;
    int relu;                                     // ReLU on the output row
};

// Rows of at most 64 pieces of 16 bytes, G = 16, 32 or 64 lanes per row (at least the number of pieces).  A
// wavefront's S = 64 / G teams of G lanes each hold the whole row and take the entries in turn (team t the entries
// t, t + S, ... of every block of 64), eight at a time per team: gathers, scores (one reduction over the team's
// lanes for all eight), one rescale of the running sums to the new maximum, then the weighted adds.  Every team
// keeps its own running maximum and sums, and the teams' states are merged pair by pair at the end.  A row of
// more than kLongRow entries is shared by the kLongWaves wavefronts of a workgroup in the same way, block of 64
// entries by block, and their states are merged in wavefront order.  Which lane takes which entry depends on the
// row's length and the width alone, so the result is the same bits on every run.

// running softmax state of one lane: maximum m, sum of weights l, weighted sum acc of its piece
template <int E>
__device__ __forceinline__ void merge_state(float& m, float& l, float (&acc)[E], float mo, float lo, const float (&acco)[E]) {
    const float mm = fmaxf(m, mo);
    // a state that has seen no entry has m = -inf and zero sums
    const float s1 = m > -INFINITY ? expf(m - mm) : 0.f, s2 = mo > -INFINITY ? expf(mo - mm) : 0.f;
    l = l * s1 + lo * s2;
#pragma unroll
    for (int i = 0; i < E; ++i) acc[i] = acc[i] * s1 + acco[i] * s2;
    m = mm;
}

// The entries of the blocks first, first + stride, ... of row v = [b, e), b < e: afterwards every team of the
// wavefront holds the merged state of all of them.
template <bool BF, int G>
__device__ __forceinline__ void gat_gather(const GatArgs& a, int64_t v, int b, int e, int first, int stride,
                                           float& m, float& l, float (&acc)[Elems<BF>::E]) {
    constexpr int E = Elems<BF>::E, EB = BF ? 2 : 4, U = 8, S = 64 / G;
    const int lane = threadIdx.x & 63, team = lane / G, tl = lane % G;
    const bool on = tl * E < a.F;
    float ad[E], ar[E], x[E];
    u32x4 t = {0u, 0u, 0u, 0u};
    if (on) t = *reinterpret_cast<const u32x4*>(a.a_dst + (int64_t)tl * E * EB);
    unpack<BF>(t, ad);
    t = u32x4{0u, 0u, 0u, 0u};
    if (on) t = *reinterpret_cast<const u32x4*>(a.a_src + (int64_t)tl * E * EB);
    unpack<BF>(t, ar);
    t = u32x4{0u, 0u, 0u, 0u};
    if (on) t = *reinterpret_cast<const u32x4*>(a.P + (v * a.ldp + (int64_t)tl * E) * EB);
    unpack<BF>(t, x);
    float sv = 0.f;
#pragma unroll
    for (int i = 0; i < E; ++i) sv += ad[i] * x[i];
    sv = team_sum<G>(sv);
    m = -INFINITY;
    l = 0.f;
#pragma unroll
    for (int i = 0; i < E; ++i) acc[i] = 0.f;
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
                    r[j] = *reinterpret_cast<const u32x4*>(a.P + ((int64_t)c * a.ldp + (int64_t)tl * E) * EB);
            }
            float sc[U], mb = m;
#pragma unroll
            for (int j = 0; j < U; ++j) {
                unpack<BF>(r[j], x);
                sc[j] = 0.f;
#pragma unroll
                for (int i = 0; i < E; ++i) sc[j] += ar[i] * x[i];
            }
            team_sum8<G>(sc);
#pragma unroll
            for (int j = 0; j < U; ++j) {
                float s = sc[j] + sv;
                s = s > 0.f ? s : a.slope * s;
                sc[j] = j0 + j * S + team < cnt ? s : -INFINITY;
                mb = fmaxf(mb, sc[j]);
            }
            if (mb > -INFINITY) {                         // a team may have had no entry of its own yet
                const float scale = expf(m - mb);         // m = -inf at the start: scale 0 on sums that are 0
                l *= scale;
#pragma unroll
                for (int i = 0; i < E; ++i) acc[i] *= scale;
#pragma unroll
                for (int j = 0; j < U; ++j) {
                    const float p = expf(sc[j] - mb);     // 0 for the padding entries
                    l += p;
                    unpack<BF>(r[j], x);
#pragma unroll
                    for (int i = 0; i < E; ++i) acc[i] += p * x[i];
                }
                m = mb;
            }
        }
    }
    // both partners of an exchange compute the same merged state
#pragma unroll
    for (int o = G; o < 64; o <<= 1) {
        const float mo = __shfl_xor(m, o), lo = __shfl_xor(l, o);
        float acco[E];
#pragma unroll
        for (int i = 0; i < E; ++i) acco[i] = __shfl_xor(acc[i], o);
        merge_state<E>(m, l, acc, mo, lo, acco);
    }
}

template <bool BF, int G>
__device__ __forceinline__ void gat_finish(const GatArgs& a, int64_t v, float l, float (&acc)[Elems<BF>::E]) {
    constexpr int E = Elems<BF>::E, EB = BF ? 2 : 4;
    const int lane = threadIdx.x & 63;
    if (lane >= G || lane * E >= a.F) return;         // team 0 stores
    const float inv = 1.f / l;
#pragma unroll
    for (int i = 0; i < E; ++i) {
        acc[i] *= inv;
        if (a.relu) acc[i] = fmaxf(acc[i], 0.f);
    }
    __builtin_nontemporal_store(pack<BF>(acc), reinterpret_cast<u32x4*>(a.Z + (v * a.ldz + (int64_t)lane * E) * EB));
}

// one wavefront per row; long rows are left to gat_long_rows_kernel
template <bool BF, int G>
__global__ __launch_bounds__(64) void gat_rows_kernel(GatArgs a) {
    constexpr int E = Elems<BF>::E, EB = BF ? 2 : 4;
    const int64_t v = blockIdx.x;
    const int lane = threadIdx.x;
    const int b = a.rowptr[v], e = a.rowptr[v + 1];
    if (e == b) {
        if (lane < G && lane * E < a.F)
            *reinterpret_cast<u32x4*>(a.Z + (v * a.ldz + (int64_t)lane * E) * EB) = u32x4{0u, 0u, 0u, 0u};
        return;
    }
    if (e - b > kLongRow) return;
    float m, l, acc[E];
    gat_gather<BF, G>(a, v, b, e, 0, 1, m, l, acc);
    gat_finish<BF, G>(a, v, l, acc);
}

// Workgroup w looks at the rows w, w + gridDim.x, ... (512 of them at a time), and every row of more than kLongRow
// entries among them is gathered by all its wavefronts together.
template <bool BF, int G>
__global__ __launch_bounds__(64 * kLongWaves) void gat_long_rows_kernel(GatArgs a) {
    constexpr int E = Elems<BF>::E, T = 64 * kLongWaves;
    __shared__ int queue[T];
    __shared__ int n_queued;
    __shared__ float red[kLongWaves][E + 2][64];
    const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
    for (int64_t r0 = blockIdx.x; r0 < a.n_rows; r0 += (int64_t)T * gridDim.x) {
        const int nq = queue_long_rows(a.rowptr, a.n_rows, r0, queue, &n_queued);
        for (int q = 0; q < nq; ++q) {
            const int64_t v = queue[q];
            const int b = a.rowptr[v], e = a.rowptr[v + 1];
            float m, l, acc[E];
            gat_gather<BF, G>(a, v, b, e, w, kLongWaves, m, l, acc);
            if (w > 0) {
                red[w][E][lane] = m;
                red[w][E + 1][lane] = l;
#pragma unroll
                for (int i = 0; i < E; ++i) red[w][i][lane] = acc[i];
            }
            __syncthreads();
            if (w == 0) {
                for (int o = 1; o < kLongWaves; ++o) {
                    float acco[E];
#pragma unroll
                    for (int i = 0; i < E; ++i) acco[i] = red[o][i][lane];
                    merge_state<E>(m, l, acc, red[o][E][lane], red[o][E + 1][lane], acco);
                }
                gat_finish<BF, G>(a, v, l, acc);
            }
            __syncthreads();
        }
    }
}

template <bool BF, int G>
void launch_rows(const GatArgs& a, hipStream_t s) {
    hipLaunchKernelGGL((gat_rows_kernel<BF, G>), dim3((unsigned)a.n_rows), dim3(64), 0, s, a);
    const unsigned blocks = long_row_blocks(a.n_rows);
    hipLaunchKernelGGL((gat_long_rows_kernel<BF, G>), dim3(blocks), dim3(64 * kLongWaves), 0, s, a);
}

template <bool BF>
void launch_vec(const GatArgs& a, hipStream_t s) {
    const int pieces = a.F / Elems<BF>::E;            // at most 64
    if (pieces <= 16) launch_rows<BF, 16>(a, s);
    else if (pieces <= 32) launch_rows<BF, 32>(a, s);
    else launch_rows<BF, 64>(a, s);
}

// any alignment, widths up to 64 * NE: lane l owns elements l, l + 64, ...; one entry at a time
template <bool BF, int NE>
__global__ __launch_bounds__(64) void gat_generic_kernel(GatArgs a) {
    const int64_t v = blockIdx.x;
    const int lane = threadIdx.x;
    auto ld = [&](const char* p, int64_t i) -> float {
        if constexpr (BF) return __uint_as_float((uint32_t)reinterpret_cast<const uint16_t*>(p)[i] << 16);
        else return reinterpret_cast<const float*>(p)[i];
    };
    const int b = a.rowptr[v], e = a.rowptr[v + 1];
    float ad[NE], ar[NE], acc[NE], x[NE];
    float sv = 0.f;
#pragma unroll
    for (int i = 0; i < NE; ++i) {
        const int f = lane + 64 * i;
        ad[i] = f < a.F ? ld(a.a_dst, f) : 0.f;
        ar[i] = f < a.F ? ld(a.a_src, f) : 0.f;
        acc[i] = 0.f;
        if (f < a.F && e > b) sv += ad[i] * ld(a.P, v * a.ldp + f);
    }
    sv = wave_sum(sv);
    float m = -INFINITY, l = 0.f;
    for (int k = b; k < e; ++k) {
        const int64_t c = a.col[k];
        float part = 0.f;
#pragma unroll
        for (int i = 0; i < NE; ++i) {
            const int f = lane + 64 * i;
            x[i] = f < a.F ? ld(a.P, c * a.ldp + f) : 0.f;
            part += ar[i] * x[i];
        }
        float s = wave_sum(part) + sv;
        s = s > 0.f ? s : a.slope * s;
        const float mb = fmaxf(m, s), scale = expf(m - mb), p = expf(s - mb);
        l = l * scale + p;
#pragma unroll
        for (int i = 0; i < NE; ++i) acc[i] = acc[i] * scale + p * x[i];
        m = mb;
    }
    const float inv = e > b ? 1.f / l : 0.f;
#pragma unroll
    for (int i = 0; i < NE; ++i) {
        const int f = lane + 64 * i;
        if (f < a.F) {
            const float y = a.relu ? fmaxf(acc[i] * inv, 0.f) : acc[i] * inv;
            if constexpr (BF) reinterpret_cast<uint16_t*>(a.Z)[v * a.ldz + f] = (uint16_t)f32_to_bf16(y);
            else reinterpret_cast<float*>(a.Z)[v * a.ldz + f] = y;
        }
    }
}

template <bool BF>
gas_status launch_generic(const GatArgs& a, hipStream_t s) {
    const dim3 grid((unsigned)a.n_rows), block(64);
    if (a.F <= 64) hipLaunchKernelGGL((gat_generic_kernel<BF, 1>), grid, block, 0, s, a);
    else if (a.F <= 256) hipLaunchKernelGGL((gat_generic_kernel<BF, 4>), grid, block, 0, s, a);
    else hipLaunchKernelGGL((gat_generic_kernel<BF, 16>), grid, block, 0, s, a);
    GAS_CHECK_HIP(hipGetLastError());
    return GAS_OK;
}

}  // namespace
}  // namespace gas

using namespace gas;

extern "C" gas_status gas_gat_aggregate(const int32_t* rowptr, const int32_t* col, int64_t n_rows, const void* P,
                                        int64_t ldp, gas_dtype dt, int32_t F, const void* a_dst, const void* a_src,
                                        float negative_slope, int relu, void* Z, int64_t ldz, void* stream) {
    if (!valid_dtype(dt)) return fail(GAS_ERR_DTYPE, "gas_gat_aggregate: unknown dtype %d", (int)dt);
    GAS_REQUIRE(n_rows >= 0 && F > 0, "gas_gat_aggregate: n_rows=%lld F=%d", (long long)n_rows, F);
    GAS_REQUIRE(F <= 1024, "gas_gat_aggregate: F=%d exceeds 1024", F);
    if (n_rows == 0) return GAS_OK;
    GAS_REQUIRE(rowptr && col && P && a_dst && a_src && Z, "gas_gat_aggregate: null pointer");
    GAS_REQUIRE(ldp >= F && ldz >= F, "gas_gat_aggregate: row stride smaller than the row");
    GAS_REQUIRE(Z != P, "gas_gat_aggregate: the output must not alias the input");
    GAS_REQUIRE(n_rows <= 0x7FFFFFFFLL, "gas_gat_aggregate: too many rows for one launch");
    GatArgs a;
    a.rowptr = rowptr; a.col = col; a.n_rows = n_rows;
    a.P = static_cast<const char*>(P); a.ldp = ldp;
    a.a_dst = static_cast<const char*>(a_dst); a.a_src = static_cast<const char*>(a_src);
    a.Z = static_cast<char*>(Z); a.ldz = ldz;
    a.F = F; a.slope = negative_slope; a.relu = relu;
    const int e = dt == GAS_BF16 ? 8 : 4;
    hipStream_t s = (hipStream_t)stream;
    const bool vec = F % e == 0 && F <= 64 * e && ldp % e == 0 && ldz % e == 0 && aligned16(P) && aligned16(Z) &&
                     aligned16(a_dst) && aligned16(a_src);
    if (vec) {
        if (dt == GAS_BF16) launch_vec<true>(a, s);
        else launch_vec<false>(a, s);
        GAS_CHECK_HIP(hipGetLastError());
        return GAS_OK;
    }
    return dt == GAS_BF16 ? launch_generic<true>(a, s) : launch_generic<false>(a, s);
}
