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

// Rows of at most 64 pieces of 16 bytes: lane l owns piece l.  Entries are taken U at a time: gathers, scores
// (one lane reduction each), one rescale of the running sums to the block's maximum, then the weighted adds in
// index order.
template <bool BF>
__global__ __launch_bounds__(64) void gat_rows_kernel(GatArgs a) {
    constexpr int E = Elems<BF>::E, EB = BF ? 2 : 4, U = 8;   // U = 8: wave_sum8 reduces one block of scores
    const int64_t v = blockIdx.x;
    const int lane = threadIdx.x;
    const int b = a.rowptr[v], e = a.rowptr[v + 1];
    const bool on = lane * E < a.F;
    char* zrow = a.Z + (v * a.ldz + (int64_t)lane * E) * EB;
    if (e == b) {
        if (on) *reinterpret_cast<u32x4*>(zrow) = u32x4{0u, 0u, 0u, 0u};
        return;
    }
    float ad[E], ar[E], x[E];
    u32x4 t = {0u, 0u, 0u, 0u};
    if (on) t = *reinterpret_cast<const u32x4*>(a.a_dst + (int64_t)lane * E * EB);
    unpack<BF>(t, ad);
    t = u32x4{0u, 0u, 0u, 0u};
    if (on) t = *reinterpret_cast<const u32x4*>(a.a_src + (int64_t)lane * E * EB);
    unpack<BF>(t, ar);
    t = u32x4{0u, 0u, 0u, 0u};
    if (on) t = *reinterpret_cast<const u32x4*>(a.P + (v * a.ldp + (int64_t)lane * E) * EB);
    unpack<BF>(t, x);
    float sv = 0.f;
#pragma unroll
    for (int i = 0; i < E; ++i) sv += ad[i] * x[i];
    sv = wave_sum(sv);
    float m = -INFINITY, l = 0.f, acc[E];
#pragma unroll
    for (int i = 0; i < E; ++i) acc[i] = 0.f;
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
                    r[j] = *reinterpret_cast<const u32x4*>(a.P + ((int64_t)c * a.ldp + (int64_t)lane * E) * EB);
            }
            float sc[U], mb = m;
#pragma unroll
            for (int j = 0; j < U; ++j) {
                unpack<BF>(r[j], x);
                sc[j] = 0.f;
#pragma unroll
                for (int i = 0; i < E; ++i) sc[j] += ar[i] * x[i];
            }
            wave_sum8(sc);
#pragma unroll
            for (int j = 0; j < U; ++j) {
                float s = sc[j] + sv;
                s = s > 0.f ? s : a.slope * s;
                sc[j] = j0 + j < cnt ? s : -INFINITY;
                mb = fmaxf(mb, sc[j]);
            }
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
    if (!on) return;
    const float inv = 1.f / l;
#pragma unroll
    for (int i = 0; i < E; ++i) {
        acc[i] *= inv;
        if (a.relu) acc[i] = fmaxf(acc[i], 0.f);
    }
    u32x4 o;
    if constexpr (BF) o = u32x4{pack_bf16(acc[0], acc[1]), pack_bf16(acc[2], acc[3]), pack_bf16(acc[4], acc[5]), pack_bf16(acc[6], acc[7])};
    else o = u32x4{__float_as_uint(acc[0]), __float_as_uint(acc[1]), __float_as_uint(acc[2]), __float_as_uint(acc[3])};
    __builtin_nontemporal_store(o, reinterpret_cast<u32x4*>(zrow));
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
        if (dt == GAS_BF16) hipLaunchKernelGGL(gat_rows_kernel<true>, dim3((unsigned)n_rows), dim3(64), 0, s, a);
        else hipLaunchKernelGGL(gat_rows_kernel<false>, dim3((unsigned)n_rows), dim3(64), 0, s, a);
        GAS_CHECK_HIP(hipGetLastError());
        return GAS_OK;
    }
    return dt == GAS_BF16 ? launch_generic<true>(a, s) : launch_generic<false>(a, s);
}
