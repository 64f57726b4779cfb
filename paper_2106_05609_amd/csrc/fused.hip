// One layer of the step in ONE launch for narrow layers (fp32, widths up to 128): the aggregation of Eq. (2) with
// its two sources (fresh in-batch rows, stored halo rows), the dense transform on the aggregated tile while it is
// still in LDS, and the Push of the result.  A deep narrow model (the 64-layer GCNII of the paper's experiments,
// width 64) spends its time on launches, not on bytes: its weight matrix is 16 KB and a whole tile of aggregated
// rows is 8 KB, so both sit in LDS and the layer needs neither the Z round trip through HBM nor a second launch.
// Wide layers (256) keep their two kernels: there the weights fill the register file of the transform.
#include "common.h"

namespace gas {
namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kRows = 32;            // rows of the batch subgraph per tile = one 32-row MFMA block
constexpr int kMaxWidth = 128;

struct FusedArgs {
    const int32_t* rowptr; const int32_t* src; const float* val;
    int64_t n_rows, n_tiles;
    const float* X; int64_t ldx;
    const float* H; int64_t ldh;
    const float* R; int64_t ldr;
    const float* W; const float* bias;
    float* Y; int64_t ldy;
    float* Zout; int64_t ldzo;       // optional copy of the aggregated rows (a training pass reads them again)
    const int32_t* push_idx; float* PH; int64_t ldp;
    int K, N, Kp, Np;                // widths, and the widths padded to the MFMA's steps (8 and 32)
    int g_log2;                      // lanes per row in the aggregation = 1 << g_log2 (>= K / 8)
    float diag, s_agg, s_res, c_id, c_w;
    int relu;
};

__device__ __forceinline__ const float* source_row(const FusedArgs& a, int s) {
    const bool fresh = s >= 0;
    return (fresh ? a.X : a.H) + (int64_t)(fresh ? s : -1 - s) * (fresh ? a.ldx : a.ldh);
}

constexpr int kThreads = 256;        // four wavefronts: eight rows of the tile each

// Workgroups of four wavefronts, looping over tiles of 32 rows.  Per tile:
//   1. aggregation: wavefront w owns rows 8w .. 8w+7; a team of G lanes owns one row at a time, lane j its
//      16-byte pieces j and j + G (two loads per gathered row, each contiguous over the team).  The team reads
//      2 G source indices (and coefficients) with two loads (the next 2 G are requested before the current ones
//      are used), gathers the rows four at a time and folds them in index order; the finished row (scaled, plus
//      the diagonal and residual terms) goes to the LDS tile Zs.  With width 64 a team is 8 lanes, so a wavefront
//      works on its 8 rows at once and the whole chain (row pointers, indices, rows) is walked once per tile.
//   2. transform: wavefront w owns output columns 32w .. 32w+31 (if the layer is that wide): 32x32x2 fp32 MFMAs
//      over Zs and the weights in LDS, then c_w * acc + c_id * Z + bias, ReLU, and the row is stored to Y and to
//      its history slot.
// The weights are staged once per workgroup, after the first row's pointers have been requested.
__global__ __launch_bounds__(kThreads) void spmm_linear_f32_kernel(FusedArgs a) {
    extern __shared__ __attribute__((aligned(16))) char smem[];
    const int ldz = a.Kp + 4, ldw = a.Np + 4;
    float* Zs = reinterpret_cast<float*>(smem);                 // [kRows][ldz]
    float* Ws = Zs + kRows * ldz;                               // [Kp][ldw]
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, li = lane & 31, lh = lane >> 5;

    const int G = 1 << a.g_log2, T = 64 >> a.g_log2;            // lanes per team, teams per wavefront
    const int team = lane >> a.g_log2, j = lane & (G - 1);
    constexpr int U = 4, RW = kRows / (kThreads / 64);          // gathers in flight per lane (two loads each), rows per wavefront
    // Workgroups go to the eight XCDs in turn and each XCD has its own L2.  Every XCD gets one contiguous eighth
    // of the tiles: consecutive rows of a batch belong to one cluster of the partition and gather mostly from that
    // cluster's rows, which then stay in that XCD's L2 instead of being fetched into all eight.
    const int64_t per_xcd = (a.n_tiles + 7) / 8;
    const int xcd = blockIdx.x & 7;
    const int64_t tile_end = min(a.n_tiles, (xcd + 1) * per_xcd), tile0 = xcd * per_xcd + (blockIdx.x >> 3);
    // the first row's pointers are requested before the weights, so the two latencies overlap
    int b_first = 0, e_first = 0;
    {
        const int64_t m = tile0 * kRows + wave * RW + team;
        if (tile0 < tile_end && team < RW && m < a.n_rows) { b_first = a.rowptr[m]; e_first = a.rowptr[m + 1]; }
    }

    // weights, zero-padded to Kp x Np
    const int nq = a.Np / 4, n_pieces = a.Kp * nq;
    for (int idx = tid; idx < n_pieces; idx += kThreads) {
        const int k = idx / nq, n = 4 * (idx % nq);
        f32x4 v = {0.f, 0.f, 0.f, 0.f};
        if (k < a.K && n < a.N) v = *reinterpret_cast<const f32x4*>(a.W + (int64_t)k * a.N + n);
        *reinterpret_cast<f32x4*>(Ws + k * ldw + n) = v;
    }
    // the padding columns of Zs are cleared once (the aggregation never writes them)
    for (int idx = tid; idx < kRows * (a.Kp - a.K); idx += kThreads)
        Zs[(idx / (a.Kp - a.K)) * ldz + a.K + idx % (a.Kp - a.K)] = 0.f;

    const bool piece0 = 4 * j < a.K, piece1 = 4 * (j + G) < a.K;
    const int off0 = piece0 ? 4 * j : 0, off1 = piece1 ? 4 * (j + G) : 0;

    for (int64_t tile = tile0; tile < tile_end; tile += gridDim.x >> 3) {
        const int64_t m_tile = tile * kRows;
        // ---- 1. aggregation
        for (int r = wave * RW + team; r < (wave + 1) * RW; r += T) {
            const int64_t m = m_tile + r;
            const bool row_on = m < a.n_rows;
            const bool have = tile == tile0 && r == wave * RW + team;      // requested before the weights
            const int b = have ? b_first : (row_on ? a.rowptr[m] : 0), e = have ? e_first : (row_on ? a.rowptr[m + 1] : 0);
            f32x4 acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};
            auto fetch = [&](int k, int& s0, int& s1, float& v0, float& v1) {
                const bool on0 = k + j < e, on1 = k + G + j < e;
                s0 = on0 ? a.src[k + j] : 0;
                s1 = on1 ? a.src[k + G + j] : 0;
                v0 = (a.val && on0) ? a.val[k + j] : 1.f;
                v1 = (a.val && on1) ? a.val[k + G + j] : 1.f;
            };
            int s0, s1, k0 = b;
            float v0, v1;
            fetch(k0, s0, s1, v0, v1);
            while (k0 < e) {
                const int cnt = min(2 * G, e - k0);
                int ns0, ns1;
                float nv0, nv1;
                fetch(k0 + 2 * G, ns0, ns1, nv0, nv1);           // the next indices, before these are used
                for (int q0 = 0; q0 < cnt; q0 += U) {
                    const bool lo = q0 < G;                       // a batch of U lies in one half (G is a multiple of U)
                    const int sh = lo ? s0 : s1, qb = lo ? q0 : q0 - G;
                    const float vh = lo ? v0 : v1;
                    f32x4 x0[U], x1[U];
                    float v[U];
                    // every load is issued, from a valid address: entries past the end re-read the batch's first
                    // row with coefficient zero, lanes past the width re-read piece 0 and drop the result
#pragma unroll
                    for (int u = 0; u < U; ++u) {
                        const bool on = q0 + u < cnt;
                        const int s = __shfl(sh, on ? qb + u : qb, G);
                        v[u] = on ? __shfl(vh, qb + u, G) : 0.f;
                        const float* row = source_row(a, s);
                        x0[u] = *reinterpret_cast<const f32x4*>(row + off0);
                        x1[u] = *reinterpret_cast<const f32x4*>(row + off1);
                    }
#pragma unroll
                    for (int u = 0; u < U; ++u) {
#pragma unroll
                        for (int c = 0; c < 4; ++c) {
                            acc0[c] = fmaf(v[u], x0[u][c], acc0[c]);
                            acc1[c] = fmaf(v[u], x1[u][c], acc1[c]);
                        }
                    }
                }
                s0 = ns0; s1 = ns1; v0 = nv0; v1 = nv1; k0 += 2 * G;
            }
            auto finish = [&](const f32x4& acc, int p) {
                f32x4 z = {0.f, 0.f, 0.f, 0.f};
                if (row_on) {
#pragma unroll
                    for (int c = 0; c < 4; ++c) z[c] = a.s_agg * acc[c];
                    if (a.diag != 0.f) {
                        const f32x4 d = *reinterpret_cast<const f32x4*>(a.X + m * a.ldx + 4 * p);
#pragma unroll
                        for (int c = 0; c < 4; ++c) z[c] = fmaf(a.diag, d[c], z[c]);
                    }
                    if (a.R) {
                        const f32x4 d = *reinterpret_cast<const f32x4*>(a.R + m * a.ldr + 4 * p);
#pragma unroll
                        for (int c = 0; c < 4; ++c) z[c] = fmaf(a.s_res, d[c], z[c]);
                    }
                }
                *reinterpret_cast<f32x4*>(Zs + r * ldz + 4 * p) = z;
            };
            if (piece0) finish(acc0, j);
            if (piece1) finish(acc1, j + G);
        }
        __syncthreads();                 // Zs (and, the first time, Ws) complete
        if (a.Zout) {                    // the aggregated rows as gas_spmm would have stored them
            const int kq4 = a.K / 4;
            for (int idx = tid; idx < kRows * kq4; idx += kThreads) {
                const int row = idx / kq4, c = 4 * (idx % kq4);
                if (m_tile + row < a.n_rows)
                    *reinterpret_cast<f32x4*>(a.Zout + (m_tile + row) * a.ldzo + c) =
                        *reinterpret_cast<const f32x4*>(Zs + row * ldz + c);
            }
        }
        // ---- 2. transform of the tile
        if (32 * wave < a.Np) {
            f32x16 acc;
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[r] = 0.f;
            const int col = 32 * wave + li;
            int slot[16];                                         // history rows of this lane's 16 output rows
            if (a.push_idx) {
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int64_t m = m_tile + 8 * (r / 4) + 4 * lh + (r % 4);
                    slot[r] = m < a.n_rows ? a.push_idx[m] : 0;
                }
            }
            for (int kq = 0; kq < a.Kp / 8; kq += 2) {            // two steps of 8 k: operands read before the products
                f32x4 fa[2];
                float fb[2][4];
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    const int kk = min(kq + h, a.Kp / 8 - 1) * 8 + lh * 4;
                    fa[h] = *reinterpret_cast<const f32x4*>(Zs + li * ldz + kk);
#pragma unroll
                    for (int q = 0; q < 4; ++q) fb[h][q] = Ws[(kk + q) * ldw + col];
                }
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    if (kq + h < a.Kp / 8) {
#pragma unroll
                        for (int q = 0; q < 4; ++q)
                            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[h][q], fb[h][q], acc, 0, 0, 0);
                    }
                }
            }
            if (col < a.N) {
                const float bv = a.bias ? a.bias[col] : 0.f;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int row = 8 * (r / 4) + 4 * lh + (r % 4);
                    const int64_t m = m_tile + row;
                    if (m >= a.n_rows) continue;
                    float y = a.c_w * acc[r] + bv;
                    if (a.c_id != 0.f) y = fmaf(a.c_id, Zs[row * ldz + col], y);
                    if (a.relu) y = fmaxf(y, 0.f);
                    a.Y[m * a.ldy + col] = y;
                    if (a.push_idx) a.PH[(int64_t)slot[r] * a.ldp + col] = y;                    // Push in the epilogue
                }
            }
        }
        __syncthreads();                 // the next tile's aggregation overwrites Zs
    }
}

}  // namespace
}  // namespace gas

using namespace gas;

extern "C" {

gas_status gas_spmm_linear(const int32_t* rowptr, const int32_t* src, const float* val, int64_t n_rows, const void* X,
                           int64_t ldx, const void* hist, int64_t n_hist_rows, int64_t ld_hist, gas_dtype dt,
                           int32_t F_in, float diag, float s_agg, const void* R, int64_t ldr, float s_res,
                           const void* W, int32_t F_out, const void* bias, float c_identity, float c_weight, int relu,
                           void* Y, int64_t ldy, void* Z_out, int64_t ldz_out, const int32_t* push_idx,
                           void* push_hist, int64_t n_push_rows, int64_t ld_push, void* stream) {
    if (!valid_dtype(dt)) return fail(GAS_ERR_DTYPE, "gas_spmm_linear: unknown dtype %d", (int)dt);
    if (dt != GAS_F32) return fail(GAS_ERR_DTYPE, "gas_spmm_linear: fp32 only (use gas_spmm_hist + gas_linear_push)");
    GAS_REQUIRE(n_rows >= 0 && n_rows < 0x7FFFFFFFLL, "gas_spmm_linear: n_rows=%lld", (long long)n_rows);
    GAS_REQUIRE(F_in > 0 && F_out > 0 && F_in <= kMaxWidth && F_out <= kMaxWidth && F_in % 4 == 0 && F_out % 4 == 0,
                "gas_spmm_linear: widths %d -> %d: multiples of 4 up to %d only (use gas_spmm_hist + gas_linear_push)",
                F_in, F_out, kMaxWidth);
    if (n_rows == 0) return GAS_OK;
    GAS_REQUIRE(rowptr && src && X && W && Y, "gas_spmm_linear: null pointer");
    GAS_REQUIRE(ldx >= F_in && ldy >= F_out && (!hist || ld_hist >= F_in) && (!R || ldr >= F_in),
                "gas_spmm_linear: row stride smaller than the width");
    GAS_REQUIRE(n_hist_rows >= 0 && n_push_rows >= 0, "gas_spmm_linear: negative table size");
    GAS_REQUIRE(c_identity == 0.f || F_in == F_out, "gas_spmm_linear: the identity term needs F_in == F_out");
    GAS_REQUIRE((push_idx == nullptr) == (push_hist == nullptr), "gas_spmm_linear: push_idx and push_hist go together");
    GAS_REQUIRE(!push_hist || ld_push >= F_out, "gas_spmm_linear: row stride of the push table smaller than F_out");
    GAS_REQUIRE(!Z_out || ldz_out >= F_in, "gas_spmm_linear: row stride of Z_out smaller than F_in");
    const bool al = aligned16(X) && ldx % 4 == 0 && aligned16(W) && (!hist || (aligned16(hist) && ld_hist % 4 == 0)) &&
                    (!R || (aligned16(R) && ldr % 4 == 0)) && (!Z_out || (aligned16(Z_out) && ldz_out % 4 == 0));
    GAS_REQUIRE(al, "gas_spmm_linear: rows must be 16-byte aligned (use gas_spmm_hist + gas_linear_push)");

    FusedArgs a{};
    a.rowptr = rowptr; a.src = src; a.val = val;
    a.n_rows = n_rows; a.n_tiles = (n_rows + kRows - 1) / kRows;
    a.X = reinterpret_cast<const float*>(X); a.ldx = ldx;
    a.H = reinterpret_cast<const float*>(hist); a.ldh = ld_hist;
    a.R = reinterpret_cast<const float*>(R); a.ldr = ldr;
    a.W = reinterpret_cast<const float*>(W); a.bias = reinterpret_cast<const float*>(bias);
    a.Y = reinterpret_cast<float*>(Y); a.ldy = ldy;
    a.Zout = reinterpret_cast<float*>(Z_out); a.ldzo = ldz_out;
    a.push_idx = push_idx; a.PH = reinterpret_cast<float*>(push_hist); a.ldp = ld_push;
    a.K = F_in; a.N = F_out; a.Kp = (F_in + 7) & ~7; a.Np = (F_out + 31) & ~31;
    a.g_log2 = 3;
    while ((8 << a.g_log2) < F_in) ++a.g_log2;          // 8 or 16 lanes per row, two 16-byte pieces each
    a.diag = diag; a.s_agg = s_agg; a.s_res = s_res; a.c_id = c_identity; a.c_w = c_weight; a.relu = relu;

    const int smem = 4 * (kRows * (a.Kp + 4) + a.Kp * (a.Np + 4));      // at most 84,480 bytes
    const int64_t per_cu = smem <= 32768 ? 4 : (smem <= 65536 ? 2 : 1);          // workgroups per CU
    const int64_t per_xcd = (a.n_tiles + 7) / 8;                                   // a multiple of eight workgroups
    const unsigned blocks = (unsigned)(8 * (per_xcd < 32 * per_cu ? per_xcd : 32 * per_cu));
    static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(spmm_linear_f32_kernel),
                                                       hipFuncAttributeMaxDynamicSharedMemorySize,
                                                       4 * (kRows * (kMaxWidth + 4) + kMaxWidth * (kMaxWidth + 4)));
    GAS_CHECK_HIP(attr);
    hipLaunchKernelGGL(spmm_linear_f32_kernel, dim3(blocks), dim3(kThreads), smem, (hipStream_t)stream, a);
    GAS_CHECK_HIP(hipGetLastError());
    return GAS_OK;
}

}  // extern "C"
