// Dense transform of the GNN operators on the matrix cores (gas_linear,
// gas_mlp2):  Y = act(c_identity * Z + c_weight * (Z W) + bias).
//
// This is the only dense contraction of the step (the W of the paper's GCN,
// GCNII and GIN operator equations), so it is the only place MFMA is used.
// fp32 data uses v_mfma_f32_32x32x2_f32, bf16 data v_mfma_f32_32x32x16_bf16
// with fp32 accumulation.
//
// Tiling (fp32): a workgroup of 4 wavefronts owns a BM x BN tile of Y, each
// wavefront a (BM/2) x (BN/2) sub-tile made of 32x32 MFMA blocks.  K is walked
// in steps of 32: the next A (rows of Z) and B (rows of W) tiles are fetched
// from global memory into registers while the current ones are consumed from
// LDS.  A is stored [m][k] so that one 128-bit LDS read gives a lane the four
// k values of four consecutive MFMAs; lanes 0-31 and 32-63 of an MFMA take
// different k, and A and B agree on which.
#include "common.h"

namespace gas {
namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));

struct LinArgs {
    const char* Z;   int64_t ldz;      // elements
    const char* W;
    const char* bias;
    char* Y;         int64_t ldy;
    int64_t M;
    int K, N;
    float c_id, c_w;
    int relu;
};

constexpr int kBK = 32;
constexpr int kPadA = 4, kPadB = 4;

// ------------------------------------------------------------------ fp32
template <int BM, int BN, bool VEC>
__global__ __launch_bounds__(256) void linear_f32_kernel(LinArgs a) {
    constexpr int TM = BM / 64, TN = BN / 64;          // 32x32 blocks per wavefront
    constexpr int A_V4 = BM * kBK / 4 / 256;           // float4 per thread per tile
    constexpr int B_V4 = kBK * BN / 4 / 256;
    __shared__ __attribute__((aligned(16))) float As[BM][kBK + kPadA];
    __shared__ __attribute__((aligned(16))) float Bs[kBK][BN + kPadB];

    const float* Z = reinterpret_cast<const float*>(a.Z);
    const float* W = reinterpret_cast<const float*>(a.W);
    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63;
    const int li = lane & 31, lh = lane >> 5;
    const int64_t m0 = (int64_t)blockIdx.x * BM;
    const int n0 = blockIdx.y * BN;
    const int wm0 = (wave >> 1) * (BM / 2), wn0 = (wave & 1) * (BN / 2);

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    f32x4 ra[A_V4], rb[B_V4];
    auto fetch = [&](int k0) {
#pragma unroll
        for (int i = 0; i < A_V4; ++i) {
            const int idx = tid + 256 * i;
            const int row = idx / (kBK / 4), c4 = idx % (kBK / 4);
            const int64_t m = m0 + row;
            const int k = k0 + 4 * c4;
            f32x4 v = {0.f, 0.f, 0.f, 0.f};
            if (m < a.M) {
                if constexpr (VEC) {
                    if (k < a.K) v = *reinterpret_cast<const f32x4*>(Z + m * a.ldz + k);
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (k + e < a.K) v[e] = Z[m * a.ldz + k + e];
                }
            }
            ra[i] = v;
        }
#pragma unroll
        for (int i = 0; i < B_V4; ++i) {
            const int idx = tid + 256 * i;
            const int kr = idx / (BN / 4), c4 = idx % (BN / 4);
            const int k = k0 + kr, n = n0 + 4 * c4;
            f32x4 v = {0.f, 0.f, 0.f, 0.f};
            if (k < a.K) {
                if constexpr (VEC) {
                    if (n < a.N) v = *reinterpret_cast<const f32x4*>(W + (int64_t)k * a.N + n);
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (n + e < a.N) v[e] = W[(int64_t)k * a.N + n + e];
                }
            }
            rb[i] = v;
        }
    };
    auto stage = [&]() {
#pragma unroll
        for (int i = 0; i < A_V4; ++i) {
            const int idx = tid + 256 * i;
            *reinterpret_cast<f32x4*>(&As[idx / (kBK / 4)][4 * (idx % (kBK / 4))]) = ra[i];
        }
#pragma unroll
        for (int i = 0; i < B_V4; ++i) {
            const int idx = tid + 256 * i;
            *reinterpret_cast<f32x4*>(&Bs[idx / (BN / 4)][4 * (idx % (BN / 4))]) = rb[i];
        }
    };

    fetch(0);
    for (int k0 = 0; k0 < a.K; k0 += kBK) {
        __syncthreads();                 // everyone is done reading the previous tile
        stage();
        __syncthreads();
        if (k0 + kBK < a.K) fetch(k0 + kBK);
#pragma unroll
        for (int kq = 0; kq < kBK / 8; ++kq) {
            f32x4 fa[TM];
#pragma unroll
            for (int i = 0; i < TM; ++i)
                fa[i] = *reinterpret_cast<const f32x4*>(&As[wm0 + 32 * i + li][kq * 8 + lh * 4]);
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                float fb[TN];
#pragma unroll
                for (int j = 0; j < TN; ++j) fb[j] = Bs[kq * 8 + lh * 4 + q][wn0 + 32 * j + li];
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[i][q], fb[j], acc[i][j], 0, 0, 0);
            }
        }
    }

    // accumulator layout of a 32x32 block: register r of lane (li, lh) holds
    // row 8*(r/4) + 4*lh + r%4, column li
    float* Y = reinterpret_cast<float*>(a.Y);
    const float* bias = reinterpret_cast<const float*>(a.bias);
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int n = n0 + wn0 + 32 * j + li;
            if (n >= a.N) continue;
            const float bv = bias ? bias[n] : 0.f;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int64_t m = m0 + wm0 + 32 * i + 8 * (r / 4) + 4 * lh + (r % 4);
                if (m >= a.M) continue;
                float y = a.c_w * acc[i][j][r] + bv;
                if (a.c_id != 0.f) y += a.c_id * Z[m * a.ldz + n];
                if (a.relu) y = fmaxf(y, 0.f);
                Y[m * a.ldy + n] = y;
            }
        }
}

template <int BM, int BN>
gas_status launch_f32(const LinArgs& a, bool vec, hipStream_t s) {
    const int64_t gm = (a.M + BM - 1) / BM;
    const int gn = (a.N + BN - 1) / BN;
    if (gm > 0x7FFFFFFF || gn > 65535) return fail(GAS_ERR_ARG, "gas_linear: problem too large for one launch");
    dim3 grid((unsigned)gm, (unsigned)gn), block(256);
    if (vec) hipLaunchKernelGGL((linear_f32_kernel<BM, BN, true>), grid, block, 0, s, a);
    else hipLaunchKernelGGL((linear_f32_kernel<BM, BN, false>), grid, block, 0, s, a);
    GAS_CHECK_HIP(hipGetLastError());
    return GAS_OK;
}

}  // namespace
}  // namespace gas

using namespace gas;

extern "C" {

gas_status gas_linear(const void* Z, int64_t ldz, int64_t n_rows, int32_t F_in, const void* W, int32_t F_out,
                      const void* bias, gas_dtype dt, float c_identity, float c_weight, int relu, void* Y,
                      int64_t ldy, void* stream) {
    if (!valid_dtype(dt)) return fail(GAS_ERR_DTYPE, "gas_linear: unknown dtype %d", (int)dt);
    GAS_REQUIRE(n_rows >= 0 && F_in > 0 && F_out > 0, "gas_linear: n_rows=%lld F_in=%d F_out=%d", (long long)n_rows,
                F_in, F_out);
    if (n_rows == 0) return GAS_OK;
    GAS_REQUIRE(Z && W && Y, "gas_linear: null pointer");
    GAS_REQUIRE(ldz >= F_in && ldy >= F_out, "gas_linear: row stride smaller than the row");
    GAS_REQUIRE(c_identity == 0.f || F_in == F_out, "gas_linear: the identity term needs F_in == F_out");
    GAS_REQUIRE(Y != Z, "gas_linear: Y must not alias Z");
    LinArgs a;
    a.Z = static_cast<const char*>(Z); a.ldz = ldz;
    a.W = static_cast<const char*>(W);
    a.bias = static_cast<const char*>(bias);
    a.Y = static_cast<char*>(Y); a.ldy = ldy;
    a.M = n_rows; a.K = F_in; a.N = F_out;
    a.c_id = c_identity; a.c_w = c_weight; a.relu = relu;
    hipStream_t s = (hipStream_t)stream;
    if (dt == GAS_F32) {
        const bool vec = aligned16(Z) && aligned16(W) && ldz % 4 == 0 && F_in % 4 == 0 && F_out % 4 == 0;
        if (F_out <= 64) return launch_f32<128, 64>(a, vec, s);
        return launch_f32<128, 128>(a, vec, s);
    }
    return fail(GAS_ERR_DTYPE, "gas_linear: bf16 is not implemented yet");
}

gas_status gas_mlp2(const void* Z, int64_t ldz, int64_t n_rows, int32_t F_in, const void* W1, int32_t F_hid,
                    const void* b1, const void* W2, int32_t F_out, const void* b2, gas_dtype dt, int relu_out,
                    void* Y, int64_t ldy, void* stream) {
    (void)Z; (void)ldz; (void)n_rows; (void)F_in; (void)W1; (void)F_hid; (void)b1; (void)W2; (void)F_out; (void)b2;
    (void)dt; (void)relu_out; (void)Y; (void)ldy; (void)stream;
    return fail(GAS_ERR_DTYPE, "gas_mlp2: not implemented yet");
}

}  // extern "C"
