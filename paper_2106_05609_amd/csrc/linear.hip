// Dense transform of the GNN operators on the matrix cores (gas_linear,
// gas_mlp2):  Y = act(c_identity * Z + c_weight * (Z W) + bias), and the fused
// two-layer MLP of the GIN operator.
//
// This is the only dense contraction of the step (the W of the paper's GCN,
// GCNII and GIN operator equations), so it is the only place MFMA is used.
// fp32 data uses v_mfma_f32_32x32x2_f32, bf16 data v_mfma_f32_32x32x16_bf16
// with fp32 accumulation.
//
// Tiling: a workgroup of 4 wavefronts (2 x 2) owns a BM x BN tile of Y, each
// wavefront a sub-tile made of 32x32 MFMA blocks.  K is walked in tiles: the
// next A (rows of Z) and B (rows of W) tiles are fetched from global memory
// into registers while the current ones are consumed from LDS.
//   fp32: A is stored [m][k] so that one 128-bit LDS read gives a lane the four
//         k values of four consecutive MFMAs; lanes 0-31 and 32-63 of an MFMA
//         take different k, and A and B agree on which.
//   bf16: both operands need eight consecutive k per lane.  Z is [m][k]
//         already; W is [k][n], so its tiles are transposed on the way into
//         LDS: a thread loads an 8(k) x 8(n) block as eight 16-byte row pieces,
//         regroups it in registers and writes eight 16-byte [n][k] pieces.
// The accumulator of a 32x32 block keeps, in register r of lane (li, lh),
// row 8*(r/4) + 4*lh + r%4 and column li.
#include <type_traits>

#include "common.h"
#include <mutex>

namespace gas {
namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

struct LinArgs {
    const char* Z;   int64_t ldz;      // elements
    const char* W;
    const char* bias;
    char* Y;         int64_t ldy;
    int64_t M;
    int K, N;
    float c_id, c_w;
    int relu;
    int trans_w;                       // W is given as [N][K] (the product is Z W^T of a [N, K] matrix)
    const char* mask; int64_t ldmask;  // optional [M, N]: outputs where mask <= 0 are set to zero
    const int32_t* push_idx = nullptr; // optional (fp32 tile kernel): row m also goes to push_hist[push_idx[m], :]
    char* push_hist = nullptr; int64_t ld_push = 0;
};

struct MlpArgs {
    const char* Z;   int64_t ldz;
    const char* W1;  const char* b1;
    const char* W2;  const char* b2;
    char* Y;         int64_t ldy;
    int64_t M;
    int K, H, N;     // F_in, F_hid (<= kHidMax), F_out
    int relu_out;
};

constexpr int kHidMax = 256;
constexpr int kMlpRowsF32 = 32, kMlpRowsBF16 = 64;     // rows per workgroup of the fused MLP kernels

template <int TM, int TN>
__device__ __forceinline__ void zero_acc(f32x16 (&acc)[TM][TN]) {
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
}

__device__ __forceinline__ float bf16_val(const uint16_t* p, int64_t i) { return __uint_as_float((uint32_t)p[i] << 16); }

// ====================================================================== fp32
constexpr int kBK = 32;                    // k per tile
constexpr int kLdA = kBK + 4;              // padded LDS row of the A tile (floats)

// Fetch / stage one BM x kBK tile of a row-major fp32 matrix with row stride ld.
template <int BM, bool VEC>
struct ATileF32 {
    static constexpr int NV = BM * kBK / 4 / 256;
    f32x4 r[NV];
    __device__ __forceinline__ void fetch(const float* Z, int64_t ld, int64_t M, int K, int64_t m0, int k0, int tid) {
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            const int idx = tid + 256 * i;
            const int64_t m = m0 + idx / (kBK / 4);
            const int k = k0 + 4 * (idx % (kBK / 4));
            f32x4 v = {0.f, 0.f, 0.f, 0.f};
            if (m < M) {
                if constexpr (VEC) {
                    if (k < K) v = *reinterpret_cast<const f32x4*>(Z + m * ld + k);
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (k + e < K) v[e] = Z[m * ld + k + e];
                }
            }
            r[i] = v;
        }
    }
    __device__ __forceinline__ void stage(float (*As)[kLdA], int tid) {
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            const int idx = tid + 256 * i;
            *reinterpret_cast<f32x4*>(&As[idx / (kBK / 4)][4 * (idx % (kBK / 4))]) = r[i];
        }
    }
};

// Fetch / stage one kBK x BN tile of a row-major fp32 [K][N] matrix.
template <int BN, bool VEC>
struct BTileF32 {
    static constexpr int NV = kBK * BN / 4 / 256;
    f32x4 r[NV];
    // trans: W is [N][K] row-major; a vector then holds 4 consecutive k of one n
    __device__ __forceinline__ void fetch(const float* W, int K, int N, int k0, int n0, int tid, bool trans = false) {
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            const int idx = tid + 256 * i;
            f32x4 v = {0.f, 0.f, 0.f, 0.f};
            if (!trans) {
                const int k = k0 + idx / (BN / 4), n = n0 + 4 * (idx % (BN / 4));
                if (k < K) {
                    if constexpr (VEC) {
                        if (n < N) v = *reinterpret_cast<const f32x4*>(W + (int64_t)k * N + n);
                    } else {
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            if (n + e < N) v[e] = W[(int64_t)k * N + n + e];
                    }
                }
            } else {
                const int n = n0 + idx / (kBK / 4), k = k0 + 4 * (idx % (kBK / 4));
                if (n < N) {
                    if constexpr (VEC) {
                        if (k < K) v = *reinterpret_cast<const f32x4*>(W + (int64_t)n * K + k);
                    } else {
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            if (k + e < K) v[e] = W[(int64_t)n * K + k + e];
                    }
                }
            }
            r[i] = v;
        }
    }
    __device__ __forceinline__ void stage(float (*Bs)[BN + 4], int tid, bool trans = false) {
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            const int idx = tid + 256 * i;
            if (!trans) {
                *reinterpret_cast<f32x4*>(&Bs[idx / (BN / 4)][4 * (idx % (BN / 4))]) = r[i];
            } else {
                const int n = idx / (kBK / 4), k = 4 * (idx % (kBK / 4));
#pragma unroll
                for (int e = 0; e < 4; ++e) Bs[k + e][n] = r[i][e];
            }
        }
    }
};

// acc += A[arow0.., acol0 .. acol0+kBK) * Bs, A an LDS array with row stride lda floats
template <int TM, int TN, int BN>
__device__ __forceinline__ void mfma_tile_f32(const float* A, int lda, int arow0, int acol0,
                                              const float (*Bs)[BN + 4], int bcol0, int li, int lh,
                                              f32x16 (&acc)[TM][TN]) {
#pragma unroll
    for (int kq = 0; kq < kBK / 8; ++kq) {
        f32x4 fa[TM];
#pragma unroll
        for (int i = 0; i < TM; ++i)
            fa[i] = *reinterpret_cast<const f32x4*>(A + (arow0 + 32 * i + li) * lda + acol0 + kq * 8 + lh * 4);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            float fb[TN];
#pragma unroll
            for (int j = 0; j < TN; ++j) fb[j] = Bs[kq * 8 + lh * 4 + q][bcol0 + 32 * j + li];
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[i][q], fb[j], acc[i][j], 0, 0, 0);
        }
    }
}

template <int BM, int BN, bool VEC, bool TRANS>
__global__ __launch_bounds__(256) void linear_f32_kernel(LinArgs a) {
    constexpr int TM = BM / 64, TN = BN / 64;
    __shared__ __attribute__((aligned(16))) float As[BM][kLdA];
    __shared__ __attribute__((aligned(16))) float Bs[kBK][BN + 4];
    const float* Z = reinterpret_cast<const float*>(a.Z);
    const float* W = reinterpret_cast<const float*>(a.W);
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, li = lane & 31, lh = lane >> 5;
    const int64_t m0 = (int64_t)blockIdx.x * BM;
    const int n0 = blockIdx.y * BN;
    const int wm0 = (wave >> 1) * (BM / 2), wn0 = (wave & 1) * (BN / 2);
    f32x16 acc[TM][TN];
    zero_acc(acc);
    ATileF32<BM, VEC> ta;
    BTileF32<BN, VEC> tb;
    constexpr bool tr = TRANS;           // compile-time: the plain path keeps its straight-line staging
    ta.fetch(Z, a.ldz, a.M, a.K, m0, 0, tid);
    tb.fetch(W, a.K, a.N, 0, n0, tid, tr);
    for (int k0 = 0; k0 < a.K; k0 += kBK) {
        __syncthreads();                 // everyone is done reading the previous tile
        ta.stage(As, tid);
        tb.stage(Bs, tid, tr);
        __syncthreads();
        if (k0 + kBK < a.K) {
            ta.fetch(Z, a.ldz, a.M, a.K, m0, k0 + kBK, tid);
            tb.fetch(W, a.K, a.N, k0 + kBK, n0, tid, tr);
        }
        mfma_tile_f32<TM, TN, BN>(&As[0][0], kLdA, wm0, 0, Bs, wn0, li, lh, acc);
    }
    // Epilogue: one output row at a time (register r of tile i), its address formed once; the optional terms
    // (identity, mask, push) are decided once per kernel, not once per element.
    float* Y = reinterpret_cast<float*>(a.Y);
    const float* bias = reinterpret_cast<const float*>(a.bias);
    const float* mask = reinterpret_cast<const float*>(a.mask);
    float* PH = reinterpret_cast<float*>(a.push_hist);
    const int nl = n0 + wn0 + li;                      // column of tile j = nl + 32 j
    float bv[TN];
#pragma unroll
    for (int j = 0; j < TN; ++j) bv[j] = (bias && nl + 32 * j < a.N) ? bias[nl + 32 * j] : 0.f;
    auto rows = [&](auto cid_tag, auto mask_tag, auto push_tag) {
        constexpr bool CID = decltype(cid_tag)::value, MASK = decltype(mask_tag)::value, PUSH = decltype(push_tag)::value;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int64_t m = m0 + wm0 + 32 * i + 8 * (r / 4) + 4 * lh + (r % 4);
                if (m >= a.M) continue;
                float* yrow = Y + m * a.ldy + nl;
                const float* zrow = CID ? Z + m * a.ldz + nl : nullptr;
                const float* krow = MASK ? mask + m * a.ldmask + nl : nullptr;
                float* hrow = PUSH ? PH + (int64_t)a.push_idx[m] * a.ld_push + nl : nullptr;
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    if (nl + 32 * j >= a.N) continue;
                    float y = a.c_w * acc[i][j][r] + bv[j];
                    if constexpr (CID) y += a.c_id * zrow[32 * j];
                    if (a.relu) y = fmaxf(y, 0.f);
                    if constexpr (MASK) { if (!(krow[32 * j] > 0.f)) y = 0.f; }
                    yrow[32 * j] = y;
                    if constexpr (PUSH) hrow[32 * j] = y;      // Push in the epilogue
                }
            }
    };
    using T = std::true_type;
    using F = std::false_type;
    const bool cid = a.c_id != 0.f;
    if (!cid && !mask && !a.push_idx) rows(F{}, F{}, F{});
    else if (!cid && !mask) rows(F{}, F{}, T{});
    else if (cid && !mask && !a.push_idx) rows(T{}, F{}, F{});
    else if (cid && !mask) rows(T{}, F{}, T{});
    else if (!cid && !a.push_idx) rows(F{}, T{}, F{});
    else if (!a.push_idx) rows(T{}, T{}, F{});
    else if (!cid) rows(F{}, T{}, T{});
    else rows(T{}, T{}, T{});
}

// fp32 fused MLP: 32 rows per workgroup; wavefront w owns hidden / output
// columns [64w, 64w+64).  Phase 1 leaves relu(Z W1 + b1) in LDS (fp32), phase 2
// multiplies it by W2 with the hidden tile as the A operand.
template <bool VEC>
__global__ __launch_bounds__(256) void mlp2_f32_kernel(MlpArgs a) {
    constexpr int BM = kMlpRowsF32, BN = 256, TN = 2;
    constexpr int kLdH = kHidMax + 4;
    extern __shared__ __attribute__((aligned(16))) char smem[];   // above the 64 KB static limit
    float (*Hs)[kLdH] = reinterpret_cast<float (*)[kLdH]>(smem);
    float (*As)[kLdA] = reinterpret_cast<float (*)[kLdA]>(smem + sizeof(float) * BM * kLdH);
    float (*Bs)[BN + 4] = reinterpret_cast<float (*)[BN + 4]>(smem + sizeof(float) * BM * (kLdH + kLdA));
    const float* Z = reinterpret_cast<const float*>(a.Z);
    const float* W1 = reinterpret_cast<const float*>(a.W1);
    const float* W2 = reinterpret_cast<const float*>(a.W2);
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, li = lane & 31, lh = lane >> 5;
    const int64_t m0 = (int64_t)blockIdx.x * BM;
    const int n0 = blockIdx.y * BN;
    const int wn0 = wave * 64;
    f32x16 acc[1][TN];
    zero_acc(acc);
    ATileF32<BM, VEC> ta;
    BTileF32<BN, VEC> tb;
    ta.fetch(Z, a.ldz, a.M, a.K, m0, 0, tid);
    tb.fetch(W1, a.K, a.H, 0, 0, tid);
    for (int k0 = 0; k0 < a.K; k0 += kBK) {
        __syncthreads();
        ta.stage(As, tid);
        tb.stage(Bs, tid);
        __syncthreads();
        if (k0 + kBK < a.K) {
            ta.fetch(Z, a.ldz, a.M, a.K, m0, k0 + kBK, tid);
            tb.fetch(W1, a.K, a.H, k0 + kBK, 0, tid);
        }
        mfma_tile_f32<1, TN, BN>(&As[0][0], kLdA, 0, 0, Bs, wn0, li, lh, acc);
    }
    const float* b1 = reinterpret_cast<const float*>(a.b1);
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int h = wn0 + 32 * j + li;
        const float bv = (b1 && h < a.H) ? b1[h] : 0.f;
#pragma unroll
        for (int r = 0; r < 16; ++r)
            Hs[8 * (r / 4) + 4 * lh + (r % 4)][h] = h < a.H ? fmaxf(acc[0][j][r] + bv, 0.f) : 0.f;
    }
    zero_acc(acc);
    tb.fetch(W2, a.H, a.N, 0, n0, tid);
    for (int k0 = 0; k0 < a.H; k0 += kBK) {
        __syncthreads();                 // Hs written / previous Bs consumed
        tb.stage(Bs, tid);
        __syncthreads();
        if (k0 + kBK < a.H) tb.fetch(W2, a.H, a.N, k0 + kBK, n0, tid);
        mfma_tile_f32<1, TN, BN>(&Hs[0][0], kLdH, 0, k0, Bs, wn0, li, lh, acc);
    }
    float* Y = reinterpret_cast<float*>(a.Y);
    const float* b2 = reinterpret_cast<const float*>(a.b2);
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int n = n0 + wn0 + 32 * j + li;
        if (n >= a.N) continue;
        const float bv = b2 ? b2[n] : 0.f;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int64_t m = m0 + 8 * (r / 4) + 4 * lh + (r % 4);
            if (m >= a.M) continue;
            float y = acc[0][j][r] + bv;
            if (a.relu_out) y = fmaxf(y, 0.f);
            Y[m * a.ldy + n] = y;
        }
    }
}

// ====================================================================== bf16
constexpr int kBKh = 64;            // k per tile
constexpr int kLdh = kBKh + 8;      // padded LDS row, in bf16 elements

__device__ __forceinline__ void transpose8x8_bf16(const u32x4 (&in)[8], u32x4 (&out)[8]) {
    // in[r] holds n = 0..7 of k-row r (two per dword); out[c] holds k = 0..7 of column c
#pragma unroll
    for (int c = 0; c < 8; ++c)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const uint32_t lo = in[2 * q][c >> 1], hi = in[2 * q + 1][c >> 1];
            out[c][q] = (c & 1) ? ((lo >> 16) | (hi & 0xFFFF0000u)) : ((lo & 0xFFFFu) | (hi << 16));
        }
}

template <int BM>
struct ATileBF16 {
    static constexpr int NV = BM * kBKh / 8 / 256;
    u32x4 r[NV];
    __device__ __forceinline__ void fetch(const uint16_t* Z, int64_t ld, int64_t M, int K, int64_t m0, int k0, int tid) {
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            const int idx = tid + 256 * i;
            const int64_t m = m0 + (idx >> 3);
            const int k = k0 + 8 * (idx & 7);
            r[i] = u32x4{0u, 0u, 0u, 0u};
            if (m < M && k < K) r[i] = *reinterpret_cast<const u32x4*>(Z + m * ld + k);
        }
    }
    __device__ __forceinline__ void stage(uint16_t (*As)[kLdh], int tid) {
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            const int idx = tid + 256 * i;
            *reinterpret_cast<u32x4*>(&As[idx >> 3][8 * (idx & 7)]) = r[i];
        }
    }
};

// One kBKh x BN tile of a bf16 weight matrix into Bs[n][k].  Row-major [K][N]: transposed on the way (8 x 8
// blocks).  trans (the matrix is [N][K] row-major): already in the layout the MFMA wants, plain 16-byte copies.
template <int BN>
struct BTileBF16 {
    u32x4 r[8];
    __device__ __forceinline__ void fetch(const uint16_t* W, int K, int N, int k0, int n0, int tid, bool trans = false) {
        if (!trans) {
            if (tid >= BN) return;              // kBKh/8 * BN/8 = BN blocks of 8 x 8
            const int kb = tid / (BN / 8), n = n0 + 8 * (tid % (BN / 8));
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int k = k0 + 8 * kb + i;
                r[i] = u32x4{0u, 0u, 0u, 0u};
                if (k < K && n < N) r[i] = *reinterpret_cast<const u32x4*>(W + (int64_t)k * N + n);
            }
        } else {
#pragma unroll
            for (int i = 0; i < BN / 32; ++i) {  // BN * 8 pieces of 16 bytes over 256 threads
                const int idx = tid + 256 * i;
                const int n = n0 + (idx >> 3), k = k0 + 8 * (idx & 7);
                r[i] = u32x4{0u, 0u, 0u, 0u};
                if (n < N && k < K) r[i] = *reinterpret_cast<const u32x4*>(W + (int64_t)n * K + k);
            }
        }
    }
    __device__ __forceinline__ void stage(uint16_t (*Bs)[kLdh], int tid, bool trans = false) {
        if (!trans) {
            if (tid >= BN) return;
            const int kb = tid / (BN / 8), nb = tid % (BN / 8);
            u32x4 t[8];
            transpose8x8_bf16(r, t);
#pragma unroll
            for (int c = 0; c < 8; ++c) *reinterpret_cast<u32x4*>(&Bs[8 * nb + c][8 * kb]) = t[c];
        } else {
#pragma unroll
            for (int i = 0; i < BN / 32; ++i) {
                const int idx = tid + 256 * i;
                *reinterpret_cast<u32x4*>(&Bs[idx >> 3][8 * (idx & 7)]) = r[i];
            }
        }
    }
};

template <int TM, int TN>
__device__ __forceinline__ void mfma_tile_bf16(const uint16_t* A, int lda, int arow0, int acol0,
                                               const uint16_t (*Bs)[kLdh], int brow0, int li, int lh,
                                               f32x16 (&acc)[TM][TN]) {
#pragma unroll
    for (int kk = 0; kk < kBKh / 16; ++kk) {
        bf16x8 fa[TM], fb[TN];
#pragma unroll
        for (int i = 0; i < TM; ++i)
            fa[i] = __builtin_bit_cast(
                bf16x8, *reinterpret_cast<const u32x4*>(A + (arow0 + 32 * i + li) * lda + acol0 + kk * 16 + 8 * lh));
#pragma unroll
        for (int j = 0; j < TN; ++j)
            fb[j] = __builtin_bit_cast(bf16x8,
                                       *reinterpret_cast<const u32x4*>(&Bs[brow0 + 32 * j + li][kk * 16 + 8 * lh]));
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
    }
}

template <int BN>
__global__ __launch_bounds__(256) void linear_bf16_kernel(LinArgs a) {
    constexpr int BM = 128, TM = 2, TN = BN / 64;
    __shared__ __attribute__((aligned(16))) uint16_t As[BM][kLdh];
    __shared__ __attribute__((aligned(16))) uint16_t Bs[BN][kLdh];
    const uint16_t* Z = reinterpret_cast<const uint16_t*>(a.Z);
    const uint16_t* W = reinterpret_cast<const uint16_t*>(a.W);
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, li = lane & 31, lh = lane >> 5;
    const int64_t m0 = (int64_t)blockIdx.x * BM;
    const int n0 = blockIdx.y * BN;
    const int wm0 = (wave >> 1) * 64, wn0 = (wave & 1) * (BN / 2);
    f32x16 acc[TM][TN];
    zero_acc(acc);
    ATileBF16<BM> ta;
    BTileBF16<BN> tb;
    const bool tr = a.trans_w != 0;
    ta.fetch(Z, a.ldz, a.M, a.K, m0, 0, tid);
    tb.fetch(W, a.K, a.N, 0, n0, tid, tr);
    for (int k0 = 0; k0 < a.K; k0 += kBKh) {
        __syncthreads();
        ta.stage(As, tid);
        tb.stage(Bs, tid, tr);
        __syncthreads();
        if (k0 + kBKh < a.K) {
            ta.fetch(Z, a.ldz, a.M, a.K, m0, k0 + kBKh, tid);
            tb.fetch(W, a.K, a.N, k0 + kBKh, n0, tid, tr);
        }
        mfma_tile_bf16<TM, TN>(&As[0][0], kLdh, wm0, 0, Bs, wn0, li, lh, acc);
    }
    uint16_t* Y = reinterpret_cast<uint16_t*>(a.Y);
    const uint16_t* bias = reinterpret_cast<const uint16_t*>(a.bias);
    const uint16_t* mask = reinterpret_cast<const uint16_t*>(a.mask);
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int n = n0 + wn0 + 32 * j + li;
            if (n >= a.N) continue;
            const float bv = bias ? bf16_val(bias, n) : 0.f;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int64_t m = m0 + wm0 + 32 * i + 8 * (r / 4) + 4 * lh + (r % 4);
                if (m >= a.M) continue;
                float y = a.c_w * acc[i][j][r] + bv;
                if (a.c_id != 0.f) y += a.c_id * bf16_val(Z, m * a.ldz + n);
                if (a.relu) y = fmaxf(y, 0.f);
                if (mask && !(bf16_val(mask, m * a.ldmask + n) > 0.f)) y = 0.f;
                Y[m * a.ldy + n] = (uint16_t)f32_to_bf16(y);
            }
        }
}

// bf16 fused MLP: 64 rows per workgroup, wavefronts 2 x 2 over (rows, columns).
// Phase 1: hidden = relu(Z W1 + b1) for all F_hid columns, rounded to bf16 into
// LDS.  Phase 2: Y = act(hidden W2 + b2), the hidden tile being the A operand.
__global__ __launch_bounds__(256) void mlp2_bf16_kernel(MlpArgs a) {
    constexpr int BM = kMlpRowsBF16, BN = 256, TN = 4;
    constexpr int kLdHid = kHidMax + 8;
    extern __shared__ __attribute__((aligned(16))) char smem[];   // above the 64 KB static limit
    uint16_t (*Hs)[kLdHid] = reinterpret_cast<uint16_t (*)[kLdHid]>(smem);
    uint16_t (*As)[kLdh] = reinterpret_cast<uint16_t (*)[kLdh]>(smem + 2 * BM * kLdHid);
    uint16_t (*Bs)[kLdh] = reinterpret_cast<uint16_t (*)[kLdh]>(smem + 2 * BM * (kLdHid + kLdh));
    const uint16_t* Z = reinterpret_cast<const uint16_t*>(a.Z);
    const uint16_t* W1 = reinterpret_cast<const uint16_t*>(a.W1);
    const uint16_t* W2 = reinterpret_cast<const uint16_t*>(a.W2);
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, li = lane & 31, lh = lane >> 5;
    const int64_t m0 = (int64_t)blockIdx.x * BM;
    const int n0 = blockIdx.y * BN;
    const int wm0 = (wave >> 1) * 32, wn0 = (wave & 1) * (BN / 2);
    f32x16 acc[1][TN];
    zero_acc(acc);
    ATileBF16<BM> ta;
    BTileBF16<BN> tb;
    ta.fetch(Z, a.ldz, a.M, a.K, m0, 0, tid);
    tb.fetch(W1, a.K, a.H, 0, 0, tid);
    for (int k0 = 0; k0 < a.K; k0 += kBKh) {
        __syncthreads();
        ta.stage(As, tid);
        tb.stage(Bs, tid);
        __syncthreads();
        if (k0 + kBKh < a.K) {
            ta.fetch(Z, a.ldz, a.M, a.K, m0, k0 + kBKh, tid);
            tb.fetch(W1, a.K, a.H, k0 + kBKh, 0, tid);
        }
        mfma_tile_bf16<1, TN>(&As[0][0], kLdh, wm0, 0, Bs, wn0, li, lh, acc);
    }
    const uint16_t* b1 = reinterpret_cast<const uint16_t*>(a.b1);
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int h = wn0 + 32 * j + li;
        const float bv = (b1 && h < a.H) ? bf16_val(b1, h) : 0.f;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const float v = h < a.H ? fmaxf(acc[0][j][r] + bv, 0.f) : 0.f;
            Hs[wm0 + 8 * (r / 4) + 4 * lh + (r % 4)][h] = (uint16_t)f32_to_bf16(v);
        }
    }
    zero_acc(acc);
    tb.fetch(W2, a.H, a.N, 0, n0, tid);
    for (int k0 = 0; k0 < a.H; k0 += kBKh) {
        __syncthreads();                 // Hs written / previous Bs consumed
        tb.stage(Bs, tid);
        __syncthreads();
        if (k0 + kBKh < a.H) tb.fetch(W2, a.H, a.N, k0 + kBKh, n0, tid);
        mfma_tile_bf16<1, TN>(&Hs[0][0], kLdHid, wm0, k0, Bs, wn0, li, lh, acc);
    }
    uint16_t* Y = reinterpret_cast<uint16_t*>(a.Y);
    const uint16_t* b2 = reinterpret_cast<const uint16_t*>(a.b2);
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int n = n0 + wn0 + 32 * j + li;
        if (n >= a.N) continue;
        const float bv = b2 ? bf16_val(b2, n) : 0.f;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int64_t m = m0 + wm0 + 8 * (r / 4) + 4 * lh + (r % 4);
            if (m >= a.M) continue;
            float y = acc[0][j][r] + bv;
            if (a.relu_out) y = fmaxf(y, 0.f);
            Y[m * a.ldy + n] = (uint16_t)f32_to_bf16(y);
        }
    }
}

// ---------------------------------------------------------------------- weights-stationary bf16 kernels
// For feature widths up to 256 the whole weight matrix fits in the registers
// of one workgroup: wavefront w of 8 keeps the MFMA B-fragments of columns
// [32w, 32w+32) for every k (K/16 fragments of 8 bf16 per lane), loaded once.
// The workgroup is persistent (one per compute unit) and streams 64-row tiles
// of Z through LDS, so after start-up the only global traffic is Z in and Y
// out: the weights are never re-staged.  ws_bf16_kernel is the single product;
// ws_mlp_bf16_kernel keeps W1 and W2 on separate wavefronts and chains the two
// products of the GIN MLP through an LDS-resident hidden tile.
struct WsArgs {
    const uint16_t* Z;  int64_t ldz;
    const uint16_t* W1; const uint16_t* b1;
    const uint16_t* W2; const uint16_t* b2;
    uint16_t* Y;        int64_t ldy;
    int64_t M, n_tiles;
    int K, H, N;        // single product: H == N is the output width and W2 is unused
    float c_id, c_w;
    int relu1, relu_out;
    int trans_w1;                          // W1 is given as [H][K] (single product only)
    const uint16_t* mask; int64_t ldmask;  // optional [M, N]: outputs where mask <= 0 are set to zero
    const int32_t* push_idx;               // optional: output row m is also stored to push_hist[push_idx[m], :]
    uint16_t* push_hist; int64_t ld_push;
    uint16_t* H_out; int64_t ldh_out;      // optional (fused MLP): the hidden activation is stored as well
};

constexpr int kWsRows = 64;

template <int KT>
__device__ __forceinline__ void load_w_frags(const uint16_t* W, int K, int ncols, int col, int lh, bf16x8 (&f)[KT],
                                             bool trans = false) {
#pragma unroll
    for (int kk = 0; kk < KT; ++kk) {
        u32x4 v = {0u, 0u, 0u, 0u};
        if (trans) {                     // [ncols][K] row-major, K a multiple of 8: the fragment is contiguous
            const int k = 16 * kk + 8 * lh;
            if (k < K && col < ncols) v = *reinterpret_cast<const u32x4*>(W + (int64_t)col * K + k);
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int k = 16 * kk + 8 * lh + e;
                uint32_t x = 0;
                if (k < K && col < ncols) x = W[(int64_t)k * ncols + col];
                v[e >> 1] |= x << (16 * (e & 1));
            }
        }
        f[kk] = __builtin_bit_cast(bf16x8, v);
    }
}

// The products are evaluated transposed, D' = W^T Z^T: the weight fragment is
// the MFMA A operand and the Z fragment the B operand (both hold 8 consecutive
// k of one row/column, so the register contents are what they would be the
// other way round).  Then a lane holds, for ONE row m of the tile, 4 groups of
// 4 consecutive output columns, which go to the [m][n] LDS tiles as 8-byte
// stores after a packed hardware fp32->bf16 conversion.
template <int KT1>
__global__ __launch_bounds__(512) void ws_bf16_kernel(WsArgs a) {
    constexpr int LDA = 16 * KT1 + 8;                 // bf16 elements per LDS row of the Z tile
    constexpr int LDY = 256 + 8;                      // ... of the output staging tile
    constexpr int VPR = 2 * KT1;                      // 16-byte vectors per Z-tile row
    constexpr int NVA = (kWsRows * VPR + 511) / 512;  // vectors per thread per tile
    constexpr int MT = kWsRows / 32;                  // 32-row blocks per tile
    extern __shared__ __attribute__((aligned(16))) char smem[];
    uint16_t* As = reinterpret_cast<uint16_t*>(smem);                       // [2][64][LDA]
    uint16_t* Ys = As + 2 * kWsRows * LDA;                                  // [64][LDY]
    const int tid = threadIdx.x, lane = tid & 63, li = lane & 31, lh = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);      // the same in every lane, and known to be

    bf16x8 w1f[KT1];
    load_w_frags<KT1>(a.W1, a.K, a.H, 32 * wave + li, lh, w1f, a.trans_w1 != 0);
    // output columns of this lane: n(q, e) = 32*wave + 8*q + 4*lh + e, q, e in 0..3
    const int nbase = 32 * wave + 4 * lh;
    // bias as fp32 in LDS (read back four at a time in the epilogue: registers are what this kernel is short of)
    float* bias1 = reinterpret_cast<float*>(Ys + kWsRows * LDY);            // [256]
    if (tid < 256) bias1[tid] = (a.b1 && tid < a.H) ? bf16_val(a.b1, tid) : 0.f;

    // Loads are issued unconditionally from a clamped address and zeroed by a select afterwards: with no
    // branch around them the compiler counts outstanding memory operations exactly, and a later wait for one
    // load does not turn into a wait for everything in flight.
    u32x4 ra[NVA];
    const bool k_whole = a.K == 16 * KT1;
    auto fetch = [&](int64_t tile) {
        const uint16_t* base = a.Z + tile * kWsRows * a.ldz;      // the same for every lane; offsets are 32-bit
        const bool full = k_whole && (tile + 1) * kWsRows <= a.M;
#pragma unroll
        for (int i = 0; i < NVA; ++i) {
            const int idx = tid + 512 * i;
            const int row = idx / VPR, k = 8 * (idx % VPR);
            uint32_t off = (uint32_t)row * (uint32_t)a.ldz + (uint32_t)k;
            if (!full) {
                const bool ok = idx < kWsRows * VPR && tile * kWsRows + row < a.M && k < a.K;
                off = ok ? off : 0u;
            } else if (kWsRows * VPR % 512 != 0 && idx >= kWsRows * VPR) {
                off = 0u;
            }
            ra[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(base + off));
        }
    };
    auto stage = [&](int buf, int64_t tile) {          // tile: the one fetch() was called for
        const bool full = k_whole && (tile + 1) * kWsRows <= a.M;
#pragma unroll
        for (int i = 0; i < NVA; ++i) {
            const int idx = tid + 512 * i;
            const int row = idx / VPR, k = 8 * (idx % VPR);
            u32x4 v = ra[i];
            if (!full) {
                const bool ok = tile * kWsRows + row < a.M && k < a.K;
                v = ok ? v : u32x4{0u, 0u, 0u, 0u};
            }
            if (idx < kWsRows * VPR) *reinterpret_cast<u32x4*>(As + (buf * kWsRows + row) * LDA + k) = v;
        }
    };

    // Order of memory operations per tile: the loads of the tile after next are issued BEFORE this tile's
    // output stores and are consumed one iteration later, so they are in flight during the stores and the next
    // tile's MFMAs, and waiting for them never waits for a store (loads and stores retire in issue order).
    constexpr int NPI = (kWsRows * 32 + 511) / 512;   // output vectors per thread per tile at the widest row
    int64_t tile = blockIdx.x;
    if (tile < a.n_tiles) {
        fetch(tile);
        stage(0, tile);
        if (tile + gridDim.x < a.n_tiles) fetch(tile + gridDim.x);
    }
    int buf = 0;
    for (; tile < a.n_tiles; tile += gridDim.x, buf ^= 1) {
        const int64_t next = tile + gridDim.x;
        __syncthreads();                               // (1) Z tile `buf` staged; previous tile fully consumed
        // output vector (row, v) of a thread: row = tid / 32 + 16 i, v = tid % 32 (the staging tile is 32 vectors
        // wide; narrower outputs leave the lanes beyond their width idle)
        const bool out_full = (tile + 1) * kWsRows <= a.M;
        int32_t prow[NPI] = {};                        // history slots of the rows this thread will store
        if (a.push_idx) {
            const int32_t* pi = a.push_idx + tile * kWsRows;
#pragma unroll
            for (int i = 0; i < NPI; ++i) {
                int row = (tid >> 5) + 16 * i;
                if (!out_full) row = tile * kWsRows + row < a.M ? row : 0;
                prow[i] = pi[row];
            }
        }
        const uint16_t* At = As + buf * kWsRows * LDA;
        f32x16 acc[MT];
#pragma unroll
        for (int t = 0; t < MT; ++t)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[t][r] = 0.f;
        if (32 * wave < a.H) {
#pragma unroll
            for (int kk = 0; kk < KT1; ++kk)
#pragma unroll
                for (int t = 0; t < MT; ++t) {
                    const bf16x8 fz = __builtin_bit_cast(
                        bf16x8, *reinterpret_cast<const u32x4*>(At + (32 * t + li) * LDA + 16 * kk + 8 * lh));
                    acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(w1f[kk], fz, acc[t], 0, 0, 0);
                }
        }
#pragma unroll
        for (int t = 0; t < MT; ++t)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                float v[4];
                const f32x4 bq = *reinterpret_cast<const f32x4*>(bias1 + nbase + 8 * q);
#pragma unroll
                for (int e = 0; e < 4; ++e) v[e] = a.c_w * acc[t][4 * q + e] + bq[e];
                if (a.c_id != 0.f && nbase + 8 * q < a.N) {      // identity term straight from the staged Z tile (K == N)
                    const u32x2 z = *reinterpret_cast<const u32x2*>(At + (32 * t + li) * LDA + nbase + 8 * q);
                    v[0] += a.c_id * bf16_lo(z[0]); v[1] += a.c_id * bf16_hi(z[0]);
                    v[2] += a.c_id * bf16_lo(z[1]); v[3] += a.c_id * bf16_hi(z[1]);
                }
                if (a.relu1) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] = fmaxf(v[e], 0.f);
                }
                *reinterpret_cast<u32x2*>(Ys + (32 * t + li) * LDY + nbase + 8 * q) =
                    u32x2{pack_bf16(v[0], v[1]), pack_bf16(v[2], v[3])};
            }
        // take delivery of the history slots before new loads are queued behind them: the stores below then
        // need no wait that the loads just issued would have to satisfy first
#pragma unroll
        for (int i = 0; i < NPI; ++i) asm volatile("" : "+v"(prow[i]));
        if (next < a.n_tiles) {
            stage(buf ^ 1, next);                      // the other buffer: nobody reads it before the next (1)
            if (next + gridDim.x < a.n_tiles) fetch(next + gridDim.x);
        }
        __syncthreads();                               // (3) output tile staged
        {
            const int vpr = a.N >> 3;                  // 16-byte vectors per output row
            uint16_t* ybase = a.Y + tile * kWsRows * a.ldy;
            const uint16_t* mbase = a.mask ? a.mask + tile * kWsRows * a.ldmask : nullptr;
            const int v = tid & 31;
            if (v < vpr) {
#pragma unroll
                for (int i = 0; i < NPI; ++i) {
                    const int row = (tid >> 5) + 16 * i;
                    if (out_full || tile * kWsRows + row < a.M) {
                        u32x4 o = *reinterpret_cast<const u32x4*>(Ys + row * LDY + 8 * v);
                        if (mbase) {
                            const u32x4 km = *reinterpret_cast<const u32x4*>(mbase + ((uint32_t)row * (uint32_t)a.ldmask + 8u * v));
#pragma unroll
                            for (int q = 0; q < 4; ++q) {
                                if (!(bf16_lo(km[q]) > 0.f)) o[q] &= 0xFFFF0000u;
                                if (!(bf16_hi(km[q]) > 0.f)) o[q] &= 0x0000FFFFu;
                            }
                        }
                        __builtin_nontemporal_store(
                            o, reinterpret_cast<u32x4*>(ybase + ((uint32_t)row * (uint32_t)a.ldy + 8u * v)));
                        if (a.push_idx)      // Push fused into the epilogue: the row goes to its history slot as well
                            __builtin_nontemporal_store(
                                o, reinterpret_cast<u32x4*>(a.push_hist + (int64_t)prow[i] * a.ld_push + 8 * v));
                    }
                }
            }
        }
    }
}

// Weight fragments for a 64-column block, through LDS: the [K][ncols] matrix is staged 128 rows at a time with
// 16-byte loads, and a lane picks the 8 consecutive k of its column out of the staged chunk (the MFMA operand
// wants the matrix transposed).  ncols is a multiple of 8 and W is 16-byte aligned.  All threads of the
// workgroup call this; only those with `mine` keep fragments.
constexpr int kLdW = 256 + 8;
template <int KT, int KTM>
__device__ __forceinline__ void load_w_block_lds(const uint16_t* W, int K, int ncols, uint16_t* Wl, bool mine, int cb,
                                                 int li, int lh, int tid, bf16x8 (&w)[2][KTM]) {
    constexpr int NCH = (KT + 7) / 8;
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
        __syncthreads();                               // the previous chunk has been read
        for (int idx = tid; idx < 128 * 32; idx += 512) {
            const int r = idx >> 5, v = idx & 31;
            const int k = 128 * c + r;
            u32x4 x = {0u, 0u, 0u, 0u};
            if (k < K && 8 * v < ncols) x = *reinterpret_cast<const u32x4*>(W + (int64_t)k * ncols + 8 * v);
            *reinterpret_cast<u32x4*>(Wl + r * kLdW + 8 * v) = x;
        }
        __syncthreads();
        if (mine) {
#pragma unroll
            for (int kk = 8 * c; kk < 8 * c + 8 && kk < KT; ++kk)
#pragma unroll
                for (int ch = 0; ch < 2; ++ch) {
                    const int col = 64 * cb + 32 * ch + li;
                    u32x4 v = {0u, 0u, 0u, 0u};
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        const uint32_t x = Wl[(16 * (kk - 8 * c) + 8 * lh + e) * kLdW + col];
                        v[e >> 1] |= x << (16 * (e & 1));
                    }
                    w[ch][kk] = __builtin_bit_cast(bf16x8, v);
                }
        }
    }
    __syncthreads();
}

// Fused two-layer MLP, weights stationary, wavefronts specialised by layer.
//
// Wavefronts 0-3 hold W1 (64 hidden columns each), wavefronts 4-7 hold W2 (64 output columns each); every SIMD
// gets one of each.  The two products are pipelined over tiles: in phase p the first group turns Z tile p into
// hidden tile p (LDS, two buffers) while the second group turns hidden tile p-1 into output tile p-1, so the
// each staged row is read from LDS by four wavefronts instead of eight.  The loads of Z tile p+1 are issued at the
// start of the phase and travel during the products; between the phase's two barriers all wavefronts move data:
// output tile p-1 from its staging tile to Y (and to the history rows), Z tile p+1 from registers to LDS.
// EXACT: K = 16 KT1 and H = N = 256, i.e. every column of every tile exists: the checks on the input columns and
// the output width are compiled out.
template <int KT1, int KT2, bool EXACT>
__global__ __launch_bounds__(512) void ws_mlp_bf16_kernel(WsArgs a) {
    constexpr int LDA = 16 * KT1 + 8, LDH = 16 * KT2 + 8, LDY = 256 + 8;
    constexpr int VPR = 2 * KT1;
    constexpr int NVA = (kWsRows * VPR + 511) / 512;
    constexpr int NPI = (kWsRows * 32 + 511) / 512;
    constexpr int MT = kWsRows / 32;
    constexpr int KTM = KT1 > KT2 ? KT1 : KT2;
    static_assert(KT2 == 16, "the hidden and output staging tiles are 256 columns wide, one 64-column block per wavefront");
    extern __shared__ __attribute__((aligned(16))) char smem[];
    uint16_t* As = reinterpret_cast<uint16_t*>(smem);                       // [64][LDA]
    uint16_t* Hs = As + kWsRows * LDA;                                      // [2][64][LDH]
    uint16_t* Ys = Hs + 2 * kWsRows * LDH;                                  // [64][LDY]
    float* bias1 = reinterpret_cast<float*>(Ys + kWsRows * LDY);            // [256]
    float* bias2 = bias1 + 256;                                             // [256]
    const int tid = threadIdx.x, lane = tid & 63, li = lane & 31, lh = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);      // the same in every lane, and known to be
    const int role = wave >> 2, cb = wave & 3;        // role 0: Z W1, role 1: H W2; 64-column block cb

    bf16x8 w[2][KTM];
    load_w_block_lds<KT1, KTM>(a.W1, a.K, a.H, As, role == 0, cb, li, lh, tid, w);
    load_w_block_lds<KT2, KTM>(a.W2, a.H, a.N, As, role == 1, cb, li, lh, tid, w);
    if (tid < 256) {
        bias1[tid] = (a.b1 && tid < a.H) ? bf16_val(a.b1, tid) : 0.f;
        bias2[tid] = (a.b2 && tid < a.N) ? bf16_val(a.b2, tid) : 0.f;
    }

    u32x4 ra[NVA];
    // Per-thread offsets (row, column, LDS address) are recomputed from the thread index where they are used
    // (the index is made opaque there): kept live across the products they would be spilled.  Addresses are a
    // tile base that is the same for every lane plus a 32-bit offset; a tile that lies wholly inside the matrix
    // (all but the last, when the width is a multiple of the MFMA depth) takes a path without per-lane checks.
    const bool k_whole = EXACT || a.K == 16 * KT1;
    auto fetch = [&](int64_t tile, int tl) {          // unconditional loads; clamped addresses where checks are needed
        const uint16_t* base = a.Z + tile * kWsRows * a.ldz;
        const bool full = k_whole && (tile + 1) * kWsRows <= a.M;
#pragma unroll
        for (int i = 0; i < NVA; ++i) {
            const int idx = tl + 512 * i;
            const int row = idx / VPR, k = 8 * (idx % VPR);
            uint32_t off = (uint32_t)row * (uint32_t)a.ldz + (uint32_t)k;
            if (!full) {
                const bool ok = idx < kWsRows * VPR && tile * kWsRows + row < a.M && k < a.K;
                off = ok ? off : 0u;
            } else if (kWsRows * VPR % 512 != 0 && idx >= kWsRows * VPR) {
                off = 0u;
            }
            ra[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(base + off));
        }
    };
    auto stage = [&](int64_t tile, int tl) {          // tile: the one fetch() was called for
        const bool full = k_whole && (tile + 1) * kWsRows <= a.M;
#pragma unroll
        for (int i = 0; i < NVA; ++i) {
            const int idx = tl + 512 * i;
            const int row = idx / VPR, k = 8 * (idx % VPR);
            u32x4 v = ra[i];
            if (!full) {
                const bool ok = tile * kWsRows + row < a.M && k < a.K;
                v = ok ? v : u32x4{0u, 0u, 0u, 0u};
            }
            if (idx < kWsRows * VPR) *reinterpret_cast<u32x4*>(As + row * LDA + k) = v;
        }
    };
    // D[m][64cb .. 64cb+63] = act(X[m][:] Wcols + bias) for the 64 rows of a tile, X and D in LDS.  Transposed
    // products: a lane ends up with 4 consecutive columns of one row per group of four accumulator registers.
    // Columns beyond the width need no check: their weight fragments and biases were loaded as zeros, so they come
    // out as exact zeros (and are zero operands of the next product).
    auto product = [&](auto kt_tag, const uint16_t* X, int ldx, uint16_t* D, int ldd, const float* bias, bool relu) {
        constexpr int KT = decltype(kt_tag)::value;
#pragma unroll
        for (int t = 0; t < MT; ++t) {                 // 32 rows at a time: two accumulator tiles live, not four
            // the accumulators start from the bias of their columns (element 4q+e of a lane is column n0(q)+e)
            f32x16 acc[2];
#pragma unroll
            for (int ch = 0; ch < 2; ++ch)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const f32x4 bq = *reinterpret_cast<const f32x4*>(bias + 64 * cb + 32 * ch + 8 * q + 4 * lh);
#pragma unroll
                    for (int e = 0; e < 4; ++e) acc[ch][4 * q + e] = bq[e];
                }
            // operand fragments are read from LDS PF steps ahead of the MFMAs that use them
            constexpr int PF = KT < 4 ? KT : 4;
            const uint16_t* xrow = X + (32 * t + li) * ldx + 8 * lh;
            u32x4 fx[PF];
#pragma unroll
            for (int j = 0; j < PF; ++j) fx[j] = *reinterpret_cast<const u32x4*>(xrow + 16 * j);
#pragma unroll
            for (int kk = 0; kk < KT; ++kk) {
                const bf16x8 cur = __builtin_bit_cast(bf16x8, fx[kk % PF]);
                if (kk + PF < KT) fx[kk % PF] = *reinterpret_cast<const u32x4*>(xrow + 16 * (kk + PF));
#pragma unroll
                for (int ch = 0; ch < 2; ++ch)
                    acc[ch] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(w[ch][kk], cur, acc[ch], 0, 0, 0);
            }
            uint16_t* drow = D + (32 * t + li) * ldd + 64 * cb + 4 * lh;
#pragma unroll
            for (int ch = 0; ch < 2; ++ch)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    float v[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        v[e] = acc[ch][4 * q + e];
                        if (relu) v[e] = fmaxf(v[e], 0.f);
                    }
                    *reinterpret_cast<u32x2*>(drow + 32 * ch + 8 * q) = u32x2{pack_bf16(v[0], v[1]), pack_bf16(v[2], v[3])};
                }
        }
    };

    const int grid = (int)gridDim.x, t0 = (int)blockIdx.x;
    const int n_my = (int)((a.n_tiles - t0 + grid - 1) / grid);   // tiles of this workgroup (>= 1)
    fetch(t0, tid);
    stage(t0, tid);
    __syncthreads();
    for (int p = 0; p <= n_my; ++p) {
        const int64_t t_out = t0 + (int64_t)(p - 1) * grid;        // tile whose output leaves in this phase
        int32_t prow[NPI] = {};
        int tl = tid;
        asm volatile("" : "+v"(tl));
        // output vector (row, v) of a thread: row = tl / 32 + 16 i, v = tl % 32 (the staging tile is 32 vectors wide;
        // narrower outputs leave the lanes beyond their width idle)
        const bool out_full = p >= 1 && (t_out + 1) * kWsRows <= a.M;
        if (a.push_idx && p >= 1) {
            const int32_t* pi = a.push_idx + t_out * kWsRows;
#pragma unroll
            for (int i = 0; i < NPI; ++i) {
                int row = (tl >> 5) + 16 * i;
                if (!out_full) row = t_out * kWsRows + row < a.M ? row : 0;
                prow[i] = pi[row];
            }
        }
        // loads of the next Z tile: issued here, they travel while the matrix pipes work, and are staged
        // between this phase's two barriers
        if (p + 1 < n_my) fetch(t0 + (int64_t)(p + 1) * grid, tl);
        if (role == 0) {
            if (p < n_my)
                product(std::integral_constant<int, KT1>{}, As, LDA, Hs + (p & 1) * kWsRows * LDH, LDH, bias1, true);
        } else {
            if (p >= 1)
                product(std::integral_constant<int, KT2>{}, Hs + ((p - 1) & 1) * kWsRows * LDH, LDH, Ys, LDY, bias2,
                        a.relu_out != 0);
        }
        __syncthreads();                               // Z tile consumed; hidden tile p and output tile p-1 complete
#pragma unroll
        for (int i = 0; i < NPI; ++i) asm volatile("" : "+v"(prow[i]));   // delivered before new loads queue up
        asm volatile("" : "+v"(tl));
        if (p + 1 < n_my) stage(t0 + (int64_t)(p + 1) * grid, tl);
        if (p >= 1) {
            const int vpr = EXACT ? 32 : a.N >> 3;     // 16-byte vectors per output row
            const int tq = __builtin_amdgcn_readfirstlane((int)t_out);   // the tile index, in a scalar register
            uint16_t* ybase = a.Y + (int64_t)tq * kWsRows * a.ldy;
            const int v = tl & 31;
            if (v < vpr) {
#pragma unroll
                for (int i = 0; i < NPI; ++i) {
                    const int row = (tl >> 5) + 16 * i;
                    if (out_full || (int64_t)tq * kWsRows + row < a.M) {
                        const u32x4 o = *reinterpret_cast<const u32x4*>(Ys + row * LDY + 8 * v);
                        __builtin_nontemporal_store(
                            o, reinterpret_cast<u32x4*>(ybase + ((uint32_t)row * (uint32_t)a.ldy + 8u * v)));
                        if (a.push_idx)
                            __builtin_nontemporal_store(
                                o, reinterpret_cast<u32x4*>(a.push_hist + (int64_t)prow[i] * a.ld_push + 8 * v));
                    }
                }
            }
            if (a.H_out) {
                // a training pass reads the hidden activation again: tile p-1 of it is complete and not written
                // before the next phase, so it leaves from its LDS buffer the same way
                const int hvpr = EXACT ? 32 : a.H >> 3;
                const uint16_t* hs = Hs + ((p - 1) & 1) * kWsRows * LDH;
                uint16_t* hbase = a.H_out + (int64_t)tq * kWsRows * a.ldh_out;
                if (v < hvpr) {
#pragma unroll
                    for (int i = 0; i < NPI; ++i) {
                        const int row = (tl >> 5) + 16 * i;
                        if (out_full || (int64_t)tq * kWsRows + row < a.M)
                            __builtin_nontemporal_store(
                                *reinterpret_cast<const u32x4*>(hs + row * LDH + 8 * v),
                                reinterpret_cast<u32x4*>(hbase + ((uint32_t)row * (uint32_t)a.ldh_out + 8u * v)));
                    }
                }
            }
        }
        __syncthreads();                               // next Z tile staged, output staging tile free again
    }
}

template <int KT1, int KT2>
gas_status launch_ws_mlp(const WsArgs& a, hipStream_t s) {
    constexpr int smem = 2 * (kWsRows * (16 * KT1 + 8) + 2 * kWsRows * (16 * KT2 + 8) + kWsRows * (256 + 8)) + 2 * 256 * 4;
    static const hipError_t attr1 = hipFuncSetAttribute(reinterpret_cast<const void*>(ws_mlp_bf16_kernel<KT1, KT2, true>),
                                                        hipFuncAttributeMaxDynamicSharedMemorySize, smem);
    static const hipError_t attr2 = hipFuncSetAttribute(reinterpret_cast<const void*>(ws_mlp_bf16_kernel<KT1, KT2, false>),
                                                        hipFuncAttributeMaxDynamicSharedMemorySize, smem);
    GAS_CHECK_HIP(attr1);
    GAS_CHECK_HIP(attr2);
    int dev = 0, cus = 256;
    if (hipGetDevice(&dev) == hipSuccess) {
        int v = 0;
        if (hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0) cus = v;
    }
    const int64_t blocks = a.n_tiles < cus ? a.n_tiles : cus;
    if (a.K == 16 * KT1 && a.H == 256 && a.N == 256)
        hipLaunchKernelGGL((ws_mlp_bf16_kernel<KT1, KT2, true>), dim3((unsigned)blocks), dim3(512), smem, s, a);
    else
        hipLaunchKernelGGL((ws_mlp_bf16_kernel<KT1, KT2, false>), dim3((unsigned)blocks), dim3(512), smem, s, a);
    GAS_CHECK_HIP(hipGetLastError());
    return GAS_OK;
}

template <int KT1>
gas_status launch_ws(const WsArgs& a, hipStream_t s) {
    constexpr int smem = 2 * (2 * kWsRows * (16 * KT1 + 8) + kWsRows * (256 + 8)) + 256 * 4;   // + the bias in fp32
    static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(ws_bf16_kernel<KT1>),
                                                       hipFuncAttributeMaxDynamicSharedMemorySize, smem);
    GAS_CHECK_HIP(attr);
    int dev = 0, cus = 256;
    if (hipGetDevice(&dev) == hipSuccess) {
        int v = 0;
        if (hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0) cus = v;
    }
    const int64_t blocks = a.n_tiles < cus ? a.n_tiles : cus;
    hipLaunchKernelGGL((ws_bf16_kernel<KT1>), dim3((unsigned)blocks), dim3(512), smem, s, a);
    GAS_CHECK_HIP(hipGetLastError());
    return GAS_OK;
}

// ====================================================================== element-wise paths
// For bf16 operands that are not 16-byte aligned (odd widths, odd strides):
// one thread per output element, fp32 accumulation.
__global__ __launch_bounds__(256) void linear_bf16_generic_kernel(LinArgs a) {
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= a.M * a.N) return;
    const int64_t m = idx / a.N;
    const int n = (int)(idx % a.N);
    const uint16_t* Z = reinterpret_cast<const uint16_t*>(a.Z);
    const uint16_t* W = reinterpret_cast<const uint16_t*>(a.W);
    float s = 0.f;
    for (int k = 0; k < a.K; ++k)
        s = fmaf(bf16_val(Z, m * a.ldz + k), bf16_val(W, a.trans_w ? (int64_t)n * a.K + k : (int64_t)k * a.N + n), s);
    float y = a.c_w * s;
    if (a.bias) y += bf16_val(reinterpret_cast<const uint16_t*>(a.bias), n);
    if (a.c_id != 0.f) y += a.c_id * bf16_val(Z, m * a.ldz + n);
    if (a.relu) y = fmaxf(y, 0.f);
    if (a.mask && !(bf16_val(reinterpret_cast<const uint16_t*>(a.mask), m * a.ldmask + n) > 0.f)) y = 0.f;
    reinterpret_cast<uint16_t*>(a.Y)[m * a.ldy + n] = (uint16_t)f32_to_bf16(y);
}

// One workgroup per row; the hidden row goes through LDS (bf16-rounded for
// bf16 data, as in the MFMA kernel).
template <bool BF>
__global__ __launch_bounds__(256) void mlp2_generic_kernel(MlpArgs a) {
    __shared__ float h[kHidMax];
    const int64_t m = blockIdx.x;
    auto ld = [](const char* p, int64_t i) -> float {
        if constexpr (BF) return bf16_val(reinterpret_cast<const uint16_t*>(p), i);
        else return reinterpret_cast<const float*>(p)[i];
    };
    for (int j = threadIdx.x; j < a.H; j += 256) {
        float s = 0.f;
        for (int k = 0; k < a.K; ++k) s = fmaf(ld(a.Z, m * a.ldz + k), ld(a.W1, (int64_t)k * a.H + j), s);
        if (a.b1) s += ld(a.b1, j);
        s = fmaxf(s, 0.f);
        if constexpr (BF) s = __uint_as_float(f32_to_bf16(s) << 16);
        h[j] = s;
    }
    __syncthreads();
    for (int n = threadIdx.x; n < a.N; n += 256) {
        float s = 0.f;
        for (int k = 0; k < a.H; ++k) s = fmaf(h[k], ld(a.W2, (int64_t)k * a.N + n), s);
        if (a.b2) s += ld(a.b2, n);
        if (a.relu_out) s = fmaxf(s, 0.f);
        if constexpr (BF) reinterpret_cast<uint16_t*>(a.Y)[m * a.ldy + n] = (uint16_t)f32_to_bf16(s);
        else reinterpret_cast<float*>(a.Y)[m * a.ldy + n] = s;
    }
}

// ====================================================================== backward kernels
// Weight gradient dW[k, j] = c_w * sum_m Z[m, k] * G[m, j]: the reduction runs over the rows.  The rows are cut
// into slabs; a workgroup forms the 128 x 128 tile (tk, tj) of the partial product of one slab in fp32 and
// writes it to the workspace; dw_reduce_kernel adds the slabs in slab order (fixed order, no atomics).
constexpr int kDwTile = 128;

// Rows per slab: a function of the shape alone (the workspace size and the order of the sum follow from it).
// About four workgroups per compute unit, at most 4096 rows (long slabs amortise the partial tile they write),
// at least 128: a small batch then still spreads over the chip instead of queueing in a handful of workgroups.
static int64_t dw_slab_rows(int64_t M, int K, int N) {
    const int64_t tiles = (int64_t)((K + kDwTile - 1) / kDwTile) * ((N + kDwTile - 1) / kDwTile);
    int64_t slab = (M * tiles + 1023) / 1024;
    slab = (slab + 63) / 64 * 64;
    return slab < 128 ? 128 : (slab > 4096 ? 4096 : slab);
}

// Slab partials for callers that can bring no workspace (gas_linear_bwd_weight_static): a zero-initialised array in
// the code object, one copy per GPU at that GPU's own address.  In host code the array's name is only a handle for
// the runtime; the address a kernel can use comes from hipGetSymbolAddress, asked once per device with that device
// current, and is what the launches are given.
constexpr int64_t kDwScratchBytes = 64ll << 20;
static __device__ __align__(256) unsigned char dw_scratch[kDwScratchBytes];
constexpr int kMaxDevices = 64;

static gas_status dw_scratch_pointer(void** out) {
    static std::mutex mu;
    static void* ptr[kMaxDevices] = {nullptr};
    int dev = -1;
    GAS_CHECK_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return fail(GAS_ERR_ARG, "gas_linear_bwd_weight_static: device %d", dev);
    std::lock_guard<std::mutex> lock(mu);
    if (!ptr[dev]) {
        void* p = nullptr;
        const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(dw_scratch));
        if (e != hipSuccess || !p)
            return fail(GAS_ERR_HIP, "gas_linear_bwd_weight_static: no address for the scratch array on device %d: %s",
                        dev, hipGetErrorString(e));
        ptr[dev] = p;
    }
    *out = ptr[dev];
    return GAS_OK;
}

struct DwArgs {
    const char* Z;  int64_t ldz;
    const char* G;  int64_t ldg;
    int64_t M;
    int K, N;                       // F_in, F_out
    float c_w;
    float* partial;                 // [n_slabs][K][N]
    float* dW;                      // [K][N]
    int n_slabs;
    int slab;                       // rows per slab
};

// fp32: both operands are read as single dwords from row-major LDS tiles (lanes run along the feature index).
template <bool VEC>
__global__ __launch_bounds__(256) void dw_f32_kernel(DwArgs a) {
    constexpr int BM = 32;                                  // rows per step
    __shared__ __attribute__((aligned(16))) float Zs[BM][kDwTile + 4];
    __shared__ __attribute__((aligned(16))) float Gs[BM][kDwTile + 4];
    const float* Z = reinterpret_cast<const float*>(a.Z);
    const float* G = reinterpret_cast<const float*>(a.G);
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, li = lane & 31, lh = lane >> 5;
    const int slab = blockIdx.x, k0 = blockIdx.y * kDwTile, n0 = blockIdx.z * kDwTile;
    const int64_t m_begin = (int64_t)slab * a.slab;
    const int64_t m_end = m_begin + a.slab < a.M ? m_begin + a.slab : a.M;
    const int wk0 = (wave >> 1) * 64, wn0 = (wave & 1) * 64;
    f32x16 acc[2][2];
    zero_acc(acc);
    f32x4 rz[4], rg[4];
    auto fetch = [&](int64_t m0) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {                       // 32 x 128 floats = 1024 float4 per operand
            const int idx = tid + 256 * i;
            const int64_t m = m0 + idx / 32;
            const int c = 4 * (idx % 32);
            f32x4 vz = {0.f, 0.f, 0.f, 0.f}, vg = {0.f, 0.f, 0.f, 0.f};
            if (m < m_end) {
                if constexpr (VEC) {
                    if (k0 + c < a.K) vz = *reinterpret_cast<const f32x4*>(Z + m * a.ldz + k0 + c);
                    if (n0 + c < a.N) vg = *reinterpret_cast<const f32x4*>(G + m * a.ldg + n0 + c);
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        if (k0 + c + e < a.K) vz[e] = Z[m * a.ldz + k0 + c + e];
                        if (n0 + c + e < a.N) vg[e] = G[m * a.ldg + n0 + c + e];
                    }
                }
            }
            rz[i] = vz;
            rg[i] = vg;
        }
    };
    fetch(m_begin);
    for (int64_t m0 = m_begin; m0 < m_end; m0 += BM) {
        __syncthreads();
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int idx = tid + 256 * i;
            *reinterpret_cast<f32x4*>(&Zs[idx / 32][4 * (idx % 32)]) = rz[i];
            *reinterpret_cast<f32x4*>(&Gs[idx / 32][4 * (idx % 32)]) = rg[i];
        }
        __syncthreads();
        if (m0 + BM < m_end) fetch(m0 + BM);
#pragma unroll
        for (int mm = 0; mm < BM; mm += 2) {                // one MFMA step covers rows mm (lanes 0-31) and mm+1
            float fa[2], fb[2];
#pragma unroll
            for (int i = 0; i < 2; ++i) fa[i] = Zs[mm + lh][wk0 + 32 * i + li];
#pragma unroll
            for (int j = 0; j < 2; ++j) fb[j] = Gs[mm + lh][wn0 + 32 * j + li];
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[i], fb[j], acc[i][j], 0, 0, 0);
        }
    }
    float* out = a.partial + (int64_t)slab * a.K * a.N;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int n = n0 + wn0 + 32 * j + li;
            if (n >= a.N) continue;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int k = k0 + wk0 + 32 * i + 8 * (r / 4) + 4 * lh + (r % 4);
                if (k < a.K) out[(int64_t)k * a.N + n] = acc[i][j][r];
            }
        }
}

// bf16: both operands need 8 consecutive rows per lane, so both tiles are transposed on the way into LDS
// (the same 8 x 8 register transposition as for the weights of the forward kernel).
__global__ __launch_bounds__(256) void dw_bf16_kernel(DwArgs a) {
    __shared__ __attribute__((aligned(16))) uint16_t Zt[kDwTile][kLdh];     // [feature][row]
    __shared__ __attribute__((aligned(16))) uint16_t Gt[kDwTile][kLdh];
    const uint16_t* Z = reinterpret_cast<const uint16_t*>(a.Z);
    const uint16_t* G = reinterpret_cast<const uint16_t*>(a.G);
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, li = lane & 31, lh = lane >> 5;
    const int slab = blockIdx.x, k0 = blockIdx.y * kDwTile, n0 = blockIdx.z * kDwTile;
    const int64_t m_begin = (int64_t)slab * a.slab;
    const int64_t m_end = m_begin + a.slab < a.M ? m_begin + a.slab : a.M;
    const int wk0 = (wave >> 1) * 64, wn0 = (wave & 1) * 64;
    f32x16 acc[2][2];
    zero_acc(acc);
    // a 64(row) x 128(feature) tile is 8 x 16 blocks of 8 x 8: threads 0-127 take Z's, threads 128-255 G's
    const bool mine_z = tid < 128;
    const int t = tid & 127, rb = t / 16, fb = t % 16;
    u32x4 r[8];
    auto fetch = [&](int64_t m0) {
        const uint16_t* src = mine_z ? Z : G;
        const int64_t ld = mine_z ? a.ldz : a.ldg;
        const int f = (mine_z ? k0 : n0) + 8 * fb, flim = mine_z ? a.K : a.N;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int64_t m = m0 + 8 * rb + i;
            r[i] = u32x4{0u, 0u, 0u, 0u};
            if (m < m_end && f < flim) r[i] = *reinterpret_cast<const u32x4*>(src + m * ld + f);
        }
    };
    fetch(m_begin);
    for (int64_t m0 = m_begin; m0 < m_end; m0 += kBKh) {
        __syncthreads();
        {
            u32x4 tt[8];
            transpose8x8_bf16(r, tt);
            uint16_t (*dst)[kLdh] = mine_z ? Zt : Gt;
#pragma unroll
            for (int c = 0; c < 8; ++c) *reinterpret_cast<u32x4*>(&dst[8 * fb + c][8 * rb]) = tt[c];
        }
        __syncthreads();
        if (m0 + kBKh < m_end) fetch(m0 + kBKh);
        mfma_tile_bf16<2, 2>(&Zt[0][0], kLdh, wk0, 0, Gt, wn0, li, lh, acc);
    }
    float* out = a.partial + (int64_t)slab * a.K * a.N;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int n = n0 + wn0 + 32 * j + li;
            if (n >= a.N) continue;
#pragma unroll
            for (int rr = 0; rr < 16; ++rr) {
                const int k = k0 + wk0 + 32 * i + 8 * (rr / 4) + 4 * lh + (rr % 4);
                if (k < a.K) out[(int64_t)k * a.N + n] = acc[i][j][rr];
            }
        }
}

// bf16, both widths at most 256: one workgroup of eight wavefronts owns the whole [K][N] partial of its slab, so
// Z and G are read once (the 128 x 128 kernel above reads each of them once per tile column / row).  Wavefront
// (wk, wn) of a 4 x 2 arrangement accumulates rows 64 wk.. of dW and columns 128 wn..: eight 32 x 32 tiles.
__global__ __launch_bounds__(512) void dw_bf16_wide_kernel(DwArgs a) {
    extern __shared__ __attribute__((aligned(16))) char smem[];               // above the 64 KB static limit
    uint16_t (*Zt)[kLdh] = reinterpret_cast<uint16_t (*)[kLdh]>(smem);        // [256 features][64 rows + pad]
    uint16_t (*Gt)[kLdh] = Zt + 256;
    const uint16_t* Z = reinterpret_cast<const uint16_t*>(a.Z);
    const uint16_t* G = reinterpret_cast<const uint16_t*>(a.G);
    const int tid = threadIdx.x, lane = tid & 63, li = lane & 31, lh = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int slab = blockIdx.x;
    const int64_t m_begin = (int64_t)slab * a.slab;
    const int64_t m_end = m_begin + a.slab < a.M ? m_begin + a.slab : a.M;
    const int wk0 = (wave >> 1) * 64, wn0 = (wave & 1) * 128;
    f32x16 acc[2][4];
    zero_acc(acc);
    // a 64(row) x 256(feature) tile is 8 x 32 blocks of 8 x 8: threads 0-255 take Z's, threads 256-511 G's
    const bool mine_z = tid < 256;
    const int t = tid & 255, rb = t / 32, fb = t % 32;
    const uint16_t* src = mine_z ? Z : G;
    const int64_t ld = mine_z ? a.ldz : a.ldg;
    const int f = 8 * fb, flim = mine_z ? a.K : a.N;
    u32x4 r[8];
    auto fetch = [&](int64_t m0) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int64_t m = m0 + 8 * rb + i;
            const bool ok = m < m_end && f < flim;
            const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(ok ? src + m * ld + f : src));
            r[i] = ok ? v : u32x4{0u, 0u, 0u, 0u};
        }
    };
    fetch(m_begin);
    for (int64_t m0 = m_begin; m0 < m_end; m0 += kBKh) {
        __syncthreads();
        {
            u32x4 tt[8];
            transpose8x8_bf16(r, tt);
            uint16_t (*dst)[kLdh] = mine_z ? Zt : Gt;
#pragma unroll
            for (int c = 0; c < 8; ++c) *reinterpret_cast<u32x4*>(&dst[8 * fb + c][8 * rb]) = tt[c];
        }
        __syncthreads();
        if (m0 + kBKh < m_end) fetch(m0 + kBKh);
        mfma_tile_bf16<2, 4>(&Zt[0][0], kLdh, wk0, 0, Gt, wn0, li, lh, acc);
    }
    float* out = a.partial + (int64_t)slab * a.K * a.N;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int n = wn0 + 32 * j + li;
            if (n >= a.N) continue;
#pragma unroll
            for (int rr = 0; rr < 16; ++rr) {
                const int k = wk0 + 32 * i + 8 * (rr / 4) + 4 * lh + (rr % 4);
                if (k < a.K) out[(int64_t)k * a.N + n] = acc[i][j][rr];
            }
        }
}

// element-wise path for bf16 operands that are not 16-byte aligned: one thread per (slab, k, j)
__global__ __launch_bounds__(256) void dw_bf16_generic_kernel(DwArgs a) {
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t per = (int64_t)a.K * a.N;
    if (idx >= per * a.n_slabs) return;
    const int slab = (int)(idx / per);
    const int k = (int)((idx % per) / a.N), n = (int)(idx % a.N);
    const uint16_t* Z = reinterpret_cast<const uint16_t*>(a.Z);
    const uint16_t* G = reinterpret_cast<const uint16_t*>(a.G);
    const int64_t m_begin = (int64_t)slab * a.slab;
    const int64_t m_end = m_begin + a.slab < a.M ? m_begin + a.slab : a.M;
    float s = 0.f;
    for (int64_t m = m_begin; m < m_end; ++m) s = fmaf(bf16_val(Z, m * a.ldz + k), bf16_val(G, m * a.ldg + n), s);
    a.partial[idx] = s;
}

// dW = c_w * (sum of the slabs' partial tiles).  A workgroup owns 32 consecutive outputs; eight threads per output
// each add every eighth slab in slab order, four loads in flight, and the eight sums are added in a fixed order.
constexpr int kDwReduceOut = 32, kDwReduceWays = 8;
__global__ __launch_bounds__(256) void dw_reduce_kernel(DwArgs a) {
    __shared__ float part[kDwReduceWays][kDwReduceOut];
    const int o = threadIdx.x % kDwReduceOut, way = threadIdx.x / kDwReduceOut;
    const int64_t idx = (int64_t)blockIdx.x * kDwReduceOut + o;
    const int64_t per = (int64_t)a.K * a.N;
    float s = 0.f;
    if (idx < per) {
        const float* p = a.partial + idx;
        int sl = way;
        for (; sl + 3 * kDwReduceWays < a.n_slabs; sl += 4 * kDwReduceWays) {
            const float v0 = p[(int64_t)sl * per], v1 = p[(int64_t)(sl + kDwReduceWays) * per],
                        v2 = p[(int64_t)(sl + 2 * kDwReduceWays) * per], v3 = p[(int64_t)(sl + 3 * kDwReduceWays) * per];
            s = ((s + v0) + v1) + v2 + v3;
        }
        for (; sl < a.n_slabs; sl += kDwReduceWays) s += p[(int64_t)sl * per];
    }
    part[way][o] = s;
    __syncthreads();
    if (way == 0 && idx < per) {
        float t = part[0][o];
#pragma unroll
        for (int w = 1; w < kDwReduceWays; ++w) t += part[w][o];
        a.dW[idx] = a.c_w * t;
    }
}

// ReLU backward, element-wise: GP = GY where Y > 0, else 0
template <bool BF>
__global__ __launch_bounds__(256) void relu_bwd_kernel(const char* GY, int64_t ldgy, const char* Y, int64_t ldy,
                                                       char* GP, int64_t ldgp, int64_t M, int F, int vec) {
    // vec: 16-byte pieces per row (0 = element-wise)
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    constexpr int EB = BF ? 2 : 4;
    if (vec > 0) {
        if (idx >= M * vec) return;
        const int64_t m = idx / vec;
        const int v = (int)(idx % vec);
        const u32x4 g = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(GY + (m * ldgy) * EB) + v);
        const u32x4 y = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(Y + (m * ldy) * EB) + v);
        u32x4 o = g;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            if constexpr (BF) {
                if (!(bf16_lo(y[q]) > 0.f)) o[q] &= 0xFFFF0000u;
                if (!(bf16_hi(y[q]) > 0.f)) o[q] &= 0x0000FFFFu;
            } else {
                if (!(__uint_as_float(y[q]) > 0.f)) o[q] = 0u;
            }
        }
        __builtin_nontemporal_store(o, reinterpret_cast<u32x4*>(GP + (m * ldgp) * EB) + v);
    } else {
        if (idx >= M * F) return;
        const int64_t m = idx / F;
        const int f = (int)(idx % F);
        if constexpr (BF) {
            const uint16_t* y = reinterpret_cast<const uint16_t*>(Y);
            const uint16_t g = reinterpret_cast<const uint16_t*>(GY)[m * ldgy + f];
            reinterpret_cast<uint16_t*>(GP)[m * ldgp + f] = bf16_val(y, m * ldy + f) > 0.f ? g : (uint16_t)0;
        } else {
            const float g = reinterpret_cast<const float*>(GY)[m * ldgy + f];
            reinterpret_cast<float*>(GP)[m * ldgp + f] = reinterpret_cast<const float*>(Y)[m * ldy + f] > 0.f ? g : 0.f;
        }
    }
}

// ====================================================================== launchers
template <int BM, int BN>
gas_status launch_f32(const LinArgs& a, bool vec, hipStream_t s) {
    const int64_t gm = (a.M + BM - 1) / BM;
    const int gn = (a.N + BN - 1) / BN;
    if (gm > 0x7FFFFFFF || gn > 65535) return fail(GAS_ERR_ARG, "gas_linear: problem too large for one launch");
    dim3 grid((unsigned)gm, (unsigned)gn), block(256);
    if (a.trans_w) {
        if (vec) hipLaunchKernelGGL((linear_f32_kernel<BM, BN, true, true>), grid, block, 0, s, a);
        else hipLaunchKernelGGL((linear_f32_kernel<BM, BN, false, true>), grid, block, 0, s, a);
    } else {
        if (vec) hipLaunchKernelGGL((linear_f32_kernel<BM, BN, true, false>), grid, block, 0, s, a);
        else hipLaunchKernelGGL((linear_f32_kernel<BM, BN, false, false>), grid, block, 0, s, a);
    }
    GAS_CHECK_HIP(hipGetLastError());
    return GAS_OK;
}

template <int BN>
gas_status launch_bf16(const LinArgs& a, hipStream_t s) {
    const int64_t gm = (a.M + 127) / 128;
    const int gn = (a.N + BN - 1) / BN;
    if (gm > 0x7FFFFFFF || gn > 65535) return fail(GAS_ERR_ARG, "gas_linear: problem too large for one launch");
    hipLaunchKernelGGL((linear_bf16_kernel<BN>), dim3((unsigned)gm, (unsigned)gn), dim3(256), 0, s, a);
    GAS_CHECK_HIP(hipGetLastError());
    return GAS_OK;
}

}  // namespace
}  // namespace gas

using namespace gas;

extern "C" {

// Y = act(c_identity * Z + c_weight * (Z op(W)) + bias) with optional output mask; op(W) = W ([F_in, F_out]) or,
// with trans_w, the transpose of a [F_out, F_in] matrix.
struct PushTarget {                 // optional fused Push: output row i also goes to hist[idx[i], :]
    const int32_t* idx = nullptr;
    void* hist = nullptr;
    int64_t n_hist_rows = 0, ld_hist = 0;
};

// rows the kernel did not scatter itself are pushed by the row-copy kernel
static gas_status push_after(const PushTarget& p, const void* Y, int64_t ldy, int64_t n_rows, int32_t F, gas_dtype dt,
                             hipStream_t s) {
    if (!p.idx) return GAS_OK;
    return gas_push(Y, ldy, p.idx, 0, n_rows, F, dt, p.hist, p.n_hist_rows, p.ld_hist, s);
}

static gas_status run_linear(const char* who, const void* Z, int64_t ldz, int64_t n_rows, int32_t F_in, const void* W,
                             int trans_w, int32_t F_out, const void* bias, gas_dtype dt, float c_identity,
                             float c_weight, int relu, const void* mask, int64_t ldmask, void* Y, int64_t ldy,
                             hipStream_t s, const PushTarget& push = PushTarget()) {
    if (push.idx) {
        GAS_REQUIRE(push.hist && push.ld_hist >= F_out && push.n_hist_rows > 0, "%s: bad history table for the fused push", who);
        GAS_REQUIRE(push.hist != Y, "%s: the history table aliases the output", who);
    }
    if (!valid_dtype(dt)) return fail(GAS_ERR_DTYPE, "%s: unknown dtype %d", who, (int)dt);
    GAS_REQUIRE(n_rows >= 0 && F_in > 0 && F_out > 0, "%s: n_rows=%lld widths %d, %d", who, (long long)n_rows, F_in, F_out);
    if (n_rows == 0) return GAS_OK;
    GAS_REQUIRE(Z && W && Y, "%s: null pointer", who);
    GAS_REQUIRE(ldz >= F_in && ldy >= F_out && (!mask || ldmask >= F_out), "%s: row stride smaller than the row", who);
    GAS_REQUIRE(c_identity == 0.f || F_in == F_out, "%s: the identity term needs equal widths", who);
    GAS_REQUIRE(Y != Z, "%s: the output must not alias the input", who);
    LinArgs a;
    a.Z = static_cast<const char*>(Z); a.ldz = ldz;
    a.W = static_cast<const char*>(W);
    a.bias = static_cast<const char*>(bias);
    a.Y = static_cast<char*>(Y); a.ldy = ldy;
    a.M = n_rows; a.K = F_in; a.N = F_out;
    a.c_id = c_identity; a.c_w = c_weight; a.relu = relu;
    a.trans_w = trans_w; a.mask = static_cast<const char*>(mask); a.ldmask = ldmask;
    if (dt == GAS_F32) {
        const bool vec = aligned16(Z) && aligned16(W) && ldz % 4 == 0 && F_in % 4 == 0 && F_out % 4 == 0;
        a.push_idx = push.idx; a.push_hist = static_cast<char*>(push.hist); a.ld_push = push.ld_hist;
        // a small batch in 128-row tiles would leave most compute units without a workgroup: 64 x 64 tiles then
        // (the same products in the same order, so the same bits)
        const int64_t tiles128 = ((n_rows + 127) / 128) * ((F_out + (F_out <= 64 ? 63 : 127)) / (F_out <= 64 ? 64 : 128));
        if (tiles128 < 512) return launch_f32<64, 64>(a, vec, s);
        return F_out <= 64 ? launch_f32<128, 64>(a, vec, s) : launch_f32<128, 128>(a, vec, s);
    }
    const bool vec = aligned16(Z) && aligned16(W) && ldz % 8 == 0 && F_in % 8 == 0 && F_out % 8 == 0;
    if (!vec) {
        const int64_t total = n_rows * (int64_t)F_out;
        const int64_t blocks = (total + 255) / 256;
        if (blocks > 0x7FFFFFFFLL) return fail(GAS_ERR_ARG, "%s: problem too large for the element-wise path", who);
        hipLaunchKernelGGL(linear_bf16_generic_kernel, dim3((unsigned)blocks), dim3(256), 0, s, a);
        GAS_CHECK_HIP(hipGetLastError());
        return push_after(push, Y, ldy, n_rows, F_out, dt, s);
    }
    if (F_in <= 256 && F_out <= 256 && aligned16(Y) && ldy % 8 == 0 && n_rows >= 4096 &&
        (!mask || (aligned16(mask) && ldmask % 8 == 0)) && ldz < (1 << 24) && ldy < (1 << 24) && ldmask < (1 << 24)) {
        const bool scatter = push.idx && aligned16(push.hist) && push.ld_hist % 8 == 0;
        WsArgs w{};
        w.Z = static_cast<const uint16_t*>(Z); w.ldz = ldz;
        w.W1 = static_cast<const uint16_t*>(W); w.b1 = static_cast<const uint16_t*>(bias);
        w.Y = static_cast<uint16_t*>(Y); w.ldy = ldy;
        w.M = n_rows; w.n_tiles = (n_rows + kWsRows - 1) / kWsRows;
        w.K = F_in; w.H = F_out; w.N = F_out;
        w.c_id = c_identity; w.c_w = c_weight; w.relu1 = relu; w.relu_out = 0;
        w.trans_w1 = trans_w; w.mask = static_cast<const uint16_t*>(mask); w.ldmask = ldmask;
        if (scatter) { w.push_idx = push.idx; w.push_hist = static_cast<uint16_t*>(push.hist); w.ld_push = push.ld_hist; }
        const gas_status st = F_in <= 64 ? launch_ws<4>(w, s) : (F_in <= 128 ? launch_ws<8>(w, s) : launch_ws<16>(w, s));
        return (st != GAS_OK || scatter) ? st : push_after(push, Y, ldy, n_rows, F_out, dt, s);
    }
    const gas_status st = F_out <= 64 ? launch_bf16<64>(a, s) : (F_out <= 128 ? launch_bf16<128>(a, s) : launch_bf16<256>(a, s));
    return st != GAS_OK ? st : push_after(push, Y, ldy, n_rows, F_out, dt, s);
}

gas_status gas_linear_push(const void* Z, int64_t ldz, int64_t n_rows, int32_t F_in, const void* W, int32_t F_out,
                           const void* bias, gas_dtype dt, float c_identity, float c_weight, int relu, void* Y,
                           int64_t ldy, const int32_t* idx, void* hist, int64_t n_hist_rows, int64_t ld_hist,
                           void* stream) {
    GAS_REQUIRE(idx || n_rows == 0, "gas_linear_push: null index array");
    PushTarget p;
    p.idx = idx; p.hist = hist; p.n_hist_rows = n_hist_rows; p.ld_hist = ld_hist;
    return run_linear("gas_linear_push", Z, ldz, n_rows, F_in, W, 0, F_out, bias, dt, c_identity, c_weight, relu,
                      nullptr, 0, Y, ldy, (hipStream_t)stream, p);
}

gas_status gas_linear(const void* Z, int64_t ldz, int64_t n_rows, int32_t F_in, const void* W, int32_t F_out,
                      const void* bias, gas_dtype dt, float c_identity, float c_weight, int relu, void* Y,
                      int64_t ldy, void* stream) {
    return run_linear("gas_linear", Z, ldz, n_rows, F_in, W, 0, F_out, bias, dt, c_identity, c_weight, relu, nullptr,
                      0, Y, ldy, (hipStream_t)stream);
}

gas_status gas_linear_bwd_input(const void* GP, int64_t ldgp, int64_t n_rows, int32_t F_out, const void* W,
                                int32_t F_in, gas_dtype dt, float c_identity, float c_weight, const void* mask,
                                int64_t ldmask, void* GZ, int64_t ldgz, void* stream) {
    // GZ = c_identity * GP + c_weight * (GP W^T): a product with the [F_in, F_out] matrix taken transposed
    return run_linear("gas_linear_bwd_input", GP, ldgp, n_rows, F_out, W, 1, F_in, nullptr, dt, c_identity, c_weight,
                      0, mask, ldmask, GZ, ldgz, (hipStream_t)stream);
}

int64_t gas_linear_bwd_weight_workspace(int64_t n_rows, int32_t F_in, int32_t F_out) {
    if (n_rows <= 0 || F_in <= 0 || F_out <= 0) return 0;
    const int64_t slab = dw_slab_rows(n_rows, F_in, F_out);
    return ((n_rows + slab - 1) / slab) * (int64_t)F_in * F_out * (int64_t)sizeof(float);
}

// Weight gradient with the slab partials in `workspace` (the caller's, or the library's static array).
static gas_status run_dw(const void* Z, int64_t ldz, const void* GP, int64_t ldgp, int64_t n_rows,
                         int32_t F_in, int32_t F_out, gas_dtype dt, float c_weight, float* dW,
                         void* workspace, int64_t workspace_bytes, bool static_scratch, void* stream) {
    if (!valid_dtype(dt)) return fail(GAS_ERR_DTYPE, "gas_linear_bwd_weight: unknown dtype %d", (int)dt);
    GAS_REQUIRE(n_rows >= 0 && F_in > 0 && F_out > 0, "gas_linear_bwd_weight: n_rows=%lld widths %d, %d",
                (long long)n_rows, F_in, F_out);
    GAS_REQUIRE(dW, "gas_linear_bwd_weight: null output");
    hipStream_t s = (hipStream_t)stream;
    DwArgs a;
    a.Z = static_cast<const char*>(Z); a.ldz = ldz;
    a.G = static_cast<const char*>(GP); a.ldg = ldgp;
    a.M = n_rows; a.K = F_in; a.N = F_out; a.c_w = c_weight;
    a.partial = static_cast<float*>(workspace); a.dW = dW;
    a.slab = (int)dw_slab_rows(n_rows, F_in, F_out);
    const int64_t n_slabs = (n_rows + a.slab - 1) / a.slab;
    GAS_REQUIRE(n_slabs <= 0x7FFFFFFFLL, "gas_linear_bwd_weight: too many rows");
    a.n_slabs = (int)n_slabs;
    const int64_t per = (int64_t)F_in * F_out;
    const unsigned rblocks = (unsigned)((per + kDwReduceOut - 1) / kDwReduceOut);
    if (n_rows == 0) {                                   // empty sum: dW = 0
        hipLaunchKernelGGL(dw_reduce_kernel, dim3(rblocks), dim3(256), 0, s, a);
        GAS_CHECK_HIP(hipGetLastError());
        return GAS_OK;
    }
    GAS_REQUIRE(Z && GP, "gas_linear_bwd_weight: null pointer");
    GAS_REQUIRE(ldz >= F_in && ldgp >= F_out, "gas_linear_bwd_weight: row stride smaller than the row");
    if (static_scratch) {
        const int64_t need = gas_linear_bwd_weight_workspace(n_rows, F_in, F_out);
        if (need > kDwScratchBytes)
            return fail(GAS_ERR_ARG, "gas_linear_bwd_weight_static: the slab partials of this shape take %lld bytes, "
                        "the library's static scratch array holds %lld; use gas_linear_bwd_weight with a workspace",
                        (long long)need, (long long)kDwScratchBytes);
        const gas_status st = dw_scratch_pointer(&workspace);
        if (st != GAS_OK) return st;
        workspace_bytes = kDwScratchBytes;
        a.partial = static_cast<float*>(workspace);
    }
    GAS_REQUIRE(workspace && workspace_bytes >= gas_linear_bwd_weight_workspace(n_rows, F_in, F_out),
                "gas_linear_bwd_weight: workspace of %lld bytes needed, %lld given",
                (long long)gas_linear_bwd_weight_workspace(n_rows, F_in, F_out), (long long)workspace_bytes);
    const unsigned tk = (unsigned)((F_in + kDwTile - 1) / kDwTile), tn = (unsigned)((F_out + kDwTile - 1) / kDwTile);
    GAS_REQUIRE(tk <= 65535 && tn <= 65535, "gas_linear_bwd_weight: widths too large");
    dim3 grid((unsigned)n_slabs, tk, tn);
    if (dt == GAS_F32) {
        const bool vec = aligned16(Z) && aligned16(GP) && ldz % 4 == 0 && ldgp % 4 == 0;
        if (vec) hipLaunchKernelGGL(dw_f32_kernel<true>, grid, dim3(256), 0, s, a);
        else hipLaunchKernelGGL(dw_f32_kernel<false>, grid, dim3(256), 0, s, a);
    } else {
        const bool vec = aligned16(Z) && aligned16(GP) && ldz % 8 == 0 && ldgp % 8 == 0 && F_in % 8 == 0 && F_out % 8 == 0;
        if (vec && F_in <= 256 && F_out <= 256 && F_in > 128 && F_out > 128) {
            constexpr int smem = 2 * 256 * kLdh * 2;
            static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(dw_bf16_wide_kernel),
                                                               hipFuncAttributeMaxDynamicSharedMemorySize, smem);
            GAS_CHECK_HIP(attr);
            hipLaunchKernelGGL(dw_bf16_wide_kernel, dim3((unsigned)n_slabs), dim3(512), smem, s, a);
        } else if (vec) {
            hipLaunchKernelGGL(dw_bf16_kernel, grid, dim3(256), 0, s, a);
        } else {
            const int64_t blocks = (per * n_slabs + 255) / 256;
            GAS_REQUIRE(blocks <= 0x7FFFFFFFLL, "gas_linear_bwd_weight: problem too large for the element-wise path");
            hipLaunchKernelGGL(dw_bf16_generic_kernel, dim3((unsigned)blocks), dim3(256), 0, s, a);
        }
    }
    hipLaunchKernelGGL(dw_reduce_kernel, dim3(rblocks), dim3(256), 0, s, a);
    GAS_CHECK_HIP(hipGetLastError());
    return GAS_OK;
}

gas_status gas_linear_bwd_weight(const void* Z, int64_t ldz, const void* GP, int64_t ldgp, int64_t n_rows,
                                 int32_t F_in, int32_t F_out, gas_dtype dt, float c_weight, float* dW,
                                 void* workspace, int64_t workspace_bytes, void* stream) {
    return run_dw(Z, ldz, GP, ldgp, n_rows, F_in, F_out, dt, c_weight, dW, workspace, workspace_bytes, false, stream);
}

gas_status gas_linear_bwd_weight_static(const void* Z, int64_t ldz, const void* GP, int64_t ldgp, int64_t n_rows,
                                        int32_t F_in, int32_t F_out, gas_dtype dt, float c_weight, float* dW,
                                        void* stream) {
    return run_dw(Z, ldz, GP, ldgp, n_rows, F_in, F_out, dt, c_weight, dW, nullptr, 0, true, stream);
}

gas_status gas_relu_bwd(const void* GY, int64_t ldgy, const void* Y, int64_t ldy, int64_t n_rows, int32_t F,
                        gas_dtype dt, void* GP, int64_t ldgp, void* stream) {
    if (!valid_dtype(dt)) return fail(GAS_ERR_DTYPE, "gas_relu_bwd: unknown dtype %d", (int)dt);
    GAS_REQUIRE(n_rows >= 0 && F > 0, "gas_relu_bwd: n_rows=%lld F=%d", (long long)n_rows, F);
    if (n_rows == 0) return GAS_OK;
    GAS_REQUIRE(GY && Y && GP, "gas_relu_bwd: null pointer");
    GAS_REQUIRE(ldgy >= F && ldy >= F && ldgp >= F, "gas_relu_bwd: row stride smaller than F");
    const int eb = elem_bytes(dt);
    const bool vec = aligned16(GY) && aligned16(Y) && aligned16(GP) && (F * eb) % 16 == 0 && (ldgy * eb) % 16 == 0 &&
                     (ldy * eb) % 16 == 0 && (ldgp * eb) % 16 == 0;
    const int v = vec ? F * eb / 16 : 0;
    const int64_t items = vec ? n_rows * v : n_rows * (int64_t)F;
    const int64_t blocks = (items + 255) / 256;
    GAS_REQUIRE(blocks <= 0x7FFFFFFFLL, "gas_relu_bwd: too many elements for one launch");
    const char* gy = static_cast<const char*>(GY);
    const char* y = static_cast<const char*>(Y);
    char* gp = static_cast<char*>(GP);
    if (dt == GAS_BF16)
        hipLaunchKernelGGL(relu_bwd_kernel<true>, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream, gy, ldgy, y,
                           ldy, gp, ldgp, n_rows, F, v);
    else
        hipLaunchKernelGGL(relu_bwd_kernel<false>, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream, gy, ldgy,
                           y, ldy, gp, ldgp, n_rows, F, v);
    GAS_CHECK_HIP(hipGetLastError());
    return GAS_OK;
}

static gas_status run_mlp2(const void* Z, int64_t ldz, int64_t n_rows, int32_t F_in, const void* W1, int32_t F_hid,
                           const void* b1, const void* W2, int32_t F_out, const void* b2, gas_dtype dt, int relu_out,
                           void* Y, int64_t ldy, void* stream, const PushTarget& push, void* H_out = nullptr,
                           int64_t ldh_out = 0) {
    if (!valid_dtype(dt)) return fail(GAS_ERR_DTYPE, "gas_mlp2: unknown dtype %d", (int)dt);
    GAS_REQUIRE(!H_out || ldh_out >= F_hid, "gas_mlp2_keep: row stride of the hidden activation smaller than F_hid");
    GAS_REQUIRE(!H_out || (H_out != Y && H_out != Z), "gas_mlp2_keep: the hidden activation aliases Z or Y");
    if (push.idx) {
        GAS_REQUIRE(push.hist && push.ld_hist >= F_out && push.n_hist_rows > 0, "gas_mlp2_push: bad history table");
        GAS_REQUIRE(push.hist != Y, "gas_mlp2_push: the history table aliases the output");
    }
    GAS_REQUIRE(n_rows >= 0 && F_in > 0 && F_hid > 0 && F_out > 0, "gas_mlp2: n_rows=%lld F_in=%d F_hid=%d F_out=%d",
                (long long)n_rows, F_in, F_hid, F_out);
    GAS_REQUIRE(F_hid <= kHidMax, "gas_mlp2: F_hid=%d exceeds %d", F_hid, kHidMax);
    if (n_rows == 0) return GAS_OK;
    GAS_REQUIRE(Z && W1 && W2 && Y, "gas_mlp2: null pointer");
    GAS_REQUIRE(ldz >= F_in && ldy >= F_out, "gas_mlp2: row stride smaller than the row");
    GAS_REQUIRE(Y != Z, "gas_mlp2: Y must not alias Z");
    MlpArgs a;
    a.Z = static_cast<const char*>(Z); a.ldz = ldz;
    a.W1 = static_cast<const char*>(W1); a.b1 = static_cast<const char*>(b1);
    a.W2 = static_cast<const char*>(W2); a.b2 = static_cast<const char*>(b2);
    a.Y = static_cast<char*>(Y); a.ldy = ldy;
    a.M = n_rows; a.K = F_in; a.H = F_hid; a.N = F_out;
    a.relu_out = relu_out;
    hipStream_t s = (hipStream_t)stream;
    const int q = dt == GAS_F32 ? 4 : 8;    // elements per 16 bytes
    const bool vec = aligned16(Z) && aligned16(W1) && aligned16(W2) && ldz % q == 0 && F_in % q == 0 &&
                     F_hid % q == 0 && F_out % q == 0;
    const bool ws_path = dt == GAS_BF16 && vec && F_in <= 256 && F_out <= 256 && aligned16(Y) && ldy % 8 == 0 &&
                         n_rows >= 4096 && ldz < (1 << 24) && ldy < (1 << 24) && H_out && aligned16(H_out) &&
                         ldh_out % 8 == 0 && ldh_out < (1 << 24);
    if (H_out && !ws_path) {
        // only the weights-stationary kernel stores the hidden activation on its way: elsewhere two stored linears
        gas_status st = run_linear("gas_mlp2_keep", Z, ldz, n_rows, F_in, W1, 0, F_hid, b1, dt, 0.f, 1.f, 1, nullptr, 0,
                                   H_out, ldh_out, s);
        if (st != GAS_OK) return st;
        return run_linear("gas_mlp2_keep", H_out, ldh_out, n_rows, F_hid, W2, 0, F_out, b2, dt, 0.f, 1.f, relu_out,
                          nullptr, 0, Y, ldy, s, push);
    }
    const int gn = (F_out + 255) / 256;
    if (n_rows > 0x7FFFFFFFLL || gn > 65535) return fail(GAS_ERR_ARG, "gas_mlp2: problem too large for one launch");
    if (dt == GAS_F32) {
        constexpr int smem = 4 * (kMlpRowsF32 * (kHidMax + 4 + kBK + 4) + kBK * (256 + 4));
        static const hipError_t e1 = hipFuncSetAttribute(reinterpret_cast<const void*>(mlp2_f32_kernel<true>),
                                                         hipFuncAttributeMaxDynamicSharedMemorySize, smem);
        static const hipError_t e2 = hipFuncSetAttribute(reinterpret_cast<const void*>(mlp2_f32_kernel<false>),
                                                         hipFuncAttributeMaxDynamicSharedMemorySize, smem);
        GAS_CHECK_HIP(e1);
        GAS_CHECK_HIP(e2);
        dim3 grid((unsigned)((n_rows + kMlpRowsF32 - 1) / kMlpRowsF32), (unsigned)gn);
        if (vec) hipLaunchKernelGGL(mlp2_f32_kernel<true>, grid, dim3(256), smem, s, a);
        else hipLaunchKernelGGL(mlp2_f32_kernel<false>, grid, dim3(256), smem, s, a);
    } else if (vec && F_in <= 256 && F_out <= 256 && aligned16(Y) && ldy % 8 == 0 && n_rows >= 4096 &&
               ldz < (1 << 24) && ldy < (1 << 24) &&      // offsets inside a 64-row tile are 32-bit
               (!H_out || (aligned16(H_out) && ldh_out % 8 == 0 && ldh_out < (1 << 24)))) {
        // the kernel scatters the rows itself if the history rows take 16-byte stores; else the row copy follows
        const bool scatter = push.idx && aligned16(push.hist) && push.ld_hist % 8 == 0;
        WsArgs w{};
        w.Z = static_cast<const uint16_t*>(Z); w.ldz = ldz;
        w.W1 = static_cast<const uint16_t*>(W1); w.b1 = static_cast<const uint16_t*>(b1);
        w.W2 = static_cast<const uint16_t*>(W2); w.b2 = static_cast<const uint16_t*>(b2);
        w.Y = static_cast<uint16_t*>(Y); w.ldy = ldy;
        w.M = n_rows; w.n_tiles = (n_rows + kWsRows - 1) / kWsRows;
        w.K = F_in; w.H = F_hid; w.N = F_out;
        w.c_id = 0.f; w.c_w = 1.f; w.relu1 = 1; w.relu_out = relu_out;
        if (scatter) { w.push_idx = push.idx; w.push_hist = static_cast<uint16_t*>(push.hist); w.ld_push = push.ld_hist; }
        w.H_out = static_cast<uint16_t*>(H_out); w.ldh_out = ldh_out;
        const gas_status st = F_in <= 128 ? launch_ws_mlp<8, 16>(w, s) : launch_ws_mlp<16, 16>(w, s);
        return (st != GAS_OK || scatter) ? st : push_after(push, Y, ldy, n_rows, F_out, dt, s);
    } else if (vec) {
        constexpr int smem = 2 * (kMlpRowsBF16 * (kHidMax + 8 + kBKh + 8) + 256 * (kBKh + 8));
        static const hipError_t e1 = hipFuncSetAttribute(reinterpret_cast<const void*>(mlp2_bf16_kernel),
                                                         hipFuncAttributeMaxDynamicSharedMemorySize, smem);
        GAS_CHECK_HIP(e1);
        hipLaunchKernelGGL(mlp2_bf16_kernel, dim3((unsigned)((n_rows + kMlpRowsBF16 - 1) / kMlpRowsBF16), (unsigned)gn),
                           dim3(256), smem, s, a);
    } else {
        hipLaunchKernelGGL(mlp2_generic_kernel<true>, dim3((unsigned)n_rows), dim3(256), 0, s, a);
    }
    GAS_CHECK_HIP(hipGetLastError());
    return push_after(push, Y, ldy, n_rows, F_out, dt, s);
}

gas_status gas_mlp2(const void* Z, int64_t ldz, int64_t n_rows, int32_t F_in, const void* W1, int32_t F_hid,
                    const void* b1, const void* W2, int32_t F_out, const void* b2, gas_dtype dt, int relu_out,
                    void* Y, int64_t ldy, void* stream) {
    return run_mlp2(Z, ldz, n_rows, F_in, W1, F_hid, b1, W2, F_out, b2, dt, relu_out, Y, ldy, stream, PushTarget());
}

gas_status gas_mlp2_push(const void* Z, int64_t ldz, int64_t n_rows, int32_t F_in, const void* W1, int32_t F_hid,
                         const void* b1, const void* W2, int32_t F_out, const void* b2, gas_dtype dt, int relu_out,
                         void* Y, int64_t ldy, const int32_t* idx, void* hist, int64_t n_hist_rows, int64_t ld_hist,
                         void* stream) {
    GAS_REQUIRE(idx || n_rows == 0, "gas_mlp2_push: null index array");
    PushTarget p;
    p.idx = idx; p.hist = hist; p.n_hist_rows = n_hist_rows; p.ld_hist = ld_hist;
    return run_mlp2(Z, ldz, n_rows, F_in, W1, F_hid, b1, W2, F_out, b2, dt, relu_out, Y, ldy, stream, p);
}

gas_status gas_mlp2_keep(const void* Z, int64_t ldz, int64_t n_rows, int32_t F_in, const void* W1, int32_t F_hid,
                         const void* b1, const void* W2, int32_t F_out, const void* b2, gas_dtype dt, int relu_out,
                         void* Y, int64_t ldy, void* H_out, int64_t ldh_out, const int32_t* idx, void* hist,
                         int64_t n_hist_rows, int64_t ld_hist, void* stream) {
    GAS_REQUIRE(H_out || n_rows == 0, "gas_mlp2_keep: null hidden activation");
    GAS_REQUIRE((idx == nullptr) == (hist == nullptr), "gas_mlp2_keep: idx and hist go together");
    PushTarget p;
    p.idx = idx; p.hist = hist; p.n_hist_rows = n_hist_rows; p.ld_hist = ld_hist;
    return run_mlp2(Z, ldz, n_rows, F_in, W1, F_hid, b1, W2, F_out, b2, dt, relu_out, Y, ldy, stream, p, H_out, ldh_out);
}

}  // extern "C"
