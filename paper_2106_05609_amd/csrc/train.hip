// Loss and parameter update that close the loop body of Algorithm 1: softmax cross-entropy over the labelled
// in-batch rows (the mini-batch loss of Section 1) and a gradient-descent step with L2 weight decay (Section 3).
// Both are element-/row-wise and HBM-bound; no atomics, the loss is summed in a fixed order.
#include "common.h"

namespace gas {
namespace {

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
    return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
}

template <bool BF>
__device__ __forceinline__ float load_logit(const char* p, int64_t i) {
    if constexpr (BF) return __uint_as_float((uint32_t)reinterpret_cast<const uint16_t*>(p)[i] << 16);
    else return reinterpret_cast<const float*>(p)[i];
}

// one wavefront per row: three passes over the row's logits (max, sum of exponentials, gradient), the second
// and third served by the cache
template <bool BF>
__global__ __launch_bounds__(256) void softmax_xent_kernel(const char* A, int64_t lda, int64_t M, int C,
                                                           const int32_t* labels, float scale, float* loss_rows,
                                                           char* G, int64_t ldg) {
    const int lane = threadIdx.x & 63;
    const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= M) return;
    const int y = labels[row];
    const int64_t a0 = row * lda, g0 = row * ldg;
    if (y < 0 || y >= C) {                              // unlabelled: no loss, no gradient
        if (lane == 0) loss_rows[row] = 0.f;
        for (int c = lane; c < C; c += 64) {
            if constexpr (BF) reinterpret_cast<uint16_t*>(G)[g0 + c] = 0;
            else reinterpret_cast<float*>(G)[g0 + c] = 0.f;
        }
        return;
    }
    float mx = -INFINITY;
    for (int c = lane; c < C; c += 64) mx = fmaxf(mx, load_logit<BF>(A, a0 + c));
    mx = wave_max(mx);
    float den = 0.f;
    for (int c = lane; c < C; c += 64) den += expf(load_logit<BF>(A, a0 + c) - mx);
    den = wave_sum(den);
    if (lane == 0) loss_rows[row] = -(load_logit<BF>(A, a0 + y) - mx - logf(den));
    const float inv = 1.f / den;
    for (int c = lane; c < C; c += 64) {
        const float p = expf(load_logit<BF>(A, a0 + c) - mx) * inv;
        const float g = scale * (p - (c == y ? 1.f : 0.f));
        if constexpr (BF) reinterpret_cast<uint16_t*>(G)[g0 + c] = (uint16_t)f32_to_bf16(g);
        else reinterpret_cast<float*>(G)[g0 + c] = g;
    }
}

// Rows of at most 64 vectors of 16 bytes (512 bf16 or 256 fp32 classes), 16-byte aligned: a team of
// 2^lpr_log2 lanes holds a whole row in registers (one vector per lane), so the logits are read once, the
// exponentials are computed once and serve the loss and the gradient, and a wavefront takes 64 / team rows.
template <bool BF>
__global__ __launch_bounds__(256) void softmax_xent_rows_kernel(const char* A, int64_t lda, int64_t M, int C,
                                                                const int32_t* labels, float scale, float* loss_rows,
                                                                char* G, int64_t ldg, int lpr_log2) {
    constexpr int EPV = BF ? 8 : 4;
    constexpr int EB = BF ? 2 : 4;
    const int lane = threadIdx.x & 63;
    const int lpr = 1 << lpr_log2, rpw = 64 >> lpr_log2;
    const int64_t row = ((int64_t)blockIdx.x * 4 + (threadIdx.x >> 6)) * rpw + (lane >> lpr_log2);
    const int c0 = (lane & (lpr - 1)) * EPV;
    const bool active = row < M && c0 < C;
    float x[EPV];
    u32x4 raw = {0u, 0u, 0u, 0u};
    if (active) raw = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(A + (row * lda + c0) * EB));
#pragma unroll
    for (int i = 0; i < EPV; ++i) {
        if constexpr (BF) x[i] = (i & 1) ? bf16_hi(raw[i >> 1]) : bf16_lo(raw[i >> 1]);
        else x[i] = __uint_as_float(raw[i]);
        if (!active) x[i] = -INFINITY;
    }
    float mx = x[0];
#pragma unroll
    for (int i = 1; i < EPV; ++i) mx = fmaxf(mx, x[i]);
    for (int o = lpr >> 1; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o));
    float e[EPV], den = 0.f;
#pragma unroll
    for (int i = 0; i < EPV; ++i) {
        e[i] = active ? expf(x[i] - mx) : 0.f;
        den += e[i];
    }
    for (int o = lpr >> 1; o > 0; o >>= 1) den += __shfl_xor(den, o);
    if (!active) return;
    const int y = labels[row];
    const bool labelled = y >= 0 && y < C;
    const float inv = labelled ? scale / den : 0.f;
    float g[EPV];
#pragma unroll
    for (int i = 0; i < EPV; ++i) {
        g[i] = e[i] * inv;
        if (labelled && c0 + i == y) {
            g[i] -= scale;
            loss_rows[row] = -(x[i] - mx - logf(den));
        }
    }
    if (!labelled && c0 == 0) loss_rows[row] = 0.f;
    u32x4 out;
    if constexpr (BF) out = u32x4{pack_bf16(g[0], g[1]), pack_bf16(g[2], g[3]), pack_bf16(g[4], g[5]), pack_bf16(g[6], g[7])};
    else out = u32x4{__float_as_uint(g[0]), __float_as_uint(g[1]), __float_as_uint(g[2]), __float_as_uint(g[3])};
    __builtin_nontemporal_store(out, reinterpret_cast<u32x4*>(G + (row * ldg + c0) * EB));
}

// sum of n floats in a fixed order: thread t adds elements t, t+1024, ... in double (eight loads in flight),
// then a tree over the block
__global__ __launch_bounds__(1024) void sum_fixed_kernel(const float* x, int64_t n, float* out) {
    __shared__ double part[1024];
    double s = 0.0;
    int64_t i = threadIdx.x;
    for (; i + 7 * 1024 < n; i += 8 * 1024) {
        float v[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) v[j] = x[i + 1024 * j];
#pragma unroll
        for (int j = 0; j < 8; ++j) s += (double)v[j];
    }
    for (; i < n; i += 1024) s += (double)x[i];
    part[threadIdx.x] = s;
    __syncthreads();
    for (int w = 512; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w) part[threadIdx.x] += part[threadIdx.x + w];
        __syncthreads();
    }
    if (threadIdx.x == 0) out[0] = (float)part[0];
}

// sum of the squares of n floats, same order and precision as sum_fixed_kernel
__global__ __launch_bounds__(1024) void sq_sum_fixed_kernel(const float* x, int64_t n, float* out) {
    __shared__ double part[1024];
    double s = 0.0;
    int64_t i = threadIdx.x;
    for (; i + 7 * 1024 < n; i += 8 * 1024) {
        float v[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) v[j] = x[i + 1024 * j];
#pragma unroll
        for (int j = 0; j < 8; ++j) s += (double)v[j] * (double)v[j];
    }
    for (; i < n; i += 1024) s += (double)x[i] * (double)x[i];
    part[threadIdx.x] = s;
    __syncthreads();
    for (int w = 512; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w) part[threadIdx.x] += part[threadIdx.x + w];
        __syncthreads();
    }
    if (threadIdx.x == 0) out[0] = (float)part[0];
}

// W <- W - lr * (c * dW + wd * W).  c = 1, or with sq_norms (the squared norms of ALL gradients of the step) the
// clipping factor min(1, max_norm / (sqrt(sum) + 1e-6)), formed once per workgroup in index order.
template <bool BF>
__global__ __launch_bounds__(256) void sgd_kernel(char* W, const float* dW, int64_t n, float lr, float wd,
                                                  const float* sq_norms, int n_norms, float max_norm) {
    __shared__ float c_shared;
    float c = 1.f;
    if (sq_norms) {
        if (threadIdx.x == 0) {
            double t = 0.0;
            for (int k = 0; k < n_norms; ++k) t += (double)sq_norms[k];
            c_shared = fminf(1.f, (float)((double)max_norm / (sqrt(t) + 1e-6)));
        }
        __syncthreads();
        c = c_shared;
    }
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    const float g = sq_norms ? c * dW[i] : dW[i];
    if constexpr (BF) {
        uint16_t* w = reinterpret_cast<uint16_t*>(W);
        const float v = __uint_as_float((uint32_t)w[i] << 16);
        w[i] = (uint16_t)f32_to_bf16(v - lr * (g + wd * v));
    } else {
        float* w = reinterpret_cast<float*>(W);
        const float v = w[i];
        w[i] = v - lr * (g + wd * v);
    }
}

// Y = X + alpha E, element-wise over [M, F] (the perturbed input of Eq. (3))
template <bool BF>
__global__ __launch_bounds__(256) void axpy_kernel(const char* X, int64_t ldx, const char* E, int64_t lde, char* Y,
                                                   int64_t ldy, int64_t M, int F, float alpha, int vec) {
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    constexpr int EB = BF ? 2 : 4;
    if (vec > 0) {                                    // vec: 16-byte pieces per row
        if (idx >= M * vec) return;
        const int64_t m = idx / vec;
        const int v = (int)(idx % vec);
        const u32x4 x = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(X + m * ldx * EB) + v);
        const u32x4 e = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(E + m * lde * EB) + v);
        u32x4 o;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            if constexpr (BF)
                o[q] = pack_bf16(bf16_lo(x[q]) + alpha * bf16_lo(e[q]), bf16_hi(x[q]) + alpha * bf16_hi(e[q]));
            else
                o[q] = __float_as_uint(__uint_as_float(x[q]) + alpha * __uint_as_float(e[q]));
        }
        __builtin_nontemporal_store(o, reinterpret_cast<u32x4*>(Y + m * ldy * EB) + v);
    } else {
        if (idx >= M * F) return;
        const int64_t m = idx / F;
        const int f = (int)(idx % F);
        if constexpr (BF) {
            const float x = __uint_as_float((uint32_t)reinterpret_cast<const uint16_t*>(X)[m * ldx + f] << 16);
            const float e = __uint_as_float((uint32_t)reinterpret_cast<const uint16_t*>(E)[m * lde + f] << 16);
            reinterpret_cast<uint16_t*>(Y)[m * ldy + f] = (uint16_t)f32_to_bf16(x + alpha * e);
        } else {
            reinterpret_cast<float*>(Y)[m * ldy + f] =
                reinterpret_cast<const float*>(X)[m * ldx + f] + alpha * reinterpret_cast<const float*>(E)[m * lde + f];
        }
    }
}

// dist[m] = || A[m, :] - B[m, :] ||_2: one wavefront per row, lanes stride over the row
template <bool BF>
__global__ __launch_bounds__(256) void row_distance_kernel(const char* A, int64_t lda, const char* B, int64_t ldb,
                                                           int64_t M, int F, float* dist) {
    const int lane = threadIdx.x & 63;
    const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= M) return;
    float s = 0.f;
    for (int f = lane; f < F; f += 64) {
        const float d = load_logit<BF>(A, row * lda + f) - load_logit<BF>(B, row * ldb + f);
        s += d * d;
    }
    s = wave_sum(s);
    if (lane == 0) dist[row] = sqrtf(s);
}

// dot[m] = sum_f A[m, f] * B[m, f]: one wavefront per row, lanes stride over the row
template <bool BF>
__global__ __launch_bounds__(256) void row_dot_kernel(const char* A, int64_t lda, const char* B, int64_t ldb,
                                                      int64_t M, int F, float* dot) {
    const int lane = threadIdx.x & 63;
    const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= M) return;
    float s = 0.f;
    for (int f = lane; f < F; f += 64) s = fmaf(load_logit<BF>(A, row * lda + f), load_logit<BF>(B, row * ldb + f), s);
    s = wave_sum(s);
    if (lane == 0) dot[row] = s;
}

// The same for rows of 16-byte pieces (both strides and bases 16-byte aligned): a team of G = 2^g lanes per row,
// a piece per lane and turn, four rows of every team in flight; the team's lanes are added in a fixed tree.
template <bool BF>
__global__ __launch_bounds__(256) void row_dot_vec_kernel(const char* A, int64_t lda, const char* B, int64_t ldb,
                                                          int64_t M, int pieces, int g_log2, float* dot) {
    constexpr int E = BF ? 8 : 4, EB = BF ? 2 : 4, R = 4;
    const int G = 1 << g_log2;
    const int team = threadIdx.x >> g_log2, tl = threadIdx.x & (G - 1);
    const int teams = 256 >> g_log2;
    const int64_t r0 = ((int64_t)blockIdx.x * teams + team) * R;
    float s[R];
#pragma unroll
    for (int j = 0; j < R; ++j) s[j] = 0.f;
    for (int p = tl; p < pieces; p += G) {
        u32x4 a[R], b[R];
#pragma unroll
        for (int j = 0; j < R; ++j) {
            a[j] = u32x4{0u, 0u, 0u, 0u};
            b[j] = u32x4{0u, 0u, 0u, 0u};
            if (r0 + j < M) {
                a[j] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(A + ((r0 + j) * lda + (int64_t)p * E) * EB));
                b[j] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(B + ((r0 + j) * ldb + (int64_t)p * E) * EB));
            }
        }
#pragma unroll
        for (int j = 0; j < R; ++j)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                if constexpr (BF) {
                    s[j] = fmaf(bf16_lo(a[j][i]), bf16_lo(b[j][i]), s[j]);
                    s[j] = fmaf(bf16_hi(a[j][i]), bf16_hi(b[j][i]), s[j]);
                } else {
                    s[j] = fmaf(__uint_as_float(a[j][i]), __uint_as_float(b[j][i]), s[j]);
                }
            }
    }
#pragma unroll
    for (int j = 0; j < R; ++j) {
        for (int o = G >> 1; o > 0; o >>= 1) s[j] += __shfl_xor(s[j], o);
        if (tl == 0 && r0 + j < M) dot[r0 + j] = s[j];
    }
}

// G[m, :] = scale * (A[m, :] - B[m, :]) / || A[m, :] - B[m, :] ||_2 (zero where the rows are equal): one wavefront
// per row, two passes over the row (the second one out of the cache)
template <bool BF>
__global__ __launch_bounds__(256) void row_distance_bwd_kernel(const char* A, int64_t lda, const char* B, int64_t ldb,
                                                               int64_t M, int F, float scale, char* G, int64_t ldg) {
    const int lane = threadIdx.x & 63;
    const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= M) return;
    float s = 0.f;
    for (int f = lane; f < F; f += 64) {
        const float d = load_logit<BF>(A, row * lda + f) - load_logit<BF>(B, row * ldb + f);
        s += d * d;
    }
    s = wave_sum(s);
    const float c = s > 0.f ? scale / sqrtf(s) : 0.f;
    for (int f = lane; f < F; f += 64) {
        const float g = c * (load_logit<BF>(A, row * lda + f) - load_logit<BF>(B, row * ldb + f));
        if constexpr (BF) reinterpret_cast<uint16_t*>(G)[row * ldg + f] = (uint16_t)f32_to_bf16(g);
        else reinterpret_cast<float*>(G)[row * ldg + f] = g;
    }
}

}  // namespace
}  // namespace gas

using namespace gas;

extern "C" {

gas_status gas_softmax_xent(const void* A, int64_t lda, int64_t n_rows, int32_t n_classes, gas_dtype dt,
                            const int32_t* labels, float scale, float* loss_rows, float* loss_sum, void* G,
                            int64_t ldg, void* stream) {
    if (!valid_dtype(dt)) return fail(GAS_ERR_DTYPE, "gas_softmax_xent: unknown dtype %d", (int)dt);
    GAS_REQUIRE(n_rows >= 0 && n_classes > 0, "gas_softmax_xent: n_rows=%lld n_classes=%d", (long long)n_rows, n_classes);
    hipStream_t s = (hipStream_t)stream;
    if (n_rows > 0) {
        GAS_REQUIRE(A && labels && loss_rows && G, "gas_softmax_xent: null pointer");
        GAS_REQUIRE(lda >= n_classes && ldg >= n_classes, "gas_softmax_xent: row stride smaller than the row");
        GAS_REQUIRE(A != G, "gas_softmax_xent: the gradient must not alias the logits");
        const int epv = dt == GAS_BF16 ? 8 : 4;
        if (n_classes % epv == 0 && n_classes <= 64 * epv && lda % epv == 0 && ldg % epv == 0 && aligned16(A) &&
            aligned16(G)) {
            int lpr_log2 = 0;
            while ((epv << lpr_log2) < n_classes) ++lpr_log2;
            const int64_t rows_per_block = 4 * (64 >> lpr_log2);
            const int64_t blocks = (n_rows + rows_per_block - 1) / rows_per_block;
            if (dt == GAS_BF16)
                hipLaunchKernelGGL(softmax_xent_rows_kernel<true>, dim3((unsigned)blocks), dim3(256), 0, s,
                                   static_cast<const char*>(A), lda, n_rows, n_classes, labels, scale, loss_rows,
                                   static_cast<char*>(G), ldg, lpr_log2);
            else
                hipLaunchKernelGGL(softmax_xent_rows_kernel<false>, dim3((unsigned)blocks), dim3(256), 0, s,
                                   static_cast<const char*>(A), lda, n_rows, n_classes, labels, scale, loss_rows,
                                   static_cast<char*>(G), ldg, lpr_log2);
            GAS_CHECK_HIP(hipGetLastError());
            if (loss_sum) {
                hipLaunchKernelGGL(sum_fixed_kernel, dim3(1), dim3(1024), 0, s, loss_rows, n_rows, loss_sum);
                GAS_CHECK_HIP(hipGetLastError());
            }
            return GAS_OK;
        }
        const int64_t blocks = (n_rows + 3) / 4;
        GAS_REQUIRE(blocks <= 0x7FFFFFFFLL, "gas_softmax_xent: too many rows for one launch");
        if (dt == GAS_BF16)
            hipLaunchKernelGGL(softmax_xent_kernel<true>, dim3((unsigned)blocks), dim3(256), 0, s,
                               static_cast<const char*>(A), lda, n_rows, n_classes, labels, scale, loss_rows,
                               static_cast<char*>(G), ldg);
        else
            hipLaunchKernelGGL(softmax_xent_kernel<false>, dim3((unsigned)blocks), dim3(256), 0, s,
                               static_cast<const char*>(A), lda, n_rows, n_classes, labels, scale, loss_rows,
                               static_cast<char*>(G), ldg);
        GAS_CHECK_HIP(hipGetLastError());
    }
    if (loss_sum) {
        hipLaunchKernelGGL(sum_fixed_kernel, dim3(1), dim3(1024), 0, s, loss_rows, n_rows, loss_sum);
        GAS_CHECK_HIP(hipGetLastError());
    }
    return GAS_OK;
}

gas_status gas_sq_norm(const float* x, int64_t n, float* out, void* stream) {
    GAS_REQUIRE(n >= 0, "gas_sq_norm: n=%lld", (long long)n);
    GAS_REQUIRE(out, "gas_sq_norm: null output");
    GAS_REQUIRE(x || n == 0, "gas_sq_norm: null pointer");
    hipLaunchKernelGGL(sq_sum_fixed_kernel, dim3(1), dim3(1024), 0, (hipStream_t)stream, x, n, out);
    GAS_CHECK_HIP(hipGetLastError());
    return GAS_OK;
}

static gas_status run_sgd(void* W, int64_t n, gas_dtype dt, const float* dW, float lr, float weight_decay,
                          const float* sq_norms, int n_norms, float max_norm, void* stream) {
    if (!valid_dtype(dt)) return fail(GAS_ERR_DTYPE, "gas_sgd_step: unknown dtype %d", (int)dt);
    GAS_REQUIRE(n >= 0, "gas_sgd_step: n=%lld", (long long)n);
    if (n == 0) return GAS_OK;
    GAS_REQUIRE(W && dW, "gas_sgd_step: null pointer");
    const int64_t blocks = (n + 255) / 256;
    GAS_REQUIRE(blocks <= 0x7FFFFFFFLL, "gas_sgd_step: too many elements for one launch");
    if (dt == GAS_BF16)
        hipLaunchKernelGGL(sgd_kernel<true>, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream,
                           static_cast<char*>(W), dW, n, lr, weight_decay, sq_norms, n_norms, max_norm);
    else
        hipLaunchKernelGGL(sgd_kernel<false>, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream,
                           static_cast<char*>(W), dW, n, lr, weight_decay, sq_norms, n_norms, max_norm);
    GAS_CHECK_HIP(hipGetLastError());
    return GAS_OK;
}

gas_status gas_sgd_step(void* W, int64_t n, gas_dtype dt, const float* dW, float lr, float weight_decay,
                        void* stream) {
    return run_sgd(W, n, dt, dW, lr, weight_decay, nullptr, 0, 0.f, stream);
}

gas_status gas_sgd_step_clipped(void* W, int64_t n, gas_dtype dt, const float* dW, float lr, float weight_decay,
                                const float* sq_norms, int32_t n_norms, float max_norm, void* stream) {
    GAS_REQUIRE(n < 0 || n == 0 || (sq_norms && n_norms > 0 && max_norm > 0.f),
                "gas_sgd_step_clipped: sq_norms=%p n_norms=%d max_norm=%g", (const void*)sq_norms, n_norms,
                (double)max_norm);
    return run_sgd(W, n, dt, dW, lr, weight_decay, sq_norms, n_norms, max_norm, stream);
}

gas_status gas_axpy(const void* X, int64_t ldx, const void* E, int64_t lde, int64_t n_rows, int32_t F, gas_dtype dt,
                    float alpha, void* Y, int64_t ldy, void* stream) {
    if (!valid_dtype(dt)) return fail(GAS_ERR_DTYPE, "gas_axpy: unknown dtype %d", (int)dt);
    GAS_REQUIRE(n_rows >= 0 && F > 0, "gas_axpy: n_rows=%lld F=%d", (long long)n_rows, F);
    if (n_rows == 0) return GAS_OK;
    GAS_REQUIRE(X && E && Y, "gas_axpy: null pointer");
    GAS_REQUIRE(ldx >= F && lde >= F && ldy >= F, "gas_axpy: row stride smaller than the row");
    const int q = dt == GAS_BF16 ? 8 : 4;
    const bool vec = F % q == 0 && ldx % q == 0 && lde % q == 0 && ldy % q == 0 && aligned16(X) && aligned16(E) && aligned16(Y);
    const int v = vec ? F / q : 0;
    const int64_t total = n_rows * (int64_t)(vec ? v : F);
    const int64_t blocks = (total + 255) / 256;
    GAS_REQUIRE(blocks <= 0x7FFFFFFFLL, "gas_axpy: problem too large for one launch");
    if (dt == GAS_BF16)
        hipLaunchKernelGGL(axpy_kernel<true>, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream,
                           static_cast<const char*>(X), ldx, static_cast<const char*>(E), lde, static_cast<char*>(Y), ldy,
                           n_rows, F, alpha, v);
    else
        hipLaunchKernelGGL(axpy_kernel<false>, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream,
                           static_cast<const char*>(X), ldx, static_cast<const char*>(E), lde, static_cast<char*>(Y), ldy,
                           n_rows, F, alpha, v);
    GAS_CHECK_HIP(hipGetLastError());
    return GAS_OK;
}

gas_status gas_row_distance(const void* A, int64_t lda, const void* B, int64_t ldb, int64_t n_rows, int32_t F,
                            gas_dtype dt, float* dist, float* dist_sum, void* stream) {
    if (!valid_dtype(dt)) return fail(GAS_ERR_DTYPE, "gas_row_distance: unknown dtype %d", (int)dt);
    GAS_REQUIRE(n_rows >= 0 && F > 0, "gas_row_distance: n_rows=%lld F=%d", (long long)n_rows, F);
    hipStream_t s = (hipStream_t)stream;
    if (n_rows > 0) {
        GAS_REQUIRE(A && B && dist, "gas_row_distance: null pointer");
        GAS_REQUIRE(lda >= F && ldb >= F, "gas_row_distance: row stride smaller than the row");
        const int64_t blocks = (n_rows + 3) / 4;
        GAS_REQUIRE(blocks <= 0x7FFFFFFFLL, "gas_row_distance: too many rows for one launch");
        if (dt == GAS_BF16)
            hipLaunchKernelGGL(row_distance_kernel<true>, dim3((unsigned)blocks), dim3(256), 0, s,
                               static_cast<const char*>(A), lda, static_cast<const char*>(B), ldb, n_rows, F, dist);
        else
            hipLaunchKernelGGL(row_distance_kernel<false>, dim3((unsigned)blocks), dim3(256), 0, s,
                               static_cast<const char*>(A), lda, static_cast<const char*>(B), ldb, n_rows, F, dist);
        GAS_CHECK_HIP(hipGetLastError());
    }
    if (dist_sum) {
        hipLaunchKernelGGL(sum_fixed_kernel, dim3(1), dim3(1024), 0, s, dist, n_rows, dist_sum);
        GAS_CHECK_HIP(hipGetLastError());
    }
    return GAS_OK;
}

gas_status gas_row_dot(const void* A, int64_t lda, const void* B, int64_t ldb, int64_t n_rows, int32_t F,
                       gas_dtype dt, float* dot, float* dot_sum, void* stream) {
    if (!valid_dtype(dt)) return fail(GAS_ERR_DTYPE, "gas_row_dot: unknown dtype %d", (int)dt);
    GAS_REQUIRE(n_rows >= 0 && F > 0, "gas_row_dot: n_rows=%lld F=%d", (long long)n_rows, F);
    hipStream_t s = (hipStream_t)stream;
    if (n_rows > 0) {
        GAS_REQUIRE(A && B && dot, "gas_row_dot: null pointer");
        GAS_REQUIRE(lda >= F && ldb >= F, "gas_row_dot: row stride smaller than the row");
        const int e = dt == GAS_BF16 ? 8 : 4;
        if (F % e == 0 && lda % e == 0 && ldb % e == 0 && aligned16(A) && aligned16(B)) {
            const int pieces = F / e;
            int g_log2 = 0;
            while ((1 << g_log2) < pieces && g_log2 < 6) ++g_log2;
            const int64_t rows_per_block = (256 >> g_log2) * 4;
            const int64_t vblocks = (n_rows + rows_per_block - 1) / rows_per_block;
            GAS_REQUIRE(vblocks <= 0x7FFFFFFFLL, "gas_row_dot: too many rows for one launch");
            if (dt == GAS_BF16)
                hipLaunchKernelGGL(row_dot_vec_kernel<true>, dim3((unsigned)vblocks), dim3(256), 0, s,
                                   static_cast<const char*>(A), lda, static_cast<const char*>(B), ldb, n_rows, pieces, g_log2, dot);
            else
                hipLaunchKernelGGL(row_dot_vec_kernel<false>, dim3((unsigned)vblocks), dim3(256), 0, s,
                                   static_cast<const char*>(A), lda, static_cast<const char*>(B), ldb, n_rows, pieces, g_log2, dot);
            GAS_CHECK_HIP(hipGetLastError());
            if (dot_sum) {
                hipLaunchKernelGGL(sum_fixed_kernel, dim3(1), dim3(1024), 0, s, dot, n_rows, dot_sum);
                GAS_CHECK_HIP(hipGetLastError());
            }
            return GAS_OK;
        }
        const int64_t blocks = (n_rows + 3) / 4;
        GAS_REQUIRE(blocks <= 0x7FFFFFFFLL, "gas_row_dot: too many rows for one launch");
        if (dt == GAS_BF16)
            hipLaunchKernelGGL(row_dot_kernel<true>, dim3((unsigned)blocks), dim3(256), 0, s,
                               static_cast<const char*>(A), lda, static_cast<const char*>(B), ldb, n_rows, F, dot);
        else
            hipLaunchKernelGGL(row_dot_kernel<false>, dim3((unsigned)blocks), dim3(256), 0, s,
                               static_cast<const char*>(A), lda, static_cast<const char*>(B), ldb, n_rows, F, dot);
        GAS_CHECK_HIP(hipGetLastError());
    }
    if (dot_sum) {
        hipLaunchKernelGGL(sum_fixed_kernel, dim3(1), dim3(1024), 0, s, dot, n_rows, dot_sum);
        GAS_CHECK_HIP(hipGetLastError());
    }
    return GAS_OK;
}

gas_status gas_row_distance_bwd(const void* A, int64_t lda, const void* B, int64_t ldb, int64_t n_rows, int32_t F,
                                gas_dtype dt, float scale, void* G, int64_t ldg, void* stream) {
    if (!valid_dtype(dt)) return fail(GAS_ERR_DTYPE, "gas_row_distance_bwd: unknown dtype %d", (int)dt);
    GAS_REQUIRE(n_rows >= 0 && F > 0, "gas_row_distance_bwd: n_rows=%lld F=%d", (long long)n_rows, F);
    if (n_rows == 0) return GAS_OK;
    GAS_REQUIRE(A && B && G, "gas_row_distance_bwd: null pointer");
    GAS_REQUIRE(lda >= F && ldb >= F && ldg >= F, "gas_row_distance_bwd: row stride smaller than the row");
    const int64_t blocks = (n_rows + 3) / 4;
    GAS_REQUIRE(blocks <= 0x7FFFFFFFLL, "gas_row_distance_bwd: too many rows for one launch");
    if (dt == GAS_BF16)
        hipLaunchKernelGGL(row_distance_bwd_kernel<true>, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream,
                           static_cast<const char*>(A), lda, static_cast<const char*>(B), ldb, n_rows, F, scale,
                           static_cast<char*>(G), ldg);
    else
        hipLaunchKernelGGL(row_distance_bwd_kernel<false>, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream,
                           static_cast<const char*>(A), lda, static_cast<const char*>(B), ldb, n_rows, F, scale,
                           static_cast<char*>(G), ldg);
    GAS_CHECK_HIP(hipGetLastError());
    return GAS_OK;
}

}  // extern "C"
