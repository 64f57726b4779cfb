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

// sum of n floats in a fixed order: thread t adds elements t, t+1024, ... in double, then a tree over the block
__global__ __launch_bounds__(1024) void sum_fixed_kernel(const float* x, int64_t n, float* out) {
    __shared__ double part[1024];
    double s = 0.0;
    for (int64_t i = threadIdx.x; i < n; i += 1024) s += (double)x[i];
    part[threadIdx.x] = s;
    __syncthreads();
    for (int w = 512; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w) part[threadIdx.x] += part[threadIdx.x + w];
        __syncthreads();
    }
    if (threadIdx.x == 0) out[0] = (float)part[0];
}

template <bool BF>
__global__ __launch_bounds__(256) void sgd_kernel(char* W, const float* dW, int64_t n, float lr, float wd) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    if constexpr (BF) {
        uint16_t* w = reinterpret_cast<uint16_t*>(W);
        const float v = __uint_as_float((uint32_t)w[i] << 16);
        w[i] = (uint16_t)f32_to_bf16(v - lr * (dW[i] + wd * v));
    } else {
        float* w = reinterpret_cast<float*>(W);
        const float v = w[i];
        w[i] = v - lr * (dW[i] + wd * v);
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

gas_status gas_sgd_step(void* W, int64_t n, gas_dtype dt, const float* dW, float lr, float weight_decay,
                        void* stream) {
    if (!valid_dtype(dt)) return fail(GAS_ERR_DTYPE, "gas_sgd_step: unknown dtype %d", (int)dt);
    GAS_REQUIRE(n >= 0, "gas_sgd_step: n=%lld", (long long)n);
    if (n == 0) return GAS_OK;
    GAS_REQUIRE(W && dW, "gas_sgd_step: null pointer");
    const int64_t blocks = (n + 255) / 256;
    GAS_REQUIRE(blocks <= 0x7FFFFFFFLL, "gas_sgd_step: too many elements for one launch");
    if (dt == GAS_BF16)
        hipLaunchKernelGGL(sgd_kernel<true>, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream,
                           static_cast<char*>(W), dW, n, lr, weight_decay);
    else
        hipLaunchKernelGGL(sgd_kernel<false>, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream,
                           static_cast<char*>(W), dW, n, lr, weight_decay);
    GAS_CHECK_HIP(hipGetLastError());
    return GAS_OK;
}

}  // extern "C"
