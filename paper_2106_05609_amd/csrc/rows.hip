// History access (gas_pull, gas_push), GCN edge coefficients, index
// validation, and the library's error plumbing.
//
// Pull and push are the Pull / Push operations of the paper's Algorithm 1:
// a row gather from, and a row scatter into, a per-layer history table.  Here
// the tables live in HBM, so both are HBM-to-HBM row copies: a group of lanes
// moves one row with 128-bit accesses, several rows are in flight per lane,
// and the accesses are non-temporal (every byte is touched once).
#include "common.h"

namespace gas {

char* last_error_buffer() {
    static thread_local char buf[512] = "no error";
    return buf;
}

gas_status fail(gas_status st, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(last_error_buffer(), 512, fmt, ap);
    va_end(ap);
    return st;
}

namespace {

constexpr int kCopyThreads = 256;
constexpr int kCopyUnroll = 4;

// One "team" of 2^g_log2 lanes moves one row of `units` vectors of type V.
// Source row i is src_idx[i] (or src_base + i), destination row likewise.
template <typename V>
__global__ __launch_bounds__(kCopyThreads) void copy_rows_kernel(
    const char* __restrict__ src, int64_t src_stride, const int32_t* __restrict__ src_idx, int64_t src_base,
    char* __restrict__ dst, int64_t dst_stride, const int32_t* __restrict__ dst_idx, int64_t dst_base,
    int64_t n, int units, int g_log2, int64_t n_blocks) {
    const int team = threadIdx.x >> g_log2;
    const int lane = threadIdx.x & ((1 << g_log2) - 1);
    const int teams = kCopyThreads >> g_log2;
    // one pass when the grid covers all row blocks (tables in HBM); a small grid striding over them otherwise
    for (int64_t blk = blockIdx.x; blk < n_blocks; blk += gridDim.x) {
        const int64_t r0 = blk * teams * kCopyUnroll + team;
        int64_t srow[kCopyUnroll], drow[kCopyUnroll];
#pragma unroll
        for (int j = 0; j < kCopyUnroll; ++j) {
            const int64_t r = r0 + (int64_t)j * teams;
            const bool ok = r < n;
            srow[j] = ok ? (src_idx ? (int64_t)src_idx[r] : src_base + r) : -1;
            drow[j] = ok ? (dst_idx ? (int64_t)dst_idx[r] : dst_base + r) : -1;
        }
        for (int u = lane; u < units; u += (1 << g_log2)) {
            V tmp[kCopyUnroll];
#pragma unroll
            for (int j = 0; j < kCopyUnroll; ++j)
                if (srow[j] >= 0)
                    tmp[j] = __builtin_nontemporal_load(
                        reinterpret_cast<const V*>(src + srow[j] * src_stride) + u);
#pragma unroll
            for (int j = 0; j < kCopyUnroll; ++j)
                if (srow[j] >= 0)
                    __builtin_nontemporal_store(tmp[j], reinterpret_cast<V*>(dst + drow[j] * dst_stride) + u);
        }
    }
}

gas_status launch_copy(const void* src, int64_t ld_src, const int32_t* src_idx, int64_t src_base,
                       void* dst, int64_t ld_dst, const int32_t* dst_idx, int64_t dst_base,
                       int64_t n, int32_t F, gas_dtype dt, hipStream_t stream, int64_t max_blocks = 0) {
    if (n == 0) return GAS_OK;
    const int eb = elem_bytes(dt);
    const int64_t row_bytes = (int64_t)F * eb, ss = ld_src * eb, ds = ld_dst * eb;
    int vec = eb;   // widest access that divides everything
    if (aligned16(src) && aligned16(dst) && row_bytes % 16 == 0 && ss % 16 == 0 && ds % 16 == 0) vec = 16;
    else if (eb == 2 && ((uintptr_t)src % 4 == 0) && ((uintptr_t)dst % 4 == 0) && row_bytes % 4 == 0 &&
             ss % 4 == 0 && ds % 4 == 0) vec = 4;
    const int units = (int)(row_bytes / vec);
    int g_log2 = 0;
    while ((1 << g_log2) < units && g_log2 < 6) ++g_log2;
    const int teams = kCopyThreads >> g_log2;
    const int64_t rows_per_block = (int64_t)teams * kCopyUnroll;
    const int64_t blocks = (n + rows_per_block - 1) / rows_per_block;
    if (blocks > 0x7FFFFFFF) return fail(GAS_ERR_ARG, "too many rows for one launch: %lld", (long long)n);
    dim3 grid((unsigned)((max_blocks > 0 && max_blocks < blocks) ? max_blocks : blocks)), block(kCopyThreads);
    const char* s = static_cast<const char*>(src);
    char* d = static_cast<char*>(dst);
    if (vec == 16)
        hipLaunchKernelGGL(copy_rows_kernel<u32x4>, grid, block, 0, stream, s, ss, src_idx, src_base, d, ds,
                           dst_idx, dst_base, n, units, g_log2, blocks);
    else if (vec == 4)
        hipLaunchKernelGGL(copy_rows_kernel<uint32_t>, grid, block, 0, stream, s, ss, src_idx, src_base, d, ds,
                           dst_idx, dst_base, n, units, g_log2, blocks);
    else
        hipLaunchKernelGGL(copy_rows_kernel<uint16_t>, grid, block, 0, stream, s, ss, src_idx, src_base, d, ds,
                           dst_idx, dst_base, n, units, g_log2, blocks);
    GAS_CHECK_HIP(hipGetLastError());
    return GAS_OK;
}

// One wavefront per row of the pattern; lanes stride over the row's entries.
__global__ __launch_bounds__(256) void gcn_norm_kernel(const int32_t* __restrict__ ptr,
                                                       const int32_t* __restrict__ ind, int64_t n_rows,
                                                       const int32_t* __restrict__ n_id,
                                                       const int32_t* __restrict__ deg,
                                                       float* __restrict__ val) {
    const int64_t r = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (r >= n_rows) return;
    const double dr = sqrt((double)deg[n_id[r]] + 1.0);
    const int end = ptr[r + 1];
    for (int k = ptr[r] + (threadIdx.x & 63); k < end; k += 64) {
        const double dc = sqrt((double)deg[n_id[ind[k]]] + 1.0);
        val[k] = (float)(1.0 / (dc * dr));
    }
}

__global__ void validate_kernel(const int32_t* __restrict__ idx, int64_t n, int64_t limit, int* flag) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) {
        const int64_t v = idx[i];
        if (v < 0 || v >= limit) *flag = 1;   // every writer stores the same value
    }
}

}  // namespace
}  // namespace gas

using namespace gas;

extern "C" {

const char* gas_last_error(void) { return last_error_buffer(); }

int gas_version(void) { return 100; }

// A transfer over the host link needs few requests in flight to run at the link's rate; a small grid leaves the
// compute units to the kernels of other streams (the overlap the paper's transfer scheme is about).
static constexpr int64_t kHostLinkBlocks = 64;

static gas_status run_pull(const void* hist, int64_t n_hist_rows, int64_t ld_hist, const int32_t* idx, int64_t base,
                           int64_t n, int32_t F, gas_dtype dt, void* dst, int64_t ld_dst, void* stream,
                           int64_t max_blocks) {
    if (!valid_dtype(dt)) return fail(GAS_ERR_DTYPE, "gas_pull: unknown dtype %d", (int)dt);
    GAS_REQUIRE(n >= 0 && F > 0 && n_hist_rows >= 0, "gas_pull: n=%lld F=%d n_hist_rows=%lld", (long long)n, F,
                (long long)n_hist_rows);
    if (n == 0) return GAS_OK;
    GAS_REQUIRE(hist && dst, "gas_pull: null table or destination");
    GAS_REQUIRE(ld_hist >= F && ld_dst >= F, "gas_pull: row stride smaller than F");
    if (!idx) GAS_REQUIRE(base >= 0 && base + n <= n_hist_rows, "gas_pull: range [%lld, %lld) outside the table",
                          (long long)base, (long long)(base + n));
    return launch_copy(hist, ld_hist, idx, base, dst, ld_dst, nullptr, 0, n, F, dt, (hipStream_t)stream, max_blocks);
}

gas_status gas_pull(const void* hist, int64_t n_hist_rows, int64_t ld_hist, const int32_t* idx, int64_t base,
                    int64_t n, int32_t F, gas_dtype dt, void* dst, int64_t ld_dst, void* stream) {
    return run_pull(hist, n_hist_rows, ld_hist, idx, base, n, F, dt, dst, ld_dst, stream, 0);
}

gas_status gas_pull_host(const void* hist, int64_t n_hist_rows, int64_t ld_hist, const int32_t* idx, int64_t base,
                         int64_t n, int32_t F, gas_dtype dt, void* dst, int64_t ld_dst, void* stream) {
    return run_pull(hist, n_hist_rows, ld_hist, idx, base, n, F, dt, dst, ld_dst, stream, kHostLinkBlocks);
}

static gas_status run_push(const void* src, int64_t ld_src, const int32_t* idx, int64_t base, int64_t n, int32_t F,
                           gas_dtype dt, void* hist, int64_t n_hist_rows, int64_t ld_hist, void* stream,
                           int64_t max_blocks) {
    if (!valid_dtype(dt)) return fail(GAS_ERR_DTYPE, "gas_push: unknown dtype %d", (int)dt);
    GAS_REQUIRE(n >= 0 && F > 0 && n_hist_rows >= 0, "gas_push: n=%lld F=%d n_hist_rows=%lld", (long long)n, F,
                (long long)n_hist_rows);
    if (n == 0) return GAS_OK;
    GAS_REQUIRE(hist && src, "gas_push: null table or source");
    GAS_REQUIRE(ld_hist >= F && ld_src >= F, "gas_push: row stride smaller than F");
    if (!idx) GAS_REQUIRE(base >= 0 && base + n <= n_hist_rows, "gas_push: range [%lld, %lld) outside the table",
                          (long long)base, (long long)(base + n));
    return launch_copy(src, ld_src, nullptr, 0, hist, ld_hist, idx, base, n, F, dt, (hipStream_t)stream, max_blocks);
}

gas_status gas_push(const void* src, int64_t ld_src, const int32_t* idx, int64_t base, int64_t n, int32_t F,
                    gas_dtype dt, void* hist, int64_t n_hist_rows, int64_t ld_hist, void* stream) {
    return run_push(src, ld_src, idx, base, n, F, dt, hist, n_hist_rows, ld_hist, stream, 0);
}

gas_status gas_push_host(const void* src, int64_t ld_src, const int32_t* idx, int64_t base, int64_t n, int32_t F,
                         gas_dtype dt, void* hist, int64_t n_hist_rows, int64_t ld_hist, void* stream) {
    return run_push(src, ld_src, idx, base, n, F, dt, hist, n_hist_rows, ld_hist, stream, kHostLinkBlocks);
}

gas_status gas_gcn_norm(const int32_t* ptr, const int32_t* ind, int64_t n_rows, const int32_t* n_id,
                        const int32_t* deg, float* val, void* stream) {
    GAS_REQUIRE(n_rows >= 0, "gas_gcn_norm: n_rows=%lld", (long long)n_rows);
    if (n_rows == 0) return GAS_OK;
    GAS_REQUIRE(ptr && ind && n_id && deg && val, "gas_gcn_norm: null pointer");
    GAS_REQUIRE(n_rows < 0x7FFFFFFFLL, "gas_gcn_norm: too many rows");
    const unsigned blocks = (unsigned)((n_rows + 3) / 4);
    hipLaunchKernelGGL(gcn_norm_kernel, dim3(blocks), dim3(256), 0, (hipStream_t)stream, ptr, ind, n_rows, n_id,
                       deg, val);
    GAS_CHECK_HIP(hipGetLastError());
    return GAS_OK;
}

gas_status gas_validate_indices(const int32_t* idx, int64_t n, int64_t limit, void* stream) {
    GAS_REQUIRE(n >= 0 && limit >= 0, "gas_validate_indices: n=%lld limit=%lld", (long long)n, (long long)limit);
    if (n == 0) return GAS_OK;
    GAS_REQUIRE(idx, "gas_validate_indices: null index array");
    int* d_flag = nullptr;
    GAS_CHECK_HIP(hipMalloc(&d_flag, sizeof(int)));
    hipStream_t s = (hipStream_t)stream;
    int h_flag = 0;
    hipError_t e = hipMemcpyAsync(d_flag, &h_flag, sizeof(int), hipMemcpyHostToDevice, s);
    if (e == hipSuccess) {
        const int64_t blocks = (n + 255) / 256;
        hipLaunchKernelGGL(validate_kernel, dim3((unsigned)blocks), dim3(256), 0, s, idx, n, limit, d_flag);
        e = hipGetLastError();
    }
    if (e == hipSuccess) e = hipMemcpyAsync(&h_flag, d_flag, sizeof(int), hipMemcpyDeviceToHost, s);
    if (e == hipSuccess) e = hipStreamSynchronize(s);
    (void)hipFree(d_flag);
    if (e != hipSuccess) return fail(GAS_ERR_HIP, "gas_validate_indices: %s", hipGetErrorString(e));
    if (h_flag) return fail(GAS_ERR_RANGE, "gas_validate_indices: an index lies outside [0, %lld)", (long long)limit);
    return GAS_OK;
}

gas_status gas_host_table_pointer(const void* host_ptr, void** device_ptr) {
    GAS_REQUIRE(host_ptr && device_ptr, "gas_host_table_pointer: null pointer");
    void* d = nullptr;
    const hipError_t e = hipHostGetDevicePointer(&d, const_cast<void*>(host_ptr), 0);
    if (e != hipSuccess || !d) {
        (void)hipGetLastError();                       // the failed query must not be reported by a later call
        return fail(GAS_ERR_ARG, "gas_host_table_pointer: not pinned host memory that this device can address (%s)",
                    hipGetErrorString(e));
    }
    *device_ptr = d;
    return GAS_OK;
}

}  // extern "C"
