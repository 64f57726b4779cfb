// gas_plan_create: the schedule of one compressed sparse pattern, built on the device.
//
// plan_host.h defines the plan (groups of light rows, chunks of heavy rows cut and ordered by L2-sized windows, the
// ranges of groups per XCD and the locality vote).  Here the same arrays are produced by kernels from the row
// pointers and indices where they lie, in device memory: only a handful of counters cross to the host (two waits),
// so building a plan costs a few passes over the indices of the heavy rows instead of a copy of all indices to the
// host and a single-threaded walk.  Algorithm 1 builds the batch subgraph once per batch and reuses it for every
// layer and epoch; so is its plan.  The host builder stays available (gas_plan_options.host_builder) as the
// reference the tests compare this one with, array by array.
//
// Steps:
//   rows    one wavefront per block of 1024 rows: row pointers into LDS, validated by all lanes; one lane walks
//           the block (the grouping rule is greedy, hence sequential, but only inside a block) - a counting pass,
//           an exclusive scan over the blocks, a writing pass.
//   chunks  one wavefront per heavy row: window keys 64 entries at a time, the positions where the window changes
//           as a ballot mask, the greedy cut rule over the set bits (wavefront-uniform) - counting pass, scan,
//           writing pass (row-major list and sort keys).
//   order   stable radix sort of the chunk list by window key, one bit per pass (a stable split by a bit is an
//           exclusive scan of the zero flags plus a scatter); the passes are short lists, not index arrays.
//   ranges  exclusive scan of the group costs, eight lower bounds, the sampled locality vote.
// All sums are integer sums: atomics on counters give the same value in any order.
#include "common.h"
#include "plan.h"
#include "plan_host.h"

#include <vector>

namespace gas {
namespace {

constexpr int kRowsPerBlock = 1024;              // PlanParams::group_block of the device builder
constexpr int kScanTile = 1024;                  // 256 threads x 4 items

// ------------------------------------------------------------------------------------------------ scans
// exclusive prefix of the calling thread's value over the 256 threads of the workgroup; *total = sum of all
__device__ __forceinline__ int64_t block_exclusive_scan(int64_t v, int64_t* total) {
    __shared__ int64_t wave_sum[4];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int64_t x = v;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const int64_t y = __shfl_up(x, off, 64);
        if (lane >= off) x += y;
    }
    __syncthreads();                              // wave_sum may still be read from a previous call
    if (lane == 63) wave_sum[wave] = x;
    __syncthreads();
    int64_t before = 0, all = 0;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        if (w < wave) before += wave_sum[w];
        all += wave_sum[w];
    }
    *total = all;
    return x - v + before;
}

template <class In>
__global__ __launch_bounds__(256) void scan_reduce_kernel(In in, int64_t n, int64_t* __restrict__ tile_sums) {
    const int64_t base = (int64_t)blockIdx.x * kScanTile + (int64_t)threadIdx.x * 4;
    int64_t s = 0;
#pragma unroll
    for (int q = 0; q < 4; ++q)
        if (base + q < n) s += in(base + q);
    int64_t total;
    (void)block_exclusive_scan(s, &total);
    if (threadIdx.x == 0) tile_sums[blockIdx.x] = total;
}

// one workgroup: tile_sums -> exclusive prefixes in place; the grand total to *total
__global__ __launch_bounds__(256) void scan_tiles_kernel(int64_t* __restrict__ tile_sums, int64_t n_tiles,
                                                         int64_t* __restrict__ total) {
    int64_t carry = 0;
    for (int64_t t0 = 0; t0 < n_tiles; t0 += 256) {
        const int64_t i = t0 + threadIdx.x;
        const int64_t v = i < n_tiles ? tile_sums[i] : 0;
        int64_t all;
        const int64_t ex = block_exclusive_scan(v, &all);
        if (i < n_tiles) tile_sums[i] = carry + ex;
        carry += all;
    }
    if (threadIdx.x == 0) *total = carry;
}

template <class In, class Out>
__global__ __launch_bounds__(256) void scan_apply_kernel(In in, int64_t n, const int64_t* __restrict__ tile_offs,
                                                         Out out) {
    const int64_t base = (int64_t)blockIdx.x * kScanTile + (int64_t)threadIdx.x * 4;
    int64_t v[4], s = 0;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        v[q] = base + q < n ? in(base + q) : 0;
        s += v[q];
    }
    int64_t total;
    int64_t ex = block_exclusive_scan(s, &total) + tile_offs[blockIdx.x];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        if (base + q < n) out(base + q, ex, v[q]);
        ex += v[q];
    }
}

struct StridedIn {
    const int64_t* p; int64_t stride;
    __device__ int64_t operator()(int64_t i) const { return p[i * stride]; }
};
struct StridedOut {
    int64_t* p; int64_t stride;
    __device__ void operator()(int64_t i, int64_t ex, int64_t) const { p[i * stride] = ex; }
};
// first chunk slot of every heavy row (int32), and the end of the last one
struct FirstSlotOut {
    int32_t* first; int64_t n;
    __device__ void operator()(int64_t i, int64_t ex, int64_t v) const {
        first[i] = (int32_t)ex;
        if (i == n - 1) first[n] = (int32_t)(ex + v);
    }
};
struct GroupCostIn {
    const int32_t* ptr; const int32_t* group;
    __device__ int64_t operator()(int64_t i) const {
        const int32_t g0 = group[2 * i], g1 = group[2 * i + 1];
        return (int64_t)(ptr[g1] - ptr[g0]) + (g1 - g0);
    }
};
struct PlainOut {
    int64_t* p;
    __device__ void operator()(int64_t i, int64_t ex, int64_t) const { p[i] = ex; }
};
// stable split of (key, idx) pairs by one bit of the key: zeros first, in order, then ones, in order
struct BitZeroIn {
    const uint32_t* key; int bit;
    __device__ int64_t operator()(int64_t i) const { return ((key[i] >> bit) & 1u) == 0u; }
};
struct SplitOut {
    const uint32_t* key; const int32_t* idx; uint32_t* key_out; int32_t* idx_out; const int64_t* zeros;
    __device__ void operator()(int64_t i, int64_t ex, int64_t is_zero) const {
        const int64_t pos = is_zero ? ex : *zeros + (i - ex);
        key_out[pos] = key[i];
        idx_out[pos] = idx[i];
    }
};

// exclusive scan of in(0..n-1) through `out`; the total goes to *total (device).  tile_sums: >= tiles(n) int64.
template <class In, class Out>
void device_scan(In in, int64_t n, Out out, int64_t* tile_sums, int64_t* total, hipStream_t s) {
    const int64_t tiles = (n + kScanTile - 1) / kScanTile;
    if (tiles > 0) hipLaunchKernelGGL((scan_reduce_kernel<In>), dim3((unsigned)tiles), dim3(256), 0, s, in, n, tile_sums);
    hipLaunchKernelGGL(scan_tiles_kernel, dim3(1), dim3(256), 0, s, tile_sums, tiles, total);
    if (tiles > 0)
        hipLaunchKernelGGL((scan_apply_kernel<In, Out>), dim3((unsigned)tiles), dim3(256), 0, s, in, n, tile_sums, out);
}

// ------------------------------------------------------------------------------------------------ rows
struct Counters {                      // one small device struct read back in two copies
    unsigned long long bad_row;        // smallest (row + 1) whose pointers are wrong; ~0 if none
    unsigned int bad_ends;             // bit 0: ptr[0] != 0, bit 1: ptr[n_rows] != nnz
    unsigned int max_key;
    int64_t n_groups, n_heavy, n_chunks, cost_total;
    int64_t xcd_start[9];
    unsigned long long local, seen;
    int64_t zeros;                     // of the current radix pass
};

struct RowsArgs {
    const int32_t* ptr; int64_t n_rows, nnz; int threshold;
    int64_t* counts;                   // [2 * n_blocks] groups, heavy rows of every block
    int32_t* group; int32_t* heavy;    // outputs of the writing pass
    Counters* ctr;
};

template <bool WRITE>
__global__ __launch_bounds__(256) void plan_rows_kernel(RowsArgs a) {
    __shared__ int32_t sp[4][kRowsPerBlock + 1];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int64_t blk = (int64_t)blockIdx.x * 4 + wave;
    const int64_t r0 = blk * kRowsPerBlock;
    const bool active = r0 < a.n_rows;
    const int n = active ? (int)min((int64_t)kRowsPerBlock, a.n_rows - r0) : 0;
    int32_t* p = sp[wave];
    if (active)
        for (int i = lane; i <= n; i += 64) p[i] = a.ptr[r0 + i];
    __syncthreads();
    if (!active) return;
    if constexpr (!WRITE) {
        for (int i = lane; i < n; i += 64) {
            const int32_t lo = p[i], hi = p[i + 1];
            if (lo < 0 || hi < lo || (int64_t)hi > a.nnz) atomicMin(&a.ctr->bad_row, (unsigned long long)(r0 + i + 1));
        }
        if (lane == 0 && r0 == 0 && p[0] != 0) atomicOr(&a.ctr->bad_ends, 1u);
        if (lane == 0 && r0 + n == a.n_rows && (int64_t)p[n] != a.nnz) atomicOr(&a.ctr->bad_ends, 2u);
    }
    if (lane != 0) return;
    int64_t ng = 0, nh = 0;
    const int64_t gbase = WRITE ? a.counts[2 * blk] : 0, hbase = WRITE ? a.counts[2 * blk + 1] : 0;   // exclusive prefixes
    int g_start = -1, g_entries = 0;
    auto close = [&](int end) {
        if (g_start >= 0) {
            if constexpr (WRITE) {
                a.group[2 * (gbase + ng)] = (int32_t)(r0 + g_start);
                a.group[2 * (gbase + ng) + 1] = (int32_t)(r0 + end);
            }
            ++ng;
        }
        g_start = -1; g_entries = 0;
    };
    for (int i = 0; i < n; ++i) {
        const int len = p[i + 1] - p[i];
        if (len > a.threshold) {
            close(i);
            if constexpr (WRITE) a.heavy[hbase + nh] = (int32_t)(r0 + i);
            ++nh;
        } else {
            if (g_start >= 0 && (g_entries + len > 64 || i - g_start >= 63)) close(i);
            if (g_start < 0) g_start = i;
            g_entries += len;
        }
    }
    close(n);
    if constexpr (!WRITE) { a.counts[2 * blk] = ng; a.counts[2 * blk + 1] = nh; }
}

// ------------------------------------------------------------------------------------------------ chunks
struct ChunkArgs {
    const int32_t* ptr; const int32_t* ind;
    const int32_t* heavy; int64_t n_heavy;      // heavy[h] row ids; heavy + n_heavy: first slots (writing pass)
    int chunk, min_chunk, wshift;
    int64_t* counts;                            // [n_heavy] chunks per heavy row (counting pass)
    int32_t* rm; uint32_t* key; int32_t* idx;   // row-major chunk list, sort keys, identity permutation (writing pass)
    Counters* ctr;
};

__device__ __forceinline__ uint32_t window_key(int32_t v, int wshift) {
    const uint32_t mag = v >= 0 ? (uint32_t)v : (uint32_t)(-1 - v);
    return ((mag >> wshift) << 1) | (v < 0 ? 1u : 0u);
}

template <bool WRITE>
__global__ __launch_bounds__(256) void plan_chunks_kernel(ChunkArgs a) {
    const int lane = threadIdx.x & 63;
    const int64_t h = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (h >= a.n_heavy) return;
    const int32_t r = a.heavy[h];
    const int b = a.ptr[r], e = a.ptr[r + 1];
    const int slot0 = WRITE ? a.heavy[a.n_heavy + h] : 0;
    int n = 0;                                   // chunks so far (wavefront-uniform)
    uint32_t maxw = 0;
    auto emit = [&](int s, int p) {              // [s, p) in pieces of at most `chunk`
        const int np = (p - s + a.chunk - 1) / a.chunk;
        if constexpr (WRITE) {
            for (int j = lane; j < np; j += 64) {
                const int k = s + j * a.chunk;
                const int at = slot0 + n + j;
                a.rm[3 * (int64_t)at] = at;
                a.rm[3 * (int64_t)at + 1] = k;
                a.rm[3 * (int64_t)at + 2] = min(k + a.chunk, p);
                a.key[at] = a.wshift < 0 ? 0u : window_key(a.ind[k], a.wshift);
                a.idx[at] = at;
            }
        }
        n += np;
    };
    int start = b;
    if (a.wshift >= 0) {
        uint32_t carry = 0;
        for (int t = b; t < e; t += 64) {
            const int k = t + lane;
            const uint32_t w = k < e ? window_key(a.ind[k], a.wshift) : 0u;
            uint32_t prev = __shfl_up(w, 1, 64);
            if (lane == 0) prev = carry;
            carry = __shfl(w, 63, 64);
            maxw = max(maxw, w);
            unsigned long long m = __ballot(k < e && k > b && w != prev);
            while (m) {                          // the positions where the window changes, ascending
                const int pos = t + __builtin_ctzll(m);
                m &= m - 1;
                if (pos - start >= a.min_chunk) { emit(start, pos); start = pos; }
            }
        }
    }
    emit(start, e);
    if constexpr (!WRITE) {
        if (lane == 0) a.counts[h] = n;
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) maxw = max(maxw, (uint32_t)__shfl_xor((int)maxw, off, 64));
        if (lane == 0 && maxw > 0) atomicMax(&a.ctr->max_key, maxw);
    }
}

__global__ __launch_bounds__(256) void plan_gather_chunks_kernel(const int32_t* __restrict__ rm,
                                                                 const int32_t* __restrict__ idx, int64_t n,
                                                                 int32_t* __restrict__ chunk) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    const int64_t src = idx[i];
#pragma unroll
    for (int q = 0; q < 3; ++q) chunk[3 * i + q] = rm[3 * src + q];
}

// ------------------------------------------------------------------------------------------------ ranges
// pre[0..ng]: exclusive prefix of the group costs, pre[ng] = total.  xcd_start[x] = lower bound of total * x / 8.
__global__ __launch_bounds__(256) void plan_xcd_kernel(const int64_t* __restrict__ pre, int64_t ng, Counters* ctr) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i > ng) return;
    const int64_t total = pre[ng];
    if (i == 0) { ctr->xcd_start[0] = 0; ctr->xcd_start[8] = ng; }
    const int64_t here = pre[i], before = i > 0 ? pre[i - 1] : -1;
#pragma unroll
    for (int x = 1; x < 8; ++x) {
        const int64_t target = total * x / 8;
        if (here >= target && before < target) ctr->xcd_start[x] = i;
    }
}

// sampled share of the entries of light rows that name a row of their own XCD range
__global__ __launch_bounds__(256) void plan_vote_kernel(const int32_t* __restrict__ ptr, const int32_t* __restrict__ ind,
                                                        const int32_t* __restrict__ group, Counters* ctr) {
    const int x = blockIdx.y;
    const int64_t lo = ctr->xcd_start[x], hi = ctr->xcd_start[x + 1];
    if (lo >= hi) return;
    const int64_t step = max((int64_t)1, (hi - lo) / 4096);
    const int64_t i = lo + ((int64_t)blockIdx.x * 256 + threadIdx.x) * step;
    if (i >= hi) return;
    const int32_t r0 = group[2 * lo], r1 = group[2 * (hi - 1) + 1];
    unsigned long long local = 0, seen = 0;
    for (int32_t k = ptr[group[2 * i]]; k < ptr[group[2 * i + 1]]; ++k) {
        ++seen;
        local += ind[k] >= r0 && ind[k] < r1;
    }
    if (seen) { atomicAdd(&ctr->seen, seen); atomicAdd(&ctr->local, local); }
}

__global__ void plan_init_counters_kernel(Counters* c) {
    if (threadIdx.x == 0 && blockIdx.x == 0) {
        Counters z = {};
        z.bad_row = ~0ull;
        *c = z;
    }
}

// device memory of one plan creation, freed when the builder leaves
struct Scratch {
    std::vector<void*> owned;
    ~Scratch() { for (void* p : owned) (void)hipFree(p); }
    template <class T> hipError_t get(T** out, int64_t count) {
        *out = nullptr;
        void* p = nullptr;
        const hipError_t e = hipMalloc(&p, (size_t)std::max<int64_t>(count, 1) * sizeof(T));
        if (e == hipSuccess) { owned.push_back(p); *out = static_cast<T*>(p); }
        return e;
    }
};

#define PLAN_HIP(expr)                                                                              \
    do {                                                                                            \
        const hipError_t e_ = (expr);                                                               \
        if (e_ != hipSuccess) {                                                                     \
            gas_plan_destroy(p);                                                                    \
            return fail(e_ == hipErrorOutOfMemory ? GAS_ERR_NOMEM : GAS_ERR_HIP, "gas_plan_create: %s: %s", #expr, \
                        hipGetErrorString(e_));                                                     \
        }                                                                                           \
    } while (0)

gas_status build_on_device(gas_plan* p, const int32_t* ptr, const int32_t* ind, int64_t n_rows, int64_t nnz,
                           const PlanParams& pp, hipStream_t s) {
    Scratch tmp;
    const int wshift = ind ? pp.wshift : -1;
    const int64_t n_blocks = (n_rows + kRowsPerBlock - 1) / kRowsPerBlock;
    Counters* ctr;
    int64_t *counts, *tiles;
    PLAN_HIP(tmp.get(&ctr, 1));
    PLAN_HIP(tmp.get(&counts, 2 * n_blocks));
    PLAN_HIP(tmp.get(&tiles, (std::max<int64_t>(n_rows, 2 * n_blocks) + kScanTile - 1) / kScanTile + 1));
    hipLaunchKernelGGL(plan_init_counters_kernel, dim3(1), dim3(64), 0, s, ctr);
    // ---- rows: count, scan, (read back), write
    RowsArgs ra = {ptr, n_rows, nnz, pp.threshold, counts, nullptr, nullptr, ctr};
    const unsigned row_grid = (unsigned)((n_blocks + 3) / 4);
    if (n_blocks > 0) hipLaunchKernelGGL(plan_rows_kernel<false>, dim3(row_grid), dim3(256), 0, s, ra);
    device_scan(StridedIn{counts, 2}, n_blocks, StridedOut{counts, 2}, tiles, &ctr->n_groups, s);
    device_scan(StridedIn{counts + 1, 2}, n_blocks, StridedOut{counts + 1, 2}, tiles, &ctr->n_heavy, s);
    Counters h;
    PLAN_HIP(hipMemcpyAsync(&h, ctr, sizeof(Counters), hipMemcpyDeviceToHost, s));
    PLAN_HIP(hipStreamSynchronize(s));
    if (h.bad_ends) {
        gas_plan_destroy(p);
        return fail(GAS_ERR_ARG, "gas_plan_create: ptr[0] or ptr[n_rows] do not match nnz=%lld", (long long)nnz);
    }
    if (h.bad_row != ~0ull) {
        gas_plan_destroy(p);
        return fail(GAS_ERR_ARG, "gas_plan_create: ptr decreases or leaves [0, nnz] at row %lld", (long long)(h.bad_row - 1));
    }
    p->n_groups = h.n_groups; p->n_heavy = h.n_heavy;
    if (p->n_groups > 0) PLAN_HIP(hipMalloc(&p->d_group, 2 * p->n_groups * sizeof(int32_t)));
    if (p->n_heavy > 0) PLAN_HIP(hipMalloc(&p->d_heavy, (2 * p->n_heavy + 1) * sizeof(int32_t)));
    ra.group = p->d_group; ra.heavy = p->d_heavy;
    if (n_blocks > 0) hipLaunchKernelGGL(plan_rows_kernel<true>, dim3(row_grid), dim3(256), 0, s, ra);
    // ---- chunks of the heavy rows: count, scan
    ChunkArgs ca = {ptr, ind, p->d_heavy, p->n_heavy, pp.chunk, pp.min_chunk, wshift, nullptr, nullptr, nullptr, nullptr, ctr};
    const unsigned heavy_grid = (unsigned)((p->n_heavy + 3) / 4);
    if (p->n_heavy > 0) {
        PLAN_HIP(tmp.get(&ca.counts, p->n_heavy));
        hipLaunchKernelGGL(plan_chunks_kernel<false>, dim3(heavy_grid), dim3(256), 0, s, ca);
        device_scan(StridedIn{ca.counts, 1}, p->n_heavy, FirstSlotOut{p->d_heavy + p->n_heavy, p->n_heavy}, tiles,
                    &ctr->n_chunks, s);
    }
    // ---- ranges of groups per XCD and the locality vote
    int64_t* pre = nullptr;
    if (p->n_groups > 0) {
        PLAN_HIP(tmp.get(&pre, p->n_groups + 1));
        device_scan(GroupCostIn{ptr, p->d_group}, p->n_groups, PlainOut{pre}, tiles, pre + p->n_groups, s);
        hipLaunchKernelGGL(plan_xcd_kernel, dim3((unsigned)((p->n_groups + 256) / 256)), dim3(256), 0, s, pre, p->n_groups, ctr);
        if (pp.xcd_mode == 0 && ind)
            hipLaunchKernelGGL(plan_vote_kernel, dim3(32, 8), dim3(256), 0, s, ptr, ind, p->d_group, ctr);
    }
    PLAN_HIP(hipMemcpyAsync(&h, ctr, sizeof(Counters), hipMemcpyDeviceToHost, s));
    PLAN_HIP(hipStreamSynchronize(s));
    p->n_chunks = h.n_chunks;
    for (int x = 0; x < 9; ++x) p->xcd_start[x] = p->n_groups > 0 ? h.xcd_start[x] : 0;
    p->xcd_ranges = p->n_groups > 0 && (pp.xcd_mode == 1 || (pp.xcd_mode == 0 && h.seen > 0 && 10 * h.local >= 3 * h.seen));
    // ---- chunk list: write row-major, order by window, gather
    if (p->n_chunks > 0) {
        if (p->n_chunks > 0x7FFFFFF0LL / 3) {
            gas_plan_destroy(p);
            return fail(GAS_ERR_ARG, "gas_plan_create: %lld chunks are too many for 32-bit positions", (long long)p->n_chunks);
        }
        PLAN_HIP(hipMalloc(&p->d_chunk, 3 * p->n_chunks * sizeof(int32_t)));
        uint32_t *key_a, *key_b;
        int32_t *idx_a, *idx_b;
        PLAN_HIP(tmp.get(&ca.rm, 3 * p->n_chunks));
        PLAN_HIP(tmp.get(&key_a, p->n_chunks));
        PLAN_HIP(tmp.get(&key_b, p->n_chunks));
        PLAN_HIP(tmp.get(&idx_a, p->n_chunks));
        PLAN_HIP(tmp.get(&idx_b, p->n_chunks));
        int64_t* sort_tiles;
        PLAN_HIP(tmp.get(&sort_tiles, (p->n_chunks + kScanTile - 1) / kScanTile + 1));
        ca.key = key_a; ca.idx = idx_a;
        hipLaunchKernelGGL(plan_chunks_kernel<true>, dim3(heavy_grid), dim3(256), 0, s, ca);
        int bits = 0;
        while (bits < 32 && (h.max_key >> bits) != 0) ++bits;
        for (int bit = 0; bit < bits; ++bit) {
            device_scan(BitZeroIn{key_a, bit}, p->n_chunks, SplitOut{key_a, idx_a, key_b, idx_b, &ctr->zeros}, sort_tiles,
                        &ctr->zeros, s);
            std::swap(key_a, key_b);
            std::swap(idx_a, idx_b);
        }
        hipLaunchKernelGGL(plan_gather_chunks_kernel, dim3((unsigned)((p->n_chunks + 255) / 256)), dim3(256), 0, s, ca.rm,
                           idx_a, p->n_chunks, p->d_chunk);
        PLAN_HIP(hipMalloc(&p->d_partial, (size_t)p->n_chunks * p->max_F * sizeof(float)));
    }
    PLAN_HIP(hipGetLastError());
    PLAN_HIP(hipStreamSynchronize(s));           // the temporaries are freed when `tmp` goes out of scope
    return GAS_OK;
}

gas_status build_on_host(gas_plan* p, const int32_t* ptr, const int32_t* ind, int64_t n_rows, int64_t nnz,
                         const PlanParams& pp, hipStream_t s) {
    std::vector<int32_t> h_ptr((size_t)n_rows + 1, 0), h_ind;
    if (n_rows > 0) {
        PLAN_HIP(hipMemcpyAsync(h_ptr.data(), ptr, sizeof(int32_t) * (n_rows + 1), hipMemcpyDeviceToHost, s));
        PLAN_HIP(hipStreamSynchronize(s));
        const int64_t bad = plan_validate_ptr(h_ptr.data(), n_rows, nnz);
        if (bad) {
            gas_plan_destroy(p);
            if (bad > n_rows)
                return fail(GAS_ERR_ARG, "gas_plan_create: ptr[0] or ptr[n_rows] do not match nnz=%lld", (long long)nnz);
            return fail(GAS_ERR_ARG, "gas_plan_create: ptr decreases or leaves [0, nnz] at row %lld", (long long)(bad - 1));
        }
    }
    if (ind && nnz > 0) {
        h_ind.resize((size_t)nnz);
        PLAN_HIP(hipMemcpyAsync(h_ind.data(), ind, sizeof(int32_t) * nnz, hipMemcpyDeviceToHost, s));
        PLAN_HIP(hipStreamSynchronize(s));
    }
    PlanArrays pa;
    build_plan_host(h_ptr.data(), h_ind.empty() ? nullptr : h_ind.data(), n_rows, nnz, pp, pa);
    p->n_heavy = pa.n_heavy; p->n_chunks = pa.n_chunks; p->n_groups = pa.n_groups;
    p->xcd_ranges = pa.xcd_ranges;
    for (int x = 0; x < 9; ++x) p->xcd_start[x] = pa.xcd_start[x];
    auto upload = [&](int32_t** dst, const std::vector<int32_t>& v) -> hipError_t {
        if (v.empty()) return hipSuccess;
        hipError_t r = hipMalloc(dst, v.size() * sizeof(int32_t));
        if (r == hipSuccess) r = hipMemcpyAsync(*dst, v.data(), v.size() * sizeof(int32_t), hipMemcpyHostToDevice, s);
        return r;
    };
    PLAN_HIP(upload(&p->d_group, pa.group));
    PLAN_HIP(upload(&p->d_chunk, pa.chunk));
    PLAN_HIP(upload(&p->d_heavy, pa.heavy));
    if (p->n_chunks > 0) PLAN_HIP(hipMalloc(&p->d_partial, (size_t)p->n_chunks * p->max_F * sizeof(float)));
    PLAN_HIP(hipStreamSynchronize(s));
    return GAS_OK;
}

}  // namespace
}  // namespace gas

using namespace gas;

extern "C" {

gas_status gas_plan_create_opt(const int32_t* ptr, const int32_t* ind, int64_t n_rows, int64_t nnz, int32_t max_F,
                               const gas_plan_options* opt, void* stream, gas_plan** out) {
    GAS_REQUIRE(out, "gas_plan_create: null output");
    *out = nullptr;
    GAS_REQUIRE(n_rows >= 0 && n_rows < 0x7FFFFFF0LL && nnz >= 0 && nnz < 0x7FFFFFF0LL && max_F > 0,
                "gas_plan_create: n_rows=%lld nnz=%lld max_F=%d", (long long)n_rows, (long long)nnz, max_F);
    GAS_REQUIRE(ptr || n_rows == 0, "gas_plan_create: null row pointer array");
    PlanParams pp;
    pp.wshift = plan_default_wshift(max_F);
    bool host_builder = false;
    if (opt) {
        GAS_REQUIRE(opt->heavy_threshold >= 0 && opt->chunk >= 0 && opt->min_chunk >= 0 && opt->window_rows >= -1 &&
                    opt->xcd_ranges >= 0 && opt->xcd_ranges <= 2 && opt->host_builder >= 0 && opt->host_builder <= 1,
                    "gas_plan_create: options out of range (threshold %d, chunk %d, min_chunk %d, window_rows %d, "
                    "xcd_ranges %d, host_builder %d)", opt->heavy_threshold, opt->chunk, opt->min_chunk,
                    opt->window_rows, opt->xcd_ranges, opt->host_builder);
        if (opt->heavy_threshold > 0) pp.threshold = opt->heavy_threshold;
        if (opt->chunk > 0) pp.chunk = opt->chunk;
        if (opt->min_chunk > 0) pp.min_chunk = opt->min_chunk;
        if (opt->window_rows < 0) pp.wshift = -1;
        else if (opt->window_rows > 0) {                 // rounded down to a power of two
            pp.wshift = 0;
            while ((2ll << pp.wshift) <= opt->window_rows) ++pp.wshift;
        }
        pp.xcd_mode = opt->xcd_ranges;
        host_builder = opt->host_builder != 0;
    }
    static_assert(kRowsPerBlock == 1024, "the device builder's blocks are the host builder's group_block");
    pp.group_block = kRowsPerBlock;
    gas_plan* p = new gas_plan();
    p->n_rows = n_rows; p->nnz = nnz; p->max_F = max_F;
    p->threshold = pp.threshold; p->chunk = pp.chunk;
    (void)hipGetDevice(&p->device);
    const gas_status st = host_builder ? build_on_host(p, ptr, ind, n_rows, nnz, pp, (hipStream_t)stream)
                                       : build_on_device(p, ptr, ind, n_rows, nnz, pp, (hipStream_t)stream);
    if (st != GAS_OK) return st;                 // p has been destroyed
    *out = p;
    return GAS_OK;
}

gas_status gas_plan_create(const int32_t* ptr, const int32_t* ind, int64_t n_rows, int64_t nnz, int32_t max_F,
                           void* stream, gas_plan** out) {
    return gas_plan_create_opt(ptr, ind, n_rows, nnz, max_F, nullptr, stream, out);
}

void gas_plan_destroy(gas_plan* p) {
    if (!p) return;
    if (p->d_chunk) (void)hipFree(p->d_chunk);
    if (p->d_heavy) (void)hipFree(p->d_heavy);
    if (p->d_partial) (void)hipFree(p->d_partial);
    if (p->d_group) (void)hipFree(p->d_group);
    delete p;
}

gas_status gas_plan_describe(const gas_plan* plan, int64_t info[16]) {
    GAS_REQUIRE(plan && info, "gas_plan_describe: null pointer");
    info[0] = plan->n_rows; info[1] = plan->nnz; info[2] = plan->n_groups; info[3] = plan->n_heavy;
    info[4] = plan->n_chunks; info[5] = plan->xcd_ranges; info[6] = plan->max_F;
    for (int x = 0; x < 9; ++x) info[7 + x] = plan->xcd_start[x];
    return GAS_OK;
}

gas_status gas_plan_copy_lists(const gas_plan* plan, int32_t* group, int32_t* heavy, int32_t* chunk, void* stream) {
    GAS_REQUIRE(plan, "gas_plan_copy_lists: null plan");
    hipStream_t s = (hipStream_t)stream;
    if (group && plan->n_groups > 0)
        GAS_CHECK_HIP(hipMemcpyAsync(group, plan->d_group, 2 * plan->n_groups * sizeof(int32_t), hipMemcpyDeviceToHost, s));
    if (heavy && plan->n_heavy > 0)
        GAS_CHECK_HIP(hipMemcpyAsync(heavy, plan->d_heavy, (2 * plan->n_heavy + 1) * sizeof(int32_t), hipMemcpyDeviceToHost, s));
    if (chunk && plan->n_chunks > 0)
        GAS_CHECK_HIP(hipMemcpyAsync(chunk, plan->d_chunk, 3 * plan->n_chunks * sizeof(int32_t), hipMemcpyDeviceToHost, s));
    GAS_CHECK_HIP(hipStreamSynchronize(s));
    return GAS_OK;
}

}  // extern "C"
