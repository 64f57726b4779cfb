// Helpers shared by the one-wavefront-per-row kernels (PNA and GAT aggregations and their backward passes):
// reductions over the 64 lanes and the 16-byte piece of a feature row that a lane owns.
#pragma once
#include "common.h"

namespace gas {

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
}

// Eight lane reductions at once: at each of the first three steps a lane keeps one half of its values, adds
// the partner's copy of that half and hands over the other half, so 4 + 2 + 1 exchanges leave one partial sum per
// lane; three more steps finish it, and the eight totals are read back from the lanes that hold them.  Ten
// exchanges instead of forty-eight.  Value j ends up in the lanes whose bits 5..3 spell j.
__device__ __forceinline__ void wave_sum8(float (&s)[8]) {
    const int lane = threadIdx.x & 63;
    float t4[4], t2[2];
    const bool h5 = lane & 32, h4 = lane & 16, h3 = lane & 8;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const float keep = h5 ? s[j + 4] : s[j], send = h5 ? s[j] : s[j + 4];
        t4[j] = keep + __shfl_xor(send, 32);
    }
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const float keep = h4 ? t4[j + 2] : t4[j], send = h4 ? t4[j] : t4[j + 2];
        t2[j] = keep + __shfl_xor(send, 16);
    }
    float t = (h3 ? t2[1] : t2[0]) + __shfl_xor(h3 ? t2[0] : t2[1], 8);
    t += __shfl_xor(t, 4);
    t += __shfl_xor(t, 2);
    t += __shfl_xor(t, 1);
    // lane bits (5, 4, 3) = (j >> 2 & 1, j >> 1 & 1, j & 1): value j sits in lanes 32 (j>>2&1) + 16 (j>>1&1) + 8 (j&1)
#pragma unroll
    for (int j = 0; j < 8; ++j)
        s[j] = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, t),
                                                                  32 * ((j >> 2) & 1) + 16 * ((j >> 1) & 1) + 8 * (j & 1)));
}

// Sum over the G lanes of a team: the wavefront's aligned groups of G lanes, G a power of two.
template <int G>
__device__ __forceinline__ float team_sum(float v) {
#pragma unroll
    for (int o = G / 2; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
}

// wave_sum8 inside every team of G = 16 or 32 lanes (G = 64: wave_sum8 itself): the same halving exchanges on the team's three upper lane
// bits, the remaining steps on the lower ones, and every lane reads the eight totals back from its own team.
template <int G>
__device__ __forceinline__ void team_sum8(float (&s)[8]) {
    static_assert(G == 16 || G == 32 || G == 64, "teams of 16, 32 or 64 lanes");
    if constexpr (G == 64) {
        wave_sum8(s);
        return;
    }
    const int lane = threadIdx.x & 63;
    float t4[4], t2[2];
    const bool ha = lane & (G / 2), hb = lane & (G / 4), hc = lane & (G / 8);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const float keep = ha ? s[j + 4] : s[j], send = ha ? s[j] : s[j + 4];
        t4[j] = keep + __shfl_xor(send, G / 2);
    }
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const float keep = hb ? t4[j + 2] : t4[j], send = hb ? t4[j] : t4[j + 2];
        t2[j] = keep + __shfl_xor(send, G / 4);
    }
    float t = (hc ? t2[1] : t2[0]) + __shfl_xor(hc ? t2[0] : t2[1], G / 8);
#pragma unroll
    for (int o = G / 16; o > 0; o >>= 1) t += __shfl_xor(t, o);
    const int base = lane & ~(G - 1);
#pragma unroll
    for (int j = 0; j < 8; ++j)
        s[j] = __shfl(t, base + (G / 2) * ((j >> 2) & 1) + (G / 4) * ((j >> 1) & 1) + (G / 8) * (j & 1));
}

// ---- rows too long for one wavefront
// The one-wavefront-per-row kernels leave a row of more than kLongRow entries to a second launch of kLongBlocks
// workgroups of kLongWaves wavefronts, which take the row's blocks of 64 entries in turn: a hub row of 17,000
// entries is thousands of dependent steps for one wavefront, which the whole launch would wait for.
constexpr int kLongRow = 2048;
constexpr int kLongWaves = 8;
constexpr int kLongBlocks = 2048;                     // 512, 8,192 and 32,768 were measured slower
inline unsigned long_row_blocks(int64_t n_rows) { return (unsigned)(n_rows < kLongBlocks ? n_rows : kLongBlocks); }

// Workgroup w of such a launch looks at the rows w, w + gridDim.x, ..., blockDim.x of them per call (r0 = w, then
// + blockDim.x * gridDim.x): the long ones among them are left in queue[0 .. return value).  Called by every thread
// of the workgroup; the caller passes a barrier between its last use of the queue and the next call.
__device__ __forceinline__ int queue_long_rows(const int32_t* rowptr, int64_t n_rows, int64_t r0, int* queue, int* n_queued,
                                               int longer_than = kLongRow) {
    if (threadIdx.x == 0) *n_queued = 0;
    __syncthreads();
    const int64_t r = r0 + (int64_t)threadIdx.x * gridDim.x;
    if (r < n_rows && rowptr[r + 1] - rowptr[r] > longer_than) queue[atomicAdd(n_queued, 1)] = (int)r;
    __syncthreads();
    return *n_queued;
}

// A value that is the same in all lanes of a wavefront, summed (or its maximum taken) over the W wavefronts of
// the workgroup in wavefront order; every thread of the workgroup calls it.
template <int W, bool MAX>
__device__ __forceinline__ float across_waves(float x, float* red) {
    if constexpr (W == 1) return x;
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = x;
    __syncthreads();
    float r = red[0];
#pragma unroll
    for (int o = 1; o < W; ++o) r = MAX ? fmaxf(r, red[o]) : r + red[o];
    __syncthreads();
    return r;
}

// elements in a 16-byte piece
template <bool BF> struct Elems { static constexpr int E = BF ? 8 : 4; };

template <bool BF>
__device__ __forceinline__ void unpack(const u32x4& r, float (&x)[Elems<BF>::E]) {
    if constexpr (BF) {
#pragma unroll
        for (int i = 0; i < 4; ++i) { x[2 * i] = bf16_lo(r[i]); x[2 * i + 1] = bf16_hi(r[i]); }
    } else {
#pragma unroll
        for (int i = 0; i < 4; ++i) x[i] = __uint_as_float(r[i]);
    }
}
template <bool BF>
__device__ __forceinline__ u32x4 pack(const float (&x)[Elems<BF>::E]) {
    if constexpr (BF) return u32x4{pack_bf16(x[0], x[1]), pack_bf16(x[2], x[3]), pack_bf16(x[4], x[5]), pack_bf16(x[6], x[7])};
    else return u32x4{__float_as_uint(x[0]), __float_as_uint(x[1]), __float_as_uint(x[2]), __float_as_uint(x[3])};
}

}  // namespace gas
