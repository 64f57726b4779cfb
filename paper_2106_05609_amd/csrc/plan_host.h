// The schedule of one compressed sparse pattern (what a gas_plan holds), built on the host in plain C++.
//
// This is the definition of the plan: the device builder in plan.hip must produce the same arrays, and the tests
// compare the two.  The file has no HIP in it, so it also compiles with g++ alone (plan_check.cpp runs it under
// the address and undefined-behaviour sanitizers on edge-case and malformed patterns).
//
// Rules (all sizes in entries or rows):
//   * A row with more than `threshold` entries is HEAVY, the others are LIGHT.
//   * Light rows are bundled into GROUPS: runs of consecutive light rows inside one block of `group_block` rows,
//     closed greedily when adding the next row would exceed 64 entries or 63 rows; a light row with more than 64
//     entries is a group of its own.  A wavefront then always has a full load of indices to work on.
//   * A heavy row is cut into CHUNKS, one wavefront each, whose partial sums are added in chunk order afterwards.
//     The entry's WINDOW is (magnitude of its index >> wshift) * 2 + (index < 0): a range of 2^wshift rows of one of
//     the two source tables, sized to fit one L2.  Walking the row, a chunk ends where the window changes if the
//     chunk has at least `min_chunk` entries by then, and in any case after `chunk` entries.  So where a row is
//     dense in a window its chunk gathers from that window only; in the sparse tail of the columns a chunk spans
//     several windows instead of shrinking below `min_chunk` entries (its partial sum would cost more than the
//     reuse saves).  wshift < 0 turns windows off (chunks of `chunk` entries).
//   * The chunks are processed in the order of their first entry's window (stable: chunks of one window keep their
//     row-major order).  Workgroups take them four at a time and go to the XCDs in turn, so all eight XCDs walk
//     the window sequence together and the window they are in fits every L2.  (Giving each XCD a range of windows
//     of its own fetches each source row into one L2 only, but the XCDs that get the sparse tail then wait on
//     their own eighth of the fabric while the others sit idle: measured slower.)  The partial sums keep their
//     row-major slots, so the order in which a row's partials are added does not depend on the processing order.
//   * The groups are also cut into eight contiguous ranges of equal cost; whether the rows kernel uses them
//     (xcd_ranges) is decided from the pattern: at least 30 % of the sampled entries of a range must name a row
//     of that range (a batch made of partition clusters does that, a graph without communities does not).
#pragma once
#include <stdint.h>

#include <algorithm>
#include <vector>

namespace gas {

struct PlanParams {
    int32_t threshold = 512;
    int32_t chunk = 256;
    int32_t min_chunk = 32;
    int32_t wshift = 11;        // 2048 rows per window; < 0: no windows
    int32_t xcd_mode = 0;       // 0 decide from the pattern, 1 always, 2 never
    int32_t group_block = 1024;
};

struct PlanArrays {
    std::vector<int32_t> group;       // [2 * n_groups] first and end row
    std::vector<int32_t> heavy;       // [n_heavy] row ids, then [n_heavy + 1] first chunk slot of each
    std::vector<int32_t> chunk;       // [3 * n_chunks] slot, begin, end, in processing order
    int64_t n_groups = 0, n_heavy = 0, n_chunks = 0;
    int64_t xcd_start[9] = {0};       // groups
    int32_t xcd_ranges = 0;
};

static inline int64_t plan_mag(int32_t v) { return v >= 0 ? (int64_t)v : -1 - (int64_t)v; }
static inline int64_t plan_window(int32_t v, int wshift) {
    return wshift < 0 ? 0 : ((plan_mag(v) >> wshift) << 1) | (v < 0 ? 1 : 0);
}

// Default window: rows of max_F floats worth 2 MiB (half of one XCD's L2), as a power of two.
static inline int32_t plan_default_wshift(int32_t max_F) {
    int64_t rows = (2ll << 20) / ((int64_t)max_F * 4);
    int32_t s = 0;
    while ((2ll << s) <= rows) ++s;
    return s < 6 ? 6 : (s > 20 ? 20 : s);
}

// 0 on success; otherwise the first row whose pointers are wrong, plus one (ptr[0] != 0 and ptr[n_rows] != nnz
// report n_rows + 1 and n_rows + 2).
static inline int64_t plan_validate_ptr(const int32_t* ptr, int64_t n_rows, int64_t nnz) {
    if (n_rows == 0) return 0;
    if (ptr[0] != 0) return n_rows + 1;
    if (ptr[n_rows] != nnz) return n_rows + 2;
    for (int64_t r = 0; r < n_rows; ++r)
        if (ptr[r] < 0 || ptr[r + 1] < ptr[r] || ptr[r + 1] > nnz) return r + 1;
    return 0;
}

// ptr must have passed plan_validate_ptr.  ind may be null (then no windows and no locality vote).
static inline void build_plan_host(const int32_t* ptr, const int32_t* ind, int64_t n_rows, int64_t nnz,
                                   const PlanParams& pp, PlanArrays& out) {
    (void)nnz;
    out = PlanArrays();
    const int wshift = ind ? pp.wshift : -1;
    // ---- groups of light rows, heavy rows
    std::vector<int32_t> heavy_row;
    for (int64_t r0 = 0; r0 < n_rows; r0 += pp.group_block) {
        const int64_t r1 = std::min<int64_t>(n_rows, r0 + pp.group_block);
        int64_t g_start = -1;
        int32_t g_entries = 0;
        auto close = [&](int64_t end_row) {
            if (g_start >= 0) { out.group.push_back((int32_t)g_start); out.group.push_back((int32_t)end_row); }
            g_start = -1; g_entries = 0;
        };
        for (int64_t r = r0; r < r1; ++r) {
            const int32_t len = ptr[r + 1] - ptr[r];
            if (len > pp.threshold) {
                close(r);
                heavy_row.push_back((int32_t)r);
            } else {
                if (g_start >= 0 && (g_entries + len > 64 || r - g_start >= 63)) close(r);
                if (g_start < 0) g_start = r;
                g_entries += len;
            }
        }
        close(r1);
    }
    out.n_groups = (int64_t)out.group.size() / 2;
    out.n_heavy = (int64_t)heavy_row.size();
    // ---- chunks of the heavy rows, row-major
    std::vector<int32_t> rm;            // [3 * n] slot, begin, end
    std::vector<int64_t> key;           // window of the first entry
    std::vector<int32_t> first;
    for (int32_t r : heavy_row) {
        first.push_back((int32_t)(rm.size() / 3));
        const int32_t b = ptr[r], e = ptr[r + 1];
        auto emit = [&](int32_t s, int32_t p) {          // [s, p) in pieces of at most `chunk`
            for (int32_t k = s; k < p; k += pp.chunk) {
                rm.push_back((int32_t)(rm.size() / 3));
                rm.push_back(k);
                rm.push_back(std::min(k + pp.chunk, p));
                key.push_back(wshift < 0 ? 0 : plan_window(ind[k], wshift));
            }
        };
        int32_t start = b;
        if (wshift >= 0)
            for (int32_t k = b + 1; k < e; ++k)
                if (plan_window(ind[k], wshift) != plan_window(ind[k - 1], wshift) && k - start >= pp.min_chunk) {
                    emit(start, k);
                    start = k;
                }
        emit(start, e);
    }
    out.n_chunks = (int64_t)rm.size() / 3;
    first.push_back((int32_t)out.n_chunks);
    out.heavy = heavy_row;
    if (out.n_heavy > 0) out.heavy.insert(out.heavy.end(), first.begin(), first.end());
    // ---- processing order: stable by window
    std::vector<int64_t> order((size_t)out.n_chunks);
    for (int64_t i = 0; i < out.n_chunks; ++i) order[i] = i;
    std::stable_sort(order.begin(), order.end(), [&](int64_t a, int64_t b) { return key[a] < key[b]; });
    out.chunk.resize(rm.size());
    for (int64_t i = 0; i < out.n_chunks; ++i)
        for (int q = 0; q < 3; ++q) out.chunk[3 * i + q] = rm[3 * order[i] + q];
    // ---- eight ranges of groups of equal cost (entries gathered + rows written), and whether to use them
    if (out.n_groups > 0) {
        const int64_t ng = out.n_groups;
        std::vector<int64_t> cost((size_t)ng + 1, 0);
        for (int64_t i = 0; i < ng; ++i)
            cost[i + 1] = cost[i] + (ptr[out.group[2 * i + 1]] - ptr[out.group[2 * i]]) +
                          (out.group[2 * i + 1] - out.group[2 * i]);
        for (int x = 0; x <= 8; ++x) {
            const int64_t target = cost[ng] * x / 8;
            out.xcd_start[x] = x == 8 ? ng : std::lower_bound(cost.begin(), cost.end(), target) - cost.begin();
        }
        out.xcd_ranges = pp.xcd_mode == 1;
        if (pp.xcd_mode == 0 && ind) {
            int64_t local = 0, seen = 0;
            for (int x = 0; x < 8; ++x) {
                if (out.xcd_start[x] >= out.xcd_start[x + 1]) continue;
                const int64_t r0 = out.group[2 * out.xcd_start[x]], r1 = out.group[2 * (out.xcd_start[x + 1] - 1) + 1];
                const int64_t step = std::max<int64_t>(1, (out.xcd_start[x + 1] - out.xcd_start[x]) / 4096);   // sample
                for (int64_t i = out.xcd_start[x]; i < out.xcd_start[x + 1]; i += step)
                    for (int32_t k = ptr[out.group[2 * i]]; k < ptr[out.group[2 * i + 1]]; ++k) {
                        ++seen;
                        local += ind[k] >= r0 && ind[k] < r1;
                    }
            }
            out.xcd_ranges = seen > 0 && 10 * local >= 3 * seen;
        }
    }
}

}  // namespace gas
