// CPU-only checker of the plan builder (plan_host.h): builds plans for seeded random, edge-case and malformed
// patterns and checks the invariants the kernels rely on (an invalid plan would be an out-of-bounds access on the
// GPU).  Compiled with g++ -fsanitize=address,undefined and run by the CPU test suite; optionally reads a pattern
// from a file (int32 little-endian: n_rows, nnz, ptr[n_rows+1], ind[nnz]) given as the first argument.
#include <stdio.h>
#include <stdlib.h>

#include <string>

#include "plan_host.h"

using namespace gas;

static int failures = 0;
#define CHECK(cond, ...)                                   \
    do {                                                   \
        if (!(cond)) {                                     \
            ++failures;                                    \
            fprintf(stderr, "FAIL %s:%d: ", __FILE__, __LINE__); \
            fprintf(stderr, __VA_ARGS__);                  \
            fprintf(stderr, "\n");                         \
            return;                                        \
        }                                                  \
    } while (0)

static uint64_t rng_state = 1;
static uint64_t rnd() {                       // splitmix64
    uint64_t z = (rng_state += 0x9E3779B97F4A7C15ull);
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

static void check_plan(const char* what, const std::vector<int32_t>& ptr, const std::vector<int32_t>& ind, bool with_ind,
                       const PlanParams& pp) {
    const int64_t n_rows = (int64_t)ptr.size() - 1, nnz = ptr.empty() ? 0 : ptr.back();
    CHECK(plan_validate_ptr(ptr.data(), n_rows, nnz) == 0, "%s: valid ptr rejected", what);
    PlanArrays pa;
    build_plan_host(ptr.data(), with_ind ? ind.data() : nullptr, n_rows, nnz, pp, pa);
    const int wshift = with_ind ? pp.wshift : -1;
    // groups: exactly the light rows, in order, within the limits, inside one block
    CHECK((int64_t)pa.group.size() == 2 * pa.n_groups, "%s: group size", what);
    int64_t next_light = 0;
    auto skip_heavy = [&]() { while (next_light < n_rows && ptr[next_light + 1] - ptr[next_light] > pp.threshold) ++next_light; };
    skip_heavy();
    for (int64_t g = 0; g < pa.n_groups; ++g) {
        const int64_t r0 = pa.group[2 * g], r1 = pa.group[2 * g + 1];
        CHECK(r0 == next_light, "%s: group %lld starts at %lld, next light row is %lld", what, (long long)g, (long long)r0, (long long)next_light);
        CHECK(r1 > r0 && r1 <= n_rows && r1 - r0 <= 63, "%s: group %lld rows [%lld,%lld)", what, (long long)g, (long long)r0, (long long)r1);
        CHECK(r0 / pp.group_block == (r1 - 1) / pp.group_block, "%s: group %lld crosses a block", what, (long long)g);
        for (int64_t r = r0; r < r1; ++r)
            CHECK(ptr[r + 1] - ptr[r] <= pp.threshold, "%s: heavy row %lld in group", what, (long long)r);
        CHECK(r1 - r0 == 1 || ptr[r1] - ptr[r0] <= 64, "%s: group %lld has %d entries in %lld rows", what, (long long)g, ptr[r1] - ptr[r0], (long long)(r1 - r0));
        next_light = r1;
        skip_heavy();
    }
    CHECK(next_light == n_rows, "%s: light rows after %lld are in no group", what, (long long)next_light);
    // heavy rows and their chunk slots
    CHECK((int64_t)pa.heavy.size() == (pa.n_heavy ? 2 * pa.n_heavy + 1 : 0), "%s: heavy size", what);
    int64_t h = 0;
    for (int64_t r = 0; r < n_rows; ++r)
        if (ptr[r + 1] - ptr[r] > pp.threshold) {
            CHECK(h < pa.n_heavy && pa.heavy[h] == r, "%s: heavy row %lld missing", what, (long long)r);
            ++h;
        }
    CHECK(h == pa.n_heavy, "%s: %lld heavy rows listed, %lld exist", what, (long long)pa.n_heavy, (long long)h);
    CHECK((int64_t)pa.chunk.size() == 3 * pa.n_chunks, "%s: chunk size", what);
    std::vector<int64_t> at((size_t)pa.n_chunks, -1);           // slot -> position in processing order
    for (int64_t i = 0; i < pa.n_chunks; ++i) {
        const int32_t slot = pa.chunk[3 * i];
        CHECK(slot >= 0 && slot < pa.n_chunks && at[slot] < 0, "%s: slot %d twice or out of range", what, slot);
        at[slot] = i;
    }
    for (int64_t hh = 0; hh < pa.n_heavy; ++hh) {
        const int32_t r = pa.heavy[hh];
        const int32_t f0 = pa.heavy[pa.n_heavy + hh], f1 = pa.heavy[pa.n_heavy + hh + 1];
        CHECK(f0 < f1 && f1 <= pa.n_chunks, "%s: heavy row %d has slots [%d,%d)", what, r, f0, f1);
        int32_t cursor = ptr[r], run_start = ptr[r];
        for (int32_t sl = f0; sl < f1; ++sl) {
            const int64_t i = at[sl];
            const int32_t b = pa.chunk[3 * i + 1], e = pa.chunk[3 * i + 2];
            CHECK(b == cursor && e > b && e - b <= pp.chunk && e <= ptr[r + 1], "%s: row %d slot %d is [%d,%d), cursor %d", what, r, sl, b, e, cursor);
            if (e < ptr[r + 1] && e - b < pp.chunk) {
                // ended early: only at a window change, and only once min_chunk entries have gone by since the
                // last such cut (the run is then stored in pieces of at most `chunk`)
                CHECK(wshift >= 0 && plan_window(ind[e], wshift) != plan_window(ind[e - 1], wshift) &&
                      e - run_start >= pp.min_chunk, "%s: row %d chunk [%d,%d) ends for no reason", what, r, b, e);
                run_start = e;
            }
            cursor = e;
        }
        CHECK(cursor == ptr[r + 1], "%s: chunks of row %d stop at %d of %d", what, r, cursor, ptr[r + 1]);
    }
    if (pa.n_heavy) CHECK(pa.heavy[2 * pa.n_heavy] == pa.n_chunks, "%s: last first-slot", what);
    // processing order: by window of the first entry, stable
    for (int64_t i = 1; i < pa.n_chunks; ++i) {
        const int64_t k0 = wshift < 0 ? 0 : plan_window(ind[pa.chunk[3 * (i - 1) + 1]], wshift);
        const int64_t k1 = wshift < 0 ? 0 : plan_window(ind[pa.chunk[3 * i + 1]], wshift);
        CHECK(k0 < k1 || (k0 == k1 && pa.chunk[3 * (i - 1)] < pa.chunk[3 * i]), "%s: processing order broken at %lld", what, (long long)i);
    }
    for (int x = 0; x < 8; ++x) {
        CHECK(pa.xcd_start[x] <= pa.xcd_start[x + 1], "%s: group ranges", what);
    }
    CHECK(pa.xcd_start[0] == 0 && pa.xcd_start[8] == pa.n_groups, "%s: group range ends", what);
}

// power-law-ish row lengths, ascending columns with an optional negative (history) half
static void random_pattern(int64_t n_rows, int64_t n_cols, int max_len, bool fused, std::vector<int32_t>& ptr,
                           std::vector<int32_t>& ind) {
    ptr.assign(1, 0);
    ind.clear();
    for (int64_t r = 0; r < n_rows; ++r) {
        const double u = (double)(rnd() >> 11) / 9007199254740992.0;
        int64_t len = (int64_t)(1.0 / (u * u + 1.0 / max_len)) - 1;          // many short, a few long
        if (rnd() % 7 == 0) len = 0;
        if (len > n_cols) len = n_cols;
        // ascending distinct columns: sample by stepping
        int64_t c = 0;
        std::vector<int32_t> row;
        for (int64_t k = 0; k < len && c < n_cols; ++k) {
            const int64_t room = (n_cols - c) / (len - k);
            c += room > 1 ? (int64_t)(rnd() % room) : 0;
            row.push_back((int32_t)c);
            ++c;
        }
        if (fused) {                       // first the in-batch half (>= 0), then history rows (< 0, magnitudes ascending)
            const size_t half = row.size() / 2;
            for (size_t k = half; k < row.size(); ++k) row[k] = -1 - row[k];
        }
        ind.insert(ind.end(), row.begin(), row.end());
        ptr.push_back((int32_t)ind.size());
    }
}

static void from_file(const char* path) {
    FILE* f = fopen(path, "rb");
    if (!f) { fprintf(stderr, "cannot open %s\n", path); ++failures; return; }
    int32_t head[2];
    if (fread(head, 4, 2, f) != 2) { fclose(f); ++failures; return; }
    std::vector<int32_t> ptr((size_t)head[0] + 1), ind((size_t)head[1]);
    const bool ok = fread(ptr.data(), 4, ptr.size(), f) == ptr.size() && fread(ind.data(), 4, ind.size(), f) == ind.size();
    fclose(f);
    if (!ok) { fprintf(stderr, "short file %s\n", path); ++failures; return; }
    PlanParams pp;
    check_plan(path, ptr, ind, true, pp);
    PlanArrays pa;
    build_plan_host(ptr.data(), ind.data(), head[0], head[1], pp, pa);
    printf("%s: rows %d nnz %d -> groups %lld heavy %lld chunks %lld xcd_ranges %d\n", path, head[0], head[1],
           (long long)pa.n_groups, (long long)pa.n_heavy, (long long)pa.n_chunks, pa.xcd_ranges);
}

int main(int argc, char** argv) {
    if (argc > 1) {
        from_file(argv[1]);
        return failures ? 1 : 0;
    }
    std::vector<int32_t> ptr, ind;
    int cases = 0;
    // seeded random patterns under many parameter sets
    for (int seed = 1; seed <= 12; ++seed) {
        rng_state = seed;
        const int64_t n_rows = 1 + rnd() % 5000, n_cols = 64 + rnd() % 200000;
        random_pattern(n_rows, n_cols, 50 + (int)(rnd() % 3000), seed % 2 == 0, ptr, ind);
        for (int t : {1, 8, 64, 512})
            for (int ws : {-1, 0, 3, 11, 20})
                for (int mc : {1, 8, 300}) {
                    PlanParams pp;
                    pp.threshold = t; pp.chunk = t < 64 ? 32 : 256; pp.min_chunk = mc; pp.wshift = ws;
                    pp.group_block = seed % 3 == 0 ? 64 : 1024;
                    pp.xcd_mode = seed % 3;
                    check_plan(("random seed " + std::to_string(seed)).c_str(), ptr, ind, true, pp);
                    ++cases;
                }
        check_plan("random, no indices", ptr, ind, false, PlanParams());
        ++cases;
    }
    // edge cases
    PlanParams pp;
    check_plan("no rows", {0}, {}, true, pp);
    check_plan("one empty row", {0, 0}, {}, true, pp);
    check_plan("empty rows only", std::vector<int32_t>(2000, 0), {}, true, pp);
    for (int len : {63, 64, 65, 511, 512, 513, 20000}) {
        ptr = {0, 0, len, len, 2 * len, 2 * len + 1};
        ind.clear();
        for (int r = 0; r < 2; ++r)
            for (int k = 0; k < len; ++k) ind.push_back(k * 3);
        ind.push_back(7);
        check_plan(("rows of " + std::to_string(len)).c_str(), ptr, ind, true, pp);
        ++cases;
    }
    {   // 70 light rows of one entry each: groups close at 63 rows / 64 entries
        ptr.assign(1, 0); ind.clear();
        for (int r = 0; r < 5000; ++r) { ind.push_back(r); ptr.push_back((int32_t)ind.size()); }
        check_plan("one entry per row", ptr, ind, true, pp);
    }
    // malformed row pointers must be rejected before anything is indexed with them
    auto rejected = [&](std::vector<int32_t> p, int64_t nnz) { return plan_validate_ptr(p.data(), (int64_t)p.size() - 1, nnz) != 0; };
    if (!rejected({0, 1000, 600}, 600)) { ++failures; fprintf(stderr, "FAIL: interior pointer above nnz accepted\n"); }
    if (!rejected({0, 5, 3, 8}, 8)) { ++failures; fprintf(stderr, "FAIL: decreasing pointer accepted\n"); }
    if (!rejected({1, 5, 8}, 8)) { ++failures; fprintf(stderr, "FAIL: ptr[0] != 0 accepted\n"); }
    if (!rejected({0, 5, 8}, 9)) { ++failures; fprintf(stderr, "FAIL: ptr[n] != nnz accepted\n"); }
    if (!rejected({0, -5, 8}, 8)) { ++failures; fprintf(stderr, "FAIL: negative pointer accepted\n"); }
    if (rejected({0, 5, 5, 8}, 8)) { ++failures; fprintf(stderr, "FAIL: valid pointers rejected\n"); }
    printf("plan_check: %d cases, %d failures\n", cases, failures);
    return failures ? 1 : 0;
}
