// Host-side check of the file-backed history table (disk.hip) under the sanitizers: tables are created, written,
// read back and compared through index lists, ranges and strides, with several I/O threads, in both I/O modes, and
// the error paths are taken.  No GPU is involved (the device transfers are covered by the GPU tests); this file
// stands in for the rest of the library, so it defines the two error helpers disk.hip needs.
// Built and run by tests/test_disk_sanitizers.py, once with -fsanitize=address,undefined and once with
// -fsanitize=thread on the host side.
#include <stdarg.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
#include <unistd.h>

#include <string>
#include <vector>

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
}  // namespace gas

static int failures = 0;
#define EXPECT(cond)                                                                 \
    do {                                                                             \
        if (!(cond)) {                                                               \
            printf("line %d: %s (%s)\n", __LINE__, #cond, gas::last_error_buffer()); \
            ++failures;                                                              \
        }                                                                            \
    } while (0)

static uint64_t state = 12345;
static uint32_t rnd() {
    state = state * 6364136223846793005ull + 1442695040888963407ull;
    return (uint32_t)(state >> 33);
}

static void round_trip(const std::string& path, int64_t n_rows, int32_t F, gas_dtype dt, int flags, int threads) {
    const int es = dt == GAS_F32 ? 4 : 2;
    gas_disk_table* t = nullptr;
    EXPECT(gas_disk_open(path.c_str(), n_rows, F, dt, GAS_DISK_CREATE | flags, threads, 0, &t) == GAS_OK);
    if (!t) return;
    std::vector<unsigned char> model((size_t)(n_rows * F * es), 0);
    for (int sweep = 0; sweep < 4; ++sweep) {
        // distinct rows: a stride walk plus one run of consecutive rows
        const int64_t n = n_rows / 2;
        std::vector<int32_t> idx((size_t)n);
        const int64_t step = 2, off = sweep & 1;
        for (int64_t i = 0; i < n; ++i) idx[(size_t)i] = (int32_t)((i * step + off) % n_rows);
        const int64_t ld = F + (sweep & 1 ? 3 : 0);
        std::vector<unsigned char> src((size_t)(n * ld * es));
        for (auto& b : src) b = (unsigned char)rnd();
        EXPECT(gas_disk_write_rows(t, idx.data(), 0, n, src.data(), ld) == GAS_OK);
        for (int64_t i = 0; i < n; ++i)
            memcpy(&model[(size_t)idx[(size_t)i] * F * es], &src[(size_t)(i * ld * es)], (size_t)F * es);
        // read back with duplicates, in any order
        const int64_t m = n_rows / 3 + 1;
        std::vector<int32_t> want((size_t)m);
        for (auto& v : want) v = (int32_t)(rnd() % (uint32_t)n_rows);
        std::vector<unsigned char> got((size_t)(m * F * es));
        EXPECT(gas_disk_read_rows(t, want.data(), 0, m, got.data(), F) == GAS_OK);
        bool same = true;
        for (int64_t i = 0; i < m && same; ++i)
            same = memcmp(&got[(size_t)(i * F * es)], &model[(size_t)want[(size_t)i] * F * es], (size_t)F * es) == 0;
        EXPECT(same);
    }
    std::vector<unsigned char> all(model.size());
    EXPECT(gas_disk_read_rows(t, nullptr, 0, n_rows, all.data(), F) == GAS_OK);
    EXPECT(all == model);
    // errors: out-of-range index and range, stride below the width, unknown ticket
    int32_t bad[3] = {0, (int32_t)n_rows, 1};
    EXPECT(gas_disk_read_rows(t, bad, 0, 3, all.data(), F) == GAS_ERR_RANGE);
    EXPECT(gas_disk_write_rows(t, nullptr, n_rows - 1, 2, all.data(), F) == GAS_ERR_RANGE);
    EXPECT(gas_disk_read_rows(t, nullptr, 0, 1, all.data(), F - 1) == GAS_ERR_ARG);
    EXPECT(gas_disk_wait(t, 7) == GAS_ERR_ARG);
    EXPECT(gas_disk_wait(t, 0) == GAS_OK);
    EXPECT(gas_disk_sync(t) == GAS_OK);
    EXPECT(gas_disk_close(t) == GAS_OK);
    // the file persists and can be opened again; another shape is refused
    EXPECT(gas_disk_open(path.c_str(), n_rows, F, dt, flags, threads, 0, &t) == GAS_OK);
    std::fill(all.begin(), all.end(), 0);
    EXPECT(gas_disk_read_rows(t, nullptr, 0, n_rows, all.data(), F) == GAS_OK);
    EXPECT(all == model);
    EXPECT(gas_disk_close(t) == GAS_OK);
    gas_disk_table* u = nullptr;
    EXPECT(gas_disk_open(path.c_str(), n_rows + 1, F, dt, flags, threads, 0, &u) == GAS_ERR_ARG && u == nullptr);
    unlink(path.c_str());
}

int main(int argc, char** argv) {
    const std::string dir = argc > 1 ? argv[1] : "/tmp";
    int cases = 0;
    for (int flags : {0, (int)GAS_DISK_CALLS})
        for (int threads : {1, 3, 8}) {
            round_trip(dir + "/disk_check_a.bin", 1000, 64, GAS_F32, flags, threads);
            round_trip(dir + "/disk_check_b.bin", 4099, 7, GAS_BF16, flags, threads);
            round_trip(dir + "/disk_check_c.bin", 20000, 100, GAS_F32, flags, threads);
            cases += 3;
        }
    gas_disk_table* t = nullptr;
    EXPECT(gas_disk_open((dir + "/no_such_dir/x.bin").c_str(), 4, 4, GAS_F32, GAS_DISK_CREATE, 0, 0, &t) == GAS_ERR_IO);
    EXPECT(gas_disk_open((dir + "/missing.bin").c_str(), 4, 4, GAS_F32, 0, 0, 0, &t) == GAS_ERR_IO);
    EXPECT(gas_disk_open(nullptr, 4, 4, GAS_F32, 0, 0, 0, &t) == GAS_ERR_ARG);
    EXPECT(gas_disk_open("x", 4, 4, GAS_F32, 64, 0, 0, &t) == GAS_ERR_ARG);
    EXPECT(gas_disk_close(nullptr) == GAS_OK);
    // an empty table
    EXPECT(gas_disk_open((dir + "/disk_check_e.bin").c_str(), 0, 4, GAS_F32, GAS_DISK_CREATE, 2, 0, &t) == GAS_OK);
    EXPECT(gas_disk_read_rows(t, nullptr, 0, 0, nullptr, 4) == GAS_OK);
    EXPECT(gas_disk_close(t) == GAS_OK);
    unlink((dir + "/disk_check_e.bin").c_str());
    printf("%d cases, %d failures\n", cases, failures);
    return failures != 0;
}
