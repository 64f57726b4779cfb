// What a gas_plan holds (internal; the C ABI only sees the opaque handle).
#pragma once
#include <stdint.h>

struct gas_plan {
    int64_t n_rows = 0, nnz = 0;
    int32_t max_F = 0;
    int32_t threshold = 0, chunk = 0;
    int64_t n_heavy = 0, n_chunks = 0;
    int32_t* d_chunk = nullptr;        // [3 * n_chunks]: slot of the partial sum, begin, end (in processing order)
    int32_t* d_heavy = nullptr;        // [n_heavy] row ids, then [n_heavy + 1] first chunk of each
    float* d_partial = nullptr;        // [n_chunks, max_F]
    int32_t* d_group = nullptr;        // [2 * n_groups] first and end row of every group of light rows
    int64_t n_groups = 0;
    int xcd_ranges = 0;                // light-row groups are handed out in one contiguous range per XCD
    int64_t xcd_start[9] = {0};        // first group of every XCD's range (and the end), equal cost per range
    int device = 0;
};

