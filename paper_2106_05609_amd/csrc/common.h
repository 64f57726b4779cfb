// Internal helpers of the GAS library (not part of the C ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdarg.h>
#include <stdio.h>

#include "gas.h"

namespace gas {

// ---- error reporting ------------------------------------------------------
char* last_error_buffer();                       // thread-local, 512 bytes
gas_status fail(gas_status st, const char* fmt, ...);

#define GAS_CHECK_HIP(expr)                                                             \
    do {                                                                                \
        hipError_t e_ = (expr);                                                         \
        if (e_ != hipSuccess)                                                           \
            return gas::fail(GAS_ERR_HIP, "%s failed: %s", #expr, hipGetErrorString(e_)); \
    } while (0)

#define GAS_REQUIRE(cond, ...)                                  \
    do {                                                        \
        if (!(cond)) return gas::fail(GAS_ERR_ARG, __VA_ARGS__); \
    } while (0)

static inline int elem_bytes(gas_dtype dt) { return dt == GAS_F32 ? 4 : 2; }
static inline bool valid_dtype(int dt) { return dt == GAS_F32 || dt == GAS_BF16; }
static inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// ---- device-side types ----------------------------------------------------
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kWave = 64;

__device__ __forceinline__ float bf16_lo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t u) { return __uint_as_float(u & 0xFFFF0000u); }

// fp32 -> bf16 bits, round to nearest even: gfx950 converts in hardware
// (v_cvt_pk_bf16_f32), two values per instruction
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2_t{lo, hi}, bf16x2_t));
}
__device__ __forceinline__ uint32_t f32_to_bf16(float f) { return pack_bf16(f, 0.f) & 0xFFFFu; }

}  // namespace gas
