// Internal helpers shared by the HIP translation units of libinsum (not part of the ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stdint.h>

#include "insum.h"

#define INSUM_HIP_TRY(expr)                      \
    do {                                         \
        hipError_t _e = (expr);                  \
        if (_e != hipSuccess) {                  \
            (void)hipGetLastError();             \
            return INSUM_ERR_HIP;                \
        }                                        \
    } while (0)

namespace insum {

constexpr int kWave = 64;

__host__ __device__ inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

inline int dtype_size(insum_dtype dt) { return dt == INSUM_F32 ? 4 : 2; }
inline bool dtype_valid(int dt) { return dt == INSUM_F32 || dt == INSUM_F16 || dt == INSUM_BF16; }

// bf16 is handled as raw 16-bit patterns: upcast is a shift, downcast rounds to nearest even.
struct bf16_t {
    uint16_t bits;
};

__device__ inline float to_float(float x) { return x; }
__device__ inline float to_float(__half x) { return __half2float(x); }
__device__ inline float to_float(bf16_t x) { return __uint_as_float(((uint32_t)x.bits) << 16); }

template <typename T>
__device__ inline T from_float(float x);
template <>
__device__ inline float from_float<float>(float x) { return x; }
template <>
__device__ inline __half from_float<__half>(float x) { return __float2half_rn(x); }
template <>
__device__ inline bf16_t from_float<bf16_t>(float x) {
    uint32_t u = __float_as_uint(x);
    if ((u & 0x7fffffffu) > 0x7f800000u) return bf16_t{(uint16_t)((u >> 16) | 0x40)};  // NaN
    u += 0x7fffu + ((u >> 16) & 1u);
    return bf16_t{(uint16_t)(u >> 16)};
}

}  // namespace insum
