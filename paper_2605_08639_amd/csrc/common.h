// Internal helpers shared by the HIP translation units of librelibra (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/relibra.h"

#define RELIBRA_HIP_TRY(expr)                      \
    do {                                           \
        hipError_t e_ = (expr);                    \
        if (e_ != hipSuccess) return RELIBRA_EHIP; \
    } while (0)

namespace relibra {

typedef uint16_t bf16_t;   // bf16 bit pattern

__device__ __forceinline__ float bf2f(bf16_t b) { return __uint_as_float((uint32_t)b << 16); }

// round-to-nearest-even fp32 -> bf16 (NaN stays NaN)
__device__ __forceinline__ bf16_t f2bf(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((u >> 16) | 0x40u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (bf16_t)(u >> 16);
}

__device__ __forceinline__ uint32_t pack2bf(float lo, float hi)
{
    return (uint32_t)f2bf(lo) | ((uint32_t)f2bf(hi) << 16);
}

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

inline hipError_t launch_check() { return hipGetLastError(); }

// Event bracketing of a launch (prof.hip); both are no-ops while profiling is off.
bool prof_before(int kernel_id, hipStream_t s);
void prof_after(int kernel_id, hipStream_t s);

// LAUNCH(kernel id, stream, kernel<<<...>>>(...)): launch, optionally timed.
#define RELIBRA_LAUNCH(id, stream, ...)                         \
    do {                                                        \
        const bool prof_ = relibra::prof_before((id), (stream)); \
        __VA_ARGS__;                                            \
        if (prof_) relibra::prof_after((id), (stream));         \
    } while (0)

}  // namespace relibra
