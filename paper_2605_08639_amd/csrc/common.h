// Internal helpers shared by the HIP translation units of librelibra (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/relibra.h"

// Assignments per unit of the permutation kernels (one wave each); sizes their count matrix.
#define RELIBRA_PERM_UNIT 128

#define RELIBRA_HIP_TRY(expr)                      \
    do {                                           \
        hipError_t e_ = (expr);                    \
        if (e_ != hipSuccess) return RELIBRA_EHIP; \
    } while (0)

namespace relibra {

typedef uint16_t bf16_t;   // bf16 bit pattern

__device__ __forceinline__ float bf2f(bf16_t b) { return __uint_as_float((uint32_t)b << 16); }

// fp32 -> bf16, round to nearest even, with the hardware conversion of gfx950
// (v_cvt_pk_bf16_f32: two values per instruction, NaN stays NaN).
typedef __bf16 hw_bf16x2_t __attribute__((ext_vector_type(2)));
typedef float hw_f32x2_t __attribute__((ext_vector_type(2)));

__device__ __forceinline__ uint32_t pack2bf(float lo, float hi)
{
    const hw_f32x2_t v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, hw_bf16x2_t));
}

__device__ __forceinline__ bf16_t f2bf(float f) { return (bf16_t)(pack2bf(f, 0.0f) & 0xffffu); }

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
