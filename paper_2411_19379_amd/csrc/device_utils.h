// Small device helpers shared by the scan kernels (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

#include "plan.h"

typedef uint16_t bf16_t;  // raw bfloat16 bits

__device__ __forceinline__ float bf16_to_f32(bf16_t v)
{
    return __uint_as_float((uint32_t)v << 16);
}

// round to nearest even; NaN stays NaN
__device__ __forceinline__ bf16_t f32_to_bf16(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u)
        return (bf16_t)((u >> 16) | 0x0040u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (bf16_t)(u >> 16);
}

template <typename IO> struct IoTraits;
template <> struct IoTraits<float> {
    static __device__ __forceinline__ float load(const float *p) { return *p; }
    static __device__ __forceinline__ void store(float *p, float v) { *p = v; }
};
template <> struct IoTraits<bf16_t> {
    static __device__ __forceinline__ float load(const bf16_t *p) { return bf16_to_f32(*p); }
    static __device__ __forceinline__ void store(bf16_t *p, float v) { *p = f32_to_bf16(v); }
};

// Arguments common to both scan kernels.  Pointers are device pointers.
struct ScanArgs {
    const void *x;
    const void *dt;
    const float *A;
    const void *B;
    const void *C;
    const float *D;
    void *y;
    float *state_out;
    const float *const *init_ptrs;  // [batch] or NULL
    const SsmTile *tiles;
    const SsmSeq *seqs;
    int32_t H, P, N, G;
    int32_t p_split;
};

// Launchers implemented next to their kernels.
hipError_t launch_scan_valu(const ssm_plan *plan, const ScanArgs &args, hipStream_t stream);
hipError_t launch_scan_mfma(const ssm_plan *plan, const ScanArgs &args, hipStream_t stream);
