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

// One element of a cached state in its storage type (ssm_state_dtype_t); the running state is always fp32 and a
// reduced-precision checkpoint is that fp32 value rounded once, to nearest even.
__device__ __forceinline__ float state_load(const void *base, size_t idx, int state_dtype)
{
    if (state_dtype == SSM_ST_F16)
        return (float)static_cast<const _Float16 *>(base)[idx];
    if (state_dtype == SSM_ST_BF16)
        return bf16_to_f32(static_cast<const bf16_t *>(base)[idx]);
    return static_cast<const float *>(base)[idx];
}

__device__ __forceinline__ void state_store(void *base, size_t idx, float v, int state_dtype)
{
    if (state_dtype == SSM_ST_F16)
        static_cast<_Float16 *>(base)[idx] = (_Float16)v;
    else if (state_dtype == SSM_ST_BF16)
        static_cast<bf16_t *>(base)[idx] = f32_to_bf16(v);
    else
        static_cast<float *>(base)[idx] = v;
}

// Arguments common to the scan kernels.  Pointers are device pointers.
struct ScanArgs {
    const void *x;
    const void *dt;
    const float *A;
    const void *B;
    const void *C;
    const float *D;
    void *y;
    void *state_out;                // [n_ckpt,H,P,N] in the state type
    const void *const *init_ptrs;   // [batch] pointers to [H,P,N] in the state type, or NULL
    const SsmTile *tiles;
    const SsmSeq *seqs;
    const SsmScanSeq *scan_seqs;    // matrix-core scan only
    int32_t H, P, N, G;
    int32_t p_split;
    int32_t state_dtype;            // ssm_state_dtype_t
};

// Launchers implemented next to their kernels.
hipError_t launch_scan_valu(const ssm_plan *plan, const ScanArgs &args, hipStream_t stream);
hipError_t launch_scan_mfma(const ssm_plan *plan, const ScanArgs &args, void *workspace, hipStream_t stream);
// events to record after the first and after the second kernel of the matrix-core scan on the calling thread
// (nullptr: none)
hipEvent_t ssm_profile_event(int which);
bool state_advance_supports(const ssm_shape_t &s);
hipError_t launch_state_advance(const ssm_plan *plan, const ScanArgs &args, void *const *d_state_ptrs,
                                hipStream_t stream);
bool conv1d_supports(int channels, int K, int io_dtype);
hipError_t launch_conv1d_prefill(const ssm_plan *plan, const SsmTile *d_tiles, const SsmSeq *d_seqs, int channels,
                                 int K, const void *in, const float *w, const float *bias,
                                 const void *const *d_init_ptrs, void *out, void *state_out, int act,
                                 hipStream_t stream);
