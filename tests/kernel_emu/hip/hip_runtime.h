// Stand-in for <hip/hip_runtime.h> in the CPU emulation of the scan kernels (test infrastructure only): the kernel
// sources compile as plain C++, run lane by lane on fibers, and the cross-lane builtins of gfx950 they use are
// routed to the emulation runtime.  Only what those sources use is provided.
#pragma once
#include <cmath>
#include <cstddef>
#include <cstdint>
#include <cstring>

#define __global__
#define __device__
#define __host__
#define __forceinline__ inline __attribute__((always_inline))
#define __launch_bounds__(...)
#define __align__(n) alignas(n)

struct uint2 { uint32_t x, y; };
struct alignas(16) uint4 { uint32_t x, y, z, w; };
struct float2 { float x, y; };
struct alignas(16) float4 { float x, y, z, w; };
struct int4 { int x, y, z, w; };
static inline uint2 make_uint2(uint32_t x, uint32_t y) { return {x, y}; }
static inline uint4 make_uint4(uint32_t x, uint32_t y, uint32_t z, uint32_t w) { return {x, y, z, w}; }
static inline float2 make_float2(float x, float y) { return {x, y}; }
static inline float4 make_float4(float x, float y, float z, float w) { return {x, y, z, w}; }
static inline float __uint_as_float(uint32_t u) { float f; memcpy(&f, &u, 4); return f; }
static inline uint32_t __float_as_uint(float f) { uint32_t u; memcpy(&u, &f, 4); return u; }

struct dim3 {
    unsigned x, y, z;
    dim3(unsigned x_ = 1, unsigned y_ = 1, unsigned z_ = 1) : x(x_), y(y_), z(z_) {}
};
typedef int hipError_t;
constexpr hipError_t hipSuccess = 0;
constexpr hipError_t hipErrorInvalidValue = 1;
constexpr hipError_t hipErrorInvalidDevice = 101;
static inline hipError_t hipGetDevice(int *dev) { *dev = 0; return hipSuccess; }
typedef void *hipStream_t;
typedef void *hipEvent_t;
static inline hipError_t hipEventRecord(hipEvent_t, hipStream_t) { return hipSuccess; }
constexpr int hipFuncAttributeMaxDynamicSharedMemorySize = 8;
static inline hipError_t hipFuncSetAttribute(const void *, int, int) { return hipSuccess; }
static inline hipError_t hipGetLastError() { return hipSuccess; }

namespace emu {
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;

struct Idx { unsigned x, y, z; };
Idx &thread_idx();
Idx &block_idx();
unsigned char *lds_base();

void barrier(int line);     // workgroup barrier
void wave_sync(int line);   // lockstep point inside a wave (stands for an LDS wait between lanes of one wave)
void wave_yield(int line);  // inside a spin-wait: the other waves of the workgroup get a turn
f32x16 mfma_32x32x16_bf16(bf16x8 a, bf16x8 b, f32x16 c, int line);
f32x16 mfma_32x32x16_f16(f16x8 a, f16x8 b, f32x16 c, int line);
f32x4 mfma_16x16x32_bf16(bf16x8 a, bf16x8 b, f32x4 c, int line);
s16x4 ds_read_tr16_b64(const void *p, int line);
int update_dpp(int old, int src, int ctrl, int row_mask, int bank_mask, bool bound_ctrl, int line);
int readlane(int v, int lane, int line);
int readfirstlane(int v, int line);
int shfl(int v, int src_lane, int line);  // any-to-any lane read (ds_bpermute)

// Buffer descriptor of the raw (stride 0) kind: a base and a size in bytes.  An access that lies inside [0, bytes)
// goes to memory; a load through a descriptor of size zero returns zeros without touching memory, as the hardware's
// range check does; any other access beyond the size is a bug of the kernel and ends the run.
struct BufRsrc {
    unsigned char *base;
    uint32_t bytes;
};
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;
void buffer_range_fault(uint32_t off, uint32_t n, uint32_t bytes, int line);
static inline BufRsrc make_buffer_rsrc(void *base, int stride, int bytes, int flags)
{
    (void)stride, (void)flags;
    return {static_cast<unsigned char *>(base), (uint32_t)bytes};
}
template <typename T> static inline T buffer_load(const BufRsrc &r, int voff, int soff, int line)
{
    T v;
    memset(&v, 0, sizeof v);
    if (r.bytes == 0)
        return v;
    const uint32_t off = (uint32_t)voff + (uint32_t)soff;
    if ((uint64_t)off + sizeof(T) > r.bytes)
        buffer_range_fault(off, sizeof(T), r.bytes, line);
    memcpy(&v, r.base + off, sizeof v);
    return v;
}
template <typename T> static inline void buffer_store(const T &v, const BufRsrc &r, int voff, int soff, int line)
{
    const uint32_t off = (uint32_t)voff + (uint32_t)soff;
    if ((uint64_t)off + sizeof(T) > r.bytes)
        buffer_range_fault(off, sizeof(T), r.bytes, line);
    memcpy(r.base + off, &v, sizeof v);
}

template <typename F> void launch(dim3 grid, dim3 block, size_t lds_bytes, F &&body);
void launch_impl(dim3 grid, dim3 block, size_t lds_bytes, void (*fn)(void *), void *arg);
template <typename F> void launch(dim3 grid, dim3 block, size_t lds_bytes, F &&body)
{
    launch_impl(grid, block, lds_bytes, [](void *p) { (*static_cast<F *>(p))(); }, &body);
}
}  // namespace emu

#define threadIdx (emu::thread_idx())
#define blockIdx (emu::block_idx())
#define __syncthreads() emu::barrier(__LINE__)

#define __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, x, y, z) emu::mfma_32x32x16_bf16((a), (b), (c), __LINE__)
#define __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, x, y, z) emu::mfma_32x32x16_f16((a), (b), (c), __LINE__)
#define __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, x, y, z) emu::mfma_16x16x32_bf16((a), (b), (c), __LINE__)
#define __builtin_amdgcn_ds_read_tr16_b64_v4i16(p) emu::ds_read_tr16_b64((const void *)(p), __LINE__)
#define __builtin_amdgcn_update_dpp(old, src, ctrl, rm, bm, bc) emu::update_dpp((old), (src), (ctrl), (rm), (bm), (bc), __LINE__)
#define __builtin_amdgcn_readlane(v, l) emu::readlane((v), (l), __LINE__)
#define __builtin_amdgcn_readfirstlane(v) emu::readfirstlane((v), __LINE__)
#define __shfl(v, l, w) __uint_as_float((uint32_t)emu::shfl((int)__float_as_uint(v), (l), __LINE__))
#define __amdgpu_buffer_rsrc_t emu::BufRsrc
#define __builtin_amdgcn_make_buffer_rsrc(p, stride, n, flags) emu::make_buffer_rsrc((p), (stride), (n), (flags))
#define __builtin_amdgcn_raw_buffer_load_b128(r, voff, soff, aux) emu::buffer_load<emu::u32x4>((r), (voff), (soff), __LINE__)
#define __builtin_amdgcn_raw_buffer_load_b16(r, voff, soff, aux) emu::buffer_load<unsigned short>((r), (voff), (soff), __LINE__)
#define __builtin_amdgcn_raw_buffer_store_b128(v, r, voff, soff, aux) emu::buffer_store((v), (r), (voff), (soff), __LINE__)
#define __builtin_amdgcn_exp2f(x) exp2f(x)
#define __builtin_amdgcn_rcpf(x) (1.0f / (x))
#define __builtin_amdgcn_s_setprio(x) ((void)0)
#define __builtin_amdgcn_sched_barrier(x) ((void)0)
#define __builtin_amdgcn_s_sleep(x) emu::wave_yield(__LINE__)
#define __builtin_amdgcn_logf(x) log2f(x)

#define hipLaunchKernelGGL(kernel, grid, block, lds, stream, ...) \
    emu::launch((grid), (block), (lds), [&]() { kernel(__VA_ARGS__); })
