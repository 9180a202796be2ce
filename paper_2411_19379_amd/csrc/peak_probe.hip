// What this GPU sustains on the two roofs the scan is priced against, measured with the simplest possible kernels:
// a streaming device copy and read (HBM) and a register-resident loop of dense 32x32x16 MFMAs in bf16 and fp16 (the
// two operand types of the scan).  Stand-alone program, not part of the library:
//     paper_2411_19379_amd/peak_probe
// prints GB/s and TFLOP/s beside nothing else; the published peaks are quoted where the figures are used.
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>

#define CK(x)                                                                              \
    do {                                                                                   \
        hipError_t e_ = (x);                                                               \
        if (e_ != hipSuccess) {                                                            \
            printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__);          \
            exit(1);                                                                       \
        }                                                                                  \
    } while (0)

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

__global__ __launch_bounds__(256) void copy_kernel(const uint4 *__restrict__ src, uint4 *__restrict__ dst, size_t n)
{
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x)
        dst[i] = src[i];
}

__global__ __launch_bounds__(256) void read_kernel(const uint4 *__restrict__ src, uint4 *__restrict__ dst, size_t n)
{
    uint4 acc = make_uint4(0, 0, 0, 0);
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) {
        const uint4 v = src[i];
        acc.x ^= v.x, acc.y ^= v.y, acc.z ^= v.z, acc.w ^= v.w;
    }
    if (acc.x == 0x12345678u && acc.y == 0x9abcdef0u)  // never true for the fill pattern: keeps the loads alive
        dst[threadIdx.x] = acc;
}

template <bool HALF>
__global__ __launch_bounds__(256) void mfma_kernel(float *out, int iters)
{
    bf16x8 a, b;
    f16x8 ah, bh;
    for (int e = 0; e < 8; ++e) {
        a[e] = (__bf16)(0.001f * (threadIdx.x + e)), b[e] = (__bf16)(0.002f * ((int)threadIdx.x - e));
        ah[e] = (_Float16)(0.001f * (threadIdx.x + e)), bh[e] = (_Float16)(0.002f * ((int)threadIdx.x - e));
    }
    f32x16 c0 = {0}, c1 = {0}, c2 = {0}, c3 = {0};  // four independent accumulators per wave
    for (int i = 0; i < iters; ++i) {
        if (HALF) {
            c0 = __builtin_amdgcn_mfma_f32_32x32x16_f16(ah, bh, c0, 0, 0, 0);
            c1 = __builtin_amdgcn_mfma_f32_32x32x16_f16(ah, bh, c1, 0, 0, 0);
            c2 = __builtin_amdgcn_mfma_f32_32x32x16_f16(ah, bh, c2, 0, 0, 0);
            c3 = __builtin_amdgcn_mfma_f32_32x32x16_f16(ah, bh, c3, 0, 0, 0);
        } else {
            c0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c0, 0, 0, 0);
            c1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c1, 0, 0, 0);
            c2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c2, 0, 0, 0);
            c3 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c3, 0, 0, 0);
        }
    }
    float s = 0;
    for (int r = 0; r < 16; ++r)
        s += c0[r] + c1[r] + c2[r] + c3[r];
    if (s == 123.456f)  // keeps the accumulators alive
        out[threadIdx.x] = s;
}

int main()
{
    const size_t bytes = (size_t)2 << 30, n = bytes / 16;
    uint4 *src, *dst;
    CK(hipMalloc(&src, bytes));
    CK(hipMalloc(&dst, bytes));
    CK(hipMemset(src, 1, bytes));
    CK(hipMemset(dst, 0, bytes));
    hipEvent_t e0, e1;
    CK(hipEventCreate(&e0));
    CK(hipEventCreate(&e1));
    float ms;
    for (int grid : {256 * 4, 256 * 8, 256 * 16, 256 * 32}) {
        hipLaunchKernelGGL(copy_kernel, dim3(grid), dim3(256), 0, 0, src, dst, n);
        CK(hipDeviceSynchronize());
        CK(hipEventRecord(e0));
        for (int i = 0; i < 5; ++i)
            hipLaunchKernelGGL(copy_kernel, dim3(grid), dim3(256), 0, 0, src, dst, n);
        CK(hipEventRecord(e1));
        CK(hipEventSynchronize(e1));
        CK(hipEventElapsedTime(&ms, e0, e1));
        printf("copy 2 GiB, %5d workgroups: %5.0f GB/s (read + write)\n", grid, 2.0 * bytes * 5 / (ms * 1e-3) / 1e9);
        hipLaunchKernelGGL(read_kernel, dim3(grid), dim3(256), 0, 0, src, dst, n);
        CK(hipDeviceSynchronize());
        CK(hipEventRecord(e0));
        for (int i = 0; i < 5; ++i)
            hipLaunchKernelGGL(read_kernel, dim3(grid), dim3(256), 0, 0, src, dst, n);
        CK(hipEventRecord(e1));
        CK(hipEventSynchronize(e1));
        CK(hipEventElapsedTime(&ms, e0, e1));
        printf("read 2 GiB, %5d workgroups: %5.0f GB/s\n", grid, 1.0 * bytes * 5 / (ms * 1e-3) / 1e9);
    }
    float *out;
    CK(hipMalloc(&out, 4096));
    const int iters = 20000;
    for (int half = 0; half < 2; ++half)
        for (int wgs_per_cu : {1, 2, 4}) {
            auto launch = [&](int it) {
                if (half)
                    hipLaunchKernelGGL(mfma_kernel<true>, dim3(256 * wgs_per_cu), dim3(256), 0, 0, out, it);
                else
                    hipLaunchKernelGGL(mfma_kernel<false>, dim3(256 * wgs_per_cu), dim3(256), 0, 0, out, it);
            };
            launch(100);
            CK(hipDeviceSynchronize());
            CK(hipEventRecord(e0));
            launch(iters);
            CK(hipEventRecord(e1));
            CK(hipEventSynchronize(e1));
            CK(hipEventElapsedTime(&ms, e0, e1));
            const double flops = 2.0 * 32 * 32 * 16 * 4.0 * iters * (256.0 * wgs_per_cu * 4);
            printf("mfma 32x32x16 %s, %d workgroups of 4 waves per CU: %5.0f TFLOP/s dense\n", half ? "fp16" : "bf16",
                   wgs_per_cu, flops / (ms * 1e-3) / 1e12);
        }
    CK(hipFree(src));
    CK(hipFree(dst));
    CK(hipFree(out));
    return 0;
}
