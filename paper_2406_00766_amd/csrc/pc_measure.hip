// Achievable peaks of the device, measured with two plain kernels (the measurement protocol, not an operation of the
// paper): a streaming copy for HBM bandwidth and a register-only MFMA loop for the fp32 matrix rate.  The benchmark
// quotes them beside the published peaks that the roofline fractions are taken against.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdint>
#include <string>

#include "pc_internal.h"

namespace pc {

typedef float floatx16 __attribute__((ext_vector_type(16)));

// 16-byte grid-stride copy: every byte is read once and written once
__global__ __launch_bounds__(256) void k_measure_copy(const float4 *__restrict__ src, float4 *__restrict__ dst, int64_t n16)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

// four independent accumulators per wave, operands in registers: nothing but v_mfma_f32_32x32x2_f32 in the loop
constexpr int kMfmaAcc = 4, kMfmaUnroll = 16;
__global__ __launch_bounds__(256) void k_measure_mfma(float *__restrict__ out, int iters, float a0, float b0)
{
    floatx16 acc[kMfmaAcc];
#pragma unroll
    for (int n = 0; n < kMfmaAcc; ++n)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[n][e] = 0.0f;
    const float a = a0 + threadIdx.x * 1e-6f, b = b0;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < kMfmaUnroll; ++u)
#pragma unroll
            for (int n = 0; n < kMfmaAcc; ++n) acc[n] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc[n], 0, 0, 0);
    }
    float s = 0.0f;
#pragma unroll
    for (int n = 0; n < kMfmaAcc; ++n)
#pragma unroll
        for (int e = 0; e < 16; ++e) s += acc[n][e];
    out[(int64_t)blockIdx.x * blockDim.x + threadIdx.x] = s;
}

static pc_status hip_fail2(hipError_t e, const char *what) { return fail(PC_ERR_HIP, std::string(what) + ": " + hipGetErrorString(e)); }
#define PC_HIP2(call)                                       \
    do {                                                    \
        hipError_t e_ = (call);                             \
        if (e_ != hipSuccess) return hip_fail2(e_, #call);  \
    } while (0)

// average milliseconds of `reps` back-to-back launches after one warm-up launch
template <typename Launch>
static pc_status time_launches(Launch launch, int reps, hipStream_t s, double *ms)
{
    hipEvent_t a = nullptr, b = nullptr;
    PC_HIP2(hipEventCreate(&a));
    PC_HIP2(hipEventCreate(&b));
    launch();
    PC_HIP2(hipEventRecord(a, s));
    for (int i = 0; i < reps; ++i) launch();
    PC_HIP2(hipEventRecord(b, s));
    PC_HIP2(hipEventSynchronize(b));
    float t = 0.0f;
    PC_HIP2(hipEventElapsedTime(&t, a, b));
    (void)hipEventDestroy(a);
    (void)hipEventDestroy(b);
    PC_HIP2(hipGetLastError());
    *ms = (double)t / reps;
    return PC_OK;
}

}  // namespace pc

using namespace pc;

extern "C" {

pc_status pc_measure_copy(const void *src, void *dst, size_t bytes, int32_t reps, void *stream, double *gb_per_s)
{
    if (!src || !dst || !gb_per_s) return fail(PC_ERR_ARG, "NULL argument");
    if (bytes < 16 || (bytes & 15) || ((uintptr_t)src & 15) || ((uintptr_t)dst & 15) || reps < 1)
        return fail(PC_ERR_ARG, "bytes must be a positive multiple of 16, buffers 16-byte aligned, reps >= 1");
    hipStream_t s = (hipStream_t)stream;
    const int64_t n16 = (int64_t)(bytes / 16);
    const unsigned grid = (unsigned)std::min<int64_t>((n16 + 255) / 256, 256 * 32);      // 32 workgroups per CU, grid-stride
    double ms = 0.0;
    pc_status st = time_launches(
        [&] { hipLaunchKernelGGL(k_measure_copy, dim3(grid), dim3(256), 0, s, (const float4 *)src, (float4 *)dst, n16); }, reps, s, &ms);
    if (st != PC_OK) return st;
    *gb_per_s = 2.0 * (double)bytes / (ms * 1e-3) / 1e9;                                  // read + written
    return PC_OK;
}

pc_status pc_measure_mfma_f32(void *out, size_t out_bytes, int32_t reps, void *stream, double *tflops)
{
    constexpr int kGrid = 256 * 8, kIters = 200;                                          // two waves per SIMD, about 3 ms per launch
    if (!out || !tflops) return fail(PC_ERR_ARG, "NULL argument");
    if (out_bytes < (size_t)kGrid * 256 * 4 || reps < 1) return fail(PC_ERR_ARG, "out must hold 2 MiB, reps >= 1");
    hipStream_t s = (hipStream_t)stream;
    double ms = 0.0;
    pc_status st = time_launches(
        [&] { hipLaunchKernelGGL(k_measure_mfma, dim3(kGrid), dim3(256), 0, s, (float *)out, kIters, 1.0f, 1e-3f); }, reps, s, &ms);
    if (st != PC_OK) return st;
    const double flop = (double)kGrid * 4 /*waves*/ * kIters * kMfmaUnroll * kMfmaAcc * (2.0 * 32 * 32 * 2);
    *tflops = flop / (ms * 1e-3) / 1e12;
    return PC_OK;
}

}  // extern "C"
