// Machine probes: what this GPU sustains on a bare MFMA issue loop and on a streaming copy.
// They carry none of the method's arithmetic; the benchmark prints their figures beside the
// published peaks so that a kernel's fraction can be read against both.
#include <hip/hip_runtime.h>

#include "../../include/sknet.h"
#include "sk_host.h"

using skh::fail;

namespace {

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 halfx8 __attribute__((ext_vector_type(8)));
typedef unsigned int uintx4 __attribute__((ext_vector_type(4)));

constexpr int kAcc = 8;   // independent accumulators per wave: hides the MFMA result latency

// Each wave issues iters * kAcc dependent-free MFMAs of one shape; nothing touches memory until
// the single store at the end (kept so the loop is not removed).  The MFMAs are written as inline
// assembly with the accumulators pinned to vector registers: with the builtin the register
// allocator shuttles the loop-carried accumulators between register files and the loop no longer
// measures the matrix pipe.  Eight independent accumulators separate dependent instructions by
// far more than the pipe's depth, and the s_nop pair covers the read of the results afterwards.
template <int DT>
__global__ void __launch_bounds__(256) mfma_issue_kernel(float *out, int iters)
{
    floatx4 acc[kAcc];
#pragma unroll
    for (int i = 0; i < kAcc; ++i) acc[i] = floatx4{0.f, 0.f, 0.f, 0.f};
    const float seed = (float)threadIdx.x * 0.001f;
    if constexpr (DT == SK_F32) {
        const float a = seed, b = 1.0f;
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int i = 0; i < kAcc; ++i) asm volatile("v_mfma_f32_16x16x4_f32 %0, %1, %2, %0" : "+v"(acc[i]) : "v"(a), "v"(b));
        }
    } else if constexpr (DT == SK_BF16) {
        bf16x8 a, b;
#pragma unroll
        for (int i = 0; i < 8; ++i) { a[i] = (__bf16)seed; b[i] = (__bf16)1.0f; }
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int i = 0; i < kAcc; ++i) asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+v"(acc[i]) : "v"(a), "v"(b));
        }
    } else {
        halfx8 a, b;
#pragma unroll
        for (int i = 0; i < 8; ++i) { a[i] = (_Float16)seed; b[i] = (_Float16)1.0f; }
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int i = 0; i < kAcc; ++i) asm volatile("v_mfma_f32_16x16x32_f16 %0, %1, %2, %0" : "+v"(acc[i]) : "v"(a), "v"(b));
        }
    }
    asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < kAcc; ++i) s += acc[i][0] + acc[i][1] + acc[i][2] + acc[i][3];
    out[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = s;
}

// 16 bytes per lane per trip, consecutive lanes on consecutive addresses, grid-stride.
__global__ void __launch_bounds__(256) stream_copy_kernel(const uintx4 *__restrict__ src, uintx4 *__restrict__ dst, size_t n16)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

template <typename F>
sk_status time_launches(hipStream_t stream, int reps, F launch, float *avg_ms)
{
    hipEvent_t e0, e1;
    SK_HIP(hipEventCreate(&e0));
    SK_HIP(hipEventCreate(&e1));
    launch();   // warm-up
    hipError_t e = hipEventRecord(e0, stream);
    for (int i = 0; i < reps; ++i) launch();
    if (e == hipSuccess) e = hipEventRecord(e1, stream);
    if (e == hipSuccess) e = hipEventSynchronize(e1);
    float ms = 0.f;
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
    if (e == hipSuccess) e = hipGetLastError();
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (e != hipSuccess) return fail(SK_EDEVICE, "probe: %s", hipGetErrorString(e));
    *avg_ms = ms / (float)reps;
    return SK_OK;
}

}  // namespace

extern "C" {

sk_status sk_probe_mfma(int32_t dtype, int32_t iters, void *hip_stream, double *tflops)
{
    if (!tflops || iters < 1 || iters > (1 << 22)) return fail(SK_EINVAL, "probe_mfma: bad arguments");
    if (dtype != SK_F32 && dtype != SK_BF16 && dtype != SK_F16) return fail(SK_EINVAL, "probe_mfma: unknown dtype %d", dtype);
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    int dev = 0, cus = 0;
    SK_HIP(hipGetDevice(&dev));
    SK_HIP(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
    const int blocks = cus * 4, threads = 256;   // 16 waves per CU, four per SIMD
    float *out = nullptr;
    SK_HIP(hipMalloc(&out, (size_t)blocks * threads * sizeof(float)));
    float ms = 0.f;
    sk_status st = time_launches(stream, 3, [&] {
        if (dtype == SK_F32) hipLaunchKernelGGL(mfma_issue_kernel<SK_F32>, dim3(blocks), dim3(threads), 0, stream, out, iters);
        else if (dtype == SK_BF16) hipLaunchKernelGGL(mfma_issue_kernel<SK_BF16>, dim3(blocks), dim3(threads), 0, stream, out, iters);
        else hipLaunchKernelGGL(mfma_issue_kernel<SK_F16>, dim3(blocks), dim3(threads), 0, stream, out, iters);
    }, &ms);
    (void)hipFree(out);
    if (st != SK_OK) return st;
    const double flop_per_mfma = dtype == SK_F32 ? 2.0 * 16 * 16 * 4 : 2.0 * 16 * 16 * 32;
    *tflops = (double)blocks * (threads / 64) * (double)iters * kAcc * flop_per_mfma / ((double)ms * 1e-3) / 1e12;
    return SK_OK;
}

sk_status sk_probe_copy(const void *src_dev, void *dst_dev, uint64_t bytes, int32_t reps, void *hip_stream, double *gb_per_s)
{
    if (!src_dev || !dst_dev || !gb_per_s || reps < 1 || bytes < 16 || (bytes & 15)) return fail(SK_EINVAL, "probe_copy: bad arguments (bytes must be a positive multiple of 16)");
    if (((uintptr_t)src_dev | (uintptr_t)dst_dev) & 15) return fail(SK_EINVAL, "probe_copy: buffers must be 16-byte aligned");
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const size_t n16 = bytes / 16;
    const size_t want = (n16 + 255) / 256;
    const int blocks = (int)(want < 16384 ? want : 16384);
    float ms = 0.f;
    SK_TRY(time_launches(stream, reps, [&] {
        hipLaunchKernelGGL(stream_copy_kernel, dim3(blocks), dim3(256), 0, stream, (const uintx4 *)src_dev, (uintx4 *)dst_dev, n16);
    }, &ms));
    *gb_per_s = 2.0 * (double)bytes / ((double)ms * 1e-3) / 1e9;   // bytes read + bytes written
    return SK_OK;
}

}  // extern "C"
