// Machine probes: what this GPU sustains on a bare MFMA issue loop and on a streaming copy.
// They carry none of the method's arithmetic; the benchmark prints their figures beside the
// published peaks so that a kernel's fraction can be read against both.
#include <hip/hip_runtime.h>

#include "../../include/sknet.h"
#include "sk_host.h"

using skh::fail;

namespace {

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef unsigned int uintx4 __attribute__((ext_vector_type(4)));

constexpr int kAcc = 8;   // independent accumulators per wave: hides the MFMA result latency

// Each wave issues iters * kAcc dependent-free MFMAs of one shape; nothing touches memory until
// the single store at the end (kept so the loop is not removed).  The MFMAs are written as inline
// assembly with the accumulators pinned to vector registers: with the builtin the register
// allocator shuttles the loop-carried accumulators between register files and the loop no longer
// measures the matrix pipe.  Eight independent accumulators separate dependent instructions by
// far more than the pipe's depth, and the s_nop pair covers the read of the results afterwards.
// VARIED = false: every MFMA multiplies the same two registers (one smooth value per lane, and ones),
// the least switching activity the pipe can see.  VARIED = true: each of the eight MFMAs of a trip
// has operands of its own, filled with hashed bit patterns that decode to values in [-1, 1); that is
// what real activations and weights look like to the multipliers, and the rate it sustains is the
// one a kernel with real data can be held against when the chip runs into its power limit.
__device__ __forceinline__ unsigned probe_hash(unsigned x)
{
    x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16;
    return x;
}
// a 16-bit float in [-1, 1) with hashed sign and mantissa (exponent field of 0.5 .. 1 minus a few steps)
template <int DT>
__device__ __forceinline__ unsigned probe_half_bits(unsigned h)
{
    if constexpr (DT == SK_BF16) return ((h & 1u) << 15) | ((0x7cu + ((h >> 1) & 3u)) << 7) | ((h >> 3) & 0x7fu);
    else return ((h & 1u) << 15) | ((0x0cu + ((h >> 1) & 3u)) << 10) | ((h >> 3) & 0x3ffu);
}

template <int DT, bool VARIED>
__global__ void __launch_bounds__(256) mfma_issue_kernel(float *out, int iters)
{
    constexpr int NOP = VARIED ? kAcc : 1;       // distinct operand pairs
    floatx4 acc[kAcc];
#pragma unroll
    for (int i = 0; i < kAcc; ++i) acc[i] = floatx4{0.f, 0.f, 0.f, 0.f};
    const float seed = (float)threadIdx.x * 0.001f;
    const unsigned tid = blockIdx.x * blockDim.x + threadIdx.x;
    if constexpr (DT == SK_F32) {
        float a[NOP], b[NOP];
#pragma unroll
        for (int i = 0; i < NOP; ++i) {
            if constexpr (VARIED) {
                a[i] = __uint_as_float(0x3f800000u | (probe_hash(tid * 16 + i) >> 9)) - 1.5f;        // [-0.5, 0.5)
                b[i] = __uint_as_float(0x3f800000u | (probe_hash(tid * 16 + 8 + i) >> 9)) - 1.5f;
            } else {
                a[i] = seed;
                b[i] = 1.0f;
            }
        }
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int i = 0; i < kAcc; ++i) asm volatile("v_mfma_f32_16x16x4_f32 %0, %1, %2, %0" : "+v"(acc[i]) : "v"(a[i % NOP]), "v"(b[i % NOP]));
        }
    } else {
        uintx4 a[NOP], b[NOP];
#pragma unroll
        for (int i = 0; i < NOP; ++i)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                if constexpr (VARIED) {
                    const unsigned ha = probe_hash((tid * 16 + i) * 8 + e), hb = probe_hash((tid * 16 + 8 + i) * 8 + e);
                    a[i][e] = probe_half_bits<DT>(ha & 0xffffu) | (probe_half_bits<DT>(ha >> 16) << 16);
                    b[i][e] = probe_half_bits<DT>(hb & 0xffffu) | (probe_half_bits<DT>(hb >> 16) << 16);
                } else if constexpr (DT == SK_BF16) {
                    const unsigned sa = __builtin_bit_cast(unsigned short, (__bf16)seed), sb = __builtin_bit_cast(unsigned short, (__bf16)1.0f);
                    a[i][e] = sa | (sa << 16);
                    b[i][e] = sb | (sb << 16);
                } else {
                    const unsigned sa = __builtin_bit_cast(unsigned short, (_Float16)seed), sb = __builtin_bit_cast(unsigned short, (_Float16)1.0f);
                    a[i][e] = sa | (sa << 16);
                    b[i][e] = sb | (sb << 16);
                }
            }
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int i = 0; i < kAcc; ++i) {
                if constexpr (DT == SK_BF16) asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+v"(acc[i]) : "v"(a[i % NOP]), "v"(b[i % NOP]));
                else asm volatile("v_mfma_f32_16x16x32_f16 %0, %1, %2, %0" : "+v"(acc[i]) : "v"(a[i % NOP]), "v"(b[i % NOP]));
            }
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

sk_status sk_probe_mfma(int32_t dtype, int32_t operands, int32_t iters, void *hip_stream, double *tflops)
{
    if (!tflops || iters < 1 || iters > (1 << 22)) return fail(SK_EINVAL, "probe_mfma: bad arguments");
    if (dtype != SK_F32 && dtype != SK_BF16 && dtype != SK_F16) return fail(SK_EINVAL, "probe_mfma: unknown dtype %d", dtype);
    if (operands != 0 && operands != 1) return fail(SK_EINVAL, "probe_mfma: operands must be 0 (constant) or 1 (varied)");
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    int dev = 0, cus = 0;
    SK_HIP(hipGetDevice(&dev));
    SK_HIP(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
    const int blocks = cus * 4, threads = 256;   // 16 waves per CU, four per SIMD
    float *out = nullptr;
    SK_HIP(hipMalloc(&out, (size_t)blocks * threads * sizeof(float)));
    float ms = 0.f;
    void (*kernel)(float *, int) = nullptr;
    if (dtype == SK_F32) kernel = operands ? mfma_issue_kernel<SK_F32, true> : mfma_issue_kernel<SK_F32, false>;
    else if (dtype == SK_BF16) kernel = operands ? mfma_issue_kernel<SK_BF16, true> : mfma_issue_kernel<SK_BF16, false>;
    else kernel = operands ? mfma_issue_kernel<SK_F16, true> : mfma_issue_kernel<SK_F16, false>;
    sk_status st = time_launches(stream, 3, [&] { hipLaunchKernelGGL(kernel, dim3(blocks), dim3(threads), 0, stream, out, iters); }, &ms);
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
