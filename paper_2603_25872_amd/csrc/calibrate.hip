// Calibration kernels for roofline denominators: what this GPU delivers for a loop of nothing but
// the GEMM's MFMA instruction, and for a plain copy.  Measurement hooks only; no step of the
// sampling path calls them.
#include "common.h"
#include "../../include/drf_measure.h"

namespace {

typedef drf::bf16_t bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kMfmaPerIter = 16, kItersPerLaunch = 4096, kWavesPerBlock = 8, kBlocks = 1024;

__device__ inline uint32_t mix(uint32_t x)
{
    x ^= x >> 16; x *= 0x7feb352dU; x ^= x >> 15; x *= 0x846ca68bU; x ^= x >> 16;
    return x;
}

// 4 x 4 operand register sets, 16 independent accumulators: no MFMA waits for another one's result.
__global__ void __launch_bounds__(kWavesPerBlock * 64) mfma_loop_kernel(int random_operands, int iters, float* sink)
{
    bf16x8 a[4], b[4];
    const uint32_t id = blockIdx.x * blockDim.x + threadIdx.x;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            // random: sign and 7 mantissa bits from a hash, exponents 2^-2 .. 2^1; constant: 1.0 / 0.5
            const uint32_t ha = mix(id * 64u + i * 8u + e), hb = mix(~id * 64u + i * 8u + e);
            const uint16_t ra = (uint16_t)((ha & 0x807fu) | ((125u + ((ha >> 8) & 3u)) << 7));
            const uint16_t rb = (uint16_t)((hb & 0x807fu) | ((125u + ((hb >> 8) & 3u)) << 7));
            const uint16_t ua = random_operands ? ra : (uint16_t)0x3f80u, ub = random_operands ? rb : (uint16_t)0x3f00u;
            a[i][e] = __builtin_bit_cast(drf::bf16_t, ua);
            b[i][e] = __builtin_bit_cast(drf::bf16_t, ub);
        }
    f32x4 acc[kMfmaPerIter];
#pragma unroll
    for (int k = 0; k < kMfmaPerIter; ++k) acc[k] = (f32x4){ 0.f, 0.f, 0.f, 0.f };
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int k = 0; k < kMfmaPerIter; ++k)
            acc[k] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[k & 3], b[k >> 2], acc[k], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int k = 0; k < kMfmaPerIter; ++k) s += acc[k][0] + acc[k][1] + acc[k][2] + acc[k][3];
    if (s == 12345.678f) sink[0] = s;               // keeps the loop alive; practically never taken
}

__global__ void __launch_bounds__(256) copy16_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t n)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) dst[i] = src[i];
}

// Mean duration (ms) of `iters` launches of `launch` between two events on `st`, after one warm-up launch.
template <typename F> drf_status time_launches(F&& launch, int iters, hipStream_t st, double* ms)
{
    hipEvent_t e0 = nullptr, e1 = nullptr;
    DRF_HIP(hipEventCreate(&e0));
    if (hipEventCreate(&e1) != hipSuccess) { (void)hipEventDestroy(e0); DRF_FAIL(DRF_EHIP, "event creation failed"); }
    launch();
    hipError_t err = hipEventRecord(e0, st);
    for (int i = 0; i < iters; ++i) launch();
    if (err == hipSuccess) err = hipEventRecord(e1, st);
    if (err == hipSuccess) err = hipEventSynchronize(e1);
    if (err == hipSuccess) err = hipGetLastError();
    float t = 0.f;
    if (err == hipSuccess) err = hipEventElapsedTime(&t, e0, e1);
    (void)hipEventDestroy(e0); (void)hipEventDestroy(e1);
    if (err != hipSuccess) DRF_FAIL(DRF_EHIP, "calibration launch failed: %s", hipGetErrorString(err));
    *ms = (double)t / iters;
    return DRF_OK;
}

}  // namespace

extern "C" drf_status drf_calibrate_mfma_bf16(int random_operands, int iters, double* tflops, void* hip_stream)
{
    if (!tflops || iters < 1 || iters > 1000) DRF_FAIL(DRF_EINVAL, "bad argument");
    hipStream_t st = (hipStream_t)hip_stream;
    float* sink = nullptr;
    if (hipMalloc((void**)&sink, 256) != hipSuccess) { (void)hipGetLastError(); DRF_FAIL(DRF_ENOMEM, "device allocation failed"); }
    double ms = 0.0;
    const drf_status rc = time_launches([&] {
        hipLaunchKernelGGL(mfma_loop_kernel, dim3(kBlocks), dim3(kWavesPerBlock * 64), 0, st, random_operands, kItersPerLaunch, sink);
    }, iters, st, &ms);
    (void)hipFree(sink);
    if (rc != DRF_OK) return rc;
    const double flops = 2.0 * 16 * 16 * 32 * kMfmaPerIter * (double)kItersPerLaunch * kWavesPerBlock * kBlocks;
    *tflops = flops / (ms * 1e-3) / 1e12;
    return DRF_OK;
}

extern "C" drf_status drf_calibrate_copy(const void* src, void* dst, size_t bytes, int iters, double* gbps, void* hip_stream)
{
    if (!src || !dst || !gbps || iters < 1 || iters > 1000 || bytes == 0 || bytes % 16 != 0 ||
        ((uintptr_t)src & 15u) || ((uintptr_t)dst & 15u))
        DRF_FAIL(DRF_EINVAL, "bad argument");
    hipStream_t st = (hipStream_t)hip_stream;
    const size_t n = bytes / 16;
    size_t blocks = (n + 255) / 256;
    if (blocks > 256 * 32) blocks = 256 * 32;
    double ms = 0.0;
    const drf_status rc = time_launches([&] {
        hipLaunchKernelGGL(copy16_kernel, dim3((unsigned)blocks), dim3(256), 0, st, (const uint4*)src, (uint4*)dst, n);
    }, iters, st, &ms);
    if (rc != DRF_OK) return rc;
    *gbps = 2.0 * (double)bytes / (ms * 1e-3) / 1e9;
    return DRF_OK;
}
