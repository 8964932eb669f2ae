// Empirical ceilings of the device: what a plain streaming copy and a register-resident
// MFMA loop reach on this GPU.  Measurement support for the benchmark: the published peaks
// (8 TB/s, 2.5 PFLOP/s dense bf16) are what fractions are quoted against; these two figures
// say how much of them any kernel could see at all.
#include "common.h"
#include <algorithm>
#include <cstdlib>

namespace fise {

// dst[i] = src[i], 16 bytes per lane, grid-stride.
__global__ __launch_bounds__(256) void calib_copy_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t n) {
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) dst[i] = src[i];
}

// The same copy with four loads in flight per lane before the first store (each a full 4 KiB per wave apart, so every
// wave-wide access stays one contiguous kilobyte); the ceiling reported is the better of the two.
__global__ __launch_bounds__(256) void calib_stream4_kernel(const uint4* __restrict__ src_, uint4* __restrict__ dst_, size_t n) {
    typedef unsigned u32x4v __attribute__((ext_vector_type(4)));
    const u32x4v* src = (const u32x4v*)src_;
    u32x4v* dst = (u32x4v*)dst_;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    for (; i + 3 * stride < n; i += 4 * stride) {
        const u32x4v v0 = __builtin_nontemporal_load(src + i), v1 = __builtin_nontemporal_load(src + i + stride);
        const u32x4v v2 = __builtin_nontemporal_load(src + i + 2 * stride), v3 = __builtin_nontemporal_load(src + i + 3 * stride);
        __builtin_nontemporal_store(v0, dst + i); __builtin_nontemporal_store(v1, dst + i + stride);
        __builtin_nontemporal_store(v2, dst + i + 2 * stride); __builtin_nontemporal_store(v3, dst + i + 3 * stride);
    }
    for (; i < n; i += stride) dst[i] = src[i];
}

// Four independent 32x32 accumulators per wave, operands never reloaded: the matrix pipe
// issues back to back.  The sums are stored so that the loop is kept.
__global__ __launch_bounds__(256) void calib_mfma_kernel(float* __restrict__ sink, int iters) {
    const int lane = threadIdx.x & 63;
    bf16x8_t a, b;
#pragma unroll
    for (int i = 0; i < 8; ++i) { a[i] = (short)(0x3f80 + ((lane + i) & 3)); b[i] = (short)(0x3f80 + ((lane * 3 + i) & 3)); }
    f32x16_t c0 = {}, c1 = {}, c2 = {}, c3 = {};
    for (int it = 0; it < iters; ++it) {
        c0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c0, 0, 0, 0);
        c1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c1, 0, 0, 0);
        c2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c2, 0, 0, 0);
        c3 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c3, 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) s += c0[i] + c1[i] + c2[i] + c3[i];
    sink[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = s;
}

namespace {
constexpr int kMfmaBlocks = 256 * 8, kMfmaIters = 2048;
constexpr size_t kSinkBytes = (size_t)kMfmaBlocks * 256 * sizeof(float);

template <typename F>
int best_of(F&& launch, int reps, hipStream_t st, double* best_ms) {
    hipEvent_t e0 = nullptr, e1 = nullptr;
    if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) {
        if (e0) (void)hipEventDestroy(e0);
        return fail(FISE_ERR_HIP, "fise_calibrate_peaks: hipEventCreate failed");
    }
    int rc = FISE_OK;
    *best_ms = 1e30;
    for (int r = 0; r < reps + 2 && rc == FISE_OK; ++r) {           // the first two passes warm caches and clocks
        (void)hipEventRecord(e0, st);
        launch();
        (void)hipEventRecord(e1, st);
        if (hipGetLastError() != hipSuccess || hipEventSynchronize(e1) != hipSuccess) {
            rc = fail(FISE_ERR_HIP, "fise_calibrate_peaks: launch or wait failed");
            break;
        }
        float ms = 0.f;
        (void)hipEventElapsedTime(&ms, e0, e1);
        if (r >= 2 && ms < *best_ms) *best_ms = ms;
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    return rc;
}
}  // namespace
}  // namespace fise

using namespace fise;

extern "C" int fise_calibrate_peaks(void* scratch, size_t scratch_bytes, double* copy_gbs, double* mfma_bf16_tflops, void* stream) {
    if (!scratch || !copy_gbs || !mfma_bf16_tflops) return fail(FISE_ERR_NULL, "fise_calibrate_peaks: null pointer");
    if (!aligned16(scratch)) return fail(FISE_ERR_ALIGN, "fise_calibrate_peaks: scratch %p not 16-byte aligned", scratch);
    if (scratch_bytes < (size_t(64) << 20))
        return fail(FISE_ERR_CAPACITY, "fise_calibrate_peaks: scratch of %zu bytes, at least 64 MiB wanted", scratch_bytes);
    hipStream_t st = as_stream(stream);
    const size_t half = (scratch_bytes / 2) & ~size_t(4095);
    const size_t n16 = half / 16;
    const uint4* src = (const uint4*)scratch;
    uint4* dst = (uint4*)((char*)scratch + half);
    double ms = 0;
    if (int e = best_of([&] { hipLaunchKernelGGL(calib_copy_kernel, dim3(256 * 16), dim3(256), 0, st, src, dst, n16); }, 5, st, &ms)) return e;
    double ms4 = 0;
    if (int e = best_of([&] { hipLaunchKernelGGL(calib_stream4_kernel, dim3(256 * 8), dim3(256), 0, st, src, dst, n16); }, 5, st, &ms4)) return e;
    if (std::getenv("FISE_DEBUG")) fprintf(stderr, "[fise] copy ceilings: plain %.0f GB/s, four in flight %.0f GB/s\n",
                                           2.0 * half / (ms * 1e-3) / 1e9, 2.0 * half / (ms4 * 1e-3) / 1e9);
    ms = std::min(ms, ms4);
    *copy_gbs = 2.0 * (double)half / (ms * 1e-3) / 1e9;              // bytes read + bytes written
    float* sink = (float*)scratch;
    static_assert(kSinkBytes <= (size_t(64) << 20), "sink fits the smallest scratch");
    if (int e = best_of([&] { hipLaunchKernelGGL(calib_mfma_kernel, dim3(kMfmaBlocks), dim3(256), 0, st, sink, kMfmaIters); }, 5, st, &ms)) return e;
    const double flops = (double)kMfmaBlocks * 4 /*waves*/ * kMfmaIters * 4 /*accumulators*/ * (2.0 * 32 * 32 * 16);
    *mfma_bf16_tflops = flops / (ms * 1e-3) / 1e12;
    return FISE_OK;
}
