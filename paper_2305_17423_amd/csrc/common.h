// Internal helpers of the fise library (gfx950 only).  Not part of the ABI.
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_bf16.h>
#include <cstdarg>
#include <cstdint>
#include <cstdio>
#include "../../include/fise.h"

namespace fise {

void set_error(const char* fmt, ...);
int fail(int code, const char* fmt, ...);

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline hipStream_t as_stream(void* s) { return reinterpret_cast<hipStream_t>(s); }
inline int ceil_div(int a, int b) { return (a + b - 1) / b; }
inline size_t align256(size_t x) { return (x + 255) & ~size_t(255); }

#define FISE_CHECK_LAUNCH(what)                                                        \
    do {                                                                               \
        hipError_t e__ = hipGetLastError();                                            \
        if (e__ != hipSuccess) return fise::fail(FISE_ERR_HIP, "%s: %s", what, hipGetErrorString(e__)); \
    } while (0)

// ---- bf16 <-> float on the device (round to nearest even) ----
typedef unsigned short bf16_t;                       // raw bits
typedef __attribute__((ext_vector_type(8))) short bf16x8_t;   // MFMA operand (8 bf16)
typedef __attribute__((ext_vector_type(16))) float f32x16_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;

typedef __bf16 hw_bf16x2_t __attribute__((ext_vector_type(2)));
typedef float hw_f32x2_t __attribute__((ext_vector_type(2)));

__device__ __forceinline__ float bf2f(bf16_t v) { return __uint_as_float(((unsigned)v) << 16); }
// two floats -> packed bf16 pair (lo in bits 0..15), round to nearest even: one v_cvt_pk_bf16_f32
__device__ __forceinline__ unsigned f2bf2(float lo, float hi) {
    hw_f32x2_t v = {lo, hi};
    hw_bf16x2_t r = __builtin_convertvector(v, hw_bf16x2_t);
    return *reinterpret_cast<unsigned*>(&r);
}
__device__ __forceinline__ bf16_t f2bf(float f) { return (bf16_t)(f2bf2(f, 0.f) & 0xffffu); }
// x * sigmoid(x); the reciprocal is the hardware approximation (1 ulp), far below bf16 resolution
__device__ __forceinline__ float silu_f(float u) { return u * __builtin_amdgcn_rcpf(1.0f + __expf(-u)); }

template <typename T> struct Elem;
template <> struct Elem<float> {
    static __device__ __forceinline__ float ld(const float* p) { return *p; }
    static __device__ __forceinline__ void st(float* p, float v) { *p = v; }
};
template <> struct Elem<bf16_t> {
    static __device__ __forceinline__ float ld(const bf16_t* p) { return bf2f(*p); }
    static __device__ __forceinline__ void st(bf16_t* p, float v) { *p = f2bf(v); }
};

// Active-pixel enumeration shared by all masked kernels: row m of the active set
// -> (y, x) on a map that is `tiles_w` tiles wide, tiles of th x tw pixels, row-major
// inside a tile.
__device__ __forceinline__ void active_pixel(const int* __restrict__ tile_idx, int m, int th, int tw, int tiles_w,
                                             int& y, int& x) {
    const int tt = th * tw;
    const int t = tile_idx[m / tt];
    const int p = m % tt;
    y = (t / tiles_w) * th + p / tw;
    x = (t % tiles_w) * tw + p % tw;
}
// square tiles of edge `tile`
__device__ __forceinline__ void active_pixel(const int* __restrict__ tile_idx, int m, int tile, int tiles_w,
                                             int& y, int& x) {
    active_pixel(tile_idx, m, tile, tile, tiles_w, y, x);
}

}  // namespace fise
