// Normalisation kernels: dense GroupNorm statistics (two-stage, deterministic),
// masked GroupNorm+SiLU with given statistics, per-row LayerNorm of compact
// token buffers.
#include <algorithm>
#include <mutex>
#include "igemm.h"

namespace fise {

constexpr int GS_PIX = 64;       // pixels per stage-1 workgroup
constexpr int GS_MAXJ = 4;       // channels per thread per pass (256 threads -> 1024 channels per pass)

// stage 1: partial[b][chunk][g] = (sum, sum of squares) over GS_PIX pixels x the group's channels.
template <typename T>
__global__ __launch_bounds__(256) void gn_partial_kernel(const T* __restrict__ x0, const T* __restrict__ x1, int HW,
                                                         int C0, int C1, int G, double2* __restrict__ partial) {
    extern __shared__ double2 chan[];                    // [C0 + C1]
    const int C = C0 + C1, cpg = C / G;
    const int b = blockIdx.y, chunk = blockIdx.x, nchunk = gridDim.x;
    const int p0 = chunk * GS_PIX, p1 = min(HW, p0 + GS_PIX);
    for (int cbase = 0; cbase < C; cbase += 256 * GS_MAXJ) {
        float s[GS_MAXJ], q[GS_MAXJ];
#pragma unroll
        for (int j = 0; j < GS_MAXJ; ++j) { s[j] = 0.f; q[j] = 0.f; }
        for (int p = p0; p < p1; ++p) {
#pragma unroll
            for (int j = 0; j < GS_MAXJ; ++j) {
                const int c = cbase + threadIdx.x + 256 * j;
                if (c < C) {
                    const float v = c < C0 ? Elem<T>::ld(x0 + ((size_t)b * HW + p) * C0 + c)
                                           : Elem<T>::ld(x1 + ((size_t)b * HW + p) * C1 + (c - C0));
                    s[j] += v; q[j] += v * v;
                }
            }
        }
#pragma unroll
        for (int j = 0; j < GS_MAXJ; ++j) {
            const int c = cbase + threadIdx.x + 256 * j;
            if (c < C) chan[c] = make_double2((double)s[j], (double)q[j]);
        }
    }
    __syncthreads();
    for (int g = threadIdx.x; g < G; g += 256) {
        double s = 0, q = 0;
        for (int c = g * cpg; c < (g + 1) * cpg; ++c) { s += chan[c].x; q += chan[c].y; }
        partial[((size_t)b * nchunk + chunk) * G + g] = make_double2(s, q);
    }
}

// stage 1 for bf16 maps whose channel counts are multiples of 8: 16-byte loads, and the chunk's pixels dealt to as
// many pixel stripes as 256 lanes allow (lane = (stripe, 8-channel piece)), so that a lane's loads do not wait for one
// another.  Stripe sums are float (a dozen terms each), added per channel in stripe order in double.
__global__ __launch_bounds__(256) void gn_partial_vec_kernel(const bf16_t* __restrict__ x0, const bf16_t* __restrict__ x1, int HW,
                                                             int C0, int C1, int G, int gps, double2* __restrict__ partial) {
    extern __shared__ double2 chan[];                    // [channels of the slab], then the stripe sums of one pass
    const int C = C0 + C1, cpg = C / G, tid = threadIdx.x;
    // blockIdx.z: a slab of gps whole groups (its channel range starts and ends on a multiple of 8)
    const int g0 = blockIdx.z * gps, g1 = min(G, g0 + gps);
    const int c_lo = g0 * cpg, CH8 = (g1 - g0) * cpg / 8;
    float2* stripe = reinterpret_cast<float2*>(chan + C);        // [stripes][pieces of the pass][8]
    const int b = blockIdx.y, chunk = blockIdx.x, nchunk = gridDim.x;
    const int p0 = chunk * GS_PIX, p1 = min(HW, p0 + GS_PIX);
    for (int pc = 0; pc < CH8; pc += 256) {
        const int CH = min(256, CH8 - pc), PS = 256 / CH;
        const int cc = tid % CH, ps = tid / CH;
        if (ps < PS) {
            const int c = c_lo + (pc + cc) * 8;
            const bf16_t* src = c < C0 ? x0 + (size_t)b * HW * C0 + c : x1 + (size_t)b * HW * C1 + (c - C0);
            const size_t pitch = c < C0 ? C0 : C1;
            float s[8], q[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) { s[j] = 0.f; q[j] = 0.f; }
            for (int p = p0 + ps; p < p1; p += PS) {
                const uint4 v = *reinterpret_cast<const uint4*>(src + (size_t)p * pitch);
                const unsigned w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const float lo = __uint_as_float(w[j] << 16), hi = __uint_as_float(w[j] & 0xffff0000u);
                    s[2 * j] += lo; q[2 * j] += lo * lo; s[2 * j + 1] += hi; q[2 * j + 1] += hi * hi;
                }
            }
#pragma unroll
            for (int j = 0; j < 8; ++j) stripe[(ps * CH + cc) * 8 + j] = make_float2(s[j], q[j]);
        }
        __syncthreads();
        for (int i = tid; i < CH * 8; i += 256) {
            double ds = 0, dq = 0;
            for (int k = 0; k < PS; ++k) { const float2 v = stripe[k * CH * 8 + i]; ds += (double)v.x; dq += (double)v.y; }
            chan[pc * 8 + i] = make_double2(ds, dq);
        }
        __syncthreads();
    }
    for (int g = g0 + tid; g < g1; g += 256) {
        double s = 0, q = 0;
        for (int c = g * cpg - c_lo; c < (g + 1) * cpg - c_lo; ++c) { s += chan[c].x; q += chan[c].y; }
        partial[((size_t)b * nchunk + chunk) * G + g] = make_double2(s, q);
    }
}

// stage 2: one wave per (b, g); lane k adds chunks k, k + 64, ... in that order, the 64 lane sums are added in a
// fixed tree.
// With ss the wave also writes the group's channels of the (scale, shift) table, from the rounded statistics it has
// just stored: ss[b, c] = (rstd * gamma[c], beta[c] - mean * rstd * gamma[c]).
__global__ __launch_bounds__(64) void gn_finish_kernel(const double2* __restrict__ partial, int nchunk, int BG, int G, double count,
                                                       float eps, float* __restrict__ mean, float* __restrict__ rstd,
                                                       const bf16_t* __restrict__ gamma, const bf16_t* __restrict__ beta, int C,
                                                       float2* __restrict__ ss) {
    const int i = blockIdx.x, lane = threadIdx.x;
    if (i >= BG) return;
    const int b = i / G, g = i % G;
    double s = 0, q = 0;
    for (int k = lane; k < nchunk; k += 64) { const double2 v = partial[((size_t)b * nchunk + k) * G + g]; s += v.x; q += v.y; }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) { s += __shfl_down(s, off); q += __shfl_down(q, off); }
    s = __shfl(s, 0); q = __shfl(q, 0);
    const double m = s / count;
    double var = q / count - m * m;
    if (var < 0) var = 0;
    const float mf = (float)m, rf = (float)(1.0 / sqrt(var + (double)eps));
    if (lane == 0) { mean[i] = mf; rstd[i] = rf; }
    if (ss) {
        const int cpg = C / G;
        for (int c = g * cpg + lane; c < (g + 1) * cpg; c += 64) {
            const float sc = rf * bf2f(gamma[c]);
            ss[(size_t)b * C + c] = make_float2(sc, fmaf(-mf, sc, bf2f(beta[c])));
        }
    }
}

template <typename T>
__global__ void masked_gn_silu_kernel(const T* __restrict__ x, const float* __restrict__ mean, const float* __restrict__ rstd,
                                      const T* __restrict__ gamma, const T* __restrict__ beta, int B, int H, int W, int C,
                                      int G, const int* __restrict__ tile_idx, int Ma, int tile, T* __restrict__ y) {
    const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    const long long total = (long long)B * Ma * C;
    if (i >= total) return;
    const int c = (int)(i % C);
    const int m = (int)((i / C) % Ma);
    const int b = (int)(i / ((long long)C * Ma));
    int py, px;
    active_pixel(tile_idx, m, tile, W / tile, py, px);
    const size_t off = (((size_t)b * H + py) * W + px) * C + c;
    const int g = c / (C / G);
    const float u = (Elem<T>::ld(x + off) - mean[b * G + g]) * rstd[b * G + g] * Elem<T>::ld(gamma + c) + Elem<T>::ld(beta + c);
    Elem<T>::st(y + off, silu_f(u));
}

// SiLU(GroupNorm(x)) with given statistics, written once for every pixel of the active tiles AND
// their one-pixel ring (clipped to the image) into a scratch map act[B,H,W,C0+C1]: the 3x3
// convolution that follows reads plain activations instead of re-evaluating the nonlinearity for
// each of its nine taps and each of its column tiles.  Neighbouring tiles write identical values
// to their shared ring.  One thread per (pixel, 8 channels).
__global__ __launch_bounds__(256) void gn_act_halo_kernel(const bf16_t* __restrict__ x0, const bf16_t* __restrict__ x1, int C0,
                                                          int C1, int H, int W, const float* __restrict__ mean,
                                                          const float* __restrict__ rstd, const bf16_t* __restrict__ gamma,
                                                          const bf16_t* __restrict__ beta, int G, int silu,
                                                          const int* __restrict__ tile_idx, int tile, bf16_t* __restrict__ act) {
    const int C = C0 + C1, chunks = C / 8, side = tile + 2;
    const int t = tile_idx[blockIdx.x], b = blockIdx.y;
    const int tiles_w = W / tile;
    const int y0 = (t / tiles_w) * tile - 1, x0p = (t % tiles_w) * tile - 1;
    const int items = side * side * chunks;
    const int cpg = C / G;
    for (int it = blockIdx.z * 256 + threadIdx.x; it < items; it += gridDim.z * 256) {
        const int p = it / chunks, ch = it % chunks;
        const int y = y0 + p / side, x = x0p + p % side;
        if (y < 0 || y >= H || x < 0 || x >= W) continue;
        const int c = ch * 8;
        const size_t pix = ((size_t)b * H + y) * W + x;
        const uint4 v = c < C0 ? *reinterpret_cast<const uint4*>(x0 + pix * C0 + c)
                               : *reinterpret_cast<const uint4*>(x1 + pix * C1 + (c - C0));
        const uint4 gv = *reinterpret_cast<const uint4*>(gamma + c), bv = *reinterpret_cast<const uint4*>(beta + c);
        const unsigned xw[4] = {v.x, v.y, v.z, v.w}, gw[4] = {gv.x, gv.y, gv.z, gv.w}, bw[4] = {bv.x, bv.y, bv.z, bv.w};
        unsigned ow[4];
        // the 8 channels of a chunk lie in one group or straddle one boundary (cpg >= 8 here; else divide per channel)
        const int g0 = c / cpg, edge = (g0 + 1) * cpg;
        const int g1 = min(g0 + 1, G - 1);
        const float mu0 = mean[b * G + g0], rs0 = rstd[b * G + g0], mu1 = mean[b * G + g1], rs1 = rstd[b * G + g1];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            float r[2];
#pragma unroll
            for (int q = 0; q < 2; ++q) {
                const int cc = c + 2 * e + q;
                float mu, rs;
                if (cpg >= 8) { const bool hi = cc >= edge; mu = hi ? mu1 : mu0; rs = hi ? rs1 : rs0; }
                else { const int g = cc / cpg; mu = mean[b * G + g]; rs = rstd[b * G + g]; }
                const float xv = q ? __uint_as_float(xw[e] & 0xffff0000u) : __uint_as_float(xw[e] << 16);
                const float ga = q ? __uint_as_float(gw[e] & 0xffff0000u) : __uint_as_float(gw[e] << 16);
                const float be = q ? __uint_as_float(bw[e] & 0xffff0000u) : __uint_as_float(bw[e] << 16);
                const float sc = rs * ga;
                float u = fmaf(xv, sc, fmaf(-mu, sc, be));      // the same two operations as the scale / shift table form
                if (silu) u = silu_f(u);
                r[q] = u;
            }
            ow[e] = f2bf2(r[0], r[1]);
        }
        *reinterpret_cast<uint4*>(act + pix * C + c) = make_uint4(ow[0], ow[1], ow[2], ow[3]);
    }
}

__global__ void gn_scale_shift_kernel(const float* __restrict__ mean, const float* __restrict__ rstd, const bf16_t* __restrict__ gamma,
                                      const bf16_t* __restrict__ beta, int B, int C, int G, float2* __restrict__ ss) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= B * C) return;
    const int b = i / C, c = i - b * C, g = c / (C / G);
    const float sc = rstd[b * G + g] * bf2f(gamma[c]);
    ss[i] = make_float2(sc, fmaf(-mean[b * G + g], sc, bf2f(beta[c])));
}

int launch_gn_scale_shift(const float* mean, const float* rstd, const void* gamma, const void* beta, int B, int C, int G, float2* ss,
                          hipStream_t st) {
    hipLaunchKernelGGL(gn_scale_shift_kernel, dim3(ceil_div(B * C, 256)), dim3(256), 0, st, mean, rstd, (const bf16_t*)gamma,
                       (const bf16_t*)beta, B, C, G, ss);
    FISE_CHECK_LAUNCH("gn scale/shift table");
    return FISE_OK;
}

int launch_gn_act_halo(const void* x0, const void* x1, int C0, int C1, int B, int H, int W, const float* mean, const float* rstd,
                       const void* gamma, const void* beta, int G, int silu, const int* tile_idx, int n_active, int tile, void* act,
                       hipStream_t st) {
    if (n_active <= 0) return FISE_OK;
    const int items = (tile + 2) * (tile + 2) * ((C0 + C1) / 8);
    const int z = std::max(1, std::min(64, ceil_div(items, 512)));
    hipLaunchKernelGGL(gn_act_halo_kernel, dim3(n_active, B, z), dim3(256), 0, st, (const bf16_t*)x0, (const bf16_t*)x1, C0, C1, H, W,
                       mean, rstd, (const bf16_t*)gamma, (const bf16_t*)beta, G, silu, tile_idx, tile, (bf16_t*)act);
    FISE_CHECK_LAUNCH("gn activation with halo");
    return FISE_OK;
}

// LayerNorm of rows -> compact out[rows, C] (bf16).  General form: one wave per row held in
// registers (C <= 2048): one read, mean, centred variance, one write.  With tile_idx the rows are
// gathered from a token map.
constexpr int LN_MAXJ = 32;
template <typename T>
__global__ __launch_bounds__(256) void ln_rows_kernel(const T* __restrict__ in, int rows, int C,
                                                      const bf16_t* __restrict__ gamma, const bf16_t* __restrict__ beta,
                                                      float eps, bf16_t* __restrict__ out, const int* __restrict__ tile_idx,
                                                      int tile, int tiles_w, int H, int W, int Ma) {
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    if (row >= rows) return;
    const T* r;
    if (tile_idx) {
        int py, px;
        active_pixel(tile_idx, row % Ma, tile, tiles_w, py, px);
        r = in + (((size_t)(row / Ma) * H + py) * W + px) * C;
    } else {
        r = in + (size_t)row * C;
    }
    float v[LN_MAXJ];
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < LN_MAXJ; ++j) {
        const int c = lane + 64 * j;
        v[j] = c < C ? Elem<T>::ld(r + c) : 0.f;
        s += v[j];
    }
    for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o);
    const float mu = s / C;
    float q = 0.f;
#pragma unroll
    for (int j = 0; j < LN_MAXJ; ++j) {
        const int c = lane + 64 * j;
        const float d = c < C ? v[j] - mu : 0.f;
        q += d * d;
    }
    for (int o = 32; o > 0; o >>= 1) q += __shfl_xor(q, o);
    const float rs = rsqrtf(q / C + eps);
#pragma unroll
    for (int j = 0; j < LN_MAXJ; ++j) {
        const int c = lane + 64 * j;
        if (c < C) out[(size_t)row * C + c] = f2bf((v[j] - mu) * rs * bf2f(gamma[c]) + bf2f(beta[c]));
    }
}

// Fast form for compact float rows with C = 20 * LPR (320 / 640 / 1280 at LPR = 16 / 32 / 64): LPR lanes
// share a row, each holds 5 x float4 = 20 consecutive channels; 16-byte loads, 8-byte bf16 stores.
template <int LPR>
__global__ __launch_bounds__(256) void ln_rows20_kernel(const float* __restrict__ in, int rows, const bf16_t* __restrict__ gamma,
                                                        const bf16_t* __restrict__ beta, float eps, bf16_t* __restrict__ out) {
    constexpr int C = 20 * LPR, RPB = 256 / LPR;
    const int row = blockIdx.x * RPB + threadIdx.x / LPR;
    const int l = threadIdx.x % LPR;
    if (row >= rows) return;                      // whole LPR-lane groups leave together
    const float4* r = reinterpret_cast<const float4*>(in + (size_t)row * C + l * 20);
    float4 v[5];
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < 5; ++j) { v[j] = r[j]; s += (v[j].x + v[j].y) + (v[j].z + v[j].w); }
#pragma unroll
    for (int o = LPR / 2; o > 0; o >>= 1) s += __shfl_xor(s, o);
    const float mu = s / C;
    float q = 0.f;
#pragma unroll
    for (int j = 0; j < 5; ++j) {
        const float a0 = v[j].x - mu, a1 = v[j].y - mu, a2 = v[j].z - mu, a3 = v[j].w - mu;
        q += (a0 * a0 + a1 * a1) + (a2 * a2 + a3 * a3);
    }
#pragma unroll
    for (int o = LPR / 2; o > 0; o >>= 1) q += __shfl_xor(q, o);
    const float rs = rsqrtf(q / C + eps);
    const uint2* g2 = reinterpret_cast<const uint2*>(gamma + l * 20);
    const uint2* b2 = reinterpret_cast<const uint2*>(beta + l * 20);
    uint2* o2 = reinterpret_cast<uint2*>(out + (size_t)row * C + l * 20);
#pragma unroll
    for (int j = 0; j < 5; ++j) {
        const uint2 gv = g2[j], bv = b2[j];
        const float y0 = (v[j].x - mu) * rs * __uint_as_float(gv.x << 16) + __uint_as_float(bv.x << 16);
        const float y1 = (v[j].y - mu) * rs * __uint_as_float(gv.x & 0xffff0000u) + __uint_as_float(bv.x & 0xffff0000u);
        const float y2 = (v[j].z - mu) * rs * __uint_as_float(gv.y << 16) + __uint_as_float(bv.y << 16);
        const float y3 = (v[j].w - mu) * rs * __uint_as_float(gv.y & 0xffff0000u) + __uint_as_float(bv.y & 0xffff0000u);
        o2[j] = make_uint2(f2bf2(y0, y1), f2bf2(y2, y3));
    }
}

int launch_ln_rows(const void* in, int in_f32, int rows, int C, const void* gamma, const void* beta, float eps, void* out,
                   const int* tile_idx, int tile, int tiles_w, int H, int W, int Ma, hipStream_t st) {
    if (rows <= 0) return FISE_OK;
    if (C > 64 * LN_MAXJ) return fail(FISE_ERR_SHAPE, "layernorm rows: C=%d > %d", C, 64 * LN_MAXJ);
    const dim3 grid(ceil_div(rows, 4)), block(256);
    if (in_f32 && !tile_idx && (C == 320 || C == 640 || C == 1280)) {
        const float* x = (const float*)in; const bf16_t* g = (const bf16_t*)gamma; const bf16_t* b = (const bf16_t*)beta;
        if (C == 320) hipLaunchKernelGGL(ln_rows20_kernel<16>, dim3(ceil_div(rows, 16)), block, 0, st, x, rows, g, b, eps, (bf16_t*)out);
        else if (C == 640) hipLaunchKernelGGL(ln_rows20_kernel<32>, dim3(ceil_div(rows, 8)), block, 0, st, x, rows, g, b, eps, (bf16_t*)out);
        else hipLaunchKernelGGL(ln_rows20_kernel<64>, dim3(ceil_div(rows, 4)), block, 0, st, x, rows, g, b, eps, (bf16_t*)out);
    } else if (in_f32)
        hipLaunchKernelGGL(ln_rows_kernel<float>, grid, block, 0, st, (const float*)in, rows, C, (const bf16_t*)gamma,
                           (const bf16_t*)beta, eps, (bf16_t*)out, tile_idx, tile, tiles_w, H, W, Ma);
    else
        hipLaunchKernelGGL(ln_rows_kernel<bf16_t>, grid, block, 0, st, (const bf16_t*)in, rows, C, (const bf16_t*)gamma,
                           (const bf16_t*)beta, eps, (bf16_t*)out, tile_idx, tile, tiles_w, H, W, Ma);
    FISE_CHECK_LAUNCH("layernorm rows");
    return FISE_OK;
}

// A few rows times a weight matrix: one wave per output column, lanes stride over K in
// 8-element (16-byte) weight loads.  K % 8 == 0.
template <int NB>
__global__ __launch_bounds__(256) void small_linear_kernel(const float* __restrict__ in, int K, const bf16_t* __restrict__ W,
                                                           const bf16_t* __restrict__ bias, int N, int silu_out,
                                                           float* __restrict__ out) {
    const int n = blockIdx.x * 4 + (threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    if (n >= N) return;
    float acc[NB];
#pragma unroll
    for (int b = 0; b < NB; ++b) acc[b] = 0.f;
    for (int k = lane * 8; k < K; k += 64 * 8) {
        const uint4 wv = *reinterpret_cast<const uint4*>(W + (size_t)n * K + k);
        const unsigned w4[4] = {wv.x, wv.y, wv.z, wv.w};
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float wf = (e & 1) ? __uint_as_float(w4[e >> 1] & 0xffff0000u) : __uint_as_float(w4[e >> 1] << 16);
#pragma unroll
            for (int b = 0; b < NB; ++b) acc[b] = fmaf(in[(size_t)b * K + k + e], wf, acc[b]);
        }
    }
#pragma unroll
    for (int b = 0; b < NB; ++b) {
        float v = acc[b];
        for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
        if (lane == 0) {
            if (bias) v += bf2f(bias[n]);
            out[(size_t)b * N + n] = silu_out ? silu_f(v) : v;
        }
    }
}

int launch_small_linear(const float* in, int B, int K, const void* W, const void* bias, int N, int silu_out, float* out,
                        hipStream_t st) {
    if (K % 8) return fail(FISE_ERR_ALIGN, "small linear: K=%d must be a multiple of 8", K);
    const dim3 grid(ceil_div(N, 4)), block(256);
    for (int b0 = 0; b0 < B; b0 += 2) {
        const float* i0 = in + (size_t)b0 * K; float* o0 = out + (size_t)b0 * N;
        if (B - b0 >= 2)
            hipLaunchKernelGGL(small_linear_kernel<2>, grid, block, 0, st, i0, K, (const bf16_t*)W, (const bf16_t*)bias, N, silu_out, o0);
        else
            hipLaunchKernelGGL(small_linear_kernel<1>, grid, block, 0, st, i0, K, (const bf16_t*)W, (const bf16_t*)bias, N, silu_out, o0);
        FISE_CHECK_LAUNCH("small linear");
    }
    return FISE_OK;
}

__global__ void iota_kernel(int* p, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = i;
}
int launch_iota(int* p, int n, hipStream_t st) {
    if (n <= 0) return FISE_OK;
    hipLaunchKernelGGL(iota_kernel, dim3(ceil_div(n, 256)), dim3(256), 0, st, p, n);
    FISE_CHECK_LAUNCH("iota");
    return FISE_OK;
}

}  // namespace fise

using namespace fise;

extern "C" size_t fise_groupnorm_stats_workspace_bytes(int B, int H, int W, int C) {
    (void)C;
    if (B < 1 || H < 1 || W < 1) return 0;
    // the group count is not known here: bound it by the channel count
    return align256((size_t)B * ceil_div(H * W, GS_PIX) * (size_t)(C > 0 ? C : 1) * sizeof(double2));
}

// Both entry points below: argument checks, then the two launches with the partial sums in `partial`.
// gamma / beta / ss (all or none): the finish launch also writes the GroupNorm's (scale, shift) table.
static int gn_stats_run(const char* fn, const void* x, const void* x1, int dtype, int B, int H, int W, int C0, int C1, int G,
                        float eps, float* mean, float* rstd, double2* partial, hipStream_t st, const void* gamma = nullptr,
                        const void* beta = nullptr, float2* ss = nullptr) {
    const int C = C0 + C1;
    const int HW = H * W, nchunk = ceil_div(HW, GS_PIX);
    const size_t shmem = (size_t)C * sizeof(double2);
    constexpr size_t kStripeBytes = 256 * 8 * sizeof(float2);
    if (shmem > 64 * 1024) return fail(FISE_ERR_SHAPE, "%s: C=%d too large", fn, C);
    const bool vec = dtype == FISE_BF16 && C0 % 8 == 0 && C1 % 8 == 0 && shmem + kStripeBytes <= 64 * 1024 && aligned16(x) &&
                     (C1 == 0 || aligned16(x1));
    if (vec) {
        // small maps have few pixel chunks: the groups are dealt to slabs as well (whole groups whose channel range
        // is a multiple of 8 wide), aiming at ~512 workgroups
        const int cpg = C / G;
        const int unit = cpg % 8 == 0 ? 1 : cpg % 4 == 0 ? 2 : cpg % 2 == 0 ? 4 : 8;       // 8 / gcd(cpg, 8) groups
        int gps = G;
        if (G % unit == 0) {
            const int want = std::max(1, 512 / (nchunk * B));
            gps = std::max(unit, ceil_div(ceil_div(G, want), unit) * unit);
        }
        hipLaunchKernelGGL(gn_partial_vec_kernel, dim3(nchunk, B, ceil_div(G, gps)), dim3(256), shmem + kStripeBytes, st, (const bf16_t*)x,
                           (const bf16_t*)x1, HW, C0, C1, G, gps, partial);
    }
    else if (dtype == FISE_F32)
        hipLaunchKernelGGL(gn_partial_kernel<float>, dim3(nchunk, B), dim3(256), shmem, st, (const float*)x, (const float*)x1, HW, C0, C1, G, partial);
    else
        hipLaunchKernelGGL(gn_partial_kernel<bf16_t>, dim3(nchunk, B), dim3(256), shmem, st, (const bf16_t*)x, (const bf16_t*)x1, HW, C0, C1, G, partial);
    FISE_CHECK_LAUNCH("fise_groupnorm_stats(partial)");
    hipLaunchKernelGGL(gn_finish_kernel, dim3(B * G), dim3(64), 0, st, partial, nchunk, B * G, G,
                       (double)HW * (C / G), eps, mean, rstd, (const bf16_t*)gamma, (const bf16_t*)beta, C, ss);
    FISE_CHECK_LAUNCH("fise_groupnorm_stats(finish)");
    return FISE_OK;
}

static int gn_stats_check(const char* fn, const void* x, const void* x1, int dtype, int B, int H, int W, int C0, int C1, int G,
                          const float* mean, const float* rstd) {
    if (!x || !mean || !rstd) return fail(FISE_ERR_NULL, "%s: null pointer", fn);
    if (dtype != FISE_F32 && dtype != FISE_BF16) return fail(FISE_ERR_DTYPE, "%s: dtype %d", fn, dtype);
    if (C1 < 0 || (C1 > 0 && !x1)) return fail(FISE_ERR_NULL, "%s: second source missing", fn);
    if (B < 1 || H < 1 || W < 1 || C0 < 1 || G < 1 || (C0 + C1) % G) return fail(FISE_ERR_SHAPE, "%s: B%d H%d W%d C%d G%d", fn, B, H, W, C0 + C1, G);
    return FISE_OK;
}

// Statistics of a bf16 map (or two concatenated ones) and, in the same two launches, the GroupNorm's scale / shift table.
int fise::launch_gn_stats_table(const void* x0, const void* x1, int B, int H, int W, int C0, int C1, int G, float eps, float* mean, float* rstd,
                          const void* gamma, const void* beta, float2* ss, void* workspace, hipStream_t st) {
    const char* fn = "groupnorm statistics + table";
    if (!workspace || !gamma || !beta || !ss) return fail(FISE_ERR_NULL, "%s: null pointer", fn);
    if (int e = gn_stats_check(fn, x0, x1, FISE_BF16, B, H, W, C0, C1, G, mean, rstd)) return e;
    return gn_stats_run(fn, x0, x1, FISE_BF16, B, H, W, C0, C1, G, eps, mean, rstd, (double2*)workspace, st, gamma, beta, ss);
}

extern "C" int fise_groupnorm_stats(const void* x, const void* x1, int dtype, int B, int H, int W, int C0, int C1, int G,
                                    float eps, float* mean, float* rstd, void* workspace, void* stream) {
    const char* fn = "fise_groupnorm_stats";
    if (!workspace) return fail(FISE_ERR_NULL, "%s: null pointer", fn);
    if (int e = gn_stats_check(fn, x, x1, dtype, B, H, W, C0, C1, G, mean, rstd)) return e;
    return gn_stats_run(fn, x, x1, dtype, B, H, W, C0, C1, G, eps, mean, rstd, (double2*)workspace, as_stream(stream));
}

// ---- the same statistics for callers that can pass no workspace: the per-chunk partial sums live in a fixed array
// in device memory that belongs to the library (one copy per GPU, held until the process ends).
constexpr size_t GN_STATIC_BYTES = 1u << 20;                      // 65536 (batch element, chunk, group) partial sums
static __device__ __align__(256) unsigned char scratch[GN_STATIC_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void* g_scratch_ptr[kMaxDevices];                                 // device address of `scratch` on each GPU (null: not asked yet)

// Device address of this GPU's copy of `scratch`.  In host code the array's name is only a handle: the address a
// kernel can use comes from hipGetSymbolAddress, asked once per device with that device current.
int static_scratch(const char* fn, void** out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return fail(FISE_ERR_HIP, "%s: no current device", fn);
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) return fail(FISE_ERR_HIP, "%s: hipGetSymbolAddress: %s", fn, hipGetErrorString(e));
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return FISE_OK;
}
}  // namespace

extern "C" size_t fise_groupnorm_stats_static_capacity_bytes(void) { return GN_STATIC_BYTES; }

extern "C" int fise_groupnorm_stats_static(const void* x, const void* x1, int dtype, int B, int H, int W, int C0, int C1, int G,
                                           float eps, float* mean, float* rstd, void* stream) {
    const char* fn = "fise_groupnorm_stats_static";
    if (int e = gn_stats_check(fn, x, x1, dtype, B, H, W, C0, C1, G, mean, rstd)) return e;
    const size_t need = (size_t)B * ceil_div(H * W, GS_PIX) * (size_t)G * sizeof(double2);
    if (need > GN_STATIC_BYTES)
        return fail(FISE_ERR_CAPACITY, "%s: B=%d x %d chunks of %d pixels x G=%d partial sums need %zu bytes, the fixed scratch holds %zu",
                    fn, B, ceil_div(H * W, GS_PIX), GS_PIX, G, need, (size_t)GN_STATIC_BYTES);
    void* partial = nullptr;
    if (int e = static_scratch(fn, &partial)) return e;
    // every partial sum the second launch reads is written by the first: nothing has to start at zero
    return gn_stats_run(fn, x, x1, dtype, B, H, W, C0, C1, G, eps, mean, rstd, (double2*)partial, as_stream(stream));
}

extern "C" int fise_masked_groupnorm_silu(const void* x, const float* mean, const float* rstd, const void* gamma,
                                          const void* beta, int dtype, int B, int H, int W, int C, int G,
                                          const int32_t* tile_idx, int n_active, int tile, void* y_cache, void* stream) {
    if (!x || !mean || !rstd || !gamma || !beta || !y_cache) return fail(FISE_ERR_NULL, "fise_masked_groupnorm_silu: null pointer");
    if (dtype != FISE_F32 && dtype != FISE_BF16) return fail(FISE_ERR_DTYPE, "fise_masked_groupnorm_silu: dtype %d", dtype);
    if (B < 1 || H < 1 || W < 1 || C < 1 || G < 1 || C % G || tile < 1 || H % tile || W % tile)
        return fail(FISE_ERR_SHAPE, "fise_masked_groupnorm_silu: B%d H%d W%d C%d G%d tile%d", B, H, W, C, G, tile);
    if (n_active < 0 || n_active > (H / tile) * (W / tile)) return fail(FISE_ERR_CAPACITY, "fise_masked_groupnorm_silu: n_active %d", n_active);
    if (n_active == 0) return FISE_OK;
    if (!tile_idx) return fail(FISE_ERR_NULL, "fise_masked_groupnorm_silu: null tile_idx");
    const int Ma = n_active * tile * tile;
    const long long total = (long long)B * Ma * C;
    const dim3 grid((unsigned)((total + 255) / 256)), block(256);
    if (dtype == FISE_F32)
        hipLaunchKernelGGL(masked_gn_silu_kernel<float>, grid, block, 0, as_stream(stream), (const float*)x, mean, rstd,
                           (const float*)gamma, (const float*)beta, B, H, W, C, G, tile_idx, Ma, tile, (float*)y_cache);
    else
        hipLaunchKernelGGL(masked_gn_silu_kernel<bf16_t>, grid, block, 0, as_stream(stream), (const bf16_t*)x, mean, rstd,
                           (const bf16_t*)gamma, (const bf16_t*)beta, B, H, W, C, G, tile_idx, Ma, tile, (bf16_t*)y_cache);
    FISE_CHECK_LAUNCH("fise_masked_groupnorm_silu");
    return FISE_OK;
}
