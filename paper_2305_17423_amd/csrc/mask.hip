// Mask generation kernels: per-pixel difference + threshold, tile OR-reduce with
// ordered compaction (wave ballot + popcount prefix), 2x2 OR-pool, multi-step
// difference accumulation, Otsu threshold search, block counts for the
// adaptive block-size choice.
#include "common.h"

namespace fise {

// ---------------------------------------------------------------------------
// d = mean_{b,c} |fresh - cached| with a fixed summation order (b outermost, c
// ascending, float adds), one pixel per lane of the first wave.  The workgroup
// stages [64 pixels x CH channels] slabs through LDS so that global reads are
// coalesced along channels while each pixel's channels are still added in
// ascending order by one lane.
// ---------------------------------------------------------------------------
constexpr int DET_PIX = 64;         // pixels per workgroup
constexpr int DET_CH = 64;          // channels staged per slab
constexpr int DET_THREADS = 256;    // all four waves load the slab; the first sums it, one pixel per lane

template <typename T>
__global__ __launch_bounds__(DET_THREADS) void pixel_diff_kernel(const T* __restrict__ cached, const T* __restrict__ fresh,
                                                                 int B, int HW, int C, float* __restrict__ d_out,
                                                                 int accumulate, float threshold, uint8_t* __restrict__ pix) {
    __shared__ float slab[DET_PIX][DET_CH + 1];
    const int p0 = blockIdx.x * DET_PIX;
    const int tid = threadIdx.x;
    float s = 0.f;
    auto absdiff = [&](int b, int pp, int c) {
        const int p = p0 + pp;
        if (p >= HW) return 0.f;
        const size_t off = ((size_t)b * HW + p) * C + c;
        return fabsf(Elem<T>::ld(fresh + off) - Elem<T>::ld(cached + off));
    };
    for (int b = 0; b < B; ++b) {
        for (int c0 = 0; c0 < C; c0 += DET_CH) {
            const int nc = min(DET_CH, C - c0);
            // cooperative load: consecutive lanes walk channels of one pixel, then the next pixel
            if (nc == DET_CH) {                 // full slab: constant trip count, all loads of a lane in flight together
                float v[DET_PIX * DET_CH / DET_THREADS];
#pragma unroll
                for (int j = 0; j < DET_PIX * DET_CH / DET_THREADS; ++j) {
                    const int e = tid + j * DET_THREADS;
                    v[j] = absdiff(b, e / DET_CH, c0 + e % DET_CH);
                }
#pragma unroll
                for (int j = 0; j < DET_PIX * DET_CH / DET_THREADS; ++j) {
                    const int e = tid + j * DET_THREADS;
                    slab[e / DET_CH][e % DET_CH] = v[j];
                }
            } else {
                for (int e = tid; e < DET_PIX * nc; e += DET_THREADS) slab[e / nc][e % nc] = absdiff(b, e / nc, c0 + e % nc);
            }
            __syncthreads();
            if (tid < DET_PIX)
                for (int cc = 0; cc < nc; ++cc) s = s + slab[tid][cc];
            __syncthreads();
        }
    }
    const int p = p0 + tid;
    if (tid < DET_PIX && p < HW) {
        const float d = s / (float)(B * C);
        if (d_out) d_out[p] = accumulate ? d_out[p] + d : d;
        if (pix) pix[p] = d > threshold ? 1 : 0;
    }
}

// ---------------------------------------------------------------------------
// tile OR + ordered compaction, one workgroup; tiles are taken 256 at a time,
// the running base keeps ids ascending across chunks.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void tile_compact_kernel(const uint8_t* __restrict__ pix, int H, int W, int tile_h, int tile_w,
                                                           uint8_t* __restrict__ tile_mask, int* __restrict__ idx,
                                                           int capacity, int* __restrict__ n_active) {
    __shared__ int wave_cnt[4];
    const int tw = W / tile_w, nt = tw * (H / tile_h);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int base = 0;
    for (int c0 = 0; c0 < nt; c0 += 256) {
        const int t = c0 + threadIdx.x;
        bool act = false;
        if (t < nt) {
            const int y0 = (t / tw) * tile_h, x0 = (t % tw) * tile_w;
            for (int yy = 0; yy < tile_h; ++yy)
                for (int xx = 0; xx < tile_w; ++xx) act |= pix[(y0 + yy) * W + x0 + xx] != 0;
            tile_mask[t] = act ? 1 : 0;
        }
        const unsigned long long bal = __ballot(act);
        const int before = __popcll(bal & ((1ull << lane) - 1ull));
        if (lane == 0) wave_cnt[wave] = __popcll(bal);
        __syncthreads();
        int off = base, total = 0;
        for (int w = 0; w < 4; ++w) {
            if (w < wave) off += wave_cnt[w];
            total += wave_cnt[w];
        }
        if (act) {
            const int pos = off + before;
            if (pos < capacity) idx[pos] = t;
        }
        base += total;
        __syncthreads();
    }
    if (threadIdx.x == 0) *n_active = base;
}

__global__ void or_pool_kernel(const uint8_t* __restrict__ m, int H, int W, uint8_t* __restrict__ out) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    const int Ho = H / 2, Wo = W / 2;
    if (i >= Ho * Wo) return;
    const int y = i / Wo, x = i % Wo;
    const uint8_t* r0 = m + (2 * y) * W + 2 * x;
    out[i] = (r0[0] | r0[1] | r0[W] | r0[W + 1]) ? 1 : 0;
}

// ---------------------------------------------------------------------------
// Otsu: one workgroup.  Values are min-max normalised in double; bin k of 257
// holds values with floor(256 v) == k, so class A of threshold k/256 is exactly
// bins [0, k).  Thread k owns bin k and walks all values in index order, which
// keeps every sum deterministic.
// ---------------------------------------------------------------------------
struct OtsuWs { double lo, hi; double cnt[257]; double sum[257]; };

__global__ __launch_bounds__(320) void otsu_kernel(const float* __restrict__ diff, int n, float* __restrict__ eps_out,
                                                   uint8_t* __restrict__ pix, OtsuWs* __restrict__ ws) {
    __shared__ double red_lo[320], red_hi[320];
    __shared__ double s_eps;
    const int t = threadIdx.x;
    double lo = 1e300, hi = -1e300;
    for (int i = t; i < n; i += 320) { const double v = diff[i]; lo = fmin(lo, v); hi = fmax(hi, v); }
    red_lo[t] = lo; red_hi[t] = hi;
    __syncthreads();
    if (t == 0) {
        for (int i = 1; i < 320; ++i) { lo = fmin(lo, red_lo[i]); hi = fmax(hi, red_hi[i]); }
        ws->lo = lo; ws->hi = hi; red_lo[0] = lo; red_hi[0] = hi;
    }
    __syncthreads();
    lo = red_lo[0]; hi = red_hi[0];
    const double range = hi - lo;
    if (t < 257) {
        double c = 0, s = 0;
        for (int i = 0; i < n; ++i) {
            const double v = range > 0 ? ((double)diff[i] - lo) / range : 0.0;
            if ((int)floor(v * 256.0) == t) { c += 1.0; s += v; }
        }
        ws->cnt[t] = c; ws->sum[t] = s;
    }
    __syncthreads();
    if (t == 0) {
        double total_c = 0, total_s = 0;
        for (int k = 0; k < 257; ++k) { total_c += ws->cnt[k]; total_s += ws->sum[k]; }
        double best = -1.0, best_eps = 0.0, ca = 0, sa = 0;
        for (int k = 0; k <= 256; ++k) {           // class A = bins [0, k)
            const double cb = total_c - ca, sb = total_s - sa;
            double obj = 0.0;
            if (ca > 0 && cb > 0) {
                const double dm = sa / ca - sb / cb;
                obj = ca * cb / (total_c * total_c) * dm * dm;
            }
            if (obj > best) { best = obj; best_eps = k / 256.0; }
            ca += ws->cnt[k]; sa += ws->sum[k];
        }
        s_eps = best_eps; *eps_out = (float)best_eps;
    }
    __syncthreads();
    const double eps = s_eps;
    for (int i = t; i < n; i += 320) {
        const double v = range > 0 ? ((double)diff[i] - lo) / range : 0.0;
        pix[i] = v >= eps ? 1 : 0;
    }
}

// one workgroup per candidate block size (h, w) = (2<<i, 2<<j)
__global__ __launch_bounds__(256) void apsc_count_kernel(const uint8_t* __restrict__ pix, int H, int W,
                                                         int* __restrict__ counts) {
    __shared__ int red[256];
    const int h = 2 << (blockIdx.x / 5), w = 2 << (blockIdx.x % 5);
    if (H % h || W % w) { if (threadIdx.x == 0) counts[blockIdx.x] = -1; return; }
    const int bw = W / w, nb = bw * (H / h);
    int c = 0;
    for (int bidx = threadIdx.x; bidx < nb; bidx += 256) {
        const int y0 = (bidx / bw) * h, x0 = (bidx % bw) * w;
        bool any = false;
        for (int yy = 0; yy < h && !any; ++yy)
            for (int xx = 0; xx < w; ++xx) if (pix[(y0 + yy) * W + x0 + xx]) { any = true; break; }
        c += any;
    }
    red[threadIdx.x] = c;
    __syncthreads();
    for (int s = 128; s > 0; s >>= 1) { if (threadIdx.x < s) red[threadIdx.x] += red[threadIdx.x + s]; __syncthreads(); }
    if (threadIdx.x == 0) counts[blockIdx.x] = red[0];
}

static int check_map(const char* fn, const void* a, const void* b, int dtype, int B, int H, int W, int C) {
    if (!a || !b) return fail(FISE_ERR_NULL, "%s: null map pointer", fn);
    if (dtype != FISE_F32 && dtype != FISE_BF16) return fail(FISE_ERR_DTYPE, "%s: dtype %d", fn, dtype);
    if (B < 1 || H < 1 || W < 1 || C < 1) return fail(FISE_ERR_SHAPE, "%s: bad shape B%d H%d W%d C%d", fn, B, H, W, C);
    return FISE_OK;
}
static int check_tile(const char* fn, int H, int W, int tile) {
    if (tile < 1 || H < 1 || W < 1 || H % tile || W % tile)
        return fail(FISE_ERR_SHAPE, "%s: H=%d, W=%d must be positive multiples of tile=%d", fn, H, W, tile);
    return FISE_OK;
}

}  // namespace fise

using namespace fise;

extern "C" int fise_mask_from_pixels(const uint8_t* pix_mask, int H, int W, int tile, uint8_t* tile_mask,
                                     int32_t* tile_idx, int capacity, int32_t* n_active, void* stream) {
    if (!pix_mask || !tile_mask || !tile_idx || !n_active) return fail(FISE_ERR_NULL, "fise_mask_from_pixels: null pointer");
    if (int e = check_tile("fise_mask_from_pixels", H, W, tile)) return e;
    if (capacity < 0) return fail(FISE_ERR_CAPACITY, "fise_mask_from_pixels: capacity %d", capacity);
    hipLaunchKernelGGL(tile_compact_kernel, dim3(1), dim3(256), 0, as_stream(stream), pix_mask, H, W, tile, tile, tile_mask,
                       tile_idx, capacity, n_active);
    FISE_CHECK_LAUNCH("fise_mask_from_pixels");
    return FISE_OK;
}

extern "C" int fise_mask_from_pixels_rect(const uint8_t* pix_mask, int H, int W, int tile_h, int tile_w, uint8_t* tile_mask,
                                          int32_t* tile_idx, int capacity, int32_t* n_active, void* stream) {
    if (!pix_mask || !tile_mask || !tile_idx || !n_active) return fail(FISE_ERR_NULL, "fise_mask_from_pixels_rect: null pointer");
    if (tile_h < 1 || tile_w < 1 || H < 1 || W < 1 || H % tile_h || W % tile_w)
        return fail(FISE_ERR_SHAPE, "fise_mask_from_pixels_rect: H=%d, W=%d must be positive multiples of the %dx%d block", H, W,
                    tile_h, tile_w);
    if (capacity < 0) return fail(FISE_ERR_CAPACITY, "fise_mask_from_pixels_rect: capacity %d", capacity);
    hipLaunchKernelGGL(tile_compact_kernel, dim3(1), dim3(256), 0, as_stream(stream), pix_mask, H, W, tile_h, tile_w, tile_mask,
                       tile_idx, capacity, n_active);
    FISE_CHECK_LAUNCH("fise_mask_from_pixels_rect");
    return FISE_OK;
}

extern "C" int fise_mask_detect(const void* cached, const void* fresh, int dtype, int B, int H, int W, int C,
                                float threshold, int tile, uint8_t* pix_mask, uint8_t* tile_mask, int32_t* tile_idx,
                                int capacity, int32_t* n_active, void* stream) {
    if (int e = check_map("fise_mask_detect", cached, fresh, dtype, B, H, W, C)) return e;
    if (!pix_mask || !tile_mask || !tile_idx || !n_active) return fail(FISE_ERR_NULL, "fise_mask_detect: null output pointer");
    if (int e = check_tile("fise_mask_detect", H, W, tile)) return e;
    if (capacity < 0) return fail(FISE_ERR_CAPACITY, "fise_mask_detect: capacity %d", capacity);
    const int HW = H * W;
    const dim3 grid(ceil_div(HW, DET_PIX)), block(DET_THREADS);
    if (dtype == FISE_F32)
        hipLaunchKernelGGL(pixel_diff_kernel<float>, grid, block, 0, as_stream(stream), (const float*)cached,
                           (const float*)fresh, B, HW, C, (float*)nullptr, 0, threshold, pix_mask);
    else
        hipLaunchKernelGGL(pixel_diff_kernel<bf16_t>, grid, block, 0, as_stream(stream), (const bf16_t*)cached,
                           (const bf16_t*)fresh, B, HW, C, (float*)nullptr, 0, threshold, pix_mask);
    FISE_CHECK_LAUNCH("fise_mask_detect(diff)");
    return fise_mask_from_pixels(pix_mask, H, W, tile, tile_mask, tile_idx, capacity, n_active, stream);
}

extern "C" int fise_diff_accumulate(const void* cached, const void* fresh, int dtype, int B, int H, int W, int C,
                                    float* diff_acc, void* stream) {
    if (int e = check_map("fise_diff_accumulate", cached, fresh, dtype, B, H, W, C)) return e;
    if (!diff_acc) return fail(FISE_ERR_NULL, "fise_diff_accumulate: null diff_acc");
    const int HW = H * W;
    const dim3 grid(ceil_div(HW, DET_PIX)), block(DET_THREADS);
    if (dtype == FISE_F32)
        hipLaunchKernelGGL(pixel_diff_kernel<float>, grid, block, 0, as_stream(stream), (const float*)cached,
                           (const float*)fresh, B, HW, C, diff_acc, 1, 0.f, (uint8_t*)nullptr);
    else
        hipLaunchKernelGGL(pixel_diff_kernel<bf16_t>, grid, block, 0, as_stream(stream), (const bf16_t*)cached,
                           (const bf16_t*)fresh, B, HW, C, diff_acc, 1, 0.f, (uint8_t*)nullptr);
    FISE_CHECK_LAUNCH("fise_diff_accumulate");
    return FISE_OK;
}

extern "C" int fise_mask_downsample(const uint8_t* mask, int H, int W, uint8_t* out, void* stream) {
    if (!mask || !out) return fail(FISE_ERR_NULL, "fise_mask_downsample: null pointer");
    if (H < 2 || W < 2 || (H & 1) || (W & 1)) return fail(FISE_ERR_SHAPE, "fise_mask_downsample: H=%d W=%d must be even", H, W);
    const int n = (H / 2) * (W / 2);
    hipLaunchKernelGGL(or_pool_kernel, dim3(ceil_div(n, 256)), dim3(256), 0, as_stream(stream), mask, H, W, out);
    FISE_CHECK_LAUNCH("fise_mask_downsample");
    return FISE_OK;
}

extern "C" size_t fise_otsu_workspace_bytes(void) { return align256(sizeof(OtsuWs)); }

extern "C" int fise_otsu_mask(const float* diff, int n, float* eps_out, uint8_t* pix_mask, void* workspace, void* stream) {
    if (!diff || !eps_out || !pix_mask || !workspace) return fail(FISE_ERR_NULL, "fise_otsu_mask: null pointer");
    if (n < 1) return fail(FISE_ERR_SHAPE, "fise_otsu_mask: n=%d", n);
    hipLaunchKernelGGL(otsu_kernel, dim3(1), dim3(320), 0, as_stream(stream), diff, n, eps_out, pix_mask, (OtsuWs*)workspace);
    FISE_CHECK_LAUNCH("fise_otsu_mask");
    return FISE_OK;
}

extern "C" int fise_apsc_block_counts(const uint8_t* pix_mask, int H, int W, int32_t* counts, void* stream) {
    if (!pix_mask || !counts) return fail(FISE_ERR_NULL, "fise_apsc_block_counts: null pointer");
    if (H < 1 || W < 1) return fail(FISE_ERR_SHAPE, "fise_apsc_block_counts: H=%d W=%d", H, W);
    hipLaunchKernelGGL(apsc_count_kernel, dim3(25), dim3(256), 0, as_stream(stream), pix_mask, H, W, counts);
    FISE_CHECK_LAUNCH("fise_apsc_block_counts");
    return FISE_OK;
}

extern "C" int fise_apsc_select(const int32_t* counts, int kh, int kw, int* h, int* w, int64_t* cost) {
    if (!counts || !h || !w) return fail(FISE_ERR_NULL, "fise_apsc_select: null pointer");
    if (kh < 1 || kw < 1) return fail(FISE_ERR_SHAPE, "fise_apsc_select: kernel %dx%d", kh, kw);
    int64_t best = -1;
    for (int i = 0; i < 5; ++i)
        for (int j = 0; j < 5; ++j) {
            const int32_t n = counts[i * 5 + j];
            if (n < 0) continue;
            const int bh = 2 << i, bw = 2 << j;
            const int64_t c = (int64_t)(bh + kh - 1) * (bw + kw - 1) * n;
            if (best < 0 || c < best) { best = c; *h = bh; *w = bw; }
        }
    if (best < 0) return fail(FISE_ERR_SHAPE, "fise_apsc_select: no candidate block size divides the map");
    if (cost) *cost = best;
    return FISE_OK;
}
