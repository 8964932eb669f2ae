// Public masked-convolution entry points.  bf16 maps whose channel counts are
// multiples of 32 go to the MFMA implicit GEMM; float maps and odd channel counts
// (e.g. the 4-channel latent) use the scalar kernel below, one output element per
// thread, same gather rules.
#include "igemm.h"

namespace fise {

template <typename T>
__global__ __launch_bounds__(256) void conv_scalar_kernel(const T* __restrict__ x0, const T* __restrict__ x1, int C0, int C1,
                                                          int B, int Hin, int Win, const T* __restrict__ w,
                                                          const T* __restrict__ bias, int Cout, int ksize, int stride, int ups,
                                                          const float* __restrict__ gn_mean, const float* __restrict__ gn_rstd,
                                                          const T* __restrict__ gn_gamma, const T* __restrict__ gn_beta, int G,
                                                          int gn_silu, const float* __restrict__ temb, const T* residual,
                                                          const int* __restrict__ tile_idx, int Ma, int tile, int tile_w, int Ho,
                                                          int Wo, T* y, int nview, GnView view0, GnView view1) {
    const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    const long long total = (long long)B * Ma * Cout;
    if (i >= total) return;
    const int co = (int)(i % Cout);
    const int m = (int)((i / Cout) % Ma);
    const int b = (int)(i / ((long long)Cout * Ma));
    int oy, ox;
    active_pixel(tile_idx, m, tile, tile_w, Wo / tile_w, oy, ox);
    const int Cin = C0 + C1, pad = ksize >> 1;
    const int cpg = gn_mean ? Cin / G : 1;
    float acc = 0.f;
    for (int ky = 0; ky < ksize; ++ky)
        for (int kx = 0; kx < ksize; ++kx) {
            int iy, ix; bool in;
            if (ups) {
                const int uy = oy + ky - pad, ux = ox + kx - pad;
                in = uy >= 0 && uy < 2 * Hin && ux >= 0 && ux < 2 * Win; iy = uy >> 1; ix = ux >> 1;
            } else {
                iy = oy * stride + ky - pad; ix = ox * stride + kx - pad;
                in = iy >= 0 && iy < Hin && ix >= 0 && ix < Win;
            }
            if (!in) continue;
            const size_t p = ((size_t)b * Hin + iy) * Win + ix;
            const T* wr = w + ((size_t)co * ksize * ksize + ky * ksize + kx) * Cin;
            for (int c = 0; c < Cin; ++c) {
                float v = c < C0 ? Elem<T>::ld(x0 + p * C0 + c) : Elem<T>::ld(x1 + p * C1 + (c - C0));
                if (gn_mean) {
                    const int g = c / cpg;
                    v = (v - gn_mean[b * G + g]) * gn_rstd[b * G + g] * Elem<T>::ld(gn_gamma + c) + Elem<T>::ld(gn_beta + c);
                    if (gn_silu) v = silu_f(v);
                }
                acc = fmaf(v, Elem<T>::ld(wr + c), acc);
            }
        }
    if (bias) acc += Elem<T>::ld(bias + co);
    if (temb) acc += temb[b * Cout + co];
    const size_t o = (((size_t)b * Ho + oy) * Wo + ox) * Cout + co;
    if (residual) acc += Elem<T>::ld(residual + o);
    Elem<T>::st(y + o, acc);
    if (nview) {                      // bf16 maps only (checked by the launcher)
        const GnView views[2] = {view0, view1};
        put_views1(views, nview, b, ((size_t)b * Ho + oy) * Wo + ox, co, acc);
    }
}

// The 4-channel latent under a 3x3 kernel (the UNet's input convolution): the 36 input
// values of one pixel are loaded once and shared by four output channels, whose 36 weights
// each are contiguous.  Same accumulation order as the scalar kernel above.
__global__ __launch_bounds__(256) void conv_latent3x3_kernel(const bf16_t* __restrict__ x, int B, int H, int W,
                                                             const bf16_t* __restrict__ w, const bf16_t* __restrict__ bias,
                                                             int Cout, const float* __restrict__ temb, const bf16_t* residual,
                                                             const int* __restrict__ tile_idx, int Ma, int tile, int tile_w, bf16_t* y,
                                                             int nview, GnView view0, GnView view1) {
    const int q4 = Cout >> 2;
    const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= (long long)B * Ma * q4) return;
    const int co = (int)(i % q4) * 4;
    const int m = (int)((i / q4) % Ma);
    const int b = (int)(i / ((long long)q4 * Ma));
    int oy, ox;
    active_pixel(tile_idx, m, tile, tile_w, W / tile_w, oy, ox);
    float xin[36];
#pragma unroll
    for (int t = 0; t < 9; ++t) {
        const int iy = oy + t / 3 - 1, ix = ox + t % 3 - 1;
        uint2 v = make_uint2(0u, 0u);
        if (iy >= 0 && iy < H && ix >= 0 && ix < W) v = *(const uint2*)(x + (((size_t)b * H + iy) * W + ix) * 4);
        xin[t * 4 + 0] = __uint_as_float(v.x << 16); xin[t * 4 + 1] = __uint_as_float(v.x & 0xffff0000u);
        xin[t * 4 + 2] = __uint_as_float(v.y << 16); xin[t * 4 + 3] = __uint_as_float(v.y & 0xffff0000u);
    }
    const size_t o = (((size_t)b * H + oy) * W + ox) * Cout + co;
    float acc[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const uint2* wr = (const uint2*)(w + (size_t)(co + j) * 36);   // 72 B per channel: 8-byte aligned
        float a = 0.f;
#pragma unroll
        for (int t = 0; t < 9; ++t) {
            const uint2 v = wr[t];
            a = fmaf(xin[t * 4 + 0], __uint_as_float(v.x << 16), a);
            a = fmaf(xin[t * 4 + 1], __uint_as_float(v.x & 0xffff0000u), a);
            a = fmaf(xin[t * 4 + 2], __uint_as_float(v.y << 16), a);
            a = fmaf(xin[t * 4 + 3], __uint_as_float(v.y & 0xffff0000u), a);
        }
        if (bias) a += Elem<bf16_t>::ld(bias + co + j);
        if (temb) a += temb[b * Cout + co + j];
        if (residual) a += Elem<bf16_t>::ld(residual + o + j);
        acc[j] = a;
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) Elem<bf16_t>::st(y + o + j, acc[j]);
    if (nview) {
        const GnView views[2] = {view0, view1};
        put_views4(views, nview, b, (unsigned)(((size_t)b * H + oy) * W + ox), co, acc);
    }
}

// fp32 convolution for channel counts that are multiples of 16 (one source, no GroupNorm prologue) on the fp32 matrix
// instruction (v_mfma_f32_32x32x2f32: full float products and sums).  A workgroup owns a 32-row x 64-column output
// tile; operands are staged through LDS in BK-wide K chunks with 16-byte loads (the next chunk is fetched into
// registers while the current one is multiplied); each of the four waves multiplies its quarter of every chunk into
// its own pair of 32x32 accumulators, and the four partial tiles are summed through LDS in wave order at the end.
typedef float f32x16v __attribute__((ext_vector_type(16)));
template <int BK>
__global__ __launch_bounds__(256) void conv_f32_tile_kernel(const float* __restrict__ x, int Cin, int B, int Hin, int Win,
                                                            const float* __restrict__ w, const float* __restrict__ bias, int Cout,
                                                            int ksize, int stride, int ups, const float* __restrict__ temb,
                                                            const float* residual, const int* __restrict__ tile_idx, int Ma, int tile,
                                                            int tile_w, int Ho, int Wo, float* y) {
    constexpr int BM = 32, BN = 64;
    constexpr int KQ = BK / 4;                           // float4 pieces per row of a chunk
    constexpr int BL = BN * KQ / 256;                    // weight pieces per thread
    constexpr int A_THREADS = BM * KQ < 256 ? BM * KQ : 256;
    __shared__ float As[BK][BM + 1];
    __shared__ __attribute__((aligned(16))) float Bs[BK][BN];
    __shared__ int rb[BM], ry[BM], rx[BM];
    const int t = threadIdx.x, rows = B * Ma;
    const int m0 = blockIdx.x * BM, n0 = blockIdx.y * BN;
    if (t < BM) {
        const int gm = m0 + t;
        int b = -1, oy = 0, ox = 0;
        if (gm < rows) { b = gm / Ma; active_pixel(tile_idx, gm % Ma, tile, tile_w, Wo / tile_w, oy, ox); }
        rb[t] = b; ry[t] = oy; rx[t] = ox;
    }
    __syncthreads();
    const int lane = t & 63, wave = t >> 6, l32 = lane & 31, hl = lane >> 5;
    const int pad = ksize >> 1;
    f32x16v acc0 = {}, acc1 = {};                        // this wave's partial sums: columns 0..31 and 32..63 of the tile
    const int la_row = (t / KQ) % BM, la_k = (t % KQ) * 4;        // A piece of this thread (threads below A_THREADS)
    const int lb_col = t / KQ, lb_k = (t % KQ) * 4;              // B pieces: columns lb_col + j * (256 / KQ)
    const int chunks = Cin / BK, total = ksize * ksize * chunks;
    float4 ra[2], rbv[2][BL];                            // two chunks in flight
    auto fetch = [&](int it, float4& a4, float4 (&b4)[BL]) {      // chunk `it` = (tap, channel offset) -> registers
        const int tap = it / chunks, c0 = (it - tap * chunks) * BK;
        const int ky = tap / ksize, kx = tap - ky * ksize;
        a4 = make_float4(0.f, 0.f, 0.f, 0.f);
        if (t < A_THREADS && rb[la_row] >= 0) {
            const int oy = ry[la_row], ox = rx[la_row], b = rb[la_row];
            long long apix = -1;
            if (ups) {
                const int uy = oy + ky - pad, ux = ox + kx - pad;
                if (uy >= 0 && uy < 2 * Hin && ux >= 0 && ux < 2 * Win) apix = ((long long)b * Hin + (uy >> 1)) * Win + (ux >> 1);
            } else {
                const int iy = oy * stride + ky - pad, ix = ox * stride + kx - pad;
                if (iy >= 0 && iy < Hin && ix >= 0 && ix < Win) apix = ((long long)b * Hin + iy) * Win + ix;
            }
            if (apix >= 0) a4 = *reinterpret_cast<const float4*>(x + apix * Cin + c0 + la_k);
        }
#pragma unroll
        for (int j = 0; j < BL; ++j) {
            const int wcol = n0 + lb_col + j * (256 / KQ);
            b4[j] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (wcol < Cout) b4[j] = *reinterpret_cast<const float4*>(w + ((size_t)wcol * ksize * ksize + tap) * Cin + c0 + lb_k);
        }
    };
    // one chunk: registers of slot S -> LDS, refill the slot with the chunk two ahead, multiply
    auto chunk = [&](int it, float4& a4, float4 (&b4)[BL]) {
        if (t < A_THREADS) { As[la_k + 0][la_row] = a4.x; As[la_k + 1][la_row] = a4.y; As[la_k + 2][la_row] = a4.z; As[la_k + 3][la_row] = a4.w; }
#pragma unroll
        for (int j = 0; j < BL; ++j) {
            const int col = lb_col + j * (256 / KQ);
            Bs[lb_k + 0][col] = b4[j].x; Bs[lb_k + 1][col] = b4[j].y; Bs[lb_k + 2][col] = b4[j].z; Bs[lb_k + 3][col] = b4[j].w;
        }
        __syncthreads();
        if (it + 2 < total) fetch(it + 2, a4, b4);       // in flight during this chunk's and the next chunk's products
        // wave w: K offsets [w * BK / 4, (w + 1) * BK / 4) of the chunk, two at a time (lane half hl takes the second)
#pragma unroll
        for (int kk = 0; kk < BK / 4; kk += 2) {
            const int k = wave * (BK / 4) + kk + hl;
            const float av = As[k][l32];
            acc0 = __builtin_amdgcn_mfma_f32_32x32x2f32(av, Bs[k][l32], acc0, 0, 0, 0);
            acc1 = __builtin_amdgcn_mfma_f32_32x32x2f32(av, Bs[k][32 + l32], acc1, 0, 0, 0);
        }
        __syncthreads();
    };
    fetch(0, ra[0], rbv[0]);
    if (total > 1) fetch(1, ra[1], rbv[1]);
    for (int it = 0; it < total; it += 2) {
        chunk(it, ra[0], rbv[0]);
        if (it + 1 < total) chunk(it + 1, ra[1], rbv[1]);
    }
    // ---- the four partial tiles through LDS, summed in wave order; then four consecutive columns of one row per thread
    __shared__ __attribute__((aligned(16))) float part[4][BM][BN + 4];
#pragma unroll
    for (int e = 0; e < 16; ++e) {
        const int r = (e >> 2) * 8 + hl * 4 + (e & 3);
        part[wave][r][l32] = acc0[e]; part[wave][r][32 + l32] = acc1[e];
    }
    __syncthreads();
    const int tr = t >> 4, tc = t & 15;                  // this thread: rows 2 tr, 2 tr + 1; columns 4 tc .. 4 tc + 3
    float acc[2][4];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            float v = 0.f;
#pragma unroll
            for (int w4 = 0; w4 < 4; ++w4) v += part[w4][tr * 2 + i][tc * 4 + q];
            acc[i][q] = v;
        }
    const int col = n0 + tc * 4;
    if (col >= Cout) return;                             // Cout % 4 == 0: a group of four is inside or outside as a whole
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int r = tr * 2 + i;
        if (rb[r] < 0) continue;
        const size_t o = (((size_t)rb[r] * Ho + ry[r]) * Wo + rx[r]) * Cout + col;
        float v[4] = {acc[i][0], acc[i][1], acc[i][2], acc[i][3]};
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            if (bias) v[q] += bias[col + q];
            if (temb) v[q] += temb[rb[r] * Cout + col + q];
            if (residual) v[q] += residual[o + q];
        }
        *reinterpret_cast<float4*>(y + o) = make_float4(v[0], v[1], v[2], v[3]);
    }
}

static int tile_cols(const fise_conv_args* a) { return a->tile_w > 0 ? a->tile_w : a->tile; }

static int validate(const fise_conv_args* a, int& Ho, int& Wo) {
    if (!a) return fail(FISE_ERR_NULL, "fise_masked_conv: null args");
    if (!a->x0 || !a->w || !a->y_cache) return fail(FISE_ERR_NULL, "fise_masked_conv: null x / w / y_cache");
    if (a->dtype != FISE_F32 && a->dtype != FISE_BF16) return fail(FISE_ERR_DTYPE, "fise_masked_conv: dtype %d", a->dtype);
    if (a->C1 < 0 || (a->C1 > 0 && !a->x1)) return fail(FISE_ERR_NULL, "fise_masked_conv: second source missing");
    if (a->B < 1 || a->H < 1 || a->W < 1 || a->C0 < 1 || a->Cout < 1) return fail(FISE_ERR_SHAPE, "fise_masked_conv: bad shape");
    if (a->ksize != 1 && a->ksize != 3) return fail(FISE_ERR_SHAPE, "fise_masked_conv: ksize %d (1 or 3)", a->ksize);
    if (a->stride != 1 && a->stride != 2) return fail(FISE_ERR_SHAPE, "fise_masked_conv: stride %d (1 or 2)", a->stride);
    if (a->upsample && a->stride != 1) return fail(FISE_ERR_SHAPE, "fise_masked_conv: upsample needs stride 1");
    if (a->stride == 2 && ((a->H & 1) || (a->W & 1))) return fail(FISE_ERR_SHAPE, "fise_masked_conv: stride 2 needs even H, W");
    Ho = a->upsample ? 2 * a->H : a->H / a->stride;
    Wo = a->upsample ? 2 * a->W : a->W / a->stride;
    if (a->tile < 1 || a->tile_w < 0) return fail(FISE_ERR_SHAPE, "fise_masked_conv: tile %d, tile_w %d", a->tile, a->tile_w);
    const int tw = tile_cols(a);
    if (Ho % a->tile || Wo % tw)
        return fail(FISE_ERR_SHAPE, "fise_masked_conv: output %dx%d not divisible by the %dx%d tile", Ho, Wo, a->tile, tw);
    if (a->n_active < 0 || a->n_active > (Ho / a->tile) * (Wo / tw))
        return fail(FISE_ERR_CAPACITY, "fise_masked_conv: n_active %d beyond the %dx%d tile grid", a->n_active, Ho / a->tile, Wo / tw);
    if (a->n_active > 0 && !a->tile_idx) return fail(FISE_ERR_NULL, "fise_masked_conv: null tile_idx");
    if (a->gn_mean) {
        if (!a->gn_rstd || !a->gn_gamma || !a->gn_beta) return fail(FISE_ERR_NULL, "fise_masked_conv: incomplete GroupNorm arguments");
        if (a->G < 1 || (a->C0 + a->C1) % a->G) return fail(FISE_ERR_SHAPE, "fise_masked_conv: C=%d %% G=%d", a->C0 + a->C1, a->G);
    }
    if (a->y_cache == a->x0 || (a->x1 && a->y_cache == a->x1)) return fail(FISE_ERR_SHAPE, "fise_masked_conv: y_cache aliases an input map");
    const void* ptrs[] = {a->x0, a->x1, a->w, a->bias, a->residual, a->y_cache, a->gn_gamma, a->gn_beta};
    for (const void* p : ptrs)
        if (p && !aligned16(p)) return fail(FISE_ERR_ALIGN, "fise_masked_conv: pointer %p not 16-byte aligned", p);
    return FISE_OK;
}

static bool mfma_path(const fise_conv_args* a) {
    return a->dtype == FISE_BF16 && a->C0 % 32 == 0 && a->C1 % 32 == 0;
}

template <typename T>
static void launch_scalar(const fise_conv_args* a, int Ho, int Wo, hipStream_t st, const GnView* views, int nview) {
    const int Ma = a->n_active * a->tile * tile_cols(a);
    const long long total = (long long)a->B * Ma * a->Cout;
    hipLaunchKernelGGL(conv_scalar_kernel<T>, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, (const T*)a->x0,
                       (const T*)a->x1, a->C0, a->C1, a->B, a->H, a->W, (const T*)a->w, (const T*)a->bias, a->Cout, a->ksize,
                       a->stride, a->upsample ? 1 : 0, a->gn_mean, a->gn_rstd, (const T*)a->gn_gamma, (const T*)a->gn_beta,
                       a->G, a->gn_silu, a->temb, (const T*)a->residual, a->tile_idx, Ma, a->tile, tile_cols(a), Ho, Wo, (T*)a->y_cache,
                       nview, nview > 0 ? views[0] : GnView{}, nview > 1 ? views[1] : GnView{});
}

int conv_dispatch(const fise_conv_args* a, void* workspace, size_t workspace_bytes, hipStream_t st, const GnView* views, int nview) {
    int Ho, Wo;
    if (int e = validate(a, Ho, Wo)) return e;
    if (a->n_active == 0) return FISE_OK;
    if (!mfma_path(a)) {
        if (a->dtype == FISE_BF16 && a->C0 == 4 && a->C1 == 0 && a->ksize == 3 && a->stride == 1 && !a->upsample &&
            !a->gn_mean && a->Cout % 4 == 0) {
            const int Ma = a->n_active * a->tile * tile_cols(a);
            const long long total = (long long)a->B * Ma * (a->Cout / 4);
            hipLaunchKernelGGL(conv_latent3x3_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st,
                               (const bf16_t*)a->x0, a->B, a->H, a->W, (const bf16_t*)a->w, (const bf16_t*)a->bias, a->Cout,
                               a->temb, (const bf16_t*)a->residual, a->tile_idx, Ma, a->tile, tile_cols(a), (bf16_t*)a->y_cache,
                               nview, nview > 0 ? views[0] : GnView{}, nview > 1 ? views[1] : GnView{});
            FISE_CHECK_LAUNCH("fise_masked_conv(latent 3x3)");
            return FISE_OK;
        }
        if (nview && a->dtype != FISE_BF16) return fail(FISE_ERR_DTYPE, "fise_masked_conv: normalised copies need bf16 maps");
        if (a->dtype == FISE_F32 && a->C1 == 0 && !a->gn_mean && a->C0 % 16 == 0 && a->Cout % 4 == 0) {
            const int Ma = a->n_active * a->tile * tile_cols(a), rows = a->B * Ma;
            const dim3 grid(ceil_div(rows, 32), ceil_div(a->Cout, 64));
#define FISE_F32_CONV(BKV) hipLaunchKernelGGL(conv_f32_tile_kernel<BKV>, grid, dim3(256), 0, st, (const float*)a->x0, a->C0, a->B, a->H, a->W, \
                               (const float*)a->w, (const float*)a->bias, a->Cout, a->ksize, a->stride, a->upsample ? 1 : 0, a->temb,            \
                               (const float*)a->residual, a->tile_idx, Ma, a->tile, tile_cols(a), Ho, Wo, (float*)a->y_cache)
            if (a->C0 % 32 == 0) FISE_F32_CONV(32); else FISE_F32_CONV(16);
#undef FISE_F32_CONV
            FISE_CHECK_LAUNCH("fise_masked_conv(fp32 tile)");
            return FISE_OK;
        }
        if (a->dtype == FISE_F32) launch_scalar<float>(a, Ho, Wo, st, nullptr, 0);
        else launch_scalar<bf16_t>(a, Ho, Wo, st, views, nview);
        FISE_CHECK_LAUNCH("fise_masked_conv(scalar)");
        return FISE_OK;
    }
    IgemmArgs g{};
    g.a0 = (const bf16_t*)a->x0; g.a1 = (const bf16_t*)a->x1; g.C0 = a->C0; g.C1 = a->C1; g.a_compact = 0;
    g.Hin = a->H; g.Win = a->W; g.ksize = a->ksize; g.stride = a->stride; g.ups = a->upsample ? 1 : 0;
    g.tile_idx = a->tile_idx; g.tile = a->tile; g.tile_w = tile_cols(a); g.tiles_w = Wo / g.tile_w; g.Ho = Ho; g.Wo = Wo; g.B = a->B;
    g.Ma = a->n_active * a->tile * g.tile_w;
    g.pro = a->gn_mean ? (a->gn_silu ? PRO_GN_SILU : PRO_GN) : PRO_NONE;
    g.gn_mean = a->gn_mean; g.gn_rstd = a->gn_rstd; g.gn_gamma = (const bf16_t*)a->gn_gamma; g.gn_beta = (const bf16_t*)a->gn_beta; g.G = a->G;
    g.w = (const bf16_t*)a->w; g.N = a->Cout; g.K = a->ksize * a->ksize * (a->C0 + a->C1); g.geglu = 0;
    g.bias = (const bf16_t*)a->bias; g.temb = a->temb; g.temb_stride = a->Cout; g.res = (const bf16_t*)a->residual; g.res_compact = 0;
    g.nsect = 1; g.sect_n = a->Cout; g.out[0] = (bf16_t*)a->y_cache; g.out_mode[0] = OUT_MAP;
    g.splits = 1; g.partial = nullptr;
    g.nview = nview;
    for (int i = 0; i < nview; ++i) g.view[i] = views[i];
    IgemmWorkspace iw;
    if (int e = igemm_workspace_init(workspace, workspace_bytes, &iw, st)) return e;
    return launch_igemm(g, &iw, st);
}

}  // namespace fise

using namespace fise;

extern "C" size_t fise_masked_conv_workspace_bytes(const fise_conv_args* a) {
    (void)a;
    return igemm_workspace_bytes();          // split-K scratch; a smaller (or null) workspace runs unsplit
}

extern "C" int fise_masked_conv(const fise_conv_args* a, void* workspace, size_t workspace_bytes, void* stream) {
    return conv_dispatch(a, workspace, workspace_bytes, as_stream(stream), nullptr, 0);
}

extern "C" int fise_masked_conv3x3(const void* x, const void* w, const void* bias, int dtype, int B, int H, int W, int Cin,
                                   int Cout, int stride, const int32_t* tile_idx, int n_active, int tile,
                                   const float* gn_mean, const float* gn_rstd, const void* gn_gamma, const void* gn_beta,
                                   int G, const float* temb, const void* residual, void* y_cache, void* workspace,
                                   size_t workspace_bytes, void* stream) {
    fise_conv_args a{};
    a.x0 = x; a.x1 = nullptr; a.C0 = Cin; a.C1 = 0; a.B = B; a.H = H; a.W = W; a.w = w; a.bias = bias; a.Cout = Cout;
    a.ksize = 3; a.stride = stride; a.upsample = 0;
    a.gn_mean = gn_mean; a.gn_rstd = gn_rstd; a.gn_gamma = gn_gamma; a.gn_beta = gn_beta; a.G = G; a.gn_silu = 1;
    a.temb = temb; a.residual = residual; a.tile_idx = tile_idx; a.n_active = n_active; a.tile = tile; a.y_cache = y_cache;
    a.dtype = dtype;
    return conv_dispatch(&a, workspace, workspace_bytes, as_stream(stream), nullptr, 0);
}
