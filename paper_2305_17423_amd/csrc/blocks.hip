// Stand-alone attention sub-layer and context K/V projection: thin host-side
// sequencing of the gathered GEMM, row LayerNorm and active-query attention kernels.
#include <cmath>
#include "igemm.h"

namespace fise {

// A linear layer on compact rows [rows, Cin] -> sections of `out`.
IgemmArgs linear_args(const void* A, int rows_per_b, int B, int Cin, const void* W, const void* bias, int N) {
    IgemmArgs g{};
    g.a0 = (const bf16_t*)A; g.a1 = nullptr; g.C0 = Cin; g.C1 = 0; g.a_compact = 1;
    g.Hin = 1; g.Win = 1; g.ksize = 1; g.stride = 1; g.ups = 0;
    g.tile_idx = nullptr; g.tile = 1; g.tiles_w = 1; g.Ho = 1; g.Wo = 1; g.B = B; g.Ma = rows_per_b;
    g.pro = PRO_NONE; g.G = 1;
    g.w = (const bf16_t*)W; g.N = N; g.K = Cin; g.geglu = 0;
    g.bias = (const bf16_t*)bias; g.temb = nullptr; g.temb_stride = 0; g.res = nullptr; g.res_compact = 1;
    g.nsect = 1; g.sect_n = N; g.out[0] = nullptr; g.out_mode[0] = OUT_COMPACT;
    g.splits = 1; g.partial = nullptr; g.counters = nullptr;
    return g;
}

}  // namespace fise

using namespace fise;

extern "C" size_t fise_context_kv_workspace_bytes(int B, int n_ctx, int Dc, int C) {
    (void)B; (void)n_ctx; (void)Dc; (void)C;
    return 256;
}

extern "C" int fise_context_kv(const void* ctx, const void* Wk, const void* Wv, int dtype, int B, int n_ctx, int Dc, int C,
                               int n_stride, void* K_ctx, void* Vt_ctx, void* workspace, size_t workspace_bytes, void* stream) {
    (void)workspace; (void)workspace_bytes;
    if (!ctx || !Wk || !Wv || !K_ctx || !Vt_ctx) return fail(FISE_ERR_NULL, "fise_context_kv: null pointer");
    if (dtype != FISE_BF16) return fail(FISE_ERR_DTYPE, "fise_context_kv: bf16 only");
    if (B < 1 || n_ctx < 1 || Dc < 1 || C < 1) return fail(FISE_ERR_SHAPE, "fise_context_kv: bad shape");
    if (Dc % 32 || C % 8) return fail(FISE_ERR_ALIGN, "fise_context_kv: Dc=%d must be a multiple of 32, C=%d of 8", Dc, C);
    if (n_stride < n_ctx || n_stride % 8) return fail(FISE_ERR_ALIGN, "fise_context_kv: n_stride %d", n_stride);
    hipStream_t st = as_stream(stream);
    IgemmArgs g = linear_args(ctx, n_ctx, B, Dc, Wk, nullptr, C);
    g.out[0] = (bf16_t*)K_ctx;
    if (int e = launch_igemm(g, st)) return e;
    g.w = (const bf16_t*)Wv; g.out[0] = (bf16_t*)Vt_ctx; g.out_mode[0] = OUT_TOKENS_T; g.Ho = 1; g.Wo = n_stride;
    return launch_igemm(g, st);
}

extern "C" size_t fise_masked_attention_workspace_bytes(int B, int C, int n_active, int tile) {
    if (B < 1 || C < 1 || n_active < 0 || tile < 1) return 0;
    const size_t rows = (size_t)B * n_active * tile * tile;
    return 3 * align256(rows * C * sizeof(bf16_t)) + 256;
}

extern "C" int fise_masked_attention(const void* x, const void* ln_gamma, const void* ln_beta, const void* Wq, const void* Wk,
                                     const void* Wv, const void* Wo, const void* bo, int dtype, int B, int H, int W, int C,
                                     int heads, void* K_cache, void* Vt_cache, const void* K_ctx, const void* Vt_ctx, int n_ctx,
                                     int n_ctx_stride, const int32_t* tile_idx, int n_active, int tile, void* y_cache,
                                     void* workspace, size_t workspace_bytes, void* stream) {
    const bool self = K_cache != nullptr || Vt_cache != nullptr;
    if (!x || !ln_gamma || !ln_beta || !Wq || !Wo || !y_cache) return fail(FISE_ERR_NULL, "fise_masked_attention: null pointer");
    if (self && (!K_cache || !Vt_cache || !Wk || !Wv)) return fail(FISE_ERR_NULL, "fise_masked_attention: self-attention needs K_cache, Vt_cache, Wk, Wv");
    if (!self && (!K_ctx || !Vt_ctx)) return fail(FISE_ERR_NULL, "fise_masked_attention: cross-attention needs K_ctx, Vt_ctx");
    if (dtype != FISE_BF16) return fail(FISE_ERR_DTYPE, "fise_masked_attention: bf16 only");
    if (B < 1 || H < 1 || W < 1 || C < 1 || heads < 1 || C % heads || tile < 1 || H % tile || W % tile)
        return fail(FISE_ERR_SHAPE, "fise_masked_attention: B%d H%d W%d C%d heads%d tile%d", B, H, W, C, heads, tile);
    const int d = C / heads;
    if (C % 32 || d % 8 || d > 160) return fail(FISE_ERR_ALIGN, "fise_masked_attention: C=%d (multiple of 32), head dim %d (multiple of 8, <= 160)", C, d);
    if (self && (H * W) % 8) return fail(FISE_ERR_ALIGN, "fise_masked_attention: H*W must be a multiple of 8");
    if (!self && (n_ctx < 1 || n_ctx_stride < n_ctx || n_ctx_stride % 8)) return fail(FISE_ERR_ALIGN, "fise_masked_attention: n_ctx %d stride %d", n_ctx, n_ctx_stride);
    if (n_active < 0 || n_active > (H / tile) * (W / tile)) return fail(FISE_ERR_CAPACITY, "fise_masked_attention: n_active %d", n_active);
    if (n_active == 0) return FISE_OK;
    if (!tile_idx) return fail(FISE_ERR_NULL, "fise_masked_attention: null tile_idx");
    if (!workspace || workspace_bytes < fise_masked_attention_workspace_bytes(B, C, n_active, tile))
        return fail(FISE_ERR_CAPACITY, "fise_masked_attention: workspace too small");
    if (y_cache == x) return fail(FISE_ERR_SHAPE, "fise_masked_attention: y_cache aliases x");

    hipStream_t st = as_stream(stream);
    const int Ma = n_active * tile * tile, rows = B * Ma;
    const size_t buf = align256((size_t)rows * C * sizeof(bf16_t));
    char* ws = (char*)workspace;
    bf16_t* nbuf = (bf16_t*)ws; bf16_t* qbuf = (bf16_t*)(ws + buf); bf16_t* obuf = (bf16_t*)(ws + 2 * buf);
    const float scale = 1.0f / sqrtf((float)d);

    if (int e = launch_ln_rows(x, rows, C, ln_gamma, ln_beta, 1e-5f, nbuf, tile_idx, tile, W / tile, H, W, Ma, st)) return e;
    IgemmArgs g = linear_args(nbuf, Ma, B, C, Wq, nullptr, C);
    g.tile_idx = tile_idx; g.tile = tile; g.tiles_w = W / tile; g.Ho = H; g.Wo = W;
    g.out[0] = qbuf;
    if (int e = launch_igemm(g, st)) return e;
    if (self) {
        g.w = (const bf16_t*)Wk; g.out[0] = (bf16_t*)K_cache; g.out_mode[0] = OUT_MAP;
        if (int e = launch_igemm(g, st)) return e;
        g.w = (const bf16_t*)Wv; g.out[0] = (bf16_t*)Vt_cache; g.out_mode[0] = OUT_TOKENS_T;
        if (int e = launch_igemm(g, st)) return e;
        if (int e = launch_attention(qbuf, K_cache, Vt_cache, B, Ma, H * W, H * W, C, heads, scale, obuf, st)) return e;
    } else {
        if (int e = launch_attention(qbuf, K_ctx, Vt_ctx, B, Ma, n_ctx, n_ctx_stride, C, heads, scale, obuf, st)) return e;
    }
    IgemmArgs o = linear_args(obuf, Ma, B, C, Wo, bo, C);
    o.tile_idx = tile_idx; o.tile = tile; o.tiles_w = W / tile; o.Ho = H; o.Wo = W;
    o.res = (const bf16_t*)x; o.res_compact = 0;
    o.out[0] = (bf16_t*)y_cache; o.out_mode[0] = OUT_MAP;
    return launch_igemm(o, st);
}
