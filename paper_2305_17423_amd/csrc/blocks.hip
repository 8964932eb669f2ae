// Masked ResNet block, masked transformer block, the stand-alone attention
// sub-layer and the context K/V projection: host-side sequencing of the gathered
// GEMM, row LayerNorm and active-query attention kernels on the caller's stream.
#include <cmath>
#include "igemm.h"

namespace fise {

// A linear layer on compact rows [rows, Cin] (bf16) -> compact bf16 out; fields are adjusted by the caller.
IgemmArgs linear_args(const void* A, int rows_per_b, int B, int Cin, const void* W, const void* bias, int N) {
    IgemmArgs g{};
    g.a0 = (const bf16_t*)A; g.a1 = nullptr; g.C0 = Cin; g.C1 = 0; g.a_compact = 1;
    g.Hin = 1; g.Win = 1; g.ksize = 1; g.stride = 1; g.ups = 0;
    g.tile_idx = nullptr; g.tile = 1; g.tiles_w = 1; g.Ho = 1; g.Wo = 1; g.B = B; g.Ma = rows_per_b;
    g.pro = PRO_NONE; g.G = 1;
    g.w = (const bf16_t*)W; g.N = N; g.K = Cin; g.geglu = 0;
    g.bias = (const bf16_t*)bias; g.temb = nullptr; g.temb_stride = 0; g.res = nullptr; g.res_compact = 1;
    g.nsect = 1; g.sect_n = N; g.out[0] = nullptr; g.out_mode[0] = OUT_COMPACT;
    g.splits = 1; g.partial = nullptr;
    return g;
}

// A convolution-shaped launch: maps in, map out.
static IgemmArgs conv_args(const void* a0, const void* a1, int C0, int C1, int B, int Hin, int Win, int Ho, int Wo, int ks,
                           int stride, int ups, const void* w, const void* bias, int N, const int* idx, int n_active, int tile,
                           void* out) {
    IgemmArgs g{};
    g.a0 = (const bf16_t*)a0; g.a1 = (const bf16_t*)a1; g.C0 = C0; g.C1 = C1; g.a_compact = 0;
    g.Hin = Hin; g.Win = Win; g.ksize = ks; g.stride = stride; g.ups = ups;
    g.tile_idx = idx; g.tile = tile; g.tiles_w = Wo / tile; g.Ho = Ho; g.Wo = Wo; g.B = B; g.Ma = n_active * tile * tile;
    g.pro = PRO_NONE; g.G = 1;
    g.w = (const bf16_t*)w; g.N = N; g.K = ks * ks * (C0 + C1); g.geglu = 0;
    g.bias = (const bf16_t*)bias; g.temb = nullptr; g.temb_stride = 0; g.res = nullptr; g.res_compact = 0;
    g.nsect = 1; g.sect_n = N; g.out[0] = (bf16_t*)out; g.out_mode[0] = OUT_MAP;
    g.splits = 1; g.partial = nullptr;
    return g;
}

static void set_views(IgemmArgs& g, const GnView* views, int nview) {
    g.nview = nview;
    for (int i = 0; i < nview; ++i) g.view[i] = views[i];
}

int run_conv(const void* a0, int C0, int B, int Hin, int Win, int stride, int ups, const void* w, const void* bias, int N,
             const int* idx, int n_active, int tile, void* out, const IgemmWorkspace* iw, hipStream_t st, const GnView* views,
             int nview) {
    const int Ho = ups ? 2 * Hin : Hin / stride, Wo = ups ? 2 * Win : Win / stride;
    IgemmArgs g = conv_args(a0, nullptr, C0, 0, B, Hin, Win, Ho, Wo, 3, stride, ups, w, bias, N, idx, n_active, tile, out);
    set_views(g, views, nview);
    return launch_igemm(g, iw, st);
}

static void set_gn(IgemmArgs& g, const float* mean, const float* rstd, const void* gamma, const void* beta, int G, bool silu) {
    g.pro = silu ? PRO_GN_SILU : PRO_GN;
    g.gn_mean = mean; g.gn_rstd = rstd; g.gn_gamma = (const bf16_t*)gamma; g.gn_beta = (const bf16_t*)beta; g.G = G;
}

// ResNet scratch: [GroupNorm statistics partials | activation map of conv1's input | of conv2's input]
static size_t resnet_gn_bytes(const fise_resnet_args* a) { return align256(fise_groupnorm_stats_workspace_bytes(a->B, a->H, a->W, a->G)); }
static size_t resnet_act_bytes(const fise_resnet_args* a, int C) { return align256((size_t)a->B * a->H * a->W * C * sizeof(bf16_t)); }
size_t resnet_ws_bytes(const fise_resnet_args* a) {
    return resnet_gn_bytes(a) + resnet_act_bytes(a, a->C0 + a->C1) + resnet_act_bytes(a, a->Cout);
}

// dv (may be null): where the block's activated inputs live between calls and who else wants the block's output
// normalised.  Without it the activations go to the workspace and are recomputed by every call.
int run_resnet(const fise_resnet_args* a, void* ws, const IgemmWorkspace* iw, hipStream_t st, const BlockDerived* dv) {
    const int Ci = a->C0 + a->C1, Co = a->Cout, B = a->B, H = a->H, W = a->W;
    char* act1 = dv ? (char*)dv->act_in : (char*)ws + resnet_gn_bytes(a);
    char* act2 = dv ? (char*)dv->act_mid : (char*)ws + resnet_gn_bytes(a) + resnet_act_bytes(a, Ci);
    // With cached statistics and a trusted cache, the producers of x0 / x1 have already written this block's
    // activated input at the active pixels (the ring outside them is unchanged), and conv1 writes conv2's.
    const bool have_acts = dv && dv->trust && !a->stats_fresh;
    if (a->stats_fresh) {
        if (dv) {
            if (int e = launch_gn_stats_table(a->x0, a->x1, B, H, W, a->C0, a->C1, a->G, 1e-5f, a->gn1_mean, a->gn1_rstd, a->gn1_gamma,
                                              a->gn1_beta, dv->ss_in, ws, st)) return e;
        } else if (int e = fise_groupnorm_stats(a->x0, a->x1, FISE_BF16, B, H, W, a->C0, a->C1, a->G, 1e-5f, a->gn1_mean, a->gn1_rstd, ws, st)) return e;
    }
    // the normalised + activated input (active tiles and their ring) is written once, then convolved
    if (!have_acts)
        if (int e = launch_gn_act_halo(a->x0, a->x1, a->C0, a->C1, B, H, W, a->gn1_mean, a->gn1_rstd, a->gn1_gamma, a->gn1_beta, a->G, 1,
                                       a->tile_idx, a->n_active, a->tile, act1, st)) return e;
    IgemmArgs c1 = conv_args(act1, nullptr, Ci, 0, B, H, W, H, W, 3, 1, 0, a->conv1_w, a->conv1_b, Co, a->tile_idx,
                             a->n_active, a->tile, a->h1_cache);
    c1.temb = a->temb; c1.temb_stride = a->temb_stride;
    if (dv && !a->stats_fresh) {       // conv2's input: SiLU(GN2(h1)) under the cached statistics, from conv1's epilogue
        c1.nview = 1;
        c1.view[0] = GnView{(bf16_t*)dv->act_mid, dv->ss_mid, Co, 0, 1, 0};
    }
    if (int e = launch_igemm(c1, iw, st)) return e;
    if (a->stats_fresh) {
        if (dv) {
            if (int e = launch_gn_stats_table(a->h1_cache, nullptr, B, H, W, Co, 0, a->G, 1e-5f, a->gn2_mean, a->gn2_rstd, a->gn2_gamma,
                                              a->gn2_beta, dv->ss_mid, ws, st)) return e;
        } else if (int e = fise_groupnorm_stats(a->h1_cache, nullptr, FISE_BF16, B, H, W, Co, 0, a->G, 1e-5f, a->gn2_mean, a->gn2_rstd, ws, st)) return e;
    }
    if (!have_acts)
        if (int e = launch_gn_act_halo(a->h1_cache, nullptr, Co, 0, B, H, W, a->gn2_mean, a->gn2_rstd, a->gn2_gamma, a->gn2_beta, a->G, 1,
                                       a->tile_idx, a->n_active, a->tile, act2, st)) return e;
    IgemmArgs c2 = conv_args(act2, nullptr, Co, 0, B, H, W, H, W, 3, 1, 0, a->conv2_w, a->conv2_b, Co, a->tile_idx,
                             a->n_active, a->tile, a->out_cache);
    if (a->sc_w) {            // 1x1 shortcut: extra K steps of the same GEMM, never stored
        c2.s0 = (const bf16_t*)a->x0; c2.s1 = (const bf16_t*)a->x1; c2.S0 = a->C0; c2.S1 = a->C1; c2.K2 = Ci;
        c2.w2 = (const bf16_t*)a->sc_w; c2.bias2 = (const bf16_t*)a->sc_b;
    } else {
        c2.res = (const bf16_t*)a->x0;
    }
    if (dv && !a->stats_fresh) set_views(c2, dv->out_view, dv->n_out_view);
    return launch_igemm(c2, iw, st);
}

struct TrWs { size_t h, h16, n, q, o, ff, gn, at, at_bytes, total; };
static TrWs tr_ws(int B, int H, int W, int C, int G, int heads, int n_active, int tile) {
    TrWs w{};
    const size_t rows = (size_t)B * n_active * tile * tile;
    size_t c = 0;
    auto take = [&](size_t bytes) { size_t o = c; c += align256(bytes); return o; };
    w.h = take(rows * C * 4); w.h16 = take(rows * C * 2); w.n = take(rows * C * 2); w.q = take(rows * C * 2); w.o = take(rows * C * 2);
    w.ff = take(rows * 4 * C * 2);
    w.gn = take(fise_groupnorm_stats_workspace_bytes(B, H, W, G));
    w.at_bytes = attention_workspace_bytes(B, n_active * tile * tile, H * W, C, heads > 0 ? heads : 1);
    w.at = take(w.at_bytes);
    w.total = c;
    return w;
}
size_t transformer_ws_bytes(const fise_transformer_args* a) {
    return tr_ws(a->B, a->H, a->W, a->C, a->G, a->heads, a->n_active, a->tile).total;
}

int run_transformer(const fise_transformer_args* a, void* workspace, const IgemmWorkspace* iw, hipStream_t st, const BlockDerived* dv) {
    const int B = a->B, H = a->H, W = a->W, C = a->C, Ma = a->n_active * a->tile * a->tile;
    const TrWs wl = tr_ws(B, H, W, C, a->G, a->heads, a->n_active, a->tile);
    char* ws = (char*)workspace;
    float* hb = (float*)(ws + wl.h);                 // residual stream of the active tokens, float
    bf16_t* nb = (bf16_t*)(ws + wl.n); bf16_t* qb = (bf16_t*)(ws + wl.q); bf16_t* ob = (bf16_t*)(ws + wl.o);
    bf16_t* fb = (bf16_t*)(ws + wl.ff);
    const float scale = 1.0f / sqrtf((float)(C / a->heads));
    auto lin = [&](const void* A, int Cin, const void* w, const void* bias, int N) {
        IgemmArgs g = linear_args(A, Ma, B, Cin, w, bias, N);
        g.tile_idx = a->tile_idx; g.tile = a->tile; g.tiles_w = W / a->tile; g.Ho = H; g.Wo = W;
        return g;
    };
    auto into_h = [&](IgemmArgs& g) { g.res = (const bf16_t*)hb; g.res_compact = 2; g.out[0] = (bf16_t*)hb; g.out_mode[0] = OUT_COMPACT_F32; };

    if (a->stats_fresh) {
        if (dv) {
            if (int e = launch_gn_stats_table(a->x, nullptr, B, H, W, C, 0, a->G, 1e-6f, a->gn_mean, a->gn_rstd, a->gn_gamma, a->gn_beta,
                                              dv->ss_in, ws + wl.gn, st)) return e;
        } else if (int e = fise_groupnorm_stats(a->x, nullptr, FISE_BF16, B, H, W, C, 0, a->G, 1e-6f, a->gn_mean, a->gn_rstd, ws + wl.gn, st)) return e;
    }
    // With a derived map the 1x1 in reads the normalised input (written by the producer of x under the cached
    // statistics, or here); without one it normalises in its own prologue.
    if (dv && !(dv->trust && !a->stats_fresh))
        if (int e = launch_gn_act_halo(a->x, nullptr, C, 0, B, H, W, a->gn_mean, a->gn_rstd, a->gn_gamma, a->gn_beta, a->G, 0,
                                       a->tile_idx, a->n_active, a->tile, dv->act_in, st)) return e;
    IgemmArgs pin = conv_args(dv ? dv->act_in : a->x, nullptr, C, 0, B, H, W, H, W, 1, 1, 0, a->pin_w, a->pin_b, C, a->tile_idx, a->n_active,
                              a->tile, hb);
    if (!dv) set_gn(pin, a->gn_mean, a->gn_rstd, a->gn_gamma, a->gn_beta, a->G, false);
    pin.out_mode[0] = OUT_COMPACT_F32;
    // every GEMM that completes the residual stream also emits the LayerNorm the next sub-block starts with
    auto with_ln = [&](IgemmArgs& g, const void* gamma, const void* beta) {
        g.ln_gamma = (const bf16_t*)gamma; g.ln_beta = (const bf16_t*)beta; g.ln_eps = 1e-5f; g.ln_out = nb;
    };
    with_ln(pin, a->ln1_g, a->ln1_b);
    if (int e = launch_igemm(pin, iw, st)) return e;
    // self-attention: LN -> stacked QKV (K, V rows scattered into the caches) -> attention -> out-proj + residual
    IgemmArgs qkv = lin(nb, C, a->qkv_w, nullptr, 3 * C);
    qkv.nsect = 3; qkv.sect_n = C;
    qkv.out[0] = qb; qkv.out_mode[0] = OUT_COMPACT;
    qkv.out[1] = (bf16_t*)a->K_cache; qkv.out_mode[1] = OUT_MAP;
    qkv.out[2] = (bf16_t*)a->Vt_cache; qkv.out_mode[2] = OUT_TOKENS_T;
    if (int e = launch_igemm(qkv, iw, st)) return e;
    if (int e = launch_attention(qb, a->K_cache, a->Vt_cache, B, Ma, H * W, H * W, C, a->heads, scale, ob, ws + wl.at, wl.at_bytes, st)) return e;
    IgemmArgs o1 = lin(ob, C, a->o1_w, a->o1_b, C); into_h(o1); with_ln(o1, a->ln2_g, a->ln2_b);
    if (int e = launch_igemm(o1, iw, st)) return e;
    // cross-attention against the context K/V
    IgemmArgs q2 = lin(nb, C, a->q2_w, nullptr, C); q2.out[0] = qb;
    if (int e = launch_igemm(q2, iw, st)) return e;
    if (int e = launch_attention(qb, a->K_ctx, a->Vt_ctx, B, Ma, a->n_ctx, a->n_ctx_stride, C, a->heads, scale, ob, nullptr, 0, st)) return e;
    IgemmArgs o2 = lin(ob, C, a->o2_w, a->o2_b, C); into_h(o2); with_ln(o2, a->ln3_g, a->ln3_b);
    if (int e = launch_igemm(o2, iw, st)) return e;
    // feed-forward: LN -> first GEMM with the GEGLU gate in its epilogue -> second GEMM + residual
    IgemmArgs f1 = lin(nb, C, a->ff1_w, a->ff1_b, 4 * C); f1.geglu = 1; f1.out[0] = fb;
    if (int e = launch_igemm(f1, iw, st)) return e;
    IgemmArgs f2 = lin(fb, 4 * C, a->ff2_w, a->ff2_b, C); into_h(f2);
    f2.mirror = (bf16_t*)(ws + wl.h16);               // bf16 copy of the final residual stream: A operand of the 1x1 out
    if (int e = launch_igemm(f2, iw, st)) return e;
    // 1x1 out + block input, scattered into the cached block output
    IgemmArgs po = lin(ws + wl.h16, C, a->pout_w, a->pout_b, C);
    po.res = (const bf16_t*)a->x; po.res_compact = 0; po.out[0] = (bf16_t*)a->out_cache; po.out_mode[0] = OUT_MAP;
    if (dv && !a->stats_fresh) set_views(po, dv->out_view, dv->n_out_view);
    return launch_igemm(po, iw, st);
}

static int check_region(const char* fn, int H, int W, int tile, int n_active, const int32_t* idx) {
    if (tile < 1 || H < 1 || W < 1 || H % tile || W % tile) return fail(FISE_ERR_SHAPE, "%s: H=%d W=%d tile=%d", fn, H, W, tile);
    if (n_active < 0 || n_active > (H / tile) * (W / tile)) return fail(FISE_ERR_CAPACITY, "%s: n_active %d", fn, n_active);
    if (n_active > 0 && !idx) return fail(FISE_ERR_NULL, "%s: null tile_idx", fn);
    return FISE_OK;
}

}  // namespace fise

using namespace fise;

extern "C" size_t fise_masked_resnet_block_workspace_bytes(const fise_resnet_args* a) {
    return a ? align256(resnet_ws_bytes(a)) + igemm_workspace_bytes() : 0;
}

extern "C" int fise_masked_resnet_block(const fise_resnet_args* a, void* workspace, size_t workspace_bytes, void* stream) {
    const char* fn = "fise_masked_resnet_block";
    if (!a) return fail(FISE_ERR_NULL, "%s: null args", fn);
    if (!a->x0 || !a->gn1_mean || !a->gn1_rstd || !a->gn1_gamma || !a->gn1_beta || !a->conv1_w || !a->gn2_mean || !a->gn2_rstd ||
        !a->gn2_gamma || !a->gn2_beta || !a->conv2_w || !a->h1_cache || !a->out_cache)
        return fail(FISE_ERR_NULL, "%s: null pointer", fn);
    if (a->C1 < 0 || (a->C1 > 0 && !a->x1)) return fail(FISE_ERR_NULL, "%s: skip source missing", fn);
    const int Ci = a->C0 + a->C1;
    if (a->B < 1 || a->C0 < 1 || a->Cout < 1 || a->G < 1 || Ci % a->G || a->Cout % a->G) return fail(FISE_ERR_SHAPE, "%s: channels %d->%d, groups %d", fn, Ci, a->Cout, a->G);
    if (a->C0 % 32 || a->C1 % 32 || a->Cout % 32) return fail(FISE_ERR_ALIGN, "%s: channel counts must be multiples of 32", fn);
    if (Ci != a->Cout && !a->sc_w) return fail(FISE_ERR_NULL, "%s: %d -> %d channels needs the 1x1 shortcut", fn, Ci, a->Cout);
    // the identity shortcut reads x0 with row pitch Cout: a concatenated input has no such map
    if (a->C1 > 0 && !a->sc_w) return fail(FISE_ERR_SHAPE, "%s: two sources (%d + %d channels) need the 1x1 shortcut", fn, a->C0, a->C1);
    if (int e = check_region(fn, a->H, a->W, a->tile, a->n_active, a->tile_idx)) return e;
    if (a->out_cache == a->x0 || a->h1_cache == a->x0 || a->out_cache == a->h1_cache) return fail(FISE_ERR_SHAPE, "%s: maps alias", fn);
    if (a->n_active == 0) return FISE_OK;
    if (!workspace || workspace_bytes < fise_masked_resnet_block_workspace_bytes(a)) return fail(FISE_ERR_CAPACITY, "%s: workspace too small", fn);
    IgemmWorkspace iw;
    const size_t off = align256(resnet_ws_bytes(a));
    if (int e = igemm_workspace_init((char*)workspace + off, workspace_bytes - off, &iw, as_stream(stream))) return e;
    return run_resnet(a, workspace, &iw, as_stream(stream), nullptr);
}

extern "C" size_t fise_masked_transformer_block_workspace_bytes(const fise_transformer_args* a) {
    return a ? align256(transformer_ws_bytes(a)) + igemm_workspace_bytes() : 0;
}

extern "C" int fise_masked_transformer_block(const fise_transformer_args* a, void* workspace, size_t workspace_bytes, void* stream) {
    const char* fn = "fise_masked_transformer_block";
    if (!a) return fail(FISE_ERR_NULL, "%s: null args", fn);
    const void* req[] = {a->x, a->gn_mean, a->gn_rstd, a->gn_gamma, a->gn_beta, a->pin_w, a->ln1_g, a->ln1_b, a->qkv_w, a->o1_w,
                         a->ln2_g, a->ln2_b, a->q2_w, a->o2_w, a->K_ctx, a->Vt_ctx, a->ln3_g, a->ln3_b, a->ff1_w, a->ff2_w,
                         a->pout_w, a->K_cache, a->Vt_cache, a->out_cache};
    for (const void* p : req) if (!p) return fail(FISE_ERR_NULL, "%s: null pointer", fn);
    if (a->B < 1 || a->C < 1 || a->G < 1 || a->heads < 1 || a->C % a->G || a->C % a->heads) return fail(FISE_ERR_SHAPE, "%s: C=%d groups=%d heads=%d", fn, a->C, a->G, a->heads);
    const int d = a->C / a->heads;
    if (a->C % 32 || d % 8 || d > 160) return fail(FISE_ERR_ALIGN, "%s: C=%d (multiple of 32), head dim %d (multiple of 8, <= 160)", fn, a->C, d);
    if (int e = check_region(fn, a->H, a->W, a->tile, a->n_active, a->tile_idx)) return e;
    if ((a->H * a->W) % 8) return fail(FISE_ERR_ALIGN, "%s: H*W must be a multiple of 8", fn);
    if (a->n_ctx < 1 || a->n_ctx_stride < a->n_ctx || a->n_ctx_stride % 8) return fail(FISE_ERR_ALIGN, "%s: n_ctx %d stride %d", fn, a->n_ctx, a->n_ctx_stride);
    if (a->x == a->out_cache) return fail(FISE_ERR_SHAPE, "%s: out_cache aliases x", fn);
    if (a->n_active == 0) return FISE_OK;
    if (!workspace || workspace_bytes < fise_masked_transformer_block_workspace_bytes(a)) return fail(FISE_ERR_CAPACITY, "%s: workspace too small", fn);
    IgemmWorkspace iw;
    const size_t off = align256(transformer_ws_bytes(a));
    if (int e = igemm_workspace_init((char*)workspace + off, workspace_bytes - off, &iw, as_stream(stream))) return e;
    return run_transformer(a, workspace, &iw, as_stream(stream), nullptr);
}

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
    const IgemmWorkspace* iw = nullptr;
    IgemmArgs g = linear_args(ctx, n_ctx, B, Dc, Wk, nullptr, C);
    g.out[0] = (bf16_t*)K_ctx;
    if (int e = launch_igemm(g, iw, st)) return e;
    g.w = (const bf16_t*)Wv; g.out[0] = (bf16_t*)Vt_ctx; g.out_mode[0] = OUT_TOKENS_T; g.Ho = 1; g.Wo = n_stride;
    return launch_igemm(g, iw, st);
}

extern "C" size_t fise_masked_attention_workspace_bytes(int B, int C, int n_active, int tile) {
    if (B < 1 || C < 1 || n_active < 0 || tile < 1) return 0;
    const size_t rows = (size_t)B * n_active * tile * tile;
    // the key-split scratch is sized for the longest key set a caller can pass (a 128 x 128 token map)
    return 3 * align256(rows * C * sizeof(bf16_t)) + attention_workspace_bytes(B, n_active * tile * tile, 128 * 128, C, 8) + 256;
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
    const IgemmWorkspace* iw = nullptr;
    const int Ma = n_active * tile * tile, rows = B * Ma;
    const size_t buf = align256((size_t)rows * C * sizeof(bf16_t));
    char* ws = (char*)workspace;
    bf16_t* nbuf = (bf16_t*)ws; bf16_t* qbuf = (bf16_t*)(ws + buf); bf16_t* obuf = (bf16_t*)(ws + 2 * buf);
    const float scale = 1.0f / sqrtf((float)d);

    if (int e = launch_ln_rows(x, 0, rows, C, ln_gamma, ln_beta, 1e-5f, nbuf, tile_idx, tile, W / tile, H, W, Ma, st)) return e;
    IgemmArgs g = linear_args(nbuf, Ma, B, C, Wq, nullptr, C);
    g.tile_idx = tile_idx; g.tile = tile; g.tiles_w = W / tile; g.Ho = H; g.Wo = W;
    g.out[0] = qbuf;
    if (int e = launch_igemm(g, iw, st)) return e;
    if (self) {
        g.w = (const bf16_t*)Wk; g.out[0] = (bf16_t*)K_cache; g.out_mode[0] = OUT_MAP;
        if (int e = launch_igemm(g, iw, st)) return e;
        g.w = (const bf16_t*)Wv; g.out[0] = (bf16_t*)Vt_cache; g.out_mode[0] = OUT_TOKENS_T;
        if (int e = launch_igemm(g, iw, st)) return e;
        if (int e = launch_attention(qbuf, K_cache, Vt_cache, B, Ma, H * W, H * W, C, heads, scale, obuf, ws + 3 * buf, workspace_bytes - 3 * buf, st)) return e;
    } else {
        if (int e = launch_attention(qbuf, K_ctx, Vt_ctx, B, Ma, n_ctx, n_ctx_stride, C, heads, scale, obuf, nullptr, 0, st)) return e;
    }
    IgemmArgs o = linear_args(obuf, Ma, B, C, Wo, bo, C);
    o.tile_idx = tile_idx; o.tile = tile; o.tiles_w = W / tile; o.Ho = H; o.Wo = W;
    o.res = (const bf16_t*)x; o.res_compact = 0;
    o.out[0] = (bf16_t*)y_cache; o.out_mode[0] = OUT_MAP;
    return launch_igemm(o, iw, st);
}

// ---- keys-restricted attention: active queries x keys / values of the active tokens only
static size_t restricted_vt_stride(int Ma) { return (size_t)((Ma + 7) / 8 * 8); }

extern "C" size_t fise_masked_attention_restricted_workspace_bytes(int B, int C, int n_active, int tile) {
    if (B < 1 || C < 1 || n_active < 0 || tile < 1) return 0;
    const int Ma = n_active * tile * tile;
    const size_t rows = (size_t)B * Ma;
    return 4 * align256(rows * C * sizeof(bf16_t)) + align256((size_t)B * C * restricted_vt_stride(Ma) * sizeof(bf16_t)) +
           attention_workspace_bytes(B, Ma, Ma, C, 8) + 256;
}

extern "C" int fise_masked_attention_restricted(const void* x, const void* ln_gamma, const void* ln_beta, const void* Wq,
                                                const void* Wk, const void* Wv, const void* Wo, const void* bo, int dtype, int B,
                                                int H, int W, int C, int heads, const int32_t* tile_idx, int n_active, int tile,
                                                void* y_cache, void* workspace, size_t workspace_bytes, void* stream) {
    const char* fn = "fise_masked_attention_restricted";
    if (!x || !ln_gamma || !ln_beta || !Wq || !Wk || !Wv || !Wo || !y_cache) return fail(FISE_ERR_NULL, "%s: null pointer", fn);
    if (dtype != FISE_BF16) return fail(FISE_ERR_DTYPE, "%s: bf16 only", fn);
    if (B < 1 || H < 1 || W < 1 || C < 1 || heads < 1 || C % heads || tile < 1 || H % tile || W % tile)
        return fail(FISE_ERR_SHAPE, "%s: B%d H%d W%d C%d heads%d tile%d", fn, B, H, W, C, heads, tile);
    const int d = C / heads;
    if (C % 32 || d % 8 || d > 160) return fail(FISE_ERR_ALIGN, "%s: C=%d (multiple of 32), head dim %d (multiple of 8, <= 160)", fn, C, d);
    if (n_active < 0 || n_active > (H / tile) * (W / tile)) return fail(FISE_ERR_CAPACITY, "%s: n_active %d", fn, n_active);
    if (n_active == 0) return FISE_OK;
    if (!tile_idx) return fail(FISE_ERR_NULL, "%s: null tile_idx", fn);
    if (!workspace || workspace_bytes < fise_masked_attention_restricted_workspace_bytes(B, C, n_active, tile))
        return fail(FISE_ERR_CAPACITY, "%s: workspace too small", fn);
    if (y_cache == x) return fail(FISE_ERR_SHAPE, "%s: y_cache aliases x", fn);

    hipStream_t st = as_stream(stream);
    const IgemmWorkspace* iw = nullptr;
    const int Ma = n_active * tile * tile, rows = B * Ma;
    const int vstride = (int)restricted_vt_stride(Ma);
    const size_t buf = align256((size_t)rows * C * sizeof(bf16_t));
    const size_t vbuf = align256((size_t)B * C * vstride * sizeof(bf16_t));
    char* ws = (char*)workspace;
    bf16_t* nbuf = (bf16_t*)ws; bf16_t* qbuf = (bf16_t*)(ws + buf); bf16_t* kbuf = (bf16_t*)(ws + 2 * buf);
    bf16_t* obuf = (bf16_t*)(ws + 3 * buf); bf16_t* vtbuf = (bf16_t*)(ws + 4 * buf);
    char* atws = ws + 4 * buf + vbuf;
    const float scale = 1.0f / sqrtf((float)d);

    if (int e = launch_ln_rows(x, 0, rows, C, ln_gamma, ln_beta, 1e-5f, nbuf, tile_idx, tile, W / tile, H, W, Ma, st)) return e;
    // Q, K as compact rows; V as compact transposed columns [B, C, vstride] (row r of batch b -> column r): these
    // launches address rows only, so they carry no tile list
    IgemmArgs g = linear_args(nbuf, Ma, B, C, Wq, nullptr, C);
    g.out[0] = qbuf;
    if (int e = launch_igemm(g, iw, st)) return e;
    g.w = (const bf16_t*)Wk; g.out[0] = kbuf;
    if (int e = launch_igemm(g, iw, st)) return e;
    g.w = (const bf16_t*)Wv; g.out[0] = vtbuf; g.out_mode[0] = OUT_TOKENS_T; g.Ho = 1; g.Wo = vstride;
    if (int e = launch_igemm(g, iw, st)) return e;
    if (int e = launch_attention(qbuf, kbuf, vtbuf, B, Ma, Ma, vstride, C, heads, scale, obuf, atws,
                                 workspace_bytes - (size_t)(atws - ws), st)) return e;
    IgemmArgs o = linear_args(obuf, Ma, B, C, Wo, bo, C);
    o.tile_idx = tile_idx; o.tile = tile; o.tiles_w = W / tile; o.Ho = H; o.Wo = W;
    o.res = (const bf16_t*)x; o.res_compact = 0;
    o.out[0] = (bf16_t*)y_cache; o.out_mode[0] = OUT_MAP;
    return launch_igemm(o, iw, st);
}
