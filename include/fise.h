/*
 * fise.h - C ABI of the MI355X (gfx950) masked UNet-step library.
 *
 * The library implements the per-denoising-step hot path of FISEdit
 * (arxiv 2305.17423, "Accelerating Text-to-Image Editing via Cache-Enabled
 * Sparse Diffusion Inference"): find the affected region from the difference
 * of cached and fresh feature maps, then recompute the U-Net only there and
 * scatter the results into the cached feature maps.
 *
 * Conventions (all entry points)
 *  - Every pointer is a DEVICE pointer unless the comment says "host".
 *  - Feature maps are [B, H, W, C], channels innermost; the same memory read as
 *    tokens is [B, H*W, C] with token = y*W + x.  Convolution weights are
 *    [C_out, k, k, C_in]; linear weights [out, in].
 *  - `dtype` selects the element type of activations AND learnable parameters
 *    (weights, biases, norm scale/shift): FISE_F32 or FISE_BF16.  GroupNorm
 *    statistics and the time-embedding projection `temb` are always float.
 *    Accumulation is float in both cases.
 *  - Active region: `tile_idx` holds `n_active` ascending row-major ids of
 *    active tiles on the (H/tile) x (W/tile) grid of the OUTPUT map; `n_active`
 *    is a host integer (read back once after fise_mask_detect).  Active pixels
 *    are enumerated tile by tile in list order, row-major inside a tile.
 *  - `y_cache`, `K_cache`, `V_cache` are read-modify-write: only active
 *    positions are written.  With n_active == 0, or on any error, no output is
 *    touched.  The same kernels run "dense" when given the full tile list.
 *  - The library allocates no device memory, keeps no device pointers and
 *    never synchronises: all work is enqueued on the caller's stream
 *    (`stream` is a hipStream_t passed as void*, NULL = default stream).
 *    Scratch space is passed in as `workspace` (256-byte aligned device memory
 *    of at least the size the matching *_workspace_bytes query returns).  A
 *    workspace must not be shared by calls that may overlap in time.
 *  - Pointers must be 16-byte aligned and channel counts of bf16 maps multiples
 *    of 8 unless noted (rows are moved as 16-byte vectors).
 *  - Return value: FISE_OK (0) or a negative fise_status; fise_last_error()
 *    returns a thread-local host string describing the last failure.
 *    Arguments are validated on the host before anything is launched.
 */
#ifndef FISE_H
#define FISE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { FISE_F32 = 0, FISE_BF16 = 1 } fise_dtype;

typedef enum {
    FISE_OK = 0,
    FISE_ERR_NULL = -1,      /* a required pointer is NULL */
    FISE_ERR_SHAPE = -2,     /* H or W not divisible by tile, C % groups, C % heads, ... */
    FISE_ERR_DTYPE = -3,     /* dtype not supported by this entry point */
    FISE_ERR_ALIGN = -4,     /* pointer not 16-byte aligned / channel count not a multiple of 8 */
    FISE_ERR_CAPACITY = -5,  /* n_active beyond the tile grid, workspace too small */
    FISE_ERR_HIP = -6        /* a HIP call (kernel launch) failed */
} fise_status;

const char* fise_last_error(void);   /* host string, thread local, never NULL */
int fise_version(void);

/* ------------------------------------------------------------------------
 * Mask generation (section "Fine-Grained Mask Generation": the |X - Y|
 * difference of cached and fresh maps and the set {diff >= eps}; section
 * "Adaptive Pixel-Wise Sparse Convolution": the blocks gathered under mask m).
 * ------------------------------------------------------------------------ */

/* d[y,x] = (1/(B*C)) * sum_b sum_c |fresh - cached| accumulated in float, b
 * outermost then c ascending; pix = d > threshold (strict); a tile is active
 * iff any of its pixels is.  Outputs: pix_mask[H*W] (uint8, required),
 * tile_mask[(H/tile)*(W/tile)] (uint8), tile_idx[capacity] (ascending ids;
 * entries beyond *n_active are not written), n_active[1] (device int32: the
 * number of active tiles, even when it exceeds `capacity`; then only the first
 * `capacity` ids are stored).  Any C >= 1 is accepted (no alignment rule). */
int fise_mask_detect(const void* cached, const void* fresh, int dtype, int B, int H, int W, int C,
                     float threshold, int tile, uint8_t* pix_mask, uint8_t* tile_mask,
                     int32_t* tile_idx, int capacity, int32_t* n_active, void* stream);

/* Same tile reduction and compaction for a user-supplied pixel mask
 * (appendix: masks drawn by the user). */
int fise_mask_from_pixels(const uint8_t* pix_mask, int H, int W, int tile, uint8_t* tile_mask,
                          int32_t* tile_idx, int capacity, int32_t* n_active, void* stream);

/* 2x2 OR-pool: out[H/2, W/2] is set where any of the four children in
 * mask[H, W] is (mask of the next coarser U-Net level; the paper notes that
 * sparsity falls as resolution does).  H, W even. */
int fise_mask_downsample(const uint8_t* mask, int H, int W, uint8_t* out, void* stream);

/* Automatic threshold (same section, the OTSU(eps) objective): diff[n] (float,
 * device) is min-max normalised to [0,1], and eps* = argmax over the grid
 * k/256, k = 0..256 (first maximiser) of N1*N2/(N1+N2)^2 * (mean_A - mean_B)^2
 * with A = {diff < eps}, B = {diff >= eps}.  Writes eps_out[1] (device float,
 * in normalised units) and pix_mask[n] = normalised diff >= eps*.
 * workspace: fise_otsu_workspace_bytes(). */
size_t fise_otsu_workspace_bytes(void);
int fise_otsu_mask(const float* diff, int n, float* eps_out, uint8_t* pix_mask, void* workspace, void* stream);

/* diff_acc[y,x] += mean over (b,c) of |fresh - cached| (float accumulation):
 * the sum over steps t1..t2 of the mask-generation equation, one call per step.
 * diff_acc[H*W] float, caller zeroes it before the first step. */
int fise_diff_accumulate(const void* cached, const void* fresh, int dtype, int B, int H, int W, int C,
                         float* diff_acc, void* stream);

/* Block-size choice of section "Adaptive Pixel-Wise Sparse Convolution":
 * counts[i*5+j] = number of (h,w) = (2<<i, 2<<j) blocks holding a masked pixel,
 * for the 25 candidate sizes (device int32[25]); sizes that do not divide the
 * map give -1.  The argmin of (h+2)(w+2)*count is a 25-element host loop. */
int fise_apsc_block_counts(const uint8_t* pix_mask, int H, int W, int32_t* counts, void* stream);

/* The argmin itself, on the host: counts is the HOST copy of the 25 counts above,
 * (kh, kw) the kernel size.  cost(h,w) = (h+kh-1)(w+kw-1)*count, the gathered
 * input pixels of all blocks (the printed (h-kh+1)(w-kw+1) is read with (h,w) as
 * the output block, since it vanishes for h < kh).  Sizes with count -1 are
 * skipped; ties go to the first size in (h, w) row-major order.  Returns
 * FISE_ERR_SHAPE when no size divides the map.  All pointers host; cost may be NULL. */
int fise_apsc_select(const int32_t* counts, int kh, int kw, int* h, int* w, int64_t* cost);

/* fise_mask_from_pixels for rectangular blocks of tile_h x tile_w pixels: tile_mask
 * [H/tile_h, W/tile_w], tile_idx ascending row-major block ids, same capacity and
 * n_active rules. */
int fise_mask_from_pixels_rect(const uint8_t* pix_mask, int H, int W, int tile_h, int tile_w, uint8_t* tile_mask,
                               int32_t* tile_idx, int capacity, int32_t* n_active, void* stream);

/* ------------------------------------------------------------------------
 * Normalisation (section "Approximate Normalization": mean and variance cached
 * from the previous generation are reused at masked positions).
 * ------------------------------------------------------------------------ */

/* Dense statistics of GroupNorm over the channel concatenation of x
 * [B,H,W,C0] and x1 [B,H,W,C1] (x1 may be NULL with C1 = 0): per (b, group)
 * mean and rstd = 1/sqrt(biased variance + eps), float [B, G].
 * (C0+C1) % G == 0.  workspace: fise_groupnorm_stats_workspace_bytes(B,H,W,C0+C1). */
size_t fise_groupnorm_stats_workspace_bytes(int B, int H, int W, int C);
int fise_groupnorm_stats(const void* x, const void* x1, int dtype, int B, int H, int W, int C0, int C1,
                         int G, float eps, float* mean, float* rstd, void* workspace, void* stream);

/* fise_groupnorm_stats for callers that cannot allocate or pass a workspace (code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc):
 * same arguments without `workspace`, same kernels, same results bit for bit.  The
 * per-chunk partial sums go to a fixed array in device memory owned by the library
 * (fise_groupnorm_stats_static_capacity_bytes() = 1 MiB per GPU, held until the
 * process ends); its device address is looked up once per GPU on the first call
 * there.  Calls need B * ceil(H*W / 64) * G * 16 bytes of it and return
 * FISE_ERR_CAPACITY beyond that (nothing is launched).  The entry point allocates
 * and frees nothing.  All calls on one GPU share the array: calls that may overlap
 * in time on one GPU (different streams) race and must be ordered by the caller. */
size_t fise_groupnorm_stats_static_capacity_bytes(void);
int fise_groupnorm_stats_static(const void* x, const void* x1, int dtype, int B, int H, int W, int C0, int C1,
                                int G, float eps, float* mean, float* rstd, void* stream);

/* y = SiLU((x - mean[b,g]) * rstd[b,g] * gamma[c] + beta[c]) at active pixels,
 * with the GIVEN statistics; other positions of y_cache keep their value. */
int fise_masked_groupnorm_silu(const void* x, const float* mean, const float* rstd, const void* gamma,
                               const void* beta, int dtype, int B, int H, int W, int C, int G,
                               const int32_t* tile_idx, int n_active, int tile, void* y_cache, void* stream);

/* ------------------------------------------------------------------------
 * Masked convolution (section "Adaptive Pixel-Wise Sparse Convolution": tiled
 * sparse convolution - gather active blocks with their halo, convolve,
 * scatter into the cached map).
 * ------------------------------------------------------------------------ */

/* General form.  y[b,p,co] = bias[co] + sum_{ky,kx,ci} w[co,ky,kx,ci] *
 * act(xcat[b, q(p,ky,kx), ci]) (+ temb[b,co]) (+ residual[b,p,co]) for p in
 * active tiles of the output map; zero outside the image; everything else in
 * y_cache untouched.  xcat = channel concatenation of x0 [B,H,W,C0] and x1
 * [B,H,W,C1] (x1 NULL, C1 0 for one source).  ksize 1 or 3 (padding ksize/2).
 * stride 1 or 2: q = stride*p + (ky,kx) - pad, output (H/stride, W/stride).
 * upsample != 0: input enlarged 2x by nearest neighbour first, q = (p + (ky,kx)
 * - pad) >> 1, output (2H, 2W); stride must be 1.  act = identity, or
 * GroupNorm(+SiLU) with the given statistics when gn_mean != NULL (gn_silu 0
 * gives the normalisation alone).  `tile` is the tile edge on the OUTPUT map.
 * y_cache must not alias x0/x1; residual may alias y_cache.
 * bf16: C0, C1 multiples of 32 use the MFMA path; other channel counts (and
 * FISE_F32) use a scalar path. */
typedef struct {
    const void* x0; const void* x1; int C0, C1;
    int B, H, W;                 /* input map */
    const void* w; const void* bias; int Cout; int ksize, stride, upsample;
    const float* gn_mean; const float* gn_rstd; const void* gn_gamma; const void* gn_beta; int G; int gn_silu;
    const float* temb;           /* [B, Cout] or NULL */
    const void* residual;        /* [B, Ho, Wo, Cout] or NULL */
    const int32_t* tile_idx; int n_active; int tile;
    void* y_cache;               /* [B, Ho, Wo, Cout] */
    int dtype;
    int tile_w;                  /* 0: square tiles of edge `tile`; else tiles of `tile` rows x `tile_w` columns,
                                    the rectangular blocks of the adaptive block-size selection (tile_idx then
                                    counts such blocks row-major, as fise_mask_from_pixels_rect writes them) */
} fise_conv_args;
size_t fise_masked_conv_workspace_bytes(const fise_conv_args* a);     /* `a` host */
int fise_masked_conv(const fise_conv_args* a /* host */, void* workspace, size_t workspace_bytes, void* stream);

/* The 3x3 case named by the paper: one source, stride 1 or 2, optional fused
 * GroupNorm+SiLU prologue (gn_mean NULL = none) and temb / residual epilogue. */
int fise_masked_conv3x3(const void* x, const void* w, const void* bias, int dtype, int B, int H, int W,
                        int Cin, int Cout, int stride, const int32_t* tile_idx, int n_active, int tile,
                        const float* gn_mean, const float* gn_rstd, const void* gn_gamma, const void* gn_beta, int G,
                        const float* temb, const void* residual, void* y_cache,
                        void* workspace, size_t workspace_bytes, void* stream);

/* ------------------------------------------------------------------------
 * Attention (section "Approximate Attention": masked tokens are gathered
 * before self- and cross-attention; only those queries are computed).
 * ------------------------------------------------------------------------ */

/* Layout of V operands: TRANSPOSED, Vt[B, C, n_stride] (keys innermost,
 * n_stride >= n_keys, multiple of 8, padding columns arbitrary), so that the
 * P*V product reads keys contiguously.  K operands are [B, n_keys, C]. */

/* out[b,m,:] = softmax_k(q[b,m,h].K[b,k,h] * scale) V[b,k,h] per head h
 * (channels [h*d,(h+1)*d), d = C/heads) over ALL n_keys keys.  q, out
 * [B, M, C].  bf16 only; d a multiple of 8, d <= 160.  With a workspace the key
 * range is split over workgroups when there are few queries (partials merged in
 * a fixed order); workspace NULL runs unsplit. */
size_t fise_attention_active_workspace_bytes(int B, int M, int n_keys, int C, int heads);
int fise_attention_active(const void* q, const void* K, const void* Vt, int dtype, int B, int M, int n_keys,
                          int n_stride, int C, int heads, float scale, void* out,
                          void* workspace, size_t workspace_bytes, void* stream);

/* K/V of the text context, once per conditioning: K_ctx[B,n_ctx,C] =
 * ctx[B,n_ctx,Dc] Wk^T, Vt_ctx[B,C,n_stride] = (ctx Wv^T)^T. */
size_t fise_context_kv_workspace_bytes(int B, int n_ctx, int Dc, int C);
int fise_context_kv(const void* ctx, const void* Wk, const void* Wv, int dtype, int B, int n_ctx, int Dc, int C,
                    int n_stride, void* K_ctx, void* Vt_ctx, void* workspace, size_t workspace_bytes, void* stream);

/* One attention sub-layer on the token map x [B,H,W,C]:
 *   y = x + Attn(LayerNorm(x)) Wo^T + bo   at active tokens, scattered into y_cache.
 * Self-attention when K_cache/Vt_cache are given: K, V rows of the active
 * tokens are refreshed in the caches (K_cache [B,H*W,C], Vt_cache [B,C,H*W]),
 * then each active query attends to every key.  Cross-attention when they are
 * NULL: keys/values K_ctx [B,n_ctx,C], Vt_ctx [B,C,n_ctx_stride].
 * LayerNorm eps 1e-5; softmax scale 1/sqrt(C/heads).  bf16 only. */
size_t fise_masked_attention_workspace_bytes(int B, int C, int n_active, int tile);
int fise_masked_attention(const void* x, const void* ln_gamma, const void* ln_beta, const void* Wq, const void* Wk,
                          const void* Wv, const void* Wo, const void* bo, int dtype, int B, int H, int W, int C,
                          int heads, void* K_cache, void* Vt_cache, const void* K_ctx, const void* Vt_ctx,
                          int n_ctx, int n_ctx_stride, const int32_t* tile_idx, int n_active, int tile,
                          void* y_cache, void* workspace, size_t workspace_bytes, void* stream);

/* ------------------------------------------------------------------------
 * Masked ResNet and transformer modules (section "Sparse Computation": the
 * U-Net is a stack of these two module kinds, each recomputed on the masked
 * region only).  bf16 only.  The UNet step below is a sequence of these two
 * calls plus resampling convolutions.
 * ------------------------------------------------------------------------ */

/* out = shortcut(x) + conv2(SiLU(GN2(h1))),  h1 = conv1(SiLU(GN1(x))) + temb,
 * at active pixels; x = channel concatenation of x0 [B,H,W,C0] and x1
 * [B,H,W,C1] (skip link; NULL / 0 for none).  h1_cache and out_cache
 * [B,H,W,Cout] are updated in place (conv2's halo reads cached h1).
 * shortcut = identity (one source: C1 == 0, C0 == Cout, sc_w NULL) or the 1x1
 * conv sc_w/sc_b (required whenever C0+C1 != Cout or a skip source is given).
 * gn*_mean/rstd [B,G] float: with stats_fresh == 0 they are inputs (statistics
 * cached from the previous generation); with stats_fresh != 0 they are
 * recomputed from the current x / updated h1 and written back (eps 1e-5).
 * temb [B, temb_stride] float, column c of this block at temb[b*temb_stride+c]
 * (NULL = none).  Channel counts multiples of 32. */
typedef struct {
    const void* x0; const void* x1; int C0, C1;
    int B, H, W, Cout, G;
    float* gn1_mean; float* gn1_rstd; const void* gn1_gamma; const void* gn1_beta;
    const void* conv1_w; const void* conv1_b;
    const float* temb; int temb_stride;
    float* gn2_mean; float* gn2_rstd; const void* gn2_gamma; const void* gn2_beta;
    const void* conv2_w; const void* conv2_b;
    const void* sc_w; const void* sc_b;
    const int32_t* tile_idx; int n_active; int tile;
    void* h1_cache; void* out_cache;
    int stats_fresh;
} fise_resnet_args;
size_t fise_masked_resnet_block_workspace_bytes(const fise_resnet_args* a /* host */);
int fise_masked_resnet_block(const fise_resnet_args* a /* host */, void* workspace, size_t workspace_bytes, void* stream);

/* out = x + P_out( FF( CA( SA( P_in(GN(x)) ) ) ) ) on active tokens:
 *   h  = pin(GN(x))                        GroupNorm eps 1e-6, no activation; 1x1 conv
 *   h += Wo1 Attn(LN1(h); K,V of all tokens) + bo1     K,V rows of active tokens refreshed first
 *   h += Wo2 Attn(LN2(h); K_ctx, Vt_ctx)   + bo2       text context of the NEW conditioning
 *   h += W2 GEGLU(W1 LN3(h) + b1) + b2
 *   out = pout(h) + x                      scattered into out_cache [B,H,W,C]
 * qkv_w is [3C, C]: Wq, Wk, Wv stacked.  K_cache [B,H*W,C], Vt_cache [B,C,H*W]
 * (transposed) are updated in place at active tokens.  gn_mean/rstd as in the
 * ResNet block.  C multiple of 32, C/heads multiple of 8 and <= 160, H*W
 * multiple of 8.  x must not alias out_cache. */
typedef struct {
    const void* x; int B, H, W, C, G, heads;
    float* gn_mean; float* gn_rstd; const void* gn_gamma; const void* gn_beta;
    const void* pin_w; const void* pin_b;
    const void* ln1_g; const void* ln1_b; const void* qkv_w; const void* o1_w; const void* o1_b;
    const void* ln2_g; const void* ln2_b; const void* q2_w; const void* o2_w; const void* o2_b;
    const void* K_ctx; const void* Vt_ctx; int n_ctx, n_ctx_stride;
    const void* ln3_g; const void* ln3_b; const void* ff1_w; const void* ff1_b; const void* ff2_w; const void* ff2_b;
    const void* pout_w; const void* pout_b;
    void* K_cache; void* Vt_cache; void* out_cache;
    const int32_t* tile_idx; int n_active; int tile;
    int stats_fresh;
} fise_transformer_args;
size_t fise_masked_transformer_block_workspace_bytes(const fise_transformer_args* a /* host */);
int fise_masked_transformer_block(const fise_transformer_args* a /* host */, void* workspace, size_t workspace_bytes, void* stream);

/* ------------------------------------------------------------------------
 * Masked UNet step (section "Sparse Computation": the U-Net's ResNet and
 * attention modules run on the masked region only, the rest is reused from
 * the cache of the previous generation; overview figure: pre-computed
 * activations of every layer are reused according to the mask).
 * The network is the Stable-Diffusion-1.x denoiser layout, parametric.
 * ------------------------------------------------------------------------ */
#define FISE_MAX_LEVELS 8
typedef struct {
    int in_ch, out_ch, base;          /* latent channels, model width of level 0 */
    int n_levels; int mults[FISE_MAX_LEVELS]; int attn[FISE_MAX_LEVELS];
    int layers;                       /* ResNet(+transformer) pairs per down level; up levels have layers+1 */
    int heads, ctx_dim, n_ctx, groups;
    int H, W, B;                      /* latent size, batch */
} fise_unet_desc;

typedef struct fise_unet fise_unet;   /* host-only plan: owns no device memory */

int fise_unet_create(const fise_unet_desc* desc /* host */, fise_unet** out /* host */);
void fise_unet_destroy(fise_unet* u);
int fise_unet_desc_get(const fise_unet* u, fise_unet_desc* out /* host */);   /* the description the plan was made from */

/* Flat buffers.  `kind` 0 = weights (bf16 elements; offset/numel in elements),
 * 1 = per-step cache, the tensors the method stores (offset/numel in BYTES; maps
 * bf16, statistics float), 2 = context K/V buffer (bytes), 3 = per-step cache, the
 * DERIVED tensors kept behind the stored ones in the same buffer (bytes): for every
 * GroupNorm its scale / shift table under the cached statistics ('<gn>.ss', float
 * pairs [B, C]) and the normalised (ResNet: + SiLU) input map of the product that
 * follows it ('<res>.a1', '<res>.a2', '<tr>.gx').  Tensor names follow the module walk
 * ("down.0.res.1.conv1.w", "up.2.tr.0.k", "mid.res.0.gn1.mean", "eps", ...);
 * '<tr>.v' entries hold V TRANSPOSED [B, C, H*W]. */
int fise_unet_num_tensors(const fise_unet* u, int kind);
int fise_unet_tensor_info(const fise_unet* u, int kind, int i, char* name /* host, >= 64 bytes */,
                          int64_t* offset /* host */, int64_t* numel /* host */);
int64_t fise_unet_weight_elems(const fise_unet* u);
size_t fise_unet_cache_bytes(const fise_unet* u);
size_t fise_unet_ctxkv_bytes(const fise_unet* u);
size_t fise_unet_workspace_bytes(const fise_unet* u, int max_active_tiles, int base_tile);

/* Recomputes every derived tensor of `cache` (kind 3 above) from its stored maps and
 * statistics: needed after stored tensors were written into the buffer by anything
 * other than this library's own steps (a FRESH pass and every masked step keep them
 * up to date by themselves).  workspace: fise_unet_refresh_derived_workspace_bytes(u). */
size_t fise_unet_refresh_derived_workspace_bytes(const fise_unet* u);
int fise_unet_refresh_derived(const fise_unet* u, const void* weights, void* cache, void* workspace,
                              size_t workspace_bytes, void* stream);

/* ------------------------------------------------------------------------
 * Moving a per-step cache between memories (section "Cache-based editing
 * pipeline": the cached activations of every denoising step are kept between
 * edits and moved between GPU and CPU memory by transfers that overlap the
 * computation).  A masked step touches little of a cache: it READS the stored
 * maps at the active tiles and the one-pixel ring around them, the K / V^T
 * caches of the attention layers in full, and the statistics; it WRITES the
 * stored maps at the active tiles and K rows / V^T columns at the active tokens.
 * These calls move exactly that, so a cache that lives in pinned host memory
 * (or in another device buffer) passes through a device slot at a fraction of
 * its size per step.
 *
 * The cache buffer is laid out in contiguous groups (byte ranges below):
 *   [maps_off, +maps_bytes)          stored maps (bf16 [B, H_l, W_l, C])
 *   [kv_off, +kv_bytes)              K [B, H_l*W_l, C] and V^T [B, C, H_l*W_l] of every transformer block
 *   [small_off, +small_bytes)        GroupNorm statistics, then the scale / shift tables
 *   [derived_maps_off, +derived_maps_bytes)   normalised copies of maps (derived)
 * stored_bytes = end of the statistics = everything the method stores.  The kv
 * and small ranges are moved by the caller with plain copies (hipMemcpyAsync).
 *
 * fise_unet_cache_move_active copies, from `src` to `dst` (both laid out as a
 * cache buffer; the same byte offsets are read and written), the pixels
 *   halo = 0: inside the active tiles,  halo = 1: those and the ring of one pixel
 * around them (clipped to the map; a pixel is moved once even where rings overlap),
 * each at its own level's resolution, of the tensor groups named in `what`:
 *   FISE_MOVE_MAPS  rows of the stored maps,  FISE_MOVE_K  rows of every K cache,
 *   FISE_MOVE_VT  columns of every V^T cache.
 * Fetch before a masked step: MAPS with halo 1 (+ plain copies of kv and small);
 * write-back after it: MAPS | K | VT with halo 0.  A slot filled this way holds no
 * valid derived maps: run the step with fise_masked_unet_modules over all modules,
 * which recomputes them where it reads them.
 * src and dst must be memory the GPU can address: device memory, or host memory
 * allocated pinned by the HIP runtime (hipHostMalloc); anything else is refused
 * (FISE_ERR_ALIGN) before a launch.  They must not overlap.  workspace (device):
 * fise_unet_cache_move_workspace_bytes(u).  n_active == 0 moves nothing.
 * Enqueued on `stream`; no allocation, no synchronisation. */
typedef struct {
    int64_t maps_off, maps_bytes, kv_off, kv_bytes, small_off, small_bytes, derived_maps_off, derived_maps_bytes;
    int64_t stored_bytes;
} fise_unet_cache_layout;
enum { FISE_MOVE_MAPS = 1, FISE_MOVE_K = 2, FISE_MOVE_VT = 4 };
int fise_unet_cache_layout_get(const fise_unet* u, fise_unet_cache_layout* out /* host */);
size_t fise_unet_cache_move_workspace_bytes(const fise_unet* u);
int fise_unet_cache_move_active(const fise_unet* u, const void* src, void* dst, const int32_t* tile_idx, int n_active,
                                int base_tile, int halo, int what, void* workspace, size_t workspace_bytes, void* stream);

/* The same move done by the copy engines instead of kernels: whole pixel rows.  tile_rows
 * (HOST int32 pairs [first, last) of rows of the base tile grid, ascending, disjoint)
 * names the tile rows that hold active tiles; for every stored map (FISE_MOVE_MAPS) and
 * every K cache (FISE_MOVE_K) the pixel rows of those tile rows at the tensor's own
 * level - plus one row above and below with halo = 1 - are copied in full width, one
 * hipMemcpyAsync per (tensor, batch element, run of rows).  A superset of what
 * fise_unet_cache_move_active moves (full rows instead of tiles), for transfers that
 * must overlap a running step: no kernel is launched.  src / dst: any memory
 * hipMemcpyAsync accepts (pinned host memory for a copy that is really asynchronous). */
int fise_unet_cache_move_tile_rows(const fise_unet* u, const void* src, void* dst, const int32_t* tile_rows /* host */,
                                   int n_ranges, int base_tile, int halo, int what, void* stream);

/* Context K/V of every transformer block for one conditioning ctx[B,n_ctx,ctx_dim]. */
int fise_unet_context_kv(const fise_unet* u, const void* weights, const void* ctx, void* ctxkv,
                         void* workspace, size_t workspace_bytes, void* stream);

typedef enum { FISE_STATS_CACHED = 0, FISE_STATS_FRESH = 1 } fise_stats_mode;

/* One masked evaluation: every ResNet / transformer / resample block is
 * recomputed at the active tiles and scattered into `cache` (in place); the
 * predicted noise is the cache tensor "eps" [B,H,W,out_ch].
 *   latent [B,H,W,in_ch] bf16 (the updated input), t_sin [B, base] float
 *   (sinusoidal time embedding), ctxkv from fise_unet_context_kv (new
 *   conditioning), tile_idx/n_active on the finest level with tile edge
 *   base_tile (divisible by 2^(n_levels-1); level l uses base_tile >> l on the
 *   same tile grid).  stats_mode CACHED uses the statistics stored in `cache`;
 *   FRESH recomputes them from the updated maps and stores them.  CACHED relies on
 *   the derived tensors of `cache` being consistent with its stored ones (see
 *   fise_unet_refresh_derived): each launch that rewrites a map at the active pixels
 *   also rewrites, there, the normalised copies its consumers read, so no launch of
 *   the step is spent on normalisation alone.
 *   level_dense (host int[n_levels], may be NULL): non-zero runs that level
 *   with the full tile list.  A dense forward is n_active = all tiles + FRESH. */
int fise_masked_unet_step(const fise_unet* u, const void* weights, void* cache, const void* latent,
                          const float* t_sin, const void* ctxkv, const int32_t* tile_idx, int n_active,
                          int base_tile, int stats_mode, const int* level_dense /* host */,
                          void* workspace, size_t workspace_bytes, void* stream);

/* The same step restricted to modules [first_module, first_module + n_modules) of the
 * walk (conv_in, ResNet / transformer blocks, resamplers, output conv, in execution
 * order); the time-embedding projections are always recomputed.  Module i reads its
 * input maps from `cache` as they stand.  Used to check or time one module at a time. */
int fise_unet_num_modules(const fise_unet* u);
int fise_unet_module_name(const fise_unet* u, int i, char* name /* host, >= 64 bytes */);
int fise_masked_unet_modules(const fise_unet* u, const void* weights, void* cache, const void* latent,
                             const float* t_sin, const void* ctxkv, const int32_t* tile_idx, int n_active,
                             int base_tile, int stats_mode, const int* level_dense /* host */,
                             int first_module, int n_modules,
                             void* workspace, size_t workspace_bytes, void* stream);

/* The keys-restricted reading of the same sub-layer (section "Approximate
 * Attention": computing with the non-zero regions only, read as restricting
 * the keys too): each active query attends to the keys and values of the ACTIVE
 * tokens of its batch element only.  No K/V cache is read or written; cost is
 * O(M_a^2) instead of O(M_a * H*W).  y = x + Attn(LayerNorm(x)) Wo^T + bo at
 * active tokens, scattered into y_cache; everything else as fise_masked_attention
 * (device pointers, bf16, caller-owned workspace of the stated size, n_active == 0
 * touches nothing, validation errors before any launch). */
size_t fise_masked_attention_restricted_workspace_bytes(int B, int C, int n_active, int tile);
int fise_masked_attention_restricted(const void* x, const void* ln_gamma, const void* ln_beta, const void* Wq, const void* Wk,
                                     const void* Wv, const void* Wo, const void* bo, int dtype, int B, int H, int W, int C,
                                     int heads, const int32_t* tile_idx, int n_active, int tile, void* y_cache,
                                     void* workspace, size_t workspace_bytes, void* stream);

/* ------------------------------------------------------------------------
 * Tracing.  With profiling enabled every launch of the gathered-GEMM and
 * attention kernels is bracketed by two HIP events on the caller's stream
 * (host objects; no device memory).  fise_profile_read(kind, ...) waits for the
 * events and returns the summed event time (ms), algorithmic FLOPs and bytes
 * and the number of launches recorded for `kind`:
 *   0 gathered GEMM, 64x64 tiles        1 gathered GEMM with the GEGLU epilogue
 *   2 attention (main kernel)           3 gathered GEMM, 128x128 tiles
 *   4 split-K reduce launches           5 gathered GEMM, 32x128 tiles (<= 32 rows)
 *   6 gathered GEMM with the GroupNorm prologue / 32-wide K steps
 *   7 attention merge launches          8 empty brackets (fise_profile_calibrate)
 *   9 wave-split GEMM (per-token products, K split inside the workgroup)
 * kind = -1 clears the log.  fise_profile_calibrate records n brackets with no
 * launch inside on `stream`: their average is what a bracket itself adds to every
 * figure above.  All pointers host.  Not thread safe.
 * ------------------------------------------------------------------------ */
int fise_profile_enable(int on);
int fise_profile_calibrate(int n, void* stream);
int fise_profile_read(int kind, double* total_ms, double* total_flops, double* total_bytes, int* launches);

/* Empirical ceilings of the current device, for the benchmark's roofline: the rate
 * of a plain streaming copy inside `scratch` (first half -> second half; bytes read +
 * bytes written per second, GB/s) and the rate of a register-resident bf16 MFMA loop
 * with no memory traffic (TFLOP/s).  Best of five timed passes each, after two
 * untimed ones.  scratch: device, 16-byte aligned, >= 64 MiB, overwritten (give well
 * over twice the 256 MB last-level cache to measure HBM and not that cache).  The two
 * results are host doubles.  WAITS for its own launches on `stream` (HIP events);
 * not to be called under graph capture. */
int fise_calibrate_peaks(void* scratch, size_t scratch_bytes, double* copy_gbs, double* mfma_bf16_tflops, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* FISE_H */
