// Gathered implicit GEMM on bf16 MFMA: the one contraction kernel behind masked
// convolutions (3x3 / 1x1, stride 2, nearest-2x upsample, two concatenated
// sources) and the per-token linears of the transformer blocks.  Internal.
#pragma once
#include "common.h"

namespace fise {

enum { PRO_NONE = 0, PRO_GN = 1, PRO_GN_SILU = 2 };
enum { OUT_COMPACT = 0, OUT_MAP = 1, OUT_TOKENS_T = 2, OUT_COMPACT_F32 = 3 };

// A second destination of a map-producing launch: the consumer's GroupNorm (+SiLU) of the value just stored,
//   dst[pix, c_off + col] = act(x * ss[b, c_off + col].x + ss[b, c_off + col].y),   x = the bf16 value stored at (pix, col)
// with ss the per-(batch element, channel) scale / shift table of that GroupNorm under its CACHED statistics.
// The consumer then reads activations instead of normalising its input in a launch of its own.
struct GnView { bf16_t* dst; const float2* ss; int dstC, c_off, silu, pad_; };

struct IgemmArgs {
    // ---- A operand: rows = B * Ma active pixels (or compact rows) x K
    const bf16_t* a0; const bf16_t* a1; int C0, C1;    // map sources [B,Hin,Win,C*] (a1 unused when C1 == 0)
    int a_compact;                                      // 1: a0 is a compact bf16 [rows, C0] buffer (ksize must be 1)
    int Hin, Win, ksize, stride, ups;
    // ---- row geometry (output map)
    const int* tile_idx; int tile, tile_w, tiles_w, Ho, Wo, B, Ma;   // tiles of tile x tile_w pixels (tile_w 0: square)
    // ---- prologue on A: GroupNorm (+SiLU) with given statistics
    int pro; const float* gn_mean; const float* gn_rstd; const bf16_t* gn_gamma; const bf16_t* gn_beta; int G;
    // ---- B operand: weights [rows_w, K], K innermost
    const bf16_t* w; int N; int K;                      // N = output columns (GEGLU: N = D, weights have 2D rows)
    int geglu;
    // ---- epilogue
    const bf16_t* bias; const float* temb; int temb_stride;
    const bf16_t* res; int res_compact;                 // 0: map at the output pixel, 1: compact bf16 rows, 2: compact float rows
    int nsect, sect_n;                                  // N = nsect * sect_n; section s goes to out[s]
    bf16_t* out[3]; int out_mode[3];
    bf16_t* mirror;                                     // OUT_COMPACT_F32 only: also store a bf16 copy here (may be null)
    // ---- optional LayerNorm of the finished rows (one OUT_COMPACT_F32 section, N = sect_n): ln_out[rows, N] bf16.
    // Fused into the split-K reduce launch where the shape allows, otherwise a separate launch.
    const bf16_t* ln_gamma; const bf16_t* ln_beta; float ln_eps; bf16_t* ln_out;
    // ---- optional side product accumulated into the same tile: 1x1 conv of the raw maps s0 | s1
    // [B,Ho,Wo,S*] at the output pixel with weights w2 [N, K2] and bias2 (K2 = S0 + S1, 0 = none)
    const bf16_t* s0; const bf16_t* s1; int S0, S1; const bf16_t* w2; const bf16_t* bias2; int K2;
    // ---- split-K (splits == 1: none)
    int splits; float* partial;
    int gx, gy;                                         // tile grid (row tiles, column tiles); set by the launcher
    int need_pix;                                       // set by the launcher: the epilogue addresses a map (else rows only)
    // ---- optional normalised copies of the output map for its consumers (one OUT_MAP section, N % 4 == 0)
    int nview; GnView view[2];
};

// What a block of the UNet step keeps in the per-step cache besides its stored maps (all derived from them and from
// the cached statistics): the activated input of its first product (ResNet: SiLU(GN1(x)); transformer: GN(x)), for a
// ResNet also conv2's activated input SiLU(GN2(h1)), the scale / shift tables of those GroupNorms, and the
// normalised copies other blocks want of this block's output.  trust: the derived maps are up to date with the
// stored maps except where this step's producers have just rewritten them (so consumers need not recompute them).
struct BlockDerived {
    void* act_in; void* act_mid; float2* ss_in; float2* ss_mid; int trust;
    GnView out_view[2]; int n_out_view;
};

#if defined(__HIPCC__)
// Four consecutive channels col .. col + 3 of pixel `pix` (batch element b): every view gets its activation.
// In two halves, so that an epilogue can request the table entries of all its items together with its other
// operands and use them later (loaded where they are used, each item pays a round trip of its own in front of
// its stores): view_ss_load fetches the four (scale, shift) pairs per view, put_views4 applies them.
struct ViewSS { float s[2][8]; };
__device__ __forceinline__ void view_ss_load(const GnView* view, int nview, int b, int col, ViewSS& o) {
    typedef float f32x4v __attribute__((ext_vector_type(4)));
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        f32x4v s01 = {0.f, 0.f, 0.f, 0.f}, s23 = s01;
        if (i < nview) {
            const GnView w = view[i];
            auto sp = (const __attribute__((address_space(1))) f32x4v*)(w.ss + (size_t)b * w.dstC + w.c_off + col);
            s01 = sp[0]; s23 = sp[1];
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) { o.s[i][q] = s01[q]; o.s[i][4 + q] = s23[q]; }
    }
}
__device__ __forceinline__ void put_views4(const GnView* view, int nview, unsigned pix, int col, const float (&v)[4], const ViewSS& ss) {
    typedef unsigned u32x2v __attribute__((ext_vector_type(2)));
    const unsigned p01 = f2bf2(v[0], v[1]), p23 = f2bf2(v[2], v[3]);      // the values as stored
    const float x[4] = {__uint_as_float(p01 << 16), __uint_as_float(p01 & 0xffff0000u), __uint_as_float(p23 << 16),
                        __uint_as_float(p23 & 0xffff0000u)};
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        if (i >= nview) break;
        const GnView w = view[i];
        float u[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) u[q] = fmaf(x[q], ss.s[i][2 * q], ss.s[i][2 * q + 1]);
        if (w.silu) {
#pragma unroll
            for (int q = 0; q < 4; ++q) u[q] = silu_f(u[q]);
        }
        auto dp = (__attribute__((address_space(1))) u32x2v*)(w.dst + (size_t)pix * w.dstC + w.c_off + col);
        *dp = u32x2v{f2bf2(u[0], u[1]), f2bf2(u[2], u[3])};
    }
}
__device__ __forceinline__ void put_views4(const GnView* view, int nview, int b, unsigned pix, int col, const float (&v)[4]) {
    ViewSS ss;
    view_ss_load(view, nview, b, col, ss);
    put_views4(view, nview, pix, col, v, ss);
}
// One channel (the element-wise epilogue of the register-staged kernel).
__device__ __forceinline__ void put_views1(const GnView* view, int nview, int b, size_t pix, int col, float v) {
    const float x = bf2f(f2bf(v));
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        if (i >= nview) break;
        const GnView w = view[i];
        const float2 s = w.ss[(size_t)b * w.dstC + w.c_off + col];
        float u = fmaf(x, s.x, s.y);
        if (w.silu) u = silu_f(u);
        w.dst[pix * w.dstC + w.c_off + col] = f2bf(u);
    }
}
#endif

// Scratch of the launcher: GroupNorm (scale, shift) table and the parked partial sums of split-K launches.
constexpr size_t IGEMM_PARTIAL_BYTES = 32u << 20;
struct IgemmWorkspace { float* partial; size_t partial_bytes; };
size_t igemm_workspace_bytes();
// Carves the scratch out of `workspace`; with a null or too
// small workspace `out` is left empty and every launch runs unsplit.
int igemm_workspace_init(void* workspace, size_t bytes, IgemmWorkspace* out, hipStream_t st);
// Enqueue; rows == 0 is a no-op.  `ws` may be null (no split-K).  Returns a fise_status.
int launch_igemm(const IgemmArgs& a, const IgemmWorkspace* ws, hipStream_t st);
// LayerNorm of rows -> compact out[rows, C].  tile_idx == nullptr: `in` is compact [rows, C];
// otherwise `in` is a token map [B, H*W, C] and row r = (b, active pixel r % Ma).
// in_f32 != 0: compact float rows (tile_idx must be nullptr).
int launch_ln_rows(const void* in, int in_f32, int rows, int C, const void* gamma, const void* beta, float eps, void* out,
                   const int* tile_idx, int tile, int tiles_w, int H, int W, int Ma, hipStream_t st);
// views / nview: normalised copies of the output map for its consumers (nullptr / 0 = none)
int conv_dispatch(const fise_conv_args* a, void* workspace, size_t workspace_bytes, hipStream_t st, const GnView* views, int nview);
// out[b, n] = act(bias[n] + sum_k in[b, k] * W[n, k]) for a handful of rows b (float in/out, bf16 weights).
int launch_small_linear(const float* in, int B, int K, const void* W, const void* bias, int N, int silu_out, float* out,
                        hipStream_t st);
int launch_iota(int* p, int n, hipStream_t st);
// ss[B, C] = (rstd * gamma, beta - mean * rstd * gamma): the scale / shift form of a GroupNorm with given statistics.
int launch_gn_scale_shift(const float* mean, const float* rstd, const void* gamma, const void* beta, int B, int C, int G, float2* ss,
                          hipStream_t st);
// mean / rstd [B, G] of the bf16 map x0 | x1 and the scale / shift table built from them (workspace as for
// fise_groupnorm_stats).
int launch_gn_stats_table(const void* x0, const void* x1, int B, int H, int W, int C0, int C1, int G, float eps, float* mean, float* rstd,
                          const void* gamma, const void* beta, float2* ss, void* workspace, hipStream_t st);
// act[B,H,W,C0+C1] = GroupNorm(x0|x1) (+SiLU) with the given statistics at the active tiles and their one-pixel ring.
int launch_gn_act_halo(const void* x0, const void* x1, int C0, int C1, int B, int H, int W, const float* mean, const float* rstd,
                       const void* gamma, const void* beta, int G, int silu, const int* tile_idx, int n_active, int tile, void* act,
                       hipStream_t st);
// ws: scratch for the key-split partials (attention_workspace_bytes; null or too small = no key split)
size_t attention_workspace_bytes(int B, int M, int n_keys, int C, int heads);
int launch_attention(const void* q, const void* K, const void* Vt, int B, int M, int n_keys, int n_stride, int C,
                     int heads, float scale, void* out, void* ws, size_t ws_bytes, hipStream_t st);

}  // namespace fise
