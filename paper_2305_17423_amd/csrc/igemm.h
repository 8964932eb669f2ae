// Gathered implicit GEMM on bf16 MFMA: the one contraction kernel behind masked
// convolutions (3x3 / 1x1, stride 2, nearest-2x upsample, two concatenated
// sources) and the per-token linears of the transformer blocks.  Internal.
#pragma once
#include "common.h"

namespace fise {

enum { PRO_NONE = 0, PRO_GN = 1, PRO_GN_SILU = 2 };
enum { OUT_COMPACT = 0, OUT_MAP = 1, OUT_TOKENS_T = 2, OUT_COMPACT_F32 = 3 };

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
};

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
int conv_dispatch(const fise_conv_args* a, void* workspace, size_t workspace_bytes, hipStream_t st);
// out[b, n] = act(bias[n] + sum_k in[b, k] * W[n, k]) for a handful of rows b (float in/out, bf16 weights).
int launch_small_linear(const float* in, int B, int K, const void* W, const void* bias, int N, int silu_out, float* out,
                        hipStream_t st);
int launch_iota(int* p, int n, hipStream_t st);
// act[B,H,W,C0+C1] = GroupNorm(x0|x1) (+SiLU) with the given statistics at the active tiles and their one-pixel ring.
int launch_gn_act_halo(const void* x0, const void* x1, int C0, int C1, int B, int H, int W, const float* mean, const float* rstd,
                       const void* gamma, const void* beta, int G, int silu, const int* tile_idx, int n_active, int tile, void* act,
                       hipStream_t st);
// ws: scratch for the key-split partials (attention_workspace_bytes; null or too small = no key split)
size_t attention_workspace_bytes(int B, int M, int n_keys, int C, int heads);
int launch_attention(const void* q, const void* K, const void* Vt, int B, int M, int n_keys, int n_stride, int C,
                     int heads, float scale, void* out, void* ws, size_t ws_bytes, hipStream_t st);

}  // namespace fise
