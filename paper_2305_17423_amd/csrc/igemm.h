// Gathered implicit GEMM on bf16 MFMA: the one contraction kernel behind masked
// convolutions (3x3 / 1x1, stride 2, nearest-2x upsample, two concatenated
// sources) and the per-token linears of the transformer blocks.  Internal.
#pragma once
#include "common.h"

namespace fise {

enum { PRO_NONE = 0, PRO_GN = 1, PRO_GN_SILU = 2 };
enum { OUT_COMPACT = 0, OUT_MAP = 1, OUT_TOKENS_T = 2 };

struct IgemmArgs {
    // ---- A operand: rows = B * Ma active pixels (or compact rows) x K
    const bf16_t* a0; const bf16_t* a1; int C0, C1;    // map sources [B,Hin,Win,C*] (a1 unused when C1 == 0)
    int a_compact;                                      // 1: a0 is a compact [rows, C0] buffer (ksize must be 1)
    int Hin, Win, ksize, stride, ups;
    // ---- row geometry (output map)
    const int* tile_idx; int tile, tiles_w, Ho, Wo, B, Ma;
    // ---- prologue on A: GroupNorm (+SiLU) with given statistics
    int pro; const float* gn_mean; const float* gn_rstd; const bf16_t* gn_gamma; const bf16_t* gn_beta; int G;
    // ---- B operand: weights [rows_w, K], K innermost
    const bf16_t* w; int N; int K;                      // N = output columns (GEGLU: N = D, weights have 2D rows)
    int geglu;
    // ---- epilogue
    const bf16_t* bias; const float* temb; int temb_stride; const bf16_t* res; int res_compact;
    int nsect, sect_n;                                  // N = nsect * sect_n; section s goes to out[s]
    bf16_t* out[3]; int out_mode[3];
    // ---- split-K (splits == 1: none)
    int splits; float* partial; int* counters;
};

// Enqueue; rows == 0 is a no-op.  Returns a fise_status.
int launch_igemm(const IgemmArgs& a, hipStream_t st);
size_t igemm_workspace_bytes(int rows, int N, int K);
// LayerNorm of rows -> compact out[rows, C].  tile_idx == nullptr: `in` is compact [rows, C];
// otherwise `in` is a token map [B, H*W, C] and row r = (b, active pixel r % Ma).
int launch_ln_rows(const void* in, int rows, int C, const void* gamma, const void* beta, float eps, void* out,
                   const int* tile_idx, int tile, int tiles_w, int H, int W, int Ma, hipStream_t st);
int conv_dispatch(const fise_conv_args* a, void* workspace, size_t workspace_bytes, hipStream_t st);
// out[b, n] = act(bias[n] + sum_k in[b, k] * W[n, k]) for a handful of rows b (float in/out, bf16 weights).
int launch_small_linear(const float* in, int B, int K, const void* W, const void* bias, int N, int silu_out, float* out,
                        hipStream_t st);
int launch_iota(int* p, int n, hipStream_t st);
int launch_attention(const void* q, const void* K, const void* Vt, int B, int M, int n_keys, int n_stride, int C,
                     int heads, float scale, void* out, hipStream_t st);

}  // namespace fise
