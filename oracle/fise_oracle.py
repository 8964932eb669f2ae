"""CPU oracle for the masked (cache-enabled sparse) UNet step of FISEdit.

TEST INFRASTRUCTURE ONLY.  Only tests/, __graft_entry__.smoke() and bench.py's
cpu_baseline leg may import this module.  It shares no code with the HIP path
and never imports it.  Everything is plain numpy in float64; tensors that the
method stores (cached feature maps, K/V caches) are rounded to the storage
dtype exactly where they are stored and, by default, nowhere else.  (An
optional mode, `scratch` / `act_dtype` / `p_dtype` = 'bf16', also rounds the
operands that pass from one product to the next without being stored: the
model of any implementation whose matrix units take bf16 operands.)

What each function follows (FISEdit, arxiv 2305.17423):
  * mask_detect ............. section "Fine-Grained Mask Generation", the
                              |X - Y| difference and the {diff >= eps} set of
                              its equation block (single pair, threshold given)
  * otsu_threshold_exact .... same equation block: argmax of the OTSU(eps)
                              objective over eps in [0, 1] (every distinct
                              partition of the values is tried)
  * otsu_threshold .......... the same objective on the grid eps = k/256
  * accumulate_diff,
    normalize_minmax ........ same equation block: the sum over steps of
                              |X_t - Y_t| and Normalize(.)
  * tiles_from_pixels ....... section "Adaptive Pixel-Wise Sparse Convolution":
                              the set of blocks gathered under a mask m
  * apsc_block_size ......... same section, the argmin over {2,4,8,16,32}^2
  * gn_stats / masked_gn_silu section "Approximate Normalization" (cached
                              mean / variance reused at masked positions)
  * masked_conv ............. section "Adaptive Pixel-Wise Sparse Convolution"
                              (tiled sparse convolution: gather, convolve,
                              scatter into the cached map)
  * attention_active,
    masked_self_attention ... section "Approximate Attention" (masked tokens
                              are gathered before self- and cross-attention)
  * resnet_block, transformer_block, unet_step
                              section "Sparse Computation": the U-Net is a
                              stack of ResNet and attention modules, each
                              recomputed only inside the mask, the rest reused
                              from the cache of the previous generation.

Layout: feature maps are [B, H, W, C] (channels innermost); token tensors are
[B, H*W, C] with token = y*W + x; conv weights [C_out, k, k, C_in]; linear
weights [out, in].  A tile list `idx` holds ascending row-major ids of active
tiles on the (H/tile) x (W/tile) tile grid.  Active pixels are enumerated tile
by tile in list order, row-major inside a tile.

Readings of points the paper leaves open are listed in the repository's design
document; the ones that matter here: strict '>' against a given threshold, mean
over batch and channels in float32 in a fixed sequential order, a tile is active
iff any of its pixels is, active queries attend to all keys of the updated K/V
cache, no mask dilation, statistics cached from the previous generation.
"""
from __future__ import annotations

import math

import numpy as np

F64 = np.float64


# ----------------------------------------------------------------------------
# storage rounding
# ----------------------------------------------------------------------------
def round_store(a, dtype: str) -> np.ndarray:
    """Value of `a` after being stored as `dtype` ('f64' | 'f32' | 'bf16'), as float64.

    bf16 keeps 8 significant bits; rounding is to nearest, ties to even, done
    once from float64 (np.rint is ties-to-even on the scaled significand).
    """
    a = np.asarray(a, F64)
    if dtype == "f64":                          # not stored: no rounding
        return a
    if dtype == "f32":
        return a.astype(np.float32).astype(F64)
    if dtype == "bf16":
        m, e = np.frexp(a)                      # a = m * 2**e, 0.5 <= |m| < 1
        return np.ldexp(np.rint(m * 256.0) / 256.0, e)
    raise ValueError(dtype)


# ----------------------------------------------------------------------------
# masks, tiles, index lists
# ----------------------------------------------------------------------------
def pixel_diff(cached: np.ndarray, fresh: np.ndarray) -> np.ndarray:
    """d[y,x] = mean over (b, c) of |fresh - cached|, in float32.

    The sum runs sequentially, b outermost then c ascending, each step
    s <- s + |f - c| rounded to float32; the final divide by float32(B*C) is a
    float32 divide.  (Order and precision are part of the contract because the
    result decides a bit.)
    """
    c32 = np.asarray(cached, np.float32)
    f32 = np.asarray(fresh, np.float32)
    B, H, W, C = c32.shape
    s = np.zeros((H, W), np.float32)
    for b in range(B):
        for c in range(C):
            s = s + np.abs(f32[b, :, :, c] - c32[b, :, :, c])
    return s / np.float32(B * C)


def tile_hw(tile):
    """A tile is a square edge (int) or a rectangular block (h, w), the shapes
    the adaptive block-size selection chooses among."""
    if isinstance(tile, (tuple, list)):
        return int(tile[0]), int(tile[1])
    return int(tile), int(tile)


def tiles_from_pixels(pix: np.ndarray, tile):
    """Pixel mask -> (tile mask, ascending tile index list).  A tile is active
    iff any pixel inside it is."""
    H, W = pix.shape
    bh, bw = tile_hw(tile)
    if H % bh or W % bw:
        raise ValueError("H, W must be multiples of tile")
    th, tw = H // bh, W // bw
    tmask = pix.reshape(th, bh, tw, bw).astype(bool).any(axis=(1, 3))
    idx = np.flatnonzero(tmask.reshape(-1)).astype(np.int32)
    return tmask.astype(np.uint8), idx


def mask_detect(cached, fresh, threshold: float, tile: int):
    """(pixel mask, tile mask, tile index list) of the region whose mean
    absolute difference exceeds `threshold` (strictly)."""
    d = pixel_diff(cached, fresh)
    pix = (d > np.float32(threshold)).astype(np.uint8)
    tmask, idx = tiles_from_pixels(pix, tile)
    return pix, tmask, idx


def mask_downsample(tmask: np.ndarray) -> np.ndarray:
    """2x2 OR-pool of a mask (pixel or tile): the mask of the next coarser
    level is set wherever any of its four children is."""
    H, W = tmask.shape
    return tmask.reshape(H // 2, 2, W // 2, 2).astype(bool).any(axis=(1, 3)).astype(np.uint8)


def active_pixels(idx, tile, W: int):
    """Coordinates (ys, xs) of the active pixels of a W-wide map, tile by tile
    in list order, row-major inside each tile."""
    idx = np.asarray(idx, np.int64)
    bh, bw = tile_hw(tile)
    tw = W // bw
    ty, tx = idx // tw, idx % tw
    oy, ox = np.divmod(np.arange(bh * bw), bw)
    ys = (ty[:, None] * bh + oy[None, :]).reshape(-1)
    xs = (tx[:, None] * bw + ox[None, :]).reshape(-1)
    return ys, xs


def full_index(H: int, W: int, tile) -> np.ndarray:
    bh, bw = tile_hw(tile)
    return np.arange((H // bh) * (W // bw), dtype=np.int32)


def normalize_minmax(a: np.ndarray) -> np.ndarray:
    """Normalize(.) of the mask-generation equation, read as min-max scaling of
    the map to [0, 1] (the threshold is searched in [0, 1])."""
    a = np.asarray(a, F64)
    lo, hi = a.min(), a.max()
    if hi == lo:
        return np.zeros_like(a)
    return (a - lo) / (hi - lo)


def accumulate_diff(cached_steps, fresh_steps) -> np.ndarray:
    """sum over steps t of the per-pixel |X_t - Y_t| (channel/batch mean)."""
    acc = None
    for X, Y in zip(cached_steps, fresh_steps):
        d = np.abs(np.asarray(Y, F64) - np.asarray(X, F64)).mean(axis=(0, 3))
        acc = d if acc is None else acc + d
    return acc


def otsu_objective(diff: np.ndarray, eps: float) -> float:
    """OTSU(eps) = N1 N2 / (N1+N2)^2 * (mean_A - mean_B)^2 with
    A = {diff < eps}, B = {diff >= eps}; 0 when either class is empty."""
    v = np.asarray(diff, F64).reshape(-1)
    A, Bs = v[v < eps], v[v >= eps]
    n1, n2 = A.size, Bs.size
    if n1 == 0 or n2 == 0:
        return 0.0
    return n1 * n2 / float(n1 + n2) ** 2 * (A.mean() - Bs.mean()) ** 2


def otsu_threshold(diff: np.ndarray, bins: int = 256):
    """argmax of OTSU(eps) over the grid eps = k / bins, k = 0..bins (the
    domain [0,1] sampled uniformly; first maximiser wins).  Returns
    (eps, mask = diff >= eps)."""
    best, best_eps = -1.0, 0.0
    for k in range(bins + 1):
        eps = k / bins
        o = otsu_objective(diff, eps)
        if o > best:
            best, best_eps = o, eps
    return best_eps, (np.asarray(diff, F64) >= best_eps).astype(np.uint8)


def otsu_threshold_exact(diff: np.ndarray):
    """argmax over eps in [0, 1] of OTSU(eps) (the paper's definition, no grid).

    The objective only changes when eps crosses a value of `diff`: with the
    distinct values v_0 < v_1 < ... every eps in (v_i, v_{i+1}] gives the same
    classes A = {diff <= v_i}, B = {diff >= v_{i+1}}, so trying one eps per
    interval tries every partition the definition can produce.  The first
    maximising interval wins (as the grid search takes its first maximiser).
    Returns (lo, hi, mask): any eps in (lo, hi] is an exact maximiser, and
    mask = diff >= hi is the unique mask they all give.  A constant map has no
    two classes: (0, 0, all ones), the value every eps <= min gives."""
    a = np.asarray(diff, F64)
    v = np.unique(a.reshape(-1))
    if v.size < 2:
        return 0.0, 0.0, np.ones(a.shape, np.uint8)
    best, lo, hi = -1.0, 0.0, 0.0
    for i in range(v.size - 1):
        o = otsu_objective(a, v[i + 1])         # eps = v_{i+1}: A = {diff <= v_i}
        if o > best:
            best, lo, hi = o, float(v[i]), float(v[i + 1])
    return lo, hi, (a >= hi).astype(np.uint8)


def otsu_grid_is_exact(diff: np.ndarray, bins: int = 256) -> bool:
    """True when the grid search must return the exact mask: some grid point k/bins
    lies in the exact maximiser's interval (lo, hi] and no grid point before it does
    better (the grid's objective values are a subset of the exact search's, so the
    first grid point inside the winning interval is the grid's first maximiser
    unless an earlier interval ties)."""
    lo, hi, _ = otsu_threshold_exact(diff)
    k = math.floor(lo * bins) + 1               # first grid point strictly above lo
    return k / bins <= hi


def apsc_cost(pix: np.ndarray, h: int, w: int, hk: int = 3, wk: int = 3, as_written: bool = False):
    """Cost of splitting into (h, w) blocks under pixel mask `pix`.

    N = number of (h, w) blocks holding at least one masked pixel.  As printed
    the per-block factor is (h-hk+1)(w-wk+1); read with (h, w) as the *output*
    block it is the gathered input patch (h+hk-1)(w+wk-1).  Both are offered.
    """
    H, W = pix.shape
    if H % h or W % w:
        return None
    n = int(pix.reshape(H // h, h, W // w, w).astype(bool).any(axis=(1, 3)).sum())
    if as_written:
        return (h - hk + 1) * (w - wk + 1) * n
    return (h + hk - 1) * (w + wk - 1) * n


def apsc_block_size(pix: np.ndarray, hk: int = 3, wk: int = 3, as_written: bool = False):
    """argmin over h, w in {2,4,8,16,32} of apsc_cost (first minimiser in
    row-major (h, w) order; block sizes that do not divide the map are
    skipped; as written, non-positive factors are skipped too)."""
    best = None
    for h in (2, 4, 8, 16, 32):
        for w in (2, 4, 8, 16, 32):
            c = apsc_cost(pix, h, w, hk, wk, as_written)
            if c is None:
                continue
            if as_written and ((h - hk + 1) <= 0 or (w - wk + 1) <= 0):
                continue
            if best is None or c < best[0]:
                best = (c, h, w)
    return best[1], best[2], best[0]


# ----------------------------------------------------------------------------
# normalisation
# ----------------------------------------------------------------------------
def _cat_sources(xs):
    """A list of maps stands for their channel concatenation (skip links)."""
    if isinstance(xs, (list, tuple)):
        return xs[0] if len(xs) == 1 else np.concatenate(xs, axis=-1)
    return xs


def gn_stats(x, groups: int, eps: float):
    """Per (batch, group) mean and 1/sqrt(biased variance + eps) over H, W and
    the group's channels; both kept as float32 values (they are cached)."""
    x = np.asarray(_cat_sources(x), F64)
    B, H, W, C = x.shape
    g = x.reshape(B, H * W, groups, C // groups)
    mean = g.mean(axis=(1, 3))
    var = ((g - mean[:, None, :, None]) ** 2).mean(axis=(1, 3))
    rstd = 1.0 / np.sqrt(var + eps)
    return round_store(mean, "f32"), round_store(rstd, "f32")


def _gn_silu(v, b, mean, rstd, gamma, beta, groups):
    """GroupNorm with given statistics, then SiLU, on rows v[n, C] of batch b."""
    C = v.shape[-1]
    gi = np.arange(C) // (C // groups)
    u = (v - mean[b][gi]) * rstd[b][gi] * gamma + beta
    return u / (1.0 + np.exp(-u))


def masked_gn_silu(x, mean, rstd, gamma, beta, groups, idx, tile, y_cache, dtype):
    """y = SiLU(GroupNorm(x)) at active pixels using the *given* statistics;
    every other position of y_cache is left as it is (in place)."""
    x = np.asarray(x, F64)
    B, H, W, C = x.shape
    ys, xs = active_pixels(idx, tile, W)
    for b in range(B):
        y_cache[b, ys, xs, :] = round_store(
            _gn_silu(x[b, ys, xs, :], b, mean, rstd, np.asarray(gamma, F64), np.asarray(beta, F64), groups), dtype)
    return y_cache


def layernorm(a, gamma, beta, eps: float = 1e-5):
    """Per-token LayerNorm over the last axis (biased variance)."""
    a = np.asarray(a, F64)
    mu = a.mean(axis=-1, keepdims=True)
    var = ((a - mu) ** 2).mean(axis=-1, keepdims=True)
    return (a - mu) / np.sqrt(var + eps) * gamma + beta


_erf = np.vectorize(math.erf, otypes=[F64])


def gelu(a):
    """Exact GELU: a * Phi(a)."""
    a = np.asarray(a, F64)
    return 0.5 * a * (1.0 + _erf(a / math.sqrt(2.0)))


def geglu(g):
    """First half of the channels times GELU of the second half."""
    D = g.shape[-1] // 2
    return g[..., :D] * gelu(g[..., D:])


# ----------------------------------------------------------------------------
# masked convolution
# ----------------------------------------------------------------------------
def masked_conv(xs, w, bias, idx, tile, y_cache, dtype, stride: int = 1, upsample: bool = False,
                gn=None, temb=None, residual=None, act_dtype: str = "f64"):
    """Convolution (k x k, zero padding k//2) evaluated only at the active
    pixels of the *output* map; results are written into y_cache in place,
    all other positions keep their cached value.

      y[b,p,co] = bias[co] + sum_{ky,kx,ci} w[co,ky,kx,ci] * xin[b, q(p,ky,kx), ci]
                  (+ temb[b,co]) (+ residual[b,p,co])

    xin is the input map as it stands (so taps that fall outside the active
    tiles read cached neighbours), optionally passed through GroupNorm+SiLU
    with the given statistics gn = dict(mean, rstd, gamma, beta, groups); taps
    outside the image contribute zero.  `xs` may be a list of maps standing for
    their channel concatenation.  stride 2: q = 2p + (ky,kx) - pad.  upsample:
    the input is first enlarged 2x by nearest neighbour (q = (p + (ky,kx) -
    pad) >> 1, zero outside the enlarged image).  `tile` is the tile edge on
    the output map.  act_dtype: precision in which the normalised + activated
    input is held before it is multiplied ('f64' = not rounded; 'bf16' models an
    implementation that materialises it as a bf16 operand, see `scratch` in the
    composite oracle).
    """
    x = np.asarray(_cat_sources(xs), F64)
    w = np.asarray(w, F64)
    B, Hi, Wi, Ci = x.shape
    Co, k = w.shape[0], w.shape[1]
    pad = k // 2
    if upsample:
        Ho, Wo = 2 * Hi, 2 * Wi
    else:
        Ho, Wo = Hi // stride, Wi // stride
    assert y_cache.shape == (B, Ho, Wo, Co), (y_cache.shape, (B, Ho, Wo, Co))
    ys, xc = active_pixels(idx, tile, Wo)
    if ys.size == 0:
        return y_cache
    for b in range(B):
        acc = np.zeros((ys.size, Co), F64)
        for ky in range(k):
            for kx in range(k):
                if upsample:
                    uy, ux = ys + ky - pad, xc + kx - pad
                    ok = (uy >= 0) & (uy < Ho) & (ux >= 0) & (ux < Wo)
                    iy, ix = uy >> 1, ux >> 1
                else:
                    iy, ix = ys * stride + ky - pad, xc * stride + kx - pad
                    ok = (iy >= 0) & (iy < Hi) & (ix >= 0) & (ix < Wi)
                v = x[b, np.clip(iy, 0, Hi - 1), np.clip(ix, 0, Wi - 1), :]
                if gn is not None:
                    v = round_store(_gn_silu(v, b, gn["mean"], gn["rstd"], np.asarray(gn["gamma"], F64),
                                             np.asarray(gn["beta"], F64), gn["groups"]), act_dtype)
                v = v * ok[:, None]
                acc += v @ w[:, ky, kx, :].T
        if bias is not None:
            acc += np.asarray(bias, F64)
        if temb is not None:
            acc += np.asarray(temb, F64)[b]
        if residual is not None:
            acc += np.asarray(residual, F64)[b, ys, xc, :]
        y_cache[b, ys, xc, :] = round_store(acc, dtype)
    return y_cache


def linear(a, w, bias=None):
    """Per-token linear map: a[..., in] @ w[out, in]^T + bias."""
    y = np.asarray(a, F64) @ np.asarray(w, F64).T
    if bias is not None:
        y = y + np.asarray(bias, F64)
    return y


# ----------------------------------------------------------------------------
# attention
# ----------------------------------------------------------------------------
def attention_active(q, K, V, heads: int, p_dtype: str = "f64"):
    """O[b,m,:] = softmax_k(q[b,m,h] . K[b,k,h] / sqrt(d)) V[b,k,h] for each
    head h (channels [h*d, (h+1)*d)), over *all* keys k.  p_dtype 'bf16' rounds
    the unnormalised weights exp(s - max) before they multiply V (the
    normalising sum stays unrounded): a bf16 P.V product."""
    q, K, V = (np.asarray(t, F64) for t in (q, K, V))
    B, M, C = q.shape
    d = C // heads
    out = np.zeros((B, M, C), F64)
    for b in range(B):
        for h in range(heads):
            sl = slice(h * d, (h + 1) * d)
            s = (q[b, :, sl] @ K[b, :, sl].T) / math.sqrt(d)
            s = s - s.max(axis=1, keepdims=True)
            p = np.exp(s)
            out[b, :, sl] = (round_store(p, p_dtype) @ V[b, :, sl]) / p.sum(axis=1, keepdims=True)
    return out


def token_ids(idx, tile, W):
    ys, xs = active_pixels(idx, tile, W)
    return ys * W + xs


def masked_self_attention(n_act, wq, wk, wv, heads, K_cache, V_cache, tok, dtype, scratch: str = "f64"):
    """Self-attention for active tokens: their K, V rows are refreshed in the
    caches (stored, hence rounded), then each active query attends to every
    key of the updated caches.  n_act[B, M, C] are the (already normalised)
    active tokens; tok their token ids.  Returns O[B, M, C] (heads merged)."""
    q = round_store(linear(n_act, wq), scratch)
    K_cache[:, tok, :] = round_store(linear(n_act, wk), dtype)
    V_cache[:, tok, :] = round_store(linear(n_act, wv), dtype)
    return attention_active(q, K_cache, V_cache, heads, scratch)


def masked_attention_block(x_map, ln_g, ln_b, wq, wk, wv, wo, bo, heads, K_cache, V_cache,
                           K_ctx, V_ctx, idx, tile, y_cache, dtype):
    """One attention sub-layer on a token map x_map[B,H,W,C]:
    y = x + (Attn(LN(x)) Wo^T + bo) at active tokens, scattered into y_cache.
    With K_cache/V_cache given it is self-attention (caches refreshed at the
    active tokens); with them None, cross-attention against K_ctx/V_ctx."""
    B, H, W, C = x_map.shape
    ys, xs = active_pixels(idx, tile, W)
    if ys.size == 0:
        return y_cache
    xa = np.asarray(x_map, F64)[:, ys, xs, :]
    n = layernorm(xa, np.asarray(ln_g, F64), np.asarray(ln_b, F64))
    if K_cache is not None:
        o = masked_self_attention(n, wq, wk, wv, heads, K_cache, V_cache, ys * W + xs, dtype)
    else:
        o = attention_active(linear(n, wq), K_ctx, V_ctx, heads)
    y_cache[:, ys, xs, :] = round_store(xa + linear(o, wo, bo), dtype)
    return y_cache


def masked_attention_restricted(x_map, ln_g, ln_b, wq, wk, wv, wo, bo, heads, idx, tile, y_cache, dtype):
    """The keys-restricted reading of Approximate Attention ("only calculate the
    results using non-zero regions"): active queries attend to the keys and
    values of the *active* tokens only; nothing outside the mask is read, so no
    K/V cache is involved.  y = x + (Attn(LN(x)) Wo^T + bo) at active tokens,
    scattered into y_cache.  K and V of the active tokens are stored tensors
    (rounded to the storage dtype) before the products, as in the cached form."""
    B, H, W, C = x_map.shape
    ys, xs = active_pixels(idx, tile, W)
    if ys.size == 0:
        return y_cache
    xa = np.asarray(x_map, F64)[:, ys, xs, :]
    n = layernorm(xa, np.asarray(ln_g, F64), np.asarray(ln_b, F64))
    k = round_store(linear(n, wk), dtype)
    v = round_store(linear(n, wv), dtype)
    o = attention_active(linear(n, wq), k, v, heads)
    y_cache[:, ys, xs, :] = round_store(xa + linear(o, wo, bo), dtype)
    return y_cache


def context_kv(ctx, wk, wv, dtype):
    """K, V of the text context, computed once per conditioning and stored."""
    return round_store(linear(ctx, wk), dtype), round_store(linear(ctx, wv), dtype)
