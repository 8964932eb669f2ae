"""CPU oracle for the composite modules: masked ResNet block, masked transformer
block and the masked UNet step (FISEdit, section "Sparse Computation": ResNet
and attention modules recomputed inside the mask, everything else reused from
the cache of the previous generation; section "Approximate Normalization":
GroupNorm statistics come from that cache too).

TEST INFRASTRUCTURE ONLY (see fise_oracle.py).  numpy float64; every tensor the
method stores in the cache is rounded to the storage dtype when stored.

The UNet is the publicly documented Stable-Diffusion-1.x denoiser layout, made
parametric (base width, level multipliers, heads, context width) so the same
walk runs a small instance in seconds.  The paper does not print it; it only
says the U-Net is a stack of ResNet and attention modules.

Cache: a dict name -> array.  A masked step updates the cache in place:
  '<res>.h1', '<res>.out'       stored maps of a ResNet block
  '<tr>.k', '<tr>.v', '<tr>.out' self-attention K/V caches and block output
  '<ds|us>.out', 'conv_in.out', 'eps'
  '<gn>.mean', '<gn>.rstd'      statistics of every GroupNorm
With stats='cached' the statistics found in the cache are used as they are; with
stats='fresh' they are recomputed from the current (updated) input map and
stored.  A dense forward is the same walk with the full index list and fresh
statistics on an all-zero cache.
"""
from __future__ import annotations

import math

import numpy as np

from . import fise_oracle as fo

F64 = np.float64


# ----------------------------------------------------------------------------
# architecture description
# ----------------------------------------------------------------------------
def sd15_desc(**over):
    d = dict(in_ch=4, out_ch=4, base=320, mults=(1, 2, 4, 4), layers=2, attn=(True, True, True, False),
             heads=8, ctx_dim=768, n_ctx=77, groups=32, H=64, W=64, B=2)
    d.update(over)
    return d


def tiny_desc(**over):
    """Same topology, 1/10 of the width, 16x16 latent: runs in a second."""
    d = sd15_desc(base=32, heads=4, ctx_dim=64, n_ctx=11, H=16, W=16)
    d.update(over)
    return d


def unet_modules(desc):
    """The module walk as a list of dicts, in execution order.  Every entry has
    'kind', 'name', level 'lvl' (0 = finest), channel counts, and for the up
    path the name of the skip map it concatenates."""
    base, mults, L = desc["base"], desc["mults"], desc["layers"]
    mods = [dict(kind="conv_in", name="conv_in", lvl=0, cin=desc["in_ch"], cout=base)]
    skips = [("conv_in.out", base)]
    ch = base
    nl = len(mults)
    for l, m in enumerate(mults):
        co = base * m
        for i in range(L):
            mods.append(dict(kind="res", name=f"down.{l}.res.{i}", lvl=l, cin=ch, cskip=0, cout=co, skip=None))
            ch = co
            last = f"down.{l}.res.{i}.out"
            if desc["attn"][l]:
                mods.append(dict(kind="tr", name=f"down.{l}.tr.{i}", lvl=l, c=ch))
                last = f"down.{l}.tr.{i}.out"
            skips.append((last, ch))
        if l != nl - 1:
            mods.append(dict(kind="ds", name=f"down.{l}.ds", lvl=l + 1, c=ch))
            skips.append((f"down.{l}.ds.out", ch))
    lb = nl - 1
    mods.append(dict(kind="res", name="mid.res.0", lvl=lb, cin=ch, cskip=0, cout=ch, skip=None))
    mods.append(dict(kind="tr", name="mid.tr.0", lvl=lb, c=ch))
    mods.append(dict(kind="res", name="mid.res.1", lvl=lb, cin=ch, cskip=0, cout=ch, skip=None))
    for j, l in enumerate(reversed(range(nl))):
        co = base * mults[l]
        for i in range(L + 1):
            sname, sch = skips.pop()
            mods.append(dict(kind="res", name=f"up.{j}.res.{i}", lvl=l, cin=ch, cskip=sch, cout=co, skip=sname))
            ch = co
            if desc["attn"][l]:
                mods.append(dict(kind="tr", name=f"up.{j}.tr.{i}", lvl=l, c=ch))
        if l != 0:
            mods.append(dict(kind="us", name=f"up.{j}.us", lvl=l - 1, c=ch))
    assert not skips
    mods.append(dict(kind="out", name="out", lvl=0, cin=ch, cout=desc["out_ch"]))
    return mods


def param_shapes(desc):
    """name -> shape for every weight tensor, in module order."""
    base, cd = desc["base"], desc["ctx_dim"]
    te = 4 * base
    sh = {"time.l1.w": (te, base), "time.l1.b": (te,), "time.l2.w": (te, te), "time.l2.b": (te,)}
    for m in unet_modules(desc):
        n, k = m["name"], m["kind"]
        if k == "conv_in":
            sh[f"{n}.w"] = (m["cout"], 3, 3, m["cin"]); sh[f"{n}.b"] = (m["cout"],)
        elif k == "res":
            ci, co = m["cin"] + m["cskip"], m["cout"]
            sh[f"{n}.gn1.g"] = (ci,); sh[f"{n}.gn1.b"] = (ci,)
            sh[f"{n}.conv1.w"] = (co, 3, 3, ci); sh[f"{n}.conv1.b"] = (co,)
            sh[f"{n}.temb.w"] = (co, te); sh[f"{n}.temb.b"] = (co,)
            sh[f"{n}.gn2.g"] = (co,); sh[f"{n}.gn2.b"] = (co,)
            sh[f"{n}.conv2.w"] = (co, 3, 3, co); sh[f"{n}.conv2.b"] = (co,)
            if ci != co:
                sh[f"{n}.sc.w"] = (co, 1, 1, ci); sh[f"{n}.sc.b"] = (co,)
        elif k == "tr":
            c = m["c"]
            sh[f"{n}.gn.g"] = (c,); sh[f"{n}.gn.b"] = (c,)
            sh[f"{n}.pin.w"] = (c, 1, 1, c); sh[f"{n}.pin.b"] = (c,)
            sh[f"{n}.ln1.g"] = (c,); sh[f"{n}.ln1.b"] = (c,)
            for t in "qkv":
                sh[f"{n}.a1.{t}.w"] = (c, c)
            sh[f"{n}.a1.o.w"] = (c, c); sh[f"{n}.a1.o.b"] = (c,)
            sh[f"{n}.ln2.g"] = (c,); sh[f"{n}.ln2.b"] = (c,)
            sh[f"{n}.a2.q.w"] = (c, c); sh[f"{n}.a2.k.w"] = (c, cd); sh[f"{n}.a2.v.w"] = (c, cd)
            sh[f"{n}.a2.o.w"] = (c, c); sh[f"{n}.a2.o.b"] = (c,)
            sh[f"{n}.ln3.g"] = (c,); sh[f"{n}.ln3.b"] = (c,)
            sh[f"{n}.ff1.w"] = (8 * c, c); sh[f"{n}.ff1.b"] = (8 * c,)
            sh[f"{n}.ff2.w"] = (c, 4 * c); sh[f"{n}.ff2.b"] = (c,)
            sh[f"{n}.pout.w"] = (c, 1, 1, c); sh[f"{n}.pout.b"] = (c,)
        elif k in ("ds", "us"):
            sh[f"{n}.w"] = (m["c"], 3, 3, m["c"]); sh[f"{n}.b"] = (m["c"],)
        elif k == "out":
            sh[f"{n}.gn.g"] = (m["cin"],); sh[f"{n}.gn.b"] = (m["cin"],)
            sh[f"{n}.conv.w"] = (m["cout"], 3, 3, m["cin"]); sh[f"{n}.conv.b"] = (m["cout"],)
    return sh


def timestep_embedding(t, dim: int):
    """Sinusoidal embedding [cos(t f_i), sin(t f_i)], f_i = 10000^(-i/(dim/2))."""
    half = dim // 2
    f = np.exp(-math.log(10000.0) * np.arange(half, dtype=F64) / half)
    a = np.asarray(t, F64)[:, None] * f[None, :]
    return np.concatenate([np.cos(a), np.sin(a)], axis=1)


# ----------------------------------------------------------------------------
# composite modules
# ----------------------------------------------------------------------------
def _stats(cache, key, src, groups, eps, stats):
    if stats == "fresh":
        cache[f"{key}.mean"], cache[f"{key}.rstd"] = fo.gn_stats(src, groups, eps)
    return cache[f"{key}.mean"], cache[f"{key}.rstd"]


def _silu(a):
    return a / (1.0 + np.exp(-a))


def resnet_block(P, name, xs, emb, cache, idx, tile, dtype, groups=32, stats="cached", scratch="f64"):
    """GN+SiLU -> conv3x3 (+ time projection) -> GN+SiLU -> conv3x3 -> + shortcut,
    at active pixels; `xs` is the input map or [map, skip map] (channel concat).
    Stores h1 and the block output in the cache; the shortcut (identity, or a
    1x1 conv when the channel count changes) is not stored, hence not rounded.
    scratch: see unet_step."""
    xs = list(xs) if isinstance(xs, (list, tuple)) else [xs]
    ci = sum(x.shape[-1] for x in xs)
    co = P[f"{name}.conv1.w"].shape[0]
    m1, r1 = _stats(cache, f"{name}.gn1", xs, groups, 1e-5, stats)
    tproj = fo.linear(_silu(np.asarray(emb, F64)), P[f"{name}.temb.w"], P[f"{name}.temb.b"])
    fo.masked_conv(xs, P[f"{name}.conv1.w"], P[f"{name}.conv1.b"], idx, tile, cache[f"{name}.h1"], dtype,
                   gn=dict(mean=m1, rstd=r1, gamma=P[f"{name}.gn1.g"], beta=P[f"{name}.gn1.b"], groups=groups),
                   temb=tproj, act_dtype=scratch)
    h1 = cache[f"{name}.h1"]
    m2, r2 = _stats(cache, f"{name}.gn2", h1, groups, 1e-5, stats)
    if ci != co:
        B, H, W, _ = h1.shape
        short = np.zeros((B, H, W, co), F64)       # only active positions get filled and read
        fo.masked_conv(xs, P[f"{name}.sc.w"], P[f"{name}.sc.b"], idx, tile, short, "f64")
    else:
        short = fo._cat_sources(xs)
    fo.masked_conv(h1, P[f"{name}.conv2.w"], P[f"{name}.conv2.b"], idx, tile, cache[f"{name}.out"], dtype,
                   gn=dict(mean=m2, rstd=r2, gamma=P[f"{name}.gn2.g"], beta=P[f"{name}.gn2.b"], groups=groups),
                   residual=short, act_dtype=scratch)
    return cache[f"{name}.out"]


def transformer_block(P, name, x, Kc, Vc, cache, idx, tile, dtype, heads, groups=32, stats="cached", scratch="f64"):
    """GN -> 1x1 in -> [LN, self-attn] -> [LN, cross-attn] -> [LN, GEGLU FF]
    -> 1x1 out -> + block input, on active tokens only.  Self-attention K/V
    rows of the active tokens are refreshed in the cache (stored => rounded);
    active queries attend to all keys.  Kc, Vc: context K/V of this block
    (computed once per conditioning).  Stores the block output.  scratch: see
    unet_step (the residual stream h itself is never rounded)."""
    x = np.asarray(x, F64)
    B, H, W, C = x.shape
    m, r = _stats(cache, f"{name}.gn", x, groups, 1e-6, stats)
    ys, xs = fo.active_pixels(idx, tile, W)
    if ys.size == 0:
        return cache[f"{name}.out"]
    gi = np.arange(C) // (C // groups)
    xa = x[:, ys, xs, :]                                              # [B, M, C]
    rs = lambda a: fo.round_store(a, scratch)                          # an operand parked in scratch memory
    g = rs((xa - m[:, None, gi]) * r[:, None, gi] * np.asarray(P[f"{name}.gn.g"], F64) + np.asarray(P[f"{name}.gn.b"], F64))
    h = fo.linear(g, np.asarray(P[f"{name}.pin.w"]).reshape(C, C), P[f"{name}.pin.b"])
    # self-attention
    n = rs(fo.layernorm(h, P[f"{name}.ln1.g"], P[f"{name}.ln1.b"]))
    o = rs(fo.masked_self_attention(n, P[f"{name}.a1.q.w"], P[f"{name}.a1.k.w"], P[f"{name}.a1.v.w"], heads,
                                    cache[f"{name}.k"], cache[f"{name}.v"], ys * W + xs, dtype, scratch))
    h = h + fo.linear(o, P[f"{name}.a1.o.w"], P[f"{name}.a1.o.b"])
    # cross-attention
    n = rs(fo.layernorm(h, P[f"{name}.ln2.g"], P[f"{name}.ln2.b"]))
    o = rs(fo.attention_active(rs(fo.linear(n, P[f"{name}.a2.q.w"])), Kc, Vc, heads, scratch))
    h = h + fo.linear(o, P[f"{name}.a2.o.w"], P[f"{name}.a2.o.b"])
    # feed-forward
    n = rs(fo.layernorm(h, P[f"{name}.ln3.g"], P[f"{name}.ln3.b"]))
    f = rs(fo.geglu(fo.linear(n, P[f"{name}.ff1.w"], P[f"{name}.ff1.b"])))
    h = h + fo.linear(f, P[f"{name}.ff2.w"], P[f"{name}.ff2.b"])
    y = fo.linear(rs(h), np.asarray(P[f"{name}.pout.w"]).reshape(C, C), P[f"{name}.pout.b"]) + xa
    cache[f"{name}.out"][:, ys, xs, :] = fo.round_store(y, dtype)
    return cache[f"{name}.out"]


def context_kv_all(P, desc, ctx, dtype):
    """Context K/V of every transformer block for one conditioning."""
    out = {}
    for m in unet_modules(desc):
        if m["kind"] == "tr":
            n = m["name"]
            out[n] = fo.context_kv(ctx, P[f"{n}.a2.k.w"], P[f"{n}.a2.v.w"], dtype)
    return out


def cache_shapes(desc):
    """name -> shape of every cached tensor (maps, K/V, statistics)."""
    B, H, W, G = desc["B"], desc["H"], desc["W"], desc["groups"]
    sh = {}
    for m in unet_modules(desc):
        n, k = m["name"], m["kind"]
        h, w = H >> m["lvl"], W >> m["lvl"]
        if k == "conv_in":
            sh[f"{n}.out"] = (B, h, w, m["cout"])
        elif k == "res":
            for g in ("gn1", "gn2"):
                sh[f"{n}.{g}.mean"] = (B, G); sh[f"{n}.{g}.rstd"] = (B, G)
            sh[f"{n}.h1"] = (B, h, w, m["cout"]); sh[f"{n}.out"] = (B, h, w, m["cout"])
        elif k == "tr":
            sh[f"{n}.gn.mean"] = (B, G); sh[f"{n}.gn.rstd"] = (B, G)
            sh[f"{n}.k"] = (B, h * w, m["c"]); sh[f"{n}.v"] = (B, h * w, m["c"])
            sh[f"{n}.out"] = (B, h, w, m["c"])
        elif k in ("ds", "us"):
            sh[f"{n}.out"] = (B, h, w, m["c"])
        elif k == "out":
            sh[f"{n}.gn.mean"] = (B, G); sh[f"{n}.gn.rstd"] = (B, G)
            sh["eps"] = (B, h, w, m["cout"])
    return sh


def empty_cache(desc):
    return {k: np.zeros(s, F64) for k, s in cache_shapes(desc).items()}


def module_output_name(m):
    return "eps" if m["kind"] == "out" else f"{m['name']}.out"


def unet_step(P, desc, cache, latent, t_sin, ctx_kv, idx, base_tile, dtype, stats="cached", level_dense=None, only=None,
              scratch="f64"):
    """One masked UNet evaluation.  `latent` [B,H,W,in_ch] is the (updated)
    input; `t_sin` [B, base] the sinusoidal time embedding; `ctx_kv` the dict
    from context_kv_all for the *new* conditioning; `idx` the active-tile list
    on the finest level with tile edge `base_tile`.  The same tile grid serves
    every level: the tile edge halves with the resolution (OR-pooling a mask
    that is a union of base tiles gives exactly that), so base_tile must be
    divisible by 2**(levels-1).  The cache is updated in place; returns the
    predicted noise map cache['eps'].  level_dense[l] = True runs level l with
    the full index list.  only = a set of module positions in the walk: the
    others are skipped and their cached output stands in for them.

    scratch: precision of the operands a module hands from one product to the
    next WITHOUT storing them in the cache (normalised / activated conv inputs,
    LayerNorm outputs, queries, softmax weights, attention outputs, the gated
    feed-forward activations, the residual stream entering the 1x1 out).  'f64'
    (default) keeps them exact: only stored tensors are rounded.  'bf16' rounds
    each of them once, which is what any implementation whose matrix units take
    bf16 operands must do; the float accumulations and the residual stream stay
    unrounded in both modes."""
    G, heads = desc["groups"], desc["heads"]
    H, W = desc["H"], desc["W"]
    nl = len(desc["mults"])
    assert base_tile % (1 << (nl - 1)) == 0
    full = fo.full_index(H, W, base_tile)

    def lv(l):
        use = full if (level_dense is not None and level_dense[l]) else idx
        return use, base_tile >> l

    emb = fo.linear(_silu(fo.linear(t_sin, P["time.l1.w"], P["time.l1.b"])), P["time.l2.w"], P["time.l2.b"])
    cur = None
    for mi, m in enumerate(unet_modules(desc)):
        n, k = m["name"], m["kind"]
        li, lt = lv(m["lvl"])
        if only is not None and mi not in only:
            cur = cache[module_output_name(m)]
            continue
        if k == "conv_in":
            cur = fo.masked_conv(np.asarray(latent, F64), P[f"{n}.w"], P[f"{n}.b"], li, lt, cache[f"{n}.out"], dtype)
        elif k == "res":
            src = [cur] if m["skip"] is None else [cur, cache[m["skip"]]]
            cur = resnet_block(P, n, src, emb, cache, li, lt, dtype, G, stats, scratch)
        elif k == "tr":
            Kc, Vc = ctx_kv[n]
            cur = transformer_block(P, n, cur, Kc, Vc, cache, li, lt, dtype, heads, G, stats, scratch)
        elif k == "ds":
            cur = fo.masked_conv(cur, P[f"{n}.w"], P[f"{n}.b"], li, lt, cache[f"{n}.out"], dtype, stride=2)
        elif k == "us":
            cur = fo.masked_conv(cur, P[f"{n}.w"], P[f"{n}.b"], li, lt, cache[f"{n}.out"], dtype, upsample=True)
        elif k == "out":
            mo, ro = _stats(cache, f"{n}.gn", cur, G, 1e-5, stats)
            cur = fo.masked_conv(cur, P[f"{n}.conv.w"], P[f"{n}.conv.b"], li, lt, cache["eps"], dtype,
                                 gn=dict(mean=mo, rstd=ro, gamma=P[f"{n}.gn.g"], beta=P[f"{n}.gn.b"], groups=G),
                                 act_dtype=scratch)
    return cache["eps"]


def unet_dense(P, desc, latent, t_sin, ctx_kv, dtype, scratch="f64"):
    """Dense forward = the same walk, full index list, fresh statistics, on an
    all-zero cache.  Returns (eps, cache)."""
    cache = empty_cache(desc)
    nl = len(desc["mults"])
    tile = 1 << (nl - 1)
    eps = unet_step(P, desc, cache, latent, t_sin, ctx_kv, fo.full_index(desc["H"], desc["W"], tile), tile,
                    dtype, stats="fresh", scratch=scratch)
    return eps, cache
