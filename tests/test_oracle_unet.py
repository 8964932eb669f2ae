"""Pins for the composite oracle (ResNet block, transformer block, UNet step).

The dense walk is checked against an independent forward written here with
torch's CPU library routines in NCHW (conv2d, group_norm, layer_norm,
scaled_dot_product_attention, interpolate, cat) following the public
Stable-Diffusion-1.x UNet layout; the architecture walk is checked against the
published parameter count of that network; the masked step against the
invariants the method promises (empty mask -> cache, full mask with fresh
statistics -> dense, untouched positions bitwise equal, idempotence)."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import fise_oracle as fo
from oracle import fise_unet_oracle as uo
from paper_2305_17423_amd import workloads as wl


def T(a):
    return torch.from_numpy(np.ascontiguousarray(np.asarray(a, np.float64)))


def conv(x, w, b, stride=1):
    w = T(w).permute(0, 3, 1, 2)
    return F.conv2d(x, w, T(b), stride=stride, padding=w.shape[-1] // 2)


def lib_res(P, n, x, emb, G):
    h = conv(F.silu(F.group_norm(x, G, T(P[f"{n}.gn1.g"]), T(P[f"{n}.gn1.b"]), 1e-5)), P[f"{n}.conv1.w"], P[f"{n}.conv1.b"])
    h = h + F.linear(F.silu(emb), T(P[f"{n}.temb.w"]), T(P[f"{n}.temb.b"]))[:, :, None, None]
    h = conv(F.silu(F.group_norm(h, G, T(P[f"{n}.gn2.g"]), T(P[f"{n}.gn2.b"]), 1e-5)), P[f"{n}.conv2.w"], P[f"{n}.conv2.b"])
    if f"{n}.sc.w" in P:
        x = conv(x, P[f"{n}.sc.w"], P[f"{n}.sc.b"])
    return x + h


def lib_attn(x, ctx, wq, wk, wv, wo, bo, heads):
    B, N, C = x.shape
    def sp(t):
        return t.reshape(B, t.shape[1], heads, C // heads).permute(0, 2, 1, 3)
    o = F.scaled_dot_product_attention(sp(F.linear(x, T(wq))), sp(F.linear(ctx, T(wk))), sp(F.linear(ctx, T(wv))))
    return F.linear(o.permute(0, 2, 1, 3).reshape(B, N, C), T(wo), T(bo))


def lib_tr(P, n, x, ctx, G, heads):
    B, C, H, W = x.shape
    h = conv(F.group_norm(x, G, T(P[f"{n}.gn.g"]), T(P[f"{n}.gn.b"]), 1e-6), P[f"{n}.pin.w"], P[f"{n}.pin.b"])
    h = h.permute(0, 2, 3, 1).reshape(B, H * W, C)
    ln = lambda t, k: F.layer_norm(t, (C,), T(P[f"{n}.{k}.g"]), T(P[f"{n}.{k}.b"]), 1e-5)
    a = ln(h, "ln1")
    h = h + lib_attn(a, a, P[f"{n}.a1.q.w"], P[f"{n}.a1.k.w"], P[f"{n}.a1.v.w"], P[f"{n}.a1.o.w"], P[f"{n}.a1.o.b"], heads)
    h = h + lib_attn(ln(h, "ln2"), ctx, P[f"{n}.a2.q.w"], P[f"{n}.a2.k.w"], P[f"{n}.a2.v.w"], P[f"{n}.a2.o.w"], P[f"{n}.a2.o.b"], heads)
    g = F.linear(ln(h, "ln3"), T(P[f"{n}.ff1.w"]), T(P[f"{n}.ff1.b"]))
    u, gate = g.chunk(2, dim=-1)
    h = h + F.linear(u * F.gelu(gate), T(P[f"{n}.ff2.w"]), T(P[f"{n}.ff2.b"]))
    h = h.reshape(B, H, W, C).permute(0, 3, 1, 2)
    return conv(h, P[f"{n}.pout.w"], P[f"{n}.pout.b"]) + x


def lib_unet(P, d, latent, t_sin, ctx):
    """Hand-written forward of the public SD-1.x UNet topology with library ops."""
    G, heads, L, nl = d["groups"], d["heads"], d["layers"], len(d["mults"])
    emb = F.linear(F.silu(F.linear(T(t_sin), T(P["time.l1.w"]), T(P["time.l1.b"]))), T(P["time.l2.w"]), T(P["time.l2.b"]))
    ctx = T(ctx)
    x = conv(T(latent).permute(0, 3, 1, 2), P["conv_in.w"], P["conv_in.b"])
    skips = [x]
    for l in range(nl):
        for i in range(L):
            x = lib_res(P, f"down.{l}.res.{i}", x, emb, G)
            if d["attn"][l]:
                x = lib_tr(P, f"down.{l}.tr.{i}", x, ctx, G, heads)
            skips.append(x)
        if l != nl - 1:
            x = conv(x, P[f"down.{l}.ds.w"], P[f"down.{l}.ds.b"], stride=2)
            skips.append(x)
    x = lib_res(P, "mid.res.0", x, emb, G)
    x = lib_tr(P, "mid.tr.0", x, ctx, G, heads)
    x = lib_res(P, "mid.res.1", x, emb, G)
    for j in range(nl):
        l = nl - 1 - j
        for i in range(L + 1):
            x = lib_res(P, f"up.{j}.res.{i}", torch.cat([x, skips.pop()], dim=1), emb, G)
            if d["attn"][l]:
                x = lib_tr(P, f"up.{j}.tr.{i}", x, ctx, G, heads)
        if l != 0:
            x = conv(F.interpolate(x, scale_factor=2.0, mode="nearest"), P[f"up.{j}.us.w"], P[f"up.{j}.us.b"])
    x = conv(F.silu(F.group_norm(x, G, T(P["out.gn.g"]), T(P["out.gn.b"]), 1e-5)), P["out.conv.w"], P["out.conv.b"])
    return x.permute(0, 2, 3, 1).numpy()


def tiny_problem(seed, dtype="f32", std=0.1, **over):
    d = uo.tiny_desc(**over)
    rng = np.random.default_rng(seed)
    P = wl.params_from_shapes(rng, uo.param_shapes(d), std, dtype)
    lat = wl.normal(rng, (d["B"], d["H"], d["W"], d["in_ch"]), 1.0, dtype)
    ctx = wl.normal(rng, (d["B"], d["n_ctx"], d["ctx_dim"]), 1.0, dtype)
    t_sin = uo.timestep_embedding(np.full(d["B"], 481.0), d["base"]).astype(np.float32)
    return d, rng, P, lat, ctx, t_sin


def test_parameter_count_of_sd15_walk():
    # the published size of the Stable Diffusion 1.x denoiser: 859,520,964 parameters
    sh = uo.param_shapes(uo.sd15_desc())
    assert sum(int(np.prod(s)) for s in sh.values()) == 859_520_964
    mods = uo.unet_modules(uo.sd15_desc())
    assert sum(m["kind"] == "res" for m in mods) == 22 and sum(m["kind"] == "tr" for m in mods) == 16
    ups = [(m["cin"] + m["cskip"], m["cout"]) for m in mods if m["name"].startswith("up.")and m["kind"] == "res"]
    assert ups == [(2560, 1280)] * 3 + [(2560, 1280), (2560, 1280), (1920, 1280), (1920, 640), (1280, 640), (960, 640),
                                       (960, 320), (640, 320), (640, 320)]


def test_timestep_embedding_closed_form():
    e = uo.timestep_embedding(np.array([0.0, 3.0]), 8)
    np.testing.assert_allclose(e[0], [1, 1, 1, 1, 0, 0, 0, 0], atol=1e-15)
    f = 10000.0 ** (-np.arange(4) / 4)
    np.testing.assert_allclose(e[1], np.concatenate([np.cos(3 * f), np.sin(3 * f)]), atol=1e-15)


def test_dense_walk_equals_library_unet():
    d, rng, P, lat, ctx, t_sin = tiny_problem(21)
    ckv = uo.context_kv_all(P, d, ctx, "f64")
    eps, cache = uo.unet_dense(P, d, lat, t_sin, ckv, "f64")
    want = lib_unet(P, d, lat, t_sin, ctx)
    assert np.abs(want).max() > 1e-3
    # GroupNorm statistics are kept in float32 (they are cached): 1e-6-level agreement
    np.testing.assert_allclose(eps, want, atol=2e-5 * np.abs(want).max())


def test_masked_step_invariants():
    d, rng, P, lat, ctx, t_sin = tiny_problem(22, dtype="bf16")
    ctx_new = wl.normal(rng, ctx.shape, 1.0, "bf16")
    kv_old = uo.context_kv_all(P, d, ctx, "bf16"); kv_new = uo.context_kv_all(P, d, ctx_new, "bf16")
    eps0, cache0 = uo.unet_dense(P, d, lat, t_sin, kv_old, "bf16")
    snap = {k: v.copy() for k, v in cache0.items()}
    H, W, bt = d["H"], d["W"], 8
    # empty mask: nothing changes, bit for bit, even with new conditioning and new latent
    lat_new = wl.perturb(rng, lat, wl.rect_pixels(rng, H, W, 5, 5), 1.0, "bf16")
    uo.unet_step(P, d, cache0, lat_new, t_sin, kv_new, np.zeros(0, np.int32), bt, "bf16")
    for k in snap:
        np.testing.assert_array_equal(cache0[k], snap[k])
    # full mask + fresh statistics == dense forward of the new inputs
    full = fo.full_index(H, W, bt)
    c1 = {k: v.copy() for k, v in snap.items()}
    e1 = uo.unet_step(P, d, c1, lat_new, t_sin, kv_new, full, bt, "bf16", stats="fresh")
    e2, c2 = uo.unet_dense(P, d, lat_new, t_sin, kv_new, "bf16")
    for k in c2:
        np.testing.assert_array_equal(c1[k], c2[k])
    # partial mask, cached statistics: untouched positions bitwise equal; statistics untouched; idempotent
    pix, tm, idx = fo.mask_detect(lat, lat_new, 0.1, bt)
    assert 0 < idx.size < full.size
    c3 = {k: v.copy() for k, v in snap.items()}
    uo.unet_step(P, d, c3, lat_new, t_sin, kv_new, idx, bt, "bf16")
    changed = 0
    for m in uo.unet_modules(d):
        t = bt >> m["lvl"]
        w = W >> m["lvl"]
        ys, xs = fo.active_pixels(idx, t, w)
        act = np.zeros((H >> m["lvl"], w), bool); act[ys, xs] = True
        names = {"res": ["h1", "out"], "tr": ["out"], "ds": ["out"], "us": ["out"], "conv_in": ["out"]}.get(m["kind"], [])
        for s in names:
            a, b = c3[f"{m['name']}.{s}"], snap[f"{m['name']}.{s}"]
            np.testing.assert_array_equal(a[:, ~act], b[:, ~act])
            changed += int((a[:, act] != b[:, act]).any())
        if m["kind"] == "tr":
            for s in ("k", "v"):
                a, b = c3[f"{m['name']}.{s}"], snap[f"{m['name']}.{s}"]
                np.testing.assert_array_equal(a[:, ~act.reshape(-1)], b[:, ~act.reshape(-1)])
    assert changed > 40
    for k in snap:
        if k.endswith(".mean") or k.endswith(".rstd"):
            np.testing.assert_array_equal(c3[k], snap[k])
    c4 = {k: v.copy() for k, v in c3.items()}
    uo.unet_step(P, d, c4, lat_new, t_sin, kv_new, idx, bt, "bf16")
    for k in c3:
        np.testing.assert_array_equal(c4[k], c3[k])
    # every stored map is bf16-representable
    for k, v in c3.items():
        if not (k.endswith(".mean") or k.endswith(".rstd")):
            np.testing.assert_array_equal(v, fo.round_store(v, "bf16"))


def test_level_dense_override_runs_that_level_with_full_list():
    d, rng, P, lat, ctx, t_sin = tiny_problem(23)
    kv = uo.context_kv_all(P, d, ctx, "f64")
    _, cache = uo.unet_dense(P, d, lat, t_sin, kv, "f64")
    lat_new = wl.perturb(rng, lat, wl.rect_pixels(rng, 16, 16, 4, 4))
    _, _, idx = fo.mask_detect(lat, lat_new, 0.1, 8)
    ca = {k: v.copy() for k, v in cache.items()}
    uo.unet_step(P, d, ca, lat_new, t_sin, kv, idx, 8, "f64", level_dense=[False, False, True, True])
    cb = {k: v.copy() for k, v in cache.items()}
    uo.unet_step(P, d, cb, lat_new, t_sin, kv, idx, 8, "f64")
    assert (ca["mid.res.0.out"] != cb["mid.res.0.out"]).any()
    np.testing.assert_array_equal(ca["down.0.res.0.out"], cb["down.0.res.0.out"])


def test_bf16_operand_rounding_alone():
    """How far does rounding ONLY the convolution inputs to bf16 (what a bf16 MFMA path has to do)
    move a ResNet block of the small instance away from the float64 oracle?  About 2e-2 in the
    elementwise metric of the GPU tests: the reason the small-instance GPU bound is 2.5e-2."""
    d = uo.tiny_desc(H=32, W=32, base=64)
    rng = np.random.default_rng(5010)
    P = wl.params_from_shapes(rng, uo.param_shapes(d), 0.04, "bf16")
    n = "up.3.res.2"
    B, H, W = 2, 32, 32
    x = wl.normal(rng, (B, H, W, 64), 1.0, "bf16"); skip = wl.normal(rng, (B, H, W, 64), 1.0, "bf16")
    emb = wl.normal(rng, (B, 256), 1.0)
    full = fo.full_index(H, W, 8)
    def run():
        cache = {f"{n}.h1": np.zeros((B, H, W, 64)), f"{n}.out": np.zeros((B, H, W, 64))}
        uo.resnet_block(P, n, [x, skip], emb, cache, full, 8, "bf16", 32, stats="fresh")
        return cache[f"{n}.out"]
    want = run()
    orig = fo._gn_silu
    try:
        fo._gn_silu = lambda *a: fo.round_store(orig(*a), "bf16")
        got = run()
    finally:
        fo._gn_silu = orig
    rms = np.sqrt(np.mean(want ** 2))
    err = np.max(np.abs(got - want) / np.maximum(np.abs(want), rms))
    assert 5e-3 < err < 2.5e-2, err
