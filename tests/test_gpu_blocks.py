"""GPU parity at the module level: masked ResNet block (config 2 shape and deeper levels)
and masked transformer block (configs 3/4 shapes), element by element against the oracle,
both sides starting from the oracle's cache of the old generation."""
import math

import numpy as np
import pytest
import torch

from oracle import fise_oracle as fo
from oracle import fise_unet_oracle as uo
from paper_2305_17423_amd import workloads as wl
from helpers import DEV, TOL, dev, host, rel_err, idx_dev, active_mask, check_map

pytestmark = pytest.mark.gpu
DT = "bf16"


@pytest.fixture(scope="module")
def fb():
    from paper_2305_17423_amd import binding
    binding.lib()
    assert torch.cuda.is_available()
    return binding


def res_shapes(n, ci, co, te):
    sh = {f"{n}.gn1.g": (ci,), f"{n}.gn1.b": (ci,), f"{n}.conv1.w": (co, 3, 3, ci), f"{n}.conv1.b": (co,),
          f"{n}.temb.w": (co, te), f"{n}.temb.b": (co,), f"{n}.gn2.g": (co,), f"{n}.gn2.b": (co,),
          f"{n}.conv2.w": (co, 3, 3, co), f"{n}.conv2.b": (co,)}
    if ci != co:
        sh[f"{n}.sc.w"] = (co, 1, 1, ci); sh[f"{n}.sc.b"] = (co,)
    return sh


def tr_shapes(n, c, cd):
    sh = {}
    for k in ("gn", "ln1", "ln2", "ln3"):
        sh[f"{n}.{k}.g"] = (c,); sh[f"{n}.{k}.b"] = (c,)
    sh.update({f"{n}.pin.w": (c, 1, 1, c), f"{n}.pin.b": (c,), f"{n}.a1.q.w": (c, c), f"{n}.a1.k.w": (c, c), f"{n}.a1.v.w": (c, c),
               f"{n}.a1.o.w": (c, c), f"{n}.a1.o.b": (c,), f"{n}.a2.q.w": (c, c), f"{n}.a2.k.w": (c, cd), f"{n}.a2.v.w": (c, cd),
               f"{n}.a2.o.w": (c, c), f"{n}.a2.o.b": (c,), f"{n}.ff1.w": (8 * c, c), f"{n}.ff1.b": (8 * c,),
               f"{n}.ff2.w": (c, 4 * c), f"{n}.ff2.b": (c,), f"{n}.pout.w": (c, 1, 1, c), f"{n}.pout.b": (c,)})
    return sh


RES_CASES = [
    # name, B, H, W, C0, C1, Cout, tile, frac, weight std
    ("cfg2-64x64-320", 2, 64, 64, 320, 0, 320, 8, 0.10, 0.02),
    ("cfg4-32x32-640", 2, 32, 32, 640, 0, 640, 4, 0.10, 0.02),
    ("cfg4-16x16-1280", 2, 16, 16, 1280, 0, 1280, 4, 0.25, 0.02),
    ("up-concat-960-to-320", 2, 32, 32, 640, 320, 320, 4, 0.05, 0.02),
    ("down-320-to-640", 2, 16, 16, 320, 0, 640, 2, 0.5, 0.03),
]


@pytest.mark.parametrize("case", RES_CASES, ids=[c[0] for c in RES_CASES])
def test_resnet_block(fb, case):
    name, B, H, W, C0, C1, Co, t, frac, std = case
    rng = np.random.default_rng(6000 + H + C0 + C1)
    te, G, n = 1280, 32, "r"
    P = wl.params_from_shapes(rng, res_shapes(n, C0 + C1, Co, te), std, DT)
    x_old = wl.normal(rng, (B, H, W, C0), 1.0, DT)
    skip = wl.normal(rng, (B, H, W, C1), 1.0, DT) if C1 else None
    emb = wl.normal(rng, (B, te), 1.0)
    pixm = wl.ellipse_pixels(rng, H, W, frac)
    x_new = wl.perturb(rng, x_old, pixm, 1.0, DT)
    _, idx = fo.tiles_from_pixels(pixm, t)
    full = fo.full_index(H, W, t)
    cache = {f"{n}.h1": np.zeros((B, H, W, Co)), f"{n}.out": np.zeros((B, H, W, Co))}
    uo.resnet_block(P, n, [x_old, skip] if C1 else x_old, emb, cache, full, t, DT, G, stats="fresh")     # old generation
    old = {k: v.copy() for k, v in cache.items()}
    want = {k: v.copy() for k, v in cache.items()}
    uo.resnet_block(P, n, [x_new, skip] if C1 else x_new, emb, want, idx, t, DT, G, stats="cached")
    tproj = fo.linear(uo._silu(emb.astype(np.float64)), P[f"{n}.temb.w"], P[f"{n}.temb.b"])                 # the step computes this once

    keep = []
    h1d, outd = dev(old[f"{n}.h1"], DT), dev(old[f"{n}.out"], DT)
    a = fb.fill_args(fb.fise_resnet_args, keep, x0=dev(x_new, DT), x1=(dev(skip, DT) if C1 else None), C0=C0, C1=C1, B=B, H=H, W=W,
                     Cout=Co, G=G, gn1_mean=dev(old[f"{n}.gn1.mean"]), gn1_rstd=dev(old[f"{n}.gn1.rstd"]),
                     gn1_gamma=dev(P[f"{n}.gn1.g"], DT), gn1_beta=dev(P[f"{n}.gn1.b"], DT), conv1_w=dev(P[f"{n}.conv1.w"], DT),
                     conv1_b=dev(P[f"{n}.conv1.b"], DT), temb=dev(tproj), temb_stride=Co,
                     gn2_mean=dev(old[f"{n}.gn2.mean"]), gn2_rstd=dev(old[f"{n}.gn2.rstd"]), gn2_gamma=dev(P[f"{n}.gn2.g"], DT),
                     gn2_beta=dev(P[f"{n}.gn2.b"], DT), conv2_w=dev(P[f"{n}.conv2.w"], DT), conv2_b=dev(P[f"{n}.conv2.b"], DT),
                     sc_w=(dev(P[f"{n}.sc.w"], DT) if C0 + C1 != Co else None), sc_b=(dev(P[f"{n}.sc.b"], DT) if C0 + C1 != Co else None),
                     tile_idx=idx_dev(idx), n_active=idx.size, tile=t, h1_cache=h1d, out_cache=outd, stats_fresh=0)
    ws = torch.zeros(max(fb.fise_masked_resnet_block_workspace_bytes(a), 256), dtype=torch.uint8, device=DEV)
    fb.fise_masked_resnet_block(a, ws)
    act = active_mask(idx, t, H, W)
    e1 = check_map(host(h1d), want[f"{n}.h1"], old[f"{n}.h1"], act, TOL[DT], name + " h1")
    e2 = check_map(host(outd), want[f"{n}.out"], old[f"{n}.out"], act, TOL[DT], name + " out")
    got = host(outd)
    fb.fise_masked_resnet_block(a, ws)                                   # idempotent
    assert np.array_equal(host(outd), got)
    # full list + fresh statistics from a zero cache reproduces the old generation (dense twin)
    h1z, outz = torch.zeros_like(h1d), torch.zeros_like(outd)
    m1, r1, m2, r2 = (torch.zeros((B, G), device=DEV) for _ in range(4))
    a2 = fb.fill_args(fb.fise_resnet_args, keep, x0=dev(x_old, DT), x1=(dev(skip, DT) if C1 else None), C0=C0, C1=C1, B=B, H=H, W=W,
                      Cout=Co, G=G, gn1_mean=m1, gn1_rstd=r1, gn1_gamma=a.gn1_gamma, gn1_beta=a.gn1_beta, conv1_w=a.conv1_w,
                      conv1_b=a.conv1_b, temb=a.temb, temb_stride=Co, gn2_mean=m2, gn2_rstd=r2, gn2_gamma=a.gn2_gamma,
                      gn2_beta=a.gn2_beta, conv2_w=a.conv2_w, conv2_b=a.conv2_b, sc_w=a.sc_w, sc_b=a.sc_b,
                      tile_idx=idx_dev(full), n_active=full.size, tile=t, h1_cache=h1z, out_cache=outz, stats_fresh=1)
    fb.fise_masked_resnet_block(a2, ws)
    assert rel_err(host(m1), old[f"{n}.gn1.mean"]) < 1e-4 and rel_err(host(r1), old[f"{n}.gn1.rstd"]) < 1e-4
    assert rel_err(host(h1z), old[f"{n}.h1"]) <= TOL[DT] and rel_err(host(outz), old[f"{n}.out"]) <= TOL[DT]
    print(f"{name}: h1 {e1:.2e} out {e2:.2e}")


TR_CASES = [
    # name, H, W, C, tile, frac
    ("cfg3-64x64-320-10pct", 64, 64, 320, 4, 0.10),
    ("cfg3-64x64-320-2pct", 64, 64, 320, 4, 0.02),
    ("cfg4-32x32-640", 32, 32, 640, 4, 0.10),
    ("cfg4-16x16-1280", 16, 16, 1280, 4, 0.25),
    ("tile1-8x8-1280", 8, 8, 1280, 1, 0.3),
]


@pytest.mark.parametrize("case", TR_CASES, ids=[c[0] for c in TR_CASES])
def test_transformer_block(fb, case):
    name, H, W, C, t, frac = case
    rng = np.random.default_rng(7000 + H + C + int(frac * 100))
    B, G, heads, cd, n_ctx, n = 2, 32, 8, 768, 77, "t"
    P = wl.params_from_shapes(rng, tr_shapes(n, C, cd), 0.02, DT)
    x_old = wl.normal(rng, (B, H, W, C), 1.0, DT)
    pixm = wl.ellipse_pixels(rng, H, W, frac)
    x_new = wl.perturb(rng, x_old, pixm, 1.0, DT)
    _, idx = fo.tiles_from_pixels(pixm, t)
    full = fo.full_index(H, W, t)
    ctx_old, ctx_new = wl.normal(rng, (B, n_ctx, cd), 1.0, DT), wl.normal(rng, (B, n_ctx, cd), 1.0, DT)
    Ko, Vo = fo.context_kv(ctx_old, P[f"{n}.a2.k.w"], P[f"{n}.a2.v.w"], DT)
    Kn, Vn = fo.context_kv(ctx_new, P[f"{n}.a2.k.w"], P[f"{n}.a2.v.w"], DT)
    cache = {f"{n}.k": np.zeros((B, H * W, C)), f"{n}.v": np.zeros((B, H * W, C)), f"{n}.out": np.zeros((B, H, W, C))}
    uo.transformer_block(P, n, x_old, Ko, Vo, cache, full, t, DT, heads, G, stats="fresh")
    old = {k: v.copy() for k, v in cache.items()}
    want = {k: v.copy() for k, v in cache.items()}
    uo.transformer_block(P, n, x_new, Kn, Vn, want, idx, t, DT, heads, G, stats="cached")

    keep = []
    ns = 80
    vt = np.zeros((B, C, ns), np.float32); vt[:, :, :n_ctx] = Vn.transpose(0, 2, 1)
    Kd, Vd, outd = dev(old[f"{n}.k"], DT), dev(old[f"{n}.v"].transpose(0, 2, 1), DT), dev(old[f"{n}.out"], DT)
    qkv = np.concatenate([P[f"{n}.a1.q.w"], P[f"{n}.a1.k.w"], P[f"{n}.a1.v.w"]], 0)
    d = lambda k: dev(P[f"{n}.{k}"], DT)
    a = fb.fill_args(fb.fise_transformer_args, keep, x=dev(x_new, DT), B=B, H=H, W=W, C=C, G=G, heads=heads,
                     gn_mean=dev(old[f"{n}.gn.mean"]), gn_rstd=dev(old[f"{n}.gn.rstd"]), gn_gamma=d("gn.g"), gn_beta=d("gn.b"),
                     pin_w=d("pin.w"), pin_b=d("pin.b"), ln1_g=d("ln1.g"), ln1_b=d("ln1.b"), qkv_w=dev(qkv, DT), o1_w=d("a1.o.w"),
                     o1_b=d("a1.o.b"), ln2_g=d("ln2.g"), ln2_b=d("ln2.b"), q2_w=d("a2.q.w"), o2_w=d("a2.o.w"), o2_b=d("a2.o.b"),
                     K_ctx=dev(Kn, DT), Vt_ctx=dev(vt, DT), n_ctx=n_ctx, n_ctx_stride=ns, ln3_g=d("ln3.g"), ln3_b=d("ln3.b"),
                     ff1_w=d("ff1.w"), ff1_b=d("ff1.b"), ff2_w=d("ff2.w"), ff2_b=d("ff2.b"), pout_w=d("pout.w"), pout_b=d("pout.b"),
                     K_cache=Kd, Vt_cache=Vd, out_cache=outd, tile_idx=idx_dev(idx), n_active=idx.size, tile=t, stats_fresh=0)
    ws = torch.zeros(fb.fise_masked_transformer_block_workspace_bytes(a), dtype=torch.uint8, device=DEV)
    fb.fise_masked_transformer_block(a, ws)
    act = active_mask(idx, t, H, W)
    av = act.reshape(-1)
    e = check_map(host(outd), want[f"{n}.out"], old[f"{n}.out"], act, TOL[DT], name + " out")
    gK, gV = host(Kd), host(Vd).transpose(0, 2, 1)
    assert rel_err(gK[:, av], want[f"{n}.k"][:, av]) <= TOL[DT] and np.array_equal(gK[:, ~av], old[f"{n}.k"][:, ~av])
    assert rel_err(gV[:, av], want[f"{n}.v"][:, av]) <= TOL[DT] and np.array_equal(gV[:, ~av], old[f"{n}.v"][:, ~av])
    got = host(outd)
    fb.fise_masked_transformer_block(a, ws)
    assert np.array_equal(host(outd), got) and np.array_equal(host(Kd), gK)
    print(f"{name}: out {e:.2e}  update/out rms {np.sqrt(np.mean((want[f'{n}.out'][:, act] - x_new.astype(np.float64)[:, act]) ** 2)):.3f}")
