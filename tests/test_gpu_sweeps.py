"""GPU parity on seeded random shapes: masked convolution and active-query attention against the CPU oracle, over
channel counts, kernel sizes, resampling, tile shapes, ragged row / column / key counts that the fixed cases do not list."""
import math

import numpy as np
import pytest
import torch

from oracle import fise_oracle as fo
from paper_2305_17423_amd import workloads as wl
from helpers import DEV, TOL, dev, host, rel_err, idx_dev, active_mask, check_map

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def fb():
    from paper_2305_17423_amd import binding
    binding.lib()
    assert torch.cuda.is_available()
    return binding


def conv_case(seed):
    r = np.random.default_rng(seed)
    k = int(r.choice([1, 3]))
    mode = r.choice(["plain", "plain", "down", "up"]) if k == 3 else "plain"
    th, tw = (int(r.choice([1, 2, 4, 8])),) * 2 if r.random() < 0.6 else (int(r.choice([1, 2, 4, 8])), int(r.choice([2, 4, 8])))
    gy, gx = int(r.integers(1, 5)), int(r.integers(1, 5))             # tile grid of the OUTPUT map
    Ho, Wo = th * gy, tw * gx
    if mode == "down":
        H, W = 2 * Ho, 2 * Wo
    elif mode == "up":
        if Ho % 2 or Wo % 2:
            Ho, Wo, th, tw = 2 * Ho, 2 * Wo, 2 * th, 2 * tw
        H, W = Ho // 2, Wo // 2
    else:
        H, W = Ho, Wo
    C0 = int(r.choice([32, 64, 96, 160, 256]))
    C1 = int(r.choice([0, 0, 32, 64, 128]))
    Co = int(r.choice([8, 40, 64, 72, 136, 320]))
    return dict(seed=seed, k=k, mode=mode, th=th, tw=tw, H=H, W=W, Ho=Ho, Wo=Wo, C0=C0, C1=C1, Co=Co, B=int(r.integers(1, 4)),
                gn=bool(r.random() < 0.4), temb=bool(r.random() < 0.5), res=bool(r.random() < 0.5), frac=float(r.uniform(0.05, 0.9)))


@pytest.mark.parametrize("seed", range(7000, 7020))
def test_conv_random_shapes(fb, seed):
    c = conv_case(seed)
    print(c, flush=True)
    rng = np.random.default_rng(seed + 100000)
    dt, B, k = "bf16", c["B"], c["k"]
    Ci = c["C0"] + c["C1"]
    x0 = wl.normal(rng, (B, c["H"], c["W"], c["C0"]), 1.0, dt, mean=0.2)
    x1 = wl.normal(rng, (B, c["H"], c["W"], c["C1"]), 1.0, dt) if c["C1"] else None
    w = wl.normal(rng, (c["Co"], k, k, Ci), 1 / math.sqrt(k * k * Ci), dt); bias = wl.normal(rng, (c["Co"],), 0.1, dt)
    xs = [x0, x1] if c["C1"] else x0
    gn = None
    if c["gn"]:
        mean, rstd = fo.gn_stats(xs, 32, 1e-5)
        gn = dict(mean=mean, rstd=rstd, gamma=wl.normal(rng, (Ci,), 0.1, dt, mean=1.0), beta=wl.normal(rng, (Ci,), 0.1, dt), groups=32)
    temb = wl.normal(rng, (B, c["Co"]), 0.3) if c["temb"] else None
    res = wl.normal(rng, (B, c["Ho"], c["Wo"], c["Co"]), 1.0, dt) if c["res"] else None
    cache = wl.normal(rng, (B, c["Ho"], c["Wo"], c["Co"]), 1.0, dt)
    tile = (c["th"], c["tw"])
    ntl = (c["Ho"] // c["th"]) * (c["Wo"] // c["tw"])
    idx = np.flatnonzero(rng.random(ntl) < c["frac"]).astype(np.int32)
    if idx.size == 0:
        idx = np.array([ntl - 1], np.int32)
    want = cache.astype(np.float64).copy()
    fo.masked_conv(xs, w, bias, idx, tile, want, dt, stride=2 if c["mode"] == "down" else 1, upsample=c["mode"] == "up", gn=gn,
                   temb=temb, residual=res)
    gnd = None
    if gn is not None:
        gnd = dict(mean=dev(gn["mean"]), rstd=dev(gn["rstd"]), gamma=dev(gn["gamma"], dt), beta=dev(gn["beta"], dt), groups=32)
    y = dev(cache, dt)
    a = fb.conv_args(dev(x0, dt), dev(w, dt), dev(bias, dt), idx_dev(idx), idx.size, c["th"], y, x1=(dev(x1, dt) if c["C1"] else None),
                     ksize=k, stride=2 if c["mode"] == "down" else 1, upsample=int(c["mode"] == "up"), gn=gnd,
                     temb=(dev(temb) if c["temb"] else None), residual=(dev(res, dt) if c["res"] else None), tile_w=c["tw"])
    ws = torch.full((fb.fise_masked_conv_workspace_bytes(a),), 0x5A, dtype=torch.uint8, device=DEV)
    fb.fise_masked_conv(a, ws)
    check_map(host(y), want, cache.astype(np.float64), active_mask(idx, tile, c["Ho"], c["Wo"]), TOL[dt], str(c))


@pytest.mark.parametrize("seed", range(7100, 7116))
def test_attention_random_shapes(fb, seed):
    r = np.random.default_rng(seed)
    heads = int(r.choice([1, 2, 4, 8]))
    d = int(r.choice([8, 16, 24, 40, 64, 80, 96, 128, 160]))
    C = heads * d
    B, M, N = int(r.integers(1, 4)), int(r.integers(1, 300)), int(r.integers(1, 1500))
    ns = (N + 7) // 8 * 8 + 8 * int(r.integers(0, 3))
    print(dict(seed=seed, B=B, M=M, N=N, C=C, heads=heads, d=d, n_stride=ns), flush=True)
    q = wl.normal(r, (B, M, C), 1.0, "bf16"); K = wl.normal(r, (B, N, C), 1.0, "bf16"); V = wl.normal(r, (B, N, C), 1.0, "bf16")
    want = fo.attention_active(q, K, V, heads)
    vt = np.full((B, C, ns), np.nan, np.float32); vt[:, :, :N] = V.transpose(0, 2, 1)
    vtd = dev(vt, "bf16")
    for use_ws in (False, True):
        out = torch.zeros((B, M, C), dtype=torch.bfloat16, device=DEV)
        ws = None
        if use_ws:
            ws = torch.full((max(fb.fise_attention_active_workspace_bytes(B, M, N, C, heads), 256),), 0x7F, dtype=torch.uint8, device=DEV)
        fb.fise_attention_active(dev(q, "bf16"), dev(K, "bf16"), vtd, heads, 1 / math.sqrt(d), out, n_keys=N, workspace=ws)
        err = rel_err(host(out), want)
        assert err <= TOL["bf16"], (err, use_ws)


@pytest.mark.parametrize("seed", range(7200, 7212))
def test_mask_detect_random_shapes(fb, seed):
    """Masks and index lists are integers: bit-exact, for random map shapes, channel counts, tiles and thresholds."""
    r = np.random.default_rng(seed)
    dtype = str(r.choice(["f32", "bf16"]))
    t = int(r.choice([1, 2, 4, 8]))
    B, C = int(r.integers(1, 4)), int(r.choice([1, 3, 4, 5, 32, 70, 320, 333]))
    H, W = t * int(r.integers(1, 20)), t * int(r.integers(1, 20))
    thr = float(r.choice([0.02, 0.1, 0.3]))
    print(dict(seed=seed, dtype=dtype, B=B, H=H, W=W, C=C, tile=t, thr=thr), flush=True)
    x_old = wl.normal(r, (B, H, W, C), 1.0, dtype)
    x_new = wl.perturb(r, x_old, wl.ellipse_pixels(r, H, W, float(r.uniform(0.05, 0.5))), float(r.choice([0.1, 1.0])), dtype)
    pix_o, tm_o, idx_o = fo.mask_detect(x_old, x_new, thr, t)
    nt = (H // t) * (W // t)
    pix = torch.full((H, W), 7, dtype=torch.uint8, device=DEV); tm = torch.full((nt,), 7, dtype=torch.uint8, device=DEV)
    idx = torch.full((nt,), -1, dtype=torch.int32, device=DEV); n = torch.full((1,), -1, dtype=torch.int32, device=DEV)
    fb.fise_mask_detect(dev(x_old, dtype), dev(x_new, dtype), thr, t, pix, tm, idx, n)
    na = int(n.item())
    assert na == idx_o.size
    np.testing.assert_array_equal(pix.cpu().numpy(), pix_o)
    np.testing.assert_array_equal(tm.cpu().numpy().reshape(tm_o.shape), tm_o)
    np.testing.assert_array_equal(idx.cpu().numpy()[:na], idx_o)
    assert (idx.cpu().numpy()[na:] == -1).all()


@pytest.mark.parametrize("seed", range(7300, 7308))
def test_masked_groupnorm_silu_random_shapes(fb, seed):
    r = np.random.default_rng(seed)
    dtype = str(r.choice(["f32", "bf16"]))
    t = int(r.choice([1, 2, 4, 8]))
    G = int(r.choice([1, 4, 32]))
    C = G * int(r.choice([1, 2, 5, 8, 10]))
    if dtype == "bf16":
        C = (C + 7) // 8 * 8
        if C % G:
            G = 1
    B, H, W = int(r.integers(1, 4)), t * int(r.integers(1, 9)), t * int(r.integers(1, 9))
    print(dict(seed=seed, dtype=dtype, B=B, H=H, W=W, C=C, G=G, tile=t), flush=True)
    x = wl.normal(r, (B, H, W, C), 1.5, dtype)
    g = wl.normal(r, (C,), 0.1, dtype, mean=1.0); bt = wl.normal(r, (C,), 0.1, dtype)
    mean, rstd = fo.gn_stats(wl.normal(r, (B, H, W, C), 1.5, dtype), G, 1e-5)
    cache = wl.normal(r, (B, H, W, C), 1.0, dtype)
    nt = (H // t) * (W // t)
    idx = np.flatnonzero(r.random(nt) < 0.4).astype(np.int32)
    want = cache.astype(np.float64).copy()
    fo.masked_gn_silu(x, mean, rstd, g, bt, G, idx, t, want, dtype)
    y = dev(cache, dtype)
    fb.fise_masked_groupnorm_silu(dev(x, dtype), dev(mean), dev(rstd), dev(g, dtype), dev(bt, dtype), G, idx_dev(idx), idx.size, t, y)
    check_map(host(y), want, cache.astype(np.float64), active_mask(idx, t, H, W), TOL[dtype], f"seed {seed}")
