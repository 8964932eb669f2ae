"""GPU parity: masked convolution (scalar float path and bf16 MFMA implicit GEMM) vs the CPU oracle."""
import math
import zlib

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


@pytest.mark.parametrize("seed", [1001, 1002, 1003])
def test_config1_fp32_conv(fb, seed):
    """Single masked conv3x3, fp32, 1x32x32x64 -> 64, mask from fise_mask_detect on the same inputs."""
    rng = np.random.default_rng(seed)
    B, H, W, C, t = 1, 32, 32, 64, 4
    x_old = wl.normal(rng, (B, H, W, C)); w = wl.normal(rng, (C, 3, 3, C), 1 / math.sqrt(576)); bias = np.zeros(C, np.float32)
    x_new = wl.perturb(rng, x_old, wl.rect_pixels(rng, H, W, 8, 8))
    full = fo.full_index(H, W, t)
    cache = np.zeros((B, H, W, C)); fo.masked_conv(x_old, w, bias, full, t, cache, "f32")
    dense_new = np.zeros((B, H, W, C)); fo.masked_conv(x_new, w, bias, full, t, dense_new, "f32")
    _, tm_o, idx_o = fo.mask_detect(x_old, x_new, 0.1, t)
    want = cache.copy(); fo.masked_conv(x_new, w, bias, idx_o, t, want, "f32")
    # device: detect, read n_active back once, convolve
    nt = (H // t) * (W // t)
    pix = torch.zeros((H, W), dtype=torch.uint8, device=DEV); tm = torch.zeros(nt, dtype=torch.uint8, device=DEV)
    idx = torch.zeros(nt, dtype=torch.int32, device=DEV); n = torch.zeros(1, dtype=torch.int32, device=DEV)
    xo, xn, wd, bd = dev(x_old), dev(x_new), dev(w), dev(bias)
    fb.fise_mask_detect(xo, xn, 0.1, t, pix, tm, idx, n)
    na = int(n.item())
    assert na == idx_o.size and 4 <= na <= 9 and np.array_equal(idx.cpu().numpy()[:na], idx_o)
    y = dev(cache)
    fb.fise_masked_conv3x3(xn, wd, bd, 1, idx, na, t, y)
    act = active_mask(idx_o, t, H, W)
    got = host(y)
    check_map(got, want, cache, act, TOL["f32"], "config 1")
    assert rel_err(got[:, act], dense_new[:, act]) <= TOL["f32"]          # == dense conv at active positions
    fb.fise_masked_conv3x3(xn, wd, bd, 1, idx, na, t, y)                  # idempotent
    assert np.array_equal(host(y), got)
    y0 = dev(cache); fb.fise_masked_conv3x3(xn, wd, bd, 1, idx, 0, t, y0)
    assert np.array_equal(host(y0), cache)                                # empty mask -> cache, bit exact
    yf = dev(cache); fb.fise_masked_conv3x3(xn, wd, bd, 1, idx_dev(full), full.size, t, yf)
    assert rel_err(host(yf), dense_new) <= TOL["f32"]                     # full mask == dense


CASES = [
    # name, B, H, W, C0, C1, Cout, k, stride, ups, tile(out), gn, silu, temb, res, frac
    ("c3-320", 2, 32, 32, 320, 0, 320, 3, 1, 0, 8, True, 1, True, True, 0.10),
    ("c3-t4", 2, 32, 32, 64, 0, 96, 3, 1, 0, 4, True, 1, False, True, 0.07),
    ("c3-t2-concat", 2, 16, 16, 64, 32, 64, 3, 1, 0, 2, True, 1, True, False, 0.2),
    ("c3-t1", 1, 8, 8, 128, 64, 128, 3, 1, 0, 1, True, 1, True, True, 0.3),
    ("c1-sc", 2, 16, 16, 96, 32, 64, 1, 1, 0, 4, False, 0, False, False, 0.15),
    ("c1-gn-nosilu", 2, 16, 16, 64, 0, 64, 1, 1, 0, 4, True, 0, False, False, 0.15),
    ("ds", 2, 32, 32, 64, 0, 64, 3, 2, 0, 4, False, 0, False, False, 0.1),
    ("us", 2, 8, 8, 64, 0, 64, 3, 1, 1, 4, False, 0, False, False, 0.1),
    ("narrow-out", 2, 16, 16, 64, 0, 4, 3, 1, 0, 4, True, 1, False, False, 0.2),
    ("ragged-n", 1, 16, 16, 32, 0, 72, 3, 1, 0, 4, False, 0, False, True, 0.1),
    ("scalar-cin4", 2, 16, 16, 4, 0, 32, 3, 1, 0, 4, False, 0, False, False, 0.2),
    ("latent-temb-res", 2, 16, 16, 4, 0, 320, 3, 1, 0, 2, False, 0, True, True, 0.2),          # the 4-channel 3x3 kernel
    ("scalar-cin4-ds", 2, 16, 16, 4, 0, 32, 3, 2, 0, 4, False, 0, False, False, 0.2),          # generic scalar kernel
    ("deep-1280-few-rows", 2, 8, 8, 1280, 1280, 1280, 3, 1, 0, 1, True, 1, True, False, 0.2),     # long K, split over workgroups
    ("deep-16x16", 2, 16, 16, 1280, 640, 1280, 3, 1, 0, 2, True, 1, True, False, 0.2),
    # no prologue and channel counts in multiples of 64: the LDS-direct kernel (zero fill at the borders, two
    # sources, ragged rows and columns, long split K)
    ("direct-concat-temb-res", 2, 16, 16, 64, 128, 192, 3, 1, 0, 2, False, 0, True, True, 0.2),
    ("direct-c1-concat", 2, 16, 16, 128, 64, 64, 1, 1, 0, 4, False, 0, False, True, 0.15),
    ("direct-ragged-n", 1, 16, 16, 64, 0, 72, 3, 1, 0, 4, False, 0, False, True, 0.1),
    ("direct-t1-ragged-rows", 1, 8, 8, 128, 0, 128, 3, 1, 0, 1, False, 0, True, False, 0.3),
    ("direct-deep", 2, 8, 8, 1280, 1280, 1280, 3, 1, 0, 1, False, 0, True, True, 0.2),
    ("direct-ds-concat", 2, 32, 32, 64, 64, 128, 3, 2, 0, 4, False, 0, False, False, 0.1),
    ("direct-us-256", 2, 8, 8, 256, 0, 256, 3, 1, 1, 4, False, 0, False, False, 0.1),
    # rectangular h x w blocks (adaptive block-size selection): LDS-direct, GroupNorm-prologue, scalar and resampling paths
    ("rect-2x8-direct", 2, 16, 16, 64, 64, 128, 3, 1, 0, (2, 8), False, 0, True, True, 0.15),
    ("rect-8x2-gn", 2, 16, 32, 64, 0, 96, 3, 1, 0, (8, 2), True, 1, True, False, 0.15),
    ("rect-4x16-c1", 1, 16, 32, 128, 0, 64, 1, 1, 0, (4, 16), False, 0, False, True, 0.2),
    ("rect-2x4-ds", 2, 32, 32, 64, 0, 64, 3, 2, 0, (2, 4), False, 0, False, False, 0.1),
    ("rect-4x2-us", 2, 8, 8, 64, 0, 64, 3, 1, 1, (4, 2), False, 0, False, False, 0.1),
    ("rect-2x4-latent", 2, 16, 16, 4, 0, 32, 3, 1, 0, (2, 4), False, 0, True, False, 0.2),
    ("rect-4x2-scalar-gn", 1, 8, 16, 8, 0, 12, 3, 1, 0, (4, 2), True, 1, False, True, 0.2),
]


@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
def test_bf16_conv_variants(fb, case):
    name, B, H, W, C0, C1, Co, k, stride, ups, t, use_gn, silu, use_temb, use_res, frac = case
    rng = np.random.default_rng(zlib.crc32(name.encode()))
    dt = "bf16"
    Ci = C0 + C1
    Ho, Wo = (2 * H, 2 * W) if ups else (H // stride, W // stride)
    x0 = wl.normal(rng, (B, H, W, C0), 1.0, dt, mean=0.3)
    x1 = wl.normal(rng, (B, H, W, C1), 1.0, dt) if C1 else None
    w = wl.normal(rng, (Co, k, k, Ci), 1 / math.sqrt(k * k * Ci), dt); bias = wl.normal(rng, (Co,), 0.1, dt)
    gn = None
    if use_gn:
        G = 32 if Ci % 32 == 0 else 4
        mean, rstd = fo.gn_stats([x0, x1] if C1 else x0, G, 1e-5)
        gn = dict(mean=mean, rstd=rstd, gamma=wl.normal(rng, (Ci,), 0.1, dt, mean=1.0), beta=wl.normal(rng, (Ci,), 0.1, dt), groups=G)
    temb = wl.normal(rng, (B, Co), 0.3) if use_temb else None
    res = wl.normal(rng, (B, Ho, Wo, Co), 1.0, dt) if use_res else None
    cache = wl.normal(rng, (B, Ho, Wo, Co), 1.0, dt)
    _, idx = fo.tiles_from_pixels(wl.ellipse_pixels(rng, Ho, Wo, frac), t)
    full = fo.full_index(Ho, Wo, t)
    xs = [x0, x1] if C1 else x0

    def oracle(ix):
        y = cache.astype(np.float64).copy()
        g2 = None
        if gn is not None:
            g2 = dict(gn)
            if not silu:      # normalisation alone: the oracle's fused path always applies SiLU, so pre-normalise here
                xc = np.concatenate([x0, x1], -1).astype(np.float64) if C1 else x0.astype(np.float64)
                gi = np.arange(Ci) // (Ci // gn["groups"])
                xn = (xc - gn["mean"][:, None, None, gi]) * gn["rstd"][:, None, None, gi] * gn["gamma"].astype(np.float64) + gn["beta"].astype(np.float64)
                return fo.masked_conv(xn, w, bias, ix, t, y, dt, stride=stride, upsample=bool(ups), temb=temb, residual=res)
        return fo.masked_conv(xs, w, bias, ix, t, y, dt, stride=stride, upsample=bool(ups), gn=g2, temb=temb, residual=res)

    gnd = None
    if gn is not None:
        gnd = dict(mean=dev(gn["mean"]), rstd=dev(gn["rstd"]), gamma=dev(gn["gamma"], dt), beta=dev(gn["beta"], dt), groups=gn["groups"])
    x0d, x1d, wd, bd = dev(x0, dt), (dev(x1, dt) if C1 else None), dev(w, dt), dev(bias, dt)
    tembd = dev(temb) if use_temb else None
    resd = dev(res, dt) if use_res else None
    th, tw = (t[0], t[1]) if isinstance(t, tuple) else (t, 0)
    for ix in (idx, full, np.zeros(0, np.int32)):
        y = dev(cache, dt)
        a = fb.conv_args(x0d, wd, bd, idx_dev(ix), ix.size, th, y, x1=x1d, ksize=k, stride=stride, upsample=ups, gn=gnd,
                         gn_silu=silu, temb=tembd, residual=resd, tile_w=tw)
        # with the split-K scratch (filled with garbage: the library zeroes what it needs) ...
        ws = torch.full((fb.fise_masked_conv_workspace_bytes(a),), 0xA5, dtype=torch.uint8, device=DEV)
        fb.fise_masked_conv(a, ws)
        got = host(y)
        check_map(got, oracle(ix), cache.astype(np.float64), active_mask(ix, t, Ho, Wo), TOL[dt], f"{name} n={ix.size}")
        fb.fise_masked_conv(a, ws)
        assert np.array_equal(host(y), got), "not idempotent"
        # ... and without it (no K split): same result up to the summation order
        y2 = dev(cache, dt)
        a2 = fb.conv_args(x0d, wd, bd, idx_dev(ix), ix.size, th, y2, x1=x1d, ksize=k, stride=stride, upsample=ups, gn=gnd,
                          gn_silu=silu, temb=tembd, residual=resd, tile_w=tw)
        fb.fise_masked_conv(a2)
        check_map(host(y2), oracle(ix), cache.astype(np.float64), active_mask(ix, t, Ho, Wo), TOL[dt], f"{name} unsplit n={ix.size}")


F32_CASES = [
    # name, B, H, W, Cin, Cout, k, stride, ups, tile(out), temb, res, frac  -- fp32 maps: the tiled float kernel (Cin % 16 == 0,
    # Cout % 4 == 0) and, for the last two, the scalar kernel it falls back to
    ("f32-c3", 2, 16, 16, 32, 64, 3, 1, 0, 4, True, True, 0.2),
    ("f32-ragged-n-rows", 1, 12, 20, 48, 76, 3, 1, 0, 2, False, True, 0.13),
    ("f32-c1-temb", 2, 16, 16, 64, 40, 1, 1, 0, 4, True, False, 0.2),
    ("f32-ds", 2, 16, 16, 16, 32, 3, 2, 0, 2, False, False, 0.2),
    ("f32-us-rect", 1, 8, 8, 32, 32, 3, 1, 1, (4, 2), False, True, 0.15),
    ("f32-wide-n", 1, 8, 8, 16, 200, 3, 1, 0, 1, True, False, 0.3),
    ("f32-scalar-cin12", 1, 8, 8, 12, 16, 3, 1, 0, 2, False, True, 0.3),
    ("f32-scalar-cout6", 1, 8, 8, 16, 6, 3, 1, 0, 2, True, False, 0.3),
]


@pytest.mark.parametrize("case", F32_CASES, ids=[c[0] for c in F32_CASES])
def test_f32_conv_variants(fb, case):
    name, B, H, W, Ci, Co, k, stride, ups, t, use_temb, use_res, frac = case
    rng = np.random.default_rng(zlib.crc32(name.encode()))
    Ho, Wo = (2 * H, 2 * W) if ups else (H // stride, W // stride)
    x = wl.normal(rng, (B, H, W, Ci), 1.0, mean=0.2)
    w = wl.normal(rng, (Co, k, k, Ci), 1 / math.sqrt(k * k * Ci)); bias = wl.normal(rng, (Co,), 0.1)
    temb = wl.normal(rng, (B, Co), 0.3) if use_temb else None
    res = wl.normal(rng, (B, Ho, Wo, Co), 1.0) if use_res else None
    cache = wl.normal(rng, (B, Ho, Wo, Co), 1.0)
    _, idx = fo.tiles_from_pixels(wl.ellipse_pixels(rng, Ho, Wo, frac), t)
    th, tw = (t[0], t[1]) if isinstance(t, tuple) else (t, 0)
    for ix in (idx, fo.full_index(Ho, Wo, t), np.zeros(0, np.int32)):
        want = fo.masked_conv(x, w, bias, ix, t, cache.astype(np.float64).copy(), "f32", stride=stride, upsample=bool(ups), temb=temb, residual=res)
        y = dev(cache)
        a = fb.conv_args(dev(x), dev(w), dev(bias), idx_dev(ix), ix.size, th, y, ksize=k, stride=stride, upsample=ups,
                         temb=dev(temb) if use_temb else None, residual=dev(res) if use_res else None, tile_w=tw)
        fb.fise_masked_conv(a)
        act = active_mask(ix, t, Ho, Wo) if ix.size else np.zeros((Ho, Wo), bool)
        check_map(host(y), want, cache.astype(np.float64), act, TOL["f32"], name)


def test_conv_residual_in_place(fb):
    """residual may alias y_cache (the ResNet shortcut is parked in the output map)."""
    rng = np.random.default_rng(77)
    B, H, W, C, t = 2, 16, 16, 64, 4
    x = wl.normal(rng, (B, H, W, C), 1.0, "bf16"); w = wl.normal(rng, (C, 3, 3, C), 0.05, "bf16"); bias = wl.normal(rng, (C,), 0.1, "bf16")
    cache = wl.normal(rng, (B, H, W, C), 1.0, "bf16")
    _, idx = fo.tiles_from_pixels(wl.ellipse_pixels(rng, H, W, 0.2), t)
    want = cache.astype(np.float64).copy()
    fo.masked_conv(x, w, bias, idx, t, want, "bf16", residual=cache)
    y = dev(cache, "bf16")
    fb.fise_masked_conv3x3(dev(x, "bf16"), dev(w, "bf16"), dev(bias, "bf16"), 1, idx_dev(idx), idx.size, t, y, residual=y)
    check_map(host(y), want, cache.astype(np.float64), active_mask(idx, t, H, W), TOL["bf16"], "in-place residual")


@pytest.mark.parametrize("seed,frac", [(31, 0.02), (32, 0.10), (33, 0.45)])
def test_apsc_selected_blocks_end_to_end(fb, seed, frac):
    """Adaptive block size: block counts on the device, argmin on the host, index list for the chosen h x w blocks,
    convolution on them.  Every stage bit-exact (integers) or within tolerance (conv) of the oracle taking the same steps."""
    rng = np.random.default_rng(seed)
    B, H, W, C, Co, dt = 2, 32, 64, 64, 64, "bf16"
    pix = wl.ellipse_pixels(rng, H, W, frac)
    counts = torch.zeros(25, dtype=torch.int32, device=DEV)
    pixd = torch.from_numpy(pix.astype(np.uint8)).to(DEV)
    fb.fise_apsc_block_counts(pixd, counts)
    h, w_, cost = fb.fise_apsc_select(counts.cpu().tolist())
    assert (h, w_, cost) == fo.apsc_block_size(pix)
    nblk = (H // h) * (W // w_)
    tm = torch.zeros(nblk, dtype=torch.uint8, device=DEV); idx = torch.full((nblk,), -1, dtype=torch.int32, device=DEV)
    n = torch.zeros(1, dtype=torch.int32, device=DEV)
    fb.fise_mask_from_pixels_rect(pixd, h, w_, tm, idx, n)
    tm_o, idx_o = fo.tiles_from_pixels(pix, (h, w_))
    na = int(n.item())
    assert na == idx_o.size and np.array_equal(idx.cpu().numpy()[:na], idx_o) and np.array_equal(tm.cpu().numpy(), tm_o.reshape(-1))
    x = wl.normal(rng, (B, H, W, C), 1.0, dt); wt = wl.normal(rng, (Co, 3, 3, C), 1 / 24, dt); bias = wl.normal(rng, (Co,), 0.1, dt)
    cache = wl.normal(rng, (B, H, W, Co), 1.0, dt)
    want = cache.astype(np.float64).copy()
    fo.masked_conv(x, wt, bias, idx_o, (h, w_), want, dt)
    y = dev(cache, dt)
    a = fb.conv_args(dev(x, dt), dev(wt, dt), dev(bias, dt), idx, na, h, y, tile_w=w_)
    ws = torch.zeros(fb.fise_masked_conv_workspace_bytes(a), dtype=torch.uint8, device=DEV)
    fb.fise_masked_conv(a, ws)
    act = active_mask(idx_o, (h, w_), H, W)
    assert act[pix.astype(bool)].all()                                   # the chosen blocks cover every masked pixel
    check_map(host(y), want, cache.astype(np.float64), act, TOL[dt], f"apsc {h}x{w_}")
