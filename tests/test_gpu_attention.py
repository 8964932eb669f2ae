"""GPU parity: active-query attention, the masked attention sub-layer and the context K/V projection."""
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


def vt_dev(V, n_stride=None, poison=False):
    """[B, N, C] -> device transposed [B, C, n_stride]; padding columns hold garbage on request."""
    B, N, C = V.shape
    ns = N if n_stride is None else n_stride
    buf = np.zeros((B, C, ns), np.float32)
    if poison:
        buf[:] = np.nan
    buf[:, :, :N] = V.transpose(0, 2, 1)
    return dev(buf, "bf16")


@pytest.mark.parametrize("B,M,N,C,heads", [
    (2, 200, 4096, 320, 8),      # config 3 shape: d = 40, ragged query count
    (2, 64, 1024, 640, 8),       # d = 80
    (1, 37, 256, 1280, 8),       # d = 160
    (2, 33, 77, 320, 8),         # cross-attention: 77 keys (tail block), stride 80
    (2, 16, 64, 32, 4),          # d = 8
    (1, 130, 200, 128, 4),       # d = 32, keys not a multiple of 64
    (1, 1, 8, 64, 4),            # one query, one partial block
])
def test_attention_active(fb, B, M, N, C, heads):
    rng = np.random.default_rng(4000 + M + N)
    q = wl.normal(rng, (B, M, C), 1.0, "bf16"); K = wl.normal(rng, (B, N, C), 1.0, "bf16"); V = wl.normal(rng, (B, N, C), 1.0, "bf16")
    want = fo.attention_active(q, K, V, heads)
    ns = (N + 7) // 8 * 8
    out = torch.zeros((B, M, C), dtype=torch.bfloat16, device=DEV)
    fb.fise_attention_active(dev(q, "bf16"), dev(K, "bf16"), vt_dev(V, ns, poison=True), heads, 1 / math.sqrt(C // heads), out, n_keys=N)
    err = rel_err(host(out), want)
    assert err <= TOL["bf16"], err
    # with scratch the key range may be split over workgroups and merged: same result
    nb = fb.fise_attention_active_workspace_bytes(B, M, N, C, heads)
    ws = torch.full((max(nb, 256),), 0x7F, dtype=torch.uint8, device=DEV)
    out2 = torch.zeros((B, M, C), dtype=torch.bfloat16, device=DEV)
    fb.fise_attention_active(dev(q, "bf16"), dev(K, "bf16"), vt_dev(V, ns, poison=True), heads, 1 / math.sqrt(C // heads), out2, n_keys=N, workspace=ws)
    err2 = rel_err(host(out2), want)
    assert err2 <= TOL["bf16"], err2


def test_attention_closed_forms_on_device(fb):
    rng = np.random.default_rng(4100)
    B, M, N, C, heads = 1, 40, 300, 320, 8
    q = wl.normal(rng, (B, M, C), 1.0, "bf16"); K = wl.normal(rng, (B, N, C), 1.0, "bf16")
    vrow = wl.normal(rng, (1, 1, C), 1.0, "bf16")
    V = np.broadcast_to(vrow, (B, N, C)).copy()
    out = torch.zeros((B, M, C), dtype=torch.bfloat16, device=DEV)
    fb.fise_attention_active(dev(q, "bf16"), dev(K, "bf16"), vt_dev(V, 304), heads, 1 / math.sqrt(40), out, n_keys=N)
    assert rel_err(host(out), np.broadcast_to(vrow, (B, M, C))) < 1e-2          # constant V -> that constant
    # sharply peaked logits: output = V of the matching key
    Kp = np.zeros((1, 64, 64), np.float32); qp = np.zeros((1, 64, 64), np.float32)
    for i in range(64):
        Kp[0, i, i] = 16.0; qp[0, i, i] = 16.0
    Vp = wl.normal(rng, (1, 64, 64), 1.0, "bf16")
    out = torch.zeros((1, 64, 64), dtype=torch.bfloat16, device=DEV)
    fb.fise_attention_active(dev(qp, "bf16"), dev(Kp, "bf16"), vt_dev(Vp), 1, 1 / 8.0, out)
    assert rel_err(host(out), Vp) < 1e-2


@pytest.mark.parametrize("C,heads,H,W,t,frac,cross", [(320, 8, 64, 64, 4, 0.05, False), (320, 8, 64, 64, 4, 0.2, False),
                                                       (320, 8, 64, 64, 4, 0.1, True), (640, 8, 32, 32, 4, 0.1, False),
                                                       (64, 4, 8, 8, 2, 0.3, False)])
def test_masked_attention_layer(fb, C, heads, H, W, t, frac, cross):
    rng = np.random.default_rng(4200 + C + int(frac * 100) + cross)
    B, dt, Dc, n_ctx = 2, "bf16", 768, 77
    x_old = wl.normal(rng, (B, H, W, C), 1.0, dt)
    pixm = wl.ellipse_pixels(rng, H, W, frac)
    x_new = wl.perturb(rng, x_old, pixm, 1.0, dt)
    _, idx = fo.tiles_from_pixels(pixm, t)
    g = wl.normal(rng, (C,), 0.02, dt, mean=1.0); b0 = wl.normal(rng, (C,), 0.02, dt)
    s = 1 / math.sqrt(C)
    wq, wo = wl.normal(rng, (C, C), s, dt), wl.normal(rng, (C, C), s, dt)
    bo = wl.normal(rng, (C,), 0.02, dt)
    full = fo.full_index(H, W, t)
    if cross:
        ctx = wl.normal(rng, (B, n_ctx, Dc), 1.0, dt)
        wk, wv = wl.normal(rng, (C, Dc), 1 / math.sqrt(Dc), dt), wl.normal(rng, (C, Dc), 1 / math.sqrt(Dc), dt)
        Kc, Vc = fo.context_kv(ctx, wk, wv, dt)
        Kd = torch.zeros((B, n_ctx, C), dtype=torch.bfloat16, device=DEV); Vd = torch.zeros((B, C, 80), dtype=torch.bfloat16, device=DEV)
        fb.fise_context_kv(dev(ctx, dt), dev(wk, dt), dev(wv, dt), Kd, Vd)
        assert rel_err(host(Kd), Kc) <= TOL[dt] and rel_err(host(Vd)[:, :, :n_ctx].transpose(0, 2, 1), Vc) <= TOL[dt]
        y_cache = wl.normal(rng, (B, H, W, C), 1.0, dt)
        want = y_cache.astype(np.float64).copy()
        fo.masked_attention_block(x_new, g, b0, wq, None, None, wo, bo, heads, None, None, Kc, Vc, idx, t, want, dt)
        y = dev(y_cache, dt)
        ws = torch.zeros(fb.fise_masked_attention_workspace_bytes(B, C, idx.size, t), dtype=torch.uint8, device=DEV)
        fb.fise_masked_attention(dev(x_new, dt), dev(g, dt), dev(b0, dt), dev(wq, dt), None, None, dev(wo, dt), dev(bo, dt), heads,
                                 None, None, dev(Kc, dt), vt_dev(Vc, 80), n_ctx, idx_dev(idx), idx.size, t, y, ws)
        check_map(host(y), want, y_cache.astype(np.float64), active_mask(idx, t, H, W), TOL[dt], "cross")
        return
    wk, wv = wl.normal(rng, (C, C), s, dt), wl.normal(rng, (C, C), s, dt)
    # caches of the old generation, from the oracle's dense pass
    K0 = np.zeros((B, H * W, C)); V0 = np.zeros((B, H * W, C)); y0 = np.zeros((B, H, W, C))
    fo.masked_attention_block(x_old, g, b0, wq, wk, wv, wo, bo, heads, K0, V0, None, None, full, t, y0, dt)
    Kw, Vw, want = K0.copy(), V0.copy(), y0.copy()
    fo.masked_attention_block(x_new, g, b0, wq, wk, wv, wo, bo, heads, Kw, Vw, None, None, idx, t, want, dt)
    Kd, Vd, y = dev(K0, dt), vt_dev(V0), dev(y0, dt)
    ws = torch.zeros(fb.fise_masked_attention_workspace_bytes(B, C, idx.size, t), dtype=torch.uint8, device=DEV)
    args = (dev(x_new, dt), dev(g, dt), dev(b0, dt), dev(wq, dt), dev(wk, dt), dev(wv, dt), dev(wo, dt), dev(bo, dt), heads,
            Kd, Vd, None, None, 0, idx_dev(idx), idx.size, t, y, ws)
    fb.fise_masked_attention(*args)
    act = active_mask(idx, t, H, W)
    got = host(y)
    check_map(got, want, y0, act, TOL[dt], "self")
    av = act.reshape(-1)
    gK, gV = host(Kd), host(Vd).transpose(0, 2, 1)
    assert rel_err(gK[:, av], Kw[:, av]) <= TOL[dt] and np.array_equal(gK[:, ~av], K0[:, ~av])
    assert rel_err(gV[:, av], Vw[:, av]) <= TOL[dt] and np.array_equal(gV[:, ~av], V0[:, ~av])
    fb.fise_masked_attention(*args)                                             # idempotent (K/V refresh included)
    assert np.array_equal(host(y), got) and np.array_equal(host(Kd), gK)


@pytest.mark.parametrize("C,heads,H,W,t,frac", [(320, 8, 64, 64, 4, 0.10), (320, 8, 64, 64, 4, 0.02), (640, 8, 32, 32, 4, 0.25),
                                                 (1280, 8, 8, 8, 1, 0.3), (64, 4, 8, 8, 2, 0.3)])
def test_keys_restricted_attention_layer(fb, C, heads, H, W, t, frac):
    """Active queries x active keys (no K/V cache): element by element against the oracle, cache kept elsewhere,
    idempotent, full mask == the cached form with every key, empty mask touches nothing.  Also prints how far the
    restricted form is from the full-key form on this synthetic input (information, not a check)."""
    rng = np.random.default_rng(4300 + C + int(frac * 100))
    B, dt = 2, "bf16"
    x_old = wl.normal(rng, (B, H, W, C), 1.0, dt)
    pixm = wl.ellipse_pixels(rng, H, W, frac)
    x_new = wl.perturb(rng, x_old, pixm, 1.0, dt)
    _, idx = fo.tiles_from_pixels(pixm, t)
    full = fo.full_index(H, W, t)
    g = wl.normal(rng, (C,), 0.02, dt, mean=1.0); b0 = wl.normal(rng, (C,), 0.02, dt)
    s = 1 / math.sqrt(C)
    wq, wk, wv, wo = (wl.normal(rng, (C, C), s, dt) for _ in range(4))
    bo = wl.normal(rng, (C,), 0.02, dt)
    y_cache = wl.normal(rng, (B, H, W, C), 1.0, dt)
    want = fo.masked_attention_restricted(x_new, g, b0, wq, wk, wv, wo, bo, heads, idx, t, y_cache.astype(np.float64).copy(), dt)
    y = dev(y_cache, dt)
    ws = torch.full((fb.fise_masked_attention_restricted_workspace_bytes(B, C, full.size, t),), 0xFF, dtype=torch.uint8, device=DEV)
    args = (dev(x_new, dt), dev(g, dt), dev(b0, dt), dev(wq, dt), dev(wk, dt), dev(wv, dt), dev(wo, dt), dev(bo, dt), heads)
    fb.fise_masked_attention_restricted(*args, idx_dev(idx), idx.size, t, y, ws)
    act = active_mask(idx, t, H, W)
    got = host(y)
    e = check_map(got, want, y_cache.astype(np.float64), act, TOL[dt], "keys-restricted")
    fb.fise_masked_attention_restricted(*args, idx_dev(idx), idx.size, t, y, ws)
    assert np.array_equal(host(y), got)                                        # idempotent
    y0 = dev(y_cache, dt)
    fb.fise_masked_attention_restricted(*args, idx_dev(idx), 0, t, y0, ws)
    assert np.array_equal(host(y0), y_cache)                                   # empty mask
    # full mask: every key is active, so this is ordinary attention = the cached form driven with the full list
    Kf = np.zeros((B, H * W, C)); Vf = np.zeros((B, H * W, C))
    wantf = fo.masked_attention_block(x_new, g, b0, wq, wk, wv, wo, bo, heads, Kf, Vf, None, None, full, t, np.zeros((B, H, W, C)), dt)
    yf = torch.zeros((B, H, W, C), dtype=torch.bfloat16, device=DEV)
    fb.fise_masked_attention_restricted(*args, idx_dev(full), full.size, t, yf, ws)
    assert rel_err(host(yf), wantf) <= TOL[dt]
    # information: distance between the two readings at the active positions (full keys from the old generation's cache)
    K0 = np.zeros((B, H * W, C)); V0 = np.zeros((B, H * W, C))
    fo.masked_attention_block(x_old, g, b0, wq, wk, wv, wo, bo, heads, K0, V0, None, None, full, t, np.zeros((B, H, W, C)), dt)
    allk = fo.masked_attention_block(x_new, g, b0, wq, wk, wv, wo, bo, heads, K0, V0, None, None, idx, t, y_cache.astype(np.float64).copy(), dt)
    print(f"C={C} {H}x{W} {idx.size} tiles: device vs oracle {e:.2e}; restricted vs all-keys reading (oracle) "
          f"{rel_err(want[:, act], allk[:, act]):.2e}")
