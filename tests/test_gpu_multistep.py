"""GPU parity over two consecutive masked UNet steps of one edit (the sparse phase of the paper's overview figure:
every remaining denoising step reuses the cache of the same timestep of the previous generation).

Old generation, on the oracle: dense step at t0, deterministic sampler update, dense step at t1 -> one cache per
timestep.  New generation, on both sides from those caches: the latent is perturbed inside a blob, the mask is
detected once, masked step at t0 with the new conditioning, the sampler update applied at active pixels only (the
rest of the latent follows the old trajectory), masked step at t1 on the second cache.  Every stored tensor of both
caches and the intermediate latent are compared with the oracle.  The same two steps are then run with the caches in
pinned host memory, passing through device slots that receive only what a masked step reads: bit-identical results."""
import numpy as np
import pytest
import torch

from oracle import fise_oracle as fo
from oracle import fise_unet_oracle as uo
from paper_2305_17423_amd import workloads as wl
from helpers import (DEV, TOL, dev, rel_err, idx_dev, active_mask, pack_weights, pack_cache, unpack_cache)
from test_gpu_unet import compare_caches

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def fb():
    from paper_2305_17423_amd import binding
    binding.lib()
    assert torch.cuda.is_available()
    return binding


@pytest.mark.parametrize("scratch", ["bf16", "f64"])
def test_two_masked_steps_vs_oracle(fb, scratch, capsys):
    def say(msg):
        with capsys.disabled():
            print(msg, flush=True)
    d = uo.tiny_desc(H=32, W=32, base=64)
    rng = np.random.default_rng(5200)
    P = wl.params_from_shapes(rng, uo.param_shapes(d), 0.04, "bf16")
    B, H, W, bt = d["B"], d["H"], d["W"], 8
    t0, t1 = 600, 580
    a, b = wl.ddim_coeffs(t0, t1)
    ts = [uo.timestep_embedding(np.full(B, float(t)), d["base"]).astype(np.float32) for t in (t0, t1)]
    ctx_old = wl.normal(rng, (B, d["n_ctx"], d["ctx_dim"]), 1.0, "bf16")
    ctx_new = wl.normal(rng, (B, d["n_ctx"], d["ctx_dim"]), 1.0, "bf16")
    kv_old = uo.context_kv_all(P, d, ctx_old, "bf16"); kv_new = uo.context_kv_all(P, d, ctx_new, "bf16")
    shapes = uo.cache_shapes(d)
    # ---- previous generation (oracle): two dense steps, one cache per timestep
    x0 = wl.normal(rng, (B, H, W, d["in_ch"]), 1.0, "bf16")
    eps0, cache0 = uo.unet_dense(P, d, x0, ts[0], kv_old, "bf16", scratch=scratch)
    x1 = fo.round_store(a * x0 + b * eps0, "bf16")
    _, cache1 = uo.unet_dense(P, d, x1, ts[1], kv_old, "bf16", scratch=scratch)
    # ---- the edit: perturbed latent, mask detected once
    pixm = wl.ellipse_pixels(rng, H, W, 0.12)
    x0n = wl.perturb(rng, x0, pixm, 1.0, "bf16")
    _, _, idx = fo.mask_detect(x0, x0n, 0.1, bt)
    ntiles = (H // bt) * (W // bt)
    assert 0 < idx.size < ntiles
    act = active_mask(idx, bt, H, W)
    # oracle: step, update at active pixels, step
    want0 = {k: v.copy() for k, v in cache0.items()}
    e0 = uo.unet_step(P, d, want0, x0n, ts[0], kv_new, idx, bt, "bf16", scratch=scratch)
    x1n = x1.copy()
    x1n[:, act] = fo.round_store(a * np.asarray(x0n, np.float64)[:, act] + b * e0[:, act], "bf16")
    want1 = {k: v.copy() for k, v in cache1.items()}
    uo.unet_step(P, d, want1, x1n, ts[1], kv_new, idx, bt, "bf16", scratch=scratch)

    # ---- device: same two steps from the same two caches, its own eps feeding its own update
    u = fb.fise_unet_create(d)
    Wd = pack_weights(fb, u, P)
    kvd = torch.zeros(fb.fise_unet_ctxkv_bytes(u), dtype=torch.uint8, device=DEV)
    fb.fise_unet_context_kv(u, Wd, dev(ctx_new, "bf16"), kvd)
    ws = torch.zeros(fb.fise_unet_workspace_bytes(u, ntiles, bt), dtype=torch.uint8, device=DEV)
    pm = torch.zeros((H, W), dtype=torch.uint8, device=DEV); tm = torch.zeros(ntiles, dtype=torch.uint8, device=DEV)
    idxd = torch.zeros(ntiles, dtype=torch.int32, device=DEV); nact = torch.zeros(1, dtype=torch.int32, device=DEV)
    x0d, x0nd = dev(x0, "bf16"), dev(x0n, "bf16")
    fb.fise_mask_detect(x0d, x0nd, 0.1, bt, pm, tm, idxd, nact)
    na = int(nact.item())
    assert na == idx.size and np.array_equal(idxd.cpu().numpy()[:na], idx)
    off, nbytes = next((o, n) for nm, o, n in fb.fise_unet_tensors(u, 1) if nm == "eps")
    actd = torch.from_numpy(act).to(DEV)
    nmod = len(fb.fise_unet_module_names(u))

    def run_device(residency):
        """The two steps with both caches resident, or living in pinned host memory and passing through device slots
        that receive only what a masked step reads (K / V^T home in host memory or on the device)."""
        from paper_2305_17423_amd.cache_ring import CacheRing
        c0, c1 = pack_cache(fb, u, cache0, Wd), pack_cache(fb, u, cache1, Wd)
        if residency == "resident":
            ring = CacheRing(2, c0.numel(), DEV)
        else:
            _, home, transfer = residency.split("-")
            ring = CacheRing(2, c0.numel(), DEV, host_spill=True, slots=2, unet=u, kv_home=home, transfer=transfer)
        ring.store(0, c0); ring.store(1, c1)
        del c0, c1
        ring.begin_edit(idxd, na, bt)

        def step(c, lat, t_sin):
            if ring.trust_derived:
                fb.fise_masked_unet_step(u, Wd, c, lat, t_sin, kvd, idxd, na, bt, fb.FISE_STATS_CACHED, None, ws)
            else:       # a slot holds no derived maps: the module walk recomputes them where it reads them
                fb.fise_masked_unet_modules(u, Wd, c, lat, t_sin, kvd, idxd, na, bt, fb.FISE_STATS_CACHED, None, 0, nmod, ws)
        c = ring.acquire(0)
        step(c, x0nd, dev(ts[0]))
        eps_d = c[off:off + nbytes].view(torch.bfloat16).reshape(B, H, W, d["out_ch"]).float()
        x1nd = dev(x1, "bf16").clone()
        upd = (a * x0nd.float() + b * eps_d).to(torch.bfloat16)              # the harness' update, float32 then stored
        x1nd[:, actd] = upd[:, actd]
        ring.release(0)
        c = ring.acquire(1)
        step(c, x1nd, dev(ts[1]))
        ring.release(1)
        g0, g1 = unpack_cache(fb, u, ring.fetch(0), shapes), unpack_cache(fb, u, ring.fetch(1), shapes)
        return g0, g1, x1nd

    got0, got1, x1nd = run_device("resident")
    for residency in ("spill-host-kernel", "spill-device-kernel", "spill-host-dma", "spill-device-dma"):
        s0, s1, sx = run_device(residency)
        assert torch.equal(sx, x1nd), residency
        for k in shapes:
            assert np.array_equal(s0[k], got0[k]), f"{residency}: {k} of the first cache differs from the resident run"
            assert np.array_equal(s1[k], got1[k]), f"{residency}: {k} of the second cache differs from the resident run"
        say(f"{residency}: both caches bit-identical to the resident run")
    torch.cuda.synchronize()

    sm = scratch == "bf16"
    say(f"two steps, oracle scratch={scratch}: first step")
    compare_caches(d, got0, want0, cache0, idx, bt, TOL["bf16"], scratch=sm, say=say, cap=False)
    lat_err = rel_err(x1nd.float().cpu().numpy()[:, act], x1n[:, act])
    assert np.array_equal(x1nd.float().cpu().numpy()[:, ~act], x1[:, ~act])
    say(f"updated latent at active pixels: rel err {lat_err:.3e}")
    # The second step starts from the second timestep's own cache; all it inherits from the first step is the latent,
    # whose deviation (the first step's eps error times the sampler's small eps coefficient) must itself be within
    # the tolerance of a stored tensor.  One branch is charged for it.
    assert lat_err <= TOL["bf16"], f"updated latent: rel err {lat_err:.3e}"
    say("second step")
    compare_caches(d, got1, want1, cache1, idx, bt, TOL["bf16"], scratch=False, start=1, say=say, cap=False)
    # statistics are inputs of the masked steps: untouched in both caches
    for k in shapes:
        if k.endswith((".mean", ".rstd")):
            assert np.array_equal(got0[k], cache0[k].astype(np.float32).astype(np.float64)), k
            assert np.array_equal(got1[k], cache1[k].astype(np.float32).astype(np.float64)), k
    fb.fise_unet_destroy(u)
