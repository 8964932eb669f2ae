"""GPU check of the per-timestep cache ring: with the caches spilled to pinned host memory and streamed through two or
three device slots, a session of masked steps gives bit for bit the caches of the all-resident session."""
import numpy as np
import pytest
import torch

from oracle import fise_oracle as fo, fise_unet_oracle as uo
from helpers import DEV, dev, idx_dev

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def fb():
    from paper_2305_17423_amd import binding
    binding.lib()
    assert torch.cuda.is_available()
    return binding


@pytest.mark.parametrize("slots,n_steps", [(3, 5), (2, 5), (3, 2), (3, 4), (3, 7)])
def test_host_spill_session_equals_resident_session(fb, slots, n_steps):
    from paper_2305_17423_amd.cache_ring import CacheRing
    d = uo.tiny_desc(H=32, W=32, base=64)
    g = torch.Generator(device="cpu").manual_seed(91)
    u = fb.fise_unet_create(d)
    H, W, bt, B = d["H"], d["W"], 8, d["B"]
    ntiles = (H // bt) * (W // bt)
    Wd = (0.04 * torch.randn(fb.fise_unet_weight_elems(u), generator=g)).to(torch.bfloat16).to(DEV)
    lat = torch.randn(B, H, W, d["in_ch"], generator=g).to(torch.bfloat16).to(DEV)
    ctx = torch.randn(B, d["n_ctx"], d["ctx_dim"], generator=g).to(torch.bfloat16).to(DEV)
    ts = [dev(uo.timestep_embedding(np.full(B, 900.0 - 150.0 * t), d["base"]).astype(np.float32)) for t in range(n_steps)]
    kv = torch.zeros(fb.fise_unet_ctxkv_bytes(u), dtype=torch.uint8, device=DEV)
    fb.fise_unet_context_kv(u, Wd, ctx, kv)
    ws = torch.zeros(fb.fise_unet_workspace_bytes(u, ntiles, bt), dtype=torch.uint8, device=DEV)
    full = idx_dev(fo.full_index(H, W, bt))
    cbytes = fb.fise_unet_cache_bytes(u)
    rings = [CacheRing(n_steps, cbytes, DEV), CacheRing(n_steps, cbytes, DEV, host_spill=True, slots=slots)]
    tmp = torch.zeros(cbytes, dtype=torch.uint8, device=DEV)
    for t in range(n_steps):                                  # the previous generation: one dense pass per step
        fb.fise_masked_unet_step(u, Wd, tmp, lat, ts[t], kv, full, ntiles, bt, fb.FISE_STATS_FRESH, None, ws)
        torch.cuda.synchronize()
        for r in rings:
            r.store(t, tmp)
    # two edits in a row over all steps: the second reads what the first wrote back
    lats = [lat.clone(), lat.clone()]
    lats[0][:, 4:13, 9:20, :] += 1.0
    lats[1][:, 16:30, 2:12, :] -= 0.5
    lists = [np.array([1, 2, 5, 6, 9], np.int32), np.array([8, 9, 12, 13], np.int32)]
    for r in rings:
        for edit in range(2):
            ix = idx_dev(lists[edit])
            for t in range(n_steps):
                c = r.acquire(t)
                fb.fise_masked_unet_step(u, Wd, c, lats[edit], ts[t], kv, ix, lists[edit].size, bt, fb.FISE_STATS_CACHED, None, ws)
                r.release(t)
    for t in range(n_steps):
        a, b = rings[0].fetch(t), rings[1].fetch(t)
        assert torch.equal(a, b), f"step {t}: spilled session differs from the resident one"
    # the edits changed something, and distinct steps hold distinct caches (no slot mix-up can hide)
    fb.fise_masked_unet_step(u, Wd, tmp, lat, ts[0], kv, full, ntiles, bt, fb.FISE_STATS_FRESH, None, ws)
    torch.cuda.synchronize()
    assert not torch.equal(rings[1].fetch(0), tmp.cpu())
    if n_steps > 1:
        assert not torch.equal(rings[1].fetch(0), rings[1].fetch(1))
    fb.fise_unet_destroy(u)
