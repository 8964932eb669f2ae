"""GPU checks of the per-timestep cache ring: with the caches spilled to pinned host memory and streamed through two or
three device slots (whole buffers, or only the part a masked step reads and writes), a session of masked steps gives
bit for bit the stored tensors of the all-resident session; and the cache-moving entry point moves exactly the bytes
its definition names (active tiles, optionally their one-pixel ring, of every map / K row / V^T column), checked
against a mask dilation written out in numpy."""
import numpy as np
import pytest
import torch

from oracle import fise_oracle as fo, fise_unet_oracle as uo
from helpers import DEV, dev, idx_dev, active_mask

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def fb():
    from paper_2305_17423_amd import binding
    binding.lib()
    assert torch.cuda.is_available()
    return binding


def level_of(name, nl):
    """Resolution level of a cache tensor, from its module's place in the walk."""
    p = name.split(".")
    if p[0] == "down":
        return int(p[1]) + (1 if p[2] == "ds" else 0)
    if p[0] == "mid":
        return nl - 1
    if p[0] == "up":
        return nl - 1 - int(p[1]) - (1 if p[2] == "us" else 0)
    return 0            # conv_in.out, eps


def check_move_active(fb, u, d, bt, tiles, halo, where, whats, seed):
    """fise_unet_cache_move_active against the definition written out: dst == src on the named bytes, untouched elsewhere."""
    H, W, B, nl = d["H"], d["W"], d["B"], len(d["mults"])
    cb = fb.fise_unet_cache_bytes(u)
    g = torch.Generator(device="cpu").manual_seed(seed)
    src_h = torch.randint(1, 256, (cb,), dtype=torch.uint8, generator=g)          # no zero byte: a moved byte shows
    idx = idx_dev(tiles)
    ws = torch.zeros(fb.fise_unet_cache_move_workspace_bytes(u), dtype=torch.uint8, device=DEV)
    src = src_h.pin_memory() if where == "host_to_device" else src_h.to(DEV)
    dst = torch.zeros(cb, dtype=torch.uint8, pin_memory=True) if where == "device_to_host" else torch.zeros(cb, dtype=torch.uint8, device=DEV)
    srcn = src_h.numpy()
    for what in whats:
        dst.zero_()
        torch.cuda.synchronize()
        fb.fise_unet_cache_move_active(u, src, dst, idx, tiles.size, bt, halo, what, ws)
        torch.cuda.synchronize()
        got = dst.cpu().numpy()
        want = np.zeros(cb, np.uint8)
        for name, off, nbytes in fb.fise_unet_tensors(u, 1):
            if name.endswith((".mean", ".rstd")):
                continue
            grp = fb.FISE_MOVE_K if name.endswith(".k") else fb.FISE_MOVE_VT if name.endswith(".v") else fb.FISE_MOVE_MAPS
            if not what & grp:
                continue
            l = level_of(name, nl)
            Hl, Wl, t = H >> l, W >> l, bt >> l
            m = active_mask(tiles, t, Hl, Wl)                # same tile grid at every level
            if halo:                                         # one-pixel dilation, clipped to the map
                p = np.pad(m, 1)
                m = np.logical_or.reduce([p[1 + dy:1 + dy + Hl, 1 + dx:1 + dx + Wl] for dy in (-1, 0, 1) for dx in (-1, 0, 1)])
            C = nbytes // (B * Hl * Wl * 2)
            sel = np.zeros((B, C, Hl * Wl, 2), bool) if name.endswith(".v") else np.zeros((B, Hl * Wl, C, 2), bool)
            if name.endswith(".v"):
                sel[:, :, m.reshape(-1)] = True
            else:
                sel[:, m.reshape(-1)] = True
            sel = sel.reshape(-1)
            want[off:off + nbytes][sel] = srcn[off:off + nbytes][sel]
        assert np.array_equal(got, want), f"what={what}: {np.count_nonzero(got != want)} bytes differ"
        assert np.count_nonzero(want) > 0
    return src, dst, idx, ws


def test_cache_move_active_at_sd15_size(fb):
    """The bench's configuration: SD-1.5 shapes, 64x64 latent, 12 of 64 tiles, pinned host memory -> device slot."""
    d = uo.sd15_desc()
    u = fb.fise_unet_create(d)
    tiles = np.array([18, 19, 20, 26, 27, 28, 29, 34, 35, 36, 37, 43], np.int32)
    check_move_active(fb, u, d, 8, tiles, 1, "host_to_device", [fb.FISE_MOVE_MAPS], 29)
    check_move_active(fb, u, d, 8, tiles, 0, "device_to_host", [fb.FISE_MOVE_MAPS | fb.FISE_MOVE_K | fb.FISE_MOVE_VT], 31)
    fb.fise_unet_destroy(u)


@pytest.mark.parametrize("halo", [0, 1])
@pytest.mark.parametrize("where", ["device", "host_to_device", "device_to_host"])
def test_cache_move_active_moves_exactly_the_named_bytes(fb, halo, where):
    d = uo.tiny_desc(H=32, W=32, base=64)
    u = fb.fise_unet_create(d)
    bt = 8
    cb = fb.fise_unet_cache_bytes(u)
    L = fb.fise_unet_cache_layout(u)
    assert 0 == L["maps_off"] < L["kv_off"] == L["maps_bytes"] and L["kv_off"] + L["kv_bytes"] == L["small_off"]
    assert L["small_off"] < L["stored_bytes"] < L["small_off"] + L["small_bytes"] == L["derived_maps_off"]
    assert L["derived_maps_off"] + L["derived_maps_bytes"] == cb
    tiles = np.array([0, 5, 6, 10, 15], np.int32)          # corners (ring clipped at the border), neighbours (rings overlap)
    src, dst, idx, ws = check_move_active(fb, u, d, bt, tiles, halo, where,
                                          (fb.FISE_MOVE_MAPS, fb.FISE_MOVE_K | fb.FISE_MOVE_VT, fb.FISE_MOVE_MAPS | fb.FISE_MOVE_K | fb.FISE_MOVE_VT), 17)
    # nothing to move, and arguments refused before any launch
    dst.zero_(); torch.cuda.synchronize()
    fb.fise_unet_cache_move_active(u, src, dst, idx, 0, bt, halo, fb.FISE_MOVE_MAPS, ws)
    torch.cuda.synchronize()
    assert int(dst.count_nonzero()) == 0
    with pytest.raises(fb.FiseError):
        fb.fise_unet_cache_move_active(u, src, dst, idx, tiles.size, bt, 2, fb.FISE_MOVE_MAPS, ws)
    with pytest.raises(fb.FiseError):
        fb.fise_unet_cache_move_active(u, src, dst, idx, tiles.size, bt, halo, 8, ws)
    with pytest.raises(fb.FiseError):
        fb.fise_unet_cache_move_active(u, src, src, idx, tiles.size, bt, halo, fb.FISE_MOVE_MAPS, ws)
    if where == "device":                                    # pageable host memory is not GPU-addressable: refused
        with pytest.raises(fb.FiseError):
            fb.fise_unet_cache_move_active(u, torch.zeros(cb, dtype=torch.uint8), dst, idx, tiles.size, bt, halo, fb.FISE_MOVE_MAPS, ws)
    fb.fise_unet_destroy(u)


@pytest.mark.parametrize("halo", [0, 1])
@pytest.mark.parametrize("where", ["device", "host_to_device", "device_to_host"])
def test_cache_move_tile_rows_moves_exactly_the_named_rows(fb, halo, where):
    d = uo.tiny_desc(H=32, W=32, base=64)
    u = fb.fise_unet_create(d)
    assert fb.fise_unet_desc_of(u) == {k: (tuple(v) if isinstance(v, (list, tuple)) else v) for k, v in d.items() if k in fb.fise_unet_desc_of(u)}
    H, W, B, bt, nl = d["H"], d["W"], d["B"], 8, len(d["mults"])
    cb = fb.fise_unet_cache_bytes(u)
    g = torch.Generator(device="cpu").manual_seed(23)
    src_h = torch.randint(1, 256, (cb,), dtype=torch.uint8, generator=g)
    src = src_h.pin_memory() if where == "host_to_device" else src_h.to(DEV)
    dst = torch.zeros(cb, dtype=torch.uint8, pin_memory=True) if where == "device_to_host" else torch.zeros(cb, dtype=torch.uint8, device=DEV)
    for ranges in ([(0, 1), (2, 3)], [(1, 2), (3, 4)], [(0, 4)], [(1, 3)]):      # rings that merge at coarse levels, borders, everything
        for what in (fb.FISE_MOVE_MAPS, fb.FISE_MOVE_K, fb.FISE_MOVE_MAPS | fb.FISE_MOVE_K):
            dst.zero_()
            torch.cuda.synchronize()
            fb.fise_unet_cache_move_tile_rows(u, src, dst, ranges, bt, halo, what)
            torch.cuda.synchronize()
            got = dst.cpu().numpy()
            want = np.zeros(cb, np.uint8)
            srcn = src_h.numpy()
            for name, off, nbytes in fb.fise_unet_tensors(u, 1):
                if name.endswith((".mean", ".rstd", ".v")):
                    continue
                if not what & (fb.FISE_MOVE_K if name.endswith(".k") else fb.FISE_MOVE_MAPS):
                    continue
                l = level_of(name, nl)
                Hl, Wl, t = H >> l, W >> l, bt >> l
                rows = np.zeros(Hl, bool)
                for a, b in ranges:
                    rows[max(0, a * t - halo):min(Hl, b * t + halo)] = True
                sel = np.zeros((B, Hl, nbytes // (B * Hl)), bool)
                sel[:, rows] = True
                sel = sel.reshape(-1)
                want[off:off + nbytes][sel] = srcn[off:off + nbytes][sel]
            assert np.array_equal(got, want), f"ranges={ranges} what={what}: {np.count_nonzero(got != want)} bytes differ"
            assert np.count_nonzero(want) > 0
    for bad in ([(1, 1)], [(2, 3), (0, 1)], [(0, 5)], [(0, 2), (1, 3)]):
        with pytest.raises(fb.FiseError):
            fb.fise_unet_cache_move_tile_rows(u, src, dst, bad, bt, halo, fb.FISE_MOVE_MAPS)
    with pytest.raises(fb.FiseError):
        fb.fise_unet_cache_move_tile_rows(u, src, dst, [(0, 1)], bt, halo, fb.FISE_MOVE_VT)
    fb.fise_unet_destroy(u)


@pytest.mark.parametrize("mode", ["whole", "active-host", "active-device", "rows-host", "rows-device"])
@pytest.mark.parametrize("slots,n_steps", [(3, 5), (2, 5), (3, 2), (3, 4), (3, 7)])
def test_host_spill_session_equals_resident_session(fb, slots, n_steps, mode):
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
    spilled = (CacheRing(n_steps, cbytes, DEV, host_spill=True, slots=slots) if mode == "whole" else
               CacheRing(n_steps, cbytes, DEV, host_spill=True, slots=slots, unet=u, kv_home=mode.split("-")[1],
                         transfer="kernel" if mode.startswith("active") else "dma"))
    rings = [CacheRing(n_steps, cbytes, DEV), spilled]
    nmod = len(fb.fise_unet_module_names(u))
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
            r.begin_edit(ix, lists[edit].size, bt)
            for t in range(n_steps):
                c = r.acquire(t)
                if r.trust_derived:
                    fb.fise_masked_unet_step(u, Wd, c, lats[edit], ts[t], kv, ix, lists[edit].size, bt, fb.FISE_STATS_CACHED, None, ws)
                else:       # a slot filled with the active part only: derived maps are recomputed where they are read
                    fb.fise_masked_unet_modules(u, Wd, c, lats[edit], ts[t], kv, ix, lists[edit].size, bt, fb.FISE_STATS_CACHED,
                                                None, 0, nmod, ws)
                r.release(t)
    n_cmp = rings[1].fetch(0).numel()         # whole buffers, or everything but the derived maps
    for t in range(n_steps):
        a, b = rings[0].fetch(t)[:n_cmp], rings[1].fetch(t)
        assert torch.equal(a, b), f"step {t}: spilled session differs from the resident one"
    # the edits changed something, and distinct steps hold distinct caches (no slot mix-up can hide)
    fb.fise_masked_unet_step(u, Wd, tmp, lat, ts[0], kv, full, ntiles, bt, fb.FISE_STATS_FRESH, None, ws)
    torch.cuda.synchronize()
    assert not torch.equal(rings[1].fetch(0), tmp.cpu()[:n_cmp])
    if n_steps > 1:
        assert not torch.equal(rings[1].fetch(0), rings[1].fetch(1))
    fb.fise_unet_destroy(u)
