"""GPU parity: the masked UNet step vs the CPU oracle on a small instance of the architecture
(element by element), and structural properties at the full SD-1.5 shape."""
import numpy as np
import pytest
import torch

from oracle import fise_oracle as fo
from oracle import fise_unet_oracle as uo
from paper_2305_17423_amd import workloads as wl
from helpers import (DEV, TOL, dev, host, rel_err, rel_l2, idx_dev, active_mask, pack_weights, pack_cache, unpack_cache,
                     chain_l2_bound, branch_depths, DRIFT_MAX_OVER_L2, SCRATCH_FLAT_STAGES)

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def fb():
    from paper_2305_17423_amd import binding
    binding.lib()
    assert torch.cuda.is_available()
    return binding


def problem(d, seed, std):
    rng = np.random.default_rng(seed)
    P = wl.params_from_shapes(rng, uo.param_shapes(d), std, "bf16")
    lat = wl.normal(rng, (d["B"], d["H"], d["W"], d["in_ch"]), 1.0, "bf16")
    ctx_old = wl.normal(rng, (d["B"], d["n_ctx"], d["ctx_dim"]), 1.0, "bf16")
    ctx_new = wl.normal(rng, (d["B"], d["n_ctx"], d["ctx_dim"]), 1.0, "bf16")
    t_sin = uo.timestep_embedding(np.full(d["B"], 481.0), d["base"]).astype(np.float32)
    return rng, P, lat, ctx_old, ctx_new, t_sin


def stored_maps(d):
    for m in uo.unet_modules(d):
        names = {"res": ["h1", "out"], "tr": ["out", "k", "v"], "ds": ["out"], "us": ["out"], "conv_in": ["out"]}.get(m["kind"], [])
        for s in names:
            yield m, f"{m['name']}.{s}"
    yield uo.unet_modules(d)[-1], "eps"


# One call of the whole step chains ~200 products (116 normalised branches) whose operands the device rounds to bf16, so
# the device and the float64 oracle drift apart with depth (helpers.py states the law and where it comes from).  Every
# stored tensor is held
#   * in relative L2 to min(tol, 3.0e-3 * sqrt(branches upstream)); cap=False holds it to the law alone, for passes
#     whose inputs already carry drift: a second step on an updated cache, and dense passes with FRESH statistics
#     (every GroupNorm's mean and rstd are then recomputed from maps that have drifted, which feeds the drift back
#     into every later branch: measured up to 2.7e-3 per sqrt(branch) there, 2.0e-2 at 62 branches),
#   * elementwise to max(tol, 10 x its own relative L2): the difference is noise of the drift's size everywhere, never
#     an isolated wrong element (a bad halo or tile edge is wrong by O(1)),
#   * bitwise at every position the step may not write.
# scratch=True: `want` comes from the oracle's bf16-operand mode, which follows the device's own roundings for the
# first modules: tensors up to SCRATCH_FLAT_STAGES branches deep are then held to the plain elementwise tolerance.
def compare_caches(d, got, want, before, idx, bt, tol, scratch=False, start=0, say=None, cap=True):
    depth = branch_depths(uo.unet_modules(d), start)
    worst_e, worst_l = ("", 0.0, 1.0), ("", 0.0, 1.0)          # name, value, bound
    for m, name in stored_maps(d):
        H, W = d["H"] >> m["lvl"], d["W"] >> m["lvl"]
        act = active_mask(idx, bt >> m["lvl"], H, W)
        g, w_, b_ = got[name], want[name], before[name]
        if g.ndim == 3:                                   # K / V caches [B, N, C]
            act = act.reshape(-1)
        err, l2 = rel_err(g[:, act], w_[:, act]), rel_l2(g[:, act], w_[:, act])
        n = depth[name]
        l2_bound = chain_l2_bound(n, tol, cap)
        e_bound = tol if (scratch and n <= SCRATCH_FLAT_STAGES) else max(tol, DRIFT_MAX_OVER_L2 * l2)
        if err / e_bound > worst_e[1] / worst_e[2]:
            worst_e = (name, err, e_bound)
        if l2 / l2_bound > worst_l[1] / worst_l[2]:
            worst_l = (name, l2, l2_bound)
        assert l2 <= l2_bound, f"{name}: relative L2 error {l2:.3e} > {l2_bound:.3e} ({n} branches upstream)"
        assert err <= e_bound, f"{name}: elementwise rel err {err:.3e} > {e_bound:.3e} ({n} branches upstream, L2 {l2:.3e})"
        assert np.array_equal(g[:, ~act], b_[:, ~act]), f"{name}: inactive positions changed"
    (say or print)(f"closest to its bound: elementwise {worst_e[0]} {worst_e[1]:.3e} (bound {worst_e[2]:.3e}); "
                   f"relative L2 {worst_l[0]} {worst_l[1]:.3e} (bound {worst_l[2]:.3e})")
    return worst_e, worst_l


@pytest.mark.parametrize("seed", [5001, 5002])
def test_tiny_unet_step_vs_oracle(fb, seed):
    d = uo.tiny_desc(H=32, W=32, base=64)          # 64..256 channels: enough terms per sum for the bf16 bar
    rng, P, lat, ctx_old, ctx_new, t_sin = problem(d, seed, 0.04)
    H, W, bt = d["H"], d["W"], 8
    shapes = uo.cache_shapes(d)
    kv_old = uo.context_kv_all(P, d, ctx_old, "bf16"); kv_new = uo.context_kv_all(P, d, ctx_new, "bf16")
    _, cache_old = uo.unet_dense(P, d, lat, t_sin, kv_old, "bf16")

    u = fb.fise_unet_create(d)
    Wd = pack_weights(fb, u, P)
    kvd_old = torch.zeros(fb.fise_unet_ctxkv_bytes(u), dtype=torch.uint8, device=DEV); kvd_new = torch.zeros_like(kvd_old)
    fb.fise_unet_context_kv(u, Wd, dev(ctx_old, "bf16"), kvd_old); fb.fise_unet_context_kv(u, Wd, dev(ctx_new, "bf16"), kvd_new)
    ntiles = (H // bt) * (W // bt)
    ws = torch.zeros(fb.fise_unet_workspace_bytes(u, ntiles, bt), dtype=torch.uint8, device=DEV)
    tsd = dev(t_sin)
    full = fo.full_index(H, W, bt)

    # (1) dense forward on the device (full list, fresh statistics, zero cache) vs the oracle's dense walk
    cd = torch.zeros(fb.fise_unet_cache_bytes(u), dtype=torch.uint8, device=DEV)
    fb.fise_masked_unet_step(u, Wd, cd, dev(lat, "bf16"), tsd, kvd_old, idx_dev(full), full.size, bt, fb.FISE_STATS_FRESH, None, ws)
    got = unpack_cache(fb, u, cd, shapes)
    zero = {k: np.zeros_like(v) for k, v in cache_old.items()}
    worst = compare_caches(d, got, cache_old, zero, full, bt, TOL["bf16"], cap=False)       # recomputed statistics: the law alone
    # statistics of the first GroupNorms see (almost) identical inputs; deeper ones inherit the drift above
    for k in ("down.0.res.0.gn1", "down.0.res.0.gn2", "down.0.tr.0.gn"):
        assert np.abs(got[k + ".mean"] - cache_old[k + ".mean"]).max() < 5e-3, k
        assert rel_err(got[k + ".rstd"], cache_old[k + ".rstd"]) < 5e-3, k
    for k in shapes:
        if k.endswith(".rstd"):
            assert rel_l2(got[k], cache_old[k]) < 2e-2, k

    # (2) masked step from the ORACLE's cache (both sides start from identical state)
    pixm = wl.rect_pixels(rng, H, W, 5, 6)
    lat_new = wl.perturb(rng, lat, pixm, 1.0, "bf16")
    _, _, idx = fo.mask_detect(lat, lat_new, 0.1, bt)
    assert 0 < idx.size < ntiles
    want = {k: v.copy() for k, v in cache_old.items()}
    uo.unet_step(P, d, want, lat_new, t_sin, kv_new, idx, bt, "bf16")
    cm = pack_cache(fb, u, cache_old, Wd)
    fb.fise_masked_unet_step(u, Wd, cm, dev(lat_new, "bf16"), tsd, kvd_new, idx_dev(idx), idx.size, bt, fb.FISE_STATS_CACHED, None, ws)
    got = unpack_cache(fb, u, cm, shapes)
    compare_caches(d, got, want, cache_old, idx, bt, TOL["bf16"])
    for k in shapes:
        if k.endswith((".mean", ".rstd")):
            assert np.array_equal(got[k], cache_old[k].astype(np.float32).astype(np.float64)), k   # cached statistics untouched
    # (3) idempotent; (4) empty mask leaves every byte alone
    snap = cm.clone()
    fb.fise_masked_unet_step(u, Wd, cm, dev(lat_new, "bf16"), tsd, kvd_new, idx_dev(idx), idx.size, bt, fb.FISE_STATS_CACHED, None, ws)
    assert torch.equal(cm, snap)
    fb.fise_masked_unet_step(u, Wd, cm, dev(lat, "bf16"), tsd, kvd_old, idx_dev(idx), 0, bt, fb.FISE_STATS_CACHED, None, ws)
    assert torch.equal(cm, snap)
    # (5) per-level dense override
    want2 = {k: v.copy() for k, v in cache_old.items()}
    ld = [False, False, True, True]
    uo.unet_step(P, d, want2, lat_new, t_sin, kv_new, idx, bt, "bf16", level_dense=ld)
    c5 = pack_cache(fb, u, cache_old, Wd)
    fb.fise_masked_unet_step(u, Wd, c5, dev(lat_new, "bf16"), tsd, kvd_new, idx_dev(idx), idx.size, bt, fb.FISE_STATS_CACHED, ld, ws)
    got5 = unpack_cache(fb, u, c5, shapes)
    assert rel_l2(got5["eps"], want2["eps"]) <= TOL["bf16"] and rel_l2(got5["mid.tr.0.out"], want2["mid.tr.0.out"]) <= TOL["bf16"]
    fb.fise_unet_destroy(u)


ARCHS = [
    ("two-levels-nonsquare", dict(base=64, mults=(1, 2), attn=(True, False), layers=1, heads=2, ctx_dim=64, n_ctx=7, H=16, W=24, B=1), 2),
    ("three-levels-batch3", dict(base=32, mults=(1, 1, 2), attn=(False, True, True), layers=2, heads=4, ctx_dim=64, n_ctx=20, H=24, W=16, B=3), 4),
    ("four-levels-8ch-latent", dict(in_ch=8, out_ch=8, base=32, mults=(1, 2, 2, 4), attn=(True, False, True, True), layers=1, heads=4,
                                    ctx_dim=96, n_ctx=77, H=32, W=32, B=2), 8),
]


@pytest.mark.parametrize("tiles", [[0], [3, 12, 15], [1, 4, 7, 13], [5, 10], list(range(16))],
                         ids=["corner", "three-corners", "edges", "diagonal-neighbours", "all-tiles-cached-stats"])
def test_tiny_unet_masks_at_the_border(fb, tiles):
    """Tile lists chosen for their geometry, not drawn: tiles in the corners and on the edges of the map (the ring of
    every level is clipped by the zero padding there, down to the 1x1 tiles of the coarsest level), tiles that touch
    only at a corner (each other's ring), and the full list under cached statistics."""
    d = uo.tiny_desc(H=32, W=32, base=64)
    rng, P, lat, ctx_old, ctx_new, t_sin = problem(d, 5050, 0.04)
    H, W, bt = d["H"], d["W"], 8
    shapes = uo.cache_shapes(d)
    kv_old = uo.context_kv_all(P, d, ctx_old, "bf16"); kv_new = uo.context_kv_all(P, d, ctx_new, "bf16")
    _, cache_old = uo.unet_dense(P, d, lat, t_sin, kv_old, "bf16")
    idx = np.asarray(tiles, np.int32)
    act = active_mask(idx, bt, H, W)
    lat_new = np.asarray(lat, np.float64).copy()
    lat_new[:, act] += rng.standard_normal(lat_new[:, act].shape)          # the whole active area changes
    lat_new = fo.round_store(lat_new, "bf16")
    want = {k: v.copy() for k, v in cache_old.items()}
    uo.unet_step(P, d, want, lat_new, t_sin, kv_new, idx, bt, "bf16")
    u = fb.fise_unet_create(d)
    Wd = pack_weights(fb, u, P)
    kvd = torch.zeros(fb.fise_unet_ctxkv_bytes(u), dtype=torch.uint8, device=DEV)
    fb.fise_unet_context_kv(u, Wd, dev(ctx_new, "bf16"), kvd)
    ws = torch.zeros(fb.fise_unet_workspace_bytes(u, 16, bt), dtype=torch.uint8, device=DEV)
    cm = pack_cache(fb, u, cache_old, Wd)
    fb.fise_masked_unet_step(u, Wd, cm, dev(lat_new, "bf16"), dev(t_sin), kvd, idx_dev(idx), idx.size, bt, fb.FISE_STATS_CACHED, None, ws)
    # With the full list nothing a branch reads is an exact cached value any more (no untouched ring, no untouched
    # keys and values to dilute the drift), as in a dense pass: that case is held to the drift law alone.
    compare_caches(d, unpack_cache(fb, u, cm, shapes), want, cache_old, idx, bt, TOL["bf16"], cap=idx.size < 16)
    fb.fise_unet_destroy(u)


@pytest.mark.parametrize("name,over,bt", ARCHS, ids=[a[0] for a in ARCHS])
def test_other_architectures_vs_oracle(fb, name, over, bt):
    """The plan is parametric: other depths, widths, attention placements, head counts, context sizes, batch sizes
    and non-square latents, dense forward and masked step against the oracle's walk of the same description."""
    d = uo.sd15_desc(**over)
    rng, P, lat, ctx_old, ctx_new, t_sin = problem(d, 5100 + bt, 0.05)
    H, W = d["H"], d["W"]
    shapes = uo.cache_shapes(d)
    kv_old = uo.context_kv_all(P, d, ctx_old, "bf16"); kv_new = uo.context_kv_all(P, d, ctx_new, "bf16")
    _, cache_old = uo.unet_dense(P, d, lat, t_sin, kv_old, "bf16")
    u = fb.fise_unet_create(d)
    assert fb.fise_unet_module_names(u) == [m["name"] for m in uo.unet_modules(d)]
    Wd = pack_weights(fb, u, P)
    kvd_old = torch.zeros(fb.fise_unet_ctxkv_bytes(u), dtype=torch.uint8, device=DEV); kvd_new = torch.zeros_like(kvd_old)
    fb.fise_unet_context_kv(u, Wd, dev(ctx_old, "bf16"), kvd_old); fb.fise_unet_context_kv(u, Wd, dev(ctx_new, "bf16"), kvd_new)
    ntiles = (H // bt) * (W // bt)
    ws = torch.zeros(fb.fise_unet_workspace_bytes(u, ntiles, bt), dtype=torch.uint8, device=DEV)
    tsd = dev(t_sin)
    full = fo.full_index(H, W, bt)
    cd = torch.zeros(fb.fise_unet_cache_bytes(u), dtype=torch.uint8, device=DEV)
    fb.fise_masked_unet_step(u, Wd, cd, dev(lat, "bf16"), tsd, kvd_old, idx_dev(full), full.size, bt, fb.FISE_STATS_FRESH, None, ws)
    zero = {k: np.zeros_like(v) for k, v in cache_old.items()}
    compare_caches(d, unpack_cache(fb, u, cd, shapes), cache_old, zero, full, bt, TOL["bf16"], cap=False)
    lat_new = wl.perturb(rng, lat, wl.rect_pixels(rng, H, W, 5, 7), 1.0, "bf16")
    _, _, idx = fo.mask_detect(lat, lat_new, 0.1, bt)
    assert 0 < idx.size < ntiles
    want = {k: v.copy() for k, v in cache_old.items()}
    uo.unet_step(P, d, want, lat_new, t_sin, kv_new, idx, bt, "bf16")
    cm = pack_cache(fb, u, cache_old, Wd)
    fb.fise_masked_unet_step(u, Wd, cm, dev(lat_new, "bf16"), tsd, kvd_new, idx_dev(idx), idx.size, bt, fb.FISE_STATS_CACHED, None, ws)
    compare_caches(d, unpack_cache(fb, u, cm, shapes), want, cache_old, idx, bt, TOL["bf16"])
    fb.fise_unet_destroy(u)


def test_tiny_unet_full_mask_fresh_equals_dense_of_new_inputs(fb):
    d = uo.tiny_desc()
    rng, P, lat, ctx_old, ctx_new, t_sin = problem(d, 5003, 0.08)
    H, W, bt = d["H"], d["W"], 8
    shapes = uo.cache_shapes(d)
    kv_old = uo.context_kv_all(P, d, ctx_old, "bf16"); kv_new = uo.context_kv_all(P, d, ctx_new, "bf16")
    _, cache_old = uo.unet_dense(P, d, lat, t_sin, kv_old, "bf16")
    lat_new = wl.perturb(rng, lat, wl.rect_pixels(rng, H, W, 7, 7), 1.0, "bf16")
    eps_new, cache_new = uo.unet_dense(P, d, lat_new, t_sin, kv_new, "bf16")
    u = fb.fise_unet_create(d)
    Wd = pack_weights(fb, u, P)
    kvd = torch.zeros(fb.fise_unet_ctxkv_bytes(u), dtype=torch.uint8, device=DEV)
    fb.fise_unet_context_kv(u, Wd, dev(ctx_new, "bf16"), kvd)
    full = fo.full_index(H, W, bt)
    ws = torch.zeros(fb.fise_unet_workspace_bytes(u, full.size, bt), dtype=torch.uint8, device=DEV)
    cm = pack_cache(fb, u, cache_old, Wd)
    fb.fise_masked_unet_step(u, Wd, cm, dev(lat_new, "bf16"), dev(t_sin), kvd, idx_dev(full), full.size, bt, fb.FISE_STATS_FRESH, None, ws)
    got = unpack_cache(fb, u, cm, shapes)
    assert rel_l2(got["eps"], cache_new["eps"]) <= TOL["bf16"]
    fb.fise_unet_destroy(u)


# ---------------------------------------------------------------------------
# One module at a time: before module i runs, the device cache is made identical to the oracle's
# state, so every module of the real plan (weight offsets, skip wiring, stacked time projections,
# per-level tile geometry) is held to the elementwise bar without chain drift.
# ---------------------------------------------------------------------------
def module_tensors(m):
    return {"res": ["h1", "out"], "tr": ["k", "v", "out"], "ds": ["out"], "us": ["out"], "conv_in": ["out"], "out": []}[m["kind"]]


def upload_tensor(fb, layout, buf, name, arr):
    off, nbytes = layout[name]
    a = np.asarray(arr, np.float32)
    if name.endswith(".v"):
        a = a.transpose(0, 2, 1)
    t = torch.from_numpy(np.ascontiguousarray(a)).to(torch.bfloat16).view(torch.uint8).reshape(-1)
    assert t.numel() == nbytes
    buf[off:off + nbytes] = t.to(DEV)


def download_tensor(layout, buf, name, shape):
    off, nbytes = layout[name]
    raw = buf[off:off + nbytes].to("cpu").view(torch.bfloat16)
    if name.endswith(".v"):
        return raw.reshape(shape[0], shape[2], shape[1]).to(torch.float64).numpy().transpose(0, 2, 1)
    return raw.reshape(shape).to(torch.float64).numpy()


def run_module_by_module(fb, d, seed, std, bt, frac, say, tol=TOL["bf16"], scratch="f64"):
    rng, P, lat, ctx_old, ctx_new, t_sin = problem(d, seed, std)
    H, W = d["H"], d["W"]
    shapes = uo.cache_shapes(d)
    mods = uo.unet_modules(d)
    kv_old = uo.context_kv_all(P, d, ctx_old, "bf16"); kv_new = uo.context_kv_all(P, d, ctx_new, "bf16")
    say(f"oracle: dense pass of the old generation, {len(mods)} modules")
    cache_old = uo.empty_cache(d)
    full = fo.full_index(H, W, bt)
    for mi in range(len(mods)):
        uo.unet_step(P, d, cache_old, lat, t_sin, kv_old, full, bt, "bf16", stats="fresh", only={mi})
        if mi % 8 == 7:
            say(f"  dense module {mi + 1}/{len(mods)}")
    pixm = wl.ellipse_pixels(rng, H, W, frac)
    lat_new = wl.perturb(rng, lat, pixm, 1.0, "bf16")
    _, _, idx = fo.mask_detect(lat, lat_new, 0.1, bt)
    ntiles = full.size
    assert 0 < idx.size < ntiles

    u = fb.fise_unet_create(d)
    assert fb.fise_unet_module_names(u) == [m["name"] for m in mods]
    Wd = pack_weights(fb, u, P)
    kvd = torch.zeros(fb.fise_unet_ctxkv_bytes(u), dtype=torch.uint8, device=DEV)
    fb.fise_unet_context_kv(u, Wd, dev(ctx_new, "bf16"), kvd)
    ws = torch.zeros(fb.fise_unet_workspace_bytes(u, ntiles, bt), dtype=torch.uint8, device=DEV)
    layout = {n: (off, nb) for n, off, nb in fb.fise_unet_tensors(u, 1)}
    cm = pack_cache(fb, u, cache_old, Wd)
    chain = cm.clone()
    latd, tsd, idxd = dev(lat_new, "bf16"), dev(t_sin), idx_dev(idx)
    want = {k: v.copy() for k, v in cache_old.items()}
    worst = ("", 0.0)
    for mi, m in enumerate(mods):
        uo.unet_step(P, d, want, lat_new, t_sin, kv_new, idx, bt, "bf16", only={mi}, scratch=scratch)
        fb.fise_masked_unet_modules(u, Wd, cm, latd, tsd, kvd, idxd, idx.size, bt, fb.FISE_STATS_CACHED, None, mi, 1, ws)
        names = [f"{m['name']}.{s}" for s in module_tensors(m)] or ["eps"]
        act = active_mask(idx, bt >> m["lvl"], H >> m["lvl"], W >> m["lvl"])
        for name in names:
            g = download_tensor(layout, cm, name, shapes[name])
            a = act.reshape(-1) if g.ndim == 3 else act
            err = rel_err(g[:, a], want[name][:, a])
            assert err <= tol, f"module {mi} {name}: rel err {err:.3e}"
            assert np.array_equal(g[:, ~a], cache_old[name][:, ~a]), f"module {mi} {name}: inactive positions changed"
            if err > worst[1]:
                worst = (name, err)
            upload_tensor(fb, layout, cm, name, want[name])            # device state := oracle state
        if mi % 8 == 7:
            say(f"  masked module {mi + 1}/{len(mods)} ok, worst so far {worst}")
    say(f"module-by-module worst elementwise rel err: {worst}")
    # the whole chain in one call, from the same starting cache: against the oracle's default mode and against its
    # bf16-operand mode (compare_caches states what each is held to)
    fb.fise_masked_unet_step(u, Wd, chain, latd, tsd, kvd, idxd, idx.size, bt, fb.FISE_STATS_CACHED, None, ws)
    got = unpack_cache(fb, u, chain, shapes)
    for mode in ("f64", "bf16"):
        ref = {k: v.copy() for k, v in cache_old.items()}
        for mi in range(len(mods)):
            uo.unet_step(P, d, ref, lat_new, t_sin, kv_new, idx, bt, "bf16", only={mi}, scratch=mode)
        say(f"whole chain vs oracle with scratch={mode}: eps L2 {rel_l2(got['eps'], ref['eps']):.3e}")
        compare_caches(d, got, ref, cache_old, idx, bt, TOL["bf16"], scratch=(mode == "bf16"), say=say)
    fb.fise_unet_destroy(u)


def test_tiny_unet_module_by_module(fb, capsys):
    def say(msg):
        with capsys.disabled():
            print(msg, flush=True)
    # 64..256 channels: sums of a few hundred terms.  Rounding the GEMM inputs to bf16 (which any bf16 MFMA path must do
    # and the float64 oracle's default mode does not) already moves single outputs of this instance by 2.05e-2 of the
    # metric (tests/test_oracle_unet.py::test_bf16_operand_rounding_alone shows it on the CPU), so the small instance
    # is teacher-forced against the oracle's bf16-operand mode, at the stated 2e-2; the SD-1.5 instance below is
    # teacher-forced against the default mode at the same 2e-2.
    run_module_by_module(fb, uo.tiny_desc(H=32, W=32, base=64), 5010, 0.04, 8, 0.1, say, scratch="bf16")


def test_sd15_unet_module_by_module(fb, capsys):
    """Config 5 at full size: SD-1.5 widths, 64x64 latent, batch 2, 10 % blob, 8x8 base tiles.
    The oracle needs about two minutes of CPU for its dense and masked passes."""
    def say(msg):
        with capsys.disabled():
            print(msg, flush=True)
    run_module_by_module(fb, uo.sd15_desc(), 5020, 0.02, 8, 0.1, say)


def test_sd15_96x96_unet_module_by_module(fb, capsys):
    """The same check at the latent size of 768x768 images: SD-1.5 widths, 96x96 latent (144 tiles of 8x8; levels
    96 / 48 / 24 / 12, none a power of two), batch 2, 10 % blob.  Every module of the plan against the oracle, its
    inputs identical on both sides."""
    def say(msg):
        with capsys.disabled():
            print(msg, flush=True)
    run_module_by_module(fb, uo.sd15_desc(H=96, W=96), 5030, 0.02, 8, 0.1, say)


def test_masked_step_under_graph_capture(fb):
    """The step allocates nothing, clears nothing with a memset node and never synchronises, so a caller can capture
    it into a HIP graph.  Each replay (with eager work and synchronisations of the test in between, and the cache
    reset to its state before the step) must reproduce the eager result bit for bit."""
    d = uo.tiny_desc(H=32, W=32, base=64)
    g = torch.Generator(device="cpu").manual_seed(77)
    u = fb.fise_unet_create(d)
    H, W, bt, B = d["H"], d["W"], 8, d["B"]
    ntiles = (H // bt) * (W // bt)
    Wd = (0.04 * torch.randn(fb.fise_unet_weight_elems(u), generator=g)).to(torch.bfloat16).to(DEV)
    lat = torch.randn(B, H, W, d["in_ch"], generator=g).to(torch.bfloat16).to(DEV)
    ctx = torch.randn(B, d["n_ctx"], d["ctx_dim"], generator=g).to(torch.bfloat16).to(DEV)
    tsd = dev(uo.timestep_embedding(np.full(B, 300.0), d["base"]).astype(np.float32))
    kv = torch.zeros(fb.fise_unet_ctxkv_bytes(u), dtype=torch.uint8, device=DEV)
    fb.fise_unet_context_kv(u, Wd, ctx, kv)
    ws = torch.zeros(fb.fise_unet_workspace_bytes(u, ntiles, bt), dtype=torch.uint8, device=DEV)
    full = idx_dev(fo.full_index(H, W, bt))
    cache0 = torch.zeros(fb.fise_unet_cache_bytes(u), dtype=torch.uint8, device=DEV)
    fb.fise_masked_unet_step(u, Wd, cache0, lat, tsd, kv, full, ntiles, bt, fb.FISE_STATS_FRESH, None, ws)   # a dense cache
    lat2 = lat.clone(); lat2[:, 4:13, 9:20, :] += 1.0
    idx = idx_dev(np.array([1, 2, 5, 6, 9], np.int32)); na = 5
    eager = cache0.clone()
    fb.fise_masked_unet_step(u, Wd, eager, lat2, tsd, kv, idx, na, bt, fb.FISE_STATS_CACHED, None, ws)
    torch.cuda.synchronize()
    assert not torch.equal(eager, cache0)

    work = cache0.clone()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        fb.fise_masked_unet_step(u, Wd, work, lat2, tsd, kv, idx, na, bt, fb.FISE_STATS_CACHED, None, ws)      # warm-up on this stream
        torch.cuda.synchronize()
        with torch.cuda.graph(graph, stream=side):
            fb.fise_masked_unet_step(u, Wd, work, lat2, tsd, kv, idx, na, bt, fb.FISE_STATS_CACHED, None, ws)
    torch.cuda.synchronize()
    for rep in range(4):
        work.copy_(cache0)
        ws.random_(0, 255)                                   # the workspace holds anything between calls
        scratch = torch.randn(1 << 20, device=DEV).sum().item()          # unrelated eager work + a synchronisation
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(work, eager), f"replay {rep} differs from the eager step ({scratch:.1f})"
    fb.fise_unet_destroy(u)


def test_sd15_96x96_properties(fb):
    """The largest shape of the paper's workloads (768 x 768 images = 96 x 96 latents, 144 base tiles, 9216 keys at the
    first level) is beyond what the oracle finishes in minutes, so it is checked through properties that hold at any
    size: a masked step with UNCHANGED inputs on a cache built from those inputs must reproduce the cached values at
    the active positions (same operators on the same data; only the K-split summation order differs) and leave every
    other byte alone; the step is idempotent; an empty mask touches nothing."""
    d = dict(uo.sd15_desc(), H=96, W=96)
    u = fb.fise_unet_create(d)
    H, W, bt, B = d["H"], d["W"], 8, d["B"]
    ntiles = (H // bt) * (W // bt)
    g = torch.Generator(device=DEV).manual_seed(96)
    Wd = (0.02 * torch.randn(fb.fise_unet_weight_elems(u), generator=g, device=DEV)).to(torch.bfloat16)
    lat = torch.randn(B, H, W, d["in_ch"], generator=g, device=DEV).to(torch.bfloat16)
    ctx = torch.randn(B, d["n_ctx"], d["ctx_dim"], generator=g, device=DEV).to(torch.bfloat16)
    tsd = dev(uo.timestep_embedding(np.full(B, 700.0), d["base"]).astype(np.float32))
    kv = torch.zeros(fb.fise_unet_ctxkv_bytes(u), dtype=torch.uint8, device=DEV)
    fb.fise_unet_context_kv(u, Wd, ctx, kv)
    ws = torch.zeros(fb.fise_unet_workspace_bytes(u, ntiles, bt), dtype=torch.uint8, device=DEV)
    cache = torch.zeros(fb.fise_unet_cache_bytes(u), dtype=torch.uint8, device=DEV)
    fb.fise_masked_unet_step(u, Wd, cache, lat, tsd, kv, idx_dev(fo.full_index(H, W, bt)), ntiles, bt, fb.FISE_STATS_FRESH, None, ws)
    rng = np.random.default_rng(9696)
    pixm = wl.ellipse_pixels(rng, H, W, 0.1)
    _, idx = fo.tiles_from_pixels(pixm, bt)
    assert 10 <= idx.size < ntiles
    before = cache.clone()
    fb.fise_masked_unet_step(u, Wd, cache, lat, tsd, kv, idx_dev(idx), idx.size, bt, fb.FISE_STATS_CACHED, None, ws)
    torch.cuda.synchronize()
    changed = 0
    for name, off, nbytes in fb.fise_unet_tensors(u, 1):
        a, b = cache[off:off + nbytes], before[off:off + nbytes]
        if name.endswith((".mean", ".rstd")):
            assert torch.equal(a, b), name                                   # cached statistics are inputs
            continue
        x, y = a.view(torch.bfloat16).float(), b.view(torch.bfloat16).float()
        diff = (x - y).abs()
        changed += int((diff > 0).sum())
        scale = float(y.abs().max()) + 1e-6
        assert float(diff.max()) <= 4e-2 * scale, f"{name}: recomputed values moved by {float(diff.max()) / scale:.2e} of the range"
        assert float((x - y).norm()) <= 1e-2 * float(y.norm()) + 1e-6, name
    # inactive positions bit-exact: check on the output map, whose layout is [B, H, W, out_ch]
    off, nbytes = next((o, n) for nm, o, n in fb.fise_unet_tensors(u, 1) if nm == "eps")
    e1 = cache[off:off + nbytes].view(torch.bfloat16).reshape(B, H, W, d["out_ch"])
    e0 = before[off:off + nbytes].view(torch.bfloat16).reshape(B, H, W, d["out_ch"])
    inactive = torch.from_numpy(~active_mask(idx, bt, H, W)).to(DEV)
    assert torch.equal(e1[:, inactive], e0[:, inactive])
    snap = cache.clone()
    fb.fise_masked_unet_step(u, Wd, cache, lat, tsd, kv, idx_dev(idx), idx.size, bt, fb.FISE_STATS_CACHED, None, ws)
    assert torch.equal(cache, snap)                                          # idempotent
    fb.fise_masked_unet_step(u, Wd, cache, lat, tsd, kv, idx_dev(idx), 0, bt, fb.FISE_STATS_CACHED, None, ws)
    assert torch.equal(cache, snap)                                          # empty mask
    fb.fise_unet_destroy(u)
