"""GPU check that independent edit sessions do not disturb one another: the library keeps no device state between calls
(every buffer and workspace is the caller's), so masked steps of different sessions, each with its own stream, cache,
mask and workspace, issued from different host threads at the same time, must give bit for bit what the same sessions
give one after the other.  The weights, the context K/V and the plan are shared."""
import threading

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


def test_concurrent_sessions_equal_serial_sessions(fb):
    d = uo.tiny_desc(H=32, W=32, base=64)
    g = torch.Generator(device="cpu").manual_seed(311)
    u = fb.fise_unet_create(d)
    H, W, bt, B = d["H"], d["W"], 8, d["B"]
    ntiles = (H // bt) * (W // bt)
    Wd = (0.04 * torch.randn(fb.fise_unet_weight_elems(u), generator=g)).to(torch.bfloat16).to(DEV)
    lat = torch.randn(B, H, W, d["in_ch"], generator=g).to(torch.bfloat16).to(DEV)
    ctx = torch.randn(B, d["n_ctx"], d["ctx_dim"], generator=g).to(torch.bfloat16).to(DEV)
    kv = torch.zeros(fb.fise_unet_ctxkv_bytes(u), dtype=torch.uint8, device=DEV)
    fb.fise_unet_context_kv(u, Wd, ctx, kv)
    full = idx_dev(fo.full_index(H, W, bt))
    n_sess, n_steps = 4, 6
    ts = [dev(uo.timestep_embedding(np.full(B, 900.0 - 100.0 * t), d["base"]).astype(np.float32)) for t in range(n_steps)]
    ws0 = torch.zeros(fb.fise_unet_workspace_bytes(u, ntiles, bt), dtype=torch.uint8, device=DEV)
    base = []                                                # the previous generation: one dense cache per step
    for t in range(n_steps):
        c = torch.zeros(fb.fise_unet_cache_bytes(u), dtype=torch.uint8, device=DEV)
        fb.fise_masked_unet_step(u, Wd, c, lat, ts[t], kv, full, ntiles, bt, fb.FISE_STATS_FRESH, None, ws0)
        base.append(c)
    torch.cuda.synchronize()
    # each session: its own perturbation of the latent and its own detected mask
    sess = []
    for j in range(n_sess):
        lj = lat.clone()
        lj[:, 3 + 5 * j:9 + 5 * j, 2 + 4 * j:12 + 4 * j, :] += 0.5 + 0.25 * j
        pm = torch.zeros((H, W), dtype=torch.uint8, device=DEV); tm = torch.zeros(ntiles, dtype=torch.uint8, device=DEV)
        ix = torch.zeros(ntiles, dtype=torch.int32, device=DEV); na = torch.zeros(1, dtype=torch.int32, device=DEV)
        fb.fise_mask_detect(lat, lj, 0.1, bt, pm, tm, ix, na)
        n = int(na.item())
        assert 0 < n < ntiles
        sess.append(dict(lat=lj, idx=ix, n=n, ws=torch.zeros_like(ws0), stream=torch.cuda.Stream(), pm=pm, tm=tm, na=na))
    assert len({s["n"] for s in sess}) > 1 or len({tuple(s["idx"][:s["n"]].tolist()) for s in sess}) > 1

    def run(s, caches, stream):
        with torch.cuda.stream(stream):
            for t in range(n_steps):
                fb.fise_mask_detect(lat, s["lat"], 0.1, bt, s["pm"], s["tm"], s["idx"], s["na"], stream=stream)
                fb.fise_masked_unet_step(u, Wd, caches[t], s["lat"], ts[t], kv, s["idx"], s["n"], bt, fb.FISE_STATS_CACHED, None,
                                         s["ws"], stream=stream)

    serial = []
    for s in sess:
        cs = [c.clone() for c in base]
        run(s, cs, torch.cuda.current_stream())
        torch.cuda.synchronize()
        serial.append(cs)
    for rep in range(3):
        conc = [[c.clone() for c in base] for _ in sess]
        torch.cuda.synchronize()
        errs = []

        def worker(j):
            try:
                run(sess[j], conc[j], sess[j]["stream"])
            except Exception as e:                           # surfaced below: a thread's exception is otherwise lost
                errs.append(e)
        th = [threading.Thread(target=worker, args=(j,)) for j in range(n_sess)]
        for t_ in th:
            t_.start()
        for t_ in th:
            t_.join()
        torch.cuda.synchronize()
        assert not errs, errs
        for j in range(n_sess):
            for t in range(n_steps):
                assert torch.equal(conc[j][t], serial[j][t]), f"repetition {rep}: session {j}, step {t} differs from the serial run"
    assert not torch.equal(serial[0][0], base[0])
    fb.fise_unet_destroy(u)
