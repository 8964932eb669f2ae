"""The C-ABI library loads and exports every symbol include/fise.h declares; host-side
argument validation returns error codes without a GPU (nothing is launched)."""
import ctypes
import os
import re

import pytest

from paper_2305_17423_amd import binding as fb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    src = open(os.path.join(ROOT, "include", "fise.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(fise_[a-z0-9_]+)\s*\(", src)))


def test_library_exports_every_declared_symbol():
    L = fb.lib()
    names = declared_symbols()
    assert len(names) >= 25
    for n in names:
        assert hasattr(L, n), f"{n} declared in fise.h but not exported"
    assert set(names) == set(fb.EXPORTS), set(names) ^ set(fb.EXPORTS)
    assert fb.fise_version() >= 1


def test_host_side_validation_without_gpu():
    L = fb.lib()
    assert L.fise_mask_detect(None, None, 0, 1, 8, 8, 4, 0.1, 4, None, None, None, 4, None, None) == -1
    a = 0x1000  # never dereferenced: validation fails first
    assert L.fise_mask_detect(a, a, 0, 1, 8, 6, 4, 0.1, 4, a, a, a, 4, a, None) == -2       # W % tile
    assert "tile" in fb.fise_last_error()
    assert L.fise_mask_detect(a, a, 7, 1, 8, 8, 4, 0.1, 4, a, a, a, 4, a, None) == -3       # dtype
    assert L.fise_mask_downsample(a, 7, 8, a, None) == -2
    assert L.fise_attention_active(a, a, a, fb.FISE_F32, 1, 4, 8, 8, 32, 4, 1.0, a, None, 0, None) == -3
    assert L.fise_attention_active(a, a, a, fb.FISE_BF16, 1, 4, 8, 8, 30, 4, 1.0, a, None, 0, None) == -2   # C % heads
    assert L.fise_attention_active(a, a, a, fb.FISE_BF16, 1, 4, 9, 9, 32, 4, 1.0, a, None, 0, None) == -4   # stride % 8
    args = fb.fise_conv_args()
    assert L.fise_masked_conv(ctypes.byref(args), None, 0, None) == -1
    args.x0 = args.w = a; args.y_cache = 0x2000; args.B = 1; args.H = args.W = 8; args.C0 = 32; args.Cout = 32
    args.ksize = 3; args.stride = 1; args.tile = 4; args.n_active = 5; args.dtype = fb.FISE_BF16
    assert L.fise_masked_conv(ctypes.byref(args), None, 0, None) == -5                       # n_active > 4 tiles
    args.n_active = 2
    assert L.fise_masked_conv(ctypes.byref(args), None, 0, None) == -1                       # tile_idx NULL
    args.n_active = 0; args.ksize = 5
    assert L.fise_masked_conv(ctypes.byref(args), None, 0, None) == -2
    args.ksize = 3; args.x0 = 0x1004
    assert L.fise_masked_conv(ctypes.byref(args), None, 0, None) == -4                       # misaligned
    args.x0 = a
    assert L.fise_masked_conv(ctypes.byref(args), None, 0, None) == 0                        # empty mask: no-op


def test_resnet_block_rejects_identity_shortcut_for_two_sources():
    """The identity shortcut reads one map of Cout channels per pixel: a concatenated input (skip link) must come
    with the 1x1 shortcut, even when C0 + C1 == Cout."""
    L = fb.lib()
    a = 0x1000
    r = fb.fise_resnet_args()
    for f in ("x0", "x1", "gn1_mean", "gn1_rstd", "gn1_gamma", "gn1_beta", "conv1_w", "gn2_mean", "gn2_rstd", "gn2_gamma",
              "gn2_beta", "conv2_w"):
        setattr(r, f, a)
    r.h1_cache, r.out_cache = 0x2000, 0x3000
    r.C0 = r.C1 = 32; r.Cout = 64; r.B = 1; r.H = r.W = 8; r.G = 32; r.tile = 4; r.n_active = 0
    assert L.fise_masked_resnet_block(ctypes.byref(r), None, 0, None) == -2
    assert "shortcut" in fb.fise_last_error()
    r.sc_w = a
    assert L.fise_masked_resnet_block(ctypes.byref(r), None, 0, None) == 0                  # empty mask: accepted, no-op
    r.sc_w = None; r.x1 = None; r.C1 = 0; r.C0 = 64
    assert L.fise_masked_resnet_block(ctypes.byref(r), None, 0, None) == 0                  # one source: identity is fine


def test_unet_plan_matches_oracle_tables():
    import numpy as np
    from oracle import fise_unet_oracle as uo
    for d in (uo.sd15_desc(), uo.tiny_desc()):
        u = fb.fise_unet_create(d)
        sh = uo.param_shapes(d)
        ws = fb.fise_unet_tensors(u, 0)
        assert {n for n, _, _ in ws} == set(sh)
        assert all(int(np.prod(sh[n])) == num and off % 8 == 0 for n, off, num in ws)
        spans = sorted((off, off + num) for _, off, num in ws)
        assert all(a[1] <= b[0] for a, b in zip(spans, spans[1:]))
        assert spans[-1][1] <= fb.fise_unet_weight_elems(u)
        csh = uo.cache_shapes(d)
        cs = fb.fise_unet_tensors(u, 1)
        assert {n for n, _, _ in cs} == set(csh)
        for n, off, nbytes in cs:
            el = 4 if n.endswith((".mean", ".rstd")) else 2
            assert nbytes == int(np.prod(csh[n])) * el and off % 256 == 0
        fb.fise_unet_destroy(u)
    bad = uo.tiny_desc(base=48)
    with pytest.raises(fb.FiseError):
        fb.fise_unet_create(bad)


def test_cache_layout_groups_and_move_argument_checks():
    """The cache buffer's tensor groups are contiguous byte ranges that hold exactly the tensors they name, and the
    cache-moving entry points refuse bad arguments before they touch the GPU."""
    import ctypes
    from oracle import fise_unet_oracle as uo
    for d in (uo.sd15_desc(), uo.tiny_desc(), uo.tiny_desc(H=32, W=32, base=64)):
        u = fb.fise_unet_create(d)
        assert fb.fise_unet_desc_of(u)["H"] == d["H"] and fb.fise_unet_desc_of(u)["mults"] == tuple(d["mults"])
        L = fb.fise_unet_cache_layout(u)
        cb = fb.fise_unet_cache_bytes(u)
        assert L["maps_off"] == 0 and L["kv_off"] == L["maps_bytes"] and L["small_off"] == L["kv_off"] + L["kv_bytes"]
        assert L["derived_maps_off"] == L["small_off"] + L["small_bytes"] and L["derived_maps_off"] + L["derived_maps_bytes"] == cb
        assert L["small_off"] < L["stored_bytes"] <= L["derived_maps_off"]
        for n, off, nbytes in fb.fise_unet_tensors(u, 1):
            if n.endswith((".mean", ".rstd")):
                lo, hi = L["small_off"], L["stored_bytes"]
            elif n.endswith((".k", ".v")):
                lo, hi = L["kv_off"], L["kv_off"] + L["kv_bytes"]
            else:
                lo, hi = 0, L["maps_bytes"]
            assert lo <= off and off + nbytes <= hi, n
        for n, off, nbytes in fb.fise_unet_tensors(u, 3):
            if n.endswith(".ss"):
                assert L["stored_bytes"] <= off and off + nbytes <= L["derived_maps_off"], n
            else:
                assert L["derived_maps_off"] <= off and off + nbytes <= cb, n
        fb.fise_unet_destroy(u)
    d = uo.tiny_desc(H=32, W=32, base=64)
    u = fb.fise_unet_create(d)
    lib, a, b = fb.lib(), 0x10000000, 0x40000000
    assert fb.fise_unet_cache_move_workspace_bytes(u) >= (32 * 32 + 16 * 16 + 8 * 8 + 4 * 4) * 4
    mv = lambda *x: lib.fise_unet_cache_move_active(u, *x)
    assert mv(a, b, a, 0, 8, 1, 1, a, 1 << 20, None) == 0                      # empty mask: nothing to do
    assert mv(a, b, a, 3, 8, 2, 1, a, 1 << 20, None) == -2                     # halo
    assert mv(a, b, a, 3, 8, 1, 8, a, 1 << 20, None) == -2                     # unknown group
    assert mv(a, b, a, 3, 6, 1, 1, a, 1 << 20, None) == -2                     # base tile must divide the map
    assert mv(a, b, a, 17, 8, 1, 1, a, 1 << 20, None) == -5                    # more active tiles than tiles
    assert mv(a, b, a, 3, 8, 1, 1, a, 16, None) == -5                          # workspace too small
    assert mv(a, a + 256, a, 3, 8, 1, 1, a, 1 << 20, None) == -2               # overlapping buffers
    assert mv(None, b, a, 3, 8, 1, 1, a, 1 << 20, None) == -1
    rows = lambda *r: (ctypes.c_int * len(r))(*r)
    tr = lambda rr, n, *x: lib.fise_unet_cache_move_tile_rows(u, a, b, rr, n, *x)
    assert tr(rows(0, 1), 0, 8, 1, 1, None) == 0                               # no ranges
    assert tr(rows(1, 1), 1, 8, 1, 1, None) == -2                              # empty range
    assert tr(rows(2, 3, 0, 1), 2, 8, 1, 1, None) == -2                        # not ascending
    assert tr(rows(0, 2, 1, 3), 2, 8, 1, 1, None) == -2                        # overlapping
    assert tr(rows(0, 5), 1, 8, 1, 1, None) == -2                              # beyond the 4 tile rows
    assert tr(rows(0, 1), 1, 8, 1, 4, None) == -2                              # V^T is not row-addressed
    assert tr(rows(0, 1), 1, 8, 3, 1, None) == -2                              # halo
    fb.fise_unet_destroy(u)


def test_apsc_select_is_the_oracle_argmin():
    """The host argmin over the 25 candidate block sizes against the oracle's selection, counts taken from the oracle."""
    import numpy as np
    from oracle import fise_oracle as fo
    from paper_2305_17423_amd import workloads as wl
    for seed, (H, W), frac in ((1, (32, 32), 0.1), (2, (64, 64), 0.03), (3, (64, 32), 0.3), (4, (48, 48), 0.1), (5, (32, 64), 0.6)):
        pix = wl.ellipse_pixels(np.random.default_rng(seed), H, W, frac)
        for kh, kw in ((3, 3), (1, 1)):
            counts = []
            for h in (2, 4, 8, 16, 32):
                for w in (2, 4, 8, 16, 32):
                    c = fo.apsc_cost(pix, h, w, kh, kw)
                    counts.append(-1 if c is None else c // ((h + kh - 1) * (w + kw - 1)))
            assert fb.fise_apsc_select(counts, kh, kw) == fo.apsc_block_size(pix, kh, kw)
    with pytest.raises(fb.FiseError):
        fb.fise_apsc_select([-1] * 25)
    L = fb.lib()
    a = 0x1000
    assert L.fise_mask_from_pixels_rect(a, 8, 8, 3, 4, a, a, 4, a, None) == -2               # H % tile_h
    assert L.fise_mask_from_pixels_rect(a, 8, 8, 2, 0, a, a, 4, a, None) == -2
    args = fb.fise_conv_args()
    args.x0 = args.w = a; args.y_cache = 0x2000; args.B = 1; args.H = args.W = 8; args.C0 = 32; args.Cout = 32
    args.ksize = 3; args.stride = 1; args.tile = 4; args.tile_w = 3; args.dtype = fb.FISE_BF16
    assert L.fise_masked_conv(ctypes.byref(args), None, 0, None) == -2                       # W % tile_w
    args.tile_w = 2; args.n_active = 9
    assert L.fise_masked_conv(ctypes.byref(args), None, 0, None) == -5                       # 2 x 4 = 8 blocks


def test_binding_refuses_numbers_where_buffers_go():
    """A Python number in a buffer position would reach a kernel as an address: the binding raises instead."""
    with pytest.raises(TypeError):
        fb._p(12)
    assert fb._p(None) is None
