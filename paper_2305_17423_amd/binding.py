"""ctypes binding of libfise.so: same names as the C ABI (include/fise.h).

Argument marshalling only: torch tensors are used as device buffers (data_ptr),
every step of the path runs in the library's kernels.  There is no fallback: if
the library has not been built, loading raises.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("FISE_LIB", os.path.join(_HERE, "libfise.so"))

FISE_F32, FISE_BF16 = 0, 1
FISE_STATS_CACHED, FISE_STATS_FRESH = 0, 1
FISE_MAX_LEVELS = 8
_lib = None

vp, i32, f32, sz, i64 = C.c_void_p, C.c_int, C.c_float, C.c_size_t, C.c_int64


class FiseError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"fise error {code}: {msg}")
        self.code = code


class fise_conv_args(C.Structure):
    _fields_ = [("x0", vp), ("x1", vp), ("C0", i32), ("C1", i32), ("B", i32), ("H", i32), ("W", i32),
                ("w", vp), ("bias", vp), ("Cout", i32), ("ksize", i32), ("stride", i32), ("upsample", i32),
                ("gn_mean", vp), ("gn_rstd", vp), ("gn_gamma", vp), ("gn_beta", vp), ("G", i32), ("gn_silu", i32),
                ("temb", vp), ("residual", vp), ("tile_idx", vp), ("n_active", i32), ("tile", i32),
                ("y_cache", vp), ("dtype", i32), ("tile_w", i32)]


class fise_resnet_args(C.Structure):
    _fields_ = [("x0", vp), ("x1", vp), ("C0", i32), ("C1", i32), ("B", i32), ("H", i32), ("W", i32), ("Cout", i32), ("G", i32),
                ("gn1_mean", vp), ("gn1_rstd", vp), ("gn1_gamma", vp), ("gn1_beta", vp), ("conv1_w", vp), ("conv1_b", vp),
                ("temb", vp), ("temb_stride", i32),
                ("gn2_mean", vp), ("gn2_rstd", vp), ("gn2_gamma", vp), ("gn2_beta", vp), ("conv2_w", vp), ("conv2_b", vp),
                ("sc_w", vp), ("sc_b", vp), ("tile_idx", vp), ("n_active", i32), ("tile", i32),
                ("h1_cache", vp), ("out_cache", vp), ("stats_fresh", i32)]


class fise_transformer_args(C.Structure):
    _fields_ = [("x", vp), ("B", i32), ("H", i32), ("W", i32), ("C", i32), ("G", i32), ("heads", i32),
                ("gn_mean", vp), ("gn_rstd", vp), ("gn_gamma", vp), ("gn_beta", vp), ("pin_w", vp), ("pin_b", vp),
                ("ln1_g", vp), ("ln1_b", vp), ("qkv_w", vp), ("o1_w", vp), ("o1_b", vp),
                ("ln2_g", vp), ("ln2_b", vp), ("q2_w", vp), ("o2_w", vp), ("o2_b", vp),
                ("K_ctx", vp), ("Vt_ctx", vp), ("n_ctx", i32), ("n_ctx_stride", i32),
                ("ln3_g", vp), ("ln3_b", vp), ("ff1_w", vp), ("ff1_b", vp), ("ff2_w", vp), ("ff2_b", vp),
                ("pout_w", vp), ("pout_b", vp), ("K_cache", vp), ("Vt_cache", vp), ("out_cache", vp),
                ("tile_idx", vp), ("n_active", i32), ("tile", i32), ("stats_fresh", i32)]


class fise_unet_desc(C.Structure):
    _fields_ = [("in_ch", i32), ("out_ch", i32), ("base", i32), ("n_levels", i32),
                ("mults", i32 * FISE_MAX_LEVELS), ("attn", i32 * FISE_MAX_LEVELS), ("layers", i32),
                ("heads", i32), ("ctx_dim", i32), ("n_ctx", i32), ("groups", i32), ("H", i32), ("W", i32), ("B", i32)]


_SIGS = {
    "fise_last_error": (C.c_char_p, []),
    "fise_version": (i32, []),
    "fise_mask_detect": (i32, [vp, vp, i32, i32, i32, i32, i32, f32, i32, vp, vp, vp, i32, vp, vp]),
    "fise_mask_from_pixels": (i32, [vp, i32, i32, i32, vp, vp, i32, vp, vp]),
    "fise_mask_downsample": (i32, [vp, i32, i32, vp, vp]),
    "fise_otsu_workspace_bytes": (sz, []),
    "fise_otsu_mask": (i32, [vp, i32, vp, vp, vp, vp]),
    "fise_diff_accumulate": (i32, [vp, vp, i32, i32, i32, i32, i32, vp, vp]),
    "fise_apsc_block_counts": (i32, [vp, i32, i32, vp, vp]),
    "fise_apsc_select": (i32, [C.POINTER(C.c_int32), i32, i32, C.POINTER(i32), C.POINTER(i32), C.POINTER(i64)]),
    "fise_mask_from_pixels_rect": (i32, [vp, i32, i32, i32, i32, vp, vp, i32, vp, vp]),
    "fise_groupnorm_stats_workspace_bytes": (sz, [i32, i32, i32, i32]),
    "fise_groupnorm_stats": (i32, [vp, vp, i32, i32, i32, i32, i32, i32, i32, f32, vp, vp, vp, vp]),
    "fise_groupnorm_stats_static_capacity_bytes": (sz, []),
    "fise_groupnorm_stats_static": (i32, [vp, vp, i32, i32, i32, i32, i32, i32, i32, f32, vp, vp, vp]),
    "fise_masked_groupnorm_silu": (i32, [vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, i32, vp, i32, i32, vp, vp]),
    "fise_masked_conv_workspace_bytes": (sz, [C.POINTER(fise_conv_args)]),
    "fise_masked_conv": (i32, [C.POINTER(fise_conv_args), vp, sz, vp]),
    "fise_masked_conv3x3": (i32, [vp, vp, vp, i32, i32, i32, i32, i32, i32, i32, vp, i32, i32, vp, vp, vp, vp, i32,
                                  vp, vp, vp, vp, sz, vp]),
    "fise_attention_active_workspace_bytes": (sz, [i32, i32, i32, i32, i32]),
    "fise_attention_active": (i32, [vp, vp, vp, i32, i32, i32, i32, i32, i32, i32, f32, vp, vp, sz, vp]),
    "fise_context_kv_workspace_bytes": (sz, [i32, i32, i32, i32]),
    "fise_context_kv": (i32, [vp, vp, vp, i32, i32, i32, i32, i32, i32, vp, vp, vp, sz, vp]),
    "fise_masked_attention_workspace_bytes": (sz, [i32, i32, i32, i32]),
    "fise_masked_attention_restricted_workspace_bytes": (sz, [i32, i32, i32, i32]),
    "fise_masked_attention_restricted": (i32, [vp, vp, vp, vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, i32, vp, i32, i32, vp,
                                               vp, sz, vp]),
    "fise_masked_attention": (i32, [vp, vp, vp, vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, i32, vp, vp, vp, vp,
                                    i32, i32, vp, i32, i32, vp, vp, sz, vp]),
    "fise_masked_resnet_block_workspace_bytes": (sz, [C.POINTER(fise_resnet_args)]),
    "fise_masked_resnet_block": (i32, [C.POINTER(fise_resnet_args), vp, sz, vp]),
    "fise_masked_transformer_block_workspace_bytes": (sz, [C.POINTER(fise_transformer_args)]),
    "fise_masked_transformer_block": (i32, [C.POINTER(fise_transformer_args), vp, sz, vp]),
    "fise_unet_create": (i32, [C.POINTER(fise_unet_desc), C.POINTER(vp)]),
    "fise_unet_destroy": (None, [vp]),
    "fise_unet_num_tensors": (i32, [vp, i32]),
    "fise_unet_tensor_info": (i32, [vp, i32, i32, C.c_char_p, C.POINTER(i64), C.POINTER(i64)]),
    "fise_unet_weight_elems": (i64, [vp]),
    "fise_unet_cache_bytes": (sz, [vp]),
    "fise_unet_ctxkv_bytes": (sz, [vp]),
    "fise_unet_workspace_bytes": (sz, [vp, i32, i32]),
    "fise_unet_refresh_derived_workspace_bytes": (sz, [vp]),
    "fise_unet_refresh_derived": (i32, [vp, vp, vp, vp, sz, vp]),
    "fise_unet_context_kv": (i32, [vp, vp, vp, vp, vp, sz, vp]),
    "fise_unet_cache_layout_get": (i32, [vp, vp]),
    "fise_unet_desc_get": (i32, [vp, vp]),
    "fise_unet_cache_move_workspace_bytes": (sz, [vp]),
    "fise_unet_cache_move_active": (i32, [vp, vp, vp, vp, i32, i32, i32, i32, vp, sz, vp]),
    "fise_unet_cache_move_tile_rows": (i32, [vp, vp, vp, C.POINTER(i32), i32, i32, i32, i32, vp]),
    "fise_masked_unet_step": (i32, [vp, vp, vp, vp, vp, vp, vp, i32, i32, i32, C.POINTER(i32), vp, sz, vp]),
    "fise_profile_enable": (i32, [i32]),
    "fise_profile_calibrate": (i32, [i32, vp]),
    "fise_calibrate_peaks": (i32, [vp, sz, C.POINTER(C.c_double), C.POINTER(C.c_double), vp]),
    "fise_profile_read": (i32, [i32, C.POINTER(C.c_double), C.POINTER(C.c_double), C.POINTER(C.c_double), C.POINTER(i32)]),
    "fise_unet_num_modules": (i32, [vp]),
    "fise_unet_module_name": (i32, [vp, i32, C.c_char_p]),
    "fise_masked_unet_modules": (i32, [vp, vp, vp, vp, vp, vp, vp, i32, i32, i32, C.POINTER(i32), i32, i32, vp, sz, vp]),
}
EXPORTS = tuple(_SIGS)


def lib():
    """The loaded library (raises if it has not been built)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(f"{LIB_PATH} is missing: run `python -m paper_2305_17423_amd.build` "
                                    "(there is no CPU or PyTorch fallback)")
        L = C.CDLL(LIB_PATH)
        for name, (res, args) in _SIGS.items():
            fn = getattr(L, name)
            fn.restype, fn.argtypes = res, args
        _lib = L
    return _lib


def _p(t):
    """Device (or host) address of a tensor, None -> NULL."""
    if t is None:
        return None
    if not hasattr(t, "data_ptr"):          # a bare number here would reach a kernel as an address
        raise TypeError(f"expected a tensor or None where a buffer is passed, got {type(t).__name__}")
    return t.data_ptr()


def _dt(t):
    if t.dtype == torch.float32:
        return FISE_F32
    if t.dtype == torch.bfloat16:
        return FISE_BF16
    raise TypeError(f"unsupported dtype {t.dtype}")


def _stream(stream):
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else stream


def _ck(code):
    if code != 0:
        raise FiseError(code, lib().fise_last_error().decode())


def fise_last_error():
    return lib().fise_last_error().decode()


def fise_version():
    return lib().fise_version()


# --------------------------------------------------------------------------- masks
def fise_mask_detect(cached, fresh, threshold, tile, pix_mask, tile_mask, tile_idx, n_active, stream=None):
    B, H, W, Cc = cached.shape
    _ck(lib().fise_mask_detect(_p(cached), _p(fresh), _dt(cached), B, H, W, Cc, threshold, tile, _p(pix_mask),
                               _p(tile_mask), _p(tile_idx), tile_idx.numel(), _p(n_active), _stream(stream)))


def fise_mask_from_pixels(pix_mask, tile, tile_mask, tile_idx, n_active, stream=None):
    H, W = pix_mask.shape
    _ck(lib().fise_mask_from_pixels(_p(pix_mask), H, W, tile, _p(tile_mask), _p(tile_idx), tile_idx.numel(),
                                    _p(n_active), _stream(stream)))


def fise_mask_from_pixels_rect(pix_mask, tile_h, tile_w, tile_mask, tile_idx, n_active, stream=None):
    H, W = pix_mask.shape
    _ck(lib().fise_mask_from_pixels_rect(_p(pix_mask), H, W, tile_h, tile_w, _p(tile_mask), _p(tile_idx), tile_idx.numel(),
                                         _p(n_active), _stream(stream)))


def fise_mask_downsample(mask, out, stream=None):
    H, W = mask.shape
    _ck(lib().fise_mask_downsample(_p(mask), H, W, _p(out), _stream(stream)))


def fise_otsu_workspace_bytes():
    return lib().fise_otsu_workspace_bytes()


def fise_otsu_mask(diff, eps_out, pix_mask, workspace, stream=None):
    _ck(lib().fise_otsu_mask(_p(diff), diff.numel(), _p(eps_out), _p(pix_mask), _p(workspace), _stream(stream)))


def fise_diff_accumulate(cached, fresh, diff_acc, stream=None):
    B, H, W, Cc = cached.shape
    _ck(lib().fise_diff_accumulate(_p(cached), _p(fresh), _dt(cached), B, H, W, Cc, _p(diff_acc), _stream(stream)))


def fise_apsc_block_counts(pix_mask, counts, stream=None):
    H, W = pix_mask.shape
    _ck(lib().fise_apsc_block_counts(_p(pix_mask), H, W, _p(counts), _stream(stream)))


def fise_apsc_select(counts_host, kh=3, kw=3):
    """(h, w, cost) from the 25 block counts (a host sequence of ints)."""
    arr = (C.c_int32 * 25)(*[int(v) for v in counts_host])
    h, w, cost = i32(), i32(), i64()
    _ck(lib().fise_apsc_select(arr, kh, kw, C.byref(h), C.byref(w), C.byref(cost)))
    return h.value, w.value, cost.value


# --------------------------------------------------------------------------- normalisation
def fise_groupnorm_stats_workspace_bytes(B, H, W, Cc):
    return lib().fise_groupnorm_stats_workspace_bytes(B, H, W, Cc)


def fise_groupnorm_stats(x, x1, G, eps, mean, rstd, workspace, stream=None):
    B, H, W, C0 = x.shape
    C1 = 0 if x1 is None else x1.shape[-1]
    _ck(lib().fise_groupnorm_stats(_p(x), _p(x1), _dt(x), B, H, W, C0, C1, G, eps, _p(mean), _p(rstd), _p(workspace),
                                   _stream(stream)))


def fise_groupnorm_stats_static_capacity_bytes():
    return lib().fise_groupnorm_stats_static_capacity_bytes()


def fise_groupnorm_stats_static(x, x1, G, eps, mean, rstd, stream=None):
    B, H, W, C0 = x.shape
    C1 = 0 if x1 is None else x1.shape[-1]
    _ck(lib().fise_groupnorm_stats_static(_p(x), _p(x1), _dt(x), B, H, W, C0, C1, G, eps, _p(mean), _p(rstd), _stream(stream)))


def fise_masked_groupnorm_silu(x, mean, rstd, gamma, beta, G, tile_idx, n_active, tile, y_cache, stream=None):
    B, H, W, Cc = x.shape
    _ck(lib().fise_masked_groupnorm_silu(_p(x), _p(mean), _p(rstd), _p(gamma), _p(beta), _dt(x), B, H, W, Cc, G,
                                         _p(tile_idx), n_active, tile, _p(y_cache), _stream(stream)))


# --------------------------------------------------------------------------- convolution
def conv_args(x0, w, bias, tile_idx, n_active, tile, y_cache, x1=None, ksize=3, stride=1, upsample=0, gn=None,
              gn_silu=1, temb=None, residual=None, tile_w=0):
    B, H, W, C0 = x0.shape
    a = fise_conv_args()
    a.x0, a.x1, a.C0, a.C1 = _p(x0), _p(x1), C0, (0 if x1 is None else x1.shape[-1])
    a.B, a.H, a.W = B, H, W
    a.w, a.bias, a.Cout, a.ksize, a.stride, a.upsample = _p(w), _p(bias), w.shape[0], ksize, stride, upsample
    if gn is not None:
        a.gn_mean, a.gn_rstd, a.gn_gamma, a.gn_beta, a.G = _p(gn["mean"]), _p(gn["rstd"]), _p(gn["gamma"]), _p(gn["beta"]), gn["groups"]
    a.gn_silu = gn_silu
    a.temb, a.residual, a.tile_idx, a.n_active, a.tile = _p(temb), _p(residual), _p(tile_idx), n_active, tile
    a.y_cache, a.dtype, a.tile_w = _p(y_cache), _dt(x0), tile_w
    return a


def fise_masked_conv_workspace_bytes(args):
    return lib().fise_masked_conv_workspace_bytes(C.byref(args))


def fise_masked_conv(args, workspace=None, stream=None):
    nbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _ck(lib().fise_masked_conv(C.byref(args), _p(workspace), nbytes, _stream(stream)))


def fise_masked_conv3x3(x, w, bias, stride, tile_idx, n_active, tile, y_cache, gn=None, temb=None, residual=None,
                        workspace=None, stream=None):
    B, H, W, Cin = x.shape
    g = gn or {}
    nbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _ck(lib().fise_masked_conv3x3(_p(x), _p(w), _p(bias), _dt(x), B, H, W, Cin, w.shape[0], stride, _p(tile_idx),
                                  n_active, tile, _p(g.get("mean")), _p(g.get("rstd")), _p(g.get("gamma")),
                                  _p(g.get("beta")), g.get("groups", 0), _p(temb), _p(residual), _p(y_cache),
                                  _p(workspace), nbytes, _stream(stream)))


# --------------------------------------------------------------------------- attention
def fise_attention_active_workspace_bytes(B, M, n_keys, Cc, heads):
    return lib().fise_attention_active_workspace_bytes(B, M, n_keys, Cc, heads)


def fise_attention_active(q, K, Vt, heads, scale, out, n_keys=None, workspace=None, stream=None):
    B, M, Cc = q.shape
    n_keys = K.shape[1] if n_keys is None else n_keys
    nbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _ck(lib().fise_attention_active(_p(q), _p(K), _p(Vt), _dt(q), B, M, n_keys, Vt.shape[2], Cc, heads, scale, _p(out),
                                    _p(workspace), nbytes, _stream(stream)))


def fise_context_kv(ctx, Wk, Wv, K_ctx, Vt_ctx, stream=None):
    B, n_ctx, Dc = ctx.shape
    _ck(lib().fise_context_kv(_p(ctx), _p(Wk), _p(Wv), _dt(ctx), B, n_ctx, Dc, Wk.shape[0], Vt_ctx.shape[2], _p(K_ctx),
                              _p(Vt_ctx), None, 0, _stream(stream)))


def fise_masked_attention_restricted_workspace_bytes(B, Cc, n_active, tile):
    return lib().fise_masked_attention_restricted_workspace_bytes(B, Cc, n_active, tile)


def fise_masked_attention_restricted(x, ln_gamma, ln_beta, Wq, Wk, Wv, Wo, bo, heads, tile_idx, n_active, tile, y_cache,
                                     workspace, stream=None):
    B, H, W, Cc = x.shape
    _ck(lib().fise_masked_attention_restricted(_p(x), _p(ln_gamma), _p(ln_beta), _p(Wq), _p(Wk), _p(Wv), _p(Wo), _p(bo), _dt(x), B,
                                               H, W, Cc, heads, _p(tile_idx), n_active, tile, _p(y_cache), _p(workspace),
                                               workspace.numel() * workspace.element_size(), _stream(stream)))


def fise_masked_attention_workspace_bytes(B, Cc, n_active, tile):
    return lib().fise_masked_attention_workspace_bytes(B, Cc, n_active, tile)


def fise_masked_attention(x, ln_gamma, ln_beta, Wq, Wk, Wv, Wo, bo, heads, K_cache, Vt_cache, K_ctx, Vt_ctx, n_ctx,
                          tile_idx, n_active, tile, y_cache, workspace, stream=None):
    B, H, W, Cc = x.shape
    nstride = 0 if Vt_ctx is None else Vt_ctx.shape[2]
    nbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _ck(lib().fise_masked_attention(_p(x), _p(ln_gamma), _p(ln_beta), _p(Wq), _p(Wk), _p(Wv), _p(Wo), _p(bo), _dt(x), B,
                                    H, W, Cc, heads, _p(K_cache), _p(Vt_cache), _p(K_ctx), _p(Vt_ctx), n_ctx, nstride,
                                    _p(tile_idx), n_active, tile, _p(y_cache), _p(workspace), nbytes, _stream(stream)))


# --------------------------------------------------------------------------- modules
def fill_args(struct_type, keep, **kw):
    """A ctypes argument struct from keyword values; tensors become addresses and are appended
    to `keep` so they outlive the (asynchronous) call.  An int in a pointer field is taken as an
    address read from another argument struct."""
    a = struct_type()
    types = dict(struct_type._fields_)
    for k, v in kw.items():
        if types[k] is vp:
            if hasattr(v, "data_ptr"):
                keep.append(v)
            setattr(a, k, v if isinstance(v, int) else _p(v))
        else:
            setattr(a, k, int(v))
    return a


def fise_masked_resnet_block_workspace_bytes(args):
    return lib().fise_masked_resnet_block_workspace_bytes(C.byref(args))


def fise_masked_resnet_block(args, workspace, stream=None):
    nbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _ck(lib().fise_masked_resnet_block(C.byref(args), _p(workspace), nbytes, _stream(stream)))


def fise_masked_transformer_block_workspace_bytes(args):
    return lib().fise_masked_transformer_block_workspace_bytes(C.byref(args))


def fise_masked_transformer_block(args, workspace, stream=None):
    nbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _ck(lib().fise_masked_transformer_block(C.byref(args), _p(workspace), nbytes, _stream(stream)))


# --------------------------------------------------------------------------- UNet
def make_desc(d):
    s = fise_unet_desc()
    s.in_ch, s.out_ch, s.base, s.n_levels = d["in_ch"], d["out_ch"], d["base"], len(d["mults"])
    for i, m in enumerate(d["mults"]):
        s.mults[i] = m
        s.attn[i] = 1 if d["attn"][i] else 0
    s.layers, s.heads, s.ctx_dim, s.n_ctx, s.groups = d["layers"], d["heads"], d["ctx_dim"], d["n_ctx"], d["groups"]
    s.H, s.W, s.B = d["H"], d["W"], d["B"]
    return s


def fise_unet_create(desc):
    h = vp()
    s = make_desc(desc) if isinstance(desc, dict) else desc
    _ck(lib().fise_unet_create(C.byref(s), C.byref(h)))
    return h


def fise_unet_destroy(u):
    lib().fise_unet_destroy(u)


def fise_unet_desc_of(u):
    """The description a plan was made from, as the dict make_desc() takes."""
    s = fise_unet_desc()
    _ck(lib().fise_unet_desc_get(u, C.byref(s)))
    n = s.n_levels
    return dict(in_ch=s.in_ch, out_ch=s.out_ch, base=s.base, mults=tuple(s.mults[i] for i in range(n)),
                attn=tuple(bool(s.attn[i]) for i in range(n)), layers=s.layers, heads=s.heads, ctx_dim=s.ctx_dim,
                n_ctx=s.n_ctx, groups=s.groups, H=s.H, W=s.W, B=s.B)


def fise_unet_tensors(u, kind):
    """[(name, offset, numel)] of the flat weight (0), cache (1) or context-K/V (2) buffer."""
    out = []
    name = C.create_string_buffer(64)
    off, num = i64(), i64()
    for i in range(lib().fise_unet_num_tensors(u, kind)):
        _ck(lib().fise_unet_tensor_info(u, kind, i, name, C.byref(off), C.byref(num)))
        out.append((name.value.decode(), off.value, num.value))
    return out


def fise_unet_weight_elems(u):
    return lib().fise_unet_weight_elems(u)


def fise_unet_cache_bytes(u):
    return lib().fise_unet_cache_bytes(u)


def fise_unet_ctxkv_bytes(u):
    return lib().fise_unet_ctxkv_bytes(u)


def fise_unet_workspace_bytes(u, max_active_tiles, base_tile):
    return lib().fise_unet_workspace_bytes(u, max_active_tiles, base_tile)


def fise_unet_refresh_derived_workspace_bytes(u):
    return lib().fise_unet_refresh_derived_workspace_bytes(u)


def fise_unet_refresh_derived(u, weights, cache, workspace, stream=None):
    _ck(lib().fise_unet_refresh_derived(u, _p(weights), _p(cache), _p(workspace), workspace.numel() * workspace.element_size(),
                                        _stream(stream)))


FISE_MOVE_MAPS, FISE_MOVE_K, FISE_MOVE_VT = 1, 2, 4
_LAYOUT_FIELDS = ("maps_off", "maps_bytes", "kv_off", "kv_bytes", "small_off", "small_bytes", "derived_maps_off",
                  "derived_maps_bytes", "stored_bytes")


def fise_unet_cache_layout(u):
    """{field: bytes} of the contiguous tensor groups of a per-step cache buffer."""
    raw = (i64 * len(_LAYOUT_FIELDS))()
    _ck(lib().fise_unet_cache_layout_get(u, raw))
    return dict(zip(_LAYOUT_FIELDS, (int(v) for v in raw)))


def fise_unet_cache_move_workspace_bytes(u):
    return lib().fise_unet_cache_move_workspace_bytes(u)


def fise_unet_cache_move_active(u, src, dst, tile_idx, n_active, base_tile, halo, what, workspace, stream=None):
    """src / dst: cache-sized uint8 tensors in device memory or pinned host memory."""
    _ck(lib().fise_unet_cache_move_active(u, _p(src), _p(dst), _p(tile_idx), n_active, base_tile, halo, what, _p(workspace),
                                          workspace.numel() * workspace.element_size(), _stream(stream)))


def fise_unet_cache_move_tile_rows(u, src, dst, tile_rows, base_tile, halo, what, stream=None):
    """tile_rows: [(first, last), ...] rows of the base tile grid (host integers)."""
    flat = [int(v) for r in tile_rows for v in r]
    arr = (i32 * max(len(flat), 1))(*flat)
    _ck(lib().fise_unet_cache_move_tile_rows(u, _p(src), _p(dst), arr, len(flat) // 2, base_tile, halo, what, _stream(stream)))


def fise_unet_context_kv(u, weights, ctx, ctxkv, stream=None):
    _ck(lib().fise_unet_context_kv(u, _p(weights), _p(ctx), _p(ctxkv), None, 0, _stream(stream)))


def fise_masked_unet_step(u, weights, cache, latent, t_sin, ctxkv, tile_idx, n_active, base_tile, stats_mode,
                          level_dense, workspace, stream=None):
    ld = None
    if level_dense is not None:
        ld = (i32 * len(level_dense))(*[int(v) for v in level_dense])
    _ck(lib().fise_masked_unet_step(u, _p(weights), _p(cache), _p(latent), _p(t_sin), _p(ctxkv), _p(tile_idx), n_active,
                                    base_tile, stats_mode, ld, _p(workspace), workspace.numel() * workspace.element_size(),
                                    _stream(stream)))


def fise_unet_module_names(u):
    name = C.create_string_buffer(64)
    out = []
    for i in range(lib().fise_unet_num_modules(u)):
        _ck(lib().fise_unet_module_name(u, i, name))
        out.append(name.value.decode())
    return out


def fise_masked_unet_modules(u, weights, cache, latent, t_sin, ctxkv, tile_idx, n_active, base_tile, stats_mode,
                             level_dense, first_module, n_modules, workspace, stream=None):
    ld = None
    if level_dense is not None:
        ld = (i32 * len(level_dense))(*[int(v) for v in level_dense])
    _ck(lib().fise_masked_unet_modules(u, _p(weights), _p(cache), _p(latent), _p(t_sin), _p(ctxkv), _p(tile_idx), n_active,
                                       base_tile, stats_mode, ld, first_module, n_modules, _p(workspace),
                                       workspace.numel() * workspace.element_size(), _stream(stream)))


def fise_profile_enable(on):
    _ck(lib().fise_profile_enable(1 if on else 0))


def fise_profile_calibrate(n, stream=None):
    _ck(lib().fise_profile_calibrate(int(n), _stream(stream)))


def fise_calibrate_peaks(scratch, stream=None):
    """(copy GB/s, bf16 MFMA TFLOP/s) measured on the current device; `scratch` is overwritten."""
    gbs, tf = C.c_double(), C.c_double()
    _ck(lib().fise_calibrate_peaks(_p(scratch), scratch.numel() * scratch.element_size(), C.byref(gbs), C.byref(tf),
                                   _stream(stream)))
    return gbs.value, tf.value


def fise_profile_read(kind):
    """(total_ms, total_flops, total_bytes, launches) of the launches recorded for `kind`; -1 clears."""
    ms, fl, by, n = C.c_double(), C.c_double(), C.c_double(), i32()
    _ck(lib().fise_profile_read(kind, C.byref(ms), C.byref(fl), C.byref(by), C.byref(n)))
    return ms.value, fl.value, by.value, n.value
