"""Seeded synthetic inputs shared by the tests, the bench and the smoke run.

Only raw random tensors and mask geometry live here: none of the method's
arithmetic (no convolution, normalisation, attention, thresholding).  Arrays are
float32 numpy holding values exactly representable in the storage dtype.
"""
from __future__ import annotations

import math

import numpy as np
import torch


def storage_round(a: np.ndarray, dtype: str) -> np.ndarray:
    """float32 array whose values are representable in `dtype` ('f32'|'bf16')."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    if dtype == "bf16":
        return torch.from_numpy(a).to(torch.bfloat16).to(torch.float32).numpy()
    return a


def normal(rng, shape, std=1.0, dtype="f32", mean=0.0):
    return storage_round(mean + std * rng.standard_normal(shape), dtype)


def rect_pixels(rng, H, W, h, w):
    """A seeded h x w rectangle, top-left uniform, not tile aligned."""
    y0 = int(rng.integers(0, H - h + 1))
    x0 = int(rng.integers(0, W - w + 1))
    m = np.zeros((H, W), np.uint8)
    m[y0:y0 + h, x0:x0 + w] = 1
    return m


def ellipse_pixels(rng, H, W, frac):
    """A seeded filled ellipse covering ~frac of the map: aspect U[0.5,2],
    angle U[0,pi), centre uniform such that the ellipse stays inside when it
    can.  At least one pixel is set."""
    area = frac * H * W
    aspect = rng.uniform(0.5, 2.0)
    ang = rng.uniform(0.0, math.pi)
    a = math.sqrt(area * aspect / math.pi)      # semi-axes, a/b = aspect
    b = a / aspect
    r = max(a, b)
    lo_y, hi_y = min(r, H / 2), max(H - r, H / 2)
    lo_x, hi_x = min(r, W / 2), max(W - r, W / 2)
    cy, cx = rng.uniform(lo_y, hi_y), rng.uniform(lo_x, hi_x)
    yy, xx = np.mgrid[0:H, 0:W]
    dy, dx = yy + 0.5 - cy, xx + 0.5 - cx
    u = dx * math.cos(ang) + dy * math.sin(ang)
    v = -dx * math.sin(ang) + dy * math.cos(ang)
    m = ((u / a) ** 2 + (v / b) ** 2 <= 1.0).astype(np.uint8)
    if m.sum() == 0:
        m[min(int(cy), H - 1), min(int(cx), W - 1)] = 1
    return m


def perturb(rng, x, pix, std=1.0, dtype="f32"):
    """x + N(0, std) at pixels where pix is set (all batch elements, channels)."""
    noise = std * rng.standard_normal(x.shape).astype(np.float32)
    return storage_round(x + noise * pix[None, :, :, None], dtype)


def params_from_shapes(rng, shapes, std=0.02, dtype="bf16"):
    """Random-init weights for a name -> shape table: weights N(0, std^2);
    1-D tensors: norm scales (names ending in '.g') 1 + N(0, std^2), everything
    else (biases, norm shifts) N(0, std^2)."""
    P = {}
    for name, shp in shapes.items():
        if name.endswith(".g"):
            P[name] = normal(rng, shp, std, dtype, mean=1.0)
        else:
            P[name] = normal(rng, shp, std, dtype)
    return P


def ddim_coeffs(t: int, t_prev: int, T: int = 1000, beta0: float = 0.00085, beta1: float = 0.012):
    """(a, b) of the deterministic sampler update x_prev = a * x + b * eps between timesteps t > t_prev of a
    scaled-linear noise schedule (harness arithmetic between two UNet evaluations; not part of the masked path)."""
    betas = np.linspace(math.sqrt(beta0), math.sqrt(beta1), T) ** 2
    ab = np.cumprod(1.0 - betas)
    at, ap = float(ab[t]), (float(ab[t_prev]) if t_prev >= 0 else 1.0)
    a = math.sqrt(ap / at)
    b = math.sqrt(1.0 - ap) - math.sqrt(ap * (1.0 - at) / at)
    return a, b
