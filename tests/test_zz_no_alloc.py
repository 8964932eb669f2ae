"""GPU check of the entry point that allocates nothing (fise_groupnorm_stats_static: the partial sums live in a
fixed device array owned by the library): through the C ABI, against the existing fise_groupnorm_stats bit for bit
and against the oracle to the fp32 bar, on two calls in a row, the second with a smaller input (the shared array
keeps the first call's contents); sizes beyond the array are refused before anything is launched."""
import ctypes

import numpy as np
import pytest
import torch

from oracle import fise_oracle as fo
from paper_2305_17423_amd import workloads as wl
from helpers import DEV, dev, host, rel_err

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def fb():
    from paper_2305_17423_amd import binding
    binding.lib()
    assert torch.cuda.is_available()
    return binding


def run_both(fb, x, x1, G, eps, dtype):
    L = fb.lib()
    B, H, W, C0 = x.shape
    C1 = 0 if x1 is None else x1.shape[-1]
    xd = dev(x, dtype); x1d = None if x1 is None else dev(x1, dtype)
    ws = torch.zeros(fb.fise_groupnorm_stats_workspace_bytes(B, H, W, C0 + C1), dtype=torch.uint8, device=DEV)
    out = [torch.full((B, G), float("nan"), dtype=torch.float32, device=DEV) for _ in range(4)]
    p = lambda t: ctypes.c_void_p(t.data_ptr()) if t is not None else None
    dt = fb.FISE_F32 if dtype == "f32" else fb.FISE_BF16
    torch.cuda.synchronize()
    assert L.fise_groupnorm_stats(p(xd), p(x1d), dt, B, H, W, C0, C1, G, eps, p(out[0]), p(out[1]), p(ws), None) == 0, fb.fise_last_error()
    assert L.fise_groupnorm_stats_static(p(xd), p(x1d), dt, B, H, W, C0, C1, G, eps, p(out[2]), p(out[3]), None) == 0, fb.fise_last_error()
    torch.cuda.synchronize()
    assert torch.equal(out[0], out[2]) and torch.equal(out[1], out[3]), "static entry point differs from the workspace one"
    src = x if x1 is None else [x, x1]
    m_o, r_o = fo.gn_stats(src, G, eps)
    assert np.abs(host(out[2]) - m_o).max() <= 1e-4 * max(1.0, np.abs(m_o).max())
    assert rel_err(host(out[3]), r_o) <= 1e-4
    return out[2], out[3]


def test_static_scratch_entry_point_two_calls(fb):
    rng = np.random.default_rng(7001)
    assert fb.fise_groupnorm_stats_static_capacity_bytes() == 1 << 20
    # first call: SD-1.5 level-0 shape (2 x 64 chunks x 32 groups of partial sums), two concatenated sources
    x = wl.normal(rng, (2, 64, 64, 320), 1.0, "bf16", mean=0.3); x1 = wl.normal(rng, (2, 64, 64, 320), 2.0, "bf16")
    run_both(fb, x, x1, 32, 1e-5, "bf16")
    # second call right after it: a smaller fp32 map with a ragged last chunk (the array still holds the first call's sums)
    y = wl.normal(rng, (1, 9, 11, 24), 1.5, "f32", mean=-0.7)
    run_both(fb, y, None, 4, 1e-6, "f32")
    # and the first shape again, one source
    run_both(fb, x, None, 32, 1e-5, "bf16")


def test_static_scratch_capacity_is_enforced(fb):
    L = fb.lib()
    a = ctypes.c_void_p(0x1000)            # never dereferenced: the size check comes first
    # 8 x ceil(256*256/64) x 64 x 16 bytes = 8 MiB > 1 MiB
    assert L.fise_groupnorm_stats_static(a, None, fb.FISE_BF16, 8, 256, 256, 64, 0, 64, 1e-5, a, a, None) == -5
    assert "scratch" in fb.fise_last_error()
    assert L.fise_groupnorm_stats_static(None, None, fb.FISE_BF16, 1, 8, 8, 32, 0, 4, 1e-5, a, a, None) == -1
    assert L.fise_groupnorm_stats_static(a, None, fb.FISE_BF16, 1, 8, 8, 30, 0, 4, 1e-5, a, a, None) == -2
