"""GPU checks of the measurement support: per-launch event log and the empirical-ceiling probe."""
import numpy as np
import pytest
import torch

from paper_2305_17423_amd import workloads as wl
from helpers import DEV, dev, idx_dev

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def fb():
    from paper_2305_17423_amd import binding
    binding.lib()
    assert torch.cuda.is_available()
    return binding


def test_calibrate_peaks_plausible_and_validated(fb):
    scratch = torch.zeros(1 << 30, dtype=torch.uint8, device=DEV)   # halves larger than the 256 MB last-level cache
    scratch[: 512 << 20] = 7
    gbs, tf = fb.fise_calibrate_peaks(scratch)
    # a copy cannot beat the 8 TB/s the memory is rated for, nor the MFMA loop the 2.5 PFLOP/s dense bf16 rating;
    # both should be well above what a broken measurement (one wave, one CU) would give
    assert 500.0 < gbs < 8000.0, gbs
    assert 200.0 < tf < 2600.0, tf
    assert int(scratch[(512 << 20) + 12345]) == 7            # the copy pass really moved the first half
    with pytest.raises(fb.FiseError) as e:
        fb.fise_calibrate_peaks(torch.zeros(1 << 20, dtype=torch.uint8, device=DEV))
    assert e.value.code == -5                               # FISE_ERR_CAPACITY


def test_profile_log_counts_launches(fb):
    """One bf16 conv with a long K: the log holds its GEMM launch (and its reduce), with the algorithmic
    FLOPs 2*M*N*K, and empty brackets are shorter than brackets around a kernel."""
    rng = np.random.default_rng(5)
    B, H, W, C, t = 2, 16, 16, 128, 4
    x = dev(wl.normal(rng, (B, H, W, C), 1.0, "bf16"), "bf16")
    w = dev(wl.normal(rng, (C, 3, 3, C), 0.03, "bf16"), "bf16")
    y = torch.zeros((B, H, W, C), dtype=torch.bfloat16, device=DEV)
    tiles = np.arange(6, dtype=np.int32)
    ws = torch.zeros(32 << 20, dtype=torch.uint8, device=DEV)
    fb.fise_profile_read(-1)
    fb.fise_profile_enable(True)
    fb.fise_masked_conv3x3(x, w, None, 1, idx_dev(tiles), tiles.size, t, y, workspace=ws)
    fb.fise_profile_enable(False)
    fb.fise_profile_calibrate(20)
    torch.cuda.synchronize()
    got = {k: fb.fise_profile_read(k) for k in range(10)}
    fb.fise_profile_read(-1)
    gemm = [k for k in (0, 3, 5, 6) if got[k][3]]
    assert len(gemm) == 1 and got[gemm[0]][3] == 1
    M = B * tiles.size * t * t
    assert got[gemm[0]][1] == pytest.approx(2.0 * M * C * 9 * C)
    assert got[8][3] == 20 and got[8][0] > 0
    assert got[gemm[0]][0] > got[8][0] / 20                  # a kernel between the events takes longer than nothing
    assert fb.fise_profile_read(0)[3] == 0                   # cleared
