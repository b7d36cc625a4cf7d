"""GPU tests of the profiling interface (per-stage event times, interval read-out, measured MFMA ceiling)."""
import pytest
import torch

import parity as P
from workloads import make_layer_inputs, scaled_config

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def moe():
    from paper_2503_09716_amd import Moe
    m = Moe(0)
    yield m
    m.close()


def test_stage_intervals_cover_every_stage_of_every_step(moe):
    from paper_2503_09716_amd import STAGES
    cfg = scaled_config("C4", T=700, H=256, F=192)          # E > 16 and shared experts: every stage but the tiled gather runs
    gl = P.GpuLayer(moe, make_layer_inputs(cfg, device="cuda"), host_weights=False)
    gl.run_layer()
    moe.profile_enable(True)
    moe.profile_read()
    steps = 5
    for _ in range(steps):
        gl.run_layer()
    iv = moe.profile_read_intervals()
    for s in STAGES:
        n = 0 if s == "permute_gather" else steps
        assert len(iv[s]) == n, (s, iv[s])
        assert all(0.0 < v < 50.0 for v in iv[s])
    assert all(len(v) == 0 for v in moe.profile_read_intervals().values())     # the read-out clears the record
    # the summed read-out agrees with the intervals
    for _ in range(steps):
        gl.run_layer()
    sums = moe.profile_read()
    moe.profile_enable(False)
    for s in STAGES:
        assert sums[s][1] == (0 if s == "permute_gather" else steps)
    gl.run_layer()
    assert all(v[1] == 0 for v in moe.profile_read().values())                   # disabled: nothing recorded


def test_mfma_ceiling_is_plausible_and_validates_its_arguments(moe):
    from paper_2503_09716_amd import MoeError
    sink = torch.empty(1 << 20, dtype=torch.uint8, device="cuda")
    a = torch.randn(1 << 20, device="cuda").to(torch.bfloat16) * 0.02
    b = torch.randn(1 << 20, device="cuda").to(torch.bfloat16)
    iters = 2000
    tf0, ms0 = moe.mfma_ceiling(None, None, iters, sink)
    tf1, ms1 = moe.mfma_ceiling(a, b, iters, sink)
    flops = 1024 * 4 * iters * 64 * 2 * 16 * 16 * 32
    for tf, ms in ((tf0, ms0), (tf1, ms1)):
        assert abs(tf - flops / (ms * 1e-3) / 1e12) < 1e-6 * tf
        assert 500.0 < tf < 2600.0              # between a fifth of and just above the published bf16 peak
    with pytest.raises(MoeError):
        moe.mfma_ceiling(None, None, iters, sink[:1000])      # sink too small
    with pytest.raises(MoeError):
        moe.mfma_ceiling(None, None, 0, sink)
