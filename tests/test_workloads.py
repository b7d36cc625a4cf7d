"""The synthetic-input generator: same bits from torch as from a numpy uint64 reference of the
same hash, the stated distributions, and the routing skew each config is meant to have."""
import numpy as np
import torch

from workloads import CONFIGS, gate_bias, normal_bf16
from workloads import gen


def test_hash_matches_numpy_reference():
    for seed, tid, start in [(1, 0, 0), (250309716, 17, 12345), (99, 500, 1 << 33)]:
        a = gen._hash_index(seed, tid, start, 4096, "cpu").numpy()
        b = gen.hash_index_reference(seed, tid, start, 4096)
        np.testing.assert_array_equal(a, b)


def test_chunking_does_not_change_bits():
    a = normal_bf16(5, 3, (1000, 37), 0.02, chunk=1 << 24)
    b = normal_bf16(5, 3, (1000, 37), 0.02, chunk=4099)
    assert torch.equal(a.view(torch.int16), b.view(torch.int16))


def test_distribution():
    x = normal_bf16(7, 0, (512, 2048)).float()
    assert abs(x.mean().item()) < 5e-3 and abs(x.std().item() - 1.0) < 5e-3
    assert 4.0 < x.abs().max().item() <= 4.4
    w = normal_bf16(7, 1, (512, 2048), 0.02).float()
    assert abs(w.std().item() - 0.02) < 2e-4
    y = normal_bf16(7, 2, (512, 2048)).float()
    assert abs((x * y).mean().item()) < 5e-3        # different tensor ids are uncorrelated


def test_gate_bias_kinds():
    assert gate_bias(CONFIGS["C1"]) is None and gate_bias(CONFIGS["C4"]) is None
    b3 = gate_bias(CONFIGS["C3"]); assert b3.shape == (8,) and b3.dtype == np.float32
    b5 = gate_bias(CONFIGS["C5"])
    assert b5.shape == (160,) and b5.max() == 0.0 and abs(b5.min() + 1.1 * np.log(160)) < 1e-5
    np.testing.assert_array_equal(b5, gate_bias(CONFIGS["C5"]))
    b5b = gate_bias(CONFIGS["C5b"]); assert b5b.max() > 10
