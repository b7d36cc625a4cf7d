"""CPU tests of the comparison helpers the GPU parity tests rely on (tests/parity.py)."""
import numpy as np
import pytest

import parity as P


def _ref(logit, k, renorm):
    logit = logit.astype(np.float32)
    p = np.exp(logit - logit.max(1, keepdims=True)).astype(np.float64)
    p = (p / p.sum(1, keepdims=True)).astype(np.float32)
    idx = np.argsort(-logit, axis=1, kind="stable")[:, :k].astype(np.int32)
    w = np.take_along_axis(p, idx.astype(np.int64), 1)
    if renorm:
        w = w / w.sum(1, keepdims=True)
    return {"idx": idx, "w": w.astype(np.float32), "logits": logit, "probs": p}


@pytest.mark.parametrize("renorm", [True, False])
def test_near_tie_tokens_must_still_carry_the_right_weights(renorm):
    k = 2
    logit = np.array([[3.0, 2.0, 1.0, 0.0],
                      [3.0, 1.0 + 4e-6, 1.0, 0.0],       # near tie between the 2nd and 3rd largest
                      [0.5, 2.0, -1.0, 1.0]], np.float32)
    ref = _ref(logit, k, renorm)
    gpu_idx = ref["idx"].copy()
    gpu_idx[1] = [0, 2]                                   # the other side of the near tie
    sel = np.take_along_axis(ref["probs"].astype(np.float64), gpu_idx.astype(np.int64), 1)
    if renorm:
        sel = sel / sel.sum(1, keepdims=True)
    gpu_w = sel.astype(np.float32)
    rep = P.compare_routing(gpu_idx, gpu_w, ref, k, renorm)
    assert rep["mismatch_set_excused"] == [1] and rep["near_ties_in_oracle"] == 1
    bad_w = gpu_w.copy()
    bad_w[1, 1] *= 1.001                                  # an excused token with a wrong weight is not excused
    with pytest.raises(AssertionError):
        P.compare_routing(gpu_idx, bad_w, ref, k, renorm)
    far = ref["idx"].copy()
    far[0] = [0, 2]                                       # a set mismatch with a wide margin is an error
    with pytest.raises(AssertionError):
        P.compare_routing(far, ref["w"], ref, k, renorm)


def test_sample_reaches_every_tile_of_every_group():
    rng = np.random.default_rng(5)
    T, E, k = 6000, 24, 3
    logit = rng.standard_normal((T, E)) - 1.1 * np.log(rng.permutation(E) + 1.0)
    idx = np.argsort(-logit, 1)[:, :k].astype(np.int32)
    tok = P.sample_tokens(idx, E, 64, 1)
    assert len(np.unique(tok)) == len(tok) and tok.min() >= 0 and tok.max() < T
    for tm in P.TILE_ROWS:
        assert P.tiles_without_a_sampled_row(idx, E, tok, tm) == 0
        assert P.tiles_without_a_sampled_row(np.zeros((T, 1), np.int64), 1, tok, tm) == 0
    # the checker itself sees a gap: a sample of one token leaves tiles uncovered
    assert P.tiles_without_a_sampled_row(idx, E, tok[:1], 256) > 0


def test_bf16_bound_is_half_a_step_of_the_values_binade():
    ref = np.array([[1.0, 3.0, 100.0, 0.0]], np.float64)
    rms = float(np.sqrt((ref ** 2).mean()))
    bar = P.OUT_BAR * rms
    assert abs(bar - 1.0004) < 1e-3
    # |ref| + bar = 2.0004, 4.0004, 101.0004, 1.0004: binades 2^1, 2^2, 2^6, 2^0; half a bf16 step = 2^(e-8)
    half = np.array([2.0 ** -7, 2.0 ** -6, 2.0 ** -2, 2.0 ** -8])
    P.assert_output_bf16(ref + bar + 0.999 * half, ref)
    for i in range(4):
        worse = ref + bar + 0.999 * half
        worse[0, i] += 0.01 * half[i]
        with pytest.raises(AssertionError):
            P.assert_output_bf16(worse, ref)
