"""The critical-path estimate of the streamed-weights layer (Sec. 4.4: longest path through the
DAG of copy and compute jobs), checked on the CPU against an independent event-driven
simulation of the two streams and the slot hand-over, and against closed forms."""
import numpy as np
import pytest

from paper_2503_09716_amd import binding


def simulate(copy_ms, comp_ms, slots):
    """Two in-order queues (copy stream, compute stream); copy g may start once compute g-slots
    has finished; compute g once copy g has finished.  Advances a clock event by event."""
    G = len(copy_ms)
    copy_done = [None] * G
    comp_done = [None] * G
    t_copy = t_comp = 0.0          # time at which each stream becomes free
    next_copy = next_comp = 0
    while next_comp < G:
        progressed = False
        if next_copy < G and (next_copy < slots or comp_done[next_copy - slots] is not None):
            start = t_copy if next_copy < slots else max(t_copy, comp_done[next_copy - slots])
            copy_done[next_copy] = start + copy_ms[next_copy]
            t_copy = copy_done[next_copy]
            next_copy += 1
            progressed = True
        if copy_done[next_comp] is not None:
            start = max(t_comp, copy_done[next_comp])
            comp_done[next_comp] = start + comp_ms[next_comp]
            t_comp = comp_done[next_comp]
            next_comp += 1
            progressed = True
        assert progressed
    return comp_done[-1]


def groups_of(rows, per_group, num_shared, T):
    out, e, E = [], 0, len(rows)
    while e < E:
        while e < E and rows[e] == 0:
            e += 1
        if e >= E:
            break
        n = r = 0
        while e < E and n < per_group:
            if rows[e] > 0:
                n += 1
                r += rows[e]
            e += 1
        out.append((n, r))
    if num_shared:
        out.append((num_shared, num_shared * T))
    return out


@pytest.mark.parametrize("seed", range(8))
def test_estimate_matches_event_simulation(seed):
    rng = np.random.default_rng(seed)
    E = int(rng.integers(1, 40))
    k = int(rng.integers(1, min(E, 6) + 1))
    T = int(rng.integers(1, 5000))
    ns = int(rng.integers(0, 3))
    H, F = 64 * int(rng.integers(1, 9)), 64 * int(rng.integers(1, 9))
    shape = binding.make_shape(T, H, F, E, k, ns)
    rows = rng.multinomial(T * k, rng.dirichlet(np.full(E, 0.3))).astype(np.int32)   # skewed, some experts empty
    per_group = int(rng.integers(1, E + 1))
    slots = int(rng.integers(2, 5))
    link, tf = float(rng.uniform(10, 100)), float(rng.uniform(0.001, 2.0))
    got = binding.estimate_streamed_ms(shape, rows, per_group, slots, link, tf)
    expert_ms = 3.0 * H * F * 2 / (link * 1e9) * 1e3
    row_ms = 6.0 * H * F / (tf * 1e12) * 1e3
    gs = groups_of(rows.tolist(), per_group, ns, T)
    want = simulate([n * expert_ms for n, _ in gs], [r * row_ms for _, r in gs], slots)
    assert got == pytest.approx(want, rel=1e-12)


def test_estimate_closed_forms():
    shape = binding.make_shape(1000, 128, 256, 4, 1)
    rows = [250, 250, 250, 250]
    expert_ms = 3.0 * 128 * 256 * 2 / 50e9 * 1e3
    # compute negligible: every copy back to back, then the last group's compute
    slow_link = binding.estimate_streamed_ms(shape, rows, 1, 2, 50.0, 1e9)
    assert slow_link == pytest.approx(4 * expert_ms, rel=1e-5)
    # copies negligible: the first copy, then all compute back to back
    row_ms = 6.0 * 128 * 256 / 1e9 * 1e3          # at 0.001 TFLOP/s
    fast_link = binding.estimate_streamed_ms(shape, rows, 1, 2, 1e9, 0.001)
    assert fast_link == pytest.approx(1000 * row_ms, rel=1e-5)
    # empty experts cost nothing
    assert binding.estimate_streamed_ms(shape, [500, 0, 0, 500], 1, 2, 50.0, 1e9) == pytest.approx(2 * expert_ms, rel=1e-5)
    # invalid arguments
    assert binding.estimate_streamed_ms(shape, rows, 0, 2, 50.0, 1.0) < 0
    assert binding.estimate_streamed_ms(shape, rows, 1, 1, 50.0, 1.0) < 0
    assert binding.estimate_streamed_ms(shape, rows, 1, 2, 0.0, 1.0) < 0
