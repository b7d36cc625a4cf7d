"""GPU parity of each staged C-ABI call against the CPU oracle, element by element, at sizes
the oracle finishes in seconds but that span several tiles and ragged tails."""
import os

import numpy as np
import pytest
import torch

from oracle import moe_oracle as orc
import parity as P
from workloads import get_config, make_layer_inputs, normal_bf16, scaled_config, torch_bf16_to_u16

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def moe():
    from paper_2503_09716_amd import Moe
    m = Moe(0)
    yield m
    m.close()


# Seeded random cases per sweep below; MOE_FUZZ_SEEDS=400 runs the long version (a minute or two on the GPU).
FUZZ_SEEDS = int(os.environ.get("MOE_FUZZ_SEEDS", "48"))


def say(*a):
    print(*a, flush=True)


ROUTE_CASES = [
    ("C1", {}),
    ("C2", dict(T=777, H=512)),
    ("C3", dict(T=300, H=256)),
    ("C4", dict(T=1000, H=512)),
    ("C5", dict(T=1500, H=1024)),
    ("C5b", dict(T=257, H=256)),
    ("C1", dict(T=1, H=64)),
    ("C1", dict(T=33, H=64, E=8, top_k=8)),      # k = E
    ("C4", dict(T=65, H=128, E=200, top_k=13)),   # E not a multiple of 32, odd k
    ("C1", dict(T=101, H=128, E=5, top_k=2)),     # few experts, not a vector width
    ("C1", dict(T=70, H=192, E=16, top_k=4)),
    ("C3", dict(T=50, H=64, E=12, top_k=3)),
    ("C1", dict(T=9, H=1088, E=1, top_k=1)),
    ("C4", dict(T=700, H=1024)),                  # matrix-core path, 4 K-splits
    ("C5", dict(T=300, H=384)),                   # 1 K-split, 160 experts padded to 160
    ("C5", dict(T=130, H=192, E=17, top_k=5)),    # 17 experts padded to 32
    ("C5", dict(T=200, H=1088, E=40, top_k=6)),   # H/32 = 34: 2 K-splits of 17 sub-tiles
    ("C4", dict(T=300, H=3520)),                  # H/32 = 110: 5 K-splits (a single chain this long misses the logit bar)
    ("C5", dict(T=260, H=6336, E=163, top_k=8)),  # H/32 = 198: 6 K-splits of 33 sub-tiles
    ("C4", dict(T=130, H=7168, E=33, top_k=4)),   # 7 K-splits
    ("C4", dict(T=140, H=4544, E=74, top_k=5)),   # H/32 = 2 * 71: 2 K-splits of 2272 terms, the longest chains in use
    ("C3", dict(T=64, H=128, E=256, top_k=8)),
    ("C4", dict(T=50, H=64, E=256, top_k=64, num_shared=0)),    # the largest expert count and k the library accepts
    ("C5", dict(T=1, H=64, E=160, top_k=6)),      # a single token through the matrix-core path
]


@pytest.mark.parametrize("name,over", ROUTE_CASES)
def test_route(moe, name, over):
    from paper_2503_09716_amd import shape_of
    cfg = scaled_config(name, **over) if over else get_config(name)
    say("route", cfg)
    li = make_layer_inputs(cfg, device="cuda", experts=False)
    shape = shape_of(cfg)
    idx = torch.empty((cfg.T, cfg.top_k), dtype=torch.int32, device="cuda")
    w = torch.empty((cfg.T, cfg.top_k), dtype=torch.float32, device="cuda")
    logits = torch.empty((cfg.T, cfg.E), dtype=torch.float32, device="cuda")
    bias = None if li.bias is None else torch.from_numpy(li.bias).cuda()
    ws = moe.new_workspace(shape)
    moe.route(shape, li.x, li.wg, bias, idx, w, logits, ws)
    torch.cuda.synchronize()
    ref = orc.route(torch_bf16_to_u16(li.x), torch_bf16_to_u16(li.wg), li.bias, cfg.top_k, cfg.renormalize,
                    cfg.routed_scale, want_logits=True, want_probs=True)
    rep = P.compare_routing(idx.cpu().numpy(), w.cpu().numpy(), ref, cfg.top_k, cfg.renormalize, cfg.routed_scale)
    say(rep)
    err = np.abs(logits.cpu().numpy() - ref["logits"]).max()
    assert err < 5e-6, err
    if cfg.renormalize:
        np.testing.assert_allclose(w.sum(1).cpu().numpy(), cfg.routed_scale, atol=2e-6)
    # without the optional logits output the result is the same, bit for bit
    idx2 = torch.empty_like(idx); w2 = torch.empty_like(w)
    moe.route(shape, li.x, li.wg, bias, idx2, w2, None, ws)
    torch.cuda.synchronize()
    assert torch.equal(idx, idx2) and torch.equal(w, w2)
    # a gate matrix packed once by the caller gives the same bits as packing per call
    wgp = moe.pack_gate(shape, li.wg)
    ws2 = torch.full_like(ws, 0x5A)          # nothing may be read from the workspace's gate region
    idx3 = torch.empty_like(idx); w3 = torch.empty_like(w)
    moe.set_option("gate_packed", 1)
    try:
        moe.route(shape, li.x, wgp, bias, idx3, w3, None, ws2)
        torch.cuda.synchronize()
    finally:
        moe.set_option("gate_packed", 0)
    assert torch.equal(idx, idx3) and torch.equal(w, w3)


@pytest.mark.parametrize("T,H,E,k", [(40, 64, 70, 3), (40, 64, 16, 16), (21, 128, 8, 2), (33, 64, 5, 5), (1, 64, 1, 1)])
def test_route_exact_ties_pick_lowest_expert(moe, T, H, E, k):
    from paper_2503_09716_amd import make_shape
    x = normal_bf16(1, 0, (T, H), 1.0, "cuda")
    wg = torch.zeros((H, E), dtype=torch.bfloat16, device="cuda")
    idx = torch.empty((T, k), dtype=torch.int32, device="cuda")
    w = torch.empty((T, k), dtype=torch.float32, device="cuda")
    shape = make_shape(T, H, 64, E, k, 0, False)
    moe.route(shape, x, wg, None, idx, w, None, moe.new_workspace(shape))
    torch.cuda.synchronize()
    assert (idx.cpu().numpy() == np.arange(k)[None, :]).all()
    np.testing.assert_allclose(w.cpu().numpy(), 1.0 / E, rtol=1e-6)


@pytest.mark.parametrize("seed", range(FUZZ_SEEDS))
def test_route_random_shapes(moe, seed):
    """Seeded random router shapes (T up to 9000, H up to 6336 in steps of 64, 1..256 experts, k up to 16, the
    three kinds of gate bias): selection against the oracle, logits within 5e-6."""
    from paper_2503_09716_amd import shape_of
    rng = np.random.default_rng(91000 + seed)
    E = int(rng.integers(1, 17)) if seed % 3 else int(rng.integers(17, 257))
    k = int(rng.integers(1, min(E, 16) + 1))
    cfg = scaled_config(["C2", "C3", "C4", "C5"][seed % 4], T=int(rng.integers(1, 9000)), H=64 * int(rng.integers(1, 100)),
                        E=E, top_k=k, bias=["none", "normal", "logzipf_rank"][seed % 3])
    say("route fuzz", seed, cfg.T, cfg.H, E, k, cfg.bias, cfg.renormalize)
    li = make_layer_inputs(cfg, device="cuda", experts=False)
    shape = shape_of(cfg)
    idx = torch.empty((cfg.T, k), dtype=torch.int32, device="cuda")
    w = torch.empty((cfg.T, k), dtype=torch.float32, device="cuda")
    logits = torch.empty((cfg.T, E), dtype=torch.float32, device="cuda")
    bias = None if li.bias is None else torch.from_numpy(li.bias).cuda()
    moe.route(shape, li.x, li.wg, bias, idx, w, logits, moe.new_workspace(shape))
    torch.cuda.synchronize()
    ref = orc.route(torch_bf16_to_u16(li.x), torch_bf16_to_u16(li.wg), li.bias, k, cfg.renormalize, cfg.routed_scale,
                    want_logits=True, want_probs=True)
    say(P.compare_routing(idx.cpu().numpy(), w.cpu().numpy(), ref, k, cfg.renormalize, cfg.routed_scale))
    err = np.abs(logits.cpu().numpy() - ref["logits"]).max()
    assert err < 5e-6, err


def random_routing(rng, T, E, k, skew=None):
    """Distinct experts per token.  skew = 'one': expert 0 stays empty, every token goes to expert 1,
    and the top third of the expert ids is hit by a single token each (tiny groups)."""
    if skew != "one":
        return np.stack([rng.permutation(E)[:k] for _ in range(T)]).astype(np.int32)
    lo = np.arange(1, E - E // 3)
    idx = np.stack([rng.permutation(lo)[:k] for _ in range(T)]).astype(np.int32)
    for t in range(T):
        if 1 not in idx[t]:
            idx[t, 0] = 1
    for i, e in enumerate(range(E - E // 3, E)):
        if k > 1:
            idx[i, 1] = e
    return idx


# One launch up to 4096 pairs, beyond that two (histogram; scan + placement), three when the table of histograms is large
PERMUTE_CASES = [(256, 8, 2, None), (1000, 64, 6, None), (777, 160, 6, "one"), (1, 4, 1, None), (300, 5, 5, None),
                 (2049, 37, 3, None), (682, 256, 6, None), (683, 256, 6, None), (500, 160, 6, "one"), (12000, 37, 6, "one"),
                 (32768, 8, 2, None), (16384, 16, 4, None), (16385, 16, 4, None), (4099, 13, 3, "one"), (1025, 17, 4, None),
                 (40000, 256, 2, None), (16384, 160, 8, None), (16640, 64, 6, "one"), (16385, 64, 1, None),
                 (16384, 256, 1, None), (16385, 256, 1, None)]


def check_permute(moe, T, E, k, idx_h, H=128):
    """moe_permute on the given routing against the oracle's stable counting sort, bit for bit."""
    from paper_2503_09716_amd import make_shape
    shape = make_shape(T, H, 64, E, k)
    x = normal_bf16(3, 0, (T, H), 1.0, "cuda")
    idx = torch.from_numpy(idx_h).cuda()
    R = T * k
    x_perm = torch.empty((R, H), dtype=torch.bfloat16, device="cuda")
    off = torch.empty(E + 1, dtype=torch.int32, device="cuda")
    perm = torch.empty(R, dtype=torch.int32, device="cuda")
    inv = torch.empty(R, dtype=torch.int32, device="cuda")
    rtok = torch.empty(R, dtype=torch.int32, device="cuda")
    ws = moe.new_workspace(shape)
    moe.permute(shape, x, idx, x_perm, off, perm, inv, rtok, ws)
    torch.cuda.synchronize()
    o_off, o_perm, o_inv = orc.permute(idx_h, E)
    np.testing.assert_array_equal(off.cpu().numpy(), o_off)
    np.testing.assert_array_equal(perm.cpu().numpy(), o_perm)
    np.testing.assert_array_equal(inv.cpu().numpy(), o_inv)
    np.testing.assert_array_equal(rtok.cpu().numpy(), o_perm // k)
    xh = torch_bf16_to_u16(x)
    np.testing.assert_array_equal(torch_bf16_to_u16(x_perm), xh[o_perm // k])
    # every token appears exactly k times
    np.testing.assert_array_equal(np.bincount(perm.cpu().numpy() // k, minlength=T), np.full(T, k))


@pytest.mark.parametrize("T,E,k,skew", PERMUTE_CASES)
def test_permute(moe, T, E, k, skew):
    say("permute", T, E, k, skew)
    rng = np.random.default_rng(T * 7 + E)
    check_permute(moe, T, E, k, random_routing(rng, T, E, k, skew))


@pytest.mark.parametrize("seed", range(FUZZ_SEEDS))
def test_permute_random_shapes(moe, seed):
    """Seeded random shapes across the one-, two- and three-launch paths (1..70000 tokens, 1..256 experts,
    k up to 8; uniform routing, one expert taking every token, or everything on k + 1 experts)."""
    rng = np.random.default_rng(55000 + seed)
    E = int(rng.integers(1, 257))
    k = int(rng.integers(1, min(E, 8) + 1))
    T = int([rng.integers(1, 600), rng.integers(600, 20000), rng.integers(20000, 70000)][seed % 3])
    idx_h = random_routing(rng, T, E, k, "one" if (seed % 5 == 0 and E >= 6) else None)
    if seed % 7 == 0 and k < E:
        idx_h = np.stack([(np.arange(k) + (t % 2)) % E for t in range(T)]).astype(np.int32)
    say("permute fuzz", seed, T, E, k)
    check_permute(moe, T, E, k, idx_h, H=64)


def run_ffn_stage(moe, cfg, idx_h, wave_rows=2, small_tiles=1, use_row_token=False, y_fp32=True, waves=4):
    """Runs moe_permute + moe_grouped_ffn for a given routing; returns (y_perm, y_shared, perm, li)."""
    from paper_2503_09716_amd import shape_of
    shape = shape_of(cfg)
    li = make_layer_inputs(cfg, device="cuda")
    w1p, w3p, w2p = moe.pack_experts(li.w1, li.w3, li.w2)
    R = cfg.T * cfg.top_k
    idx = torch.from_numpy(idx_h).cuda()
    x_perm = torch.empty((R, cfg.H), dtype=torch.bfloat16, device="cuda")
    off = torch.empty(cfg.E + 1, dtype=torch.int32, device="cuda")
    perm = torch.empty(R, dtype=torch.int32, device="cuda")
    inv = torch.empty(R, dtype=torch.int32, device="cuda")
    rtok = torch.empty(R, dtype=torch.int32, device="cuda")
    ws = moe.new_workspace(shape)
    moe.permute(shape, li.x, idx, x_perm, off, perm, inv, rtok, ws)
    h = moe.new_h_scratch(shape)
    ydt = torch.float32 if y_fp32 else torch.bfloat16
    y = torch.full((R, cfg.H), float("nan"), dtype=ydt, device="cuda")
    ysh = torch.full((cfg.T, cfg.H), float("nan"), dtype=ydt, device="cuda") if cfg.num_shared else None
    moe.set_option("gemm_waves", waves)
    moe.set_option("gemm_wave_rows", wave_rows)
    moe.set_option("small_tiles", small_tiles)
    moe.set_option("y_fp32", 1 if y_fp32 else 0)
    try:
        moe.grouped_ffn(shape, None if use_row_token else x_perm, rtok if use_row_token else None, li.x, off,
                        w1p, w3p, w2p, h, y, ysh, ws)
        torch.cuda.synchronize()
    finally:
        moe.set_option("gemm_waves", DEFAULT_WAVES)
        moe.set_option("gemm_wave_rows", DEFAULT_WAVE_ROWS)
        moe.set_option("small_tiles", 1)
        moe.set_option("y_fp32", 1)
    return y, ysh, perm.cpu().numpy(), off.cpu().numpy(), li


DEFAULT_WAVES, DEFAULT_WAVE_ROWS = 4, 1

FFN_CASES = [
    # name, overrides, skew, waves, wave_rows, small_tiles, row_token
    ("C1", {}, None, 4, 2, 1, False),
    ("C1", {}, None, 4, 1, 1, True),
    ("C1", {}, None, 8, 2, 1, True),
    ("C1", dict(T=333, H=192, F=320), None, 4, 2, 0, False),        # ragged rows, N not a multiple of the tile
    ("C1", dict(T=333, H=192, F=320), None, 8, 4, 0, False),
    ("C4", dict(T=512, H=256, F=192, E=16, top_k=4), None, 4, 2, 1, True),   # shared experts, K-concatenated down proj
    ("C4", dict(T=512, H=256, F=192, E=16, top_k=4), None, 8, 2, 1, True),
    ("C4", dict(T=300, H=128, F=128, E=16, top_k=4), None, 4, 1, 1, False),
    ("C4", dict(T=300, H=128, F=128, E=16, top_k=4), None, 8, 4, 1, False),
    ("C5", dict(T=700, H=256, F=128, E=40, top_k=3), "one", 4, 2, 1, False),  # one hot expert, tiny and empty experts
    ("C5", dict(T=700, H=256, F=128, E=40, top_k=3), "one", 8, 2, 1, False),
    ("C5", dict(T=700, H=256, F=128, E=40, top_k=3), "one", 4, 1, 1, False),
    ("C1", dict(T=40, H=64, F=64, E=4, top_k=1), None, 4, 2, 1, False),
    ("C1", dict(T=40, H=64, F=64, E=4, top_k=1), None, 8, 4, 1, False),
]


@pytest.mark.parametrize("name,over,skew,waves,wave_rows,small_tiles,row_token", FFN_CASES)
def test_grouped_ffn(moe, name, over, skew, waves, wave_rows, small_tiles, row_token):
    cfg = scaled_config(name, **over) if over else get_config(name)
    say("grouped_ffn", cfg, skew, waves, wave_rows, small_tiles, row_token)
    rng = np.random.default_rng(cfg.T + cfg.E)
    idx_h = random_routing(rng, cfg.T, cfg.E, cfg.top_k, skew)
    y, ysh, perm, off, li = run_ffn_stage(moe, cfg, idx_h, wave_rows, small_tiles, row_token, waves=waves)
    u = torch_bf16_to_u16
    hw1 = [u(t) for t in li.w1]; hw3 = [u(t) for t in li.w3]; hw2 = [u(t) for t in li.w2]
    hx = u(li.x)
    rows_x = hx[perm // cfg.top_k]
    eid = np.repeat(np.arange(cfg.E, dtype=np.int32), np.diff(off))
    ref = orc.expert_rows(rows_x, eid, hw1, hw3, hw2)
    rep = P.assert_output(y.float().cpu().numpy(), ref, "y_perm")
    say(rep)
    if cfg.num_shared:
        ref_s = np.zeros((cfg.T, cfg.H), np.float32)
        for s in range(cfg.num_shared):
            ref_s += orc.expert_rows(hx, np.full(cfg.T, cfg.E + s, np.int32), hw1, hw3, hw2)
        say(P.assert_output(ysh.float().cpu().numpy(), ref_s, "y_shared"))


TAIL_COUNTS = [256 + 1, 256 + 32, 256 + 33, 256 + 64, 256 + 65, 512 + 40, 255, 1, 0, 300, 256, 768 + 64, 129, 64]


@pytest.mark.parametrize("F,num_shared,tall", [(128, 0, -1), (128, 2, -1), (512, 0, -1), (512, 1, -1), (512, 1, 1), (128, 2, 0)])
def test_grouped_ffn_every_tail_class(moe, F, num_shared, tall):
    """Prescribed rows per expert (top-1 routing laid out by hand) so that one launch holds every
    kind of m-tile: tails of 1, 32, 33 and 64 rows that join a full tile (288- and 320-row tiles),
    a 65-row tail that does not, short tails that are moved (and cut along K when F = 512), tails
    above half a tile, an empty expert, single-row and exact-multiple groups; T itself ends in a
    short tail for the shared experts.  Every row against the oracle."""
    counts = np.array(TAIL_COUNTS)
    E, T = len(counts), int(counts.sum())
    cfg = scaled_config("C4", T=T, H=192, F=F, E=E, top_k=1, num_shared=num_shared)
    idx_h = np.repeat(np.arange(E, dtype=np.int32), counts)
    idx_h = idx_h[np.random.default_rng(5).permutation(T)].reshape(T, 1)
    say("tail classes", cfg, "tall_tiles", tall)
    moe.set_option("tall_tiles", tall)
    moe.set_option("down_tail_splits", 2)   # cut every eligible tail (the library's own rule would not, in a launch this short)
    try:
        y, ysh, perm, off, li = run_ffn_stage(moe, cfg, idx_h, wave_rows=1)
    finally:
        moe.set_option("tall_tiles", -1)
        moe.set_option("down_tail_splits", 1)
    np.testing.assert_array_equal(np.diff(off), counts)
    u = torch_bf16_to_u16
    hw1 = [u(t) for t in li.w1]; hw3 = [u(t) for t in li.w3]; hw2 = [u(t) for t in li.w2]
    hx = u(li.x)
    eid = np.repeat(np.arange(E, dtype=np.int32), counts)
    ref = orc.expert_rows(hx[perm], eid, hw1, hw3, hw2)
    say(P.assert_output(y.float().cpu().numpy(), ref, "y_perm"))
    if num_shared:
        ref_s = np.zeros((T, cfg.H), np.float32)
        for sh in range(num_shared):
            ref_s += orc.expert_rows(hx, np.full(T, E + sh, np.int32), hw1, hw3, hw2)
        say(P.assert_output(ysh.float().cpu().numpy(), ref_s, "y_shared"))


def test_grouped_ffn_bf16_y(moe):
    """Option y_fp32 = 0: y in bf16 is the RNE rounding of the fp32 y, bit for bit."""
    cfg = scaled_config("C4", T=300, H=256, F=192, E=16, top_k=4)
    rng = np.random.default_rng(3)
    idx_h = random_routing(rng, cfg.T, cfg.E, cfg.top_k)
    y32, s32, _, _, _ = run_ffn_stage(moe, cfg, idx_h)
    y16, s16, _, _, _ = run_ffn_stage(moe, cfg, idx_h, y_fp32=False)
    assert torch.equal(y32.to(torch.bfloat16).view(torch.int16), y16.view(torch.int16))
    assert torch.equal(s32.to(torch.bfloat16).view(torch.int16), s16.view(torch.int16))


def test_grouped_ffn_single_expert_is_dense_mlp(moe):
    """E = 1, top-1: the grouped FFN is a dense SwiGLU MLP; checked against torch fp64 on the CPU."""
    cfg = scaled_config("C1", T=200, H=128, F=256, E=1, top_k=1)
    idx_h = np.zeros((cfg.T, 1), np.int32)
    y, _, perm, off, li = run_ffn_stage(moe, cfg, idx_h)
    assert (perm == np.arange(cfg.T)).all()
    x = li.x.double().cpu()
    ref = (torch.nn.functional.silu(x @ li.w1[0].double().cpu()) * (x @ li.w3[0].double().cpu())) @ li.w2[0].double().cpu()
    say(P.assert_output(y.float().cpu().numpy(), ref.numpy(), "dense"))


def test_grouped_ffn_exact_scaling(moe):
    """Doubling W2 doubles y bit-exactly (power-of-two scaling commutes with every rounding)."""
    from paper_2503_09716_amd import shape_of
    cfg = scaled_config("C1", T=128, H=128, F=128, E=4, top_k=2)
    rng = np.random.default_rng(5)
    idx_h = random_routing(rng, cfg.T, cfg.E, cfg.top_k)
    y1, _, _, _, li = run_ffn_stage(moe, cfg, idx_h)
    shape = shape_of(cfg)
    w1p, w3p, w2p = moe.pack_experts(li.w1, li.w3, [w * 2 for w in li.w2])
    R = cfg.T * cfg.top_k
    idx = torch.from_numpy(idx_h).cuda()
    x_perm = torch.empty((R, cfg.H), dtype=torch.bfloat16, device="cuda")
    off = torch.empty(cfg.E + 1, dtype=torch.int32, device="cuda")
    perm = torch.empty(R, dtype=torch.int32, device="cuda"); inv = torch.empty_like(perm)
    ws = moe.new_workspace(shape)
    moe.permute(shape, li.x, idx, x_perm, off, perm, inv, None, ws)
    h = moe.new_h_scratch(shape)
    y2 = torch.empty((R, cfg.H), dtype=torch.float32, device="cuda")
    moe.grouped_ffn(shape, x_perm, None, None, off, w1p, w3p, w2p, h, y2, None, ws)
    torch.cuda.synchronize()
    assert torch.equal(y1 * 2, y2)


COMBINE_CASES = [(256, 512, 2, False, True), (333, 2048, 6, True, True), (1, 64, 1, False, True),
                 (100, 5120, 6, True, False), (77, 1024, 2, False, False)]


@pytest.mark.parametrize("T,H,k,shared,y_fp32", COMBINE_CASES)
def test_combine(moe, T, H, k, shared, y_fp32):
    from paper_2503_09716_amd import make_shape
    say("combine", T, H, k, shared, y_fp32)
    rng = np.random.default_rng(T + H)
    shape = make_shape(T, H, 64, max(k, 8), k, 1 if shared else 0, False)
    y = normal_bf16(9, 0, (T * k, H), 1.0, "cuda")
    ysh = normal_bf16(9, 1, (T, H), 1.0, "cuda") if shared else None
    if y_fp32:   # fp32 values with a full mantissa
        y = y.float() * 1.0009765625
        ysh = None if ysh is None else ysh.float() * 0.9990234375
    to_host = (lambda t: t.cpu().numpy()) if y_fp32 else torch_bf16_to_u16
    inv_h = rng.permutation(T * k).astype(np.int32)
    w_h = rng.random((T, k)).astype(np.float32)
    inv = torch.from_numpy(inv_h).cuda(); w = torch.from_numpy(w_h).cuda()
    ref = orc.combine(to_host(y), inv_h, w_h, None if ysh is None else to_host(ysh))
    moe.set_option("y_fp32", 1 if y_fp32 else 0)
    try:
        out32 = torch.empty((T, H), dtype=torch.float32, device="cuda")
        moe.set_option("out_fp32", 1)
        moe.combine(shape, y, inv, w, ysh, out32)
        moe.set_option("out_fp32", 0)
        out16 = torch.empty((T, H), dtype=torch.bfloat16, device="cuda")
        moe.combine(shape, y, inv, w, ysh, out16)
        torch.cuda.synchronize()
        # fp32 sums in the same order; the GPU fuses each multiply-add (one rounding instead of two)
        np.testing.assert_allclose(out32.cpu().numpy(), ref, rtol=2e-6, atol=2e-6)
        assert torch.equal(out32.to(torch.bfloat16).view(torch.int16), out16.view(torch.int16))
        # k = 1, w = 1 is a pure gather: bit-exact
        inv1 = rng.permutation(T).astype(np.int32)
        shape1 = make_shape(T, H, 64, 8, 1, 0, False)
        y1 = y[:T].contiguous()
        moe.set_option("out_fp32", 1 if y_fp32 else 0)
        out1 = torch.empty((T, H), dtype=y.dtype, device="cuda")
        moe.combine(shape1, y1, torch.from_numpy(inv1).cuda(), torch.ones((T, 1), device="cuda"), None, out1)
        torch.cuda.synchronize()
        assert torch.equal(out1, y1[torch.from_numpy(inv1.astype(np.int64)).cuda()])
    finally:
        moe.set_option("y_fp32", 1)
        moe.set_option("out_fp32", 0)


def packed_reference(w: np.ndarray) -> np.ndarray:
    """The packed layout as include/moe.h words it, written out element by element."""
    K, N = w.shape
    out = np.empty(K * N, w.dtype)
    for n in range(N):
        src = n                         # rows keep their logical order
        g, r = divmod(n, 16)
        for kt in range(K // 32):
            base = (g * (K // 32) + kt) * 512
            for c in range(4):
                slot = c ^ ((4 - r // 4) & 3)
                out[base + r * 32 + slot * 8: base + r * 32 + slot * 8 + 8] = w[kt * 32 + c * 8: kt * 32 + c * 8 + 8, src]
    return out


def test_pack_weight_layout(moe):
    w = normal_bf16(4, 0, (96, 160), 0.02, "cuda")
    p = moe.pack_weight(w)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(torch_bf16_to_u16(p), packed_reference(torch_bf16_to_u16(w)))


def test_error_paths(moe):
    """Argument errors are reported before anything is enqueued."""
    from paper_2503_09716_amd import MoeError, make_shape
    shape = make_shape(64, 64, 64, 4, 2)
    x = torch.zeros((64, 64), dtype=torch.bfloat16, device="cuda")
    idx = torch.zeros((64, 2), dtype=torch.int32, device="cuda")
    w = torch.zeros((64, 2), dtype=torch.float32, device="cuda")
    ws = torch.empty(1024, dtype=torch.uint8, device="cuda")
    with pytest.raises(MoeError) as e:
        moe.route(shape, None, x, None, idx, w, None, ws)
    assert e.value.status == 1
    with pytest.raises(MoeError) as e:
        moe.route(make_shape(64, 60, 64, 4, 2), x, x, None, idx, w, None, ws)
    assert e.value.status == 2
    with pytest.raises(MoeError) as e:
        moe.route(shape, x, x, None, idx, w, None, ws)
    assert e.value.status == 3
    off = torch.zeros(5, dtype=torch.int32, device="cuda")
    perm = torch.zeros(128, dtype=torch.int32, device="cuda")
    with pytest.raises(MoeError) as e:
        moe.permute(shape, x, idx, None, off, perm, perm.clone(), None, ws)
    assert e.value.status == 3 and "workspace" in str(e.value)
    with pytest.raises(MoeError):
        moe.set_option("no_such_option", 1)
    with pytest.raises(MoeError):
        moe.set_option("gemm_wave_rows", 3)
    torch.cuda.synchronize()


def test_empty_batch_is_a_no_op(moe):
    """T = 0: every entry point returns MOE_OK without touching its buffers; moe_permute still
    reports E empty groups."""
    from paper_2503_09716_amd import make_shape
    E, k, H, F = 8, 2, 128, 192
    shape = make_shape(0, H, F, E, k, num_shared=1, renormalize=False)
    dev = "cuda"
    empty16 = torch.empty((0, H), dtype=torch.bfloat16, device=dev)
    idx = torch.empty((0, k), dtype=torch.int32, device=dev)
    w = torch.empty((0, k), dtype=torch.float32, device=dev)
    wg = normal_bf16(9, 0, (H, E), 0.02, dev)
    ws = torch.empty(1 << 16, dtype=torch.uint8, device=dev)
    off = torch.full((E + 1,), 7, dtype=torch.int32, device=dev)
    none_i = torch.empty(0, dtype=torch.int32, device=dev)
    moe.route(shape, empty16, wg, None, idx, w, None, ws)
    moe.permute(shape, empty16, idx, empty16, off, none_i, none_i, none_i, ws)
    torch.cuda.synchronize()
    assert (off == 0).all()
    w1 = [normal_bf16(9, 1 + e, (H, F), 0.02, dev) for e in range(E + 1)]
    w2 = [normal_bf16(9, 20 + e, (F, H), 0.02, dev) for e in range(E + 1)]
    w1p, w3p, w2p = moe.pack_experts(w1, w1, w2)
    y = torch.empty((0, H), dtype=torch.float32, device=dev)
    moe.grouped_ffn(shape, empty16, None, empty16, off, w1p, w3p, w2p, ws, y, y, ws)
    moe.combine(shape, y, none_i, w, y, empty16)
    moe.layer(shape, empty16, wg, None, w1p, w3p, w2p, empty16, ws)
    moe.layer_chunked(shape, empty16, wg, None, w1p, w3p, w2p, 16, empty16, ws)
    torch.cuda.synchronize()
