"""Pins for the CPU oracle: each test fixes it to something other than itself (brute force,
closed forms, invariants, a library routine on a special case, a hand-worked example), so
that a dropped term, a wrong sign or index, or a transposed operand fails at least one."""
import json
import os

import numpy as np
import pytest
import torch

from oracle import moe_oracle as orc
from workloads import (bf16_bits_to_f32, f32_to_bf16_bits, get_config, make_layer_inputs, scaled_config,
                       torch_bf16_to_u16)

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def bits(a):
    return f32_to_bf16_bits(np.asarray(a, dtype=np.float32))


def rnd_bits(rng, shape, std):
    return bits(rng.standard_normal(shape).astype(np.float32) * std)


def small_layer(rng, T=24, H=16, F=24, E=6, Ns=0, wstd=0.3):
    x = rnd_bits(rng, (T, H), 1.0)
    wg = rnd_bits(rng, (H, E), 0.5)
    w1 = [rnd_bits(rng, (H, F), wstd) for _ in range(E + Ns)]
    w3 = [rnd_bits(rng, (H, F), wstd) for _ in range(E + Ns)]
    w2 = [rnd_bits(rng, (F, H), wstd) for _ in range(E + Ns)]
    return x, wg, w1, w3, w2


def f64(b):
    return bf16_bits_to_f32(b).astype(np.float64)


def dense_swiglu_torch(xb, w1b, w3b, w2b):
    """Independent library formulation in float64 torch CPU ops."""
    x = torch.from_numpy(f64(xb)); w1 = torch.from_numpy(f64(w1b))
    w3 = torch.from_numpy(f64(w3b)); w2 = torch.from_numpy(f64(w2b))
    return ((torch.nn.functional.silu(x @ w1) * (x @ w3)) @ w2).numpy()


# ----------------------------------------------------------------------------- router
def test_router_hand_example_and_layer():
    g = json.load(open(os.path.join(GOLDEN, "hand_example.json")))
    x, wg = bits(g["x"]), bits(g["wg"])
    w1 = [bits(m) for m in g["w1"]]; w3 = [bits(m) for m in g["w3"]]; w2 = [bits(m) for m in g["w2"]]
    r = orc.route(x, wg, None, 1, False)
    assert r["idx"].tolist() == g["expect_idx"]
    np.testing.assert_allclose(r["w"], np.array(g["expect_w"]), rtol=2e-7)
    out = orc.layer(x, r["idx"], r["w"], w1, w3, w2, 2, 0)
    np.testing.assert_allclose(out, np.array(g["expect_out"]), rtol=5e-7)


def test_hand_example_mixed_experts():
    """Two tokens that pick DIFFERENT experts with different non-zero weights, top-2 with
    renormalisation and one shared expert: an expert mix-up, a dropped shared term, a missing
    renormalisation or a transposed matrix each change the expected numbers."""
    g = json.load(open(os.path.join(GOLDEN, "hand_example_mixed_experts.json")))
    x, wg = bits(g["x"]), bits(g["wg"])
    w1 = [bits(m) for m in g["w1"]]; w3 = [bits(m) for m in g["w3"]]; w2 = [bits(m) for m in g["w2"]]
    E, Ns, k = 3, g["num_shared"], g["top_k"]
    r = orc.route(x, wg, None, k, bool(g["renormalize"]))
    assert r["idx"].tolist() == g["expect_idx"]
    np.testing.assert_allclose(r["w"], np.array(g["expect_w"]), rtol=3e-7)
    out = orc.layer(x, r["idx"], r["w"], w1, w3, w2, E, Ns)
    np.testing.assert_allclose(out, np.array(g["expect_out"]), rtol=1e-6)
    # the same experts row by row through the stage-level entry (expert ids 0, 1, 2, 1, shared, shared)
    ey = g["expect_expert_y"]
    rows = orc.expert_rows(bits(ey["rows_x"]), np.array(ey["rows_expert"], np.int32), w1, w3, w2)
    np.testing.assert_allclose(rows, np.array(ey["y"]), rtol=1e-6)
    # and the combine stage on those rows: y_perm in expert order (e0:t0 | e1:t0,t1 | e2:t1), fp32 input
    y = np.array(ey["y"], np.float32)
    y_perm = np.stack([y[0], y[1], y[3], y[2]])
    inv = np.array([0, 1, 3, 2], np.int32)          # (t0,j0)->e0 row 0, (t0,j1)->e1 row 1, (t1,j0)->e2 row 3, (t1,j1)->e1 row 2
    o, p, i = orc.permute(r["idx"], E)
    assert o.tolist() == [0, 1, 3, 4] and i.tolist() == inv.tolist() and p.tolist() == [0, 1, 3, 2]
    comb = orc.combine(y_perm, inv, r["w"], np.stack([y[4], y[5]]))
    np.testing.assert_allclose(comb, np.array(g["expect_out"]), rtol=1e-6)


@pytest.mark.parametrize("E,k", [(4, 1), (8, 2), (16, 6), (11, 11)])
def test_router_brute_force_sort(E, k):
    rng = np.random.default_rng(E * 100 + k)
    T, H = 64, 32
    x = rnd_bits(rng, (T, H), 1.0); wg = rnd_bits(rng, (H, E), 0.5)
    bias = rng.standard_normal(E).astype(np.float32)
    r = orc.route(x, wg, bias, k, True, want_logits=True, want_probs=True)
    logit = (f64(x) @ f64(wg) + bias.astype(np.float64)).astype(np.float32)
    np.testing.assert_array_equal(r["logits"], logit)      # correctly rounded fp64 dot product
    for t in range(T):
        order = sorted(range(E), key=lambda e: (-logit[t, e], e))[:k]
        assert r["idx"][t].tolist() == order
    p = torch.softmax(torch.from_numpy(logit.astype(np.float64)), dim=-1).numpy()
    np.testing.assert_allclose(r["probs"], p, rtol=1e-6, atol=1e-9)
    sel = np.take_along_axis(p, r["idx"].astype(np.int64), axis=1)
    np.testing.assert_allclose(r["w"], sel / sel.sum(1, keepdims=True), rtol=2e-6)
    np.testing.assert_allclose(r["w"].sum(1), 1.0, atol=1e-6)
    # no renormalisation: the raw probabilities of the selected experts
    r0 = orc.route(x, wg, bias, k, False)
    np.testing.assert_array_equal(r0["idx"], r["idx"])
    np.testing.assert_allclose(r0["w"], sel, rtol=2e-6)
    assert (r0["w"].sum(1) <= 1 + 1e-6).all()
    # torch.topk agrees as a set (no exact ties in random data)
    tk = torch.topk(torch.from_numpy(logit), k, dim=-1).indices.numpy()
    assert (np.sort(tk, 1) == np.sort(r["idx"], 1)).all()


def test_router_closed_forms():
    T, H, E = 5, 8, 6
    x = bits(np.arange(T * H).reshape(T, H) % 7 - 3.0)
    wg0 = bits(np.zeros((H, E)))
    for k in (1, 3, 6):
        r = orc.route(x, wg0, None, k, True, want_probs=True)
        assert (r["idx"] == np.arange(k)[None, :]).all()          # exact ties -> lowest ids, in order
        np.testing.assert_allclose(r["probs"], 1.0 / E, rtol=1e-7)
        np.testing.assert_allclose(r["w"], 1.0 / k, rtol=1e-7)
        r = orc.route(x, wg0, None, k, False)
        np.testing.assert_allclose(r["w"], 1.0 / E, rtol=1e-7)
    # one-hot gate columns: logit[t,e] = x[t,e] (+ bias[e]); checkable by eye
    wg1 = bits(np.eye(H)[:, :E])
    bias = np.array([0, 0, 0, 10, 0, 0], np.float32)
    r = orc.route(x, wg1, bias, 2, False, want_logits=True)
    xf = bf16_bits_to_f32(x)
    np.testing.assert_array_equal(r["logits"], xf[:, :E] + bias)
    assert (r["idx"][:, 0] == 3).all()
    # routed_scale multiplies the weights, bias shifts by a constant change nothing
    ra = orc.route(x, wg1, bias, 2, True, routed_scale=1.0)
    rb = orc.route(x, wg1, bias + 4.0, 2, True, routed_scale=2.0)
    np.testing.assert_array_equal(ra["idx"], rb["idx"])
    np.testing.assert_allclose(rb["w"], 2.0 * ra["w"], rtol=1e-6)


def test_router_token_subset_matches_full():
    rng = np.random.default_rng(7)
    x = rnd_bits(rng, (40, 16), 1.0); wg = rnd_bits(rng, (16, 8), 0.5)
    full = orc.route(x, wg, None, 2, True, want_logits=True)
    tok = np.array([3, 39, 0, 17], np.int32)
    sub = orc.route(x, wg, None, 2, True, tokens=tok, want_logits=True)
    for key in ("idx", "w", "logits"):
        np.testing.assert_array_equal(sub[key], full[key][tok])


# ----------------------------------------------------------------------------- permutation
@pytest.mark.parametrize("T,k,E", [(1, 1, 1), (37, 2, 8), (200, 6, 16), (64, 4, 4)])
def test_permute_properties_and_brute_force(T, k, E):
    rng = np.random.default_rng(T + k + E)
    idx = np.stack([rng.permutation(E)[:k] for _ in range(T)]).astype(np.int32)
    off, perm, inv = orc.permute(idx, E)
    R = T * k
    assert off[0] == 0 and off[E] == R
    np.testing.assert_array_equal(np.diff(off), np.bincount(idx.reshape(-1), minlength=E))
    assert sorted(perm.tolist()) == list(range(R))
    np.testing.assert_array_equal(inv[perm], np.arange(R))
    np.testing.assert_array_equal(np.bincount(perm // k, minlength=T), np.full(T, k))
    flat = idx.reshape(-1)
    for e in range(E):
        rows = perm[off[e]:off[e + 1]]
        assert (flat[rows] == e).all()
        assert (np.diff(rows // k) > 0).all()                 # strictly ascending tokens
    # brute force: stable sort of the pairs by expert
    np.testing.assert_array_equal(perm, np.argsort(flat, kind="stable").astype(np.int32))


def test_permute_empty_and_single_expert():
    idx = np.zeros((10, 1), np.int32) + 2
    off, perm, inv = orc.permute(idx, 5)
    assert off.tolist() == [0, 0, 0, 10, 10, 10]
    assert perm.tolist() == list(range(10)) and inv.tolist() == list(range(10))


# ----------------------------------------------------------------------------- experts / layer
def test_single_expert_top1_is_dense_swiglu():
    rng = np.random.default_rng(11)
    T, H, F = 9, 20, 28            # non-square so a transposed operand cannot pass
    x = rnd_bits(rng, (T, H), 1.0)
    wg = rnd_bits(rng, (H, 1), 0.5)
    w1 = [rnd_bits(rng, (H, F), 0.3)]; w3 = [rnd_bits(rng, (H, F), 0.3)]; w2 = [rnd_bits(rng, (F, H), 0.3)]
    out, r = orc.moe_forward(x, wg, None, w1, w3, w2, 1, 0, True)
    assert (r["idx"] == 0).all() and np.allclose(r["w"], 1.0)
    ref = dense_swiglu_torch(x, w1[0], w3[0], w2[0])
    np.testing.assert_allclose(out, ref, rtol=2e-6, atol=1e-6)
    rows = orc.expert_rows(x, np.zeros(T, np.int32), w1, w3, w2)
    np.testing.assert_array_equal(rows, out)


def test_expert_rows_mixed_experts_are_each_experts_dense_swiglu():
    """Stage-level entry with a shuffled multi-expert row -> expert map: every row must be the
    dense SwiGLU MLP of ITS expert's weights (independent float64 library formulation), and of no
    other expert's."""
    rng = np.random.default_rng(31)
    n, H, F, E = 23, 20, 28, 5        # non-square, so a transposed operand cannot pass
    x = rnd_bits(rng, (n, H), 1.0)
    w1 = [rnd_bits(rng, (H, F), 0.3) for _ in range(E)]
    w3 = [rnd_bits(rng, (H, F), 0.3) for _ in range(E)]
    w2 = [rnd_bits(rng, (F, H), 0.3) for _ in range(E)]
    eid = rng.integers(0, E, n).astype(np.int32)
    eid[:E] = rng.permutation(E)      # every expert appears, in no particular order
    y = orc.expert_rows(x, eid, w1, w3, w2)
    dense = [dense_swiglu_torch(x, w1[e], w3[e], w2[e]) for e in range(E)]
    ref = np.stack([dense[eid[i]][i] for i in range(n)])
    np.testing.assert_allclose(y, ref, rtol=3e-6, atol=2e-6)
    # the check has teeth: another expert's output for the same row is far away
    scale = np.abs(ref).mean()
    for i in range(n):
        other = dense[(eid[i] + 1) % E][i]
        assert np.abs(y[i] - other).max() > 0.05 * scale
    # the stage-level entry and the layer agree bit for bit when the layer is one expert with weight 1
    out = orc.layer(x, eid[:, None], np.ones((n, 1), np.float32), w1, w3, w2, E, 0)
    np.testing.assert_array_equal(out, y)


def test_identical_experts_reduce_to_dense():
    rng = np.random.default_rng(12)
    T, H, F, E, k, Ns = 12, 16, 24, 5, 3, 2
    x = rnd_bits(rng, (T, H), 1.0); wg = rnd_bits(rng, (H, E), 0.5)
    a1, a3, a2 = rnd_bits(rng, (H, F), 0.3), rnd_bits(rng, (H, F), 0.3), rnd_bits(rng, (F, H), 0.3)
    s1, s3, s2 = rnd_bits(rng, (H, F), 0.3), rnd_bits(rng, (H, F), 0.3), rnd_bits(rng, (F, H), 0.3)
    w1 = [a1] * E + [s1] * Ns; w3 = [a3] * E + [s3] * Ns; w2 = [a2] * E + [s2] * Ns
    mlp = dense_swiglu_torch(x, a1, a3, a2); mlp_s = dense_swiglu_torch(x, s1, s3, s2)
    out, r = orc.moe_forward(x, wg, None, w1, w3, w2, k, Ns, True)
    np.testing.assert_allclose(out, mlp + Ns * mlp_s, rtol=3e-6, atol=2e-6)
    out0, r0 = orc.moe_forward(x, wg, None, w1, w3, w2, k, Ns, False)
    wsum = r0["w"].astype(np.float64).sum(1, keepdims=True)
    np.testing.assert_allclose(out0, wsum * mlp + Ns * mlp_s, rtol=3e-6, atol=2e-6)


def test_metamorphic_exact():
    rng = np.random.default_rng(13)
    x, wg, w1, w3, w2 = small_layer(rng, Ns=1)
    E, k = 6, 2
    out, r = orc.moe_forward(x, wg, None, w1, w3, w2, k, 1, True)
    # power-of-two scaling of W2 commutes with every rounding: bit-exact doubling
    w2d = [bits(bf16_bits_to_f32(m) * 2.0) for m in w2]
    outd, _ = orc.moe_forward(x, wg, None, w1, w3, w2d, k, 1, True)
    np.testing.assert_array_equal(outd, 2.0 * out)
    w3d = [bits(bf16_bits_to_f32(m) * 2.0) for m in w3]
    outd, _ = orc.moe_forward(x, wg, None, w1, w3d, w2, k, 1, True)
    np.testing.assert_array_equal(outd, 2.0 * out)
    # zero input -> zero output
    z, _ = orc.moe_forward(np.zeros_like(x), wg, None, w1, w3, w2, k, 1, True)
    assert (z == 0).all()
    # permuting tokens permutes output rows bit-exactly
    p = rng.permutation(x.shape[0])
    outp, _ = orc.moe_forward(x[p], wg, None, w1, w3, w2, k, 1, True)
    np.testing.assert_array_equal(outp, out[p])
    # relabelling the routed experts (gate columns and weight tables together) changes nothing
    q = rng.permutation(E)
    sh = [E]
    wq = lambda ws: [ws[i] for i in q] + [ws[i] for i in sh]
    outq, rq = orc.moe_forward(x, np.ascontiguousarray(wg[:, q]), None, wq(w1), wq(w3), wq(w2), k, 1, True)
    np.testing.assert_array_equal(q[rq["idx"]], r["idx"])
    np.testing.assert_array_equal(outq, out)
    # token subset == rows of the full result
    tok = np.array([5, 0, 23], np.int32)
    rs = orc.route(x, wg, None, k, True, tokens=tok)
    outs = orc.layer(x, rs["idx"], rs["w"], w1, w3, w2, E, 1, tokens=tok)
    np.testing.assert_array_equal(outs, out[tok])


def second_formulation(li, r):
    """Independent plumbing: group rows by expert, per-expert float64 matmuls in torch, index_add."""
    cfg = li.cfg
    x = li.x.double()
    idx = torch.from_numpy(r["idx"].astype(np.int64)); w = torch.from_numpy(r["w"].astype(np.float64))
    out = torch.zeros(cfg.T, cfg.H, dtype=torch.float64)

    def mlp(xe, e):
        return (torch.nn.functional.silu(xe @ li.w1[e].double()) * (xe @ li.w3[e].double())) @ li.w2[e].double()
    for e in range(cfg.E):
        tok, j = torch.nonzero(idx == e, as_tuple=True)
        if len(tok):
            out.index_add_(0, tok, mlp(x[tok], e) * w[tok, j][:, None])
    for s in range(cfg.num_shared):
        out += mlp(x, cfg.E + s)
    return out.numpy()


@pytest.mark.parametrize("name,over", [
    ("C1", {}),
    ("C4", dict(T=192, H=128, F=192)),
    ("C5", dict(T=256, H=128, F=64)),
])
def test_whole_layer_vs_second_formulation(name, over):
    cfg = scaled_config(name, **over) if over else get_config(name)
    li = make_layer_inputs(cfg)
    u = torch_bf16_to_u16
    w1 = [u(t) for t in li.w1]; w3 = [u(t) for t in li.w3]; w2 = [u(t) for t in li.w2]
    out, r = orc.moe_forward(u(li.x), u(li.wg), li.bias, w1, w3, w2, cfg.top_k, cfg.num_shared,
                             cfg.renormalize, cfg.routed_scale)
    ref = second_formulation(li, r)
    scale = np.sqrt((ref ** 2).mean())
    assert np.abs(out - ref).max() <= 5e-6 * scale
    if cfg.renormalize:
        np.testing.assert_allclose(r["w"].sum(1), 1.0, atol=1e-6)
    off, perm, inv = orc.permute(r["idx"], cfg.E)
    assert off[-1] == cfg.T * cfg.top_k
    if name == "C5":
        cnt = np.diff(off)
        assert cnt.max() > 5 * cnt.mean()            # the log-Zipf bias skews the routing


# ----------------------------------------------------------------------------- combine
def test_combine_pins():
    rng = np.random.default_rng(21)
    T, H, k = 13, 10, 3
    y = rnd_bits(rng, (T * k, H), 1.0)
    inv = rng.permutation(T * k).astype(np.int32)
    w = rng.random((T, k)).astype(np.float32)
    ys = rnd_bits(rng, (T, H), 1.0)
    out = orc.combine(y, inv, w, ys)
    yf = bf16_bits_to_f32(y).astype(np.float64)
    ref = (w.astype(np.float64)[:, :, None] * yf[inv.reshape(T, k)]).sum(1) + f64(ys)
    np.testing.assert_allclose(out, ref, rtol=1e-6, atol=1e-6)
    # k = 1, w = 1: a pure row gather, bit-exact
    inv1 = rng.permutation(T).astype(np.int32)
    o1 = orc.combine(y[:T], inv1, np.ones((T, 1), np.float32))
    np.testing.assert_array_equal(o1, bf16_bits_to_f32(y[:T])[inv1])
    # linear in w (power-of-two scale is exact)
    np.testing.assert_array_equal(orc.combine(y, inv, 2 * w), 2 * orc.combine(y, inv, w))


def test_combine_fp32_inputs():
    """The float32-input form of the combine (what the down projection hands over by default):
    values with full 24-bit mantissas against the float64 sum; gather and linearity bit-exact."""
    rng = np.random.default_rng(22)
    T, H, k = 11, 14, 3
    y = (rng.standard_normal((T * k, H)) * np.pi).astype(np.float32)      # full mantissas, not bf16-representable
    assert (f32_to_bf16_bits(y).astype(np.uint32) << 16 != y.view(np.uint32)).mean() > 0.9
    ys = (rng.standard_normal((T, H)) * np.e).astype(np.float32)
    inv = rng.permutation(T * k).astype(np.int32)
    w = rng.random((T, k)).astype(np.float32)
    out = orc.combine(y, inv, w, ys)
    ref = (w.astype(np.float64)[:, :, None] * y.astype(np.float64)[inv.reshape(T, k)]).sum(1) + ys.astype(np.float64)
    np.testing.assert_allclose(out, ref, rtol=1e-6, atol=1e-6)
    # every element is read where it is: a one-hot y_perm lands in exactly one output element
    for (r, h) in [(0, 0), (5, 13), (T * k - 1, 7), (17, 1)]:
        hot = np.zeros((T * k, H), np.float32); hot[r, h] = 1.0
        o = orc.combine(hot, inv, w)
        t, j = divmod(int(np.nonzero(inv == r)[0][0]), k)
        expect = np.zeros((T, H), np.float32); expect[t, h] = w[t, j]
        np.testing.assert_array_equal(o, expect)
    # k = 1, w = 1: a pure row gather, bit-exact (float32 values pass through unrounded)
    inv1 = rng.permutation(T).astype(np.int32)
    np.testing.assert_array_equal(orc.combine(y[:T], inv1, np.ones((T, 1), np.float32)), y[:T][inv1])
    # shared rows are added with weight 1 to the right token
    z = np.zeros((T * k, H), np.float32)
    np.testing.assert_array_equal(orc.combine(z, inv, w, ys), ys)
    # power-of-two scale is exact; bf16-representable float32 input equals the bf16-bits form
    np.testing.assert_array_equal(orc.combine(y, inv, 2 * w), 2 * orc.combine(y, inv, w))
    yb = rnd_bits(rng, (T * k, H), 1.0); ysb = rnd_bits(rng, (T, H), 1.0)
    np.testing.assert_array_equal(orc.combine(bf16_bits_to_f32(yb), inv, w, bf16_bits_to_f32(ysb)),
                                  orc.combine(yb, inv, w, ysb))


def test_oracle_reports_threads():
    assert orc.num_threads() >= 1
