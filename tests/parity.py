"""Helpers shared by the GPU parity tests: run the HIP path through the binding, run the
oracle on the same bytes, compare to the stated bars.

Bars:  routing indices and the permutation bit-exact, except at reported top-k near-ties
(oracle logit margin < 1e-5); routing weights to 1e-5 relative; FFN / layer output
max-abs error <= 2e-2 x RMS(oracle output), asserted on the fp32 form of the result.  A bf16
result must be the round-to-nearest-even of that fp32 result bit for bit; against the oracle
it is held to the same bar widened by the rounding it cannot avoid (half a bf16 ulp = up to
2^-8 |value|, which alone is 1.7e-2..2.2e-2 x RMS for an element 4.3..5.7 sigma out)."""
from __future__ import annotations

import numpy as np
import torch

from oracle import moe_oracle as orc
from workloads import torch_bf16_to_u16

TIE_MARGIN = 1e-5
OUT_BAR = 2e-2
W_RTOL = 1e-5


def host_u16(t: torch.Tensor) -> np.ndarray:
    return torch_bf16_to_u16(t)


def compare_routing(gpu_idx: np.ndarray, gpu_w: np.ndarray, ref: dict, top_k: int, renormalize: bool = True,
                    routed_scale: float = 1.0):
    """ref: oracle.route(..., want_logits=True, want_probs=True) for the same tokens.  Returns a
    report; raises on an unexcused mismatch.  A set mismatch at token t is excused iff the oracle's
    k-th and (k+1)-th largest logits differ by < TIE_MARGIN; an order-only mismatch iff every
    displaced pair of logits differs by < TIE_MARGIN.  The weights of an excused token must still
    be the oracle's softmax probabilities at the experts the GPU chose (renormalised over them
    when the layer renormalises)."""
    idx_o, w_o, logit, probs = ref["idx"], ref["w"], ref["logits"], ref["probs"]
    n, E = logit.shape
    bad = np.nonzero((gpu_idx != idx_o).any(axis=1))[0]
    excused_set, excused_order = [], []
    for t in bad:
        so = np.sort(logit[t])[::-1]
        same_set = set(gpu_idx[t].tolist()) == set(idx_o[t].tolist())
        if same_set:
            d = np.abs(logit[t, gpu_idx[t]] - logit[t, idx_o[t]]).max()
            assert d < TIE_MARGIN, "token %d: order mismatch with logit gap %g" % (t, d)
            excused_order.append(int(t))
        else:
            margin = so[top_k - 1] - so[top_k] if top_k < E else np.inf
            assert margin < TIE_MARGIN, "token %d: top-k set mismatch with margin %g (gpu %s, oracle %s)" % (
                t, margin, gpu_idx[t].tolist(), idx_o[t].tolist())
            assert len(set(gpu_idx[t].tolist())) == top_k
            excused_set.append(int(t))
    good = np.setdiff1d(np.arange(n), bad)
    if len(good):
        np.testing.assert_allclose(gpu_w[good], w_o[good], rtol=W_RTOL, atol=1e-7)
    if len(bad):
        sel = np.take_along_axis(probs[bad].astype(np.float64), gpu_idx[bad].astype(np.int64), axis=1)
        if renormalize:
            sel = sel / sel.sum(axis=1, keepdims=True)
        np.testing.assert_allclose(gpu_w[bad], sel * routed_scale, rtol=W_RTOL, atol=1e-7,
                                   err_msg="weights of near-tie tokens are not the oracle's probabilities at the chosen experts")
    so = np.sort(logit, axis=1)[:, ::-1]
    near = int((so[:, top_k - 1] - so[:, top_k] < TIE_MARGIN).sum()) if top_k < E else 0
    return {"tokens": int(n), "mismatch_set_excused": excused_set, "mismatch_order_excused": excused_order,
            "near_ties_in_oracle": near}


def output_report(out_gpu: np.ndarray, out_ref: np.ndarray):
    """Error of a bf16 GPU result against the fp32 oracle, relative to the oracle's RMS."""
    ref = out_ref.astype(np.float64)
    got = out_gpu.astype(np.float64)
    rms = float(np.sqrt((ref ** 2).mean()))
    err = np.abs(got - ref)
    rel = err / np.maximum(np.abs(ref), 1e-30)
    big = np.abs(ref) > 0.1 * rms
    ref_bf16 = torch.from_numpy(out_ref.astype(np.float32)).to(torch.bfloat16).float().numpy().astype(np.float64)
    return {
        "rms": rms,
        "max_abs_over_rms": float(err.max() / rms) if rms > 0 else float(err.max()),
        "max_abs_vs_bf16_rounded_oracle_over_rms": float(np.abs(got - ref_bf16).max() / rms) if rms > 0 else 0.0,
        "rel_p50": float(np.median(rel[big])) if big.any() else 0.0,
        "rel_p99": float(np.percentile(rel[big], 99)) if big.any() else 0.0,
        "rel_max": float(rel[big].max()) if big.any() else 0.0,
    }


def assert_output(out_gpu: np.ndarray, out_ref: np.ndarray, what: str = "output"):
    rep = output_report(out_gpu, out_ref)
    assert rep["max_abs_over_rms"] <= OUT_BAR, "%s: max-abs error %.4g x RMS exceeds %.2g (%s)" % (
        what, rep["max_abs_over_rms"], OUT_BAR, rep)
    return rep


def assert_output_bf16(out_gpu: np.ndarray, out_ref: np.ndarray, what: str = "output"):
    """Per-element bound for a result stored in bf16: the fp32 result v may be off by the error bar
    (OUT_BAR x RMS), so |v| <= |ref| + bar, and rounding v to bf16 (8 significant bits, round to
    nearest even) moves it by at most half a bf16 step of its binade: 2^(floor(log2 |v|) - 8)."""
    ref = out_ref.astype(np.float64)
    rms = float(np.sqrt((ref ** 2).mean()))
    err = np.abs(out_gpu.astype(np.float64) - ref)
    vmax = np.abs(ref) + OUT_BAR * rms
    _, ex = np.frexp(vmax)                               # vmax = m * 2^ex, m in [0.5, 1): floor(log2 vmax) = ex - 1
    half_step = np.ldexp(1.0, np.maximum(ex - 1, -126) - 8)
    bound = OUT_BAR * rms + half_step
    worst = float((err / bound).max())
    assert worst <= 1.0, "%s: bf16 result off by %.3f x its bound" % (what, worst)
    return output_report(out_gpu, out_ref)


class GpuLayer:
    """One synthetic layer resident on the GPU with packed weights, plus host copies for the oracle."""

    def __init__(self, moe, li, host_weights: bool = True):
        from paper_2503_09716_amd import shape_of
        self.moe, self.li, self.cfg = moe, li, li.cfg
        self.shape = shape_of(li.cfg)
        self.x, self.wg = li.x, li.wg
        self.bias = None if li.bias is None else torch.from_numpy(li.bias).cuda()
        self.w1p, self.w3p, self.w2p = moe.pack_experts(li.w1, li.w3, li.w2)
        torch.cuda.synchronize()
        self.ws = moe.new_workspace(self.shape)
        self.tables = moe.tables(self.w1p, self.w3p, self.w2p)
        if host_weights:
            self.hx, self.hwg = host_u16(li.x), host_u16(li.wg)
            self.hw1 = [host_u16(w) for w in li.w1]
            self.hw3 = [host_u16(w) for w in li.w3]
            self.hw2 = [host_u16(w) for w in li.w2]

    def run_layer(self, out_fp32: bool = False):
        cfg = self.cfg
        out = torch.empty((cfg.T, cfg.H), dtype=torch.float32 if out_fp32 else torch.bfloat16, device="cuda")
        self.moe.set_option("out_fp32", 1 if out_fp32 else 0)
        try:
            self.moe.layer(self.shape, self.x, self.wg, self.bias, self.w1p, self.w3p, self.w2p, out, self.ws,
                           tables=self.tables)
            torch.cuda.synchronize()
        finally:
            self.moe.set_option("out_fp32", 0)
        return out

    def run_layer_both(self):
        """fp32 output (held to the bar) and bf16 output (must be its exact RNE rounding)."""
        o32 = self.run_layer(True)
        o16 = self.run_layer(False)
        assert torch.equal(o32.to(torch.bfloat16).view(torch.int16), o16.view(torch.int16)), \
            "bf16 output is not the round-to-nearest-even of the fp32 output"
        return o32, o16

    def oracle_route(self, tokens=None):
        cfg = self.cfg
        return orc.route(self.hx, self.hwg, self.li.bias, cfg.top_k, cfg.renormalize, cfg.routed_scale,
                         tokens=tokens, want_logits=True, want_probs=True)

    def oracle_layer(self, idx, w, tokens=None):
        cfg = self.cfg
        return orc.layer(self.hx, idx, w, self.hw1, self.hw3, self.hw2, cfg.E, cfg.num_shared, tokens=tokens)


def check_layer_against_oracle(gl: GpuLayer, out: torch.Tensor, tokens=None, check_all_routing: bool = True,
                               out16: torch.Tensor = None, progress=None):
    """Full check of one moe_layer result.  tokens=None: every token through the oracle;
    otherwise the FFN/combine part only for the listed tokens (routing still for all tokens
    when check_all_routing)."""
    cfg = gl.cfg
    views = gl.moe.layer_views(gl.shape, gl.ws)
    idx = views["topk_idx"].cpu().numpy()
    w = views["topk_w"].cpu().numpy()
    off = views["expert_offsets"].cpu().numpy()
    inv = views["inv_perm"].cpu().numpy()
    report = {}
    # permutation: bit-exact against the oracle's stable counting sort of the GPU's own routing
    o_off, o_perm, o_inv = orc.permute(idx, cfg.E)
    np.testing.assert_array_equal(off, o_off)
    np.testing.assert_array_equal(inv, o_inv)
    cnt = np.diff(off)
    report["rows_per_expert"] = {"max": int(cnt.max()), "mean": float(cnt.mean()), "min": int(cnt.min()),
                                 "empty": int((cnt == 0).sum())}
    # routing
    rt_tokens = None if (check_all_routing or tokens is None) else tokens
    ref = gl.oracle_route(rt_tokens)
    sel = slice(None) if rt_tokens is None else rt_tokens
    report["routing"] = compare_routing(idx[sel], w[sel], ref, cfg.top_k, cfg.renormalize, cfg.routed_scale)
    # FFN + combine: the oracle runs with the GPU's routing, so an excused near-tie cannot fail it
    if tokens is None:
        tokens = np.arange(cfg.T, dtype=np.int32)
    tokens = np.asarray(tokens, dtype=np.int32)
    if progress is None:
        out_ref = gl.oracle_layer(idx[tokens], w[tokens], tokens=tokens)
    else:       # long runs: the oracle in pieces, a line after each, so that the run is seen to be alive
        parts = []
        for lo in range(0, len(tokens), 1024):
            tk = tokens[lo:lo + 1024]
            parts.append(gl.oracle_layer(idx[tk], w[tk], tokens=tk))
            progress("  oracle: %d of %d tokens" % (min(lo + 1024, len(tokens)), len(tokens)))
        out_ref = np.concatenate(parts)
    out_gpu = out[torch.from_numpy(tokens.astype(np.int64)).cuda()].float().cpu().numpy()
    report["output"] = assert_output(out_gpu, out_ref, "layer output (%s)" % cfg.name)
    if out16 is not None:
        got16 = out16[torch.from_numpy(tokens.astype(np.int64)).cuda()].float().cpu().numpy()
        report["output_bf16"] = assert_output_bf16(got16, out_ref, "bf16 layer output (%s)" % cfg.name)
    return report


TILE_ROWS = (128, 256, 320)      # every m-tile height the grouped GEMMs use for full tiles


def sample_tokens(idx: np.ndarray, E: int, n: int, seed: int, every_tile: bool = True) -> np.ndarray:
    """At least n tokens chosen so that EVERY m-tile of every expert's row group holds a checked
    row, whichever tile height a launch uses: per group (rows are in ascending token order) one
    random row from each block of 128, of 256 and of 320 rows; the rows on both sides of the first
    tile boundaries (127..129, 255..257, 319..321); the first and the last row; the rows on both
    sides of the place where a short tail (the rows past the last multiple of 256) joins the last
    full tile.  The same positions of the token range itself cover the shared experts, whose
    groups are all T tokens.  The rest uniformly at random.  every_tile=False keeps only the
    boundary rows of each group (no row per block): about 20 tokens per expert."""
    rng = np.random.default_rng(seed)
    T, k = idx.shape
    flat_e = idx.reshape(-1).astype(np.int64)
    flat_tok = np.repeat(np.arange(T, dtype=np.int64), k)
    order = np.lexsort((flat_tok, flat_e))               # rows of the permuted batch: by expert, then token
    row_tok = flat_tok[order]
    off = np.concatenate([[0], np.cumsum(np.bincount(flat_e, minlength=E))])

    def positions(rows: int) -> np.ndarray:
        """Row positions inside a group of `rows` rows."""
        pos = [0, rows - 1]
        for tm in TILE_ROWS:
            starts = np.arange(0, rows, tm)
            if every_tile:
                pos.extend((starts + rng.integers(0, np.minimum(tm, rows - starts))).tolist())
            pos.extend([tm - 1, tm, tm + 1])
        full = (rows // 256) * 256
        pos.extend([full - 1, full, full + 1, full - 256, full - 257])
        p = np.array(pos, dtype=np.int64)
        return np.unique(p[(p >= 0) & (p < rows)])

    chosen = [positions(T)]                                          # shared experts: the token range itself
    for e in range(E):
        rows = int(off[e + 1] - off[e])
        if rows:
            chosen.append(row_tok[off[e] + positions(rows)])
    chosen = np.unique(np.concatenate(chosen))
    rest = rng.permutation(T)[:max(0, n - len(chosen))]
    return np.unique(np.concatenate([chosen, rest])).astype(np.int32)


def tiles_without_a_sampled_row(idx: np.ndarray, E: int, tokens: np.ndarray, tile_rows: int) -> int:
    """Number of m-tiles (blocks of tile_rows rows of an expert's group) none of whose rows belongs
    to a sampled token; 0 means the sample reaches every tile."""
    T, k = idx.shape
    flat_e = idx.reshape(-1).astype(np.int64)
    flat_tok = np.repeat(np.arange(T, dtype=np.int64), k)
    order = np.lexsort((flat_tok, flat_e))
    hit = np.isin(flat_tok[order], tokens)
    off = np.concatenate([[0], np.cumsum(np.bincount(flat_e, minlength=E))])
    missing = 0
    for e in range(E):
        for r0 in range(int(off[e]), int(off[e + 1]), tile_rows):
            if not hit[r0:min(r0 + tile_rows, int(off[e + 1]))].any():
                missing += 1
    return missing
