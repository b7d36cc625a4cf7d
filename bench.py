"""Benchmark of the MoE expert module on one MI355X.

A step = one moe_layer call (route -> permute -> grouped SwiGLU FFN -> combine) over one
synthetic accumulated batch that is already resident in HBM.  Prints ONE JSON line:

  * value / ms_per_step: tokens/s of the whole layer on the headline workload (C2), from a timed
    loop of exactly K steps with no profiling events in it;
  * step_ms / stage_ms: median and min per step and per stage, from a second loop with HIP events
    (the library's own per-stage events on the launch stream, torch events around each step);
  * roofline: the gate/up grouped GEMM against the published bf16 MFMA peak and against the rate a
    register-only MFMA loop sustains on this machine (on zeros and on the workload's own data);
  * hbm_stages: route / permute / combine through the staged calls on rotating buffer sets larger
    than the last-level cache, bytes as the algorithm defines them, against 8 TB/s and a measured copy;
  * all_workloads: step and grouped-GEMM figures of the other named workloads (C1, C3, C4, C5);
  * cpu_baseline: the CPU oracle timed on this machine's host cores on a bounded sample.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload C2] [--no-cpu-baseline]
                    [--no-all-workloads] [--no-hbm-stages] [--no-ceiling]
    python bench.py --sweep C2|C5      tokens-per-expert sweep (markdown table; resident and streamed weights)
"""
from __future__ import annotations

import argparse
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA peak
PEAK_HBM_GBS = 8000.0
TARGET_FRAC = 0.60          # grouped FFN on the 8-expert large-batch workloads (C2, C3)
LLC_BYTES = 256 << 20       # last-level (memory-side) cache; rotating buffer sets must exceed it
METRIC = "expert-module tokens/s and grouped-FFN TFLOP/s (% bf16 MFMA peak), 1 GPU"


def med_min(v):
    v = [float(a) for a in v]
    return {"median": statistics.median(v), "min": min(v), "n": len(v)} if v else {"median": 0.0, "min": 0.0, "n": 0}


def cpu_baseline(cfg, li, target_seconds: float = 12.0):
    """The oracle as it stands, on a bounded sample of tokens of the same workload."""
    import numpy as np
    from oracle import moe_oracle as orc
    from workloads import torch_bf16_to_u16 as u
    hx, hwg = u(li.x), u(li.wg)
    hw1 = [u(w) for w in li.w1]; hw3 = [u(w) for w in li.w3]; hw2 = [u(w) for w in li.w2]
    threads = orc.num_threads()
    rng = np.random.default_rng(cfg.seed)
    order = rng.permutation(cfg.T).astype(np.int32)
    done, t0 = 0, time.perf_counter()
    while done < cfg.T:
        tok = order[done:done + threads]
        r = orc.route(hx, hwg, li.bias, cfg.top_k, cfg.renormalize, cfg.routed_scale, tokens=tok)
        orc.layer(hx, r["idx"], r["w"], hw1, hw3, hw2, cfg.E, cfg.num_shared, tokens=tok)
        done += len(tok)
        if time.perf_counter() - t0 >= target_seconds:
            break
    dt = time.perf_counter() - t0
    return {"value": done / dt, "unit": "tokens/s", "cores": threads, "kind": "oracle",
            "sample": "%d seeded random tokens of %s through route + experts + combine, %.1f s" % (done, cfg.name, dt)}


class Layer:
    """One synthetic workload resident on the GPU with packed weights."""

    def __init__(self, moe, cfg, keep_logical_weights: bool = False):
        import torch
        from paper_2503_09716_amd import shape_of
        from workloads import make_layer_inputs
        self.moe, self.cfg = moe, cfg
        self.li = make_layer_inputs(cfg, device="cuda")
        self.shape = shape_of(cfg)
        self.w1p, self.w3p, self.w2p = moe.pack_experts(self.li.w1, self.li.w3, self.li.w2)
        torch.cuda.synchronize()
        if not keep_logical_weights:
            self.li.w1 = self.li.w3 = self.li.w2 = None
        self.bias = None if self.li.bias is None else torch.from_numpy(self.li.bias).cuda()
        # the gate matrix is static like the expert weights: packed once, outside the timed path (E > 16 only)
        self.wg_packed = moe.pack_gate(self.shape, self.li.wg)
        self.wg = self.li.wg if self.wg_packed is None else self.wg_packed
        self.ws = moe.new_workspace(self.shape)
        self.out = torch.empty((cfg.T, cfg.H), dtype=torch.bfloat16, device="cuda")
        self.tables = moe.tables(self.w1p, self.w3p, self.w2p)
        torch.cuda.synchronize()

    def activate(self):
        """Context options that go with this layer's buffers (the context is shared by all workloads)."""
        self.moe.set_option("gate_packed", 0 if self.wg_packed is None else 1)

    def step(self):
        self.moe.layer(self.shape, self.li.x, self.wg, self.bias, self.w1p, self.w3p, self.w2p, self.out, self.ws,
                       tables=self.tables)

    def settle(self, seconds: float):
        """Untimed steps: the chip needs about 0.1 s of this load before its clocks stop moving
        (the first 70 ms measure ~2 % slow), whatever warm-up count the caller passes."""
        import torch
        self.activate()
        t = time.perf_counter()
        while time.perf_counter() - t < seconds:
            for _ in range(10 if self.cfg.T * self.cfg.H < (1 << 26) else 2):
                self.step()
            torch.cuda.synchronize()

    def rows_per_expert(self):
        cnt = self.moe.layer_views(self.shape, self.ws)["expert_offsets"].cpu().diff()
        return cnt

    def timed(self, steps: int, warmup: int):
        """(a) K steps bracketed by synchronisation, nothing else on the stream: the headline;
        (b) K more steps with an event pair around each step and the library's per-stage events."""
        import torch
        from paper_2503_09716_amd import STAGES
        moe, cfg = self.moe, self.cfg
        self.activate()
        for _ in range(warmup):
            self.step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            self.step()
        torch.cuda.synchronize()
        ms_per_step = (time.perf_counter() - t0) / steps * 1e3
        moe.profile_enable(True)
        moe.profile_read()
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
        for a, b in ev:
            a.record()
            self.step()
            b.record()
        torch.cuda.synchronize()
        per_stage = moe.profile_read_intervals()
        moe.profile_enable(False)
        step_ms = med_min([a.elapsed_time(b) for a, b in ev])
        stage_ms = {s: med_min(per_stage[s]) for s in STAGES}
        R, Rs = cfg.T * cfg.top_k, cfg.T * cfg.num_shared
        f1, f2 = 4.0 * (R + Rs) * cfg.H * cfg.F, 2.0 * (R + Rs) * cfg.H * cfg.F
        g1, g2 = stage_ms["ffn_gate_up"]["median"], stage_ms["ffn_down"]["median"]
        tf = lambda f, ms: f / (ms * 1e-3) / 1e12 if ms > 0 else 0.0
        ffn = tf(f1 + f2, g1 + g2)
        cnt = self.rows_per_expert()
        return {
            "workload": "%s: T=%d H=%d F=%d E=%d top_k=%d shared=%d, weights resident in HBM" % (
                cfg.name, cfg.T, cfg.H, cfg.F, cfg.E, cfg.top_k, cfg.num_shared),
            "seed": cfg.seed,
            "rows_per_expert": {"max": int(cnt.max()), "mean": float(cnt.float().mean()), "min": int(cnt.min())},
            "steps": steps, "ms_per_step": ms_per_step, "tokens_per_s": cfg.T / (ms_per_step * 1e-3),
            "step_ms": step_ms, "stage_ms": stage_ms,
            "gate_up": {"flops_per_launch": f1, "TFLOP/s": tf(f1, g1), "frac_of_bf16_peak": tf(f1, g1) / PEAK_BF16_TFLOPS,
                        "TFLOP/s_at_min": tf(f1, stage_ms["ffn_gate_up"]["min"])},
            "down": {"flops_per_launch": f2, "TFLOP/s": tf(f2, g2), "frac_of_bf16_peak": tf(f2, g2) / PEAK_BF16_TFLOPS,
                     "TFLOP/s_at_min": tf(f2, stage_ms["ffn_down"]["min"])},
            "grouped_ffn_tflops": ffn, "grouped_ffn_frac_of_bf16_peak": ffn / PEAK_BF16_TFLOPS,
        }


def device_copy_gbs():
    """Measured ceiling beside the published HBM peak: a plain device-to-device copy of 1 GiB (read + write bytes)."""
    import torch
    src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
    dst = torch.empty_like(src)
    for _ in range(2):
        dst.copy_(src)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    ev[0].record()
    for _ in range(5):
        dst.copy_(src)
    ev[1].record()
    torch.cuda.synchronize()
    return 5 * 2 * src.numel() / (ev[0].elapsed_time(ev[1]) * 1e-3) / 1e9


def hbm_stages(moe, L: Layer, copy_gbs: float, reps: int = 5):
    """route / permute / combine through the staged entry points, each call on the next of N buffer
    sets whose total size exceeds twice the last-level cache, so that every call reads from HBM.
    Bytes are the algorithm's: route T*H*2 + 8*R (E <= 16 only: beyond that the router is a GEMM);
    permute T*H*2 read + R*H*2 written + 16*R of indices; combine R*H*y + T*H*y shared + 8*R + T*H*2
    with y = 2 or 4 bytes per element of y_perm (both measured; moe_layer's own choice is named)."""
    import torch
    cfg, sh = L.cfg, L.shape
    T, H, k, E, Ns = cfg.T, cfg.H, cfg.top_k, cfg.E, cfg.num_shared
    R = T * k
    dev = "cuda"

    def timed_calls(nsets, fn):
        for i in range(nsets):          # one untimed pass over every set
            fn(i)
        torch.cuda.synchronize()
        ev = []
        for r in range(reps):
            for i in range(nsets):
                a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                a.record()
                fn(i)
                b.record()
                ev.append((a, b))
        torch.cuda.synchronize()
        return med_min([a.elapsed_time(b) for a, b in ev])

    def nsets_for(set_bytes):
        return max(4, -(-2 * LLC_BYTES // set_bytes))

    def entry(bytes_, t, nsets, extra=None):
        gbs = bytes_ / (t["median"] * 1e-3) / 1e9 if t["median"] > 0 else 0.0
        e = {"bytes": bytes_, "ms": t, "GB/s": gbs, "frac_of_8TB/s": gbs / PEAK_HBM_GBS, "frac_of_device_copy": gbs / copy_gbs,
             "buffer_sets": nsets}
        if extra:
            e.update(extra)
        return e

    res = {"device_copy_1GiB_GB/s": copy_gbs,
           "how": "staged calls, each on the next of N buffer sets (N sets > 2x the 256 MB last-level cache), median over %d passes" % reps}
    idx = torch.empty((T, k), dtype=torch.int32, device=dev)
    w = torch.empty((T, k), dtype=torch.float32, device=dev)
    L.activate()
    moe.route(sh, L.li.x, L.wg, L.bias, idx, w, None, L.ws)
    torch.cuda.synchronize()
    # route
    n = nsets_for(T * H * 2)
    xs = [L.li.x.clone() for _ in range(n)]
    t = timed_calls(n, lambda i: moe.route(sh, xs[i], L.wg, L.bias, idx, w, None, L.ws))
    if E <= 16:
        res["route"] = entry(T * H * 2 + 8 * R, t, n)
    else:
        res["route_gemm"] = {"ms": t, "buffer_sets": n, "note": "E > 16: gate GEMM on the matrix cores + top-k kernel, not HBM-bound",
                             "TFLOP/s": 2.0 * T * H * E / (t["median"] * 1e-3) / 1e12}
    # permute (indices + row-major gather)
    n = nsets_for((T + R) * H * 2)
    xs = xs[:n] + [L.li.x.clone() for _ in range(max(0, n - len(xs)))]
    xp = [torch.empty((R, H), dtype=torch.bfloat16, device=dev) for _ in range(n)]
    off = torch.empty(E + 1, dtype=torch.int32, device=dev)
    perm = torch.empty(R, dtype=torch.int32, device=dev)
    inv = torch.empty(R, dtype=torch.int32, device=dev)
    t = timed_calls(n, lambda i: moe.permute(sh, xs[i], idx, xp[i], off, perm, inv, None, L.ws))
    res["permute"] = entry((T + R) * H * 2 + 16 * R, t, n, {"what": "moe_permute: histogram + scan + placement + row gather"})
    del xs, xp
    # combine, for both dtypes of y_perm
    layer_y32 = not (k >= 4 and Ns > 0)   # moe_layer's rule (option "layer_y_fp32" = -1)
    for y32 in (True, False):
        ysz = 4 if y32 else 2
        ydt = torch.float32 if y32 else torch.bfloat16
        set_bytes = R * H * ysz + (T * H * ysz if Ns else 0) + T * H * 2
        n = nsets_for(set_bytes)
        ys = [torch.randn((R, H), dtype=torch.float32, device=dev).to(ydt) for _ in range(n)]
        ysh = [torch.randn((T, H), dtype=torch.float32, device=dev).to(ydt) if Ns else None for _ in range(n)]
        outs = [torch.empty((T, H), dtype=torch.bfloat16, device=dev) for _ in range(n)]
        moe.set_option("y_fp32", 1 if y32 else 0)
        try:
            t = timed_calls(n, lambda i: moe.combine(sh, ys[i], inv, w, ysh[i], outs[i]))
        finally:
            moe.set_option("y_fp32", 1)
        res["combine_y_%s" % ("fp32" if y32 else "bf16")] = entry(
            set_bytes + 8 * R, t, n, {"y_perm_dtype": "fp32" if y32 else "bf16",
                                      "is_moe_layer_choice": y32 == layer_y32})
        del ys, ysh, outs
    res["note"] = ("moe_layer on this workload keeps y_perm in %s (y_shared always fp32); the in-layer stage_ms of combine "
                   "reads y_perm that the down projection has just written (partly cache-resident), these figures do not"
                   % ("fp32" if layer_y32 else "bf16"))
    torch.cuda.empty_cache()
    return res


def measured_ceiling(moe, L: Layer, iters: int = 40000, launches: int = 3):
    """Register-only loop of the GEMM's MFMA instruction, on zeros and on this workload's data."""
    import torch
    sink = torch.empty(1 << 20, dtype=torch.uint8, device="cuda")
    a = L.w1p[0]
    b = L.li.x.reshape(-1)
    out = {"kernel": "mfma_ceiling_kernel: v_mfma_f32_16x16x32_bf16, 64 accumulator blocks per wave, no LDS or memory traffic in the loop",
           "iters": iters, "launches": launches}
    for name, (pa, pb) in (("zeros", (None, None)), ("workload_data", (a, b)), ("zeros_again", (None, None))):
        runs = [moe.mfma_ceiling(pa, pb, iters, sink) for _ in range(launches)]
        out[name] = {"TFLOP/s": [r[0] for r in runs], "ms": [r[1] for r in runs]}
    out["operands"] = "a = packed W1 of expert 0 (N(0, 0.02^2)), b = x (N(0, 1)) of %s" % L.cfg.name
    out["TFLOP/s_on_workload_data"] = statistics.median(out["workload_data"]["TFLOP/s"])
    out["TFLOP/s_on_zeros"] = statistics.median(out["zeros"]["TFLOP/s"] + out["zeros_again"]["TFLOP/s"])
    return out


def blas_reference(cfg, steps):
    """Context only: the vendor BLAS (torch.bmm, bf16) on the two dense batched GEMMs that the grouped FFN
    would be with exactly T*k/E rows per expert, on data of the same distribution."""
    import torch
    from workloads import normal_bf16
    R = cfg.T * cfg.top_k
    rows = max(1, R // cfg.E)
    a1 = normal_bf16(cfg.seed, 101, (cfg.E, rows, cfg.H), 1.0, "cuda")
    b1 = normal_bf16(cfg.seed, 102, (cfg.E, cfg.H, 2 * cfg.F), 0.02, "cuda")
    a2 = normal_bf16(cfg.seed, 103, (cfg.E, rows, cfg.F), 1.0, "cuda")
    b2 = normal_bf16(cfg.seed, 104, (cfg.E, cfg.F, cfg.H), 0.02, "cuda")
    ref = {}
    for nm, a, b in (("gate_up", a1, b1), ("down", a2, b2)):
        for _ in range(3):
            torch.bmm(a, b)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(steps):
            torch.bmm(a, b)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / steps
        ref[nm] = {"ms": ms, "TFLOP/s": 2.0 * a.shape[0] * a.shape[1] * a.shape[2] * b.shape[2] / (ms * 1e-3) / 1e12}
    return {"what": "torch.bmm bf16, %d x [%d rows], no routing raggedness, no SiLU epilogue" % (cfg.E, rows), **ref}


def sweep(args):
    """Grouped-FFN throughput against the number of tokens per expert (the paper's Fig. 3 on this GPU),
    with the weights resident in HBM (left panel) and streamed from pinned host memory expert by
    expert through two staging slots (right panel: the share of the streamed layer's time during
    which the GPU waits for weights, measured, beside the critical-path estimate).  Markdown table."""
    import torch
    from paper_2503_09716_amd import Moe, STAGES, estimate_streamed_ms, shape_of
    from workloads import make_layer_inputs, scaled_config

    # C5's expert shape with 32 experts and no shared expert, so that large n stays inside the 4 GiB-per-matrix limit
    base = dict(C2=dict(), C5=dict(E=32, num_shared=0, bias="none"))[args.sweep]
    probe = scaled_config(args.sweep, **base)
    moe = Moe(0)
    expert_bytes = 3 * probe.H * probe.F * 2
    print("| tokens/expert | T | resident FFN ms | FFN TFLOP/s | % of 2.5 PF | streamed layer ms | host link GB/s | "
          "idle fraction measured | estimated layer ms | idle fraction estimated |")
    print("|---|---|---|---|---|---|---|---|---|---|")
    weights = host = None
    points = sorted(set([1 << lg for lg in range(4, args.max_log2 + 1)] + [75]))   # 75: the decode row of Table 1
    for n in points:
        T = n * probe.E // probe.top_k
        cfg = scaled_config(args.sweep, T=T, **base)
        li = make_layer_inputs(cfg, device="cuda", experts=weights is None)
        if weights is None:
            weights = moe.pack_experts(li.w1, li.w3, li.w2)   # the weights do not depend on T
            li.w1 = li.w3 = li.w2 = None
            host = [[w.cpu().pin_memory() for w in ws_] for ws_ in weights]
        w1p, w3p, w2p = weights
        shape = shape_of(cfg)
        ws = moe.new_workspace(shape)
        out = torch.empty((cfg.T, cfg.H), dtype=torch.bfloat16, device="cuda")
        bias = None if li.bias is None else torch.from_numpy(li.bias).cuda()
        tables = moe.tables(w1p, w3p, w2p)
        # untimed settling phase, as in the benchmark proper: after the idle stretches of the streamed
        # runs the chip's clocks need some tens of milliseconds of this load to stop moving
        t_end = time.perf_counter() + 0.25
        while time.perf_counter() < t_end:
            for _ in range(4):
                moe.layer(shape, li.x, li.wg, bias, w1p, w3p, w2p, out, ws, tables=tables)
            torch.cuda.synchronize()
        moe.profile_enable(True)
        moe.profile_read()
        for _ in range(args.steps):
            moe.layer(shape, li.x, li.wg, bias, w1p, w3p, w2p, out, ws, tables=tables)
        torch.cuda.synchronize()
        prof = moe.profile_read_intervals()
        moe.profile_enable(False)
        ffn_ms = statistics.median(prof["ffn_gate_up"]) + statistics.median(prof["ffn_down"])
        tf = cfg.ffn_flops / (ffn_ms * 1e-3) / 1e12
        # streamed: one expert per group, two slots (the double buffer of Sec. 4.2)
        slots = torch.empty(2 * expert_bytes, dtype=torch.uint8, device="cuda")
        moe.layer_streamed(shape, li.x, li.wg, bias, host[0], host[1], host[2], slots, 2, 1, out, ws)
        torch.cuda.synchronize()
        times = []
        for _ in range(3):
            t0 = time.perf_counter()
            moe.layer_streamed(shape, li.x, li.wg, bias, host[0], host[1], host[2], slots, 2, 1, out, ws)
            torch.cuda.synchronize()
            times.append((time.perf_counter() - t0) * 1e3)
        st_ms = statistics.median(times)
        stats = moe.stream_stats()
        link = stats["bytes_copied"] / (st_ms * 1e-3) / 1e9
        idle = max(0.0, 1.0 - ffn_ms / st_ms)
        cnt = moe.layer_views(shape, ws)["expert_offsets"].cpu().diff().tolist()
        est = estimate_streamed_ms(shape, cnt, 1, 2, args.link_gbs, tf)
        idle_est = max(0.0, 1.0 - ffn_ms / est) if est > 0 else 0.0
        print("| %d | %d | %.3f | %.0f | %.1f | %.2f | %.1f | %.3f | %.2f | %.3f |" % (
            n, T, ffn_ms, tf, 100 * tf / PEAK_BF16_TFLOPS, st_ms, link, idle, est, idle_est), flush=True)
        del ws, out, li, slots
        torch.cuda.empty_cache()
    moe.close()


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="C2")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-all-workloads", action="store_true", help="skip the figures of the other named workloads")
    ap.add_argument("--no-hbm-stages", action="store_true", help="skip the rotating-buffer timing of route / permute / combine")
    ap.add_argument("--no-ceiling", action="store_true", help="skip the register-only MFMA ceiling measurement")
    ap.add_argument("--option", action="append", default=[], help="library tuning knob key=value")
    ap.add_argument("--max-tokens-per-pass", type=int, default=0, metavar="B_E",
                    help="also time moe_layer_chunked with this many tokens per pass (workspace sized for one pass) "
                         "and report it in a 'chunked' object")
    ap.add_argument("--streamed", type=int, default=0, metavar="G",
                    help="also time moe_layer_streamed (expert weights in pinned host memory, G experts per group, "
                         "two staging slots) and report it in a 'streamed' object")
    ap.add_argument("--blas-reference", action="store_true",
                    help="context only: time the vendor BLAS (torch.bmm, bf16) on the two dense batched GEMMs that the "
                         "grouped FFN would be with exactly T*k/E rows per expert, on data of the same distribution")
    ap.add_argument("--calibrate-copy", type=int, default=0, metavar="MIB",
                    help="after the timed steps, run one plain device copy of this many MiB (a kernel of known "
                         "HBM traffic for scaling the profiler's FETCH_SIZE / WRITE_SIZE counters)")
    ap.add_argument("--sweep", choices=["C2", "C5"], help="tokens-per-expert sweep of this expert shape instead of the benchmark")
    ap.add_argument("--max-log2", type=int, default=14, help="--sweep: largest tokens-per-expert point")
    ap.add_argument("--link-gbs", type=float, default=56.0, help="--sweep: host-to-device rate the estimate assumes")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)
    if args.sweep:
        if args.steps == 50:
            args.steps = 5
        return sweep(args)

    import numpy
    import torch
    from paper_2503_09716_amd import Moe, estimate_streamed_ms, shape_of
    from workloads import get_config

    cfg = get_config(args.workload)
    moe = Moe(0)
    for kv in args.option:
        k, v = kv.split("=")
        moe.set_option(k, int(v))
    L = Layer(moe, cfg, keep_logical_weights=not args.no_cpu_baseline)
    L.settle(0.2)
    head = L.timed(args.steps, args.warmup)
    if args.calibrate_copy:
        src = torch.empty(args.calibrate_copy << 20, dtype=torch.uint8, device="cuda").random_(0, 255)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)   # reads and writes calibrate_copy MiB each
        torch.cuda.synchronize()
        del src, dst

    g1 = head["gate_up"]
    traffic, traffic_source = None, None
    tpath = os.path.join(ROOT, "profiles", "traffic_%s.json" % cfg.name)
    if os.path.exists(tpath):
        tj = json.load(open(tpath))
        traffic = tj.get("ffn_gate_up_hbm_bytes_per_launch")
        traffic_source = "profiles/traffic_%s.json: %s (an earlier profiler run of this command, not this run)" % (cfg.name, tj.get("source", ""))
    roofline = {"bound": "mfma", "kernel": "ffn_gemm_kernel<gated> (gate/up projection + SiLU-gate)",
                "achieved": g1["TFLOP/s"], "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                "frac": g1["frac_of_bf16_peak"], "traffic": traffic, "traffic_source": traffic_source,
                "avg_launch_ms": head["stage_ms"]["ffn_gate_up"]["median"], "min_launch_ms": head["stage_ms"]["ffn_gate_up"]["min"],
                "flops_per_launch": g1["flops_per_launch"],
                "target_frac": TARGET_FRAC, "target_met": bool(head["grouped_ffn_frac_of_bf16_peak"] >= TARGET_FRAC)}
    if not args.no_ceiling:
        ceil = measured_ceiling(moe, L)
        roofline["measured_ceiling"] = ceil
        roofline["frac_of_measured_ceiling"] = g1["TFLOP/s"] / ceil["TFLOP/s_on_workload_data"]
        roofline["frac_of_measured_ceiling_on_zeros"] = g1["TFLOP/s"] / ceil["TFLOP/s_on_zeros"]

    result = {
        "metric": METRIC,
        "value": head["tokens_per_s"],
        "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": head["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": head["workload"], "rows_per_expert": head["rows_per_expert"], "seed": cfg.seed,
                   "generator": "workloads.gen.normal_bf16: splitmix64 counter -> 65536-point quantile table of N(0, std^2), bf16 RNE; "
                                "x std 1, weights std 0.02; same bits on CPU and GPU",
                   "versions": {"torch": torch.__version__, "numpy": numpy.__version__, "hip": getattr(torch.version, "hip", None),
                                "device": torch.cuda.get_device_name(0)}},
        "step_ms": head["step_ms"],
        "grouped_ffn_tflops": head["grouped_ffn_tflops"],
        "grouped_ffn_frac_of_bf16_peak": head["grouped_ffn_frac_of_bf16_peak"],
        "gate_up": head["gate_up"], "down": head["down"],
        "stage_ms": head["stage_ms"],
        "timing": "ms_per_step / value: %d steps between two synchronisations, no events on the stream; step_ms and stage_ms: "
                  "a second loop of %d steps with HIP events (median, min)" % (args.steps, args.steps),
        "roofline": roofline,
    }
    if not args.no_hbm_stages:
        result["hbm_stages"] = hbm_stages(moe, L, device_copy_gbs())
    ffn_tflops = head["grouped_ffn_tflops"]
    shape, li, bias, w1p, w3p, w2p, out, ws, tables = L.shape, L.li, L.bias, L.w1p, L.w3p, L.w2p, L.out, L.ws, L.tables
    if args.max_tokens_per_pass:
        be = min(args.max_tokens_per_pass, cfg.T)
        from dataclasses import replace
        ws_pass = moe.new_workspace(shape_of(replace(cfg, T=be)))
        for _ in range(3):
            moe.layer_chunked(shape, li.x, L.wg, bias, w1p, w3p, w2p, be, out, ws_pass, tables=tables)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            moe.layer_chunked(shape, li.x, L.wg, bias, w1p, w3p, w2p, be, out, ws_pass, tables=tables)
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) / args.steps * 1e3
        result["chunked"] = {"max_tokens_per_pass": be, "passes": -(-cfg.T // be), "ms_per_step": ms,
                             "tokens/s": cfg.T / (ms * 1e-3), "workspace_bytes": ws_pass.numel(),
                             "workspace_bytes_unchunked": ws.numel()}
    if args.streamed:
        G = args.streamed
        host = [[w.cpu().pin_memory() for w in ws_] for ws_ in (w1p, w3p, w2p)]
        expert_bytes = 3 * cfg.H * cfg.F * 2
        slots = torch.empty(2 * max(G, cfg.num_shared) * expert_bytes, dtype=torch.uint8, device="cuda")
        for _ in range(2):
            moe.layer_streamed(shape, li.x, L.wg, bias, host[0], host[1], host[2], slots, 2, G, out, ws)
        torch.cuda.synchronize()
        n = max(3, args.steps // 4)
        t0 = time.perf_counter()
        for _ in range(n):
            moe.layer_streamed(shape, li.x, L.wg, bias, host[0], host[1], host[2], slots, 2, G, out, ws)
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) / n * 1e3
        st = moe.stream_stats()
        est = estimate_streamed_ms(shape, L.rows_per_expert().tolist(), G, 2, 56.0, ffn_tflops)   # 56 GB/s: this pool's pinned host-to-device rate
        result["streamed"] = {"experts_per_group": G, "slots": 2, "ms_per_step": ms, "tokens/s": cfg.T / (ms * 1e-3),
                              "critical_path_estimate_ms_expert_phase": est,
                              "host_to_device_GB/s": st["bytes_copied"] / (ms * 1e-3) / 1e9,
                              "bytes_copied_per_step": st["bytes_copied"], "groups": st["groups"],
                              "experts_skipped": st["experts_skipped"]}
        del host, slots
    if args.blas_reference:
        result["blas_reference"] = blas_reference(cfg, args.steps)
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(cfg, L.li)
    if not args.no_all_workloads:
        # the other named workloads: 20 steps each, same protocol, no oracle leg
        L = li = w1p = w3p = w2p = out = ws = tables = None
        torch.cuda.empty_cache()
        others = {}
        for name in ("C1", "C2", "C3", "C4", "C5"):
            if name == cfg.name:
                continue
            Lw = Layer(moe, get_config(name))
            Lw.settle(0.15)
            r = Lw.timed(20 if name != "C1" else 50, 3)
            r["target_frac"] = TARGET_FRAC if name in ("C2", "C3") else None
            others[name] = r
            Lw = None
            torch.cuda.empty_cache()
        result["all_workloads"] = others
    print(json.dumps(result))
    moe.close()


if __name__ == "__main__":
    main()
