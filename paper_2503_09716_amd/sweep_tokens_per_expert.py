"""Grouped-FFN throughput against the number of tokens per expert (the paper's Fig. 3 on this GPU).

For a fixed expert shape the script runs moe_layer on synthetic batches whose size gives each
expert about n rows, n = 2^4 .. 2^max, and prints a markdown table: achieved TFLOP/s of the two
grouped GEMMs (weights resident in HBM), the time one expert's n rows take, and the fraction of
time the GPU would idle if that expert's weights had to arrive over the host link meanwhile
(Sec. 4.2: the batch must be large enough for expert compute to cover the weight prefetch).

    python -m paper_2503_09716_amd.sweep_tokens_per_expert [--shape C2|C5] [--max-log2 14] [--link-gbs 56]
"""
from __future__ import annotations

import argparse
import os
import sys

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--shape", default="C2", choices=["C2", "C5"])
    ap.add_argument("--max-log2", type=int, default=14)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--link-gbs", type=float, default=56.0, help="measured host-to-device rate of the streamed path")
    args = ap.parse_args()

    import torch
    from paper_2503_09716_amd import Moe, STAGES, shape_of
    from workloads import make_layer_inputs, scaled_config

    # C5's expert shape with 32 experts and no shared expert, so that large n stays inside the 4 GiB-per-matrix limit
    base = dict(C2=dict(), C5=dict(E=32, num_shared=0, bias="none"))[args.shape]
    probe = scaled_config(args.shape, **base)
    moe = Moe(0)
    expert_bytes = 3 * probe.H * probe.F * 2
    print("| tokens/expert | T | FFN ms | FFN TFLOP/s | %% of 2.5 PF | us per expert | weight fetch us @ %.0f GB/s | idle fraction if streamed |" % args.link_gbs)
    print("|---|---|---|---|---|---|---|---|")
    weights = None
    for lg in range(4, args.max_log2 + 1):
        n = 1 << lg
        T = n * probe.E // probe.top_k
        cfg = scaled_config(args.shape, T=T, **base)
        li = make_layer_inputs(cfg, device="cuda", experts=weights is None)
        if weights is None:
            weights = moe.pack_experts(li.w1, li.w3, li.w2)   # the weights do not depend on T
            li.w1 = li.w3 = li.w2 = None
        w1p, w3p, w2p = weights
        shape = shape_of(cfg)
        ws = moe.new_workspace(shape)
        out = torch.empty((cfg.T, cfg.H), dtype=torch.bfloat16, device="cuda")
        bias = None if li.bias is None else torch.from_numpy(li.bias).cuda()
        tables = moe.tables(w1p, w3p, w2p)
        for _ in range(2):
            moe.layer(shape, li.x, li.wg, bias, w1p, w3p, w2p, out, ws, tables=tables)
        torch.cuda.synchronize()
        moe.profile_enable(True)
        moe.profile_read()
        for _ in range(args.steps):
            moe.layer(shape, li.x, li.wg, bias, w1p, w3p, w2p, out, ws, tables=tables)
        torch.cuda.synchronize()
        prof = moe.profile_read()
        moe.profile_enable(False)
        ms = {s: prof[s][0] / max(1, prof[s][1]) for s in STAGES}
        ffn_ms = ms["ffn_gate_up"] + ms["ffn_down"]
        tf = cfg.ffn_flops / (ffn_ms * 1e-3) / 1e12
        per_expert_us = ffn_ms * 1e3 / cfg.E
        fetch_us = expert_bytes / (args.link_gbs * 1e9) * 1e6
        idle = max(0.0, 1.0 - per_expert_us / fetch_us)
        print("| %d | %d | %.3f | %.0f | %.1f | %.1f | %.0f | %.3f |" % (n, T, ffn_ms, tf, 100 * tf / 2500.0, per_expert_us, fetch_us, idle),
              flush=True)
        del ws, out, li
        torch.cuda.empty_cache()
    moe.close()


if __name__ == "__main__":
    main()
