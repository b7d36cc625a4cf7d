"""moe_layer_static: the layer for callers that cannot allocate (its workspace is a scratch array
inside the library's device image).  Called through the C ABI; its output must equal moe_layer's
bit for bit, on two calls in a row of which the second has a smaller input (the scratch still
holds the first call's intermediates)."""
import pytest
import torch

import parity as P
from workloads import make_layer_inputs, scaled_config

pytestmark = pytest.mark.gpu


def test_static_scratch_layer_equals_layer_twice_in_a_row_second_smaller():
    from paper_2503_09716_amd import Moe, MoeError
    from paper_2503_09716_amd.binding import workspace_bytes, STATIC_WORKSPACE_BYTES
    moe = Moe(0)
    try:
        first = scaled_config("C4", T=640, H=256, F=192)                    # 64 experts top-6 + 2 shared
        second = scaled_config("C2", T=97, H=128, F=320, E=8, top_k=2)      # smaller in every dimension, no shared experts
        for fp32 in (0, 1):
            moe.set_option("out_fp32", fp32)
            for cfg in (first, second):
                print("static", cfg, "out_fp32", fp32, flush=True)
                gl = P.GpuLayer(moe, make_layer_inputs(cfg, device="cuda"), host_weights=False)
                assert workspace_bytes(gl.shape) <= STATIC_WORKSPACE_BYTES
                dt = torch.float32 if fp32 else torch.bfloat16
                ref = torch.empty((cfg.T, cfg.H), dtype=dt, device="cuda")
                moe.layer(gl.shape, gl.x, gl.wg, gl.bias, gl.w1p, gl.w3p, gl.w2p, ref, gl.ws, tables=gl.tables)
                got = torch.full_like(ref, float("nan"))
                torch.cuda.synchronize()
                held = torch.cuda.memory_allocated()
                moe.layer_static(gl.shape, gl.x, gl.wg, gl.bias, gl.w1p, gl.w3p, gl.w2p, got, tables=gl.tables)
                assert torch.cuda.memory_allocated() == held
                torch.cuda.synchronize()
                assert torch.isfinite(ref.float()).all()
                assert torch.equal(ref.view(torch.int32 if fp32 else torch.int16), got.view(torch.int32 if fp32 else torch.int16))
        moe.set_option("out_fp32", 0)
        # a shape whose intermediates do not fit the scratch is refused before anything is enqueued
        big = scaled_config("C2", T=4096, H=1024, F=2048)
        gl = P.GpuLayer(moe, make_layer_inputs(big, device="cuda"), host_weights=False)
        assert workspace_bytes(gl.shape) > STATIC_WORKSPACE_BYTES
        out = torch.zeros((big.T, big.H), dtype=torch.bfloat16, device="cuda")
        with pytest.raises(MoeError) as ei:
            moe.layer_static(gl.shape, gl.x, gl.wg, gl.bias, gl.w1p, gl.w3p, gl.w2p, out, tables=gl.tables)
        assert ei.value.status == 3 and "scratch" in str(ei.value)
        torch.cuda.synchronize()
        assert (out == 0).all()
    finally:
        moe.close()


def test_static_scratch_layer_in_a_hip_graph():
    """The callers the entry point is for: captured once (after one eager call, which uploads the
    weight pointer table), replayed with eager work and synchronisations in between; every replay
    gives moe_layer's bits."""
    from paper_2503_09716_amd import Moe
    moe = Moe(0)
    try:
        cfg = scaled_config("C4", T=333, H=256, F=192)
        gl = P.GpuLayer(moe, make_layer_inputs(cfg, device="cuda"), host_weights=False)
        ref = gl.run_layer().clone()
        out = torch.empty_like(ref)

        def step():
            moe.layer_static(gl.shape, gl.x, gl.wg, gl.bias, gl.w1p, gl.w3p, gl.w2p, out, tables=gl.tables)

        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            step()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        assert torch.equal(out, ref)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step()
        torch.cuda.synchronize()
        for _ in range(3):
            out.zero_()
            graph.replay()
            torch.cuda.synchronize()
            assert torch.equal(out, ref)
            assert torch.equal(gl.run_layer(), ref)      # eager work of the library between replays
    finally:
        moe.close()
