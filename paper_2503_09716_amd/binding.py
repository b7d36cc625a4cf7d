"""Thin ctypes binding of libmoe_mi355.so (the C ABI declared in include/moe.h).

Argument marshalling only: torch supplies device memory and the current stream; every step
of the MoE expert module runs in the library's HIP kernels.  There is no fallback: if the
library is missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence

import torch

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libmoe_mi355.so")

STATIC_WORKSPACE_BYTES = 32 << 20   # MOE_STATIC_WORKSPACE_BYTES of include/moe.h

STAGES = ["route", "permute_index", "permute_gather", "plan", "ffn_gate_up", "ffn_down", "combine"]

EXPORTS = [
    "moe_create", "moe_destroy", "moe_last_error", "moe_workspace_bytes", "moe_h_scratch_bytes", "moe_set_option", "moe_pack_weight",
    "moe_gate_packed_bytes", "moe_pack_gate",
    "moe_route", "moe_permute", "moe_grouped_ffn", "moe_combine", "moe_layer", "moe_layer_static", "moe_layer_views",
    "moe_layer_streamed", "moe_stream_stats", "moe_estimate_streamed_ms", "moe_accumulate", "moe_layer_chunked",
    "moe_profile_enable", "moe_profile_read", "moe_profile_read_intervals", "moe_profile_mfma_ceiling",
]


class MoeShape(C.Structure):
    _fields_ = [("T", C.c_int32), ("H", C.c_int32), ("F", C.c_int32), ("E", C.c_int32), ("top_k", C.c_int32),
                ("num_shared", C.c_int32), ("renormalize", C.c_int32), ("routed_scale", C.c_float)]


class MoeError(RuntimeError):
    def __init__(self, status: int, msg: str):
        super().__init__("moe status %d: %s" % (status, msg))
        self.status = status


_lib = None


def load_library():
    """Loads the in-tree library (building it first only if it does not exist yet)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        from .build import build
        build()
    lib = C.CDLL(LIB_PATH)
    vp, i32p, f32p = C.c_void_p, C.c_void_p, C.c_void_p
    sp = C.POINTER(MoeShape)
    tab = C.POINTER(C.c_void_p)
    lib.moe_create.argtypes = [C.POINTER(C.c_void_p), C.c_int]
    lib.moe_destroy.argtypes = [C.c_void_p]
    lib.moe_destroy.restype = None
    lib.moe_last_error.argtypes = [C.c_void_p]
    lib.moe_last_error.restype = C.c_char_p
    lib.moe_workspace_bytes.argtypes = [sp]
    lib.moe_workspace_bytes.restype = C.c_size_t
    lib.moe_h_scratch_bytes.argtypes = [sp]
    lib.moe_h_scratch_bytes.restype = C.c_size_t
    lib.moe_gate_packed_bytes.argtypes = [sp]
    lib.moe_gate_packed_bytes.restype = C.c_size_t
    lib.moe_pack_gate.argtypes = [C.c_void_p, sp, vp, vp, vp]
    lib.moe_set_option.argtypes = [C.c_void_p, C.c_char_p, C.c_int32]
    lib.moe_pack_weight.argtypes = [C.c_void_p, vp, C.c_int32, C.c_int32, vp, vp]
    lib.moe_route.argtypes = [C.c_void_p, sp, vp, vp, f32p, i32p, f32p, f32p, vp, C.c_size_t, vp]
    lib.moe_permute.argtypes = [C.c_void_p, sp, vp, i32p, vp, i32p, i32p, i32p, i32p, vp, C.c_size_t, vp]
    lib.moe_grouped_ffn.argtypes = [C.c_void_p, sp, vp, i32p, vp, i32p, tab, tab, tab, vp, vp, vp, vp, C.c_size_t, vp]
    lib.moe_combine.argtypes = [C.c_void_p, sp, vp, i32p, f32p, vp, vp, vp]
    lib.moe_layer.argtypes = [C.c_void_p, sp, vp, vp, f32p, tab, tab, tab, vp, vp, C.c_size_t, vp]
    lib.moe_layer_static.argtypes = [C.c_void_p, sp, vp, vp, f32p, tab, tab, tab, vp, vp]
    lib.moe_layer_streamed.argtypes = [C.c_void_p, sp, vp, vp, f32p, tab, tab, tab, vp, C.c_size_t, C.c_int32, C.c_int32,
                                       vp, vp, C.c_size_t, vp]
    lib.moe_accumulate.argtypes = [C.c_void_p, vp, C.c_int32, C.c_int32, C.POINTER(C.c_int32), vp, C.c_int32, vp]
    lib.moe_layer_chunked.argtypes = [C.c_void_p, sp, vp, vp, f32p, tab, tab, tab, C.c_int32, vp, vp, C.c_size_t, vp]
    lib.moe_stream_stats.argtypes = [C.c_void_p, C.POINTER(C.c_uint64), C.POINTER(C.c_int32), C.POINTER(C.c_int32)]
    lib.moe_layer_views.argtypes = [sp, vp, C.POINTER(C.c_void_p), C.POINTER(C.c_void_p), C.POINTER(C.c_void_p),
                                    C.POINTER(C.c_void_p)]
    lib.moe_profile_enable.argtypes = [C.c_void_p, C.c_int32]
    lib.moe_profile_read.argtypes = [C.c_void_p, C.POINTER(C.c_double), C.POINTER(C.c_int32)]
    lib.moe_profile_read_intervals.argtypes = [C.c_void_p, C.POINTER(C.c_int32), C.POINTER(C.c_float), C.c_int32,
                                               C.POINTER(C.c_int32)]
    lib.moe_profile_mfma_ceiling.argtypes = [C.c_void_p, vp, vp, C.c_size_t, C.c_int32, vp, C.c_size_t,
                                             C.POINTER(C.c_double), C.POINTER(C.c_double), vp]
    lib.moe_estimate_streamed_ms.argtypes = [sp, C.POINTER(C.c_int32), C.c_int32, C.c_int32, C.c_double, C.c_double]
    lib.moe_estimate_streamed_ms.restype = C.c_double
    for name in EXPORTS:
        if name not in ("moe_destroy", "moe_last_error", "moe_workspace_bytes", "moe_h_scratch_bytes", "moe_gate_packed_bytes",
                        "moe_estimate_streamed_ms"):
            getattr(lib, name).restype = C.c_int
    _lib = lib
    return lib


def make_shape(T, H, F, E, top_k, num_shared=0, renormalize=True, routed_scale=1.0) -> MoeShape:
    return MoeShape(int(T), int(H), int(F), int(E), int(top_k), int(num_shared), 1 if renormalize else 0,
                    float(routed_scale))


def shape_of(cfg) -> MoeShape:
    return make_shape(cfg.T, cfg.H, cfg.F, cfg.E, cfg.top_k, cfg.num_shared, cfg.renormalize, cfg.routed_scale)


def workspace_bytes(shape: MoeShape) -> int:
    return int(load_library().moe_workspace_bytes(C.byref(shape)))


def h_scratch_bytes(shape: MoeShape) -> int:
    return int(load_library().moe_h_scratch_bytes(C.byref(shape)))


def estimate_streamed_ms(shape: MoeShape, rows_per_expert, experts_per_group: int, num_slots: int, link_gbs: float,
                         ffn_tflops: float) -> float:
    """Critical-path estimate of the expert phase of Moe.layer_streamed (host arithmetic)."""
    rows = (C.c_int32 * shape.E)(*[int(r) for r in rows_per_expert])
    return float(load_library().moe_estimate_streamed_ms(C.byref(shape), rows, experts_per_group, num_slots,
                                                         link_gbs, ffn_tflops))


def _ptr(t: Optional[torch.Tensor]):
    if t is None:
        return None
    assert t.is_cuda and t.is_contiguous(), "device-resident contiguous tensor required"
    return C.c_void_p(t.data_ptr())


def _table(ws: Sequence[torch.Tensor]):
    for w in ws:
        assert w.is_cuda and w.is_contiguous()
    return (C.c_void_p * len(ws))(*[w.data_ptr() for w in ws])


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


class Moe:
    """One library context on one GPU.  Methods mirror the C entry points one to one."""

    def __init__(self, device: int = 0):
        self.lib = load_library()
        self.device = device
        h = C.c_void_p()
        st = self.lib.moe_create(C.byref(h), device)
        if st != 0 or not h:
            raise MoeError(st, "moe_create failed on device %d" % device)
        self.h = h

    def close(self):
        if getattr(self, "h", None):
            self.lib.moe_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, st: int):
        if st != 0:
            raise MoeError(st, self.lib.moe_last_error(self.h).decode())

    def set_option(self, key: str, value: int):
        self._check(self.lib.moe_set_option(self.h, key.encode(), int(value)))

    def new_workspace(self, shape: MoeShape) -> torch.Tensor:
        n = workspace_bytes(shape)
        if n == 0:
            raise MoeError(2, "unsupported or invalid shape")
        return torch.empty(n, dtype=torch.uint8, device="cuda:%d" % self.device)

    # ---- one-time weight packing -------------------------------------------------------
    def new_h_scratch(self, shape: MoeShape) -> torch.Tensor:
        return torch.empty(h_scratch_bytes(shape), dtype=torch.uint8, device="cuda:%d" % self.device)

    def pack_weight(self, w: torch.Tensor) -> torch.Tensor:
        """Logical [K, N] weight -> packed form (opaque 1-D bf16 tensor of K*N elements)."""
        rows, cols = w.shape
        out = torch.empty(rows * cols, dtype=torch.bfloat16, device=w.device)
        self._check(self.lib.moe_pack_weight(self.h, _ptr(w), rows, cols, _ptr(out), _stream()))
        return out

    def pack_gate(self, shape, wg: torch.Tensor):
        """Packed gate matrix for option "gate_packed"."""
        n = int(self.lib.moe_gate_packed_bytes(C.byref(shape)))
        if n == 0:
            return None
        out = torch.empty(n // 2, dtype=torch.bfloat16, device=wg.device)
        self._check(self.lib.moe_pack_gate(self.h, C.byref(shape), _ptr(wg), _ptr(out), _stream()))
        return out

    def pack_experts(self, w1: Sequence[torch.Tensor], w3: Sequence[torch.Tensor], w2: Sequence[torch.Tensor]):
        return ([self.pack_weight(w) for w in w1], [self.pack_weight(w) for w in w3],
                [self.pack_weight(w) for w in w2])

    # ---- staged calls ------------------------------------------------------------------
    def route(self, shape, x, wg, bias, topk_idx, topk_w, logits, workspace):
        self._check(self.lib.moe_route(self.h, C.byref(shape), _ptr(x), _ptr(wg), _ptr(bias), _ptr(topk_idx),
                                       _ptr(topk_w), _ptr(logits), _ptr(workspace), workspace.numel(), _stream()))

    def permute(self, shape, x, topk_idx, x_perm, expert_offsets, perm, inv_perm, row_token, workspace):
        self._check(self.lib.moe_permute(self.h, C.byref(shape), _ptr(x), _ptr(topk_idx), _ptr(x_perm),
                                         _ptr(expert_offsets), _ptr(perm), _ptr(inv_perm), _ptr(row_token),
                                         _ptr(workspace), workspace.numel(), _stream()))

    def grouped_ffn(self, shape, x_perm, row_token, x, expert_offsets, w1p, w3p, w2p, h_scratch, y_perm, y_shared,
                    workspace):
        self._check(self.lib.moe_grouped_ffn(self.h, C.byref(shape), _ptr(x_perm), _ptr(row_token), _ptr(x),
                                             _ptr(expert_offsets), _table(w1p), _table(w3p), _table(w2p),
                                             _ptr(h_scratch), _ptr(y_perm), _ptr(y_shared), _ptr(workspace),
                                             workspace.numel(), _stream()))

    def combine(self, shape, y_perm, inv_perm, topk_w, y_shared, out):
        self._check(self.lib.moe_combine(self.h, C.byref(shape), _ptr(y_perm), _ptr(inv_perm), _ptr(topk_w),
                                         _ptr(y_shared), _ptr(out), _stream()))

    # ---- fused call --------------------------------------------------------------------
    def layer(self, shape, x, wg, bias, w1p, w3p, w2p, out, workspace, tables=None):
        t1, t3, t2 = tables if tables is not None else (_table(w1p), _table(w3p), _table(w2p))
        self._check(self.lib.moe_layer(self.h, C.byref(shape), _ptr(x), _ptr(wg), _ptr(bias), t1, t3, t2,
                                       _ptr(out), _ptr(workspace), workspace.numel(), _stream()))

    def layer_static(self, shape, x, wg, bias, w1p, w3p, w2p, out, tables=None):
        """moe_layer with the library's built-in scratch as workspace (allocates nothing)."""
        t1, t3, t2 = tables if tables is not None else (_table(w1p), _table(w3p), _table(w2p))
        self._check(self.lib.moe_layer_static(self.h, C.byref(shape), _ptr(x), _ptr(wg), _ptr(bias), t1, t3, t2,
                                              _ptr(out), _stream()))

    def layer_streamed(self, shape, x, wg, bias, host_w1p, host_w3p, host_w2p, slots, num_slots, experts_per_group,
                       out, workspace):
        """Expert weights in pinned HOST tensors (packed layout); `slots` is a device byte buffer
        cut into num_slots equal staging slots."""
        def host_table(ws):
            for w in ws:
                assert (not w.is_cuda) and w.is_pinned() and w.is_contiguous(), "pinned host tensor required"
            return (C.c_void_p * len(ws))(*[w.data_ptr() for w in ws])
        slot_bytes = (slots.numel() * slots.element_size() // num_slots) & ~255
        self._check(self.lib.moe_layer_streamed(self.h, C.byref(shape), _ptr(x), _ptr(wg), _ptr(bias),
                                                host_table(host_w1p), host_table(host_w3p), host_table(host_w2p),
                                                _ptr(slots), slot_bytes, num_slots, experts_per_group, _ptr(out),
                                                _ptr(workspace), workspace.numel(), _stream()))

    def layer_chunked(self, shape, x, wg, bias, w1p, w3p, w2p, max_tokens_per_pass, out, workspace, tables=None):
        t1, t3, t2 = tables if tables is not None else (_table(w1p), _table(w3p), _table(w2p))
        self._check(self.lib.moe_layer_chunked(self.h, C.byref(shape), _ptr(x), _ptr(wg), _ptr(bias), t1, t3, t2,
                                               max_tokens_per_pass, _ptr(out), _ptr(workspace), workspace.numel(),
                                               _stream()))

    def accumulate(self, staging, rows_filled: int, x_microbatch) -> int:
        """Appends x_microbatch's rows to staging at row rows_filled; returns the new fill count."""
        n = C.c_int32(rows_filled)
        self._check(self.lib.moe_accumulate(self.h, _ptr(staging), staging.shape[0], staging.shape[1], C.byref(n),
                                            _ptr(x_microbatch), x_microbatch.shape[0], _stream()))
        return n.value

    def stream_stats(self):
        b, g, k = C.c_uint64(), C.c_int32(), C.c_int32()
        self._check(self.lib.moe_stream_stats(self.h, C.byref(b), C.byref(g), C.byref(k)))
        return {"bytes_copied": b.value, "groups": g.value, "experts_skipped": k.value}

    def tables(self, w1p, w3p, w2p):
        """Pre-marshalled pointer tables, so a timed loop does not rebuild them per call."""
        return _table(w1p), _table(w3p), _table(w2p)

    def layer_views(self, shape, workspace):
        """Routing results of the last layer() call, as torch views into the workspace."""
        p = [C.c_void_p() for _ in range(4)]
        st = self.lib.moe_layer_views(C.byref(shape), _ptr(workspace), *[C.byref(q) for q in p])
        if st != 0:
            raise MoeError(st, "moe_layer_views")
        base = workspace.data_ptr()
        R = shape.T * shape.top_k

        def view(ptr, nbytes, dtype, shp):
            off = ptr.value - base
            return workspace[off:off + nbytes].view(dtype).view(*shp)
        return {
            "topk_idx": view(p[0], R * 4, torch.int32, (shape.T, shape.top_k)),
            "topk_w": view(p[1], R * 4, torch.float32, (shape.T, shape.top_k)),
            "expert_offsets": view(p[2], (shape.E + 1) * 4, torch.int32, (shape.E + 1,)),
            "inv_perm": view(p[3], R * 4, torch.int32, (R,)),
        }

    # ---- profiling ---------------------------------------------------------------------
    def profile_enable(self, on: bool):
        self._check(self.lib.moe_profile_enable(self.h, 1 if on else 0))

    def profile_read_intervals(self, capacity: int = 8192):
        """{stage name: [ms, ...]} of every interval recorded since the last read, in order."""
        st = (C.c_int32 * capacity)()
        ms = (C.c_float * capacity)()
        n = C.c_int32()
        self._check(self.lib.moe_profile_read_intervals(self.h, st, ms, capacity, C.byref(n)))
        out = {s: [] for s in STAGES}
        for i in range(n.value):
            out[STAGES[st[i]]].append(float(ms[i]))
        return out

    def mfma_ceiling(self, a, b, iters: int, sink):
        """One timed launch of the register-only MFMA loop; a, b: bf16 device tensors of equal size or None.
        Returns (TFLOP/s, ms)."""
        tf, ms = C.c_double(), C.c_double()
        nbytes = 0 if a is None else min(a.numel() * a.element_size(), b.numel() * b.element_size())
        self._check(self.lib.moe_profile_mfma_ceiling(self.h, _ptr(a), _ptr(b), nbytes, iters, _ptr(sink),
                                                      sink.numel() * sink.element_size(), C.byref(tf), C.byref(ms),
                                                      _stream()))
        return tf.value, ms.value

    def profile_read(self):
        ms = (C.c_double * len(STAGES))()
        n = (C.c_int32 * len(STAGES))()
        self._check(self.lib.moe_profile_read(self.h, ms, n))
        return {s: (ms[i], n[i]) for i, s in enumerate(STAGES)}
