"""ctypes front end of the CPU oracle (oracle/moe_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, __graft_entry__.smoke() and bench.py's
cpu_baseline leg.  It shares nothing with the HIP path and the product never calls it.

All bf16 tensors are passed as numpy uint16 bit patterns, row-major:
  x [T,H], wg [H,E], w1/w3 [H,F] per expert, w2 [F,H] per expert (routed first, then shared).
"""
from __future__ import annotations

import ctypes as C
from typing import Optional, Sequence

import numpy as np

from .build import build

_lib = None

_u16p = C.POINTER(C.c_uint16)
_i32p = C.POINTER(C.c_int32)
_f32p = C.POINTER(C.c_float)


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.oracle_num_threads.restype = C.c_int
    return _lib


def _p(a: Optional[np.ndarray], ty):
    if a is None:
        return None
    assert a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(ty)


def _u16(a) -> np.ndarray:
    a = np.ascontiguousarray(a)
    assert a.dtype == np.uint16, a.dtype
    return a


def _ptr_table(ws: Sequence[np.ndarray]):
    keep = [_u16(w) for w in ws]
    arr = (_u16p * len(keep))(*[w.ctypes.data_as(_u16p) for w in keep])
    return arr, keep


def num_threads() -> int:
    return int(lib().oracle_num_threads())


def route(x, wg, bias, top_k: int, renormalize: bool, routed_scale: float = 1.0,
          tokens=None, want_logits: bool = False, want_probs: bool = False):
    """Router for all tokens (tokens=None) or for the listed token ids.

    Returns dict(idx int32 [n,k], w float32 [n,k], logits/probs float32 [n,E] if asked)."""
    x = _u16(x); wg = _u16(wg)
    T, H = x.shape
    H2, E = wg.shape
    assert H2 == H and 1 <= top_k <= E
    tok = None if tokens is None else np.ascontiguousarray(tokens, dtype=np.int32)
    n = T if tok is None else len(tok)
    b = None if bias is None else np.ascontiguousarray(bias, dtype=np.float32)
    idx = np.empty((n, top_k), np.int32)
    w = np.empty((n, top_k), np.float32)
    logits = np.empty((n, E), np.float32) if want_logits else None
    probs = np.empty((n, E), np.float32) if want_probs else None
    lib().oracle_route(_p(x, _u16p), _p(wg, _u16p), _p(b, _f32p), C.c_int(T), C.c_int(H), C.c_int(E),
                       C.c_int(top_k), C.c_int(1 if renormalize else 0), C.c_float(routed_scale),
                       _p(tok, _i32p), C.c_int(n), _p(idx, _i32p), _p(w, _f32p),
                       _p(logits, _f32p), _p(probs, _f32p))
    out = {"idx": idx, "w": w}
    if want_logits:
        out["logits"] = logits
    if want_probs:
        out["probs"] = probs
    return out


def permute(idx, E: int):
    """Stable per-expert grouping.  Returns (offsets [E+1], perm [T*k], inv_perm [T*k]) int32."""
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    T, k = idx.shape
    assert idx.min(initial=0) >= 0 and idx.max(initial=0) < E
    offsets = np.empty(E + 1, np.int32)
    perm = np.empty(T * k, np.int32)
    inv = np.empty(T * k, np.int32)
    lib().oracle_permute(_p(idx, _i32p), C.c_int(T), C.c_int(k), C.c_int(E),
                         _p(offsets, _i32p), _p(perm, _i32p), _p(inv, _i32p))
    return offsets, perm, inv


def expert_rows(xrows, eid, w1, w3, w2):
    """y[n,:] = SwiGLU expert eid[n] applied to row n.  Returns float32 [n,H]."""
    xrows = _u16(xrows)
    n, H = xrows.shape
    F = w1[0].shape[1]
    eid = np.ascontiguousarray(eid, dtype=np.int32)
    assert len(eid) == n and eid.min(initial=0) >= 0 and eid.max(initial=0) < len(w1)
    for a, b_, c in zip(w1, w3, w2):
        assert a.shape == (H, F) and b_.shape == (H, F) and c.shape == (F, H)
    t1, k1 = _ptr_table(w1); t3, k3 = _ptr_table(w3); t2, k2 = _ptr_table(w2)
    y = np.empty((n, H), np.float32)
    lib().oracle_expert_rows(_p(xrows, _u16p), _p(eid, _i32p), C.c_int(n), t1, t3, t2,
                             C.c_int(H), C.c_int(F), _p(y, _f32p))
    return y


def layer(x, idx, w, w1, w3, w2, E: int, num_shared: int, tokens=None):
    """Layer output (float32 [n,H]) for the listed tokens given their routing idx/w [n,k]."""
    x = _u16(x)
    T, H = x.shape
    F = w1[0].shape[1]
    assert len(w1) == len(w3) == len(w2) == E + num_shared
    for a, b_, c in zip(w1, w3, w2):
        assert a.shape == (H, F) and b_.shape == (H, F) and c.shape == (F, H)
    tok = None if tokens is None else np.ascontiguousarray(tokens, dtype=np.int32)
    n = T if tok is None else len(tok)
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    w = np.ascontiguousarray(w, dtype=np.float32)
    k = idx.shape[1]
    assert idx.shape == (n, k) and w.shape == (n, k)
    assert idx.min(initial=0) >= 0 and idx.max(initial=0) < E
    t1, k1 = _ptr_table(w1); t3, k3 = _ptr_table(w3); t2, k2 = _ptr_table(w2)
    out = np.empty((n, H), np.float32)
    lib().oracle_layer(_p(x, _u16p), _p(tok, _i32p), C.c_int(n), _p(idx, _i32p), _p(w, _f32p),
                       t1, t3, t2, C.c_int(H), C.c_int(F), C.c_int(E), C.c_int(k),
                       C.c_int(num_shared), _p(out, _f32p))
    return out


def combine(y_perm, inv_perm, w, y_shared=None):
    """out[t] = sum_j w[t,j] * y_perm[inv_perm[t*k+j]] (+ y_shared[t]); float32 [T,H].
    y_perm / y_shared: float32 arrays, or uint16 arrays of bf16 bit patterns."""
    y_perm = np.ascontiguousarray(y_perm)
    f32 = y_perm.dtype == np.float32
    assert f32 or y_perm.dtype == np.uint16
    R, H = y_perm.shape
    w = np.ascontiguousarray(w, dtype=np.float32)
    T, k = w.shape
    assert R == T * k
    inv = np.ascontiguousarray(inv_perm, dtype=np.int32).reshape(-1)
    assert len(inv) == R and inv.min(initial=0) >= 0 and inv.max(initial=0) < R
    ys = None
    if y_shared is not None:
        ys = np.ascontiguousarray(y_shared)
        assert ys.dtype == y_perm.dtype and ys.shape == (T, H)
    out = np.empty((T, H), np.float32)
    lib().oracle_combine(C.c_void_p(y_perm.ctypes.data), C.c_int(1 if f32 else 0), _p(inv, _i32p), _p(w, _f32p),
                         None if ys is None else C.c_void_p(ys.ctypes.data),
                         C.c_int(T), C.c_int(H), C.c_int(k), _p(out, _f32p))
    return out


def moe_forward(x, wg, bias, w1, w3, w2, top_k, num_shared, renormalize, routed_scale=1.0, tokens=None):
    """route + layer for convenience.  Returns (out [n,H], routing dict)."""
    E = wg.shape[1]
    r = route(x, wg, bias, top_k, renormalize, routed_scale, tokens=tokens, want_logits=True)
    out = layer(x, r["idx"], r["w"], w1, w3, w2, E, num_shared, tokens=tokens)
    return out, r
