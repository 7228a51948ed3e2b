"""fp64 CPU oracle for the LV-XAttn single-worker compute path (ctypes front end).

TEST INFRASTRUCTURE ONLY: imported by tests/, by ``__graft_entry__.smoke()`` and
by the ``cpu_baseline`` leg of ``bench.py``.  The product package never imports
this module and this module never imports the product package.

All the arithmetic lives in ``lvx_oracle.c`` (plain C, double precision); this
file only builds that C file with gcc, loads it, and marshals numpy arrays.
Inputs are float32 arrays holding values already rounded to the workload's
storage type; every result is float64.

Functions follow the paper as stated in the header of ``lvx_oracle.c``:
the attention definition of Section 2, the Rescale step of Algorithm 1, the
derivative of the definition (Table 1 counts its FLOPs, Section 3.2 names
what is saved for it), and the projections x W_Q, y W_K, y W_V of Section 2
that Section 3.2 recomputes in the backward pass, with the chain rule through
them (gradients of the weights and of the tokens).
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "lvx_oracle.c")
_LIB = os.path.join(_HERE, "liblvx_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile lvx_oracle.c with gcc (OpenMP) into liblvx_oracle.so next to it."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-march=x86-64-v3", "-fopenmp", "-fPIC", "-shared", "-std=c11",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


class _Problem(C.Structure):
    _fields_ = [("B", C.c_int), ("Hq", C.c_int), ("Hkv", C.c_int), ("Sq", C.c_int),
                ("Skv", C.c_int), ("D", C.c_int), ("scale", C.c_double),
                ("allow", C.c_void_p), ("q_chunk", C.c_int), ("kv_block", C.c_int),
                ("n_q_chunks", C.c_int), ("n_kv_blocks", C.c_int), ("mask_sb", C.c_long)]


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = C.CDLL(_LIB)
        _lib.lvx_oracle_threads.restype = C.c_int
    return _lib


def threads() -> int:
    """Number of OpenMP threads the oracle will use."""
    return int(_load().lvx_oracle_threads())


@dataclass
class Mask:
    """allow[b or 0][i // q_chunk][j // kv_block] != 0  <=>  query i may attend key j."""
    allow: np.ndarray            # uint8, [n_q_chunks, n_kv_blocks] or [B, n_q_chunks, n_kv_blocks]
    q_chunk: int
    kv_block: int


def _f32(a) -> np.ndarray:
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a


def _ptr(a: np.ndarray):
    return a.ctypes.data_as(C.c_void_p)


def _problem(q, k, scale, mask: Optional[Mask]):
    B, Hq, Sq, D = q.shape
    Bk, Hkv, Skv, Dk = k.shape
    assert Bk == B and Dk == D and Hq % Hkv == 0
    p = _Problem()
    p.B, p.Hq, p.Hkv, p.Sq, p.Skv, p.D = B, Hq, Hkv, Sq, Skv, D
    p.scale = float(1.0 / np.sqrt(D)) if scale is None else float(scale)
    keep = None
    if mask is not None:
        a = np.ascontiguousarray(mask.allow, dtype=np.uint8)
        if a.ndim == 2:
            a = a[None]
            p.mask_sb = 0
        else:
            assert a.shape[0] == B
            p.mask_sb = a.shape[1] * a.shape[2]
        assert a.shape[1] * mask.q_chunk >= Sq and a.shape[2] * mask.kv_block >= Skv
        p.allow = a.ctypes.data
        p.q_chunk, p.kv_block = int(mask.q_chunk), int(mask.kv_block)
        p.n_q_chunks, p.n_kv_blocks = a.shape[1], a.shape[2]
        keep = a
    else:
        p.allow = None
    return p, keep


def prob_row(q, k, b, hq, i, scale=None, mask=None) -> np.ndarray:
    """Softmax probabilities of one query row over all keys."""
    q, k = _f32(q), _f32(k)
    p, keep = _problem(q, k, scale, mask)
    out = np.empty(k.shape[2], dtype=np.float64)
    _load().lvx_oracle_prob_row(C.byref(p), _ptr(q), _ptr(k), C.c_int(b), C.c_int(hq), C.c_int(i),
                                _ptr(out))
    return out


def fwd(q, k, v, scale=None, mask=None):
    """O [B,Hq,Sq,D] and L [B,Hq,Sq] by the attention definition."""
    q, k, v = _f32(q), _f32(k), _f32(v)
    p, keep = _problem(q, k, scale, mask)
    O = np.empty(q.shape, dtype=np.float64)
    L = np.empty(q.shape[:3], dtype=np.float64)
    _load().lvx_oracle_fwd(C.byref(p), _ptr(q), _ptr(k), _ptr(v), _ptr(O), _ptr(L))
    return O, L


def fwd_rows(q, k, v, rows, scale=None, mask=None):
    """Forward for sampled query rows; rows is [n,3] of (b, hq, i)."""
    q, k, v = _f32(q), _f32(k), _f32(v)
    rows = np.ascontiguousarray(rows, dtype=np.int32).reshape(-1, 3)
    p, keep = _problem(q, k, scale, mask)
    O = np.empty((rows.shape[0], q.shape[3]), dtype=np.float64)
    L = np.empty(rows.shape[0], dtype=np.float64)
    _load().lvx_oracle_fwd_rows(C.byref(p), _ptr(q), _ptr(k), _ptr(v), C.c_int(rows.shape[0]),
                                _ptr(rows), _ptr(O), _ptr(L))
    return O, L


def merge(O_parts, L_parts):
    """Rescale of Algorithm 1 over n parts: O_parts [n, ..., D], L_parts [n, ...]."""
    O_parts = np.ascontiguousarray(O_parts, dtype=np.float64)
    L_parts = np.ascontiguousarray(L_parts, dtype=np.float64)
    n = O_parts.shape[0]
    D = O_parts.shape[-1]
    assert L_parts.shape == O_parts.shape[:-1]
    rows = int(np.prod(L_parts.shape[1:], dtype=np.int64))
    O = np.empty(O_parts.shape[1:], dtype=np.float64)
    L = np.empty(L_parts.shape[1:], dtype=np.float64)
    _load().lvx_oracle_merge(C.c_int(n), C.c_long(rows), C.c_int(D), _ptr(O_parts), _ptr(L_parts),
                             _ptr(O), _ptr(L))
    return O, L


def bwd(q, k, v, dO, scale=None, mask=None):
    """dQ, dK, dV of loss = sum(O * dO), naive, through the explicit softmax Jacobian."""
    q, k, v, dO = _f32(q), _f32(k), _f32(v), _f32(dO)
    p, keep = _problem(q, k, scale, mask)
    dQ = np.empty(q.shape, dtype=np.float64)
    dK = np.empty(k.shape, dtype=np.float64)
    dV = np.empty(k.shape, dtype=np.float64)
    _load().lvx_oracle_bwd(C.byref(p), _ptr(q), _ptr(k), _ptr(v), _ptr(dO), _ptr(dQ), _ptr(dK),
                           _ptr(dV))
    return dQ, dK, dV


def bwd_q_rows(q, k, v, dO, rows, scale=None, mask=None):
    """dQ for sampled query rows; rows is [n,3] of (b, hq, i)."""
    q, k, v, dO = _f32(q), _f32(k), _f32(v), _f32(dO)
    rows = np.ascontiguousarray(rows, dtype=np.int32).reshape(-1, 3)
    p, keep = _problem(q, k, scale, mask)
    dQ = np.empty((rows.shape[0], q.shape[3]), dtype=np.float64)
    _load().lvx_oracle_bwd_q_rows(C.byref(p), _ptr(q), _ptr(k), _ptr(v), _ptr(dO),
                                  C.c_int(rows.shape[0]), _ptr(rows), _ptr(dQ))
    return dQ


def bwd_kv_rows(q, k, v, dO, rows, scale=None, mask=None):
    """dK, dV for sampled key rows; rows is [n,3] of (b, hkv, j)."""
    q, k, v, dO = _f32(q), _f32(k), _f32(v), _f32(dO)
    rows = np.ascontiguousarray(rows, dtype=np.int32).reshape(-1, 3)
    p, keep = _problem(q, k, scale, mask)
    dK = np.empty((rows.shape[0], q.shape[3]), dtype=np.float64)
    dV = np.empty((rows.shape[0], q.shape[3]), dtype=np.float64)
    _load().lvx_oracle_bwd_kv_rows(C.byref(p), _ptr(q), _ptr(k), _ptr(v), _ptr(dO),
                                   C.c_int(rows.shape[0]), _ptr(rows), _ptr(dK), _ptr(dV))
    return dK, dV


def bwd_block(q, k, v, dO, O, L, kv0, kv1, scale=None, mask=None):
    """One worker's backward step for key rows [kv0,kv1) given the final O and L.

    Returns (dQ addend [B,Hq,Sq,D], dK [B,Hkv,kv1-kv0,D], dV likewise)."""
    q, k, v, dO = _f32(q), _f32(k), _f32(v), _f32(dO)
    O = np.ascontiguousarray(O, dtype=np.float64)
    L = np.ascontiguousarray(L, dtype=np.float64)
    p, keep = _problem(q, k, scale, mask)
    nb = kv1 - kv0
    dQ = np.empty(q.shape, dtype=np.float64)
    dK = np.empty((k.shape[0], k.shape[1], nb, k.shape[3]), dtype=np.float64)
    dV = np.empty_like(dK)
    _load().lvx_oracle_bwd_block(C.byref(p), _ptr(q), _ptr(k), _ptr(v), _ptr(dO), _ptr(O), _ptr(L),
                                 C.c_int(kv0), C.c_int(kv1), _ptr(dQ), _ptr(dK), _ptr(dV))
    return dQ, dK, dV


def project(x, w, n_heads: int, rows=None) -> np.ndarray:
    """The projection of Section 2 cut into heads: x [B,S,E], w [n_heads*D, E] (the transposed
    projection matrix, one row per output column) -> [B, n_heads, S, D]; with rows ([n,2] of
    (b, s)) only those tokens, [n, n_heads, D]."""
    x, w = _f32(x), _f32(w)
    B, S, E = x.shape
    N, Ew = w.shape
    assert Ew == E and N % n_heads == 0
    D = N // n_heads
    if rows is None:
        out = np.empty((B, n_heads, S, D), dtype=np.float64)
        _load().lvx_oracle_project(C.c_int(B), C.c_int(S), C.c_int(E), C.c_int(n_heads), C.c_int(D),
                                   _ptr(x), _ptr(w), C.c_int(0), None, _ptr(out))
        return out
    rows = np.ascontiguousarray(rows, dtype=np.int32).reshape(-1, 2)
    out = np.empty((rows.shape[0], n_heads, D), dtype=np.float64)
    _load().lvx_oracle_project(C.c_int(B), C.c_int(S), C.c_int(E), C.c_int(n_heads), C.c_int(D),
                               _ptr(x), _ptr(w), C.c_int(rows.shape[0]), _ptr(rows), _ptr(out))
    return out


def project_bwd(x, w, g, n_heads: int, cols=None, rows=None):
    """The chain rule through project (Section 2's linear maps, which Section 3.2 evaluates again
    in the backward pass): x [B,S,E], w [n_heads*D, E], g = d loss / d out [B, n_heads, S, D] ->
    (dw [n_heads*D, E], dx [B,S,E]).  With cols (output columns h*D + c) only those rows of dw,
    [n, E]; with rows ([n,2] of (b, s)) only those tokens of dx, [n, E]."""
    x, w, g = _f32(x), _f32(w), _f32(g)
    B, S, E = x.shape
    N, Ew = w.shape
    assert Ew == E and N % n_heads == 0
    D = N // n_heads
    assert g.shape == (B, n_heads, S, D)
    dims = (C.c_int(B), C.c_int(S), C.c_int(E), C.c_int(n_heads), C.c_int(D))
    if cols is None:
        dw = np.empty((N, E), dtype=np.float64)
        _load().lvx_oracle_project_bwd_w(*dims, _ptr(x), _ptr(g), C.c_int(0), None, _ptr(dw))
    else:
        cols = np.ascontiguousarray(cols, dtype=np.int32).reshape(-1)
        assert cols.size == 0 or (cols.min() >= 0 and cols.max() < N)
        dw = np.empty((cols.size, E), dtype=np.float64)
        _load().lvx_oracle_project_bwd_w(*dims, _ptr(x), _ptr(g), C.c_int(cols.size), _ptr(cols), _ptr(dw))
    if rows is None:
        dx = np.empty((B, S, E), dtype=np.float64)
        _load().lvx_oracle_project_bwd_x(*dims, _ptr(w), _ptr(g), C.c_int(0), None, _ptr(dx))
    else:
        rows = np.ascontiguousarray(rows, dtype=np.int32).reshape(-1, 2)
        dx = np.empty((rows.shape[0], E), dtype=np.float64)
        _load().lvx_oracle_project_bwd_x(*dims, _ptr(w), _ptr(g), C.c_int(rows.shape[0]), _ptr(rows), _ptr(dx))
    return dw, dx
