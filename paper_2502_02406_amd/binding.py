"""Thin ctypes binding of liblvx.so (include/lvx.h).  Argument marshalling only.

PyTorch is used for device memory and streams; every step of the attention path runs in the
HIP kernels behind the C ABI.  There is no CPU fallback: if the library is missing or no GPU
is present the calls raise.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
# (LVX_LIB: another build of the same library, e.g. one with measurement switches compiled in)
LIB_PATH = os.environ.get("LVX_LIB") or os.path.join(_HERE, "liblvx.so")

LVX_F32, LVX_BF16 = 0, 1
LVX_WS_FWD, LVX_WS_BWD, LVX_WS_FWD_MERGE = 0, 1, 2
LVX_MAX_PARTS = 64

LVX_BWD_DELTA, LVX_BWD_DKDV, LVX_BWD_DQ, LVX_BWD_ALL = 1, 2, 4, 7
LVX_BWD_FUSED, LVX_BWD_SPLIT = 8, 16

LVX_STATIC_SCRATCH_BYTES = 64 << 20

EXPORTS = ("lvx_xattn_workspace_bytes", "lvx_xattn_fwd", "lvx_xattn_fwd_static", "lvx_xattn_fwd_merge", "lvx_xattn_merge", "lvx_xattn_bwd",
           "lvx_xattn_bwd_stages", "lvx_xattn_bwd_error_word", "lvx_xattn_dq_finalize", "lvx_xattn_project", "lvx_xattn_project_bwd", "lvx_strerror")


class LvxError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {strerror(code)} (status {code})")


class lvx_problem(C.Structure):
    _fields_ = [("B", C.c_int32), ("Hq", C.c_int32), ("Hkv", C.c_int32), ("Sq", C.c_int32),
                ("Skv", C.c_int32), ("D", C.c_int32),
                ("q_sb", C.c_int64), ("q_sh", C.c_int64), ("q_ss", C.c_int64),
                ("kv_sb", C.c_int64), ("kv_sh", C.c_int64), ("kv_ss", C.c_int64),
                ("softmax_scale", C.c_float)]


class lvx_mask(C.Structure):
    _fields_ = [("allow", C.c_void_p), ("q_chunk", C.c_int32), ("kv_block", C.c_int32),
                ("n_q_chunks", C.c_int32), ("n_kv_blocks", C.c_int32),
                ("stride_b", C.c_int64), ("stride_q", C.c_int64)]


class lvx_projection(C.Structure):
    _fields_ = [("B", C.c_int32), ("S", C.c_int32), ("E", C.c_int32), ("H", C.c_int32),
                ("D", C.c_int32), ("x_sb", C.c_int64), ("x_ss", C.c_int64)]


_lib = None


def load() -> C.CDLL:
    """Load liblvx.so (built by paper_2502_02406_amd.build); raises if it is not there."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} not found: build it with `python -m paper_2502_02406_amd.build`")
        lib = C.CDLL(LIB_PATH)
        lib.lvx_xattn_workspace_bytes.restype = C.c_size_t
        lib.lvx_xattn_workspace_bytes.argtypes = [C.POINTER(lvx_problem), C.c_int, C.c_int]
        lib.lvx_xattn_fwd.restype = C.c_int
        lib.lvx_xattn_fwd.argtypes = [C.POINTER(lvx_problem), C.c_int, C.c_void_p, C.c_void_p,
                                      C.c_void_p, C.POINTER(lvx_mask), C.c_void_p, C.c_int,
                                      C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        lib.lvx_xattn_fwd_static.restype = C.c_int
        lib.lvx_xattn_fwd_static.argtypes = lib.lvx_xattn_fwd.argtypes[:9] + [C.c_void_p]
        lib.lvx_xattn_fwd_merge.restype = C.c_int
        lib.lvx_xattn_fwd_merge.argtypes = [C.POINTER(lvx_problem), C.c_int, C.c_void_p, C.c_void_p,
                                            C.c_void_p, C.POINTER(lvx_mask), C.c_void_p, C.c_void_p,
                                            C.c_void_p, C.c_size_t, C.c_void_p]
        lib.lvx_xattn_merge.restype = C.c_int
        lib.lvx_xattn_merge.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_int32,
                                        C.POINTER(C.c_void_p), C.POINTER(C.c_void_p), C.c_int,
                                        C.c_void_p, C.c_int, C.c_void_p, C.c_void_p]
        lib.lvx_xattn_bwd.restype = C.c_int
        lib.lvx_xattn_bwd.argtypes = [C.POINTER(lvx_problem), C.c_int, C.c_void_p, C.c_void_p,
                                      C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                      C.POINTER(lvx_mask), C.c_void_p, C.c_void_p, C.c_void_p,
                                      C.c_void_p, C.c_size_t, C.c_void_p]
        lib.lvx_xattn_bwd_stages.restype = C.c_int
        lib.lvx_xattn_bwd_stages.argtypes = lib.lvx_xattn_bwd.argtypes + [C.c_uint]
        lib.lvx_xattn_bwd_error_word.restype = C.c_int
        lib.lvx_xattn_bwd_error_word.argtypes = [C.POINTER(lvx_problem), C.c_int, C.POINTER(lvx_mask), C.c_void_p,
                                                 C.c_size_t, C.POINTER(C.c_void_p)]
        lib.lvx_xattn_dq_finalize.restype = C.c_int
        lib.lvx_xattn_dq_finalize.argtypes = [C.POINTER(lvx_problem), C.c_void_p, C.c_void_p,
                                              C.c_int, C.c_void_p]
        lib.lvx_xattn_project.restype = C.c_int
        lib.lvx_xattn_project.argtypes = [C.POINTER(lvx_projection), C.c_int, C.c_void_p, C.c_void_p,
                                          C.c_int, C.POINTER(C.c_void_p), C.c_void_p]
        lib.lvx_xattn_project_bwd.restype = C.c_int
        lib.lvx_xattn_project_bwd.argtypes = [C.POINTER(lvx_projection), C.c_int, C.c_void_p, C.c_void_p,
                                              C.c_int, C.POINTER(C.c_void_p), C.c_void_p, C.c_void_p,
                                              C.c_void_p]
        lib.lvx_strerror.restype = C.c_char_p
        lib.lvx_strerror.argtypes = [C.c_int]
        _lib = lib
    return _lib


def strerror(code: int) -> str:
    return load().lvx_strerror(int(code)).decode()


def dtype_code(dt: torch.dtype) -> int:
    if dt == torch.float32:
        return LVX_F32
    if dt == torch.bfloat16:
        return LVX_BF16
    raise TypeError(f"unsupported dtype {dt}")


def _stream() -> int:
    return int(torch.cuda.current_stream().cuda_stream)


def make_problem(q: torch.Tensor, k: torch.Tensor, softmax_scale: float = 0.0) -> lvx_problem:
    """Shape and strides of Q [B,Hq,Sq,D] and K [B,Hkv,Skv,D] (K may be a strided view)."""
    assert q.dim() == 4 and k.dim() == 4 and q.stride(3) == 1 and k.stride(3) == 1
    p = lvx_problem()
    p.B, p.Hq, p.Sq, p.D = q.shape
    p.Hkv, p.Skv = k.shape[1], k.shape[2]
    p.q_sb, p.q_sh, p.q_ss = q.stride(0), q.stride(1), q.stride(2)
    p.kv_sb, p.kv_sh, p.kv_ss = k.stride(0), k.stride(1), k.stride(2)
    p.softmax_scale = float(softmax_scale)
    return p


def make_mask(allow: torch.Tensor, q_chunk: int, kv_block: int, kv_block0: int = 0,
              n_kv_blocks: Optional[int] = None) -> lvx_mask:
    """allow: uint8 device tensor [n_q_chunks, n_kv_blocks_total] or [B, ...]; kv_block0 offsets
    the bitmap columns for a K/V block that starts at key kv_block0 * kv_block."""
    assert allow.dtype == torch.uint8 and allow.is_cuda and allow.stride(-1) == 1
    m = lvx_mask()
    m.allow = allow.data_ptr() + kv_block0
    m.q_chunk, m.kv_block = int(q_chunk), int(kv_block)
    m.n_q_chunks = allow.shape[-2]
    m.n_kv_blocks = (allow.shape[-1] - kv_block0) if n_kv_blocks is None else int(n_kv_blocks)
    m.stride_q = allow.stride(-2)
    m.stride_b = allow.stride(0) if allow.dim() == 3 else 0
    return m


def lvx_xattn_workspace_bytes(p: lvx_problem, dtype: int, which: int) -> int:
    return int(load().lvx_xattn_workspace_bytes(C.byref(p), dtype, which))


def _check(code: int, where: str) -> None:
    if code != 0:
        raise LvxError(code, where)


def lvx_xattn_fwd(p: lvx_problem, q, k, v, mask: Optional[lvx_mask], o, lse, workspace) -> None:
    """o (dtype of q, or float32) and lse (float32 [B,Hq,Sq]) are overwritten."""
    if not q.is_cuda:
        raise RuntimeError("lvx_xattn_fwd needs device tensors")
    code = load().lvx_xattn_fwd(C.byref(p), dtype_code(q.dtype), q.data_ptr(), k.data_ptr(),
                                v.data_ptr(), C.byref(mask) if mask is not None else None,
                                o.data_ptr(), dtype_code(o.dtype), lse.data_ptr(),
                                workspace.data_ptr(), workspace.numel() * workspace.element_size(),
                                _stream())
    _check(code, "lvx_xattn_fwd")


def lvx_xattn_fwd_static(p: lvx_problem, q, k, v, mask: Optional[lvx_mask], o, lse) -> None:
    """lvx_xattn_fwd without a workspace: scratch is the library's own fixed device array."""
    if not q.is_cuda:
        raise RuntimeError("lvx_xattn_fwd_static needs device tensors")
    code = load().lvx_xattn_fwd_static(C.byref(p), dtype_code(q.dtype), q.data_ptr(), k.data_ptr(),
                                       v.data_ptr(), C.byref(mask) if mask is not None else None,
                                       o.data_ptr(), dtype_code(o.dtype), lse.data_ptr(), _stream())
    _check(code, "lvx_xattn_fwd_static")


def lvx_xattn_fwd_merge(p: lvx_problem, q, k, v, mask: Optional[lvx_mask], o_acc, lse_acc, workspace) -> None:
    """One visit merged into the running result: o_acc (float32, contiguous [B,Hq,Sq,D]) and
    lse_acc (float32 [B,Hq,Sq]) are updated in place."""
    if not q.is_cuda:
        raise RuntimeError("lvx_xattn_fwd_merge needs device tensors")
    assert o_acc.dtype == torch.float32 and o_acc.is_contiguous() and lse_acc.is_contiguous()
    code = load().lvx_xattn_fwd_merge(C.byref(p), dtype_code(q.dtype), q.data_ptr(), k.data_ptr(),
                                      v.data_ptr(), C.byref(mask) if mask is not None else None,
                                      o_acc.data_ptr(), lse_acc.data_ptr(), workspace.data_ptr(),
                                      workspace.numel() * workspace.element_size(), _stream())
    _check(code, "lvx_xattn_fwd_merge")


def lvx_xattn_merge(o_parts: Sequence[torch.Tensor], lse_parts: Sequence[torch.Tensor],
                    o_out: torch.Tensor, lse_out: torch.Tensor) -> None:
    """Rescale of Algorithm 1 over the given parts (each contiguous [B,Hq,Sq,D] / [B,Hq,Sq])."""
    n = len(o_parts)
    B, Hq, Sq, D = o_out.shape
    if not o_out.is_cuda:
        raise RuntimeError("lvx_xattn_merge needs device tensors")
    for t in list(o_parts) + list(lse_parts) + [o_out, lse_out]:
        assert t.is_contiguous()
    op = (C.c_void_p * max(n, 1))(*[t.data_ptr() for t in o_parts])
    lp = (C.c_void_p * max(n, 1))(*[t.data_ptr() for t in lse_parts])
    code = load().lvx_xattn_merge(B, Hq, Sq, D, n, op, lp, dtype_code(o_parts[0].dtype) if n else 0,
                                  o_out.data_ptr(), dtype_code(o_out.dtype), lse_out.data_ptr(),
                                  _stream())
    _check(code, "lvx_xattn_merge")


def lvx_xattn_bwd(p: lvx_problem, q, k, v, o, lse, d_o, mask: Optional[lvx_mask], dq_accum, dk, dv,
                  workspace, stages: int = LVX_BWD_ALL) -> None:
    """dk/dv (views with K's strides) overwritten; dq_accum (float32, contiguous) accumulated.
    With stages != LVX_BWD_ALL this is lvx_xattn_bwd_stages (a subset of the kernels)."""
    if not q.is_cuda:
        raise RuntimeError("lvx_xattn_bwd needs device tensors")
    assert dq_accum.dtype == torch.float32 and dq_accum.is_contiguous()
    assert dk.stride() == k.stride() and dv.stride() == k.stride()
    assert o.stride() == q.stride() and d_o.stride() == q.stride()
    args = (C.byref(p), dtype_code(q.dtype), q.data_ptr(), k.data_ptr(),
            v.data_ptr(), o.data_ptr(), lse.data_ptr(), d_o.data_ptr(),
            C.byref(mask) if mask is not None else None, dq_accum.data_ptr(),
            dk.data_ptr(), dv.data_ptr(), workspace.data_ptr(),
            workspace.numel() * workspace.element_size(), _stream())
    if stages == LVX_BWD_ALL:
        _check(load().lvx_xattn_bwd(*args), "lvx_xattn_bwd")
    else:
        _check(load().lvx_xattn_bwd_stages(*args, stages), "lvx_xattn_bwd_stages")


def lvx_xattn_bwd_error_word(p: lvx_problem, dtype: int, mask: Optional[lvx_mask], workspace) -> int:
    """Device address (0 if none) of the word that a backward call with these arguments sets when
    it could not finish dQ."""
    out = C.c_void_p()
    code = load().lvx_xattn_bwd_error_word(C.byref(p), dtype, C.byref(mask) if mask is not None else None,
                                           workspace.data_ptr(), workspace.numel() * workspace.element_size(),
                                           C.byref(out))
    _check(code, "lvx_xattn_bwd_error_word")
    return int(out.value or 0)


def lvx_xattn_dq_finalize(p: lvx_problem, dq_accum, dq) -> None:
    code = load().lvx_xattn_dq_finalize(C.byref(p), dq_accum.data_ptr(), dq.data_ptr(),
                                        dtype_code(dq.dtype), _stream())
    _check(code, "lvx_xattn_dq_finalize")


def _token_strides(x):
    """(batch stride, token stride) of x [B, S, E]; with one batch the batch stride means nothing (a
    window of a longer token sequence reports the whole sequence's), so it is set to what the
    entry points ask for: batches that follow each other."""
    return (x.stride(0) if x.shape[0] > 1 else x.shape[1] * x.stride(1)), x.stride(1)


def lvx_xattn_project(x, w, outs) -> None:
    """outs: one or two tensors [B, H, S, D] (contiguous, dtype of x), overwritten with the heads of
    x [B, S, E] times the rows of w [len(outs) * H * D, E]."""
    if not x.is_cuda:
        raise RuntimeError("lvx_xattn_project needs device tensors")
    assert x.dim() == 3 and x.stride(2) == 1 and w.dim() == 2 and w.is_contiguous()
    assert all(o.dim() == 4 and o.is_contiguous() and o.dtype == x.dtype for o in outs) and w.dtype == x.dtype
    p = lvx_projection()
    p.B, p.S, p.E = x.shape
    _, p.H, _, p.D = outs[0].shape
    assert all(tuple(o.shape) == (p.B, p.H, p.S, p.D) for o in outs) and tuple(w.shape) == (len(outs) * p.H * p.D, p.E)
    p.x_sb, p.x_ss = _token_strides(x)
    arr = (C.c_void_p * len(outs))(*[o.data_ptr() for o in outs])
    code = load().lvx_xattn_project(C.byref(p), dtype_code(x.dtype), x.data_ptr(), w.data_ptr(),
                                    len(outs), arr, _stream())
    _check(code, "lvx_xattn_project")


def lvx_xattn_project_bwd(x, w, d_outs, dx=None, dw=None) -> None:
    """d_outs: one or two tensors [B, H, S, D] (contiguous, dtype of x), the gradients of the heads
    that lvx_xattn_project made from x [B, S, E] and w [len(d_outs) * H * D, E].  dx (x's shape,
    strides and dtype) is overwritten with the gradient of x; dw (w's shape, float32) has the
    gradient of w added to it."""
    if not x.is_cuda:
        raise RuntimeError("lvx_xattn_project_bwd needs device tensors")
    assert x.dim() == 3 and x.stride(2) == 1 and w.dim() == 2 and w.is_contiguous() and w.dtype == x.dtype
    assert all(g.dim() == 4 and g.is_contiguous() and g.dtype == x.dtype for g in d_outs)
    assert dx is not None or dw is not None
    p = lvx_projection()
    p.B, p.S, p.E = x.shape
    _, p.H, _, p.D = d_outs[0].shape
    assert all(tuple(g.shape) == (p.B, p.H, p.S, p.D) for g in d_outs)
    assert tuple(w.shape) == (len(d_outs) * p.H * p.D, p.E)
    p.x_sb, p.x_ss = _token_strides(x)
    if dx is not None:
        assert dx.shape == x.shape and dx.stride() == x.stride() and dx.dtype == x.dtype and dx.is_cuda
    if dw is not None:
        assert dw.shape == w.shape and dw.is_contiguous() and dw.dtype == torch.float32 and dw.is_cuda
    arr = (C.c_void_p * len(d_outs))(*[g.data_ptr() for g in d_outs])
    code = load().lvx_xattn_project_bwd(C.byref(p), dtype_code(x.dtype), x.data_ptr(), w.data_ptr(),
                                        len(d_outs), arr, dx.data_ptr() if dx is not None else None,
                                        dw.data_ptr() if dw is not None else None, _stream())
    _check(code, "lvx_xattn_project_bwd")
