"""Host-side checks that need no GPU: the C-ABI library loads, exports every function that
include/lvx.h declares, rejects bad arguments before launching anything, and sizes workspaces."""
import ctypes as C
import os
import re

import pytest

from paper_2502_02406_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(B.LIB_PATH):
        from paper_2502_02406_amd import build
        build.build()
    return B.load()


def declared_functions():
    text = open(os.path.join(ROOT, "include", "lvx.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(lvx_[a-z_]+)\s*\(", text)))


def test_header_functions_are_exported(lib):
    names = declared_functions()
    assert {"lvx_xattn_fwd", "lvx_xattn_merge", "lvx_xattn_bwd"} <= set(names)
    for n in names:
        assert hasattr(lib, n), f"{n} declared in lvx.h but not exported"
    assert set(B.EXPORTS) == set(names)


def problem(**kw):
    p = B.lvx_problem()
    d = dict(B=1, Hq=4, Hkv=2, Sq=100, Skv=1000, D=128)
    d.update(kw)
    for k, v in d.items():
        setattr(p, k, v)
    p.q_ss, p.q_sh, p.q_sb = p.D, p.Sq * p.D, p.Hq * p.Sq * p.D
    p.kv_ss, p.kv_sh, p.kv_sb = p.D, p.Skv * p.D, p.Hkv * p.Skv * p.D
    for k, v in kw.items():
        if k.endswith(("_ss", "_sh", "_sb")):
            setattr(p, k, v)
    return p


FAKE = 0x1000      # non-null, 256-byte aligned; never dereferenced because validation fails first


def fwd(lib, p, dtype=B.LVX_BF16, q=FAKE, k=FAKE, v=FAKE, mask=None, o=FAKE, o_dtype=None, lse=FAKE,
        ws=FAKE, ws_bytes=1 << 40):
    return lib.lvx_xattn_fwd(C.byref(p) if p is not None else None, dtype, q, k, v, mask, o,
                             dtype if o_dtype is None else o_dtype, lse, ws, ws_bytes, None)


def test_fwd_argument_errors(lib):
    assert fwd(lib, None) == -1
    assert fwd(lib, problem(), q=None) == -1
    assert fwd(lib, problem(), lse=None) == -1
    assert fwd(lib, problem(Sq=0)) == -2
    assert fwd(lib, problem(Hq=3)) == -2                       # Hq % Hkv != 0
    assert fwd(lib, problem(), dtype=7) == -3
    assert fwd(lib, problem(), dtype=B.LVX_F32, o_dtype=B.LVX_BF16) == -3
    assert fwd(lib, problem(D=80)) == -7
    assert fwd(lib, problem(kv_ss=64)) == -4                   # row stride smaller than D
    assert fwd(lib, problem(kv_ss=132)) == -4                  # breaks 16-byte row alignment
    assert fwd(lib, problem(), k=FAKE + 2) == -4               # misaligned pointer
    assert fwd(lib, problem(), ws=None) == -6
    assert fwd(lib, problem(), ws=FAKE + 16) == -6
    assert fwd(lib, problem(), ws_bytes=8) == -6


def test_mask_errors(lib):
    m = B.lvx_mask()
    m.allow, m.q_chunk, m.kv_block, m.n_q_chunks, m.n_kv_blocks = FAKE, 32, 256, 4, 4
    m.stride_q, m.stride_b = 4, 0
    assert fwd(lib, problem(Sq=129), mask=C.byref(m)) == -5    # 4 chunks * 32 < 129 rows
    assert fwd(lib, problem(Skv=1025), mask=C.byref(m)) == -5
    m.stride_q = 2
    assert fwd(lib, problem(), mask=C.byref(m)) == -5
    m.stride_q, m.allow = 4, None
    assert fwd(lib, problem(), mask=C.byref(m)) == -1
    m.allow, m.q_chunk = FAKE, 0
    assert fwd(lib, problem(), mask=C.byref(m)) == -5


def test_merge_and_bwd_errors(lib):
    arr = (C.c_void_p * 2)(FAKE, FAKE)
    one = (C.c_void_p * 2)(FAKE, None)
    assert lib.lvx_xattn_merge(1, 2, 8, 128, 2, arr, arr, 0, None, 0, FAKE, None) == -1
    assert lib.lvx_xattn_merge(1, 2, 8, 128, 2, one, arr, 0, FAKE, 0, FAKE, None) == -1
    assert lib.lvx_xattn_merge(1, 2, 8, 128, 0, arr, arr, 0, FAKE, 0, FAKE, None) == -2
    assert lib.lvx_xattn_merge(1, 2, 8, 128, 65, arr, arr, 0, FAKE, 0, FAKE, None) == -2
    assert lib.lvx_xattn_merge(1, 2, 8, 80, 2, arr, arr, 0, FAKE, 0, FAKE, None) == -7
    assert lib.lvx_xattn_merge(1, 2, 8, 128, 2, arr, arr, 5, FAKE, 0, FAKE, None) == -3
    p = problem()
    args = [C.byref(p), B.LVX_BF16] + [FAKE] * 6 + [None, FAKE, FAKE, FAKE, FAKE, 1 << 40, None]
    bad = list(args); bad[9] = None                              # dq_accum
    assert lib.lvx_xattn_bwd(*bad) == -1
    bad = list(args); bad[13] = 16                               # workspace too small
    assert lib.lvx_xattn_bwd(*bad) == -6
    assert lib.lvx_xattn_bwd_stages(*args, 0) == -2
    assert lib.lvx_xattn_bwd_stages(*args, 8) == -2          # a kernel choice without a stage
    assert lib.lvx_xattn_bwd_stages(*args, 32 | 7) == -2     # unknown bit
    assert lib.lvx_xattn_bwd_stages(*args, 7 | 8 | 16) == -2  # both kernel choices
    assert lib.lvx_xattn_dq_finalize(C.byref(p), None, FAKE, B.LVX_BF16, None) == -1


def test_fwd_merge_errors(lib):
    p = problem()
    args = [C.byref(p), B.LVX_BF16, FAKE, FAKE, FAKE, None, FAKE, FAKE, FAKE, 1 << 40, None]
    bad = list(args); bad[6] = None                              # o_acc
    assert lib.lvx_xattn_fwd_merge(*bad) == -1
    bad = list(args); bad[7] = None                              # lse_acc
    assert lib.lvx_xattn_fwd_merge(*bad) == -1
    bad = list(args); bad[9] = 16                                # workspace too small
    assert lib.lvx_xattn_fwd_merge(*bad) == -6
    bad = list(args); bad[2] = FAKE + 4                          # misaligned q
    assert lib.lvx_xattn_fwd_merge(*bad) == -4
    strided = problem()
    strided.q_ss = 2 * strided.D                                 # float32 kernels need a contiguous Q here
    assert lib.lvx_xattn_fwd_merge(C.byref(strided), B.LVX_F32, *args[2:]) == -4
    assert lib.lvx_xattn_fwd_merge(C.byref(problem(D=80)), B.LVX_BF16, *args[2:]) == -7
    n = B.lvx_xattn_workspace_bytes(p, B.LVX_F32, B.LVX_WS_FWD_MERGE)
    assert n >= p.B * p.Hq * p.Sq * (p.D + 1) * 4                # one float32 partial result and its L
    assert B.lvx_xattn_workspace_bytes(p, B.LVX_BF16, B.LVX_WS_FWD_MERGE) >= 256


def test_project_errors(lib):
    p = B.lvx_projection()
    p.B, p.S, p.E, p.H, p.D = 1, 100, 256, 2, 128
    p.x_ss, p.x_sb = p.E, p.S * p.E
    outs = (C.c_void_p * 2)(FAKE, FAKE)
    one = (C.c_void_p * 2)(FAKE, None)

    def call(pp=p, dtype=B.LVX_BF16, x=FAKE, w=FAKE, n_out=2, out=outs):
        return lib.lvx_xattn_project(C.byref(pp) if pp is not None else None, dtype, x, w, n_out, out, None)

    assert call(pp=None) == -1
    assert call(x=None) == -1
    assert call(out=one) == -1
    assert call(n_out=3) == -2
    assert call(dtype=5) == -3
    assert call(x=FAKE + 2) == -4
    bad = B.lvx_projection.from_buffer_copy(p); bad.S = 0
    assert call(pp=bad) == -2
    bad = B.lvx_projection.from_buffer_copy(p); bad.x_ss = p.E - 8
    assert call(pp=bad) == -4
    bad = B.lvx_projection.from_buffer_copy(p); bad.x_sb = p.S * p.E + 64     # batches must follow each other
    assert call(pp=bad) == -4
    bad = B.lvx_projection.from_buffer_copy(p); bad.E = 96; bad.x_ss = 96; bad.x_sb = 96 * p.S
    assert call(pp=bad) == -7                                                 # E % 64 != 0 on the matrix cores
    bad = B.lvx_projection.from_buffer_copy(p); bad.D = 64                    # 2 * 2 * 64 = 256 columns, heads of 64: fine shape-wise ...
    assert call(pp=bad, n_out=1) == -7                                        # ... but one output of 128 columns is not a tile


def test_project_bwd_errors(lib):
    p = B.lvx_projection()
    p.B, p.S, p.E, p.H, p.D = 1, 100, 256, 2, 128
    p.x_ss, p.x_sb = p.E, p.S * p.E
    gs = (C.c_void_p * 2)(FAKE, FAKE)
    one = (C.c_void_p * 2)(FAKE, None)

    def call(pp=p, dtype=B.LVX_BF16, x=FAKE, w=FAKE, n_out=2, g=gs, dx=FAKE, dw=FAKE):
        return lib.lvx_xattn_project_bwd(C.byref(pp) if pp is not None else None, dtype, x, w, n_out, g,
                                         dx, dw, None)

    assert call(pp=None) == -1
    assert call(w=None) == -1
    assert call(g=one) == -1
    assert call(dx=None, dw=None) == -1            # nothing asked for
    assert call(n_out=0) == -2
    assert call(dtype=5) == -3
    assert call(dw=FAKE + 4) == -4
    assert call(dx=FAKE + 2) == -4
    bad = B.lvx_projection.from_buffer_copy(p); bad.H = 0
    assert call(pp=bad) == -2
    bad = B.lvx_projection.from_buffer_copy(p); bad.x_sb = p.S * p.E + 64
    assert call(pp=bad) == -4


def test_workspace_sizes_and_strerror(lib):
    p = problem(B=1, Hq=32, Hkv=8, Sq=2048, Skv=32768)
    rows = 32 * 2048
    # delta + 2 padded stats, + the dQ kernel's partial sums for the most it may split this problem
    # (a masked call on 256 compute units, the count assumed without a device: 4 splits)
    # + for the fused kernel (dense, D = 128): dQ tiles of 32 rows x 128 float32, a lock word per tile
    # (rounded up to 256 bytes) and 256 bytes that hold the error word
    ws_bwd = B.lvx_xattn_workspace_bytes(p, B.LVX_BF16, B.LVX_WS_BWD)
    tiles = 32 * (2048 // 32)
    fused = tiles * 32 * 128 * 4 + (tiles * 4 + 255) // 256 * 256 + 256
    assert ws_bwd >= 3 * rows * 4 + fused and (ws_bwd - 3 * rows * 4 - fused) % (rows * 128 * 4) == 0
    # 64-wide heads use the two-kernel backward: no tiles
    p64 = problem(B=1, Hq=32, Hkv=8, Sq=2048, Skv=32768, D=64)
    assert (B.lvx_xattn_workspace_bytes(p64, B.LVX_BF16, B.LVX_WS_BWD) - 3 * rows * 4) % (rows * 64 * 4) == 0
    assert B.lvx_xattn_workspace_bytes(p, B.LVX_F32, B.LVX_WS_BWD) == 3 * rows * 4
    assert B.lvx_xattn_workspace_bytes(p, B.LVX_BF16, B.LVX_WS_FWD) >= 256
    assert B.lvx_xattn_workspace_bytes(p, B.LVX_F32, B.LVX_WS_FWD) == 256
    assert B.lvx_xattn_workspace_bytes(problem(D=80), B.LVX_BF16, B.LVX_WS_FWD) == 0
    assert B.lvx_xattn_workspace_bytes(p, B.LVX_BF16, 9) == 0
    small = problem(B=1, Hq=2, Hkv=2, Sq=64, Skv=1 << 20)       # few query tiles: split-KV
    n = B.lvx_xattn_workspace_bytes(small, B.LVX_BF16, B.LVX_WS_FWD)
    assert n > 2 * 64 * 128 * 4 and n % 256 == 0
    assert B.strerror(0) == "ok"
    for code in range(-8, 0):
        assert B.strerror(code) not in ("ok", "unknown status")
    assert B.strerror(-99) == "unknown status"


def test_binding_refuses_cpu_tensors():
    import torch
    if torch.cuda.is_available():
        pytest.skip("host-only check")
    q = torch.zeros(1, 2, 8, 128, dtype=torch.bfloat16)
    p = B.make_problem(q, q)
    with pytest.raises(RuntimeError):
        B.lvx_xattn_fwd(p, q, q, q, None, q, torch.zeros(1, 2, 8), torch.zeros(256, dtype=torch.uint8))
    from paper_2502_02406_amd.blockloop import BlockLoop
    with pytest.raises(RuntimeError):
        BlockLoop((1, 2, 8, 128), (1, 2, 64, 128), torch.bfloat16)


def test_static_scratch_forward_refuses_what_does_not_fit(lib):
    """lvx_xattn_fwd_static turns down, before any HIP call, a problem whose split-KV partial results
    exceed its fixed array; bad arguments get the same codes as from lvx_xattn_fwd."""
    p = problem(Hq=64, Hkv=8, Sq=700, Skv=1 << 20)
    assert B.lvx_xattn_workspace_bytes(p, B.LVX_BF16, B.LVX_WS_FWD) > B.LVX_STATIC_SCRATCH_BYTES
    call = lambda pp, q=FAKE: lib.lvx_xattn_fwd_static(C.byref(pp), B.LVX_BF16, q, FAKE, FAKE, None, FAKE,
                                                       B.LVX_BF16, FAKE, None)
    assert call(p) == -6
    text = open(os.path.join(ROOT, "include", "lvx.h")).read()
    assert re.search(r"LVX_STATIC_SCRATCH_BYTES\s*=\s*64\s*<<\s*20", text) and B.LVX_STATIC_SCRATCH_BYTES == 64 << 20
