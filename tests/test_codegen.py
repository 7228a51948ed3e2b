"""Generated-code checks of the matrix-core kernels (no GPU needed: hipcc cross-compiles).

The kernels write some matrix instructions out by hand so that accumulators and stationary
operands stay in the accumulation register file.  The compiler does not know that those
statements are matrix instructions, so it would not wait for their results before a register move
or a spill of its own.  That is safe only while the steady-state loops of the dense kernels contain
no such move: this test compiles the sources exactly as the build does and looks at the loops."""
import functools
import os
import re
import subprocess
import tempfile

import pytest

from paper_2502_02406_amd import build as B

CSRC = B.CSRC


@functools.lru_cache(maxsize=None)
def _asm(src):
    with tempfile.TemporaryDirectory() as tmp:
        out = os.path.join(tmp, "k.s")
        cmd = [B.HIPCC] + B.FLAGS + B.FILE_FLAGS.get(src, []) + ["--cuda-device-only", "-S",
                                                                   os.path.join(CSRC, src), "-o", out]
        r = subprocess.run(cmd, capture_output=True, text=True, timeout=900)
        assert r.returncode == 0, r.stderr[-2000:]
        return open(out).read()


def _kernel(asm, pattern):
    # (up to the end of the function: an early exit may put an s_endpgm ahead of the loops)
    m = re.search(r"^(_ZN[^\n]*" + pattern + r"[^\n]*):.*?^\.Lfunc_end\d+:", asm, re.S | re.M)
    assert m, f"kernel {pattern} not found"
    return m.group(0)


def _blocks(body):
    """basic blocks: split at labels"""
    return re.split(r"^\.LBB\d+_\d+:.*$", body, flags=re.M)


@pytest.mark.parametrize("src,kernel,loop_mfma", [
    ("lvx_bwd_dkdv_bf16.hip", "bwd_dkdv_bf16_kernelILi128ELb0ELb0E", 128),   # two steps of 64 per trip
    ("lvx_bwd_dkdv_bf16.hip", "bwd_dkdv_bf16_kernelILi128ELb0ELb1E", 128),   # the same loop over a list of steps
    ("lvx_bwd_dq_bf16.hip", "bwd_dq_bf16_kernelILi128ELb0ELi0E", 96),        # one tile = two halves of 48
    ("lvx_bwd_dq_bf16.hip", "bwd_dq_bf16_kernelILi128ELb0ELi1E", 96),        # the same loop over a list of tiles
    ("lvx_bwd_dq_bf16.hip", "bwd_dq_bf16_kernelILi128ELb0ELi2E", 96),        # ... with row blocks that skip tiles
    # the instantiations for 64-wide heads: half the matrix instructions per step or tile
    ("lvx_bwd_dkdv_bf16.hip", "bwd_dkdv_bf16_kernelILi64ELb0ELb0E", 64),
    ("lvx_bwd_dkdv_bf16.hip", "bwd_dkdv_bf16_kernelILi64ELb0ELb1E", 64),
    ("lvx_bwd_dq_bf16.hip", "bwd_dq_bf16_kernelILi64ELb0ELi0E", 48),
    ("lvx_bwd_dq_bf16.hip", "bwd_dq_bf16_kernelILi64ELb0ELi1E", 48),
    # ... and for 96-wide heads: three quarters of them
    ("lvx_bwd_dkdv_bf16.hip", "bwd_dkdv_bf16_kernelILi96ELb0ELb0E", 96),
    ("lvx_bwd_dkdv_bf16.hip", "bwd_dkdv_bf16_kernelILi96ELb0ELb1E", 96),
    ("lvx_bwd_dq_bf16.hip", "bwd_dq_bf16_kernelILi96ELb0ELi0E", 72),
    ("lvx_bwd_dq_bf16.hip", "bwd_dq_bf16_kernelILi96ELb0ELi2E", 72),
    # the fused backward: scoring of one step and contraction of the next in one block
    ("lvx_bwd_fused_bf16.hip", "bwd_fused_bf16_kernelILi128E", 80),
])
def test_dense_loop_moves_no_accumulator(src, kernel, loop_mfma):
    body = _kernel(_asm(src), kernel)
    loops = [b for b in _blocks(body) if b.count("v_mfma_f32_32x32x16_bf16") == loop_mfma]
    assert len(loops) == 1, "steady-state loop not found as one basic block"
    loop = loops[0]
    assert "v_accvgpr" not in loop, "an accumulator or operand leaves the accumulation file inside the loop"
    assert "scratch_" not in loop, "register spill inside the loop"
    # LDS waits must be exact (no tile copy known to the compiler forces them to zero)
    waits = re.findall(r"lgkmcnt\((\d+)\)", loop)
    assert sum(1 for w in waits if w != "0") > len(waits) // 2


def test_general_dkdv_leaves_half_the_accumulation_file():
    asm = _asm("lvx_bwd_dkdv_bf16.hip")
    body = _kernel(asm, "bwd_dkdv_bf16_kernelILi128ELb1ELb0E")
    for blk in _blocks(body):
        if "v_mfma_f32_32x32x16_bf16" in blk:
            assert "v_accvgpr" not in blk, "accumulator moved next to matrix instructions"
    # kernel metadata: ".agpr_count: N" precedes the ".name:" entry of its kernel
    m = re.search(r"\.agpr_count:\s*(\d+)\n(?:(?!\.agpr_count).*\n)*?\s*\.name:\s*\S*bwd_dkdv_bf16_kernelILi128ELb1ELb0E", asm)
    assert m and int(m.group(1)) <= 128


@pytest.mark.parametrize("src,kernel", [
    ("lvx_fwd_bf16.hip", "fwd_bf16_kernelILi128ELi0EE"),
    ("lvx_fwd_bf16.hip", "fwd_bf16_kernelILi128ELi1EE"),     # the same kernel over a list of tiles
    ("lvx_fwd_bf16.hip", "fwd_bf16_kernelILi128ELi2EE"),     # ... with row blocks that skip tiles
    ("lvx_bwd_dq_bf16.hip", "bwd_dq_bf16_kernelILi128ELb1ELi0E"),
    ("lvx_fwd_bf16.hip", "fwd_bf16_kernelILi64ELi0EE"),      # 64-wide heads
    ("lvx_fwd_bf16.hip", "fwd_bf16_kernelILi64ELi1EE"),
    ("lvx_fwd_bf16.hip", "fwd_bf16_kernelILi64ELi2EE"),
    ("lvx_bwd_dq_bf16.hip", "bwd_dq_bf16_kernelILi64ELb1ELi0E"),
    ("lvx_bwd_dkdv_bf16.hip", "bwd_dkdv_bf16_kernelILi64ELb1ELb0E"),
    ("lvx_fwd_bf16.hip", "fwd_bf16_kernelILi96ELi0EE"),      # 96-wide heads
    ("lvx_fwd_bf16.hip", "fwd_bf16_kernelILi96ELi2EE"),
    ("lvx_bwd_dq_bf16.hip", "bwd_dq_bf16_kernelILi96ELb1ELi0E"),
    ("lvx_bwd_dkdv_bf16.hip", "bwd_dkdv_bf16_kernelILi96ELb1ELb0E"),
])
def test_blocks_with_matrix_instructions_move_no_accumulator(src, kernel):
    """The dense forward's loop has (rare) branches and the general dQ kernel has mask code, so
    their loops are several basic blocks; the rule is then per block: where matrix instructions are
    issued, no accumulator move and no spill.  The moves of the (rare) rescale of O^T sit in
    blocks of their own, behind an explicit wait."""
    body = _kernel(_asm(src), kernel)
    n = 0
    for blk in _blocks(body):
        if "v_mfma_f32_32x32x16_bf16" in blk:
            n += 1
            assert "v_accvgpr" not in blk, "accumulator moved next to matrix instructions"
            assert "scratch_" not in blk, "register spill next to matrix instructions"
    assert n > 0


def test_fused_backward_accumulators_stay_put():
    """The fused backward writes only its dK / dV accumulations by hand (into the accumulation file);
    S, dP and dQ are matrix instructions the compiler knows.  Wherever a hand-written one is issued,
    no accumulator may move.  (Spills of ordinary registers are the compiler's own business: it knows
    every instruction that wrote them; the steady-state block, checked above, has none.)"""
    body = _kernel(_asm("lvx_bwd_fused_bf16.hip"), "bwd_fused_bf16_kernelILi128E")
    n = 0
    for blk in _blocks(body):
        if re.search(r"v_mfma_f32_32x32x16_bf16 a\[", blk):
            n += 1
            assert "v_accvgpr" not in blk, "accumulator moved next to hand-written matrix instructions"
    assert n > 0
