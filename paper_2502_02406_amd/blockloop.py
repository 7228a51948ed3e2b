"""Algorithm 1 of the paper on ONE GPU: the query block visits N key/value blocks in turn.

The distributed schedule keeps each K/V block on its worker and passes (Q_j, O_j, L_j) around a
ring; each visit is FlashAttention(Q_j, K_i, V_i) followed by Rescale.  Here the send/recv steps
are dropped and the N blocks are N windows of one GPU's K/V tensors, so the loop is

    (O, L) <- (0, -inf);  for n in blocks:  (dO, dL) <- lvx_xattn_fwd(Q, K[n], V[n]);
                                             (O, L) <- lvx_xattn_merge((O, L), (dO, dL))

and the backward pass runs lvx_xattn_bwd once per block with the FINAL (O, L): dK/dV of a block
are complete after its call, dQ accumulates over blocks (no rescaling appears in backward).

This module only sequences C-ABI calls and owns the buffers between them (allocated once, in
the constructor, so the timed loop allocates nothing); all arithmetic is in the kernels.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Optional, Tuple

import torch

from . import binding as B


@dataclass
class MediaMask:
    allow: torch.Tensor      # uint8 device tensor [n_q_chunks, n_kv_blocks] (or [B, ., .])
    q_chunk: int
    kv_block: int


class BlockLoop:
    def __init__(self, q_shape, kv_shape, dtype: torch.dtype, n_blocks: int = 1,
                 mask: Optional[MediaMask] = None, softmax_scale: float = 0.0,
                 device: str = "cuda", bwd_flags: int = 0):
        if not torch.cuda.is_available():
            raise RuntimeError("BlockLoop needs a GPU: there is no CPU fallback")
        B.load()
        self.Bsz, self.Hq, self.Sq, self.D = q_shape
        _, self.Hkv, self.Skv, _ = kv_shape
        assert self.Skv % n_blocks == 0, "blocks must be equal (the paper's Skv/n)"
        self.n_blocks = n_blocks
        self.bwd_flags = bwd_flags      # B.LVX_BWD_FUSED / B.LVX_BWD_SPLIT: which backward kernels (0: the library's choice)
        self.blk = self.Skv // n_blocks
        if mask is not None and n_blocks > 1:
            assert self.blk % mask.kv_block == 0, "block boundaries must fall on mask blocks"
        self.dtype, self.mask, self.scale, self.dev = dtype, mask, softmax_scale, device
        f32 = dict(dtype=torch.float32, device=device)
        rows = (self.Bsz, self.Hq, self.Sq)
        self.lse = torch.empty(rows, **f32)
        self.o = torch.empty(q_shape, dtype=dtype, device=device)
        if n_blocks > 1:
            self.o_acc = torch.empty(q_shape, **f32)       # running O_j of Algorithm 1 (L_j lives in self.lse)
        self.dq_accum = torch.empty(q_shape, **f32)
        self.dq = torch.empty(q_shape, dtype=dtype, device=device)
        # one workspace sized for the larger of the two passes
        qd = torch.empty(q_shape, dtype=dtype, device="meta")
        kd = torch.empty((self.Bsz, self.Hkv, self.blk, self.D), dtype=dtype, device="meta")
        p = B.make_problem(qd, kd, softmax_scale)
        p.kv_sh = self.Skv * self.D
        p.kv_sb = self.Hkv * self.Skv * self.D
        code = B.dtype_code(dtype)
        nbytes = max(B.lvx_xattn_workspace_bytes(p, code, B.LVX_WS_FWD),
                     B.lvx_xattn_workspace_bytes(p, code, B.LVX_WS_FWD_MERGE),
                     B.lvx_xattn_workspace_bytes(p, code, B.LVX_WS_BWD))
        if nbytes == 0:
            raise B.LvxError(-2, "lvx_xattn_workspace_bytes")
        self.ws = torch.empty(nbytes, dtype=torch.uint8, device=device)

    def _mask_for(self, n: int) -> Optional[B.lvx_mask]:
        if self.mask is None:
            return None
        per = self.blk // self.mask.kv_block if self.n_blocks > 1 else 0
        nkb = (self.blk + self.mask.kv_block - 1) // self.mask.kv_block
        return B.make_mask(self.mask.allow, self.mask.q_chunk, self.mask.kv_block, n * per, nkb)

    def forward(self, q, k, v) -> Tuple[torch.Tensor, torch.Tensor]:
        """Returns (O in the input dtype, L float32); both are buffers owned by this object."""
        # (the running O of the block loop is written with Q's strides by the first visit and read as
        # a contiguous tensor by the others)
        assert self.n_blocks == 1 or q.is_contiguous(), "the block loop needs a contiguous Q"
        if self.n_blocks == 1:
            p = B.make_problem(q, k, self.scale)
            B.lvx_xattn_fwd(p, q, k, v, self._mask_for(0), self.o, self.lse, self.ws)
            return self.o, self.lse
        for n in range(self.n_blocks):
            kb = k[:, :, n * self.blk:(n + 1) * self.blk]
            vb = v[:, :, n * self.blk:(n + 1) * self.blk]
            p = B.make_problem(q, kb, self.scale)
            if n == 0:      # merging with the identity (0, -inf) is a no-op: write the state directly
                B.lvx_xattn_fwd(p, q, kb, vb, self._mask_for(n), self.o_acc, self.lse, self.ws)
            else:           # the FlashAttention call and Rescale of Algorithm 1 in one call
                B.lvx_xattn_fwd_merge(p, q, kb, vb, self._mask_for(n), self.o_acc, self.lse, self.ws)
        B.lvx_xattn_merge([self.o_acc], [self.lse], self.o, self.lse)    # round to the output dtype
        return self.o, self.lse

    def backward(self, q, k, v, o, lse, d_o, dk, dv) -> torch.Tensor:
        """dk/dv (same shape and strides as k) are overwritten; returns dQ in the input dtype."""
        self.dq_accum.zero_()
        for n in range(self.n_blocks):
            sl = slice(n * self.blk, (n + 1) * self.blk)
            kb, vb = k[:, :, sl], v[:, :, sl]
            p = B.make_problem(q, kb, self.scale)
            # delta = rowsum(dO * O) depends on the query block only: the first visit computes it
            # into the workspace, the others reuse it
            stages = (B.LVX_BWD_ALL if n == 0 else (B.LVX_BWD_DKDV | B.LVX_BWD_DQ)) | self.bwd_flags
            B.lvx_xattn_bwd(p, q, kb, vb, o, lse, d_o, self._mask_for(n), self.dq_accum,
                            dk[:, :, sl], dv[:, :, sl], self.ws, stages)
        p = B.make_problem(q, k, self.scale)
        B.lvx_xattn_dq_finalize(p, self.dq_accum, self.dq)
        return self.dq


class RecomputeLayer:
    """One cross-attention layer under the activation recomputation of Section 3.2, on one GPU: the
    forward pass keeps the token features x, y and (O, L) and nothing else; the backward pass makes
    Q again from x and, block by block, K and V again from the block's visual tokens, runs the
    attention backward on them, and carries dQ, dK, dV on through the projections to dx, dy and the
    weights' gradients.  K and V exist for one block at a time.

    x [B, Sq, E] text tokens, y [B, Skv, E] visual tokens (B > 1: n_blocks must be 1, the
    projection entry points want the batches of a call to follow each other), wq [Hq D, E],
    wkv [2 Hkv D, E] (W_K^T on top of W_V^T).  Only sequences C-ABI calls."""

    def __init__(self, Bsz, Sq, Skv, E, Hq, Hkv, D, dtype: torch.dtype, n_blocks: int = 1,
                 softmax_scale: float = 0.0, device: str = "cuda"):
        assert Skv % n_blocks == 0 and (Bsz == 1 or n_blocks == 1)
        self.n_blocks, self.blk = n_blocks, Skv // n_blocks
        self.loop = BlockLoop((Bsz, Hq, Sq, D), (Bsz, Hkv, self.blk, D), dtype, 1, None, softmax_scale, device)
        kw = dict(dtype=dtype, device=device)
        self.q = torch.empty((Bsz, Hq, Sq, D), **kw)
        self.k = torch.empty((Bsz, Hkv, self.blk, D), **kw)
        self.v = torch.empty_like(self.k)
        self.dk, self.dv = torch.empty_like(self.k), torch.empty_like(self.k)
        self.o_acc = torch.empty((Bsz, Hq, Sq, D), dtype=torch.float32, device=device)
        self.dx = torch.empty((Bsz, Sq, E), **kw)
        self.dy = torch.empty((Bsz, Skv, E), **kw)
        self.dwq = torch.empty((Hq * D, E), dtype=torch.float32, device=device)
        self.dwkv = torch.empty((2 * Hkv * D, E), dtype=torch.float32, device=device)

    def _kv_of_block(self, y, wkv, n):
        yb = y[:, n * self.blk:(n + 1) * self.blk]
        B.lvx_xattn_project(yb, wkv, [self.k, self.v])
        return yb

    def forward(self, x, y, wq, wkv) -> Tuple[torch.Tensor, torch.Tensor]:
        """(O in the input dtype, L float32); Q, K, V are not kept."""
        lp = self.loop
        B.lvx_xattn_project(x, wq, [self.q])
        p = B.make_problem(self.q, self.k, lp.scale)
        for n in range(self.n_blocks):
            self._kv_of_block(y, wkv, n)
            if self.n_blocks == 1:
                B.lvx_xattn_fwd(p, self.q, self.k, self.v, None, lp.o, lp.lse, lp.ws)
                return lp.o, lp.lse
            if n == 0:
                B.lvx_xattn_fwd(p, self.q, self.k, self.v, None, self.o_acc, lp.lse, lp.ws)
            else:
                B.lvx_xattn_fwd_merge(p, self.q, self.k, self.v, None, self.o_acc, lp.lse, lp.ws)
        B.lvx_xattn_merge([self.o_acc], [lp.lse], lp.o, lp.lse)
        return lp.o, lp.lse

    def backward(self, x, y, wq, wkv, o, lse, d_o):
        """(dx, dy in the input dtype, dW_Q, dW_KV float32) from x, y, (O, L) and dO alone."""
        lp = self.loop
        B.lvx_xattn_project(x, wq, [self.q])                       # Q again
        lp.dq_accum.zero_()
        self.dwq.zero_()
        self.dwkv.zero_()
        p = B.make_problem(self.q, self.k, lp.scale)
        for n in range(self.n_blocks):
            yb = self._kv_of_block(y, wkv, n)                       # K, V of the block again
            stages = B.LVX_BWD_ALL if n == 0 else (B.LVX_BWD_DKDV | B.LVX_BWD_DQ)
            B.lvx_xattn_bwd(p, self.q, self.k, self.v, o, lse, d_o, None, lp.dq_accum, self.dk, self.dv, lp.ws, stages)
            B.lvx_xattn_project_bwd(yb, wkv, [self.dk, self.dv],
                                    dx=self.dy[:, n * self.blk:(n + 1) * self.blk], dw=self.dwkv)
        B.lvx_xattn_dq_finalize(p, lp.dq_accum, lp.dq)
        B.lvx_xattn_project_bwd(x, wq, [lp.dq], dx=self.dx, dw=self.dwq)
        return self.dx, self.dy, self.dwq, self.dwkv
