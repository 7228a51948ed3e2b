"""Seeded synthetic inputs for the LV-XAttn cross-attention path.

This module holds NO attention arithmetic.  It only draws random tensors,
scales them, rounds them to the storage type and builds mask bitmaps, so that
the GPU path and the CPU oracle can be fed the very same values.  The paper
benchmarks on randomly generated inputs of given sizes (Section 4.1, the
benchmarking-methodology paragraph), so synthetic tensors of the stated shapes
are its workload.

Shapes: Q, dO [B, Hq, Sq, D];  K, V [B, Hkv, Skv, D];  mask allow
[n_q_chunks, n_kv_blocks] uint8 (1 = the text chunk may attend the visual block).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, Optional

import numpy as np
import torch

BASE_SEED = 20250204
_TENSOR_ID = {"q": 0, "k": 1, "v": 2, "do": 3, "outliers": 4, "tokens": 5, "weights": 6, "head_grads": 7}


@dataclass(frozen=True)
class Workload:
    name: str
    B: int
    Hq: int
    Hkv: int
    D: int
    Sq: int
    Skv: int
    dtype: str                 # "f32" or "bf16": storage type of Q, K, V, dO
    std: float                 # Q, K, V, dO ~ N(0,1) * std
    n_blocks: int = 1          # K/V blocks the query block visits in turn (Algorithm 1 on one GPU)
    q_chunk: int = 0           # >0: media mask over text chunks of q_chunk rows and visual blocks of kv_block keys
    kv_block: int = 0
    mask_kind: str = "causal"  # "causal": text chunk i sees visual blocks <= i; "recent": only block i
    outlier_frac: float = 0.0  # fraction of key tokens whose K row is scaled
    outlier_scale: float = 1.0
    note: str = ""

    @property
    def masked(self) -> bool:
        return self.q_chunk > 0

    def fwd_flops(self) -> float:
        """Paper's convention (Table 1): 4 * Sq * Skv * h * d; masked pairs are not counted."""
        return 4.0 * self.B * self.Hq * self.D * self.visible_pairs()

    def bwd_flops(self) -> float:
        """Paper's convention (Table 1): 10 * Sq * Skv * h * d."""
        return 10.0 * self.B * self.Hq * self.D * self.visible_pairs()

    def visible_pairs(self) -> float:
        if not self.masked:
            return float(self.Sq) * float(self.Skv)
        allow = media_mask(self)
        # (ragged last chunk / block: count the rows and keys that exist)
        rows = np.minimum(self.q_chunk, self.Sq - np.arange(allow.shape[0]) * self.q_chunk)
        keys = np.minimum(self.kv_block, self.Skv - np.arange(allow.shape[1]) * self.kv_block)
        return float(rows.astype(np.float64) @ allow.astype(np.float64) @ keys.astype(np.float64))


WORKLOADS: Dict[str, Workload] = {
    "c1_tiny": Workload("c1_tiny", B=1, Hq=2, Hkv=2, D=64, Sq=128, Skv=1024, dtype="f32", std=1.0,
                        n_blocks=4, note="tiny exact check, 4 blocks of 256"),
    "c2_llama_64k": Workload("c2_llama_64k", B=1, Hq=32, Hkv=8, D=128, Sq=2048, Skv=65536,
                             dtype="bf16", std=0.5, note="Llama-3-V-like layer, one KV share"),
    "c3_longvideo_256k": Workload("c3_longvideo_256k", B=1, Hq=32, Hkv=8, D=128, Sq=2048,
                                  Skv=262144, dtype="bf16", std=0.5, n_blocks=8,
                                  note="256 frames x 1024 tokens, 8 blocks of 32768 merged via LSE"),
    "c4_flamingo_masked": Workload("c4_flamingo_masked", B=2, Hq=16, Hkv=16, D=128, Sq=1024,
                                   Skv=131072, dtype="bf16", std=0.5, q_chunk=32, kv_block=1024,
                                   note="32 text chunks x 32 tokens, 128 frames x 1024 tokens, "
                                        "chunk i sees frames <= i"),
    "c5_extreme_1m": Workload("c5_extreme_1m", B=1, Hq=32, Hkv=8, D=128, Sq=512, Skv=1048576,
                              dtype="bf16", std=0.5, n_blocks=16, outlier_frac=0.01,
                              outlier_scale=8.0, note="16 blocks of 65536, 1% of key tokens x8"),
    # further shapes (the paper's models with short visual blocks have much longer text sides,
    # Section 4): measured for the record, not part of the graded set
    "x1_sq32k_skv64k": Workload("x1_sq32k_skv64k", B=1, Hq=32, Hkv=8, D=128, Sq=32768, Skv=65536,
                                dtype="bf16", std=0.5, note="text side as long as half the visual side"),
    "x2_d64_sq8k_skv256k": Workload("x2_d64_sq8k_skv256k", B=1, Hq=32, Hkv=8, D=64, Sq=8192, Skv=262144,
                                    dtype="bf16", std=0.5, n_blocks=4, note="64-wide heads, 4 blocks of 65536"),
    "x4_ragged_5514x64040": Workload("x4_ragged_5514x64040", B=1, Hq=32, Hkv=8, D=128, Sq=5514, Skv=64040,
                                     dtype="bf16", std=0.5, n_blocks=2,
                                     note="sizes that are no tile multiples: the paper's Video-MME text length, "
                                          "ten frames of 6404 visual tokens in two blocks"),
    "x3_sq65k_skv8k": Workload("x3_sq65k_skv8k", B=1, Hq=32, Hkv=8, D=128, Sq=65536, Skv=8192,
                               dtype="bf16", std=0.5, note="text side longer than the visual side"),
    "x5_d96_skv256k": Workload("x5_d96_skv256k", B=1, Hq=32, Hkv=8, D=96, Sq=2048, Skv=262144,
                               dtype="bf16", std=0.5, n_blocks=8, note="96-wide heads on the shape of c3"),
    # One worker's share of rows of the paper's comparison table (Section 4.2, 16 workers: the
    # worker keeps 1/16 of the text and meets all 16 K/V blocks), with the models' visual tokens
    # per frame (Section 4.1): 729 and 64
    "m1_owl7b_729": Workload("m1_owl7b_729", B=1, Hq=28, Hkv=4, D=128, Sq=512, Skv=1458000,
                             dtype="bf16", std=0.5, n_blocks=16,
                             note="8K text, 2000 frames of 729 tokens: 512 text rows, 16 blocks of 125 frames "
                                  "(91125 keys, no tile multiple), head groups of 7"),
    "m2_flamingo9b_64": Workload("m2_flamingo9b_64", B=1, Hq=8, Hkv=8, D=64, Sq=4096, Skv=2097152,
                                 dtype="bf16", std=0.5, n_blocks=16,
                                 note="64K text, 32K frames of 64 tokens: 4096 text rows, 16 blocks of 2048 frames"),
    "m3_flamingo_recent_frame": Workload("m3_flamingo_recent_frame", B=1, Hq=8, Hkv=8, D=64, Sq=4096, Skv=131072,
                                         dtype="bf16", std=0.5, q_chunk=2, kv_block=64, mask_kind="recent",
                                         note="the same worker's text against its own 2048 frames when every "
                                              "text chunk (2 tokens per frame) sees only the frame before it"),
}


def scaled(w: Workload, **kw) -> Workload:
    """A copy of a workload with some fields replaced (used for reduced-size parity cases)."""
    d = {f: getattr(w, f) for f in w.__dataclass_fields__}
    d.update(kw)
    return Workload(**d)


def torch_dtype(name: str) -> torch.dtype:
    return {"f32": torch.float32, "bf16": torch.bfloat16}[name]


def _normal(shape, seed: int, std: float) -> torch.Tensor:
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)
    n0 = shape[0] * shape[1]
    out = torch.empty(shape, dtype=torch.float32)
    flat = out.view(n0, shape[2], shape[3])
    for r in range(n0):                       # one (b, head) slab at a time bounds peak memory
        flat[r].normal_(0.0, 1.0, generator=g)
    if std != 1.0:
        out.mul_(std)
    return out


def outlier_tokens(w: Workload, seed: int = BASE_SEED) -> Optional[np.ndarray]:
    """Per batch, the sorted key-token indices whose K rows are scaled: [B, n_out]."""
    if w.outlier_frac <= 0.0:
        return None
    n_out = int(round(w.outlier_frac * w.Skv))
    rng = np.random.Generator(np.random.Philox(seed + _TENSOR_ID["outliers"]))
    return np.stack([np.sort(rng.choice(w.Skv, size=n_out, replace=False)) for _ in range(w.B)])


def block_causal_mask(w: Workload) -> np.ndarray:
    """allow[i, f] = 1 iff visual block f <= text chunk i (shared across batch)."""
    nq = (w.Sq + w.q_chunk - 1) // w.q_chunk
    nk = (w.Skv + w.kv_block - 1) // w.kv_block
    i = np.arange(nq)[:, None]
    f = np.arange(nk)[None, :]
    return (f <= i).astype(np.uint8)


def recent_frame_mask(w: Workload) -> np.ndarray:
    """allow[i, f] = 1 iff f == i: a text chunk sees only the visual block inserted right before it
    (the most recent frame); chunks past the last block see the last one."""
    nq = (w.Sq + w.q_chunk - 1) // w.q_chunk
    nk = (w.Skv + w.kv_block - 1) // w.kv_block
    i = np.minimum(np.arange(nq), nk - 1)[:, None]
    f = np.arange(nk)[None, :]
    return (f == i).astype(np.uint8)


def media_mask(w: Workload) -> np.ndarray:
    """The workload's mask bitmap [n_q_chunks, n_kv_blocks] (shared across the batch)."""
    return {"causal": block_causal_mask, "recent": recent_frame_mask}[w.mask_kind](w)


def make_inputs(w: Workload, seed: int = BASE_SEED, with_do: bool = True) -> Dict[str, torch.Tensor]:
    """CPU tensors in the workload's storage dtype: q, k, v, (do), plus 'allow' (uint8) if masked.

    Values are rounded to the storage type here, once; both the GPU path and the
    oracle consume these rounded values."""
    dt = torch_dtype(w.dtype)
    out: Dict[str, torch.Tensor] = {}
    out["q"] = _normal((w.B, w.Hq, w.Sq, w.D), seed + _TENSOR_ID["q"], w.std).to(dt)
    k = _normal((w.B, w.Hkv, w.Skv, w.D), seed + _TENSOR_ID["k"], w.std)
    tok = outlier_tokens(w, seed)
    if tok is not None:
        for b in range(w.B):
            k[b, :, torch.from_numpy(tok[b]), :] *= w.outlier_scale
    out["k"] = k.to(dt)
    del k
    out["v"] = _normal((w.B, w.Hkv, w.Skv, w.D), seed + _TENSOR_ID["v"], w.std).to(dt)
    if with_do:
        out["do"] = _normal((w.B, w.Hq, w.Sq, w.D), seed + _TENSOR_ID["do"], w.std).to(dt)
    if w.masked:
        out["allow"] = torch.from_numpy(media_mask(w))
    return out


def as_f32_numpy(t: torch.Tensor) -> np.ndarray:
    """Exact widening of a storage-typed tensor to float32 numpy (what the oracle reads)."""
    return t.detach().to("cpu", torch.float32).contiguous().numpy()


def projection_inputs(B: int, S: int, E: int, N: int, dtype: str, seed: int = BASE_SEED,
                      std_out: float = 0.5) -> Dict[str, torch.Tensor]:
    """CPU tensors for the projections of Section 2 (recomputed in the backward pass, Section 3.2):
    token features 'x' [B, S, E] ~ N(0, 1) (what a normalisation layer hands over) and stacked,
    transposed projection weights 'w' [N, E] ~ N(0, std_out^2 / E), so that the projected heads
    have the spread the attention workloads use.  Rounded to the storage type here, once."""
    dt = torch_dtype(dtype)
    g = torch.Generator(device="cpu")
    g.manual_seed(seed + _TENSOR_ID["tokens"])
    x = torch.empty((B, S, E), dtype=torch.float32).normal_(0.0, 1.0, generator=g)
    g.manual_seed(seed + _TENSOR_ID["weights"])
    w = torch.empty((N, E), dtype=torch.float32).normal_(0.0, std_out / float(E) ** 0.5, generator=g)
    return {"x": x.to(dt), "w": w.to(dt)}


def projection_grad_inputs(B: int, S: int, H: int, D: int, n_out: int, dtype: str,
                           seed: int = BASE_SEED, std: float = 0.05) -> list:
    """CPU tensors standing in for the gradients of the projected heads (what the attention
    backward hands over as dQ, or as dK and dV): n_out tensors [B, H, S, D] ~ N(0, std^2), rounded
    to the storage type here, once."""
    dt = torch_dtype(dtype)
    g = torch.Generator(device="cpu")
    outs = []
    for o in range(n_out):
        g.manual_seed(seed + _TENSOR_ID["head_grads"] + 16 * o)
        outs.append(torch.empty((B, H, S, D), dtype=torch.float32).normal_(0.0, std, generator=g).to(dt))
    return outs
