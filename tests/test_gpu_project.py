"""GPU parity of the projection kernels (Q = x W_Q, K, V = y W_K, y W_V of Section 2, recomputed
in the backward pass per Section 3.2) against the fp64 oracle, element by element, through the C
ABI.

Tolerance, from the arithmetic: the matrix-core kernel forms exact bf16 x bf16 products, adds
them in float32 and rounds the sum once to bf16.  With A = sum_e |x_e| |w_e| the float32 sum is
off by at most about E 2^-24 A (taken as 2^-20 A for E <= 16384 with room to spare) and the final
rounding by 2^-9 |ref| (taken as 2^-8): |out - ref| <= 2^-8 |ref| + 2^-20 A.  float32 tensors:
2^-20 A alone."""
import numpy as np
import pytest
import torch

import oracle
from paper_2502_02406_amd import workloads as W

pytestmark = pytest.mark.gpu


def run(B, S, E, H, D, n_out, dtype, seed, x_pad=0):
    from paper_2502_02406_amd import binding as Bn
    inp = W.projection_inputs(B, S, E, n_out * H * D, dtype, seed=seed)
    x, w = inp["x"], inp["w"]
    if x_pad:                                   # a strided view: rows E + x_pad apart
        buf = torch.zeros((B, S, E + x_pad), dtype=x.dtype)
        buf[:, :, :E] = x
        xd = buf.cuda()[:, :, :E]
    else:
        xd = x.cuda()
    outs = [torch.full((B, H, S, D), float("nan"), dtype=x.dtype, device="cuda") for _ in range(n_out)]
    Bn.lvx_xattn_project(xd, w.cuda(), outs)
    torch.cuda.synchronize()
    return x, w, [o.float().cpu().numpy().astype(np.float64) for o in outs]


def check(x, w, outs, H, dtype, tag, rows=None):
    xf, wf = x.float().numpy(), w.float().numpy()
    HD = wf.shape[0] // len(outs)
    for o, got in enumerate(outs):
        wo = wf[o * HD:(o + 1) * HD]
        ref = oracle.project(xf, wo, H, rows=rows)
        mag = oracle.project(np.abs(xf), np.abs(wo), H, rows=rows)
        if rows is not None:
            got = np.stack([got[b, :, s] for b, s in rows])
        assert np.isfinite(got).all(), f"{tag}: non-finite output {o}"
        bound = (2.0 ** -8 * np.abs(ref) if dtype == "bf16" else 0.0) + 2.0 ** -20 * mag
        worst = (np.abs(got - ref) / bound).max()
        assert worst <= 1.0, f"{tag}: output {o} off by {worst:.2f} of the bound"


CASES = [
    # B, S, E, H, D, n_out, x_pad
    ("one_tile_two_pairs", 1, 256, 128, 2, 128, 1, 0),
    ("one_pair", 1, 100, 64, 2, 128, 1, 0),
    ("ragged_tokens_three_pairs", 1, 300, 192, 2, 128, 2, 0),
    ("four_pairs", 1, 260, 256, 2, 128, 1, 0),
    ("d64_batches_fold", 2, 333, 320, 4, 64, 2, 0),
    ("llama_like_kv", 1, 1000, 1024, 8, 128, 2, 0),
    ("strided_tokens", 1, 515, 256, 2, 128, 1, 64),
    ("q_like_many_column_tiles", 1, 257, 512, 16, 64, 1, 0),
]


@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
def test_project_bf16(case):
    tag, B, S, E, H, D, n_out, x_pad = case
    x, w, outs = run(B, S, E, H, D, n_out, "bf16", seed=77 + len(tag), x_pad=x_pad)
    check(x, w, outs, H, "bf16", tag)


def test_project_f32_any_shape():
    x, w, outs = run(2, 37, 50, 3, 20, 2, "f32", seed=5)
    check(x, w, outs, 3, "f32", "f32")


def test_project_repeats_bit_for_bit():
    """What the backward pass recomputes must be what the forward pass used: no run-to-run
    variation (fixed summation order, no atomics)."""
    from paper_2502_02406_amd import binding as Bn
    inp = W.projection_inputs(2, 700, 512, 2 * 4 * 128, "bf16", seed=9)
    x, w = inp["x"].cuda(), inp["w"].cuda()
    outs = [[torch.empty((2, 4, 700, 128), dtype=torch.bfloat16, device="cuda") for _ in range(2)] for _ in range(2)]
    Bn.lvx_xattn_project(x, w, outs[0])
    torch.cuda.synchronize()
    Bn.lvx_xattn_project(x, w, outs[1])
    torch.cuda.synchronize()
    assert torch.equal(outs[0][0], outs[1][0]) and torch.equal(outs[0][1], outs[1][1])


def test_project_unsupported_shapes_are_refused():
    from paper_2502_02406_amd import binding as Bn
    x = torch.zeros((1, 64, 96), dtype=torch.bfloat16, device="cuda")        # E % 64 != 0
    w = torch.zeros((256, 96), dtype=torch.bfloat16, device="cuda")
    out = torch.zeros((1, 2, 64, 128), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(Bn.LvxError) as e:
        Bn.lvx_xattn_project(x, w, [out])
    assert e.value.code == -7


def test_project_full_size_block_sampled():
    """One K/V block of the long-video workload from its tokens: 32768 tokens of width 4096 onto 8
    K heads and 8 V heads of 128 -- the launch bench.py times -- on sampled tokens."""
    B, S, E, H, D = 1, 32768, 4096, 8, 128
    x, w, outs = run(B, S, E, H, D, 2, "bf16", seed=W.BASE_SEED)
    rng = np.random.default_rng(3)
    rows = np.stack([np.zeros(48, dtype=np.int64), np.sort(rng.choice(S, 48, replace=False))], axis=1)
    rows[0, 1], rows[-1, 1] = 0, S - 1
    check(x, w, outs, H, "bf16", "full", rows=rows.astype(np.int32))
    # projected keys feed the attention: their spread is the attention workloads'
    assert 0.4 < outs[0].std() < 0.6
