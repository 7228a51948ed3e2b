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


# ---- gradients of the projection -----------------------------------------------------------------
# Tolerance, from the arithmetic: exact bf16 x bf16 products added in float32.  dx is a sum of
# N = n_out H D terms rounded once to the tensors' type: 2^-8 |ref| + 2^-20 A with A the sum of the
# terms' magnitudes, as for the forward.  dw stays float32 and is a sum over the M tokens, taken 16
# at a time by a matrix instruction and then added to a running float32 value: M / 16 roundings of
# at most 2^-24 A each in the worst case, i.e. 2^-28 M A, and never less than 2^-20 A allowed.


def run_bwd(B, S, E, H, D, n_out, dtype, seed, x_pad=0, want=("dx", "dw"), dw0=None):
    from paper_2502_02406_amd import binding as Bn
    inp = W.projection_inputs(B, S, E, n_out * H * D, dtype, seed=seed)
    gs = W.projection_grad_inputs(B, S, H, D, n_out, dtype, seed=seed)
    x, w = inp["x"], inp["w"]
    if x_pad:
        buf = torch.zeros((B, S, E + x_pad), dtype=x.dtype)
        buf[:, :, :E] = x
        xd = buf.cuda()[:, :, :E]
        dxd = torch.full((B, S, E + x_pad), float("nan"), dtype=x.dtype, device="cuda")[:, :, :E]
    else:
        xd = x.cuda()
        dxd = torch.full((B, S, E), float("nan"), dtype=x.dtype, device="cuda")
    dwd = (torch.zeros((n_out * H * D, E), dtype=torch.float32) if dw0 is None else dw0.clone()).cuda()
    Bn.lvx_xattn_project_bwd(xd, w.cuda(), [g.cuda() for g in gs],
                             dx=dxd if "dx" in want else None, dw=dwd if "dw" in want else None)
    torch.cuda.synchronize()
    return x, w, gs, dxd.float().cpu().numpy().astype(np.float64), dwd.cpu().numpy().astype(np.float64)


def check_bwd(x, w, gs, dx, dw, H, dtype, tag, cols=None, rows=None, dw0=None, want=("dx", "dw")):
    xf, wf = x.float().numpy(), w.float().numpy()
    gf = np.concatenate([g.float().numpy() for g in gs], axis=1)          # heads of all outputs stacked
    Ht = H * len(gs)
    M = xf.shape[0] * xf.shape[1]
    ref_w, ref_x = oracle.project_bwd(xf, wf, gf, Ht, cols=cols, rows=rows)
    mag_w, mag_x = oracle.project_bwd(np.abs(xf), np.abs(wf), np.abs(gf), Ht, cols=cols, rows=rows)
    if "dx" in want:
        got = dx if rows is None else np.stack([dx[b, s] for b, s in rows])
        assert np.isfinite(got).all(), f"{tag}: non-finite dx"
        bound = (2.0 ** -8 * np.abs(ref_x) if dtype == "bf16" else 0.0) + 2.0 ** -20 * mag_x
        worst = (np.abs(got - ref_x) / bound).max()
        assert worst <= 1.0, f"{tag}: dx off by {worst:.2f} of the bound"
    if "dw" in want:
        got = dw if cols is None else dw[cols]
        if dw0 is not None:
            base = dw0.numpy().astype(np.float64)
            base = base if cols is None else base[cols]
            ref_w = ref_w + base
            mag_w = mag_w + np.abs(base)
        assert np.isfinite(got).all(), f"{tag}: non-finite dw"
        bound = max(2.0 ** -20, 2.0 ** -28 * M) * mag_w
        worst = (np.abs(got - ref_w) / bound).max()
        assert worst <= 1.0, f"{tag}: dw off by {worst:.2f} of the bound"


BWD_CASES = [
    # B, S, E, H, D, n_out, x_pad
    ("one_tile_four_pairs", 1, 256, 256, 2, 128, 1, 0),
    ("less_than_one_pair_of_tokens", 1, 40, 256, 2, 128, 1, 0),
    ("two_pairs", 1, 128, 256, 2, 128, 1, 0),
    ("ragged_tokens_two_outputs", 1, 300, 256, 2, 128, 2, 0),
    ("d64_batches_fold", 2, 333, 512, 4, 64, 2, 0),
    ("short_batches_inside_a_pair", 3, 70, 256, 2, 128, 1, 0),
    ("llama_like_kv", 1, 1000, 1024, 8, 128, 2, 0),
    ("strided_tokens", 1, 515, 256, 2, 128, 1, 64),
    ("q_like_many_column_tiles", 1, 257, 512, 16, 64, 1, 0),
    # one tile of dw and 63 tile pairs of tokens (the last with 32 rows): seven parts of the token
    # range take turns on the tile
    ("dw_parts_take_turns", 1, 4000, 256, 2, 128, 1, 0),
    ("dw_parts_two_outputs_batches", 2, 1300, 256, 2, 128, 2, 0),
    # 96-wide heads: a tile pair's 64 columns straddle two heads, eight heads fill three column tiles
    ("d96_heads_straddle_tile_pairs", 2, 150, 256, 8, 96, 2, 0),
    # shapes the matrix-core kernels do not take: the plain kernels
    ("plain_heads_of_96", 1, 130, 64, 2, 96, 2, 0),
    ("plain_narrow_output", 2, 65, 128, 1, 128, 1, 0),
]


@pytest.mark.parametrize("case", BWD_CASES, ids=[c[0] for c in BWD_CASES])
def test_project_bwd_bf16(case):
    tag, B, S, E, H, D, n_out, x_pad = case
    print(f"[project_bwd] {tag}", flush=True)
    x, w, gs, dx, dw = run_bwd(B, S, E, H, D, n_out, "bf16", seed=31 + len(tag), x_pad=x_pad)
    check_bwd(x, w, gs, dx, dw, H, "bf16", tag)


def test_project_bwd_f32_any_shape():
    x, w, gs, dx, dw = run_bwd(2, 37, 50, 3, 20, 2, "f32", seed=6)
    check_bwd(x, w, gs, dx, dw, 3, "f32", "f32")


def test_project_bwd_accumulates_into_dw_and_takes_either_output_alone():
    B, S, E, H, D, n_out = 1, 200, 256, 2, 128, 2
    dw0 = torch.empty((n_out * H * D, E), dtype=torch.float32).normal_(0.0, 1.0, generator=torch.Generator().manual_seed(4))
    x, w, gs, dx, dw = run_bwd(B, S, E, H, D, n_out, "bf16", seed=12, dw0=dw0)
    check_bwd(x, w, gs, dx, dw, H, "bf16", "accumulate", dw0=dw0)
    x, w, gs, dx1, dw1 = run_bwd(B, S, E, H, D, n_out, "bf16", seed=12, want=("dx",), dw0=dw0)
    assert np.array_equal(dx1, dx) and np.array_equal(dw1, dw0.numpy().astype(np.float64))   # dw untouched
    x, w, gs, dx2, dw2 = run_bwd(B, S, E, H, D, n_out, "bf16", seed=12, want=("dw",), dw0=dw0)
    assert np.array_equal(dw2, dw) and np.isnan(dx2).all()                                     # dx untouched


@pytest.mark.parametrize("S", [700, 5000])      # (5000 tokens: the parts of dw's token range take turns)
def test_project_bwd_repeats_bit_for_bit(S):
    a = run_bwd(2, S, 512, 4, 128, 2, "bf16", seed=9)
    b = run_bwd(2, S, 512, 4, 128, 2, "bf16", seed=9)
    assert np.array_equal(a[3], b[3]) and np.array_equal(a[4], b[4])


def test_project_bwd_wide_projection_takes_tall_tiles_sampled():
    """A projection with at least as many 256 x 256 tiles of dw as three quarters of the chip's
    compute units (the query projection of the bench model: 4096 columns from 4096 features) runs
    the 256-row tiles; narrower ones, every other case here, the 128-row tiles."""
    B, S, E, H, D = 1, 200, 4096, 32, 128
    x, w, gs, dx, dw = run_bwd(B, S, E, H, D, 1, "bf16", seed=44)
    rng = np.random.default_rng(6)
    rows = np.stack([np.zeros(6, dtype=np.int64), np.sort(rng.choice(S, 6, replace=False))], axis=1)
    cols = np.sort(rng.choice(H * D, 24, replace=False))
    cols[0], cols[-1] = 0, H * D - 1
    check_bwd(x, w, gs, dx, dw, H, "bf16", "wide", cols=cols.astype(np.int32), rows=rows.astype(np.int32))
    assert np.isfinite(dw).all() and np.isfinite(dx).all()


@pytest.mark.parametrize("tag,S,E,H,D", [
    # the long-video workload's K/V block: 128 tiles of dw, the tokens of each in two parts
    ("long_video_block", 32768, 4096, 8, 128),
    # a block of the 64-token-frame model (embedding width 512, 8 heads of 64): 8 tiles of dw, the
    # tokens of each in 32 parts that take turns
    ("short_frame_block", 131072, 512, 8, 64),
])
def test_project_bwd_full_size_block_sampled(tag, S, E, H, D):
    """The gradients of one K/V block at full size -- the launches bench.py times -- on sampled
    tokens (dx) and sampled columns of the projection (dw)."""
    B = 1
    print(f"[project_bwd] full size {tag}: GPU", flush=True)
    x, w, gs, dx, dw = run_bwd(B, S, E, H, D, 2, "bf16", seed=W.BASE_SEED)
    rng = np.random.default_rng(5)
    rows = np.stack([np.zeros(24, dtype=np.int64), np.sort(rng.choice(S, 24, replace=False))], axis=1)
    rows[0, 1], rows[-1, 1] = 0, S - 1
    cols = np.sort(rng.choice(2 * H * D, 12, replace=False))
    cols[0], cols[-1] = 0, 2 * H * D - 1
    print("[project_bwd] full size: oracle on sampled tokens and columns", flush=True)
    check_bwd(x, w, gs, dx, dw, H, "bf16", "full", cols=cols.astype(np.int32), rows=rows.astype(np.int32))
