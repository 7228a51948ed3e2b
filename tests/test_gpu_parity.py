"""GPU parity: the HIP path (through the C ABI) against the fp64 CPU oracle, element by element,
on the same seeded inputs.  Sizes here are ones the oracle finishes in seconds; they span
several tiles (128 query rows, 64 keys) and ragged tails.

Tolerances (bf16 inputs, fp32 accumulation): max-abs 1e-2 on O, 1e-3 on L, relative 2e-2 on
dQ/dK/dV (both Frobenius ratio and max-abs ratio).  Because |O| can be far below 1e-2 for
zero-mean V, O must also match to 2e-2 in relative Frobenius norm.  float32 inputs are held to
1e-5 / 1e-5 / 1e-4."""
import numpy as np
import pytest
import torch

import oracle
from paper_2502_02406_amd import workloads as W

pytestmark = pytest.mark.gpu

TOL = {"bf16": dict(o=1e-2, lse=1e-3, grad=2e-2, o_rel=2e-2),
       "f32": dict(o=1e-5, lse=1e-5, grad=1e-4, o_rel=1e-5)}


def _loop(*a, **k):
    from paper_2502_02406_amd.blockloop import BlockLoop
    return BlockLoop(*a, **k)


def rel_fro(x, ref):
    return float(np.linalg.norm(x - ref) / max(np.linalg.norm(ref), 1e-30))


def rel_max(x, ref):
    return float(np.abs(x - ref).max() / max(np.abs(ref).max(), 1e-30))


def check_fwd(O, L, Oref, Lref, tol, tag):
    O = O.float().cpu().numpy().astype(np.float64)
    L = L.float().cpu().numpy().astype(np.float64)
    inf_ref = np.isneginf(Lref)
    assert np.array_equal(np.isneginf(L), inf_ref), f"{tag}: -inf pattern of L differs"
    fin = ~inf_ref
    if fin.any():
        assert np.abs(L[fin] - Lref[fin]).max() <= tol["lse"], f"{tag}: L err {np.abs(L[fin] - Lref[fin]).max()}"
    assert np.isfinite(O).all(), f"{tag}: non-finite O"
    assert np.abs(O - Oref).max() <= tol["o"], f"{tag}: O max-abs err {np.abs(O - Oref).max()}"
    assert rel_fro(O, Oref) <= tol["o_rel"], f"{tag}: O rel err {rel_fro(O, Oref)}"
    if inf_ref.any():
        assert np.all(O[inf_ref] == 0.0), f"{tag}: rows without keys must give O = 0"


def check_grad(g, ref, tol, tag, cancel_atol=0.0):
    """cancel_atol > 0 is for references that vanish only by cancellation (a single key: dS =
    p (dP - delta) with dP and delta two float32 sums of the same D products taken in different
    orders); zeros that are structural (masked or dead rows, p = 0) must be exact."""
    g = g.float().cpu().numpy().astype(np.float64)
    assert np.isfinite(g).all(), f"{tag}: non-finite gradient"
    if np.abs(ref).max() == 0.0:
        assert np.abs(g).max() <= cancel_atol, f"{tag}: expected zeros, got {np.abs(g).max()}"
        return
    assert rel_fro(g, ref) <= tol["grad"], f"{tag}: Frobenius rel err {rel_fro(g, ref)}"
    assert rel_max(g, ref) <= tol["grad"], f"{tag}: max-abs rel err {rel_max(g, ref)}"


def run_case(w: W.Workload, seed=W.BASE_SEED, do_bwd=True, v_mean=0.0, k_ramp=0.0, allow=None, bwd_flags=0):
    x = W.make_inputs(w, seed)
    if allow is not None:                # a bitmap other than the workload's block-causal one
        x["allow"] = torch.from_numpy(np.ascontiguousarray(allow, dtype=np.uint8))
    if v_mean:
        x["v"] = (x["v"].float() + v_mean).to(x["v"].dtype)
    if k_ramp:      # key norms grow along the sequence by a factor 1 + k_ramp in all
        ramp = 1.0 + k_ramp * torch.arange(w.Skv, dtype=torch.float32) / max(w.Skv - 1, 1)
        x["k"] = (x["k"].float() * ramp[None, None, :, None]).to(x["k"].dtype)
    qn, kn, vn, gn = (W.as_f32_numpy(x[n]) for n in ("q", "k", "v", "do"))
    omask = dmask = None
    dev = {n: t.cuda() for n, t in x.items()}
    if w.masked:
        omask = oracle.Mask(x["allow"].numpy(), w.q_chunk, w.kv_block)
        from paper_2502_02406_amd.blockloop import MediaMask
        dmask = MediaMask(dev["allow"], w.q_chunk, w.kv_block)
    tol = TOL[w.dtype]
    loop = _loop(tuple(x["q"].shape), tuple(x["k"].shape), W.torch_dtype(w.dtype), w.n_blocks, dmask,
                 bwd_flags=bwd_flags)
    O, L = loop.forward(dev["q"], dev["k"], dev["v"])
    torch.cuda.synchronize()
    Oref, Lref = oracle.fwd(qn, kn, vn, mask=omask)
    check_fwd(O, L, Oref, Lref, tol, w.name)
    if not do_bwd:
        return
    dk, dv = torch.empty_like(dev["k"]), torch.empty_like(dev["v"])
    dq = loop.backward(dev["q"], dev["k"], dev["v"], O, L, dev["do"], dk, dv)
    torch.cuda.synchronize()
    # the oracle differentiates the exact forward; the GPU was handed its own (rounded) O and L,
    # as a real backward pass would be
    dQr, dKr, dVr = oracle.bwd(qn, kn, vn, gn, mask=omask)
    # One key: O = V and p = 1, so dS, dQ and dK vanish by cancellation of sums of magnitude
    # D * |dO| * |V| ~ 30, i.e. up to a few float32 ulps (1e-6) times |Q| or |K| times the scale.
    atol = 1e-5 if w.Skv == 1 else 0.0
    check_grad(dq, dQr, tol, w.name + " dQ", atol)
    check_grad(dk, dKr, tol, w.name + " dK", atol)
    check_grad(dv, dVr, tol, w.name + " dV")
    if bwd_flags:       # the fused kernel reports a lock it could not get; there must be none
        from paper_2502_02406_amd import binding as B
        kb = dev["k"][:, :, :loop.blk]
        ew = B.lvx_xattn_bwd_error_word(B.make_problem(dev["q"], kb), B.dtype_code(dev["q"].dtype), None, loop.ws)
        if ew and (bwd_flags & B.LVX_BWD_FUSED):
            import ctypes
            word = torch.ones(1, dtype=torch.int32, device="cuda")
            assert ctypes.CDLL("libamdhip64.so").hipMemcpy(ctypes.c_void_p(word.data_ptr()), ctypes.c_void_p(ew), 4, 3) == 0
            torch.cuda.synchronize()
            assert int(word.item()) == 0, f"{w.name}: a workgroup gave up on a dQ tile lock"


def small(name, **kw):
    base = dict(name=name, B=1, Hq=2, Hkv=2, D=128, Sq=128, Skv=512, dtype="bf16", std=0.5)
    base.update(kw)
    return W.Workload(**base)


FWD_BWD_CASES = [
    W.WORKLOADS["c1_tiny"],                                                    # fp32, 4 blocks of 256
    small("f32_d128_gqa_ragged", dtype="f32", std=1.0, Hq=4, Sq=37, Skv=203),
    small("f32_masked", dtype="f32", std=1.0, D=64, Hq=4, Sq=64, Skv=256, q_chunk=8, kv_block=32),
    small("bf16_one_tile", Sq=32, Skv=64),
    small("bf16_multi_tile", Hq=4, Sq=256, Skv=1024),
    small("bf16_ragged", Hq=4, Sq=200, Skv=1000 + 37),
    small("bf16_sq1_skv1", Sq=1, Skv=1),
    small("bf16_d64", D=64, Hq=4, Sq=160, Skv=777),
    small("bf16_gqa4_blocks", B=2, Hq=8, Hkv=2, Sq=192, Skv=2048, n_blocks=4),
    small("bf16_blockcausal", B=2, Hq=4, Hkv=4, Sq=256, Skv=2048, q_chunk=32, kv_block=256),
    small("bf16_mixed_mask", Hq=2, Sq=100, Skv=600, q_chunk=5, kv_block=24),
    small("bf16_outliers", Hq=4, Sq=128, Skv=4096, outlier_frac=0.01, outlier_scale=8.0, n_blocks=2),
    small("bf16_splitkv", Hq=2, Sq=64, Skv=16384),
    # as many workgroups as the chip has compute units: the key range is not split, so that the
    # Rescale of the block loop runs in the forward kernel's own epilogue
    small("bf16_fused_rescale", B=4, Hq=64, Hkv=8, D=64, Sq=32, Skv=512, n_blocks=4),
    small("bf16_long_q", Sq=1100, Skv=384),                                    # five query tiles, six key tiles
    small("bf16_gqa8_d64_blocks", D=64, Hq=8, Hkv=1, Sq=96, Skv=1536, n_blocks=3),
    # 64-wide heads through every kind of kernel, six or more tiles / steps each: dense; a mask
    # that selects whole steps and whole key tiles (step lists in dK/dV, tile lists plus the general
    # kernels on the partly visible tiles in the forward and dQ); a mask that cuts through tiles
    small("bf16_d64_dense_long", D=64, Hq=2, Sq=224, Skv=1024),
    small("bf16_d64_blockcausal_lists", D=64, Hq=4, Hkv=2, Sq=256, Skv=4096, q_chunk=32, kv_block=512),
    small("bf16_d64_mixed_mask", D=64, Hq=4, Hkv=2, Sq=200, Skv=1500, q_chunk=5, kv_block=24),
    # the structure of the masked bench workload at a size the oracle does in seconds: 32-row
    # chunks, 1024-key frames, chunk i sees frames <= i -- every wave meets tiles that are
    # visible to one of its two row blocks only, inside the pipelined loop
    small("bf16_blockcausal_frames", Sq=512, Skv=16384, q_chunk=32, kv_block=1024),
    small("bf16_mask_unaligned_d64", D=64, Hq=4, Sq=300, Skv=3000, q_chunk=50, kv_block=700),
    small("bf16_mask_many_chunks", Sq=256, Skv=1024, q_chunk=4, kv_block=64),   # 64 chunks per workgroup
    # text lengths are arbitrary: a last query tile of 13 rows per head, several heads per group
    small("bf16_ragged_rows_gqa_d64", D=64, Hq=8, Hkv=2, Sq=77, Skv=640, n_blocks=2),
    small("bf16_ragged_rows_one_short_tile", Hq=2, Sq=3, Skv=512),
    # one text token per head against a long key range: the four heads of a group share a tile,
    # the key range is split
    small("bf16_single_token_gqa", Hq=8, Hkv=2, Sq=1, Skv=8192),
    # a worker's share of the text: 345 rows per head, tiles that straddle the heads of a group
    small("bf16_short_block_gqa", Hq=8, Hkv=2, Sq=345, Skv=1024),
    # 96-wide heads (three 32-column blocks, six k-steps, rows of 192 bytes: 12 chunks per row,
    # so copies and row-wise stores have idle lanes) through every kind of kernel
    small("f32_d96_gqa_ragged", dtype="f32", std=1.0, D=96, Hq=4, Sq=37, Skv=203),
    small("bf16_d96_one_tile", D=96, Sq=32, Skv=64),
    small("bf16_d96_dense_long", D=96, Hq=2, Sq=224, Skv=1024),
    small("bf16_d96_ragged", D=96, Hq=4, Sq=200, Skv=1037),
    small("bf16_d96_gqa4_blocks", D=96, B=2, Hq=8, Hkv=2, Sq=192, Skv=2048, n_blocks=4),
    small("bf16_d96_blockcausal_lists", D=96, Hq=4, Hkv=2, Sq=256, Skv=4096, q_chunk=32, kv_block=512),
    small("bf16_d96_mixed_mask", D=96, Hq=4, Hkv=2, Sq=200, Skv=1500, q_chunk=5, kv_block=24),
    small("bf16_d96_splitkv", D=96, Hq=2, Sq=64, Skv=16384),
    small("bf16_d96_single_token_gqa", D=96, Hq=8, Hkv=2, Sq=1, Skv=8192),
    small("bf16_d96_fused_rescale", D=96, B=4, Hq=64, Hkv=8, Sq=32, Skv=512, n_blocks=4),
    # a head group of seven (28 query heads on 4 K/V heads), 729 keys per frame: tiles straddle
    # the heads of a group and the frames
    small("bf16_gqa7_frames_of_729", Hq=14, Hkv=2, Sq=150, Skv=4 * 729, n_blocks=2),
]


# Both forms of the bf16 backward on the shapes the fused kernel takes (dense, D = 128, >= 256 keys,
# >= 32 query rows): one kernel for all five products (dQ tiles added under locks by every key
# tile's workgroup), and the dK/dV + dQ kernel pair.  Shapes: many key tiles against few steps (every
# workgroup meets every other on the same dQ tiles), walks cut into segments of one, two and three
# steps, a ragged Sq (overlapping last step) and a ragged Skv (tail on the kernel pair), GQA 8:1,
# K/V blocks (dQ accumulated over calls), two batches.
FUSED_CASES = [
    small("fz_contended", Hq=2, Sq=32, Skv=8192),
    small("fz_two_steps", Hq=2, Sq=64, Skv=4096),
    small("fz_segments", Hq=4, Sq=128, Skv=2048),
    small("fz_ragged", Hq=4, Sq=200, Skv=2048 + 100),
    small("fz_gqa8_blocks", B=2, Hq=8, Hkv=1, Sq=96, Skv=3072, n_blocks=3),
    small("fz_outliers", Hq=4, Sq=160, Skv=4096, outlier_frac=0.01, outlier_scale=8.0, n_blocks=2),
    small("fz_long_q", Hq=2, Sq=1100, Skv=512),
]


@pytest.mark.parametrize("mode", ["fused", "split"])
@pytest.mark.parametrize("w", FUSED_CASES, ids=lambda w: w.name)
def test_backward_forms(w, mode):
    from paper_2502_02406_amd import binding as B
    run_case(w, bwd_flags=B.LVX_BWD_FUSED if mode == "fused" else B.LVX_BWD_SPLIT)


@pytest.mark.parametrize("w", FWD_BWD_CASES, ids=lambda w: w.name)
def test_fwd_parity(w):
    run_case(w, do_bwd=False)


@pytest.mark.parametrize("w", FWD_BWD_CASES, ids=lambda w: w.name)
def test_fwd_bwd_parity(w):
    run_case(w, do_bwd=True)


def test_fwd_structured_values_order_one():
    # V with mean 1 makes |O| = O(1), so the absolute tolerance on O is a real constraint
    run_case(small("bf16_vmean1", Hq=4, Sq=256, Skv=2048), do_bwd=True, v_mean=1.0)


def test_rising_scores_raise_the_reference_often():
    # keys grow 12-fold along the sequence, so the row maxima keep rising and the forward's lazy
    # reference is raised (and O rescaled) again and again, in every wave, instead of once
    run_case(small("bf16_rising", Hq=4, Sq=256, Skv=4096), do_bwd=True, k_ramp=11.0)
    run_case(small("bf16_rising_blocks", Hq=2, Sq=128, Skv=8192, n_blocks=2), do_bwd=False, k_ramp=23.0)


@pytest.mark.parametrize("name,kw,per_batch,p_on", [
    ("bf16_randmask_batch", dict(B=2, Hq=4, Hkv=2, Sq=384, Skv=4096, q_chunk=16, kv_block=128), True, 0.5),
    ("bf16_randmask_unaligned_d64", dict(D=64, Hq=4, Sq=200, Skv=2500, q_chunk=7, kv_block=100), False, 0.3),
    ("bf16_randmask_half_tiles", dict(Sq=256, Skv=2048, q_chunk=32, kv_block=32), False, 0.7),
    ("bf16_randmask_blocks", dict(Hq=4, Hkv=1, Sq=128, Skv=4096, q_chunk=32, kv_block=256, n_blocks=2), False, 0.4),
    ("bf16_randmask_sparse", dict(Sq=512, Skv=8192, q_chunk=64, kv_block=512), False, 0.1),
])
def test_random_media_masks(name, kw, per_batch, p_on):
    # seeded random bitmaps: mixed tiles everywhere, rows and keys that nobody pairs with,
    # a different bitmap per batch entry in the first case
    w = small(name, **kw)
    rng = np.random.Generator(np.random.Philox(1234 + len(name)))
    nq, nk = -(-w.Sq // w.q_chunk), -(-w.Skv // w.kv_block)
    shape = (w.B, nq, nk) if per_batch else (nq, nk)
    run_case(w, do_bwd=True, allow=(rng.random(shape) < p_on))


@pytest.mark.parametrize("name,kw,per_batch,p_on", [
    ("bf16_stepmask_gqa", dict(B=2, Hq=8, Hkv=2, Sq=256, Skv=2048, q_chunk=32, kv_block=256), True, 0.4),
    ("bf16_stepmask_d64_ragged_keys", dict(D=64, Hq=4, Hkv=2, Sq=192, Skv=1900, q_chunk=64, kv_block=512), False, 0.5),
    ("bf16_stepmask_single_steps", dict(Hq=2, Sq=320, Skv=1536, q_chunk=32, kv_block=256), False, 0.12),
    ("bf16_stepmask_ragged_rows", dict(Hq=4, Hkv=2, Sq=200, Skv=1024, q_chunk=32, kv_block=256), False, 0.6),
])
def test_step_aligned_media_masks(name, kw, per_batch, p_on):
    # chunks that are multiples of 32 rows and key blocks that are multiples of 256 keys: the
    # dK/dV kernel then runs its dense loop over a list of visible steps (several heads per
    # group walk the list again; lists of one entry; key blocks nobody sees; a ragged last block)
    w = small(name, **kw)
    rng = np.random.Generator(np.random.Philox(4321 + len(name)))
    nq, nk = -(-w.Sq // w.q_chunk), -(-w.Skv // w.kv_block)
    shape = (w.B, nq, nk) if per_batch else (nq, nk)
    run_case(w, do_bwd=True, allow=(rng.random(shape) < p_on))


@pytest.mark.parametrize("kind", ["recent", "random"])
def test_masks_whose_window_stays_in_global_memory(kind):
    # chunks of 2 rows against 320 frames of 16 keys: the 128 chunks of a workgroup's rows times
    # all frames are more bytes than the window areas in LDS hold, so the kernels plan their tiles
    # from the bitmap where it lies (the one-frame mask of the short-frame models at a small size,
    # and a random bitmap with rows and frames that pair with nothing)
    w = small(f"bf16_{kind}_tiny_chunks", D=64, Hq=4, Hkv=2, Sq=512, Skv=5120, q_chunk=2, kv_block=16)
    nq, nk = w.Sq // w.q_chunk, w.Skv // w.kv_block
    if kind == "recent":
        allow = np.arange(nk)[None, :] == np.minimum(np.arange(nq)[:, None] + 40, nk - 1)
    else:
        allow = np.random.Generator(np.random.Philox(77)).random((nq, nk)) < 0.02
    run_case(w, do_bwd=True, allow=allow)


def _random_case(it, rng, wide=False):
    """A small random problem: head dims, group sizes, query lengths around the tile sizes, key
    blocks that are and are not tile multiples, block loops, and media masks of three kinds
    (wide: also 96-wide heads, head groups of 7, and masks that show each text chunk one frame)."""
    D, Hkv, G, B = int(rng.choice([64, 96, 96, 128] if wide else [64, 128])), int(rng.choice([1, 2, 3])), \
        int(rng.choice([1, 2, 4, 7] if wide else [1, 2, 4])), int(rng.choice([1, 2]))
    Sq = int(rng.choice([1, 7, 31, 32, 33, 64, 100, 200, 256, 257, 345, 512]))
    n_blocks = int(rng.choice([1, 1, 2, 3]))
    masked = rng.random() < 0.5
    q_chunk = kv_block = 0
    if masked:
        q_chunk, kv_block = int(rng.choice([8, 16, 32, 64, 50])), int(rng.choice([64, 128, 256, 512, 100, 729]))
        blk = kv_block * int(rng.integers(1, 5))              # block boundaries fall on mask blocks
        if rng.random() < 0.3 and n_blocks == 1:
            blk += int(rng.integers(1, kv_block))             # ragged last mask block
    else:
        blk = int(rng.choice([64, 128, 192, 500, 1000, 1024, 2048, 3000]))
    Skv = blk * n_blocks
    if Skv * Sq * B * Hkv * G > 6e7:
        return None, None
    w = W.Workload(f"random{it}", B=B, Hq=Hkv * G, Hkv=Hkv, D=D, Sq=Sq, Skv=Skv, dtype="bf16", std=0.5,
                   n_blocks=n_blocks, q_chunk=q_chunk, kv_block=kv_block)
    allow = None
    if masked:
        nq, nk = -(-Sq // q_chunk), -(-Skv // kv_block)
        kind = int(rng.integers(0, 4 if wide else 3))
        if kind == 3:        # each text chunk sees one frame, the most recent one
            allow = np.arange(nk)[None, :] == np.minimum(np.arange(nq)[:, None], nk - 1)
        elif kind == 0:
            allow = rng.random((nq, nk)) < rng.choice([0.2, 0.5, 0.9])
        elif kind == 1:
            allow = np.arange(nk)[None, :] <= np.arange(nq)[:, None]
        else:
            allow = rng.random((B, nq, nk)) < 0.5
    return w, allow


@pytest.mark.parametrize("seed", [11, 12, 13, 21, 22])
def test_random_shapes(seed):
    rng = np.random.Generator(np.random.Philox(seed))
    done = 0
    for it in range(16):
        w, allow = _random_case(it, rng, wide=seed > 20)
        if w is None:
            continue
        run_case(w, seed=seed * 100 + it, do_bwd=True, allow=allow)
        done += 1
    assert done >= 8


def test_masked_rows_without_keys():
    # block-causal mask whose first chunks see nothing inside the second K/V block
    w = small("bf16_blockcausal_blocks", B=1, Hq=2, Sq=128, Skv=1024, q_chunk=32, kv_block=256,
              n_blocks=2)
    run_case(w, do_bwd=True)


@pytest.mark.parametrize("D,n", [(128, 5), (96, 5), (128, 11), (64, 19)])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_merge_matches_oracle(dtype, D, n):
    # (the kernel keeps the statistics of eight parts in registers and fetches the parts' elements
    # four parts at a time: 5, 11 and 19 parts end inside a group of four, of eight, and past both)
    from paper_2502_02406_amd import binding as B
    rng = np.random.default_rng(5)
    shape = (2, 3, 50, D)
    O = rng.standard_normal((n,) + shape)
    L = rng.standard_normal((n,) + shape[:3]) * 4
    L[1, :, :, :7] = -np.inf
    L[:, 0, 0, 10:13] = -np.inf          # rows empty in every part
    td = W.torch_dtype(dtype)
    parts = [torch.from_numpy(O[i]).to(td).cuda() for i in range(n)]
    lses = [torch.from_numpy(L[i]).float().cuda() for i in range(n)]
    Oin = np.stack([p.float().cpu().numpy().astype(np.float64) for p in parts])
    Lin = np.stack([l.cpu().numpy().astype(np.float64) for l in lses])
    Oref, Lref = oracle.merge(Oin, Lin)
    for out_dtype in (torch.float32, td):
        o_out = torch.empty(shape, dtype=out_dtype, device="cuda")
        l_out = torch.empty(shape[:3], dtype=torch.float32, device="cuda")
        B.lvx_xattn_merge(parts, lses, o_out, l_out)
        torch.cuda.synchronize()
        # The parts are exact in float32 (the oracle reads their rounded values), the weights and
        # sums are float32 arithmetic (1e-5 of the largest value is far above its noise), and a
        # bf16 output adds ONE rounding: half a unit in the last of 8 mantissa bits, at most 2^-8 |O|
        # (reached just above a power of two).
        got = o_out.float().cpu().numpy().astype(np.float64)
        bound = 1e-5 * max(1.0, np.abs(Oref).max())
        if out_dtype == torch.bfloat16:
            bound = bound + 2.0 ** -8 * np.abs(Oref)
        assert np.all(np.abs(got - Oref) <= bound), f"merge error {np.abs(got - Oref).max()}"

        Lg = l_out.cpu().numpy().astype(np.float64)
        assert np.array_equal(np.isneginf(Lg), np.isneginf(Lref))
        fin = np.isfinite(Lref)
        assert np.abs(Lg[fin] - Lref[fin]).max() <= 1e-5
        assert np.all(got[~fin] == 0.0)
    # in-place pairwise update of the running state, as Algorithm 1 does each round
    if dtype == "f32":
        run_o, run_l = parts[0].clone(), lses[0].clone()
        for i in range(1, n):
            B.lvx_xattn_merge([run_o, parts[i]], [run_l, lses[i]], run_o, run_l)
        torch.cuda.synchronize()
        assert np.abs(run_o.cpu().numpy() - Oref).max() <= 1e-5 * max(1.0, np.abs(Oref).max())
        Lg = run_l.cpu().numpy().astype(np.float64)
        fin = np.isfinite(Lref)
        assert np.abs(Lg[fin] - Lref[fin]).max() <= 1e-5
