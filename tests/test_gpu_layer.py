"""GPU parity of a whole cross-attention layer under the activation recomputation of Section 3.2:
projections (Section 2), Algorithm 1 over the K/V blocks, the recompute-P backward, and the chain
rule back through the projections -- the sequence of C-ABI calls of `RecomputeLayer`, which keeps
x, y, O and L only -- against the oracle's functions chained on the CPU.

Both sides round Q, K and V to the storage type where they are stored (the attention reads bf16
heads).  The GPU also rounds dQ, dK, dV (and dx, dy) to bf16 on their way; the oracle chain does not,
which stays inside the gradient tolerance."""
import numpy as np
import pytest
import torch

import oracle
from paper_2502_02406_amd import workloads as W

pytestmark = pytest.mark.gpu


def rel_fro(x, ref):
    return float(np.linalg.norm(x - ref) / max(np.linalg.norm(ref), 1e-30))


def bf16_round(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).bfloat16().float().numpy()


CASES = [
    # name, B, Sq, Skv, E, Hq, Hkv, D, n_blocks
    ("two_blocks_gqa", 1, 96, 512, 256, 4, 2, 128, 2),
    ("one_block_two_batches", 2, 64, 320, 256, 2, 2, 128, 1),
    ("four_blocks_d64", 1, 200, 1024, 256, 8, 4, 64, 4),
]


@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
def test_layer_with_recomputation(case):
    from paper_2502_02406_amd.blockloop import RecomputeLayer
    name, B, Sq, Skv, E, Hq, Hkv, D, n_blocks = case
    print(f"[layer] {name}", flush=True)
    seed = 500 + len(name)
    tx = W.projection_inputs(B, Sq, E, Hq * D, "bf16", seed=seed)
    ty = W.projection_inputs(B, Skv, E, 2 * Hkv * D, "bf16", seed=seed + 50)
    x, wq, y, wkv = tx["x"], tx["w"] * 2.0, ty["x"], ty["w"] * 2.0       # heads of spread ~1: a softmax that is not flat
    wq, wkv = wq.bfloat16(), wkv.bfloat16()
    d_o = W.projection_grad_inputs(B, Sq, Hq, D, 1, "bf16", seed=seed, std=0.5)[0]

    layer = RecomputeLayer(B, Sq, Skv, E, Hq, Hkv, D, torch.bfloat16, n_blocks)
    xd, yd, wqd, wkvd, dod = (t.cuda() for t in (x, y, wq, wkv, d_o))
    O, L = layer.forward(xd, yd, wqd, wkvd)
    O, L = O.clone(), L.clone()
    dx, dy, dwq, dwkv = layer.backward(xd, yd, wqd, wkvd, O, L, dod)
    torch.cuda.synchronize()

    xf, yf, wqf, wkvf, gof = (t.float().numpy() for t in (x, y, wq, wkv, d_o))
    wkf, wvf = wkvf[:Hkv * D], wkvf[Hkv * D:]
    q = bf16_round(oracle.project(xf, wqf, Hq))
    k = bf16_round(oracle.project(yf, wkf, Hkv))
    v = bf16_round(oracle.project(yf, wvf, Hkv))
    Oref, Lref = oracle.fwd(q, k, v)
    assert np.abs(L.cpu().numpy() - Lref).max() <= 1e-3
    assert np.abs(O.float().cpu().numpy() - Oref).max() <= 1e-2
    assert rel_fro(O.float().cpu().numpy(), Oref) <= 2e-2
    dQ, dK, dV = oracle.bwd(q, k, v, gof)
    dwq_ref, dx_ref = oracle.project_bwd(xf, wqf, dQ.astype(np.float32), Hq)
    dwk_ref, dyk = oracle.project_bwd(yf, wkf, dK.astype(np.float32), Hkv)
    dwv_ref, dyv = oracle.project_bwd(yf, wvf, dV.astype(np.float32), Hkv)
    for tag, got, ref in (("dx", dx, dx_ref), ("dy", dy, dyk + dyv), ("dW_Q", dwq, dwq_ref),
                          ("dW_KV", dwkv, np.concatenate([dwk_ref, dwv_ref]))):
        g = got.float().cpu().numpy().astype(np.float64)
        assert np.isfinite(g).all(), f"{name} {tag}: non-finite"
        assert rel_fro(g, ref) <= 2e-2, f"{name} {tag}: Frobenius rel err {rel_fro(g, ref)}"
        assert np.abs(g - ref).max() <= 3e-2 * np.abs(ref).max(), f"{name} {tag}: max err {np.abs(g - ref).max() / np.abs(ref).max()}"
