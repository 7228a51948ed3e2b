#!/usr/bin/env python3
"""Benchmark of the LV-XAttn cross-attention path on ONE MI355X.

A "step" is one pass of the whole hot path over one batch of synthetic input: the forward
block loop (Algorithm 1 with the send/recv removed: lvx_xattn_fwd for the first K/V block, then
lvx_xattn_fwd_merge -- the FlashAttention call and Rescale in one call -- for each further block)
followed by the backward block loop (per block lvx_xattn_bwd, then lvx_xattn_dq_finalize).
The workload is the long-video share: B=1, Hq=32, Hkv=8, D=128, Sq=2048, Skv=262144 in 8 blocks
of 32768, bf16.  FLOPs follow the paper's Table 1 convention (forward 4, backward 10 times
Sq*Skv*h*d).  Inputs are seeded, synthetic and resident in HBM before the timed region.

Prints ONE JSON line.  `roofline` is for the dominant kernel, timed live with HIP events on the
stream the kernels run on; `cpu_baseline` is the fp64 oracle timed on the host cores on a bounded
sample of the same workload.  `recompute` times the projections that the backward pass would
run again under the activation recomputation of Section 3.2 (lvx_xattn_project); it is reported
beside the attention figures and is no part of `value`; `model` is the paper's per-round runtime
model (Section 3.1) evaluated with the measured forward visit.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0
# HBM bytes per launch (read + written) of the three matrix kernels on one K/V block of the bench
# workload, from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this file scaled by what the same
# counters read for a plain copy of known size.  Counters cannot be read from inside this process,
# so the figures are carried here together with where and when they were measured; they describe
# the kernels of that commit and are refreshed with the profile.
MEASURED_HBM = {"profile": "profiles/bench_c3_longvideo_256k_hbm_traffic.md", "kernels_of_commit": "261ce80",
                "bytes": {"bwd_dkdv": int((258.5 + 128.0) * 2**20), "bwd_dq": int((192.9 + 32.0) * 2**20),
                          "fwd": int((170.0 + 32.3) * 2**20)}}


def cpu_baseline(w, seed):
    """Oracle forward + backward on a slice of the workload: one K/V head (its 4 query heads),
    the first `sq` query rows and the first `skv` keys."""
    import numpy as np
    import oracle
    from paper_2502_02406_amd import workloads as W
    sq, skv = 2048, 131072
    G = w.Hq // w.Hkv
    small = W.scaled(w, name="cpu_sample", B=1, Hq=G, Hkv=1, Sq=sq, Skv=skv, n_blocks=1)
    x = W.make_inputs(small, seed)
    q, k, v, g = (W.as_f32_numpy(x[n]) for n in ("q", "k", "v", "do"))
    oracle.fwd(q[:, :, :8], k[:, :, :512], v[:, :, :512])          # warm the thread pool
    t0 = time.perf_counter()
    oracle.fwd(q, k, v)
    oracle.bwd(q, k, v, g)
    dt = time.perf_counter() - t0
    flops = small.fwd_flops() + small.bwd_flops()
    return {"value": flops / dt * 1e-12, "unit": "TFLOP/s", "cores": oracle.threads(),
            "kind": "oracle", "seconds": dt,
            "sample": f"fp64 oracle fwd+bwd on B=1 Hq={G} Hkv=1 Sq={sq} Skv={skv} D={w.D} "
                      f"(one K/V head, first {sq} query rows, first {skv} keys of the workload)"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="c3_longvideo_256k")
    ap.add_argument("--seed", type=int, default=None)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calib-copy", action="store_true",
                    help="also run one plain 256 MiB device copy (a reference of known HBM traffic "
                         "for rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures ONE GPU (the kernel on one GPU's K/V share); "
              "--gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2502_02406_amd import binding as B
    from paper_2502_02406_amd import workloads as W
    from paper_2502_02406_amd.blockloop import BlockLoop, MediaMask

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(1)
    B.load()
    w = W.WORKLOADS[args.workload]
    seed = W.BASE_SEED if args.seed is None else args.seed
    x = W.make_inputs(w, seed)
    dev = {n: t.cuda() for n, t in x.items()}
    del x
    mask = MediaMask(dev["allow"], w.q_chunk, w.kv_block) if w.masked else None
    dt = W.torch_dtype(w.dtype)
    loop = BlockLoop(tuple(dev["q"].shape), tuple(dev["k"].shape), dt, w.n_blocks, mask)
    q, k, v, g = dev["q"], dev["k"], dev["v"], dev["do"]
    dk, dv = torch.empty_like(k), torch.empty_like(v)

    def step():
        o, lse = loop.forward(q, k, v)
        loop.backward(q, k, v, o, lse, g, dk, dv)

    if args.calib_copy:
        src = torch.empty(64 * 1024 * 1024, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    sec = (time.perf_counter() - t0) / args.steps
    flops = w.fwd_flops() + w.bwd_flops()
    value = flops / sec * 1e-12

    # ---- per-kernel timing with HIP events on the launch stream (torch's current stream)
    def timed(fn, reps):
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(reps + 1)]
        fn()
        torch.cuda.synchronize()
        ev[0].record()
        for i in range(reps):
            fn()
            ev[i + 1].record()
        torch.cuda.synchronize()
        return sum(ev[i].elapsed_time(ev[i + 1]) for i in range(reps)) / reps   # ms

    o, lse = loop.forward(q, k, v)
    blk = loop.blk
    kb, vb = k[:, :, :blk], v[:, :, :blk]
    p = B.make_problem(q, kb)
    m0 = loop._mask_for(0)
    reps = max(3, args.steps)
    unit = float(w.B * w.Hq * w.D) * (w.visible_pairs() / w.n_blocks)    # Sq*Skv_blk*h*d
    B.lvx_xattn_bwd(p, q, kb, vb, o, lse, g, m0, loop.dq_accum, dk[:, :, :blk], dv[:, :, :blk],
                    loop.ws, B.LVX_BWD_DELTA)
    ms_dkdv = timed(lambda: B.lvx_xattn_bwd(p, q, kb, vb, o, lse, g, m0, loop.dq_accum,
                                            dk[:, :, :blk], dv[:, :, :blk], loop.ws, B.LVX_BWD_DKDV), reps)
    ms_dq = timed(lambda: B.lvx_xattn_bwd(p, q, kb, vb, o, lse, g, m0, loop.dq_accum,
                                          dk[:, :, :blk], dv[:, :, :blk], loop.ws, B.LVX_BWD_DQ), reps)
    o_part = torch.empty(q.shape, dtype=torch.float32, device="cuda")
    l_part = torch.empty(q.shape[:3], dtype=torch.float32, device="cuda")
    ms_fwd = timed(lambda: B.lvx_xattn_fwd(p, q, kb, vb, m0, o_part, l_part, loop.ws), reps)
    o_acc = torch.zeros_like(o_part)
    l_acc = torch.zeros_like(l_part)
    ms_merge = timed(lambda: B.lvx_xattn_merge([o_acc, o_part], [l_acc, l_part], o_acc, l_acc), reps)
    rows = w.B * w.Hq * w.Sq
    merge_bytes = 3 * rows * w.D * 4 + 3 * rows * 4
    # the N-way form of Rescale: one partial result per K/V block (at least two), combined in one
    # launch into an output of the input dtype: reads N * (O + L) float32, writes O (bf16) + L
    n_way = max(2, w.n_blocks)
    o_parts = [torch.randn_like(o_part) for _ in range(n_way)]
    l_parts = [torch.randn_like(l_part) for _ in range(n_way)]
    o_fin, l_fin = torch.empty_like(q), torch.empty_like(l_part)
    ms_merge_n = timed(lambda: B.lvx_xattn_merge(o_parts, l_parts, o_fin, l_fin), reps)
    merge_n_bytes = n_way * (rows * w.D * 4 + rows * 4) + rows * w.D * o_fin.element_size() + rows * 4
    del o_parts, l_parts, o_fin, l_fin
    # the backward in its one-kernel form (all five products in one pass), where the problem allows it
    ms_fused = None
    if w.dtype == "bf16" and not w.masked and w.D == 128 and blk >= 256 and w.Sq >= 32:
        fused = B.LVX_BWD_DKDV | B.LVX_BWD_DQ | B.LVX_BWD_FUSED
        ms_fused = timed(lambda: B.lvx_xattn_bwd(p, q, kb, vb, o, lse, g, m0, loop.dq_accum,
                                                 dk[:, :, :blk], dv[:, :, :blk], loop.ws, fused), reps)
    kernels = {
        "bwd_dkdv": {"ms": ms_dkdv, "flops": 8 * unit, "tflops": 8 * unit / ms_dkdv * 1e-9},
        "bwd_dq": {"ms": ms_dq, "flops": 6 * unit, "tflops": 6 * unit / ms_dq * 1e-9},
        "fwd": {"ms": ms_fwd, "flops": 4 * unit, "tflops": 4 * unit / ms_fwd * 1e-9},
        "merge": {"ms": ms_merge, "bytes": merge_bytes, "gbs": merge_bytes / ms_merge * 1e-6,
                  "frac_hbm": merge_bytes / ms_merge * 1e-6 / PEAK_HBM_GBS},
        "merge_nway": {"parts": n_way, "ms": ms_merge_n, "bytes": merge_n_bytes,
                       "gbs": merge_n_bytes / ms_merge_n * 1e-6,
                       "frac_hbm": merge_n_bytes / ms_merge_n * 1e-6 / PEAK_HBM_GBS},
    }
    if ms_fused is not None:
        kernels["bwd_fused"] = {"ms": ms_fused, "flops": 10 * unit, "tflops": 10 * unit / ms_fused * 1e-9,
                                "note": "the optional one-kernel backward (LVX_BWD_FUSED) on the same block; "
                                        "compare with bwd_dkdv + bwd_dq, which lvx_xattn_bwd runs by default"}
    # ---- the recomputation of Section 3.2 beside it (not part of `value`): K and V of one block
    # from that block's visual tokens, and Q from the text tokens, with an embedding width of
    # Hq * D (the width of the language model the shapes stand for) and seeded synthetic weights
    recompute = None
    if w.dtype == "bf16" and (w.Hq * w.D) % 64 == 0 and (w.Hkv * w.D) % 128 == 0:
        E = w.Hq * w.D
        pin = W.projection_inputs(w.B, blk, E, 2 * w.Hkv * w.D, w.dtype, seed)
        y_d, wkv_d = pin["x"].cuda(), pin["w"].cuda()
        pin = W.projection_inputs(w.B, w.Sq, E, w.Hq * w.D, w.dtype, seed + 100)
        x_d, wq_d = pin["x"].cuda(), pin["w"].cuda()
        del pin
        k_re, v_re = torch.empty_like(kb, memory_format=torch.contiguous_format), torch.empty_like(kb, memory_format=torch.contiguous_format)
        q_re = torch.empty_like(q)
        ms_kv = timed(lambda: B.lvx_xattn_project(y_d, wkv_d, [k_re, v_re]), reps)
        ms_q = timed(lambda: B.lvx_xattn_project(x_d, wq_d, [q_re]), reps)
        f_kv = 2.0 * w.B * blk * E * 2 * w.Hkv * w.D
        f_q = 2.0 * w.B * w.Sq * E * w.Hq * w.D
        extra_ms = w.n_blocks * ms_kv + ms_q
        # the chain rule through the same projections (lvx_xattn_project_bwd): dy and dW_K, dW_V of a
        # block from its dK, dV (stood in for by the recomputed heads: timing only), dx and dW_Q from dQ
        dy_d, dwkv_d = torch.empty_like(y_d), torch.zeros(wkv_d.shape, dtype=torch.float32, device="cuda")
        dxq_d, dwq_d = torch.empty_like(x_d), torch.zeros(wq_d.shape, dtype=torch.float32, device="cuda")
        ms_gkv_x = timed(lambda: B.lvx_xattn_project_bwd(y_d, wkv_d, [k_re, v_re], dx=dy_d), reps)
        ms_gkv_w = timed(lambda: B.lvx_xattn_project_bwd(y_d, wkv_d, [k_re, v_re], dw=dwkv_d), reps)
        ms_gq = timed(lambda: B.lvx_xattn_project_bwd(x_d, wq_d, [q_re], dx=dxq_d, dw=dwq_d), reps)
        grad_ms = w.n_blocks * (ms_gkv_x + ms_gkv_w) + ms_gq
        del dy_d, dwkv_d, dxq_d, dwq_d
        recompute = {"embed": E,
                     "kv_block": {"ms": ms_kv, "flops": f_kv, "tflops": f_kv / ms_kv * 1e-9,
                                  "frac": f_kv / ms_kv * 1e-9 / PEAK_BF16_TFLOPS},
                     "q": {"ms": ms_q, "flops": f_q, "tflops": f_q / ms_q * 1e-9},
                     "ms_per_step": extra_ms, "overhead_of_step": extra_ms / (sec * 1e3),
                     "gradients": {
                         "kv_block_dx": {"ms": ms_gkv_x, "flops": f_kv, "tflops": f_kv / ms_gkv_x * 1e-9,
                                         "frac": f_kv / ms_gkv_x * 1e-9 / PEAK_BF16_TFLOPS},
                         "kv_block_dw": {"ms": ms_gkv_w, "flops": f_kv, "tflops": f_kv / ms_gkv_w * 1e-9,
                                         "frac": f_kv / ms_gkv_w * 1e-9 / PEAK_BF16_TFLOPS},
                         "q": {"ms": ms_gq, "flops": 2 * f_q, "tflops": 2 * f_q / ms_gq * 1e-9},
                         "ms_per_step": grad_ms,
                         "note": "lvx_xattn_project_bwd: dy, dW_K, dW_V of every block and dx, dW_Q; work any "
                                 "training step does with or without recomputation, not an overhead of it"},
                     "note": "lvx_xattn_project: K and V of every block and Q made again in the backward "
                             "pass; overhead = that time over the attention forward + backward above"}
        del y_d, k_re, v_re, q_re
        # the whole layer with recomputation (RecomputeLayer: keeps x, y, O, L; makes Q, and K, V block by
        # block, again in the backward pass and carries the gradients through the projections), timed as
        # a sequence of C-ABI calls like the attention step above
        if not w.masked and w.B == 1 and w.Skv * E * 2 <= 8 << 30:
            from paper_2502_02406_amd.blockloop import RecomputeLayer
            layer = RecomputeLayer(w.B, w.Sq, w.Skv, E, w.Hq, w.Hkv, w.D, q.dtype, w.n_blocks)
            y_all = W.projection_inputs(w.B, w.Skv, E, 8, w.dtype, seed + 200)["x"].cuda()
            lo, ll = layer.forward(x_d, y_all, wq_d, wkv_d)
            ms_lf = timed(lambda: layer.forward(x_d, y_all, wq_d, wkv_d), max(1, reps // 2))
            ms_lb = timed(lambda: layer.backward(x_d, y_all, wq_d, wkv_d, lo, ll, g), max(1, reps // 2))
            recompute["layer"] = {
                "fwd_ms": ms_lf, "bwd_ms": ms_lb,
                "attention_only_ms": sec * 1e3,
                "bwd_share_recompute": extra_ms / ms_lb,
                "note": "projections + attention forward; backward with Q, K, V made again and the projections' "
                        "gradients: a whole cross-attention layer's share of a training step (no output "
                        "projection, no residual path); bwd_share_recompute = the recomputed projections' "
                        "time over the layer's backward"}
            del layer, y_all, lo, ll
        del wkv_d, x_d, wq_d
    dom = max(("bwd_dkdv", "bwd_dq", "fwd"), key=lambda n: kernels[n]["ms"])
    roofline = {"bound": "mfma", "kernel": dom, "achieved": kernels[dom]["tflops"],
                "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                "frac": kernels[dom]["tflops"] / PEAK_BF16_TFLOPS,
                "traffic": MEASURED_HBM["bytes"][dom] if args.workload == "c3_longvideo_256k" else None,
                "traffic_source": {k: MEASURED_HBM[k] for k in ("profile", "kernels_of_commit")},
                "launch_ms": kernels[dom]["ms"],
                "note": "flops = the matrix products this kernel itself performs per launch "
                        "(one K/V block of the workload)"}

    out = {
        "metric": f"cross-attn fwd+bwd TFLOP/s, Sq={w.Sq} Skv={w.Skv // 1024}K, 1 GPU",
        "value": value, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": sec * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": w.name, "B": w.B, "Hq": w.Hq, "Hkv": w.Hkv, "D": w.D, "Sq": w.Sq,
                   "Skv": w.Skv, "kv_blocks": w.n_blocks, "masked": w.masked, "seed": seed},
        "frac_of_bf16_mfma_peak": value / PEAK_BF16_TFLOPS,
        "flops_per_step": flops,
        "roofline": roofline,
        "kernels": kernels,
    }
    if recompute is not None:
        out["recompute"] = recompute
    # ---- Section 3.1's runtime model fed with the measured visit: what a forward round would take
    # with the transfers of LV-XAttn (Q, running O, L) or of Ring Attention (K, V) on one link
    from dataclasses import asdict
    from paper_2502_02406_amd import runtime_model as RM
    out["model"] = {"f_ms": ms_fwd, "note": "per-round max(f, comm) of Equations 1 and 2 with the measured forward visit; "
                                            "one xGMI link, and the paper's two slower interconnects",
                    "rounds": [asdict(RM.predict_forward_round(ms_fwd, w.Sq, blk, w.D, w.Hq, w.Hkv, name, gbs))
                               for name, gbs in (("xgmi_link", 153.0), ("net_25GBs", 25.0), ("net_1.25GBs", 1.25))],
                    "f_bwd_ms": ms_dkdv + ms_dq,
                    "rounds_bwd": [asdict(RM.predict_backward_round(ms_dkdv + ms_dq, w.Sq, blk, w.D, w.Hq, w.Hkv, name, gbs))
                                   for name, gbs in (("xgmi_link", 153.0), ("net_25GBs", 25.0), ("net_1.25GBs", 1.25))]}
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, seed)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
