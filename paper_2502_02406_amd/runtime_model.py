"""The paper's analytic runtime model (Section 3.1, "Runtime Analysis"; Equations 1 and 2; Table 1),
as plain host arithmetic.  Nothing here touches the GPU: bench.py feeds it the measured time of
one visit (the kernel on one worker's K/V share) and prints what the model predicts per round
for a given link bandwidth.

Per round, a worker of LV-XAttn computes attention of a visiting query block against its K/V
block and meanwhile passes (Q_j, O_j, L_j) on; a worker of Ring Attention passes (K_i, V_i) on
instead.  Both take  max(f, comm)  per round, with f the attention time.  Sizes are counted in
elements per head in the paper (2 S_Q d / n + S_Q / n against 2 S_KV d / n) and multiplied by the
number of heads h in Table 1; here they are turned into bytes by the caller's element sizes.
"""
from __future__ import annotations

from dataclasses import dataclass


def lvxattn_round_elements(sq_per_worker: int, d: int, h: int = 1) -> int:
    """Elements a worker of LV-XAttn sends per round (Equation 1): Q_j and O_j, S_Q/n x d each,
    and L_j, S_Q/n, for each of the h heads."""
    return h * (2 * sq_per_worker * d + sq_per_worker)


def ring_round_elements(skv_per_worker: int, d: int, h: int = 1) -> int:
    """Elements a worker of Ring Attention sends per round (Equation 2): K_i and V_i, S_KV/n x d
    each, for each of the h heads."""
    return h * 2 * skv_per_worker * d


def volume_ratio(sq: int, skv: int, d: int) -> float:
    """LV-XAttn's communication volume over Ring Attention's (the worker count and the head count
    cancel)."""
    return lvxattn_round_elements(sq, d) / ring_round_elements(skv, d)


def round_time(f_seconds: float, comm_bytes: float, bandwidth_bytes_per_s: float) -> float:
    """max(f, comm): the transfer of a round overlaps its attention (Equations 1 and 2)."""
    return max(f_seconds, comm_bytes / bandwidth_bytes_per_s)


def table1_speedup(sq_per_worker: int, gpu_flops: float, net_elements_per_s: float, backward: bool = False) -> float:
    """Table 1's last row: Ring Attention bound by its transfers over LV-XAttn bound by its
    attention FLOPs (4 units forward, 10 backward, of S_Q/n S_KV/n h d; Ring sends 2 units of
    S_KV/n h d forward and 4 backward: K, V and their gradients)."""
    c = (2.0 / 5.0) if backward else 0.5
    return c / sq_per_worker * gpu_flops / net_elements_per_s


@dataclass
class RoundPrediction:
    link: str
    bandwidth_gbs: float
    lvxattn_comm_ms: float
    lvxattn_round_ms: float
    ring_comm_ms: float
    ring_round_ms: float
    speedup: float
    lvxattn_hidden: bool        # the transfer fits under the attention of the round


def predict_forward_round(f_ms: float, sq: int, skv_block: int, d: int, h_q: int, h_kv: int, link: str,
                          bandwidth_gbs: float, q_bytes: int = 2, o_bytes: int = 4, l_bytes: int = 4,
                          kv_bytes: int = 2) -> RoundPrediction:
    """One forward round with the measured attention time f_ms of a visit (query block of sq rows
    against a K/V block of skv_block keys).  LV-XAttn sends Q (q_bytes per element), the running O
    (o_bytes) and L (l_bytes) of the h_q query heads; Ring Attention sends K and V (kv_bytes) of
    the h_kv key/value heads."""
    bw = bandwidth_gbs * 1e9
    lv_bytes = h_q * (sq * d * q_bytes + sq * d * o_bytes + sq * l_bytes)
    ring_bytes = h_kv * 2 * skv_block * d * kv_bytes
    f = f_ms * 1e-3
    lv = round_time(f, lv_bytes, bw)
    rg = round_time(f, ring_bytes, bw)
    return RoundPrediction(link, bandwidth_gbs, lv_bytes / bw * 1e3, lv * 1e3, ring_bytes / bw * 1e3, rg * 1e3,
                           rg / lv, lv_bytes / bw <= f)


def predict_backward_round(f_ms: float, sq: int, skv_block: int, d: int, h_q: int, h_kv: int, link: str,
                           bandwidth_gbs: float, q_bytes: int = 2, do_bytes: int = 2, dq_bytes: int = 4,
                           stat_bytes: int = 4, kv_bytes: int = 2, dkv_bytes: int = 4) -> RoundPrediction:
    """One backward round with the measured backward time f_ms of a visit.  The paper gives the
    backward pass only through Table 1 (Ring Attention moves 4 units of S_KV/n h d: K, V and their
    gradients); for LV-XAttn this build's reading is that the query side keeps travelling: Q, dO,
    the two row statistics (L and rowsum(dO * O)) and the running dQ of the h_q query heads, while
    K, V, dK and dV stay where they are."""
    bw = bandwidth_gbs * 1e9
    lv_bytes = h_q * (sq * d * (q_bytes + do_bytes + dq_bytes) + 2 * sq * stat_bytes)
    ring_bytes = h_kv * 2 * skv_block * d * (kv_bytes + dkv_bytes)
    f = f_ms * 1e-3
    lv = round_time(f, lv_bytes, bw)
    rg = round_time(f, ring_bytes, bw)
    return RoundPrediction(link, bandwidth_gbs, lv_bytes / bw * 1e3, lv * 1e3, ring_bytes / bw * 1e3, rg * 1e3,
                           rg / lv, lv_bytes / bw <= f)
