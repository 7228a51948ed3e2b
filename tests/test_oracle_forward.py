"""Pins of the oracle's forward (attention definition, Section 2 of the paper) against
things other than itself: an independent numpy brute force, closed forms, invariants."""
import numpy as np
import pytest

import oracle


def rnd(shape, seed, grid=2.0 ** -8):
    r = np.random.default_rng(seed).standard_normal(shape)
    return (np.round(r / grid) * grid).astype(np.float32)


def brute_force(q, k, v, scale, allow=None, q_chunk=1, kv_block=1):
    """Independent triple loop in python floats (float64)."""
    B, Hq, Sq, D = q.shape
    _, Hkv, Skv, _ = k.shape
    G = Hq // Hkv
    O = np.zeros((B, Hq, Sq, D))
    L = np.full((B, Hq, Sq), -np.inf)
    for b in range(B):
        for h in range(Hq):
            hk = h // G
            for i in range(Sq):
                s = []
                for j in range(Skv):
                    if allow is not None and not allow[i // q_chunk][j // kv_block]:
                        s.append(None)
                        continue
                    s.append(scale * sum(float(q[b, h, i, d]) * float(k[b, hk, j, d]) for d in range(D)))
                vis = [x for x in s if x is not None]
                if not vis:
                    continue
                m = max(vis)
                z = sum(np.exp(x - m) for x in vis)
                L[b, h, i] = m + np.log(z)
                for j in range(Skv):
                    if s[j] is None:
                        continue
                    pj = np.exp(s[j] - m) / z
                    for d in range(D):
                        O[b, h, i, d] += pj * float(v[b, hk, j, d])
    return O, L


def test_matches_brute_force_dense_gqa():
    q, k, v = rnd((2, 4, 5, 4), 1), rnd((2, 2, 11, 4), 2), rnd((2, 2, 11, 4), 3)
    O, L = oracle.fwd(q, k, v)
    Ob, Lb = brute_force(q, k, v, 1 / np.sqrt(4))
    np.testing.assert_allclose(O, Ob, rtol=0, atol=1e-13)
    np.testing.assert_allclose(L, Lb, rtol=0, atol=1e-13)


def test_matches_brute_force_masked_and_scale_override():
    q, k, v = rnd((1, 2, 8, 4), 4), rnd((1, 1, 12, 4), 5), rnd((1, 1, 12, 4), 6)
    allow = np.random.default_rng(7).integers(0, 2, size=(4, 4)).astype(np.uint8)
    allow[1, :] = 0                       # chunk 1 (rows 2,3) sees nothing
    m = oracle.Mask(allow, q_chunk=2, kv_block=3)
    O, L = oracle.fwd(q, k, v, scale=0.37, mask=m)
    Ob, Lb = brute_force(q, k, v, 0.37, allow, 2, 3)
    np.testing.assert_allclose(O, Ob, rtol=0, atol=1e-13)
    assert np.array_equal(np.isinf(L), np.isinf(Lb))
    np.testing.assert_allclose(L[np.isfinite(L)], Lb[np.isfinite(Lb)], rtol=0, atol=1e-13)
    assert np.all(L[0, :, 2:4] == -np.inf) and np.all(O[0, :, 2:4] == 0.0)


def test_two_key_closed_form():
    # scores ln(1) and ln(3) -> p = (1/4, 3/4), L = ln 4
    D = 4
    scale = 0.5
    q = np.zeros((1, 1, 1, D), np.float32); q[..., 0] = 1.0
    k = np.zeros((1, 1, 2, D), np.float32)
    k[0, 0, 1, 0] = np.float32(np.log(3.0) / scale)
    v = np.array([[[[1, 0, 2, 0], [0, 1, 0, 4]]]], np.float32)
    O, L = oracle.fwd(q, k, v, scale=scale)
    s1 = scale * float(k[0, 0, 1, 0])
    p1 = np.exp(s1) / (1 + np.exp(s1))
    assert abs(p1 - 0.75) < 1e-6
    np.testing.assert_allclose(O[0, 0, 0], [(1 - p1), p1, 2 * (1 - p1), 4 * p1], atol=1e-14)
    np.testing.assert_allclose(L[0, 0, 0], np.log(1 + np.exp(s1)), atol=1e-14)


def test_probability_rows_sum_to_one():
    q, k = rnd((1, 2, 6, 8), 8), rnd((1, 2, 40, 8), 9)
    for hq in range(2):
        for i in range(6):
            p = oracle.prob_row(q, k, 0, hq, i)
            assert np.all(p >= 0)
            assert abs(p.sum() - 1.0) < 1e-14


def test_constant_v_gives_constant_o():
    q, k = rnd((1, 4, 7, 8), 10), rnd((1, 2, 33, 8), 11)
    v = np.full((1, 2, 33, 8), 0.625, np.float32)
    O, _ = oracle.fwd(q, k, v)
    np.testing.assert_allclose(O, 0.625, atol=1e-14)


def test_zero_k_gives_mean_v_and_log_skv():
    q, v = rnd((1, 2, 5, 8), 12), rnd((1, 1, 29, 8), 13)
    k = np.zeros((1, 1, 29, 8), np.float32)
    O, L = oracle.fwd(q, k, v)
    np.testing.assert_allclose(L, np.log(29.0), atol=1e-14)
    np.testing.assert_allclose(O, np.broadcast_to(v.astype(np.float64).mean(axis=2)[:, :, None], O.shape)[:, [0, 0]], atol=1e-14)


def test_single_key():
    q, k, v = rnd((1, 2, 3, 8), 14), rnd((1, 2, 1, 8), 15), rnd((1, 2, 1, 8), 16)
    O, L = oracle.fwd(q, k, v)
    np.testing.assert_allclose(O, np.broadcast_to(v.astype(np.float64), O.shape), atol=0)
    s = np.einsum("bhid,bhjd->bhij", q.astype(np.float64), k.astype(np.float64))[..., 0] / np.sqrt(8)
    np.testing.assert_allclose(L, s, atol=1e-14)


def test_dominant_key_selects_its_value():
    q, k, v = rnd((1, 1, 2, 4), 17), rnd((1, 1, 9, 4), 18), rnd((1, 1, 9, 4), 19)
    q[0, 0, :, :] = [[1, 0, 0, 0], [0, 1, 0, 0]]
    k[0, 0, 5] = [400, 400, 0, 0]
    O, _ = oracle.fwd(q, k, v)
    np.testing.assert_allclose(O[0, 0], np.stack([v[0, 0, 5]] * 2), atol=1e-12)


def test_key_shift_invariance():
    q, k, v = rnd((1, 2, 4, 8), 20), rnd((1, 2, 17, 8), 21), rnd((1, 2, 17, 8), 22)
    c = rnd((8,), 23)
    O0, L0 = oracle.fwd(q, k, v)
    O1, L1 = oracle.fwd(q, k + c, v)
    np.testing.assert_allclose(O1, O0, atol=1e-13)
    shift = (q.astype(np.float64) @ c.astype(np.float64)) / np.sqrt(8)
    np.testing.assert_allclose(L1 - L0, shift, atol=1e-13)


def test_gqa_equals_repeated_heads():
    q, k, v = rnd((2, 6, 4, 8), 24), rnd((2, 3, 13, 8), 25), rnd((2, 3, 13, 8), 26)
    O0, L0 = oracle.fwd(q, k, v)
    kr, vr = np.repeat(k, 2, axis=1), np.repeat(v, 2, axis=1)   # head hq reads hq // 2
    O1, L1 = oracle.fwd(q, kr, vr)
    np.testing.assert_allclose(O0, O1, atol=0)
    np.testing.assert_allclose(L0, L1, atol=0)
    # and it is NOT the interleaved mapping hq % Hkv
    ki, vi = np.tile(k, (1, 2, 1, 1)), np.tile(v, (1, 2, 1, 1))
    O2, _ = oracle.fwd(q, ki, vi)
    assert np.abs(O2 - O0).max() > 1e-3


def test_mask_all_ones_is_dense_and_mask_is_row_deletion():
    q, k, v = rnd((1, 2, 6, 8), 27), rnd((1, 2, 20, 8), 28), rnd((1, 2, 20, 8), 29)
    O0, L0 = oracle.fwd(q, k, v)
    ones = oracle.Mask(np.ones((3, 5), np.uint8), 2, 4)
    O1, L1 = oracle.fwd(q, k, v, mask=ones)
    assert np.array_equal(O0, O1) and np.array_equal(L0, L1)
    allow = np.ones((3, 5), np.uint8); allow[:, [1, 3]] = 0      # delete kv blocks 1 and 3 for everyone
    O2, L2 = oracle.fwd(q, k, v, mask=oracle.Mask(allow, 2, 4))
    keep = np.r_[0:4, 8:12, 16:20]
    O3, L3 = oracle.fwd(q, k[:, :, keep], v[:, :, keep])
    np.testing.assert_allclose(O2, O3, atol=1e-14)
    np.testing.assert_allclose(L2, L3, atol=1e-14)


def test_per_batch_mask():
    q, k, v = rnd((2, 1, 4, 4), 30), rnd((2, 1, 6, 4), 31), rnd((2, 1, 6, 4), 32)
    allow = np.ones((2, 2, 3), np.uint8); allow[1, 0, 2] = 0
    O, L = oracle.fwd(q, k, v, mask=oracle.Mask(allow, 2, 2))
    Od, Ld = oracle.fwd(q, k, v)
    assert np.array_equal(O[0], Od[0])
    assert np.array_equal(O[1, :, 2:], Od[1, :, 2:])
    assert np.abs(O[1, :, :2] - Od[1, :, :2]).max() > 1e-4


def test_fwd_rows_matches_full():
    q, k, v = rnd((2, 4, 9, 8), 33), rnd((2, 2, 21, 8), 34), rnd((2, 2, 21, 8), 35)
    O, L = oracle.fwd(q, k, v)
    rows = np.array([[0, 0, 0], [1, 3, 8], [0, 2, 4], [1, 1, 7]], np.int32)
    Or, Lr = oracle.fwd_rows(q, k, v, rows)
    for n, (b, h, i) in enumerate(rows):
        assert np.array_equal(Or[n], O[b, h, i]) and Lr[n] == L[b, h, i]


def test_lse_statistics_for_gaussian_scores():
    # i.i.d. Gaussian scores of std sigma: LSE ~ ln(Skv) + sigma^2/2
    D, Skv = 64, 8192
    rng = np.random.default_rng(36)
    q = (rng.standard_normal((1, 1, 8, D)) * 0.5).astype(np.float32)
    k = (rng.standard_normal((1, 1, Skv, D)) * 0.5).astype(np.float32)
    v = (rng.standard_normal((1, 1, Skv, D)) * 0.5).astype(np.float32)
    _, L = oracle.fwd(q, k, v)
    sig2 = (np.linalg.norm(q.astype(np.float64), axis=-1) ** 2) * 0.25 / D
    np.testing.assert_allclose(L[0, 0], np.log(Skv) + sig2[0, 0] / 2, atol=0.03)
