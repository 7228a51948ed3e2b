"""Pins of the oracle's projection (Section 2: Q = x W_Q, K, V = y W_K, y W_V; Section 3.2
recomputes them in the backward pass) against what the mathematics fixes: selections, closed
forms, a brute-force loop, a library matrix product, and the attention built on top of it."""
import numpy as np
import pytest

import oracle


def rnd(seed, *shape):
    return np.random.default_rng(seed).standard_normal(shape).astype(np.float32)


def test_identity_weights_only_cut_the_columns_into_heads():
    B, S, H, D = 2, 5, 3, 4
    x = rnd(1, B, S, H * D)
    out = oracle.project(x, np.eye(H * D, dtype=np.float32), H)
    assert out.shape == (B, H, S, D)
    for h in range(H):
        assert np.array_equal(out[:, h], x[:, :, h * D:(h + 1) * D].astype(np.float64))


def test_single_weight_selects_one_input_feature():
    # w[n, e] = 1 alone: output column n copies input feature e (a transposed w would copy
    # feature n into column e instead)
    B, S, E, H, D = 1, 4, 7, 2, 3
    x = rnd(2, B, S, E)
    n, e = 4, 6
    w = np.zeros((H * D, E), dtype=np.float32)
    w[n, e] = 1.0
    out = oracle.project(x, w, H)
    expect = np.zeros((B, H, S, D))
    expect[:, n // D, :, n % D] = x[:, :, e]
    assert np.array_equal(out, expect)


def test_ones_input_gives_row_sums_of_the_weights():
    E, H, D = 9, 2, 4
    w = rnd(3, H * D, E)
    out = oracle.project(np.ones((1, 3, E), dtype=np.float32), w, H)
    sums = w.astype(np.float64).sum(axis=1).reshape(H, D)
    assert np.allclose(out[0, :, 0], sums, rtol=0, atol=1e-12)
    assert np.array_equal(out[0, :, 0], out[0, :, 2])


def test_brute_force_loop_and_library_product():
    B, S, E, H, D = 2, 6, 10, 2, 3
    x, w = rnd(4, B, S, E), rnd(5, H * D, E)
    out = oracle.project(x, w, H)
    for b in range(B):
        for s in range(S):
            for n in range(H * D):
                acc = 0.0
                for e in range(E):
                    acc += float(x[b, s, e]) * float(w[n, e])
                assert abs(out[b, n // D, s, n % D] - acc) < 1e-12
    lib = np.einsum("bse,ne->bsn", x.astype(np.float64), w.astype(np.float64))
    lib = lib.reshape(B, S, H, D).transpose(0, 2, 1, 3)
    assert np.allclose(out, lib, rtol=0, atol=1e-12)


def test_linearity_and_sampled_rows():
    B, S, E, H, D = 2, 8, 12, 3, 4
    x1, x2, w = rnd(6, B, S, E), rnd(7, B, S, E), rnd(8, H * D, E)
    a = oracle.project(x1, w, H)
    b = oracle.project(x2, w, H)
    both = oracle.project((x1.astype(np.float64) + 2.0 * x2).astype(np.float32), w, H)
    # (the sum is rounded to float32 before it is projected: compare against the rounded input)
    xs = (x1.astype(np.float64) + 2.0 * x2).astype(np.float32).astype(np.float64)
    err = np.abs(xs - (x1.astype(np.float64) + 2.0 * x2)).max() * np.abs(w).sum(axis=1).max()
    assert np.abs(both - (a + 2.0 * b)).max() <= err + 1e-12
    rows = np.array([[1, 7], [0, 0], [1, 3]], dtype=np.int32)
    picked = oracle.project(x1, w, H, rows=rows)
    for r, (bb, ss) in enumerate(rows):
        assert np.array_equal(picked[r], a[bb, :, ss])


def test_attention_of_projected_inputs_matches_a_dense_evaluation():
    # the whole of Section 2's cross-attention from x and y, heads of the oracle's projection fed
    # to the oracle's attention, against numpy on the definition with per-head weight slices
    B, Sq, Skv, E, H, D = 1, 3, 6, 8, 2, 4
    x, y = rnd(9, B, Sq, E), rnd(10, B, Skv, E)
    wq, wk, wv = rnd(11, H * D, E), rnd(12, H * D, E), rnd(13, H * D, E)
    q = oracle.project(x, wq, H).astype(np.float32)
    k = oracle.project(y, wk, H).astype(np.float32)
    v = oracle.project(y, wv, H).astype(np.float32)
    O, _ = oracle.fwd(q, k, v)
    for h in range(H):
        sl = slice(h * D, (h + 1) * D)
        qh = (x[0].astype(np.float64) @ wq[sl].astype(np.float64).T).astype(np.float32).astype(np.float64)
        kh = (y[0].astype(np.float64) @ wk[sl].astype(np.float64).T).astype(np.float32).astype(np.float64)
        vh = (y[0].astype(np.float64) @ wv[sl].astype(np.float64).T).astype(np.float32).astype(np.float64)
        s = qh @ kh.T / np.sqrt(D)
        p = np.exp(s - s.max(axis=1, keepdims=True))
        p /= p.sum(axis=1, keepdims=True)
        assert np.allclose(O[0, h], p @ vh, rtol=0, atol=1e-10)
