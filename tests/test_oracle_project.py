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


# ---- gradients of the projection: loss = sum(out * g) is linear in x and in w, so its exact
# ---- derivatives are fixed by the (pinned) forward alone


def test_gradients_match_differences_of_the_forward():
    # loss(x, w) = sum(project(x, w) * g) is bilinear: a central difference in one argument is
    # exact up to rounding whatever the step, so the tolerance is rounding only.  Inputs are
    # small dyadic numbers and the step a power of two: x +- h and w +- h stay exact in float32.
    B, S, E, H, D = 2, 5, 6, 2, 3
    rng = np.random.default_rng(20)
    x = rng.integers(-8, 9, (B, S, E)).astype(np.float32) / 8
    w = rng.integers(-8, 9, (H * D, E)).astype(np.float32) / 8
    g = rng.integers(-8, 9, (B, H, S, D)).astype(np.float32) / 8
    dw, dx = oracle.project_bwd(x, w, g, H)
    assert dw.shape == (H * D, E) and dx.shape == (B, S, E)
    g64, h = g.astype(np.float64), 0.5

    def loss(xx, ww):
        return float((oracle.project(xx, ww, H) * g64).sum())

    for n in range(H * D):
        for e in range(E):
            wp, wm = w.copy(), w.copy()
            wp[n, e] += h
            wm[n, e] -= h
            assert abs((loss(x, wp) - loss(x, wm)) / (2 * h) - dw[n, e]) < 1e-11, (n, e)
    for b in range(B):
        for s in range(S):
            for e in range(E):
                xp, xm = x.copy(), x.copy()
                xp[b, s, e] += h
                xm[b, s, e] -= h
                assert abs((loss(xp, w) - loss(xm, w)) / (2 * h) - dx[b, s, e]) < 1e-11, (b, s, e)


def test_gradients_match_a_library_product():
    B, S, E, H, D = 2, 7, 9, 3, 4
    x, w, g = rnd(21, B, S, E), rnd(22, H * D, E), rnd(23, B, H, S, D)
    dw, dx = oracle.project_bwd(x, w, g, H)
    g2 = g.astype(np.float64).transpose(0, 2, 1, 3).reshape(B * S, H * D)      # [tokens, columns]
    x2 = x.astype(np.float64).reshape(B * S, E)
    assert np.allclose(dw, g2.T @ x2, rtol=0, atol=1e-12)
    assert np.allclose(dx.reshape(B * S, E), g2 @ w.astype(np.float64), rtol=0, atol=1e-12)


def test_single_entries_pick_single_terms():
    # g with one nonzero entry at (b, h, s, c): dw has ONE nonzero row, n = h D + c, equal to
    # x[b, s, :], and dx ONE nonzero token, (b, s), equal to w[n, :].  A head/column or a
    # batch/token mix-up, or g read token-major, lands elsewhere.
    B, S, E, H, D = 2, 4, 5, 3, 2
    x, w = rnd(24, B, S, E), rnd(25, H * D, E)
    b, h, s, c = 1, 2, 3, 1
    g = np.zeros((B, H, S, D), dtype=np.float32)
    g[b, h, s, c] = 2.0
    dw, dx = oracle.project_bwd(x, w, g, H)
    want_w = np.zeros((H * D, E))
    want_w[h * D + c] = 2.0 * x[b, s].astype(np.float64)
    want_x = np.zeros((B, S, E))
    want_x[b, s] = 2.0 * w[h * D + c].astype(np.float64)
    assert np.array_equal(dw, want_w)
    assert np.array_equal(dx, want_x)


def test_identity_weights_regroup_the_gradient_and_ones_sum_it():
    B, S, H, D = 2, 3, 2, 4
    g = rnd(26, B, H, S, D)
    x = np.ones((B, S, H * D), dtype=np.float32)
    dw, dx = oracle.project_bwd(x, np.eye(H * D, dtype=np.float32), g, H)
    # identity weights: dx is g with the heads laid side by side again
    assert np.array_equal(dx, g.astype(np.float64).transpose(0, 2, 1, 3).reshape(B, S, H * D))
    # x of ones: every entry of row n of dw is the sum of g's column n over all tokens
    col = g.astype(np.float64).sum(axis=(0, 2)).reshape(H * D)
    assert np.allclose(dw, np.repeat(col[:, None], H * D, axis=1), rtol=0, atol=1e-12)


def test_sampled_gradient_rows_are_the_full_ones():
    B, S, E, H, D = 2, 6, 7, 2, 3
    x, w, g = rnd(27, B, S, E), rnd(28, H * D, E), rnd(29, B, H, S, D)
    dw, dx = oracle.project_bwd(x, w, g, H)
    cols = np.array([5, 0, 3], dtype=np.int32)
    rows = np.array([[1, 5], [0, 0], [1, 2], [0, 4]], dtype=np.int32)
    dws, dxs = oracle.project_bwd(x, w, g, H, cols=cols, rows=rows)
    assert np.array_equal(dws, dw[cols])
    for r, (b, s) in enumerate(rows):
        assert np.array_equal(dxs[r], dx[b, s])


def test_gradients_through_attention_match_differences_of_the_whole_layer():
    # the chain of Section 2 end to end: loss = sum(attention(x W_Q, y W_K, y W_V) * dO); the
    # oracle's attention backward gives dQ, dK, dV, the projection backward carries them to the
    # weights and the tokens.  Compared with central differences of the loss in fp64 numpy.
    B, Sq, Skv, E, H, D = 1, 3, 5, 4, 2, 2
    rng = np.random.default_rng(30)
    x, y = rng.standard_normal((B, Sq, E)), rng.standard_normal((B, Skv, E))
    wq, wk, wv = (rng.standard_normal((H * D, E)) * 0.5 for _ in range(3))
    dO = rng.standard_normal((B, H, Sq, D))
    f32 = lambda a: a.astype(np.float32)
    x, y, wq, wk, wv, dO = map(f32, (x, y, wq, wk, wv, dO))

    def heads(t, wt):                     # fp64 numpy: [B,S,E] x [H D, E] -> [B,H,S,D]
        o = t.astype(np.float64) @ wt.astype(np.float64).T
        return o.reshape(t.shape[0], t.shape[1], H, D).transpose(0, 2, 1, 3)

    def loss(x_, y_, wq_, wk_, wv_):
        q, k, v = heads(x_, wq_), heads(y_, wk_), heads(y_, wv_)
        s = np.einsum("bhid,bhjd->bhij", q, k) / np.sqrt(D)
        p = np.exp(s - s.max(axis=-1, keepdims=True))
        p /= p.sum(axis=-1, keepdims=True)
        return float((np.einsum("bhij,bhjd->bhid", p, v) * dO.astype(np.float64)).sum())

    # the oracle's chain; its attention takes float32 operands, so hand it exactly representable
    # heads: the loss above is evaluated at the same (rounded) heads only to first order, hence
    # the tolerance of a few float32 roundings times the gradients' size
    q, k, v = (f32(heads(t, wt)) for t, wt in ((x, wq), (y, wk), (y, wv)))
    dQ, dK, dV = oracle.bwd(q, k, v, dO)
    dwq, dx = oracle.project_bwd(x, wq, f32(dQ), H)
    dwk, dy_k = oracle.project_bwd(y, wk, f32(dK), H)
    dwv, dy_v = oracle.project_bwd(y, wv, f32(dV), H)
    dy = dy_k + dy_v
    args = [x, y, wq, wk, wv]
    h = 1e-3
    for idx, grad in ((0, dx), (1, dy), (2, dwq), (3, dwk), (4, dwv)):
        for pos in np.ndindex(*args[idx].shape):
            ap = [a.astype(np.float64) for a in args]
            am = [a.astype(np.float64) for a in args]
            ap[idx][pos] += h
            am[idx][pos] -= h
            fd = (loss(*ap) - loss(*am)) / (2 * h)
            assert abs(fd - grad[pos]) < 2e-5, (idx, pos, fd, grad[pos])
