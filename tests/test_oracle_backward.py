"""Pins of the oracle's backward.  The paper states only its cost (Table 1) and what is saved
for it (Section 3.2), so the pins are mathematical: central finite differences of
loss = sum(O * dO) evaluated with the (separately pinned) forward, invariants of the
softmax Jacobian, and the block-wise rule summed over blocks."""
import numpy as np
import pytest

import oracle
from test_oracle_forward import rnd

H = 2.0 ** -10      # exactly representable step for inputs on a 2^-8 grid of magnitude < 8


def loss(q, k, v, dO, **kw):
    O, _ = oracle.fwd(q, k, v, **kw)
    return float((O * dO.astype(np.float64)).sum())


def fd_grad(q, k, v, dO, which, idxs, **kw):
    out = []
    for idx in idxs:
        arrs = {"q": q.copy(), "k": k.copy(), "v": v.copy()}
        arrs[which][idx] += np.float32(H)
        lp = loss(arrs["q"], arrs["k"], arrs["v"], dO, **kw)
        arrs[which][idx] -= np.float32(2 * H)
        lm = loss(arrs["q"], arrs["k"], arrs["v"], dO, **kw)
        out.append((lp - lm) / (2 * H))
    return np.array(out)


def some_indices(shape, n, seed):
    rng = np.random.default_rng(seed)
    return [tuple(int(rng.integers(0, s)) for s in shape) for _ in range(n)]


@pytest.mark.parametrize("case", ["dense_mha", "gqa", "masked_gqa", "scale"])
def test_finite_differences(case):
    kw = {}
    if case == "dense_mha":
        q, k, v, dO = rnd((1, 2, 4, 8), 50), rnd((1, 2, 9, 8), 51), rnd((1, 2, 9, 8), 52), rnd((1, 2, 4, 8), 53)
    elif case == "gqa":
        q, k, v, dO = rnd((2, 4, 3, 8), 54), rnd((2, 2, 7, 8), 55), rnd((2, 2, 7, 8), 56), rnd((2, 4, 3, 8), 57)
    elif case == "masked_gqa":
        q, k, v, dO = rnd((1, 4, 6, 8), 58), rnd((1, 2, 8, 8), 59), rnd((1, 2, 8, 8), 60), rnd((1, 4, 6, 8), 61)
        allow = np.array([[1, 0, 1, 0], [0, 0, 0, 0], [1, 1, 1, 1]], np.uint8)
        kw["mask"] = oracle.Mask(allow, 2, 2)
    else:
        q, k, v, dO = rnd((1, 1, 3, 4), 62), rnd((1, 1, 5, 4), 63), rnd((1, 1, 5, 4), 64), rnd((1, 1, 3, 4), 65)
        kw["scale"] = 0.8
    dQ, dK, dV = oracle.bwd(q, k, v, dO, **kw)
    for name, g, x in (("q", dQ, q), ("k", dK, k), ("v", dV, v)):
        idxs = some_indices(x.shape, 12, 66)
        fd = fd_grad(q, k, v, dO, name, idxs, **kw)
        an = np.array([g[i] for i in idxs])
        np.testing.assert_allclose(an, fd, rtol=2e-5, atol=2e-6, err_msg=f"{case} d{name}")
    if case == "masked_gqa":
        assert np.all(dQ[:, :, 2:4] == 0.0)          # chunk 1 sees nothing
        assert np.all(dK[:, :, 2:4] != 0.0) and np.all(dV[:, :, 2:4] != 0.0)


def test_dv_column_sums_equal_do_sums():
    # rows of P sum to one  =>  sum_j dV[hkv, j, :] = sum over the head group and rows of dO
    q, k, v, dO = rnd((2, 4, 5, 8), 70), rnd((2, 2, 19, 8), 71), rnd((2, 2, 19, 8), 72), rnd((2, 4, 5, 8), 73)
    _, _, dV = oracle.bwd(q, k, v, dO)
    want = dO.astype(np.float64).reshape(2, 2, 2, 5, 8).sum(axis=(2, 3))
    np.testing.assert_allclose(dV.sum(axis=2), want, atol=1e-13)


def test_equal_keys_give_zero_dq_and_dk_sums_to_zero():
    q, v, dO = rnd((1, 2, 4, 8), 74), rnd((1, 1, 11, 8), 75), rnd((1, 2, 4, 8), 76)
    k = np.broadcast_to(rnd((1, 1, 1, 8), 77), (1, 1, 11, 8)).copy()
    dQ, dK, _ = oracle.bwd(q, k, v, dO)
    np.testing.assert_allclose(dQ, 0.0, atol=1e-14)          # dS rows sum to zero
    k2 = rnd((1, 1, 11, 8), 78)
    _, dK2, _ = oracle.bwd(q, k2, v, dO)
    np.testing.assert_allclose(dK2.sum(axis=2), 0.0, atol=1e-13)   # sum_j dS_ij = 0 for each i


def test_gqa_dk_dv_sum_over_group():
    q, k, v, dO = rnd((1, 4, 3, 8), 79), rnd((1, 2, 6, 8), 80), rnd((1, 2, 6, 8), 81), rnd((1, 4, 3, 8), 82)
    dQ, dK, dV = oracle.bwd(q, k, v, dO)
    kr, vr = np.repeat(k, 2, axis=1), np.repeat(v, 2, axis=1)
    dQr, dKr, dVr = oracle.bwd(q, kr, vr, dO)
    np.testing.assert_allclose(dQ, dQr, atol=1e-15)
    np.testing.assert_allclose(dK, dKr.reshape(1, 2, 2, 6, 8).sum(axis=2), atol=1e-14)
    np.testing.assert_allclose(dV, dVr.reshape(1, 2, 2, 6, 8).sum(axis=2), atol=1e-14)


def test_dense_matrix_form_on_tiny_case():
    # the textbook matrix expressions, evaluated with numpy
    q, k, v, dO = rnd((1, 1, 5, 4), 83), rnd((1, 1, 7, 4), 84), rnd((1, 1, 7, 4), 85), rnd((1, 1, 5, 4), 86)
    Q, K, V, G = (a[0, 0].astype(np.float64) for a in (q, k, v, dO))
    sc = 0.5
    S = Q @ K.T * sc
    P = np.exp(S - S.max(1, keepdims=True)); P /= P.sum(1, keepdims=True)
    dP = G @ V.T
    dS = P * (dP - (P * dP).sum(1, keepdims=True))
    dQ, dK, dV = oracle.bwd(q, k, v, dO)
    np.testing.assert_allclose(dQ[0, 0], dS @ K * sc, atol=1e-14)
    np.testing.assert_allclose(dK[0, 0], dS.T @ Q * sc, atol=1e-14)
    np.testing.assert_allclose(dV[0, 0], P.T @ G, atol=1e-14)


@pytest.mark.parametrize("masked", [False, True])
def test_blockwise_with_global_lse_sums_to_unsplit(masked):
    q, k, v, dO = rnd((2, 4, 6, 8), 87), rnd((2, 2, 24, 8), 88), rnd((2, 2, 24, 8), 89), rnd((2, 4, 6, 8), 90)
    kw = {}
    if masked:
        allow = np.random.default_rng(91).integers(0, 2, size=(3, 6)).astype(np.uint8)
        allow[2, :] = 0
        allow[0, 0] = 1
        kw["mask"] = oracle.Mask(allow, 2, 4)
    O, L = oracle.fwd(q, k, v, **kw)
    dQ, dK, dV = oracle.bwd(q, k, v, dO, **kw)
    acc = np.zeros_like(dQ)
    for a, b in ((0, 5), (5, 6), (6, 16), (16, 24)):
        dq, dk, dv = oracle.bwd_block(q, k, v, dO, O, L, a, b, **kw)
        acc += dq
        np.testing.assert_allclose(dk, dK[:, :, a:b], atol=1e-13)
        np.testing.assert_allclose(dv, dV[:, :, a:b], atol=1e-13)
    np.testing.assert_allclose(acc, dQ, atol=1e-13)


def test_sampled_rows_match_full():
    q, k, v, dO = rnd((2, 4, 7, 8), 92), rnd((2, 2, 15, 8), 93), rnd((2, 2, 15, 8), 94), rnd((2, 4, 7, 8), 95)
    allow = np.ones((4, 3), np.uint8); allow[1, 2] = 0; allow[3, 0] = 0
    mask = oracle.Mask(allow, 2, 5)
    dQ, dK, dV = oracle.bwd(q, k, v, dO, mask=mask)
    qr = np.array([[0, 0, 0], [1, 3, 6], [0, 2, 3]], np.int32)
    got = oracle.bwd_q_rows(q, k, v, dO, qr, mask=mask)
    for n, (b, h, i) in enumerate(qr):
        np.testing.assert_allclose(got[n], dQ[b, h, i], atol=1e-15)
    kr = np.array([[0, 1, 14], [1, 0, 0], [1, 1, 7]], np.int32)
    gk, gv = oracle.bwd_kv_rows(q, k, v, dO, kr, mask=mask)
    for n, (b, h, j) in enumerate(kr):
        np.testing.assert_allclose(gk[n], dK[b, h, j], atol=1e-15)
        np.testing.assert_allclose(gv[n], dV[b, h, j], atol=1e-15)
