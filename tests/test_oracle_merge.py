"""Pins of the oracle's merge (the Rescale step of Algorithm 1): merging the partial results
of ANY split of the keys must reproduce the unsplit attention definition (the block-wise
decomposition of Section 2), plus the algebraic properties of a log-sum-exp merge."""
import numpy as np

import oracle
from test_oracle_forward import rnd


def parts_for(q, k, v, cuts, mask=None):
    Os, Ls = [], []
    for a, b in zip(cuts[:-1], cuts[1:]):
        m = None
        if mask is not None:          # kv_block == 1 in these tests so a column window is a slice
            m = oracle.Mask(mask.allow[:, a:b], mask.q_chunk, 1)
        O, L = oracle.fwd(q, k[:, :, a:b], v[:, :, a:b], mask=m)
        Os.append(O); Ls.append(L)
    return np.stack(Os), np.stack(Ls)


def test_any_split_equals_unsplit():
    q, k, v = rnd((2, 4, 6, 8), 40), rnd((2, 2, 37, 8), 41), rnd((2, 2, 37, 8), 42)
    O, L = oracle.fwd(q, k, v)
    for cuts in ([0, 37], [0, 10, 20, 30, 37], [0, 1, 2, 36, 37], [0, 5, 37], list(range(38))):
        Op, Lp = parts_for(q, k, v, cuts)
        Om, Lm = oracle.merge(Op, Lp)
        np.testing.assert_allclose(Om, O, atol=1e-13)
        np.testing.assert_allclose(Lm, L, atol=1e-13)
        perm = np.random.default_rng(len(cuts)).permutation(len(cuts) - 1)
        Om2, Lm2 = oracle.merge(Op[perm], Lp[perm])
        np.testing.assert_allclose(Om2, O, atol=1e-13)
        np.testing.assert_allclose(Lm2, L, atol=1e-13)


def test_split_with_mask_and_empty_parts():
    q, k, v = rnd((1, 2, 4, 8), 43), rnd((1, 2, 12, 8), 44), rnd((1, 2, 12, 8), 45)
    allow = np.ones((2, 12), np.uint8)
    allow[0, :6] = 0          # chunk 0 sees nothing in the first half
    allow[1, 3:] = 0          # chunk 1 sees only keys 0..2
    mask = oracle.Mask(allow, 2, 1)
    O, L = oracle.fwd(q, k, v, mask=mask)
    Op, Lp = parts_for(q, k, v, [0, 3, 6, 12], mask)
    assert np.isneginf(Lp[0, 0, :, :2]).all() and np.isneginf(Lp[2, 0, :, 2:]).all()
    Om, Lm = oracle.merge(Op, Lp)
    np.testing.assert_allclose(Om, O, atol=1e-13)
    np.testing.assert_allclose(Lm, L, atol=1e-13)


def test_pairwise_chain_from_identity_equals_nway():
    # Algorithm 1 applies Rescale once per round to a running (O, L); start = (0, -inf)
    q, k, v = rnd((1, 2, 5, 8), 46), rnd((1, 1, 40, 8), 47), rnd((1, 1, 40, 8), 48)
    Op, Lp = parts_for(q, k, v, [0, 10, 20, 30, 40])
    On, Ln = oracle.merge(Op, Lp)
    Or, Lr = np.zeros_like(Op[0]), np.full_like(Lp[0], -np.inf)
    for n in range(4):
        Or, Lr = oracle.merge(np.stack([Or, Op[n]]), np.stack([Lr, Lp[n]]))
    np.testing.assert_allclose(Or, On, atol=1e-13)
    np.testing.assert_allclose(Lr, Ln, atol=1e-13)


def test_identity_self_merge_and_all_empty():
    rng = np.random.default_rng(49)
    O = rng.standard_normal((3, 7, 4)); L = rng.standard_normal((3, 7)) * 5
    Z, NI = np.zeros_like(O), np.full_like(L, -np.inf)
    Om, Lm = oracle.merge(np.stack([O, Z]), np.stack([L, NI]))
    assert np.array_equal(Om, O) and np.array_equal(Lm, L)
    Om, Lm = oracle.merge(np.stack([O, O]), np.stack([L, L]))
    np.testing.assert_allclose(Om, O, atol=1e-15)
    np.testing.assert_allclose(Lm, L + np.log(2.0), atol=1e-14)
    Om, Lm = oracle.merge(np.stack([Z, Z]), np.stack([NI, NI]))
    assert np.all(Om == 0) and np.isneginf(Lm).all()


def test_weights_closed_form():
    # L = (ln 1, ln 3) -> weights (1/4, 3/4), L' = ln 4
    O = np.array([[[2.0, 0.0]], [[0.0, 8.0]]]); L = np.array([[0.0], [np.log(3.0)]])
    Om, Lm = oracle.merge(O, L)
    np.testing.assert_allclose(Om, [[0.5, 6.0]], atol=1e-15)
    np.testing.assert_allclose(Lm, [np.log(4.0)], atol=1e-15)


def test_large_magnitude_lse_is_stable():
    O = np.ones((2, 1, 3)); O[1] *= 3
    L = np.array([[800.0], [801.0]])
    Om, Lm = oracle.merge(O, L)
    w1 = 1 / (1 + np.exp(-1.0))
    np.testing.assert_allclose(Om, 1 * (1 - w1) + 3 * w1, atol=1e-14)
    np.testing.assert_allclose(Lm, 801 + np.log1p(np.exp(-1.0)), atol=1e-12)
