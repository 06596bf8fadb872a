"""Pins of the Graph SGD oracle (oracle/sgd.c) against things other than itself (Section 6.1.4 names the method;
the update is the textbook one of Koren et al. 2009, the order stratified after Gemulla et al. 2011)."""
import numpy as np
import pytest

from oracle import sgd as osgd
from workloads import ratings as wl


def _one_rating(p, q, r):
    F = len(p)
    return (np.array([0, 1], np.int32), np.array([0], np.int32), np.array([r], np.float32),
            np.array([p], np.float64).reshape(1, F), np.array([q], np.float64).reshape(1, F))


def test_hand_worked_update():
    # p = (1, 2), q = (3, 4), r = 5, gamma = 0.1, lambda = 0.5: <p, q> = 11, e = -6,
    # p' = p + 0.1 (-6 q - 0.5 p) = (1 - 1.85, 2 - 2.5), q' = q + 0.1 (-6 p - 0.5 q) = (3 - 0.75, 4 - 1.4)
    rp, it, ra, P0, Q0 = _one_rating([1.0, 2.0], [3.0, 4.0], 5.0)
    P, Q = osgd.sgd(rp, it, ra, P0, Q0, 0.1, 0.5, 1, 1)
    assert np.allclose(P, [[-0.85, -0.5]], rtol=0, atol=1e-15)
    assert np.allclose(Q, [[2.25, 2.6]], rtol=0, atol=1e-15)
    P32, Q32 = osgd.sgd(rp, it, ra, P0, Q0, 0.1, 0.5, 1, 1, ordered_fp32=True)
    assert np.allclose(P32, [[-0.85, -0.5]], atol=1e-6) and np.allclose(Q32, [[2.25, 2.6]], atol=1e-6)


def test_update_is_a_gradient_step_of_the_regularised_squared_error():
    # (x' - x) / gamma must equal minus the gradient of L = 1/2 (r - <p, q>)^2 + lambda/2 (|p|^2 + |q|^2), taken here
    # by central differences of L itself.  Catches a wrong sign, p and q swapped, a dropped or doubled lambda term.
    rng = np.random.default_rng(3)
    F, lam, gamma, r = 5, 0.3, 1e-3, 2.5
    p, q = rng.standard_normal(F), rng.standard_normal(F)
    loss = lambda p_, q_: 0.5 * (r - p_ @ q_) ** 2 + 0.5 * lam * (p_ @ p_ + q_ @ q_)
    h = 1e-6
    gp = np.array([(loss(p + h * np.eye(F)[l], q) - loss(p - h * np.eye(F)[l], q)) / (2 * h) for l in range(F)])
    gq = np.array([(loss(p, q + h * np.eye(F)[l]) - loss(p, q - h * np.eye(F)[l])) / (2 * h) for l in range(F)])
    rp, it, ra, P0, Q0 = _one_rating(list(p), list(q), r)
    P, Q = osgd.sgd(rp, it, ra, P0, Q0, gamma, lam, 1, 1)
    assert np.allclose((P[0] - p) / gamma, -gp, atol=1e-7)
    assert np.allclose((Q[0] - q) / gamma, -gq, atol=1e-7)


def test_exact_low_rank_ratings_are_a_fixed_point_without_regularisation():
    rng = np.random.default_rng(5)
    U, I, F = 12, 9, 4
    A, Bm = rng.standard_normal((U, F)), rng.standard_normal((I, F))
    dense = rng.random((U, I)) < 0.5
    rp = np.concatenate([[0], np.cumsum(dense.sum(1))]).astype(np.int32)
    it = np.concatenate([np.flatnonzero(row) for row in dense]).astype(np.int32)
    users = np.repeat(np.arange(U), np.diff(rp))
    exact = np.einsum("ef,ef->e", A[users], Bm[it])
    # ratings are stored as fp32: make them exactly representable so that the error is exactly the rounding of <p, q>
    ra = exact.astype(np.float32)
    P, Q = osgd.sgd(rp, it, ra, A, Bm, 0.05, 0.0, 3, 3)
    assert np.abs(P - A).max() < 1e-6 and np.abs(Q - Bm).max() < 1e-6      # only the fp32 rounding of the ratings moves them
    P, Q = osgd.sgd(rp, it, ra, A, Bm, 0.05, 0.1, 1, 3)
    assert np.abs(P - A).max() > 1e-3                                      # with lambda > 0 the factors shrink


def _block_starts(rp, it, U, I, B):
    """Block k begins at the first id with ceil(k E / B) ratings or more before it (numpy, independent of the C code)."""
    E = int(rp[U])
    want = [-(-k * E // B) for k in range(1, B)]
    before_item = np.concatenate([[0], np.cumsum(np.bincount(it, minlength=I))])
    us = [0] + [int(np.searchsorted(rp, w, side="left")) for w in want] + [U]
    is_ = [0] + [int(np.searchsorted(before_item, w, side="left")) for w in want] + [I]
    return us, is_


def _brute_order(rp, it, U, I, B):
    us, is_ = _block_starts(rp, it, U, I, B)
    out = []
    for s in range(B):
        for a in range(B):
            b = (a + s) % B
            for u in range(us[a], us[a + 1]):
                for e in range(rp[u], rp[u + 1]):
                    if is_[b] <= it[e] < is_[b + 1]:
                        out.append(e)
    return out


@pytest.mark.parametrize("B", [1, 2, 3, 7, 16])
def test_order_is_the_stratified_one(B):
    r = wl.rmat_ratings(6, 700, seed=2)
    got = osgd.order(r.row_ptr, r.item, r.n_items, B)
    assert sorted(got) == list(range(r.n_ratings))                         # every rating once per iteration
    assert list(got) == _brute_order(r.row_ptr, r.item, r.n_users, r.n_items, B)
    us, is_ = _block_starts(r.row_ptr, r.item, r.n_users, r.n_items, B)
    ous, ois = osgd.blocks(r.row_ptr, r.item, r.n_items, B)
    assert list(ous) == us and list(ois) == is_
    # the cells of one stratum share neither a user block nor an item block
    users = np.repeat(np.arange(r.n_users), np.diff(r.row_ptr))
    a = np.searchsorted(np.array(us[1:B]), users[got], side="right")
    b = np.searchsorted(np.array(is_[1:B]), r.item[got], side="right")
    s = (b - a) % B
    assert np.all(np.diff(s) >= 0)                                         # strata in order
    for k in range(B):
        cells = set(zip(a[s == k], b[s == k]))
        assert len({x for x, _ in cells}) == len(cells) == len({y for _, y in cells})


def test_blocks_hold_about_the_same_number_of_ratings():
    r = wl.rmat_ratings(10, 1 << 15, seed=5)
    B = 16
    us, is_ = osgd.blocks(r.row_ptr, r.item, r.n_items, B)
    per_user_block = np.diff(r.row_ptr[us])
    per_item_block = np.diff(np.concatenate([[0], np.cumsum(np.bincount(r.item, minlength=r.n_items))])[is_])
    share = r.n_ratings / B
    assert per_user_block.sum() == per_item_block.sum() == r.n_ratings
    assert per_user_block.max() <= share + np.diff(r.row_ptr).max()        # a block overshoots by less than one row
    assert per_item_block.max() <= share + np.bincount(r.item).max()
    assert per_user_block.max() < 1.5 * share and per_item_block.max() < 1.5 * share   # on this graph: well balanced


def test_with_one_block_the_order_is_plain_row_order_and_matches_a_python_loop():
    r = wl.rmat_ratings(5, 200, seed=4)
    P0, Q0 = wl.initial_factors(r.n_users, r.n_items, 4, seed=1)
    gamma, lam = 0.02, 0.05
    P, Q = P0.astype(np.float64), Q0.astype(np.float64)
    for _ in range(2):
        for u in range(r.n_users):
            for e in range(r.row_ptr[u], r.row_ptr[u + 1]):
                i = r.item[e]
                err = float(r.rating[e]) - P[u] @ Q[i]
                P[u], Q[i] = P[u] + gamma * (err * Q[i] - lam * P[u]), Q[i] + gamma * (err * P[u] - lam * Q[i])
    Po, Qo = osgd.sgd(r.row_ptr, r.item, r.rating, P0, Q0, gamma, lam, 2, 1)
    assert np.abs(Po - P).max() < 1e-12 and np.abs(Qo - Q).max() < 1e-12


def test_rmse_falls_on_planted_low_rank_ratings():
    r = wl.rmat_ratings(9, 1 << 14, seed=7)
    P0, Q0 = wl.initial_factors(r.n_users, r.n_items, 16, seed=1)
    before = osgd.rmse(r.row_ptr, r.item, r.rating, P0, Q0)
    P, Q = osgd.sgd(r.row_ptr, r.item, r.rating, P0, Q0, 0.02, 0.02, 10, 8)
    after = osgd.rmse(r.row_ptr, r.item, r.rating, P, Q)
    assert after < 0.5 * before, (before, after)


def test_fp32_with_pinned_roundings_stays_close_to_fp64():
    r = wl.rmat_ratings(9, 1 << 14, seed=8)
    P0, Q0 = wl.initial_factors(r.n_users, r.n_items, 64, seed=2)
    P64, Q64 = osgd.sgd(r.row_ptr, r.item, r.rating, P0, Q0, 0.02, 0.02, 5, 8)
    P32, Q32 = osgd.sgd(r.row_ptr, r.item, r.rating, P0, Q0, 0.02, 0.02, 5, 8, ordered_fp32=True)
    assert np.abs(P32 - P64).max() < 1e-4 and np.abs(Q32 - Q64).max() < 1e-4
    assert np.abs(P32 - P64).max() > 0          # they are different computations


def test_inputs_are_seeded_sorted_and_distinct():
    a, b = wl.rmat_ratings(8, 5000, seed=3), wl.rmat_ratings(8, 5000, seed=3)
    assert np.array_equal(a.item, b.item) and np.array_equal(a.rating, b.rating) and np.array_equal(a.row_ptr, b.row_ptr)
    for u in range(a.n_users):
        row = a.item[a.row_ptr[u]:a.row_ptr[u + 1]]
        assert np.all(np.diff(row) > 0)
    assert a.row_ptr[-1] == a.n_ratings == len(a.rating) and 1.0 < a.rating.mean() < 5.0
