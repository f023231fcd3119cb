"""Pins for the oracle's neighbourhood definition (CPU only).

What fixes the expected values here is the paper, not the oracle:
  * Section 3.1: a query attends to its k nearest neighbours (per axis: the k positions
    closest to it) -- checked by brute-force nearest-k selection;
  * Section 1 / Appendix figure "3x3 NA on a 7x7 map": every query keeps exactly k*k keys,
    the window being repeated at corners -- checked against the hand-written fixture
    tests/golden/na_3x3_on_7x7_windows.txt and by counting.
"""
import os

import numpy as np
import pytest

KS = (3, 5, 7, 9, 11, 13, 15, 17, 21)   # the sizes the paper tunes for, and a few beyond them


def nearest_k_bruteforce(i, L, k):
    """The k positions of [0, L) closest to i, by explicit sorting on distance.
    Also checks that the choice is unambiguous: the (k+1)-th candidate is strictly farther."""
    order = sorted(range(L), key=lambda j: abs(j - i))
    if L > k:
        assert abs(order[k] - i) > abs(order[k - 1] - i), (i, L, k)
    return sorted(order[:k])


@pytest.mark.parametrize("k", KS)
def test_window_is_the_k_nearest_positions(oracle, k):
    for L in range(k, max(21, k + 8)):
        for i in range(L):
            s = oracle.window_start(i, L, k)
            assert list(range(s, s + k)) == nearest_k_bruteforce(i, L, k), (L, k, i)


def test_golden_3x3_on_7x7(oracle):
    path = os.path.join(os.path.dirname(__file__), "golden", "na_3x3_on_7x7_windows.txt")
    key_index, _ = oracle.indices(7, 7, 3)
    n = 0
    for line in open(path):
        if line.startswith("#") or not line.strip():
            continue
        lhs, rhs = line.split(":")
        qy, qx = map(int, lhs.split())
        fy, fx = map(int, rhs.split())
        expect = [(fy + a) * 7 + (fx + c) for a in range(3) for c in range(3)]
        assert key_index[qy, qx].tolist() == expect
        n += 1
    assert n == 49


@pytest.mark.parametrize("H,W,k", [(7, 7, 3), (14, 14, 3), (9, 12, 5), (7, 7, 7), (20, 13, 13), (56, 56, 7), (10, 17, 9),
                                   (15, 15, 15), (23, 30, 15), (25, 22, 21)])
def test_every_query_sees_exactly_kk_distinct_inbounds_keys(oracle, H, W, k):
    key_index, rpb_index = oracle.indices(H, W, k)
    assert key_index.shape == (H, W, k * k)
    assert key_index.min() >= 0 and key_index.max() < H * W
    for qy in range(H):
        for qx in range(W):
            keys = key_index[qy, qx]
            assert len(set(keys.tolist())) == k * k
            ky, kx = keys // W, keys % W
            # the span is a k x k square that contains the query
            assert ky.max() - ky.min() == k - 1 and kx.max() - kx.min() == k - 1
            assert ky.min() <= qy <= ky.max() and kx.min() <= qx <= kx.max()
            # raster order over ascending key coordinates
            assert np.all(np.diff(keys.reshape(k, k), axis=1) == 1)
            assert np.all(np.diff(keys.reshape(k, k), axis=0) == W)
            # bias cell = relative offset + (k - 1) on each axis
            u, v = rpb_index[qy, qx] // (2 * k - 1), rpb_index[qy, qx] % (2 * k - 1)
            assert np.array_equal(u, ky - qy + k - 1) and np.array_equal(v, kx - qx + k - 1)
            assert u.min() >= 0 and u.max() <= 2 * k - 2 and v.min() >= 0 and v.max() <= 2 * k - 2


def test_interior_queries_are_centred(oracle):
    H, W, k = 16, 19, 7
    r = k // 2
    key_index, rpb_index = oracle.indices(H, W, k)
    for qy in range(r, H - r):
        for qx in range(r, W - r):
            assert key_index[qy, qx, (k * k) // 2] == qy * W + qx
            # interior queries only touch the central k x k block of the bias table
            u = rpb_index[qy, qx] // (2 * k - 1)
            assert u.min() == r and u.max() == r + k - 1


def test_max_neighbourhood_is_the_whole_map(oracle):
    # Section 3.1: at the maximum neighbourhood size NA's span is all of self attention's
    for L in (3, 5, 7, 13):
        key_index, _ = oracle.indices(L, L, L)
        assert np.array_equal(key_index, np.broadcast_to(np.arange(L * L, dtype=np.int32), (L, L, L * L)))
