"""Pins for the oracle's topologies: facts the paper's definitions and the
mathematics fix, none of which re-use the oracle's own formulas."""

import math
import os

import numpy as np
import pytest

from oracle import topology as T


def test_five_node_example_in_and_out_sets(golden_dir):
    # Section "Network topology": N(5) = {1,2,3,4}, M(5) = {1,3}.
    edges = []
    with open(os.path.join(golden_dir, "five_node_example.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                a, b = line.split()
                edges.append((int(a) - 1, int(b) - 1))
    out = {j: sorted(b for a, b in edges if a == j) for j in range(5)}
    inn = T.in_lists_from_out_lists(out)
    assert [v + 1 for v in inn[4]] == [1, 2, 3, 4]
    assert [v + 1 for v in out[4]] == [1, 3]
    # a pull matrix on this graph: w_ij nonzero only if (j,i) is an edge or i == j (eq. wij)
    W = T.uniform_from_neighbor_sets(inn)
    D = T.to_dense(W)
    for i in range(5):
        for j in range(5):
            assert (D[i, j] != 0) == (i == j or (j, i) in edges)
    assert T.in_lists(W) == inn and T.out_lists(W) == out
    np.testing.assert_allclose(D.sum(axis=1), 1.0, atol=1e-15)     # pull: W 1 = 1
    assert abs(D.sum(axis=0) - 1.0).max() > 0.1                    # but not push


def test_ring16_is_the_third_third_third_circulant():
    n = 16
    D = T.to_dense(T.ring(n))
    expect = np.zeros((n, n))
    for i in range(n):
        for j in (i - 1, i, i + 1):
            expect[i, j % n] = 1 / 3
    np.testing.assert_allclose(D, expect, atol=1e-16)
    # circulant closed form: eigenvalues (1 + 2 cos(2 pi m / n)) / 3
    ev = np.sort(np.linalg.eigvalsh(D))[::-1]
    closed = np.sort([(1 + 2 * math.cos(2 * math.pi * m / n)) / 3 for m in range(n)])[::-1]
    np.testing.assert_allclose(ev, closed, atol=1e-14)
    assert abs(ev[1] - 0.9492530216741911) < 1e-14


@pytest.mark.parametrize("n,deg,lam2", [(64, 11, 2 / 3), (32, 9, 3 / 5), (8, 5, 1 / 3), (16, 7, 0.5)])
def test_static_exponential_structure_and_lambda2(n, deg, lam2):
    W = T.static_exponential(n)
    D = T.to_dense(W)
    p = int(math.log2(n))
    S = set()
    for k in range(p):
        S.add(2 ** k % n)
        S.add(-(2 ** k) % n)
    assert len(S) == deg
    for i in range(n):
        nz = {j for j in range(n) if D[i, j] != 0}
        assert nz == {(i + s) % n for s in S} | {i}
        assert all(abs(D[i, j] - 1 / (deg + 1)) < 1e-16 for j in nz)
    np.testing.assert_allclose(D, D.T, atol=0)                       # symmetric
    np.testing.assert_allclose(D.sum(0), 1.0, atol=1e-15)            # doubly stochastic
    np.testing.assert_allclose(D.sum(1), 1.0, atol=1e-15)
    mags = np.sort(np.abs(np.linalg.eigvalsh(D)))[::-1]
    assert abs(mags[0] - 1) < 1e-14
    assert abs(mags[1] - lam2) < 1e-13        # |lambda_2| = (p-2)/p, at the alternating vector


def test_static_exponential_non_power_of_two():
    n = 12                                    # offsets 1,2,4,8 -> +-: {1,11,2,10,4,8} (8 == -4)
    D = T.to_dense(T.static_exponential(n))
    assert {j for j in range(n) if D[0, j] != 0} == {0, 1, 11, 2, 10, 4, 8}
    np.testing.assert_allclose(D.sum(0), 1.0, atol=1e-15)
    np.testing.assert_allclose(D.sum(1), 1.0, atol=1e-15)


@pytest.mark.parametrize("n", [2, 8, 256])
def test_one_peer_product_is_exact_average(n):
    # prod_r (I + P^(2^r))/2 = 11^T / n : every shift s in [0,n) has one binary expansion.
    R = T.one_peer_rounds(n)
    assert R == int(math.log2(n))
    P = np.eye(n)
    for r in range(R):
        D = T.to_dense(T.one_peer_exponential(n, r))
        for i in range(n):                    # pulls from the higher index, weights 1/2, 1/2
            assert D[i, i] == 0.5 and D[i, (i + 2 ** r) % n] == 0.5
        np.testing.assert_allclose(D.sum(0), 1.0, atol=0)
        P = D @ P
    assert np.array_equal(P, np.full((n, n), 1.0 / n))               # dyadic: exact in fp64
    # the schedule is periodic with period R
    assert T.one_peer_exponential(n, R + 1) == T.one_peer_exponential(n, 1)


def test_one_peer_degenerate_sizes():
    assert T.one_peer_exponential(1, 0) == {0: [(0, 1.0)]}
    assert T.one_peer_rounds(1) == 1
    D = T.to_dense(T.one_peer_exponential(3, 1))   # offsets 1,2 ; round 1 -> +2
    assert D[0, 2] == 0.5 and D[1, 0] == 0.5 and D[2, 1] == 0.5


def test_splitmix64_known_answers():
    # First outputs of the published splitmix64 generator seeded with 0 and with
    # 1234567 (widely reproduced test vectors of the reference C program).
    g = T.SplitMix64(0)
    assert [g.next() for _ in range(3)] == [
        0xE220A8397B1DCDAF, 0x6E789E6AA1B965F4, 0x06C45D188009454F]
    g = T.SplitMix64(1234567)
    assert [g.next() for _ in range(2)] == [6457827717110365317, 3203168211198807973]


def test_random_directed_push_graph_structure():
    n, k = 128, 4
    W, seed = T.random_directed_push(n, k, 401)
    assert seed >= 401
    D = T.to_dense(W)
    np.testing.assert_allclose(D.sum(axis=0), 1.0, atol=1e-15)      # push: 1^T W = 1^T
    assert abs(D.sum(axis=1) - 1).max() > 1e-3                      # not a pull matrix
    for j in range(n):
        col = D[:, j]
        assert col[j] == 0.2
        assert (col != 0).sum() == k + 1 and set(col[col != 0]) == {0.2}
    out = T.out_lists(W)
    assert all(len(out[j]) == k and j not in out[j] for j in range(n))
    assert T.is_strongly_connected(out)
    # strong connectivity the hard way: (I + A)^(n-1) has no zero entry
    A = (D != 0).astype(np.float64)
    R = np.linalg.matrix_power(A, n - 1)
    assert (R > 0).all()
    # the draw is a pure function of the seed, and the earlier seeds were rejected
    W2, seed2 = T.random_directed_push(n, k, 401)
    assert W2 == W and seed2 == seed
    for s in range(401, seed):
        assert not T.is_strongly_connected(T.draw_out_targets(n, k, s))


def test_strong_connectivity_checker_on_known_graphs():
    cyc = {0: [1], 1: [2], 2: [0]}
    assert T.is_strongly_connected(cyc)
    chain = {0: [1], 1: [2], 2: []}
    assert not T.is_strongly_connected(chain)
    src = {0: [1], 1: [2], 2: [1]}            # node 0 has no in-neighbor
    assert not T.is_strongly_connected(src)


def test_draw_uses_every_target_about_equally():
    # Fisher-Yates prefix: each other agent is a target with probability k/(n-1).
    n, k = 16, 4
    cnt = np.zeros((n, n))
    for s in range(400):
        out = T.draw_out_targets(n, k, 9000 + s)
        for j in range(n):
            assert len(set(out[j])) == k and j not in out[j]
            for i in out[j]:
                cnt[j, i] += 1
    off = cnt[~np.eye(n, dtype=bool)]
    assert abs(off.mean() - 400 * k / (n - 1)) < 1e-9
    assert off.min() > 60 and off.max() < 160          # expectation 106.7, sd ~ 8.8


def test_csr_round_trip():
    W = T.static_exponential(8)
    rowptr, col, wgt = [0], [], []
    for i in range(8):
        for j, w in W[i]:
            col.append(j)
            wgt.append(w)
        rowptr.append(len(col))
    assert T.from_csr(rowptr, col, wgt) == W
