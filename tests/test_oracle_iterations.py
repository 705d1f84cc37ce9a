"""Pins for the oracle's iterations against library routines, closed forms,
invariants and limiting cases.  A transposed operand, a dropped term, a wrong
sign or a wrong index in ``oracle.iterations`` fails at least one test here."""

import math

import numpy as np
import pytest
import scipy.sparse as sp
import torch

from oracle import iterations as O
from oracle import topology as T


def _rand_W(n, rng, density=0.4):
    """A random non-symmetric, non-stochastic weight matrix with a full diagonal."""
    D = rng.normal(size=(n, n)) * (rng.random((n, n)) < density)
    D[np.arange(n), np.arange(n)] = rng.normal(size=n) + 2.0
    return D


# ---------------------------------------------------------------- mix
def test_mix_equals_dense_and_scipy_spmm():
    rng = np.random.default_rng(1)
    n, d = 7, 13
    D = _rand_W(n, rng)
    assert abs(D - D.T).max() > 0.5                      # asymmetric: catches a transposed W
    X = rng.normal(size=(n, d))
    got = O.mix(X, T.from_dense(D))
    np.testing.assert_allclose(got, D @ X, rtol=0, atol=1e-13)
    np.testing.assert_allclose(got, sp.csr_matrix(D) @ X, rtol=0, atol=1e-13)


def test_mix_brute_force_scalar_loops():
    rng = np.random.default_rng(2)
    n, d = 5, 3
    D = _rand_W(n, rng)
    X = rng.normal(size=(n, d))
    got = O.mix(X, T.from_dense(D))
    for i in range(n):
        for c in range(d):
            s = 0.0
            for j in range(n):
                s += D[i, j] * X[j, c]       # w_ij scales x_j (eq. wij)
            assert abs(got[i, c] - s) < 1e-13


def test_mix_mean_preserved_iff_columns_sum_to_one():
    rng = np.random.default_rng(3)
    X = rng.normal(size=(64, 50))
    W = T.static_exponential(64)
    Xn = O.mix(X, W)
    np.testing.assert_allclose(Xn.sum(0), X.sum(0), atol=64 * 1e-15 * 10)
    # a pull-only (row-stochastic) matrix fixes consensus but does not preserve the mean
    inn = {i: [(i + 1) % 5] if i else [1, 2, 3, 4] for i in range(5)}
    Wp = T.uniform_from_neighbor_sets(inn)
    Xc = np.tile(rng.normal(size=(1, 6)), (5, 1))
    np.testing.assert_allclose(O.mix(Xc, Wp), Xc, atol=1e-15)
    X5 = rng.normal(size=(5, 6))
    assert abs(O.mix(X5, Wp).sum(0) - X5.sum(0)).max() > 1e-3


def test_mix_does_not_modify_input_and_empty_width():
    X = np.ones((4, 3))
    X0 = X.copy()
    O.mix(X, T.ring(4))
    assert np.array_equal(X, X0)
    assert O.mix(np.zeros((4, 0)), T.ring(4)).shape == (4, 0)


def test_consensus_contracts_at_lambda2_ring_and_static_exp():
    rng = np.random.default_rng(4)
    for W, lam2 in ((T.ring(16), 0.9492530216741911), (T.static_exponential(64), 2 / 3)):
        n = len(W)
        X = rng.uniform(-1, 1, size=(n, 40))
        e_prev = O.consensus_error(X)
        ratios = []
        for k in range(50):
            X = O.mix(X, W)
            e = O.consensus_error(X)
            assert e <= lam2 * e_prev * (1 + 1e-12)       # hard bound every round
            ratios.append(e / e_prev)
            e_prev = e
        assert ratios[-1] <= lam2 + 1e-12
        assert ratios[-1] > 0.9 * lam2                     # and approaches it from below
    # static exp: error after 50 rounds is below (2/3)^50 of the start
    assert (2 / 3) ** 50 < 1.6e-9


def test_consensus_error_definition():
    X = np.array([[1.0, 2.0], [3.0, 6.0]])
    # means (2,4): deviations (+-1, +-2) -> sqrt(1+1+4+4)
    assert abs(O.consensus_error(X) - math.sqrt(10)) < 1e-15
    np.testing.assert_allclose(O.column_mean(X), [2.0, 4.0])


def test_one_peer_eight_rounds_give_exact_mean():
    rng = np.random.default_rng(5)
    n = 256
    X = rng.normal(size=(n, 17))
    mean = X.mean(0)
    Y = X
    for r in range(8):
        Y = O.mix(Y, T.one_peer_exponential(n, r))
        if r < 7:
            assert abs(Y - mean).max() > 1e-3
    np.testing.assert_allclose(Y, np.tile(mean, (n, 1)), atol=4e-16 * 8)


def test_static_is_special_case_of_push_pull_split():
    # eq. 2bzbz09 with r*s = w reduces to eq. dsgd-2; pure push (r=1,s=w) == pure pull (r=w,s=1).
    rng = np.random.default_rng(6)
    n = 9
    D = _rand_W(n, rng)
    W = T.from_dense(D)
    X = rng.normal(size=(n, 5))
    selfw = {i: D[i, i] for i in range(n)}
    nb = {i: [(j, w) for j, w in W[i] if j != i] for i in range(n)}
    ones = {i: [(j, 1.0) for j, _ in nb[i]] for i in range(n)}
    pull = O.mix_push_pull(X, selfw, nb, ones)
    push = O.mix_push_pull(X, selfw, ones, nb)
    np.testing.assert_allclose(pull, D @ X, atol=1e-13)
    np.testing.assert_allclose(push, D @ X, atol=1e-13)
    half = {i: [(j, math.sqrt(abs(w))) for j, w in nb[i]] for i in range(n)}
    halfs = {i: [(j, math.copysign(math.sqrt(abs(w)), w)) for j, w in nb[i]] for i in range(n)}
    np.testing.assert_allclose(O.mix_push_pull(X, selfw, half, halfs), D @ X, atol=1e-13)


# ---------------------------------------------------------------- push-sum
def test_pushsum_invariants_and_limit():
    rng = np.random.default_rng(7)
    n = 128
    W, _ = T.random_directed_push(n, 4, 401)
    X = rng.normal(5, 2, size=(n, 11))
    xbar = X.mean(0)
    p = np.ones(n)
    s0 = X.sum(0)
    for k in range(100):
        X, p, Y = O.pushsum_step(X, p, W)
        np.testing.assert_allclose(X.sum(0), s0, rtol=1e-13)      # 1^T W = 1^T
        assert abs(p.sum() - n) < 1e-11                           # sum of p stays n
        if k == 0:
            assert abs(Y - xbar).max() > 0.1
    np.testing.assert_allclose(Y, np.tile(xbar, (n, 1)), atol=1e-12)
    assert abs(X / p[:, None] - Y).max() == 0.0
    assert abs(p - 1).max() > 0.05                                 # the correction is not trivial


def test_pushsum_weights_converge_to_perron_vector_tiny():
    # brute force at n=6: p_k = W^k 1 -> n * pi, pi the right Perron vector of column-stochastic W
    W, _ = T.random_directed_push(6, 2, 7)
    D = T.to_dense(W)
    ev, V = np.linalg.eig(D)
    k = int(np.argmax(ev.real))
    pi = np.real(V[:, k])
    pi = pi / pi.sum()
    X = np.arange(12.0).reshape(6, 2)
    p = np.ones(6)
    for _ in range(200):
        X, p, Y = O.pushsum_step(X, p, W)
    np.testing.assert_allclose(p, 6 * pi, atol=1e-12)
    np.testing.assert_allclose(p, np.linalg.matrix_power(D, 200) @ np.ones(6), atol=1e-12)
    np.testing.assert_allclose(Y, np.tile(np.arange(12.0).reshape(6, 2).mean(0), (6, 1)), atol=1e-11)


def test_pushsum_without_correction_is_biased():
    # the plain iterate x (no division by p) does not reach the mean on a push-only graph
    W, _ = T.random_directed_push(16, 3, 11)
    rng = np.random.default_rng(8)
    X = rng.normal(size=(16, 4))
    xbar = X.mean(0)
    p = np.ones(16)
    for _ in range(300):
        X, p, Y = O.pushsum_step(X, p, W)
    assert abs(Y - xbar).max() < 1e-12
    assert abs(X - xbar).max() > 1e-2


# ---------------------------------------------------------------- least-squares gradient
def test_ls_grad_is_gradient_of_half_squared_residual():
    rng = np.random.default_rng(9)
    n, m, d = 3, 4, 6
    A = rng.normal(size=(n, m, d))
    b = rng.normal(size=(n, m))
    X = rng.normal(size=(n, d))
    G = O.ls_grad(A, b, X)
    f = lambda i, x: 0.5 * np.sum((A[i] @ x - b[i]) ** 2)
    h = 1e-6
    for i in range(n):
        for c in range(d):
            e = np.zeros(d)
            e[c] = h
            fd = (f(i, X[i] + e) - f(i, X[i] - e)) / (2 * h)
            assert abs(G[i, c] - fd) < 1e-6
    At = torch.tensor(A)
    xt = torch.tensor(X, requires_grad=True)
    loss = 0.5 * ((torch.einsum("imd,id->im", At, xt) - torch.tensor(b)) ** 2).sum()
    loss.backward()
    np.testing.assert_allclose(G, xt.grad.numpy(), atol=1e-12)


# ---------------------------------------------------------------- ATC / AWC
def test_atc_single_agent_is_gradient_descent_closed_form():
    # n=1, W=[1]: x_k = (I - alpha A^T A)^k x_0 + ... ; closed form through the SVD of A.
    rng = np.random.default_rng(10)
    m, d, alpha, K = 4, 7, 0.05, 60
    A = rng.normal(size=(1, m, d))
    b = rng.normal(size=(1, m))
    W = {0: [(0, 1.0)]}
    X = np.zeros((1, d))
    for _ in range(K):
        X = O.atc_step(X, O.ls_grad(A, b, X), W, alpha)
    U, s, Vt = np.linalg.svd(A[0], full_matrices=False)
    coef = (1 - (1 - alpha * s ** 2) ** K) / s * (U.T @ b[0])
    np.testing.assert_allclose(X[0], Vt.T @ coef, atol=1e-12)
    # and the limit is the pseudo-inverse solution
    for _ in range(5000):
        X = O.atc_step(X, O.ls_grad(A, b, X), W, alpha)
    np.testing.assert_allclose(X[0], np.linalg.pinv(A[0]) @ b[0], atol=1e-9)


def test_atc_with_global_averaging_is_centralized_gd():
    # W = 11^T/n and equal starts: x <- x - (alpha/n) sum_i g_i  (eq. sgd-2)
    rng = np.random.default_rng(11)
    n, m, d, alpha = 4, 3, 5, 0.02
    A = rng.normal(size=(n, m, d))
    b = rng.normal(size=(n, m))
    W = T.from_dense(np.full((n, n), 1.0 / n))
    x = rng.normal(size=d)
    X = np.tile(x, (n, 1))
    for _ in range(7):
        g = sum(A[i].T @ (A[i] @ x - b[i]) for i in range(n))
        x = x - alpha / n * g
        X = O.atc_step(X, O.ls_grad(A, b, X), W, alpha)
    np.testing.assert_allclose(X, np.tile(x, (n, 1)), atol=1e-13)


def test_atc_and_awc_against_dense_formulas():
    rng = np.random.default_rng(12)
    n, d, alpha = 6, 4, 0.3
    D = _rand_W(n, rng)
    W = T.from_dense(D)
    X = rng.normal(size=(n, d))
    G = rng.normal(size=(n, d))
    np.testing.assert_allclose(O.atc_step(X, G, W, alpha), D @ (X - alpha * G), atol=1e-13)
    np.testing.assert_allclose(O.awc_step(X, G, W, alpha), D @ X - alpha * G, atol=1e-13)
    assert abs(O.atc_step(X, G, W, alpha) - O.awc_step(X, G, W, alpha)).max() > 1e-2
    Z = np.zeros_like(G)
    np.testing.assert_allclose(O.atc_step(X, Z, W, alpha), O.awc_step(X, Z, W, alpha), atol=0)
    np.testing.assert_allclose(O.atc_step(X, G, W, 0.0), O.mix(X, W), atol=0)
    np.testing.assert_allclose(O.awc_step(X, G, W, 0.0), O.mix(X, W), atol=0)


def test_dgd_on_ring_converges_near_least_squares_solution():
    # DGD (eqs. dgd-1, dgd-2) with a small step lands in a neighbourhood of x*; all agents agree
    rng = np.random.default_rng(13)
    n, m, d, alpha = 8, 6, 5, 0.01
    A = rng.normal(size=(n, m, d))
    xs = rng.normal(size=d)
    b = np.einsum("imd,d->im", A, xs)            # consistent system: x* is every agent's minimiser
    W = T.ring(n)
    X = np.zeros((n, d))
    for _ in range(4000):
        X = O.atc_step(X, O.ls_grad(A, b, X), W, alpha)
    np.testing.assert_allclose(X, np.tile(xs, (n, 1)), atol=1e-8)


# ---------------------------------------------------------------- momentum
def test_dmsgd_beta_zero_is_atc():
    rng = np.random.default_rng(14)
    W = T.static_exponential(8)
    X, M, G = (rng.normal(size=(8, 5)) for _ in range(3))
    Xn, Mn = O.dmsgd_atc_step(X, M, G, W, 0.1, 0.0)
    np.testing.assert_allclose(Xn, O.atc_step(X, G, W, 0.1), atol=0)
    np.testing.assert_allclose(Mn, G, atol=0)


def test_dmsgd_single_agent_matches_torch_sgd_momentum():
    rng = np.random.default_rng(15)
    d, alpha, beta, lam = 6, 0.1, 0.9, 1.0
    c = rng.normal(size=d)
    noise = rng.normal(size=(12, d))
    p = torch.zeros(d, dtype=torch.float64, requires_grad=True)
    opt = torch.optim.SGD([p], lr=alpha, momentum=beta, dampening=0, nesterov=False)
    X = np.zeros((1, d))
    M = np.zeros((1, d))
    W = {0: [(0, 1.0)]}
    for k in range(12):
        G = O.quadratic_noise_grad(X, c[None], noise[k][None], lam, 0.1)
        X, M = O.dmsgd_atc_step(X, M, G, W, alpha, beta)
        opt.zero_grad()
        p.grad = lam * (p.detach() - torch.tensor(c)) + 0.1 * torch.tensor(noise[k])
        opt.step()
        np.testing.assert_allclose(X[0], p.detach().numpy(), atol=1e-13)


def test_dmsgd_noise_free_two_by_two_recurrence():
    # per coordinate, W = I: [x;m]' = [[1-a l, -a b],[l, b]] [x;m] + [a l c; -l c]; fixed point x=c, m=0
    alpha, beta, lam, c = 0.1, 0.9, 1.0, 0.7
    Amat = np.array([[1 - alpha * lam, -alpha * beta], [lam, beta]])
    off = np.array([alpha * lam * c, -lam * c])
    ev, V = np.linalg.eig(Amat)
    z0 = np.array([0.0, 0.0]) - np.array([c, 0.0])
    X = np.zeros((1, 1))
    M = np.zeros((1, 1))
    W = {0: [(0, 1.0)]}
    for k in range(1, 30):
        G = O.quadratic_noise_grad(X, np.array([[c]]), np.zeros((1, 1)), lam, 0.1)
        X, M = O.dmsgd_atc_step(X, M, G, W, alpha, beta)
        zk = np.real(V @ (ev ** k * np.linalg.solve(V, z0.astype(complex)))) + np.array([c, 0.0])
        assert abs(X[0, 0] - zk[0]) < 1e-12 and abs(M[0, 0] - zk[1]) < 1e-12
    assert np.allclose(Amat @ np.array([c, 0.0]) + off, [c, 0.0])


def test_dmsgd_column_sums():
    rng = np.random.default_rng(16)
    W = T.static_exponential(32)
    X, M, G = (rng.normal(size=(32, 9)) for _ in range(3))
    Xn, Mn = O.dmsgd_atc_step(X, M, G, W, 0.1, 0.9)
    np.testing.assert_allclose(Xn.sum(0), (X - 0.1 * Mn).sum(0), atol=1e-12)
    np.testing.assert_allclose(Mn, 0.9 * M + G, atol=0)


def test_dmsgd_bf16_storage_equals_plain_step_when_nothing_needs_rounding():
    # One-peer weights (1/2, 1/2), alpha = 1/4, beta = 1/2, X integers, G multiples of 4, M multiples
    # of 8: m' = beta m + g is a multiple of 4, x - alpha m' an integer, the mix a multiple of 1/2
    # below 64 in magnitude -- seven significant bits, exact in bfloat16.  The storage twin then has
    # nothing to round and must return the plain step's values bit for bit.
    rng = np.random.default_rng(41)
    n, d = 8, 33
    W = T.one_peer_exponential(n, 1)
    X = rng.integers(-8, 9, size=(n, d)).astype(np.float32)
    G = (4 * rng.integers(-4, 5, size=(n, d))).astype(np.float32)
    M = (8 * rng.integers(-4, 5, size=(n, d))).astype(np.float32)
    Xs, Ms = O.dmsgd_atc_step_bf16_storage(X, M, G, W, 0.25, 0.5)
    Xp, Mp = O.dmsgd_atc_step(X, M, G, W, 0.25, 0.5)
    assert Xs.dtype == np.float32 and Ms.dtype == np.float32
    np.testing.assert_array_equal(Xs.astype(np.float64), Xp)
    np.testing.assert_array_equal(Ms.astype(np.float64), Mp)
    assert np.array_equal(O.round_to_bf16(Xs), Xs)           # the guard: the result is a bfloat16 value


def test_dmsgd_bf16_storage_hand_worked_ties_and_rounding_order():
    one = {0: [(0, 1.0)]}
    f = lambda v: np.array([[v]], dtype=np.float32)
    # x' = 1 - 2^-8 * (-1) = 1 + 2^-8: halfway between the bfloat16 values 1 (even) and 1 + 2^-7 (odd)
    Xs, Ms = O.dmsgd_atc_step_bf16_storage(f(1.0), f(0.0), f(-1.0), one, 2.0 ** -8, 0.0)
    assert Xs[0, 0] == 1.0 and Ms[0, 0] == -1.0
    # x' = 1 + 3 * 2^-8: halfway between 1 + 2^-7 (odd) and 1 + 2^-6 (even)
    Xs, _ = O.dmsgd_atc_step_bf16_storage(f(1.0), f(0.0), f(-3.0), one, 2.0 ** -8, 0.0)
    assert Xs[0, 0] == 1.0 + 2.0 ** -6
    # just above / below a tie go to the nearer neighbour
    Xs, _ = O.dmsgd_atc_step_bf16_storage(f(1.0), f(0.0), f(-1.0 - 2.0 ** -7), one, 2.0 ** -8, 0.0)
    assert Xs[0, 0] == 1.0 + 2.0 ** -7
    # the momentum is rounded to fp32 (ties to even): 1 + 2^-24 -> 1, 1 + 3 * 2^-24 -> 1 + 2^-22
    _, Ms = O.dmsgd_atc_step_bf16_storage(f(0.0), f(1.0), f(2.0 ** -24), one, 0.0, 1.0)
    assert Ms[0, 0] == np.float32(1.0)
    _, Ms = O.dmsgd_atc_step_bf16_storage(f(0.0), f(1.0), f(3 * 2.0 ** -24), one, 0.0, 1.0)
    assert Ms[0, 0] == np.float32(1.0 + 2.0 ** -22)
    # order of the roundings: x' is formed from the STORED (fp32) momentum.  m' = 1 + 2^-8 + 2^-30
    # stores as 1 + 2^-8; x' = 0 - (-1) m' is then exactly the tie 1 + 2^-8 and goes to 1 (even).
    # Rounding the unrounded m' straight to bfloat16 would give 1 + 2^-7 instead.
    Xs, Ms = O.dmsgd_atc_step_bf16_storage(f(0.0), f(1.0 + 2.0 ** -8), f(2.0 ** -30), one, -1.0, 1.0)
    assert Ms[0, 0] == np.float32(1.0 + 2.0 ** -8)
    assert Xs[0, 0] == 1.0


# ---------------------------------------------------------------- Exact-Diffusion (next row)
def test_exact_diffusion_fixed_point_is_least_squares_solution():
    rng = np.random.default_rng(17)
    n, m, d, alpha = 8, 4, 6, 0.02          # n*m >= d: the stacked system has full column rank
    A = rng.normal(size=(n, m, d))
    b = rng.normal(size=(n, m))
    W = T.ring(n)
    X = np.zeros((n, d))
    psi_prev = X.copy()                     # psi^{(-1)} = x^{(0)}
    for _ in range(20000):
        X, psi_prev = O.exact_diffusion_step(X, psi_prev, O.ls_grad(A, b, X), W, alpha)
    xs = np.linalg.lstsq(A.reshape(n * m, d), b.reshape(n * m), rcond=None)[0]
    np.testing.assert_allclose(X, np.tile(xs, (n, 1)), atol=1e-8)


def test_exact_diffusion_step_against_dense_formula_and_two_step_recursion():
    rng = np.random.default_rng(42)
    n, d, alpha = 7, 4, 0.05
    D = _rand_W(n, rng)
    W = T.from_dense(D)
    X, Psi, G = (rng.normal(size=(n, d)) for _ in range(3))
    Xn, psi = O.exact_diffusion_step(X, Psi, G, W, alpha)
    # eqs. ed-1..ed-3 in matrix form: psi = X - alpha G, X' = W (2X - alpha G - Psi_prev)
    np.testing.assert_allclose(psi, X - alpha * G, atol=0)
    np.testing.assert_allclose(Xn, D @ (2 * X - alpha * G - Psi), atol=1e-13)
    # Eliminating psi from two consecutive iterations leaves the two-step recursion
    #   x^{k+1} = W (2 x^k - x^{k-1} - alpha (g^k - g^{k-1})),  started with x^1 = W (x^0 - alpha g^0).
    A = rng.normal(size=(n, 3, d))
    b = rng.normal(size=(n, 3))
    X0 = rng.normal(size=(n, d))
    xs, gs = [X0], [O.ls_grad(A, b, X0)]
    Xk, Pk = X0, X0.copy()
    for k in range(6):
        Xk, Pk = O.exact_diffusion_step(Xk, Pk, gs[-1], W, alpha)
        if k == 0:
            expect = D @ (xs[0] - alpha * gs[0])
        else:
            expect = D @ (2 * xs[-1] - xs[-2] - alpha * (gs[-1] - gs[-2]))
        np.testing.assert_allclose(Xk, expect, rtol=1e-11, atol=1e-11)
        xs.append(Xk)
        gs.append(O.ls_grad(A, b, Xk))


# ---------------------------------------------------------------- bf16 rounding and fp32 chain
def test_round_to_bf16_matches_torch():
    rng = np.random.default_rng(18)
    vals = np.concatenate([
        rng.normal(size=4000).astype(np.float32),
        (rng.normal(size=2000) * 1e-40).astype(np.float32),            # subnormals
        np.array([0.0, -0.0, np.inf, -np.inf, np.nan, 1.0, 1.00390625, 1.01171875,
                  3.3895314e38, -3.3895314e38, 3.4028235e38], dtype=np.float32),
        # exact ties: bf16 has 8 significant bits; 1 + (2k+1) 2^-8 lies halfway
        np.array([1 + (2 * k + 1) * 2.0 ** -8 for k in range(64)], dtype=np.float32),
    ])
    got = O.round_to_bf16(vals)
    ref = torch.from_numpy(vals).to(torch.bfloat16).to(torch.float32).numpy()
    nan = np.isnan(ref)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan].view(np.uint32), ref[~nan].view(np.uint32))


def test_mix_fp32_chain_one_peer_is_single_rounded_add():
    rng = np.random.default_rng(19)
    X = rng.normal(size=(8, 33)).astype(np.float32)
    W = T.one_peer_exponential(8, 1)
    got = O.mix_fp32_chain(X, W)
    ref = np.empty_like(X)
    for i in range(8):
        ref[i] = (X[i] + X[(i + 2) % 8]) / np.float32(2)   # one rounded add, exact halving
    assert np.array_equal(got.view(np.uint32), ref.view(np.uint32))
    np.testing.assert_allclose(got, O.mix(X, W), rtol=1e-7, atol=1e-7)


# ---------------------------------------------------------------- push-sum gradient tracking (next row)
def _gt_problem(seed, n=8, m=4, d=6):
    rng = np.random.default_rng(seed)
    A = rng.normal(size=(n, m, d))
    b = rng.normal(size=(n, m))
    xs = np.linalg.lstsq(A.reshape(n * m, d), b.reshape(n * m), rcond=None)[0]
    return A, b, xs


def test_gradient_tracking_invariants_and_exact_limit_on_directed_graph():
    n = 8
    A, b, xs = _gt_problem(20, n=n)
    W, _ = T.random_directed_push(n, 2, 5)
    grad = lambda X: O.ls_grad(A, b, X)
    X = np.zeros((n, 6))
    U, v = X.copy(), np.ones(n)
    G = grad(X)
    Y = G.copy()
    for k in range(6000):
        U, v, X, Y, G = O.pushsum_gradient_tracking_step(U, v, Y, G, W, 0.01, grad)
        if k % 500 == 0:
            np.testing.assert_allclose(Y.sum(0), G.sum(0), atol=1e-9)     # 1^T y = 1^T g (column-stochastic W)
            assert abs(v.sum() - n) < 1e-10
    np.testing.assert_allclose(X, np.tile(xs, (n, 1)), atol=1e-7)         # exact solution, no DGD bias
    assert abs(v - 1).max() > 0.05                                         # push-sum weights are not trivial


def test_gradient_tracking_on_time_varying_one_peer_graph():
    n = 8
    A, b, xs = _gt_problem(21, n=n)
    grad = lambda X: O.ls_grad(A, b, X)
    X = np.zeros((n, 6))
    U, v = X.copy(), np.ones(n)
    G = grad(X)
    Y = G.copy()
    for k in range(6000):
        U, v, X, Y, G = O.pushsum_gradient_tracking_step(U, v, Y, G, T.one_peer_exponential(n, k), 0.01, grad)
    np.testing.assert_allclose(X, np.tile(xs, (n, 1)), atol=1e-7)
    np.testing.assert_allclose(v, 1.0, atol=1e-12)                          # doubly stochastic rounds keep v = 1


def test_gradient_tracking_step_against_dense_formulas():
    rng = np.random.default_rng(22)
    n, d = 5, 3
    D = np.abs(_rand_W(n, rng))
    D = D / D.sum(0, keepdims=True)                                         # column stochastic, asymmetric
    W = T.from_dense(D)
    U, Y, Gp = (rng.normal(size=(n, d)) for _ in range(3))
    v = rng.random(n) + 0.5
    Q = rng.normal(size=(d, d))
    grad = lambda X: X @ Q + 1.0
    Un, vn, Xn, Yn, Gn = O.pushsum_gradient_tracking_step(U, v, Y, Gp, W, 0.3, grad)
    np.testing.assert_allclose(Un, D @ (U - 0.3 * Y), atol=1e-13)
    np.testing.assert_allclose(vn, D @ v, atol=1e-13)
    np.testing.assert_allclose(Xn, (D @ (U - 0.3 * Y)) / (D @ v)[:, None], atol=1e-13)
    np.testing.assert_allclose(Gn, Xn @ Q + 1.0, atol=1e-13)
    np.testing.assert_allclose(Yn, D @ (Y + Gn - Gp), atol=1e-13)


# ------------------------------------------------------------------ two-level (hierarchical) averaging
def test_hierarchical_equals_kronecker_product_operator():
    # stages 1-3 compose to the n x n matrix kron(W_machine, 11^T / L): a dense product by a library
    # routine, independent of the oracle's staged loops
    rng = np.random.default_rng(21)
    for M, L, topo in [(4, 3, T.ring(4)), (8, 2, T.static_exponential(8)), (5, 4, T.random_directed_push(5, 2, 7)[0])]:
        X = rng.standard_normal((M * L, 6))
        Wd = T.to_dense(topo)
        ref = np.kron(Wd, np.full((L, L), 1.0 / L)) @ X
        got = O.hierarchical_neighbor_allreduce(X, topo, L)
        np.testing.assert_allclose(got, ref, rtol=0, atol=1e-14)


def test_hierarchical_special_cases():
    rng = np.random.default_rng(22)
    X = rng.standard_normal((12, 5))
    ring = T.ring(12)
    # one agent per machine: nothing but the flat neighbor average
    np.testing.assert_allclose(O.hierarchical_neighbor_allreduce(X, ring, 1), O.mix(X, ring), atol=1e-15)
    # one machine holding everybody, W = [1]: the global average
    one = {0: [(0, 1.0)]}
    np.testing.assert_allclose(O.hierarchical_neighbor_allreduce(X, one, 12), np.tile(X.mean(0), (12, 1)), atol=1e-15)
    # agents of a machine end up equal; a doubly stochastic machine matrix keeps the global mean
    out = O.hierarchical_neighbor_allreduce(X, T.ring(4), 3)
    for a in range(4):
        assert np.ptp(out[3 * a:3 * a + 3], axis=0).max() == 0.0
    np.testing.assert_allclose(out.mean(0), X.mean(0), atol=1e-15)
    # worked example by hand: 2 machines x 2 agents, W = [[3/4, 1/4], [1/4, 3/4]], scalars 0, 2, 4, 10
    W2 = {0: [(0, 0.75), (1, 0.25)], 1: [(0, 0.25), (1, 0.75)]}
    got = O.hierarchical_neighbor_allreduce(np.array([[0.0], [2.0], [4.0], [10.0]]), W2, 2)
    np.testing.assert_allclose(got[:, 0], [2.5, 2.5, 5.5, 5.5], atol=1e-15)
    with pytest.raises(ValueError):
        O.hierarchical_neighbor_allreduce(X, ring, 5)


# ------------------------------------------------------------------ window primitives
def _push_graph(n, k, seed):
    return T.random_directed_push(n, k, seed)[0]


def test_window_all_active_accumulate_then_collect_is_one_pushsum_round():
    rng = np.random.default_rng(31)
    W = _push_graph(9, 3, 5)
    X = rng.standard_normal((9, 4))
    p = np.ones(9)
    E = O.window_slots(W)[0][-1]
    X1, p1, Win, wp = O.win_accumulate(X, p, np.zeros((E, 4)), np.zeros(E), W)
    X2, p2, Win2, wp2 = O.win_update_then_collect(X1, p1, Win, wp, W)
    Xs, ps, _ = O.pushsum_step(X, p, W)
    np.testing.assert_allclose(X2, Xs, atol=1e-14)
    np.testing.assert_allclose(p2, ps, atol=1e-14)
    assert np.abs(Win2).max() == 0.0 and np.abs(wp2).max() == 0.0


def test_window_put_then_update_all_active_is_one_mix_round():
    rng = np.random.default_rng(32)
    W = T.static_exponential(8)
    X = rng.standard_normal((8, 3))
    E = O.window_slots(W)[0][-1]
    Win = O.win_put(X, np.full((E, 3), 99.0), W)             # stale contents are overwritten
    np.testing.assert_allclose(O.win_update(X, Win, W), O.mix(X, W), atol=1e-14)


def test_window_get_is_the_pull_side_of_put():
    rng = np.random.default_rng(34)
    W = _push_graph(10, 3, 2)
    X = rng.standard_normal((10, 3))
    slot_ptr, slot_src, _, _ = O.window_slots(W)
    E = slot_ptr[-1]
    stale = np.full((E, 3), -7.0)
    # everybody active: pulling every slot and pushing every slot fill the window identically
    np.testing.assert_array_equal(O.win_get(X, stale, W), O.win_put(X, stale, W))
    np.testing.assert_allclose(O.win_update(X, O.win_get(X, stale, W), W), O.mix(X, W), atol=1e-14)
    # masks act on different ends: get refreshes the slots OWNED by active agents, put those FED by them
    act = np.zeros(10, dtype=int); act[3] = 1
    got = O.win_get(X, stale, W, act)
    put = O.win_put(X, stale, W, act)
    for e in range(E):
        owner = next(i for i in range(10) if slot_ptr[i] <= e < slot_ptr[i + 1])
        assert (got[e] == (X[slot_src[e]] if owner == 3 else -7.0)).all()
        assert (put[e] == (X[3] if slot_src[e] == 3 else -7.0)).all()


def test_window_hand_worked_two_agents_with_a_late_receiver():
    # W = [[1/2, 1/3], [1/2, 2/3]] (columns sum to one); x = (6, 12), p = (1, 1).
    W = {0: [(0, 0.5), (1, 1.0 / 3.0)], 1: [(0, 0.5), (1, 2.0 / 3.0)]}
    X = np.array([[6.0], [12.0]])
    p = np.ones(2)
    Win, wp = np.zeros((2, 1)), np.zeros(2)
    # both send: slot of agent 0 (from 1) holds 4, slot of agent 1 (from 0) holds 3
    X, p, Win, wp = O.win_accumulate(X, p, Win, wp, W)
    np.testing.assert_allclose(X[:, 0], [3.0, 8.0]); np.testing.assert_allclose(Win[:, 0], [4.0, 3.0])
    np.testing.assert_allclose(p, [0.5, 2.0 / 3.0]); np.testing.assert_allclose(wp, [1.0 / 3.0, 0.5])
    # only agent 0 collects; agent 1 is late and its slot keeps waiting
    X, p, Win, wp = O.win_update_then_collect(X, p, Win, wp, W, active=[1, 0])
    np.testing.assert_allclose(X[:, 0], [7.0, 8.0]); np.testing.assert_allclose(Win[:, 0], [0.0, 3.0])
    np.testing.assert_allclose(p, [5.0 / 6.0, 2.0 / 3.0]); np.testing.assert_allclose(wp, [0.0, 0.5])
    # agent 0 sends again before agent 1 has collected: the slot adds up (3 + 3.5)
    X, p, Win, wp = O.win_accumulate(X, p, Win, wp, W, active=[1, 0])
    np.testing.assert_allclose(X[:, 0], [3.5, 8.0]); np.testing.assert_allclose(Win[:, 0], [0.0, 6.5])
    X, p, Win, wp = O.win_update_then_collect(X, p, Win, wp, W, active=[0, 1])
    np.testing.assert_allclose(X[:, 0], [3.5, 14.5])
    assert abs(X.sum() + Win.sum() - 18.0) < 1e-14 and abs(p.sum() + wp.sum() - 2.0) < 1e-14


def test_window_mass_is_conserved_and_ratio_converges_under_random_activity():
    rng = np.random.default_rng(33)
    n, d = 12, 3
    W = _push_graph(n, 3, 11)
    X = rng.standard_normal((n, d)) * 3 + 1
    mean = X.mean(0)
    total = X.sum(0)
    p = np.ones(n)
    E = O.window_slots(W)[0][-1]
    Win, wp = np.zeros((E, d)), np.zeros(E)
    for k in range(400):
        act = rng.random(n) < 0.6
        X, p, Win, wp = O.win_accumulate(X, p, Win, wp, W, act)
        act = rng.random(n) < 0.6
        X, p, Win, wp = O.win_update_then_collect(X, p, Win, wp, W, act)
        np.testing.assert_allclose(X.sum(0) + Win.sum(0), total, atol=1e-11)
        assert abs(p.sum() + wp.sum() - n) < 1e-12
    assert np.abs(X / p[:, None] - mean).max() < 1e-8
    assert np.abs(X - mean).max() > 1e-3                     # x alone is biased


def test_window_slots_paper_sizing_example(golden_dir):
    # The paper's example (section "Asynchronous decentralized communication"): node 1 with in-coming
    # neighbors 3 and 5 and a 5 x 5 x 3 tensor registers one chunk of 150 = 5*5*3*2 values, first
    # half for node 3, second half for node 5.
    fx = {}
    for line in open(golden_dir + "/window_sizing_example.txt"):
        if line.strip() and not line.startswith("#"):
            k, v = line.split(":")
            fx[k.strip()] = [int(t) for t in v.split()]
    node, senders, shape = fx["node"][0], fx["in_coming"], fx["tensor_shape"]
    numel = int(np.prod(shape))
    n = 5
    W = {i: [(i, 1.0)] for i in range(n)}
    W[node - 1] = sorted([(node - 1, 1.0 / 3.0)] + [(s_ - 1, 1.0 / 3.0) for s_ in senders])
    slot_ptr, slot_src, slot_w, self_w = O.window_slots(W)
    lo, hi = slot_ptr[node - 1], slot_ptr[node]
    assert (hi - lo) * numel == fx["chunk_length"][0]
    assert [j + 1 for j in slot_src[lo:hi]] == senders                 # first half node 3, second half node 5
    assert slot_ptr[-1] == len(senders)                                # nobody else owns a slot
    assert self_w[node - 1] == 1.0 / 3.0 and slot_w[lo:hi] == [1.0 / 3.0] * 2
    # filling the window: the chunk is x_3 followed by x_5
    X = np.arange(n * numel, dtype=np.float64).reshape(n, numel)
    chunk = O.win_put(X, np.zeros((slot_ptr[-1], numel)), W)[lo:hi].reshape(-1)
    assert chunk.shape == (fx["chunk_length"][0],)
    np.testing.assert_array_equal(chunk[:numel], X[senders[0] - 1])
    np.testing.assert_array_equal(chunk[numel:], X[senders[1] - 1])


def test_window_update_hand_worked_three_agents_with_a_mask():
    # rows of W: agent 0 hears 1 and 2, agent 1 hears 0, agent 2 hears 1.  Slots in order:
    # (0 <- 1), (0 <- 2), (1 <- 0), (2 <- 1).
    W = {0: [(0, 0.5), (1, 0.25), (2, 0.25)], 1: [(0, 0.5), (1, 0.5)], 2: [(1, 1.0 / 3.0), (2, 2.0 / 3.0)]}
    slot_ptr, slot_src, slot_w, self_w = O.window_slots(W)
    assert slot_ptr == [0, 2, 3, 4] and slot_src == [1, 2, 0, 1]
    assert slot_w == [0.25, 0.25, 0.5, 1.0 / 3.0] and self_w == [0.5, 0.5, 2.0 / 3.0]
    X = np.array([[4.0], [8.0], [12.0]])
    Win = np.array([[1.0], [2.0], [3.0], [5.0]])
    # agents 0 and 2 update, agent 1 is busy elsewhere: x0 = 4/2 + 1/4 + 2/4, x2 = 2*12/3 + 5/3
    out = O.win_update(X, Win, W, active=[1, 0, 1])
    np.testing.assert_allclose(out[:, 0], [2.75, 8.0, 8.0 + 5.0 / 3.0], rtol=1e-15)
    # only agent 1: x1 = 8/2 + 3/2
    out = O.win_update(X, Win, W, active=[0, 1, 0])
    np.testing.assert_allclose(out[:, 0], [4.0, 5.5, 12.0], rtol=1e-15)
    # nobody: nothing moves; the window is never written by an update
    np.testing.assert_array_equal(O.win_update(X, Win, W, active=[0, 0, 0]), X)
    np.testing.assert_array_equal(Win[:, 0], [1.0, 2.0, 3.0, 5.0])


# ------------------------------------------------------------------ window primitives with per-call weights
def test_weighted_window_calls_without_arguments_are_the_plain_calls():
    rng = np.random.default_rng(51)
    W = _push_graph(9, 3, 5)
    n, d = 9, 4
    X = rng.standard_normal((n, d)); p = rng.random(n) + 0.5
    E = O.window_slots(W)[0][-1]
    Win = rng.standard_normal((E, d)); wp = rng.random(E)
    act = rng.random(n) < 0.6
    Xo, Wo = O.win_put_weighted(X, Win, W, act)
    np.testing.assert_array_equal(Wo, O.win_put(X, Win, W, act)); np.testing.assert_array_equal(Xo, X)
    np.testing.assert_array_equal(O.win_get_weighted(X, Win, W, act), O.win_get(X, Win, W, act))
    for a, b in zip(O.win_accumulate_weighted(X, p, Win, wp, W, act), O.win_accumulate(X, p, Win, wp, W, act)):
        np.testing.assert_allclose(a, b, rtol=0, atol=1e-15)
    np.testing.assert_allclose(O.win_update_weighted(X, Win, W, act), O.win_update(X, Win, W, act), rtol=0, atol=1e-15)


def test_weighted_window_calls_hand_worked_subsets():
    # rows of W: agent 0 hears 1 and 2, agent 1 hears 0, agent 2 hears 1 (slots: 0<-1, 0<-2, 1<-0, 2<-1)
    W = {0: [(0, 0.5), (1, 0.25), (2, 0.25)], 1: [(0, 0.5), (1, 0.5)], 2: [(1, 1.0 / 3.0), (2, 2.0 / 3.0)]}
    X = np.array([[4.0], [8.0], [12.0]])
    Win = np.array([[1.0], [2.0], [3.0], [5.0]])
    # agent 1 puts 2 x_1 to agent 0 only and keeps x_1 / 4; agent 2 puts nothing (empty subset)
    Xo, Wo = O.win_put_weighted(X, Win, W, None, self_weight=[1.0, 0.25, 1.0], dst_weights={0: {}, 1: {0: 2.0}, 2: {}})
    np.testing.assert_array_equal(Wo[:, 0], [16.0, 2.0, 3.0, 5.0]); np.testing.assert_array_equal(Xo[:, 0], [4.0, 2.0, 12.0])
    # accumulate: agent 1 adds x_1 / 2 at agent 2 (slot 3) and p_1 / 2 with it, keeps half
    p = np.array([1.0, 2.0, 1.0]); wp = np.zeros(4)
    Xo, po, Wo, wpo = O.win_accumulate_weighted(X, p, Win, wp, W, [0, 1, 0], self_weight=[9.0, 0.5, 9.0],
                                                dst_weights={0: {}, 1: {2: 0.5}, 2: {}})
    np.testing.assert_array_equal(Wo[:, 0], [1.0, 2.0, 3.0, 9.0]); np.testing.assert_array_equal(wpo, [0.0, 0.0, 0.0, 1.0])
    np.testing.assert_array_equal(Xo[:, 0], [4.0, 4.0, 12.0]); np.testing.assert_array_equal(po, [1.0, 1.0, 1.0])
    assert Xo.sum() + Wo.sum() == X.sum() + Win.sum() and po.sum() + wpo.sum() == p.sum()      # mass stays
    # get: agent 0 fetches 3 x_2 only
    Wo = O.win_get_weighted(X, Win, W, None, src_weights={0: {2: 3.0}, 1: {}, 2: {}})
    np.testing.assert_array_equal(Wo[:, 0], [1.0, 36.0, 3.0, 5.0])
    # update: agent 0 averages itself (weight 1/2) with the slot of agent 2 only (weight 1/2)
    Xo = O.win_update_weighted(X, Win, W, [1, 0, 0], self_weight=[0.5, 1.0, 1.0], src_weights={0: {2: 0.5}, 1: {}, 2: {}})
    np.testing.assert_array_equal(Xo[:, 0], [3.0, 8.0, 12.0])
    # an edge outside the static topology is refused (the paper: the ranks must be a subset of the neighbors)
    with pytest.raises(ValueError):
        O.win_put_weighted(X, Win, W, None, dst_weights={0: {2: 1.0}, 1: {}, 2: {}})


def test_weighted_accumulate_with_any_column_stochastic_split_conserves_mass_and_converges():
    # asynchronous push-sum over a dynamic sub-topology: each call, every active sender picks a random
    # subset of its out-neighbors and splits its mass evenly between them and itself
    rng = np.random.default_rng(52)
    n, d = 10, 2
    W = _push_graph(n, 3, 4)
    outs = T.out_lists(W)
    X = rng.standard_normal((n, d)) + 2.0
    mean, total = X.mean(0), X.sum(0)
    p = np.ones(n)
    E = O.window_slots(W)[0][-1]
    Win, wp = np.zeros((E, d)), np.zeros(E)
    for k in range(600):
        act = rng.random(n) < 0.7
        dst, sw = {}, np.ones(n)
        for j in range(n):
            nb = [i for i in outs[j] if i != j and rng.random() < 0.6]
            dst[j] = {i: 1.0 / (len(nb) + 1) for i in nb}
            sw[j] = 1.0 / (len(nb) + 1)
        X, p, Win, wp = O.win_accumulate_weighted(X, p, Win, wp, W, act, sw, dst)
        X, p, Win, wp = O.win_update_then_collect(X, p, Win, wp, W, rng.random(n) < 0.7)
        np.testing.assert_allclose(X.sum(0) + Win.sum(0), total, atol=1e-11)
        assert abs(p.sum() + wp.sum() - n) < 1e-12
    assert np.abs(X / p[:, None] - mean).max() < 1e-6
