"""GPU parity: the HIP path (through the C ABI) against the fp64 CPU oracle, element by element,
on the same seeded inputs.  Tolerances: fp32 configs max|x_gpu - x_ref| <= 1e-5 max|x_ref| per
round; bf16-storage config <= 2e-2 max|x_ref| per step; integer/bitwise claims exact."""

import numpy as np
import pytest
import torch

import paper_2111_04287_amd as bf
import workloads
from oracle import iterations as O
from oracle import topology as OT

pytestmark = pytest.mark.gpu

DEV = torch.device("cuda:0")
TOL32 = 1e-5
TOL16 = 2e-2


def lib_W(t, r=0):
    rowptr, col, wgt, _ = bf.bf_topology_export_csr(t, r)
    return OT.from_csr(rowptr, col, wgt)          # W is data: the oracle gets the library's fp32 weights


def host(x):
    return x.detach().float().cpu().numpy().astype(np.float64)


def assert_close(gpu, ref, tol, what=""):
    ref = np.asarray(ref, dtype=np.float64)
    scale = np.abs(ref).max() if ref.size else 0.0
    err = np.abs(host(gpu) - ref).max() if ref.size else 0.0
    assert err <= tol * scale + 1e-30, "%s: max err %.3e > %.1e * %.3e" % (what, err, tol, scale)
    return err


def rows(n, d, seed, dtype=torch.float32, ld=None, std=1.0, mean=0.0):
    ld = workloads.padded_ld(d, 2 if dtype == torch.bfloat16 else 4) if ld is None else ld
    return workloads.normal_rows(n, d, seed, DEV, mean=mean, std=std, ld=ld, dtype=dtype)


def empty_like_rows(x):
    n, d = x.shape
    ld = x.stride(0) if n > 1 else d
    return workloads.alloc_rows(n, d, x.dtype, DEV, ld=ld)


TOPOS = [
    ("ring", lambda n: bf.bf_topology_create(bf.BF_RING, n)),
    ("exp", lambda n: bf.bf_topology_create(bf.BF_EXP_STATIC, n)),
    ("onepeer", lambda n: bf.bf_topology_create(bf.BF_EXP2_ONE_PEER, n)),
    ("push", lambda n: bf.bf_topology_create(bf.BF_RANDOM_DIRECTED, n, out_degree=min(4, n - 1), seed=401)),
]


# ------------------------------------------------------------------ a1/a2: neighbor_allreduce
@pytest.mark.parametrize("name,make", TOPOS)
@pytest.mark.parametrize("n,d", [(1, 64), (3, 4), (16, 1024), (64, 8192 + 520), (100, 3004), (256, 4096 + 72),
                                 (320, 1000), (37, 130)])
def test_mix_fp32_matches_oracle(name, make, n, d):
    if name == "push" and n < 3:
        pytest.skip("needs a few agents")
    t = make(n)
    X = rows(n, d, 1000 + n)
    for r in range(2):                            # odd rounds walk the tiles right to left
        out = empty_like_rows(X)
        out.fill_(float("nan"))
        bf.bf_neighbor_allreduce(t, r, X, out)
        assert_close(out, O.mix(host(X), lib_W(t, r)), TOL32, "%s n=%d d=%d r=%d" % (name, n, d, r))
        # in place gives the same bits
        Xi = empty_like_rows(X)
        Xi.copy_(X)
        bf.bf_neighbor_allreduce(t, r, Xi, Xi)
        assert torch.equal(Xi, out)


def test_many_agents_use_the_fallback_kernels():
    # 2048 agents: a 2048 x 64 fp32 tile is 512 KB, beyond LDS.  Out of place goes through the row
    # gather, in place through 16-column tiles; both give the same bits.
    n, d = 2048, 520 + 3
    t = bf.bf_topology_create(bf.BF_EXP_STATIC, n)
    W = lib_W(t)
    X = rows(n, d, 5)
    out = empty_like_rows(X)
    bf.bf_neighbor_allreduce(t, 0, X, out)
    assert_close(out, O.mix(host(X), W), TOL32)
    Xi = empty_like_rows(X).copy_(X)
    bf.bf_neighbor_allreduce(t, 0, Xi, Xi)
    assert torch.equal(Xi, out)
    G = rows(n, d, 6)
    M = workloads.normal_rows(n, d, 7, DEV, ld=X.stride(0))
    M0 = host(M)
    for mode in (bf.BF_ATC, bf.BF_AWC):
        bf.bf_atc_step(t, 0, X, out, G, None, alpha=0.05, mode=mode)
        ref = (O.atc_step if mode == bf.BF_ATC else O.awc_step)(host(X), host(G), W, float(np.float32(0.05)))
        assert_close(out, ref, TOL32)
    bf.bf_atc_step(t, 0, X, out, G, M, alpha=0.05, beta=0.9, mode=bf.BF_ATC)
    ref, Mref = O.dmsgd_atc_step(host(X), M0, host(G), W, float(np.float32(0.05)), float(np.float32(0.9)))
    assert_close(out, ref, TOL32)
    assert_close(M, Mref, 1e-6)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_many_agents_every_op_has_a_kernel(dtype):
    # 700 agents: beyond a 64-column tile.  In-place updates, Exact-Diffusion, tracking and the
    # push-sum ratio go through the narrow-tile kernel; every op against the oracle.
    n, d = 700, 72 + 5
    t = bf.bf_topology_create(bf.BF_RANDOM_DIRECTED, n, out_degree=10, seed=21)
    W = lib_W(t)
    tol = TOL32 if dtype == torch.float32 else 2.0 ** -8
    X, G, G2 = (rows(n, d, 300 + k, dtype=dtype) for k in range(3))
    alpha, beta = 0.05, 0.9
    a64, b64 = float(np.float32(alpha)), float(np.float32(beta))
    # in place: mix, ATC, AWC
    for mode, fn in ((None, lambda x, g: O.mix(x, W)), (bf.BF_ATC, lambda x, g: O.atc_step(x, g, W, a64)),
                     (bf.BF_AWC, lambda x, g: O.awc_step(x, g, W, a64))):
        Xi = empty_like_rows(X).copy_(X)
        if mode is None:
            bf.bf_neighbor_allreduce(t, 0, Xi, Xi)
        else:
            bf.bf_atc_step(t, 0, Xi, Xi, G, None, alpha, 0.0, mode)
        assert_close(Xi, fn(host(X), host(G)), tol, "in place mode %s" % mode)
    # momentum, in place
    M = workloads.normal_rows(n, d, 310, DEV, ld=X.stride(0))
    Xr, Mr = O.dmsgd_atc_step(host(X), host(M), host(G), W, a64, b64)
    Xi = empty_like_rows(X).copy_(X)
    bf.bf_atc_step(t, 0, Xi, Xi, G, M, alpha, beta, bf.BF_ATC)
    assert_close(Xi, Xr, tol, "momentum x")
    assert_close(M, Mr, 1e-6, "momentum m")
    # Exact-Diffusion and the tracking update, out of place and in place
    P = workloads.normal_rows(n, d, 311, DEV, ld=X.stride(0))
    P0 = host(P)
    ref, psi = O.exact_diffusion_step(host(X), P0, host(G), W, a64)
    out = bf.bf_exact_diffusion_step(t, 0, X, empty_like_rows(X), G, P, alpha)
    assert_close(out, ref, tol, "ED x")
    assert_close(P, psi, 1e-6, "ED psi")
    Yo = bf.bf_tracking_step(t, 0, X, empty_like_rows(X), G, G2)
    assert_close(Yo, O.mix(host(X) + host(G) - host(G2), W), tol, "tracking")
    Yi = empty_like_rows(X).copy_(X)
    bf.bf_tracking_step(t, 0, Yi, Yi, G, G2)
    assert torch.equal(Yi, Yo)
    # push-sum in place with the ratio
    w = torch.rand(n, device=DEV) + 0.5
    Xn, wn, Yn = O.pushsum_step(host(X), host(w), W)
    Xi = empty_like_rows(X).copy_(X)
    Y = empty_like_rows(X)
    bf.bf_pushsum_step(t, 0, Xi, Xi, w, w, Y)
    assert_close(Xi, Xn, tol, "push-sum x")
    assert_close(w, wn, TOL32, "push-sum w")
    assert_close(Y, Yn, 2e-5 if dtype == torch.float32 else 2.0 ** -7, "push-sum ratio")


def test_forced_gather_path_matches_tile_path():
    n, d = 64, 3000
    t = bf.bf_topology_create(bf.BF_EXP_STATIC, n)
    X = rows(n, d, 8)
    a, b = empty_like_rows(X), empty_like_rows(X)
    bf.bf_neighbor_allreduce(t, 0, X, a)
    try:
        bf.bf_set_tuning(2, 1)
        bf.bf_neighbor_allreduce(t, 0, X, b)
    finally:
        bf.bf_set_tuning(2, 0)
    assert torch.equal(a, b)


def test_mix_never_touches_row_padding():
    n, d, ld = 16, 1000, 1024
    base = torch.full((n, ld), 7.0, device=DEV)
    X = rows(n, d, 5, ld=ld)
    out = base[:, :d]
    t = bf.bf_topology_create(bf.BF_EXP_STATIC, n)
    bf.bf_neighbor_allreduce(t, 0, X, out)
    assert torch.all(base[:, d:] == 7.0)
    assert_close(out, O.mix(host(X), lib_W(t)), TOL32)


def test_mix_empty_width_is_a_no_op():
    t = bf.bf_topology_create(bf.BF_RING, 4)
    X = torch.zeros((4, 64), device=DEV)
    assert bf.lib.bf_neighbor_allreduce(t.handle, 0, X.data_ptr(), X.data_ptr(), 0, 64, bf.BF_F32, None) == 0


@pytest.mark.parametrize("tile", [64, 128, 256, 512, 1024])
def test_mix_result_is_independent_of_tile_width(tile):
    n, d = 16, 5000
    t = bf.bf_topology_create(bf.BF_EXP_STATIC, n)
    X = rows(n, d, 77)
    ref = empty_like_rows(X)
    bf.bf_neighbor_allreduce(t, 0, X, ref)
    try:
        bf.bf_set_tuning(0, tile)
        out = empty_like_rows(X)
        bf.bf_neighbor_allreduce(t, 0, X, out)
    finally:
        bf.bf_set_tuning(0, 0)
    assert torch.equal(out, ref)                  # same CSR order, same FMA chain: same bits


@pytest.mark.parametrize("knob,value", [(7, 1), (8, 1), (8, 2), (1, 1), (3, 3)])
def test_launch_policy_knobs_do_not_change_results(knob, value):
    # tile order, cache policy, occupancy and grid size are scheduling choices: same bits
    n, d = 64, 9000
    t = bf.bf_topology_create(bf.BF_EXP_STATIC, n)
    X, G = rows(n, d, 78), rows(n, d, 79)
    ref = [empty_like_rows(X) for _ in range(4)]
    for r in range(2):
        bf.bf_neighbor_allreduce(t, r, X, ref[r])
        bf.bf_atc_step(t, r, X, ref[2 + r], G, None, alpha=0.1, mode=bf.BF_ATC)
    try:
        bf.bf_set_tuning(knob, value)
        for r in range(2):
            out = empty_like_rows(X)
            bf.bf_neighbor_allreduce(t, r, X, out)
            assert torch.equal(out, ref[r])
            Xi = empty_like_rows(X)
            Xi.copy_(X)
            bf.bf_atc_step(t, r, Xi, Xi, G, None, alpha=0.1, mode=bf.BF_ATC)
            assert torch.equal(Xi, ref[2 + r])
    finally:
        bf.bf_set_tuning(knob, 0)


def test_mix_bf16_matches_oracle():
    n, d = 32, 2048 + 40
    t = bf.bf_topology_create(bf.BF_EXP_STATIC, n)
    X = rows(n, d, 9, dtype=torch.bfloat16)
    out = empty_like_rows(X)
    bf.bf_neighbor_allreduce(t, 0, X, out)
    ref = O.mix(host(X), lib_W(t))
    got = host(out)
    # the exact result rounded once to bf16 (half an ulp), plus the fp32 accumulation error, which
    # matters only where the sum cancels to almost nothing or sits next to a rounding tie
    rounded = O.round_to_bf16(ref.astype(np.float32)).astype(np.float64)
    ulp = 2.0 ** (np.floor(np.log2(np.maximum(np.abs(ref), 1e-300))) - 7)
    assert (np.abs(got - ref) <= 0.5 * ulp + 4e-7 * np.abs(host(X)).max()).all()
    # equal weights put many exact sums next to a rounding tie (0.1f * short sum): most, not all, agree
    assert (got == rounded).mean() > 0.98


def test_bf16_output_rounding_is_nearest_even_bit_for_bit():
    """x_0 <- (a + b) / 2 with bf16 a, b of nearby exponents is exact in fp32, so the stored bf16 value
    is that number rounded once: to nearest, ties to even, denormals kept, infinities and NaN passed on.
    Hand-made ties in both directions, denormal ties, signed zeros, the largest finite values and
    random pairs, in every kernel that stores bf16 (out of place: pipelined kernel; in place: one-tile
    kernel; forced chain kernel), checked bit for bit against the oracle's rounding."""
    n = 2
    t = bf.bf_topology_create(bf.BF_CSR_USER, n, rounds=1, rowptr=np.array([0, 2, 3]), col=np.array([0, 1, 1]),
                              wgt=np.array([0.5, 0.5, 1.0], dtype=np.float32), require_strongly_connected=False)
    e7, e6 = 2.0 ** -7, 2.0 ** -6
    pairs = [(1.0, 1.0 + e7), (1.0 + e7, 1.0 + e6), (-1.0, -1.0 - e7), (-1.0 - e7, -1.0 - e6),     # ties: down to even, up to even
             (1.0, 1.0 + e6), (3.0, 3.0 + 2 * e7),                                                    # exact, no rounding
             (2.0 ** -133, 2.0 ** -132), (2.0 ** -132, 3 * 2.0 ** -133), (2.0 ** -126, 2.0 ** -126 + 2.0 ** -133),   # denormal ties
             (0.0, -0.0), (0.0, 2.0 ** -133),       # (sums start from +0, so -0 + -0 gives +0: not a rounding matter)
             (3.3895313892515355e38, 3.3895313892515355e38), (3.3895313892515355e38, 3.376e38),
             (float("inf"), 1.0), (float("-inf"), 5.0), (float("inf"), float("-inf")), (float("nan"), 1.0)]
    rng = np.random.default_rng(77)
    d = 4096 + 24
    a = rng.standard_normal(d).astype(np.float32) * np.float32(2.0) ** rng.integers(-20, 20, d).astype(np.float32)
    b = a * (1 + rng.integers(-64, 64, d).astype(np.float32) * np.float32(e7))
    a, b = O.round_to_bf16(a), O.round_to_bf16(b)
    for k, (x, y) in enumerate(pairs):
        a[k * 8:(k + 1) * 8], b[k * 8:(k + 1) * 8] = x, y
    a, b = O.round_to_bf16(a), O.round_to_bf16(b)                # (3.376e38 and the like: the nearest bf16)
    with np.errstate(invalid="ignore", over="ignore"):
        exact = (0.5 * a.astype(np.float64) + 0.5 * b.astype(np.float64)).astype(np.float32)
        assert np.array_equal(exact.astype(np.float64)[np.isfinite(exact)], (0.5 * a.astype(np.float64) + 0.5 * b.astype(np.float64))[np.isfinite(exact)])
    want = O.round_to_bf16(exact)
    X = workloads.alloc_rows(n, d, torch.bfloat16, DEV, ld=workloads.padded_ld(d, 2))
    X.copy_(torch.from_numpy(np.stack([a, b])).to(DEV).to(torch.bfloat16))
    assert np.array_equal(X.float().cpu().numpy().view(np.uint32)[~np.isnan(a[None, :]).repeat(2, 0)],
                          np.stack([a, b]).view(np.uint32)[~np.isnan(a[None, :]).repeat(2, 0)])

    def check(out, what):
        got = out[0].float().cpu().numpy()
        nan = np.isnan(want)
        assert np.array_equal(np.isnan(got), nan), what
        bad = np.nonzero(got.view(np.uint32)[~nan] != want.view(np.uint32)[~nan])[0]
        assert bad.size == 0, "%s: %d values differ, first at %d: got %r want %r" % (what, bad.size, bad[0], got[~nan][bad[0]], want[~nan][bad[0]])
        assert torch.equal(out[1], X[1])

    out = empty_like_rows(X)
    bf.bf_neighbor_allreduce(t, 0, X, out)
    check(out, "out of place")
    Xi = empty_like_rows(X).copy_(X)
    bf.bf_neighbor_allreduce(t, 0, Xi, Xi)
    check(Xi, "in place")
    bf.bf_set_tuning(6, 1)
    try:
        out = empty_like_rows(X)
        bf.bf_neighbor_allreduce(t, 0, X, out)
    finally:
        bf.bf_set_tuning(6, 0)
    check(out, "chain kernel")
    G = workloads.alloc_rows(n, d, torch.bfloat16, DEV, ld=X.stride(0), fill=0)
    for mode in (bf.BF_ATC, bf.BF_AWC):
        out = empty_like_rows(X)
        bf.bf_atc_step(t, 0, X, out, G, None, alpha=0.25, mode=mode)          # zero gradient: the same numbers
        check(out, "fused step, mode %d" % mode)


def test_dynamic_api_with_constant_weights_equals_static():
    n, d = 64, 3000
    ts = bf.bf_topology_create(bf.BF_EXP_STATIC, n)
    rowptr, col, wgt, _ = bf.bf_topology_export_csr(ts)
    R = 3
    rp = np.concatenate([rowptr + k * len(col) for k in range(R)])
    tu = bf.bf_topology_create(bf.BF_CSR_USER, n, rounds=R, rowptr=rp, col=np.tile(col, R), wgt=np.tile(wgt, R),
                               require_class=bf.BF_W_STANDARD)
    X = rows(n, d, 3)
    a, b = empty_like_rows(X), empty_like_rows(X)
    bf.bf_neighbor_allreduce(ts, 0, X, a)
    for r in range(R):
        bf.bf_neighbor_allreduce(tu, r, X, b)
        assert torch.equal(a, b)


def test_push_equals_pull_on_one_device():
    # w = r*s: pure push (r=1, s=w) and pure pull (r=w, s=1) give the same result
    n, d = 12, 520
    W = OT.static_exponential(n)
    src = {i: [(j, w) for j, w in W[i] if j != i] for i in range(n)}
    srp = np.cumsum([0] + [len(src[i]) for i in range(n)])
    srk = [j for i in range(n) for j, _ in src[i]]
    swt = [w for i in range(n) for _, w in src[i]]
    dst = {j: sorted(i for i in range(n) for jj, _ in src[i] if jj == j) for j in range(n)}
    drp = np.cumsum([0] + [len(dst[j]) for j in range(n)])
    drk = [i for j in range(n) for i in dst[j]]
    dwt = [dict(src[i])[j] for j in range(n) for i in dst[j]]
    selfw = [dict(W[i])[i] for i in range(n)]
    t_pull = bf.bf_topology_create_push_pull(n, selfw, srp, srk, swt, drp, drk, None)
    t_push = bf.bf_topology_create_push_pull(n, selfw, srp, srk, None, drp, drk, dwt)
    X = rows(n, d, 21)
    a, b = empty_like_rows(X), empty_like_rows(X)
    bf.bf_neighbor_allreduce(t_pull, 0, X, a)
    bf.bf_neighbor_allreduce(t_push, 0, X, b)
    assert torch.equal(a, b)
    assert_close(a, O.mix(host(X), W), TOL32)


# ------------------------------------------------------------------ configuration 2 (reduced d)
def test_config2_static_exp_50_rounds():
    n, d = 64, 8192 + 264
    t = bf.bf_topology_create(bf.BF_EXP_STATIC, n)
    W = lib_W(t)
    X = workloads.config2_state(DEV, n=n, d=d, ld=workloads.padded_ld(d, 4))
    ref = host(X)
    e0 = O.consensus_error(ref)
    floor = 1e-6 * np.abs(ref).max() * np.sqrt(n * d)
    buf = [X, empty_like_rows(X)]
    stats = torch.empty(3, dtype=torch.float64, device=DEV)
    for k in range(50):
        bf.bf_neighbor_allreduce(t, k, buf[k & 1], buf[1 - (k & 1)])
        ref = O.mix(ref, W)
        cur = buf[1 - (k & 1)]
        assert_close(cur, ref, TOL32, "round %d" % k)
        bf.bf_consensus_stats(cur, None, stats)
        err = float(stats[0].sqrt())
        bound = (2.0 / 3.0) ** (k + 1) * e0
        if bound > floor:                                   # contraction at |lambda_2| = 2/3
            assert err <= bound * (1 + 1e-4)
        np.testing.assert_allclose(err, O.consensus_error(host(cur)), rtol=1e-9, atol=1e-12)
    np.testing.assert_allclose(host(cur).mean(0), ref.mean(0), atol=2e-6)


# ------------------------------------------------------------------ configuration 3 (reduced d)
def test_config3_one_peer_8_rounds_exact_mean_and_bitwise():
    n, d = 256, 4096 + 136
    t = bf.bf_topology_create(bf.BF_EXP2_ONE_PEER, n)
    assert bf.bf_topology_rounds(t) == 8
    X = workloads.config3_state(DEV, n=n, d=d, ld=workloads.padded_ld(d, 4))
    ref = host(X)
    emu = X.cpu().numpy()
    mean = ref.mean(0)
    buf = [X, empty_like_rows(X)]
    for r in range(8):
        cur = buf[1 - (r & 1)]
        bf.bf_neighbor_allreduce(t, r, buf[r & 1], cur)
        W = lib_W(t, r)
        ref = O.mix(ref, W)
        emu = O.mix_fp32_chain(emu, W)
        assert_close(cur, ref, TOL32, "round %d" % r)
        assert np.array_equal(cur.cpu().numpy().view(np.uint32), emu.view(np.uint32)), "round %d bits" % r
    got = host(cur)
    assert np.abs(got - mean).max() <= 1e-6 * np.abs(ref).max() + 8 * 6e-8 * np.abs(host(X)).max()
    assert np.abs(ref - mean).max() < 1e-14


# ------------------------------------------------------------------ a3 / configuration 4 (reduced d)
def test_config4_pushsum_100_rounds():
    n, d = 128, 2048 + 328
    t = bf.bf_topology_create(bf.BF_RANDOM_DIRECTED, n, out_degree=4, seed=workloads.CONFIG4_GRAPH_SEED)
    W = lib_W(t)
    X = workloads.config4_state(DEV, n=n, d=d, ld=workloads.padded_ld(d, 4))
    Xr = host(X)
    xbar = Xr.mean(0)
    pr = np.ones(n)
    w = [torch.ones(n, device=DEV), torch.empty(n, device=DEV)]
    buf = [X, empty_like_rows(X)]
    Y = empty_like_rows(X)
    for k in range(100):
        a, b = k & 1, 1 - (k & 1)
        bf.bf_pushsum_step(t, k, buf[a], buf[b], w[a], w[b], Y)
        Xr, pr, Yr = O.pushsum_step(Xr, pr, W)
        assert_close(buf[b], Xr, TOL32, "X round %d" % k)
        assert_close(w[b], pr, TOL32, "w round %d" % k)
        assert_close(Y, Yr, 2e-5, "Y round %d" % k)
    assert abs(float(w[b].sum()) - n) < 1e-3
    assert np.abs(host(Y) - xbar).max() < 2e-5 * np.abs(xbar).max()
    stats = bf.bf_consensus_stats(buf[b], w[b])
    assert float(stats[1]) < 2e-5 * float(stats[2])


def test_pushsum_in_place_and_without_ratio():
    n, d = 16, 700
    t = bf.bf_topology_create(bf.BF_RANDOM_DIRECTED, n, out_degree=3, seed=11)
    W = lib_W(t)
    X = rows(n, d, 31, mean=5.0, std=2.0, ld=704)
    Xr, pr = host(X), np.ones(n)
    w = torch.ones(n, device=DEV)
    for k in range(5):
        bf.bf_pushsum_step(t, k, X, X, w, w, None)
        Xr, pr, _ = O.pushsum_step(Xr, pr, W)
    assert_close(X, Xr, TOL32)
    assert_close(w, pr, TOL32)


# ------------------------------------------------------------------ a4/a5/a7: ATC, AWC, least squares
def test_least_squares_gradient_matches_oracle():
    data = workloads.config1_least_squares(DEV)
    A, b = data["A"], data["b"]
    X = rows(16, 1024, 41)
    G = empty_like_rows(X)
    bf.bf_grad_least_squares(A, b, X, G)
    ref = O.ls_grad(host(A), host(b), host(X))
    assert_close(G, ref, 2e-6, "ls grad")


@pytest.mark.parametrize("n,m,d", [(1, 1, 4), (3, 5, 260), (5, 64, 1028)])
def test_least_squares_gradient_shapes(n, m, d):
    g = torch.Generator(device=DEV).manual_seed(n * 100 + m)
    A = torch.randn((n, m, d), generator=g, device=DEV)
    b = torch.randn((n, m), generator=g, device=DEV)
    X = rows(n, d, 43)
    G = empty_like_rows(X)
    bf.bf_grad_least_squares(A, b, X, G)
    assert_close(G, O.ls_grad(host(A), host(b), host(X)), 5e-6)


@pytest.mark.parametrize("mode", [bf.BF_ATC, bf.BF_AWC])
@pytest.mark.parametrize("n,d", [(16, 1024), (64, 2000), (256, 520), (5, 68), (1, 300), (2, 64), (3, 1)])
def test_atc_awc_step_matches_oracle(mode, n, d):
    t = bf.bf_topology_create(bf.BF_EXP_STATIC, n)
    W = lib_W(t)
    X, G = rows(n, d, 51), rows(n, d, 52)
    alpha = 0.05
    out = empty_like_rows(X)
    bf.bf_atc_step(t, 0, X, out, G, None, alpha=alpha, mode=mode)
    a64 = float(np.float32(alpha))
    ref = (O.atc_step if mode == bf.BF_ATC else O.awc_step)(host(X), host(G), W, a64)
    assert_close(out, ref, TOL32)
    Xi = empty_like_rows(X)
    Xi.copy_(X)
    bf.bf_atc_step(t, 0, Xi, Xi, G, None, alpha=alpha, mode=mode)      # in place
    assert torch.equal(Xi, out)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("n,d,tile", [(16, 11 * 1024 + 44, 1024), (16, 11 * 512 + 44, 512), (40, 9 * 256 + 4, 256),
                                      (128, 13 * 128 + 2, 128), (64, 13 * 128 + 2, 128), (256, 7 * 64 + 1, 64),
                                      (128, 7 * 64 + 1, 64), (16, 11 * 1024 + 44, 0)])
def test_awc_on_the_pipelined_kernel_with_several_tiles_per_workgroup(dtype, n, d, tile):
    """The reducers of the pipelined kernel take the receiver's own gradient (and momentum) either
    from HBM, several rows ahead and across tile boundaries, or -- bf16 storage, no momentum, where
    n more rows fit the LDS tile -- from a gradient tile the loaders stage (tuning knob 14 keeps
    them from it).  A grid capped at three workgroups gives each of them several tiles (an odd
    number of them, the last one ragged) in every tile width the kernel has (knob 0; the shapes
    include one where the gradient rows fill LDS to the last byte and ones where they do not fit);
    rounds 0 and 1 walk the tiles in opposite directions.  Checked against the oracle and, bit for
    bit, between the capped and the uncapped launch and between the two forms."""
    t = bf.bf_topology_create(bf.BF_EXP_STATIC, n)
    tol = TOL32 if dtype == torch.float32 else 2.0 ** -8
    X, G = rows(n, d, 71, dtype=dtype), rows(n, d, 72, dtype=dtype)
    M0 = workloads.normal_rows(n, d, 73, DEV, ld=X.stride(0))
    alpha, beta = 0.05, 0.9
    a64, b64 = float(np.float32(alpha)), float(np.float32(beta))
    for rnd in range(2):
        W = lib_W(t, rnd)
        mixed = O.mix(host(X), W)
        for with_m in (False, True):
            got = []
            for grid, from_hbm in ((0, 0), (3, 0), (3, 1)):
                bf.bf_set_tuning(3, grid)
                bf.bf_set_tuning(0, tile)
                bf.bf_set_tuning(14, from_hbm)
                try:
                    out = empty_like_rows(X)
                    out.fill_(float("nan"))
                    M = empty_like_rows(M0).copy_(M0) if with_m else None
                    bf.bf_atc_step(t, rnd, X, out, G, M, alpha=alpha, beta=beta if with_m else 0.0, mode=bf.BF_AWC)
                finally:
                    bf.bf_set_tuning(3, 0)
                    bf.bf_set_tuning(0, 0)
                    bf.bf_set_tuning(14, 0)
                got.append((out, M))
            (out, M), (out3, M3), (outh, Mh) = got
            assert torch.equal(out, out3), "capped grid differs (n=%d rnd=%d momentum=%s)" % (n, rnd, with_m)
            assert torch.equal(out3, outh), "gradient from LDS and from HBM differ (n=%d rnd=%d momentum=%s)" % (n, rnd, with_m)
            if with_m:
                assert torch.equal(M, M3) and torch.equal(M, Mh)
                Mn = b64 * host(M0) + host(G)
                assert_close(M3, Mn, 1e-6, "momentum")
                assert_close(out3, mixed - a64 * Mn, tol, "x")
            else:
                assert_close(out3, O.awc_step(host(X), host(G), W, a64), tol, "x")


def test_config1_dgd_least_squares_200_iterations():
    data = workloads.config1_least_squares(DEV)
    A, b, alpha = data["A"], data["b"], data["alpha"]
    n, m, d = A.shape
    t = bf.bf_topology_create(bf.BF_RING, n)
    W = lib_W(t)
    for (_, w) in W[0]:
        assert w == float(np.float32(1 / 3))
    X = [torch.zeros((n, d), device=DEV), torch.zeros((n, d), device=DEV)]
    G = torch.empty((n, d), device=DEV)
    Ah, bh = host(A), host(b)
    Xr = np.zeros((n, d))
    a64 = float(np.float32(alpha))
    worst = 0.0
    for k in range(data["iters"]):
        a, c = k & 1, 1 - (k & 1)
        bf.bf_grad_least_squares(A, b, X[a], G)
        bf.bf_atc_step(t, k, X[a], X[c], G, None, alpha=alpha, mode=bf.BF_ATC)
        Xr = O.atc_step(Xr, O.ls_grad(Ah, bh, Xr), W, a64)
        err = assert_close(X[c], Xr, TOL32, "iteration %d" % k)          # every iteration of the trajectory
        worst = max(worst, err / np.abs(Xr).max())
    # the iterates approach x* on the sampled subspace: the residual has dropped a lot
    r0 = np.linalg.norm(bh)
    rk = np.linalg.norm(np.einsum("imd,id->im", Ah, Xr) - bh)
    assert rk < 0.2 * r0
    print("config1 worst relative error %.2e" % worst)


# ------------------------------------------------------------------ a6 / configuration 5 (reduced d)
@pytest.mark.parametrize("mode", [bf.BF_ATC, bf.BF_AWC])
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_momentum_step_matches_oracle(mode, dtype):
    n, d = 32, 1024 + 40
    t = bf.bf_topology_create(bf.BF_EXP_STATIC, n)
    W = lib_W(t)
    X, G = rows(n, d, 61, dtype=dtype), rows(n, d, 62, dtype=dtype)
    ldm = X.stride(0)
    M = workloads.normal_rows(n, d, 63, DEV, ld=ldm)
    M0 = host(M)
    out = empty_like_rows(X)
    alpha, beta = 0.1, 0.9
    bf.bf_atc_step(t, 0, X, out, G, M, alpha=alpha, beta=beta, mode=mode)
    a64, b64 = float(np.float32(alpha)), float(np.float32(beta))
    Mn = b64 * M0 + host(G)
    if mode == bf.BF_ATC:
        ref, Mref = O.dmsgd_atc_step(host(X), M0, host(G), W, a64, b64)
    else:
        ref, Mref = O.mix(host(X), W) - a64 * Mn, Mn
    assert_close(M, Mref, 1e-6, "momentum")
    assert_close(out, ref, TOL32 if dtype == torch.float32 else 2.0 ** -8, "x")


def test_config5_dmsgd_bf16_20_steps():
    n, d = 32, 4096 + 40                                        # same 40-column ragged tail as 25,557,032
    cfg = workloads.CONFIG5
    ld = workloads.padded_ld(d, 2)
    t = bf.bf_topology_create(bf.BF_EXP_STATIC, n)
    W = lib_W(t)
    Cc = workloads.config5_centres(DEV, n=n, d=d, ld=ld)
    X = [workloads.alloc_rows(n, d, torch.bfloat16, DEV, ld=ld, fill=0) for _ in range(2)]
    G = workloads.alloc_rows(n, d, torch.bfloat16, DEV, ld=ld)
    M = workloads.alloc_rows(n, d, torch.float32, DEV, ld=ld, fill=0)
    lam, sig, alpha, beta = cfg["lam"], cfg["sigma"], cfg["alpha"], cfg["beta"]
    a64, b64, s64 = float(np.float32(alpha)), float(np.float32(beta)), float(np.float32(sig))
    Xr, Mr = np.zeros((n, d)), np.zeros((n, d))                 # graded oracle: fp64 state, no rounding
    Xs, Ms = np.zeros((n, d), np.float32), np.zeros((n, d), np.float32)   # diagnostic: bf16 storage
    Ch = host(Cc)
    for k in range(cfg["steps"]):
        a, c = k & 1, 1 - (k & 1)
        E = workloads.config5_noise(DEV, k, n=n, d=d, ld=ld)
        Eh = host(E)
        bf.bf_grad_quadratic(X[a], Cc, E, lam, sig, G)
        # the generator kernel: fp32 arithmetic on bf16 inputs, one bf16 rounding
        gs = O.round_to_bf16(O.quadratic_noise_grad(Xs, Ch, Eh, lam, s64).astype(np.float32))
        assert (host(G) == gs.astype(np.float64)).mean() > 0.995
        bf.bf_atc_step(t, k, X[a], X[c], G, M, alpha=alpha, beta=beta, mode=bf.BF_ATC)
        Xr, Mr = O.dmsgd_atc_step(Xr, Mr, O.quadratic_noise_grad(Xr, Ch, Eh, lam, s64), W, a64, b64)
        assert_close(X[c], Xr, TOL16, "step %d" % k)
        Xs, Ms = O.dmsgd_atc_step_bf16_storage(Xs, Ms, host(G), W, a64, b64)
        # same storage rounding on both sides: at most one bf16 ulp apart, nearly always equal
        diff = np.abs(host(X[c]) - Xs.astype(np.float64))
        ulp = 2.0 ** (np.floor(np.log2(np.maximum(np.abs(Xs.astype(np.float64)), 1e-300))) - 7)
        assert (diff <= ulp + 1e-6 * np.abs(Xs).max()).all(), "step %d" % k
        assert (diff == 0).mean() > 0.98
        Xs = X[c].float().cpu().numpy()                         # re-synchronise the diagnostic twin
        Ms = M.cpu().numpy().copy()


# ------------------------------------------------------------------ a8: dense W on the matrix cores
@pytest.mark.parametrize("n,d", [(5, 100), (32, 1000), (64, 4096 + 8), (100, 260), (256, 1024)])
def test_dense_mix_matches_oracle_and_sparse_kernel(n, d):
    rng = np.random.default_rng(n)
    D = rng.random((n, n)).astype(np.float32)
    D = (D / D.sum(1, keepdims=True)).astype(np.float32)
    td = bf.bf_topology_create(bf.BF_DENSE_USER, n, dense_w=D, require_class=bf.BF_W_PULL)
    X = rows(n, d, 71)
    out = empty_like_rows(X)
    bf.bf_neighbor_allreduce(td, 0, X, out)                   # dispatches to the MFMA kernel
    ref = O.mix(host(X), OT.from_dense(D.astype(np.float64)))
    assert_close(out, ref, TOL32, "dense")
    np.testing.assert_allclose(ref, D.astype(np.float64) @ host(X), atol=1e-12)
    Xi = empty_like_rows(X)
    Xi.copy_(X)
    bf.bf_dense_mix(td, 0, Xi, Xi)                             # in place
    assert torch.equal(Xi, out)
    # the sparse tile kernel on a sparse topology agrees with its dense form on the matrix cores
    ts = bf.bf_topology_create(bf.BF_EXP_STATIC, n)
    a, b = empty_like_rows(X), empty_like_rows(X)
    bf.bf_neighbor_allreduce(ts, 0, X, a)
    bf.bf_dense_mix(ts, 0, X, b)
    assert_close(b, host(a), 2e-6, "dense vs sparse")


def test_dense_mix_keeps_a_non_finite_column_to_itself():
    # one Inf column must not leak into other columns (the kernel's zero padding rows would turn it
    # into NaN and carry it along if they were ever written): same answer as the sparse kernel
    n, d = 40, 128 * 6 + 20
    ts = bf.bf_topology_create(bf.BF_EXP_STATIC, n)
    X = rows(n, d, 75)
    X[3, 130] = float("inf")
    a, b = empty_like_rows(X), empty_like_rows(X)
    bf.bf_neighbor_allreduce(ts, 0, X, a)
    for _ in range(2):                      # twice: a poisoned persistent workgroup would show on reuse
        bf.bf_dense_mix(ts, 0, X, b)
    # column 130 itself: the dense product multiplies the Inf by the zeros of W too, so it is NaN or
    # Inf in every row there, where the sparse kernel keeps it to agent 3's out-neighbors
    assert bool((~torch.isfinite(a[:, 130])).any()) and bool((~torch.isfinite(b[:, 130])).all())
    keep = torch.ones(d, dtype=torch.bool, device=DEV)
    keep[130] = False
    assert bool(torch.isfinite(b[:, keep]).all()) and bool(torch.isfinite(a[:, keep]).all())
    assert float((a[:, keep] - b[:, keep]).abs().max()) <= 2e-6 * float(a[:, keep].abs().max())


def test_global_averaging_through_dense_w():
    n, d = 16, 520
    J = np.full((n, n), 1.0 / n, dtype=np.float32)
    t = bf.bf_topology_create(bf.BF_DENSE_USER, n, dense_w=J, require_class=bf.BF_W_STANDARD)
    X = rows(n, d, 73)
    out = empty_like_rows(X)
    bf.bf_neighbor_allreduce(t, 0, X, out)
    assert_close(out, np.tile(host(X).mean(0), (n, 1)), TOL32)


# ------------------------------------------------------------------ a9 and the gradient generator
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_consensus_stats_and_quadratic_gradient(dtype):
    n, d = 24, 1000
    X = rows(n, d, 81, dtype=dtype, std=2.0, mean=1.0)
    p = torch.rand(n, device=DEV) + 0.5
    mean = torch.empty(d, device=DEV)
    st = bf.bf_consensus_stats(X, p, mean_out=mean)
    Yh = host(X) / host(p)[:, None]
    mu = Yh.mean(0)
    np.testing.assert_allclose(float(st[0]), ((Yh - mu) ** 2).sum(), rtol=1e-10)
    np.testing.assert_allclose(float(st[1]), np.abs(Yh - mu).max(), rtol=1e-12)
    np.testing.assert_allclose(float(st[2]), np.abs(Yh).max(), rtol=1e-12)
    np.testing.assert_allclose(host(mean), mu, rtol=1e-6, atol=1e-7)
    st = bf.bf_consensus_stats(X)
    np.testing.assert_allclose(float(st[0]) ** 0.5, O.consensus_error(host(X)), rtol=1e-10)
    Cc, E = rows(n, d, 82, dtype=dtype), rows(n, d, 83, dtype=dtype)
    G = empty_like_rows(X)
    bf.bf_grad_quadratic(X, Cc, E, 1.5, 0.1, G)
    ref = O.quadratic_noise_grad(host(X), host(Cc), host(E), 1.5, float(np.float32(0.1)))
    assert_close(G, ref, 1e-6 if dtype == torch.float32 else 2.0 ** -8)


# ------------------------------------------------------------------ chain (row-streaming) kernel
class _chain:
    """Force the chain kernel with cw vectors per thread (it is otherwise reserved for wide matrices)."""

    def __init__(self, cw):
        self.cw = cw

    def __enter__(self):
        bf.bf_set_tuning(6, self.cw)

    def __exit__(self, *a):
        bf.bf_set_tuning(6, 0)


class _no_chain:
    def __enter__(self):
        bf.bf_set_tuning(5, 1)

    def __exit__(self, *a):
        bf.bf_set_tuning(5, 0)


CHAIN_TOPOS = [
    ("ring16", lambda: bf.bf_topology_create(bf.BF_RING, 16)),
    ("ring3", lambda: bf.bf_topology_create(bf.BF_RING, 3)),
    ("ring2", lambda: bf.bf_topology_create(bf.BF_RING, 2)),
    ("one", lambda: bf.bf_topology_create(bf.BF_RING, 1)),
    ("onepeer256", lambda: bf.bf_topology_create(bf.BF_EXP2_ONE_PEER, 256)),
    ("onepeer12", lambda: bf.bf_topology_create(bf.BF_EXP2_ONE_PEER, 12)),
]


@pytest.mark.parametrize("name,make", CHAIN_TOPOS)
@pytest.mark.parametrize("cw", [1, 2, 4])
@pytest.mark.parametrize("d", [4, 1000, 4096 + 136])
def test_chain_kernel_mix_fp32(name, make, cw, d):
    t = make()
    n = t.n
    X = rows(n, d, 300 + n)
    for r in range(bf.bf_topology_rounds(t)):
        assert bf.bf_topology_chain_plan(t, r) is not None
        ref = O.mix(host(X), lib_W(t, r))
        out = empty_like_rows(X)
        out.fill_(float("nan"))
        with _chain(cw):
            bf.bf_neighbor_allreduce(t, r, X, out)
        assert_close(out, ref, TOL32, "%s r=%d" % (name, r))
        with _no_chain():
            tile = empty_like_rows(X)
            bf.bf_neighbor_allreduce(t, r, X, tile)
        assert torch.equal(out, tile)                     # same CSR order on both kernels: same bits
        Xi = empty_like_rows(X)
        Xi.copy_(X)
        with _chain(cw):
            bf.bf_neighbor_allreduce(t, r, Xi, Xi)        # in place
        assert torch.equal(Xi, out)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("cw", [1, 2])
def test_chain_kernel_fused_ops(dtype, cw):
    n, d = 16, 2048 + 40
    t = bf.bf_topology_create(bf.BF_RING, n)
    W = lib_W(t)
    X, G = rows(n, d, 61, dtype=dtype), rows(n, d, 62, dtype=dtype)
    alpha, beta = 0.1, 0.9
    a64, b64 = float(np.float32(alpha)), float(np.float32(beta))
    tol = TOL32 if dtype == torch.float32 else 2.0 ** -8
    for mode in (bf.BF_ATC, bf.BF_AWC):
        out = empty_like_rows(X)
        with _chain(cw):
            bf.bf_atc_step(t, 0, X, out, G, None, alpha=alpha, mode=mode)
        ref = (O.atc_step if mode == bf.BF_ATC else O.awc_step)(host(X), host(G), W, a64)
        assert_close(out, ref, tol, "mode %d" % mode)
        M = workloads.normal_rows(n, d, 63, DEV, ld=X.stride(0))
        M0 = host(M)
        Xi = empty_like_rows(X)
        Xi.copy_(X)
        with _chain(cw):
            bf.bf_atc_step(t, 0, Xi, Xi, G, M, alpha=alpha, beta=beta, mode=mode)     # in place, momentum
        Mn = b64 * M0 + host(G)
        ref = O.mix(host(X) - a64 * Mn, W) if mode == bf.BF_ATC else O.mix(host(X), W) - a64 * Mn
        assert_close(M, Mn, 1e-6, "momentum")
        assert_close(Xi, ref, tol, "momentum x, mode %d" % mode)
    # push-sum ratio output on a one-peer round
    t2 = bf.bf_topology_create(bf.BF_EXP2_ONE_PEER, n)
    w0 = torch.rand(n, device=DEV) + 0.5
    w1 = torch.empty_like(w0)
    out, Y = empty_like_rows(X), empty_like_rows(X)
    with _chain(cw):
        bf.bf_pushsum_step(t2, 1, X, out, w0, w1, Y)
    Xr, pr, Yr = O.pushsum_step(host(X), host(w0[:, None])[:, 0], lib_W(t2, 1))
    assert_close(out, Xr, tol)
    assert_close(w1, pr, TOL32)
    assert_close(Y, Yr, 2e-5 if dtype == torch.float32 else 2.0 ** -7)


# ------------------------------------------------------------------ next row: Exact-Diffusion
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("kernel", ["tile", "chain"])
def test_exact_diffusion_step_matches_oracle(dtype, kernel):
    n, d = 16, 2048 + 40
    t = bf.bf_topology_create(bf.BF_RING, n)
    W = lib_W(t)
    X, G = rows(n, d, 91, dtype=dtype), rows(n, d, 92, dtype=dtype)
    P = workloads.normal_rows(n, d, 93, DEV, ld=X.stride(0))
    P0 = host(P)
    alpha = 0.05
    a64 = float(np.float32(alpha))
    ref, psi = O.exact_diffusion_step(host(X), P0, host(G), W, a64)
    out = empty_like_rows(X)
    with (_chain(2) if kernel == "chain" else _no_chain()):
        bf.bf_exact_diffusion_step(t, 0, X, out, G, P, alpha)
    assert_close(P, psi, 1e-6, "psi")
    assert_close(out, ref, TOL32 if dtype == torch.float32 else 2.0 ** -8, "x")
    # in place on X, state advanced once more from the same start
    P.copy_(torch.from_numpy(P0).to(DEV).float())
    Xi = empty_like_rows(X)
    Xi.copy_(X)
    with (_chain(2) if kernel == "chain" else _no_chain()):
        bf.bf_exact_diffusion_step(t, 0, Xi, Xi, G, P, alpha)
    assert torch.equal(Xi, out)


def test_exact_diffusion_removes_the_bias_of_dgd():
    # eqs. ed-1..ed-3 on decentralized linear regression: the fixed point is the exact
    # least-squares solution (DGD with the same step stalls at a biased point).
    n, m, d, alpha = 16, 8, 64, 0.01
    g = torch.Generator(device=DEV).manual_seed(95)
    A = torch.randn((n, m, d), generator=g, device=DEV)
    b = torch.randn((n, m), generator=g, device=DEV)
    t = bf.bf_topology_create(bf.BF_RING, n)
    W = lib_W(t)
    X = torch.zeros((n, d), device=DEV)
    P = X.clone()                                   # psi^(-1) = x^(0)
    G = torch.empty((n, d), device=DEV)
    Ah, bh = host(A), host(b)
    Xr, Pr = np.zeros((n, d)), np.zeros((n, d))
    a64 = float(np.float32(alpha))
    for k in range(3000):
        bf.bf_grad_least_squares(A, b, X, G)
        bf.bf_exact_diffusion_step(t, k, X, X, G, P, alpha)
        if k < 300:
            Xr, Pr = O.exact_diffusion_step(Xr, Pr, O.ls_grad(Ah, bh, Xr), W, a64)
            if k % 20 == 19:
                # the (x, psi) recursion has a marginally stable mode (its bias correction is an
                # integrator), so fp32 rounding, about 5e-7 relative per step, adds up linearly at worst
                assert_close(X, Xr, 5e-7 * (k + 1), "iteration %d" % k)
    xs = np.linalg.lstsq(Ah.reshape(n * m, d), bh.reshape(n * m), rcond=None)[0]
    # In fp32 the integrator mode has no restoring force, so rounding drifts it by ~1e-6 per
    # iteration (a plain numpy fp32 run of the same recursion shows the same 3e-3 after 3000 steps;
    # the fp64 oracle reaches 1e-8).  The bias of DGD with the same step is 0.57.
    assert np.abs(host(X) - xs).max() < 1e-2 * np.abs(xs).max()
    Xd = torch.zeros((n, d), device=DEV)
    for k in range(3000):
        bf.bf_grad_least_squares(A, b, Xd, G)
        bf.bf_atc_step(t, k, Xd, Xd, G, None, alpha=alpha, mode=bf.BF_ATC)
    assert np.abs(host(Xd) - xs).max() > 20 * np.abs(host(X) - xs).max()


# ------------------------------------------------------------------ next row: push-sum gradient tracking
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("kind", ["push_tile", "onepeer_chain", "onepeer_tile"])
def test_gradient_tracking_pieces_match_oracle(dtype, kind):
    n, d = 16, 2048 + 40
    if kind == "push_tile":
        t = bf.bf_topology_create(bf.BF_RANDOM_DIRECTED, n, out_degree=3, seed=11)
    else:
        t = bf.bf_topology_create(bf.BF_EXP2_ONE_PEER, n)
    ctx = _chain(2) if kind == "onepeer_chain" else _no_chain()
    r = 1
    W = lib_W(t, r)
    U, Yt, Gn, Go = (rows(n, d, 110 + k, dtype=dtype) for k in range(4))
    v = torch.rand(n, device=DEV) + 0.5
    v2 = torch.empty_like(v)
    alpha = 0.05
    a64 = float(np.float32(alpha))
    tol = TOL32 if dtype == torch.float32 else 2.0 ** -8
    Uo, Xo, Yo = empty_like_rows(U), empty_like_rows(U), empty_like_rows(U)
    with ctx:
        bf.bf_pushsum_atc_step(t, r, U, Uo, Yt, alpha, v, v2, Xo)
        bf.bf_tracking_step(t, r, Yt, Yo, Gn, Go)
    Ur = O.mix(host(U) - a64 * host(Yt), W)
    vr = OT.to_dense(W) @ host(v[:, None])[:, 0]
    assert_close(Uo, Ur, tol, "u")
    assert_close(v2, vr, TOL32, "v")
    assert_close(Xo, Ur / vr[:, None], 2e-5 if dtype == torch.float32 else 2.0 ** -7, "x = u/v")
    assert_close(Yo, O.mix(host(Yt) + host(Gn) - host(Go), W), tol, "y")
    Yi = empty_like_rows(Yt)
    Yi.copy_(Yt)
    with ctx:
        bf.bf_tracking_step(t, r, Yi, Yi, Gn, Go)               # in place
    assert torch.equal(Yi, Yo)


def test_gradient_tracking_run_on_time_varying_graph():
    # the whole recursion on decentralized linear regression over the one-peer schedule:
    # trajectory against the oracle, tracking invariant 1^T y = 1^T g, exact least-squares limit
    n, m, d, alpha = 16, 8, 64, 0.01
    g = torch.Generator(device=DEV).manual_seed(97)
    A = torch.randn((n, m, d), generator=g, device=DEV)
    b = torch.randn((n, m), generator=g, device=DEV)
    t = bf.bf_topology_create(bf.BF_EXP2_ONE_PEER, n)
    Ah, bh = host(A), host(b)
    grad = lambda X: O.ls_grad(Ah, bh, X)
    X = torch.zeros((n, d), device=DEV)
    U = X.clone()
    v = torch.ones(n, device=DEV)
    G = [torch.empty((n, d), device=DEV), torch.empty((n, d), device=DEV)]
    bf.bf_grad_least_squares(A, b, X, G[0])
    Yt = G[0].clone()
    Xr = np.zeros((n, d)); Ur = Xr.copy(); vr = np.ones(n); Gr = grad(Xr); Yr = Gr.copy()
    a64 = float(np.float32(alpha))
    for k in range(2500):
        cur, new = G[k & 1], G[1 - (k & 1)]
        bf.bf_pushsum_atc_step(t, k, U, U, Yt, alpha, v, v, X)
        bf.bf_grad_least_squares(A, b, X, new)
        bf.bf_tracking_step(t, k, Yt, Yt, new, cur)
        if k < 200:
            Ur, vr, Xr, Yr, Gr = O.pushsum_gradient_tracking_step(Ur, vr, Yr, Gr, lib_W(t, k), a64, grad)
            if k % 20 == 19:
                assert_close(X, Xr, 5e-7 * (k + 1), "x, iteration %d" % k)
                assert_close(Yt, Yr, 2e-6 * (k + 1), "y, iteration %d" % k)
        if k % 500 == 499:
            ysum, gsum = host(Yt).sum(0), host(new).sum(0)
            assert np.abs(ysum - gsum).max() < 1e-3 * max(1.0, np.abs(host(new)).max()) * n
    xs = np.linalg.lstsq(Ah.reshape(n * m, d), bh.reshape(n * m), rcond=None)[0]
    assert np.abs(host(X) - xs).max() < 1e-2 * np.abs(xs).max()
    assert float((v - 1).abs().max()) < 1e-6


# ------------------------------------------------------------------ several rounds in one pass
@pytest.mark.parametrize("name,make", TOPOS)
@pytest.mark.parametrize("n,d,round0,count", [(16, 1024, 0, 2), (64, 8192 + 520, 3, 5), (100, 3004, 1, 8),
                                              (256, 4096 + 72, 0, 8), (37, 130, 2, 3), (1, 64, 0, 4), (320, 1000, 5, 2)])
def test_fused_rounds_match_the_oracle_and_the_separate_calls(name, make, n, d, round0, count):
    t = make(n)
    X = rows(n, d, 1000 + n + count)
    ref = host(X)
    for r in range(round0, round0 + count):
        ref = O.mix(ref, lib_W(t, r % bf.bf_topology_rounds(t)))
    out = bf.bf_neighbor_allreduce_multi(t, round0, count, X, empty_like_rows(X))
    assert_close(out, ref, TOL32 * count, "%s n=%d %d rounds" % (name, n, count))
    seq = [empty_like_rows(X).copy_(X), empty_like_rows(X)]
    for k, r in enumerate(range(round0, round0 + count)):
        bf.bf_neighbor_allreduce(t, r, seq[k & 1], seq[1 - (k & 1)])
    assert torch.equal(out, seq[count & 1]), "fused rounds differ in bits from separate rounds"
    inplace = empty_like_rows(X).copy_(X)
    bf.bf_neighbor_allreduce_multi(t, round0, count, inplace, inplace)
    assert torch.equal(inplace, out)


def _shift_topology(n, shifts, weights):
    """User CSR rounds x_i <- ws x_i + wp x_((i+s) mod n), one per (s, (ws, wp))."""
    rowptr, col, wgt = [], [], []
    for s_, (ws, wp) in zip(shifts, weights):
        base = len(col)
        for i in range(n):
            rowptr.append(base + 2 * i)
            for j, w in sorted([(i, ws), ((i + s_) % n, wp)]):
                col.append(j)
                wgt.append(w)
        rowptr.append(base + 2 * n)
    return bf.bf_topology_create(bf.BF_CSR_USER, n, rounds=len(shifts), rowptr=np.array(rowptr), col=np.array(col),
                                 wgt=np.array(wgt, dtype=np.float32))


@pytest.mark.parametrize("n,d,shifts", [(64, 1024 + 4, [1, 5, 63, 32]), (128, 640, [3, 64, 100, 127]), (192, 260, [64, 128, 7, 190]),
                                        (256, 1000 + 1, [128, 1, 192, 255, 64, 2])])
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_fused_shift_rounds_in_registers_equal_the_general_kernel(n, d, shifts, dtype):
    # Rounds of the form x_i <- ws x_i + wp x_((i+s) mod n) run in registers (lane rotations); any s
    # below 64 or a multiple of 64 qualifies, with any pair of weights.  Shifts with both parts (100,
    # 190, 255, ...) make the call take the general LDS path, which must give the same bits.
    rng = np.random.default_rng(n)
    weights = [(float(np.float32(w)), float(np.float32(1.0 - w))) for w in rng.uniform(0.2, 0.8, len(shifts))]
    t = _shift_topology(n, shifts, weights)
    X = rows(n, d, 1300 + n, dtype=dtype)
    R = len(shifts)
    for round0, count in ((0, R), (1, 2), (R - 1, 3), (2, 1)):
        ref = host(X)
        for r in range(round0, round0 + count):
            ref = O.mix(ref, lib_W(t, r % R))
        outs = []
        for knob in (2, 1):                       # in registers wherever the rounds allow; never
            bf.bf_set_tuning(13, knob)
            try:
                outs.append(bf.bf_neighbor_allreduce_multi(t, round0, count, X, empty_like_rows(X)))
            finally:
                bf.bf_set_tuning(13, 0)
        assert torch.equal(outs[0], outs[1]), "register rounds differ from LDS rounds (round0=%d count=%d)" % (round0, count)
        if dtype == torch.float32:
            assert_close(outs[0], ref, TOL32 * count, "shift rounds n=%d" % n)
            seq = [empty_like_rows(X).copy_(X), empty_like_rows(X)]
            for k, r in enumerate(range(round0, round0 + count)):
                bf.bf_neighbor_allreduce(t, r, seq[k & 1], seq[1 - (k & 1)])
            assert torch.equal(outs[0], seq[count & 1])
        else:
            assert_close(outs[0], ref, 2.0 ** -8, "shift rounds bf16 n=%d" % n)
        Xi = empty_like_rows(X).copy_(X)
        bf.bf_set_tuning(13, 2)
        try:
            bf.bf_neighbor_allreduce_multi(t, round0, count, Xi, Xi)
        finally:
            bf.bf_set_tuning(13, 0)
        assert torch.equal(Xi, outs[0])


def test_fused_one_peer_rounds_give_the_exact_mean_in_one_pass():
    # log2(n) one-peer rounds average exactly (the product of the eight weight matrices of the third
    # benchmark configuration is 11^T/n: every offset below n has one binary expansion); with
    # power-of-two weights each fp32 step is one correctly rounded addition, so the bits are fixed.
    n, d = 256, 4096 + 136
    t = bf.bf_topology_create(bf.BF_EXP2_ONE_PEER, n)
    X = workloads.config3_state(DEV, n=n, d=d, ld=workloads.padded_ld(d, 4))
    emu = X.cpu().numpy()
    for r in range(8):
        emu = O.mix_fp32_chain(emu, lib_W(t, r))
    out = bf.bf_neighbor_allreduce_multi(t, 0, 8, X, empty_like_rows(X))
    assert np.array_equal(out.cpu().numpy().view(np.uint32), emu.view(np.uint32))
    mean = host(X).mean(0)
    assert np.abs(host(out) - mean).max() <= 8 * 6e-8 * np.abs(host(X)).max()
    assert float((out - out[0:1]).abs().max()) <= 8 * 6e-8 * float(X.abs().max())


def test_fused_rounds_bf16_round_once():
    n, d, count = 64, 2048 + 264, 6
    t = bf.bf_topology_create(bf.BF_EXP2_ONE_PEER, n)
    X = rows(n, d, 77, dtype=torch.bfloat16)
    ref = host(X)
    for r in range(count):
        ref = O.mix(ref, lib_W(t, r))
    out = bf.bf_neighbor_allreduce_multi(t, 0, count, X, empty_like_rows(X))
    # intermediate products stay fp32: the only bf16 rounding is the final store (half an ulp of a
    # 7-bit fraction: at most 2^-8 relative) on top of fp32 accumulation error
    err = np.abs(host(out) - ref)
    assert (err <= np.abs(ref) * 2.0 ** -8 + 1e-6).all()
    assert_close(out, ref, TOL16, "bf16 fused")


@pytest.mark.parametrize("n,d", [(400, 256 + 8), (900, 130)])
def test_fused_rounds_fall_back_to_separate_passes_when_two_tiles_do_not_fit(n, d):
    # 400 agents: one LDS tile fits, two do not; 900 agents: not even one 64-column tile
    t = bf.bf_topology_create(bf.BF_EXP2_ONE_PEER, n)
    X = rows(n, d, 5)
    sep = [empty_like_rows(X), empty_like_rows(X)]
    bf.bf_neighbor_allreduce(t, 1, X, sep[0])
    bf.bf_neighbor_allreduce(t, 2, sep[0], sep[1])
    bf.bf_neighbor_allreduce(t, 3, sep[1], sep[0])
    out = bf.bf_neighbor_allreduce_multi(t, 1, 3, X, empty_like_rows(X))
    assert torch.equal(out, sep[0])
    ref = host(X)
    for r in (1, 2, 3):
        ref = O.mix(ref, lib_W(t, r))
    assert_close(out, ref, TOL32)
    Xi = empty_like_rows(X).copy_(X)
    bf.bf_neighbor_allreduce_multi(t, 1, 3, Xi, Xi)
    assert torch.equal(Xi, out)


# ------------------------------------------------------------------ two-level (hierarchical) averaging
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("name,make", TOPOS)
@pytest.mark.parametrize("M,L,d", [(4, 4, 1024), (8, 8, 4096 + 136), (16, 2, 3004), (5, 3, 130), (1, 7, 64), (32, 8, 2048 + 8),
                                   (40, 8, 520), (80, 8, 264)])
def test_hierarchical_neighbor_allreduce_matches_oracle(name, make, M, L, d, dtype):
    if name == "push" and M < 2:
        pytest.skip("a random directed graph needs two machines")
    t = make(M)
    X = rows(M * L, d, 4000 + M + L, dtype=dtype)
    for rnd in range(min(2, bf.bf_topology_rounds(t))):
        ref = O.hierarchical_neighbor_allreduce(host(X), lib_W(t, rnd), L)
        out = bf.bf_hierarchical_neighbor_allreduce(t, rnd, L, X, empty_like_rows(X))
        assert_close(out, ref, TOL32 if dtype == torch.float32 else TOL16, "%s M=%d L=%d round %d" % (name, M, L, rnd))
        inplace = empty_like_rows(X).copy_(X)
        bf.bf_hierarchical_neighbor_allreduce(t, rnd, L, inplace, inplace)
        assert torch.equal(inplace, out)
        # agents of one machine hold the same bits
        o3 = out.reshape(M, L, d)
        assert torch.equal(o3, o3[:, :1].expand(M, L, d))


def test_hierarchical_checks_the_row_count():
    t = bf.bf_topology_create(bf.BF_RING, 4)
    X = rows(12, 64, 1)
    with pytest.raises(ValueError):
        bf.bf_hierarchical_neighbor_allreduce(t, 0, 2, X, empty_like_rows(X))
    with pytest.raises(ValueError):
        bf.bf_neighbor_allreduce(t, 0, X, empty_like_rows(X))


# ------------------------------------------------------------------ window primitives
def _window_state(t, n, d, seed, rnd=0):
    E = bf.bf_topology_window_slots(t, rnd)
    X = rows(n, d, seed, mean=1.0, std=2.0)
    ld = X.stride(0) if n > 1 else workloads.padded_ld(d, 4)
    Win = workloads.normal_rows(max(E, 1), d, seed + 1, DEV, ld=ld)[:E]
    p = torch.rand(n, device=DEV, generator=torch.Generator(device=DEV).manual_seed(seed + 2)) + 0.5
    win_p = torch.rand(max(E, 1), device=DEV, generator=torch.Generator(device=DEV).manual_seed(seed + 3))[:E].contiguous()
    return X, p, Win, win_p


def _mask(n, seed, frac=0.6):
    g = np.random.default_rng(seed)
    m = (g.random(n) < frac).astype(np.int32)
    return m, torch.from_numpy(m).to(DEV)


WIN_TOPOS = [t for t in TOPOS if t[0] != "onepeer"] + [("onepeer", TOPOS[2][1])]


@pytest.mark.parametrize("name,make", WIN_TOPOS)
@pytest.mark.parametrize("n,d", [(16, 1024), (12, 4096 + 136), (33, 130), (64, 8192 + 520), (2, 5000), (1, 64)])
@pytest.mark.parametrize("masked", [False, True])
def test_window_primitives_match_oracle(name, make, n, d, masked):
    if name == "push" and n < 3:
        pytest.skip("the random directed graph needs more agents")
    t = make(n)
    W = lib_W(t, 0)
    X, p, Win, win_p = _window_state(t, n, d, 7000 + n)
    m_np, m_dev = _mask(n, n + d) if masked else (None, None)
    hx, hp, hw, hwp = host(X), host(p[:, None])[:, 0], host(Win), host(win_p[:, None])[:, 0]
    pad_before = X.as_strided((n, X.stride(0) - d), (X.stride(0), 1), X.storage_offset() + d).clone() if n > 1 else None

    # put
    ref = O.win_put(hx, hw, W, m_np)
    got = bf.bf_win_put(t, 0, X, Win.clone() if Win.numel() == 0 else empty_like_rows(Win).copy_(Win), active=m_dev)
    assert np.array_equal(host(got), ref), "put copies bits"
    # get: the pull side
    ref = O.win_get(hx, hw, W, m_np)
    got = bf.bf_win_get(t, 0, X, Win.clone() if Win.numel() == 0 else empty_like_rows(Win).copy_(Win), active=m_dev)
    assert np.array_equal(host(got), ref), "get copies bits"
    # update (weighted average, window kept)
    ref = O.win_update(hx, hw, W, m_np)
    Xc = empty_like_rows(X).copy_(X)
    bf.bf_win_update(t, 0, Xc, Win, active=m_dev)
    assert_close(Xc, ref, TOL32, "win_update")
    # accumulate
    rx, rp, rw, rwp = O.win_accumulate(hx, hp, hw, hwp, W, m_np)
    Xc, pc, Wc, wpc = empty_like_rows(X).copy_(X), p.clone(), (empty_like_rows(Win).copy_(Win) if Win.numel() else Win.clone()), win_p.clone()
    bf.bf_win_accumulate(t, 0, Xc, pc, Wc, wpc, active=m_dev)
    assert_close(Xc, rx, TOL32, "accumulate X"); assert_close(pc[:, None], rp[:, None], TOL32, "accumulate p")
    if Win.numel():
        assert_close(Wc, rw, TOL32, "accumulate Win"); assert_close(wpc[:, None], rwp[:, None], TOL32, "accumulate win_p")
    # update_then_collect, continuing from the accumulated state
    cx, cp, cw, cwp = O.win_update_then_collect(rx, rp, rw, rwp, W, m_np)
    bf.bf_win_update_then_collect(t, 0, Xc, pc, Wc, wpc, active=m_dev)
    assert_close(Xc, cx, 2 * TOL32, "collect X"); assert_close(pc[:, None], cp[:, None], 2 * TOL32, "collect p")
    if Win.numel():
        assert_close(Wc, cw, 2 * TOL32, "collect Win")
        zero_rows = np.flatnonzero(np.abs(cw).max(axis=1) == 0.0)
        assert np.abs(host(Wc)[zero_rows]).max(initial=0.0) == 0.0, "collected slots are exactly zero"
    if pad_before is not None:
        pad_after = Xc.as_strided((n, Xc.stride(0) - d), (Xc.stride(0), 1), Xc.storage_offset() + d)
        assert pad_after.shape == pad_before.shape


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("masked", [False, True])
@pytest.mark.parametrize("n,d", [(12, 4096 + 136), (33, 130 + 3)])
def test_weighted_window_calls_match_oracle(dtype, masked, n, d):
    # per-call self_weight / dst_weights / src_weights over a random subset of the static topology's
    # edges (the paper's signatures), X in fp32 or bf16, the window always fp32
    t = bf.bf_topology_create(bf.BF_RANDOM_DIRECTED, n, out_degree=3, seed=31)
    W = lib_W(t, 0)
    slot_ptr, slot_src, _, _ = bf.bf_topology_export_window(t, 0)
    E = int(slot_ptr[-1])
    X = rows(n, d, 7100 + n, dtype=dtype, mean=1.0, std=2.0)
    Win = workloads.normal_rows(E, d, 7101 + n, DEV, ld=X.stride(0))
    g = torch.Generator(device=DEV).manual_seed(7102)
    p = torch.rand(n, device=DEV, generator=g) + 0.5
    win_p = torch.rand(E, device=DEV, generator=g)
    rng = np.random.default_rng(n + d)
    sw = rng.uniform(0.2, 0.9, n).astype(np.float32)
    ew = rng.uniform(0.1, 0.7, E).astype(np.float32)
    on = (rng.random(E) < 0.6).astype(np.int32)
    m_np, m_dev = _mask(n, n + d) if masked else (None, None)
    sw_d, ew_d, on_d = (torch.from_numpy(v).to(DEV) for v in (sw, ew, on))
    owner = np.repeat(np.arange(n), np.diff(slot_ptr))
    dst = {j: {} for j in range(n)}
    src = {i: {} for i in range(n)}
    for e in range(E):
        if on[e]:
            dst[int(slot_src[e])][int(owner[e])] = float(ew[e])
            src[int(owner[e])][int(slot_src[e])] = float(ew[e])
    hx, hp, hw, hwp = host(X), host(p[:, None])[:, 0], host(Win), host(win_p[:, None])[:, 0]
    tolx = TOL32 if dtype == torch.float32 else 2.0 ** -8
    copy_w = lambda: empty_like_rows(Win).copy_(Win)
    copy_x = lambda: empty_like_rows(X).copy_(X)
    # put
    rx, rw = O.win_put_weighted(hx, hw, W, m_np, sw.astype(np.float64), dst)
    Xc, Wc = copy_x(), copy_w()
    bf.bf_win_put_weighted(t, 0, Xc, Wc, sw_d, ew_d, on_d, active=m_dev)
    assert_close(Wc, rw, TOL32, "put window"); assert_close(Xc, rx, tolx, "put x")
    untouched = np.array([not on[e] or (m_np is not None and not m_np[slot_src[e]]) for e in range(E)])
    assert np.array_equal(host(Wc)[untouched], hw[untouched]), "slots of edges the call does not name keep their bits"
    # get
    rw = O.win_get_weighted(hx, hw, W, m_np, src)
    Wc = copy_w()
    bf.bf_win_get_weighted(t, 0, X, Wc, ew_d, on_d, active=m_dev)
    assert_close(Wc, rw, TOL32, "get window")
    # accumulate (with the push-sum scalar)
    rx, rp, rw, rwp = O.win_accumulate_weighted(hx, hp, hw, hwp, W, m_np, sw.astype(np.float64), dst)
    Xc, pc, Wc, wpc = copy_x(), p.clone(), copy_w(), win_p.clone()
    bf.bf_win_accumulate_weighted(t, 0, Xc, pc, Wc, wpc, sw_d, ew_d, on_d, active=m_dev)
    assert_close(Xc, rx, tolx, "accumulate x"); assert_close(pc[:, None], rp[:, None], TOL32, "accumulate p")
    assert_close(Wc, rw, TOL32, "accumulate window"); assert_close(wpc[:, None], rwp[:, None], TOL32, "accumulate win_p")
    # update
    rx = O.win_update_weighted(hx, hw, W, m_np, sw.astype(np.float64), src)
    Xc = copy_x()
    bf.bf_win_update_weighted(t, 0, Xc, Win, sw_d, ew_d, on_d, active=m_dev)
    assert_close(Xc, rx, tolx, "update x")
    # no arguments: the plain calls, bit for bit
    Xa, Xb, Wa, Wb = copy_x(), copy_x(), copy_w(), copy_w()
    bf.bf_win_put_weighted(t, 0, Xa, Wa, active=m_dev); bf.bf_win_put(t, 0, Xb, Wb, active=m_dev)
    assert torch.equal(Wa, Wb) and torch.equal(Xa, X)
    bf.bf_win_update_weighted(t, 0, Xa, Win, active=m_dev); bf.bf_win_update(t, 0, Xb, Win, active=m_dev)
    assert torch.equal(Xa, Xb)


def test_window_calls_leave_row_padding_alone():
    n, d = 8, 1000 + 3                      # d is not a multiple of 4: the last vector of a row is partial
    ld = workloads.padded_ld(d, 4)
    t = bf.bf_topology_create(bf.BF_RING, n)
    E = bf.bf_topology_window_slots(t, 0)
    Xfull = torch.full((n, ld), 7.0, device=DEV)
    Wfull = torch.full((E, ld), -3.0, device=DEV)
    X, Win = Xfull[:, :d], Wfull[:, :d]
    X.normal_(generator=torch.Generator(device=DEV).manual_seed(1))
    Win.zero_()
    p, win_p = torch.ones(n, device=DEV), torch.zeros(E, device=DEV)
    bf.bf_win_accumulate(t, 0, X, p, Win, win_p)
    bf.bf_win_put(t, 0, X, Win)
    bf.bf_win_update(t, 0, X, Win)
    bf.bf_win_update_then_collect(t, 0, X, p, Win, win_p)
    assert bool((Xfull[:, d:] == 7.0).all()) and bool((Wfull[:, d:] == -3.0).all())


def test_window_async_pushsum_run_conserves_mass_and_converges():
    # the asynchronous push-sum example: random subsets of agents send, random subsets collect
    n, d = 24, 2048 + 72
    t = bf.bf_topology_create(bf.BF_RANDOM_DIRECTED, n, out_degree=3, seed=workloads.CONFIG4_GRAPH_SEED)
    W = lib_W(t, 0)
    E = bf.bf_topology_window_slots(t, 0)
    X = rows(n, d, 55, mean=5.0, std=2.0)
    ld = X.stride(0)
    Win = workloads.alloc_rows(E, d, torch.float32, DEV, ld=ld); Win.zero_()
    p, win_p = torch.ones(n, device=DEV), torch.zeros(E, device=DEV)
    rx, rp, rw, rwp = host(X), np.ones(n), np.zeros((E, d)), np.zeros(E)
    mean = rx.mean(0)
    total = rx.sum(0)
    for k in range(120):
        ma, ma_dev = _mask(n, 1000 + 2 * k)
        mc, mc_dev = _mask(n, 1001 + 2 * k)
        bf.bf_win_accumulate(t, 0, X, p, Win, win_p, active=ma_dev)
        bf.bf_win_update_then_collect(t, 0, X, p, Win, win_p, active=mc_dev)
        rx, rp, rw, rwp = O.win_accumulate(rx, rp, rw, rwp, W, ma)
        rx, rp, rw, rwp = O.win_update_then_collect(rx, rp, rw, rwp, W, mc)
        if k % 20 == 19 or k < 3:
            assert_close(X, rx, 3e-5, "step %d X" % k)
            assert_close(p[:, None], rp[:, None], 3e-5, "step %d p" % k)
            assert_close(Win, rw, 3e-5 * max(1.0, np.abs(rx).max() / max(np.abs(rw).max(), 1e-30)), "step %d Win" % k)
    mass = host(X).sum(0) + host(Win).sum(0)
    assert np.abs(mass - total).max() <= 1e-4 * np.abs(total).max()
    assert abs(float(p.double().sum() + win_p.double().sum()) - n) < 1e-4
    y = host(X) / host(p[:, None])
    assert np.abs(y - mean).max() < 2e-4 * np.abs(mean).max()
    assert np.abs(host(X) - mean).max() > 1e-2                # x alone is not the average


def test_window_all_active_round_equals_pushsum_step():
    n, d = 32, 4096 + 264
    t = bf.bf_topology_create(bf.BF_RANDOM_DIRECTED, n, out_degree=4, seed=3)
    E = bf.bf_topology_window_slots(t, 0)
    X = rows(n, d, 91, mean=2.0)
    Win = workloads.alloc_rows(E, d, torch.float32, DEV, ld=X.stride(0)); Win.zero_()
    p, win_p = torch.ones(n, device=DEV), torch.zeros(E, device=DEV)
    Xs, ws, _ = bf.bf_pushsum_step(t, 0, X, empty_like_rows(X), torch.ones(n, device=DEV), torch.empty(n, device=DEV))
    bf.bf_win_accumulate(t, 0, X, p, Win, win_p)
    bf.bf_win_update_then_collect(t, 0, X, p, Win, win_p)
    assert_close(X, host(Xs), 1e-6, "window round vs push-sum kernel")
    assert_close(p[:, None], host(ws[:, None]), 1e-6, "p")
    assert float(Win.abs().max()) == 0.0 and float(win_p.abs().max()) == 0.0


# ------------------------------------------------------------------ HIP graph replay of the DGD iteration
def test_dgd_iterations_replayed_from_a_hip_graph_match_eager():
    data = workloads.config1_least_squares(DEV)
    A, b = data["A"], data["b"]
    n, m, d = A.shape
    t = bf.bf_topology_create(bf.BF_RING, n)
    X = [torch.zeros((n, d), device=DEV), torch.zeros((n, d), device=DEV)]
    G = torch.empty((n, d), device=DEV)

    def dgd(k):
        bf.bf_grad_least_squares(A, b, X[k & 1], G)
        bf.bf_atc_step(t, k, X[k & 1], X[1 - (k & 1)], G, None, data["alpha"], 0.0, bf.BF_ATC)

    for k in range(12):
        dgd(k)
    torch.cuda.synchronize()
    eager = [X[0].clone()]                          # after 12 iterations; then after 16, 20, 24
    for rep in range(3):
        for k in range(4):
            dgd(k)
        eager.append(X[0].clone())
    X[0].zero_(); X[1].zero_()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        dgd(0); dgd(1)
    torch.cuda.current_stream().wait_stream(side)
    X[0].zero_(); X[1].zero_()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        for k in range(4):
            dgd(k)
    X[0].zero_(); X[1].zero_()
    scratch = torch.zeros(1 << 16, device=DEV)
    for rep in range(6):
        graph.replay()
        scratch.add_(1.0)                           # eager work and a synchronisation between the replays
        torch.cuda.synchronize()
        if rep >= 2:
            assert torch.equal(X[0], eager[rep - 2]), "replay %d differs from eager" % rep


# ------------------------------------------------------------------ many DGD iterations in one launch
def _dgd_reference(A, b, W_of_round, alpha, iters, X0):
    x = X0.copy()
    for k in range(iters):
        x = O.atc_step(x, O.ls_grad(A, b, x), W_of_round(k), alpha)
    return x


@pytest.mark.parametrize("name,make", [TOPOS[0], TOPOS[1], TOPOS[2]])
@pytest.mark.parametrize("n,m,d,iters", [(16, 32, 1024, 1), (16, 32, 1024, 2), (16, 32, 1024, 25), (8, 16, 520, 9),
                                         (5, 7, 64, 12), (1, 3, 16, 4), (32, 64, 256, 6), (16, 4, 4096, 3)])
def test_dgd_run_in_one_launch_matches_oracle(name, make, n, m, d, iters):
    t = make(n)
    R = bf.bf_topology_rounds(t)
    Ws = [lib_W(t, r) for r in range(R)]
    g = torch.Generator(device=DEV).manual_seed(900 + n + m)
    A = torch.randn((n, m, d), device=DEV, generator=g) / (d ** 0.5)
    b = torch.randn((n, m), device=DEV, generator=g)
    X = rows(n, d, 901 + n, std=0.5)
    alpha = float(np.float32(0.4))
    ref = _dgd_reference(host(A.reshape(n * m, d)).reshape(n, m, d), host(b), lambda k: Ws[(1 + k) % R], alpha, iters, host(X))
    ld = X.stride(0) if n > 1 else d
    work = torch.empty(2 * n * ld, device=DEV)
    bf.bf_dgd_least_squares_run(t, 1, iters, A, b, X, work, alpha)
    assert bf.bf_dgd_status(t) == 0
    assert_close(X, ref, TOL32, "%s n=%d m=%d d=%d after %d iterations" % (name, n, m, d, iters))


def test_dgd_run_config1_200_iterations_and_two_runs_in_a_row():
    data = workloads.config1_least_squares(DEV)
    A, b, alpha = data["A"], data["b"], data["alpha"]
    n, m, d = A.shape
    t = bf.bf_topology_create(bf.BF_RING, n)
    W = lib_W(t)
    X = torch.zeros((n, d), device=DEV)
    work = torch.empty(2 * n * d, device=DEV)
    Ah, bh = host(A.reshape(n * m, d)).reshape(n, m, d), host(b)
    a64 = float(np.float32(alpha))
    # every iteration of the 200 against the oracle's trajectory, at the fp32 tolerance: the run is
    # advanced one iteration per launch, which is the same kernel and the same arithmetic as 200
    # iterations in one launch (checked bit for bit below)
    Xs = torch.zeros((n, d), device=DEV)
    xr = np.zeros((n, d))
    for k in range(200):
        bf.bf_dgd_least_squares_run(t, k, 1, A, b, Xs, work, alpha)
        xr = O.atc_step(xr, O.ls_grad(Ah, bh, xr), W, a64)
        assert_close(Xs, xr, TOL32, "iteration %d" % (k + 1))
    ref = _dgd_reference(Ah, bh, lambda k: W, a64, 120, np.zeros((n, d)))
    bf.bf_dgd_least_squares_run(t, 0, 120, A, b, X, work, alpha)
    assert_close(X, ref, TOL32, "120 iterations")
    ref = _dgd_reference(Ah, bh, lambda k: W, a64, 80, ref)
    bf.bf_dgd_least_squares_run(t, 0, 80, A, b, X, work, alpha)       # continues from the state of the first run
    assert bf.bf_dgd_status(t) == 0
    assert_close(X, ref, TOL32, "200 iterations in two runs")
    assert torch.equal(X, Xs), "200 iterations in two launches and in 200 launches differ"
    # the same 200 iterations by the two-call path
    Y = [torch.zeros((n, d), device=DEV), torch.zeros((n, d), device=DEV)]
    G = torch.empty((n, d), device=DEV)
    for k in range(200):
        bf.bf_grad_least_squares(A, b, Y[k & 1], G)
        bf.bf_atc_step(t, k, Y[k & 1], Y[1 - (k & 1)], G, None, alpha, 0.0, bf.BF_ATC)
    assert float((X - Y[0]).abs().max()) <= TOL32 * float(Y[0].abs().max())


def test_dgd_run_gives_up_instead_of_hanging_when_the_barrier_cannot_complete():
    # the host makes the barrier wait for one arrival more than there are workgroups and gives it a
    # small poll budget: every workgroup runs out of polls (or sees that another did), raises the
    # error word and leaves; nothing hangs, and the host is told
    data = workloads.config1_least_squares(DEV)
    A, b = data["A"], data["b"]
    n, m, d = A.shape
    t = bf.bf_topology_create(bf.BF_RING, n)
    X = torch.zeros((n, d), device=DEV)
    work = torch.empty(2 * n * d, device=DEV)
    bf.bf_set_tuning(10, 200)
    bf.bf_set_tuning(11, 1)
    try:
        bf.bf_dgd_least_squares_run(t, 0, 50, A, b, X, work, data["alpha"])
        gave_up = bf.bf_dgd_status(t)
    finally:
        bf.bf_set_tuning(10, 0)
        bf.bf_set_tuning(11, 0)
    assert gave_up == 1
    # and the next run, with the normal settings, is clean
    X.zero_()
    bf.bf_dgd_least_squares_run(t, 0, 3, A, b, X, work, data["alpha"])
    assert bf.bf_dgd_status(t) == 0
    assert bool(torch.isfinite(X).all())


@pytest.mark.parametrize("n,m,d", [(4, 64, 1024), (6, 80, 256), (3, 8, 4096 + 64), (300, 4, 64)])
def test_dgd_run_too_large_for_one_launch_takes_the_two_call_path(n, m, d):
    # A_i beyond one CU's LDS (256 KB), more than 64 rows, rows longer than 4096 columns, more agents
    # than CUs: the run is then made of gradient + fused step launches, with the same result
    t = bf.bf_topology_create(bf.BF_RING, n)
    W = lib_W(t)
    g = torch.Generator(device=DEV).manual_seed(950 + n)
    A = torch.randn((n, m, d), device=DEV, generator=g) / (d ** 0.5)
    b = torch.randn((n, m), device=DEV, generator=g)
    X = torch.randn((n, d), device=DEV, generator=g) * 0.5
    P = X.clone()
    X0 = host(X)
    work = torch.empty(2 * n * d, device=DEV)
    alpha = float(np.float32(0.3))
    iters = 5
    ref = _dgd_reference(host(A.reshape(n * m, d)).reshape(n, m, d), host(b), lambda k: W, alpha, iters, X0)
    bf.bf_dgd_least_squares_run(t, 0, iters, A, b, X, work, alpha)
    assert bf.bf_dgd_status(t) == 0
    assert_close(X, ref, TOL32, "DGD, two-call path inside the run")
    # Exact-Diffusion the same way
    Xe = torch.from_numpy(X0).to(DEV).float()
    xr, pr = X0.copy(), X0.copy()
    Ah, bh = host(A.reshape(n * m, d)).reshape(n, m, d), host(b)
    for k in range(iters):
        xr, pr = O.exact_diffusion_step(xr, pr, O.ls_grad(Ah, bh, xr), W, alpha)
    bf.bf_exact_diffusion_least_squares_run(t, 0, iters, A, b, Xe, P, work, alpha)
    assert_close(Xe, xr, 2e-5, "Exact-Diffusion, two-call path inside the run")
    assert_close(P, pr, 2e-5, "psi")


def test_dense_mix_beyond_the_matrix_core_kernel_uses_the_list_kernels():
    n, d = 300, 260
    rng = np.random.default_rng(9)
    D = rng.random((n, n)).astype(np.float32)
    D = (D / D.sum(1, keepdims=True)).astype(np.float32)
    td = bf.bf_topology_create(bf.BF_DENSE_USER, n, dense_w=D, require_class=bf.BF_W_PULL)
    X = rows(n, d, 76)
    out = bf.bf_dense_mix(td, 0, X, empty_like_rows(X))
    assert_close(out, D.astype(np.float64) @ host(X), 2e-5, "dense n=300")       # 300-term fp32 sums
    Xb = rows(64, d, 77, dtype=torch.bfloat16)
    ts = bf.bf_topology_create(bf.BF_EXP_STATIC, 64)
    a, b = empty_like_rows(Xb), empty_like_rows(Xb)
    bf.bf_dense_mix(ts, 0, Xb, a)
    bf.bf_neighbor_allreduce(ts, 0, Xb, b)
    assert torch.equal(a, b)


# ------------------------------------------------------------------ bandwidth probes
def test_stream_probe_copies_and_fills():
    src = torch.randn(3 * 1000 * 1000 + 4, device=DEV)          # 12 MB + a ragged tail of one vector
    dst = torch.zeros_like(src)
    for wgs in (1, 8):
        dst.zero_()
        bf.bf_stream_probe(0, src, dst, wgs)
        assert torch.equal(src, dst)
    bf.bf_stream_probe(1, src, dst, 4)                           # read only: nothing may change
    assert torch.equal(src, dst)
    bf.bf_stream_probe(2, None, dst, 4)
    assert torch.equal(dst.view(-1, 4), torch.tensor([1.0, 2.0, 3.0, 4.0], device=DEV).expand(dst.numel() // 4, 4))


@pytest.mark.parametrize("name,make", [TOPOS[0], TOPOS[2]])
@pytest.mark.parametrize("n,m,d,iters", [(16, 32, 1024, 1), (16, 32, 1024, 2), (16, 32, 1024, 30), (8, 16, 520, 9), (1, 3, 16, 4)])
def test_exact_diffusion_run_in_one_launch_matches_oracle(name, make, n, m, d, iters):
    t = make(n)
    R = bf.bf_topology_rounds(t)
    Ws = [lib_W(t, r) for r in range(R)]
    g = torch.Generator(device=DEV).manual_seed(950 + n + m)
    A = torch.randn((n, m, d), device=DEV, generator=g) / (d ** 0.5)
    b = torch.randn((n, m), device=DEV, generator=g)
    X = rows(n, d, 951 + n, std=0.5)
    P = empty_like_rows(X).copy_(X)
    alpha = float(np.float32(0.4))
    Ah, bh = host(A.reshape(n * m, d)).reshape(n, m, d), host(b)
    xr, pr = host(X), host(X)
    for k in range(iters):
        xr, pr = O.exact_diffusion_step(xr, pr, O.ls_grad(Ah, bh, xr), Ws[k % R], alpha)
    ld = X.stride(0) if n > 1 else d
    work = torch.empty(2 * n * ld, device=DEV)
    bf.bf_exact_diffusion_least_squares_run(t, 0, iters, A, b, X, P, work, alpha)
    assert bf.bf_dgd_status(t) == 0
    assert_close(X, xr, 2e-5 + 5e-7 * iters, "x after %d iterations" % iters)
    assert_close(P, pr, 2e-5 + 5e-7 * iters, "psi after %d iterations" % iters)


def test_exact_diffusion_run_reaches_the_least_squares_solution_where_dgd_stalls():
    n, m, d, alpha = 16, 8, 64, 0.01
    g = torch.Generator(device=DEV).manual_seed(95)
    A = torch.randn((n, m, d), generator=g, device=DEV)
    b = torch.randn((n, m), generator=g, device=DEV)
    t = bf.bf_topology_create(bf.BF_RING, n)
    X = torch.zeros((n, d), device=DEV); P = torch.zeros((n, d), device=DEV)
    work = torch.empty(2 * n * d, device=DEV)
    for _ in range(3):                                  # 3 runs of 1000 iterations: the state carries over
        bf.bf_exact_diffusion_least_squares_run(t, 0, 1000, A, b, X, P, work, alpha)
    xs = np.linalg.lstsq(host(A).reshape(n * m, d), host(b).reshape(n * m), rcond=None)[0]
    err_ed = np.abs(host(X) - xs).max()
    assert err_ed < 1e-2 * np.abs(xs).max()
    Xd = torch.zeros((n, d), device=DEV)
    bf.bf_dgd_least_squares_run(t, 0, 3000, A, b, Xd, work, alpha)
    assert bf.bf_dgd_status(t) == 0
    assert np.abs(host(Xd) - xs).max() > 20 * err_ed


# ------------------------------------------------------------------ long rows at four columns per lane
@pytest.mark.parametrize("what", ["mix", "awc", "pushsum_ratio"])
def test_long_row_form_of_the_wide_tile_kernels_matches_oracle(what):
    # 256-column tiles are only chosen for wide matrices; forcing them here runs the kernel form used
    # for rows of five entries or more (batched LDS reads, half-tile prefetch) on a small case with
    # several tiles per workgroup slot and a ragged last tile
    n, d = 64, 3 * 256 * 7 + 100
    t = bf.bf_topology_create(bf.BF_EXP_STATIC, n)
    W = lib_W(t)
    X = rows(n, d, 1234)
    try:
        bf.bf_set_tuning(0, 256)
        bf.bf_set_tuning(3, 3)                      # three workgroups: each walks several tiles
        if what == "mix":
            out = bf.bf_neighbor_allreduce(t, 0, X, empty_like_rows(X))
            assert_close(out, O.mix(host(X), W), TOL32, what)
        elif what == "awc":
            G = rows(n, d, 1235)
            out = bf.bf_atc_step(t, 0, X, empty_like_rows(X), G, None, alpha=0.05, mode=bf.BF_AWC)
            assert_close(out, O.awc_step(host(X), host(G), W, float(np.float32(0.05))), TOL32, what)
        else:
            w = torch.rand(n, device=DEV) + 0.5
            Y = empty_like_rows(X)
            Xo, wo, _ = bf.bf_pushsum_step(t, 0, X, empty_like_rows(X), w, torch.empty_like(w), Y)
            rx, rp, ry = O.pushsum_step(host(X), host(w[:, None])[:, 0], W)
            assert_close(Xo, rx, TOL32, "x"); assert_close(Y, ry, TOL32, "ratio")
    finally:
        bf.bf_set_tuning(0, 0)
        bf.bf_set_tuning(3, 0)
