"""Parity at the benchmark's full sizes, in the launch configuration bench.py times (library-chosen
leading dimension and tile shape).  The path is column separable, so the fp64 oracle run on a set
of sampled columns computes exactly what a full-width oracle would compute for those columns; the
sample covers the first tile, tile boundaries, random interior spans and the ragged tail.
Whole-matrix properties (mean preservation, consensus) are checked with the library's fp64
diagnostics kernel."""

import numpy as np
import pytest
import torch

import paper_2111_04287_amd as bf
import workloads
from oracle import iterations as O
from oracle import topology as OT

pytestmark = pytest.mark.gpu
DEV = torch.device("cuda:0")


def lib_W(t, r=0):
    rowptr, col, wgt, _ = bf.bf_topology_export_csr(t, r)
    return OT.from_csr(rowptr, col, wgt)


def sample_columns(d, seed):
    rng = np.random.default_rng(seed)
    cols = set(range(0, min(d, 300)))                       # first tile(s)
    cols |= set(range(max(0, d - 64), d))                   # ragged tail
    for c in (64, 128, 256, 512, 1024):                     # around tile boundaries of every width
        for k in rng.integers(1, max(2, d // c), size=6):
            cols |= set(range(max(0, k * c - 5), min(d, k * c + 5)))
    for s in rng.integers(0, max(1, d - 40), size=20):      # random interior spans
        cols |= set(range(int(s), int(s) + 33))
    return torch.tensor(sorted(c for c in cols if 0 <= c < d), device=DEV)


def take(X, cols):
    return X[:, cols].float().cpu().numpy().astype(np.float64)


def check(X, cols, ref, tol, what):
    got = take(X, cols)
    err = np.abs(got - ref).max()
    assert err <= tol * np.abs(ref).max(), "%s: %.3e vs %.1e * %.3e" % (what, err, tol, np.abs(ref).max())


def test_config2_full_size_50_rounds():
    n, d = 64, 1 << 20
    t = bf.bf_topology_create(bf.BF_EXP_STATIC, n)
    W = lib_W(t)
    ld = bf.bf_recommended_ld(d, bf.BF_F32)
    X = [workloads.config2_state(DEV, n=n, d=d, ld=ld), workloads.alloc_rows(n, d, torch.float32, DEV, ld=ld)]
    cols = sample_columns(d, 2)
    ref = take(X[0], cols)
    mean0 = torch.empty(d, device=DEV)
    s0 = bf.bf_consensus_stats(X[0], None, mean_out=mean0).clone()
    e0 = float(s0[0]) ** 0.5
    floor = 2e-7 * float(s0[2]) * np.sqrt(n * d)
    mean = torch.empty(d, device=DEV)
    for k in range(50):
        a, b = k & 1, 1 - (k & 1)
        bf.bf_neighbor_allreduce(t, k, X[a], X[b])
        ref = O.mix(ref, W)
        check(X[b], cols, ref, 1e-5, "round %d" % k)
        st = bf.bf_consensus_stats(X[b], None, mean_out=mean)
        bound = (2.0 / 3.0) ** (k + 1) * e0
        if bound > floor:
            assert float(st[0]) ** 0.5 <= bound * (1 + 1e-4), "contraction, round %d" % k
    assert float((mean - mean0).abs().max()) < 2e-6           # doubly stochastic W keeps the mean


def test_config3_full_size_8_rounds_reach_the_exact_mean():
    n, d = 256, 1 << 22
    t = bf.bf_topology_create(bf.BF_EXP2_ONE_PEER, n)
    ld = bf.bf_recommended_ld(d, bf.BF_F32)
    X = [workloads.config3_state(DEV, n=n, d=d, ld=ld), workloads.alloc_rows(n, d, torch.float32, DEV, ld=ld)]
    cols = sample_columns(d, 3)
    ref = take(X[0], cols)
    emu = X[0][:, cols].cpu().numpy()
    mean0 = torch.empty(d, device=DEV)
    s0 = bf.bf_consensus_stats(X[0], None, mean_out=mean0).clone()
    for r in range(8):
        a, b = r & 1, 1 - (r & 1)
        bf.bf_neighbor_allreduce(t, r, X[a], X[b])
        W = lib_W(t, r)
        ref = O.mix(ref, W)
        emu = O.mix_fp32_chain(emu, W)
        check(X[b], cols, ref, 1e-5, "round %d" % r)
        assert np.array_equal(X[b][:, cols].cpu().numpy().view(np.uint32), emu.view(np.uint32)), "bits, round %d" % r
    mean = torch.empty(d, device=DEV)
    st = bf.bf_consensus_stats(X[b], None, mean_out=mean)
    # every row equals the column mean up to fp32 rounding of eight halving additions
    assert float(st[1]) <= 8 * 6e-8 * float(s0[2])
    assert float((mean - mean0).abs().max()) <= 8 * 6e-8 * float(s0[2])
    assert np.abs(ref - ref.mean(0)).max() < 1e-14


def test_config4_full_size_pushsum_100_rounds():
    n, d = 128, 1 << 21
    t = bf.bf_topology_create(bf.BF_RANDOM_DIRECTED, n, out_degree=4, seed=workloads.CONFIG4_GRAPH_SEED)
    W = lib_W(t)
    ld = bf.bf_recommended_ld(d, bf.BF_F32)
    X = [workloads.config4_state(DEV, n=n, d=d, ld=ld), workloads.alloc_rows(n, d, torch.float32, DEV, ld=ld)]
    Y = workloads.alloc_rows(n, d, torch.float32, DEV, ld=ld)
    w = [torch.ones(n, device=DEV), torch.empty(n, device=DEV)]
    cols = sample_columns(d, 4)
    Xr, pr = take(X[0], cols), np.ones(n)
    mean0 = torch.empty(d, device=DEV)
    bf.bf_consensus_stats(X[0], None, mean_out=mean0)
    for k in range(100):
        a, b = k & 1, 1 - (k & 1)
        want_y = k % 10 == 9
        bf.bf_pushsum_step(t, k, X[a], X[b], w[a], w[b], Y if want_y else None)
        Xr, pr, Yr = O.pushsum_step(Xr, pr, W)
        check(X[b], cols, Xr, 1e-5, "X round %d" % k)
        assert np.abs(w[b].cpu().numpy() - pr).max() <= 1e-5 * pr.max()
        if want_y:
            check(Y, cols, Yr, 2e-5, "Y round %d" % k)
    mean = torch.empty(d, device=DEV)
    st = bf.bf_consensus_stats(X[b], w[b], mean_out=mean)      # ratios x_i / w_i against their mean
    assert float(st[1]) < 2e-5 * float(st[2])
    assert float((mean - mean0).abs().max()) < 2e-5 * float(st[2])   # and that mean is the initial average


def test_config5_full_size_momentum_20_steps():
    n, d = 32, workloads.RESNET50_PARAMS
    cfg = workloads.CONFIG5
    ld = bf.bf_recommended_ld(d, bf.BF_BF16)
    t = bf.bf_topology_create(bf.BF_EXP_STATIC, n)
    W = lib_W(t)
    Cc = workloads.config5_centres(DEV, n=n, d=d, ld=ld)
    X = [workloads.alloc_rows(n, d, torch.bfloat16, DEV, ld=ld, fill=0) for _ in range(2)]
    G = workloads.alloc_rows(n, d, torch.bfloat16, DEV, ld=ld)
    E = workloads.alloc_rows(n, d, torch.bfloat16, DEV, ld=ld)
    M = workloads.alloc_rows(n, d, torch.float32, DEV, ld=ld, fill=0)
    cols = sample_columns(d, 5)
    assert int(cols[-1]) == d - 1 and d % 1024 == 40                 # the 40-column ragged tail is sampled
    a64, b64, s64 = (float(np.float32(cfg[k])) for k in ("alpha", "beta", "sigma"))
    Xr, Mr = np.zeros((n, len(cols))), np.zeros((n, len(cols)))
    Ch = take(Cc, cols)
    for k in range(cfg["steps"]):
        a, b = k & 1, 1 - (k & 1)
        workloads.config5_noise(DEV, k, n=n, d=d, out=E)
        bf.bf_grad_quadratic(X[a], Cc, E, cfg["lam"], cfg["sigma"], G)
        bf.bf_atc_step(t, k, X[a], X[b], G, M, alpha=cfg["alpha"], beta=cfg["beta"], mode=bf.BF_ATC)
        Xr, Mr = O.dmsgd_atc_step(Xr, Mr, O.quadratic_noise_grad(Xr, Ch, take(E, cols), cfg["lam"], s64), W, a64, b64)
        check(X[b], cols, Xr, 2e-2, "step %d" % k)
        check(M, cols, Mr, 2e-2, "momentum, step %d" % k)


# ------------------------------------------------------------------ rows beyond the five configurations
def test_fused_eight_rounds_full_size_reach_the_exact_mean_in_one_pass():
    n, d = 256, 1 << 22
    t = bf.bf_topology_create(bf.BF_EXP2_ONE_PEER, n)
    ld = bf.bf_recommended_ld(d, bf.BF_F32)
    X = workloads.config3_state(DEV, n=n, d=d, ld=ld)
    cols = sample_columns(d, 13)
    ref = take(X, cols)
    emu = X[:, cols].cpu().numpy()
    mean0 = torch.empty(d, device=DEV)
    bf.bf_consensus_stats(X, None, mean_out=mean0)
    for r in range(8):
        W = lib_W(t, r)
        ref = O.mix(ref, W)
        emu = O.mix_fp32_chain(emu, W)
    bf.bf_neighbor_allreduce_multi(t, 0, 8, X, X)             # in place, as bench.py runs it
    check(X, cols, ref, 1e-5, "8 fused rounds")
    assert np.array_equal(X[:, cols].cpu().numpy().view(np.uint32), emu.view(np.uint32))
    st = bf.bf_consensus_stats(X, None)
    assert float(st[1]) <= 8 * 6e-8 * float(st[2]) + 1e-30, "every row is the column mean"
    assert float((X[0] - mean0).abs().max()) <= 2e-6


def test_hierarchical_full_size():
    M, L, d = 8, 8, 1 << 22
    t = bf.bf_topology_create(bf.BF_EXP_STATIC, M)
    ld = bf.bf_recommended_ld(d, bf.BF_F32)
    X = workloads.normal_rows(M * L, d, 601, DEV, ld=ld)
    cols = sample_columns(d, 14)
    ref = O.hierarchical_neighbor_allreduce(take(X, cols), lib_W(t), L)
    out = bf.bf_hierarchical_neighbor_allreduce(t, 0, L, X, workloads.alloc_rows(M * L, d, torch.float32, DEV, ld=ld))
    check(out, cols, ref, 1e-5, "hierarchical")
    bf.bf_hierarchical_neighbor_allreduce(t, 0, L, X, X)
    assert torch.equal(X[:, cols], out[:, cols])
    o3 = out[:, cols].reshape(M, L, -1)
    assert torch.equal(o3, o3[:, :1].expand_as(o3))


def test_window_pushsum_round_full_size():
    n, d = 128, 1 << 21
    t = bf.bf_topology_create(bf.BF_RANDOM_DIRECTED, n, out_degree=4, seed=workloads.CONFIG4_GRAPH_SEED)
    W = lib_W(t)
    E = bf.bf_topology_window_slots(t, 0)
    ld = bf.bf_recommended_ld(d, bf.BF_F32)
    X = workloads.config4_state(DEV, n=n, d=d, ld=ld)
    Win = workloads.alloc_rows(E, d, torch.float32, DEV, ld=ld, fill=0)
    p, win_p = torch.ones(n, device=DEV), torch.zeros(E, device=DEV)
    cols = sample_columns(d, 15)
    rx, rp, rw, rwp = take(X, cols), np.ones(n), np.zeros((E, len(cols))), np.zeros(E)
    rng = np.random.default_rng(15)
    for k in range(6):
        ma = (rng.random(n) < 0.7).astype(np.int32)
        mc = (rng.random(n) < 0.7).astype(np.int32)
        bf.bf_win_accumulate(t, 0, X, p, Win, win_p, active=torch.from_numpy(ma).to(DEV))
        rx, rp, rw, rwp = O.win_accumulate(rx, rp, rw, rwp, W, ma)
        check(X, cols, rx, 1e-5, "accumulate %d X" % k)
        check(Win, cols, rw, 1e-5, "accumulate %d Win" % k)
        bf.bf_win_update_then_collect(t, 0, X, p, Win, win_p, active=torch.from_numpy(mc).to(DEV))
        rx, rp, rw, rwp = O.win_update_then_collect(rx, rp, rw, rwp, W, mc)
        check(X, cols, rx, 1e-5, "collect %d X" % k)
        got_w = take(Win, cols)
        assert np.abs(got_w - rw).max() <= 1e-5 * max(np.abs(rw).max(), np.abs(rx).max())
        np.testing.assert_allclose(p.cpu().numpy(), rp, rtol=1e-5)
    assert abs(float(p.double().sum() + win_p.double().sum()) - n) < 1e-4


def test_more_than_two_to_the_31_columns():
    """Column indices beyond 32 bits: two agents on a ring (weights 1/2, 1/2), d = 2^31 + 1000, fp32,
    on agent-major rows and in column blocks; constant rows with three marked columns."""
    n, d = 2, (1 << 31) + 1000
    t = bf.bf_topology_create(bf.BF_RING, n)
    ld = bf.bf_recommended_ld(d, bf.BF_F32)
    X = torch.empty((n, ld), device=DEV)[:, :d]
    X[0].fill_(1.0)
    X[1].fill_(3.0)
    marks = {d - 1: (5.0, 9.0), (1 << 31) + 7: (-1.0, 3.0), 1 << 31: (1.0, 3.0), 0: (1.0, 3.0), 12345678: (1.0, 3.0)}
    for c, (a, b) in marks.items():
        X[0, c] = a
        X[1, c] = b
    out = torch.empty((n, ld), device=DEV)[:, :d]
    bf.bf_neighbor_allreduce(t, 0, X, out)
    for c, (a, b) in marks.items():
        assert float(out[0, c]) == (a + b) / 2 and float(out[1, c]) == (a + b) / 2, c
    B = 16384
    Xb = bf.Blocked(torch.empty(((d + B - 1) // B, n, B), device=DEV), d)
    bf.bf_blocked_pack(X, Xb)
    bf.bf_neighbor_allreduce(t, 0, Xb, Xb)
    out.fill_(0.0)
    bf.bf_blocked_unpack(Xb, out)
    for c, (a, b) in marks.items():
        assert float(out[0, c]) == (a + b) / 2 and float(out[1, c]) == (a + b) / 2, c
    st = bf.bf_consensus_stats(out)
    assert float(st[0]) == 0.0 and float(st[2]) == 7.0           # both rows equal everywhere; the largest value is (5 + 9) / 2
