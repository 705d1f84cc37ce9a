"""GPU parity of the column-block layout: the conversion kernels against the layout's definition
written out in numpy, every call that accepts the layout against the same call on agent-major
matrices (bit for bit: same kernels' arithmetic, other addresses) and against the fp64 oracle, and
the momentum step at the benchmark's full size in the launch configuration bench.py times."""

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


def lib_W(t, r=0):
    rowptr, col, wgt, _ = bf.bf_topology_export_csr(t, r)
    return OT.from_csr(rowptr, col, wgt)


def host(x):
    return x.detach().float().cpu().numpy().astype(np.float64)


def rows(n, d, seed, dtype=torch.float32):
    ld = workloads.padded_ld(d, 2 if dtype == torch.bfloat16 else 4)
    return workloads.normal_rows(n, d, seed, DEV, ld=ld, dtype=dtype)


def empty_blocked(n, d, B, dtype, fill=float("nan")):
    data = torch.full(((d + B - 1) // B, n, B), fill, dtype=dtype, device=DEV)
    return bf.Blocked(data, d)


def to_blocked(X, B):
    n, d = X.shape
    return bf.bf_blocked_pack(X, empty_blocked(n, d, B, X.dtype))


def from_blocked(Xb, like):
    out = torch.full((like.shape[0], like.stride(0)), 7.0, dtype=like.dtype, device=DEV)[:, :like.shape[1]]
    return bf.bf_blocked_unpack(Xb, out)


def blocked_by_definition(X, B):
    """Column c of agent i is element (c // B, i, c % B); the columns past d of the last block are zero."""
    n, d = X.shape
    nb = (d + B - 1) // B
    full = torch.zeros((n, nb * B), dtype=X.dtype, device=X.device)
    full[:, :d] = X
    return full.reshape(n, nb, B).permute(1, 0, 2).contiguous()


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("n,d,B", [(1, 64, 64), (3, 5, 64), (7, 1000, 128), (32, 3 * 512 + 37, 512), (5, 4096 * 2 + 1, 4096),
                                   (64, 256 * 9, 256), (130, 77, 1024)])
def test_pack_and_unpack_follow_the_layout_definition(dtype, n, d, B):
    X = rows(n, d, 10 + n, dtype=dtype)
    Xb = to_blocked(X, B)
    assert Xb.data.numel() == bf.bf_blocked_elems(n, d, B)
    assert torch.equal(Xb.data.view(torch.int16 if dtype == torch.bfloat16 else torch.int32),
                       blocked_by_definition(X, B).view(torch.int16 if dtype == torch.bfloat16 else torch.int32))
    back = torch.full((n, X.stride(0)), 7.0, dtype=dtype, device=DEV)
    bf.bf_blocked_unpack(Xb, back[:, :d])
    assert torch.equal(back[:, :d], X)
    assert bool((back[:, d:] == 7.0).all()), "columns past d of the agent-major rows are not written"


CASES = [(1, 100, 64), (3, 20, 64), (5, 300, 64), (32, 3 * 512 + 37, 512), (64, 2 * 256 + 100, 256), (128, 1000, 1024), (32, 9000, 8192),
         (16, 70000, 1 << 16), (300, 200, 64), (700, 150, 64)]


def _knobs(setting):
    for k, v in setting:
        bf.bf_set_tuning(k, v)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("n,d,B", CASES)
@pytest.mark.parametrize("setting", [(), ((12, 1),), ((12, 2),)], ids=["auto", "pipelined", "one-tile"])
def test_every_accepting_call_gives_the_agent_major_bits(dtype, n, d, B, setting):
    t = bf.bf_topology_create(bf.BF_RANDOM_DIRECTED, n, out_degree=min(10, n - 1), seed=77) if n > 1 \
        else bf.bf_topology_create(bf.BF_RING, 1)
    W = lib_W(t)
    tol = TOL32 if dtype == torch.float32 else 2.0 ** -8
    X, G, G2 = (rows(n, d, 40 + k, dtype=dtype) for k in range(3))
    M0 = workloads.normal_rows(n, d, 49, DEV, ld=X.stride(0))
    w0 = torch.rand(n, device=DEV) + 0.5
    alpha, beta = 0.05, 0.9
    a64, b64 = float(np.float32(alpha)), float(np.float32(beta))
    Xb, Gb, G2b = (to_blocked(A, B) for A in (X, G, G2))

    def fresh(A):
        return torch.empty((n, A.stride(0)), dtype=A.dtype, device=DEV)[:, :d].copy_(A)

    def both(call, in_place, state=None, ratio=False):
        """Runs call(x_in, x_out, state, y) in both layouts; returns the agent-major results after
        checking that the column-block ones hold the same bits and that block padding is untouched."""
        xi = fresh(X)
        xo = xi if in_place else torch.empty((n, X.stride(0)), dtype=dtype, device=DEV)[:, :d]
        st = None if state is None else fresh(state)
        y = torch.empty((n, X.stride(0)), dtype=dtype, device=DEV)[:, :d] if ratio else None
        bxi = to_blocked(X, B)
        bxo = bxi if in_place else empty_blocked(n, d, B, dtype, fill=3.0)
        bst = None if state is None else to_blocked(state, B)
        by = empty_blocked(n, d, B, dtype, fill=3.0) if ratio else None
        try:
            _knobs(setting)
            call(xi, xo, st, y)
            call(bxi, bxo, bst, by)
        finally:
            _knobs(tuple((k, 0) for k, _ in setting))
        assert torch.equal(from_blocked(bxo, X), xo)
        if st is not None:
            assert torch.equal(from_blocked(bst, st), st)
        if ratio:
            assert torch.equal(from_blocked(by, X), y)
        pad = bxo.data[-1, :, d - (bxo.data.shape[0] - 1) * B:]
        if not in_place and pad.numel():
            assert bool((pad == 3.0).all()), "the padding columns of the last block are never written"
        return xo, st, y

    for in_place in (False, True):
        out, _, _ = both(lambda a, b, s, y: bf.bf_neighbor_allreduce(t, 1, a, b), in_place)
        ref = O.mix(host(X), W)
        assert np.abs(host(out) - ref).max() <= tol * np.abs(ref).max()
        for mode, fn in ((bf.BF_ATC, O.atc_step), (bf.BF_AWC, O.awc_step)):
            out, _, _ = both(lambda a, b, s, y: bf.bf_atc_step(t, 0, a, b, (Gb if isinstance(a, bf.Blocked) else G), None,
                                                               alpha=alpha, mode=mode), in_place)
            ref = fn(host(X), host(G), W, a64)
            assert np.abs(host(out) - ref).max() <= tol * np.abs(ref).max()
            out, Mn, _ = both(lambda a, b, s, y: bf.bf_atc_step(t, 0, a, b, (Gb if isinstance(a, bf.Blocked) else G), s,
                                                                alpha=alpha, beta=beta, mode=mode), in_place, state=M0)
            Mref = b64 * host(M0) + host(G)
            ref = O.dmsgd_atc_step(host(X), host(M0), host(G), W, a64, b64)[0] if mode == bf.BF_ATC \
                else O.mix(host(X), W) - a64 * Mref
            assert np.abs(host(Mn) - Mref).max() <= 1e-6 * np.abs(Mref).max()
            assert np.abs(host(out) - ref).max() <= tol * np.abs(ref).max()
        # Exact-Diffusion (state: psi of the step before), tracking, push-sum with the ratio
        out, Pn, _ = both(lambda a, b, s, y: bf.bf_exact_diffusion_step(t, 0, a, b, (Gb if isinstance(a, bf.Blocked) else G), s,
                                                                        alpha), in_place, state=M0)
        ref, Pref = O.exact_diffusion_step(host(X), host(M0), host(G), W, a64)
        assert np.abs(host(out) - ref).max() <= tol * np.abs(ref).max()
        assert np.abs(host(Pn) - Pref).max() <= 1e-6 * np.abs(Pref).max()
        out, _, _ = both(lambda a, b, s, y: bf.bf_tracking_step(t, 0, a, b, *((Gb, G2b) if isinstance(a, bf.Blocked) else (G, G2))),
                         in_place)
        ref = O.mix(host(X) + host(G) - host(G2), W)
        assert np.abs(host(out) - ref).max() <= tol * max(np.abs(ref).max(), 1.0)
        for with_g in (False, True):
            w1 = torch.empty_like(w0)

            def ps(a, b, s, y):
                if with_g:
                    bf.bf_pushsum_atc_step(t, 0, a, b, (Gb if isinstance(a, bf.Blocked) else G), alpha, w0, w1, y)
                else:
                    bf.bf_pushsum_step(t, 0, a, b, w0, w1, y)
            out, _, y = both(ps, in_place, ratio=True)
            xin = host(X) - a64 * host(G) if with_g else host(X)
            ref = O.mix(xin, W)
            wref = O.mix(host(w0)[:, None], W)[:, 0]
            assert np.abs(host(out) - ref).max() <= tol * np.abs(ref).max()
            assert np.abs(host(w1) - wref).max() <= TOL32 * np.abs(wref).max()
            yref = ref / wref[:, None]
            assert np.abs(host(y) - yref).max() <= 2 * tol * np.abs(yref).max()


def test_layout_mismatch_and_agent_major_only_calls_are_refused():
    n, d, B = 8, 300, 64
    t = bf.bf_topology_create(bf.BF_RING, n)
    X = rows(n, d, 1)
    Xb = to_blocked(X, B)
    with pytest.raises(ValueError):
        bf.bf_neighbor_allreduce(t, 0, Xb, X)                      # mixed layouts
    with pytest.raises(ValueError):
        bf.bf_neighbor_allreduce(t, 0, Xb, to_blocked(X, 128))     # two block widths
    A = torch.zeros((n, 4, d - d % 4), device=DEV)
    with pytest.raises((bf.BfError, ValueError, AttributeError)):
        bf.bf_grad_least_squares(A, torch.zeros((n, 4), device=DEV), Xb, Xb)   # whole-row access: agent-major only


def sample_columns(d, seed):
    rng = np.random.default_rng(seed)
    cols = set(range(0, 300)) | set(range(d - 64, d))
    for c in (256, 512, 1024):
        for k in rng.integers(1, d // c, size=6):
            cols |= set(range(k * c - 5, k * c + 5))
    for s in rng.integers(0, d - 40, size=20):
        cols |= set(range(int(s), int(s) + 33))
    return torch.tensor(sorted(c for c in cols if 0 <= c < d), device=DEV)


def test_config5_full_size_momentum_steps_in_column_blocks():
    """The headline workload as bench.py times it: n = 32, d = 25,557,032, bf16 X and G, fp32 momentum,
    in place, blocks of bf_recommended_block columns.  Oracle on sampled columns (the path is column
    separable), which include the ragged tail inside the last block."""
    n, d = 32, workloads.RESNET50_PARAMS
    cfg = workloads.CONFIG5
    t = bf.bf_topology_create(bf.BF_EXP_STATIC, n)
    B = bf.bf_recommended_block(t, d, bf.BF_BF16)
    ld = bf.bf_recommended_ld(d, bf.BF_BF16)
    W = lib_W(t)
    cols = sample_columns(d, 5)
    assert int(cols[-1]) == d - 1 and d % B == 6184     # the last block is ragged
    scratch = workloads.alloc_rows(n, d, torch.bfloat16, DEV, ld=ld)          # agent-major staging for the recipe
    scratch32 = workloads.alloc_rows(n, d, torch.float32, DEV, ld=ld)
    Cc = workloads.config5_centres(DEV, n=n, d=d, ld=ld)
    Ch = Cc[:, cols].float().cpu().numpy().astype(np.float64)
    Cb = to_blocked(Cc, B)
    del Cc
    Xb = empty_blocked(n, d, B, torch.bfloat16, fill=0.0)
    Gb = empty_blocked(n, d, B, torch.bfloat16, fill=0.0)
    Eb = empty_blocked(n, d, B, torch.bfloat16, fill=0.0)
    Mb = empty_blocked(n, d, B, torch.float32, fill=0.0)
    a64, b64, s64 = (float(np.float32(cfg[k])) for k in ("alpha", "beta", "sigma"))
    Xr, Mr = np.zeros((n, len(cols))), np.zeros((n, len(cols)))
    for k in range(6):
        workloads.config5_noise(DEV, k, n=n, d=d, out=scratch)
        Eh = scratch[:, cols].float().cpu().numpy().astype(np.float64)
        bf.bf_blocked_pack(scratch, Eb)
        bf.bf_grad_quadratic(Xb, Cb, Eb, cfg["lam"], cfg["sigma"], Gb)
        bf.bf_atc_step(t, k, Xb, Xb, Gb, Mb, alpha=cfg["alpha"], beta=cfg["beta"], mode=bf.BF_ATC)
        Xr, Mr = O.dmsgd_atc_step(Xr, Mr, O.quadratic_noise_grad(Xr, Ch, Eh, cfg["lam"], s64), W, a64, b64)
        bf.bf_blocked_unpack(Xb, scratch)
        got = scratch[:, cols].float().cpu().numpy().astype(np.float64)
        assert np.abs(got - Xr).max() <= 2e-2 * np.abs(Xr).max(), "step %d" % k
        bf.bf_blocked_unpack(Mb, scratch32)
        gotm = scratch32[:, cols].cpu().numpy().astype(np.float64)
        assert np.abs(gotm - Mr).max() <= 2e-2 * np.abs(Mr).max(), "momentum, step %d" % k
    pad = Xb.data[-1, :, d - (Xb.data.shape[0] - 1) * B:]
    assert bool((pad == 0).all()) and bool((Mb.data[-1, :, d - (Mb.data.shape[0] - 1) * B:] == 0).all())


@pytest.mark.parametrize("dtype,n,d", [(torch.bfloat16, 32, workloads.RESNET50_PARAMS), (torch.float32, 128, 1 << 22)])
def test_steps_without_a_state_matrix_full_size_in_column_blocks(dtype, n, d):
    """The plain mix and the ATC and AWC steps on the static exponential graph, out of place, at the
    sizes and block width bench.py times them at beside the five configurations (bf16 with 32 agents
    and ResNet-50's parameter count -- where AWC takes its gradients from the LDS tile --, fp32 with
    128 agents and fourteen entries per row).  Oracle on sampled columns, ragged tail included."""
    t = bf.bf_topology_create(bf.BF_EXP_STATIC, n)
    code = bf.BF_BF16 if dtype == torch.bfloat16 else bf.BF_F32
    B = bf.bf_recommended_block(t, d, code)
    ld = bf.bf_recommended_ld(d, code)
    W = lib_W(t)
    tol = 2.0 ** -8 if dtype == torch.bfloat16 else TOL32
    cols = sample_columns(d, 11)
    assert int(cols[-1]) == d - 1
    X = workloads.normal_rows(n, d, 160, DEV, ld=ld, dtype=dtype)
    G = workloads.normal_rows(n, d, 161, DEV, ld=ld, dtype=dtype)
    Xh, Gh = host(X[:, cols]), host(G[:, cols])
    Xb, Gb = to_blocked(X, B), to_blocked(G, B)
    Yb = empty_blocked(n, d, B, dtype)
    alpha = 0.05
    a64 = float(np.float32(alpha))
    for what, run, ref in (
            ("mix", lambda: bf.bf_neighbor_allreduce(t, 0, Xb, Yb), lambda: O.mix(Xh, W)),
            ("ATC", lambda: bf.bf_atc_step(t, 0, Xb, Yb, Gb, None, alpha=alpha, mode=bf.BF_ATC), lambda: O.atc_step(Xh, Gh, W, a64)),
            ("AWC", lambda: bf.bf_atc_step(t, 0, Xb, Yb, Gb, None, alpha=alpha, mode=bf.BF_AWC), lambda: O.awc_step(Xh, Gh, W, a64))):
        Yb.data.fill_(float("nan"))
        run()
        bf.bf_blocked_unpack(Yb, X)                      # X is free by now: Xb holds the input
        got, want = host(X[:, cols]), ref()
        assert np.abs(got - want).max() <= tol * np.abs(want).max(), what
        assert bool((Yb.data[-1, :, d - (Yb.data.shape[0] - 1) * B:] != Yb.data[-1, :, d - (Yb.data.shape[0] - 1) * B:]).all()), \
            what + ": the padding of the last block was written"


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("cw", [1, 2, 4])
@pytest.mark.parametrize("kind,n", [(bf.BF_RING, 16), (bf.BF_EXP2_ONE_PEER, 100), (bf.BF_EXP2_ONE_PEER, 256)])
@pytest.mark.parametrize("d,B", [(3 * 1024 + 77, 1024), (2 * 8192 + 4100, 8192), (5000, 2048)])
def test_row_streaming_kernel_on_column_blocks(dtype, cw, kind, n, d, B):
    """Rounds whose graph is a union of paths and cycles: the chain kernel's sweeps stay inside a
    block (blocks narrower than a sweep go to the tile kernels); same bits as agent-major rows."""
    t = bf.bf_topology_create(kind, n)
    X, G, G2 = (rows(n, d, 70 + k, dtype=dtype) for k in range(3))
    S = workloads.normal_rows(n, d, 79, DEV, ld=X.stride(0))
    w0 = torch.rand(n, device=DEV) + 0.5
    Xb, Gb, G2b = (to_blocked(A, B) for A in (X, G, G2))

    def fresh(A):
        return torch.empty((n, A.stride(0)), dtype=A.dtype, device=DEV)[:, :d].copy_(A)

    bf.bf_set_tuning(6, cw)
    try:
        for rnd in (0, 3):
            for in_place in (False, True):
                # plain mix
                xi = fresh(X); xo = xi if in_place else fresh(X)
                bi = to_blocked(X, B); bo = bi if in_place else empty_blocked(n, d, B, dtype)
                bf.bf_neighbor_allreduce(t, rnd, xi, xo)
                bf.bf_neighbor_allreduce(t, rnd, bi, bo)
                assert torch.equal(from_blocked(bo, X), xo)
                ref = O.mix(host(X), lib_W(t, rnd))
                assert np.abs(host(xo) - ref).max() <= (TOL32 if dtype == torch.float32 else 2.0 ** -8) * np.abs(ref).max()
                # momentum ATC and AWC, Exact-Diffusion (fp32 state updated in place)
                for call in (lambda a, b, g, s: bf.bf_atc_step(t, rnd, a, b, g, s, alpha=0.05, beta=0.9, mode=bf.BF_ATC),
                             lambda a, b, g, s: bf.bf_atc_step(t, rnd, a, b, g, s, alpha=0.05, beta=0.9, mode=bf.BF_AWC),
                             lambda a, b, g, s: bf.bf_exact_diffusion_step(t, rnd, a, b, g, s, 0.05)):
                    xi = fresh(X); xo = xi if in_place else fresh(X); st = fresh(S)
                    bi = to_blocked(X, B); bo = bi if in_place else empty_blocked(n, d, B, dtype); bs = to_blocked(S, B)
                    call(xi, xo, G, st)
                    call(bi, bo, Gb, bs)
                    assert torch.equal(from_blocked(bo, X), xo) and torch.equal(from_blocked(bs, S), st)
                # tracking, push-sum with the ratio
                xi = fresh(X); xo = xi if in_place else fresh(X)
                bi = to_blocked(X, B); bo = bi if in_place else empty_blocked(n, d, B, dtype)
                bf.bf_tracking_step(t, rnd, xi, xo, G, G2)
                bf.bf_tracking_step(t, rnd, bi, bo, Gb, G2b)
                assert torch.equal(from_blocked(bo, X), xo)
                xi = fresh(X); xo = xi if in_place else fresh(X); y = fresh(X)
                bi = to_blocked(X, B); bo = bi if in_place else empty_blocked(n, d, B, dtype); by = empty_blocked(n, d, B, dtype)
                w1, w2 = torch.empty_like(w0), torch.empty_like(w0)
                bf.bf_pushsum_step(t, rnd, xi, xo, w0, w1, y)
                bf.bf_pushsum_step(t, rnd, bi, bo, w0, w2, by)
                assert torch.equal(from_blocked(bo, X), xo) and torch.equal(from_blocked(by, X), y) and torch.equal(w1, w2)
    finally:
        bf.bf_set_tuning(6, 0)


def _shift_topology(n, shifts, weights):
    rp, cols, wg = [], [], []
    for s, (ws, wp) in zip(shifts, weights):
        base = len(cols)
        for i in range(n):
            rp.append(len(cols))
            for j, w in sorted(((i, ws), ((i + s) % n, wp))):
                cols.append(j); wg.append(w)
        rp.append(len(cols))
    return bf.bf_topology_create(bf.BF_CSR_USER, n, rounds=len(shifts), rowptr=rp, col=cols, wgt=wg)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("case", ["onepeer64", "onepeer256", "shift128", "exp100", "push300", "ring700"])
@pytest.mark.parametrize("B", [64, 256, 8192])
def test_fused_rounds_on_column_blocks(dtype, case, B):
    """Several rounds per pass: in registers (uniform shift rounds), LDS tile to LDS tile, and as
    separate passes when two tiles do not fit; each gives the agent-major bits."""
    if case == "onepeer64":
        t, n = bf.bf_topology_create(bf.BF_EXP2_ONE_PEER, 64), 64
    elif case == "onepeer256":
        t, n = bf.bf_topology_create(bf.BF_EXP2_ONE_PEER, 256), 256
    elif case == "shift128":
        t, n = _shift_topology(128, [3, 64, 100 - 36, 127 - 64 - 1], [(0.5, 0.5), (0.25, 0.75), (0.7, 0.3), (0.5, 0.5)]), 128
    elif case == "exp100":
        t, n = bf.bf_topology_create(bf.BF_EXP_STATIC, 100), 100
    elif case == "push300":
        t, n = bf.bf_topology_create(bf.BF_RANDOM_DIRECTED, 300, out_degree=5, seed=3), 300
    else:
        t, n = bf.bf_topology_create(bf.BF_RING, 700), 700
    d = 2 * B + 100 if B <= 256 else B + 1000
    X = rows(n, d, 90, dtype=dtype)
    for round0, count in ((0, 2), (1, 5), (3, 8)):
        for in_place in (False, True):
            xi = torch.empty((n, X.stride(0)), dtype=dtype, device=DEV)[:, :d].copy_(X)
            xo = xi if in_place else torch.empty((n, X.stride(0)), dtype=dtype, device=DEV)[:, :d]
            bi = to_blocked(X, B)
            bo = bi if in_place else empty_blocked(n, d, B, dtype)
            bf.bf_neighbor_allreduce_multi(t, round0, count, xi, xo)
            bf.bf_neighbor_allreduce_multi(t, round0, count, bi, bo)
            assert torch.equal(from_blocked(bo, X), xo), (case, B, round0, count, in_place)
    ref = host(X)
    for r in range(3, 11):
        ref = O.mix(ref, lib_W(t, r))
    tol = TOL32 if dtype == torch.float32 else 8 * 2.0 ** -8
    assert np.abs(host(xo) - ref).max() <= tol * np.abs(ref).max()


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("M,L,d,B", [(4, 4, 1000, 256), (8, 8, 8192 + 136, 8192), (5, 3, 130, 64), (40, 20, 300, 128)])
def test_hierarchical_averaging_on_column_blocks(dtype, M, L, d, B):
    t = bf.bf_topology_create(bf.BF_EXP_STATIC, M)
    n = M * L
    X = rows(n, d, 95, dtype=dtype)
    xo = torch.empty((n, X.stride(0)), dtype=dtype, device=DEV)[:, :d]
    bo = empty_blocked(n, d, B, dtype)
    bf.bf_hierarchical_neighbor_allreduce(t, 1, L, X, xo)
    bf.bf_hierarchical_neighbor_allreduce(t, 1, L, to_blocked(X, B), bo)
    assert torch.equal(from_blocked(bo, X), xo)
    ref = O.hierarchical_neighbor_allreduce(host(X), lib_W(t, 1), L)
    assert np.abs(host(xo) - ref).max() <= (TOL32 if dtype == torch.float32 else 2.0 ** -7) * np.abs(ref).max()
    bi = to_blocked(X, B)
    bf.bf_hierarchical_neighbor_allreduce(t, 1, L, bi, bi)
    assert torch.equal(from_blocked(bi, X), xo)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("n,d,B", [(12, 4096 + 136, 1024), (33, 130 + 3, 64), (16, 2 * 8192 + 5000, 8192)])
def test_window_calls_on_column_blocks(dtype, n, d, B):
    """One asynchronous push-sum round (accumulate, update_then_collect), put / get / update and a
    weighted call: X and the window in column blocks give the agent-major bits."""
    t = bf.bf_topology_create(bf.BF_RANDOM_DIRECTED, n, out_degree=3, seed=5)
    E = bf.bf_topology_window_slots(t, 0)
    X = rows(n, d, 110, dtype=dtype)
    W0 = workloads.normal_rows(E, d, 111, DEV, ld=X.stride(0))
    active = torch.tensor([1 if (i * 7) % 5 else 0 for i in range(n)], dtype=torch.int32, device=DEV)
    self_w = torch.rand(n, device=DEV)
    edge_w = torch.rand(E, device=DEV)

    def run(call):
        x = torch.empty((n, X.stride(0)), dtype=dtype, device=DEV)[:, :d].copy_(X)
        w = torch.empty((E, X.stride(0)), device=DEV)[:, :d].copy_(W0)
        p, wp = torch.ones(n, device=DEV), torch.full((E,), 0.25, device=DEV)
        xb, wb = to_blocked(X, B), to_blocked(W0, B)
        pb, wpb = torch.ones(n, device=DEV), torch.full((E,), 0.25, device=DEV)
        call(x, w, p, wp)
        call(xb, wb, pb, wpb)
        assert torch.equal(from_blocked(xb, X), x) and torch.equal(from_blocked(wb, W0), w)
        assert torch.equal(p, pb) and torch.equal(wp, wpb)

    for act in (None, active):
        run(lambda x, w, p, wp: bf.bf_win_put(t, 0, x, w, active=act))
        run(lambda x, w, p, wp: bf.bf_win_get(t, 0, x, w, active=act))
        run(lambda x, w, p, wp: bf.bf_win_update(t, 0, x, w, active=act))
        run(lambda x, w, p, wp: (bf.bf_win_accumulate(t, 0, x, p, w, wp, active=act),
                                 bf.bf_win_update_then_collect(t, 0, x, p, w, wp, active=act)))
        run(lambda x, w, p, wp: bf.bf_win_accumulate_weighted(t, 0, x, p, w, wp, self_weight=self_w, dst_weight=edge_w, active=act))
        run(lambda x, w, p, wp: bf.bf_win_update_weighted(t, 0, x, w, self_weight=self_w, src_weight=edge_w, active=act))


@pytest.mark.parametrize("n,d,B", [(5, 300, 64), (64, 3 * 256 + 10, 256), (100, 1000, 128), (256, 2 * 1024 + 72, 1024), (200, 500, 64)])
def test_dense_mix_on_column_blocks(n, d, B):
    """Dense W on the matrix cores with the matrices in column blocks (blocks narrower than the
    kernel's tile go to the list kernels): the agent-major bits or, from the list kernels, the
    oracle's values."""
    rng = np.random.default_rng(n)
    D = rng.random((n, n)).astype(np.float32)
    D /= D.sum(axis=1, keepdims=True)
    t = bf.bf_topology_create(bf.BF_DENSE_USER, n, dense_w=D)
    X = rows(n, d, 120)
    out = torch.empty((n, X.stride(0)), device=DEV)[:, :d]
    bf.bf_dense_mix(t, 0, X, out)
    ob = empty_blocked(n, d, B, torch.float32)
    bf.bf_dense_mix(t, 0, to_blocked(X, B), ob)
    ref = O.mix(host(X), lib_W(t))
    got = from_blocked(ob, X)
    assert np.abs(host(got) - ref).max() <= TOL32 * np.abs(ref).max()
    assert np.abs(host(out) - ref).max() <= TOL32 * np.abs(ref).max()
    xb = to_blocked(X, B)
    bf.bf_dense_mix(t, 0, xb, xb)                                  # in place
    assert torch.equal(from_blocked(xb, X), got)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("n,d,B", [(5, 300, 64), (32, 3 * 512 + 37, 512), (16, 9000, 8192)])
def test_gradient_generator_and_diagnostics_on_column_blocks(dtype, n, d, B):
    X, Cc, E = (rows(n, d, 130 + k, dtype=dtype) for k in range(3))
    G = torch.empty((n, X.stride(0)), dtype=dtype, device=DEV)[:, :d]
    bf.bf_grad_quadratic(X, Cc, E, 0.7, 0.3, G)
    Gb = empty_blocked(n, d, B, dtype, fill=3.0)
    bf.bf_grad_quadratic(to_blocked(X, B), to_blocked(Cc, B), to_blocked(E, B), 0.7, 0.3, Gb)
    assert torch.equal(from_blocked(Gb, X), G)
    pad = Gb.data[-1, :, d - (Gb.data.shape[0] - 1) * B:]
    assert bool((pad == 3.0).all()), "the padding columns of the last block are never written"
    p = torch.rand(n, device=DEV) + 0.5
    for pv in (None, p):
        m1, m2 = torch.empty(d, device=DEV), torch.empty(d, device=DEV)
        s1 = bf.bf_consensus_stats(X, pv, mean_out=m1).clone()
        s2 = bf.bf_consensus_stats(to_blocked(X, B), pv, mean_out=m2).clone()
        assert torch.equal(m1, m2)
        assert torch.equal(s1[1:], s2[1:]) and abs(float(s1[0]) - float(s2[0])) <= 1e-12 * float(s1[0])   # sums: atomics, any order


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("n,d,B", [(5, 300, 64), (32, 3 * 512 + 37, 512), (64, 9000, 8192), (300, 200, 64), (700, 150, 64)])
@pytest.mark.parametrize("kind", [bf.BF_EXP_STATIC, bf.BF_RING])
def test_a_layout_per_matrix(dtype, n, d, B, kind):
    """Every mix of agent-major rows and column blocks for (X, G, M): the bits of the all-agent-major
    call, for ATC, AWC and both momentum forms, in place and not."""
    t = bf.bf_topology_create(kind, n)
    X, G = rows(n, d, 140, dtype=dtype), rows(n, d, 141, dtype=dtype)
    M0 = workloads.normal_rows(n, d, 142, DEV, ld=X.stride(0))
    Gb = to_blocked(G, B)

    def fresh(A):
        return torch.empty((n, A.stride(0)), dtype=A.dtype, device=DEV)[:, :d].copy_(A)

    for cw in (0, 2):                                            # 2: the row-streaming kernel where the round allows it
        bf.bf_set_tuning(6, cw)
        try:
            for mode in (bf.BF_ATC, bf.BF_AWC):
                for with_m in (False, True):
                    for in_place in (False, True):
                        xi = fresh(X); xo = xi if in_place else fresh(X); m = fresh(M0) if with_m else None
                        bf.bf_atc_step(t, 1, xi, xo, G, m, alpha=0.05, beta=0.9, mode=mode)
                        for xb, gb, mb in ((1, 0, 1), (0, 1, 0), (0, 0, 1), (1, 1, 0), (1, 0, 0), (0, 1, 1)):
                            if not with_m and (xb, gb, mb) in ((0, 0, 1), (1, 1, 0), (0, 1, 1)):
                                continue                          # the same call as another one without M
                            yi = to_blocked(X, B) if xb else fresh(X)
                            yo = yi if in_place else (empty_blocked(n, d, B, dtype) if xb else fresh(X))
                            ym = None if not with_m else (to_blocked(M0, B) if mb else fresh(M0))
                            bf.bf_atc_step_layouts(t, 1, yi, yo, Gb if gb else G, ym, alpha=0.05, beta=0.9, mode=mode)
                            assert torch.equal(from_blocked(yo, X) if xb else yo, xo), (xb, gb, mb, mode, with_m, in_place)
                            if with_m:
                                assert torch.equal(from_blocked(ym, M0) if mb else ym, m), (xb, gb, mb, mode, in_place)
            # Exact-Diffusion: psi of the step before is the state
            for in_place in (False, True):
                xi = fresh(X); xo = xi if in_place else fresh(X); ps = fresh(M0)
                bf.bf_exact_diffusion_step(t, 1, xi, xo, G, ps, 0.05)
                for xb, gb, pb in ((0, 0, 1), (1, 0, 1), (0, 1, 0), (1, 1, 0)):
                    yi = to_blocked(X, B) if xb else fresh(X)
                    yo = yi if in_place else (empty_blocked(n, d, B, dtype) if xb else fresh(X))
                    yp = to_blocked(M0, B) if pb else fresh(M0)
                    bf.bf_exact_diffusion_step_layouts(t, 1, yi, yo, Gb if gb else G, yp, 0.05)
                    assert torch.equal(from_blocked(yo, X) if xb else yo, xo), (xb, gb, pb, in_place)
                    assert torch.equal(from_blocked(yp, M0) if pb else yp, ps), (xb, gb, pb, in_place)
        finally:
            bf.bf_set_tuning(6, 0)


@pytest.mark.parametrize("config", ["c2", "c3", "c4", "hier"])
def test_full_size_configs_in_column_blocks_give_the_agent_major_bits(config):
    """Configs 2, 3 and 4 and the hierarchical pass at the benchmark's sizes and block widths (the
    launch configurations bench.py times): three rounds in column blocks equal the same rounds on
    agent-major rows bit for bit; tests/test_gpu_fullsize.py holds the latter against the oracle."""
    if config == "c2":
        n, d = 64, 1 << 20
        t = bf.bf_topology_create(bf.BF_EXP_STATIC, n)
        step = lambda k, a, b: bf.bf_neighbor_allreduce(t, k, a, b)
        in_place = False
    elif config == "c3":
        n, d = 256, 1 << 22
        t = bf.bf_topology_create(bf.BF_EXP2_ONE_PEER, n)
        step = lambda k, a, b: bf.bf_neighbor_allreduce(t, k, a, b)
        in_place = True
    elif config == "c4":
        n, d = 128, 1 << 21
        t = bf.bf_topology_create(bf.BF_RANDOM_DIRECTED, n, out_degree=4, seed=workloads.CONFIG4_GRAPH_SEED)
        in_place = True
    else:
        n, d = 64, 1 << 22
        t = bf.bf_topology_create(bf.BF_EXP_STATIC, 8)
        step = lambda k, a, b: bf.bf_hierarchical_neighbor_allreduce(t, k, 8, a, b)
        in_place = True
    B = 16384 if config == "hier" else bf.bf_recommended_block(t, d, bf.BF_F32)
    ld = bf.bf_recommended_ld(d, bf.BF_F32)
    X = workloads.normal_rows(n, d, 150, DEV, ld=ld)
    Xb = to_blocked(X, B)
    Y = X if in_place else workloads.alloc_rows(n, d, torch.float32, DEV, ld=ld)
    Yb = Xb if in_place else empty_blocked(n, d, B, torch.float32)
    if config == "c4":
        w1, w2 = torch.ones(n, device=DEV), torch.ones(n, device=DEV)
    cur, curb, nxt, nxtb = X, Xb, Y, Yb
    for k in range(3):
        if config == "c4":
            bf.bf_pushsum_step(t, k, cur, nxt, w1, w1, None)
            bf.bf_pushsum_step(t, k, curb, nxtb, w2, w2, None)
        else:
            step(k, cur, nxt)
            step(k, curb, nxtb)
        cur, curb, nxt, nxtb = nxt, nxtb, cur, curb
    back = workloads.alloc_rows(n, d, torch.float32, DEV, ld=ld)
    bf.bf_blocked_unpack(curb, back)
    assert torch.equal(back, cur)
    if config == "c4":
        assert torch.equal(w1, w2)
