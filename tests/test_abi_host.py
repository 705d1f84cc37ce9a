"""Host-side checks of the C ABI that need no GPU: the library loads and exports every declared
symbol, its topologies equal the oracle's, and every argument error is reported before any launch."""

import ctypes as C
import os
import re

import numpy as np
import pytest

import paper_2111_04287_amd as bf
from oracle import iterations as O
from oracle import topology as OT

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_every_declared_symbol_is_exported():
    text = open(os.path.join(ROOT, "include", "bf.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(bf_[a-z0-9_]+)\s*\(", text))
    assert {"bf_topology_create", "bf_neighbor_allreduce", "bf_pushsum_step", "bf_atc_step"} <= declared
    raw = C.CDLL(bf.LIB_PATH)
    for name in sorted(declared):
        assert hasattr(raw, name), name
    assert declared == set(bf.EXPORTS)


def _lib_W(t, r=0):
    rowptr, col, wgt, seed = bf.bf_topology_export_csr(t, r)
    return OT.from_csr(rowptr, col, wgt), seed


def _assert_same(Wlib, Wor):
    assert set(Wlib) == set(Wor)
    for i in Wor:
        assert [j for j, _ in Wlib[i]] == [j for j, _ in Wor[i]], i
        for (_, a), (_, b) in zip(Wlib[i], Wor[i]):
            assert a == float(np.float32(b))            # the fp32 rounding of the exact weight


@pytest.mark.parametrize("n", [1, 2, 3, 5, 16, 33])
def test_ring_matches_oracle(n):
    t = bf.bf_topology_create(bf.BF_RING, n)
    _assert_same(_lib_W(t)[0], OT.ring(n))
    assert bf.bf_topology_class(t) == bf.BF_W_STANDARD and bf.bf_topology_rounds(t) == 1


@pytest.mark.parametrize("n", [1, 2, 7, 12, 32, 64, 100])
def test_static_exponential_matches_oracle(n):
    t = bf.bf_topology_create(bf.BF_EXP_STATIC, n)
    _assert_same(_lib_W(t)[0], OT.static_exponential(n))
    assert bf.bf_topology_class(t) == bf.BF_W_STANDARD


def test_static_exponential_degrees_at_benchmark_sizes():
    for n, deg in ((64, 12), (32, 10)):
        t = bf.bf_topology_create(bf.BF_EXP_STATIC, n)
        assert bf.bf_topology_max_degree(t) == deg and bf.bf_topology_nnz(t) == n * deg


@pytest.mark.parametrize("n", [1, 2, 3, 8, 256])
def test_one_peer_matches_oracle(n):
    t = bf.bf_topology_create(bf.BF_EXP2_ONE_PEER, n)
    R = bf.bf_topology_rounds(t)
    assert R == OT.one_peer_rounds(n)
    for r in range(R + 2):                                  # round index wraps
        _assert_same(_lib_W(t, r)[0], OT.one_peer_exponential(n, r))
        assert bf.bf_topology_class(t, r) == bf.BF_W_STANDARD


@pytest.mark.parametrize("n,k,seed", [(128, 4, 401), (16, 3, 11), (6, 2, 7), (5, 4, 3), (4, 0, 1)])
def test_random_directed_matches_oracle(n, k, seed):
    strong = k > 0
    t = bf.bf_topology_create(bf.BF_RANDOM_DIRECTED, n, out_degree=k, seed=seed,
                              require_strongly_connected=strong)
    Wl, s_lib = _lib_W(t)
    Wo, s_or = OT.random_directed_push(n, k, seed, require_strongly_connected=strong)
    assert s_lib == s_or
    _assert_same(Wl, Wo)
    assert bf.bf_topology_class(t) & bf.BF_W_PUSH


def test_random_directed_rejects_bad_degree_and_unconnectable():
    with pytest.raises(bf.BfError) as e:
        bf.bf_topology_create(bf.BF_RANDOM_DIRECTED, 8, out_degree=8, seed=1)
    assert e.value.code == bf.BF_ERR_SIZE
    with pytest.raises(bf.BfError) as e:                    # out-degree 0 can never be connected
        bf.bf_topology_create(bf.BF_RANDOM_DIRECTED, 4, out_degree=0, seed=1)
    assert e.value.code == bf.BF_ERR_NOT_CONNECTED


def _csr(W):
    rowptr, col, wgt = [0], [], []
    for i in range(len(W)):
        for j, w in W[i]:
            col.append(j)
            wgt.append(w)
        rowptr.append(len(col))
    return rowptr, col, wgt


def test_user_csr_round_trip_and_rounds():
    n = 8
    parts = [_csr(OT.one_peer_exponential(n, r)) for r in range(3)]
    rowptr, col, wgt = [], [], []
    for rp, c, w in parts:
        rowptr += [v + len(col) for v in rp]
        col += c
        wgt += w
    t = bf.bf_topology_create(bf.BF_CSR_USER, n, rounds=3, rowptr=rowptr, col=col, wgt=wgt,
                              require_class=bf.BF_W_STANDARD)
    assert bf.bf_topology_rounds(t) == 3
    for r in range(3):
        _assert_same(_lib_W(t, r)[0], OT.one_peer_exponential(n, r))


def test_user_csr_validation():
    n = 4
    rowptr, col, wgt = _csr(OT.ring(n))

    def create(**kw):
        a = dict(rowptr=rowptr, col=col, wgt=wgt)
        a.update(kw)
        return bf.bf_topology_create(bf.BF_CSR_USER, n, **a)

    def code(**kw):
        with pytest.raises(bf.BfError) as e:
            create(**kw)
        return e.value.code

    create()
    bad = list(col); bad[1] = 7
    assert code(col=bad) == bf.BF_ERR_CSR                       # dangling column
    bad = list(col); bad[0], bad[1] = bad[1], bad[0]
    assert code(col=bad) == bf.BF_ERR_CSR                       # unsorted row
    bad = list(col); bad[1] = bad[0]
    assert code(col=bad) == bf.BF_ERR_CSR                       # duplicate
    bad = list(rowptr); bad[2] = bad[1] - 1
    assert code(rowptr=bad) == bf.BF_ERR_CSR                    # decreasing rowptr
    bad = list(wgt); bad[0] = float("nan")
    assert code(wgt=bad) == bf.BF_ERR_CSR
    bad = list(wgt); bad[0] = 0.5
    assert code(wgt=bad, require_class=bf.BF_W_PULL) == bf.BF_ERR_NOT_STOCHASTIC
    create(wgt=bad, require_class=bf.BF_W_ANY)                  # allowed when no class is required
    assert code(require_class=8) == bf.BF_ERR_KIND


def test_dense_user_and_classes():
    rng = np.random.default_rng(0)
    n = 5
    D = rng.random((n, n)).astype(np.float32)
    D[0, 3] = 0.0
    rowst = (D / D.sum(1, keepdims=True)).astype(np.float32)
    colst = (D / D.sum(0, keepdims=True)).astype(np.float32)
    t = bf.bf_topology_create(bf.BF_DENSE_USER, n, dense_w=rowst, require_class=bf.BF_W_PULL)
    assert bf.bf_topology_class(t) == bf.BF_W_PULL
    Wl, _ = _lib_W(t)
    np.testing.assert_array_equal(OT.to_dense(Wl), rowst.astype(np.float64))
    t = bf.bf_topology_create(bf.BF_DENSE_USER, n, dense_w=colst, require_class=bf.BF_W_PUSH)
    assert bf.bf_topology_class(t) == bf.BF_W_PUSH
    with pytest.raises(bf.BfError) as e:
        bf.bf_topology_create(bf.BF_DENSE_USER, n, dense_w=colst, require_class=bf.BF_W_STANDARD)
    assert e.value.code == bf.BF_ERR_NOT_STOCHASTIC
    J = np.full((n, n), 1.0 / n, dtype=np.float32)              # periodic global averaging
    t = bf.bf_topology_create(bf.BF_DENSE_USER, n, dense_w=J, require_class=bf.BF_W_STANDARD)
    assert bf.bf_topology_nnz(t) == n * n


def test_push_pull_local_views_and_topology_check(golden_dir):
    # the 5-node example: N(5) = {1,2,3,4}, M(5) = {1,3}
    edges = []
    with open(os.path.join(golden_dir, "five_node_example.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                a, b = line.split()
                edges.append((int(a) - 1, int(b) - 1))
    n = 5
    src = {i: sorted(j for j, k in edges if k == i) for i in range(n)}
    dst = {j: sorted(k for a, k in edges if a == j) for j in range(n)}
    srp = np.cumsum([0] + [len(src[i]) for i in range(n)])
    drp = np.cumsum([0] + [len(dst[j]) for j in range(n)])
    srk = [j for i in range(n) for j in src[i]]
    drk = [k for j in range(n) for k in dst[j]]
    selfw = [1.0 / (len(dst[j]) + 1) for j in range(n)]
    dwt = [1.0 / (len(dst[j]) + 1) for j in range(n) for _ in dst[j]]
    # pure push: r = 1, s = 1/(outdeg+1) -> column stochastic
    t = bf.bf_topology_create_push_pull(n, selfw, srp, srk, None, drp, drk, dwt)
    assert bf.bf_topology_class(t) == bf.BF_W_PUSH
    Wl, _ = _lib_W(t)
    assert OT.in_lists(Wl) == src and OT.out_lists(Wl) == dst
    assert sorted(j + 1 for j in OT.in_lists(Wl)[4]) == [1, 2, 3, 4]
    assert sorted(j + 1 for j in OT.out_lists(Wl)[4]) == [1, 3]
    # pure pull: s = 1, r = 1/(indeg+1) -> row stochastic
    selfr = [1.0 / (len(src[i]) + 1) for i in range(n)]
    swt = [1.0 / (len(src[i]) + 1) for i in range(n) for _ in src[i]]
    t = bf.bf_topology_create_push_pull(n, selfr, srp, srk, swt, drp, drk, None)
    assert bf.bf_topology_class(t) == bf.BF_W_PULL
    # push-pull: w = r*s
    t = bf.bf_topology_create_push_pull(n, selfr, srp, srk, swt, drp, drk, dwt)
    D = OT.to_dense(_lib_W(t)[0])
    for j, i in edges:
        assert D[i, j] == float(np.float32(1.0 / (len(src[i]) + 1)) * np.float32(1.0 / (len(dst[j]) + 1)))
    # a receiver that expects a sender who does not send: reported, not hung
    dst_bad = dict(dst)
    dst_bad[4] = [1, 2]                                         # node 5 sends to 2 instead of 1
    bad_drk = [k for j in range(n) for k in dst_bad[j]]
    with pytest.raises(bf.BfError) as e:
        bf.bf_topology_create_push_pull(n, selfw, srp, srk, None, drp, bad_drk, dwt)
    assert e.value.code == bf.BF_ERR_TOPO_MISMATCH
    # one edge missing on the sender side
    drp2 = drp.copy(); drp2[5:] -= 1
    with pytest.raises(bf.BfError) as e:
        bf.bf_topology_create_push_pull(n, selfw, srp, srk, None, drp2, drk[:-1], dwt[:-1])
    assert e.value.code == bf.BF_ERR_TOPO_MISMATCH


def test_create_argument_errors():
    h = C.c_void_p()
    assert bf.lib.bf_topology_create(None, bf.BF_RING, 4, None) == bf.BF_ERR_NULL
    assert bf.lib.bf_topology_create(C.byref(h), bf.BF_RING, 0, None) == bf.BF_ERR_SIZE
    assert bf.lib.bf_topology_create(C.byref(h), 99, 4, None) == bf.BF_ERR_KIND
    assert bf.lib.bf_topology_create(C.byref(h), bf.BF_RANDOM_DIRECTED, 4, None) == bf.BF_ERR_NULL
    assert bf.lib.bf_topology_create(C.byref(h), bf.BF_CSR_USER, 4, None) == bf.BF_ERR_NULL
    assert h.value is None
    assert bf.lib.bf_topology_destroy(None) == bf.BF_OK
    assert bf.lib.bf_topology_n(None) == bf.BF_ERR_NULL
    assert b"aligned" in bf.lib.bf_strerror(bf.BF_ERR_ALIGN)


def test_compute_calls_validate_before_touching_the_device():
    # Fake but well-formed device addresses: every call below must fail on the host.
    t = bf.bf_topology_create(bf.BF_RING, 4)
    h = t.handle
    A, B = 0x10000000, 0x20000000
    L = bf.lib
    na = L.bf_neighbor_allreduce
    assert na(None, 0, A, B, 64, 64, bf.BF_F32, None) == bf.BF_ERR_NULL
    assert na(h, 0, None, B, 64, 64, bf.BF_F32, None) == bf.BF_ERR_NULL
    assert na(h, -1, A, B, 64, 64, bf.BF_F32, None) == bf.BF_ERR_ROUND
    assert na(h, 0, A, B, 64, 32, bf.BF_F32, None) == bf.BF_ERR_SIZE          # ld < d
    assert na(h, 0, A, B, -1, 64, bf.BF_F32, None) == bf.BF_ERR_SIZE
    assert na(h, 0, A, B, 62, 62, bf.BF_F32, None) == bf.BF_ERR_ALIGN         # row pitch 248 B
    assert na(h, 0, A + 4, B, 64, 64, bf.BF_F32, None) == bf.BF_ERR_ALIGN
    assert na(h, 0, A, B, 64, 64, 7, None) == bf.BF_ERR_KIND
    assert na(h, 0, A, A + 256, 64, 64, bf.BF_F32, None) == bf.BF_ERR_ALIAS    # partial overlap
    assert na(h, 0, A, B, 0, 64, bf.BF_F32, None) == bf.BF_OK                  # empty: nothing to launch
    assert na(h, 0, A, A, 0, 64, bf.BF_F32, None) == bf.BF_OK
    assert L.bf_dense_mix(h, 0, A, A + 256, 64, 64, bf.BF_BF16, None) == bf.BF_ERR_ALIAS
    W1b, W2b = 0x60000000, 0x60001000
    wa = L.bf_win_accumulate
    ww = L.bf_win_accumulate_weighted
    assert ww(h, 0, None, A, None, B, None, W1b + 2, None, None, 64, 64, bf.BF_BF16, None) == bf.BF_ERR_ALIGN   # self_weight
    assert ww(h, 0, None, A, None, B, None, None, None, W1b + 1, 64, 64, bf.BF_F32, None) == bf.BF_ERR_ALIGN    # dst_on
    assert ww(h, 0, None, None, None, B, None, None, None, None, 64, 64, bf.BF_F32, None) == bf.BF_ERR_NULL
    assert L.bf_win_update_weighted(h, 0, None, A, A + 512, None, None, None, 64, 64, bf.BF_F32, None) == bf.BF_ERR_ALIAS
    assert wa(h, 0, None, A, W1b, B, None, 64, 64, bf.BF_F32, None) == bf.BF_ERR_NULL        # p without win_p
    assert wa(h, 0, None, A, None, A + 512, None, 64, 64, bf.BF_F32, None) == bf.BF_ERR_ALIAS  # Win inside X
    assert wa(h, 0, None, A, W1b, B, W1b + 8, 64, 64, bf.BF_F32, None) == bf.BF_ERR_ALIAS
    assert wa(h, 0, A + 2, A, None, B, None, 64, 64, bf.BF_F32, None) == bf.BF_ERR_ALIGN
    assert wa(h, -1, None, A, None, B, None, 64, 64, bf.BF_F32, None) == bf.BF_ERR_ROUND
    assert L.bf_win_put(h, 0, None, None, B, 64, 64, bf.BF_F32, None) == bf.BF_ERR_NULL
    assert L.bf_win_update(h, 0, None, A, B + 4, 64, 64, bf.BF_F32, None) == bf.BF_ERR_ALIGN
    assert L.bf_win_update_then_collect(h, 0, None, A, W1b, B, W2b, 62, 62, bf.BF_F32, None) == bf.BF_ERR_ALIGN
    dg = L.bf_dgd_least_squares_run
    WK, G = 0x70000000, 0x40000000
    assert dg(None, 0, 5, 32, A, B, G, WK, 1e-3, 1024, 1024, None) == bf.BF_ERR_NULL
    assert dg(h, 0, 5, 32, A, B, G, None, 1e-3, 1024, 1024, None) == bf.BF_ERR_NULL
    assert dg(h, -1, 5, 32, A, B, G, WK, 1e-3, 1024, 1024, None) == bf.BF_ERR_ROUND
    assert dg(h, 0, -1, 32, A, B, G, WK, 1e-3, 1024, 1024, None) == bf.BF_ERR_SIZE
    assert dg(h, 0, 5, 0, A, B, G, WK, 1e-3, 1024, 1024, None) == bf.BF_ERR_SIZE
    assert dg(h, 0, 5, 8193, A, B, G, WK, 1e-3, 1024, 1024, None) == bf.BF_ERR_SIZE
    assert dg(h, 0, 5, 32, A, B, G, WK, 1e-3, 1022, 1024, None) == bf.BF_ERR_SIZE      # d not a multiple of 4
    assert dg(h, 0, 5, 32, A, B, G, WK, 1e-3, 1024, 1000, None) == bf.BF_ERR_SIZE      # ld < d
    assert dg(h, 0, 5, 32, A, B, G + 4, WK, 1e-3, 1024, 1024, None) == bf.BF_ERR_ALIGN
    assert dg(h, 0, 5, 32, A, B, G, G + 4096, 1e-3, 1024, 1024, None) == bf.BF_ERR_ALIAS  # work inside X
    assert dg(h, 0, 0, 32, A, B, G, WK, 1e-3, 1024, 1024, None) == bf.BF_OK              # nothing to do
    assert L.bf_dgd_status(None, None, None) == bf.BF_ERR_NULL
    ed = L.bf_exact_diffusion_least_squares_run
    assert ed(h, 0, 5, 32, A, B, G, None, WK, 1e-3, 1024, 1024, None) == bf.BF_ERR_NULL
    assert ed(h, 0, 5, 32, A, B, G, G + 16, WK, 1e-3, 1024, 1024, None) == bf.BF_ERR_ALIAS
    assert ed(h, 0, 0, 32, A, B, G, 0x50000000, WK, 1e-3, 1024, 1024, None) == bf.BF_OK
    sp = L.bf_stream_probe
    assert sp(3, A, B, 1024, 1, None) == bf.BF_ERR_KIND
    assert sp(0, None, B, 1024, 1, None) == bf.BF_ERR_NULL
    assert sp(2, None, None, 1024, 1, None) == bf.BF_ERR_NULL
    assert sp(0, A, B, 1000, 1, None) == bf.BF_ERR_SIZE
    assert sp(0, A, B, 1024, 0, None) == bf.BF_ERR_SIZE
    assert sp(0, A, A + 512, 1024, 1, None) == bf.BF_ERR_ALIAS
    assert sp(0, A + 8, B, 1024, 1, None) == bf.BF_ERR_ALIGN
    assert sp(0, A, B, 0, 1, None) == bf.BF_OK
    hn = L.bf_hierarchical_neighbor_allreduce
    assert hn(h, 0, 0, A, B, 64, 64, bf.BF_F32, None) == bf.BF_ERR_SIZE       # local_size < 1
    assert hn(h, 0, 1 << 19, A, B, 64, 64, bf.BF_F32, None) == bf.BF_ERR_SIZE
    assert hn(None, 0, 2, A, B, 64, 64, bf.BF_F32, None) == bf.BF_ERR_NULL
    assert hn(h, -1, 2, A, B, 64, 64, bf.BF_F32, None) == bf.BF_ERR_ROUND
    assert hn(h, 0, 2, A, A + 256, 64, 64, bf.BF_F32, None) == bf.BF_ERR_ALIAS
    assert hn(h, 0, 2, A, B, 0, 64, bf.BF_F32, None) == bf.BF_OK
    nm = L.bf_neighbor_allreduce_multi
    assert nm(h, 0, 0, A, B, 64, 64, bf.BF_F32, None) == bf.BF_ERR_SIZE       # count out of [1, 8]
    assert nm(h, 0, 9, A, B, 64, 64, bf.BF_F32, None) == bf.BF_ERR_SIZE
    assert nm(h, -2, 2, A, B, 64, 64, bf.BF_F32, None) == bf.BF_ERR_ROUND
    assert nm(h, 0, 2, A, A + 256, 64, 64, bf.BF_F32, None) == bf.BF_ERR_ALIAS
    assert nm(h, 0, 2, None, B, 64, 64, bf.BF_F32, None) == bf.BF_ERR_NULL
    assert nm(h, 0, 2, A, B, 0, 64, bf.BF_F32, None) == bf.BF_OK
    ps = L.bf_pushsum_step
    W1, W2 = 0x30000000, 0x30001000
    assert ps(h, 0, A, B, None, W2, None, 64, 64, bf.BF_F32, None) == bf.BF_ERR_NULL
    assert ps(h, 0, A, B, W1, W1 + 8, None, 64, 64, bf.BF_F32, None) == bf.BF_ERR_ALIAS
    assert ps(h, 0, A, B, W1, W2, A, 64, 64, bf.BF_F32, None) == bf.BF_ERR_ALIAS   # Y aliases X_in
    assert ps(h, 0, A, B, W1, A, None, 64, 64, bf.BF_F32, None) == bf.BF_ERR_ALIAS  # w_out inside X
    at = L.bf_atc_step
    G, M = 0x40000000, 0x50000000
    assert at(h, 0, A, B, None, None, 0.1, 0.0, bf.BF_ATC, 64, 64, bf.BF_F32, None) == bf.BF_ERR_NULL
    assert at(h, 0, A, B, G, None, 0.1, 0.0, 5, 64, 64, bf.BF_F32, None) == bf.BF_ERR_KIND
    assert at(h, 0, A, B, B, None, 0.1, 0.0, bf.BF_ATC, 64, 64, bf.BF_F32, None) == bf.BF_ERR_ALIAS
    assert at(h, 0, A, B, G, A, 0.1, 0.9, bf.BF_ATC, 64, 64, bf.BF_F32, None) == bf.BF_ERR_ALIAS
    assert at(h, 0, A, B, G, M + 8, 0.1, 0.9, bf.BF_ATC, 64, 64, bf.BF_F32, None) == bf.BF_ERR_ALIGN
    ls = L.bf_grad_least_squares
    assert ls(4, 0, 64, A, B, G, 64, M, 64, None) == bf.BF_ERR_SIZE
    assert ls(4, 8193, 64, A, B, G, 64, M, 64, None) == bf.BF_ERR_SIZE
    assert ls(4, 8, 62, A, B, G, 64, M, 64, None) == bf.BF_ERR_SIZE
    assert ls(4, 8, 64, A, B, G, 64, G, 64, None) == bf.BF_ERR_ALIAS
    assert ls(4, 8, 64, A, None, G, 64, M, 64, None) == bf.BF_ERR_NULL
    gq = L.bf_grad_quadratic
    assert gq(4, 64, 64, A, B, G, 1.0, 0.1, A, bf.BF_F32, None) == bf.BF_ERR_ALIAS
    assert gq(0, 64, 64, A, B, G, 1.0, 0.1, M, bf.BF_F32, None) == bf.BF_ERR_SIZE
    cs = L.bf_consensus_stats
    assert cs(4, 64, 64, A, None, bf.BF_F32, None, None, None) == bf.BF_ERR_NULL
    assert cs(4, 64, 64, A, None, bf.BF_F32, M + 4, None, None) == bf.BF_ERR_ALIGN
    assert L.bf_set_tuning(99, 1) == bf.BF_ERR_KIND
    assert L.bf_pushsum_atc_step(h, 0, A, B, None, 0.1, W1, W2, None, 64, 64, bf.BF_F32, None) == bf.BF_ERR_NULL
    assert L.bf_pushsum_atc_step(h, 0, A, B, B, 0.1, W1, W2, None, 64, 64, bf.BF_F32, None) == bf.BF_ERR_ALIAS
    assert L.bf_tracking_step(h, 0, A, B, G, None, 64, 64, bf.BF_F32, None) == bf.BF_ERR_NULL
    assert L.bf_tracking_step(h, 0, A, B, B, G, 64, 64, bf.BF_F32, None) == bf.BF_ERR_ALIAS
    assert L.bf_tracking_step(h, -1, A, B, G, M, 64, 64, bf.BF_F32, None) == bf.BF_ERR_ROUND
    assert L.bf_exact_diffusion_step(h, 0, A, B, G, None, 0.1, 64, 64, bf.BF_F32, None) == bf.BF_ERR_NULL
    assert L.bf_exact_diffusion_step(h, 0, A, B, G, A, 0.1, 64, 64, bf.BF_F32, None) == bf.BF_ERR_ALIAS
    assert L.bf_set_tuning(0, 0) == bf.BF_OK


def test_column_block_layout_argument_checks():
    t = bf.bf_topology_create(bf.BF_RING, 4)
    h = t.handle
    A, B = 0x10000000, 0x20000000
    L = bf.lib
    assert bf.bf_blocked_elems(4, 1000, 256) == 4 * 1024
    assert bf.bf_blocked_elems(3, 0, 64) == 0
    assert L.bf_blocked_elems(4, 1000, 100) == bf.BF_ERR_SIZE              # not a power of two
    assert L.bf_blocked_elems(4, 1000, 32) == bf.BF_ERR_SIZE
    assert L.bf_blocked_elems(4, 1000, 1 << 21) == bf.BF_ERR_SIZE
    assert L.bf_blocked_elems(0, 1000, 64) == bf.BF_ERR_SIZE
    rb = lambda kind, n, d, dt=bf.BF_F32: bf.bf_recommended_block(bf.bf_topology_create(kind, n), d, dt)
    assert rb(bf.BF_EXP_STATIC, 32, 25557032, bf.BF_BF16) == 8192 and rb(bf.BF_EXP_STATIC, 64, 1 << 20) == 16384
    assert rb(bf.BF_EXP_STATIC, 128, 1 << 21) == 8192 and rb(bf.BF_EXP_STATIC, 256, 1 << 22) == 4096
    assert rb(bf.BF_EXP_STATIC, 3000, 1 << 22) == 2048 and rb(bf.BF_EXP_STATIC, 5, 4096) == 4096
    assert rb(bf.BF_RING, 5, 100) == 128 and rb(bf.BF_RING, 5, 3) == 64 and rb(bf.BF_RING, 5, 0) == 64
    # rounds that are unions of paths and cycles, more agents than 128-column tiles allow: the row-streaming kernel
    assert rb(bf.BF_EXP2_ONE_PEER, 256, 1 << 22) == 65536 and rb(bf.BF_RING, 200, 1 << 22) == 65536
    assert rb(bf.BF_EXP2_ONE_PEER, 128, 1 << 22) == 8192 and rb(bf.BF_EXP2_ONE_PEER, 256, 20000) == 32768
    assert L.bf_recommended_block(None, 100, bf.BF_F32) == bf.BF_ERR_NULL
    assert L.bf_recommended_block(h, 100, 9) == bf.BF_ERR_KIND and L.bf_recommended_block(h, -1, bf.BF_F32) == bf.BF_ERR_SIZE
    na = L.bf_neighbor_allreduce
    assert na(h, 0, A, B, 100, -100, bf.BF_F32, None) == bf.BF_ERR_SIZE       # block width not a power of two
    assert na(h, 0, A, B, 100, -32, bf.BF_F32, None) == bf.BF_ERR_SIZE
    assert na(h, 0, A, B, 100, -(1 << 21), bf.BF_F32, None) == bf.BF_ERR_SIZE
    assert na(h, 0, A, B, 0, -64, bf.BF_F32, None) == bf.BF_OK               # empty
    assert na(h, 0, A, A + 1024, 100, -64, bf.BF_F32, None) == bf.BF_ERR_ALIAS   # 2 blocks x 4 x 64 x 4 = 2048 bytes each
    assert na(h, 0, A, A + 2048, 0, -64, bf.BF_F32, None) == bf.BF_OK
    # calls that take agent-major matrices only
    assert L.bf_neighbor_allreduce_multi(h, 0, 2, A, A + 1024, 100, -64, bf.BF_F32, None) == bf.BF_ERR_ALIAS
    assert L.bf_hierarchical_neighbor_allreduce(h, 0, 2, A, A + 2048, 100, -64, bf.BF_F32, None) == bf.BF_ERR_ALIAS   # 8 rows
    assert L.bf_neighbor_allreduce_multi(h, 0, 2, A, B, 0, -64, bf.BF_F32, None) == bf.BF_OK
    assert L.bf_dense_mix(h, 0, A, A + 1024, 100, -64, bf.BF_F32, None) == bf.BF_ERR_ALIAS
    assert L.bf_win_put(h, 0, None, A, A + 1024, 100, -64, bf.BF_F32, None) == bf.BF_ERR_ALIAS
    assert L.bf_dgd_least_squares_run(h, 0, 5, 32, A, B, 0x40000000, 0x70000000, 1e-3, 1024, -1024, None) == bf.BF_ERR_SIZE
    assert L.bf_consensus_stats(4, 100, -100, A, None, bf.BF_F32, B, None, None) == bf.BF_ERR_SIZE
    assert L.bf_grad_quadratic(4, 100, -64, A, B, 0x40000000, 1.0, 0.1, A + 1024, bf.BF_F32, None) == bf.BF_ERR_ALIAS
    # the state matrix of a momentum step has the layout of X: its extent follows the blocks
    G, M = 0x40000000, 0x50000000
    at = L.bf_atc_step
    assert at(h, 0, A, A, G, A + 512, 0.1, 0.9, bf.BF_ATC, 100, -64, bf.BF_BF16, None) == bf.BF_ERR_ALIAS
    assert at(h, 0, A, A, G, G + 1024, 0.1, 0.9, bf.BF_ATC, 100, -64, bf.BF_F32, None) == bf.BF_ERR_ALIAS    # M inside G (2048 bytes)
    ag = L.bf_atc_step_layouts
    assert ag(h, 0, A, A, None, None, 0.1, 0.0, bf.BF_ATC, 100, -64, 104, 104, bf.BF_F32, None) == bf.BF_ERR_NULL
    assert ag(h, 0, A, A, G, None, 0.1, 0.0, bf.BF_ATC, 100, -64, 96, 104, bf.BF_F32, None) == bf.BF_ERR_SIZE      # ld_g < d
    assert ag(h, 0, A, A, G, None, 0.1, 0.0, bf.BF_ATC, 100, -64, -100, 104, bf.BF_F32, None) == bf.BF_ERR_SIZE
    assert ag(h, 0, A, A, G, M, 0.1, 0.9, bf.BF_ATC, 100, 104, 104, -100, bf.BF_F32, None) == bf.BF_ERR_SIZE        # ld_m
    assert ag(h, 0, A, A, G, M, 0.1, 0.9, bf.BF_ATC, 100, 104, 104, 102, bf.BF_BF16, None) == bf.BF_ERR_ALIGN       # M is fp32: 408-byte rows
    assert ag(h, 0, A, A, A + 1024, None, 0.1, 0.0, bf.BF_ATC, 100, -64, 104, 104, bf.BF_F32, None) == bf.BF_ERR_ALIAS   # G inside X_out
    assert ag(h, 0, A, A, G, G + 256, 0.1, 0.9, bf.BF_ATC, 100, -64, 104, -64, bf.BF_F32, None) == bf.BF_ERR_ALIAS       # M inside G's rows
    assert ag(h, 0, A, A, G, A + 1600, 0.1, 0.9, bf.BF_ATC, 100, 104, 104, -64, bf.BF_F32, None) == bf.BF_ERR_ALIAS      # M (blocks) inside X (rows)
    el = L.bf_exact_diffusion_step_layouts
    assert el(h, 0, A, A, G, None, 0.1, 100, 104, 104, -64, bf.BF_F32, None) == bf.BF_ERR_NULL
    assert el(h, 0, A, A, G, M, 0.1, 100, 104, 104, -100, bf.BF_F32, None) == bf.BF_ERR_SIZE
    assert el(h, 0, A, A, G, G + 1024, 0.1, 100, 104, -64, -64, bf.BF_F32, None) == bf.BF_ERR_ALIAS
    pk, up = L.bf_blocked_pack, L.bf_blocked_unpack
    assert pk(4, 100, 104, None, 64, B, bf.BF_F32, None) == bf.BF_ERR_NULL
    assert pk(4, 100, 104, A, 100, B, bf.BF_F32, None) == bf.BF_ERR_SIZE
    assert pk(4, 100, 96, A, 64, B, bf.BF_F32, None) == bf.BF_ERR_SIZE       # ld < d
    assert pk(4, 100, 102, A, 64, B, bf.BF_F32, None) == bf.BF_ERR_ALIGN
    assert pk(4, 100, 104, A, 64, A + 1024, bf.BF_F32, None) == bf.BF_ERR_ALIAS
    assert pk(0, 100, 104, A, 64, B, bf.BF_F32, None) == bf.BF_ERR_SIZE
    assert pk(4, 0, 104, A, 64, B, bf.BF_F32, None) == bf.BF_OK
    assert up(4, 100, 64, A, 104, A + 1024, bf.BF_F32, None) == bf.BF_ERR_ALIAS
    assert up(4, 100, 64, A, 104, B + 8, bf.BF_F32, None) == bf.BF_ERR_ALIGN
    assert up(4, 0, 64, A, 104, B, bf.BF_F32, None) == bf.BF_OK


def _walk_chain_plan(steps, X):
    """Replay a chain plan the way the streaming kernel does: three live rows, each row loaded once."""
    n = X.shape[0]
    out = np.full_like(X, np.nan)
    loads = []

    def load(r):
        loads.append(int(r))
        return X[r].copy()

    prev = cur = nxt = first = last = None
    for k in range(n):
        row, flags, last_row, next_row, slots = (int(v) for v in steps[k, :5])
        w = steps[k, 5:8].view(np.float32).astype(np.float64)
        if flags & 1:
            prev = first = last = None
            if flags & 2:
                last = load(last_row)
                prev = last
            cur = load(row)
            first = cur
        nk = (flags >> 2) & 3
        nxt = load(next_row) if nk == 0 else last if nk == 1 else first if nk == 2 else None
        acc = np.zeros(X.shape[1])
        for e in range(3):
            code = (slots >> (4 * e)) & 15
            if code != 15:
                acc += w[e] * (prev, cur, nxt)[code]
        assert np.isnan(out[row]).all()
        out[row] = acc
        prev, cur = cur, nxt
    assert sorted(loads) == list(range(n))             # every row read exactly once
    return out


@pytest.mark.parametrize("make,rounds", [
    (lambda: bf.bf_topology_create(bf.BF_RING, 16), 1),
    (lambda: bf.bf_topology_create(bf.BF_RING, 3), 1),
    (lambda: bf.bf_topology_create(bf.BF_RING, 2), 1),
    (lambda: bf.bf_topology_create(bf.BF_RING, 1), 1),
    (lambda: bf.bf_topology_create(bf.BF_EXP2_ONE_PEER, 256), 8),
    (lambda: bf.bf_topology_create(bf.BF_EXP2_ONE_PEER, 12), 4),
    (lambda: bf.bf_topology_create(bf.BF_EXP2_ONE_PEER, 2), 1),
    (lambda: bf.bf_topology_create(bf.BF_EXP_STATIC, 4), 1),      # neighbors +-1, 2: three partners -> no plan
])
def test_chain_plan_replays_to_the_oracle_mix(make, rounds):
    from oracle import iterations as O
    t = make()
    n = bf.bf_topology_n(t) if hasattr(bf, "bf_topology_n") else t.n
    rng = np.random.default_rng(n)
    X = rng.normal(size=(n, 5))
    for r in range(rounds):
        steps = bf.bf_topology_chain_plan(t, r)
        W = _lib_W(t, r)[0]
        partners = max(len(set(j for j, _ in W[i] if j != i) | set(k for k in W if any(j == i for j, _ in W[k]) and k != i))
                       for i in W)
        if partners > 2:
            assert steps is None
            continue
        assert steps is not None and steps.shape == (n, 8)
        np.testing.assert_allclose(_walk_chain_plan(steps, X), O.mix(X, W), atol=1e-14)


def test_chain_plan_on_a_directed_path_and_a_matching():
    from oracle import iterations as O
    # rows pull from the next row only, last row keeps itself: a path, not a cycle
    n = 5
    D = np.eye(n, dtype=np.float32) * 0.25
    for i in range(n - 1):
        D[i, i + 1] = 0.75
    D[n - 1, n - 1] = 1.0
    t = bf.bf_topology_create(bf.BF_DENSE_USER, n, dense_w=D)
    steps = bf.bf_topology_chain_plan(t, 0)
    X = np.random.default_rng(1).normal(size=(n, 3))
    np.testing.assert_allclose(_walk_chain_plan(steps, X), D.astype(np.float64) @ X, atol=1e-14)
    assert not (steps[:, 1] & 2).any()
    # a perfect matching with asymmetric weights, plus one isolated agent
    n = 7
    D = np.zeros((n, n), dtype=np.float32)
    for a, b in ((0, 4), (1, 5), (2, 3)):
        D[a, a], D[a, b], D[b, b], D[b, a] = 0.3, 0.7, 0.6, 0.4
    D[6, 6] = 1.0
    t = bf.bf_topology_create(bf.BF_DENSE_USER, n, dense_w=D)
    steps = bf.bf_topology_chain_plan(t, 0)
    X = np.random.default_rng(2).normal(size=(n, 3))
    np.testing.assert_allclose(_walk_chain_plan(steps, X), D.astype(np.float64) @ X, atol=1e-14)


@pytest.mark.parametrize("kind,n,kw", [(bf.BF_RING, 7, {}), (bf.BF_EXP_STATIC, 16, {}), (bf.BF_EXP2_ONE_PEER, 8, {}),
                                       (bf.BF_RANDOM_DIRECTED, 12, dict(out_degree=3, seed=9)), (bf.BF_RING, 1, {})])
def test_window_layout_matches_the_oracle(kind, n, kw):
    t = bf.bf_topology_create(kind, n, **kw)
    for rnd in range(bf.bf_topology_rounds(t)):
        rowptr, col, wgt, _ = bf.bf_topology_export_csr(t, rnd)
        W = OT.from_csr(rowptr, col, wgt)
        slot_ptr, slot_src, slot_w, self_w = O.window_slots(W)
        rp, src, sw, selfw = bf.bf_topology_export_window(t, rnd)
        assert bf.bf_topology_window_slots(t, rnd) == slot_ptr[-1]
        assert list(rp) == slot_ptr and list(src) == slot_src
        np.testing.assert_array_equal(sw, np.asarray(slot_w, dtype=np.float32))
        np.testing.assert_array_equal(selfw, np.asarray(self_w, dtype=np.float32))
    assert bf.lib.bf_topology_window_slots(None, 0) == bf.BF_ERR_NULL
    assert bf.lib.bf_topology_window_slots(t.handle, -1) == bf.BF_ERR_ROUND


def test_host_code_is_clean_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    """The topology code (generators, validators, chain / window / two-level plans, exports) built
    with g++ -fsanitize=address,undefined and driven over every kind and a range of sizes."""
    import shutil
    import subprocess
    if shutil.which("g++") is None:
        pytest.skip("no g++")
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    exe = str(tmp_path / "driver")
    cmd = ["g++", "-O1", "-g", "-std=c++17", "-fsanitize=address,undefined", "-static-libasan", "-static-libubsan",
           "-fno-omit-frame-pointer", "-I" + os.path.join(root, "include"),
           "-I" + os.path.join(root, "paper_2111_04287_amd", "csrc"),
           os.path.join(root, "tests", "host_sanitizer_driver.cpp"),
           os.path.join(root, "paper_2111_04287_amd", "csrc", "bf_topology.cpp"), "-o", exe]
    b = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if b.returncode != 0 and "sanitize" in b.stdout:
        pytest.skip("this g++ has no sanitizer runtime")
    assert b.returncode == 0, b.stdout
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0", UBSAN_OPTIONS="halt_on_error=1")
    r = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, env=env, timeout=300)
    assert r.returncode == 0 and "0 failures" in r.stdout, r.stdout[-2000:]
