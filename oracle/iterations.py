"""Oracle iterations in fp64 numpy.  TEST INFRASTRUCTURE ONLY.

State layout: ``X`` is an (n, d) array whose row i is agent i's vector x_i.
``W`` is a dictionary of in-neighbor lists (see ``oracle.topology``).
Every function returns new arrays and leaves its arguments untouched.
Each function is the definition it cites written out row by row; there is no
blocking, fusion or reordering.
"""

import numpy as np


def _f64(a):
    return np.asarray(a, dtype=np.float64)


def mix(X, W):
    """Partial averaging (eq. dsgd-2, eq. dgd-2):
    x_i <- w_ii x_i + sum_{j in N(i)} w_ij x_j, for every agent i."""
    X = _f64(X)
    out = np.zeros_like(X)
    for i in range(X.shape[0]):
        for j, w in W[i]:
            out[i, :] += w * X[j, :]
    return out


def mix_push_pull(X, self_w, r, s):
    """Time-varying partial averaging with sender-side scaling s_ij and
    receiver-side scaling r_ij (eqs. 2bzbz09, dyn-push-comm, dyn-pull-comm):
    y_ij = s_ij x_j ;  x_i <- w_ii x_i + sum_j r_ij y_ij.
    ``r`` and ``s`` are dictionaries i -> [(j, weight)] over N(i); ``self_w[i]``
    is w_ii."""
    X = _f64(X)
    out = np.zeros_like(X)
    for i in range(X.shape[0]):
        out[i, :] += self_w[i] * X[i, :]
        sj = dict(s[i])
        for j, rij in r[i]:
            y_ij = sj[j] * X[j, :]
            out[i, :] += rij * y_ij
    return out


def pushsum_step(X, p, W):
    """One synchronous push-sum round (push-sum recursion with all delays equal
    to one; identical to the u, v, x lines of push-sum gradient tracking with a
    zero step): x <- W x, p <- W p, y_i = x_i / p_i.  W is column stochastic
    and p starts at one.  Returns (X', p', Y)."""
    X = _f64(X)
    p = _f64(p)
    Xn = mix(X, W)
    pn = np.zeros_like(p)
    for i in range(p.shape[0]):
        for j, w in W[i]:
            pn[i] += w * p[j]
    Y = Xn / pn[:, None]
    return Xn, pn, Y


def atc_step(X, G, W, alpha):
    """Adapt-then-combine (eq. eq.atc; eqs. dsgd-1/dsgd-2; dgd-1/dgd-2):
    x_i <- sum_{j in N(i) or j=i} w_ij (x_j - alpha g_j), g_j the gradient of
    agent j at its own previous iterate."""
    X = _f64(X)
    G = _f64(G)
    half = X - alpha * G
    return mix(half, W)


def awc_step(X, G, W, alpha):
    """Adapt-while-communicate (eq. eq.awc):
    x_i <- sum_{j in N(i) or j=i} w_ij x_j - alpha g_i."""
    X = _f64(X)
    G = _f64(G)
    return mix(X, W) - alpha * G


def dmsgd_atc_step(X, M, G, W, alpha, beta):
    """Heavy-ball decentralized momentum SGD in adapt-then-combine order.
    The paper names decentralized momentum SGD in its accuracy tables but gives
    no recursion; this is the plain form: m_i <- beta m_i + g_i, then eq.atc
    with m_i in the place of the gradient.  Returns (X', M')."""
    X = _f64(X)
    M = _f64(M)
    G = _f64(G)
    Mn = beta * M + G
    return mix(X - alpha * Mn, W), Mn


def ls_grad(A, b, X):
    """Local least-squares gradients used by decentralized gradient descent
    (eq. dgd-1): g_i = A_i^T (A_i x_i - b_i).  A is (n, m, d), b is (n, m)."""
    A = _f64(A)
    b = _f64(b)
    X = _f64(X)
    G = np.zeros_like(X)
    for i in range(X.shape[0]):
        resid = A[i] @ X[i] - b[i]
        G[i, :] = A[i].T @ resid
    return G


def quadratic_noise_grad(X, C, E, lam, sigma):
    """Synthetic local gradient of f_i(x) = lam/2 |x - c_i|^2 plus additive
    noise: g_i = lam (x_i - c_i) + sigma e_i (the benchmark's stand-in for a
    network's stochastic gradient)."""
    return lam * (_f64(X) - _f64(C)) + sigma * _f64(E)


def exact_diffusion_step(X, psi_prev, G, W, alpha):
    """Exact-Diffusion (eqs. ed-1, ed-2, ed-3): psi = x - alpha g;
    phi = psi + x - psi_prev; x <- W phi.  Returns (X', psi)."""
    X = _f64(X)
    psi = X - alpha * _f64(G)
    phi = psi + X - _f64(psi_prev)
    return mix(phi, W), psi


def column_mean(X):
    return _f64(X).mean(axis=0)


def consensus_error(X):
    """Frobenius distance of X from the consensus matrix 1 xbar^T."""
    X = _f64(X)
    return float(np.linalg.norm(X - X.mean(axis=0, keepdims=True)))


def round_to_bf16(x32):
    """Round fp32 values to the nearest bfloat16 (ties to even), returned as
    fp32.  bfloat16 is the top 16 bits of the IEEE-754 binary32 pattern; NaNs
    are kept quiet."""
    a = np.ascontiguousarray(x32, dtype=np.float32)
    u = a.view(np.uint32).astype(np.uint64)
    lsb = (u >> 16) & 1
    r = ((u + 0x7FFF + lsb) >> 16) << 16
    nan = np.isnan(a)
    r = np.where(nan, (u | 0x00400000) & 0xFFFF0000, r)
    return (r & 0xFFFFFFFF).astype(np.uint32).view(np.float32).reshape(a.shape)


def dmsgd_atc_step_bf16_storage(X_bf, M32, G_bf, W, alpha, beta):
    """Diagnostic twin of ``dmsgd_atc_step`` for the bf16-storage layout: X and
    G hold bf16 values, M holds fp32 values; arithmetic is exact fp64 and each
    result is rounded once to its storage type (M to fp32, X to fp32 then
    bf16).  Returns (X' as fp32 holding bf16 values, M' as fp32)."""
    Mn = (beta * _f64(M32) + _f64(G_bf)).astype(np.float32)
    Xn = mix(_f64(X_bf) - alpha * _f64(Mn), W)
    return round_to_bf16(Xn.astype(np.float32)), Mn


def mix_fp32_chain(X32, W):
    """fp32 emulation of a fused-multiply-add chain over each in-neighbor list
    in list order: acc = fl(w_0 x_0); acc = fl(w_p x_p + acc).  Each product is
    exact in fp64 (24+24 bits); the fp64 sum is then rounded to fp32.  This is
    bit-identical to a hardware FMA chain whenever w_p x_p + acc is exact in
    fp64 before the final rounding, in particular for power-of-two weights
    (the one-peer exponential graph, where each round is one correctly rounded
    fp32 addition of two exactly halved values)."""
    X32 = np.asarray(X32, dtype=np.float32)
    out = np.zeros_like(X32)
    for i in range(X32.shape[0]):
        acc = None
        for j, w in W[i]:
            prod = np.float64(np.float32(w)) * X32[j, :].astype(np.float64)
            if acc is None:
                acc = prod.astype(np.float32)
            else:
                acc = (prod + acc.astype(np.float64)).astype(np.float32)
        out[i, :] = acc
    return out


def pushsum_gradient_tracking_step(U, v, Y, G_prev, W, alpha, grad):
    """One iteration of push-sum gradient tracking over a (possibly time-varying) column-stochastic
    W (appendix "Application example: Push-sum gradient tracking algorithm"):
        u' = W (u - alpha y);  v' = W v;  x' = u' / v';  g' = grad(x');  y' = W (y + g' - g_prev).
    ``grad`` maps the (n, d) matrix of iterates to the (n, d) matrix of local gradients.
    Start: v = 1, y = g_prev = grad(x^0), u = x^0.  Returns (U', v', X', Y', G')."""
    U = _f64(U)
    v = _f64(v)
    Y = _f64(Y)
    G_prev = _f64(G_prev)
    Un = mix(U - alpha * Y, W)
    vn = np.zeros_like(v)
    for i in range(v.shape[0]):
        for j, w in W[i]:
            vn[i] += w * v[j]
    Xn = Un / vn[:, None]
    Gn = _f64(grad(Xn))
    Yn = mix(Y + Gn - G_prev, W)
    return Un, vn, Xn, Yn, Gn


def hierarchical_neighbor_allreduce(X, W_machine, local_size):
    """Two-level neighbor averaging (section "Enabling hierarchical communication"): machine a owns
    the agents a*local_size .. (a+1)*local_size-1 (machine_rank = rank // local_size).
    Stage 1: each machine averages its agents.  Stage 2: one round of partial averaging of those
    machine values over the machine-level W.  Stage 3: every agent takes its machine's result."""
    X = _f64(X)
    n = X.shape[0]
    L = int(local_size)
    if L < 1 or n % L:
        raise ValueError("the number of agents must be a multiple of local_size")
    M = n // L
    local_avg = np.zeros((M, X.shape[1]))
    for a in range(M):
        for l in range(L):
            local_avg[a, :] += X[a * L + l, :]
        local_avg[a, :] /= L
    machine_out = np.zeros_like(local_avg)
    for a in range(M):
        for b, w in W_machine[a]:
            machine_out[a, :] += w * local_avg[b, :]
    out = np.zeros_like(X)
    for i in range(n):
        out[i, :] = machine_out[i // L, :]
    return out


# --------------------------------------------------------------------------------------------------
# Window (one-sided) primitives, section "Asynchronous decentralized communication".  Agent i owns a
# window with one slot per in-neighbor, in the order of its in-neighbor list with the self entry
# left out.  ``Win`` is the (E, d) matrix of all slots, agent 0's slots first; ``win_p`` the (E,)
# vector of the matching slots of the push-sum scalar p.  ``active`` says which agents execute the
# call (an agent that is not active does nothing, which is how the lack of a common clock is
# simulated on one device); None means everybody.

def window_slots(W):
    """(slot_ptr, slot_src, slot_w, self_w): agent i's slots are slot_ptr[i] .. slot_ptr[i+1]-1,
    slot e receives from agent slot_src[e] with weight slot_w[e] = w_{i,src}; self_w[i] = w_ii
    (zero when the list has no self entry)."""
    n = len(W)
    slot_ptr, slot_src, slot_w, self_w = [0], [], [], [0.0] * n
    for i in range(n):
        for j, w in W[i]:
            if j == i:
                self_w[i] = w
            else:
                slot_src.append(j)
                slot_w.append(w)
        slot_ptr.append(len(slot_src))
    return slot_ptr, slot_src, slot_w, self_w


def _is_active(active, j):
    return True if active is None else bool(active[j])


def win_put(X, Win, W, active=None):
    """neighbor_win_put without weights: every active agent j overwrites its slot in the window of
    each of its out-neighbors with x_j.  Returns Win'."""
    X = _f64(X)
    Win = _f64(Win).copy()
    slot_ptr, slot_src, _, _ = window_slots(W)
    for e, j in enumerate(slot_src):
        if _is_active(active, j):
            Win[e, :] = X[j, :]
    return Win


def win_get(X, Win, W, active=None):
    """neighbor_win_get without weights: every active agent i fetches x_j of each in-neighbor j
    into its own slot for j (pull style).  Returns Win'."""
    X = _f64(X)
    Win = _f64(Win).copy()
    slot_ptr, slot_src, _, _ = window_slots(W)
    for i in range(X.shape[0]):
        if _is_active(active, i):
            for e in range(slot_ptr[i], slot_ptr[i + 1]):
                Win[e, :] = X[slot_src[e], :]
    return Win


def win_accumulate(X, p, Win, win_p, W, active=None):
    """neighbor_win_accumulate in the push-sum use of the section "Asynchronous push-style partial
    averaging": every active agent j adds w_ij x_j (and w_ij p_j) to its slot at each out-neighbor
    i, then keeps w_jj x_j (and w_jj p_j) for itself.  Returns (X', p', Win', win_p')."""
    X = _f64(X).copy()
    p = _f64(p).copy()
    Win = _f64(Win).copy()
    win_p = _f64(win_p).copy()
    slot_ptr, slot_src, slot_w, self_w = window_slots(W)
    for e, j in enumerate(slot_src):
        if _is_active(active, j):
            Win[e, :] += slot_w[e] * X[j, :]
            win_p[e] += slot_w[e] * p[j]
    for j in range(X.shape[0]):
        if _is_active(active, j):
            X[j, :] *= self_w[j]
            p[j] *= self_w[j]
    return X, p, Win, win_p


def win_update_then_collect(X, p, Win, win_p, W, active=None):
    """win_update_then_collect: every active agent i adds all its slots to its own tensor and
    resets them to zero, as one atomic step (so that the sum of p over tensors and windows never
    changes).  Returns (X', p', Win', win_p')."""
    X = _f64(X).copy()
    p = _f64(p).copy()
    Win = _f64(Win).copy()
    win_p = _f64(win_p).copy()
    slot_ptr, _, _, _ = window_slots(W)
    for i in range(X.shape[0]):
        if _is_active(active, i):
            for e in range(slot_ptr[i], slot_ptr[i + 1]):
                X[i, :] += Win[e, :]
                p[i] += win_p[e]
                Win[e, :] = 0.0
                win_p[e] = 0.0
    return X, p, Win, win_p


def win_update(X, Win, W, active=None):
    """win_update with the topology's weights: every active agent i returns
    w_ii x_i + sum_j w_ij (slot of j); the window keeps its contents.  Returns X'."""
    X = _f64(X).copy()
    Win = _f64(Win)
    slot_ptr, _, slot_w, self_w = window_slots(W)
    for i in range(X.shape[0]):
        if _is_active(active, i):
            acc = self_w[i] * X[i, :]
            for e in range(slot_ptr[i], slot_ptr[i + 1]):
                acc = acc + slot_w[e] * Win[e, :]
            X[i, :] = acc
    return X


# --------------------------------------------------------------------------------------------------
# The same primitives with the per-call weight arguments of the section "Asynchronous decentralized
# communication": neighbor_win_put / neighbor_win_accumulate(tensor, name, [self_weight,
# dst_weights]), neighbor_win_get(tensor, name, [src_weights]), win_update(name, [self_weight,
# src_weights]).  ``dst_weights[j]`` is a dictionary {i: weight} over a SUBSET of j's out-neighbors
# in the static topology, ``src_weights[i]`` a dictionary {j: weight} over a subset of i's
# in-neighbors; an edge that is not named is not touched (put, accumulate, get) or not included
# (update).  ``self_weight[j]`` scales the caller's own tensor.  None means: no such argument.

def _slot_index(W):
    """{(receiver i, sender j): slot number} in the layout of ``window_slots``."""
    slot_ptr, slot_src, _, _ = window_slots(W)
    index = {}
    for i in range(len(W)):
        for e in range(slot_ptr[i], slot_ptr[i + 1]):
            index[(i, slot_src[e])] = e
    return index


def _check_subset(index, i, j):
    if (i, j) not in index:
        raise ValueError("edge %d -> %d is not in the static topology" % (j, i))
    return index[(i, j)]


def win_put_weighted(X, Win, W, active=None, self_weight=None, dst_weights=None):
    """neighbor_win_put(tensor, name, [self_weight, dst_weights]): every active agent j overwrites
    its slot at each named out-neighbor i with dst_weights[j][i] * x_j (all out-neighbors, weight 1,
    without the argument), then keeps self_weight[j] * x_j (x_j itself without the argument).
    Returns (X', Win')."""
    X = _f64(X).copy()
    Win = _f64(Win).copy()
    index = _slot_index(W)
    n = X.shape[0]
    for j in range(n):
        if not _is_active(active, j):
            continue
        if dst_weights is None:
            targets = {i: 1.0 for (i, jj) in index if jj == j}
        else:
            targets = dst_weights[j]
        for i, w in targets.items():
            Win[_check_subset(index, i, j), :] = w * X[j, :]
    if self_weight is not None:
        for j in range(n):
            if _is_active(active, j):
                X[j, :] *= self_weight[j]
    return X, Win


def win_accumulate_weighted(X, p, Win, win_p, W, active=None, self_weight=None, dst_weights=None):
    """neighbor_win_accumulate(tensor, name, [self_weight, dst_weights]): as the put, but the slot
    is added to; the push-sum scalar p travels with x.  Without the arguments the topology's own
    column of weights is used, as in ``win_accumulate``.  Returns (X', p', Win', win_p')."""
    X = _f64(X).copy()
    p = _f64(p).copy()
    Win = _f64(Win).copy()
    win_p = _f64(win_p).copy()
    index = _slot_index(W)
    _, _, slot_w, self_w = window_slots(W)
    n = X.shape[0]
    for j in range(n):
        if not _is_active(active, j):
            continue
        if dst_weights is None:
            targets = {i: slot_w[e] for (i, jj), e in index.items() if jj == j}
        else:
            targets = dst_weights[j]
        for i, w in targets.items():
            e = _check_subset(index, i, j)
            Win[e, :] += w * X[j, :]
            win_p[e] += w * p[j]
    for j in range(n):
        if _is_active(active, j):
            sw = self_w[j] if self_weight is None else self_weight[j]
            X[j, :] *= sw
            p[j] *= sw
    return X, p, Win, win_p


def win_get_weighted(X, Win, W, active=None, src_weights=None):
    """neighbor_win_get(tensor, name, [src_weights]): every active agent i fetches
    src_weights[i][j] * x_j of each named in-neighbor j into its own slot for j (all in-neighbors,
    weight 1, without the argument).  Returns Win'."""
    X = _f64(X)
    Win = _f64(Win).copy()
    index = _slot_index(W)
    for i in range(X.shape[0]):
        if not _is_active(active, i):
            continue
        if src_weights is None:
            sources = {j: 1.0 for (ii, j) in index if ii == i}
        else:
            sources = src_weights[i]
        for j, w in sources.items():
            Win[_check_subset(index, i, j), :] = w * X[j, :]
    return Win


def win_update_weighted(X, Win, W, active=None, self_weight=None, src_weights=None):
    """win_update(name, [self_weight, src_weights]): every active agent i returns
    self_weight[i] x_i + sum over the named in-neighbors j of src_weights[i][j] * (slot of j); the
    window keeps its contents.  Without the arguments the topology's weights are used, as in
    ``win_update``.  Returns X'."""
    X = _f64(X).copy()
    Win = _f64(Win)
    index = _slot_index(W)
    _, _, slot_w, self_w = window_slots(W)
    out = X.copy()
    for i in range(X.shape[0]):
        if not _is_active(active, i):
            continue
        sw = self_w[i] if self_weight is None else self_weight[i]
        if src_weights is None:
            sources = {j: slot_w[e] for (ii, j), e in index.items() if ii == i}
        else:
            sources = src_weights[i]
        acc = sw * X[i, :]
        for j in sorted(sources):
            acc = acc + sources[j] * Win[_check_subset(index, i, j), :]
        out[i, :] = acc
    return out
