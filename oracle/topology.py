"""Oracle topologies: weight matrices as dictionaries of in-neighbor lists.

TEST INFRASTRUCTURE ONLY -- see the package docstring.

``W[i]`` is the list ``[(j, w_ij), ...]`` over ``j`` in N(i) united with {i},
where N(i) = {j : (j, i) is an edge} is the in-coming neighbor set
(eq. in-neighbor) and ``w_ij`` multiplies data sent from j to i (eq. wij).
The out-going sets M(j) = {i : (j, i) is an edge} (eq. out-neighbor) are
obtained by ``out_lists``.

The paper names its built-in graphs (ring, static exponential, one-peer
exponential) without defining them; the definitions here are the ones the
benchmark configurations state:

* ring: self and both ring neighbors, equal weights;
* static exponential: neighbors i +/- 2^k (mod n) for every 2^k < n, taken as a
  set (for n a power of two +n/2 and -n/2 coincide), equal weights over the set
  plus self;
* one-peer exponential-2, round r: agent i averages 1/2, 1/2 with agent
  (i + 2^(r mod R)) mod n, R = number of powers of two below n;
* random directed push graph: every sender j draws ``out_degree`` distinct
  targets other than itself; column j of W holds 1/(out_degree+1) on the
  targets and on the diagonal, the sender-side rule of the push-sum listing
  (weights 1/(outdegree+1)).
"""

from collections import deque

_MASK64 = (1 << 64) - 1


def _dedup_sorted(items):
    return sorted(set(items))


def uniform_from_neighbor_sets(nbrs):
    """Equal weight 1/(|N(i)|+1) on self and every in-neighbor."""
    W = {}
    for i, ns in nbrs.items():
        ns = [j for j in _dedup_sorted(ns) if j != i]
        w = 1.0 / (len(ns) + 1)
        W[i] = [(j, w) for j in sorted(ns + [i])]
    return W


def ring(n):
    return uniform_from_neighbor_sets(
        {i: [(i - 1) % n, (i + 1) % n] for i in range(n)})


def powers_of_two_below(n):
    out, p = [], 1
    while p < n:
        out.append(p)
        p *= 2
    return out


def static_exponential(n):
    offs = powers_of_two_below(n)
    return uniform_from_neighbor_sets(
        {i: [(i + o) % n for o in offs] + [(i - o) % n for o in offs]
         for i in range(n)})


def one_peer_rounds(n):
    return max(1, len(powers_of_two_below(n)))


def one_peer_exponential(n, r):
    offs = powers_of_two_below(n)
    if not offs:
        return {0: [(0, 1.0)]}
    o = offs[r % len(offs)]
    W = {}
    for i in range(n):
        j = (i + o) % n
        W[i] = [(i, 1.0)] if j == i else sorted([(i, 0.5), (j, 0.5)])
    return W


class SplitMix64:
    """The splitmix64 sequence: a 64-bit counter advanced by the golden-ratio
    increment and passed through two xor-shift-multiply rounds."""

    def __init__(self, seed):
        self.s = seed & _MASK64

    def next(self):
        self.s = (self.s + 0x9E3779B97F4A7C15) & _MASK64
        z = self.s
        z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _MASK64
        z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _MASK64
        return z ^ (z >> 31)


def draw_out_targets(n, out_degree, seed):
    """One draw of the random directed graph: targets[j] = M(j).

    For sender j = 0..n-1 in order: list the other n-1 agents in increasing
    order and run ``out_degree`` steps of a Fisher-Yates shuffle, step t
    swapping position t with position t + (u mod (n-1-t)), u the next
    splitmix64 output; the first ``out_degree`` entries are the targets.
    """
    if not (0 <= out_degree <= n - 1):
        raise ValueError("out_degree must lie in [0, n-1]")
    g = SplitMix64(seed)
    targets = {}
    for j in range(n):
        cand = [a for a in range(n) if a != j]
        for t in range(out_degree):
            p = t + g.next() % (n - 1 - t)
            cand[t], cand[p] = cand[p], cand[t]
        targets[j] = cand[:out_degree]
    return targets


def in_lists_from_out_lists(out):
    """N(i) from M(j): i in M(j)  <=>  j in N(i)."""
    n = len(out)
    inn = {i: [] for i in range(n)}
    for j in range(n):
        for i in out[j]:
            inn[i].append(j)
    return {i: sorted(v) for i, v in inn.items()}


def out_lists(W):
    """M(j) of the graph a weight matrix induces (edge (j,i) iff w_ij != 0, i != j)."""
    out = {j: [] for j in W}
    for i, row in W.items():
        for j, w in row:
            if j != i and w != 0.0:
                out[j].append(i)
    return {j: sorted(v) for j, v in out.items()}


def in_lists(W):
    return {i: sorted(j for j, w in row if j != i and w != 0.0)
            for i, row in W.items()}


def _reaches_all(adj, n):
    seen = [False] * n
    seen[0] = True
    q = deque([0])
    while q:
        u = q.popleft()
        for v in adj[u]:
            if not seen[v]:
                seen[v] = True
                q.append(v)
    return all(seen)


def is_strongly_connected(out):
    n = len(out)
    if n == 0:
        return False
    return _reaches_all(out, n) and _reaches_all(in_lists_from_out_lists(out), n)


def random_directed_push(n, out_degree, seed, require_strongly_connected=True,
                         max_tries=10000):
    """Column-stochastic W of a random out-regular digraph.

    Seeds seed, seed+1, ... are tried in turn until the draw is strongly
    connected (push-sum reaches the average only on such graphs).  Returns
    (W, accepted_seed).
    """
    for a in range(max_tries):
        s = (seed + a) & _MASK64
        out = draw_out_targets(n, out_degree, s)
        if not require_strongly_connected or is_strongly_connected(out):
            w = 1.0 / (out_degree + 1)
            W = {i: [(i, w)] for i in range(n)}
            for j in range(n):
                for i in out[j]:
                    W[i].append((j, w))
            return {i: sorted(r) for i, r in W.items()}, s
    raise RuntimeError("no strongly connected draw found")


def from_dense(Wd, drop_zeros=True):
    """Dictionary form of a dense n x n array (entry [i][j] = w_ij)."""
    n = len(Wd)
    return {i: [(j, float(Wd[i][j])) for j in range(n)
                if (not drop_zeros) or Wd[i][j] != 0.0] for i in range(n)}


def to_dense(W):
    import numpy as np
    n = len(W)
    D = np.zeros((n, n), dtype=np.float64)
    for i, row in W.items():
        for j, w in row:
            D[i, j] += w
    return D


def row_sums(W):
    return [sum(w for _, w in W[i]) for i in range(len(W))]


def col_sums(W):
    s = [0.0] * len(W)
    for i, row in W.items():
        for j, w in row:
            s[j] += w
    return s


def from_csr(rowptr, col, wgt):
    """Dictionary form of a receiver-major CSR triple (used to feed the oracle
    the library's fp32 weight values: W is data on both sides)."""
    n = len(rowptr) - 1
    return {i: [(int(col[p]), float(wgt[p])) for p in range(int(rowptr[i]), int(rowptr[i + 1]))]
            for i in range(n)}
