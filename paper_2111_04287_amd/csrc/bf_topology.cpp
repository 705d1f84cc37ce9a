// Host side of libbf: topology generators, weight-matrix checks and CSR export.
// Plain C++17; nothing in this file touches the GPU, so every path here runs on a CPU-only host.
//
// Definitions follow the paper's sections "Network topology" (in-coming sets N(i), out-going sets
// M(j)) and "Weight matrix" (w_ij is nonzero only on an edge j -> i or on the diagonal; pull, push
// and standard classes).  The named graphs are the ones the benchmark configurations define.

#include <algorithm>
#include <cmath>
#include <cstring>
#include <new>
#include <utility>

#include "bf_internal.h"

namespace bf {

namespace {

constexpr double kStochasticTol = 1e-6;

// Turn per-receiver neighbor sets (self excluded) into a uniform-weight round:
// every entry of row i, the diagonal included, gets 1/(|N(i)|+1).
Round uniform_round(const std::vector<std::vector<int32_t>>& in_nbrs) {
  const int32_t n = static_cast<int32_t>(in_nbrs.size());
  Round r;
  r.rowptr.assign(n + 1, 0);
  for (int32_t i = 0; i < n; ++i) {
    std::vector<int32_t> row(in_nbrs[i]);
    row.push_back(i);
    std::sort(row.begin(), row.end());
    row.erase(std::unique(row.begin(), row.end()), row.end());
    const float w = static_cast<float>(1.0 / static_cast<double>(row.size()));
    for (int32_t j : row) {
      r.col.push_back(j);
      r.wgt.push_back(w);
    }
    r.rowptr[i + 1] = static_cast<int64_t>(r.col.size());
  }
  return r;
}

std::vector<int32_t> powers_of_two_below(int32_t n) {
  std::vector<int32_t> v;
  for (int64_t p = 1; p < n; p *= 2) v.push_back(static_cast<int32_t>(p));
  return v;
}

Round make_ring(int32_t n) {
  std::vector<std::vector<int32_t>> nb(n);
  for (int32_t i = 0; i < n; ++i) {
    nb[i].push_back((i + 1) % n);
    nb[i].push_back((i + n - 1) % n);
  }
  return uniform_round(nb);
}

Round make_exp_static(int32_t n) {
  const auto offs = powers_of_two_below(n);
  std::vector<std::vector<int32_t>> nb(n);
  for (int32_t i = 0; i < n; ++i)
    for (int32_t o : offs) {
      nb[i].push_back(static_cast<int32_t>((static_cast<int64_t>(i) + o) % n));
      nb[i].push_back(static_cast<int32_t>((static_cast<int64_t>(i) + n - o) % n));
    }
  return uniform_round(nb);
}

// Round r of the one-peer exponential-2 schedule: pull from (i + 2^(r mod R)) mod n, weights 1/2.
Round make_one_peer(int32_t n, int32_t offset) {
  Round r;
  r.rowptr.assign(n + 1, 0);
  for (int32_t i = 0; i < n; ++i) {
    const int32_t j = static_cast<int32_t>((static_cast<int64_t>(i) + offset) % n);
    if (j == i) {
      r.col.push_back(i);
      r.wgt.push_back(1.0f);
    } else {
      const int32_t lo = std::min(i, j), hi = std::max(i, j);
      r.col.push_back(lo);
      r.wgt.push_back(0.5f);
      r.col.push_back(hi);
      r.wgt.push_back(0.5f);
    }
    r.rowptr[i + 1] = static_cast<int64_t>(r.col.size());
  }
  return r;
}

struct SplitMix64 {
  uint64_t s;
  uint64_t next() {
    s += 0x9E3779B97F4A7C15ull;
    uint64_t z = s;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
  }
};

// out[j] = M(j): out_degree distinct targets other than j, by a Fisher-Yates prefix.
std::vector<std::vector<int32_t>> draw_targets(int32_t n, int32_t k, uint64_t seed) {
  SplitMix64 g{seed};
  std::vector<std::vector<int32_t>> out(n);
  std::vector<int32_t> cand;
  cand.reserve(n);
  for (int32_t j = 0; j < n; ++j) {
    cand.clear();
    for (int32_t a = 0; a < n; ++a)
      if (a != j) cand.push_back(a);
    for (int32_t t = 0; t < k; ++t) {
      const uint64_t span = static_cast<uint64_t>(n - 1 - t);
      const int32_t p = t + static_cast<int32_t>(g.next() % span);
      std::swap(cand[t], cand[p]);
    }
    out[j].assign(cand.begin(), cand.begin() + k);
  }
  return out;
}

bool reaches_all(const std::vector<std::vector<int32_t>>& adj) {
  const int32_t n = static_cast<int32_t>(adj.size());
  std::vector<char> seen(n, 0);
  std::vector<int32_t> stack{0};
  seen[0] = 1;
  int32_t count = 1;
  while (!stack.empty()) {
    const int32_t u = stack.back();
    stack.pop_back();
    for (int32_t v : adj[u])
      if (!seen[v]) {
        seen[v] = 1;
        ++count;
        stack.push_back(v);
      }
  }
  return count == n;
}

bool strongly_connected(const std::vector<std::vector<int32_t>>& out) {
  const int32_t n = static_cast<int32_t>(out.size());
  if (n == 0) return false;
  std::vector<std::vector<int32_t>> in(n);
  for (int32_t j = 0; j < n; ++j)
    for (int32_t i : out[j]) in[i].push_back(j);
  return reaches_all(out) && reaches_all(in);
}

// Column-stochastic W from out-lists: column j holds 1/(k+1) on M(j) and on the diagonal.
Round push_round_from_targets(const std::vector<std::vector<int32_t>>& out, int32_t k) {
  const int32_t n = static_cast<int32_t>(out.size());
  const float w = static_cast<float>(1.0 / (static_cast<double>(k) + 1.0));
  std::vector<std::vector<int32_t>> rows(n);
  for (int32_t j = 0; j < n; ++j) {
    rows[j].push_back(j);
    for (int32_t i : out[j]) rows[i].push_back(j);
  }
  Round r;
  r.rowptr.assign(n + 1, 0);
  for (int32_t i = 0; i < n; ++i) {
    std::sort(rows[i].begin(), rows[i].end());
    for (int32_t j : rows[i]) {
      r.col.push_back(j);
      r.wgt.push_back(w);
    }
    r.rowptr[i + 1] = static_cast<int64_t>(r.col.size());
  }
  return r;
}

}  // namespace

int finalize_round(Round& r, int32_t n) {
  if (static_cast<int32_t>(r.rowptr.size()) != n + 1 || r.rowptr[0] != 0) return BF_ERR_CSR;
  const int64_t nnz = r.rowptr[n];
  if (nnz < 0 || nnz != static_cast<int64_t>(r.col.size()) || r.col.size() != r.wgt.size() ||
      nnz > INT32_MAX)
    return BF_ERR_CSR;
  std::vector<double> rs(n, 0.0), cs(n, 0.0);
  int32_t maxdeg = 0;
  for (int32_t i = 0; i < n; ++i) {
    const int64_t b = r.rowptr[i], e = r.rowptr[i + 1];
    if (e < b) return BF_ERR_CSR;
    maxdeg = std::max<int32_t>(maxdeg, static_cast<int32_t>(e - b));
    for (int64_t p = b; p < e; ++p) {
      const int32_t j = r.col[p];
      if (j < 0 || j >= n) return BF_ERR_CSR;
      if (p > b && r.col[p - 1] >= j) return BF_ERR_CSR;      // ascending and unique
      if (!std::isfinite(r.wgt[p])) return BF_ERR_CSR;
      rs[i] += static_cast<double>(r.wgt[p]);
      cs[j] += static_cast<double>(r.wgt[p]);
    }
  }
  bool pull = true, push = true;
  for (int32_t i = 0; i < n; ++i) {
    if (std::fabs(rs[i] - 1.0) > kStochasticTol) pull = false;
    if (std::fabs(cs[i] - 1.0) > kStochasticTol) push = false;
  }
  r.max_degree = maxdeg;
  r.wclass = (pull ? BF_W_PULL : 0) | (push ? BF_W_PUSH : 0);
  if (maxdeg <= 3) build_chain_plan(r, n);
  // uniform shift round?  Two entries per row, the diagonal and (i + s) mod n, same s and the same
  // two weights (bit for bit) in every row.
  r.shift = 0;
  if (n >= 2 && nnz == 2 * static_cast<int64_t>(n)) {
    int32_t s = -1;
    float ws = 0.0f, wp = 0.0f;
    bool ok = true;
    for (int32_t i = 0; i < n && ok; ++i) {
      const int64_t b = r.rowptr[i];
      if (r.rowptr[i + 1] - b != 2) { ok = false; break; }
      const int q_self = r.col[b] == i ? 0 : (r.col[b + 1] == i ? 1 : -1);
      if (q_self < 0) { ok = false; break; }
      const int32_t j = r.col[b + 1 - q_self];
      const int32_t si = ((j - i) % n + n) % n;
      const float wsi = r.wgt[b + q_self], wpi = r.wgt[b + 1 - q_self];
      if (i == 0) { s = si; ws = wsi; wp = wpi; }
      else if (si != s || std::memcmp(&wsi, &ws, 4) != 0 || std::memcmp(&wpi, &wp, 4) != 0) ok = false;
    }
    if (ok && s > 0) { r.shift = s; r.shift_w_self = ws; r.shift_w_peer = wp; }
  }
  return BF_OK;
}

// Chain plan.  Take the undirected graph on agents with an edge {i, j} whenever w_ij or w_ji is
// stored off the diagonal.  If no agent has more than two such partners the graph is a disjoint
// union of paths and cycles (the ring; every round of the one-peer exponential schedule; any
// matching), and walking each path or cycle in order visits, for every row, its in-neighbors
// immediately before or after it.  A kernel can then stream the rows of a column strip through
// three registers (previous, current, next) instead of staging all n rows.
void build_chain_plan(Round& r, int32_t n) {
  r.chain.clear();
  std::vector<std::vector<int32_t>> adj(n);
  for (int32_t i = 0; i < n; ++i)
    for (int64_t p = r.rowptr[i]; p < r.rowptr[i + 1]; ++p) {
      const int32_t j = r.col[p];
      if (j == i) continue;
      if (std::find(adj[i].begin(), adj[i].end(), j) == adj[i].end()) adj[i].push_back(j);
      if (std::find(adj[j].begin(), adj[j].end(), i) == adj[j].end()) adj[j].push_back(i);
      if (adj[i].size() > 2 || adj[j].size() > 2) return;
    }
  std::vector<char> done(n, 0);
  std::vector<ChainStep> steps;
  steps.reserve(n);
  auto emit = [&](const std::vector<int32_t>& seq, bool cycle) {
    const int32_t L = static_cast<int32_t>(seq.size());
    for (int32_t k = 0; k < L; ++k) {
      ChainStep st{};
      st.row = seq[k];
      const int32_t pred = k > 0 ? seq[k - 1] : (cycle ? seq[L - 1] : -1);
      int32_t next_kind;
      st.next_row = -1;
      if (k + 1 < L) {
        if (cycle && k + 1 == L - 1) next_kind = 1;          // the last row was loaded at the start
        else { next_kind = 0; st.next_row = seq[k + 1]; }
      } else {
        next_kind = cycle ? 2 : 3;
      }
      st.flags = (k == 0 ? 1 : 0) | (cycle ? 2 : 0) | (next_kind << 2);
      st.last_row = (k == 0 && cycle) ? seq[L - 1] : -1;
      int32_t slots = 0xFFF;
      int e = 0;
      for (int64_t p = r.rowptr[st.row]; p < r.rowptr[st.row + 1]; ++p, ++e) {
        const int32_t j = r.col[p];
        const int32_t code = (j == st.row) ? 1 : (j == pred ? 0 : 2);
        slots = (slots & ~(0xF << (4 * e))) | (code << (4 * e));
        st.w[e] = r.wgt[p];
      }
      st.slots = slots;
      steps.push_back(st);
    }
  };
  // paths first (start from an end point), then cycles
  for (int pass = 0; pass < 2; ++pass)
    for (int32_t s0 = 0; s0 < n; ++s0) {
      if (done[s0]) continue;
      if (pass == 0 && adj[s0].size() == 2) continue;
      std::vector<int32_t> seq;
      int32_t prev = -1, cur = s0;
      while (cur >= 0 && !done[cur]) {
        done[cur] = 1;
        seq.push_back(cur);
        int32_t nxt = -1;
        for (int32_t v : adj[cur])
          if (v != prev && !done[v]) { nxt = v; break; }
        prev = cur;
        cur = nxt;
      }
      const bool cycle = pass == 1 && seq.size() >= 3;
      emit(seq, cycle);
    }
  // a row with more than three stored entries cannot occur here (self + two partners at most)
  r.chain = std::move(steps);
}

int make_two_level(const bf_topology& machine, int32_t local_size, bf_topology** out) {
  const int32_t M = machine.n, L = local_size;
  if (L < 1 || static_cast<int64_t>(M) * L > (1 << 20)) return BF_ERR_SIZE;
  const int32_t n = M * L;
  auto* t = new (std::nothrow) bf_topology;
  if (!t) return BF_ERR_NOMEM;
  t->n = n;
  t->kind = machine.kind;
  t->accepted_seed = machine.accepted_seed;
  for (const Round& mr : machine.rounds) {
    Round avg, mix, copy;
    avg.rowptr.assign(1, 0);
    mix.rowptr.assign(1, 0);
    copy.rowptr.assign(1, 0);
    const float inv = 1.0f / static_cast<float>(L);
    // The machine values live in rows 0 .. M-1 between the stages (row a for machine a), so the
    // rows that carry work are contiguous; the last stage hands row i / L to agent i.
    for (int32_t i = 0; i < n; ++i) {
      if (i < M) {
        const int32_t a = i;
        for (int32_t l = 0; l < L; ++l) { avg.col.push_back(a * L + l); avg.wgt.push_back(inv); }
        for (int64_t q = mr.rowptr[a]; q < mr.rowptr[a + 1]; ++q) {
          mix.col.push_back(mr.col[q]);
          mix.wgt.push_back(mr.wgt[q]);
        }
      }
      copy.col.push_back(i / L);                     // machine_rank = rank // local_size
      copy.wgt.push_back(1.0f);
      avg.rowptr.push_back(static_cast<int64_t>(avg.col.size()));
      mix.rowptr.push_back(static_cast<int64_t>(mix.col.size()));
      copy.rowptr.push_back(static_cast<int64_t>(copy.col.size()));
    }
    for (Round* r : {&avg, &mix, &copy}) {
      const int st = finalize_round(*r, n);
      if (st != BF_OK) { delete t; return st; }
      r->chain.clear();                              // these rounds only run inside the fused kernel
      t->rounds.push_back(std::move(*r));
    }
  }
  *out = t;
  return BF_OK;
}

void build_window_plan(const Round& r, int32_t n, WindowPlan* out) {
  WindowPlan& w = *out;
  w = WindowPlan{};
  w.in_ptr.assign(1, 0);
  w.self_w.assign(n, 0.0f);
  std::vector<int32_t> out_count(n, 0);
  for (int32_t i = 0; i < n; ++i) {
    for (int64_t q = r.rowptr[i]; q < r.rowptr[i + 1]; ++q) {
      if (r.col[q] == i) { w.self_w[i] = r.wgt[q]; continue; }
      w.slot_src.push_back(r.col[q]);
      w.slot_w.push_back(r.wgt[q]);
      ++out_count[r.col[q]];
    }
    w.in_ptr.push_back(static_cast<int32_t>(w.slot_src.size()));
  }
  const size_t E = w.slot_src.size();
  w.out_ptr.assign(n + 1, 0);
  for (int32_t j = 0; j < n; ++j) w.out_ptr[j + 1] = w.out_ptr[j] + out_count[j];
  w.out_slot.assign(E, 0);
  w.out_w.assign(E, 0.0f);
  std::vector<int32_t> fill(w.out_ptr.begin(), w.out_ptr.end() - 1);
  for (size_t e = 0; e < E; ++e) {             // ascending e, so each sender's list is ascending
    const int32_t j = w.slot_src[e];
    w.out_slot[fill[j]] = static_cast<int32_t>(e);
    w.out_w[fill[j]] = w.slot_w[e];
    ++fill[j];
  }
}

void dense_transposed(const Round& r, int32_t n, int32_t n_pad, float* out) {
  std::fill(out, out + static_cast<size_t>(n_pad) * n_pad, 0.0f);
  for (int32_t i = 0; i < n; ++i)
    for (int64_t p = r.rowptr[i]; p < r.rowptr[i + 1]; ++p)
      out[static_cast<size_t>(r.col[p]) * n_pad + i] = r.wgt[p];
}

}  // namespace bf

using bf::Round;

namespace {

int slice_index(const bf_topology_t* t, int32_t round) {
  return static_cast<int>(round % static_cast<int32_t>(t->rounds.size()));
}

int check_class(const Round& r, int32_t required) {
  if ((required & ~3) != 0) return BF_ERR_KIND;
  return ((r.wclass & required) == required) ? BF_OK : BF_ERR_NOT_STOCHASTIC;
}

}  // namespace

extern "C" {

int bf_topology_create(bf_topology_t** out, bf_topo_kind_t kind, int32_t n, const bf_topo_params_t* p) {
  if (!out) return BF_ERR_NULL;
  *out = nullptr;
  if (n < 1 || n > (1 << 20)) return BF_ERR_SIZE;
  bf_topology_t* t = new (std::nothrow) bf_topology_t();
  if (!t) return BF_ERR_NOMEM;
  t->n = n;
  t->kind = static_cast<int32_t>(kind);
  t->accepted_seed = p ? p->seed : 0;
  int st = BF_OK;
  try {
    switch (kind) {
      case BF_RING:
        t->rounds.push_back(bf::make_ring(n));
        break;
      case BF_EXP_STATIC:
        t->rounds.push_back(bf::make_exp_static(n));
        break;
      case BF_EXP2_ONE_PEER: {
        const auto offs = bf::powers_of_two_below(n);
        if (offs.empty()) t->rounds.push_back(bf::make_one_peer(n, 0));
        for (int32_t o : offs) t->rounds.push_back(bf::make_one_peer(n, o));
        break;
      }
      case BF_RANDOM_DIRECTED: {
        if (!p) { st = BF_ERR_NULL; break; }
        if (p->out_degree < 0 || p->out_degree > n - 1) { st = BF_ERR_SIZE; break; }
        const int tries = p->require_strongly_connected ? 10000 : 1;
        st = BF_ERR_NOT_CONNECTED;
        for (int a = 0; a < tries; ++a) {
          const uint64_t s = p->seed + static_cast<uint64_t>(a);
          auto targets = bf::draw_targets(n, p->out_degree, s);
          if (!p->require_strongly_connected || bf::strongly_connected(targets)) {
            t->rounds.push_back(bf::push_round_from_targets(targets, p->out_degree));
            t->accepted_seed = s;
            st = BF_OK;
            break;
          }
        }
        break;
      }
      case BF_CSR_USER: {
        if (!p || !p->rowptr || !p->col || !p->wgt) { st = BF_ERR_NULL; break; }
        const int32_t R = p->rounds == 0 ? 1 : p->rounds;
        if (R < 1 || R > 65536) { st = BF_ERR_SIZE; break; }
        for (int32_t r = 0; r < R && st == BF_OK; ++r) {
          const int64_t* rp = p->rowptr + static_cast<size_t>(r) * (n + 1);
          Round rd;
          rd.rowptr.resize(n + 1);
          const int64_t base = rp[0];
          if (base < 0) { st = BF_ERR_CSR; break; }
          for (int32_t i = 0; i <= n; ++i) {
            if (rp[i] < base || (i > 0 && rp[i] < rp[i - 1]) || rp[i] - base > INT32_MAX) { st = BF_ERR_CSR; break; }
            rd.rowptr[i] = rp[i] - base;
          }
          if (st != BF_OK) break;
          rd.col.assign(p->col + base, p->col + rp[n]);
          rd.wgt.assign(p->wgt + base, p->wgt + rp[n]);
          t->rounds.push_back(std::move(rd));
        }
        break;
      }
      case BF_DENSE_USER: {
        if (!p || !p->dense_w) { st = BF_ERR_NULL; break; }
        if (n > 4096) { st = BF_ERR_SIZE; break; }
        const int32_t R = p->rounds == 0 ? 1 : p->rounds;
        if (R < 1 || R > 65536) { st = BF_ERR_SIZE; break; }
        for (int32_t r = 0; r < R; ++r) {
          const float* D = p->dense_w + static_cast<size_t>(r) * n * n;
          Round rd;
          rd.rowptr.assign(n + 1, 0);
          for (int32_t i = 0; i < n; ++i) {
            for (int32_t j = 0; j < n; ++j) {
              const float w = D[static_cast<size_t>(i) * n + j];
              if (w != 0.0f || i == j) {     // w != 0 is also true for NaN: caught by finalize
                rd.col.push_back(j);
                rd.wgt.push_back(w);
              }
            }
            rd.rowptr[i + 1] = static_cast<int64_t>(rd.col.size());
          }
          t->rounds.push_back(std::move(rd));
        }
        break;
      }
      default:
        st = BF_ERR_KIND;
    }
    for (auto& r : t->rounds) {
      if (st != BF_OK) break;
      st = bf::finalize_round(r, n);
      if (st == BF_OK && p && (kind == BF_CSR_USER || kind == BF_DENSE_USER))
        st = check_class(r, p->require_class);
    }
  } catch (const std::bad_alloc&) {
    st = BF_ERR_NOMEM;
  }
  if (st != BF_OK) {
    delete t;
    return st;
  }
  *out = t;
  return BF_OK;
}

int bf_topology_create_push_pull(bf_topology_t** out, int32_t n, const float* self_weight,
                                 const int64_t* src_rowptr, const int32_t* src_rank, const float* src_weight,
                                 const int64_t* dst_rowptr, const int32_t* dst_rank, const float* dst_weight) {
  if (!out) return BF_ERR_NULL;
  *out = nullptr;
  if (!self_weight || !src_rowptr || !src_rank || !dst_rowptr || !dst_rank) return BF_ERR_NULL;
  if (n < 1 || n > (1 << 20)) return BF_ERR_SIZE;
  try {
    // Structural checks of both views.
    for (int pass = 0; pass < 2; ++pass) {
      const int64_t* rp = pass ? dst_rowptr : src_rowptr;
      const int32_t* rk = pass ? dst_rank : src_rank;
      if (rp[0] != 0) return BF_ERR_CSR;
      for (int32_t i = 0; i < n; ++i) {
        if (rp[i + 1] < rp[i]) return BF_ERR_CSR;
        for (int64_t q = rp[i]; q < rp[i + 1]; ++q) {
          if (rk[q] < 0 || rk[q] >= n || rk[q] == i) return BF_ERR_CSR;
          if (q > rp[i] && rk[q - 1] >= rk[q]) return BF_ERR_CSR;
        }
      }
    }
    if (src_rowptr[n] != dst_rowptr[n]) return BF_ERR_TOPO_MISMATCH;
    // The topology check: receiver i lists j as a source  <=>  sender j lists i as a destination.
    Round rd;
    rd.rowptr.assign(n + 1, 0);
    for (int32_t i = 0; i < n; ++i) {
      bool self_done = false;
      auto push_self = [&]() {
        rd.col.push_back(i);
        rd.wgt.push_back(self_weight[i]);
        self_done = true;
      };
      for (int64_t q = src_rowptr[i]; q < src_rowptr[i + 1]; ++q) {
        const int32_t j = src_rank[q];
        const int32_t* b = dst_rank + dst_rowptr[j];
        const int32_t* e = dst_rank + dst_rowptr[j + 1];
        const int32_t* hit = std::lower_bound(b, e, i);
        if (hit == e || *hit != i) return BF_ERR_TOPO_MISMATCH;
        const float rr = src_weight ? src_weight[q] : 1.0f;
        const float ss = dst_weight ? dst_weight[hit - dst_rank] : 1.0f;
        if (!self_done && j > i) push_self();
        rd.col.push_back(j);
        rd.wgt.push_back(rr * ss);
      }
      if (!self_done) push_self();
      rd.rowptr[i + 1] = static_cast<int64_t>(rd.col.size());
    }
    // Equal edge counts plus src-edge-in-dst for every edge means the two edge sets coincide.
    bf_topology_t* t = new (std::nothrow) bf_topology_t();
    if (!t) return BF_ERR_NOMEM;
    t->n = n;
    t->kind = BF_CSR_USER;
    const int st = bf::finalize_round(rd, n);
    if (st != BF_OK) {
      delete t;
      return st;
    }
    t->rounds.push_back(std::move(rd));
    *out = t;
    return BF_OK;
  } catch (const std::bad_alloc&) {
    return BF_ERR_NOMEM;
  }
}

int32_t bf_topology_n(const bf_topology_t* t) { return t ? t->n : BF_ERR_NULL; }

int32_t bf_topology_rounds(const bf_topology_t* t) {
  return t ? static_cast<int32_t>(t->rounds.size()) : BF_ERR_NULL;
}

int64_t bf_topology_nnz(const bf_topology_t* t, int32_t round) {
  if (!t) return BF_ERR_NULL;
  if (round < 0) return BF_ERR_ROUND;
  return t->rounds[slice_index(t, round)].rowptr[t->n];
}

int32_t bf_topology_max_degree(const bf_topology_t* t, int32_t round) {
  if (!t) return BF_ERR_NULL;
  if (round < 0) return BF_ERR_ROUND;
  return t->rounds[slice_index(t, round)].max_degree;
}

int32_t bf_topology_class(const bf_topology_t* t, int32_t round) {
  if (!t) return BF_ERR_NULL;
  if (round < 0) return BF_ERR_ROUND;
  return t->rounds[slice_index(t, round)].wclass;
}

int32_t bf_topology_chain_plan(const bf_topology_t* t, int32_t round, int32_t* steps) {
  if (!t) return BF_ERR_NULL;
  if (round < 0) return BF_ERR_ROUND;
  const Round& r = t->rounds[slice_index(t, round)];
  if (r.chain.empty()) return 0;
  static_assert(sizeof(bf::ChainStep) == 32, "ChainStep is exported as eight 32-bit words");
  if (steps) std::memcpy(steps, r.chain.data(), r.chain.size() * sizeof(bf::ChainStep));
  return t->n;
}

int bf_topology_export_csr(const bf_topology_t* t, int32_t round, int64_t* rowptr, int32_t* col,
                           float* wgt, uint64_t* accepted_seed) {
  if (!t) return BF_ERR_NULL;
  if (round < 0) return BF_ERR_ROUND;
  const Round& r = t->rounds[slice_index(t, round)];
  if (rowptr) std::memcpy(rowptr, r.rowptr.data(), r.rowptr.size() * sizeof(int64_t));
  if (col) std::memcpy(col, r.col.data(), r.col.size() * sizeof(int32_t));
  if (wgt) std::memcpy(wgt, r.wgt.data(), r.wgt.size() * sizeof(float));
  if (accepted_seed) *accepted_seed = t->accepted_seed;
  return BF_OK;
}

int64_t bf_topology_window_slots(const bf_topology_t* t, int32_t round) {
  if (!t) return BF_ERR_NULL;
  if (round < 0) return BF_ERR_ROUND;
  const int k = slice_index(t, round);
  const Round& r = t->rounds[k];
  int64_t diag = 0;
  for (int32_t i = 0; i < t->n; ++i)
    for (int64_t q = r.rowptr[i]; q < r.rowptr[i + 1]; ++q) diag += r.col[q] == i;
  return r.rowptr[t->n] - diag;
}

int bf_topology_export_window(const bf_topology_t* t, int32_t round, int64_t* slot_rowptr, int32_t* slot_src,
                              float* slot_weight, float* self_weight) {
  if (!t) return BF_ERR_NULL;
  if (round < 0) return BF_ERR_ROUND;
  const int k = slice_index(t, round);
  bf::WindowPlan w;
  bf::build_window_plan(t->rounds[k], t->n, &w);
  if (slot_rowptr) for (int32_t i = 0; i <= t->n; ++i) slot_rowptr[i] = w.in_ptr[i];
  if (slot_src) std::copy(w.slot_src.begin(), w.slot_src.end(), slot_src);
  if (slot_weight) std::copy(w.slot_w.begin(), w.slot_w.end(), slot_weight);
  if (self_weight) std::copy(w.self_w.begin(), w.self_w.end(), self_weight);
  return BF_OK;
}

int64_t bf_recommended_ld(int64_t d, bf_dtype_t dt) {
  if (dt != BF_F32 && dt != BF_BF16) return BF_ERR_KIND;
  if (d < 0 || d > (int64_t{1} << 40)) return BF_ERR_SIZE;
  const int64_t eb = dt == BF_F32 ? 4 : 2;
  const int64_t pitch = (d * eb + 127) / 128 * 128 + 4224;
  return pitch / eb;
}

int64_t bf_blocked_elems(int32_t n, int64_t d, int64_t block) {
  if (n < 1 || d < 0 || d > (int64_t{1} << 40) || block < 64 || block > (int64_t{1} << 20) || (block & (block - 1)) != 0)
    return BF_ERR_SIZE;
  return (d + block - 1) / block * block * n;
}

int64_t bf_recommended_block(const bf_topology_t* t, int64_t d, bf_dtype_t dt) {
  if (!t) return BF_ERR_NULL;
  if (dt != BF_F32 && dt != BF_BF16) return BF_ERR_KIND;
  if (d < 0 || d > (int64_t{1} << 40)) return BF_ERR_SIZE;
  const int64_t n = t->n;
  // Measured on MI355X (block widths 128 .. 2^20; n = 32 bf16 with fp32 momentum, n = 64 and
  // n = 128 fp32): bandwidth peaks where a block of fp32 values is about 4 MB -- 16384 columns at
  // n = 64, 8192 at n = 128; n = 32 is flat between 8192 and 16384 -- and falls off on both sides
  // (narrower: fewer neighbouring tiles share a block row; wider: the rows of a block drift apart
  // like agent-major rows).
  // bf16 matrices usually come with an fp32 state matrix of the same shape (momentum), which doubles
  // the bytes of a block: 8192 columns measure best there (n = 32: 6.27 TB/s against 6.20 at 16384).
  int64_t b = dt == BF_BF16 ? 8192 : 16384;
  while (b > 2048 && b * n > (int64_t{1} << 20)) b >>= 1;
  // More agents than give the pipelined kernel 128-column tiles (two n x 128 fp32 tiles in 160 KB
  // of LDS): rounds that are unions of paths and cycles go to the row-streaming kernel, whose
  // workgroups sweep 4096 to 16384 columns of a row at a time; it measures best on blocks of 65536
  // (n = 256 fp32: 5.88 TB/s against 5.55 agent-major and 4.9 on blocks of 4096).
  if (2 * n * 128 * 4 > 160 * 1024) {
    bool chains = !t->rounds.empty();
    for (const auto& r : t->rounds) chains = chains && !r.chain.empty();
    if (chains) b = 65536;
  }
  // a matrix narrower than that is one block
  while (b > 64 && b / 2 >= d) b >>= 1;
  return b;
}

const char* bf_strerror(int code) {
  switch (code) {
    case BF_OK: return "ok";
    case BF_ERR_NULL: return "required pointer is NULL";
    case BF_ERR_SIZE: return "size argument out of range";
    case BF_ERR_ALIGN: return "pointer or row pitch not 16-byte aligned";
    case BF_ERR_ALIAS: return "operands overlap (only exact in-place X_in == X_out is allowed)";
    case BF_ERR_KIND: return "unknown topology kind, dtype, mode or class";
    case BF_ERR_ROUND: return "negative round index";
    case BF_ERR_NOT_STOCHASTIC: return "weight matrix is not in the required pull/push/standard class";
    case BF_ERR_NOT_CONNECTED: return "graph is not strongly connected";
    case BF_ERR_CSR: return "malformed CSR or neighbor list";
    case BF_ERR_TOPO_MISMATCH: return "source and destination lists describe different edges";
    case BF_ERR_UNSUPPORTED: return "no kernel for this shape (n too large for the tile kernels, or tuning override not honourable)";
    case BF_ERR_HIP: return "HIP runtime call failed";
    case BF_ERR_NOMEM: return "host allocation failed";
    default: return "unknown status";
  }
}

}  // extern "C"
