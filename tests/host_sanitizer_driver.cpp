// host-only sanitizer run of the topology code: every generator, the validators, plans and exports
#include <cstdio>
#include <cstdlib>
#include <vector>
#include "bf_internal.h"
static void free_topo(bf_topology_t* t) { for (auto& kv : t->two_level) free_topo(kv.second); delete t; }
int main() {
  int fails = 0;
  for (int n : {1, 2, 3, 5, 16, 37, 64, 100, 256, 641}) {
    for (int kind : {BF_RING, BF_EXP_STATIC, BF_EXP2_ONE_PEER, BF_RANDOM_DIRECTED}) {
      bf_topo_params_t p{};
      p.out_degree = n > 4 ? 4 : (n > 1 ? n - 1 : 0);
      p.seed = 401; p.require_strongly_connected = 1;
      bf_topology_t* t = nullptr;
      int rc = bf_topology_create(&t, static_cast<bf_topo_kind_t>(kind), n, &p);
      if (rc != BF_OK) {
        // a random directed graph needs two agents, and may find no strongly connected draw at all
        if (kind != BF_RANDOM_DIRECTED) { printf("create kind %d n %d -> %d\n", kind, n, rc); ++fails; }
        continue;
      }
      for (int r = 0; r < bf_topology_rounds(t); ++r) {
        const int64_t nnz = bf_topology_nnz(t, r);
        std::vector<int64_t> rp(n + 1); std::vector<int32_t> col(nnz); std::vector<float> w(nnz); uint64_t seed;
        if (bf_topology_export_csr(t, r, rp.data(), col.data(), w.data(), &seed) != BF_OK) ++fails;
        std::vector<int32_t> steps(8 * n);
        bf_topology_chain_plan(t, r, steps.data());
        const int64_t E = bf_topology_window_slots(t, r);
        std::vector<int64_t> srp(n + 1); std::vector<int32_t> src(E > 0 ? E : 1); std::vector<float> sw(E > 0 ? E : 1), self(n);
        if (bf_topology_export_window(t, r, srp.data(), src.data(), sw.data(), self.data()) != BF_OK) ++fails;
        if (srp[n] != E) ++fails;
        // user CSR round trip
        bf_topo_params_t q{}; q.rounds = 1; q.rowptr = rp.data(); q.col = col.data(); q.wgt = w.data();
        bf_topology_t* u = nullptr;
        if (bf_topology_create(&u, BF_CSR_USER, n, &q) != BF_OK) ++fails; else free_topo(u);
      }
      for (int L : {1, 3, 8}) {
        bf_topology_t* two = nullptr;
        if (bf::make_two_level(*t, L, &two) != BF_OK) ++fails; else free_topo(two);
      }
      if (n <= 64) {
        std::vector<float> dense(static_cast<size_t>(n) * n, 1.0f / n);
        bf_topo_params_t q{}; q.rounds = 1; q.dense_w = dense.data();
        bf_topology_t* u = nullptr;
        if (bf_topology_create(&u, BF_DENSE_USER, n, &q) != BF_OK) ++fails; else free_topo(u);
      }
      free_topo(t);
    }
  }
  // malformed inputs must be rejected, not crash
  {
    int64_t rp[4] = {0, 2, 1, 3}; int32_t col[3] = {0, 5, -1}; float w[3] = {1.f, 1.f, 1.f};
    bf_topo_params_t q{}; q.rounds = 1; q.rowptr = rp; q.col = col; q.wgt = w;
    bf_topology_t* u = nullptr;
    if (bf_topology_create(&u, BF_CSR_USER, 3, &q) == BF_OK) { ++fails; free_topo(u); }
  }
  printf("host sanitizer driver: %d failures\n", fails);
  return fails != 0;
}
