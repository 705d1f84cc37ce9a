// Private to libbf: host-side representation of a topology and the launch interface between the
// C-ABI layer (argument checks, dispatch) and the HIP kernels.
#ifndef BF_INTERNAL_H_
#define BF_INTERNAL_H_

#include <cstdint>
#include <list>
#include <map>
#include <mutex>
#include <vector>

#include "bf.h"

namespace bf {

// One step of a chain walk (see build_chain_plan): the row to produce, what to load next, and the
// row's at most three CSR entries as (slot, weight) in CSR order.  32 bytes: one scalar load.
struct ChainStep {
  int32_t row;        // output row of this step
  int32_t flags;      // bit 0: first row of a chain; bit 1: the chain is a cycle;
                      // bits 2-3: where the next row comes from: 0 load next_row, 1 the kept last
                      // row of the cycle, 2 the kept first row of the cycle, 3 there is none
  int32_t last_row;   // at the first step of a cycle: the cycle's last row (loaded up front)
  int32_t next_row;   // row to load when bits 2-3 are 0
  int32_t slots;      // three 4-bit codes, entry e in bits 4e..4e+3: 0 previous, 1 this row, 2 next, 15 none
  float   w[3];       // the entries' weights, in CSR order
};

// One weight matrix W^(r) as receiver-major CSR: row i lists (j, w_ij), j ascending.
struct Round {
  std::vector<int64_t> rowptr;   // n+1
  std::vector<int32_t> col;      // nnz
  std::vector<float>   wgt;      // nnz
  int32_t max_degree = 0;
  int32_t wclass = 0;            // bf_wclass_t bit mask
  std::vector<ChainStep> chain;  // n steps when the off-diagonal graph is a union of paths and cycles
  // Uniform shift round: every row is {i, (i + shift) mod n} with the same two weights (every round
  // of the one-peer exponential graph is); shift == 0 otherwise.
  int32_t shift = 0;
  float   shift_w_self = 0.0f, shift_w_peer = 0.0f;
};

// Window layout of a round (one slot per off-diagonal entry, agent 0's slots first, in CSR order)
// seen from both ends: receivers walk in_ptr, senders walk out_ptr.
struct WindowPlan {
  std::vector<int32_t> in_ptr;    // n+1: agent i owns slots in_ptr[i] .. in_ptr[i+1]-1
  std::vector<int32_t> slot_src;  // E: sender of each slot
  std::vector<float>   slot_w;    // E: w_{i,src}
  std::vector<float>   self_w;    // n: w_ii, 0 when row i has no diagonal entry
  std::vector<int32_t> out_ptr;   // n+1: sender j writes the slots out_slot[out_ptr[j] .. out_ptr[j+1]-1]
  std::vector<int32_t> out_slot;  // E, ascending within a sender
  std::vector<float>   out_w;     // E: weight of that slot
};

// Device-resident copy of all rounds, built on first use on a device.
struct DeviceCopy {
  int      device = -1;
  char*    blob = nullptr;               // round table | per round: int32 rowptr[n+1] | {int32 col, f32 w}[nnz] |
                                         // chain plan | sliced copy (headers, records of four rows side by side)
  std::vector<size_t> rowptr_off;        // byte offsets into blob, per round
  std::vector<size_t> entry_off;
  std::vector<size_t> chain_off;         // byte offset of the round's ChainStep[n], or SIZE_MAX
  float*   dense_t = nullptr;            // [round][k][i] = w_ik, n_pad x n_pad, lazily built
  int32_t  n_pad = 0;
  // Window plans, one allocation per round, built on first use: int32 in_ptr[n+1] | f32 slot_w[E] |
  // f32 self_w[n] | int32 out_ptr[n+1] | {int32 slot, f32 w} out_ent[E] | int32 slot_src[E], each
  // part 16-byte aligned.
  std::vector<char*>  win_blob;
  std::vector<size_t> win_off;           // 6 byte offsets per round
  std::vector<int32_t> win_slots;        // E per round
  unsigned int* sync = nullptr;          // arrival counter and error word of the grid-barrier kernel
  unsigned int* last_sync = nullptr;     // the words the last grid-barrier run on this device used (sync, or the
                                         // library's static scratch); not owned
};

}  // namespace bf

struct bf_topology {
  int32_t  n = 0;
  int32_t  kind = 0;
  uint64_t accepted_seed = 0;
  std::vector<bf::Round> rounds;
  std::mutex mu;                          // guards dev and two_level
  std::list<bf::DeviceCopy> dev;           // a list: pointers to entries stay valid when one is added
  // Two-level operators built from this (machine-level) topology, keyed by local_size; owned.
  std::map<int32_t, bf_topology*> two_level;
};

namespace bf {

// Host-only helpers implemented in bf_topology.cpp.
int  finalize_round(Round& r, int32_t n);           // sort check, class, max degree; returns status
void dense_transposed(const Round& r, int32_t n, int32_t n_pad, float* out);  // out[k*n_pad+i] = w_ik
void build_chain_plan(Round& r, int32_t n);          // fills r.chain when the structure allows
// Three rounds over M*local_size agents per round of the M-machine topology: machine a's local
// average into row a, the machine-level round among rows 0..M-1, row i/local_size back to agent i.
int  make_two_level(const bf_topology& machine, int32_t local_size, bf_topology** out);
void build_window_plan(const Round& r, int32_t n, WindowPlan* out);

}  // namespace bf

#endif  // BF_INTERNAL_H_
