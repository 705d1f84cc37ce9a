/*
 * bf.h -- C ABI of libbf: decentralized neighbor averaging for n simulated agents on one MI355X.
 *
 * The n agents of the paper's problem statement (eq. dist-opt: min (1/n) sum_i f_i(x)) live on one
 * GPU.  Agent i's vector x_i is row i of an agent-major matrix X (n x d) in device memory, and the
 * paper's "communication" -- partial averaging over a topology with weight matrix W -- becomes a
 * sparse gather-reduce over the rows of X.
 *
 * Conventions shared by every entry point
 *   - w_ij scales the copy of x_j that flows from agent j to agent i (eq. wij).  A topology stores,
 *     per round, the in-neighbor lists N(i) united with {i} as a receiver-major CSR: row i of the
 *     CSR lists (j, w_ij) with j ascending.
 *   - Matrices are agent-major.  Row i starts at base + i*ld*s bytes, s = 4 (BF_F32) or 2 (BF_BF16);
 *     ld >= d is the leading dimension in elements.  base and ld*s must be multiples of 16 bytes.
 *     Columns d..ld-1 of a row are never written.  Kernels read whole 16-byte vectors, so of the
 *     padding they may read (and discard) what shares a 16-byte vector with a column below d: a
 *     matrix must be readable up to (n-1)*ld*s + d*s rounded up to 16 bytes, which is also the
 *     extent the overlap checks use.
 *   - The column-block layout is the second layout of a matrix, for the calls that say they accept
 *     it: ld = BF_LD_BLOCKED(B), B a power of two in [64, 2^20].  The d columns are cut into
 *     ceil(d/B) blocks of B columns; block k is an n x B row-major matrix at element k*n*B, so
 *     column c of agent i is element (c/B)*n*B + i*B + c%B, and a matrix has bf_blocked_elems(n, d,
 *     B) elements, all of which the kernels may read; the columns at or past d of the last block are
 *     never written (bf_blocked_pack zero-fills them).  Every matrix of one call (X_in, X_out, G,
 *     M, Y, ...) has the same layout.  Why it exists: a column tile of the agent-major layout is n
 *     row segments in n distant places of every matrix (n x 3 streams and as many memory pages per
 *     tile with gradient and momentum), a tile of this layout is one contiguous piece per matrix.
 *     Measured on the n = 32, d = 25.5 M momentum step with blocks of 8192 columns: 6.3 TB/s
 *     against 5.06 TB/s agent-major.  A call that does not accept the layout answers
 *     BF_ERR_UNSUPPORTED.
 *   - Pointers named X*, G, M, Y, A, b, C, E, w_in/w_out and stats are DEVICE pointers owned by the
 *     caller; the library never allocates, frees or resizes them.  Pointers inside
 *     bf_topo_params_t and the export arrays are HOST pointers.
 *   - hip_stream is a hipStream_t passed as void* (NULL = the null stream).  Compute calls enqueue
 *     on it and return at once: they are the paper's nonblocking primitive, and waiting on the
 *     stream is its wait(handle).  No call synchronizes the device or reads results back.
 *   - X_out may be exactly X_in (in place) or must not overlap it at all; any partial overlap, or an
 *     output overlapping another operand, is BF_ERR_ALIAS.  Two calls that touch the same buffers
 *     on different streams race; ordering them is the caller's job.
 *   - `round` selects the weight matrix W^(round mod rounds) of a time-varying topology (the paper
 *     passes per-iteration weights to neighbor_allreduce); static topologies have rounds == 1.
 *   - Every function returns BF_OK (0) or a negative bf_status_t.  All argument checks happen on the
 *     host before anything is launched, so no error path touches the device.  Nothing throws or
 *     aborts across this boundary.
 */
#ifndef BF_H_
#define BF_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  BF_OK = 0,
  BF_ERR_NULL = -1,            /* a required pointer is NULL                                   */
  BF_ERR_SIZE = -2,            /* n, d, ld, m, out_degree or rounds out of range               */
  BF_ERR_ALIGN = -3,           /* base pointer or row pitch not a multiple of 16 bytes         */
  BF_ERR_ALIAS = -4,           /* operands overlap in a way other than exact in-place          */
  BF_ERR_KIND = -5,            /* unknown topology kind / dtype / mode                         */
  BF_ERR_ROUND = -6,           /* negative round index                                         */
  BF_ERR_NOT_STOCHASTIC = -7,  /* required row / column sums differ from 1 by more than 1e-6   */
  BF_ERR_NOT_CONNECTED = -8,   /* no strongly connected draw found / user graph not connected  */
  BF_ERR_CSR = -9,             /* malformed CSR: bad rowptr, column out of range, unsorted or
                                  duplicate columns, non-finite weight                        */
  BF_ERR_TOPO_MISMATCH = -10,  /* a sender's dst list and a receiver's src list disagree       */
  BF_ERR_UNSUPPORTED = -11,    /* valid request this build has no kernel for (says which)      */
  BF_ERR_HIP = -12,            /* a HIP runtime call failed; bf_last_hip_error() has the code  */
  BF_ERR_NOMEM = -13           /* host allocation failed                                       */
} bf_status_t;

typedef enum {
  BF_RING = 0,             /* self and both ring neighbors, equal weights (1/3 for n >= 3)       */
  BF_EXP_STATIC = 1,       /* neighbors i +/- 2^k mod n for every 2^k < n, as a set; equal weights
                              over the set plus self (1/12 at n = 64, 1/10 at n = 32)            */
  BF_EXP2_ONE_PEER = 2,    /* round r: x_i <- x_i/2 + x_((i + 2^(r mod R)) mod n)/2,
                              R = number of powers of two below n (log2 n for n = 2^p)           */
  BF_RANDOM_DIRECTED = 3,  /* push graph: each sender draws out_degree distinct targets != self;
                              column j holds 1/(out_degree+1) on targets and diagonal            */
  BF_CSR_USER = 4,         /* caller supplies receiver-major CSR slices, one per round           */
  BF_DENSE_USER = 5        /* caller supplies dense row-major n x n matrices, one per round      */
} bf_topo_kind_t;

typedef enum { BF_F32 = 0, BF_BF16 = 1 } bf_dtype_t;
typedef enum { BF_ATC = 0, BF_AWC = 1 } bf_mode_t;

/* Classes of weight matrix (section "Weight matrix"): pull = rows sum to 1, push = columns sum to
 * 1, standard = both.  Bit mask: bit 0 = pull, bit 1 = push. */
typedef enum { BF_W_ANY = 0, BF_W_PULL = 1, BF_W_PUSH = 2, BF_W_STANDARD = 3 } bf_wclass_t;

typedef struct {
  /* BF_RANDOM_DIRECTED */
  int32_t  out_degree;                  /* 0 <= out_degree <= n-1                                */
  int32_t  require_strongly_connected;  /* nonzero: try seed, seed+1, ... until strongly connected
                                           (at most 10000 tries, else BF_ERR_NOT_CONNECTED)      */
  uint64_t seed;
  /* BF_CSR_USER / BF_DENSE_USER */
  int32_t  rounds;                      /* number of slices, >= 1 (0 is read as 1)               */
  int32_t  require_class;               /* bf_wclass_t every slice must satisfy (the paper's
                                           topology check, done once at create time)             */
  const int64_t* rowptr;                /* rounds*(n+1) entries; slice r uses rowptr[r*(n+1)..],
                                           offsets are absolute positions in col/wgt             */
  const int32_t* col;                   /* ascending and unique within a row; a row may be empty  */
  const float*   wgt;
  const float*   dense_w;               /* rounds*n*n, entry [r][i][j] = w_ij of round r         */
} bf_topo_params_t;

typedef struct bf_topology bf_topology_t;   /* opaque; immutable after creation; may be shared by
                                               streams and threads                               */

/* Build a topology and its weights (the paper's set_topology(graph), sections "Network topology",
 * "Weight matrix" and "Static topology").  `p` may be NULL for the first three kinds.  The random
 * directed draw is specified as: splitmix64 seeded with the attempt's seed; for sender j = 0..n-1,
 * list the other agents ascending and run out_degree Fisher-Yates steps, step t swapping slot t
 * with slot t + (next() mod (n-1-t)); the first out_degree slots are M(j).
 * On success *out owns host memory (and, lazily, a few KB of device memory per device used). */
int bf_topology_create(bf_topology_t** out, bf_topo_kind_t kind, int32_t n, const bf_topo_params_t* p);

/* Build a one-round topology from each agent's local view (section "Push- and pull-style
 * communication over time-varying topology", eqs. dyn-push-comm / dyn-pull-comm): agent i passes
 * self_weight[i] = w_ii, its source list (j, r_ij) over N(i) and its destination list (i', s_i'i)
 * over M(i), both as CSR with ascending ranks.  A NULL src_weight means r = 1, a NULL dst_weight
 * means s = 1 (pure push / pure pull).  The resulting weight is w_ij = r_ij * s_ij.  The lists are
 * cross-checked: edge (j -> i) must appear in i's sources and in j's destinations, else
 * BF_ERR_TOPO_MISMATCH (the paper's automatic topology check, which exists so that an unmatched
 * send/receive pair is reported instead of hanging). */
int bf_topology_create_push_pull(bf_topology_t** out, int32_t n, const float* self_weight,
                                 const int64_t* src_rowptr, const int32_t* src_rank, const float* src_weight,
                                 const int64_t* dst_rowptr, const int32_t* dst_rank, const float* dst_weight);

int     bf_topology_destroy(bf_topology_t* t);          /* NULL is accepted                      */
int32_t bf_topology_n(const bf_topology_t* t);          /* number of agents, or negative status  */
int32_t bf_topology_rounds(const bf_topology_t* t);     /* 1 for static graphs                   */
int64_t bf_topology_nnz(const bf_topology_t* t, int32_t round);       /* self loops included     */
int32_t bf_topology_max_degree(const bf_topology_t* t, int32_t round);/* longest CSR row         */
int32_t bf_topology_class(const bf_topology_t* t, int32_t round);     /* bf_wclass_t bit mask,
                                                            sums tested to 1e-6 in fp64          */
/* Copy round's CSR to caller-sized host arrays: rowptr[n+1] (starting at 0), col[nnz], wgt[nnz].
 * Any output pointer may be NULL.  accepted_seed receives the seed a random draw settled on
 * (the params seed for other kinds).  The fp32 weights exported here are the exact values the
 * kernels multiply by. */
int bf_topology_export_csr(const bf_topology_t* t, int32_t round, int64_t* rowptr, int32_t* col,
                           float* wgt, uint64_t* accepted_seed);

/* Diagnostic: the row-walk plan of a round whose off-diagonal graph is a union of paths and cycles
 * (ring, one-peer rounds, matchings), which lets the kernels stream rows through registers.
 * Returns n and, if steps is not NULL, writes n records of eight 32-bit words {row, flags,
 * last_row, next_row, slots, w0, w1, w2 (float bits)}: flags bit 0 = first row of a chain, bit 1 =
 * the chain is a cycle, bits 2-3 = source of the next row (0 load next_row, 1 the cycle's last row
 * kept from its start, 2 the cycle's first row, 3 none); slots holds three 4-bit codes in CSR order
 * (0 previous row of the walk, 1 this row, 2 next row, 15 no entry).  Returns 0 when the round has
 * no such plan, negative on error. */
int32_t bf_topology_chain_plan(const bf_topology_t* t, int32_t round, int32_t* steps);

/* Window layout of a round (section "Asynchronous decentralized communication": every agent owns
 * one slot per in-coming neighbor, in one contiguous chunk).  Slots are numbered over all agents,
 * agent 0's first, within an agent in the order of its CSR row with the diagonal entry left out.
 * bf_topology_window_slots returns their number E (or a negative status);
 * bf_topology_export_window copies to caller-sized host arrays slot_rowptr[n+1] (agent i owns
 * slots slot_rowptr[i] .. slot_rowptr[i+1]-1), slot_src[E] (the sender of each slot),
 * slot_weight[E] (w_{i,src}) and self_weight[n] (w_ii, 0 without a diagonal entry); any may be
 * NULL. */
int64_t bf_topology_window_slots(const bf_topology_t* t, int32_t round);
int bf_topology_export_window(const bf_topology_t* t, int32_t round, int64_t* slot_rowptr, int32_t* slot_src,
                              float* slot_weight, float* self_weight);

/* Partial averaging (eq. dsgd-2, eq. dgd-2; the neighbor_allreduce primitive):
 *   X_out[i,:] = sum_{(j,w) in row i of W^(round)} w * X_in[j,:].
 * Accumulation is fp32 in CSR order; BF_BF16 rounds the result to nearest-even on store.
 * Kernel choice (all give the same bits for BF_F32): column tiles staged in LDS while n x 64 fp32
 * values fit one CU's LDS (n <= 640 on MI355X), rows streamed through registers for wide matrices
 * whose round is a union of paths and cycles, and beyond that a row gather through the caches (out
 * of place) or 4..32-column LDS tiles (in place, n <= 10240); more agents than that in place is
 * BF_ERR_UNSUPPORTED.  The same holds for every call below that mixes a matrix.
 * ld may be BF_LD_BLOCKED(B): the matrices are then in column blocks of B columns, and the LDS tile
 * kernels run with tiles of at most B columns and the row-streaming kernel with sweeps inside a
 * block (same arithmetic, same bits).  bf_neighbor_allreduce_multi,
 * bf_hierarchical_neighbor_allreduce, bf_pushsum_step, bf_pushsum_atc_step, bf_tracking_step,
 * bf_atc_step, bf_exact_diffusion_step, bf_dense_mix, the bf_win_* calls (X with n rows and the
 * window with E rows, both in blocks of B), bf_grad_quadratic and bf_consensus_stats accept it too;
 * the least-squares calls (bf_grad_least_squares, the bf_*_least_squares_run family), whose access
 * is by whole rows of small matrices, take agent-major matrices only. */
int bf_neighbor_allreduce(const bf_topology_t* t, int32_t round, const void* X_in, void* X_out,
                          int64_t d, int64_t ld, bf_dtype_t dt, void* hip_stream);

/* `count` consecutive rounds of partial averaging in one pass over the matrix: the per-round
 * recursion of eq. dsgd-2 applied `count` times with the time-varying weights of section "Push- and
 * pull-style communication over time-varying topology" (the one-peer exponential graph, which the
 * paper names in "Concepts and Theoretical Foundations" and uses in its DNN experiments, averages
 * exactly in log2 n such rounds):  X_out = W^(round0+count-1) ... W^(round0+1) W^(round0) X_in.
 * Every intermediate product stays on chip in fp32 (also for BF_BF16, which therefore rounds once,
 * at the end, unlike `count` separate calls); for BF_F32 the result is bit-identical to `count`
 * calls of bf_neighbor_allreduce.  1 <= count <= 8, else BF_ERR_SIZE.  One pass needs two n x 64
 * fp32 tiles in one CU's LDS (n <= 320 on MI355X); with more agents the call runs `count` separate
 * passes instead (BF_BF16 then rounds after every round).  X_out may equal X_in. */
int bf_neighbor_allreduce_multi(const bf_topology_t* t, int32_t round0, int32_t count, const void* X_in,
                                void* X_out, int64_t d, int64_t ld, bf_dtype_t dt, void* hip_stream);

/* Two-level neighbor averaging (section "Enabling hierarchical communication"): agents are grouped
 * into machines of `local_size` consecutive ranks (machine_rank = rank / local_size); each machine
 * first averages its agents, the machines then do one round of partial averaging over
 * `machine_topology` (whose n is the number of machines M), and every agent of a machine takes its
 * machine's result:  X_out[i,:] = sum_b W_machine[a(i), b] * (1/local_size) sum_{j in b} X_in[j,:].
 * X has M * local_size rows.  One pass over X when an (M*local_size + M) x 64 fp32 tile fits one
 * CU's LDS (the M machine values sit beside the staged rows), three passes otherwise (up to an
 * (M*local_size) x 64 tile; beyond that BF_ERR_UNSUPPORTED).  The derived
 * operator is built on first use and kept inside machine_topology (freed with it).  X_out may equal
 * X_in.  local_size < 1: BF_ERR_SIZE. */
int bf_hierarchical_neighbor_allreduce(const bf_topology_t* machine_topology, int32_t round, int32_t local_size,
                                       const void* X_in, void* X_out, int64_t d, int64_t ld, bf_dtype_t dt,
                                       void* hip_stream);

/* Window primitives (sections "Asynchronous decentralized communication" and "Asynchronous
 * push-style partial averaging"), all agents simulated on one device.  X: n x d device matrix of
 * dtype dt, row pitch ld elements.  Win: E x d device matrix, ALWAYS fp32 (slots accumulate), with
 * the same pitch ld in elements (so ld * 4 bytes), row e being slot e of the layout above (the
 * caller allocates it and zeroes it once, as win_create does).  p: n device floats, win_p: E
 * device floats, the push-sum scalar and its slots (both NULL to leave them out).  active: n
 * device int32 flags, or NULL for everybody; an agent whose flag is 0 does nothing in that call,
 * which is how agents that run at different speeds are simulated.  With BF_BF16 the arithmetic is
 * fp32 and X is rounded to nearest-even when it is written.  Calls on one stream execute one after the other, which gives
 * the mutual exclusion and the atomic read-and-reset the paper asks for; calls on different
 * streams that share X or Win race.  X, Win, p, win_p may not overlap (BF_ERR_ALIAS).  A topology
 * without edges has E = 0 slots; Win and win_p may then be NULL.
 *   bf_win_put:        every active j copies x_j into its slot at each out-neighbor (no weights).
 *   bf_win_get:        every active i copies x_j of each in-neighbor j into its own slot for j.
 *   bf_win_accumulate: every active j adds w_ij x_j (w_ij p_j) to its slot at each out-neighbor i,
 *                      then keeps w_jj x_j (w_jj p_j).
 *   bf_win_update:     every active i sets x_i = w_ii x_i + sum over its slots of w_ij * slot;
 *                      the window is left as it is.
 *   bf_win_update_then_collect: every active i adds its slots to x_i (p_i) and zeroes them.
 * With W column stochastic, sum(p) + sum(win_p) stays n and sum(X) + sum(Win) stays what it was
 * (up to fp32 rounding) whatever the activity pattern. */
int bf_win_put(const bf_topology_t* t, int32_t round, const int32_t* active, const void* X, void* Win,
               int64_t d, int64_t ld, bf_dtype_t dt, void* hip_stream);
int bf_win_get(const bf_topology_t* t, int32_t round, const int32_t* active, const void* X, void* Win,
               int64_t d, int64_t ld, bf_dtype_t dt, void* hip_stream);
int bf_win_accumulate(const bf_topology_t* t, int32_t round, const int32_t* active, void* X, float* p,
                      void* Win, float* win_p, int64_t d, int64_t ld, bf_dtype_t dt, void* hip_stream);
int bf_win_update(const bf_topology_t* t, int32_t round, const int32_t* active, void* X, const void* Win,
                  int64_t d, int64_t ld, bf_dtype_t dt, void* hip_stream);
int bf_win_update_then_collect(const bf_topology_t* t, int32_t round, const int32_t* active, void* X, float* p,
                               void* Win, float* win_p, int64_t d, int64_t ld, bf_dtype_t dt, void* hip_stream);

/* The same calls with the per-call weight arguments of the paper's signatures (section
 * "Asynchronous decentralized communication"): neighbor_win_put / neighbor_win_accumulate(tensor,
 * name, [self_weight, dst_weights]), neighbor_win_get(tensor, name, [src_weights]), win_update(name,
 * [self_weight, src_weights]).  The window is laid out over the static topology; a call may name
 * any SUBSET of its edges, with any weights ("the ranks used in dst_weights and src_weights should
 * be the subset of the neighbors defined under the global static topology").  On one device the
 * dictionaries of all agents together are arrays in the window's slot order:
 *   self_weight: n device floats, agent j's self_weight; NULL = no such argument.
 *   dst_weight / src_weight: E device floats, the weight of the edge that slot e stands for (slot e
 *       of receiver i holds what sender slot_src[e] pushes to i, or what i pulls from it); NULL = no
 *       such argument.
 *   dst_on / src_on: E device int32 flags, nonzero for the edges the call names; NULL = all edges.
 * Without an argument the call behaves as its plain form above (put, get: weight 1 and X unchanged;
 * accumulate, update: the topology's own weights).
 *   put:        every active j writes dst_weight * x_j into its slot at each named out-neighbor,
 *               then, if self_weight is given, keeps self_weight[j] * x_j.
 *   accumulate: every active j adds dst_weight * x_j (and dst_weight * p_j) to those slots, then
 *               keeps self_weight[j] * x_j (and p_j likewise).
 *   get:        every active i writes src_weight * x_j into its own slot for each named in-neighbor j.
 *   update:     every active i sets x_i = self_weight[i] x_i + sum over its named slots of
 *               src_weight * slot; the window is left as it is.
 * Edges that are not named are neither written nor read.  Other arguments and errors as above. */
int bf_win_put_weighted(const bf_topology_t* t, int32_t round, const int32_t* active, void* X, void* Win,
                        const float* self_weight, const float* dst_weight, const int32_t* dst_on,
                        int64_t d, int64_t ld, bf_dtype_t dt, void* hip_stream);
int bf_win_get_weighted(const bf_topology_t* t, int32_t round, const int32_t* active, const void* X, void* Win,
                        const float* src_weight, const int32_t* src_on, int64_t d, int64_t ld, bf_dtype_t dt,
                        void* hip_stream);
int bf_win_accumulate_weighted(const bf_topology_t* t, int32_t round, const int32_t* active, void* X, float* p,
                               void* Win, float* win_p, const float* self_weight, const float* dst_weight,
                               const int32_t* dst_on, int64_t d, int64_t ld, bf_dtype_t dt, void* hip_stream);
int bf_win_update_weighted(const bf_topology_t* t, int32_t round, const int32_t* active, void* X, const void* Win,
                           const float* self_weight, const float* src_weight, const int32_t* src_on,
                           int64_t d, int64_t ld, bf_dtype_t dt, void* hip_stream);

/* Same product through the dense n x n form of W^(round) on the fp32 matrix cores (BF_F32 with
 * n <= 256; anything else is computed by the list kernels of bf_neighbor_allreduce).  Intended for
 * dense / fully connected W (periodic global averaging is W = 11^T/n) and as an independent
 * cross-check of the sparse kernels. */
int bf_dense_mix(const bf_topology_t* t, int32_t round, const void* X_in, void* X_out,
                 int64_t d, int64_t ld, bf_dtype_t dt, void* hip_stream);

/* One synchronous push-sum round (section "Asynchronous push-style partial averaging" with unit
 * delays; the u, v, x lines of push-sum gradient tracking): X_out = W X_in, w_out = W w_in and, if
 * Y is not NULL, Y[i,:] = X_out[i,:] / w_out[i].  W should be column stochastic and w start at 1;
 * this is not enforced.  w_in, w_out: n fp32 values (the paper's scalar p_i; kept apart from X so
 * rows stay 16-byte aligned).  w_out may equal w_in; Y has the layout of X_out and may not alias
 * anything. */
int bf_pushsum_step(const bf_topology_t* t, int32_t round, const void* X_in, void* X_out,
                    const float* w_in, float* w_out, void* Y, int64_t d, int64_t ld,
                    bf_dtype_t dt, void* hip_stream);

/* Push-sum round with a local update folded in -- the u, v, x lines of push-sum gradient tracking
 * (appendix "Application example: Push-sum gradient tracking algorithm"):
 *   X_out = W (X_in - alpha G),  w_out = W w_in,  Y[i,:] = X_out[i,:] / w_out[i]  (Y optional).
 * With G the tracker y this is  u' = W(u - alpha y), v' = W v, x' = u'/v'.  Arguments as in
 * bf_pushsum_step; G has the dtype and layout of X and may not overlap an output. */
int bf_pushsum_atc_step(const bf_topology_t* t, int32_t round, const void* X_in, void* X_out, const void* G,
                        float alpha, const float* w_in, float* w_out, void* Y, int64_t d, int64_t ld,
                        bf_dtype_t dt, void* hip_stream);

/* Tracker update of gradient tracking (same appendix, last line of the recursion):
 *   Y_out = W (Y_in + G_new - G_old).
 * All four matrices share dtype and layout; Y_out may equal Y_in. */
int bf_tracking_step(const bf_topology_t* t, int32_t round, const void* Y_in, void* Y_out, const void* G_new,
                     const void* G_old, int64_t d, int64_t ld, bf_dtype_t dt, void* hip_stream);

/* Local update fused with partial averaging (eqs. eq.atc / eq.awc; dsgd-1 + dsgd-2):
 *   M == NULL, BF_ATC:  X_out[i,:] = sum_j w_ij (X_in[j,:] - alpha G[j,:])
 *   M == NULL, BF_AWC:  X_out[i,:] = sum_j w_ij X_in[j,:] - alpha G[i,:]
 *   M != NULL (heavy-ball momentum, fp32, n x d with leading dimension ld, updated in place):
 *       M[j,:] <- beta M[j,:] + G[j,:], then the formulas above with M in the place of G.
 * G has the dtype and leading dimension of X.  beta is ignored when M is NULL. */
int bf_atc_step(const bf_topology_t* t, int32_t round, const void* X_in, void* X_out, const void* G,
                float* M, float alpha, float beta, bf_mode_t mode, int64_t d, int64_t ld,
                bf_dtype_t dt, void* hip_stream);

/* bf_atc_step with a layout per matrix: ld describes X_in and X_out, ld_g describes G, ld_m
 * describes M (ignored when M is NULL); each is a row pitch or BF_LD_BLOCKED(B).  What the agent-major
 * layout costs is the scattered in-place read-write of the state; scattered read-only streams cost
 * nothing.  Measured on the n = 32, d = 25.5 M bf16 momentum step (TB/s): everything on agent-major
 * rows 5.06; X and G on rows -- one contiguous parameter and gradient vector per agent, as a
 * per-agent producer and consumer have them -- and only the momentum, which nobody else looks at,
 * in column blocks 5.96; X and M in blocks with G on rows 6.3, as with everything in blocks.
 * Same arithmetic, same bits as bf_atc_step. */
int bf_atc_step_layouts(const bf_topology_t* t, int32_t round, const void* X_in, void* X_out, const void* G,
                        float* M, float alpha, float beta, bf_mode_t mode, int64_t d, int64_t ld, int64_t ld_g,
                        int64_t ld_m, bf_dtype_t dt, void* hip_stream);

/* One Exact-Diffusion iteration (appendix "Application example: Exact-Diffusion algorithm",
 * eqs. ed-1, ed-2, ed-3), fused into one pass:
 *   psi_i = x_i - alpha g_i;   phi_i = psi_i + x_i - psi_prev_i;   X_out[i,:] = sum_j w_ij phi_j;
 *   Psi_prev[i,:] <- psi_i.
 * Psi_prev is fp32, n x d with leading dimension ld, updated in place; before the first iteration
 * the caller sets it to X (so that phi^(0) = psi^(0)).  G has the dtype and layout of X. */
int bf_exact_diffusion_step(const bf_topology_t* t, int32_t round, const void* X_in, void* X_out,
                            const void* G, float* Psi_prev, float alpha, int64_t d, int64_t ld,
                            bf_dtype_t dt, void* hip_stream);

/* bf_exact_diffusion_step with a layout per matrix, as bf_atc_step_layouts: ld describes X_in and
 * X_out, ld_g describes G, ld_p describes Psi_prev (the state only this call reads: the one to keep in
 * column blocks next to per-agent parameter and gradient vectors). */
int bf_exact_diffusion_step_layouts(const bf_topology_t* t, int32_t round, const void* X_in, void* X_out,
                                    const void* G, float* Psi_prev, float alpha, int64_t d, int64_t ld,
                                    int64_t ld_g, int64_t ld_p, bf_dtype_t dt, void* hip_stream);

/* Decentralized gradient descent on least squares (section "Decentralized linear regression",
 * eqs. dgd-1 and dgd-2; the adapt-then-combine form of bf_grad_least_squares + bf_atc_step):
 * `iterations` iterations in ONE launch,
 *   x_i <- sum_j w_ij^(round0+k) (x_j - alpha A_j^T (A_j x_j - b_j)),   k = 0 .. iterations-1,
 * when one agent's A_i (m x d fp32) fits one CU's LDS next to 20 KB of working storage (the paper's
 * example, m = 32, d = 1024, does), m <= 64, d <= 4096 and n is at most the number of CUs: one
 * workgroup per agent keeps A_i in LDS for the whole run and the agents meet at a grid barrier once
 * per iteration.  Larger problems run the same iterations as two launches each (bf_grad_least_squares
 * into the first half of `work`, then bf_atc_step in place).
 * A: n x m x d row-major fp32, b: n x m, X: n x d with pitch ld, updated in place; work: device
 * scratch of 2 * n * ld floats (contents undefined afterwards).  1 <= m <= 8192, d a multiple of 4,
 * d >= 4.  Every barrier wait is bounded: if the workgroups cannot all be resident at once
 * (the device is busy with other kernels for about a second) the run gives up, X is undefined and
 * bf_dgd_status reports it.  One such run at a time per topology object (they share the barrier
 * words); runs on one stream are ordered and safe.
 * bf_dgd_status: waits for `hip_stream` and writes 1 to *timed_out (host) if the last run on this
 * topology gave up, else 0. */
int bf_dgd_least_squares_run(const bf_topology_t* t, int32_t round0, int32_t iterations, int32_t m,
                             const float* A, const float* b, float* X, float* work, float alpha,
                             int64_t d, int64_t ld, void* hip_stream);
int bf_dgd_status(const bf_topology_t* t, int32_t* timed_out, void* hip_stream);

/* bf_dgd_least_squares_run for callers that cannot allocate device memory: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same computation, same kernel and
 * bit-identical results; the only difference is where the scratch lives.  The half steps
 * (2 * n * ld floats) and the two barrier words sit in a static device array of the library
 * (2 MiB + 256 bytes per GPU, held until the process ends) instead of a caller workspace and a
 * lazily allocated pair of words, and the call performs no hipMalloc / hipFree of any kind.
 *   - 2 * n * ld * 4 bytes must not exceed 2 MiB (2,097,152), else BF_ERR_SIZE.
 *   - Only the one-launch form exists here (m <= 64, d <= 4096, A_i in one CU's LDS, n <= CUs); a
 *     larger problem is BF_ERR_UNSUPPORTED.
 *   - The topology's device copy is never created here: if `t` has not been used by any compute call
 *     on the current device yet (which is what uploads it), the call returns BF_ERR_UNSUPPORTED.
 *   - Every call on a GPU shares that GPU's one array, whatever the topology: calls that overlap in
 *     time on one GPU (different streams) race; calls on one stream are ordered and safe.  The
 *     barrier words are cleared by a small kernel at the start of each call; the half steps need no
 *     clearing (each is written before it is read).
 * All other arguments, limits and error codes as for bf_dgd_least_squares_run; bf_dgd_status
 * reports on whichever of the two variants ran last on the topology. */
int bf_dgd_least_squares_run_static(const bf_topology_t* t, int32_t round0, int32_t iterations, int32_t m,
                                    const float* A, const float* b, float* X, float alpha, int64_t d, int64_t ld,
                                    void* hip_stream);

/* Exact-Diffusion on the same problem in the same way (appendix "Application example:
 * Exact-Diffusion algorithm", eqs. ed-1, ed-2, ed-3 with the least-squares gradient):
 *   psi_i = x_i - alpha A_i^T (A_i x_i - b_i);  phi_i = psi_i + x_i - psi_prev_i;  x_i <- sum_j w_ij phi_j.
 * Psi_prev: n x d with pitch ld, in and out (set it to X before the first run).  Everything else,
 * bf_dgd_status included, as for bf_dgd_least_squares_run; needs 4 * d more bytes of LDS. */
int bf_exact_diffusion_least_squares_run(const bf_topology_t* t, int32_t round0, int32_t iterations, int32_t m,
                                         const float* A, const float* b, float* X, float* Psi_prev, float* work,
                                         float alpha, int64_t d, int64_t ld, void* hip_stream);

/* Local least-squares gradients of decentralized linear regression (eq. dgd-1):
 *   G[i,:] = A_i^T (A_i x_i - b_i),  A: n x m x d row-major fp32, b: n x m fp32.
 * 1 <= m <= 8192, d a multiple of 4.  G must not alias X. */
int bf_grad_least_squares(int32_t n, int32_t m, int64_t d, const float* A, const float* b,
                          const float* X, int64_t ldx, float* G, int64_t ldg, void* hip_stream);

/* Synthetic stochastic gradient of f_i(x) = lam/2 |x - c_i|^2: G = lam (X - C) + sigma E, all
 * n x d with leading dimension ld and dtype dt; computed in fp32.  Used to drive the momentum
 * benchmark; not part of the timed path. */
int bf_grad_quadratic(int32_t n, int64_t d, int64_t ld, const void* X, const void* C, const void* E,
                      float lam, float sigma, void* G, bf_dtype_t dt, void* hip_stream);

/* Diagnostics (average consensus problem, section "Asynchronous push-style partial averaging"):
 * with y_i = x_i (p == NULL) or x_i / p[i], and ybar the column mean of the y_i, writes to the
 * device array stats[3] (fp64): sum_ic (y_ic - ybar_c)^2, max_ic |y_ic - ybar_c|, max_ic |y_ic|.
 * If mean_out is not NULL it receives ybar as d fp32 values.  Accumulation is fp64. */
int bf_consensus_stats(int32_t n, int64_t d, int64_t ld, const void* X, const float* p, bf_dtype_t dt,
                       double* stats, float* mean_out, void* hip_stream);

/* The column-block layout (see the conventions at the top).  BF_LD_BLOCKED(B) is what a call takes
 * as ld for matrices in blocks of B columns. */
#define BF_LD_BLOCKED(B) (-(int64_t)(B))

/* Elements of an n x d matrix in column blocks of `block` columns: ceil(d/block) * n * block.
 * Negative (BF_ERR_SIZE) if block is not a power of two in [64, 2^20] or n, d are out of range. */
int64_t bf_blocked_elems(int32_t n, int64_t d, int64_t block);

/* Block width this library suggests for n x d matrices mixed over topology t (measured on MI355X):
 * the power of two nearest to 2^20 / n within [2048, 16384] (16384 columns at n <= 64, 8192 at
 * n = 128; at most 8192 for BF_BF16, whose steps usually carry an fp32 state matrix as well); 65536 when n > 160 and every round of t is a union of paths and cycles (those go to the
 * row-streaming kernel); the power of two that covers d when d is smaller.  Negative on error. */
int64_t bf_recommended_block(const bf_topology_t* t, int64_t d, bf_dtype_t dt);

/* Layout conversion, device to device: X (agent-major, n x d, pitch ld) to X_blocked (column blocks
 * of `block` columns, bf_blocked_elems(n, d, block) elements; the padding columns of the last block
 * are set to zero), and back (columns d..ld-1 of X are not written).  The two must not overlap.
 * One pass over the matrix each; not part of a step: a state that lives in column blocks is
 * converted once. */
int bf_blocked_pack(int32_t n, int64_t d, int64_t ld, const void* X, int64_t block, void* X_blocked,
                    bf_dtype_t dt, void* hip_stream);
int bf_blocked_unpack(int32_t n, int64_t d, int64_t block, const void* X_blocked, int64_t ld, void* X,
                      bf_dtype_t dt, void* hip_stream);

/* Leading dimension (elements) this library suggests for an n x d matrix of dtype dt: the row pitch
 * is d rounded up to 128 bytes plus 4224 bytes (one 4 KB page and one 128-byte line).  A pitch that
 * is a large power of two sends the same column of every agent to the same HBM channel and bank;
 * the offset spreads the n concurrent row streams of a tile (measured +5..10 % bandwidth).
 * Any ld >= d with a 16-byte-multiple pitch is accepted by the compute calls.  Negative on error. */
int64_t bf_recommended_ld(int64_t d, bf_dtype_t dt);

/* Plain streaming kernels with 128-bit accesses, for measuring the practical bandwidth ceilings the
 * mixing kernels are compared with (not part of the method).  mode 0: dst <- src (bytes read and
 * bytes written); mode 1: read src only (dst, at least 16 * 256 * workgroups bytes, is written
 * only if the data sum to a particular value, which keeps the loads alive); mode 2: fill dst with
 * a constant.  bytes is a multiple of 16; workgroups_per_cu (1..64) sets the size of the
 * persistent grid. */
int bf_stream_probe(int32_t mode, const void* src, void* dst, int64_t bytes, int32_t workgroups_per_cu,
                    void* hip_stream);

const char* bf_strerror(int code);
int         bf_last_hip_error(void);   /* hipError_t of the last BF_ERR_HIP on this thread        */

/* Launch-shape override for experiments and sweeps; value 0 restores the built-in heuristic.
 *   knob 0: column-tile width of the LDS tile kernel in elements (power of two, 64..1024)
 *   knob 1: workgroups per compute unit for the tile kernel
 *   knob 2: 1 forces the fallbacks for large agent counts (row gather, narrow tiles)
 *   knob 3: upper bound on the number of persistent workgroups (for the window calls: their number,
 *           which may also exceed the default of one per compute unit)
 *   knob 5: 1 disables the row-streaming chain kernel
 *   knob 8: 1 forces non-temporal loads/stores in the tile kernels, 2 forbids them
 *   knob 12: 1 uses the pipelined tile kernel (loader and reducer waves) also for cache-resident
 *           in-place rounds, 2 never uses it
 *   knob 13: 1 keeps bf_neighbor_allreduce_multi from running shift rounds in registers, 2 makes
 *           it do so whenever the rounds have that form (the default also weighs n and count)
 *   knob 14: 1 makes the pipelined kernel's AWC step with bf16 storage fetch the receiver's own
 *           gradient from HBM in the reducer waves, as with fp32 storage, instead of staging the
 *           gradients in LDS
 *   knob 9: 1 keeps the chain kernel at 256-thread workgroups
 *   knob 7: 1 disables the alternating (odd rounds right-to-left) tile order
 *   knob 6: forces the chain kernel (where the round has a chain plan) with 1, 2 or 4 16-byte
 *           vectors per thread, whatever the matrix shape
 *   knob 10: number of polls a grid-barrier wait of bf_dgd_least_squares_run may take before it
 *           gives up
 *   knob 11: 1 makes that barrier wait for one arrival more than there are workgroups, so that it
 *           must give up (with knob 10 small, the test of the give-up path: the kernel still exits)
 * Values the kernels cannot honour give BF_ERR_UNSUPPORTED at the next compute call.  Process-wide,
 * not thread safe: for benchmarks and tests only. */
int bf_set_tuning(int32_t knob, int32_t value);

#ifdef __cplusplus
}
#endif
#endif /* BF_H_ */
