// HIP kernels of libbf for gfx950 (MI355X) and their C-ABI entry points.
//
// Core idea.  Partial averaging X_out = W X_in (eq. dsgd-2) is column separable: column c of the
// result depends on column c of the input only.  A workgroup therefore owns a tile of C columns for
// ALL n agents: it streams the n x C tile from HBM once (16-byte loads, long coalesced row
// segments), forms the local update x_j - alpha g_j (eq. dsgd-1 / eq. eq.atc) while staging the
// tile into LDS, then produces every output row of the tile from LDS -- one wave per (row, 64-lane
// span), the row's in-neighbor list read through the scalar cache, accumulation in registers --
// and writes each output element once.  HBM traffic is the compulsory read-once / write-once; the
// (nnz) x d gather traffic stays inside LDS.  Because no other workgroup touches those columns the
// update may be in place.
//
// Workgroups are persistent: tile t+1's global loads are issued into registers before tile t is
// reduced, so HBM requests are in flight during the LDS phase.

#include <new>

#include "bf_device.h"

thread_local int bf::g_last_hip_error = 0;

namespace {

using namespace bf;

// ---------------------------------------------------------------------------------------------
// Push-sum weights: w_out = W w_in for n scalars (the p_i of the push-sum recursion).  One
// workgroup; w_in is copied to LDS first so that w_out may be w_in.
__global__ __launch_bounds__(1024) void bf_pushsum_w_kernel(const int32_t* rowptr, const u32x2* ent,
                                                           const float* w_in, float* w_out, int n) {
  extern __shared__ f32x4 lds_raw[];
  float* wl = reinterpret_cast<float*>(lds_raw);
  for (int i = threadIdx.x; i < n; i += blockDim.x) wl[i] = w_in[i];
  __syncthreads();
  for (int i = threadIdx.x; i < n; i += blockDim.x) {
    float acc = 0.0f;
    for (int q = rowptr[i]; q < rowptr[i + 1]; ++q) {
      const u32x2 en = ent[q];
      acc = fmaf(__uint_as_float(en.y), wl[en.x], acc);
    }
    w_out[i] = acc;
  }
}

// ---------------------------------------------------------------------------------------------
// Window primitives (section "Asynchronous decentralized communication").  The window of agent i
// is one row per in-neighbor; all windows form one E x d matrix with the row pitch of X.  A
// workgroup takes one agent and one 4096-column chunk of its row (four 16-byte vectors per thread,
// so the loads of an edge's slot are all in flight together) and walks the agent's out-edges
// (sender side: put, accumulate) or its own slots (receiver side: update, update_then_collect).
// Every slot has exactly one sender and one owner, so within a call no two workgroups touch the
// same bytes; successive calls on one stream give the atomicity the paper asks of
// update_then_collect.  Agents whose `active` entry is zero do nothing.
struct WinParams {
  char* x;                   // n x ld, fp32 or bf16
  float* win;                // E x ld, always fp32 (slots accumulate)
  const int32_t* active;     // n flags, or null: everybody
  const int32_t* in_ptr;
  const float* slot_w;
  const int32_t* slot_src;
  const float* self_w;
  const int32_t* out_ptr;
  const u32x2* out_ent;      // {slot, weight bits}
  // per-call arguments of the paper's signatures (all optional, all in the window's slot order):
  const float* call_self_w;  // n: self_weight of this call
  const float* call_edge_w;  // E: dst_weights (put, accumulate) / src_weights (get, update) of this call
  const int32_t* call_edge_on;  // E flags: the subset of edges this call names; null: all
  int64_t d, ld;
  int32_t n, chunks;
  int32_t block_log;         // 0: agent-major rows; else X (n rows) and the window (E rows) in column blocks of 1 << block_log
  int32_t slots;             // E
};

enum { WIN_PUT = 0, WIN_ACCUMULATE = 1, WIN_COLLECT = 2, WIN_AVERAGE = 3, WIN_GET = 4 };

// Scalar-cache views of the window plan and of the per-call arrays (one value per agent or per
// edge, the same for every lane): uniform addresses into these become s_load instructions, which
// leaves the vector-memory counter to the row traffic.
typedef const float __attribute__((address_space(4)))* win_f32_ptr;

// One unit of work: agent a, columns [c * 4096, (c + 1) * 4096).  FULL: every one of the workgroup's
// 16-byte vectors lies inside [0, d), so nothing is predicated per lane.
template <int MODE, int DT, bool STREAM, bool FULL>
__device__ __forceinline__ void win_unit(const WinParams& p, int a, int c, int tid) {
  constexpr int U = 4;
  const bf::csr_i32_ptr in_ptr = (bf::csr_i32_ptr)(uintptr_t)p.in_ptr;
  const bf::csr_i32_ptr out_ptr = (bf::csr_i32_ptr)(uintptr_t)p.out_ptr;
  const bf::csr_i32_ptr slot_src = (bf::csr_i32_ptr)(uintptr_t)p.slot_src;
  const bf::csr_i32_ptr edge_flags = (bf::csr_i32_ptr)(uintptr_t)p.call_edge_on;
  const bf::csr_ent_ptr out_ent = (bf::csr_ent_ptr)(uintptr_t)p.out_ent;
  const win_f32_ptr slot_w = (win_f32_ptr)(uintptr_t)p.slot_w;
  const win_f32_ptr self_w = (win_f32_ptr)(uintptr_t)p.self_w;
  const win_f32_ptr call_self_w = (win_f32_ptr)(uintptr_t)p.call_self_w;
  const win_f32_ptr call_edge_w = (win_f32_ptr)(uintptr_t)p.call_edge_w;
  int64_t xcol[U], wcol[U];      // where the column lies within a row of pitch ld, in X and in the window
  int valid[U];
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const int64_t col = (static_cast<int64_t>(c) * U + u) * 1024 + tid * 4;
    const int64_t rem = p.d - col;
    valid[u] = FULL ? 4 : (rem >= 4 ? 4 : (rem > 0 ? static_cast<int>(rem) : 0));
    const int64_t blk = p.block_log ? col >> p.block_log : 0;
    xcol[u] = col + ((blk * (p.n - 1)) << p.block_log);
    wcol[u] = col + ((blk * (p.slots - 1)) << p.block_log);
  }
  // four columns of a row of X (storage type DT) or of the window (fp32); a vector that starts
  // inside the row may end in the row's padding: rows are 16-byte multiples
  auto load_x = [&](int64_t row, int u) -> f32x4 {
    if (!FULL && !valid[u]) return f32x4{0.f, 0.f, 0.f, 0.f};
    float v[4];
    load_in<DT, 4, STREAM>(p.x, row * p.ld + xcol[u], v);
    return f32x4{v[0], v[1], v[2], v[3]};
  };
  auto store_x = [&](int64_t row, int u, f32x4 v) {
    const float e[4] = {v.x, v.y, v.z, v.w};
    if (FULL || valid[u]) store_out<DT, 4, STREAM>(p.x, row * p.ld + xcol[u], e, FULL ? 4 : valid[u]);      // never the padding
  };
  auto load_w = [&](const float* row, int u) -> f32x4 {
    return (FULL || valid[u]) ? ld_stream<STREAM>(reinterpret_cast<const f32x4*>(row + wcol[u])) : f32x4{0.f, 0.f, 0.f, 0.f};
  };
  auto store_w = [&](float* row, int u, f32x4 v) {
    if (FULL || valid[u] == 4) { st_stream<STREAM>(reinterpret_cast<f32x4*>(row + wcol[u]), v); return; }
    const float e[4] = {v.x, v.y, v.z, v.w};
    for (int k = 0; k < valid[u]; ++k) row[wcol[u] + k] = e[k];
  };
  auto edge_on = [&](int e) { return !p.call_edge_on || edge_flags[e] != 0; };
  if constexpr (MODE == WIN_GET) {
    const int end = in_ptr[a + 1];
    for (int e = in_ptr[a]; e < end; ++e) {
      if (!edge_on(e)) continue;
      float* wrow = p.win + static_cast<int64_t>(e) * p.ld;
      f32x4 v[U];
#pragma unroll
      for (int u = 0; u < U; ++u) v[u] = load_x(slot_src[e], u);
      if (p.call_edge_w) {
        const float w = call_edge_w[e];
#pragma unroll
        for (int u = 0; u < U; ++u) { v[u].x *= w; v[u].y *= w; v[u].z *= w; v[u].w *= w; }
      }
#pragma unroll
      for (int u = 0; u < U; ++u) store_w(wrow, u, v[u]);
    }
    return;
  }
  f32x4 x[U];
#pragma unroll
  for (int u = 0; u < U; ++u) x[u] = load_x(a, u);
  if constexpr (MODE == WIN_PUT || MODE == WIN_ACCUMULATE) {
    const int end = out_ptr[a + 1];
    for (int q = out_ptr[a]; q < end; ++q) {
      const u32x2 en = out_ent[q];
      const int e = static_cast<int>(en.x);
      if (!edge_on(e)) continue;
      float* wrow = p.win + static_cast<int64_t>(e) * p.ld;
      if constexpr (MODE == WIN_PUT) {
        if (p.call_edge_w) {
          const float w = call_edge_w[e];
#pragma unroll
          for (int u = 0; u < U; ++u) store_w(wrow, u, f32x4{w * x[u].x, w * x[u].y, w * x[u].z, w * x[u].w});
        } else {
#pragma unroll
          for (int u = 0; u < U; ++u) store_w(wrow, u, x[u]);
        }
      } else {
        const float w = p.call_edge_w ? call_edge_w[e] : __uint_as_float(en.y);
        f32x4 v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) v[u] = load_w(wrow, u);
#pragma unroll
        for (int u = 0; u < U; ++u) {
          v[u].x = fmaf(w, x[u].x, v[u].x); v[u].y = fmaf(w, x[u].y, v[u].y);
          v[u].z = fmaf(w, x[u].z, v[u].z); v[u].w = fmaf(w, x[u].w, v[u].w);
          store_w(wrow, u, v[u]);
        }
      }
    }
    if (MODE == WIN_ACCUMULATE || p.call_self_w) {
      const float sw = p.call_self_w ? call_self_w[a] : self_w[a];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        x[u].x *= sw; x[u].y *= sw; x[u].z *= sw; x[u].w *= sw;
        store_x(a, u, x[u]);
      }
    }
  } else {
    if constexpr (MODE == WIN_AVERAGE) {
      const float sw = p.call_self_w ? call_self_w[a] : self_w[a];
#pragma unroll
      for (int u = 0; u < U; ++u) { x[u].x *= sw; x[u].y *= sw; x[u].z *= sw; x[u].w *= sw; }
    }
    const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
    const int end = in_ptr[a + 1];
    if (MODE == WIN_AVERAGE && !p.call_edge_on) {
      // Every slot counts: the loads of the next slot are issued before this one is summed, so a wave
      // has two slots (eight vectors per lane) in flight instead of one (n = 128, 512 slots,
      // d = 2^21: 5.4 -> 5.7 TB/s).  The two register sets alternate, because a copy of a loaded
      // register would wait for its load; the sum runs in slot order as in the loop below.
      struct Slot { float w; f32x4 v[U]; };
      auto fetch = [&](int e, Slot& s) __attribute__((always_inline)) {
        const float* wrow = p.win + static_cast<int64_t>(e) * p.ld;
        s.w = p.call_edge_w ? call_edge_w[e] : slot_w[e];
#pragma unroll
        for (int u = 0; u < U; ++u) s.v[u] = load_w(wrow, u);
      };
      auto add = [&](const Slot& s) __attribute__((always_inline)) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
          x[u].x = fmaf(s.w, s.v[u].x, x[u].x); x[u].y = fmaf(s.w, s.v[u].y, x[u].y);
          x[u].z = fmaf(s.w, s.v[u].z, x[u].z); x[u].w = fmaf(s.w, s.v[u].w, x[u].w);
        }
      };
      int e = in_ptr[a];
      if (e < end) {
        Slot s0, s1;
        fetch(e, s0);
        for (;;) {
          if (++e >= end) { add(s0); break; }
          fetch(e, s1);
          add(s0);
          if (++e >= end) { add(s1); break; }
          fetch(e, s0);
          add(s1);
        }
      }
    } else
    for (int e = in_ptr[a]; e < end; ++e) {
      if (MODE == WIN_AVERAGE && !edge_on(e)) continue;
      float* wrow = p.win + static_cast<int64_t>(e) * p.ld;
      f32x4 v[U];
#pragma unroll
      for (int u = 0; u < U; ++u) v[u] = load_w(wrow, u);
      if constexpr (MODE == WIN_COLLECT) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
          x[u].x += v[u].x; x[u].y += v[u].y; x[u].z += v[u].z; x[u].w += v[u].w;
          store_w(wrow, u, zero);
        }
      } else {
        const float w = p.call_edge_w ? call_edge_w[e] : slot_w[e];
#pragma unroll
        for (int u = 0; u < U; ++u) {
          x[u].x = fmaf(w, v[u].x, x[u].x); x[u].y = fmaf(w, v[u].y, x[u].y);
          x[u].z = fmaf(w, v[u].z, x[u].z); x[u].w = fmaf(w, v[u].w, x[u].w);
        }
      }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) store_x(a, u, x[u]);
  }
}

template <int MODE, int DT, bool STREAM>
__global__ __launch_bounds__(256) void bf_win_kernel(const WinParams p) {
  const int tid = threadIdx.x;
  const bf::csr_i32_ptr active = (bf::csr_i32_ptr)(uintptr_t)p.active;
  const int64_t units = static_cast<int64_t>(p.n) * p.chunks;
  for (int64_t unit = blockIdx.x; unit < units; unit += gridDim.x) {
    // consecutive workgroups walk along an agent's row in either layout (measured on column blocks:
    // walking down the agents of a chunk instead is 5 % slower)
    const int a = static_cast<int>(unit / p.chunks);
    const int c = static_cast<int>(unit - static_cast<int64_t>(a) * p.chunks);
    if (p.active && active[a] == 0) continue;
    if ((static_cast<int64_t>(c) + 1) * 4096 <= p.d) win_unit<MODE, DT, STREAM, true>(p, a, c, tid);
    else win_unit<MODE, DT, STREAM, false>(p, a, c, tid);
  }
}

// The push-sum scalars of the same two calls: p_j and one scalar per slot.  One workgroup.
template <int MODE>
__global__ __launch_bounds__(1024) void bf_win_p_kernel(const WinParams p, float* pv, float* win_p) {
  for (int a = threadIdx.x; a < p.n; a += blockDim.x) {
    if (p.active && p.active[a] == 0) continue;
    if constexpr (MODE == WIN_ACCUMULATE) {
      const float pa = pv[a];
      for (int q = p.out_ptr[a]; q < p.out_ptr[a + 1]; ++q) {
        const u32x2 en = p.out_ent[q];
        if (p.call_edge_on && p.call_edge_on[en.x] == 0) continue;
        const float w = p.call_edge_w ? p.call_edge_w[en.x] : __uint_as_float(en.y);
        win_p[en.x] = fmaf(w, pa, win_p[en.x]);
      }
      pv[a] = pa * (p.call_self_w ? p.call_self_w[a] : p.self_w[a]);
    } else {
      float pa = pv[a];
      for (int e = p.in_ptr[a]; e < p.in_ptr[a + 1]; ++e) { pa += win_p[e]; win_p[e] = 0.0f; }
      pv[a] = pa;
    }
  }
}

// ---------------------------------------------------------------------------------------------
// Least-squares gradient g_i = A_i^T (A_i x_i - b_i) (eq. dgd-1).  One workgroup per agent.
// Phase 1: one wave per row of A_i forms the residual (fp32 products, per-lane partial sums, wave
// tree).  Phase 2: each thread owns 4 columns and accumulates A_i^T r over the m rows.
__global__ __launch_bounds__(1024) void bf_ls_grad_kernel(const float* A, const float* b, const float* X,
                                                         float* G, int m, int64_t d, int64_t ldx, int64_t ldg) {
  extern __shared__ f32x4 lds_raw[];
  float* resid = reinterpret_cast<float*>(lds_raw);            // m residuals
  const int i = blockIdx.x;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, nw = blockDim.x >> 6;
  const float* Ai = A + static_cast<int64_t>(i) * m * d;
  const float* xi = X + static_cast<int64_t>(i) * ldx;
  for (int k = wave; k < m; k += nw) {
    const float* row = Ai + static_cast<int64_t>(k) * d;
    float s = 0.0f;
    for (int64_t c = lane * 4; c < d; c += 256) {
      const f32x4 a = *reinterpret_cast<const f32x4*>(row + c);
      const f32x4 x = *reinterpret_cast<const f32x4*>(xi + c);
      s = fmaf(a.x, x.x, s); s = fmaf(a.y, x.y, s); s = fmaf(a.z, x.z, s); s = fmaf(a.w, x.w, s);
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
    if (lane == 0) resid[k] = s - b[static_cast<int64_t>(i) * m + k];
  }
  __syncthreads();
  float* gi = G + static_cast<int64_t>(i) * ldg;
  for (int64_t c = static_cast<int64_t>(tid) * 4; c < d; c += static_cast<int64_t>(blockDim.x) * 4) {
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    for (int k = 0; k < m; ++k) {
      const f32x4 a = *reinterpret_cast<const f32x4*>(Ai + static_cast<int64_t>(k) * d + c);
      const float r = resid[k];
      acc.x = fmaf(a.x, r, acc.x); acc.y = fmaf(a.y, r, acc.y);
      acc.z = fmaf(a.z, r, acc.z); acc.w = fmaf(a.w, r, acc.w);
    }
    *reinterpret_cast<f32x4*>(gi + c) = acc;
  }
}

// ---------------------------------------------------------------------------------------------
// Synthetic gradient G = lam (X - C) + sigma E, elementwise in fp32.
template <int DT>
__global__ __launch_bounds__(256) void bf_grad_quadratic_kernel(const char* X, const char* C, const char* E, char* G,
                                                               int n, int64_t d, int64_t ld, int block_log, float lam, float sigma) {
  constexpr int UC = Elem<DT>::per16;
  constexpr int EB = Elem<DT>::bytes;
  const int64_t upr = (d + UC - 1) / UC;
  const int64_t total = upr * n;
  for (int64_t u = blockIdx.x * static_cast<int64_t>(blockDim.x) + threadIdx.x; u < total;
       u += static_cast<int64_t>(gridDim.x) * blockDim.x) {
    const int64_t row = u / upr, col = (u % upr) * UC;
    const int64_t off = row * ld + col + (block_log ? ((col >> block_log) * (n - 1)) << block_log : int64_t{0});
    float xv[UC], cv[UC], ev[UC], gv[UC];
    widen<DT>(*reinterpret_cast<const u32x4*>(X + off * EB), xv);
    widen<DT>(*reinterpret_cast<const u32x4*>(C + off * EB), cv);
    widen<DT>(*reinterpret_cast<const u32x4*>(E + off * EB), ev);
#pragma unroll
    for (int e = 0; e < UC; ++e) gv[e] = fmaf(sigma, ev[e], lam * (xv[e] - cv[e]));
    const int64_t rem = d - col;
    if (rem >= UC) {
      u32x4 o;
      if constexpr (DT == DT_F32) {
        o.x = __float_as_uint(gv[0]); o.y = __float_as_uint(gv[1]); o.z = __float_as_uint(gv[2]); o.w = __float_as_uint(gv[3]);
      } else {
        o.x = pack_bf16x2(gv[0], gv[1]); o.y = pack_bf16x2(gv[2], gv[3]);
        o.z = pack_bf16x2(gv[4], gv[5]); o.w = pack_bf16x2(gv[6], gv[7]);
      }
      *reinterpret_cast<u32x4*>(G + off * EB) = o;
    } else {
      for (int e = 0; e < UC; ++e)
        if (e < rem) {
          if constexpr (DT == DT_F32) reinterpret_cast<float*>(G)[off + e] = gv[e];
          else reinterpret_cast<uint16_t*>(G)[off + e] = static_cast<uint16_t>(f32_to_bf16_bits(gv[e]));
        }
    }
  }
}

// ---------------------------------------------------------------------------------------------
// Decentralized gradient descent on least squares (eqs. dgd-1, dgd-2), many iterations in ONE
// launch, for problems small enough that each agent's A_i fits the LDS of one CU (the paper's
// linear-regression example: 32 x 1024 fp32 = 128 KB).  One 1024-thread workgroup per agent keeps
// A_i, b_i and x_i in LDS for the whole run.  Per iteration: residual r = A_i x_i - b_i (a wave per
// row), half step h_i = x_i - alpha A_i^T r (rows split over the threads that share a column
// vector), publish h_i to global memory, cross the grid barrier, combine the neighbors' half steps
// in list order.  The half steps are double buffered by iteration parity, so one barrier per
// iteration is enough: nobody can be more than one iteration ahead.
//
// The barrier is a monotonic arrival counter.  Every wait is bounded: after `spin_limit` polls (or
// as soon as anyone has set the error word) a workgroup sets the error word and leaves, and so
// does everybody else, so the grid always drains; the result is then undefined and the error word
// tells the host.  The exchange uses agent-scope atomic stores and loads (the L2 caches of the
// XCDs are not coherent with each other for ordinary accesses).
struct DgdParams {
  const float* A;
  const float* b;
  float* X;
  float* H;                  // 2 x n x ld half steps
  float* Psi;                // null: DGD.  Else Exact-Diffusion: n x ld, psi of the previous iteration, in/out
  const char* blob;          // round table + CSR of every round
  unsigned int* sync;        // [0] arrivals, [1] error
  int64_t d, ld;
  int32_t n, m, iters, round_k0, nrounds;
  float alpha;
  uint32_t spin_limit;
  uint32_t extra_arrivals;   // 0; a test sets 1 so that the barrier can never complete and must give up
};

__global__ __launch_bounds__(1024) void bf_dgd_ls_kernel(const DgdParams p) {
  extern __shared__ f32x4 lds_raw[];
  float* As = reinterpret_cast<float*>(lds_raw);                 // m x d
  float* xs = As + static_cast<size_t>(p.m) * p.d;               // d
  f32x4* part = reinterpret_cast<f32x4*>(xs + p.d);              // 1024 partial column sums
  float* resid = reinterpret_cast<float*>(part + 1024);          // 64
  float* bs = resid + 64;                                        // 64
  float* psi_prev = bs + 64;                                     // d, Exact-Diffusion only
  __shared__ int failed;
  const int i = blockIdx.x;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int d = static_cast<int>(p.d), m = p.m;
  const int nvec = d >> 2;
  {
    const f32x4* src = reinterpret_cast<const f32x4*>(p.A + static_cast<int64_t>(i) * m * d);
    f32x4* dst = reinterpret_cast<f32x4*>(As);
    for (int v = tid; v < m * nvec; v += 1024) dst[v] = src[v];
    for (int c = tid; c < d; c += 1024) xs[c] = p.X[static_cast<int64_t>(i) * p.ld + c];
    if (tid < m) bs[tid] = p.b[static_cast<int64_t>(i) * m + tid];
    if (p.Psi)
      for (int c = tid; c < d; c += 1024) psi_prev[c] = p.Psi[static_cast<int64_t>(i) * p.ld + c];
    if (tid == 0) failed = 0;
  }
  __syncthreads();
  int vt = 1024;                                                  // threads side by side on column vectors
  while (vt > 16 && vt / 2 >= nvec) vt >>= 1;
  const int rg_count = 1024 / vt, cv = tid % vt, rg = tid / vt;
  typedef const u32x4 __attribute__((address_space(4)))* csr_u4_ptr;
  const csr_u4_ptr round_tab = (csr_u4_ptr)(uintptr_t)p.blob;
  int k_round = p.round_k0;
  for (int it = 0; it < p.iters; ++it) {
    // residual
    for (int k = wave; k < m; k += 16) {
      const float* row = As + k * d;
      float s0 = 0.0f, s1 = 0.0f;
      int c = lane * 4;
      for (; c + 256 < d; c += 512) {
        const f32x4 a0 = *reinterpret_cast<const f32x4*>(row + c), x0 = *reinterpret_cast<const f32x4*>(xs + c);
        const f32x4 a1 = *reinterpret_cast<const f32x4*>(row + c + 256), x1 = *reinterpret_cast<const f32x4*>(xs + c + 256);
        s0 = fmaf(a0.x, x0.x, s0); s0 = fmaf(a0.y, x0.y, s0); s0 = fmaf(a0.z, x0.z, s0); s0 = fmaf(a0.w, x0.w, s0);
        s1 = fmaf(a1.x, x1.x, s1); s1 = fmaf(a1.y, x1.y, s1); s1 = fmaf(a1.z, x1.z, s1); s1 = fmaf(a1.w, x1.w, s1);
      }
      if (c < d) {
        const f32x4 a0 = *reinterpret_cast<const f32x4*>(row + c), x0 = *reinterpret_cast<const f32x4*>(xs + c);
        s0 = fmaf(a0.x, x0.x, s0); s0 = fmaf(a0.y, x0.y, s0); s0 = fmaf(a0.z, x0.z, s0); s0 = fmaf(a0.w, x0.w, s0);
      }
      float sum = s0 + s1;
#pragma unroll
      for (int o = 32; o > 0; o >>= 1) sum += __shfl_xor(sum, o, 64);
      if (lane == 0) resid[k] = sum - bs[k];
    }
    __syncthreads();
    // half step, published for the neighbors
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    if (cv < nvec) {
      for (int k = rg; k < m; k += rg_count) {
        const f32x4 a = *reinterpret_cast<const f32x4*>(As + k * d + (cv << 2));
        const float r = resid[k];
        acc.x = fmaf(a.x, r, acc.x); acc.y = fmaf(a.y, r, acc.y); acc.z = fmaf(a.z, r, acc.z); acc.w = fmaf(a.w, r, acc.w);
      }
    }
    part[tid] = acc;
    __syncthreads();
    float* hbase = p.H + (static_cast<int64_t>(it & 1) * p.n) * p.ld;
    if (rg == 0 && cv < nvec) {
      for (int q = 1; q < rg_count; ++q) {
        const f32x4 t = part[q * vt + cv];
        acc.x += t.x; acc.y += t.y; acc.z += t.z; acc.w += t.w;
      }
      const f32x4 x = *reinterpret_cast<const f32x4*>(xs + (cv << 2));
      float hv[4] = {fmaf(-p.alpha, acc.x, x.x), fmaf(-p.alpha, acc.y, x.y), fmaf(-p.alpha, acc.z, x.z),
                     fmaf(-p.alpha, acc.w, x.w)};
      if (p.Psi) {
        // Exact-Diffusion (eqs. ed-1, ed-2): psi = x - alpha g;  phi = psi + x - psi_prev is what goes out
        const float xv[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float psi = hv[e];
          hv[e] = (psi + xv[e]) - psi_prev[(cv << 2) + e];
          psi_prev[(cv << 2) + e] = psi;
        }
      }
      float* h = hbase + static_cast<int64_t>(i) * p.ld + (cv << 2);
#pragma unroll
      for (int e = 0; e < 4; ++e) __hip_atomic_store(h + e, hv[e], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    // Grid barrier number it+1.  Why the neighbors see the half steps: they went out as AGENT-scope
    // atomic stores, i.e. each store is itself performed at the memory the XCDs share, not just in
    // this XCD's L2.  The workgroup-scope release fence makes every wave wait until its own stores
    // have been acknowledged from there (on this hardware: s_waitcnt vmcnt(0); the scope of a fence
    // decides which caches are written back, not how long outstanding stores are waited for); the
    // workgroup barrier orders all those waits before thread 0's arrival, which is an agent-scope
    // release on the counter.  In the memory model's terms: store -> workgroup release fence ->
    // barrier -> agent-scope release is one happens-before chain (release is cumulative), and the
    // reader's agent-scope acquire after seeing the counter completes it.  An agent-scope fence per
    // wave instead was measured: 6.4 us per iteration against 4.6, for no additional guarantee.
    // Thread 0 polls with relaxed loads (an acquire load per poll would invalidate the L2 each time)
    // and takes one agent-scope acquire fence at the end.
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __syncthreads();
    if (tid == 0) {
      __hip_atomic_fetch_add(p.sync, 1u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
      const unsigned int target = static_cast<unsigned int>(p.n) * static_cast<unsigned int>(it + 1) + p.extra_arrivals;
      uint32_t polls = 0;
      while (__hip_atomic_load(p.sync, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < target) {
        if (++polls > p.spin_limit || __hip_atomic_load(p.sync + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u) {
          __hip_atomic_store(p.sync + 1, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          failed = 1;
          break;
        }
        __builtin_amdgcn_s_sleep(1);
      }
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
    }
    __syncthreads();
    if (failed) break;                                            // uniform: every thread reads the same LDS word
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
    // combine (eq. dgd-2) in list order
    const u32x4 offs = round_tab[k_round];
    const csr_i32_ptr rp = (csr_i32_ptr)(reinterpret_cast<uintptr_t>(p.blob) + offs.x);
    const csr_ent_ptr en = (csr_ent_ptr)(reinterpret_cast<uintptr_t>(p.blob) + offs.y);
    k_round = k_round + 1 == p.nrounds ? 0 : k_round + 1;
    const int beg = rp[i], end = rp[i + 1];
    for (int c = tid; c < d; c += 1024) {
      float a = 0.0f;
      // up to eight neighbors' values are requested before the first is used: each is a round trip
      // to the memory the XCDs share
      for (int q0 = beg; q0 < end; q0 += 8) {
        const int cnt = end - q0 < 8 ? end - q0 : 8;
        float hv[8], wv[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          if (u < cnt) {
            const u32x2 e = en[q0 + u];
            wv[u] = __uint_as_float(e.y);
            hv[u] = __hip_atomic_load(hbase + static_cast<int64_t>(e.x) * p.ld + c, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          }
        }
#pragma unroll
        for (int u = 0; u < 8; ++u)
          if (u < cnt) a = fmaf(wv[u], hv[u], a);
      }
      xs[c] = a;
    }
    __syncthreads();
  }
  for (int c = tid; c < d; c += 1024) p.X[static_cast<int64_t>(i) * p.ld + c] = xs[c];
  if (p.Psi)
    for (int c = tid; c < d; c += 1024) p.Psi[static_cast<int64_t>(i) * p.ld + c] = psi_prev[c];
}

__global__ void bf_sync_clear_kernel(unsigned int* sync) {
  if (threadIdx.x < 2) sync[threadIdx.x] = 0u;
}

// Scratch of the entry point that may not allocate (bf_dgd_least_squares_run_static): the double
// buffered half steps, then the two barrier words.  One copy per device, held until the process
// ends.  In host code the array's name is only a handle; the device address comes from
// hipGetSymbolAddress, once per device, and is what kernels and copies are given.
constexpr size_t kStaticHalfStepBytes = size_t{2} << 20;          // 2 * n * ld * 4 must fit
constexpr size_t kStaticScratchBytes = kStaticHalfStepBytes + 256;
static __device__ __align__(256) unsigned char bf_static_scratch[kStaticScratchBytes];

int static_scratch_address(int dev, unsigned char** out) {
  static std::mutex mu;
  static std::vector<std::pair<int, unsigned char*>> known;       // device -> address of its copy
  std::lock_guard<std::mutex> lk(mu);
  for (auto& k : known)
    if (k.first == dev) { *out = k.second; return BF_OK; }
  void* ptr = nullptr;
  BF_HIP_TRY(hipGetSymbolAddress(&ptr, HIP_SYMBOL(bf_static_scratch)));   // of the current device, which is dev
  known.emplace_back(dev, static_cast<unsigned char*>(ptr));
  *out = static_cast<unsigned char*>(ptr);
  return BF_OK;
}

// ---------------------------------------------------------------------------------------------
// Plain streaming kernels with 128-bit accesses: the practical ceilings (copy, read only, write
// only) that the mixing kernels' bandwidth is compared with.  Persistent grid-stride loops, four
// vectors in flight per thread, non-temporal hints.
template <int MODE>
__global__ __launch_bounds__(256) void bf_stream_probe_kernel(const f32x4* src, f32x4* dst, int64_t n4) {
  const int64_t stride = static_cast<int64_t>(gridDim.x) * 256;
  int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
  const f32x4 fill = {1.f, 2.f, 3.f, 4.f};
  for (; i + 3 * stride < n4; i += 4 * stride) {
    f32x4 v[4];
    if constexpr (MODE != 2) {
#pragma unroll
      for (int u = 0; u < 4; ++u) v[u] = __builtin_nontemporal_load(src + i + u * stride);
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      if constexpr (MODE == 0) __builtin_nontemporal_store(v[u], dst + i + u * stride);
      else if constexpr (MODE == 1) acc += v[u];
      else __builtin_nontemporal_store(fill, dst + i + u * stride);
    }
  }
  for (; i < n4; i += stride) {
    if constexpr (MODE == 0) dst[i] = src[i];
    else if constexpr (MODE == 1) acc += src[i];
    else dst[i] = fill;
  }
  if constexpr (MODE == 1) {
    // one partial sum per thread of the first workgroup's worth of slots keeps the loads alive
    if (acc.x + acc.y + acc.z + acc.w == 0.12345f) dst[blockIdx.x] = acc;
  }
}

// ---------------------------------------------------------------------------------------------
// Consensus diagnostics in fp64: one thread per column, two passes over the n rows.
__global__ void bf_stats_clear_kernel(double* stats) {
  if (threadIdx.x < 3) stats[threadIdx.x] = 0.0;
}

__device__ __forceinline__ void atomic_max_nonneg(double* addr, double v) {
  // non-negative doubles order like their bit patterns
  atomicMax(reinterpret_cast<unsigned long long*>(addr), static_cast<unsigned long long>(__double_as_longlong(v)));
}

template <int DT>
__global__ __launch_bounds__(256) void bf_stats_kernel(const char* X, const float* p, int n, int64_t d, int64_t ld,
                                                      int block_log, double* stats, float* mean_out) {
  __shared__ double red[3][4];
  double ss = 0.0, mdev = 0.0, mabs = 0.0;
  for (int64_t c = blockIdx.x * static_cast<int64_t>(blockDim.x) + threadIdx.x; c < d;
       c += static_cast<int64_t>(gridDim.x) * blockDim.x) {
    // column blocks: column c of agent i is at i * ld + c plus the start of its block (ld = block width)
    const int64_t co = c + (block_log ? ((c >> block_log) * (n - 1)) << block_log : int64_t{0});
    double sum = 0.0;
    for (int i = 0; i < n; ++i) {
      float v;
      load_in<DT, 1>(X, static_cast<int64_t>(i) * ld + co, &v);
      sum += p ? static_cast<double>(v) / static_cast<double>(p[i]) : static_cast<double>(v);
    }
    const double mean = sum / n;
    if (mean_out) mean_out[c] = static_cast<float>(mean);
    for (int i = 0; i < n; ++i) {
      float v;
      load_in<DT, 1>(X, static_cast<int64_t>(i) * ld + co, &v);
      const double y = p ? static_cast<double>(v) / static_cast<double>(p[i]) : static_cast<double>(v);
      const double dev = fabs(y - mean);
      ss += dev * dev;
      mdev = fmax(mdev, dev);
      mabs = fmax(mabs, fabs(y));
    }
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    ss += __shfl_xor(ss, o, 64);
    mdev = fmax(mdev, __shfl_xor(mdev, o, 64));
    mabs = fmax(mabs, __shfl_xor(mabs, o, 64));
  }
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  if (lane == 0) { red[0][wave] = ss; red[1][wave] = mdev; red[2][wave] = mabs; }
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int w = 1; w < 4; ++w) { ss += red[0][w]; mdev = fmax(mdev, red[1][w]); mabs = fmax(mabs, red[2][w]); }
    atomicAdd(&stats[0], ss);
    atomic_max_nonneg(&stats[1], mdev);
    atomic_max_nonneg(&stats[2], mabs);
  }
}

// ---------------------------------------------------------------------------------------------
// Host side: device copies of a topology, launch-shape heuristic, argument checks.

struct DeviceInfo {
  int cus = 0;
  size_t lds_per_cu = 0;
  size_t lds_per_block_optin = 0;
};

int device_info(int dev, DeviceInfo* out) {
  static std::mutex mu;
  static std::vector<std::pair<int, DeviceInfo>> cache;
  std::lock_guard<std::mutex> lk(mu);
  for (auto& c : cache)
    if (c.first == dev) { *out = c.second; return BF_OK; }
  hipDeviceProp_t prop;
  BF_HIP_TRY(hipGetDeviceProperties(&prop, dev));
  DeviceInfo di;
  di.cus = prop.multiProcessorCount;
  di.lds_per_cu = prop.maxSharedMemoryPerMultiProcessor;
  di.lds_per_block_optin = prop.sharedMemPerBlock;
  int v = 0;
  if (hipDeviceGetAttribute(&v, hipDeviceAttributeSharedMemPerBlockOptin, dev) == hipSuccess && v > 0)
    di.lds_per_block_optin = std::max<size_t>(di.lds_per_block_optin, static_cast<size_t>(v));
  cache.emplace_back(dev, di);
  *out = di;
  return BF_OK;
}

int get_device_copy(bf_topology_t* t, bool need_dense, bf::DeviceCopy** out) {
  int dev = 0;
  BF_HIP_TRY(hipGetDevice(&dev));
  std::lock_guard<std::mutex> lk(t->mu);
  bf::DeviceCopy* dc = nullptr;
  for (auto& c : t->dev)
    if (c.device == dev) dc = &c;
  if (!dc) {
    bf::DeviceCopy c;
    c.device = dev;
    // Head of the blob: four byte offsets per round {rowptr, entries, slice headers, slice entries},
    // for kernels that walk several rounds themselves.  The sliced copy of a round groups rows in
    // fours: a header {first 32-byte record, number of records, 1 if the four rows differ in
    // length} per group, and per record the q-th entry of each of the four rows side by side
    // {col, weight} x 4, so one 32-byte scalar load feeds four rows.  A row shorter than its group
    // is filled with {0x80000000 | row, 0}, which the kernel skips.
    const size_t ngroups = (static_cast<size_t>(t->n) + 3) / 4;
    size_t bytes = (t->rounds.size() * 16 + 31) / 32 * 32;
    std::vector<size_t> slice_hdr_off, slice_ent_off;
    std::vector<std::vector<uint32_t>> slice_hdr(t->rounds.size()), slice_ent(t->rounds.size());
    for (size_t k = 0; k < t->rounds.size(); ++k) {
      auto& r = t->rounds[k];
      c.rowptr_off.push_back(bytes);
      bytes += ((static_cast<size_t>(t->n) + 1 + 1) / 2) * 8;
      c.entry_off.push_back(bytes);
      bytes += r.col.size() * 8;
      bytes = (bytes + 31) / 32 * 32;
      c.chain_off.push_back(r.chain.empty() ? SIZE_MAX : bytes);
      bytes += r.chain.size() * sizeof(bf::ChainStep);
      bytes = (bytes + 31) / 32 * 32;
      auto& hdr = slice_hdr[k];
      auto& ent = slice_ent[k];
      for (size_t g = 0; g < ngroups; ++g) {
        int64_t longest = 0, shortest = INT64_MAX;
        for (size_t u = 0; u < 4; ++u) {
          const size_t row = g * 4 + u;
          const int64_t len = row < static_cast<size_t>(t->n) ? r.rowptr[row + 1] - r.rowptr[row] : 0;
          longest = std::max(longest, len);
          shortest = std::min(shortest, len);
        }
        hdr.push_back(static_cast<uint32_t>(ent.size() / 8));
        hdr.push_back(static_cast<uint32_t>(longest));
        hdr.push_back(shortest != longest ? 1u : 0u);
        hdr.push_back(0u);
        for (int64_t q = 0; q < longest; ++q)
          for (size_t u = 0; u < 4; ++u) {
            const size_t row = std::min(g * 4 + u, static_cast<size_t>(t->n) - 1);
            const bool live = g * 4 + u < static_cast<size_t>(t->n) && r.rowptr[row] + q < r.rowptr[row + 1];
            uint32_t wbits = 0;
            if (live) std::memcpy(&wbits, &r.wgt[r.rowptr[row] + q], 4);
            ent.push_back(live ? static_cast<uint32_t>(r.col[r.rowptr[row] + q]) : (0x80000000u | static_cast<uint32_t>(row)));
            ent.push_back(wbits);
          }
      }
      slice_hdr_off.push_back(bytes);
      bytes += (hdr.size() * 4 + 31) / 32 * 32;
      slice_ent_off.push_back(bytes);
      bytes += (ent.size() * 4 + 31) / 32 * 32;
    }
    bytes += 64;   // wide scalar loads may read past the last record
    if (bytes > UINT32_MAX) return BF_ERR_SIZE;
    std::vector<char> host(bytes, 0);
    for (size_t k = 0; k < t->rounds.size(); ++k) {
      auto& r = t->rounds[k];
      uint32_t* tab = reinterpret_cast<uint32_t*>(host.data());
      tab[4 * k] = static_cast<uint32_t>(c.rowptr_off[k]);
      tab[4 * k + 1] = static_cast<uint32_t>(c.entry_off[k]);
      tab[4 * k + 2] = static_cast<uint32_t>(slice_hdr_off[k]);
      tab[4 * k + 3] = static_cast<uint32_t>(slice_ent_off[k]);
      if (!slice_hdr[k].empty()) std::memcpy(host.data() + slice_hdr_off[k], slice_hdr[k].data(), slice_hdr[k].size() * 4);
      if (!slice_ent[k].empty()) std::memcpy(host.data() + slice_ent_off[k], slice_ent[k].data(), slice_ent[k].size() * 4);
      int32_t* rp = reinterpret_cast<int32_t*>(host.data() + c.rowptr_off[k]);
      for (int32_t i = 0; i <= t->n; ++i) rp[i] = static_cast<int32_t>(r.rowptr[i]);
      uint32_t* en = reinterpret_cast<uint32_t*>(host.data() + c.entry_off[k]);
      for (size_t q = 0; q < r.col.size(); ++q) {
        en[2 * q] = static_cast<uint32_t>(r.col[q]);
        std::memcpy(&en[2 * q + 1], &r.wgt[q], 4);
      }
      if (!r.chain.empty()) std::memcpy(host.data() + c.chain_off[k], r.chain.data(), r.chain.size() * sizeof(bf::ChainStep));
    }
    BF_HIP_TRY(hipMalloc(reinterpret_cast<void**>(&c.blob), std::max<size_t>(bytes, 16)));
    hipError_t e = hipMemcpy(c.blob, host.data(), bytes, hipMemcpyHostToDevice);
    if (e != hipSuccess) { (void)hipFree(c.blob); g_last_hip_error = e; return BF_ERR_HIP; }
    t->dev.push_back(std::move(c));
    dc = &t->dev.back();
  }
  if (need_dense && !dc->dense_t) {
    const int32_t n_pad = (t->n + 31) / 32 * 32;
    const size_t per = static_cast<size_t>(n_pad) * n_pad;
    std::vector<float> host(per * t->rounds.size());
    for (size_t k = 0; k < t->rounds.size(); ++k) bf::dense_transposed(t->rounds[k], t->n, n_pad, host.data() + per * k);
    float* dptr = nullptr;
    BF_HIP_TRY(hipMalloc(reinterpret_cast<void**>(&dptr), host.size() * sizeof(float)));
    hipError_t e = hipMemcpy(dptr, host.data(), host.size() * sizeof(float), hipMemcpyHostToDevice);
    if (e != hipSuccess) { (void)hipFree(dptr); g_last_hip_error = e; return BF_ERR_HIP; }
    dc->dense_t = dptr;
    dc->n_pad = n_pad;
  }
  *out = dc;
  return BF_OK;
}

int g_tune_tile = 0;      // column-tile width override (elements)
int g_tune_wgs = 0;       // workgroups per CU override
int g_tune_gather = 0;    // 1: force the gather fallback
int g_tune_grid = 0;      // total workgroups override (capped by the resident slots)
int g_tune_nochain = 0;   // 1: never use the chain kernel
int g_tune_noserp = 0;    // 1: always walk tiles left to right
int g_tune_chain256 = 0;  // 1: chain kernel never uses 1024-thread workgroups
int g_tune_stream = 0;    // 1: always non-temporal, 2: never
int g_tune_cw = 0;        // chain kernel: 16-byte vectors per thread (1, 2 or 4)
int g_tune_spin = 0;      // polls a grid-barrier wait may take before it gives up (0: default)
int g_tune_extra = 0;     // 1: the grid barrier waits for an arrival that never comes (give-up test)
int g_tune_noshift = 0;   // 1: fused rounds never take the in-register form, 2: whenever it applies
int g_tune_pipe = 0;      // 1: the pipelined kernel also for cache-resident rounds, 2: never
int g_tune_awc = 0;       // 1: AWC on the pipelined kernel always fetches its own gradient from HBM


int ilog2(int64_t v) { int l = 0; while ((int64_t{1} << (l + 1)) <= v) ++l; return l; }

// Choose the tile: the widest power-of-two C in [64, 1024] whose n x C fp32 tile fits the LDS share
// of one of `wgs` workgroups per CU (two 1024-thread workgroups per CU when possible, so one can
// stream while the other reduces), narrowed while the launch would leave workgroup slots idle.
int choose_shape(int n, int64_t d, const DeviceInfo& di, Shape* s, int max_wgs = 2, int max_log_c = 10) {
  const size_t lds_cu = di.lds_per_cu ? di.lds_per_cu : 65536;
  const size_t lds_blk = di.lds_per_block_optin ? di.lds_per_block_optin : lds_cu;
  int wgs = g_tune_wgs > 0 ? g_tune_wgs : max_wgs;
  int log_c = -1;
  if (g_tune_tile > 0) {
    const int lc = ilog2(g_tune_tile);
    if ((1 << lc) != g_tune_tile || lc < 6 || lc > 10) return BF_ERR_UNSUPPORTED;
    const size_t bytes = static_cast<size_t>(n) * g_tune_tile * 4;
    if (bytes > lds_blk || bytes > lds_cu || lc > max_log_c) return BF_ERR_UNSUPPORTED;
    if (g_tune_wgs == 0) wgs = static_cast<int>(std::max<size_t>(1, lds_cu / bytes));
    if (bytes * wgs > lds_cu) return BF_ERR_UNSUPPORTED;
    log_c = lc;
  } else {
    auto widest = [&](int w) {
      const size_t budget = std::min(lds_cu / w, lds_blk);
      for (int lc = max_log_c; lc >= 6; --lc)
        if (static_cast<size_t>(n) * (size_t{1} << lc) * 4 <= budget) return lc;
      return -1;
    };
    for (; wgs >= 1; --wgs) {
      log_c = widest(wgs);
      if (log_c >= 0) break;
    }
    if (log_c < 0) return BF_ERR_UNSUPPORTED;
    wgs = std::max(wgs, 1);
    // 64-column tiles use 256 bytes of each of n row pages (12 % TLB misses at n = 256): one
    // workgroup per CU with a tile twice as wide is faster there (58 % vs 45-57 % of peak).
    if (g_tune_wgs == 0 && wgs == 2 && log_c == 6 && widest(1) > 6) { wgs = 1; log_c = widest(1); }
    const int64_t slots = static_cast<int64_t>(di.cus) * std::min(wgs, 2);
    while (log_c > 6 && ((d + (int64_t{1} << log_c) - 1) >> log_c) < slots) --log_c;
  }
  s->log_c = log_c;
  s->lw = log_c >= 8 ? 4 : (log_c == 7 ? 2 : 1);
  s->threads = 1024;
  s->wgs_per_cu = std::max(1, std::min(wgs, 2048 / s->threads));
  s->lds_bytes = static_cast<size_t>(n) * (size_t{1} << log_c) * 4;
  return BF_OK;
}

// Tile of the pipelined kernel: two n x C fp32 tiles share one CU's LDS; the widest power-of-two C in
// [64, 1024] that fits, narrowed while the launch would leave CUs without a tile.
int choose_pipe_shape(int n, int64_t d, const DeviceInfo& di, Shape* s, int max_log_c = 10) {
  const size_t lds_cu = di.lds_per_cu ? di.lds_per_cu : 65536;
  const size_t budget = std::min(lds_cu, di.lds_per_block_optin ? di.lds_per_block_optin : lds_cu);
  int log_c = -1;
  if (g_tune_tile > 0) {
    const int lc = ilog2(g_tune_tile);
    if ((1 << lc) != g_tune_tile || lc < 6 || lc > 10) return BF_ERR_UNSUPPORTED;
    if (2 * static_cast<size_t>(n) * g_tune_tile * 4 > budget || lc > max_log_c) return BF_ERR_UNSUPPORTED;
    log_c = lc;
  } else {
    for (int lc = max_log_c; lc >= 6 && log_c < 0; --lc)
      if (2 * static_cast<size_t>(n) * (size_t{1} << lc) * 4 <= budget) log_c = lc;
    if (log_c < 0) return BF_ERR_UNSUPPORTED;
    while (log_c > 6 && ((d + (int64_t{1} << log_c) - 1) >> log_c) < di.cus) --log_c;
  }
  s->log_c = log_c;
  s->lw = log_c >= 8 ? 4 : (log_c == 7 ? 2 : 1);
  s->threads = 0;
  s->wgs_per_cu = 1;
  s->lds_bytes = 2 * static_cast<size_t>(n) * (size_t{1} << log_c) * 4;
  return BF_OK;
}

// Overlap test on byte ranges [a, a+na) and [b, b+nb).
bool overlaps(const void* a, size_t na, const void* b, size_t nb) {
  const uintptr_t pa = reinterpret_cast<uintptr_t>(a), pb = reinterpret_cast<uintptr_t>(b);
  return pa < pb + nb && pb < pa + na;
}

struct MatArgs {
  int64_t d, ld; int dt; int n;
  size_t bytes;       // extent of a matrix of the call's element type
  int block_log;      // 0: agent-major; else log2 of the block width of the column-block layout
  // extent of a matrix of `eb`-byte elements in the same layout (momentum and the like are fp32)
  size_t extent(int eb) const {
    if (block_log) return static_cast<size_t>((d + ld - 1) / ld) * n * ld * eb;
    return static_cast<size_t>(n - 1) * ld * eb + ((static_cast<size_t>(d) * eb + 15) & ~size_t{15});
  }
};

// Common checks of an n x d matrix argument set.  A negative ld = -B names the column-block layout
// with blocks of B columns (a power of two in [64, 2^20]): accepted only where the caller says so,
// else BF_ERR_UNSUPPORTED.  ma->ld is then B.  ma->bytes is what the kernels may touch: for
// agent-major rows whole 16-byte vectors up to the one that holds column d-1, for column blocks
// every block in full.
int check_matrix_shape(int32_t n, int64_t d, int64_t ld, int dt, MatArgs* ma, bool blocked_ok = false) {
  if (dt != BF_F32 && dt != BF_BF16) return BF_ERR_KIND;
  const int eb = dt == BF_F32 ? 4 : 2;
  ma->d = d; ma->dt = dt; ma->n = n; ma->block_log = 0;
  if (ld < 0) {
    const int64_t blk = -ld;
    if (d < 0 || blk < 64 || blk > (int64_t{1} << 20) || (blk & (blk - 1)) != 0 || d > (int64_t{1} << 40)) return BF_ERR_SIZE;
    if (!blocked_ok) return BF_ERR_UNSUPPORTED;
    ma->ld = blk;
    ma->block_log = ilog2(blk);
    ma->bytes = ma->extent(eb);
    return BF_OK;
  }
  if (d < 0 || ld < d || ld < 1 || ld > (int64_t{1} << 40)) return BF_ERR_SIZE;
  if ((ld * eb) % 16 != 0) return BF_ERR_ALIGN;
  ma->ld = ld;
  ma->bytes = ma->extent(eb);
  return BF_OK;
}

bool misaligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

// Choose the kernel for one call and launch it.  With `dry` set nothing is launched: the return
// value then only says whether a kernel exists for the request, so that an entry point made of
// several launches can find out before the first of them touches the caller's data.
int run_tile(bf_topology_t* t, int32_t round, int op, bool with_y, TileParams tp, int dt, hipStream_t st, bool dry = false) {
  if (tp.d == 0) return BF_OK;
  bf::DeviceCopy* dc = nullptr;
  int rc = get_device_copy(t, false, &dc);
  if (rc != BF_OK) return rc;
  DeviceInfo di;
  rc = device_info(dc->device, &di);
  if (rc != BF_OK) return rc;
  const size_t k = static_cast<size_t>(round) % t->rounds.size();
  tp.rowptr = reinterpret_cast<const int32_t*>(dc->blob + dc->rowptr_off[k]);
  tp.ent = reinterpret_cast<const u32x2*>(dc->blob + dc->entry_off[k]);
  tp.n = t->n;
  tp.long_rows = t->rounds[k].max_degree >= 5 ? 1 : 0;
  tp.reverse = g_tune_noserp ? 0 : (round & 1);
  const int fuse = tp.fuse > 1 ? tp.fuse : 1;
  tp.fuse = fuse;
  if (fuse > 1) {
    // Several consecutive rounds in one pass: the earlier rounds' lists go in the side arrays, the
    // last round's in the usual place.  Only the plain mix has this form.
    if (op != OP_MIX || with_y || fuse > 8) return BF_ERR_UNSUPPORTED;
    tp.blob = dc->blob;
    tp.round_k0 = static_cast<int32_t>(k);
    tp.nrounds = static_cast<int32_t>(t->rounds.size());
    const size_t kl = (static_cast<size_t>(round) + fuse - 1) % t->rounds.size();
    tp.rowptr = reinterpret_cast<const int32_t*>(dc->blob + dc->rowptr_off[kl]);
    tp.ent = reinterpret_cast<const u32x2*>(dc->blob + dc->entry_off[kl]);
    tp.reverse = g_tune_noserp ? 0 : ((round / fuse) & 1);
  }
  // Column-block layout: tiles stay inside a block (so do the chain kernel's sweeps of one 16-byte
  // vector per thread), and the gather fallback, which walks whole rows, does not apply.
  if (tp.g_ld == 0) { tp.g_ld = tp.ld; tp.g_block_log = tp.block_log; }     // gradients and state matrix laid out like X
  if (tp.m_ld == 0) { tp.m_ld = tp.ld; tp.m_block_log = tp.block_log; }
  const bool same_layout = tp.g_ld == tp.ld && tp.g_block_log == tp.block_log && tp.m_ld == tp.ld && tp.m_block_log == tp.block_log;
  const bool blocked = tp.block_log > 0;
  const int64_t block_cols = blocked ? int64_t{1} << tp.block_log : INT64_MAX;
  const int cap_log_c = blocked ? std::min(tp.block_log, 10) : 10;
  // (On column blocks the pipelined kernel keeps the lead up to 128-column tiles: n = 128 one-peer
  // rounds on blocks of 8192 measure 6.2 TB/s there against 5.9 for the chain kernel at its best
  // block width; on agent-major rows the chain kernel wins from 256-column tiles down.)
  const size_t lds_cu_bytes = di.lds_per_cu ? di.lds_per_cu : 65536;
  const bool chain_pays = blocked ? 2 * static_cast<size_t>(t->n) * 128 * 4 > lds_cu_bytes
                                  : static_cast<size_t>(t->n) * 256 * 4 > lds_cu_bytes / 2;
  if (fuse == 1 && dc->chain_off[k] != SIZE_MAX && !g_tune_nochain && !g_tune_gather && (g_tune_cw > 0 || chain_pays)) {
    // Chain-structured round with too many agents for a 256-column LDS tile (measured: the tile
    // kernels win below that, the row-streaming kernel above): stream rows through registers when
    // the matrix is wide enough to give every CU several 256-thread workgroups.
    const int per16 = dt == BF_F32 ? 4 : 8;
    int cw = g_tune_cw > 0 ? g_tune_cw : (dt == BF_F32 ? 4 : 2);
    if (cw != 1 && cw != 2 && cw != 4) return BF_ERR_UNSUPPORTED;
    if (dt != BF_F32 && cw == 4) cw = 2;
    // Widest first: 1024 threads x 4 vectors read 64 KB of a row per step (a plain row-walk copy
    // peaks there: 5.55 TB/s vs 5.35 with 16 KB); needs at least one such chunk per CU.
    const int64_t wide_cols = static_cast<int64_t>(1024) * per16 * (dt == BF_F32 ? 4 : 2);
    const int64_t wide_chunks = (tp.d + wide_cols - 1) / wide_cols;
    const bool wide = g_tune_cw == 0 && !g_tune_chain256 && wide_chunks >= di.cus && op != OP_MOM_ATC && op != OP_ED &&
                      block_cols >= 1024 * per16;
    const int64_t chunk_cols = wide ? wide_cols : static_cast<int64_t>(256) * per16 * cw;
    const int64_t nchunks = (tp.d + chunk_cols - 1) / chunk_cols;
    if ((nchunks >= 2 * static_cast<int64_t>(di.cus) || g_tune_cw > 0 || wide) && block_cols >= 256 * per16) {
      if (dry) return BF_OK;
      tp.chain = reinterpret_cast<const bf::ChainStep*>(dc->blob + dc->chain_off[k]);
      int grid = static_cast<int>(std::min<int64_t>(nchunks, static_cast<int64_t>(di.cus) * (wide ? 1 : 8)));
      if (g_tune_grid > 0) grid = std::min(grid, g_tune_grid);
      return dt == BF_F32 ? launch_chain_f32(op, with_y, cw, wide, tp, nchunks, grid, st)
                          : launch_chain_bf16(op, with_y, cw, wide, tp, nchunks, grid, st);
    }
  }
  // Cache policy.  MI355X has a 256 MB memory-side cache.  An in-place update whose whole state
  // is about that size is best left cacheable (the next round, walking the tiles in the opposite
  // direction, finds most of it there: measured 71 % vs 65 % of HBM peak on 64 x 2^20 fp32);
  // anything larger, or out of place, streams with non-temporal loads and stores.
  bool cacheable = false;
  {
    const size_t eb = dt == BF_F32 ? 4 : 2;
    const size_t row_elems = blocked ? static_cast<size_t>((tp.d + tp.ld - 1) / tp.ld * tp.ld) : static_cast<size_t>(tp.ld);
    size_t footprint = static_cast<size_t>(t->n) * row_elems * eb;
    if (tp.g) footprint *= 2;
    if (tp.g2) footprint += static_cast<size_t>(t->n) * row_elems * eb;
    if (tp.m) footprint += static_cast<size_t>(t->n) * row_elems * 4;
    cacheable = tp.x_in == tp.x_out && footprint <= (size_t{320} << 20);
  }
  const bool stream = g_tune_stream == 1 ? true : (g_tune_stream == 2 ? false : !cacheable);
  if (fuse == 1 && !g_tune_gather && (g_tune_pipe == 1 || (g_tune_pipe == 0 && stream))) {
    // One streaming round: the pipelined kernel (loader waves and reducer waves, two LDS tiles per
    // CU) measures 2-3 points of HBM peak above the one-tile kernel on matrices that do not fit the
    // memory-side cache.  A cache-resident in-place round is left to the one-tile kernel, whose two
    // workgroups per CU do better there (76 % vs 75 % on 64 x 2^20).
    Shape ps;
    // (column blocks: tiles of 512 columns below 32 agents and 256 from there on measure best --
    // n = 8: 512 columns 6.2 TB/s, 1024 6.0, 256 3.1; n = 32: 256 columns 6.04, 512 5.67)
    const int pipe_cap = blocked ? std::min(cap_log_c, t->n < 32 ? 9 : 8) : cap_log_c;
    bool pipe_fits = choose_pipe_shape(t->n, tp.d, di, &ps, pipe_cap) == BF_OK;
    if (pipe_fits && ps.log_c < 7 && g_tune_pipe != 1) {
      // More than 160 agents leave the two tiles 64 columns each (256-byte row pieces, one column per
      // lane in the reduce phase).  The one-tile kernel gets 128 columns there and measures 10-60 %
      // faster (n = 256, static exponential graph, bf16 momentum step: 4.0 against 3.2 TB/s; fp32
      // ATC 4.9 against 4.3), so it takes those sizes.
      Shape ts;
      if (choose_shape(t->n, tp.d, di, &ts, 2, cap_log_c) == BF_OK && ts.log_c > ps.log_c) pipe_fits = false;
    }
    if (pipe_fits) {
      if (dry) return BF_OK;
      // AWC with bf16 storage: the reducers are short of issue slots, and fetching their own gradient
      // from HBM between their stores costs them a third of their rate.  Where n more fp32 rows fit
      // each LDS tile at 256 columns or more (or without narrowing it), the loaders stage the gradients there instead (n = 32,
      // static exponential graph: 4.2 -> 5.6 TB/s on column blocks, 4.1 -> 5.2 on agent-major rows,
      // where the tile narrows from 512 to 256 columns).  With fp32 storage the reducers have the
      // slots and the loaders the bytes: the fetch from HBM measures the same or better (n = 32: 6.36
      // against 6.17 TB/s), so it stays.
      int pipe_op = op;
      if (op == OP_AWC && dt == BF_BF16 && !g_tune_awc) {
        Shape ps2;
        if (choose_pipe_shape(2 * t->n, tp.d, di, &ps2, pipe_cap) == BF_OK && (ps2.log_c >= 8 || ps2.log_c == ps.log_c)) { ps = ps2; pipe_op = OP_AWC_LDS; }
      }
      ps.stream = stream;
      tp.log_c = ps.log_c;
      tp.ntiles = (tp.d + (int64_t{1} << ps.log_c) - 1) >> ps.log_c;
      // Two workgroups per CU where both fit: the plain mix stays within 64 registers, and with small
      // tiles (32 agents and fewer) two pairs of LDS tiles fit a CU.  That doubles the reducer waves,
      // which is what a bf16 mix is short of (n = 32: 3.3 -> 4.0 TB/s); fp32 mixes do not change.
      const size_t lds_cu_pipe = std::min(di.lds_per_cu ? di.lds_per_cu : size_t{65536},
                                          di.lds_per_block_optin ? di.lds_per_block_optin : size_t{65536});
      const int per_cu = (op == OP_MIX && g_tune_wgs != 1 && 2 * ps.lds_bytes <= lds_cu_pipe) ? 2 : 1;
      int grid = static_cast<int>(std::min<int64_t>(tp.ntiles, static_cast<int64_t>(di.cus) * per_cu));
      if (g_tune_grid > 0) grid = std::min(grid, g_tune_grid);
      return dt == BF_F32 ? launch_pipe_op_f32(pipe_op, with_y, tp, ps, grid, st)
                          : launch_pipe_op_bf16(pipe_op, with_y, tp, ps, grid, st);
    }
  }
  Shape s;
  // (the fused kernel needs more than 64 registers, so one workgroup per CU is all that runs)
  const int rows_b = fuse > 1 ? (tp.rows_b > 0 && tp.rows_b < t->n ? tp.rows_b : t->n) : 0;
  rc = g_tune_gather ? BF_ERR_UNSUPPORTED : choose_shape(t->n + rows_b, tp.d, di, &s, fuse > 1 ? 1 : 2,
                                                                 fuse > 1 ? std::min(8, cap_log_c) : cap_log_c);   // fused: 256 columns at most (512 measured slower)
  if (fuse > 1 && rc != BF_OK) return rc;   // fused rounds exist only as the two-tile LDS kernel
  if (rc == BF_ERR_UNSUPPORTED && g_tune_tile == 0) {
    // Too many agents for a 64-column LDS tile.
    const bool gatherable = tp.x_in != tp.x_out && op != OP_ED && op != OP_TRACK && !blocked && same_layout;
    if (gatherable) {
      // row gather through the caches (out of place only; no state matrix in the sum)
      if (dry) return BF_OK;
      const int per16 = dt == BF_F32 ? 4 : 8;
      const int64_t units = (tp.d + per16 - 1) / per16 * t->n;
      const int grid = static_cast<int>(std::min<int64_t>((units + 255) / 256, static_cast<int64_t>(di.cus) * 32));
      if (op == OP_MOM_ATC || op == OP_MOM_AWC) {
        const int64_t u4 = (tp.d + 3) / 4 * t->n;
        const int g2 = static_cast<int>(std::min<int64_t>((u4 + 255) / 256, static_cast<int64_t>(di.cus) * 32));
        rc = launch_momentum(dt, tp.m, tp.g, t->n, tp.d, tp.ld, tp.beta, g2, st);
        if (rc != BF_OK) return rc;
      }
      return dt == BF_F32 ? launch_gather_f32(op, with_y, tp, grid, st) : launch_gather_bf16(op, with_y, tp, grid, st);
    }
    // in place, or an op the gather cannot express: tiles of 32, 16, 8 or 4 columns
    const size_t lds_max = std::min(di.lds_per_cu ? di.lds_per_cu : size_t{65536},
                                    di.lds_per_block_optin ? di.lds_per_block_optin : size_t{65536});
    int lc = 5;
    while (lc >= 2 && static_cast<size_t>(t->n) * (size_t{1} << lc) * 4 > lds_max) --lc;
    if (lc < 2) return BF_ERR_UNSUPPORTED;
    if (dry) return BF_OK;
    tp.log_c = lc;
    tp.ntiles = (tp.d + (int64_t{1} << lc) - 1) >> lc;
    const int grid = static_cast<int>(std::min<int64_t>(tp.ntiles, static_cast<int64_t>(di.cus)));
    const size_t lds = static_cast<size_t>(t->n) * (size_t{1} << lc) * 4;
    return dt == BF_F32 ? launch_narrow_f32(op, with_y, tp, lds, grid, st) : launch_narrow_bf16(op, with_y, tp, lds, grid, st);
  }
  if (rc != BF_OK) return rc;
  if (dry) return BF_OK;
  s.stream = stream;
  tp.log_c = s.log_c;
  tp.ntiles = (tp.d + (int64_t{1} << s.log_c) - 1) >> s.log_c;
  int grid = static_cast<int>(std::min<int64_t>(tp.ntiles, static_cast<int64_t>(di.cus) * s.wgs_per_cu));
  if (g_tune_grid > 0) grid = std::min(grid, g_tune_grid);
  return dt == BF_F32 ? launch_tile_op_f32(op, with_y, tp, s, grid, st)
                      : launch_tile_op_bf16(op, with_y, tp, s, grid, st);
}

// `count` rounds in registers when every one of them is a uniform shift round and the agents fill
// whole waves (bf_shift.hip).  BF_ERR_UNSUPPORTED when the request has no such form: the caller
// then takes the general path.
int run_shift_rounds(bf_topology_t* t, int32_t round0, int32_t count, const TileParams& tp, int dt, hipStream_t st) {
  const int32_t n = t->n;
  if (g_tune_noshift == 1 || n % 64 != 0 || n > 256 || count < 1 || count > 8) return BF_ERR_UNSUPPORTED;
  // Measured at d = 2^21..2^22: with 64-column tiles (n >= 192) the register rounds always win (n = 256:
  // 1.8 / 1.8 / 2.0 ms for 2 / 4 / 8 rounds against 2.2 / 3.5 / 6.0 ms); with the wider tiles of fewer
  // agents the LDS rounds hide behind the HBM transfers for the first few rounds and win there.
  if (g_tune_noshift == 0 && ((n == 128 && count < 3) || (n == 64 && count < 5))) return BF_ERR_UNSUPPORTED;
  ShiftParams sp{};
  const size_t R = t->rounds.size();
  for (int32_t j = 0; j < count; ++j) {
    const bf::Round& r = t->rounds[(static_cast<size_t>(round0) + j) % R];
    if (r.shift <= 0 || (r.shift >= 64 && r.shift % 64 != 0)) return BF_ERR_UNSUPPORTED;   // lane part or register part, not both
    sp.shift[j] = r.shift; sp.w_self[j] = r.shift_w_self; sp.w_peer[j] = r.shift_w_peer;
  }
  int dev = 0;
  BF_HIP_TRY(hipGetDevice(&dev));
  DeviceInfo di;
  int rc = device_info(dev, &di);
  if (rc != BF_OK) return rc;
  // a 64 KB tile: n x C fp32 with C = 16384 / n (64 columns at n = 256), two workgroups per CU
  int log_c = ilog2(16384 / n);
  if (n == 192) log_c = 6;
  if (tp.block_log) log_c = std::min(log_c, tp.block_log);
  while (log_c > 6 && ((tp.d + (int64_t{1} << log_c) - 1) >> log_c) < 2 * static_cast<int64_t>(di.cus)) --log_c;
  const size_t lds = static_cast<size_t>(n) * ((size_t{1} << log_c) + 4) * 4;
  if (2 * lds + 256 > (di.lds_per_cu ? di.lds_per_cu : 65536)) return BF_ERR_UNSUPPORTED;
  sp.x_in = tp.x_in; sp.x_out = tp.x_out; sp.d = tp.d; sp.ld = tp.ld;
  sp.n = n; sp.log_c = log_c; sp.count = count; sp.block_log = tp.block_log;
  sp.ntiles = (tp.d + (int64_t{1} << log_c) - 1) >> log_c;
  sp.reverse = g_tune_noserp ? 0 : ((round0 / count) & 1);
  int grid = static_cast<int>(std::min<int64_t>(sp.ntiles, static_cast<int64_t>(di.cus) * 2));
  if (g_tune_grid > 0) grid = std::min(grid, g_tune_grid);
  return launch_shift_rounds(dt, sp, grid, lds, st);
}

// Device copy of a round's window plan, built on first use.
int get_window_plan(bf_topology_t* t, size_t k, bf::DeviceCopy* dc, WinParams* wp) {
  std::lock_guard<std::mutex> lk(t->mu);
  const size_t R = t->rounds.size();
  if (dc->win_blob.empty()) { dc->win_blob.assign(R, nullptr); dc->win_off.assign(R * 6, 0); dc->win_slots.assign(R, 0); }
  if (!dc->win_blob[k]) {
    bf::WindowPlan w;
    bf::build_window_plan(t->rounds[k], t->n, &w);
    const size_t E = w.slot_src.size();
    auto pad = [](size_t b) { return (b + 15) / 16 * 16; };
    size_t off[6];
    size_t bytes = 0;
    off[0] = bytes; bytes += pad((static_cast<size_t>(t->n) + 1) * 4);
    off[1] = bytes; bytes += pad(E * 4);
    off[2] = bytes; bytes += pad(static_cast<size_t>(t->n) * 4);
    off[3] = bytes; bytes += pad((static_cast<size_t>(t->n) + 1) * 4);
    off[4] = bytes; bytes += pad(E * 8);
    off[5] = bytes; bytes += pad(E * 4);
    std::vector<char> host(bytes + 16, 0);
    std::memcpy(host.data() + off[0], w.in_ptr.data(), w.in_ptr.size() * 4);
    if (E) std::memcpy(host.data() + off[1], w.slot_w.data(), E * 4);
    std::memcpy(host.data() + off[2], w.self_w.data(), w.self_w.size() * 4);
    std::memcpy(host.data() + off[3], w.out_ptr.data(), w.out_ptr.size() * 4);
    if (E) std::memcpy(host.data() + off[5], w.slot_src.data(), E * 4);
    uint32_t* oe = reinterpret_cast<uint32_t*>(host.data() + off[4]);
    for (size_t q = 0; q < E; ++q) {
      oe[2 * q] = static_cast<uint32_t>(w.out_slot[q]);
      std::memcpy(&oe[2 * q + 1], &w.out_w[q], 4);
    }
    char* blob = nullptr;
    BF_HIP_TRY(hipMalloc(reinterpret_cast<void**>(&blob), host.size()));
    hipError_t e = hipMemcpy(blob, host.data(), host.size(), hipMemcpyHostToDevice);
    if (e != hipSuccess) { (void)hipFree(blob); g_last_hip_error = e; return BF_ERR_HIP; }
    dc->win_blob[k] = blob;
    for (int q = 0; q < 6; ++q) dc->win_off[k * 6 + q] = off[q];
    dc->win_slots[k] = static_cast<int32_t>(E);
  }
  const char* b = dc->win_blob[k];
  const size_t* off = &dc->win_off[k * 6];
  wp->in_ptr = reinterpret_cast<const int32_t*>(b + off[0]);
  wp->slot_w = reinterpret_cast<const float*>(b + off[1]);
  wp->self_w = reinterpret_cast<const float*>(b + off[2]);
  wp->out_ptr = reinterpret_cast<const int32_t*>(b + off[3]);
  wp->out_ent = reinterpret_cast<const u32x2*>(b + off[4]);
  wp->slot_src = reinterpret_cast<const int32_t*>(b + off[5]);
  return BF_OK;
}

// Shared body of the four window calls.
int win_common(int mode, const bf_topology_t* tc, int32_t round, const int32_t* active, void* X, float* pv,
               void* Win, float* win_p, int64_t d, int64_t ld, bf_dtype_t dt, void* hip_stream,
               const float* call_self_w = nullptr, const float* call_edge_w = nullptr, const int32_t* call_edge_on = nullptr) {
  if (!tc || !X) return BF_ERR_NULL;
  if (round < 0) return BF_ERR_ROUND;
  bf_topology_t* t = const_cast<bf_topology_t*>(tc);
  const int64_t E = bf_topology_window_slots(t, round);
  if (E < 0) return static_cast<int>(E);
  // a topology without edges has no slots: Win and win_p may then be NULL
  if (E > 0 && (!Win || (pv == nullptr) != (win_p == nullptr))) return BF_ERR_NULL;
  MatArgs ma;
  int rc = check_matrix_shape(t->n, d, ld, dt, &ma, true);
  if (rc != BF_OK) return rc;
  if (misaligned16(X) || misaligned16(Win)) return BF_ERR_ALIGN;
  if ((active && (reinterpret_cast<uintptr_t>(active) & 3u)) || (pv && (reinterpret_cast<uintptr_t>(pv) & 3u)) ||
      (win_p && (reinterpret_cast<uintptr_t>(win_p) & 3u)) || (reinterpret_cast<uintptr_t>(call_self_w) & 3u) ||
      (reinterpret_cast<uintptr_t>(call_edge_w) & 3u) || (reinterpret_cast<uintptr_t>(call_edge_on) & 3u))
    return BF_ERR_ALIGN;
  // the window is fp32 whatever the storage type of X (slots accumulate), with X's pitch in elements
  MatArgs mw = ma;
  mw.n = static_cast<int>(E);
  const size_t win_bytes = E > 0 ? mw.extent(4) : 0;
  if (E > 0 && overlaps(X, ma.bytes, Win, win_bytes)) return BF_ERR_ALIAS;
  if (pv && E > 0 && (overlaps(pv, static_cast<size_t>(t->n) * 4, X, ma.bytes) || overlaps(pv, static_cast<size_t>(t->n) * 4, Win, win_bytes) ||
             overlaps(win_p, static_cast<size_t>(E) * 4, X, ma.bytes) || overlaps(win_p, static_cast<size_t>(E) * 4, Win, win_bytes) ||
             overlaps(pv, static_cast<size_t>(t->n) * 4, win_p, static_cast<size_t>(E) * 4)))
    return BF_ERR_ALIAS;
  bf::DeviceCopy* dc = nullptr;
  rc = get_device_copy(t, false, &dc);
  if (rc != BF_OK) return rc;
  DeviceInfo di;
  rc = device_info(dc->device, &di);
  if (rc != BF_OK) return rc;
  WinParams wp{};
  rc = get_window_plan(t, static_cast<size_t>(round) % t->rounds.size(), dc, &wp);
  if (rc != BF_OK) return rc;
  wp.x = static_cast<char*>(X);
  wp.win = static_cast<float*>(Win);
  wp.active = active;
  wp.call_self_w = call_self_w; wp.call_edge_w = call_edge_w; wp.call_edge_on = call_edge_on;
  wp.d = d; wp.ld = ma.ld; wp.n = t->n; wp.block_log = ma.block_log; wp.slots = static_cast<int32_t>(E);
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  if (pv && (mode == WIN_ACCUMULATE || mode == WIN_COLLECT)) {
    if (mode == WIN_ACCUMULATE) hipLaunchKernelGGL(bf_win_p_kernel<WIN_ACCUMULATE>, dim3(1), dim3(1024), 0, st, wp, pv, win_p);
    else hipLaunchKernelGGL(bf_win_p_kernel<WIN_COLLECT>, dim3(1), dim3(1024), 0, st, wp, pv, win_p);
    BF_HIP_TRY(hipGetLastError());
  }
  if (d == 0) return BF_OK;
  const int64_t chunk_cols = 4 * 1024;
  const int64_t chunks = (d + chunk_cols - 1) / chunk_cols;
  if (chunks > INT32_MAX) return BF_ERR_SIZE;
  wp.chunks = static_cast<int32_t>(chunks);
  const int64_t units = chunks * t->n;
  // One 256-thread workgroup per CU, as for a plain copy: these kernels only move data, and with more
  // workgroups per CU the memory system serves the same streams more slowly (n = 128, 512 slots,
  // d = 2^21: accumulate 5.14 -> 5.4 TB/s, update_then_collect 5.18 -> 5.5, put 5.1 -> 5.3, update
  // 5.65 -> 6.0 against eight per CU; two per CU already lose the gain).
  // (win_get with bf16 storage is the exception: it reads every X row once per out-edge in 8-byte
  // pieces and lives on cache hits, which more resident workgroups raise: n = 32, 288 slots,
  // d = 12.8 M: 4.3 ms with eight per CU, 6.1 ms with one.)
  const int per_cu = (mode == WIN_GET && dt != BF_F32) ? 8 : 1;
  int grid = static_cast<int>(std::min<int64_t>(units, static_cast<int64_t>(di.cus) * per_cu));
  if (g_tune_grid > 0) grid = static_cast<int>(std::min<int64_t>(units, g_tune_grid));     // (the knob may also raise it)
  // Cache policy as for the mixing kernels: state and window beyond what the memory-side cache can
  // keep between two calls stream with non-temporal loads and stores.
  const size_t eb = dt == BF_F32 ? 4 : 2;
  const bool stream = g_tune_stream == 1 ? true : (g_tune_stream == 2 ? false : ma.extent(static_cast<int>(eb)) + win_bytes > (size_t{320} << 20));
#define BF_WIN(M)                                                                                                \
  do {                                                                                                           \
    if (dt == BF_F32) {                                                                                          \
      if (stream) hipLaunchKernelGGL((bf_win_kernel<M, DT_F32, true>), dim3(grid), dim3(256), 0, st, wp);        \
      else hipLaunchKernelGGL((bf_win_kernel<M, DT_F32, false>), dim3(grid), dim3(256), 0, st, wp);              \
    } else {                                                                                                     \
      if (stream) hipLaunchKernelGGL((bf_win_kernel<M, DT_BF16, true>), dim3(grid), dim3(256), 0, st, wp);       \
      else hipLaunchKernelGGL((bf_win_kernel<M, DT_BF16, false>), dim3(grid), dim3(256), 0, st, wp);             \
    }                                                                                                            \
  } while (0)
  switch (mode) {
    case WIN_PUT: BF_WIN(WIN_PUT); break;
    case WIN_ACCUMULATE: BF_WIN(WIN_ACCUMULATE); break;
    case WIN_COLLECT: BF_WIN(WIN_COLLECT); break;
    case WIN_GET: BF_WIN(WIN_GET); break;
    default: BF_WIN(WIN_AVERAGE); break;
  }
#undef BF_WIN
  BF_HIP_TRY(hipGetLastError());
  return BF_OK;
}

// Layout conversion between agent-major rows and column blocks: one thread per 16 bytes of the
// block side (coalesced there; row segments of B elements on the agent-major side).  PACK also
// zero-fills the columns at or past d of the last block, UNPACK never writes them.
template <int EB, bool PACK>
__global__ __launch_bounds__(256) void bf_layout_kernel(const char* src, char* dst, int n, int64_t d, int64_t ld,
                                                        int block_log, int64_t nunits) {
  constexpr int PER = 16 / EB;
  const int upb_log = block_log - (EB == 4 ? 2 : 3);          // 16-byte units per block row (log2)
  for (int64_t u = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x; u < nunits;
       u += static_cast<int64_t>(gridDim.x) * 256) {
    const int64_t rowu = u >> upb_log;                          // block * n + row
    const int64_t blk = rowu / n;
    const int row = static_cast<int>(rowu - blk * n);
    const int64_t col = (blk << block_log) + ((u & ((int64_t{1} << upb_log) - 1)) * PER);
    const char* rowmajor = (PACK ? src : dst) + (static_cast<int64_t>(row) * ld + col) * EB;
    const char* blocked = (PACK ? dst : src) + u * 16;
    if (col + PER <= d) {
      if (PACK) *reinterpret_cast<u32x4*>(const_cast<char*>(blocked)) = *reinterpret_cast<const u32x4*>(rowmajor);
      else *reinterpret_cast<u32x4*>(const_cast<char*>(rowmajor)) = *reinterpret_cast<const u32x4*>(blocked);
    } else {
      // the unit that straddles d (element by element), and the padding behind it
      for (int e = 0; e < PER; ++e) {
        const bool in = col + e < d;
        for (int b = 0; b < EB; ++b) {
          if (PACK) const_cast<char*>(blocked)[e * EB + b] = in ? rowmajor[e * EB + b] : char{0};
          else if (in) const_cast<char*>(rowmajor)[e * EB + b] = blocked[e * EB + b];
        }
      }
    }
  }
}

int layout_common(bool pack, int32_t n, int64_t d, int64_t ld, const void* src, int64_t block, void* dst,
                         bf_dtype_t dt, void* hip_stream) {
  if (!src || !dst) return BF_ERR_NULL;
  if (n < 1) return BF_ERR_SIZE;
  MatArgs rm, bl;
  int rc = check_matrix_shape(n, d, ld, dt, &rm);
  if (rc != BF_OK) return rc;
  if (block < 1) return BF_ERR_SIZE;
  rc = check_matrix_shape(n, d, -block, dt, &bl, true);
  if (rc != BF_OK) return rc;
  if (misaligned16(src) || misaligned16(dst)) return BF_ERR_ALIGN;
  if (overlaps(src, pack ? rm.bytes : bl.bytes, dst, pack ? bl.bytes : rm.bytes)) return BF_ERR_ALIAS;
  if (d == 0) return BF_OK;
  int dev = 0;
  BF_HIP_TRY(hipGetDevice(&dev));
  DeviceInfo di;
  rc = device_info(dev, &di);
  if (rc != BF_OK) return rc;
  const int64_t nunits = static_cast<int64_t>(bl.bytes / 16);
  const int grid = static_cast<int>(std::min<int64_t>((nunits + 255) / 256, static_cast<int64_t>(di.cus) * 16));
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  const char* s8 = static_cast<const char*>(src);
  char* d8 = static_cast<char*>(dst);
  if (dt == BF_F32) {
    if (pack) hipLaunchKernelGGL((bf_layout_kernel<4, true>), dim3(grid), dim3(256), 0, st, s8, d8, n, d, ld, bl.block_log, nunits);
    else hipLaunchKernelGGL((bf_layout_kernel<4, false>), dim3(grid), dim3(256), 0, st, s8, d8, n, d, ld, bl.block_log, nunits);
  } else {
    if (pack) hipLaunchKernelGGL((bf_layout_kernel<2, true>), dim3(grid), dim3(256), 0, st, s8, d8, n, d, ld, bl.block_log, nunits);
    else hipLaunchKernelGGL((bf_layout_kernel<2, false>), dim3(grid), dim3(256), 0, st, s8, d8, n, d, ld, bl.block_log, nunits);
  }
  BF_HIP_TRY(hipGetLastError());
  return BF_OK;
}

}  // namespace

extern "C" {

int bf_last_hip_error(void) { return g_last_hip_error; }

int bf_set_tuning(int32_t knob, int32_t value) {
  if (value < 0) return BF_ERR_SIZE;
  if (knob == 0) g_tune_tile = value;
  else if (knob == 1) g_tune_wgs = value;
  else if (knob == 2) g_tune_gather = value;
  else if (knob == 3) g_tune_grid = value;
  else if (knob == 5) g_tune_nochain = value;
  else if (knob == 7) g_tune_noserp = value;
  else if (knob == 9) g_tune_chain256 = value;
  else if (knob == 8) g_tune_stream = value;
  else if (knob == 6) g_tune_cw = value;
  else if (knob == 10) g_tune_spin = value;
  else if (knob == 11) g_tune_extra = value;
  else if (knob == 12) g_tune_pipe = value;
  else if (knob == 13) g_tune_noshift = value;
  else if (knob == 14) g_tune_awc = value;
  else return BF_ERR_KIND;
  return BF_OK;
}

int bf_topology_destroy(bf_topology_t* t) {
  if (!t) return BF_OK;
  int rc = BF_OK;
  for (auto& kv : t->two_level)
    if (bf_topology_destroy(kv.second) != BF_OK) rc = BF_ERR_HIP;
  for (auto& c : t->dev) {
    if (c.blob && hipFree(c.blob) != hipSuccess) rc = BF_ERR_HIP;
    if (c.dense_t && hipFree(c.dense_t) != hipSuccess) rc = BF_ERR_HIP;
    for (char* wb : c.win_blob)
      if (wb && hipFree(wb) != hipSuccess) rc = BF_ERR_HIP;
    if (c.sync && hipFree(c.sync) != hipSuccess) rc = BF_ERR_HIP;
  }
  delete t;
  return rc;
}

int bf_neighbor_allreduce(const bf_topology_t* t, int32_t round, const void* X_in, void* X_out,
                          int64_t d, int64_t ld, bf_dtype_t dt, void* hip_stream) {
  if (!t || !X_in || !X_out) return BF_ERR_NULL;
  if (round < 0) return BF_ERR_ROUND;
  MatArgs ma;
  int rc = check_matrix_shape(t->n, d, ld, dt, &ma, true);
  if (rc != BF_OK) return rc;
  if (misaligned16(X_in) || misaligned16(X_out)) return BF_ERR_ALIGN;
  if (X_in != X_out && overlaps(X_in, ma.bytes, X_out, ma.bytes)) return BF_ERR_ALIAS;
  if (t->kind == BF_DENSE_USER && dt == BF_F32 && t->n <= 256)
    return bf_dense_mix(t, round, X_in, X_out, d, ld, dt, hip_stream);
  TileParams tp{};
  tp.x_in = static_cast<const char*>(X_in);
  tp.x_out = static_cast<char*>(X_out);
  tp.d = d; tp.ld = ma.ld; tp.block_log = ma.block_log;
  return run_tile(const_cast<bf_topology_t*>(t), round, OP_MIX, false, tp, dt, static_cast<hipStream_t>(hip_stream));
}

int bf_neighbor_allreduce_multi(const bf_topology_t* t, int32_t round0, int32_t count, const void* X_in,
                                void* X_out, int64_t d, int64_t ld, bf_dtype_t dt, void* hip_stream) {
  if (!t || !X_in || !X_out) return BF_ERR_NULL;
  if (round0 < 0) return BF_ERR_ROUND;
  if (count < 1 || count > 8) return BF_ERR_SIZE;
  MatArgs ma;
  int rc = check_matrix_shape(t->n, d, ld, dt, &ma, true);
  if (rc != BF_OK) return rc;
  if (misaligned16(X_in) || misaligned16(X_out)) return BF_ERR_ALIGN;
  if (X_in != X_out && overlaps(X_in, ma.bytes, X_out, ma.bytes)) return BF_ERR_ALIAS;
  TileParams tp{};
  tp.x_in = static_cast<const char*>(X_in);
  tp.x_out = static_cast<char*>(X_out);
  tp.d = d; tp.ld = ma.ld; tp.block_log = ma.block_log;
  tp.fuse = count;
  bf_topology_t* tt = const_cast<bf_topology_t*>(t);
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  if (d == 0) return BF_OK;
  rc = run_shift_rounds(tt, round0, count, tp, dt, st);
  if (rc != BF_ERR_UNSUPPORTED) return rc;
  rc = run_tile(tt, round0, OP_MIX, false, tp, dt, st);
  if (rc != BF_ERR_UNSUPPORTED || count == 1) return rc;
  // No room for two LDS tiles (many agents): `count` separate passes, the first from X_in to X_out,
  // the others in place on X_out.  For BF_F32 the result is the same bits either way; BF_BF16 then
  // rounds after every round, as separate calls do.  Every pass is checked for a kernel first.
  tp.fuse = 1;
  TileParams tq = tp;
  tq.x_in = tq.x_out;
  // round numbers modulo twice the period: same weight matrix, same tile direction, no overflow
  const int64_t period2 = 2 * static_cast<int64_t>(tt->rounds.size());
  auto rnd = [&](int32_t j) { return static_cast<int32_t>((static_cast<int64_t>(round0) + j) % period2); };
  for (int32_t j = 0; j < count; ++j)
    if ((rc = run_tile(tt, rnd(j), OP_MIX, false, j == 0 ? tp : tq, dt, st, true)) != BF_OK) return rc;
  for (int32_t j = 0; j < count; ++j)
    if ((rc = run_tile(tt, rnd(j), OP_MIX, false, j == 0 ? tp : tq, dt, st)) != BF_OK) return rc;
  return BF_OK;
}

int bf_hierarchical_neighbor_allreduce(const bf_topology_t* machine_topology, int32_t round, int32_t local_size,
                                       const void* X_in, void* X_out, int64_t d, int64_t ld, bf_dtype_t dt,
                                       void* hip_stream) {
  if (!machine_topology || !X_in || !X_out) return BF_ERR_NULL;
  if (round < 0) return BF_ERR_ROUND;
  if (local_size < 1 || static_cast<int64_t>(machine_topology->n) * local_size > (1 << 20)) return BF_ERR_SIZE;
  const int32_t n = machine_topology->n * local_size;
  MatArgs ma;
  int rc = check_matrix_shape(n, d, ld, dt, &ma, true);
  if (rc != BF_OK) return rc;
  if (misaligned16(X_in) || misaligned16(X_out)) return BF_ERR_ALIGN;
  if (X_in != X_out && overlaps(X_in, ma.bytes, X_out, ma.bytes)) return BF_ERR_ALIAS;
  bf_topology_t* mt = const_cast<bf_topology_t*>(machine_topology);
  bf_topology_t* two = nullptr;
  {
    std::lock_guard<std::mutex> lk(mt->mu);
    auto it = mt->two_level.find(local_size);
    if (it == mt->two_level.end()) {
      rc = bf::make_two_level(*mt, local_size, &two);
      if (rc != BF_OK) return rc;
      mt->two_level[local_size] = two;
    } else {
      two = it->second;
    }
  }
  const int32_t r3 = static_cast<int32_t>((static_cast<int64_t>(round) % static_cast<int64_t>(mt->rounds.size())) * 3);
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  TileParams tp{};
  tp.x_in = static_cast<const char*>(X_in);
  tp.x_out = static_cast<char*>(X_out);
  tp.d = d; tp.ld = ma.ld; tp.block_log = ma.block_log;
  tp.fuse = 3;
  // stage A writes rows 0..M-1 of the second LDS tile and stage B reads only those: the tile needs M rows
  tp.rows_b = mt->n;
  rc = run_tile(two, r3, OP_MIX, false, tp, dt, st);
  if (rc != BF_ERR_UNSUPPORTED) return rc;
  // Too many agents for two LDS tiles: the three stages as three passes.  The first may write
  // X_out, the other two update it in place (every row of X_out is overwritten in the end, so the
  // zeros the first two stages leave in rows M and up are never seen).  All three are checked for a
  // kernel before the first is launched.
  tp.fuse = 1;
  tp.rows_b = 0;
  TileParams tq = tp;
  tq.x_in = tq.x_out;
  if ((rc = run_tile(two, r3, OP_MIX, false, tp, dt, st, true)) != BF_OK) return rc;
  if ((rc = run_tile(two, r3 + 1, OP_MIX, false, tq, dt, st, true)) != BF_OK) return rc;
  if ((rc = run_tile(two, r3 + 2, OP_MIX, false, tq, dt, st, true)) != BF_OK) return rc;
  if ((rc = run_tile(two, r3, OP_MIX, false, tp, dt, st)) != BF_OK) return rc;
  if ((rc = run_tile(two, r3 + 1, OP_MIX, false, tq, dt, st)) != BF_OK) return rc;
  return run_tile(two, r3 + 2, OP_MIX, false, tq, dt, st);
}

int bf_win_put(const bf_topology_t* t, int32_t round, const int32_t* active, const void* X, void* Win,
               int64_t d, int64_t ld, bf_dtype_t dt, void* hip_stream) {
  return win_common(WIN_PUT, t, round, active, const_cast<void*>(X), nullptr, Win, nullptr, d, ld, dt, hip_stream);
}

int bf_win_get(const bf_topology_t* t, int32_t round, const int32_t* active, const void* X, void* Win,
               int64_t d, int64_t ld, bf_dtype_t dt, void* hip_stream) {
  return win_common(WIN_GET, t, round, active, const_cast<void*>(X), nullptr, Win, nullptr, d, ld, dt, hip_stream);
}

int bf_win_accumulate(const bf_topology_t* t, int32_t round, const int32_t* active, void* X, float* p,
                      void* Win, float* win_p, int64_t d, int64_t ld, bf_dtype_t dt, void* hip_stream) {
  return win_common(WIN_ACCUMULATE, t, round, active, X, p, Win, win_p, d, ld, dt, hip_stream);
}

int bf_win_update(const bf_topology_t* t, int32_t round, const int32_t* active, void* X, const void* Win,
                  int64_t d, int64_t ld, bf_dtype_t dt, void* hip_stream) {
  return win_common(WIN_AVERAGE, t, round, active, X, nullptr, const_cast<void*>(Win), nullptr, d, ld, dt, hip_stream);
}

int bf_win_update_then_collect(const bf_topology_t* t, int32_t round, const int32_t* active, void* X, float* p,
                               void* Win, float* win_p, int64_t d, int64_t ld, bf_dtype_t dt, void* hip_stream) {
  return win_common(WIN_COLLECT, t, round, active, X, p, Win, win_p, d, ld, dt, hip_stream);
}

int bf_win_put_weighted(const bf_topology_t* t, int32_t round, const int32_t* active, void* X, void* Win,
                        const float* self_weight, const float* dst_weight, const int32_t* dst_on,
                        int64_t d, int64_t ld, bf_dtype_t dt, void* hip_stream) {
  return win_common(WIN_PUT, t, round, active, X, nullptr, Win, nullptr, d, ld, dt, hip_stream, self_weight, dst_weight, dst_on);
}

int bf_win_get_weighted(const bf_topology_t* t, int32_t round, const int32_t* active, const void* X, void* Win,
                        const float* src_weight, const int32_t* src_on, int64_t d, int64_t ld, bf_dtype_t dt,
                        void* hip_stream) {
  return win_common(WIN_GET, t, round, active, const_cast<void*>(X), nullptr, Win, nullptr, d, ld, dt, hip_stream, nullptr,
                    src_weight, src_on);
}

int bf_win_accumulate_weighted(const bf_topology_t* t, int32_t round, const int32_t* active, void* X, float* p,
                               void* Win, float* win_p, const float* self_weight, const float* dst_weight,
                               const int32_t* dst_on, int64_t d, int64_t ld, bf_dtype_t dt, void* hip_stream) {
  return win_common(WIN_ACCUMULATE, t, round, active, X, p, Win, win_p, d, ld, dt, hip_stream, self_weight, dst_weight, dst_on);
}

int bf_win_update_weighted(const bf_topology_t* t, int32_t round, const int32_t* active, void* X, const void* Win,
                           const float* self_weight, const float* src_weight, const int32_t* src_on,
                           int64_t d, int64_t ld, bf_dtype_t dt, void* hip_stream) {
  return win_common(WIN_AVERAGE, t, round, active, X, nullptr, const_cast<void*>(Win), nullptr, d, ld, dt, hip_stream,
                    self_weight, src_weight, src_on);
}

int bf_dense_mix(const bf_topology_t* t, int32_t round, const void* X_in, void* X_out,
                 int64_t d, int64_t ld, bf_dtype_t dt, void* hip_stream) {
  if (!t || !X_in || !X_out) return BF_ERR_NULL;
  if (round < 0) return BF_ERR_ROUND;
  MatArgs ma;
  int rc = check_matrix_shape(t->n, d, ld, dt, &ma, true);
  if (rc != BF_OK) return rc;
  if (misaligned16(X_in) || misaligned16(X_out)) return BF_ERR_ALIGN;
  if (X_in != X_out && overlaps(X_in, ma.bytes, X_out, ma.bytes)) return BF_ERR_ALIAS;
  if (d == 0) return BF_OK;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  if (dt == BF_F32 && t->n <= 256) {
    bf::DeviceCopy* dc = nullptr;
    rc = get_device_copy(const_cast<bf_topology_t*>(t), true, &dc);
    if (rc != BF_OK) return rc;
    DeviceInfo di;
    rc = device_info(dc->device, &di);
    if (rc != BF_OK) return rc;
    const int n_pad = dc->n_pad;
    const size_t k = static_cast<size_t>(round) % t->rounds.size();
    const float* wt = dc->dense_t + k * static_cast<size_t>(n_pad) * n_pad;
    const size_t lds_cu = std::min(di.lds_per_cu ? di.lds_per_cu : size_t{65536},
                                   di.lds_per_block_optin ? di.lds_per_block_optin : size_t{65536});
    rc = launch_dense(n_pad / 32, static_cast<const float*>(X_in), static_cast<float*>(X_out), wt, t->n, d, ma.ld,
                      ma.block_log, di.cus, lds_cu, st);
    if (rc != BF_ERR_UNSUPPORTED) return rc;
  }
  // no matrix-core kernel for this storage type, this many agents, this little LDS or blocks this
  // narrow: the list kernels compute the same product (a dense W is a CSR with full rows)
  TileParams tp{};
  tp.x_in = static_cast<const char*>(X_in);
  tp.x_out = static_cast<char*>(X_out);
  tp.d = d; tp.ld = ma.ld; tp.block_log = ma.block_log;
  return run_tile(const_cast<bf_topology_t*>(t), round, OP_MIX, false, tp, dt, st);
}

// Shared body of the push-sum entry points: optional local update x - alpha g before the mix.
static int pushsum_common(const bf_topology_t* t, int32_t round, const void* X_in, void* X_out, const void* G,
                          float alpha, const float* w_in, float* w_out, void* Y, int64_t d, int64_t ld,
                          bf_dtype_t dt, void* hip_stream) {
  if (!t || !X_in || !X_out || !w_in || !w_out) return BF_ERR_NULL;
  if (round < 0) return BF_ERR_ROUND;
  MatArgs ma;
  int rc = check_matrix_shape(t->n, d, ld, dt, &ma, true);
  if (rc != BF_OK) return rc;
  if (misaligned16(X_in) || misaligned16(X_out) || (Y && misaligned16(Y)) || (G && misaligned16(G))) return BF_ERR_ALIGN;
  if ((reinterpret_cast<uintptr_t>(w_in) & 3u) || (reinterpret_cast<uintptr_t>(w_out) & 3u)) return BF_ERR_ALIGN;
  const size_t wb = static_cast<size_t>(t->n) * 4;
  if (X_in != X_out && overlaps(X_in, ma.bytes, X_out, ma.bytes)) return BF_ERR_ALIAS;
  if (w_in != w_out && overlaps(w_in, wb, w_out, wb)) return BF_ERR_ALIAS;
  if (overlaps(w_out, wb, X_out, ma.bytes) || overlaps(w_out, wb, X_in, ma.bytes) ||
      overlaps(w_in, wb, X_out, ma.bytes))
    return BF_ERR_ALIAS;
  if (Y && (overlaps(Y, ma.bytes, X_in, ma.bytes) || overlaps(Y, ma.bytes, X_out, ma.bytes) ||
            overlaps(Y, ma.bytes, w_in, wb) || overlaps(Y, ma.bytes, w_out, wb)))
    return BF_ERR_ALIAS;
  if (G && (overlaps(G, ma.bytes, X_out, ma.bytes) || overlaps(G, ma.bytes, w_out, wb) ||
            (Y && overlaps(G, ma.bytes, Y, ma.bytes))))
    return BF_ERR_ALIAS;
  if (static_cast<size_t>(t->n) * 4 > 160 * 1024) return BF_ERR_UNSUPPORTED;
  bf_topology_t* tt = const_cast<bf_topology_t*>(t);
  bf::DeviceCopy* dc = nullptr;
  rc = get_device_copy(tt, false, &dc);
  if (rc != BF_OK) return rc;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  const size_t k = static_cast<size_t>(round) % t->rounds.size();
  const size_t wl = std::max<size_t>(wb, 16);
  if (wl > 48 * 1024) {
    static thread_local size_t raised = 0;
    if (raised < wl) {
      BF_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(bf_pushsum_w_kernel),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(wl)));
      raised = wl;
    }
  }
  TileParams tp{};
  tp.x_in = static_cast<const char*>(X_in);
  tp.x_out = static_cast<char*>(X_out);
  tp.g = static_cast<const char*>(G);
  tp.alpha = alpha;
  tp.y = static_cast<char*>(Y);
  tp.p_out = w_out;
  tp.d = d; tp.ld = ma.ld; tp.block_log = ma.block_log;
  // is there a kernel for the matrix part?  Asked before w is advanced, so that an error leaves
  // the caller's push-sum state as it was
  rc = run_tile(tt, round, G ? OP_ATC : OP_MIX, Y != nullptr, tp, dt, st, true);
  if (rc != BF_OK) return rc;
  // w first (one small workgroup, in-place safe); the tile kernel then reads w_out for the ratio.
  hipLaunchKernelGGL(bf_pushsum_w_kernel, dim3(1), dim3(1024), wl, st,
                     reinterpret_cast<const int32_t*>(dc->blob + dc->rowptr_off[k]),
                     reinterpret_cast<const u32x2*>(dc->blob + dc->entry_off[k]), w_in, w_out, t->n);
  BF_HIP_TRY(hipGetLastError());
  return run_tile(tt, round, G ? OP_ATC : OP_MIX, Y != nullptr, tp, dt, st);
}

int bf_pushsum_step(const bf_topology_t* t, int32_t round, const void* X_in, void* X_out,
                    const float* w_in, float* w_out, void* Y, int64_t d, int64_t ld,
                    bf_dtype_t dt, void* hip_stream) {
  return pushsum_common(t, round, X_in, X_out, nullptr, 0.0f, w_in, w_out, Y, d, ld, dt, hip_stream);
}

int bf_pushsum_atc_step(const bf_topology_t* t, int32_t round, const void* X_in, void* X_out, const void* G,
                        float alpha, const float* w_in, float* w_out, void* Y, int64_t d, int64_t ld,
                        bf_dtype_t dt, void* hip_stream) {
  if (!G) return BF_ERR_NULL;
  return pushsum_common(t, round, X_in, X_out, G, alpha, w_in, w_out, Y, d, ld, dt, hip_stream);
}

int bf_tracking_step(const bf_topology_t* t, int32_t round, const void* Y_in, void* Y_out, const void* G_new,
                     const void* G_old, int64_t d, int64_t ld, bf_dtype_t dt, void* hip_stream) {
  if (!t || !Y_in || !Y_out || !G_new || !G_old) return BF_ERR_NULL;
  if (round < 0) return BF_ERR_ROUND;
  MatArgs ma;
  int rc = check_matrix_shape(t->n, d, ld, dt, &ma, true);
  if (rc != BF_OK) return rc;
  if (misaligned16(Y_in) || misaligned16(Y_out) || misaligned16(G_new) || misaligned16(G_old)) return BF_ERR_ALIGN;
  if (Y_in != Y_out && overlaps(Y_in, ma.bytes, Y_out, ma.bytes)) return BF_ERR_ALIAS;
  if (overlaps(G_new, ma.bytes, Y_out, ma.bytes) || overlaps(G_old, ma.bytes, Y_out, ma.bytes)) return BF_ERR_ALIAS;
  TileParams tp{};
  tp.x_in = static_cast<const char*>(Y_in);
  tp.x_out = static_cast<char*>(Y_out);
  tp.g = static_cast<const char*>(G_new);
  tp.g2 = static_cast<const char*>(G_old);
  tp.d = d; tp.ld = ma.ld; tp.block_log = ma.block_log;
  return run_tile(const_cast<bf_topology_t*>(t), round, OP_TRACK, false, tp, dt, static_cast<hipStream_t>(hip_stream));
}

// Shared body of bf_atc_step and bf_atc_step_layouts: ld names the layout of X_in and X_out, ld_g that
// of G, ld_m that of M.
static int atc_common(const bf_topology_t* t, int32_t round, const void* X_in, void* X_out, const void* G,
                      float* M, float alpha, float beta, bf_mode_t mode, int64_t d, int64_t ld, int64_t ld_g,
                      int64_t ld_m, bf_dtype_t dt, void* hip_stream) {
  if (!t || !X_in || !X_out || !G) return BF_ERR_NULL;
  if (round < 0) return BF_ERR_ROUND;
  if (mode != BF_ATC && mode != BF_AWC) return BF_ERR_KIND;
  MatArgs ma, mg, mm;
  int rc = check_matrix_shape(t->n, d, ld, dt, &ma, true);
  if (rc != BF_OK) return rc;
  rc = check_matrix_shape(t->n, d, ld_g, dt, &mg, true);
  if (rc != BF_OK) return rc;
  mm = ma;
  if (M) {
    rc = check_matrix_shape(t->n, d, ld_m, BF_F32, &mm, true);
    if (rc != BF_OK) return rc;
  }
  if (misaligned16(X_in) || misaligned16(X_out) || misaligned16(G) || (M && misaligned16(M))) return BF_ERR_ALIGN;
  const size_t mb = M ? mm.bytes : 0;
  if (X_in != X_out && overlaps(X_in, ma.bytes, X_out, ma.bytes)) return BF_ERR_ALIAS;
  if (overlaps(G, mg.bytes, X_out, ma.bytes)) return BF_ERR_ALIAS;
  if (M && (overlaps(M, mb, X_out, ma.bytes) || overlaps(M, mb, X_in, ma.bytes) || overlaps(M, mb, G, mg.bytes)))
    return BF_ERR_ALIAS;
  TileParams tp{};
  tp.x_in = static_cast<const char*>(X_in);
  tp.x_out = static_cast<char*>(X_out);
  tp.g = static_cast<const char*>(G);
  tp.m = M;
  tp.alpha = alpha; tp.beta = beta;
  tp.d = d; tp.ld = ma.ld; tp.block_log = ma.block_log;
  tp.g_ld = mg.ld; tp.g_block_log = mg.block_log;
  tp.m_ld = mm.ld; tp.m_block_log = mm.block_log;
  const int op = M ? (mode == BF_ATC ? OP_MOM_ATC : OP_MOM_AWC) : (mode == BF_ATC ? OP_ATC : OP_AWC);
  return run_tile(const_cast<bf_topology_t*>(t), round, op, false, tp, dt, static_cast<hipStream_t>(hip_stream));
}

int bf_atc_step(const bf_topology_t* t, int32_t round, const void* X_in, void* X_out, const void* G,
                float* M, float alpha, float beta, bf_mode_t mode, int64_t d, int64_t ld,
                bf_dtype_t dt, void* hip_stream) {
  return atc_common(t, round, X_in, X_out, G, M, alpha, beta, mode, d, ld, ld, ld, dt, hip_stream);
}

int bf_atc_step_layouts(const bf_topology_t* t, int32_t round, const void* X_in, void* X_out, const void* G,
                        float* M, float alpha, float beta, bf_mode_t mode, int64_t d, int64_t ld, int64_t ld_g,
                        int64_t ld_m, bf_dtype_t dt, void* hip_stream) {
  return atc_common(t, round, X_in, X_out, G, M, alpha, beta, mode, d, ld, ld_g, ld_m, dt, hip_stream);
}

// Shared body of bf_exact_diffusion_step and its _layouts form: ld names the layout of X_in and X_out,
// ld_g that of G, ld_p that of Psi_prev.
static int ed_common(const bf_topology_t* t, int32_t round, const void* X_in, void* X_out, const void* G,
                     float* Psi_prev, float alpha, int64_t d, int64_t ld, int64_t ld_g, int64_t ld_p,
                     bf_dtype_t dt, void* hip_stream) {
  if (!t || !X_in || !X_out || !G || !Psi_prev) return BF_ERR_NULL;
  if (round < 0) return BF_ERR_ROUND;
  MatArgs ma, mg, mp;
  int rc = check_matrix_shape(t->n, d, ld, dt, &ma, true);
  if (rc != BF_OK) return rc;
  rc = check_matrix_shape(t->n, d, ld_g, dt, &mg, true);
  if (rc != BF_OK) return rc;
  rc = check_matrix_shape(t->n, d, ld_p, BF_F32, &mp, true);
  if (rc != BF_OK) return rc;
  if (misaligned16(X_in) || misaligned16(X_out) || misaligned16(G) || misaligned16(Psi_prev)) return BF_ERR_ALIGN;
  const size_t pb = mp.bytes;
  if (X_in != X_out && overlaps(X_in, ma.bytes, X_out, ma.bytes)) return BF_ERR_ALIAS;
  if (overlaps(G, mg.bytes, X_out, ma.bytes)) return BF_ERR_ALIAS;
  if (overlaps(Psi_prev, pb, X_out, ma.bytes) || overlaps(Psi_prev, pb, X_in, ma.bytes) || overlaps(Psi_prev, pb, G, mg.bytes))
    return BF_ERR_ALIAS;
  TileParams tp{};
  tp.x_in = static_cast<const char*>(X_in);
  tp.x_out = static_cast<char*>(X_out);
  tp.g = static_cast<const char*>(G);
  tp.m = Psi_prev;
  tp.alpha = alpha;
  tp.d = d; tp.ld = ma.ld; tp.block_log = ma.block_log;
  tp.g_ld = mg.ld; tp.g_block_log = mg.block_log;
  tp.m_ld = mp.ld; tp.m_block_log = mp.block_log;
  return run_tile(const_cast<bf_topology_t*>(t), round, OP_ED, false, tp, dt, static_cast<hipStream_t>(hip_stream));
}

int bf_exact_diffusion_step(const bf_topology_t* t, int32_t round, const void* X_in, void* X_out,
                            const void* G, float* Psi_prev, float alpha, int64_t d, int64_t ld,
                            bf_dtype_t dt, void* hip_stream) {
  return ed_common(t, round, X_in, X_out, G, Psi_prev, alpha, d, ld, ld, ld, dt, hip_stream);
}

int bf_exact_diffusion_step_layouts(const bf_topology_t* t, int32_t round, const void* X_in, void* X_out,
                                    const void* G, float* Psi_prev, float alpha, int64_t d, int64_t ld,
                                    int64_t ld_g, int64_t ld_p, bf_dtype_t dt, void* hip_stream) {
  return ed_common(t, round, X_in, X_out, G, Psi_prev, alpha, d, ld, ld_g, ld_p, dt, hip_stream);
}

// static_scratch: the half steps and barrier words live in the library's static device array and
// nothing is allocated (the topology must already be resident on the device).
static int dgd_run_common(const bf_topology_t* tc, int32_t round0, int32_t iterations, int32_t m,
                          const float* A, const float* b, float* X, float* Psi, bool want_psi, float* work,
                          float alpha, int64_t d, int64_t ld, void* hip_stream, bool static_scratch = false) {
  if (!tc || !A || !b || !X || (!work && !static_scratch) || (want_psi && !Psi)) return BF_ERR_NULL;
  if (round0 < 0) return BF_ERR_ROUND;
  bf_topology_t* t = const_cast<bf_topology_t*>(tc);
  const int32_t n = t->n;
  if (iterations < 0 || m < 1 || m > 8192 || d < 4 || (d % 4) != 0 || ld < d || (ld % 4) != 0) return BF_ERR_SIZE;
  if (static_cast<uint64_t>(n) * static_cast<uint64_t>(iterations) >= (uint64_t{1} << 32)) return BF_ERR_SIZE;
  if (misaligned16(A) || misaligned16(X) || (work && misaligned16(work)) || (reinterpret_cast<uintptr_t>(b) & 3u)) return BF_ERR_ALIGN;
  const size_t xb = (static_cast<size_t>(n - 1) * ld + d) * 4, wb = (static_cast<size_t>(2 * n - 1) * ld + d) * 4;
  const size_t ab = static_cast<size_t>(n) * m * d * 4, bb = static_cast<size_t>(n) * m * 4;
  if (static_scratch && static_cast<size_t>(2) * n * ld * 4 > kStaticHalfStepBytes) return BF_ERR_SIZE;
  if (overlaps(X, xb, A, ab) || overlaps(X, xb, b, bb)) return BF_ERR_ALIAS;
  if (work && (overlaps(X, xb, work, wb) || overlaps(work, wb, A, ab) || overlaps(work, wb, b, bb))) return BF_ERR_ALIAS;
  if (Psi && (misaligned16(Psi))) return BF_ERR_ALIGN;
  if (Psi && (overlaps(Psi, xb, X, xb) || (work && overlaps(Psi, xb, work, wb)) || overlaps(Psi, xb, A, ab) || overlaps(Psi, xb, b, bb)))
    return BF_ERR_ALIAS;
  if (iterations == 0) return BF_OK;
  bf::DeviceCopy* dc = nullptr;
  int rc = BF_OK;
  unsigned char* scratch = nullptr;
  // Does the problem fit the one-launch kernel?  One workgroup per agent, all resident at once, A_i
  // and 20 KB of working storage in one CU's LDS, rows of at most 4096 columns.
  bool fits = d <= 4096 && m <= 64;
  if (fits) {
    int dev = 0;
    BF_HIP_TRY(hipGetDevice(&dev));
    DeviceInfo di0;
    rc = device_info(dev, &di0);
    if (rc != BF_OK) return rc;
    const size_t need = static_cast<size_t>(m) * d * 4 + static_cast<size_t>(d) * 4 * (Psi ? 2 : 1) + 1024 * 16 + 128 * 4 + 64;
    const size_t have = std::min(di0.lds_per_cu ? di0.lds_per_cu : size_t{65536},
                                 di0.lds_per_block_optin ? di0.lds_per_block_optin : size_t{65536});
    fits = need <= have && n <= di0.cus;
  }
  if (!fits) {
    // Too large for that: the same iterations as two launches each (gradient, then the fused
    // adapt-then-combine or Exact-Diffusion step in place), the first half of `work` holding the
    // gradients.  The static-scratch variant has no room for this and refuses.
    if (static_scratch) return BF_ERR_UNSUPPORTED;
    const int64_t period2 = 2 * static_cast<int64_t>(t->rounds.size());
    for (int32_t k = 0; k < iterations; ++k) {
      const int32_t r = static_cast<int32_t>((static_cast<int64_t>(round0) + k) % period2);
      rc = bf_grad_least_squares(n, m, d, A, b, X, ld, work, ld, hip_stream);
      if (rc != BF_OK) return rc;
      rc = Psi ? bf_exact_diffusion_step(t, r, X, X, work, Psi, alpha, d, ld, BF_F32, hip_stream)
               : bf_atc_step(t, r, X, X, work, nullptr, alpha, 0.0f, BF_ATC, d, ld, BF_F32, hip_stream);
      if (rc != BF_OK) return rc;
    }
    return BF_OK;
  }
  if (static_scratch) {
    // never allocates: the topology's device copy must be there already
    int dev = 0;
    BF_HIP_TRY(hipGetDevice(&dev));
    {
      std::lock_guard<std::mutex> lk(t->mu);
      for (auto& c : t->dev)
        if (c.device == dev) dc = &c;
    }
    if (!dc) return BF_ERR_UNSUPPORTED;
    rc = static_scratch_address(dev, &scratch);
    if (rc != BF_OK) return rc;
    work = reinterpret_cast<float*>(scratch);
  } else {
    rc = get_device_copy(t, false, &dc);
  }
  if (rc != BF_OK) return rc;
  DeviceInfo di;
  rc = device_info(dc->device, &di);
  if (rc != BF_OK) return rc;
  // one workgroup per agent, all resident at once, A_i in LDS
  const size_t lds = static_cast<size_t>(m) * d * 4 + static_cast<size_t>(d) * 4 * (Psi ? 2 : 1) + 1024 * 16 + 128 * 4;
  const size_t lds_max = std::min(di.lds_per_cu ? di.lds_per_cu : size_t{65536},
                                  di.lds_per_block_optin ? di.lds_per_block_optin : size_t{65536});
  if (lds + 64 > lds_max || n > di.cus) return BF_ERR_UNSUPPORTED;   // (checked above; 64: the kernel's static LDS)
  unsigned int* sync = nullptr;
  {
    std::lock_guard<std::mutex> lk(t->mu);
    if (static_scratch) {
      sync = reinterpret_cast<unsigned int*>(scratch + kStaticHalfStepBytes);
    } else {
      if (!dc->sync) BF_HIP_TRY(hipMalloc(reinterpret_cast<void**>(&dc->sync), 256));
      sync = dc->sync;
    }
    dc->last_sync = sync;
  }
  if (lds > 48 * 1024) {
    static thread_local size_t raised = 0;
    if (raised < lds) {
      BF_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(bf_dgd_ls_kernel),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds)));
      raised = lds;
    }
  }
  DgdParams p{};
  p.A = A; p.b = b; p.X = X; p.H = work; p.Psi = Psi;
  p.blob = dc->blob;
  p.sync = sync;
  p.d = d; p.ld = ld; p.n = n; p.m = m; p.iters = iterations;
  p.round_k0 = static_cast<int32_t>(static_cast<size_t>(round0) % t->rounds.size());
  p.nrounds = static_cast<int32_t>(t->rounds.size());
  p.alpha = alpha;
  p.extra_arrivals = g_tune_extra ? 1u : 0u;
  p.spin_limit = g_tune_spin > 0 ? static_cast<uint32_t>(g_tune_spin) : (1u << 20);   // of the order of a second of polling
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  hipLaunchKernelGGL(bf_sync_clear_kernel, dim3(1), dim3(64), 0, st, sync);
  BF_HIP_TRY(hipGetLastError());
  hipLaunchKernelGGL(bf_dgd_ls_kernel, dim3(n), dim3(1024), lds, st, p);
  BF_HIP_TRY(hipGetLastError());
  return BF_OK;
}

int bf_dgd_least_squares_run(const bf_topology_t* t, int32_t round0, int32_t iterations, int32_t m,
                             const float* A, const float* b, float* X, float* work, float alpha,
                             int64_t d, int64_t ld, void* hip_stream) {
  return dgd_run_common(t, round0, iterations, m, A, b, X, nullptr, false, work, alpha, d, ld, hip_stream);
}

int bf_exact_diffusion_least_squares_run(const bf_topology_t* t, int32_t round0, int32_t iterations, int32_t m,
                                         const float* A, const float* b, float* X, float* Psi_prev, float* work,
                                         float alpha, int64_t d, int64_t ld, void* hip_stream) {
  return dgd_run_common(t, round0, iterations, m, A, b, X, Psi_prev, true, work, alpha, d, ld, hip_stream);
}

int bf_dgd_least_squares_run_static(const bf_topology_t* t, int32_t round0, int32_t iterations, int32_t m,
                                    const float* A, const float* b, float* X, float alpha, int64_t d, int64_t ld,
                                    void* hip_stream) {
  return dgd_run_common(t, round0, iterations, m, A, b, X, nullptr, false, nullptr, alpha, d, ld, hip_stream, true);
}

int bf_dgd_status(const bf_topology_t* tc, int32_t* timed_out, void* hip_stream) {
  if (!tc || !timed_out) return BF_ERR_NULL;
  bf_topology_t* t = const_cast<bf_topology_t*>(tc);
  bf::DeviceCopy* dc = nullptr;
  int rc = get_device_copy(t, false, &dc);
  if (rc != BF_OK) return rc;
  *timed_out = 0;
  unsigned int* sync = nullptr;
  {
    std::lock_guard<std::mutex> lk(t->mu);
    sync = dc->last_sync;
  }
  if (!sync) return BF_OK;                           // never run on this device
  unsigned int host[2] = {0u, 0u};
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  BF_HIP_TRY(hipMemcpyAsync(host, sync, sizeof(host), hipMemcpyDeviceToHost, st));
  BF_HIP_TRY(hipStreamSynchronize(st));
  *timed_out = host[1] != 0u ? 1 : 0;
  return BF_OK;
}

int bf_blocked_pack(int32_t n, int64_t d, int64_t ld, const void* X, int64_t block, void* X_blocked,
                    bf_dtype_t dt, void* hip_stream) {
  return layout_common(true, n, d, ld, X, block, X_blocked, dt, hip_stream);
}

int bf_blocked_unpack(int32_t n, int64_t d, int64_t block, const void* X_blocked, int64_t ld, void* X,
                      bf_dtype_t dt, void* hip_stream) {
  return layout_common(false, n, d, ld, X_blocked, block, X, dt, hip_stream);
}

int bf_stream_probe(int32_t mode, const void* src, void* dst, int64_t bytes, int32_t workgroups_per_cu,
                    void* hip_stream) {
  if (mode < 0 || mode > 2) return BF_ERR_KIND;
  if ((mode != 2 && !src) || !dst) return BF_ERR_NULL;
  if (bytes < 0 || (bytes % 16) != 0 || workgroups_per_cu < 1 || workgroups_per_cu > 64) return BF_ERR_SIZE;
  if ((src && misaligned16(src)) || misaligned16(dst)) return BF_ERR_ALIGN;
  if (mode == 0 && overlaps(src, static_cast<size_t>(bytes), dst, static_cast<size_t>(bytes))) return BF_ERR_ALIAS;
  if (bytes == 0) return BF_OK;
  int dev = 0;
  BF_HIP_TRY(hipGetDevice(&dev));
  DeviceInfo di;
  int rc = device_info(dev, &di);
  if (rc != BF_OK) return rc;
  const int64_t n4 = bytes / 16;
  const int grid = static_cast<int>(std::min<int64_t>((n4 + 255) / 256, static_cast<int64_t>(di.cus) * workgroups_per_cu));
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  const f32x4* s4 = static_cast<const f32x4*>(src);
  f32x4* d4 = static_cast<f32x4*>(dst);
  if (mode == 0) hipLaunchKernelGGL(bf_stream_probe_kernel<0>, dim3(grid), dim3(256), 0, st, s4, d4, n4);
  else if (mode == 1) hipLaunchKernelGGL(bf_stream_probe_kernel<1>, dim3(grid), dim3(256), 0, st, s4, d4, n4);
  else hipLaunchKernelGGL(bf_stream_probe_kernel<2>, dim3(grid), dim3(256), 0, st, s4, d4, n4);
  BF_HIP_TRY(hipGetLastError());
  return BF_OK;
}

int bf_grad_least_squares(int32_t n, int32_t m, int64_t d, const float* A, const float* b,
                          const float* X, int64_t ldx, float* G, int64_t ldg, void* hip_stream) {
  if (!A || !b || !X || !G) return BF_ERR_NULL;
  if (n < 1 || m < 1 || m > 8192 || d < 0 || (d % 4) != 0 || ldx < d || ldg < d) return BF_ERR_SIZE;
  if ((ldx % 4) != 0 || (ldg % 4) != 0) return BF_ERR_ALIGN;
  if (misaligned16(A) || misaligned16(X) || misaligned16(G) || (reinterpret_cast<uintptr_t>(b) & 3u)) return BF_ERR_ALIGN;
  const size_t xb = (static_cast<size_t>(n - 1) * ldx + d) * 4, gb = (static_cast<size_t>(n - 1) * ldg + d) * 4;
  const size_t ab = static_cast<size_t>(n) * m * d * 4, bb = static_cast<size_t>(n) * m * 4;
  if (overlaps(G, gb, X, xb) || overlaps(G, gb, A, ab) || overlaps(G, gb, b, bb)) return BF_ERR_ALIAS;
  if (d == 0) return BF_OK;
  hipLaunchKernelGGL(bf_ls_grad_kernel, dim3(n), dim3(1024), static_cast<size_t>(m) * 4, static_cast<hipStream_t>(hip_stream),
                     A, b, X, G, m, d, ldx, ldg);
  BF_HIP_TRY(hipGetLastError());
  return BF_OK;
}

int bf_grad_quadratic(int32_t n, int64_t d, int64_t ld, const void* X, const void* C, const void* E,
                      float lam, float sigma, void* G, bf_dtype_t dt, void* hip_stream) {
  if (!X || !C || !E || !G) return BF_ERR_NULL;
  if (n < 1) return BF_ERR_SIZE;
  MatArgs ma;
  int rc = check_matrix_shape(n, d, ld, dt, &ma, true);
  if (rc != BF_OK) return rc;
  if (misaligned16(X) || misaligned16(C) || misaligned16(E) || misaligned16(G)) return BF_ERR_ALIGN;
  if (overlaps(G, ma.bytes, X, ma.bytes) || overlaps(G, ma.bytes, C, ma.bytes) || overlaps(G, ma.bytes, E, ma.bytes))
    return BF_ERR_ALIAS;
  if (d == 0) return BF_OK;
  const int per16 = dt == BF_F32 ? 4 : 8;
  const int64_t units = (d + per16 - 1) / per16 * n;
  const int grid = static_cast<int>(std::min<int64_t>((units + 255) / 256, 256 * 32));
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  if (dt == BF_F32)
    hipLaunchKernelGGL(bf_grad_quadratic_kernel<DT_F32>, dim3(grid), dim3(256), 0, st, static_cast<const char*>(X),
                       static_cast<const char*>(C), static_cast<const char*>(E), static_cast<char*>(G), n, d, ma.ld, ma.block_log, lam, sigma);
  else
    hipLaunchKernelGGL(bf_grad_quadratic_kernel<DT_BF16>, dim3(grid), dim3(256), 0, st, static_cast<const char*>(X),
                       static_cast<const char*>(C), static_cast<const char*>(E), static_cast<char*>(G), n, d, ma.ld, ma.block_log, lam, sigma);
  BF_HIP_TRY(hipGetLastError());
  return BF_OK;
}

int bf_consensus_stats(int32_t n, int64_t d, int64_t ld, const void* X, const float* p, bf_dtype_t dt,
                       double* stats, float* mean_out, void* hip_stream) {
  if (!X || !stats) return BF_ERR_NULL;
  if (n < 1) return BF_ERR_SIZE;
  MatArgs ma;
  int rc = check_matrix_shape(n, d, ld, dt, &ma, true);
  if (rc != BF_OK) return rc;
  if (misaligned16(X) || (reinterpret_cast<uintptr_t>(stats) & 7u)) return BF_ERR_ALIGN;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  hipLaunchKernelGGL(bf_stats_clear_kernel, dim3(1), dim3(64), 0, st, stats);
  BF_HIP_TRY(hipGetLastError());
  if (d == 0) return BF_OK;
  const int grid = static_cast<int>(std::min<int64_t>((d + 255) / 256, 256 * 16));
  if (dt == BF_F32)
    hipLaunchKernelGGL(bf_stats_kernel<DT_F32>, dim3(grid), dim3(256), 0, st, static_cast<const char*>(X), p, n, d, ma.ld, ma.block_log, stats, mean_out);
  else
    hipLaunchKernelGGL(bf_stats_kernel<DT_BF16>, dim3(grid), dim3(256), 0, st, static_cast<const char*>(X), p, n, d, ma.ld, ma.block_log, stats, mean_out);
  BF_HIP_TRY(hipGetLastError());
  return BF_OK;
}

}  // extern "C"
