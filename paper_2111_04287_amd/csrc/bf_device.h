// Device-side building blocks shared by the HIP translation units of libbf (gfx950): vector types,
// bf16 conversion, streaming loads and stores, the parameter block of the tile / chain / gather
// kernels, and the launchers each translation unit exports to the dispatch code in bf_kernels.hip.
// The kernels are split over several files only so that they compile in parallel.
#ifndef BF_DEVICE_H_
#define BF_DEVICE_H_

#include <hip/hip_runtime.h>
#include <type_traits>

#include <algorithm>
#include <cstdint>
#include <cstring>

#include "bf_internal.h"

namespace bf {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

extern thread_local int g_last_hip_error;   // last failing hipError_t of this thread (defined in bf_kernels.hip)

#define BF_HIP_TRY(expr)                                  \
  do {                                                    \
    hipError_t e_ = (expr);                               \
    if (e_ != hipSuccess) {                               \
      ::bf::g_last_hip_error = static_cast<int>(e_);      \
      return BF_ERR_HIP;                                  \
    }                                                     \
  } while (0)

// ---------------------------------------------------------------------------------------------
// bf16 <-> fp32 (bfloat16 = upper half of binary32; round to nearest, ties to even)
__device__ __forceinline__ float bf16_lo(uint32_t packed) { return __uint_as_float(packed << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t packed) { return __uint_as_float(packed & 0xFFFF0000u); }
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (u >> 16) | 0x0040u;   // quiet NaN
  return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}
// Two results at once: gfx950's v_cvt_pk_bf16_f32 (round to nearest even, denormals kept, NaN made
// quiet), one instruction where the integer form above takes about eight per value.  The stores of
// the mixing kernels go through here; with bf16 storage and no fp32 state matrix those kernels are
// bound by the number of vector instructions they issue, not by HBM.
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  const f32x2 v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}

// Streaming accesses.  Every element of X, G and M is read once and written once per call, so
// loads of X and G and stores of X_out and Y carry the non-temporal hint (measured +2..5 %).
// The momentum matrix does not: with bf16 storage a lane's two 16-byte halves of M are moved by
// separate instructions, and with the hint every 128-byte line became two partial transfers
// (-25 % on the store, -2 % on the load).
template <bool NT, typename T> __device__ __forceinline__ T ld_stream(const T* ptr) {
  if constexpr (NT) return __builtin_nontemporal_load(ptr);
  else return *ptr;
}
template <bool NT, typename T> __device__ __forceinline__ void st_stream(T* ptr, const T& v) {
  if constexpr (NT) __builtin_nontemporal_store(v, ptr);
  else *ptr = v;
}

// Workgroup barrier for kernels whose waves hand data to each other through LDS only.
// __syncthreads() also waits for every outstanding GLOBAL access of the wave (vmcnt(0)), which
// drains a streaming kernel's store queue - and the loads it has prefetched - once per tile.  Here
// only the LDS accesses are waited for; global loads and stores stay in flight across the barrier.
// Safe where no wave reads global memory that another wave of the workgroup writes in the same
// launch (every kernel here: a workgroup's tiles are disjoint column ranges).
__device__ __forceinline__ void lds_barrier() {
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// Scalar-cache view of the topology: uniform addresses into these become s_load instructions.
typedef const int32_t __attribute__((address_space(4)))* csr_i32_ptr;
typedef const u32x2 __attribute__((address_space(4)))* csr_ent_ptr;

enum { OP_MIX = 0, OP_ATC = 1, OP_AWC = 2, OP_MOM_ATC = 3, OP_MOM_AWC = 4, OP_ED = 5, OP_TRACK = 6 };
// (pipelined kernel only) AWC with the gradient tile staged in LDS beside the X tile
enum { OP_AWC_LDS = 7 };
enum { DT_F32 = 0, DT_BF16 = 1 };

struct TileParams {
  const char* x_in;      // n x ld, dtype DT
  char*       x_out;
  const char* g;         // gradient, dtype DT (ATC/AWC/momentum)
  const char* g2;        // previous gradient, dtype DT (gradient-tracking update)
  float*      m;         // momentum, fp32 (momentum ops)
  char*       y;         // push-sum ratio output, dtype DT (optional)
  const float* p_out;    // push-sum weights after this round (for y)
  const int32_t* rowptr; // device CSR of the round
  const u32x2*   ent;    // {col, weight bits}
  const bf::ChainStep* chain;  // walk order of the round when it has chain structure, else null
  int64_t d, ld;
  int64_t ntiles;
  int32_t n;
  int32_t log_c;         // tile width C = 1 << log_c elements
  int64_t g_ld, m_ld;    // layouts of the gradient matrices (g, g2) and of the fp32 state matrix (m), which
  int32_t g_block_log, m_block_log;   // may differ from that of X and Y: pitch and block width as ld / block_log below
  int32_t block_log;     // 0: agent-major rows of pitch ld.  Else the column-block layout: blocks of
                         // B = 1 << block_log columns, block k an n x B row-major matrix at element
                         // k n B (ld = B; tiles never straddle a block: log_c <= block_log)
  int32_t reverse;       // walk the column tiles from the last to the first
  int32_t fuse;          // rounds applied per pass (1 = a single mix); >1 needs two LDS tiles
  // Fused rounds: the rounds before the last one (rowptr/ent hold the last) are found through the
  // table at the head of the topology's device blob, {rowptr byte offset, entry byte offset} per
  // round.  (A per-round pointer array in this struct would be indexed at run time, i.e. read from
  // the kernel-argument segment inside the tile loop, which costs microseconds per read.)
  const char* blob;
  int32_t round_k0;      // first fused round, already reduced modulo nrounds
  int32_t nrounds;
  int32_t long_rows;     // 1: the round's longest row has 5 entries or more (fp32 mix: batched LDS reads)
  int32_t rows_b;        // rows of the second LDS tile (0: n).  Smaller when the rounds that write it leave
                         // all rows from rows_b on empty and the rounds that read it never refer to them
  float alpha, beta;
};

// What to add to row * ld + column for the columns of the tile that starts at column c0: nothing
// for agent-major rows; in the column-block layout block k = c0 / B starts (n - 1) B k elements
// later than agent-major rows of pitch B would put it.
__device__ __forceinline__ int64_t tile_origin(const TileParams& p, int64_t c0) {
  return p.block_log ? ((c0 >> p.block_log) * (p.n - 1)) << p.block_log : int64_t{0};
}

// Element offset of column `col` of agent `row` in the gradient matrices, whose layout is their own.
__device__ __forceinline__ int64_t g_offset(const TileParams& p, int64_t row, int64_t col) {
  return row * p.g_ld + col + (p.g_block_log ? ((col >> p.g_block_log) * (p.n - 1)) << p.g_block_log : int64_t{0});
}
// The same for the fp32 state matrix (momentum, psi of Exact-Diffusion).
__device__ __forceinline__ int64_t m_offset(const TileParams& p, int64_t row, int64_t col) {
  return row * p.m_ld + col + (p.m_block_log ? ((col >> p.m_block_log) * (p.n - 1)) << p.m_block_log : int64_t{0});
}

// Parameters of the kernel that runs uniform shift rounds in registers (bf_shift.hip).
struct ShiftParams {
  const char* x_in;
  char*       x_out;
  int64_t d, ld, ntiles;
  int32_t n;             // 64, 128, 192 or 256
  int32_t log_c;         // tile width
  int32_t block_log;     // as in TileParams: 0 agent-major, else column blocks of 1 << block_log (ld = that)
  int32_t reverse;
  int32_t count;         // rounds per pass, 1..8
  int32_t shift[8];      // per round: s in x_i <- w_self x_i + w_peer x_((i+s) mod n)
  float   w_self[8], w_peer[8];
};

template <int DT> struct Elem { static constexpr int bytes = DT == DT_F32 ? 4 : 2; static constexpr int per16 = 16 / bytes; };

// Load 16 bytes of X/G and widen to fp32.
template <int DT>
__device__ __forceinline__ void widen(const u32x4& raw, float* out) {
  if constexpr (DT == DT_F32) {
    out[0] = __uint_as_float(raw.x); out[1] = __uint_as_float(raw.y);
    out[2] = __uint_as_float(raw.z); out[3] = __uint_as_float(raw.w);
  } else {
    out[0] = bf16_lo(raw.x); out[1] = bf16_hi(raw.x); out[2] = bf16_lo(raw.y); out[3] = bf16_hi(raw.y);
    out[4] = bf16_lo(raw.z); out[5] = bf16_hi(raw.z); out[6] = bf16_lo(raw.w); out[7] = bf16_hi(raw.w);
  }
}

// Store LW consecutive results of dtype DT at element offset `off` of row base `base`;
// `valid` = how many of them lie below d.
template <int DT, int LW, bool NT = true>
__device__ __forceinline__ void store_out(char* base, int64_t off, const float* v, int valid) {
  if constexpr (DT == DT_F32) {
    float* ptr = reinterpret_cast<float*>(base) + off;
    if (valid >= LW) {
      if constexpr (LW == 4) { f32x4 t = {v[0], v[1], v[2], v[3]}; st_stream<NT>(reinterpret_cast<f32x4*>(ptr), t); }
      else if constexpr (LW == 2) { f32x2 t = {v[0], v[1]}; st_stream<NT>(reinterpret_cast<f32x2*>(ptr), t); }
      else { st_stream<NT>(ptr, v[0]); }
    } else {
      for (int k = 0; k < LW; ++k) if (k < valid) ptr[k] = v[k];
    }
  } else {
    uint16_t* ptr = reinterpret_cast<uint16_t*>(base) + off;
    if (valid >= LW) {
      if constexpr (LW == 4) { u32x2 t = {pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3])}; st_stream<NT>(reinterpret_cast<u32x2*>(ptr), t); }
      else if constexpr (LW == 2) { st_stream<NT>(reinterpret_cast<uint32_t*>(ptr), pack_bf16x2(v[0], v[1])); }
      else { ptr[0] = static_cast<uint16_t>(f32_to_bf16_bits(v[0])); }
    } else {
      for (int k = 0; k < LW; ++k) if (k < valid) ptr[k] = static_cast<uint16_t>(f32_to_bf16_bits(v[k]));
    }
  }
}

// Load LW consecutive values of dtype DT (all below ld, so in bounds) and widen.
template <int DT, int LW, bool NT = false>
__device__ __forceinline__ void load_in(const char* base, int64_t off, float* v) {
  if constexpr (DT == DT_F32) {
    const float* ptr = reinterpret_cast<const float*>(base) + off;
    if constexpr (LW == 4) { f32x4 t = ld_stream<NT>(reinterpret_cast<const f32x4*>(ptr)); v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w; }
    else if constexpr (LW == 2) { f32x2 t = *reinterpret_cast<const f32x2*>(ptr); v[0] = t.x; v[1] = t.y; }
    else { v[0] = ptr[0]; }
  } else {
    const uint16_t* ptr = reinterpret_cast<const uint16_t*>(base) + off;
    if constexpr (LW == 4) { u32x2 t = ld_stream<NT>(reinterpret_cast<const u32x2*>(ptr)); v[0] = bf16_lo(t.x); v[1] = bf16_hi(t.x); v[2] = bf16_lo(t.y); v[3] = bf16_hi(t.y); }
    else if constexpr (LW == 2) { uint32_t t = *reinterpret_cast<const uint32_t*>(ptr); v[0] = bf16_lo(t); v[1] = bf16_hi(t); }
    else { v[0] = __uint_as_float(static_cast<uint32_t>(ptr[0]) << 16); }
  }
}

// Local update of four columns of one agent while its row is staged, for the ops that carry an
// fp32 state matrix.  In: xv = x, gv = g, st = state.  Out: xv = the value to be mixed, st = the new
// state to write back.
//   OP_MOM_ATC (heavy-ball momentum, adapt-then-combine): m <- beta m + g;  mixed value x - alpha m.
//   OP_ED (Exact-Diffusion, eqs. ed-1, ed-2): psi = x - alpha g;  phi = psi + x - psi_prev;
//          mixed value phi, state <- psi.
template <int OP>
__device__ __forceinline__ void local_update4(float* xv, const float* gv, float* st, float alpha, float beta) {
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    if constexpr (OP == OP_ED) {
      const float psi = fmaf(-alpha, gv[e], xv[e]);
      xv[e] = (psi + xv[e]) - st[e];
      st[e] = psi;
    } else {
      st[e] = fmaf(beta, st[e], gv[e]);
      xv[e] = fmaf(-alpha, st[e], xv[e]);
    }
  }
}

// Launch shape of the tile kernel, chosen on the host.
struct Shape { int log_c; int lw; int wgs_per_cu; int threads; size_t lds_bytes; bool stream; };

// Launchers, one translation unit per storage type for the tile kernel.  All return a bf status.
int launch_tile_op_f32(int op, bool with_y, const TileParams& tp, const Shape& s, int grid, hipStream_t st);
int launch_tile_op_bf16(int op, bool with_y, const TileParams& tp, const Shape& s, int grid, hipStream_t st);
int launch_pipe_op_f32(int op, bool with_y, const TileParams& tp, const Shape& s, int grid, hipStream_t st);
int launch_pipe_op_bf16(int op, bool with_y, const TileParams& tp, const Shape& s, int grid, hipStream_t st);
int launch_chain_f32(int op, bool with_y, int cw, bool wide, const TileParams& tp, int64_t nchunks, int grid, hipStream_t st);
int launch_chain_bf16(int op, bool with_y, int cw, bool wide, const TileParams& tp, int64_t nchunks, int grid, hipStream_t st);
int launch_gather_f32(int op, bool with_y, const TileParams& tp, int grid, hipStream_t st);
int launch_gather_bf16(int op, bool with_y, const TileParams& tp, int grid, hipStream_t st);
int launch_narrow_f32(int op, bool with_y, const TileParams& tp, size_t lds, int grid, hipStream_t st);
int launch_narrow_bf16(int op, bool with_y, const TileParams& tp, size_t lds, int grid, hipStream_t st);
// M <- beta M + G for the gather fallback's momentum ops; G has storage type dt (BF_F32 / BF_BF16).
int launch_dense(int rb, const float* xi, float* xo, const float* wt, int n, int64_t d, int64_t ld, int block_log,
                 int cus, size_t lds_cu, hipStream_t st);
int launch_shift_rounds(int dt, const ShiftParams& p, int grid, size_t lds, hipStream_t st);
int launch_momentum(int dt, float* M, const char* G, int n, int64_t d, int64_t ld, float beta, int grid, hipStream_t st);

}  // namespace bf

#endif  // BF_DEVICE_H_
