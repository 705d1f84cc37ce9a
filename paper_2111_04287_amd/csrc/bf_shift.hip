// Several rounds of partial averaging per pass for rounds of the form
//     x_i <- w_self x_i + w_peer x_((i + s) mod n)        (same s and weights for every agent),
// which is what every round of the one-peer exponential graph is (s = 2^r, weights 1/2, 1/2).
// A column tile is staged into LDS once, and the rounds then run in REGISTERS: agent i = 64 q + lane
// sits in register q of lane `lane`, so for s < 64 the partner (i + s) mod n is a rotation of the
// wave by s lanes (ds_bpermute: the LDS crossbar, no memory) with a carry into the next register,
// and for s = 64 a it is the same lane of register q + a, which costs nothing.  (Shifts with both a
// lane part and a register part are left to the general kernel.)  No LDS traffic and no
// list lookups per round; a pass costs one read and one write of the matrix whatever the number of
// rounds.  The arithmetic per round and row is the two-entry list of the general kernels, in the
// same order (lower agent index first), so fp32 results are bit-identical to separate rounds.
#include "bf_device.h"

namespace bf {

// 512 threads, two workgroups per CU (64 KB tile each): the kernel needs about 100 vector registers,
// which two 8-wave workgroups can have and two 16-wave ones could not.
template <int DT, int R>
__global__ __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(4, 4))) void bf_shift_rounds_kernel(const ShiftParams p) {
  extern __shared__ f32x4 lds_raw[];
  float* lds = reinterpret_cast<float*>(lds_raw);
  __shared__ int32_t sh_shift[8];
  __shared__ float sh_ws[8], sh_wp[8];

  constexpr int N = 64 * R;
  constexpr int EB = Elem<DT>::bytes;
  constexpr int UC = Elem<DT>::per16;               // columns per 16-byte unit of storage
  constexpr int UC_LOG = DT == DT_F32 ? 2 : 3;
  constexpr int MAXPF = DT == DT_F32 ? 8 : 4;       // units per thread: a 64 KB fp32 tile, 512 threads
  constexpr int THREADS = 512, NW = 8;

  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lane = tid & 63;
  const int log_c = p.log_c;
  // Row pitch C + 4 floats: rows stay 16-byte aligned, and the 64 lanes of a transposed 16-byte
  // read (lane = agent, stride one row) fall on distinct banks eight lanes at a time.
  const int pitch = (1 << log_c) + 4;
  const int upr_log = log_c - UC_LOG;
  const int upr_mask = (1 << upr_log) - 1;
  const int nunits = N << upr_log;
  const int64_t d = p.d, ld = p.ld;
  const int64_t last_vec = d > 0 ? ((d - 1) >> UC_LOG) << UC_LOG : 0;

  // the rounds' parameters go to LDS once: indexing the kernel-argument arrays with a run-time
  // round number inside the tile loop would read the argument segment again and again
  if (tid < p.count) { sh_shift[tid] = p.shift[tid]; sh_ws[tid] = p.w_self[tid]; sh_wp[tid] = p.w_peer[tid]; }

  // A thread's MAXPF units lie in the same columns of rows row0, row0 + rstep, ...: one address and
  // uniform strides, instead of MAXPF 64-bit addresses held in registers across the tile loop.
  const int row0 = tid >> upr_log;
  const int cit0 = (tid & upr_mask) << UC_LOG;
  const int rstep = THREADS >> upr_log;             // rows per step (N * C / UC is a multiple of THREADS)
  const int64_t step_bytes = static_cast<int64_t>(rstep) * ld * EB;
  const int nsteps = nunits / THREADS;              // <= MAXPF: the host keeps N * C within 16384 elements
  u32x4 xr[MAXPF];
  // column blocks: block k of the tile's columns starts (n - 1) B k elements later than rows of pitch B would put it
  auto block_origin = [&](int64_t c0) {
    return p.block_log ? ((c0 >> p.block_log) * (N - 1)) << p.block_log : int64_t{0};
  };
  auto issue_loads = [&](int64_t tile) {
    const int64_t col = min((tile << log_c) + cit0, last_vec);
    const char* src = p.x_in + (static_cast<int64_t>(row0) * ld + col + block_origin(tile << log_c)) * EB;
#pragma unroll
    for (int k = 0; k < MAXPF; ++k)
      if (k < nsteps) xr[k] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(src + k * step_bytes));
  };

  auto phys = [&](int64_t seq) { return p.reverse ? p.ntiles - 1 - seq : seq; };
  int64_t seq = blockIdx.x;
  if (seq < p.ntiles) issue_loads(phys(seq));
  while (seq < p.ntiles) {
    const int64_t tile = phys(seq);
    const int64_t c0 = tile << log_c;
    // stage: fp32 values into the padded tile (columns at or past d hold copies of the last vector
    // and are never stored)
    float* const mine = lds + row0 * pitch + cit0;
#pragma unroll
    for (int k = 0; k < MAXPF; ++k) {
      if (k >= nsteps) break;
      float xv[UC];
      widen<DT>(xr[k], xv);
      float* dst = mine + k * rstep * pitch;
#pragma unroll
      for (int q = 0; q < UC / 4; ++q) {
        f32x4 t = {xv[4 * q], xv[4 * q + 1], xv[4 * q + 2], xv[4 * q + 3]};
        *reinterpret_cast<f32x4*>(dst + 4 * q) = t;
      }
    }
    lds_barrier();
    const int64_t next = seq + gridDim.x;
    if (next < p.ntiles) issue_loads(phys(next));     // in flight during the rounds

    // the rounds, four columns per wave at a time
    for (int cg = wave; cg < (1 << (log_c - 2)); cg += NW) {
      float x[R][4];
#pragma unroll
      for (int q = 0; q < R; ++q) {
        const f32x4 t = *reinterpret_cast<const f32x4*>(lds + (64 * q + lane) * pitch + 4 * cg);
        x[q][0] = t.x; x[q][1] = t.y; x[q][2] = t.z; x[q][3] = t.w;
      }
      for (int r = 0; r < p.count; ++r) {
        const int s = __builtin_amdgcn_readfirstlane(sh_shift[r]);
        const float ws = __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(sh_ws[r])));
        const float wp = __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(sh_wp[r])));
        if (s < 64) {
          // Rotation by s lanes.  Register q's partner is lane + s of the same register, or of the
          // next one where lane + s runs past the wave.  The row's list is {i, (i+s) mod n} in
          // ascending order, so the partner comes first where i + s wraps round n: only in the last
          // register, in the lanes that carry.  One column at a time keeps the live values few.
          const int src = ((lane + s) & 63) << 2;
          const bool carry = lane + s >= 64;
          const float wf = carry ? wp : ws, wl = carry ? ws : wp;
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            float rot[R];
#pragma unroll
            for (int q = 0; q < R; ++q) rot[q] = __int_as_float(__builtin_amdgcn_ds_bpermute(src, __float_as_int(x[q][e])));
#pragma unroll
            for (int q = 0; q < R; ++q) {
              const float peer = carry ? rot[(q + 1) % R] : rot[q];
              if (q < R - 1) {
                x[q][e] = fmaf(wp, peer, fmaf(ws, x[q][e], 0.0f));
              } else {
                const float first = carry ? peer : x[q][e], last = carry ? x[q][e] : peer;
                x[q][e] = fmaf(wl, last, fmaf(wf, first, 0.0f));
              }
            }
          }
        } else {
          // s = 64 a: the partner is the same lane of register (q + a) mod R, and i + s wraps round n
          // exactly in the registers with q + a >= R.  a is uniform: one unrolled case each.
          auto apply = [&](auto ac) {
            constexpr int A = decltype(ac)::value;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              float old[R];
#pragma unroll
              for (int q = 0; q < R; ++q) old[q] = x[q][e];
#pragma unroll
              for (int q = 0; q < R; ++q) {
                const float peer = old[(q + A) % R];
                x[q][e] = (q + A >= R) ? fmaf(ws, old[q], fmaf(wp, peer, 0.0f)) : fmaf(wp, peer, fmaf(ws, old[q], 0.0f));
              }
            }
          };
          switch (s >> 6) {
            case 1: if constexpr (R > 1) apply(std::integral_constant<int, 1>{}); break;
            case 2: if constexpr (R > 2) apply(std::integral_constant<int, 2>{}); break;
            default: if constexpr (R > 3) apply(std::integral_constant<int, 3>{}); break;
          }
        }
      }
#pragma unroll
      for (int q = 0; q < R; ++q) {
        f32x4 t = {x[q][0], x[q][1], x[q][2], x[q][3]};
        *reinterpret_cast<f32x4*>(lds + (64 * q + lane) * pitch + 4 * cg) = t;
      }
    }
    lds_barrier();
    // store the tile, row-major and coalesced
    {
      const int64_t col = c0 + cit0;
      const int64_t rem = d - col;                   // columns of this thread's units that exist
      char* dstp = p.x_out + (static_cast<int64_t>(row0) * ld + col + block_origin(c0)) * EB;
      if (rem >= UC) {
#pragma unroll
        for (int k = 0; k < MAXPF; ++k) {
          if (k >= nsteps) break;
          const float* src = mine + k * rstep * pitch;
          if constexpr (DT == DT_BF16) {
            const f32x4 t0 = *reinterpret_cast<const f32x4*>(src), t1 = *reinterpret_cast<const f32x4*>(src + 4);
            u32x4 o = {pack_bf16x2(t0.x, t0.y), pack_bf16x2(t0.z, t0.w), pack_bf16x2(t1.x, t1.y), pack_bf16x2(t1.z, t1.w)};
            __builtin_nontemporal_store(o, reinterpret_cast<u32x4*>(dstp + k * step_bytes));
          } else {
            const f32x4 t = *reinterpret_cast<const f32x4*>(src);
            __builtin_nontemporal_store(t, reinterpret_cast<f32x4*>(dstp + k * step_bytes));
          }
        }
      } else if (rem > 0) {
        // the ragged end of the last tile, element by element
        for (int k = 0; k < nsteps; ++k)
          for (int e = 0; e < static_cast<int>(rem); ++e) {
            const float v = mine[k * rstep * pitch + e];
            store_out<DT, 1, false>(dstp + k * step_bytes, e, &v, 1);
          }
      }
    }
    lds_barrier();
    seq = next;
  }
}

template <int DT>
int launch_shift_dt(const ShiftParams& p, int grid, size_t lds, hipStream_t st) {
#define BF_SHIFT(RV)                                                                                         \
  do {                                                                                                       \
    auto kern = bf_shift_rounds_kernel<DT, RV>;                                                              \
    if (lds > 48 * 1024) {                                                                                   \
      static thread_local size_t raised = 0;                                                                 \
      if (raised < lds) {                                                                                    \
        BF_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(kern),                                  \
                                       hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds))); \
        raised = lds;                                                                                        \
      }                                                                                                      \
    }                                                                                                        \
    hipLaunchKernelGGL(kern, dim3(grid), dim3(512), lds, st, p);                                             \
  } while (0)
  switch (p.n / 64) {
    case 1: BF_SHIFT(1); break;
    case 2: BF_SHIFT(2); break;
    case 3: BF_SHIFT(3); break;
    case 4: BF_SHIFT(4); break;
    default: return BF_ERR_UNSUPPORTED;
  }
#undef BF_SHIFT
  BF_HIP_TRY(hipGetLastError());
  return BF_OK;
}

int launch_shift_rounds(int dt, const ShiftParams& p, int grid, size_t lds, hipStream_t st) {
  return dt == BF_F32 ? launch_shift_dt<DT_F32>(p, grid, lds, st) : launch_shift_dt<DT_BF16>(p, grid, lds, st);
}

}  // namespace bf
