// Dense W X on the fp32 matrix cores (v_mfma_f32_32x32x2_f32: true fp32 operands, fp32 accumulate),
// for weight matrices given in dense form (fully connected W, periodic global averaging) and as an
// independent cross-check of the list kernels.
//
// v_mfma_f32_32x32x2_f32 operand layout (wave64): A lane l holds A[l%32][l/32], B lane l holds
// B[l/32][l%32], D register v of lane l holds D[8*(v/4) + 4*(l/32) + v%4][l%32].
//
// A persistent workgroup owns two LDS tiles of NP x TC input values (NP = n rounded up to 32).  A
// wave owns ONE block of 32 output rows and keeps that block's slice of W -- 32 x NP values, NP/2
// registers per lane -- in registers for the whole launch, so the multiply loop reads nothing but
// the B operand from LDS (one 4-byte read per lane per MFMA).  Waves that share a row block split
// the tile's 32-column blocks between them.  The next tile's loads are issued before the multiply
// loop and land in the other LDS tile after it, so HBM reads run under the MFMAs; results go from
// the accumulators straight to global memory (each store instruction writes two 128-byte row
// pieces), so there is one workgroup barrier per tile.
#include "bf_device.h"

namespace bf {


// RB: 32-row blocks of W.  WPR: waves per row block.  CPW: 32-column blocks per wave.
template <int RB, int WPR, int CPW>
__global__ __launch_bounds__(RB * WPR * 64) void bf_dense_kernel(const float* x_in, float* x_out, const float* wt,
                                                                  int n, int64_t d, int64_t ld, int64_t ntiles,
                                                                  int block_log) {
  constexpr int NP = RB * 32;
  constexpr int NW = RB * WPR;
  constexpr int THREADS = NW * 64;
  constexpr int TC = 32 * WPR * CPW;          // tile width in columns
  // LDS rows are TC floats with no padding; odd rows keep their columns XOR 32, so that the two
  // half-waves of a B read (rows 2 k2 and 2 k2 + 1, the same 32 columns) fall on disjoint banks
  constexpr int P = TC;
  constexpr int UPR = TC / 4;                 // 16-byte units per tile row
  constexpr int PF = 4 * CPW;                 // units per thread: NP * UPR / THREADS
  static_assert(TC >= 64, "the swizzle exchanges 32-column halves of a 64-column group");
  static_assert(NP * UPR == PF * THREADS, "a tile is a whole number of units per thread");
  extern __shared__ f32x4 lds_raw[];
  float* lds = reinterpret_cast<float*>(lds_raw);
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, lh = lane >> 5;
  const int rb = wave / WPR, cw = wave % WPR;
  const int64_t last_vec = ((d - 1) >> 2) << 2;

  // this wave's slice of W: A[i = rb*32 + l32][k = 2*k2 + lh] = w_ik = wt[k * NP + i]
  float areg[NP / 2];
#pragma unroll
  for (int k2 = 0; k2 < NP / 2; ++k2) areg[k2] = wt[static_cast<size_t>(2 * k2 + lh) * NP + rb * 32 + l32];

  // the padding rows n..NP-1 of both tiles are zero for the whole launch (never loaded into)
  for (int u = tid; u < (NP - n) * UPR; u += THREADS) {
    const f32x4 z = {0.f, 0.f, 0.f, 0.f};
    const int row = n + u / UPR, cit = (u % UPR) * 4;       // (zeros: the swizzle does not matter)
    *reinterpret_cast<f32x4*>(lds + row * P + cit) = z;
    *reinterpret_cast<f32x4*>(lds + NP * P + row * P + cit) = z;
  }

  auto origin = [&](int64_t c0) {             // column blocks: see tile_origin() in bf_device.h
    return block_log ? ((c0 >> block_log) * (n - 1)) << block_log : int64_t{0};
  };
  f32x4 pf[PF];
  auto issue_loads = [&](int64_t tile) {
    const int64_t c0 = tile * TC;
    const int64_t t0 = origin(c0);
#pragma unroll
    for (int k = 0; k < PF; ++k) {
      const int u = tid + k * THREADS;
      const int row = min(u / UPR, n - 1);
      const int64_t col = min(c0 + (u % UPR) * 4, last_vec);
      pf[k] = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(x_in + static_cast<int64_t>(row) * ld + col + t0));
    }
  };
  auto land = [&](float* buf) {
#pragma unroll
    for (int k = 0; k < PF; ++k) {
      const int u = tid + k * THREADS;
      const int row = u / UPR;
      if (row < n) *reinterpret_cast<f32x4*>(buf + row * P + (((u % UPR) * 4) ^ ((row & 1) << 5))) = pf[k];
    }
  };

  int64_t tile = blockIdx.x;
  if (tile >= ntiles) return;
  issue_loads(tile);
  land(lds);
  lds_barrier();
  int cur = 0;
  while (tile < ntiles) {
    const int64_t next = tile + gridDim.x;
    if (next < ntiles) issue_loads(next);
    const float* brow = lds + cur * (NP * P) + lh * P;        // row 2 k2 + lh has the parity of lh
    int bcol[CPW];
#pragma unroll
    for (int j = 0; j < CPW; ++j) bcol[j] = ((cw * CPW + j) * 32 + l32) ^ (lh << 5);
    f32x16 acc[CPW];
#pragma unroll
    for (int j = 0; j < CPW; ++j) acc[j] = f32x16{0};
#pragma unroll
    for (int k2 = 0; k2 < NP / 2; ++k2) {
#pragma unroll
      for (int j = 0; j < CPW; ++j)
        acc[j] = __builtin_amdgcn_mfma_f32_32x32x2f32(areg[k2], brow[2 * k2 * P + bcol[j]], acc[j], 0, 0, 0);
    }
    const int64_t c0 = tile * TC;
    const int64_t t0 = origin(c0);
#pragma unroll
    for (int j = 0; j < CPW; ++j) {
      const int64_t col = c0 + (cw * CPW + j) * 32 + l32;
      if (col < d) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int row = rb * 32 + 8 * (v / 4) + 4 * lh + (v % 4);
          if (row < n) __builtin_nontemporal_store(acc[j][v], x_out + static_cast<int64_t>(row) * ld + col + t0);
        }
      }
    }
    if (next < ntiles) land(lds + (cur ^ 1) * (NP * P));
    lds_barrier();
    tile = next;
    cur ^= 1;
  }
}

template <int RB, int WPR, int CPW>
int launch_dense_shape(const float* xi, float* xo, const float* wt, int n, int64_t d, int64_t ld, int block_log,
                       int cus, size_t lds_cu, hipStream_t st) {
  constexpr int TC = 32 * WPR * CPW;
  if (block_log && (int64_t{1} << block_log) < TC) return BF_ERR_UNSUPPORTED;
  const size_t lds = 2 * static_cast<size_t>(RB * 32) * TC * 4;
  if (lds > lds_cu) return BF_ERR_UNSUPPORTED;
  const int64_t ntiles = (d + TC - 1) / TC;
  // as many workgroups per CU as LDS and the 2048-thread limit allow, at most two
  const int per_cu = static_cast<int>(std::max<size_t>(1, std::min<size_t>({size_t{2}, lds_cu / lds, size_t{2048} / (RB * WPR * 64)})));
  const int grid = static_cast<int>(std::min<int64_t>(ntiles, static_cast<int64_t>(cus) * per_cu));
  auto kern = bf_dense_kernel<RB, WPR, CPW>;
  if (lds > 48 * 1024) {
    static thread_local size_t raised = 0;
    if (raised < lds) {
      BF_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                     static_cast<int>(lds)));
      raised = lds;
    }
  }
  hipLaunchKernelGGL(kern, dim3(grid), dim3(RB * WPR * 64), lds, st, xi, xo, wt, n, d, ld, ntiles, block_log);
  BF_HIP_TRY(hipGetLastError());
  return BF_OK;
}

// rb = n_pad / 32 in 1..8.  Waves per row block and column blocks per wave: 8 to 12 waves per
// workgroup where the registers allow (the W slice is 16 rb registers per lane), tiles of 64
// columns for the large matrices so that two tiles fit 160 KB of LDS.
int launch_dense(int rb, const float* xi, float* xo, const float* wt, int n, int64_t d, int64_t ld, int block_log,
                 int cus, size_t lds_cu, hipStream_t st) {
  switch (rb) {
    case 1: return launch_dense_shape<1, 8, 1>(xi, xo, wt, n, d, ld, block_log, cus, lds_cu, st);
    case 2: return launch_dense_shape<2, 4, 1>(xi, xo, wt, n, d, ld, block_log, cus, lds_cu, st);
    case 3: return launch_dense_shape<3, 4, 1>(xi, xo, wt, n, d, ld, block_log, cus, lds_cu, st);
    case 4: return launch_dense_shape<4, 2, 2>(xi, xo, wt, n, d, ld, block_log, cus, lds_cu, st);
    case 5: return launch_dense_shape<5, 2, 1>(xi, xo, wt, n, d, ld, block_log, cus, lds_cu, st);
    case 6: return launch_dense_shape<6, 2, 1>(xi, xo, wt, n, d, ld, block_log, cus, lds_cu, st);
    case 7: return launch_dense_shape<7, 1, 2>(xi, xo, wt, n, d, ld, block_log, cus, lds_cu, st);
    case 8: return launch_dense_shape<8, 1, 2>(xi, xo, wt, n, d, ld, block_log, cus, lds_cu, st);
    default: return BF_ERR_UNSUPPORTED;
  }
}

}  // namespace bf
