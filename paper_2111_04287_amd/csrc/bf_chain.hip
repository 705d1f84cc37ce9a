// Row-streaming chain kernel, the gather fallback and its momentum pre-pass, with their launchers.
#include "bf_device.h"

namespace bf {

// ---------------------------------------------------------------------------------------------
// Chain kernel.  When every agent exchanges with at most two partners (ring, one-peer exponential
// rounds, matchings) the rows can be ordered into paths and cycles such that a row's in-neighbors
// sit directly before or after it.  Each thread then owns CW 16-byte column vectors and walks the
// rows in that order with three live values per vector (previous, this, next): every row is loaded
// once, combined in CSR order, and stored once.  No LDS, no barriers; all 256 threads of a
// workgroup read 4 KB of one row per step, and all workgroups walk the rows in the same order, so
// at any moment the device streams through a few rows over their whole width, like a plain copy.
// A cycle keeps its first and last rows in registers so that it closes without re-reading (which
// also makes in-place updates safe: a row is stored only after its last use as an operand).
static_assert(sizeof(bf::ChainStep) == 32, "ChainStep is read as eight dwords");

template <int DT, int OP, bool WITH_Y, int CW, int THR>
__global__ __launch_bounds__(THR) void bf_chain_kernel(const TileParams p, const int64_t nchunks) {
  constexpr int EB = Elem<DT>::bytes;
  constexpr int UC = Elem<DT>::per16;
  constexpr int UC_LOG = DT == DT_F32 ? 2 : 3;
  constexpr bool MOM = (OP == OP_MOM_ATC || OP == OP_MOM_AWC);
  constexpr bool G_ON_LOAD = (OP == OP_ATC || OP == OP_MOM_ATC || OP == OP_ED || OP == OP_TRACK);
  constexpr bool G_ON_STORE = (OP == OP_AWC || OP == OP_MOM_AWC);
  constexpr bool STATE_ON_LOAD = (OP == OP_MOM_ATC || OP == OP_ED);
  constexpr int CHUNK_LOG = (THR == 1024 ? 10 : 8) + UC_LOG;   // columns per workgroup sweep
  const int64_t d = p.d, ld = p.ld;
  const int64_t last_vec = ((d - 1) >> UC_LOG) << UC_LOG;
  const csr_i32_ptr steps = (csr_i32_ptr)(uintptr_t)p.chain;
  const int tid = threadIdx.x;

  for (int64_t cseq = blockIdx.x; cseq < nchunks; cseq += gridDim.x) {
    const int64_t chunk = p.reverse ? nchunks - 1 - cseq : cseq;   // odd rounds run right to left
    int64_t col[CW], acol[CW];     // the column, and where it lies within a row of pitch ld
    bool live[CW];
#pragma unroll
    for (int w = 0; w < CW; ++w) {
      const int64_t c = ((chunk * CW + w) << CHUNK_LOG) + (static_cast<int64_t>(tid) << UC_LOG);
      live[w] = c < d;
      col[w] = min(c, last_vec);
      acol[w] = col[w] + tile_origin(p, col[w]);
    }
    float prev[CW][UC], cur[CW][UC], nxt[CW][UC], first[CW][UC], last[CW][UC];

    // y_j = x_j, or x_j - alpha g_j, or (momentum) x_j - alpha (beta m_j + g_j) with m_j written back
    auto load_y = [&](int row, float (*out)[UC]) {
      u32x4 xr[CW], gr[CW], g2r[CW];
      f32x4 mr[CW][UC / 4];
#pragma unroll
      for (int w = 0; w < CW; ++w) {
        const int64_t off = static_cast<int64_t>(row) * ld + acol[w];
        xr[w] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p.x_in + off * EB));
        if constexpr (G_ON_LOAD) gr[w] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p.g + g_offset(p, row, col[w]) * EB));
        if constexpr (OP == OP_TRACK) g2r[w] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p.g2 + g_offset(p, row, col[w]) * EB));
        if constexpr (STATE_ON_LOAD) {
#pragma unroll
          for (int q = 0; q < UC / 4; ++q) mr[w][q] = *reinterpret_cast<const f32x4*>(p.m + m_offset(p, row, col[w]) + 4 * q);
        }
      }
#pragma unroll
      for (int w = 0; w < CW; ++w) {
        widen<DT>(xr[w], out[w]);
        if constexpr (G_ON_LOAD) {
          float gv[UC];
          widen<DT>(gr[w], gv);
          if constexpr (STATE_ON_LOAD) {
            const int64_t off = m_offset(p, row, col[w]);
#pragma unroll
            for (int q = 0; q < UC / 4; ++q) {
              float sv[4] = {mr[w][q].x, mr[w][q].y, mr[w][q].z, mr[w][q].w};
              local_update4<OP>(out[w] + 4 * q, gv + 4 * q, sv, p.alpha, p.beta);
              if (live[w]) {
                const int64_t rem = d - (col[w] + 4 * q);
                if (rem >= 4) { f32x4 t = {sv[0], sv[1], sv[2], sv[3]}; *reinterpret_cast<f32x4*>(p.m + off + 4 * q) = t; }
                else for (int e = 0; e < 4; ++e) if (e < rem) p.m[off + 4 * q + e] = sv[e];
              }
            }
          } else if constexpr (OP == OP_TRACK) {
            float hv[UC];
            widen<DT>(g2r[w], hv);
#pragma unroll
            for (int e = 0; e < UC; ++e) out[w][e] = (out[w][e] + gv[e]) - hv[e];
          } else {
#pragma unroll
            for (int e = 0; e < UC; ++e) out[w][e] = fmaf(-p.alpha, gv[e], out[w][e]);
          }
        }
      }
    };

    for (int k = 0; k < p.n; ++k) {
      // one ChainStep = eight dwords through the scalar cache
      struct { int row, flags, last_row, next_row, slots; float w[3]; } st;
      st.row = steps[8 * k + 0]; st.flags = steps[8 * k + 1]; st.last_row = steps[8 * k + 2];
      st.next_row = steps[8 * k + 3]; st.slots = steps[8 * k + 4];
      st.w[0] = __int_as_float(steps[8 * k + 5]); st.w[1] = __int_as_float(steps[8 * k + 6]);
      st.w[2] = __int_as_float(steps[8 * k + 7]);
      const int flags = st.flags;
      if (flags & 1) {
        if (flags & 2) {
          load_y(st.last_row, last);
#pragma unroll
          for (int w = 0; w < CW; ++w)
#pragma unroll
            for (int e = 0; e < UC; ++e) prev[w][e] = last[w][e];
        }
        load_y(st.row, cur);
#pragma unroll
        for (int w = 0; w < CW; ++w)
#pragma unroll
          for (int e = 0; e < UC; ++e) first[w][e] = cur[w][e];
      }
      const int nk = (flags >> 2) & 3;
      if (nk == 0) {
        load_y(st.next_row, nxt);
      } else if (nk == 1) {
#pragma unroll
        for (int w = 0; w < CW; ++w)
#pragma unroll
          for (int e = 0; e < UC; ++e) nxt[w][e] = last[w][e];
      } else if (nk == 2) {
#pragma unroll
        for (int w = 0; w < CW; ++w)
#pragma unroll
          for (int e = 0; e < UC; ++e) nxt[w][e] = first[w][e];
      }
      float acc[CW][UC];
#pragma unroll
      for (int w = 0; w < CW; ++w)
#pragma unroll
        for (int e = 0; e < UC; ++e) acc[w][e] = 0.0f;
#pragma unroll
      for (int en = 0; en < 3; ++en) {
        const int code = (st.slots >> (4 * en)) & 15;
        if (code != 15) {
          const float wt = st.w[en];
#pragma unroll
          for (int w = 0; w < CW; ++w)
#pragma unroll
            for (int e = 0; e < UC; ++e) {
              const float v = code == 0 ? prev[w][e] : (code == 1 ? cur[w][e] : nxt[w][e]);
              acc[w][e] = fmaf(wt, v, acc[w][e]);
            }
        }
      }
      // finish row st.row
#pragma unroll
      for (int w = 0; w < CW; ++w) {
        if (live[w]) {
          const int64_t off = static_cast<int64_t>(st.row) * ld + acol[w];
          const int64_t rem = d - col[w];
          if constexpr (G_ON_STORE) {
            float gv[UC];
            widen<DT>(*reinterpret_cast<const u32x4*>(p.g + g_offset(p, st.row, col[w]) * EB), gv);
            if constexpr (MOM) {
#pragma unroll
              for (int q = 0; q < UC / 4; ++q) {
                float mv[4];
                load_in<DT_F32, 4>(reinterpret_cast<const char*>(p.m), m_offset(p, st.row, col[w]) + 4 * q, mv);
#pragma unroll
                for (int e = 0; e < 4; ++e) { mv[e] = fmaf(p.beta, mv[e], gv[4 * q + e]); gv[4 * q + e] = mv[e]; }
                const int64_t r4 = rem - 4 * q;
                if (r4 > 0) {
                  float* mp = p.m + m_offset(p, st.row, col[w]) + 4 * q;
                  if (r4 >= 4) { f32x4 t = {mv[0], mv[1], mv[2], mv[3]}; *reinterpret_cast<f32x4*>(mp) = t; }
                  else for (int e = 0; e < 4; ++e) if (e < r4) mp[e] = mv[e];
                }
              }
            }
#pragma unroll
            for (int e = 0; e < UC; ++e) acc[w][e] = fmaf(-p.alpha, gv[e], acc[w][e]);
          }
          float rcp = 1.0f;
          if constexpr (WITH_Y) rcp = 1.0f / p.p_out[st.row];
#pragma unroll
          for (int h = 0; h < UC / 4; ++h) {
            const int64_t r4 = rem - 4 * h;
            if (r4 > 0) {
              const int valid = r4 >= 4 ? 4 : static_cast<int>(r4);
              if constexpr (DT == DT_BF16) if (h == 0 && rem >= 8) {
                // both halves at once: one 16-byte store of eight bf16
                u32x4 t = {pack_bf16x2(acc[w][0], acc[w][1]), pack_bf16x2(acc[w][2], acc[w][3]),
                           pack_bf16x2(acc[w][4], acc[w][5]), pack_bf16x2(acc[w][6], acc[w][7])};
                st_stream<true>(reinterpret_cast<u32x4*>(p.x_out + off * EB), t);
                if constexpr (WITH_Y) {
                  u32x4 ty = {pack_bf16x2(acc[w][0] * rcp, acc[w][1] * rcp), pack_bf16x2(acc[w][2] * rcp, acc[w][3] * rcp),
                              pack_bf16x2(acc[w][4] * rcp, acc[w][5] * rcp), pack_bf16x2(acc[w][6] * rcp, acc[w][7] * rcp)};
                  st_stream<true>(reinterpret_cast<u32x4*>(p.y + off * EB), ty);
                }
                break;
              }
              store_out<DT, 4>(p.x_out, off + 4 * h, acc[w] + 4 * h, valid);
              if constexpr (WITH_Y) {
                float yv[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) yv[e] = acc[w][4 * h + e] * rcp;
                store_out<DT, 4>(p.y, off + 4 * h, yv, valid);
              }
            }
          }
        }
      }
#pragma unroll
      for (int w = 0; w < CW; ++w)
#pragma unroll
        for (int e = 0; e < UC; ++e) { prev[w][e] = cur[w][e]; cur[w][e] = nxt[w][e]; }
    }
  }
}

// ---------------------------------------------------------------------------------------------
// Fallback for agent counts whose n x 64 tile does not fit LDS: a plain row gather.  Each thread
// owns one 16-byte vector of one output row and walks the row's in-neighbor list, reading neighbor
// vectors from global memory (re-reads are served by L2 / Infinity Cache as far as they fit).
// Out of place only.  For the momentum ops M has already been advanced by bf_momentum_kernel and
// stands in for the gradient.
template <int DT, int OP, bool WITH_Y>
__global__ __launch_bounds__(256) void bf_gather_kernel(const TileParams p) {
  constexpr int EB = Elem<DT>::bytes;
  constexpr int UC = Elem<DT>::per16;
  constexpr bool MOM = (OP == OP_MOM_ATC || OP == OP_MOM_AWC);
  constexpr bool G_IN_SUM = (OP == OP_ATC || OP == OP_MOM_ATC);
  constexpr bool G_AFTER = (OP == OP_AWC || OP == OP_MOM_AWC);
  const int64_t d = p.d, ld = p.ld;
  const int64_t upr = (d + UC - 1) / UC;
  const int64_t total = upr * p.n;
  auto load_g = [&](int64_t off, float* gv) {
    if constexpr (MOM) {
#pragma unroll
      for (int q = 0; q < UC / 4; ++q) {
        const f32x4 t = *reinterpret_cast<const f32x4*>(p.m + off + 4 * q);
        gv[4 * q] = t.x; gv[4 * q + 1] = t.y; gv[4 * q + 2] = t.z; gv[4 * q + 3] = t.w;
      }
    } else {
      widen<DT>(*reinterpret_cast<const u32x4*>(p.g + off * EB), gv);
    }
  };
  for (int64_t u = blockIdx.x * static_cast<int64_t>(blockDim.x) + threadIdx.x; u < total;
       u += static_cast<int64_t>(gridDim.x) * blockDim.x) {
    const int i = static_cast<int>(u / upr);
    const int64_t col = (u % upr) * UC;
    float acc[UC];
#pragma unroll
    for (int e = 0; e < UC; ++e) acc[e] = 0.0f;
    for (int q = p.rowptr[i]; q < p.rowptr[i + 1]; ++q) {
      const u32x2 en = p.ent[q];
      const float w = __uint_as_float(en.y);
      const int64_t off = static_cast<int64_t>(en.x) * ld + col;
      float xv[UC];
      widen<DT>(*reinterpret_cast<const u32x4*>(p.x_in + off * EB), xv);
      if constexpr (G_IN_SUM) {
        float gv[UC];
        load_g(off, gv);
#pragma unroll
        for (int e = 0; e < UC; ++e) xv[e] = fmaf(-p.alpha, gv[e], xv[e]);
      }
#pragma unroll
      for (int e = 0; e < UC; ++e) acc[e] = fmaf(w, xv[e], acc[e]);
    }
    const int64_t off = static_cast<int64_t>(i) * ld + col;
    if constexpr (G_AFTER) {
      float gv[UC];
      load_g(off, gv);
#pragma unroll
      for (int e = 0; e < UC; ++e) acc[e] = fmaf(-p.alpha, gv[e], acc[e]);
    }
    const int64_t rem = d - col;
#pragma unroll
    for (int h = 0; h < UC / 4; ++h) {
      const int valid = rem - 4 * h >= 4 ? 4 : (rem - 4 * h > 0 ? static_cast<int>(rem - 4 * h) : 0);
      if (valid > 0) {
        store_out<DT, 4>(p.x_out, off + 4 * h, acc + 4 * h, valid);
        if constexpr (WITH_Y) {
          const float rcp = 1.0f / p.p_out[i];
          float yv[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) yv[e] = acc[4 * h + e] * rcp;
          store_out<DT, 4>(p.y, off + 4 * h, yv, valid);
        }
      }
    }
  }
}

// Second fallback for large agent counts, for what the row gather cannot do: updates in place and
// the ops that carry a state or a second gradient (Exact-Diffusion, tracking).  The column-owned LDS
// tile of the main kernels narrowed to C = 32, 16, 8 or 4 columns, so that n x C fp32 values still
// fit one CU's LDS for thousands of agents; a workgroup stages its tile (local update included),
// then every thread produces 4-column pieces of output rows, walking the row's in-neighbor list
// itself (lists come through the vector caches: rows differ between the lanes of a wave).  Row
// segments of 16..128 bytes make this slow; it exists so that no valid call is refused.
template <int DT, int OP, bool WITH_Y>
__global__ __launch_bounds__(1024) void bf_narrow_kernel(const TileParams p) {
  extern __shared__ f32x4 lds_raw[];
  float* lds = reinterpret_cast<float*>(lds_raw);
  constexpr bool STAGE_G = (OP == OP_ATC || OP == OP_MOM_ATC || OP == OP_ED || OP == OP_TRACK);
  constexpr bool STAGE_M = (OP == OP_MOM_ATC || OP == OP_ED);
  const int log_c = p.log_c;                       // 2..5
  const int vpr_log = log_c - 2;                   // 4-column pieces per tile row (log2)
  const int npieces = p.n << vpr_log;
  const int64_t d = p.d, ld = p.ld;
  for (int64_t tile = blockIdx.x; tile < p.ntiles; tile += gridDim.x) {
    const int64_t c0 = tile << log_c;
    for (int u = threadIdx.x; u < npieces; u += blockDim.x) {
      const int row = u >> vpr_log;
      const int cit = (u & ((1 << vpr_log) - 1)) << 2;
      const int64_t col = c0 + cit;
      float xv[4] = {0.f, 0.f, 0.f, 0.f};
      if (col < d) {
        const int64_t off = static_cast<int64_t>(row) * ld + col + tile_origin(p, c0);
        const int64_t rem = d - col;
        // element by element: a piece may straddle d, and bf16 pieces are only 8-byte aligned
        float gv[4] = {0.f, 0.f, 0.f, 0.f}, hv[4] = {0.f, 0.f, 0.f, 0.f}, sv[4] = {0.f, 0.f, 0.f, 0.f};
        for (int e = 0; e < 4; ++e)
          if (e < rem) {
            load_in<DT, 1>(p.x_in, off + e, &xv[e]);
            if constexpr (STAGE_G) load_in<DT, 1>(p.g, g_offset(p, row, col) + e, &gv[e]);
            if constexpr (OP == OP_TRACK) load_in<DT, 1>(p.g2, g_offset(p, row, col) + e, &hv[e]);
            if constexpr (STAGE_M) sv[e] = p.m[m_offset(p, row, col) + e];
          }
        if constexpr (STAGE_M) {
          local_update4<OP>(xv, gv, sv, p.alpha, p.beta);
          for (int e = 0; e < 4; ++e) if (e < rem) p.m[m_offset(p, row, col) + e] = sv[e];
        } else if constexpr (OP == OP_TRACK) {
          for (int e = 0; e < 4; ++e) xv[e] = (xv[e] + gv[e]) - hv[e];
        } else if constexpr (STAGE_G) {
          for (int e = 0; e < 4; ++e) xv[e] = fmaf(-p.alpha, gv[e], xv[e]);
        }
      }
      f32x4 t = {xv[0], xv[1], xv[2], xv[3]};
      *reinterpret_cast<f32x4*>(lds + (row << log_c) + cit) = t;
    }
    __syncthreads();
    for (int u = threadIdx.x; u < npieces; u += blockDim.x) {
      const int i = u >> vpr_log;
      const int cit = (u & ((1 << vpr_log) - 1)) << 2;
      const int64_t col = c0 + cit;
      if (col >= d) continue;
      float acc[4] = {0.f, 0.f, 0.f, 0.f};
      for (int q = p.rowptr[i]; q < p.rowptr[i + 1]; ++q) {
        const u32x2 en = p.ent[q];
        const float w = __uint_as_float(en.y);
        const f32x4 v = *reinterpret_cast<const f32x4*>(lds + (static_cast<int>(en.x) << log_c) + cit);
        acc[0] = fmaf(w, v.x, acc[0]); acc[1] = fmaf(w, v.y, acc[1]);
        acc[2] = fmaf(w, v.z, acc[2]); acc[3] = fmaf(w, v.w, acc[3]);
      }
      const int64_t off = static_cast<int64_t>(i) * ld + col + tile_origin(p, c0);
      const int64_t rem = d - col;
      const int valid = rem >= 4 ? 4 : static_cast<int>(rem);
      if constexpr (OP == OP_AWC || OP == OP_MOM_AWC) {
        for (int e = 0; e < valid; ++e) {
          float g;
          load_in<DT, 1>(p.g, g_offset(p, i, col) + e, &g);
          if constexpr (OP == OP_MOM_AWC) { const int64_t mo = m_offset(p, i, col) + e; g = fmaf(p.beta, p.m[mo], g); p.m[mo] = g; }
          acc[e] = fmaf(-p.alpha, g, acc[e]);
        }
      }
      float rcp = 1.0f;
      if constexpr (WITH_Y) rcp = 1.0f / p.p_out[i];
      for (int e = 0; e < valid; ++e) {
        store_out<DT, 1, false>(p.x_out, off + e, &acc[e], 1);
        if constexpr (WITH_Y) { const float y = acc[e] * rcp; store_out<DT, 1, false>(p.y, off + e, &y, 1); }
      }
    }
    __syncthreads();
  }
}

// M <- beta M + G, elementwise (pre-pass of the gather fallback's momentum ops).
template <int DT>
__global__ __launch_bounds__(256) void bf_momentum_kernel(float* M, const char* G, int n, int64_t d, int64_t ld, float beta) {
  constexpr int EB = Elem<DT>::bytes;
  const int64_t upr = (d + 3) / 4;
  const int64_t total = upr * n;
  for (int64_t u = blockIdx.x * static_cast<int64_t>(blockDim.x) + threadIdx.x; u < total;
       u += static_cast<int64_t>(gridDim.x) * blockDim.x) {
    const int64_t off = (u / upr) * ld + (u % upr) * 4;
    const int64_t rem = d - (u % upr) * 4;
    float gv[4], mv[4];
    load_in<DT, 4>(G, off, gv);
    load_in<DT_F32, 4>(reinterpret_cast<const char*>(M), off, mv);
#pragma unroll
    for (int e = 0; e < 4; ++e) mv[e] = fmaf(beta, mv[e], gv[e]);
    store_out<DT_F32, 4, false>(reinterpret_cast<char*>(M), off, mv, rem >= 4 ? 4 : static_cast<int>(rem));
  }
}

template <int DT, int CW, int THR>
int launch_chain_cw(int op, bool with_y, const TileParams& tp, int64_t nchunks, int grid, hipStream_t st) {
#define BF_CHAIN(OPV, YV) hipLaunchKernelGGL((bf_chain_kernel<DT, OPV, YV, CW, THR>), dim3(grid), dim3(THR), 0, st, tp, nchunks)
  switch (op) {
    case OP_MIX: if (with_y) BF_CHAIN(OP_MIX, true); else BF_CHAIN(OP_MIX, false); break;
    case OP_ATC: if (with_y) BF_CHAIN(OP_ATC, true); else BF_CHAIN(OP_ATC, false); break;
    case OP_TRACK: BF_CHAIN(OP_TRACK, false); break;
    case OP_AWC: BF_CHAIN(OP_AWC, false); break;
    case OP_MOM_AWC: BF_CHAIN(OP_MOM_AWC, false); break;
    default:
      // the ops that carry a state matrix through the load path need more than the 128 registers
      // a 1024-thread workgroup allows: 256-thread variant only
      if constexpr (THR == 256) {
        if (op == OP_MOM_ATC) BF_CHAIN(OP_MOM_ATC, false); else BF_CHAIN(OP_ED, false);
      } else {
        return BF_ERR_UNSUPPORTED;
      }
      break;
  }
#undef BF_CHAIN
  BF_HIP_TRY(hipGetLastError());
  return BF_OK;
}

template <int DT>
int launch_chain(int op, bool with_y, int cw, bool wide, const TileParams& tp, int64_t nchunks, int grid, hipStream_t st) {
  if (wide) {   // 1024 threads: 64 KB of a row per workgroup per step
    if constexpr (DT == DT_F32) return launch_chain_cw<DT, 4, 1024>(op, with_y, tp, nchunks, grid, st);
    else return launch_chain_cw<DT, 2, 1024>(op, with_y, tp, nchunks, grid, st);
  }
  if constexpr (DT == DT_F32) {
    if (cw == 4) return launch_chain_cw<DT, 4, 256>(op, with_y, tp, nchunks, grid, st);
  }
  if (cw == 2) return launch_chain_cw<DT, 2, 256>(op, with_y, tp, nchunks, grid, st);
  return launch_chain_cw<DT, 1, 256>(op, with_y, tp, nchunks, grid, st);
}

template <int DT>
int launch_gather(int op, bool with_y, const TileParams& tp, int grid, hipStream_t st) {
#define BF_GATHER(OPV, YV) hipLaunchKernelGGL((bf_gather_kernel<DT, OPV, YV>), dim3(grid), dim3(256), 0, st, tp)
  switch (op) {
    case OP_MIX: if (with_y) BF_GATHER(OP_MIX, true); else BF_GATHER(OP_MIX, false); break;
    case OP_ATC: if (with_y) BF_GATHER(OP_ATC, true); else BF_GATHER(OP_ATC, false); break;
    case OP_AWC: BF_GATHER(OP_AWC, false); break;
    case OP_MOM_ATC: BF_GATHER(OP_MOM_ATC, false); break;
    default: BF_GATHER(OP_MOM_AWC, false); break;
  }
#undef BF_GATHER
  BF_HIP_TRY(hipGetLastError());
  return BF_OK;
}

template <int DT>
int launch_narrow(int op, bool with_y, const TileParams& tp, size_t lds, int grid, hipStream_t st) {
#define BF_NARROW(OPV, YV)                                                                                    \
  do {                                                                                                        \
    auto kern = bf_narrow_kernel<DT, OPV, YV>;                                                                \
    if (lds > 48 * 1024) {                                                                                    \
      static thread_local size_t raised = 0;                                                                  \
      if (raised < lds) {                                                                                     \
        BF_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(kern),                                   \
                                       hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds)));   \
        raised = lds;                                                                                         \
      }                                                                                                       \
    }                                                                                                         \
    hipLaunchKernelGGL(kern, dim3(grid), dim3(1024), lds, st, tp);                                            \
  } while (0)
  switch (op) {
    case OP_MIX: if (with_y) BF_NARROW(OP_MIX, true); else BF_NARROW(OP_MIX, false); break;
    case OP_ATC: if (with_y) BF_NARROW(OP_ATC, true); else BF_NARROW(OP_ATC, false); break;
    case OP_TRACK: BF_NARROW(OP_TRACK, false); break;
    case OP_AWC: BF_NARROW(OP_AWC, false); break;
    case OP_MOM_ATC: BF_NARROW(OP_MOM_ATC, false); break;
    case OP_ED: BF_NARROW(OP_ED, false); break;
    default: BF_NARROW(OP_MOM_AWC, false); break;
  }
#undef BF_NARROW
  BF_HIP_TRY(hipGetLastError());
  return BF_OK;
}

int launch_chain_f32(int op, bool with_y, int cw, bool wide, const TileParams& tp, int64_t nchunks, int grid, hipStream_t st) {
  return launch_chain<DT_F32>(op, with_y, cw, wide, tp, nchunks, grid, st);
}
int launch_chain_bf16(int op, bool with_y, int cw, bool wide, const TileParams& tp, int64_t nchunks, int grid, hipStream_t st) {
  return launch_chain<DT_BF16>(op, with_y, cw, wide, tp, nchunks, grid, st);
}
int launch_gather_f32(int op, bool with_y, const TileParams& tp, int grid, hipStream_t st) {
  return launch_gather<DT_F32>(op, with_y, tp, grid, st);
}
int launch_gather_bf16(int op, bool with_y, const TileParams& tp, int grid, hipStream_t st) {
  return launch_gather<DT_BF16>(op, with_y, tp, grid, st);
}
int launch_narrow_f32(int op, bool with_y, const TileParams& tp, size_t lds, int grid, hipStream_t st) {
  return launch_narrow<DT_F32>(op, with_y, tp, lds, grid, st);
}
int launch_narrow_bf16(int op, bool with_y, const TileParams& tp, size_t lds, int grid, hipStream_t st) {
  return launch_narrow<DT_BF16>(op, with_y, tp, lds, grid, st);
}
int launch_momentum(int dt, float* M, const char* G, int n, int64_t d, int64_t ld, float beta, int grid, hipStream_t st) {
  if (dt == BF_F32) hipLaunchKernelGGL(bf_momentum_kernel<DT_F32>, dim3(grid), dim3(256), 0, st, M, G, n, d, ld, beta);
  else hipLaunchKernelGGL(bf_momentum_kernel<DT_BF16>, dim3(grid), dim3(256), 0, st, M, G, n, d, ld, beta);
  BF_HIP_TRY(hipGetLastError());
  return BF_OK;
}

}  // namespace bf
