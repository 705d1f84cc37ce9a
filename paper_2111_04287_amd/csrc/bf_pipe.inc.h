// The pipelined column-tile kernel and its launchers (template code; included by bf_tile_f32.hip
// and bf_tile_bf16.hip, which instantiate it for one storage type each).
#ifndef BF_PIPE_INC_H_
#define BF_PIPE_INC_H_

#include "bf_device.h"

namespace bf {

template <int NB> struct RawVec;
template <> struct RawVec<16> { typedef u32x4 type; };
template <> struct RawVec<8> { typedef u32x2 type; };

// Widen one staging unit of UC columns of storage type DT to fp32.
template <int DT, int UC, typename R>
__device__ __forceinline__ void widen_unit(const R& raw, float* out) {
  if constexpr (DT == DT_F32) {
    out[0] = __uint_as_float(raw.x); out[1] = __uint_as_float(raw.y);
    out[2] = __uint_as_float(raw.z); out[3] = __uint_as_float(raw.w);
  } else if constexpr (UC == 8) {
    out[0] = bf16_lo(raw.x); out[1] = bf16_hi(raw.x); out[2] = bf16_lo(raw.y); out[3] = bf16_hi(raw.y);
    out[4] = bf16_lo(raw.z); out[5] = bf16_hi(raw.z); out[6] = bf16_lo(raw.w); out[7] = bf16_hi(raw.w);
  } else {
    out[0] = bf16_lo(raw.x); out[1] = bf16_hi(raw.x); out[2] = bf16_lo(raw.y); out[3] = bf16_hi(raw.y);
  }
}

// ---------------------------------------------------------------------------------------------
// One persistent workgroup per CU owns two n x C fp32 tiles in LDS and splits its waves into two
// roles.  The NL loader waves stream the next column tile from HBM, U 16-byte vectors per lane in
// flight at a time, apply the local update (x - alpha g; momentum; Exact-Diffusion; tracking) and
// put the values to be mixed into one LDS tile.  The NR reducer waves meanwhile produce the output
// rows of the previous tile from the other LDS tile -- one wave per (row, 64*LW-column span), the
// row's in-neighbor list read through the scalar cache, fp32 accumulation in list order -- and
// store them.  The two roles meet at one workgroup barrier per tile.  A CU thus issues loads and
// stores all the time, a few KB of each in flight, instead of a tile-sized burst of one kind
// followed by a burst of the other.
//
// DT: storage type of X/G/Y.  OP: what is staged and what is subtracted.  WITH_Y: also write the
// push-sum ratio.  LW: columns per lane in the reduce phase.
template <int DT, int OP, bool WITH_Y, int LW, int NL, int NR, int U, bool STREAM>
__global__ __launch_bounds__((NL + NR) * 64) void bf_pipe_kernel(const TileParams p) {
  extern __shared__ f32x4 lds_raw[];
  float* lds = reinterpret_cast<float*>(lds_raw);

  constexpr int EB = Elem<DT>::bytes;
  // OP_AWC_LDS: adapt-while-communicate with the gradients staged, as fp32, in n more rows of each
  // LDS tile (row n + i holds agent i's): the reducer then takes its own gradient as one more LDS
  // read behind the row's list instead of fetching it from HBM between its stores.
  constexpr bool G_LDS = (OP == OP_AWC_LDS);
  constexpr bool STAGE_G = (OP == OP_ATC || OP == OP_MOM_ATC || OP == OP_ED || OP == OP_TRACK || G_LDS);
  constexpr bool STAGE_G2 = (OP == OP_TRACK);
  constexpr bool STAGE_M = (OP == OP_MOM_ATC || OP == OP_ED);
  // A staging unit is 16 bytes of X, except next to an fp32 state matrix with bf16 storage: there
  // it is four columns (8 bytes of X and G, 16 bytes of M), so that every wave-wide access of M is
  // one contiguous kilobyte.
  constexpr int UC = (DT == DT_BF16 && !STAGE_M) ? 8 : 4;
  constexpr int UC_LOG = UC == 8 ? 3 : 2;
  typedef typename RawVec<UC * EB>::type raw_t;
  constexpr int LT = NL * 64;                       // loader threads

  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lane = tid & 63;
  const int log_c = p.log_c;
  const int upr_log = log_c - UC_LOG;               // staging units per tile row (log2)
  const int upr_mask = (1 << upr_log) - 1;
  const int nunits = p.n << upr_log;
  const int64_t d = p.d, ld = p.ld;
  // A row of a tile is at most 256 staging units and LT is a multiple of 256: a loader lane keeps
  // its column through all its units of a tile and moves down LT / (units per row) rows from one
  // unit to the next, so an address is the previous one plus a wave-uniform step -- two additions
  // where row x pitch would be a 64-bit product.  Within a step the loads are not predicated per
  // lane, only the LDS write and the M store are: a unit past the tile's end reads row 0 of its
  // column, a column at or past d the row's last in-range vector.
  static_assert(LT % 256 == 0, "a lane's units of a tile share one column");
  const int64_t last_vec = d > 0 ? ((d - 1) >> UC_LOG) << UC_LOG : 0;
  const int rows_step = LT >> upr_log;
  const int lcit = (tid & upr_mask) << UC_LOG;      // column inside the tile
  const int row0 = tid >> upr_log;

  auto load_tile = [&](int64_t tile, float* buf) {
    const int64_t c0 = tile << log_c;
    const int64_t t0 = tile_origin(p, c0);
    const int64_t col = min(c0 + lcit, last_vec);
    const bool col_live = c0 + lcit < d;
    const int64_t x_row0 = col + t0;
    int64_t xo = static_cast<int64_t>(row0) * ld + x_row0;
    const int64_t xs = static_cast<int64_t>(rows_step) * ld;
    [[maybe_unused]] int64_t g_row0 = 0, go = 0, gs = 0, m_row0 = 0, mo = 0, ms = 0;
    if constexpr (STAGE_G) { g_row0 = g_offset(p, 0, col); go = g_offset(p, row0, col); gs = static_cast<int64_t>(rows_step) * p.g_ld; }
    if constexpr (STAGE_M) { m_row0 = m_offset(p, 0, col); mo = m_offset(p, row0, col); ms = static_cast<int64_t>(rows_step) * p.m_ld; }
    int row = row0;                                  // this lane's row in the step about to be requested
    for (int base = 0; base < nunits; base += LT * U) {
      raw_t xr[U];
      raw_t gr[STAGE_G ? U : 1];
      raw_t g2r[STAGE_G2 ? U : 1];
      f32x4 mr[STAGE_M ? U : 1];
      // a small tile ends before the U-th unit of a lane: those steps are skipped as a whole
      const int steps = (nunits - base + LT - 1) / LT;
      const int row_b = row;
      [[maybe_unused]] const int64_t mo_b = mo;
#pragma unroll
      for (int k = 0; k < U; ++k) {
        if (k >= steps) break;
        const bool in = row < p.n;
        xr[k] = ld_stream<STREAM>(reinterpret_cast<const raw_t*>(p.x_in + (in ? xo : x_row0) * EB));
        xo += xs;
        if constexpr (STAGE_G) {
          gr[k] = ld_stream<STREAM>(reinterpret_cast<const raw_t*>(p.g + (in ? go : g_row0) * EB));
          if constexpr (STAGE_G2) g2r[k] = ld_stream<STREAM>(reinterpret_cast<const raw_t*>(p.g2 + (in ? go : g_row0) * EB));
          go += gs;
        }
        if constexpr (STAGE_M) {
          mr[k] = ld_stream<STREAM>(reinterpret_cast<const f32x4*>(p.m + (in ? mo : m_row0)));
          mo += ms;
        }
        row += rows_step;
      }
#pragma unroll
      for (int k = 0; k < U; ++k) {
        if (k >= steps) break;
        const int rk = row_b + k * rows_step;
        const bool live = rk < p.n && col_live;
        float xv[UC];
        [[maybe_unused]] float gv[UC];
        widen_unit<DT, UC>(xr[k], xv);
        if constexpr (STAGE_G) {
          widen_unit<DT, UC>(gr[k], gv);
          if constexpr (STAGE_M) {
            float sv[4] = {mr[k].x, mr[k].y, mr[k].z, mr[k].w};
            local_update4<OP>(xv, gv, sv, p.alpha, p.beta);
            if (live) {
              float* mp = p.m + (mo_b + k * ms);
              const int64_t rem = d - col;
              if (rem >= 4) { f32x4 t = {sv[0], sv[1], sv[2], sv[3]}; st_stream<STREAM>(reinterpret_cast<f32x4*>(mp), t); }
              else for (int e = 0; e < 4; ++e) if (e < rem) mp[e] = sv[e];
            }
          } else if constexpr (STAGE_G2) {
            // gradient tracking: the mixed value is y + g_new - g_old
            float hv[UC];
            widen_unit<DT, UC>(g2r[k], hv);
#pragma unroll
            for (int e = 0; e < UC; ++e) xv[e] = (xv[e] + gv[e]) - hv[e];
          } else if constexpr (!G_LDS) {
#pragma unroll
            for (int e = 0; e < UC; ++e) xv[e] = fmaf(-p.alpha, gv[e], xv[e]);
          }
        }
        if (live) {
          float* dst = buf + (rk << log_c) + lcit;
#pragma unroll
          for (int q = 0; q < UC / 4; ++q) {
            f32x4 t = {xv[4 * q], xv[4 * q + 1], xv[4 * q + 2], xv[4 * q + 3]};
            *reinterpret_cast<f32x4*>(dst + 4 * q) = t;
          }
          if constexpr (G_LDS) {
            float* gdst = dst + (p.n << log_c);
#pragma unroll
            for (int q = 0; q < UC / 4; ++q) {
              f32x4 t = {gv[4 * q], gv[4 * q + 1], gv[4 * q + 2], gv[4 * q + 3]};
              *reinterpret_cast<f32x4*>(gdst + 4 * q) = t;
            }
          }
        }
      }
    }
  };

  constexpr int SPAN_LOG = (LW == 4 ? 8 : (LW == 2 ? 7 : 6));      // log2(64*LW)
  const int spans_log = log_c - SPAN_LOG;
  const int nops = p.n << spans_log;
  const int tile_floats = (G_LDS ? 2 * p.n : p.n) << log_c;

  const csr_i32_ptr rowptr = (csr_i32_ptr)(uintptr_t)p.rowptr;
  const csr_ent_ptr ent = (csr_ent_ptr)(uintptr_t)p.ent;

  // Reducer wave w takes the ops w, w + NR, w + 2 NR, ... of a tile, op = row * spans + span.  NR is a
  // multiple of the number of spans per row (1, 2 or 4), so a wave stays in one span: the columns of
  // its lanes are fixed, and what depends on them -- the LDS address, the global column offset, the
  // tail predicate -- is worked out once per tile, not once per op.
  static_assert(NR % 4 == 0, "a reducer wave keeps its span");
  const int cit = (((wave - NL) & ((1 << spans_log) - 1)) << SPAN_LOG) + lane * LW;    // column inside the tile
  // Adapt-while-communicate: the receiver's own gradient (and momentum) values, which the reducers
  // read from HBM themselves.  A wave's memory operations complete in issue order, so waiting for a
  // value just requested also waits for every store before it.  The values are therefore requested
  // AHEAD ops ahead, across tile boundaries, into AHEAD register sets used in turn (the op loop is
  // unrolled AHEAD times so that every set has a fixed name; every wave is given a multiple of AHEAD
  // ops per tile, those past the tile's end being empty): a store then has that many ops' time to
  // complete before anything waits behind it.  Like the loaders' reads, a request is not predicated:
  // a column at or past d re-reads the row's last vector.  For the compiler to know how many
  // operations were issued after the request it waits for, that number must be the same on every
  // path into the op loop: in tiles without a ragged tail nothing in the loop is conditional, and
  // the two other ways in (the start of the kernel, a tile with a ragged tail) drain the queue first.
  constexpr bool AWC = (OP == OP_AWC || OP == OP_MOM_AWC);
  constexpr int AHEAD = 4;
  const int nops_even = (nops + AHEAD * NR - 1) / (AHEAD * NR) * (AHEAD * NR);
  const int64_t last_own = d > 0 ? (d - 1) / LW * LW : 0;
  [[maybe_unused]] float gq[AHEAD][LW], mq[AHEAD][LW];
  auto fetch_own = [&](int64_t tile, int op, float* gv, float* mv) {
    // (an empty op still issues its request, so that the number of requests in flight at each wait is
    // the same on every path and known to the compiler; all its lanes read one and the same vector)
    const int i = min(op, nops - 1) >> spans_log;
    const int64_t col = min((tile << log_c) + (op >= nops ? cit - lane * LW : cit), last_own);
    load_in<DT, LW>(p.g, g_offset(p, i, col), gv);
    if constexpr (OP == OP_MOM_AWC) load_in<DT_F32, LW>(reinterpret_cast<const char*>(p.m), m_offset(p, i, col), mv);
  };

  // Output rows of one tile: reducer wave w takes the (row, 64*LW-column span) pairs w, w+NR, ...
  // Each is the weighted sum over the row's in-neighbor list, read from the LDS tile in list order
  // with fp32 accumulation; the list comes through the scalar cache, and entries go in batches of
  // eight (then four, two, one) so that a wave waits once per batch of LDS reads.
  // `next_tile`: the tile this workgroup reduces after this one (this one again if it is the last).
  // FULL: the tile has no ragged tail, so no store is predicated.
  auto reduce_tile_as = [&](int64_t tile, int64_t next_tile, const float* buf, auto full_c) __attribute__((always_inline)) {
    constexpr bool FULL = decltype(full_c)::value;
    const int64_t c0 = tile << log_c;
    const int64_t t0 = tile_origin(p, c0);
    // this lane's columns in this tile
    const float* src = buf + cit;
    const int64_t col = c0 + cit;
    const bool live = FULL || col < d;
    const int valid = (FULL || d - col >= LW) ? LW : static_cast<int>(d - col);
    const int64_t out_col = col + t0;
    [[maybe_unused]] const int64_t m_col = OP == OP_MOM_AWC ? m_offset(p, 0, col) : 0;
    // one batch of K list entries of one row: K LDS vectors, then K x LW FMAs in list order
    auto batch = [&](const float* src, float* acc, int q, auto kc) {
      constexpr int K = decltype(kc)::value;
      u32x2 en[K];
#pragma unroll
      for (int u = 0; u < K; ++u) en[u] = ent[q + u];
      float v[K][LW];
#pragma unroll
      for (int u = 0; u < K; ++u) {
        const float* sp = src + (static_cast<int>(en[u].x) << log_c);
        if constexpr (LW == 4) {
          const f32x4 t = *reinterpret_cast<const f32x4*>(sp);
          v[u][0] = t.x; v[u][1] = t.y; v[u][2] = t.z; v[u][3] = t.w;
        } else if constexpr (LW == 2) {
          const f32x2 t = *reinterpret_cast<const f32x2*>(sp);
          v[u][0] = t.x; v[u][1] = t.y;
        } else {
          v[u][0] = sp[0];
        }
      }
#pragma unroll
      for (int u = 0; u < K; ++u) {
        const float w = __uint_as_float(en[u].y);
#pragma unroll
        for (int e = 0; e < LW; ++e) acc[e] = fmaf(w, v[u][e], acc[e]);
      }
    };
    auto rest = [&](const float* src, float* acc, int q, int end) {
      for (; q + 8 <= end; q += 8) batch(src, acc, q, std::integral_constant<int, 8>{});
      if (q + 4 <= end) { batch(src, acc, q, std::integral_constant<int, 4>{}); q += 4; }
      if (q + 2 <= end) { batch(src, acc, q, std::integral_constant<int, 2>{}); q += 2; }
      if (q < end) batch(src, acc, q, std::integral_constant<int, 1>{});
    };
    // One output vector: the weighted sum, minus the own gradient step (AWC); mn is the new momentum.
    auto reduce_one = [&](int op, const float* gv, const float* mv, float* acc, float* mn) {
      const int i = op >> spans_log;
#pragma unroll
      for (int e = 0; e < LW; ++e) acc[e] = 0.0f;
      [[maybe_unused]] float own[LW];
      if constexpr (G_LDS) {
        const float* gp = src + ((p.n + i) << log_c);
#pragma unroll
        for (int e = 0; e < LW; ++e) own[e] = gp[e];
      }
      rest(src, acc, rowptr[i], rowptr[i + 1]);
      if constexpr (G_LDS) {
#pragma unroll
        for (int e = 0; e < LW; ++e) acc[e] = fmaf(-p.alpha, own[e], acc[e]);
      }
      if constexpr (AWC) {
#pragma unroll
        for (int e = 0; e < LW; ++e) {
          mn[e] = OP == OP_MOM_AWC ? fmaf(p.beta, mv[e], gv[e]) : gv[e];
          acc[e] = fmaf(-p.alpha, mn[e], acc[e]);
        }
      }
    };
    auto store_one = [&](int op, const float* acc, const float* mn) {
      const int i = op >> spans_log;
      if (live) {
        const int64_t off = static_cast<int64_t>(i) * ld + out_col;
        if constexpr (OP == OP_MOM_AWC) store_out<DT_F32, LW, false>(reinterpret_cast<char*>(p.m), static_cast<int64_t>(i) * p.m_ld + m_col, mn, valid);
        store_out<DT, LW, STREAM>(p.x_out, off, acc, valid);
        if constexpr (WITH_Y) {
          const float rcp = 1.0f / p.p_out[i];
          float yv[LW];
#pragma unroll
          for (int e = 0; e < LW; ++e) yv[e] = acc[e] * rcp;
          store_out<DT, LW, STREAM>(p.y, off, yv, valid);
        }
      }
    };
    if constexpr (AWC) {
      float acc[LW], mn[LW];
      for (int op = wave - NL; op < nops_even; op += AHEAD * NR) {
#pragma unroll
        for (int j = 0; j < AHEAD; ++j) {
          const int oj = op + j * NR;
          if (oj < nops) reduce_one(oj, gq[j], mq[j], acc, mn);
          const int nx = oj + AHEAD * NR;              // the op that uses this register set next
          const bool here = nx < nops_even;
          fetch_own(here ? tile : next_tile, here ? nx : nx - nops_even, gq[j], mq[j]);
          if (oj < nops) store_one(oj, acc, mn);
        }
      }
      if constexpr (!FULL) __builtin_amdgcn_s_waitcnt(0x0F70);      // vmcnt(0): see above
    } else {
      for (int op = wave - NL; op < nops; op += NR) {
        float acc[LW];
        reduce_one(op, nullptr, nullptr, acc, nullptr);
        store_one(op, acc, nullptr);
      }
    }
  };

  auto reduce_tile = [&](int64_t tile, int64_t next_tile, const float* buf) __attribute__((always_inline)) {
    if (((tile + 1) << log_c) <= d) reduce_tile_as(tile, next_tile, buf, std::true_type{});
    else reduce_tile_as(tile, next_tile, buf, std::false_type{});
  };

  // Odd rounds walk the tiles backwards: the columns a round wrote last are the first ones the
  // next round reads, so whatever the memory-side cache still holds of them is reused.
  auto phys = [&](int64_t seq) { return p.reverse ? p.ntiles - 1 - seq : seq; };
  // Each role runs a loop of its own (both meet at the same barriers, one per tile): in one loop
  // shared by both, the compiler sees the loaders' outstanding loads at the loop head and makes
  // every wave wait there for all its memory operations, which for a reducer means waiting for
  // the write acknowledgements of the tile it has just stored.
  int64_t seq = blockIdx.x;
  if (seq >= p.ntiles) return;
  int cur = 0;
  if (wave < NL) {
    load_tile(phys(seq), lds);
    lds_barrier();
    for (; seq < p.ntiles; seq += gridDim.x, cur ^= 1) {
      const int64_t next = seq + gridDim.x;
      if (next < p.ntiles) load_tile(phys(next), lds + (cur ^ 1) * tile_floats);
      lds_barrier();
    }
  } else {
    if constexpr (AWC) {
#pragma unroll
      for (int j = 0; j < AHEAD; ++j) fetch_own(phys(seq), wave - NL + j * NR, gq[j], mq[j]);
      __builtin_amdgcn_s_waitcnt(0x0F70);                           // vmcnt(0)
    }
    lds_barrier();
    for (; seq < p.ntiles; seq += gridDim.x, cur ^= 1) {
      const int64_t next = seq + gridDim.x;
      reduce_tile(phys(seq), phys(next < p.ntiles ? next : seq), lds + cur * tile_floats);
      lds_barrier();
    }
  }
}

template <int DT, int OP, bool WITH_Y, int LW, int NL, int NR, int U, bool STREAM>
int launch_pipe_shape(const TileParams& tp, int grid, size_t lds, hipStream_t st) {
  auto kern = bf_pipe_kernel<DT, OP, WITH_Y, LW, NL, NR, U, STREAM>;
  if (lds > 48 * 1024) {
    static thread_local size_t raised = 0;
    if (raised < lds) {
      BF_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                     static_cast<int>(lds)));
      raised = lds;
    }
  }
  hipLaunchKernelGGL(kern, dim3(grid), dim3((NL + NR) * 64), lds, st, tp);
  BF_HIP_TRY(hipGetLastError());
  return BF_OK;
}

// The wave split.  Plain mixing and the ops that stage X (and G) only: four loader waves with eight
// (narrow tiles: four) vectors per lane in flight and twelve reducer waves, the measured best of the splits tried (4+8
// and 8+8 waves leave the reducers short; two or three loader waves cannot keep enough loads in
// flight).  The ops that also read and write an fp32 state matrix while staging (momentum,
// Exact-Diffusion) do most of their work in the loaders: eight loader waves with four vectors in
// flight and eight reducers measure 2-3 % above the 4+12 split there on column blocks (n = 32 bf16
// momentum: 6.25 against 6.08 TB/s; with eight vectors in flight 5.75) and within 1 % of it on
// agent-major rows.
template <int DT, int OP, bool WITH_Y, int LW>
int launch_pipe_lw(const TileParams& tp, int grid, size_t lds, bool stream, hipStream_t st) {
  if constexpr (OP == OP_MOM_ATC || OP == OP_ED) {
    // (vectors in flight per loader lane: four with bf16 storage, two with fp32, where a unit of X and G
    // is twice the bytes: fp32 momentum 6.09-6.21 -> 6.19-6.30 TB/s at n = 32, 64, 128)
    constexpr int UU = DT == DT_F32 ? 2 : 4;
    return stream ? launch_pipe_shape<DT, OP, WITH_Y, LW, 8, 8, UU, true>(tp, grid, lds, st)
                  : launch_pipe_shape<DT, OP, WITH_Y, LW, 8, 8, UU, false>(tp, grid, lds, st);
  } else {
    // (tiles narrower than 256 columns -- more than 80 agents -- do better with four vectors in flight
    // than with eight: config 4 in place on column blocks 6.18 -> 6.35 TB/s, n = 160 5.89 -> 6.20;
    // at 256 columns and more eight stay ahead by a percent)
    constexpr int UU = LW == 4 ? 8 : 4;
    return stream ? launch_pipe_shape<DT, OP, WITH_Y, LW, 4, 12, UU, true>(tp, grid, lds, st)
                  : launch_pipe_shape<DT, OP, WITH_Y, LW, 4, 12, UU, false>(tp, grid, lds, st);
  }
}

template <int DT, int OP, bool WITH_Y>
int launch_pipe(const TileParams& tp, const Shape& s, int grid, hipStream_t st) {
  switch (s.lw) {
    case 4: return launch_pipe_lw<DT, OP, WITH_Y, 4>(tp, grid, s.lds_bytes, s.stream, st);
    case 2: return launch_pipe_lw<DT, OP, WITH_Y, 2>(tp, grid, s.lds_bytes, s.stream, st);
    default: return launch_pipe_lw<DT, OP, WITH_Y, 1>(tp, grid, s.lds_bytes, s.stream, st);
  }
}

template <int DT>
int launch_pipe_op(int op, bool with_y, const TileParams& tp, const Shape& s, int grid, hipStream_t st) {
  switch (op) {
    case OP_MIX: return with_y ? launch_pipe<DT, OP_MIX, true>(tp, s, grid, st) : launch_pipe<DT, OP_MIX, false>(tp, s, grid, st);
    case OP_ATC: return with_y ? launch_pipe<DT, OP_ATC, true>(tp, s, grid, st) : launch_pipe<DT, OP_ATC, false>(tp, s, grid, st);
    case OP_TRACK: return launch_pipe<DT, OP_TRACK, false>(tp, s, grid, st);
    case OP_AWC: return launch_pipe<DT, OP_AWC, false>(tp, s, grid, st);
    case OP_AWC_LDS:
      if constexpr (DT == DT_BF16) return launch_pipe<DT, OP_AWC_LDS, false>(tp, s, grid, st);
      else return BF_ERR_UNSUPPORTED;                  // (the dispatcher takes this form with bf16 storage only)
    case OP_MOM_ATC: return launch_pipe<DT, OP_MOM_ATC, false>(tp, s, grid, st);
    case OP_ED: return launch_pipe<DT, OP_ED, false>(tp, s, grid, st);
    default: return launch_pipe<DT, OP_MOM_AWC, false>(tp, s, grid, st);
  }
}

}  // namespace bf

#endif  // BF_PIPE_INC_H_
