// The column-owned LDS tile kernel and its launchers (template code; included by bf_tile_f32.hip
// and bf_tile_bf16.hip, which instantiate it for one storage type each).
#ifndef BF_TILE_INC_H_
#define BF_TILE_INC_H_

#include "bf_device.h"

namespace bf {

// ---------------------------------------------------------------------------------------------
// The tile kernel.  DT: storage type of X/G/Y.  OP: what is staged and what is subtracted.
// WITH_Y: also write the push-sum ratio.  LW: columns per lane in the reduce phase (a wave spans
// 64*LW columns of one output row).  MAXPF: staging units (16-byte vectors of X) per thread.
template <int DT, int OP, bool WITH_Y, int LW, int THREADS, int MAXPF, bool STREAM, bool MULTI = false>
__global__ __launch_bounds__(THREADS) void bf_tile_kernel(const TileParams p) {
  extern __shared__ f32x4 lds_raw[];
  float* lds = reinterpret_cast<float*>(lds_raw);

  constexpr int EB = Elem<DT>::bytes;
  constexpr int UC = Elem<DT>::per16;               // columns per staging unit
  constexpr int UC_LOG = DT == DT_F32 ? 2 : 3;
  constexpr bool STAGE_G = (OP == OP_ATC || OP == OP_MOM_ATC || OP == OP_ED || OP == OP_TRACK);
  constexpr bool STAGE_G2 = (OP == OP_TRACK);
  constexpr bool STAGE_M = (OP == OP_MOM_ATC || OP == OP_ED);
  constexpr int MV = UC / 4;                        // 16-byte vectors of M per unit

  const int tid = threadIdx.x;
  const int log_c = p.log_c;
  const int upr_log = log_c - UC_LOG;               // staging units per tile row (log2)
  const int upr_mask = (1 << upr_log) - 1;
  const int nunits = p.n << upr_log;
  const int64_t d = p.d, ld = p.ld;

  u32x4 xr[MAXPF];
  u32x4 gr[STAGE_G ? MAXPF : 1];
  u32x4 g2r[STAGE_G2 ? MAXPF : 1];
  f32x4 mr[STAGE_M ? MAXPF * MV : 1];

  // Loads are unconditional (uniform control flow keeps all of a tile's loads in flight at
  // once): a unit past the tile's end re-reads the last unit, a column at or past d re-reads the
  // row's last in-range vector.  Only the LDS write and the M store are predicated.
  const int64_t last_vec = d > 0 ? ((d - 1) >> UC_LOG) << UC_LOG : 0;
  auto issue_one = [&](int64_t tile, int k) {
    const int64_t c0 = tile << log_c;
    {
      const int u = min(tid + k * THREADS, nunits - 1);
      const int row = u >> upr_log;
      const int64_t col = min(c0 + (static_cast<int64_t>(u & upr_mask) << UC_LOG), last_vec);
      const int64_t off = static_cast<int64_t>(row) * ld + col + tile_origin(p, c0);
      xr[k] = ld_stream<STREAM>(reinterpret_cast<const u32x4*>(p.x_in + off * EB));
      if constexpr (STAGE_G) gr[k] = ld_stream<STREAM>(reinterpret_cast<const u32x4*>(p.g + g_offset(p, row, col) * EB));
      if constexpr (STAGE_G2) g2r[k] = ld_stream<STREAM>(reinterpret_cast<const u32x4*>(p.g2 + g_offset(p, row, col) * EB));
      if constexpr (STAGE_M) {
#pragma unroll
        for (int q = 0; q < MV; ++q) mr[k * MV + q] = *reinterpret_cast<const f32x4*>(p.m + m_offset(p, row, col) + 4 * q);
      }
    }
  };
  auto issue_loads = [&](int64_t tile) {
#pragma unroll
    for (int k = 0; k < MAXPF; ++k) issue_one(tile, k);
  };

  // Transform one staging unit (local update, momentum) and put it into the LDS tile.
  auto stage_unit = [&](int u, int64_t c0, const u32x4& xraw, const u32x4& graw, const u32x4& g2raw, const f32x4* mraw) {
    const int row = u >> upr_log;
    const int cit = (u & upr_mask) << UC_LOG;       // column inside the tile
    const int64_t col = c0 + cit;
    const bool live = u < nunits && col < d;
    float xv[UC];
    widen<DT>(xraw, xv);
    if constexpr (STAGE_G) {
      float gv[UC];
      widen<DT>(graw, gv);
      if constexpr (STAGE_M) {
        const int64_t off = m_offset(p, row, col);
#pragma unroll
        for (int q = 0; q < MV; ++q) {
          float sv[4] = {mraw[q].x, mraw[q].y, mraw[q].z, mraw[q].w};
          local_update4<OP>(xv + 4 * q, gv + 4 * q, sv, p.alpha, p.beta);
          if (live) {
            const int64_t rem = d - (col + 4 * q);
            if (rem >= 4) { f32x4 t = {sv[0], sv[1], sv[2], sv[3]}; *reinterpret_cast<f32x4*>(p.m + off + 4 * q) = t; }
            else for (int e = 0; e < 4; ++e) if (e < rem) p.m[off + 4 * q + e] = sv[e];
          }
        }
      } else if constexpr (STAGE_G2) {
        // gradient tracking: the mixed value is y + g_new - g_old
        float hv[UC];
        widen<DT>(g2raw, hv);
#pragma unroll
        for (int e = 0; e < UC; ++e) xv[e] = (xv[e] + gv[e]) - hv[e];
      } else {
#pragma unroll
        for (int e = 0; e < UC; ++e) xv[e] = fmaf(-p.alpha, gv[e], xv[e]);
      }
    }
    if (live) {
      float* dst = lds + (row << log_c) + cit;
#pragma unroll
      for (int q = 0; q < MV; ++q) {
        f32x4 t = {xv[4 * q], xv[4 * q + 1], xv[4 * q + 2], xv[4 * q + 3]};
        *reinterpret_cast<f32x4*>(dst + 4 * q) = t;
      }
    }
  };

  auto stage = [&](int64_t tile) {
    const int64_t c0 = tile << log_c;
#pragma unroll
    for (int k = 0; k < MAXPF; ++k)
      stage_unit(tid + k * THREADS, c0, xr[k], gr[STAGE_G ? k : 0], g2r[STAGE_G2 ? k : 0], &mr[STAGE_M ? k * MV : 0]);
    // Tiles taller than THREADS*MAXPF units (many agents): the rest is loaded here, unprefetched.
    for (int u = tid + MAXPF * THREADS; u < nunits; u += THREADS) {
      const int row = u >> upr_log;
      const int64_t col = min(c0 + (static_cast<int64_t>(u & upr_mask) << UC_LOG), last_vec);
      const int64_t off = static_cast<int64_t>(row) * ld + col + tile_origin(p, c0);
      const u32x4 xraw = ld_stream<STREAM>(reinterpret_cast<const u32x4*>(p.x_in + off * EB));
      u32x4 graw = {0, 0, 0, 0}, g2raw = {0, 0, 0, 0};
      f32x4 mraw[MV];
      if constexpr (STAGE_G) graw = ld_stream<STREAM>(reinterpret_cast<const u32x4*>(p.g + g_offset(p, row, col) * EB));
      if constexpr (STAGE_G2) g2raw = ld_stream<STREAM>(reinterpret_cast<const u32x4*>(p.g2 + g_offset(p, row, col) * EB));
      if constexpr (STAGE_M) {
#pragma unroll
        for (int q = 0; q < MV; ++q) mraw[q] = *reinterpret_cast<const f32x4*>(p.m + m_offset(p, row, col) + 4 * q);
      }
      stage_unit(u, c0, xraw, graw, g2raw, mraw);
    }
  };

  const csr_i32_ptr rowptr = (csr_i32_ptr)(uintptr_t)p.rowptr;
  const csr_ent_ptr ent = (csr_ent_ptr)(uintptr_t)p.ent;

  constexpr int NW = THREADS / 64;
  constexpr int SPAN_LOG = (LW == 4 ? 8 : (LW == 2 ? 7 : 6));      // log2(64*LW)
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lane = tid & 63;
  const int spans_log = log_c - SPAN_LOG;
  const int nops = p.n << spans_log;
  // Weighted sum of one output row-span over the row's in-neighbor list, read from an LDS tile.
  auto gather = [&](const float* tile_base, csr_i32_ptr rp, csr_ent_ptr en_list, int i, int cit, float* acc) {
    const int beg = rp[i], end = rp[i + 1];
#pragma unroll
    for (int e = 0; e < LW; ++e) acc[e] = 0.0f;
    const float* src = tile_base + cit;
    // Entries go in batches of K (4, then 2, then 1): the K list entries and the K LDS reads of a
    // batch are issued together and only then consumed, in list order, so a wave waits once per
    // batch instead of once per entry.
    auto batch = [&](int q, auto kc) {
      constexpr int K = decltype(kc)::value;
      u32x2 en[K];
#pragma unroll
      for (int u = 0; u < K; ++u) en[u] = en_list[q + u];
      float v[K][LW];
#pragma unroll
      for (int u = 0; u < K; ++u) {
        const float* s = src + (static_cast<int>(en[u].x) << log_c);
        if constexpr (LW == 4) {
          const f32x4 t = *reinterpret_cast<const f32x4*>(s);
          v[u][0] = t.x; v[u][1] = t.y; v[u][2] = t.z; v[u][3] = t.w;
        } else if constexpr (LW == 2) {
          const f32x2 t = *reinterpret_cast<const f32x2*>(s);
          v[u][0] = t.x; v[u][1] = t.y;
        } else {
          v[u][0] = s[0];
        }
      }
#pragma unroll
      for (int u = 0; u < K; ++u) {
        const float w = __uint_as_float(en[u].y);
#pragma unroll
        for (int e = 0; e < LW; ++e) acc[e] = fmaf(w, v[u][e], acc[e]);
      }
    };
    // The fp32 kernels with four columns per lane and no gradient operand fit two 1024-thread
    // workgroups per CU only while they stay within 64 registers, which the batch of four would
    // cost them (unless they prefetch only half the tile, MAXPF == 2, the form used for long rows);
    // every other kernel is either well below or already above that line.
    constexpr bool BATCHED =
        !(DT == DT_F32 && LW == 4 && (OP == OP_MIX || OP == OP_AWC || OP == OP_MOM_AWC) && !MULTI && MAXPF == 4);
    int q = beg;
    if constexpr (BATCHED) {
      for (; q + 4 <= end; q += 4) batch(q, std::integral_constant<int, 4>{});
      if (q + 2 <= end) { batch(q, std::integral_constant<int, 2>{}); q += 2; }
    }
    for (; q < end; ++q) batch(q, std::integral_constant<int, 1>{});
  };
  const float* final_src = lds;     // the LDS tile the last round reads (moves when rounds are fused)
  // One output row-span: gather from LDS in CSR order, finish, store.
  auto row_op = [&](int64_t tile, int op) {
    const int64_t c0 = tile << log_c;
    {
      const int i = op >> spans_log;
      const int cit = ((op & ((1 << spans_log) - 1)) << SPAN_LOG) + lane * LW;
      const int64_t col = c0 + cit;
      float acc[LW];
      gather(final_src, rowptr, ent, i, cit, acc);
      if (col < d) {
        const int64_t rem = d - col;
        const int valid = rem >= LW ? LW : static_cast<int>(rem);
        const int64_t off = static_cast<int64_t>(i) * ld + col + tile_origin(p, c0);
        if constexpr (OP == OP_AWC || OP == OP_MOM_AWC) {
          // Adapt-while-communicate: the receiver's own gradient is subtracted after the mix.
          float gv[LW];
          load_in<DT, LW>(p.g, g_offset(p, i, col), gv);
          if constexpr (OP == OP_MOM_AWC) {
            float mv[LW];
            load_in<DT_F32, LW>(reinterpret_cast<const char*>(p.m), m_offset(p, i, col), mv);
#pragma unroll
            for (int e = 0; e < LW; ++e) gv[e] = fmaf(p.beta, mv[e], gv[e]);
            store_out<DT_F32, LW, false>(reinterpret_cast<char*>(p.m), m_offset(p, i, col), gv, valid);
          }
#pragma unroll
          for (int e = 0; e < LW; ++e) acc[e] = fmaf(-p.alpha, gv[e], acc[e]);
        }
        store_out<DT, LW, STREAM>(p.x_out, off, acc, valid);
        if constexpr (WITH_Y) {
          const float rcp = 1.0f / p.p_out[i];
          float yv[LW];
#pragma unroll
          for (int e = 0; e < LW; ++e) yv[e] = acc[e] * rcp;
          store_out<DT, LW, STREAM>(p.y, off, yv, valid);
        }
      }
    }
  };
  // Reduce phase of `tile`; the loads of tile `next` (if any) are issued one by one between the
  // first row-spans so that reads and writes alternate on the memory pipe.
  auto reduce_and_store = [&](int64_t tile, int64_t next, bool has_next) {
    int op = wave;
#pragma unroll
    for (int k = 0; k < MAXPF; ++k) {
      if (has_next) issue_one(next, k);
      if (op < nops) { row_op(tile, op); op += NW; }
    }
    for (; op < nops; op += NW) row_op(tile, op);
  };

  // Odd rounds walk the tiles backwards: the columns a round wrote last are the first ones the
  // next round reads, so whatever the memory-side cache still holds of them is reused.
  auto phys = [&](int64_t seq) { return p.reverse ? p.ntiles - 1 - seq : seq; };
  int64_t seq = blockIdx.x;
  if (seq < p.ntiles) issue_loads(phys(seq));
  while (seq < p.ntiles) {
    const int64_t tile = phys(seq);
    stage(tile);
    lds_barrier();
    if constexpr (MULTI) {
      // Only one such workgroup fits a CU (two tiles), so nothing else keeps the memory pipe busy
      // during the LDS rounds: the next tile's loads go out now, not during the last round.
      if (seq + gridDim.x < p.ntiles) issue_loads(phys(seq + gridDim.x));
      // Fused rounds: apply the first fuse-1 weight matrices LDS tile to LDS tile (two tiles, used
      // alternately); the last one goes through the normal reduce-and-store below.
      float* tile_a = lds;
      float* tile_b = lds + (p.n << log_c);
      typedef const u32x4 __attribute__((address_space(4)))* csr_u4_ptr;
      typedef const u32x8 __attribute__((address_space(4)))* csr_u8_ptr;
      const csr_u4_ptr round_tab = (csr_u4_ptr)(uintptr_t)p.blob;
      const int rows_b = p.rows_b > 0 ? p.rows_b : p.n;
      int k = p.round_k0;
      for (int r = 0; r + 1 < p.fuse; ++r) {
        const float* src_t = (r & 1) ? tile_b : tile_a;
        float* dst_t = (r & 1) ? tile_a : tile_b;
        const int row_limit = (r & 1) ? p.n : rows_b;          // rows the destination tile has
        const int ngroups = (row_limit + 3) >> 2;
        const int nitems = ngroups << spans_log;
        const u32x4 offs = round_tab[k];
        const csr_u4_ptr hdrs = (csr_u4_ptr)(reinterpret_cast<uintptr_t>(p.blob) + offs.z);
        const uintptr_t recs = reinterpret_cast<uintptr_t>(p.blob) + offs.w;
        k = k + 1 == p.nrounds ? 0 : k + 1;
        // NG groups of four rows per wave at a time, from the sliced copy of the round: one 32-byte
        // scalar load brings the q-th entry of a group's four rows, the LDS reads of all groups go
        // out together, and each row still adds its entries in list order, as the one-round path
        // does.  (One group at a time leaves the wave waiting on each lookup: 16 waves per CU are
        // all there is to hide it, because the two tiles fill the LDS.)
        constexpr int NG = 1;
        for (int item0 = wave; item0 < nitems; item0 += NW * NG) {
          int g[NG], cit[NG];
          u32x4 hdr[NG];
          uint32_t longest = 0;
          bool ragged = false;
#pragma unroll
          for (int j = 0; j < NG; ++j) {
            const int item = item0 + j * NW;
            const int itc = item < nitems ? item : item0;
            g[j] = itc >> spans_log;
            cit[j] = ((itc & ((1 << spans_log) - 1)) << SPAN_LOG) + lane * LW;
            hdr[j] = hdrs[g[j]];
            if (item >= nitems) hdr[j].y = 0;
          }
#pragma unroll
          for (int j = 0; j < NG; ++j) {
            longest = max(longest, hdr[j].y);
            ragged = ragged || hdr[j].z != 0 || hdr[j].y != hdr[0].y;
          }
          float acc[NG][4][LW];
#pragma unroll
          for (int j = 0; j < NG; ++j)
#pragma unroll
            for (int u = 0; u < 4; ++u)
#pragma unroll
              for (int e = 0; e < LW; ++e) acc[j][u][e] = 0.0f;
          auto records = [&](auto ragged_c) {
            constexpr bool RAGGED = decltype(ragged_c)::value;
            for (uint32_t q = 0; q < longest; ++q) {
              u32x8 e8[NG];
#pragma unroll
              for (int j = 0; j < NG; ++j) {
                // a group that has run out re-reads its last record (or record 0 of the table when
                // it has none); every entry of such a read is skipped below
                const uint32_t qc = RAGGED ? (q < hdr[j].y ? q : (hdr[j].y ? hdr[j].y - 1 : 0)) : q;
                const uint32_t first = RAGGED && hdr[j].y == 0 ? 0 : hdr[j].x;
                e8[j] = ((csr_u8_ptr)(recs + (static_cast<uintptr_t>(first + qc) << 5)))[0];
              }
              float v[NG][4][LW];
#pragma unroll
              for (int j = 0; j < NG; ++j) {
                const uint32_t col[4] = {e8[j].s0, e8[j].s2, e8[j].s4, e8[j].s6};
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                  const float* sp = src_t + cit[j] + (static_cast<int>(RAGGED ? (col[u] & 0x7fffffffu) : col[u]) << log_c);
                  if constexpr (LW == 4) {
                    const f32x4 t = *reinterpret_cast<const f32x4*>(sp);
                    v[j][u][0] = t.x; v[j][u][1] = t.y; v[j][u][2] = t.z; v[j][u][3] = t.w;
                  } else if constexpr (LW == 2) {
                    const f32x2 t = *reinterpret_cast<const f32x2*>(sp);
                    v[j][u][0] = t.x; v[j][u][1] = t.y;
                  } else {
                    v[j][u][0] = sp[0];
                  }
                }
              }
#pragma unroll
              for (int j = 0; j < NG; ++j) {
                const uint32_t col[4] = {e8[j].s0, e8[j].s2, e8[j].s4, e8[j].s6};
                const uint32_t wb[4] = {e8[j].s1, e8[j].s3, e8[j].s5, e8[j].s7};
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                  const float w = __uint_as_float(wb[u]);
                  const bool live = !RAGGED || (static_cast<int32_t>(col[u]) >= 0 && q < hdr[j].y);
#pragma unroll
                  for (int e = 0; e < LW; ++e) {
                    const float f = fmaf(w, v[j][u][e], acc[j][u][e]);
                    acc[j][u][e] = live ? f : acc[j][u][e];
                  }
                }
              }
            }
          };
          if (ragged) records(std::true_type{}); else records(std::false_type{});
#pragma unroll
          for (int j = 0; j < NG; ++j) {
            if (item0 + j * NW < nitems) {
#pragma unroll
              for (int u = 0; u < 4; ++u) {
                const int row = (g[j] << 2) + u;
                if (row < row_limit) {
                  float* o = dst_t + (row << log_c) + cit[j];
                  if constexpr (LW == 4) { f32x4 t = {acc[j][u][0], acc[j][u][1], acc[j][u][2], acc[j][u][3]}; *reinterpret_cast<f32x4*>(o) = t; }
                  else if constexpr (LW == 2) { f32x2 t = {acc[j][u][0], acc[j][u][1]}; *reinterpret_cast<f32x2*>(o) = t; }
                  else { o[0] = acc[j][u][0]; }
                }
              }
            }
          }
        }
        lds_barrier();
      }
      final_src = ((p.fuse - 1) & 1) ? tile_b : tile_a;
    }
    const int64_t next = seq + gridDim.x;
    reduce_and_store(tile, phys(next), !MULTI && next < p.ntiles);
    lds_barrier();
    seq = next;
  }
}

template <int DT, int OP, bool WITH_Y, int LW, int THREADS, bool STREAM, bool MULTI = false, bool LONG_ROWS = false>
int launch_tile_thr(const TileParams& tp, int grid, size_t lds, hipStream_t st) {
  // prefetch depth: a 64 KB tile is 4 (fp32) / 2 (bf16) vectors per thread at 1024 threads.  The
  // long-row form of the fp32 mix prefetches half the tile and spends the registers on batched LDS
  // reads instead (see the kernel's reduce phase).
  constexpr int MAXPF = DT == DT_F32 ? (LONG_ROWS ? 2 : 4) : 2;
  auto kern = bf_tile_kernel<DT, OP, WITH_Y, LW, THREADS, MAXPF, STREAM, MULTI>;
  if (lds > 48 * 1024) {
    static thread_local size_t raised = 0;
    if (raised < lds) {
      BF_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                     static_cast<int>(lds)));
      raised = lds;
    }
  }
  hipLaunchKernelGGL(kern, dim3(grid), dim3(THREADS), lds, st, tp);
  BF_HIP_TRY(hipGetLastError());
  return BF_OK;
}

// 1024 threads, two workgroups per CU: smaller workgroups (256, 512 threads, more per CU) were
// measured 5..25 % slower at every tile width.
template <int DT, int OP, bool WITH_Y, int LW>
int launch_tile_lw(const TileParams& tp, int grid, size_t lds, bool stream, hipStream_t st) {
  if constexpr (OP == OP_MIX && !WITH_Y) {
    // the several-rounds-per-pass form is a kernel of its own, so its extra registers cost the
    // one-round kernel nothing
    if (tp.fuse > 1)
      return stream ? launch_tile_thr<DT, OP, WITH_Y, LW, 1024, true, true>(tp, grid, lds, st)
                    : launch_tile_thr<DT, OP, WITH_Y, LW, 1024, false, true>(tp, grid, lds, st);
  }
  if constexpr (DT == DT_F32 && LW == 4 && (OP == OP_MIX || OP == OP_AWC)) {
    // Rows with many entries (the static exponential graph has 12): the reduce phase, one LDS read
    // at a time, is then as long as the tile's HBM transfers.  Batching the reads needs 12 more
    // registers, which a prefetch of half the tile pays for, so two workgroups still fit a CU:
    // config 2 in place 72 -> 75 % of peak; rows of 2 or 3 entries lose about 1 %, so they keep
    // the full prefetch.
    if (tp.long_rows)
      return stream ? launch_tile_thr<DT, OP, WITH_Y, LW, 1024, true, false, true>(tp, grid, lds, st)
                    : launch_tile_thr<DT, OP, WITH_Y, LW, 1024, false, false, true>(tp, grid, lds, st);
  }
  return stream ? launch_tile_thr<DT, OP, WITH_Y, LW, 1024, true>(tp, grid, lds, st)
                : launch_tile_thr<DT, OP, WITH_Y, LW, 1024, false>(tp, grid, lds, st);
}

template <int DT, int OP, bool WITH_Y>
int launch_tile(const TileParams& tp, const Shape& s, int grid, hipStream_t st) {
  switch (s.lw) {
    case 4: return launch_tile_lw<DT, OP, WITH_Y, 4>(tp, grid, s.lds_bytes, s.stream, st);
    case 2: return launch_tile_lw<DT, OP, WITH_Y, 2>(tp, grid, s.lds_bytes, s.stream, st);
    default: return launch_tile_lw<DT, OP, WITH_Y, 1>(tp, grid, s.lds_bytes, s.stream, st);
  }
}

template <int DT>
int launch_tile_op(int op, bool with_y, const TileParams& tp, const Shape& s, int grid, hipStream_t st) {
  switch (op) {
    case OP_MIX: return with_y ? launch_tile<DT, OP_MIX, true>(tp, s, grid, st) : launch_tile<DT, OP_MIX, false>(tp, s, grid, st);
    case OP_ATC: return with_y ? launch_tile<DT, OP_ATC, true>(tp, s, grid, st) : launch_tile<DT, OP_ATC, false>(tp, s, grid, st);
    case OP_TRACK: return launch_tile<DT, OP_TRACK, false>(tp, s, grid, st);
    case OP_AWC: return launch_tile<DT, OP_AWC, false>(tp, s, grid, st);
    case OP_MOM_ATC: return launch_tile<DT, OP_MOM_ATC, false>(tp, s, grid, st);
    case OP_ED: return launch_tile<DT, OP_ED, false>(tp, s, grid, st);
    default: return launch_tile<DT, OP_MOM_AWC, false>(tp, s, grid, st);
  }
}

}  // namespace bf

#endif  // BF_TILE_INC_H_
