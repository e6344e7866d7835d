// bf16 dk/dv kernel (see hstu_mfma.h for the common parts).
#include "hstu_mfma.h"

namespace hstu {

namespace {

// =============================================================================================
// dk/dv pass: owners are key rows (K and V rows in registers), Q and dO are streamed.
//   S  = Q K^T   (A = Q tile rows,  B = K registers)   lane: key n, query rows in registers
//   dP = dO V^T  (A = dO tile rows, B = V registers)
//   dV^T += dO^T P   (A = dO tile transposed read, B = P registers)   lane: key n, columns in registers
//   dK^T += Q^T dS   (A = Q tile transposed read,  B = dS registers)
// (The transposes of dV and dK are what is accumulated, so that a lane ends up with four
// consecutive elements of its key row per accumulator group and the epilogue writes 8 bytes per
// lane and instruction; with the operands the other way round it wrote single elements.)
// Each key tile belongs to exactly one workgroup, so dk and dv need no atomics.
// =============================================================================================

// The stream of query rows is processed in blocks of 32 rows, software-pipelined across blocks
// and across tiles.  Step i issues, interleaved,
//   the matrix instructions of the scores of block i+1       (S, dP: KS + VS instructions),
//   the matrix instructions of the contraction of block i-1  (dV, dK: VS + KS instructions),
//   the elementwise work that turns S(i), dP(i) into P(i), dS(i) (vector instructions),
// which are independent of each other, so the matrix pipe and the vector pipe are both busy for
// the whole step.  (With one wave per SIMD nothing else overlaps them: a tile-at-a-time order has
// the first and the last quarter of every tile without vector work and the middle half bound by
// it.)  Two accumulator sets for S/dP and two operand sets for P/dS alternate by block parity.
//
// Causal mask of a block the diagonal touches: query row r (accumulator element) of the block is
// visible to the lane's key iff rel <= 8*(r/4) + 4*hh + r%4, rel = key position - block position.
// It is applied to the finished elementwise results under a wave-uniform branch, so the matrix
// instructions and their accumulators follow one path whether or not a block is masked; a block
// no row of which is visible comes out as zeros and contributes nothing.
template <int DQK, int DV, bool CONTR, class Init, class Vis>
__device__ __forceinline__ void dkdv_step(const Init& init, const char* qn, const char* gn, int bn,
                                          const char* qp, const char* gp, int bp,
                                          const RowAddr<DQK>& raq, const RowAddr<DV>& rag,
                                          const ColAddr<DQK>& caq, const ColAddr<DV>& cag,
                                          const bf16x8 (&kreg)[DQK / 16],
                                          const bf16x8 (&vreg)[DV / 16],
                                          const f32x16& s_in, const f32x16& d_in,
                                          f32x16& s_out, f32x16& d_out,
                                          const bf16x8 (&pd_prev)[4], bf16x8 (&pd_cur)[4],
                                          f32x16 (&dkacc)[DQK / 32], f32x16 (&dvacc)[DV / 32],
                                          float c1, float alpha, bool mask, const Vis& vis_of) {
  constexpr int KS = DQK / 16, VS = DV / 16, NS = KS + VS;
  constexpr int AHEAD = NS < 4 ? NS : 4;  // operand reads in flight ahead of their use
  constexpr int GRP = 4;                  // slots between scheduling fences
  bf16x8 op[NS];  // row-wise operands of block i+1: Q rows, then dO rows
  bf16x8 tp[NS];  // transposed operands of block i-1: dO^T, then Q^T
  auto read_rows = [&](int m) { return m < KS ? raq.read(qn, bn, m) : rag.read(gn, bn, m - KS); };
  auto read_cols = [&](int m) {
    return m < VS ? cag.read(gp, bp * 2 + (m & 1), m >> 1)
                  : caq.read(qp, bp * 2 + ((m - VS) & 1), (m - VS) >> 1);
  };
  auto fence = [] { __builtin_amdgcn_sched_barrier(0); };
  init(s_out);
#pragma unroll
  for (int r = 0; r < 16; ++r) d_out[r] = 0.f;
#pragma unroll
  for (int m = 0; m < AHEAD; ++m) {
    op[m] = read_rows(m);
    if (CONTR) tp[m] = read_cols(m);
  }
  fence();
  float p[16], ds[16];
  // The elementwise work of a group of four slots is done in four stages over the group's
  // 64 / NS elements, one stage per slot, so that an instruction's operands were produced a few
  // instructions earlier and not by its predecessor (a lone wave pays every such dependence, most
  // of all behind exp and rcp, in stalled cycles and hazard nops).
  // (Only where a wave has the whole register file: the variants built for two workgroups per CU
  // are at their limit of 256, and the values in flight would spill.)
  constexpr bool STAGED = DQK + DV > 128 && (NS == 8 || NS == 16);
  constexpr int EPG = STAGED ? 64 / NS : 1;
  float st_t[EPG], st_g[EPG];
#pragma unroll
  for (int m = 0; m < NS; ++m) {
    if (m < KS) s_out = mfma(op[m], kreg[m], s_out);
    else d_out = mfma(op[m], vreg[m - KS], d_out);
    if (CONTR) {
      if (m < VS) dvacc[m >> 1] = mfma(tp[m], pd_prev[m & 1], dvacc[m >> 1]);
      else dkacc[(m - VS) >> 1] = mfma(tp[m], pd_prev[2 + ((m - VS) & 1)], dkacc[(m - VS) >> 1]);
    }
    if (m + AHEAD < NS) {
      op[m + AHEAD] = read_rows(m + AHEAD);
      if (CONTR) tp[m + AHEAD] = read_cols(m + AHEAD);
    }
    if constexpr (STAGED) {
      const int e0 = (m / 4) * EPG, ph = m % 4;
      if (ph == 0) {
#pragma unroll
        for (int j = 0; j < EPG; ++j) st_t[j] = s_in[e0 + j] * c1;
#pragma unroll
        for (int j = 0; j < EPG; ++j) st_t[j] = __builtin_amdgcn_exp2f(st_t[j]);
      } else if (ph == 1) {
#pragma unroll
        for (int j = 0; j < EPG; ++j) st_t[j] = 1.0f + st_t[j];
#pragma unroll
        for (int j = 0; j < EPG; ++j) st_g[j] = __builtin_amdgcn_rcpf(st_t[j]);
      } else if (ph == 2) {  // p' = s * sg, p' * (1 - sg) as p' - p' * sg
#pragma unroll
        for (int j = 0; j < EPG; ++j) p[e0 + j] = s_in[e0 + j] * st_g[j];
#pragma unroll
        for (int j = 0; j < EPG; ++j) st_t[j] = __builtin_fmaf(-p[e0 + j], st_g[j], p[e0 + j]);
      } else {               // ds' = dp * (sg + alpha * p' * (1 - sg)): two fused multiply-adds after p'
#pragma unroll
        for (int j = 0; j < EPG; ++j) st_t[j] = __builtin_fmaf(alpha, st_t[j], st_g[j]);
#pragma unroll
        for (int j = 0; j < EPG; ++j) ds[e0 + j] = d_in[e0 + j] * st_t[j];
      }
    } else {
#pragma unroll
      for (int e = m * 16 / NS; e < (m + 1) * 16 / NS; ++e) bwd_elem(s_in[e], d_in[e], c1, alpha, p[e], ds[e]);
    }
    if (m % GRP == GRP - 1) fence();
  }
  if (mask) {
    asm volatile("" ::: "memory");  // not speculable: keeps the selects off the unmasked path
    const auto vis = vis_of();      // (the block's position is worked out on this path only)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const bool on = vis(r);
      p[r] = on ? p[r] : 0.f;
      ds[r] = on ? ds[r] : 0.f;
    }
  }
  pd_cur[0] = pack8(p); pd_cur[1] = pack8(p + 8);
  pd_cur[2] = pack8(ds); pd_cur[3] = pack8(ds + 8);
  fence();
}

// Head dimensions up to 64 + 64 fit two workgroups per CU (256 registers per lane, a handful
// spilled at 64 + 64): measured 1.36x faster than one on long sequences (H = 8, d = 64, the skewed
// 96 K-row batch: 4.32 -> 3.18 ms) and 1.67x on 4096 short ones.  At d = 128 the two accumulator
// sets alone take 128 registers and the kernel runs one wave per SIMD with the full register file.
// One item (owner tile) of one head.
template <int DQK, int DV, int NW, bool BIAS, bool PACKED>
__device__ __forceinline__ void dkdv_item(const AttnArgs& a, const Item& it, int h) {
  constexpr int QB = ST * DQK * 2, GB = ST * DV * 2;
  // Three tile buffers: an iteration of the main loop touches tiles j and j+1 while the copy of
  // tile j+2 is in flight.  One array per buffer, so that the compiler can see that a copy into
  // one cannot alias operand reads from another.
  __shared__ __attribute__((aligned(1024))) char smem0[QB + GB];
  __shared__ __attribute__((aligned(1024))) char smem1[QB + GB];
  __shared__ __attribute__((aligned(1024))) char smem2[QB + GB];
  __shared__ __attribute__((aligned(1024))) char tmem0[BIAS ? REC_TILE : 16];
  __shared__ __attribute__((aligned(1024))) char tmem1[BIAS ? REC_TILE : 16];
  __shared__ __attribute__((aligned(1024))) char tmem2[BIAS ? REC_TILE : 16];
  __shared__ float wtab[BIAS ? MAX_TS_BUCKETS : 1];
  auto qbuf = [&](int b) { return b == 0 ? smem0 : (b == 1 ? smem1 : smem2); };
  auto gbuf = [&](int b) { return qbuf(b) + QB; };
  auto tbuf = [&](int b) { return b == 0 ? tmem0 : (b == 1 ? tmem1 : tmem2); };

  const int H = a.num_heads;
  const int tid = threadIdx.x, lane = tid & 63, n = lane & 31, hh = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int64_t sq = (int64_t)H * DQK, sv = (int64_t)H * DV;
  const __bf16* qg = (const __bf16*)a.q + h * DQK;
  const __bf16* gg = (const __bf16*)a.d_o + h * DV;
  const __bf16* kg = (const __bf16*)a.k + (int64_t)it.row0 * sq + h * DQK;
  const __bf16* vg = (const __bf16*)a.v + (int64_t)it.row0 * sv + h * DV;

  const int orow = wave * 32 + n;
  const bool wave_on = wave * 32 < it.nrows;
  int2 wsq = {};
  if constexpr (PACKED) wsq = window_bounds(a.row_seq, it.row0 + orow, orow < it.nrows);
  bf16x8 kreg[DQK / 16], vreg[DV / 16];
  load_owner<DQK>(kreg, kg, sq, orow, it.nrows, hh);
  load_owner<DV>(vreg, vg, sv, orow, it.nrows, hh);
  BiasCtx bias = {};
  if constexpr (BIAS) bias = bias_setup<NW * 64>(a, wtab, it, orow, tid, hh);
  auto init_of = [&](const char* trec, int blk, const BlockBias& bb) {
    return ScoreInit<BIAS>{&bias, trec, blk, bb};
  };

  f32x16 dkacc[DQK / 32], dvacc[DV / 32];
#pragma unroll
  for (int i = 0; i < DQK / 32; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) dkacc[i][r] = 0.f;
#pragma unroll
  for (int i = 0; i < DV / 32; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) dvacc[i][r] = 0.f;

  const Stream st = make_stream<1>(it, a.causal);
  const int T = st.total, NB = 2 * T;  // tiles and 32-row blocks of the stream
  const float c1 = -a.alpha * 1.4426950408889634f;
  const int k_lo = it.pos0 + wave * 32, k_hi = k_lo + 31;

  RowAddr<DQK> raq; RowAddr<DV> rag; ColAddr<DQK> caq; ColAddr<DV> cag;
  raq.init(n, hh); rag.init(n, hh); caq.init(lane); cag.init(lane);

  auto copy_tile = [&](int j, int buf) {
    const TileRef t = tile_ref(it, st, j);
    tile_copy_async<DQK, NW>(qbuf(buf), qg + (int64_t)t.row * sq, sq, t.valid, wave, lane);
    tile_copy_async<DV, NW>(gbuf(buf), gg + (int64_t)t.row * sv, sv, t.valid, wave, lane);
    if (BIAS && wave == 0) rec_copy_async(tbuf(buf), a.ts_rec + t.row, t.valid, lane);
  };
  // Position of block i of the stream (i in [0, NB)); the positions grow with i.
  auto block_pos = [&](int i) { return tile_ref(it, st, i >> 1).pos + (i & 1) * 32; };
  Window win = {};  // (packed tiles: set below, once the first tile copies are on their way)
  // Plain tiles: the block positions grow by 32 inside a segment, so the first block any query of
  // which sees a key of this wave (first_on) and the last block the diagonal touches (last_masked:
  // position < k_hi) have closed forms, worked out once; a step then costs two comparisons instead
  // of the scalar arithmetic of a block position.
  int first_on = 0, last_masked = -1;
  if (!PACKED && a.causal) {
    first_on = NB;
#pragma unroll
    for (int g = 1; g >= 0; --g) {
      const int i0 = g ? 2 * st.n[0] : 0, nb = 2 * st.n[g];     // the segment's blocks [i0, i0 + nb)
      const int p0 = it.seg_pos0[g] + st.beg[g];                 // position of its first block
      if (nb > 0) {
        const int q = (k_lo - 31 - p0 + 31) >> 5;                // first block with pos + 31 >= k_lo
        const int f = q < 0 ? 0 : q;
        if (f < nb) first_on = i0 + f;
        const int m = (k_hi - 1 - p0) >> 5;                      // last block with pos < k_hi
        if (m >= 0 && last_masked < 0) last_masked = i0 + (m < nb - 1 ? m : nb - 1);
      }
    }
  }
  // Does any query of block i see a key of this wave?  Once true it stays true.
  auto block_on = [&](int i) {
    if constexpr (PACKED) return wave_on && block_pos(i) + 31 >= win.lo_min;
    else return wave_on && i >= first_on;
  };
  // Packed tiles: block i is not yet beyond the last row that sees a key of the wave (i < 0: no
  // such block).  Once false it stays false; a step is skipped when the block it would contract
  // is beyond, and with it every later step.
  auto not_past = [&](int i) { return !PACKED || i < 0 || block_pos(i) <= win.hi_max; };
  // Block i may hold pairs the mask hides ...
  auto mask_of = [&](int i) {
    if constexpr (PACKED) return win.masks(block_pos(i));
    else return i <= last_masked;
  };
  // ... and which of its rows the lane's key sees (made on the masked path only).
  auto vis_of = [&](int i) {
    return [&, i] {
      const int pos = block_pos(i);
      if constexpr (PACKED) return win.vis(pos, hh);
      else return VisAfter{k_lo + n - pos, hh};
    };
  };

  if (T > 0) copy_tile(0, 0);
  if (T > 1) copy_tile(1, 1);
  if constexpr (PACKED) {
    __builtin_amdgcn_sched_barrier(0);
    win = make_window(wsq, it.row0 + orow, orow < it.nrows, 1, a.causal);
  }
  tile_copy_wait<0>();
  tile_barrier();
  if (T > 0) {  // (no visible query at all: a context-parallel pair with every query before the keys)

  f32x16 sacc[2], dacc[2];  // S and dP of the blocks of even / odd index
  bf16x8 pd[2][4];          // P (2 halves) and dS (2 halves) of the blocks of even / odd index
#pragma unroll
  for (int x = 0; x < 2; ++x) {
#pragma unroll
    for (int r = 0; r < 16; ++r) { sacc[x][r] = 0.f; dacc[x][r] = 0.f; }
#pragma unroll
    for (int y = 0; y < 4; ++y)
#pragma unroll
      for (int e = 0; e < 8; ++e) pd[x][y][e] = (__bf16)0.f;
  }

  BlockTable tab = {};
  if constexpr (BIAS) {
    tab.fill(bias, 0, NB, it, st, lane);
    tab.fill(bias, 64, NB, it, st, lane);
  }
  auto bb_of = [&](int i) { return BIAS ? tab.get(i) : BlockBias{}; };

  // scores of block 0 on their own
  if (block_on(0)) {
    init_of(tbuf(0), 0, bb_of(0))(sacc[0]);
#pragma unroll
    for (int ks = 0; ks < DQK / 16; ++ks) sacc[0] = mfma(raq.read(qbuf(0), 0, ks), kreg[ks], sacc[0]);
#pragma unroll
    for (int ks = 0; ks < DV / 16; ++ks) dacc[0] = mfma(rag.read(gbuf(0), 0, ks), vreg[ks], dacc[0]);
  }
  // step 0: scores of block 1, elementwise of block 0, nothing to contract yet
  if (block_on(1)) {
    dkdv_step<DQK, DV, false>(init_of(tbuf(0), 1, bb_of(1)), qbuf(0), gbuf(0), 1, qbuf(0), gbuf(0), 0, raq, rag,
                              caq, cag, kreg, vreg, sacc[0], dacc[0], sacc[1], dacc[1], pd[1], pd[0],
                              dkacc, dvacc, c1, a.alpha, mask_of(0), vis_of(0));
  }

  // Iteration j: steps 2j+1 and 2j+2, which touch tiles j and j+1 only.
  auto iter = [&](int j, auto buf_tag) {
    constexpr int B0 = decltype(buf_tag)::value, B1 = (B0 + 1) % 3, B2 = (B0 + 2) % 3;
    if constexpr (BIAS)  // the iteration enters one set of the block table: refill the other
      if (((2 * j + 2) & 63) == 0) tab.fill(bias, 2 * j + 2 + 64, NB, it, st, lane);
    if (j + 2 < T) copy_tile(j + 2, B2);  // every wave left tile j-1 before the last barrier
    {
      const int i = 2 * j + 1;  // scores of (tile j+1, block 0), contraction of (tile j, block 0)
      if (block_on(i + 1 < NB ? i + 1 : i) && not_past(i - 1)) {
        dkdv_step<DQK, DV, true>(init_of(tbuf(B1), 0, bb_of(i + 1)), qbuf(B1), gbuf(B1), 0, qbuf(B0), gbuf(B0), 0, raq,
                                 rag, caq, cag, kreg, vreg, sacc[1], dacc[1], sacc[0], dacc[0], pd[0],
                                 pd[1], dkacc, dvacc, c1, a.alpha, mask_of(i), vis_of(i));
      }
    }
    if (j + 1 < T) {
      const int i = 2 * j + 2;  // scores of (tile j+1, block 1), contraction of (tile j, block 1)
      if (block_on(i + 1) && not_past(i - 1)) {
        dkdv_step<DQK, DV, true>(init_of(tbuf(B1), 1, bb_of(i + 1)), qbuf(B1), gbuf(B1), 1, qbuf(B0), gbuf(B0), 1, raq,
                                 rag, caq, cag, kreg, vreg, sacc[0], dacc[0], sacc[1], dacc[1], pd[1],
                                 pd[0], dkacc, dvacc, c1, a.alpha, mask_of(i), vis_of(i));
      }
    }
    tile_copy_wait<0>();
    tile_barrier();
  };
  for (int j = 0; j < T; j += 3) {
    iter(j, std::integral_constant<int, 0>{});
    if (j + 1 < T) iter(j + 1, std::integral_constant<int, 1>{});
    if (j + 2 < T) iter(j + 2, std::integral_constant<int, 2>{});
  }

  // contraction of the last block (tile T-1, block 1) on its own, if the step before it ran
  if (block_on(NB - 1) && not_past(NB - 2)) {
    const int lb = (T - 1) % 3;
    const char* qt = qbuf(lb);
    const char* gt = gbuf(lb);
#pragma unroll
    for (int c = 0; c < DV / 32; ++c) {
      dvacc[c] = mfma(cag.read(gt, 2, c), pd[1][0], dvacc[c]);
      dvacc[c] = mfma(cag.read(gt, 3, c), pd[1][1], dvacc[c]);
    }
#pragma unroll
    for (int c = 0; c < DQK / 32; ++c) {
      dkacc[c] = mfma(caq.read(qt, 2, c), pd[1][2], dkacc[c]);
      dkacc[c] = mfma(caq.read(qt, 3, c), pd[1][3], dkacc[c]);
    }
  }
  }  // T > 0

  // dK^T and dV^T accumulators: lane holds key row n, elements c*32 + 8*(r/4) + 4*hh + r%4.
  // (P is held without its factor alpha / N, like dS.)
  if (orow < it.nrows) {
    store_owner_major<DQK>(a.dk, ((int64_t)it.row0 + orow) * sq + h * DQK, dkacc, a.alpha * a.inv_n, hh,
                           a.accumulate, a.out_f32);
    store_owner_major<DV>(a.dv, ((int64_t)it.row0 + orow) * sv + h * DV, dvacc, a.alpha * a.inv_n, hh,
                          a.accumulate, a.out_f32);
  }
}

// One workgroup per (item, head), handed out by the hardware in index order, which is what
// balances items of very different cost - unless the grid is smaller than the number of (item,
// head) pairs: then a workgroup walks over every gridDim.x-th pair and fetches the descriptions of
// the next ones while it works on the current one, so that the stores of one item overlap the
// loads of the next and neither a workgroup launch nor the description's round trips lie between
// them.  With one workgroup per CU nothing else would overlap them; the host asks for it where
// items are many and of about equal cost (packed tiles, large batches).
template <int DQK, int DV, int NW, bool BIAS, bool PACKED>
__global__ void __launch_bounds__(NW * 64, (DQK + DV <= 128 ? 2 : 1)) hstu_dkdv_bf16(AttnArgs a) {
  Item it;
  const int64_t bound = a.xcd_parts <= 1 ? (int64_t)a.max_items * a.num_heads
                                         : 8 * (((int64_t)a.max_items + a.xcd_parts - 1) / a.xcd_parts);
  // (The variants built for two workgroups per CU never walk - the host launches them on the whole
  // grid - and are compiled without that path, whose prefetched descriptions would cost them
  // registers they do not have.)
  constexpr bool CAN_WALK = DQK + DV > 128;
  if (!CAN_WALK || (!PACKED && gridDim.x >= bound)) {
    const Unit un = unit_of(a, blockIdx.x);
    if (!un.on || !fetch_item<PACKED>(a.plan, un.slot, it)) return;
    dkdv_item<DQK, DV, NW, BIAS, PACKED>(a, it, un.h);
    return;
  }
  if constexpr (CAN_WALK) {
  const int n = a.plan.header[0];
  const int units = unit_count(a, n);
  // Every gridDim.x-th unit from blockIdx.x on - or, for a schedule in natural order (walk_chunks),
  // one contiguous run of this XCD's units (unit = 8 * j + XCD, see unit_of): whole sequences, whose
  // tiles then follow each other in time on one CU and find their streamed rows in the caches,
  // where a stride would beat against the number of tiles per sequence.
  int u = blockIdx.x, stride = (int)gridDim.x, end = units;
  if (a.walk_chunks && (gridDim.x & 7) == 0) {
    const int x = u & 7, m = u >> 3, wgs = (int)(gridDim.x >> 3), per = (units + 7) >> 3;
    const int c = (per + wgs - 1) / wgs;
    const int64_t last = (int64_t)8 * (m + 1) * c;
    u = 8 * m * c + x;
    stride = 8;
    end = last < units ? (int)last : units;
  }
  // The description of unit u, as loaded (all zeros, i.e. no rows, for a unit that is none).
  // (The items of packed tiles are in schedule order already: no indirection.)
  auto index_of = [&](const Unit& un) { return PACKED ? un.slot : a.plan.order[un.slot]; };
  auto valid = [&](const Unit& un) { return un.on && un.slot < n; };
  if (u >= end) return;
  Unit cur = unit_of(a, u);
  RawItem raw = {};
  if (valid(cur)) raw = load_raw_item(a.plan.items + index_of(cur));
  Unit nxt = {};
  int next = 0;
  if ((int64_t)u + stride < end) {
    nxt = unit_of(a, u + stride);
    if (valid(nxt)) next = index_of(nxt);
  }
  while (true) {
    const bool on = valid(cur) && decode_item(raw, it);
    const int h = cur.h;
    const bool more = (int64_t)u + stride < end;
    u += more ? stride : 0;
    if (more) {  // in flight while this item is worked on
      cur = nxt;
      raw = RawItem{};
      if (valid(cur)) raw = load_raw_item(a.plan.items + next);
      next = 0;
      if ((int64_t)u + stride < end) {
        nxt = unit_of(a, u + stride);
        if (valid(nxt)) next = index_of(nxt);
      }
    }
    if (on) dkdv_item<DQK, DV, NW, BIAS, PACKED>(a, it, h);
    if (!more) break;
    tile_barrier();  // every wave has left the item's tiles before the next item's copies land
  }
  }  // CAN_WALK
}

}  // namespace

hipError_t launch_dkdv_bf16(const AttnArgs& a, int d_qk, int d_v, hipStream_t stream) {
  if (a.waves != 4) return hipErrorInvalidValue;
  if (dkdv_pair_supported(a, d_qk, d_v) && !a.dkdv_one_wave)
    return launch_dkdv_pair_bf16(a, d_qk, d_v, stream);
  if (a.ts_rec && (a.nb < 1 || a.nb > MAX_TS_BUCKETS || !a.ts_w || !a.ts_rec_own)) return hipErrorInvalidValue;
  // One workgroup per CU is resident at the larger head dimensions: as many workgroups as CUs,
  // each walking over its share of the items.  Two per CU overlap each other's memory round
  // trips already, and the hardware's own dispatch serves them better (measured).
  const int64_t cap = (a.large_batch || a.walk_chunks) && d_qk + d_v > 128 ? 256 : 0;
  if (a.row_seq) {  // packed tiles: walking whatever the size of the batch
    if (a.ts_rec) HSTU_DISPATCH_G(d_qk + d_v > 128 ? 256 : 0, hstu_dkdv_bf16, 4, 4, true, true);
    HSTU_DISPATCH_G(d_qk + d_v > 128 ? 256 : 0, hstu_dkdv_bf16, 4, 4, false, true);
  }
  if (a.ts_rec) HSTU_DISPATCH_G(cap, hstu_dkdv_bf16, 4, 4, true, false);
  HSTU_DISPATCH_G(cap, hstu_dkdv_bf16, 4, 4, false, false);
}

}  // namespace hstu
