// bf16 forward kernel and the transposed copy of V it reads (see hstu_mfma.h for the common parts).
#include "hstu_mfma.h"

namespace hstu {

namespace {

// =============================================================================================
// Forward: owners are query rows, keys and values are streamed.
//   S^T = K Q^T (A = K tile rows, B = Q registers)  ->  P^T in accumulator layout
//   O^T += V^T P^T (A = V tile transposed read, B = P^T registers)
// =============================================================================================

// The stream of keys is processed in blocks of 32, software-pipelined across blocks and tiles.
// Step i issues, interleaved and independent of each other,
//   the matrix instructions of S(i+1) = K(i+1) Q^T              (DQK/16 instructions),
//   the matrix instructions of O^T += V(i-1)^T P(i-1)^T          (DV/16 instructions),
//   the SiLU that turns S(i) into P(i)                           (vector instructions),
// so that every wave's instruction stream is an even mix of matrix and vector work: two waves
// of a SIMD then keep both pipes busy whatever their relative phase (a matrix instruction
// holds its own wave's issue for a while, the other wave's vector instructions fill that time).
// Two S accumulator sets and two P operand sets alternate by block parity.
//
// Causal mask: key r (accumulator element) of block i is visible to the lane's query iff
// 8*(r/4) + 4*hh + r%4 <= rel, rel = query position - block position; applied to the finished
// P under a wave-uniform branch, so the matrix instructions follow one path whether or not a
// block is masked.  A block none of whose keys is visible comes out as zeros.
template <int DQK, int DV, bool PV, class VAddr, class Init, class Vis>
__device__ __forceinline__ void fwd_step(const Init& init, const char* kn, int bn, const char* vp, int bp,
                                         const RowAddr<DQK>& ra, const VAddr& ca,
                                         const bf16x8 (&qreg)[DQK / 16], const f32x16& s_in,
                                         f32x16& s_out, const bf16x8 (&p_prev)[2],
                                         bf16x8 (&p_cur)[2], f32x16 (&oacc)[DV / 32], float c1,
                                         bool mask, const Vis& vis_of) {
  constexpr int KS = DQK / 16, NPV = DV / 16, NSL = KS > NPV ? KS : NPV;
  constexpr int AHEAD = 3;  // operand reads in flight ahead of their use
  bf16x8 ka[KS], va[NPV];
  auto fence = [] { __builtin_amdgcn_sched_barrier(0); };
  init(s_out);
#pragma unroll
  for (int m = 0; m < AHEAD; ++m) {
    if (m < KS) ka[m] = ra.read(kn, bn, m);
    if (PV && m < NPV) va[m] = ca.read(vp, bp * 2 + (m & 1), m >> 1);
  }
  fence();
  float p[16];
#pragma unroll
  for (int m = 0; m < NSL; ++m) {
    const int e0 = m * 16 / NSL, e1 = (m + 1) * 16 / NSL, em = (e0 + e1 + 1) / 2;
    if (m < KS) s_out = mfma(ka[m], qreg[m], s_out);
    if (m + AHEAD < KS) ka[m + AHEAD] = ra.read(kn, bn, m + AHEAD);
#pragma unroll
    for (int e = e0; e < em; ++e) p[e] = s_in[e] * sigmoid_scaled(s_in[e], c1);
    fence();
    if (PV && m < NPV) oacc[m >> 1] = mfma(va[m], p_prev[m & 1], oacc[m >> 1]);
    if (PV && m + AHEAD < NPV) va[m + AHEAD] = ca.read(vp, bp * 2 + ((m + AHEAD) & 1), (m + AHEAD) >> 1);
#pragma unroll
    for (int e = em; e < e1; ++e) p[e] = s_in[e] * sigmoid_scaled(s_in[e], c1);
    fence();
  }
  if (mask) {
    asm volatile("" ::: "memory");  // not speculable: keeps the selects off the unmasked path
    const auto vis = vis_of();      // (the block's position is worked out on this path only)
#pragma unroll
    for (int r = 0; r < 16; ++r) p[r] = vis(r) ? p[r] : 0.f;
  }
  p_cur[0] = pack8(p);
  p_cur[1] = pack8(p + 8);
  fence();
}

// VT: the V tiles come from the transposed copy (plain row reads, one LDS instruction per matrix
// instruction); otherwise from V itself, row-major, through transposing reads (two per matrix
// instruction, but no transposed copy has to be built first: the choice for small problems).
// BIAS: with the timestamp bias (the records of the streamed rows travel with the K tiles).
// PACKED: packed tiles (see Window).
template <int DQK, int DV, int NW, bool VT, bool BIAS, bool PACKED>
__global__ void __launch_bounds__(NW * 64, 2) hstu_fwd_bf16(AttnArgs a) {
  static_assert(!(PACKED && VT), "packed tiles: row-major V tiles");
  constexpr int KB = ST * DQK * 2, VB = ST * DV * 2;
  // NBUF buffers each for the K tiles and the transposed V tiles; copies run PD tiles ahead.
  // Eight waves (one workgroup per CU) use three, four waves (two workgroups per CU) two.
  // One array per buffer, K and V apart (an iteration reads the K tile of one index and the V
  // tile of another while copies into the remaining ones are in flight): the compiler can then
  // see that a copy cannot alias the operand reads, and does not wait for it before them.
  constexpr int NBUF = NW >= 8 ? 3 : 2, PD = NBUF - 1;
  __shared__ __attribute__((aligned(1024))) char kmem0[KB];
  __shared__ __attribute__((aligned(1024))) char kmem1[KB];
  __shared__ __attribute__((aligned(1024))) char kmem2[NBUF > 2 ? KB : 1024];
  __shared__ __attribute__((aligned(1024))) char vmem0[VB];
  __shared__ __attribute__((aligned(1024))) char vmem1[VB];
  __shared__ __attribute__((aligned(1024))) char vmem2[NBUF > 2 ? VB : 1024];
  __shared__ __attribute__((aligned(1024))) char tmem0[BIAS ? REC_TILE : 16];
  __shared__ __attribute__((aligned(1024))) char tmem1[BIAS ? REC_TILE : 16];
  __shared__ __attribute__((aligned(1024))) char tmem2[BIAS && NBUF > 2 ? REC_TILE : 16];
  __shared__ float wtab[BIAS ? MAX_TS_BUCKETS : 1];
  auto kbuf = [&](int b) { return b == 0 ? kmem0 : (b == 1 ? kmem1 : kmem2); };
  auto vbuf = [&](int b) { return b == 0 ? vmem0 : (b == 1 ? vmem1 : vmem2); };
  auto tbuf = [&](int b) { return b == 0 ? tmem0 : (b == 1 ? tmem1 : tmem2); };

  const int H = a.num_heads;
  const Unit un = unit_of(a, blockIdx.x);
  const int slot = un.slot, h = un.h;
  Item it;
  if (!un.on || !fetch_item<PACKED>(a.plan, slot, it)) return;

  const int tid = threadIdx.x, lane = tid & 63, n = lane & 31, hh = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int64_t sq = (int64_t)H * DQK, sv = (int64_t)H * DV;
  const __bf16* qg = (const __bf16*)a.q + (int64_t)it.row0 * sq + h * DQK;
  const __bf16* kg = (const __bf16*)a.k + h * DQK;
  const int64_t tcols = (int64_t)ST * a.plan.max_stiles;           // columns of the transposed copy
  const __bf16* vtg = (const __bf16*)a.vt + (int64_t)h * DV * tcols;  // V^T of this head: [DV][tcols]
  const __bf16* vg = (const __bf16*)a.v + h * DV;

  const int orow = wave * 32 + n;  // this lane's owner row inside the tile
  const bool wave_on = wave * 32 < it.nrows;
  int2 wsq = {};
  if constexpr (PACKED) wsq = window_bounds(a.row_seq, it.row0 + orow, orow < it.nrows);
  bf16x8 qreg[DQK / 16];
  load_owner<DQK>(qreg, qg, sq, orow, it.nrows, hh);
  BiasCtx bias = {};
  if constexpr (BIAS) bias = bias_setup<NW * 64>(a, wtab, it, orow, tid, hh);
  auto init_of = [&](const char* trec, int blk, const BlockBias& bb) {
    return ScoreInit<BIAS>{&bias, trec, blk, bb};
  };

  f32x16 oacc[DV / 32];
#pragma unroll
  for (int i = 0; i < DV / 32; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) oacc[i][r] = 0.f;

  const Stream st = make_stream<0>(it, a.causal);
  const int T = st.total, NB = 2 * T;  // tiles and 32-key blocks of the stream
  const float c1 = -a.alpha * 1.4426950408889634f;
  const int q_lo = it.pos0 + wave * 32, q_hi = q_lo + 31;

  // K tile t lives in K buffer t % NBUF, V tile t in V buffer t % NBUF.
  auto copy_k = [&](int t, int buf) {
    const TileRef r = tile_ref(it, st, t);
    tile_copy_async<DQK, NW>(kbuf(buf), kg + (int64_t)r.row * sq, sq, r.valid, wave, lane);
    if (BIAS && wave == 0) rec_copy_async(tbuf(buf), a.ts_rec + r.row, r.valid, lane);
  };
  auto copy_v = [&](int t, int buf) {
    const TileRef r = tile_ref(it, st, t);
    if (VT) ttile_copy_async<DV, NW>(vbuf(buf), vtg + r.tcol, tcols, wave, lane);
    else tile_copy_async<DV, NW>(vbuf(buf), vg + (int64_t)r.row * sv, sv, r.valid, wave, lane);
  };
  // Position of block i (i in [0, NB)); positions grow with i.
  auto block_pos = [&](int i) { return tile_ref(it, st, i >> 1).pos + (i & 1) * 32; };
  Window win = {};  // (packed tiles: set below, once the first tile copies are on their way)
  // Does any key of block i precede (or equal) a query of this wave?  Once false it stays false.
  // (Packed tiles: no block lies beyond the last row that some row of the wave sees.)
  // Plain tiles: the block positions grow by 32 inside a segment, so the last block with a key
  // some query of the wave sees (last_on: position <= q_hi) and the first block the diagonal touches
  // (first_masked: position + 31 > q_lo) have closed forms, worked out once; a step then costs two
  // comparisons instead of the scalar arithmetic of a block position.
  int last_on = NB - 1, first_masked = NB;
  if (!PACKED && a.causal) {
    last_on = -1;
#pragma unroll
    for (int g = 1; g >= 0; --g) {
      const int i0 = g ? 2 * st.n[0] : 0, nb = 2 * st.n[g];  // the segment's blocks [i0, i0 + nb)
      const int p0 = it.seg_pos0[g] + st.beg[g];              // position of its first block
      if (nb > 0) {
        const int m = (q_hi - p0) >> 5;                       // last block with pos <= q_hi
        if (m >= 0 && last_on < 0) last_on = i0 + (m < nb - 1 ? m : nb - 1);
        const int f0 = ((q_lo - 31 - p0) >> 5) + 1;           // first block with pos + 31 > q_lo
        const int f = f0 < 0 ? 0 : f0;
        if (f < nb) first_masked = i0 + f;
      }
    }
  }
  auto block_on = [&](int i) {
    if constexpr (PACKED) return wave_on && i < NB && block_pos(i) <= win.hi_max;
    else return wave_on && i <= last_on;
  };
  // Packed tiles: has the stream reached the first row that some row of the wave sees by block i?
  // Once true it stays true.  A step skipped before that leaves its accumulators at their initial
  // zeros, from which the first step that runs derives P = 0 for the block before its own.
  auto started = [&](int i) { return !PACKED || block_pos(i < NB ? i : NB - 1) + 31 >= win.lo_min; };

  RowAddr<DQK> ra;
  ra.init(n, hh);
  typename std::conditional<VT, TrAddr<DV>, ColAddr<DV>>::type ca;
  if constexpr (VT) ca.init(n, hh); else ca.init(lane);
  static_assert(tile_loads<DV>() == DV / 8, "both kinds of V tile take the same number of loads");
  // wave-wide loads one wave issues per iteration (the in-flight count the waits below allow)
  constexpr int LPT = (tile_loads<DQK>() + NW - 1) / NW + (DV / 8 + NW - 1) / NW;

  // Iteration j of the main loop reads K tile j+1 and V tile j; K(0) is read before it.
  if (T > 0) { copy_k(0, 0); copy_v(0, 0); }
  if (T > 1) copy_k(1, 1);
  if (PD > 1 && T > 1) copy_v(1, 1);
  if (PD > 1 && T > 2) copy_k(2, 2);
  if constexpr (PACKED) {
    __builtin_amdgcn_sched_barrier(0);
    win = make_window(wsq, it.row0 + orow, orow < it.nrows, 0, a.causal);
  }
  tile_copy_wait<0>();
  tile_barrier();

  if (T > 0) {
    f32x16 sacc[2];   // S of the blocks of even / odd index
    bf16x8 pb[2][2];  // P (two 16-key halves) of the blocks of even / odd index
#pragma unroll
    for (int x = 0; x < 2; ++x) {
#pragma unroll
      for (int r = 0; r < 16; ++r) sacc[x][r] = 0.f;
#pragma unroll
      for (int y = 0; y < 2; ++y)
#pragma unroll
        for (int e = 0; e < 8; ++e) pb[x][y][e] = (__bf16)0.f;
    }
    auto mask_of = [&](int i) {
      if constexpr (PACKED) return win.masks(block_pos(i));
      else return i >= first_masked;
    };
    auto vis_of = [&](int i) {  // (made on the masked path only)
      return [&, i] {
        const int pos = block_pos(i);
        if constexpr (PACKED) return win.vis(pos, hh);
        else return VisBefore{q_lo + n - pos, hh};
      };
    };
    BlockTable tab = {};
    if constexpr (BIAS) {
      tab.fill(bias, 0, NB, it, st, lane);
      tab.fill(bias, 64, NB, it, st, lane);
    }
    auto bb_of = [&](int i) { return BIAS ? tab.get(i) : BlockBias{}; };

    // S of block 0 on its own, then step 0 (nothing to multiply by V yet)
    if (block_on(0) && started(1)) {
      init_of(tbuf(0), 0, bb_of(0))(sacc[0]);
#pragma unroll
      for (int ks = 0; ks < DQK / 16; ++ks) sacc[0] = mfma(ra.read(kbuf(0), 0, ks), qreg[ks], sacc[0]);
      fwd_step<DQK, DV, false>(init_of(tbuf(0), 1, bb_of(1)), kbuf(0), 1, vbuf(0), 0, ra, ca, qreg, sacc[0],
                               sacc[1], pb[1], pb[0], oacc, c1, mask_of(0), vis_of(0));
    }
    tile_barrier();  // iteration 0 copies over K tile 0, which the lines above read

    // Iteration j: steps 2j+1 and 2j+2.  Step i runs while block i-1 is visible: it finishes
    // P(i-1) V(i-1); whatever it computes for invisible blocks is masked to zero or unused.
    auto iter = [&](int j, auto buf_tag) {
      constexpr int B0 = decltype(buf_tag)::value, B1 = (B0 + 1) % NBUF;
      // tiles j-1 (V) and j (K) were left by every wave before the last barrier
      const bool both = j + 1 + PD < T;
      if constexpr (BIAS)  // the iteration enters one set of the block table: refill the other
        if (((2 * j + 2) & 63) == 0) tab.fill(bias, 2 * j + 2 + 64, NB, it, st, lane);
      if (both) copy_k(j + 1 + PD, (B0 + 1 + PD) % NBUF);
      if (j + PD < T) copy_v(j + PD, (B0 + PD) % NBUF);
      {
        const int i = 2 * j + 1;  // S of (tile j+1, block 0), P V of (tile j, block 0)
        if (block_on(i - 1) && started(i + 1))
          fwd_step<DQK, DV, true>(init_of(tbuf(B1), 0, bb_of(i + 1)), kbuf(B1), 0, vbuf(B0), 0, ra, ca, qreg, sacc[1],
                                  sacc[0], pb[0], pb[1], oacc, c1, mask_of(i), vis_of(i));
      }
      if (j + 1 < T) {
        const int i = 2 * j + 2;  // S of (tile j+1, block 1), P V of (tile j, block 1)
        if (block_on(i - 1) && started(i + 1))
          fwd_step<DQK, DV, true>(init_of(tbuf(B1), 1, bb_of(i + 1)), kbuf(B1), 1, vbuf(B0), 1, ra, ca, qreg, sacc[0],
                                  sacc[1], pb[1], pb[0], oacc, c1, mask_of(i), vis_of(i));
      }
      // what the next iteration reads must have landed; with copies two tiles ahead the ones
      // just issued may stay in flight
      if (PD > 1 && both) tile_copy_wait<LPT>(); else tile_copy_wait<0>();
      tile_barrier();
    };
    for (int j = 0; j < T; j += NBUF) {
      iter(j, std::integral_constant<int, 0>{});
      if (j + 1 < T) iter(j + 1, std::integral_constant<int, 1>{});
      if (NBUF > 2 && j + 2 < T) iter(j + 2, std::integral_constant<int, (NBUF > 2 ? 2 : 0)>{});
    }

    // P V of the last block (tile T-1, block 1) on its own
    if (block_on(NB - 1)) {
      const char* vt = vbuf((T - 1) % NBUF);
#pragma unroll
      for (int dvb = 0; dvb < DV / 32; ++dvb) {
        oacc[dvb] = mfma(ca.read(vt, 2, dvb), pb[1][0], oacc[dvb]);
        oacc[dvb] = mfma(ca.read(vt, 3, dvb), pb[1][1], oacc[dvb]);
      }
    }
  }

  // O^T accumulators: lane holds query row n, elements dvb*32 + 8*(r/4) + 4*hh + r%4.
  if (orow < it.nrows) {
    if (it.part > 0)  // one part of a split tile: an fp32 partial result, summed by the reduce kernel
      store_owner_major<DV>(a.partial, (((int64_t)(it.part - 1) * H + h) * (NW * 32) + orow) * DV, oacc,
                            a.alpha * a.inv_n, hh, 0, 1);
    else
      store_owner_major<DV>(a.o, ((int64_t)it.row0 + orow) * sv + h * DV, oacc, a.alpha * a.inv_n, hh,
                            a.accumulate, a.out_f32);
  }
}

// =============================================================================================
// Transposed copies of streamed tensors (see TrAddr): src [rows][H][D] -> dst [H][D][columns].
// One workgroup per (64-row streamed tile, head); memory bound, a few percent of a pass.
// =============================================================================================
template <int D>
__global__ void __launch_bounds__(256) hstu_transpose_bf16(const uint16_t* __restrict__ src,
                                                           uint16_t* __restrict__ dst, Plan plan,
                                                           int H) {
  constexpr int LD = D + 2;  // padded row length in elements (rows stay 4-byte aligned)
  __shared__ __attribute__((aligned(16))) uint16_t tile[ST * LD];
  const int i = blockIdx.x / H, h = blockIdx.x % H;
  if (i >= plan.header[1]) return;
  const int row0 = plan.ttile[2 * i], nrows = plan.ttile[2 * i + 1];
  const int64_t cols = (int64_t)ST * plan.max_stiles;
  const int tid = threadIdx.x;
  for (int c = tid; c < ST * (D / 8); c += 256) {
    const int r = c / (D / 8), ch = c % (D / 8);
    u32x4 v = {0u, 0u, 0u, 0u};
    if (r < nrows) v = *(const u32x4*)(src + ((int64_t)(row0 + r) * H + h) * D + ch * 8);
    uint32_t* t = (uint32_t*)(tile + r * LD + ch * 8);
    t[0] = v[0]; t[1] = v[1]; t[2] = v[2]; t[3] = v[3];
  }
  __syncthreads();
  for (int c = tid; c < D * 8; c += 256) {
    const int d = c >> 3, q = c & 7;                 // output row d, 16-byte chunk q of its 64 columns
    const int base = (q >> 1) * 16 + (q & 1) * 4;    // rows base+0..3 and base+8..11
    uint16_t e[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) e[j] = tile[(base + (j & 3) + ((j >> 2) << 3)) * LD + d];
    u32x4 v;
#pragma unroll
    for (int j = 0; j < 4; ++j) v[j] = (uint32_t)e[2 * j] | ((uint32_t)e[2 * j + 1] << 16);
    *(u32x4*)(dst + ((int64_t)h * D + d) * cols + (int64_t)ST * i + q * 8) = v;
  }
}

}  // namespace

int waves_bf16(int pass, int64_t owner_rows, int heads) {
  if (pass == PASS_FWD) {
    return (owner_rows / 256) * heads >= 2048 ? 8 : 4;
  }
  return 4;
}

hipError_t launch_transpose_bf16(const void* src, void* dst, const Plan& plan, int num_heads, int d,
                                 hipStream_t stream) {
  const dim3 grid((unsigned)((int64_t)plan.max_stiles * num_heads)), block(256);
  const uint16_t* s = (const uint16_t*)src;
  uint16_t* t = (uint16_t*)dst;
  if (d == 128) hipLaunchKernelGGL((hstu_transpose_bf16<128>), grid, block, 0, stream, s, t, plan, num_heads);
  else if (d == 64) hipLaunchKernelGGL((hstu_transpose_bf16<64>), grid, block, 0, stream, s, t, plan, num_heads);
  else if (d == 32) hipLaunchKernelGGL((hstu_transpose_bf16<32>), grid, block, 0, stream, s, t, plan, num_heads);
  else return hipErrorInvalidValue;
  return hipGetLastError();
}

hipError_t launch_fwd_bf16(const AttnArgs& a, int d_qk, int d_v, hipStream_t stream) {
  if (a.vt == nullptr) {  // no transposed copy of V was built
    if (a.waves != 4) return hipErrorInvalidValue;
    if (a.row_seq) {
      if (a.ts_rec) HSTU_DISPATCH_BIAS(hstu_fwd_bf16, 4, 4, false, true, true);
      HSTU_DISPATCH_D(hstu_fwd_bf16, 4, 4, false, false, true);
    }
    if (a.ts_rec) HSTU_DISPATCH_BIAS(hstu_fwd_bf16, 4, 4, false, true, false);
    HSTU_DISPATCH_D(hstu_fwd_bf16, 4, 4, false, false, false);
  }
  if (a.row_seq) return hipErrorInvalidValue;  // packed tiles read V row-major
  if (a.waves == 8) {
    if (a.ts_rec) HSTU_DISPATCH_BIAS(hstu_fwd_bf16, 8, 8, true, true, false);
    HSTU_DISPATCH_D(hstu_fwd_bf16, 8, 8, true, false, false);
  }
  if (a.waves == 4) {
    if (a.ts_rec) HSTU_DISPATCH_BIAS(hstu_fwd_bf16, 4, 4, true, true, false);
    HSTU_DISPATCH_D(hstu_fwd_bf16, 4, 4, true, false, false);
  }
  return hipErrorInvalidValue;
}

}  // namespace hstu
