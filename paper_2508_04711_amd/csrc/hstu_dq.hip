// bf16 dq kernel (see hstu_mfma.h for the common parts).
#include "hstu_mfma.h"

namespace hstu {

namespace {

// =============================================================================================
// dq pass: owners are query rows (Q and dO rows in registers), K and V are streamed.
//   S^T  = K Q^T   (A = K tile rows, B = Q registers)
//   dP^T = V dO^T  (A = V tile rows, B = dO registers)
//   dQ^T += K^T dS^T (A = K tile transposed read, B = dS^T registers)
// A second recomputation of S instead of atomics: dq is deterministic.
//
// One 32-key block at a time: scores, elementwise, contraction.  Two workgroups share a CU, so
// every SIMD has two waves of different workgroups, which are at unrelated points of this
// sequence and fill each other's gaps.  Keeping two blocks in flight per wave instead (as the
// other two passes do) needs more than the 256 registers a wave may have at this occupancy; the
// spills it caused cost more than the overlap gained (their reloads also wait for the tile
// copy in flight, because vector memory operations complete in order).
// =============================================================================================
// Sum of dS per bucket for the gradient of the bias table (dq pass only: it visits every pair once).
// A run of blocks that fall into one bucket adds up in a register per lane and goes to the
// workgroup's LDS table when the bucket changes; the pairs of a block that spans several
// buckets go there one by one.  The LDS table is 64-bit fixed point (see dw_to_fixed) and holds
// 2^shift copies of every bucket, a lane adds to copy (lane mod 2^shift).
constexpr int DW_LDS = 1024;  // entries of the workgroup's table
__host__ __device__ constexpr int dw_shift(int nb) {
  int s = 0;
  while (s < 5 && (nb << (s + 1)) <= DW_LDS) ++s;
  return s;
}
struct DwAcc {
  unsigned long long* dwl;  // LDS, 2^shift entries per bucket
  float sum;                // per lane: dS of the current run
  int cur;                  // bucket of the current run (uniform; -1: none)
  int shift;
  __device__ __forceinline__ void add(int bucket, int lane, float x) {
    atomicAdd(dwl + (bucket << shift) + (lane & ((1 << shift) - 1)), dw_to_fixed(x));
  }
  __device__ __forceinline__ void flush(int lane) {
    if (cur >= 0) {
      const float t = wave_sum(sum);
      if (lane == 0) atomicAdd(dwl + (cur << shift), dw_to_fixed(t));
    }
    sum = 0.f;
  }
};
static_assert(MAX_TS_BUCKETS <= DW_LDS, "one entry per bucket at least");

template <int DQK, int DV, bool BIAS, class Vis>
__device__ __forceinline__ void dq_block(const BiasCtx& bias, const char* trec,
                                                const BlockBias& bb, DwAcc& dwa,
                                                const char* kt, const char* vt, int blk,
                                                const RowAddr<DQK>& rak, const RowAddr<DV>& rav,
                                                const ColAddr<DQK>& cak,
                                                const bf16x8 (&qreg)[DQK / 16],
                                                const bf16x8 (&greg)[DV / 16],
                                                f32x16 (&dqacc)[DQK / 32], float c1, float alpha,
                                                bool mask, const Vis& vis, int n, int hh) {
  f32x16 s, dp;
  int bk[16];
#pragma unroll
  for (int r = 0; r < 16; ++r) { s[r] = 0.f; dp[r] = 0.f; }
  if constexpr (BIAS) bias_block(s, trec, blk, bias, bb, bk);
#pragma unroll
  for (int ks = 0; ks < DQK / 16; ++ks) s = mfma(rak.read(kt, blk, ks), qreg[ks], s);
#pragma unroll
  for (int ks = 0; ks < DV / 16; ++ks) dp = mfma(rav.read(vt, blk, ks), greg[ks], dp);
  // Stage by stage over eight elements at a time, so that no instruction consumes the result of
  // its predecessor (exp and rcp results are late: a dependent successor costs a hazard nop and
  // stalled cycles).  ds' = dp * (sg + alpha * s * (sg - sg^2)).
  // (Not with the bias: its variants are at the register limit, and the sixteen values in flight
  // would spill.)
  float ds[16];
  // silu'(x) = sg + x * (sg - sg^2), x = alpha * s: the dq pass needs no p, which saves an
  // instruction per score against the form the dk/dv pass uses.
  if constexpr (BIAS) {
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const float sg = sigmoid_scaled(s[r], c1);
      ds[r] = dp[r] * __builtin_fmaf(alpha * s[r], __builtin_fmaf(-sg, sg, sg), sg);
    }
  } else {
#pragma unroll
  for (int h = 0; h < 16; h += 8) {
    float t[8], g[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) t[j] = s[h + j] * c1;
#pragma unroll
    for (int j = 0; j < 8; ++j) t[j] = __builtin_amdgcn_exp2f(t[j]);
#pragma unroll
    for (int j = 0; j < 8; ++j) t[j] = 1.0f + t[j];
#pragma unroll
    for (int j = 0; j < 8; ++j) g[j] = __builtin_amdgcn_rcpf(t[j]);
#pragma unroll
    for (int j = 0; j < 8; ++j) t[j] = __builtin_fmaf(-g[j], g[j], g[j]);
#pragma unroll
    for (int j = 0; j < 8; ++j) t[j] = __builtin_fmaf(alpha * s[h + j], t[j], g[j]);
#pragma unroll
    for (int j = 0; j < 8; ++j) ds[h + j] = dp[h + j] * t[j];
  }
  }
  if (mask) {
#pragma unroll
    for (int r = 0; r < 16; ++r) ds[r] = vis(r) ? ds[r] : 0.f;
  }
  if constexpr (BIAS) {
    if (bb.uni) {
      if (bb.b0 != dwa.cur) {
        dwa.flush(n + 32 * hh);
        dwa.cur = bb.b0;
      }
      float t = 0.f;
#pragma unroll
      for (int r = 0; r < 16; ++r) t += ds[r];
      dwa.sum += t;
    } else {
#pragma unroll
      for (int r = 0; r < 16; ++r) dwa.add(bk[r], n + 32 * hh, ds[r]);
    }
  }
  const bf16x8 db0 = pack8(ds), db1 = pack8(ds + 8);
#pragma unroll
  for (int c = 0; c < DQK / 32; ++c) {
    dqacc[c] = mfma(cak.read(kt, blk * 2, c), db0, dqacc[c]);
    dqacc[c] = mfma(cak.read(kt, blk * 2 + 1, c), db1, dqacc[c]);
  }
}

template <int DQK, int DV, int NW, bool BIAS, bool PACKED>
__global__ void __launch_bounds__(NW * 64, 2) hstu_dq_bf16(AttnArgs a) {
  constexpr int KB = ST * DQK * 2, VB = ST * DV * 2;
  __shared__ __attribute__((aligned(1024))) char smem0[KB + VB];
  __shared__ __attribute__((aligned(1024))) char smem1[KB + VB];
  __shared__ __attribute__((aligned(1024))) char tmem0[BIAS ? REC_TILE : 16];
  __shared__ __attribute__((aligned(1024))) char tmem1[BIAS ? REC_TILE : 16];
  __shared__ float wtab[BIAS ? MAX_TS_BUCKETS : 1];
  __shared__ unsigned long long dwl[BIAS ? DW_LDS : 1];
  auto kbuf = [&](int b) { return b ? smem1 : smem0; };
  auto vbuf = [&](int b) { return (b ? smem1 : smem0) + KB; };
  auto tbuf = [&](int b) { return b ? tmem1 : tmem0; };

  const int H = a.num_heads;
  const Unit un = unit_of(a, blockIdx.x);
  const int slot = un.slot, h = un.h;
  Item it;
  if (!un.on || !fetch_item<PACKED>(a.plan, slot, it)) return;

  const int tid = threadIdx.x, lane = tid & 63, n = lane & 31, hh = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int64_t sq = (int64_t)H * DQK, sv = (int64_t)H * DV;
  const __bf16* qg = (const __bf16*)a.q + (int64_t)it.row0 * sq + h * DQK;
  const __bf16* gg = (const __bf16*)a.d_o + (int64_t)it.row0 * sv + h * DV;
  const __bf16* kg = (const __bf16*)a.k + h * DQK;
  const __bf16* vg = (const __bf16*)a.v + h * DV;

  const int orow = wave * 32 + n;
  const bool wave_on = wave * 32 < it.nrows;
  int2 wsq = {};
  if constexpr (PACKED) wsq = window_bounds(a.row_seq, it.row0 + orow, orow < it.nrows);
  bf16x8 qreg[DQK / 16], greg[DV / 16];
  load_owner<DQK>(qreg, qg, sq, orow, it.nrows, hh);
  load_owner<DV>(greg, gg, sv, orow, it.nrows, hh);
  BiasCtx bias = {};
  DwAcc dwa = {dwl, 0.f, -1, 0};
  if constexpr (BIAS) {
    dwa.shift = dw_shift(a.nb);
    for (int i = tid; i < (a.nb << dwa.shift); i += NW * 64) dwl[i] = 0ull;
    bias = bias_setup<NW * 64>(a, wtab, it, orow, tid, hh);
  }

  f32x16 dqacc[DQK / 32];
#pragma unroll
  for (int i = 0; i < DQK / 32; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) dqacc[i][r] = 0.f;

  const Stream st = make_stream<0>(it, a.causal);
  const float c1 = -a.alpha * 1.4426950408889634f;
  const int q_lo = it.pos0 + wave * 32, q_hi = q_lo + 31;

  RowAddr<DQK> rak; RowAddr<DV> rav; ColAddr<DQK> cak;
  rak.init(n, hh); rav.init(n, hh); cak.init(lane);

  if (st.total > 0) {
    const TileRef t0 = tile_ref(it, st, 0);
    tile_copy_async<DQK, NW>(kbuf(0), kg + (int64_t)t0.row * sq, sq, t0.valid, wave, lane);
    tile_copy_async<DV, NW>(vbuf(0), vg + (int64_t)t0.row * sv, sv, t0.valid, wave, lane);
    if (BIAS && wave == 0) rec_copy_async(tbuf(0), a.ts_rec + t0.row, t0.valid, lane);
  }
  Window win = {};
  if constexpr (PACKED) {  // (looked at only now that the first tile copies are on their way)
    __builtin_amdgcn_sched_barrier(0);
    win = make_window(wsq, it.row0 + orow, orow < it.nrows, 0, a.causal);
  }
  tile_copy_wait<0>();
  tile_barrier();

  BlockTable tab = {};
  if constexpr (BIAS) {
    tab.fill(bias, 0, 2 * st.total, it, st, lane);
    tab.fill(bias, 64, 2 * st.total, it, st, lane);
  }

  auto step = [&](int j, auto buf_tag) {
    constexpr int BUF = decltype(buf_tag)::value;
    const TileRef tj = tile_ref(it, st, j);
    if constexpr (BIAS)  // the step enters one set of the block table: refill the other
      if (j > 0 && ((2 * j) & 63) == 0) tab.fill(bias, 2 * j + 64, 2 * st.total, it, st, lane);
    if (j + 1 < st.total) {
      const TileRef tn = tile_ref(it, st, j + 1);
      tile_copy_async<DQK, NW>(kbuf(BUF ^ 1), kg + (int64_t)tn.row * sq, sq, tn.valid, wave, lane);
      tile_copy_async<DV, NW>(vbuf(BUF ^ 1), vg + (int64_t)tn.row * sv, sv, tn.valid, wave, lane);
      if (BIAS && wave == 0) rec_copy_async(tbuf(BUF ^ 1), a.ts_rec + tn.row, tn.valid, lane);
    }
    const char* kt = kbuf(BUF);
    const char* vt = vbuf(BUF);
    if (wave_on) {
#pragma unroll
      for (int blk = 0; blk < ST / 32; ++blk) {
        const int k_lo = tj.pos + blk * 32;
        // no key of the block is visible (packed tiles: to no row of the wave)
        if (blk * 32 >= tj.valid || (!PACKED && a.causal && k_lo > q_hi)) continue;
        if (PACKED && (k_lo > win.hi_max || k_lo + 31 < win.lo_min)) continue;
        const BlockBias bb = BIAS ? tab.get(2 * j + blk) : BlockBias{};
        if constexpr (PACKED)
          dq_block<DQK, DV, BIAS>(bias, tbuf(BUF), bb, dwa, kt, vt, blk, rak, rav, cak, qreg, greg, dqacc, c1,
                                  a.alpha, win.masks(k_lo), win.vis(k_lo, hh), n, hh);
        else
          dq_block<DQK, DV, BIAS>(bias, tbuf(BUF), bb, dwa, kt, vt, blk, rak, rav, cak, qreg, greg, dqacc, c1,
                                  a.alpha, a.causal && k_lo + 31 > q_lo, VisBefore{q_lo + n - k_lo, hh}, n, hh);
      }
    }
    tile_copy_wait<0>();
    tile_barrier();
  };
  for (int j = 0; j < st.total; j += 2) {
    step(j, std::integral_constant<int, 0>{});
    if (j + 1 < st.total) step(j + 1, std::integral_constant<int, 1>{});
  }

  if constexpr (BIAS) {
    // the workgroup's sums go to the call's table (double precision atomics: their order can
    // change the result by a unit of the 53rd bit, far below the fp32 it is rounded to)
    dwa.flush(lane);
    __syncthreads();
    for (int i = tid; i < a.nb; i += NW * 64) {
      unsigned long long t = 0ull;
      const int cm = (1 << dwa.shift) - 1;  // (rotated by i: neighbouring threads read different banks)
      for (int c = 0; c <= cm; ++c) t += dwl[(i << dwa.shift) + ((c + i) & cm)];
      if (t != 0ull) atomicAdd(a.d_ts_acc + i, dw_from_fixed(t));
    }
  }

  // dQ^T accumulators: lane holds query row n, elements c*32 + 8*(r/4) + 4*hh + r%4.
  if (orow < it.nrows) {
    if (it.part > 0)
      store_owner_major<DQK>(a.partial, (((int64_t)(it.part - 1) * H + h) * (NW * 32) + orow) * DQK, dqacc,
                             a.alpha * a.inv_n, hh, 0, 1);
    else
      store_owner_major<DQK>(a.dq, ((int64_t)it.row0 + orow) * sq + h * DQK, dqacc, a.alpha * a.inv_n,
                             hh, a.accumulate, a.out_f32);
  }
}

}  // namespace

hipError_t launch_dq_bf16(const AttnArgs& a, int d_qk, int d_v, hipStream_t stream) {
  if (a.waves != 4 || (a.ts_rec && !a.d_ts_acc)) return hipErrorInvalidValue;
  if (a.row_seq) {
    if (a.ts_rec) HSTU_DISPATCH_BIAS(hstu_dq_bf16, 4, 4, true, true);
    HSTU_DISPATCH_D(hstu_dq_bf16, 4, 4, false, true);
  }
  if (a.ts_rec) HSTU_DISPATCH_BIAS(hstu_dq_bf16, 4, 4, true, false);
  HSTU_DISPATCH_D(hstu_dq_bf16, 4, 4, false, false);
}

}  // namespace hstu
