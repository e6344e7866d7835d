// bf16 dk/dv kernel for the large head dimensions, two waves per SIMD (see hstu_mfma.h for the
// common parts and hstu_dkdv.hip for the one-wave-per-SIMD kernel it replaces on long sequences).
#include "hstu_mfma.h"

namespace hstu {

namespace {

// =============================================================================================
// The dk/dv pass of section 2.1's attention (gradient derived: with x = alpha*s, sg = sigmoid(x),
// p = x*sg/N, dp = <dO_i, V_j>/N, ds = dp*silu'(x): dV_j += p*dO_i, dK_j += alpha*ds*Q_i).
//
// At d_qk + d_v > 128 one wave cannot hold K, V and both accumulators in the 256 registers it
// has when two waves share a SIMD, and with one wave per SIMD nothing overlaps that wave's own
// matrix and vector instructions.  Here two waves share every 32 keys of the tile and split the
// work without repeating any of it:
//   role A (waves 0..3):  S = Q K^T,  the SiLU arithmetic (p' = s*sg and silu'),  dV^T += dO^T P
//   role B (waves 4..7):  dP = dO V^T,  dS = dP * silu' (silu' handed over by A),   dK^T += Q^T dS
// Each role issues 16 of the step's 32 matrix instructions; A holds K and the dV accumulators, B
// holds V and the dK accumulators (about half of the one-wave kernel's registers each).  silu'
// travels from A to B through LDS as fp32 in the accumulator layout (the two waves of a pair
// have identical lane layouts, so the exchange is a plain 16-byte write and read per four
// values); the mask is applied by A alone (a hidden pair has p' = silu' = 0, which zeroes dS too).
// (Handing over sg and p' instead, with silu' worked out by B, balances the two roles' vector
// work but doubles the exchange, and the LDS pipe is what this kernel is shortest of: measured
// 7.1 ms against 5.9 ms on the long skewed batch.)
//
// The stream of query rows is processed in blocks of 32 rows that live in a ring of six LDS
// buffers.  Step t:
//   A: scores of block t | SiLU of block t-1 (writes silu' of t-1) | dV contraction of block t-2
//   B: dP of block t-1   | dS of block t-2 (reads silu' of t-2)    | dK contraction of block t-3
//   B: the copy of block t+2 is issued at the start; block t+1 has landed at the end.
// One workgroup barrier per step orders the hand-over (the exchange buffers alternate by parity)
// and the reuse of ring buffers.  Steps run from 0 to blocks + 2; the blocks before block 0 are
// zeros (their ring buffers are cleared at the start) and blocks at or beyond the end are treated
// as wholly masked, so one step body serves the whole item.
// Role A is the longer role (the SiLU arithmetic is its alone) and the two meet at the barrier,
// so the step's time is A's: inside the loop A issues no copies, keeps no cursor and waits for no
// memory (B's waves do), and its last exchange write leaves a slot before the step ends.
// With the timestamp bias (BIAS) role A writes the block's bias into its score accumulator before
// the block's first product (see bias_block); the table's gradient belongs to the dq pass.
// =============================================================================================

constexpr int BR = 32;     // streamed rows per block
constexpr int NSLOT = 6;   // ring buffers
constexpr int PW = 8;      // waves per workgroup
constexpr int AHEAD_COPY = 2;  // the copy of block t + AHEAD_COPY is issued in step t

// Where the next block to copy lies: the rows of one head of Q and dO (the same rows of both
// tensors, which have equal row lengths here) and how many of the rows from there on are visible.
// Advancing costs a handful of scalar instructions per block; the segment is looked up again
// only where the stream passes from its first segment to the second.
template <int D>
struct BlockCursor {
  const __bf16* q;
  const __bf16* g;
  int valid;  // visible rows from the block's first row on (<= 0: none)
  int b;      // block index
  int row;    // the block's first row in the streamed tensors (the bias variant copies its records)
  __device__ __forceinline__ void seek(const AttnArgs& a, const Item& it, const Stream& st, int h, int blk) {
    const TileRef t = tile_ref(it, st, blk >> 1);
    const int o = (blk & 1) * BR;
    const int64_t off = (int64_t)(t.row + o) * a.num_heads * D + h * D;
    q = (const __bf16*)a.q + off;
    g = (const __bf16*)a.d_o + off;
    valid = t.valid - o;
    b = blk;
    row = t.row + o;
  }
  __device__ __forceinline__ void next(const AttnArgs& a, const Item& it, const Stream& st, int h) {
    if (b + 1 == 2 * st.n[0]) {
      seek(a, it, st, h, b + 1);
    } else {
      const int64_t step = (int64_t)BR * a.num_heads * D;
      q += step; g += step; valid -= BR; ++b; row += BR;
    }
  }
};

// Asynchronous copy of one block (BR rows of one head) into its swizzled LDS layout; see
// tile_copy_async.  Rows >= valid arrive as zeros.  One wave-wide load per wave at D = 128.
template <int D>
__device__ __forceinline__ void block_copy_async(char* buf, const __bf16* base, int rs, int valid,
                                                 int wave, int voff) {
  constexpr int CPR = D / 8, RPL = 64 / CPR, LOADS = BR / RPL;
  static_assert(LOADS == PW, "one load per wave");
  const int rows = valid < 0 ? 0 : (valid < BR ? valid : BR);
  // (readfirstlane: the size is uniform, and must be seen to be, or the load is wrapped in a loop
  // over the distinct resources of the lanes)
  const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
      (void*)base, 0, __builtin_amdgcn_readfirstlane(rows * rs), 0x00020000);
  __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, HSTU_LDS(void, buf + wave * 1024), 16, voff, 0, 0, 0);
}

// The same copy issued by the four waves of role B alone (two wave-wide loads per wave): inside the
// loop role A, whose vector work makes it the longer of the two, issues no copies, keeps no
// cursor and waits for no memory.
template <int D>
__device__ __forceinline__ void block_copy_async_half(char* buf, const __bf16* base, int rs, int valid,
                                                      int w, const int (&voff2)[2]) {
  static_assert(BR / (64 / (D / 8)) == PW, "two loads per wave of one role");
  const int rows = valid < 0 ? 0 : (valid < BR ? valid : BR);
  const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
      (void*)base, 0, __builtin_amdgcn_readfirstlane(rows * rs), 0x00020000);
  __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, HSTU_LDS(void, buf + (2 * w) * 1024), 16, voff2[0], 0, 0, 0);
  __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, HSTU_LDS(void, buf + (2 * w + 1) * 1024), 16, voff2[1], 0, 0, 0);
}

// Asynchronous copy of the timestamp records of one block into a 1 KB buffer (one wave-wide load:
// 32 records of 16 bytes; the lanes beyond them and rows >= valid arrive as zeros).
__device__ __forceinline__ void rec_block_copy_async(char* buf, const TsRecord* rec, int valid, int lane) {
  const int rows = valid < 0 ? 0 : (valid < BR ? valid : BR);
  const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
      (void*)rec, 0, __builtin_amdgcn_readfirstlane(rows * (int)sizeof(TsRecord)), 0x00020000);
  __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, HSTU_LDS(void, buf), 16, lane * 16, 0, 0, 0);
}

__device__ __forceinline__ void lds_writes_done() { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); }

typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;

// Exchange buffer of one (parity, 32 keys): [four accumulator elements][lane] as 16-byte groups;
// xw points at the lane's first group.
constexpr int XG = 256;        // floats between the groups of four elements
constexpr int XK = 4 * XG;     // floats per 32 keys

// Role A, one step: scores of the block at qn into s_out, SiLU of s_in (p' packed into p_cur,
// silu' written to xw), dV^T += dO^T P with the block at gp and p_prev.
template <int D, class Init, class Vis>
__device__ __forceinline__ void role_a_step(const Init& init, const char* qn, const char* gp, const RowAddr<D>& raq,
                                            const ColAddr<D>& cag, const bf16x8 (&kreg)[D / 16],
                                            const f32x16& s_in, f32x16& s_out,
                                            const bf16x8 (&p_prev)[2], bf16x8 (&p_cur)[2],
                                            f32x16 (&dvacc)[D / 32], float* xw, float c1, float alpha,
                                            bool mask, const Vis& vis_of) {
  constexpr int NS = D / 16;
  constexpr int AHEAD = 3;  // operand reads in flight ahead of their use
  static_assert(NS == 8, "eight slots per step: two groups of four stages");
  bf16x8 op[NS], tp[NS];
  auto fence = [] { __builtin_amdgcn_sched_barrier(0); };
  init(s_out);  // zeros, or the block's bias
#pragma unroll
  for (int m = 0; m < AHEAD; ++m) {
    op[m] = raq.read(qn, 0, m);
    tp[m] = cag.read(gp, m & 1, m >> 1);
  }
  fence();
  // The arithmetic of eight elements per group, one stage per slot, so that no instruction consumes
  // its predecessor's result; a group's results leave the registers (silu' to the exchange buffer,
  // p' packed) as soon as they are complete.  The first group takes slots 0..3, the second slots
  // 3..6: the last slot has no stage, so the wave's exchange writes are under way while its last
  // matrix instructions issue, and the wait for them that ends the step finds them done.
  float p[2][8], st_t[2][8], st_g[2][8];
  auto stage = [&](auto gtag, int ph) {
    constexpr int G = decltype(gtag)::value, e0 = G * 8;
    if (ph == 0) {
#pragma unroll
      for (int j = 0; j < 8; ++j) st_t[G][j] = s_in[e0 + j] * c1;
#pragma unroll
      for (int j = 0; j < 8; ++j) st_t[G][j] = __builtin_amdgcn_exp2f(st_t[G][j]);
    } else if (ph == 1) {
#pragma unroll
      for (int j = 0; j < 8; ++j) st_t[G][j] = 1.0f + st_t[G][j];
#pragma unroll
      for (int j = 0; j < 8; ++j) st_g[G][j] = __builtin_amdgcn_rcpf(st_t[G][j]);
    } else if (ph == 2) {  // p' = s * sg, p' * (1 - sg) as p' - p' * sg
#pragma unroll
      for (int j = 0; j < 8; ++j) p[G][j] = s_in[e0 + j] * st_g[G][j];
#pragma unroll
      for (int j = 0; j < 8; ++j) st_t[G][j] = __builtin_fmaf(-p[G][j], st_g[G][j], p[G][j]);
    } else {               // silu' = sg + alpha * p' * (1 - sg): two fused multiply-adds after p'
#pragma unroll
      for (int j = 0; j < 8; ++j) st_g[G][j] = __builtin_fmaf(alpha, st_t[G][j], st_g[G][j]);
      if (mask) {
        asm volatile("" ::: "memory");  // not speculable: keeps the selects off the unmasked path
        const auto vis = vis_of();
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          const bool on = vis(e0 + j);
          p[G][j] = on ? p[G][j] : 0.f;
          st_g[G][j] = on ? st_g[G][j] : 0.f;
        }
      }
#pragma unroll
      for (int q4 = 0; q4 < 2; ++q4) {
        const f32x4 vf = {st_g[G][4 * q4], st_g[G][4 * q4 + 1], st_g[G][4 * q4 + 2], st_g[G][4 * q4 + 3]};
        *HSTU_LDS(f32x4, xw + (e0 / 4 + q4) * XG) = vf;
      }
      p_cur[G] = pack8(p[G]);
    }
  };
#pragma unroll
  for (int m = 0; m < NS; ++m) {
    s_out = mfma(op[m], kreg[m], s_out);
    dvacc[m >> 1] = mfma(tp[m], p_prev[m & 1], dvacc[m >> 1]);
    if (m + AHEAD < NS) {
      op[m + AHEAD] = raq.read(qn, 0, m + AHEAD);
      tp[m + AHEAD] = cag.read(gp, (m + AHEAD) & 1, (m + AHEAD) >> 1);
    }
    if (m < 4) stage(std::integral_constant<int, 0>{}, m);
    if (m >= 3 && m < 7) stage(std::integral_constant<int, 1>{}, m - 3);
    fence();
  }
}

// Role B, one step: dP of the block at gn into d_out, dS = d_in * silu' (read from xr) packed into
// ds_cur, dK^T += Q^T dS with the block at qp and ds_prev.
template <int D>
__device__ __forceinline__ void role_b_step(const char* gn, const char* qp, const RowAddr<D>& rag,
                                            const ColAddr<D>& caq, const bf16x8 (&vreg)[D / 16],
                                            const f32x16& d_in, f32x16& d_out,
                                            const bf16x8 (&ds_prev)[2], bf16x8 (&ds_cur)[2],
                                            f32x16 (&dkacc)[D / 32], const float* xr) {
  constexpr int NS = D / 16;
  constexpr int AHEAD = 3;
  bf16x8 op[NS], tp[NS];
  auto fence = [] { __builtin_amdgcn_sched_barrier(0); };
#pragma unroll
  for (int r = 0; r < 16; ++r) d_out[r] = 0.f;
  f32x4 x4[4];
#pragma unroll
  for (int q4 = 0; q4 < 4; ++q4) x4[q4] = *HSTU_LDS(const f32x4, xr + q4 * XG);
#pragma unroll
  for (int m = 0; m < AHEAD; ++m) {
    op[m] = rag.read(gn, 0, m);
    tp[m] = caq.read(qp, m & 1, m >> 1);
  }
  fence();
  float ds[16];
#pragma unroll
  for (int m = 0; m < NS; ++m) {
    d_out = mfma(op[m], vreg[m], d_out);
    dkacc[m >> 1] = mfma(tp[m], ds_prev[m & 1], dkacc[m >> 1]);
    if (m + AHEAD < NS) {
      op[m + AHEAD] = rag.read(gn, 0, m + AHEAD);
      tp[m + AHEAD] = caq.read(qp, (m + AHEAD) & 1, (m + AHEAD) >> 1);
    }
#pragma unroll
    for (int e = m * 16 / NS; e < (m + 1) * 16 / NS; ++e) ds[e] = d_in[e] * x4[e >> 2][e & 3];
    fence();
  }
  ds_cur[0] = pack8(ds);
  ds_cur[1] = pack8(ds + 8);
  fence();
}

// The whole item for one role (ROLE 0: A, 1: B).
template <int D, int ROLE, bool BIAS>
__device__ __forceinline__ void pair_body(const AttnArgs& a, const Item& it, int h, char* ring0,
                                          char* ring1, char* ring2, char* ring3, char* ring4,
                                          char* ring5, float* xbuf0, float* xbuf1, char* rec0, char* rec1,
                                          char* rec2, char* rec3, char* rec4, char* rec5, float* wtab) {
  constexpr int QB = BR * D * 2;
  auto ring = [&](int b) {
    return b == 0 ? ring0 : (b == 1 ? ring1 : (b == 2 ? ring2 : (b == 3 ? ring3 : (b == 4 ? ring4 : ring5))));
  };
  auto recb = [&](int b) {  // the records of the block in ring buffer b (bias variant)
    return b == 0 ? rec0 : (b == 1 ? rec1 : (b == 2 ? rec2 : (b == 3 ? rec3 : (b == 4 ? rec4 : rec5))));
  };
  const int H = a.num_heads;
  const int tid = threadIdx.x, lane = tid & 63, n = lane & 31, hh = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int g = wave & 3;  // which 32 keys of the tile
  const int64_t sr = (int64_t)H * D;
  const int rs = H * D * 2;  // bytes per row
  const int orow = g * 32 + n;

  const Stream st = make_stream<1>(it, a.causal);
  const int NBLK = 2 * st.total;  // 32-row blocks of the stream
  // the lane's part of a block copy: row wave * RPL + lane / CPR, swizzled chunk
  const int crow = wave * (64 / (D / 8)) + lane / (D / 8);
  const int voff = crow * rs + (((lane % (D / 8)) ^ swz<D>(crow)) << 4);
  BlockCursor<D> cur;
  auto copy_next = [&](char* buf, char* rbuf) {  // copies block cur.b, then moves on
    block_copy_async<D>(buf, cur.q, rs, cur.valid, wave, voff);
    block_copy_async<D>(buf + QB, cur.g, rs, cur.valid, wave, voff);
    if (BIAS && wave == 0) rec_block_copy_async(rbuf, a.ts_rec + cur.row, cur.valid, lane);
    cur.next(a, it, st, h);
  };
  // The copy issued in every step, by role B: block cur.b while the stream lasts, afterwards a copy
  // of no rows (zeros arrive; the buffer is one that no later step reads for anything that counts).
  // Every step thus issues the same four loads and waits with the same count, with no branch around
  // either: the compiler's own bookkeeping of copies in flight follows that, whereas with a
  // condition evaluated at both places it assumed older copies pending and put a wait for
  // everything in front of some steps' first operand reads, i.e. right behind the copy just issued.
  int voff2[2] = {0, 0};
  if constexpr (ROLE == 1) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int r2 = (2 * g + i) * (64 / (D / 8)) + lane / (D / 8);
      voff2[i] = r2 * rs + (((lane % (D / 8)) ^ swz<D>(r2)) << 4);
    }
  }
  // (With the bias every wave of role B also issues the load of the block's records: the same
  // kilobyte four times, so that all four keep the same count of loads in flight.)
  auto copy_step = [&](char* buf, char* rbuf, bool live) {
    const int valid = live ? cur.valid : 0;
    block_copy_async_half<D>(buf, cur.q, rs, valid, g, voff2);
    block_copy_async_half<D>(buf + QB, cur.g, rs, valid, g, voff2);
    if constexpr (BIAS) rec_block_copy_async(rbuf, a.ts_rec + (live ? cur.row : 0), valid, lane);
    if (live) cur.next(a, it, st, h);
  };
  auto block_pos = [&](int b) { return tile_ref(it, st, b >> 1).pos + (b & 1) * BR; };

  // Ring buffers 4 and 5 stand for the two blocks before the first one (the contractions of the
  // first two steps read them against operands that are zero): cleared, so that those products
  // are zeros whatever the memory held.
  {
    const u32x4 z = {0u, 0u, 0u, 0u};
    for (int i = tid; i < 2 * QB / 16; i += PW * 64) {
      *HSTU_LDS(u32x4, ring4 + i * 16) = z;
      *HSTU_LDS(u32x4, ring5 + i * 16) = z;
    }
  }
  bf16x8 oreg[D / 16];  // A: the K rows, B: the V rows
  {
    const __bf16* og = (const __bf16*)(ROLE == 0 ? a.k : a.v) + (int64_t)it.row0 * sr + h * D;
    load_owner<D>(oreg, og, sr, orow, it.nrows, hh);
  }
  if (NBLK > 0) {
    cur.seek(a, it, st, h, 0);
    copy_next(ring0, rec0);
    copy_next(ring1, rec1);  // (NBLK is even)
  }
  // The bias enters the scores only, i.e. role A's product (the table's gradient is the dq pass's).
  BiasCtx bias = {};
  if constexpr (BIAS) bias = bias_setup<PW * 64>(a, wtab, it, orow, tid, hh);  // (all waves: has a barrier)

  const float c1 = -a.alpha * 1.4426950408889634f;
  const int k_lo = it.pos0 + g * 32, k_hi = k_lo + 31;
  // The last block the diagonal touches (position < k_hi); block positions grow with the index.
  int last_masked = -1;
  if (ROLE == 0 && a.causal) {
#pragma unroll
    for (int s = 1; s >= 0; --s) {
      const int i0 = s ? 2 * st.n[0] : 0, nb = 2 * st.n[s];
      const int p0 = it.seg_pos0[s] + st.beg[s];
      if (nb > 0) {
        const int m = (k_hi - 1 - p0) >> 5;
        if (m >= 0 && last_masked < 0) last_masked = i0 + (m < nb - 1 ? m : nb - 1);
      }
    }
  }

  f32x16 acc[D / 32];  // A: dV^T, B: dK^T
#pragma unroll
  for (int i = 0; i < D / 32; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;

  RowAddr<D> ra;  // A: rows of Q, B: rows of dO
  ColAddr<D> ca;  // A: dO transposed, B: Q transposed
  ra.init(n, hh); ca.init(lane);

  lds_writes_done();
  tile_copy_wait<0>();
  tile_barrier();

  if (NBLK > 0) {
    f32x16 sd[2];     // A: S, B: dP of the blocks of even / odd index
    bf16x8 pk[2][2];  // A: P, B: dS of the blocks of even / odd index
#pragma unroll
    for (int x = 0; x < 2; ++x) {
#pragma unroll
      for (int r = 0; r < 16; ++r) sd[x][r] = 0.f;
#pragma unroll
      for (int y = 0; y < 2; ++y)
#pragma unroll
        for (int e = 0; e < 8; ++e) pk[x][y][e] = (__bf16)0.f;
    }
    float* xa0 = xbuf0 + g * XK + lane * 4;
    float* xa1 = xbuf1 + g * XK + lane * 4;
    const int nsteps = NBLK + 3;
    BlockTable tab = {};
    if constexpr (BIAS && ROLE == 0) {
      tab.fill(bias, 0, NBLK, it, st, lane);
      tab.fill(bias, 64, NBLK, it, st, lane);
    }

    auto step = [&](int t, auto tag) {
      constexpr int S = decltype(tag)::value;  // t mod 6; S & 1 is the parity of t
      if constexpr (ROLE == 1)
        copy_step(ring((S + AHEAD_COPY) % NSLOT), recb((S + AHEAD_COPY) % NSLOT), t + AHEAD_COPY < NBLK);
      if constexpr (ROLE == 0) {
        if constexpr (BIAS)  // the stream enters one set of the block table: refill the other
          if (t > 0 && (t & 63) == 0) tab.fill(bias, t + 64, NBLK, it, st, lane);
        if (t <= NBLK + 1) {  // (nothing left to contract in the last step)
          // block t-1: masked when the diagonal touches it or when it lies beyond the stream
          const int b = t - 1;
          const bool mask = b <= last_masked || b >= NBLK;
          auto vis_of = [&] {
            const int rel = b >= NBLK ? (1 << 20) : k_lo + n - block_pos(b < 0 ? 0 : b);
            return VisAfter{rel, hh};
          };
          const ScoreInit<BIAS> init = {&bias, recb(S), 0, BIAS ? tab.get(t) : BlockBias{}};
          role_a_step<D>(init, ring(S), ring((S + 4) % NSLOT) + QB, ra, ca, oreg, sd[(S + 1) & 1], sd[S & 1],
                         pk[S & 1], pk[(S + 1) & 1], acc, (S + 1) & 1 ? xa1 : xa0, c1, a.alpha, mask, vis_of);
          lds_writes_done();
        }
      } else {
        if (t >= 1)  // (nothing to work on in the first step)
          role_b_step<D>(ring((S + 5) % NSLOT) + QB, ring((S + 3) % NSLOT), ra, ca, oreg, sd[S & 1],
                         sd[(S + 1) & 1], pk[(S + 1) & 1], pk[S & 1], acc, S & 1 ? xa1 : xa0);
      }
      // block t+1 must have landed; the copies of the later blocks may stay in flight
      if constexpr (ROLE == 1) tile_copy_wait<(BIAS ? 5 : 4) * (AHEAD_COPY - 1)>();
      tile_barrier();
    };
    for (int t = 0; t < nsteps; t += NSLOT) {
      step(t, std::integral_constant<int, 0>{});
      if (t + 1 < nsteps) step(t + 1, std::integral_constant<int, 1>{});
      if (t + 2 < nsteps) step(t + 2, std::integral_constant<int, 2>{});
      if (t + 3 < nsteps) step(t + 3, std::integral_constant<int, 3>{});
      if (t + 4 < nsteps) step(t + 4, std::integral_constant<int, 4>{});
      if (t + 5 < nsteps) step(t + 5, std::integral_constant<int, 5>{});
    }
    tile_copy_wait<0>();  // (the last steps' empty copies: nothing may be in flight when the workgroup's LDS is released)
  }

  // Accumulators: lane holds key row n, elements c*32 + 8*(r/4) + 4*hh + r%4 (P and dS are held
  // without their factor alpha / N).
  if (orow < it.nrows)
    store_owner_major<D>(ROLE == 0 ? a.dv : a.dk, ((int64_t)it.row0 + orow) * sr + h * D, acc,
                         a.alpha * a.inv_n, hh, a.accumulate, a.out_f32);
}

template <int D, bool BIAS>
__global__ void __launch_bounds__(PW * 64) hstu_dkdv_pair_bf16(AttnArgs a) {
  constexpr int QB = BR * D * 2;
  // One array per ring buffer (the Q block, then the dO block), so that the compiler can see that
  // a copy into one cannot alias operand reads from another.
  __shared__ __attribute__((aligned(1024))) char ring0[2 * QB];
  __shared__ __attribute__((aligned(1024))) char ring1[2 * QB];
  __shared__ __attribute__((aligned(1024))) char ring2[2 * QB];
  __shared__ __attribute__((aligned(1024))) char ring3[2 * QB];
  __shared__ __attribute__((aligned(1024))) char ring4[2 * QB];
  __shared__ __attribute__((aligned(1024))) char ring5[2 * QB];
  __shared__ __attribute__((aligned(1024))) float xbuf0[4 * XK];  // silu' of blocks of even index
  __shared__ __attribute__((aligned(1024))) float xbuf1[4 * XK];  // ... of odd index
  // bias variant: the timestamp records of the blocks in the ring buffers, and the table
  __shared__ __attribute__((aligned(1024))) char rec0[BIAS ? 1024 : 16];
  __shared__ __attribute__((aligned(1024))) char rec1[BIAS ? 1024 : 16];
  __shared__ __attribute__((aligned(1024))) char rec2[BIAS ? 1024 : 16];
  __shared__ __attribute__((aligned(1024))) char rec3[BIAS ? 1024 : 16];
  __shared__ __attribute__((aligned(1024))) char rec4[BIAS ? 1024 : 16];
  __shared__ __attribute__((aligned(1024))) char rec5[BIAS ? 1024 : 16];
  __shared__ float wtab[BIAS ? MAX_TS_BUCKETS : 1];

  const Unit un = unit_of(a, blockIdx.x);
  Item it;
  if (!un.on || !fetch_item<false>(a.plan, un.slot, it)) return;
  const int role = __builtin_amdgcn_readfirstlane(threadIdx.x >> 8);
  if (role == 0)
    pair_body<D, 0, BIAS>(a, it, un.h, ring0, ring1, ring2, ring3, ring4, ring5, xbuf0, xbuf1, rec0, rec1, rec2,
                          rec3, rec4, rec5, wtab);
  else
    pair_body<D, 1, BIAS>(a, it, un.h, ring0, ring1, ring2, ring3, ring4, ring5, xbuf0, xbuf1, rec0, rec1, rec2,
                          rec3, rec4, rec5, wtab);
}

}  // namespace

// The pair kernel serves per-sequence schedules, with or without the timestamp bias (no packed
// tiles, no walking workgroups), of the head dimensions that do not fit two workgroups per CU.
bool dkdv_pair_supported(const AttnArgs& a, int d_qk, int d_v) {
  if (a.ts_rec && (a.nb < 1 || a.nb > MAX_TS_BUCKETS || !a.ts_w || !a.ts_rec_own)) return false;
  return d_qk == 128 && d_v == 128 && !a.row_seq && !a.large_batch && !a.walk_chunks && a.waves == 4;
}

hipError_t launch_dkdv_pair_bf16(const AttnArgs& a, int d_qk, int d_v, hipStream_t stream) {
  if (!dkdv_pair_supported(a, d_qk, d_v)) return hipErrorInvalidValue;
  const int64_t units = a.xcd_parts <= 1 ? (int64_t)a.max_items * a.num_heads
                                         : 8 * (((int64_t)a.max_items + a.xcd_parts - 1) / a.xcd_parts);
  if (a.ts_rec) hipLaunchKernelGGL((hstu_dkdv_pair_bf16<128, true>), dim3((unsigned)units), dim3(PW * 64), 0, stream, a);
  else hipLaunchKernelGGL((hstu_dkdv_pair_bf16<128, false>), dim3((unsigned)units), dim3(PW * 64), 0, stream, a);
  return hipGetLastError();
}

}  // namespace hstu
