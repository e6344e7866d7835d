// bf16 jagged HSTU attention on the gfx950 matrix cores: what the forward, dk/dv and dq kernels
// (hstu_fwd.hip, hstu_dkdv.hip, hstu_dq.hip: one translation unit each, so that they compile in
// parallel) share.
//
// Paper, section 2.1: O = Mask(SiLU(alpha * Q K^T)) V (bias absent), here divided by max_len.
// All three kernels share one shape.  A workgroup takes one schedule item for one head: a
// tile of "owner" rows, 32 per wavefront, whose data a wave keeps in registers as MFMA B
// operands, and streams the other side's rows through LDS in tiles of 64 (two or three tile
// buffers, filled by asynchronous copies one or two tiles ahead) as MFMA A operands.  Scores
// are produced transposed with respect to the owner rows so that the accumulator registers of
// the first product are, lane for lane, the B (or A) operand of the second one; nothing but
// the streamed tiles ever goes through LDS.
//
//   v_mfma_f32_32x32x16_bf16  D[32x32] += A[32x16] * B[16x32]   (lane l: n = l%32, hh = l/32)
//     A: lane holds row n,    k = 8*hh .. 8*hh+7          B: lane holds column n, same k
//     D: lane holds column n, rows 8*(r/4) + 4*hh + r%4   for r = 0..15
//
// Products whose contraction runs over streamed rows (P V, P^T dO, dS^T Q, dS K) need the
// streamed tile transposed; ds_read_b64_tr_b16 delivers that straight from the row-major
// tile: within each group of 16 lanes, lane i receives the four 16-bit elements that lanes
// i/4, i/4+4, i/4+8, i/4+12 address at element index i%4, i.e. a 4x16 block comes back as
// one column per lane.
//
// LDS tiles are dense [64 rows][D] bf16 with the 16-byte chunk index XOR-swizzled by the row
// so that both the row-wise 16-byte operand reads and the transposing 8-byte reads are free
// of bank conflicts without padding.
//
// SiLU, its derivative and the mask are evaluated in fp32 on the accumulator registers; P and
// dS are rounded to bf16 only as operands of the second product; alpha and 1/max_len are
// folded into one fp32 scale at the output, which is rounded to bf16 once.
#pragma once
#include <cstdlib>
#include <type_traits>

#include "hstu_common.h"

namespace hstu {

namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4;
typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;
typedef __attribute__((__vector_size__(4 * sizeof(short)))) short s16x4;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4;
typedef __attribute__((__vector_size__(2 * sizeof(uint32_t)))) uint32_t u32x2;

#define HSTU_LDS(T, p) ((__attribute__((address_space(3))) T*)(p))

constexpr int ST = 64;  // streamed rows per LDS tile

// Swizzle of the 16-byte chunk index by the row.  LDS has 64 banks of 4 bytes, i.e. 16 chunk
// positions per 256 bytes.  The position of (row, chunk) is its byte offset / 16 mod 16; the
// swizzle makes (a) 16 consecutive rows at one logical chunk (a row-wise operand read) and
// (b) 4 consecutive rows x 4 consecutive chunks (what 32 lanes of a transposing read touch)
// each land on 16 different positions, with no padding.  RB is the row length in bytes.
template <int RB>
__device__ __forceinline__ int swz_rb(int row) {
  if (RB == 256) return ((row & 3) << 2) | ((row >> 2) & 3);       // 1 row per 256 bytes
  if (RB == 128) return (((row >> 1) & 1) << 2) | ((row >> 2) & 3);  // 2 rows per 256 bytes
  return (row >> 2) & 3;                                           // 4 rows per 256 bytes
}
template <int D>
__device__ __forceinline__ int swz(int row) { return swz_rb<D * 2>(row); }

// Byte offset inside a tile with RB-byte rows of 16-byte chunk `chunk` of row `row`.
template <int RB>
__device__ __forceinline__ int lds_off_rb(int row, int chunk) {
  return row * RB + ((chunk ^ swz_rb<RB>(row)) << 4);
}
template <int D>
__device__ __forceinline__ int lds_off(int row, int chunk) { return lds_off_rb<D * 2>(row, chunk); }

// Per-lane byte offsets of operand reads inside a tile, computed once per kernel.  A row-wise
// operand is 8 consecutive elements of one row (one 16-byte chunk); a transposed operand for a
// 32x32x16 product gives lane (n, hh), for column col0 + n, the rows 4*hh + {0..3} and
// 8 + 4*hh + {0..3} of a 16-row group: exactly the streamed rows a lane's accumulator registers
// 8c..8c+7 belong to.  The swizzle
// depends on row mod 16 only, so a read of block blk (rows 32*blk + ...) is the same offset plus
// a constant, which the compiler folds into the instruction's immediate offset.
template <int D>
struct RowAddr {  // row-wise operand reads of row n (+32*blk): one address per 16-element step
  int a[D / 16];
  __device__ __forceinline__ void init(int n, int hh) {
#pragma unroll
    for (int ks = 0; ks < D / 16; ++ks) a[ks] = lds_off<D>(n, ks * 2 + hh);
  }
  __device__ __forceinline__ bf16x8 read(const char* tile, int blk, int ks) const {
    return *HSTU_LDS(bf16x8, tile + blk * 32 * D * 2 + a[ks]);
  }
};

template <int D>
struct ColAddr {  // transposing reads: per 32-column block, the lane's address in rows 0..7 and 8..15
  int a[D / 32][2];
  __device__ __forceinline__ void init(int lane) {
    const int i = lane & 15, g = lane >> 4;
    const int row = ((g >> 1) << 2) + (i >> 2);
#pragma unroll
    for (int c = 0; c < D / 32; ++c) {
      const int col = c * 32 + ((g & 1) << 4) + ((i & 3) << 2);
      a[c][0] = lds_off<D>(row, col >> 3) + ((col & 7) << 1);
      a[c][1] = lds_off<D>(row + 8, col >> 3) + ((col & 7) << 1);
    }
  }
  // operand for streamed rows 16*half16 .. 16*half16+15 of the tile (half16 = 2*blk + c), columns 32*cb ..
  __device__ __forceinline__ bf16x8 read(const char* tile, int half16, int cb) const {
    const char* base = tile + half16 * 16 * D * 2;
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(HSTU_LDS(s16x4, base + a[cb][0]));
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(HSTU_LDS(s16x4, base + a[cb][1]));
    typedef __attribute__((__vector_size__(8 * sizeof(short)))) short s16x8;
    const s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, both);
  }
};

// Transposed streamed tiles.  A transposed copy of a streamed tensor lives in the workspace as
// [H][D][columns], 64 columns (= 64 streamed rows) per tile, and inside every group of 16
// columns the rows are stored in the order 0-3, 8-11, 4-7, 12-15: exactly the order in which the
// accumulator registers of a 32x32 score block hold them, so that a plain 16-byte row read of
// the transposed tile is the operand of the second product (no transposing LDS reads needed).
// In LDS such a tile is [D rows][128 bytes], swizzled like any tile with 128-byte rows.
constexpr int TRB = ST * 2;  // bytes per row of a transposed tile

template <int D>
struct TrAddr {  // lane (n, hh): row n (+32*cb), chunk 2*half16 + hh for half16 = 0..3
  int a[4];
  __device__ __forceinline__ void init(int n, int hh) {
#pragma unroll
    for (int q = 0; q < 4; ++q) a[q] = lds_off_rb<TRB>(n, q * 2 + hh);
  }
  // operand for streamed rows 16*half16 .. +15 of the tile and output columns 32*cb .. +31
  __device__ __forceinline__ bf16x8 read(const char* tile, int half16, int cb) const {
    return *HSTU_LDS(bf16x8, tile + cb * 32 * TRB + a[half16]);
  }
};

// Asynchronous copy of one transposed tile: D rows of 128 bytes, row r at src + r * col_stride.
template <int D, int NW>
__device__ __forceinline__ void ttile_copy_async(char* tile, const __bf16* src, int64_t col_stride,
                                                 int wave, int lane) {
  constexpr int LOADS = D / 8;  // 8 rows of 128 bytes per wave-wide load
  const int rs = (int)col_stride * 2;
  const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
      (void*)src, 0, __builtin_amdgcn_readfirstlane((D - 1) * rs + TRB), 0x00020000);
#pragma unroll
  for (int i = 0; i < (LOADS + NW - 1) / NW; ++i) {
    const int idx = i * NW + wave;
    if (LOADS % NW != 0 && idx >= LOADS) break;
    const int row = idx * 8 + (lane >> 3);
    const int chunk = (lane & 7) ^ swz_rb<TRB>(row);
    __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, HSTU_LDS(void, tile + idx * 1024), 16,
                                             row * rs + chunk * 16, 0, 0, 0);
  }
}

// Asynchronous copy of one streamed tile (ST rows of one head) from global memory straight into
// its swizzled LDS layout: each wave-wide load moves 64 x 16 bytes into 1 KB of consecutive LDS
// (lane l lands at byte 16*l), so the lane that fills physical chunk pc of a row fetches the
// logical chunk pc ^ swz(row).  Rows >= valid are outside the buffer resource and arrive as
// zeros.  `tile` must be 1 KB aligned and uniform across the wave.
template <int D, int NW>
__device__ __forceinline__ void tile_copy_async(char* tile, const __bf16* base, int64_t row_stride,
                                                int valid, int wave, int lane) {
  constexpr int CPR = D / 8;            // 16-byte chunks per row
  constexpr int RPL = 64 / CPR;         // rows per wave-wide load
  constexpr int LOADS = ST / RPL;       // wave-wide loads per tile
  const int rs = (int)row_stride * 2;   // bytes
  const int rows = valid < 0 ? 0 : (valid < ST ? valid : ST);
  const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
      (void*)base, 0, __builtin_amdgcn_readfirstlane(rows * rs), 0x00020000);
#pragma unroll
  for (int i = 0; i < (LOADS + NW - 1) / NW; ++i) {
    const int idx = i * NW + wave;
    if (LOADS % NW != 0 && idx >= LOADS) break;
    const int row = idx * RPL + lane / CPR;
    const int chunk = (lane % CPR) ^ swz<D>(row);
    __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, HSTU_LDS(void, tile + idx * 1024), 16,
                                             row * rs + chunk * 16, 0, 0, 0);
  }
}

// Wave-wide loads that make up one row-major tile copy.
template <int D>
constexpr int tile_loads() { return ST / (64 / (D / 8)); }

// Waits until at most N of this wave's vector memory loads (tile copies included) are still in
// flight; loads complete in order, so the N newest may remain outstanding.
template <int N = 0>
__device__ __forceinline__ void tile_copy_wait() {
  static_assert(N >= 0 && N < 16, "vmcnt immediate");
  __builtin_amdgcn_s_waitcnt(0x0f70 | N);
}

// Workgroup barrier between tiles without the memory fence of __syncthreads(), which would wait
// for every outstanding load and with it for the tile copies that are meant to stay in flight.
// What has to be complete is waited for explicitly with tile_copy_wait<>() just before: a wave's
// own copies of the next tile (other waves see them after the barrier) - its LDS operand reads of
// the current tile have already been consumed by matrix instructions.  The empty asm statements
// keep the compiler from moving memory accesses across the barrier.
__device__ __forceinline__ void tile_barrier() {
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}

// (The owner rows are fetched with ordinary loads just before the first tile copies are issued,
// and nothing waits in between: the prologue's wait for the first tiles covers them, so a
// workgroup pays one memory round trip for both.)

// 32 owner rows of one head as B operands: lane (n, hh) holds row n, elements 16*s + 8*hh + e.
// base points at (row 0 of the owner tile, this head); rows >= nrows read as zero.
template <int D>
__device__ __forceinline__ void load_owner(bf16x8 (&reg)[D / 16], const __bf16* base,
                                           int64_t row_stride, int row, int nrows, int hh) {
  const int rs = (int)row_stride * 2;
  const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
      (void*)base, 0, __builtin_amdgcn_readfirstlane(nrows * rs), 0x00020000);
#pragma unroll
  for (int s = 0; s < D / 16; ++s) {
    const u32x4 z = __builtin_amdgcn_raw_buffer_load_b128(rsrc, row * rs + s * 32 + hh * 16, 0, 0);
    reg[s] = __builtin_bit_cast(bf16x8, z);
  }
}

__device__ __forceinline__ f32x16 mfma(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// sigmoid(alpha * s) with c1 = -alpha * log2(e).  exp2 overflow gives rcp(inf) = 0.
__device__ __forceinline__ float sigmoid_scaled(float s, float c1) {
  return __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(s * c1));
}

__device__ __forceinline__ bf16x8 pack8(const float* x) {
  bf16x8 r;
#pragma unroll
  for (int e = 0; e < 8; ++e) r[e] = (__bf16)x[e];
  return r;
}

// Streamed rows of a segment that matter to an owner tile, as [beg, end) in segment rows.
// side 0 (owners are queries): keys at positions <= the tile's last position.
// side 1 (owners are keys): queries at positions >= the tile's first position.
template <int SIDE>
__device__ __forceinline__ void visible_range(const Item& it, int g, int causal, int& beg, int& end) {
  beg = 0;
  end = it.seg_len[g];
  if (causal) {
    if (SIDE == 0) {
      const int e = it.pos0 + it.nrows - it.seg_pos0[g];
      end = e < 0 ? 0 : (e < end ? e : end);
    } else {
      const int b = it.pos0 - it.seg_pos0[g];
      beg = b < 0 ? 0 : (b < end ? b : end);
      beg &= ~(ST - 1);
    }
  }
}

// The streamed tiles of an item, flattened over its segments.
struct Stream {
  int n[2];    // tiles per segment
  int beg[2];  // first streamed row (segment-relative) of tile 0
  int end[2];  // end of the visible range (segment-relative)
  int total;
};

template <int SIDE>
__device__ __forceinline__ Stream make_stream(const Item& it, int causal) {
  Stream s;
#pragma unroll
  for (int g = 0; g < 2; ++g) {
    s.n[g] = 0; s.beg[g] = 0; s.end[g] = 0;
    if (g < it.nseg) {
      visible_range<SIDE>(it, g, causal, s.beg[g], s.end[g]);
      s.n[g] = (s.end[g] - s.beg[g] + ST - 1) / ST;
    }
  }
  s.total = s.n[0] + s.n[1];
  return s;
}

// Tile j of the stream: segment, first segment-relative row, valid rows, first position.
struct TileRef { int row; int valid; int pos; int tcol; };

__device__ __forceinline__ TileRef tile_ref(const Item& it, const Stream& s, int j) {
  const int g = j < s.n[0] ? 0 : 1;
  const int t = g ? j - s.n[0] : j;
  const int rel = s.beg[g] + t * ST;
  TileRef r;
  r.row = it.seg_row0[g] + rel;
  r.valid = s.end[g] - rel;  // may exceed ST; callers clamp by ST through the loader
  r.pos = it.seg_pos0[g] + rel;
  r.tcol = it.seg_tcol0[g] + rel;  // a multiple of 64: streams start on tile boundaries
  return r;
}

// Epilogue for accumulators held "owner row per lane": blk[c][r] is element
// c*32 + 8*(r/4) + 4*hh + r%4 of the lane's row.  `elem` is the element offset of the row start.
// Lanes n and n + 32 hold the same row (hh = 0, 1) and must both be active.
template <int D>
__device__ __forceinline__ void store_owner_major(void* out, int64_t elem, const f32x16 (&acc)[D / 32],
                                                  float scale, int hh, int accumulate, int out_f32) {
  if (!out_f32 && !accumulate) {
    // Plain bf16 output.  The two lanes of a row hold alternating runs of four elements; after one
    // exchange between the wave's halves per register (the upper half of the first operand against
    // the lower half of the second) the lower lane holds elements 0..7 of a run of sixteen and the
    // upper lane elements 8..15, so a store is 16 bytes per lane and 32 contiguous bytes per row.
    // (A store instruction touches the cache lines of 32 rows whatever it writes to each: half as
    // many instructions take half as long, 3 us of a short item's 15 before.)
#pragma unroll
    for (int c = 0; c < D / 32; ++c)
#pragma unroll
      for (int pr = 0; pr < 2; ++pr) {
        uint32_t w[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          bf16x2 t;
          t[0] = (__bf16)(acc[c][8 * pr + 2 * e] * scale);
          t[1] = (__bf16)(acc[c][8 * pr + 2 * e + 1] * scale);
          w[e] = __builtin_bit_cast(uint32_t, t);
        }
        // w[0..1]: run 2*pr, w[2..3]: run 2*pr + 1 of this lane's half
        const auto s0 = __builtin_amdgcn_permlane32_swap(w[0], w[2], false, false);
        const auto s1 = __builtin_amdgcn_permlane32_swap(w[1], w[3], false, false);
        u32x4 v;
        v[0] = s0[0]; v[1] = s1[0]; v[2] = s0[1]; v[3] = s1[1];
        *(u32x4*)((__bf16*)out + elem + c * 32 + 16 * pr + 8 * hh) = v;
      }
    return;
  }
#pragma unroll
  for (int c = 0; c < D / 32; ++c)
#pragma unroll
    for (int q4 = 0; q4 < 4; ++q4) {
      const int64_t e0 = elem + c * 32 + 8 * q4 + 4 * hh;
      float x[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) x[e] = acc[c][4 * q4 + e] * scale;
      if (out_f32) {
        float4* dst = (float4*)((float*)out + e0);
        if (accumulate) {
          const float4 old = *dst;
          x[0] += old.x; x[1] += old.y; x[2] += old.z; x[3] += old.w;
        }
        *dst = make_float4(x[0], x[1], x[2], x[3]);
      } else {
        bf16x4* dst = (bf16x4*)((__bf16*)out + e0);
        if (accumulate) {
          const bf16x4 old = *dst;
#pragma unroll
          for (int e = 0; e < 4; ++e) x[e] += (float)old[e];
        }
        bf16x4 o4;
#pragma unroll
        for (int e = 0; e < 4; ++e) o4[e] = (__bf16)x[e];
        *dst = o4;
      }
    }
}

// One element of an output tensor, either dtype, optionally added to what is there.
__device__ __forceinline__ void store_one(void* out, int64_t elem, float x, int accumulate, int out_f32) {
  if (out_f32) {
    float* d = (float*)out + elem;
    *d = accumulate ? *d + x : x;
  } else {
    __bf16* d = (__bf16*)out + elem;
    *d = (__bf16)(accumulate ? (float)*d + x : x);
  }
}

// Which (item of the schedule, head) a workgroup-sized unit of work is (see AttnArgs::xcd_parts).
// on == false: none (the grid is sized from bounds).
struct Unit { int slot, h; bool on; };
__device__ __forceinline__ Unit unit_of(const AttnArgs& a, int u) {
  const int H = a.num_heads;
  Unit r;
  if (a.xcd_parts <= 1) {
    r.slot = u / H; r.h = u % H; r.on = true;  // (the item fetch checks the slot)
    return r;
  }
  const int n = a.plan.header[0];
  const int per = (n + a.xcd_parts - 1) / a.xcd_parts;
  const int x = u & 7, j = u >> 3;
  r.h = x % H;
  r.slot = (x / H) * per + j;
  r.on = j < per && r.slot < n;
  return r;
}
// Units the (item, head) pairs of a schedule of n items are spread over.
__device__ __forceinline__ int unit_count(const AttnArgs& a, int n) {
  return a.xcd_parts <= 1 ? n * a.num_heads : 8 * ((n + a.xcd_parts - 1) / a.xcd_parts);
}

// An item as it lies in memory, loaded by every lane alike (what a workgroup that walks over items
// fetches ahead of time) ...
struct RawItem { u32x4 w[4]; };
__device__ __forceinline__ RawItem load_raw_item(const Item* src) {
  RawItem r;
#pragma unroll
  for (int i = 0; i < 4; ++i) r.w[i] = ((const u32x4*)src)[i];
  return r;
}
// ... and brought into scalar registers when its turn comes.  False: no owner rows.
__device__ __forceinline__ bool decode_item(const RawItem& r, Item& it) {
  auto word = [&](int i) { return (int)__builtin_amdgcn_readfirstlane(r.w[i >> 2][i & 3]); };
  it.row0 = word(0); it.nrows = word(1); it.pos0 = word(2); it.nseg = word(3);
#pragma unroll
  for (int g = 0; g < 2; ++g) {
    it.seg_row0[g] = word(4 + g); it.seg_len[g] = word(6 + g);
    it.seg_pos0[g] = word(8 + g); it.seg_tcol0[g] = word(10 + g);
  }
  it.cost = 0;
  it.part = word(13);
  return it.nrows > 0;
}

// DIRECT: the items are in schedule order already (packed tiles), no indirection.
template <bool DIRECT = false>
__device__ __forceinline__ bool fetch_item(const Plan& plan, int slot, Item& it) {
  if (slot >= plan.header[0]) return false;
  const Item* src = plan.items + (DIRECT ? slot : plan.order[slot]);
  // The item is the same for every lane: keep it in scalar registers so that everything derived
  // from it (addresses, buffer resources, loop bounds) is uniform.
  it.row0 = __builtin_amdgcn_readfirstlane(src->row0);
  it.nrows = __builtin_amdgcn_readfirstlane(src->nrows);
  it.pos0 = __builtin_amdgcn_readfirstlane(src->pos0);
  it.nseg = __builtin_amdgcn_readfirstlane(src->nseg);
#pragma unroll
  for (int g = 0; g < 2; ++g) {
    it.seg_row0[g] = __builtin_amdgcn_readfirstlane(src->seg_row0[g]);
    it.seg_len[g] = __builtin_amdgcn_readfirstlane(src->seg_len[g]);
    it.seg_pos0[g] = __builtin_amdgcn_readfirstlane(src->seg_pos0[g]);
    it.seg_tcol0[g] = __builtin_amdgcn_readfirstlane(src->seg_tcol0[g]);
  }
  it.cost = 0;
  it.part = __builtin_amdgcn_readfirstlane(src->part);
  return it.nrows > 0;
}

// =============================================================================================
// Which streamed rows of a 32-row block the lane's owner row sees; r is the accumulator element,
// i.e. streamed row 8*(r/4) + 4*hh + r%4 of the block.
// =============================================================================================
struct VisBefore {  // owners are queries, causal: keys at or before the query; rel = query - block position
  int rel, hh;
  __device__ __forceinline__ bool operator()(int r) const { return 8 * (r >> 2) + 4 * hh + (r & 3) <= rel; }
};
struct VisAfter {   // owners are keys, causal: queries at or after the key; rel = key - block position
  int rel, hh;
  __device__ __forceinline__ bool operator()(int r) const { return rel <= 8 * (r >> 2) + 4 * hh + (r & 3); }
};
struct VisWindow {  // packed tiles: positions [lo, lo + span]; base = block position - lo
  int base;
  uint32_t span;
  int hh;
  __device__ __forceinline__ bool operator()(int r) const {
    return (uint32_t)(base + 8 * (r >> 2) + 4 * hh + (r & 3)) <= span;
  }
};

// Packed tiles (batches of short sequences): an owner tile is 128 consecutive rows of the batch
// whatever sequences they belong to, the streamed rows run from the start of the first of those
// sequences to the end of the last, positions are row numbers, and every owner row sees the
// window of rows [lo, lo + span] of its own sequence (cut at the row itself when causal).
struct Window {
  int lo;
  uint32_t span;
  int lo_min, lo_max, hi_min, hi_max;  // over the wave's valid rows (uniform)
  // some row of the block at position b may be hidden from some owner row of the wave
  __device__ __forceinline__ bool masks(int b) const { return b < lo_max || b + 31 > hi_min; }
  __device__ __forceinline__ VisWindow vis(int b, int hh) const { return VisWindow{b - lo, span, hh}; }
};

__device__ __forceinline__ int wave_min(int x);
__device__ __forceinline__ int wave_max(int x);

// side 0: owners are queries, 1: owners are keys.  row_seq[row] = {first row, end row} of the
// row's sequence.  Lanes without a valid owner row get an empty window.
// The bounds are loaded on their own (window_bounds) so that a kernel can request them first of
// all and look at them only after it has issued its first tile copies: one memory round trip for
// both instead of two in a row.
__device__ __forceinline__ int2 window_bounds(const int2* row_seq, int row, bool valid) {
  return valid ? row_seq[row] : make_int2(0, 0);
}
__device__ __forceinline__ Window make_window(const int2& sq, int row, bool valid, int side, int causal) {
  Window w;
  int hi = -1;
  w.lo = 0x3fffffff;
  w.span = 0;
  if (valid) {
    w.lo = (causal && side == 1) ? row : sq.x;
    hi = (causal && side == 0) ? row : sq.y - 1;
    w.span = (uint32_t)(hi - w.lo);
  }
  w.lo_min = wave_min(w.lo);
  w.lo_max = wave_max(valid ? w.lo : (int)0x80000000);
  w.hi_min = wave_min(valid ? hi : 0x7fffffff);
  w.hi_max = wave_max(valid ? hi : (int)0x80000000);
  return w;
}

// =============================================================================================
// Timestamp bias.  Paper, section 2.1: the scores get "+ Bias" inside the SiLU, the bias being a
// learnable table indexed by a bucket of the difference of two rows' timestamps; the bucket
// function (a logarithm with 2^f groups per octave, in integers) is this library's reading:
//   delta = |ts_i - ts_j|;  bucket = 0 if delta <= 1, else min(nb - 1, e * 2^f + m) with
//   e = floor(log2 delta) and m the f bits below delta's leading one.
// The bias of a 32x32 block of pairs is written into the accumulator of the score product before
// its first matrix instruction, so that the elementwise code sees scores that already contain it
// (x = alpha * (q.k + w) in the forward pass and in both backward passes alike).
// The bucket grows with delta, so when the smallest and the largest difference a block can contain
// (from the ranges of the two sides' timestamps) fall into one bucket, the whole block takes that
// one table entry; otherwise every lane works out the buckets of its 16 pairs.  Which case a
// block is, and the table entry of the first case, is worked out for 64 blocks of the stream at a
// time, one block per lane (BlockTable), so that a block of the first case costs two cross-lane
// reads when its turn comes.  (Measured alternatives: the range through an LDS read and the two
// buckets in scalar arithmetic per block, or through scalar loads issued a tile ahead, cost 7 to
// 13 % of a pass even when every block is of the first case.)
// =============================================================================================

constexpr int REC_TILE = ST * (int)sizeof(TsRecord);  // bytes of the records of one streamed tile

// Asynchronous copy of the records of one streamed tile (one wave-wide load; rows >= valid
// arrive as zeros).  Called by one wave.
__device__ __forceinline__ void rec_copy_async(char* tile, const TsRecord* rec, int valid, int lane) {
  const int rows = valid < 0 ? 0 : (valid < ST ? valid : ST);
  const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
      (void*)rec, 0, __builtin_amdgcn_readfirstlane(rows * (int)sizeof(TsRecord)), 0x00020000);
  __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, HSTU_LDS(void, tile), 16, lane * 16, 0, 0, 0);
}

__device__ __forceinline__ int wave_min(int x) {
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) { const int y = __shfl_xor(x, m); x = y < x ? y : x; }
  return __builtin_amdgcn_readfirstlane(x);
}
__device__ __forceinline__ int wave_max(int x) {
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) { const int y = __shfl_xor(x, m); x = y > x ? y : x; }
  return __builtin_amdgcn_readfirstlane(x);
}
__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) x += __shfl_xor(x, m);
  return x;
}

// What a wave knows about the bias: its own rows' timestamps and the table.
struct BiasCtx {
  const float* wtab;     // LDS copy of the table
  const TsRecord* rec;   // the records of all rows, padded by 64
  bf16x8 ones;           // A operand with 1.0 in the first two slots of every row (see bias_block)
  int t_own;             // timestamp of the lane's owner row
  int o_lo, o_hi;        // range of the timestamps of the wave's valid owner rows (uniform)
  int nb, f, hh;
  int per_pair;          // every block works out its pairs' buckets one by one (AttnArgs::bias_per_pair)
};

// The uniform part of a block's bias: whether all its pairs fall into one bucket, that bucket
// (else the bucket of the smallest difference) and its table entry.
struct BlockBias {
  int b0;
  bool uni;
  bool small;      // every difference of the block is below BIAS_SMALL_DELTA
  uint32_t wpair;  // the table entry as two bf16 halves, high part in the low 16 bits (see bias_block)
};

// BlockBias of the stream's blocks, one block per lane: blocks [128k, 128k + 64) in set 0,
// [128k + 64, 128k + 128) in set 1; a set is refilled when the stream enters the other one.
struct BlockTable {
  int code0, code1;  // bucket | NONUNIFORM | SMALL
  float w0, w1;
  static constexpr int NONUNIFORM = 1 << 30, SMALL = 1 << 29;

  // Fills the set of blocks [first, first + 64), first a multiple of 64; blocks >= nblocks (past
  // the end of the stream: their scores are computed and discarded) get a zero bias.
  __device__ __forceinline__ void fill(const BiasCtx& c, int first, int nblocks, const Item& it,
                                       const Stream& st, int lane) {
    const int i = first + lane;
    int code = 0;
    float w = 0.f;
    if (i < nblocks) {
      const int t = i >> 1;
      const bool g = t >= st.n[0];
      const int rel = (g ? st.beg[1] + (t - st.n[0]) * ST : st.beg[0] + t * ST) + (i & 1) * 32;
      const int row = (g ? it.seg_row0[1] : it.seg_row0[0]) + rel;  // inside the padded table
      const u32x2 head = *(const u32x2*)&c.rec[row].lo;
      const int s_lo = (int)head[0], s_hi = (int)head[1];
      // differences of int32 values as uint32 (exact up to 2^32 - 1); of d1, d2 one is not negative
      const uint32_t d1 = c.o_hi >= s_lo ? (uint32_t)c.o_hi - (uint32_t)s_lo : 0u;
      const uint32_t d2 = s_hi >= c.o_lo ? (uint32_t)s_hi - (uint32_t)c.o_lo : 0u;
      const uint32_t dmax = d1 > d2 ? d1 : d2;
      const uint32_t dmin = c.o_lo > s_hi ? (uint32_t)c.o_lo - (uint32_t)s_hi
                                          : (s_lo > c.o_hi ? (uint32_t)s_lo - (uint32_t)c.o_hi : 0u);
      const int b0 = bias_bucket(dmin, c.nb, c.f), b1 = bias_bucket(dmax, c.nb, c.f);
      code = b0 | (b0 != b1 || c.per_pair ? NONUNIFORM : 0) | (dmax < BIAS_SMALL_DELTA ? SMALL : 0);
      // the entry as hi + lo, both bf16: exact to 2^-16 of its value
      const float wv = *HSTU_LDS(float, c.wtab + b0);
      const __bf16 hi = (__bf16)wv;
      const __bf16 lo = (__bf16)(wv - (float)hi);
      w = __builtin_bit_cast(float, (uint32_t)__builtin_bit_cast(uint16_t, hi) |
                                        ((uint32_t)__builtin_bit_cast(uint16_t, lo) << 16));
    }
    const bool odd = (first >> 6) & 1;
    code0 = odd ? code0 : code; w0 = odd ? w0 : w;
    code1 = odd ? code : code1; w1 = odd ? w : w1;
  }

  // Block i (uniform), which must be in one of the two sets filled last.
  __device__ __forceinline__ BlockBias get(int i) const {
    const int l = i & 63;
    const bool odd = (i >> 6) & 1;
    const int c0 = __builtin_amdgcn_readlane(code0, l), c1 = __builtin_amdgcn_readlane(code1, l);
    const int x0 = __builtin_amdgcn_readlane(__builtin_bit_cast(int, w0), l);
    const int x1 = __builtin_amdgcn_readlane(__builtin_bit_cast(int, w1), l);
    const int c = odd ? c1 : c0;
    BlockBias b;
    b.b0 = c & (SMALL - 1);
    b.uni = (c & NONUNIFORM) == 0;
    b.small = (c & SMALL) != 0;
    b.wpair = (uint32_t)(odd ? x1 : x0);
    return b;
  }
};

// Bias of block blk of a streamed tile whose records are at trec (LDS): s[r] = w[bucket of the
// pair (lane's owner row, streamed row 8*(r/4) + 4*hh + r%4 of the block)].  bb: the uniform
// part; bk: the buckets of the lane's pairs when the block spans several.
__device__ __forceinline__ void bias_block(f32x16& s, const char* trec, int blk, const BiasCtx& c,
                                           const BlockBias& bb, int (&bk)[16]) {
  if (bb.uni) {
    // One matrix instruction writes the entry into all 32x32 accumulator elements: every row of A has
    // ones in its first two slots, every column of B the entry's two bf16 halves there, so that
    // D = 1*hi + 1*lo.  (Sixteen register moves cost the vector pipe four times what this costs
    // the matrix pipe, and the vector pipe is the fuller one.)  bk stays unset: only blocks of
    // several buckets use it.
    const u32x4 bq = {c.hh == 0 ? bb.wpair : 0u, 0u, 0u, 0u};
    const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    s = mfma(c.ones, __builtin_bit_cast(bf16x8, bq), zero);
  } else if (bb.small) {  // (the common case: a third of the instructions of the general one)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int row = blk * 32 + 8 * (r >> 2) + 4 * c.hh + (r & 3);
      const int t = *HSTU_LDS(int, trec + row * (int)sizeof(TsRecord));
      bk[r] = bias_bucket_small(abs_diff(c.t_own, t), c.nb, c.f);
      s[r] = *HSTU_LDS(float, c.wtab + bk[r]);
    }
  } else {
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int row = blk * 32 + 8 * (r >> 2) + 4 * c.hh + (r & 3);
      const int t = *HSTU_LDS(int, trec + row * (int)sizeof(TsRecord));
      bk[r] = bias_bucket(abs_diff(c.t_own, t), c.nb, c.f);
      s[r] = *HSTU_LDS(float, c.wtab + bk[r]);
    }
  }
}

// Initial value of a score accumulator: zero, or the bias of the block.
template <bool BIAS>
struct ScoreInit {
  const BiasCtx* c;
  const char* trec;
  int blk;
  BlockBias bb;
  __device__ __forceinline__ void operator()(f32x16& s) const {
    if constexpr (BIAS) {
      int bk[16];
      bias_block(s, trec, blk, *c, bb, bk);
    } else {
#pragma unroll
      for (int r = 0; r < 16; ++r) s[r] = 0.f;
    }
  }
};

// Loads the table into LDS and works out the wave's owner-side context.  All threads of the
// workgroup call it (it contains a barrier).
template <int NT>
__device__ __forceinline__ BiasCtx bias_setup(const AttnArgs& a, float* wtab, const Item& it, int orow,
                                              int tid, int hh) {
  for (int i = tid; i < a.nb; i += NT) wtab[i] = a.ts_w[i];
  BiasCtx c;
  c.wtab = wtab;
  c.rec = a.ts_rec;
  c.nb = a.nb; c.f = a.fbits; c.hh = hh;
  c.per_pair = a.bias_per_pair;
  {
    const u32x4 o = {hh == 0 ? 0x3f803f80u : 0u, 0u, 0u, 0u};
    c.ones = __builtin_bit_cast(bf16x8, o);
  }
  const bool ok = orow < it.nrows;
  c.t_own = ok ? a.ts_rec_own[it.row0 + orow].ts : 0;
  c.o_lo = wave_min(ok ? c.t_own : 0x7fffffff);
  c.o_hi = wave_max(ok ? c.t_own : (int)0x80000000);
  __syncthreads();
  return c;
}

// p' = s*sg (p = alpha*p'/N);  silu'(alpha*s) = sg + alpha*p'*(1-sg);  ds' = dp*silu' (ds = ds'/N)
__device__ __forceinline__ void bwd_elem(float s, float dp, float c1, float alpha, float& p, float& ds) {
  const float sg = sigmoid_scaled(s, c1);
  p = s * sg;
  ds = dp * __builtin_fmaf(alpha, __builtin_fmaf(-p, sg, p), sg);
}

// CAP > 0: at most that many workgroups (for kernels that walk over the (item, head) pairs).
#define HSTU_DISPATCH_D(KERNEL, NW, ...) HSTU_DISPATCH_G(0, KERNEL, NW, __VA_ARGS__)
#define HSTU_DISPATCH_G(CAP, KERNEL, NW, ...)                                           \
  do {                                                                                  \
    const int64_t units_ = a.xcd_parts <= 1 ? (int64_t)a.max_items * a.num_heads        \
                               : 8 * (((int64_t)a.max_items + a.xcd_parts - 1) / a.xcd_parts); \
    const int64_t cap_ = (CAP);                                                         \
    const dim3 grid((unsigned)(cap_ > 0 && units_ > cap_ ? cap_ : units_)), block(NW * 64); \
    if (d_qk == 128 && d_v == 128) hipLaunchKernelGGL((KERNEL<128, 128, __VA_ARGS__>), grid, block, 0, stream, a); \
    else if (d_qk == 64 && d_v == 64) hipLaunchKernelGGL((KERNEL<64, 64, __VA_ARGS__>), grid, block, 0, stream, a); \
    else if (d_qk == 32 && d_v == 32) hipLaunchKernelGGL((KERNEL<32, 32, __VA_ARGS__>), grid, block, 0, stream, a); \
    else if (d_qk == 128 && d_v == 64) hipLaunchKernelGGL((KERNEL<128, 64, __VA_ARGS__>), grid, block, 0, stream, a); \
    else if (d_qk == 64 && d_v == 128) hipLaunchKernelGGL((KERNEL<64, 128, __VA_ARGS__>), grid, block, 0, stream, a); \
    else if (d_qk == 128 && d_v == 32) hipLaunchKernelGGL((KERNEL<128, 32, __VA_ARGS__>), grid, block, 0, stream, a); \
    else if (d_qk == 32 && d_v == 128) hipLaunchKernelGGL((KERNEL<32, 128, __VA_ARGS__>), grid, block, 0, stream, a); \
    else if (d_qk == 64 && d_v == 32) hipLaunchKernelGGL((KERNEL<64, 32, __VA_ARGS__>), grid, block, 0, stream, a); \
    else if (d_qk == 32 && d_v == 64) hipLaunchKernelGGL((KERNEL<32, 64, __VA_ARGS__>), grid, block, 0, stream, a); \
    else return hipErrorInvalidValue;                                                   \
    return hipGetLastError();                                                           \
  } while (0)

// The kernels with the timestamp bias: the same dispatch after a check of the bias arguments.
#define HSTU_DISPATCH_BIAS(KERNEL, NW, ...)                                             \
  do {                                                                                  \
    if (a.nb < 1 || a.nb > MAX_TS_BUCKETS || !a.ts_w || !a.ts_rec_own) return hipErrorInvalidValue; \
    HSTU_DISPATCH_D(KERNEL, NW, __VA_ARGS__);                                           \
  } while (0)

}  // namespace

}  // namespace hstu
