// bf16 jagged HSTU attention on the gfx950 matrix cores: forward, dk/dv pass, dq pass.
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
#include <cstdlib>
#include <type_traits>

#include "hstu_common.h"

namespace hstu {

namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4;
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
template <int D>
__device__ __forceinline__ void store_owner_major(void* out, int64_t elem, const f32x16 (&acc)[D / 32],
                                                  float scale, int hh, int accumulate, int out_f32) {
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

__device__ __forceinline__ bool fetch_item(const Plan& plan, int slot, Item& it) {
  if (slot >= plan.header[0]) return false;
  const Item* src = plan.items + plan.order[slot];
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
__device__ __forceinline__ Window make_window(const int2* row_seq, int row, bool valid, int side, int causal) {
  Window w;
  int hi = -1;
  w.lo = 0x3fffffff;
  w.span = 0;
  if (valid) {
    const int2 sq = row_seq[row];
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

__device__ __forceinline__ int bias_bucket(uint32_t delta, int nb, int f) {
  const uint32_t d = delta > 2u ? delta : 2u;  // (no branch: the result for delta <= 1 is selected below)
  const int e = 31 - __builtin_clz(d);
  const uint32_t top = e >= f ? d >> (e - f) : d << (f - e);
  int b = (e << f) + (int)top - (1 << f);
  b = b < nb - 1 ? b : nb - 1;
  return delta <= 1u ? 0 : b;
}

__device__ __forceinline__ uint32_t abs_diff(int a, int b) {
  return a > b ? (uint32_t)a - (uint32_t)b : (uint32_t)b - (uint32_t)a;
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
  int t_own;             // timestamp of the lane's owner row
  int o_lo, o_hi;        // range of the timestamps of the wave's valid owner rows (uniform)
  int nb, f, hh;
};

// The uniform part of a block's bias: whether all its pairs fall into one bucket, that bucket
// (else the bucket of the smallest difference) and its table entry.
struct BlockBias {
  int b0;
  bool uni;
  float wb;
};

// BlockBias of the stream's blocks, one block per lane: blocks [128k, 128k + 64) in set 0,
// [128k + 64, 128k + 128) in set 1; a set is refilled when the stream enters the other one.
struct BlockTable {
  int code0, code1;  // bucket | NONUNIFORM
  float w0, w1;
  static constexpr int NONUNIFORM = 1 << 30;

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
      code = b0 | (b0 != b1 ? NONUNIFORM : 0);
      w = *HSTU_LDS(float, c.wtab + b0);
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
    b.b0 = c & (NONUNIFORM - 1);
    b.uni = (c & NONUNIFORM) == 0;
    b.wb = __builtin_bit_cast(float, odd ? x1 : x0);
    return b;
  }
};

// Bias of block blk of a streamed tile whose records are at trec (LDS): s[r] = w[bucket of the
// pair (lane's owner row, streamed row 8*(r/4) + 4*hh + r%4 of the block)].  bb: the uniform
// part; bk: the buckets of the lane's pairs when the block spans several.
__device__ __forceinline__ void bias_block(f32x16& s, const char* trec, int blk, const BiasCtx& c,
                                           const BlockBias& bb, int (&bk)[16]) {
  if (bb.uni) {
#pragma unroll
    for (int r = 0; r < 16; ++r) { s[r] = bb.wb; bk[r] = bb.b0; }
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
  const bool ok = orow < it.nrows;
  c.t_own = ok ? a.ts_rec_own[it.row0 + orow].ts : 0;
  c.o_lo = wave_min(ok ? c.t_own : 0x7fffffff);
  c.o_hi = wave_max(ok ? c.t_own : (int)0x80000000);
  __syncthreads();
  return c;
}

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
                                         bool mask, const Vis& vis) {
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
  static_assert(!(PACKED && (VT || BIAS)), "packed tiles: row-major V tiles, no bias");
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
  const int slot = blockIdx.x / H, h = blockIdx.x % H;
  Item it;
  if (!fetch_item(a.plan, slot, it)) return;

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
  Window win = {};
  if constexpr (PACKED) win = make_window(a.row_seq, it.row0 + orow, orow < it.nrows, 0, a.causal);
  // Does any key of block i precede (or equal) a query of this wave?  Once false it stays false.
  // (Packed tiles: the few blocks of a tile's stream all run; the windows do the rest.)
  auto block_on = [&](int i) {
    return wave_on && i < NB && (PACKED || !a.causal || block_pos(i) <= q_hi);
  };

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
      return PACKED ? win.masks(block_pos(i)) : (a.causal && block_pos(i) + 31 > q_lo);
    };
    auto vis_of = [&](int i) {
      if constexpr (PACKED) return win.vis(block_pos(i), hh);
      else return VisBefore{q_lo + n - block_pos(i), hh};
    };
    BlockTable tab = {};
    if constexpr (BIAS) {
      tab.fill(bias, 0, NB, it, st, lane);
      tab.fill(bias, 64, NB, it, st, lane);
    }
    auto bb_of = [&](int i) { return BIAS ? tab.get(i) : BlockBias{}; };

    // S of block 0 on its own, then step 0 (nothing to multiply by V yet)
    if (block_on(0)) {
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
        if (block_on(i - 1))
          fwd_step<DQK, DV, true>(init_of(tbuf(B1), 0, bb_of(i + 1)), kbuf(B1), 0, vbuf(B0), 0, ra, ca, qreg, sacc[1],
                                  sacc[0], pb[0], pb[1], oacc, c1, mask_of(i), vis_of(i));
      }
      if (j + 1 < T) {
        const int i = 2 * j + 2;  // S of (tile j+1, block 1), P V of (tile j, block 1)
        if (block_on(i - 1))
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
// dk/dv pass: owners are key rows (K and V rows in registers), Q and dO are streamed.
//   S  = Q K^T   (A = Q tile rows,  B = K registers)   lane: key n, query rows in registers
//   dP = dO V^T  (A = dO tile rows, B = V registers)
//   dV += P^T dO   (A = P registers,  B = dO tile transposed read)
//   dK += dS^T Q   (A = dS registers, B = Q tile transposed read)
// Each key tile belongs to exactly one workgroup, so dk and dv need no atomics.
// =============================================================================================

// p' = s*sg (p = alpha*p'/N);  silu'(alpha*s) = sg + alpha*p'*(1-sg);  ds' = dp*silu' (ds = ds'/N)
__device__ __forceinline__ void bwd_elem(float s, float dp, float c1, float alpha, float& p, float& ds) {
  const float sg = sigmoid_scaled(s, c1);
  p = s * sg;
  ds = dp * (sg + alpha * p * (1.0f - sg));
}

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
                                          float c1, float alpha, bool mask, const Vis& vis) {
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
#pragma unroll
  for (int m = 0; m < NS; ++m) {
    if (m < KS) s_out = mfma(op[m], kreg[m], s_out);
    else d_out = mfma(op[m], vreg[m - KS], d_out);
    if (CONTR) {
      if (m < VS) dvacc[m >> 1] = mfma(pd_prev[m & 1], tp[m], dvacc[m >> 1]);
      else dkacc[(m - VS) >> 1] = mfma(pd_prev[2 + ((m - VS) & 1)], tp[m], dkacc[(m - VS) >> 1]);
    }
    if (m + AHEAD < NS) {
      op[m + AHEAD] = read_rows(m + AHEAD);
      if (CONTR) tp[m + AHEAD] = read_cols(m + AHEAD);
    }
#pragma unroll
    for (int e = m * 16 / NS; e < (m + 1) * 16 / NS; ++e) bwd_elem(s_in[e], d_in[e], c1, alpha, p[e], ds[e]);
    if (m % GRP == GRP - 1) fence();
  }
  if (mask) {
    asm volatile("" ::: "memory");  // not speculable: keeps the selects off the unmasked path
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
template <int DQK, int DV, int NW, bool BIAS, bool PACKED>
__global__ void __launch_bounds__(NW * 64, (DQK + DV <= 128 ? 2 : 1)) hstu_dkdv_bf16(AttnArgs a) {
  static_assert(!(PACKED && BIAS), "packed tiles: no bias");
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
  const int slot = blockIdx.x / H, h = blockIdx.x % H;
  Item it;
  if (!fetch_item(a.plan, slot, it)) return;

  const int tid = threadIdx.x, lane = tid & 63, n = lane & 31, hh = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int64_t sq = (int64_t)H * DQK, sv = (int64_t)H * DV;
  const __bf16* qg = (const __bf16*)a.q + h * DQK;
  const __bf16* gg = (const __bf16*)a.d_o + h * DV;
  const __bf16* kg = (const __bf16*)a.k + (int64_t)it.row0 * sq + h * DQK;
  const __bf16* vg = (const __bf16*)a.v + (int64_t)it.row0 * sv + h * DV;

  const int orow = wave * 32 + n;
  const bool wave_on = wave * 32 < it.nrows;
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
  Window win = {};
  if constexpr (PACKED) win = make_window(a.row_seq, it.row0 + orow, orow < it.nrows, 1, a.causal);
  // Does any query of block i see a key of this wave?  Once true it stays true.
  // (Packed tiles: the few blocks of a tile's stream all run; the windows do the rest.)
  auto block_on = [&](int i) { return wave_on && (PACKED || !a.causal || block_pos(i) + 31 >= k_lo); };
  auto mask_of = [&](int pos) { return PACKED ? win.masks(pos) : (a.causal && pos < k_hi); };
  auto vis_of = [&](int pos) {
    if constexpr (PACKED) return win.vis(pos, hh);
    else return VisAfter{k_lo + n - pos, hh};
  };

  if (T > 0) copy_tile(0, 0);
  if (T > 1) copy_tile(1, 1);
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
    const int pos = block_pos(0);
    dkdv_step<DQK, DV, false>(init_of(tbuf(0), 1, bb_of(1)), qbuf(0), gbuf(0), 1, qbuf(0), gbuf(0), 0, raq, rag,
                              caq, cag, kreg, vreg, sacc[0], dacc[0], sacc[1], dacc[1], pd[1], pd[0],
                              dkacc, dvacc, c1, a.alpha, mask_of(pos), vis_of(pos));
  }

  // Iteration j: steps 2j+1 and 2j+2, which touch tiles j and j+1 only.
  auto iter = [&](int j, auto buf_tag) {
    constexpr int B0 = decltype(buf_tag)::value, B1 = (B0 + 1) % 3, B2 = (B0 + 2) % 3;
    if constexpr (BIAS)  // the iteration enters one set of the block table: refill the other
      if (((2 * j + 2) & 63) == 0) tab.fill(bias, 2 * j + 2 + 64, NB, it, st, lane);
    if (j + 2 < T) copy_tile(j + 2, B2);  // every wave left tile j-1 before the last barrier
    {
      const int i = 2 * j + 1;  // scores of (tile j+1, block 0), contraction of (tile j, block 0)
      if (block_on(i + 1 < NB ? i + 1 : i)) {
        const int pos = block_pos(i);
        dkdv_step<DQK, DV, true>(init_of(tbuf(B1), 0, bb_of(i + 1)), qbuf(B1), gbuf(B1), 0, qbuf(B0), gbuf(B0), 0, raq,
                                 rag, caq, cag, kreg, vreg, sacc[1], dacc[1], sacc[0], dacc[0], pd[0],
                                 pd[1], dkacc, dvacc, c1, a.alpha, mask_of(pos), vis_of(pos));
      }
    }
    if (j + 1 < T) {
      const int i = 2 * j + 2;  // scores of (tile j+1, block 1), contraction of (tile j, block 1)
      if (block_on(i + 1)) {
        const int pos = block_pos(i);
        dkdv_step<DQK, DV, true>(init_of(tbuf(B1), 1, bb_of(i + 1)), qbuf(B1), gbuf(B1), 1, qbuf(B0), gbuf(B0), 1, raq,
                                 rag, caq, cag, kreg, vreg, sacc[0], dacc[0], sacc[1], dacc[1], pd[1],
                                 pd[0], dkacc, dvacc, c1, a.alpha, mask_of(pos), vis_of(pos));
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

  // contraction of the last block (tile T-1, block 1) on its own
  if (block_on(NB - 1)) {
    const int lb = (T - 1) % 3;
    const char* qt = qbuf(lb);
    const char* gt = gbuf(lb);
#pragma unroll
    for (int c = 0; c < DV / 32; ++c) {
      dvacc[c] = mfma(pd[1][0], cag.read(gt, 2, c), dvacc[c]);
      dvacc[c] = mfma(pd[1][1], cag.read(gt, 3, c), dvacc[c]);
    }
#pragma unroll
    for (int c = 0; c < DQK / 32; ++c) {
      dkacc[c] = mfma(pd[1][2], caq.read(qt, 2, c), dkacc[c]);
      dkacc[c] = mfma(pd[1][3], caq.read(qt, 3, c), dkacc[c]);
    }
  }
  }  // T > 0

  // Accumulators: lane holds column c*32 + n of key rows 8*(r/4) + 4*hh + r%4 of its wave.
  if (wave_on) {
    const float scale = a.alpha * a.inv_n;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int row = wave * 32 + 8 * (r >> 2) + 4 * hh + (r & 3);
      if (row >= it.nrows) continue;
      const int64_t ek = ((int64_t)it.row0 + row) * sq + h * DQK + n;
      const int64_t ev = ((int64_t)it.row0 + row) * sv + h * DV + n;
#pragma unroll
      for (int c = 0; c < DQK / 32; ++c)
        store_one(a.dk, ek + c * 32, dkacc[c][r] * scale, a.accumulate, a.out_f32);
#pragma unroll
      for (int c = 0; c < DV / 32; ++c)
        store_one(a.dv, ev + c * 32, dvacc[c][r] * scale, a.accumulate, a.out_f32);
    }
  }
}

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
// buckets go there one by one.  The LDS table holds 2^shift copies of every bucket, a lane adds
// to copy (lane mod 2^shift): lanes that hit the same bucket at once then mostly hit different
// addresses (same-address LDS atomics are served one after the other).
constexpr int DW_LDS = 2048;  // floats of the workgroup's table
__host__ __device__ constexpr int dw_shift(int nb) {
  int s = 0;
  while (s < 5 && (nb << (s + 1)) <= DW_LDS) ++s;
  return s;
}
struct DwAcc {
  float* dwl;   // LDS, 2^shift entries per bucket
  float sum;    // per lane: dS of the current run
  int cur;      // bucket of the current run (uniform; -1: none)
  int shift;
  __device__ __forceinline__ void add(int bucket, int lane, float x) {
    atomicAdd(dwl + (bucket << shift) + (lane & ((1 << shift) - 1)), x);
  }
  __device__ __forceinline__ void flush(int lane) {
    if (cur >= 0) {
      const float t = wave_sum(sum);
      if (lane == 0) atomicAdd(dwl + (cur << shift), t);
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
  float ds[16];
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    float p;
    bwd_elem(s[r], dp[r], c1, alpha, p, ds[r]);
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
  static_assert(!(PACKED && BIAS), "packed tiles: no bias");
  constexpr int KB = ST * DQK * 2, VB = ST * DV * 2;
  __shared__ __attribute__((aligned(1024))) char smem0[KB + VB];
  __shared__ __attribute__((aligned(1024))) char smem1[KB + VB];
  __shared__ __attribute__((aligned(1024))) char tmem0[BIAS ? REC_TILE : 16];
  __shared__ __attribute__((aligned(1024))) char tmem1[BIAS ? REC_TILE : 16];
  __shared__ float wtab[BIAS ? MAX_TS_BUCKETS : 1];
  __shared__ float dwl[BIAS ? DW_LDS : 1];
  auto kbuf = [&](int b) { return b ? smem1 : smem0; };
  auto vbuf = [&](int b) { return (b ? smem1 : smem0) + KB; };
  auto tbuf = [&](int b) { return b ? tmem1 : tmem0; };

  const int H = a.num_heads;
  const int slot = blockIdx.x / H, h = blockIdx.x % H;
  Item it;
  if (!fetch_item(a.plan, slot, it)) return;

  const int tid = threadIdx.x, lane = tid & 63, n = lane & 31, hh = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int64_t sq = (int64_t)H * DQK, sv = (int64_t)H * DV;
  const __bf16* qg = (const __bf16*)a.q + (int64_t)it.row0 * sq + h * DQK;
  const __bf16* gg = (const __bf16*)a.d_o + (int64_t)it.row0 * sv + h * DV;
  const __bf16* kg = (const __bf16*)a.k + h * DQK;
  const __bf16* vg = (const __bf16*)a.v + h * DV;

  const int orow = wave * 32 + n;
  const bool wave_on = wave * 32 < it.nrows;
  bf16x8 qreg[DQK / 16], greg[DV / 16];
  load_owner<DQK>(qreg, qg, sq, orow, it.nrows, hh);
  load_owner<DV>(greg, gg, sv, orow, it.nrows, hh);
  BiasCtx bias = {};
  DwAcc dwa = {dwl, 0.f, -1, 0};
  if constexpr (BIAS) {
    dwa.shift = dw_shift(a.nb);
    for (int i = tid; i < (a.nb << dwa.shift); i += NW * 64) dwl[i] = 0.f;
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
  Window win = {};
  if constexpr (PACKED) win = make_window(a.row_seq, it.row0 + orow, orow < it.nrows, 0, a.causal);

  if (st.total > 0) {
    const TileRef t0 = tile_ref(it, st, 0);
    tile_copy_async<DQK, NW>(kbuf(0), kg + (int64_t)t0.row * sq, sq, t0.valid, wave, lane);
    tile_copy_async<DV, NW>(vbuf(0), vg + (int64_t)t0.row * sv, sv, t0.valid, wave, lane);
    if (BIAS && wave == 0) rec_copy_async(tbuf(0), a.ts_rec + t0.row, t0.valid, lane);
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
        // no key of the block is visible (packed tiles: the windows decide)
        if (blk * 32 >= tj.valid || (!PACKED && a.causal && k_lo > q_hi)) continue;
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
    // the workgroup's sums go to the table gradient (fp32 atomics: the order of the additions,
    // and with it the last bits of the result, varies from run to run)
    dwa.flush(lane);
    __syncthreads();
    const float scale = a.alpha * a.inv_n;
    for (int i = tid; i < a.nb; i += NW * 64) {
      float t = 0.f;
      const int cm = (1 << dwa.shift) - 1;  // (rotated by i: neighbouring threads read different banks)
      for (int c = 0; c <= cm; ++c) t += dwl[(i << dwa.shift) + ((c + i) & cm)];
      if (t != 0.f) atomicAdd(a.d_ts_w + i, t * scale);
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
    // HSTU_ATTN_FWD_TILE=128|256 overrides the choice (testing and tuning)
    if (const char* e = getenv("HSTU_ATTN_FWD_TILE")) {
      if (e[0] == '1') return 4;
      if (e[0] == '2') return 8;
    }
    return (owner_rows / 256) * heads >= 2048 ? 8 : 4;
  }
  return 4;
}

#define HSTU_DISPATCH_D(KERNEL, NW, ...)                                                \
  do {                                                                                  \
    const dim3 grid((unsigned)((int64_t)a.max_items * a.num_heads)), block(NW * 64);    \
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

// The kernels with the timestamp bias exist for equal head dimensions of Q/K and V only.
#define HSTU_DISPATCH_BIAS(KERNEL, NW, ...)                                             \
  do {                                                                                  \
    const dim3 grid((unsigned)((int64_t)a.max_items * a.num_heads)), block(NW * 64);    \
    if (a.nb < 1 || a.nb > MAX_TS_BUCKETS || !a.ts_w || !a.ts_rec_own) return hipErrorInvalidValue; \
    if (d_qk == 128 && d_v == 128) hipLaunchKernelGGL((KERNEL<128, 128, __VA_ARGS__>), grid, block, 0, stream, a); \
    else if (d_qk == 64 && d_v == 64) hipLaunchKernelGGL((KERNEL<64, 64, __VA_ARGS__>), grid, block, 0, stream, a); \
    else if (d_qk == 32 && d_v == 32) hipLaunchKernelGGL((KERNEL<32, 32, __VA_ARGS__>), grid, block, 0, stream, a); \
    else return hipErrorInvalidValue;                                                   \
    return hipGetLastError();                                                           \
  } while (0)

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
      if (a.ts_rec) return hipErrorInvalidValue;
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
hipError_t launch_dkdv_bf16(const AttnArgs& a, int d_qk, int d_v, hipStream_t stream) {
  if (a.waves != 4 || (a.row_seq && a.ts_rec)) return hipErrorInvalidValue;
  if (a.row_seq) HSTU_DISPATCH_D(hstu_dkdv_bf16, 4, 4, false, true);
  if (a.ts_rec) HSTU_DISPATCH_BIAS(hstu_dkdv_bf16, 4, 4, true, false);
  HSTU_DISPATCH_D(hstu_dkdv_bf16, 4, 4, false, false);
}
hipError_t launch_dq_bf16(const AttnArgs& a, int d_qk, int d_v, hipStream_t stream) {
  if (a.waves != 4 || (a.row_seq && a.ts_rec)) return hipErrorInvalidValue;
  if (a.row_seq) HSTU_DISPATCH_D(hstu_dq_bf16, 4, 4, false, true);
  if (a.ts_rec) {
    if (!a.d_ts_w) return hipErrorInvalidValue;
    HSTU_DISPATCH_BIAS(hstu_dq_bf16, 4, 4, true, false);
  }
  HSTU_DISPATCH_D(hstu_dq_bf16, 4, 4, false, false);
}

}  // namespace hstu

