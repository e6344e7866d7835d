// Internal declarations shared by the library's translation units (not part of the C ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace hstu {

// One unit of scheduled work: a tile of "owner" rows (query rows for the forward and dq
// passes, key rows for the dk/dv pass) plus up to two segments of "streamed" rows of the
// same sequence that the tile is computed against.  Rows index the caller's buffers;
// positions are in-sequence positions and drive the causal mask, so the same kernels serve
// whole-batch attention (one segment, row == offset + position) and a context-parallel
// rank's share (two mini-chunks per side, section 2.3 of the paper).
struct Item {
  int32_t row0;         // first owner row of the tile
  int32_t nrows;        // valid owner rows (0..tile)
  int32_t pos0;         // in-sequence position of row0
  int32_t nseg;         // streamed segments in use (0..2)
  int32_t seg_row0[2];  // first streamed row of each segment
  int32_t seg_len[2];   // rows in each segment
  int32_t seg_pos0[2];  // in-sequence position of each segment's first row
  int32_t seg_tcol0[2]; // column of each segment's first row in the transposed streamed copies
  int32_t cost;         // visible 32-row streamed blocks (the sort key)
  int32_t part;         // 0: the item writes its output rows; p > 0: it covers only a part of the
                        // streamed rows and writes an fp32 partial result into slot p - 1
  int32_t pad[2];
};
static_assert(sizeof(Item) == 64, "Item is one 64-byte record");

// Device view of a built schedule.
struct Plan {
  const int32_t* header;  // [0] = number of items, [1] = number of 64-row streamed tiles,
                          // [2] = number of owner tiles whose partial results have to be summed
  const int32_t* red;     // per such tile: first owner row, rows, first partial slot, slots
  const int32_t* order;   // order[slot] = item index, non-increasing cost
  const Item* items;
  const int32_t* ttile;   // per 64-row streamed tile: first row, valid rows
  int32_t max_stiles;     // host bound on the streamed tiles; transposed copies have 64x this many columns
};

// Byte offsets of one schedule's arrays inside the workspace.
struct PlanLayout {
  size_t header, owner_base, streamed_base, tile_base, stile_base, ttile, order, items, red, end;
};

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// max_items bounds the items the kernels see (parts included), max_tiles the owner tiles.
inline PlanLayout plan_layout(size_t base, int64_t batch, int64_t max_items, int64_t max_stiles,
                              int64_t max_tiles = 0) {
  PlanLayout l;
  size_t p = align_up(base, 256);
  l.header = p;        p += 64;
  l.owner_base = p;    p = align_up(p + (size_t)(batch + 1) * 4, 64);
  l.streamed_base = p; p = align_up(p + (size_t)(batch + 1) * 4, 64);
  l.tile_base = p;     p = align_up(p + (size_t)(batch + 1) * 4, 64);
  l.stile_base = p;    p = align_up(p + (size_t)(batch + 1) * 4, 64);
  l.ttile = p;         p = align_up(p + (size_t)max_stiles * 8, 64);
  l.order = p;         p = align_up(p + (size_t)max_items * 4, 64);
  l.items = p;         p = align_up(p + (size_t)max_items * sizeof(Item), 64);
  l.red = p;           p = align_up(p + (size_t)max_tiles * 16, 64);
  l.end = p;
  return l;
}

// Upper bound on the number of items when `rows` owner rows of `batch` sequences, each cut
// into at most `segs` segments, are tiled by `tile` rows.
inline int64_t max_items_bound(int64_t rows, int64_t batch, int segs, int tile) {
  return rows / tile + (int64_t)segs * batch + 1;
}

struct PlanArgs {
  const int32_t* off;     // device, batch + 1
  int32_t batch;
  int32_t total_rows;     // rows of the global layout
  int32_t cp;             // context-parallel size (1 for whole-batch attention)
  int32_t owner_rank;     // -1: owner side is in the global layout
  int32_t streamed_rank;  // -1: streamed side is in the global layout
  int32_t side;           // 0: owners are queries, 1: owners are keys
  int32_t tile;           // owner rows per item
  int32_t causal;
  int32_t owner_rows;     // rows the caller declared for the owner-side buffers
  int32_t streamed_rows;  // rows the caller declared for the streamed-side buffers
  int32_t max_items;      // bound on the items written (parts of split tiles included)
  int32_t max_stiles;     // bound on the 64-row tiles of the streamed side
  int32_t cost_shift;     // cost >> cost_shift selects the sort bin
  int32_t split_max;      // an owner tile is cut into at most this many parts along its streamed
                          // rows (1: never); side 0 only
  int32_t split_blocks;   // ... of at least this many visible 32-row blocks each
  int32_t* red;           // reduce table (see Plan), split_max > 1 only
  int32_t* header;
  int32_t* owner_base;
  int32_t* streamed_base;
  int32_t* tile_base;
  int32_t* stile_base;
  int32_t* ttile;
  int32_t want_ttile;     // the streamed side's tile table is needed (a transposed copy will be built from it)
  int32_t* order;
  Item* items;
};

// Builds up to three schedules in one launch (one workgroup each).
hipError_t launch_plans(const PlanArgs* a, int count, hipStream_t stream);

// What the kernels need to know about a row's timestamp: the timestamp itself and the range of
// the timestamps of the (up to) 32 rows of the same sequence that start at this row, from which
// a 32-row block whose first row this is decides whether one bucket covers all its pairs.
struct TsRecord {
  int32_t ts, lo, hi, pad;
};
static_assert(sizeof(TsRecord) == 16, "one 16-byte record per row");
constexpr int MAX_TS_BUCKETS = 512;

// The bucket of a timestamp difference (the library's reading of section 2.1's sketch of the
// bias; see include/hstu_attn.h): 0 for delta <= 1, else min(nb - 1, e * 2^f + m) with
// e = floor(log2 delta) and m the f bits below delta's leading one.  Integer arithmetic only.
__device__ __forceinline__ int bias_bucket(uint32_t delta, int nb, int f) {
  const uint32_t d = delta > 2u ? delta : 2u;  // (no branch: the result for delta <= 1 is selected below)
  const int e = 31 - __builtin_clz(d);
  const uint32_t top = e >= f ? d >> (e - f) : d << (f - e);
  int b = (e << f) + (int)top - (1 << f);
  b = b < nb - 1 ? b : nb - 1;
  return delta <= 1u ? 0 : b;
}
// The same bucket for delta < 2^24, where the conversion to float is exact: the float's exponent
// and its top f mantissa bits are e and m.  (127 + e) * 2^f + m comes out of one shift of the bit
// pattern; delta = 0 and 1 land at or below zero and are clamped to bucket 0 like the rest.
constexpr uint32_t BIAS_SMALL_DELTA = 1u << 24;
__device__ __forceinline__ int bias_bucket_small(uint32_t delta, int nb, int f) {
  const int b = (int)(__builtin_bit_cast(uint32_t, (float)delta) >> (23 - f)) - (127 << f);
  const int lo = b > 0 ? b : 0;
  return lo < nb - 1 ? lo : nb - 1;
}
// |a - b| of two int32 values, exact up to 2^32 - 1.
__device__ __forceinline__ uint32_t abs_diff(int a, int b) {
  return (uint32_t)(a > b ? a : b) - (uint32_t)(a > b ? b : a);
}

// The gradient of the bias table is a sum of dS over all visible pairs of a bucket.  A workgroup
// of the dq pass sums its share in LDS as 64-bit fixed point with 32 fraction bits: LDS integer
// adds are served ten times faster than LDS float adds (measured: 8 against 80 ns per wave-wide
// instruction and CU), and the sum does not depend on the order of the additions.  Terms below
// 2^-32 are lost and a workgroup's sum for one bucket must stay below 2^31 in magnitude (128
// query rows against all their keys, dS unscaled: dP times SiLU').  The workgroups' sums are then
// added in double precision to a table of the call (acc), which a last small kernel scales and
// rounds to the caller's fp32 table.
constexpr float DW_FIXED_ONE = 4294967296.f;
__device__ __forceinline__ unsigned long long dw_to_fixed(float x) {
  return (unsigned long long)(long long)(x * DW_FIXED_ONE);
}
__device__ __forceinline__ double dw_from_fixed(unsigned long long q) {
  return (double)(long long)q * (1.0 / 4294967296.0);
}
// d_w[i] = (accumulate ? d_w[i] : 0) + scale * acc[i] for the nb buckets.
hipError_t launch_dw_finish(const double* acc, float* d_w, int nb, double scale, int accumulate,
                            hipStream_t stream);

// Builds the records of `total_rows` rows (rec has total_rows + 64 entries; the surplus is
// cleared) and, if acc is not null, clears the nb entries of the call's table of sums.  off: the
// offsets of the whole-batch layout (a row's range stops at the end of its sequence), or null for
// any other layout of rows (the range covers the next 32 rows whatever they belong to: a superset,
// which only makes the one-bucket test of a block more cautious).
hipError_t launch_ts_records(const int32_t* ts, const int32_t* off, int batch, int64_t total_rows,
                             TsRecord* rec, double* acc, int nb, hipStream_t stream);

// Packed tiles: schedules whose owner tiles are `tile` consecutive rows of the batch whatever
// sequences they belong to (item t = rows [t * tile, (t + 1) * tile), in natural order), for both
// sides at once, plus the per-row sequence bounds the kernels' windows come from.  Positions are
// row numbers.  Rows at or beyond off[batch] (clamped to total_rows) belong to no item.
struct PackedPlanArgs {
  const int32_t* off;
  int32_t batch, total_rows, tile, causal;
  int2* row_seq;                    // total_rows entries
  int32_t* header[2];               // per side (0: owners are queries, 1: keys): see Plan
  int32_t* order[2];
  Item* items[2];
};
hipError_t launch_packed_plan(const PackedPlanArgs& a, hipStream_t stream);

// Arguments of the attention kernels.
struct AttnArgs {
  const void* q;
  const void* k;
  const void* v;
  const void* d_o;
  const void* vt;   // transposed copy of v (bf16 forward; see launch_transpose_bf16)
  void* o;
  void* dq;
  void* dk;
  void* dv;
  Plan plan;
  int32_t num_heads;
  int32_t causal;
  int32_t accumulate;
  int32_t max_items;
  int32_t waves;    // wavefronts per workgroup (bf16 kernels): owner tile = 32 * waves rows
  int32_t out_f32;  // outputs are fp32 (bf16 kernels only; the fp32 kernels always write fp32)
  float* partial;   // partial results of split tiles: [slot][head][tile row][d] fp32 (or null)
  float alpha;
  float inv_n;
  // Timestamp bias (ts_rec == null: no bias).
  const TsRecord* ts_rec;      // per row of the streamed side's buffers, built by launch_ts_records
  const TsRecord* ts_rec_own;  // per row of the owner side's buffers (the same array for whole batches)
  const float* ts_w;       // bucket table, nb entries
  double* d_ts_acc;        // the call's sums of dS per bucket (dq pass: added with atomics), or null
  int32_t nb;              // buckets
  int32_t fbits;           // log2 of the groups per octave
  int32_t bias_per_pair;   // no block takes the one-bucket path (HSTU_FLAG_BIAS_PER_PAIR)
  // Packed tiles (bf16 kernels, whole-batch layout, batches of short sequences; null: not packed):
  // per row the first row and the end row of its sequence, built by launch_packed_plan.
  const int2* row_seq;
  // Large batch (many items, none of them a large share of the whole): kernels that run one
  // workgroup per CU may launch as many workgroups as CUs and let each walk over its share.
  int32_t large_batch;
  // Schedules in natural order (the items of a sequence are neighbours in the list) with a head
  // count that divides 8: the hardware hands workgroup i to XCD i % 8, each XCD with an L2 of
  // its own, so the unit -> (item, head) map gives every XCD one head and one contiguous part
  // of the list (8 / heads parts) and the tiles of a sequence, which stream the same rows, meet
  // in one L2.  1: the plain map, unit = item * heads + head (with 8 heads that already is one
  // head per XCD).
  int32_t xcd_parts;
  // Walking workgroups take contiguous runs of their XCD's units instead of every n-th unit
  // (natural order with a head count that divides 8).
  int32_t walk_chunks;
  // dk/dv pass: keep to the kernel with one wave per 32 keys where the two-wave kernel would serve.
  int32_t dkdv_one_wave;
};

// Owner rows per item each kernel family expects (pass: 0 forward, 1 dk/dv, 2 dq); the
// schedule must be built with the same value.
enum { PASS_FWD = 0, PASS_DKDV = 1, PASS_DQ = 2 };
// Wavefronts per workgroup (32 owner rows each) the bf16 kernels of a pass use for a problem
// with `owner_rows` owner rows and `heads` heads: large problems take the wider workgroup, which
// halves the traffic of streamed tiles; small ones keep enough workgroups to fill the chip.
int waves_bf16(int pass, int64_t owner_rows, int heads);
int tile_rows_f32(int pass);

// Transposed copy of a streamed bf16 tensor: src [rows, H, D] -> dst [H, D, 64 * max_stiles], one
// 64-column group per streamed tile, columns permuted inside each group of 16 into the order
// the matrix instructions consume them, zero beyond the valid rows.
hipError_t launch_transpose_bf16(const void* src, void* dst, const Plan& plan, int num_heads, int d,
                                 hipStream_t stream);

// Load-balance reorder (section 2.3): copies the 64-row tiles of a rank's local layout from / to
// their place in the global layout, for `count` tensors whose rows are row_bytes[i] long.
struct ReorderArgs {
  const char* src[4];
  char* dst[4];
  int64_t row_bytes[4];
  const int32_t* off;
  int32_t count;
  int32_t scatter;  // 0: dst is local, src global (gather); 1: dst is global, src local
  int32_t batch, total_rows, local_rows, cp, rank;
  int32_t split;    // workgroups per 64-row tile (a divisor of 64)
};
// max_tiles: an upper bound on the 64-row tiles of the local layout (the grid's first dimension).
hipError_t launch_reorder(const ReorderArgs& a, int64_t max_tiles, hipStream_t stream);

// Sums the partial results of split owner tiles (in slot order: deterministic) into `out`
// [rows, H, d] with the output conventions of the attention kernels.
hipError_t launch_reduce_partials(const Plan& plan, int64_t max_tiles, const float* partial, void* out,
                                  int num_heads, int d, int tile_rows, int accumulate, int out_f32,
                                  hipStream_t stream);

hipError_t launch_fwd_bf16(const AttnArgs& a, int d_qk, int d_v, hipStream_t stream);
hipError_t launch_dkdv_bf16(const AttnArgs& a, int d_qk, int d_v, hipStream_t stream);
// The dk/dv pass with two waves per 32 keys (plain per-sequence schedules at d_qk = d_v = 128).
bool dkdv_pair_supported(const AttnArgs& a, int d_qk, int d_v);
hipError_t launch_dkdv_pair_bf16(const AttnArgs& a, int d_qk, int d_v, hipStream_t stream);
hipError_t launch_dq_bf16(const AttnArgs& a, int d_qk, int d_v, hipStream_t stream);
hipError_t launch_fwd_f32(const AttnArgs& a, int d_qk, int d_v, hipStream_t stream);
hipError_t launch_dkdv_f32(const AttnArgs& a, int d_qk, int d_v, hipStream_t stream);
hipError_t launch_dq_f32(const AttnArgs& a, int d_qk, int d_v, hipStream_t stream);

// Measurement kernels (hstu_probe.hip): a loop of matrix instructions only (flops per launch
// returned), and fp32 atomic adds in the pattern of a dq produced by the dk/dv pass (payload
// bytes per launch returned).
hipError_t launch_mfma_loop(int iters, int random, float* sink, double* flops, hipStream_t stream);
hipError_t launch_dq_atomic(float* buf, int64_t rows, int heads, int nblk, int local, double* bytes,
                            hipStream_t stream);

}  // namespace hstu
