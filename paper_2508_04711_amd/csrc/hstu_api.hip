// C ABI of the jagged HSTU attention library: argument checks, workspace carving, launches.
// See include/hstu_attn.h for the contract of every entry point.
#include <atomic>
#include <cmath>
#include <cstdlib>
#include <mutex>
#include <vector>

#include "../../include/hstu_attn.h"
#include "hstu_common.h"

namespace {

using namespace hstu;

bool dim_ok(int d) { return d == 32 || d == 64 || d == 128; }

// Optional per-launch timing (hstu_debug_timing_begin/end): thread-local, off by default.
struct Timing {
  bool on = false;
  std::vector<hipEvent_t> start, stop;
  std::vector<int> kind;
  size_t used = 0;
};
thread_local Timing g_timing;

struct TimedLaunch {
  hipStream_t stream;
  bool active;
  TimedLaunch(int kind, hipStream_t s) : stream(s), active(false) {
    Timing& t = g_timing;
    if (t.on && t.used < t.start.size()) {
      active = true;
      t.kind[t.used] = kind;
      (void)hipEventRecord(t.start[t.used], stream);
    }
  }
  ~TimedLaunch() {
    if (active) {
      Timing& t = g_timing;
      (void)hipEventRecord(t.stop[t.used], stream);
      ++t.used;
    }
  }
};

int check_params(const hstu_attn_params* p) {
  if (!p) return HSTU_ERR_NULL_PTR;
  if (p->batch < 0 || p->num_heads < 1 || p->total_rows < 0 || p->total_rows >= (1ll << 31) ||
      p->max_len < 1 || !std::isfinite(p->alpha))
    return HSTU_ERR_BAD_SHAPE;
  if (!dim_ok(p->d_qk) || !dim_ok(p->d_v)) return HSTU_ERR_UNSUPPORTED;
  if (p->dtype != HSTU_BF16 && p->dtype != HSTU_F32) return HSTU_ERR_UNSUPPORTED;
  if (p->out_dtype != p->dtype && p->out_dtype != HSTU_F32) return HSTU_ERR_UNSUPPORTED;
  if (p->flags & ~HSTU_FLAGS_ALL) return HSTU_ERR_UNSUPPORTED;
  if ((p->flags & HSTU_FLAG_FWD_TILE_128) && (p->flags & HSTU_FLAG_FWD_TILE_256)) return HSTU_ERR_UNSUPPORTED;
  return HSTU_OK;
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Short sequences on average (the host knows the mean length, total_rows / batch, without
// reading the offsets): such batches keep the natural item order where they are large, and their
// dk/dv workgroups may walk over items (see prepare_plan).
bool short_sequences(const hstu_attn_params* p) {
  // a forced tile height means the forms of long sequences
  if (p->flags & (HSTU_FLAG_FWD_TILE_128 | HSTU_FLAG_FWD_TILE_256)) return false;
  return p->batch > 0 && p->total_rows / p->batch <= 1024;
}

// Whether the bf16 forward pass reads V through a transposed copy built first (see
// launch_transpose_bf16): only when a tile height is forced.  The copy buys one LDS instruction per
// matrix instruction instead of one and a half and costs a launch and the copy's traffic.  Measured
// on one box, the default (row-major V, 128-row tiles) against the copy with 256-row tiles: forward
// 2.71 against 2.92 + 0.07 ms on the long skewed batch, the step within +-0.7 % (under the chip's
// power limit a faster forward pass slows the passes after it); the context-parallel workload -3 %
// per step, the 16-sequence workload -1.5 %, the ring form -3 % (a launch less per step).
bool fwd_transposed_v(const hstu_attn_params* p) {
  return p->dtype == HSTU_BF16 && (p->flags & (HSTU_FLAG_FWD_TILE_128 | HSTU_FLAG_FWD_TILE_256)) != 0;
}

// Batches of very short sequences (mean length at most PACKED_MEAN_LEN): the whole-batch entry
// points tile the rows of the batch regardless of sequence boundaries (packed tiles), so that no
// tile is mostly padding.  HSTU_FLAG_NO_PACK turns this off, HSTU_FLAG_PACK_SHORT moves the
// threshold up to the 1024 of the short-sequence form.
// Measured, fwd + bwd, H = 4, d = 128, per-sequence tiles -> packed: 8192 sequences of 16..64 rows
// 1.98 -> 1.35 ms (the per-sequence schedule build alone is 0.16 ms); 4096 of 32..256 rows 2.82 ->
// 2.65 ms; 2048 of 200..400 rows 3.13 -> 3.06 ms; 1536 of 300..600 rows 3.94 -> 3.92 ms: beyond a mean
// of ~300 rows the two are within noise of each other.
constexpr int PACKED_TILE = 128;
constexpr int64_t PACKED_MEAN_LEN = 256;
bool packed_tiles(const hstu_attn_params* p) {
  if (p->dtype != HSTU_BF16 || !short_sequences(p) || (p->flags & HSTU_FLAG_NO_PACK)) return false;
  const int64_t limit = (p->flags & HSTU_FLAG_PACK_SHORT) ? 1024 : PACKED_MEAN_LEN;
  return p->total_rows / p->batch <= limit;
}
size_t packed_bytes(const hstu_attn_params* p) {
  const size_t nt = (size_t)(p->total_rows + PACKED_TILE - 1) / PACKED_TILE;
  return align_up((size_t)p->total_rows * sizeof(int2), 256) +
         2 * (256 + align_up(nt * 4, 256) + align_up(nt * sizeof(Item), 256));
}

// Wavefronts per workgroup and owner rows per item of a pass on a problem of the given size.
int pass_waves(const hstu_attn_params* p, int pass, int64_t owner_rows) {
  if (p->dtype != HSTU_BF16 || short_sequences(p)) return 4;
  if (pass == PASS_FWD && !fwd_transposed_v(p)) return 4;  // (the eight-wave forward reads the transposed copy)
  if (pass == PASS_FWD && (p->flags & HSTU_FLAG_FWD_TILE_128)) return 4;
  if (pass == PASS_FWD && (p->flags & HSTU_FLAG_FWD_TILE_256)) return 8;
  return waves_bf16(pass, owner_rows, p->num_heads);
}
int tile_rows(const hstu_attn_params* p, int pass, int64_t owner_rows) {
  return p->dtype == HSTU_BF16 ? 32 * pass_waves(p, pass, owner_rows) : tile_rows_f32(pass);
}

// One schedule: who owns, who is streamed, how many rows each side's buffers hold.
struct SideSpec {
  int side;           // 0: owners are queries, 1: owners are keys
  int pass;           // which kernel family consumes it (tile height)
  int owner_rank, streamed_rank;
  int64_t owner_rows, streamed_rows;
  int segs;           // segments per sequence on the owner side (1 global, 2 rank-local)
  int ssegs;          // segments per sequence on the streamed side
};

struct BuiltPlan {
  Plan plan;
  int64_t max_items;  // items the kernels may see (grid bound), parts of split tiles included
  int64_t max_tiles;  // owner tiles (bound on the reduce table)
  int split;          // parts an owner tile may be cut into (1: none)
  size_t end;
  int waves;
  bool large;         // short sequences, and even the heaviest item is a small share of one workgroup slot's work
  bool natural;       // the items are in their natural order (those of a sequence are neighbours)
  bool chunks;        // dK/dV workgroups walk over contiguous runs of the list
};

// Bound on the items of a schedule, taken with the smallest tile any kernel variant uses so that
// it holds whichever variant the problem size selects (surplus workgroups exit at once).
int64_t items_bound(const hstu_attn_params* p, const SideSpec& s) {
  return max_items_bound(s.owner_rows, p->batch, s.segs,
                         p->dtype == HSTU_BF16 ? 128 : tile_rows_f32(s.pass));
}

// Bound on the 64-row tiles of the streamed side (the transposed copies have 64 columns each).
int64_t stiles_bound(const hstu_attn_params* p, const SideSpec& s) {
  return max_items_bound(s.streamed_rows, p->batch, s.ssegs, 64);
}

// Query-side passes (forward, dQ) on a problem with too few owner tiles to fill the chip cut
// their heavy tiles along the keys into up to this many parts, each an item of its own that
// writes an fp32 partial result; a small kernel then sums the parts in a fixed order.  What is
// gained: with fewer workgroups than slots the pass lasts as long as its heaviest tile, which
// under a causal mask sees twice the average number of keys (a context-parallel rank's share
// and small batches of long sequences are such problems).
constexpr int SPLIT_BLOCKS = 64;  // a part covers at least this many visible 32-row blocks
int split_of(const hstu_attn_params* p, const SideSpec& s) {
  if (p->dtype != HSTU_BF16 || s.side != 0 || (p->flags & HSTU_FLAG_NO_SPLIT)) return 1;
  // no sequence is long enough for two parts (when the lengths respect max_len)
  if ((int64_t)p->max_len < 2 * SPLIT_BLOCKS * 32) return 1;
  const int64_t wgs = items_bound(p, s) * p->num_heads;
  const int64_t slots = pass_waves(p, s.pass, s.owner_rows) == 8 ? 256 : 512;
  // Measured on the context-parallel workload (548 workgroups for 512 slots): two parts of at
  // least 64 blocks 574 TFLOP/s for the step, four parts of 16 blocks 522, none 507; on the
  // 16-sequence workload (1224 workgroups) splitting loses to the cost of the partial results.
  const int64_t n = (2 * slots + wgs - 1) / wgs;
  return n < 1 ? 1 : (n > 8 ? 8 : (int)n);
}

// Bounds for the workspace query that hold for every number of owner rows up to s.owner_rows
// (a context-parallel rank's share is not known when the workspace is sized):
// tiles * split <= tiles + 2 * slots / heads + 1 because split <= 2 * slots / (tiles * heads) + 1.
int64_t split_items_bound(const hstu_attn_params* p, const SideSpec& s) {
  const int64_t tiles = items_bound(p, s);
  if (p->dtype != HSTU_BF16 || s.side != 0 || (p->flags & HSTU_FLAG_NO_SPLIT) ||
      (int64_t)p->max_len < 2 * SPLIT_BLOCKS * 32)
    return tiles;
  return tiles + 2 * 512 / p->num_heads + 1;
}

size_t plan_bytes(const hstu_attn_params* p, const SideSpec& s, size_t base) {
  return plan_layout(base, p->batch, split_items_bound(p, s), stiles_bound(p, s), items_bound(p, s)).end;
}

// Bytes of the partial results of a pass whose outputs have head dimension d: exact for a call
// (slots = the schedule's item bound), an upper bound for the workspace query.
size_t partial_bytes(const hstu_attn_params* p, int64_t slots, int tile, int d) {
  return align_up((size_t)slots * p->num_heads * tile * d * 4, 256);
}
size_t partial_bytes_bound(const hstu_attn_params* p, const SideSpec& s, int d) {
  if (split_items_bound(p, s) == items_bound(p, s)) return 0;
  // 128-row tiles: the 256-row forward is chosen only for problems with thousands of tiles,
  // which are never cut
  return partial_bytes(p, split_items_bound(p, s), 128, d);
}

// Bytes of one transposed copy of a streamed tensor with head dimension d (bf16 only).
size_t tcopy_bytes(const hstu_attn_params* p, const SideSpec& s, int d) {
  if (!fwd_transposed_v(p)) return 0;
  return align_up((size_t)p->num_heads * d * 64 * stiles_bound(p, s) * 2, 256);
}

// Carves one schedule out of the workspace at byte offset `base` and fills the arguments of
// its build (launched by launch_built).
int prepare_plan(const hstu_attn_params* p, int cp_size, const SideSpec& s, const int32_t* off,
                 char* ws, size_t ws_bytes, size_t base, PlanArgs* args, BuiltPlan* out) {
  const int split = split_of(p, s);
  const int64_t max_tiles = items_bound(p, s), max_items = max_tiles * split, max_stiles = stiles_bound(p, s);
  // only the forward pass with a transposed copy of V reads the streamed side's tile table (see make_tcopy)
  const bool want_ttile = s.pass == PASS_FWD && fwd_transposed_v(p);
  if (max_items * p->num_heads >= (1ll << 31) || max_stiles * p->num_heads >= (1ll << 31) ||
      // (the rows of the transposed copy are addressed with 32-bit byte offsets)
      (want_ttile && max_stiles * 64 * 2 * 128 >= (1ll << 31)))
    return HSTU_ERR_BAD_SHAPE;
  const PlanLayout l = plan_layout(base, p->batch, max_items, max_stiles, max_tiles);
  if (l.end > ws_bytes) return HSTU_ERR_WORKSPACE_TOO_SMALL;
  PlanArgs a;
  a.off = off;
  a.batch = p->batch;
  a.total_rows = (int32_t)p->total_rows;
  a.cp = cp_size;
  a.owner_rank = s.owner_rank;
  a.streamed_rank = s.streamed_rank;
  a.side = s.side;
  a.tile = tile_rows(p, s.pass, s.owner_rows);
  a.causal = p->causal ? 1 : 0;
  a.owner_rows = (int32_t)s.owner_rows;
  a.streamed_rows = (int32_t)s.streamed_rows;
  a.max_items = (int32_t)max_items;
  a.max_stiles = (int32_t)max_stiles;
  // cost bins: an item's cost is at most the 32-row blocks of one sequence's streamed side, which
  // max_len bounds when the caller's lengths respect it (longer ones share the last bin)
  const int64_t longest = s.streamed_rows < p->max_len ? s.streamed_rows : (int64_t)p->max_len;
  int shift = 0;
  while (((longest / 32 + 4) >> shift) >= 2048) ++shift;
  // When even the heaviest possible item is a small fraction of what one workgroup slot gets
  // to do in total (large batches), the order cannot unbalance the tail, and the natural order
  // keeps the items of a sequence, which share their streamed rows, together in time: one bin.
  // Both sides of the comparison in (owner row, streamed row) pairs: the heaviest item has at
  // most tile x longest; all items together at least batch x mean owner rows x mean streamed
  // rows (half of it under the causal mask), the sum of products being smallest when every
  // sequence has the mean length.
  // Measured, H = 4, d = 128, sorted -> natural: 1536 sequences of 300..600 rows forward 1.18 ->
  // 0.86 ms, dQ 1.32 -> 1.07, dK/dV 1.94 -> 2.06; 768 of 600..1200 forward 1.68 -> 1.15, dQ 1.83 ->
  // 1.53, dK/dV 2.68 -> 2.94; 512 of 1000..2000 forward 2.17 -> 2.10, dQ 2.91 -> 2.29, dK/dV 4.25
  // -> 3.96: the passes whose owners are queries always gain; the dK/dV pass at two workgroups per
  // CU gains 4 % (H = 8, d = 64, 1024 sequences of 400..800 rows 1.76 -> 1.69 ms); at one workgroup
  // per CU (d_qk + d_v > 128) it gains beyond the short-sequence form, and below it when its
  // walking workgroups take contiguous runs (2 to 5 %), but loses 4 % when they take every 256th
  // item, whose stride beats against the tiles per sequence.
  const int64_t batch = p->batch > 0 ? p->batch : 1;
  const int64_t all_pairs = s.owner_rows / batch * (s.streamed_rows / batch) / (p->causal ? 2 : 1) * batch;
  const int64_t per_slot = all_pairs / 512 * p->num_heads;
  const bool large = (int64_t)tile_rows(p, s.pass, s.owner_rows) * longest * 8 < per_slot;
  // The dK/dV pass at one workgroup per CU walks over the list (see launch_dkdv_bf16): in natural
  // order when its workgroups can take contiguous runs of one XCD's share, which needs a head
  // count that divides 8; sorted by cost, every 256th item, otherwise.
  const bool chunks = large && s.side == 1 && short_sequences(p) && p->d_qk + p->d_v > 128 &&
                      p->dtype == HSTU_BF16 && p->num_heads <= 8 && 8 % p->num_heads == 0;
  out->chunks = chunks;
  if (large && (s.side == 0 || !short_sequences(p) || p->d_qk + p->d_v <= 128 || chunks)) shift = 30;
  out->natural = shift == 30 && split <= 1;
  // (Walking workgroups take every 256th item: fine for a sorted list of short items, but in the
  // natural order of longer sequences the stride beats against the tiles per sequence: measured
  // 7 % slower on 512 sequences of 1000..2000 rows, 3 to 5 % faster on 200..1200 rows.)
  out->large = large && short_sequences(p);
  a.cost_shift = shift;
  a.split_max = split;
  a.split_blocks = SPLIT_BLOCKS;
  a.red = reinterpret_cast<int32_t*>(ws + l.red);
  a.header = reinterpret_cast<int32_t*>(ws + l.header);
  a.owner_base = reinterpret_cast<int32_t*>(ws + l.owner_base);
  a.streamed_base = reinterpret_cast<int32_t*>(ws + l.streamed_base);
  a.tile_base = reinterpret_cast<int32_t*>(ws + l.tile_base);
  a.stile_base = reinterpret_cast<int32_t*>(ws + l.stile_base);
  a.ttile = reinterpret_cast<int32_t*>(ws + l.ttile);
  a.want_ttile = want_ttile ? 1 : 0;
  a.order = reinterpret_cast<int32_t*>(ws + l.order);
  a.items = reinterpret_cast<Item*>(ws + l.items);
  *args = a;
  out->plan.header = a.header;
  out->plan.order = a.order;
  out->plan.items = a.items;
  out->plan.ttile = a.ttile;
  out->plan.red = a.red;
  out->plan.max_stiles = a.max_stiles;
  out->max_items = max_items;
  out->max_tiles = max_tiles;
  out->split = split;
  out->waves = pass_waves(p, s.pass, s.owner_rows);
  out->end = l.end;
  return HSTU_OK;
}

// Packed tiles: carves the row bounds and both sides' schedules out of the workspace at `base`
// and launches their construction.
struct PackedPlans {
  BuiltPlan side[2];
  const int2* row_seq;
};
int build_packed(const hstu_attn_params* p, const int32_t* off, char* ws, size_t ws_bytes, size_t base,
                 hipStream_t stream, PackedPlans* out) {
  const size_t nt = (size_t)(p->total_rows + PACKED_TILE - 1) / PACKED_TILE;
  if ((int64_t)nt * p->num_heads >= (1ll << 31)) return HSTU_ERR_BAD_SHAPE;
  size_t at = align_up(base, 256);
  if (at + packed_bytes(p) > ws_bytes) return HSTU_ERR_WORKSPACE_TOO_SMALL;
  PackedPlanArgs a = {};
  a.off = off;
  a.batch = p->batch;
  a.total_rows = (int32_t)p->total_rows;
  a.tile = PACKED_TILE;
  a.causal = p->causal ? 1 : 0;
  a.row_seq = reinterpret_cast<int2*>(ws + at);
  at += align_up((size_t)p->total_rows * sizeof(int2), 256);
  for (int side = 0; side < 2; ++side) {
    a.header[side] = reinterpret_cast<int32_t*>(ws + at); at += 256;
    a.order[side] = reinterpret_cast<int32_t*>(ws + at);  at += align_up(nt * 4, 256);
    a.items[side] = reinterpret_cast<Item*>(ws + at);     at += align_up(nt * sizeof(Item), 256);
    BuiltPlan& bp = out->side[side];
    bp.plan = Plan{};
    bp.plan.header = a.header[side];
    bp.plan.order = a.order[side];
    bp.plan.items = a.items[side];
    bp.max_items = (int64_t)nt;
    bp.max_tiles = (int64_t)nt;
    bp.split = 1;
    bp.waves = PACKED_TILE / 32;
    bp.large = false;  // (the packed dK/dV kernel walks whatever the size)
    bp.natural = true;
    bp.chunks = false;
    bp.end = at;
  }
  out->row_seq = a.row_seq;
  TimedLaunch timed(3, stream);
  return launch_packed_plan(a, stream) == hipSuccess ? HSTU_OK : HSTU_ERR_HIP;
}

// Carves a transposed copy out of the workspace at *base and launches its construction.
int make_tcopy(const hstu_attn_params* p, const SideSpec& s, const BuiltPlan& bp, const void* src,
               int d, char* ws, size_t ws_bytes, size_t* base, hipStream_t stream, const void** out) {
  *out = nullptr;
  if (!fwd_transposed_v(p)) return HSTU_OK;
  const size_t at = align_up(*base, 256), bytes = tcopy_bytes(p, s, d);
  if (at + bytes > ws_bytes) return HSTU_ERR_WORKSPACE_TOO_SMALL;
  {
    TimedLaunch timed(4, stream);
    if (launch_transpose_bf16(src, ws + at, bp.plan, p->num_heads, d, stream) != hipSuccess)
      return HSTU_ERR_HIP;
  }
  *out = ws + at;
  *base = at + bytes;
  return HSTU_OK;
}

int launch_built(const PlanArgs* args, int count, hipStream_t stream) {
  TimedLaunch timed(3, stream);
  return launch_plans(args, count, stream) == hipSuccess ? HSTU_OK : HSTU_ERR_HIP;
}

// One schedule: prepare and launch.
int build_plan(const hstu_attn_params* p, int cp_size, const SideSpec& s, const int32_t* off,
               char* ws, size_t ws_bytes, size_t base, hipStream_t stream, BuiltPlan* out) {
  PlanArgs args;
  const int rc = prepare_plan(p, cp_size, s, off, ws, ws_bytes, base, &args, out);
  if (rc != HSTU_OK) return rc;
  return launch_built(&args, 1, stream);
}

AttnArgs base_args(const hstu_attn_params* p, const BuiltPlan& bp, int accumulate) {
  AttnArgs a = {};
  a.plan = bp.plan;
  a.num_heads = p->num_heads;
  a.causal = p->causal ? 1 : 0;
  a.accumulate = accumulate;
  a.max_items = (int32_t)bp.max_items;
  a.waves = bp.waves;
  a.large_batch = bp.large ? 1 : 0;
  a.walk_chunks = bp.chunks ? 1 : 0;
  a.xcd_parts = bp.natural && p->dtype == HSTU_BF16 && p->num_heads < 8 && 8 % p->num_heads == 0
                    ? 8 / p->num_heads : 1;
  a.out_f32 = p->out_dtype == HSTU_F32 ? 1 : 0;
  a.dkdv_one_wave = (p->flags & HSTU_FLAG_DKDV_ONE_WAVE) ? 1 : 0;
  a.bias_per_pair = (p->flags & HSTU_FLAG_BIAS_PER_PAIR) ? 1 : 0;
  a.alpha = p->alpha;
  a.inv_n = 1.0f / (float)p->max_len;
  return a;
}

int run_pass(const hstu_attn_params* p, int pass, const AttnArgs& a, hipStream_t stream) {
  hipError_t e;
  TimedLaunch timed(pass, stream);
  if (p->dtype == HSTU_BF16) {
    e = pass == PASS_FWD ? launch_fwd_bf16(a, p->d_qk, p->d_v, stream)
        : pass == PASS_DKDV ? launch_dkdv_bf16(a, p->d_qk, p->d_v, stream)
                            : launch_dq_bf16(a, p->d_qk, p->d_v, stream);
  } else {
    e = pass == PASS_FWD ? launch_fwd_f32(a, p->d_qk, p->d_v, stream)
        : pass == PASS_DKDV ? launch_dkdv_f32(a, p->d_qk, p->d_v, stream)
                            : launch_dq_f32(a, p->d_qk, p->d_v, stream);
  }
  return e == hipSuccess ? HSTU_OK : HSTU_ERR_HIP;
}

// A query-side pass (forward or dQ) whose schedule may contain parts of split tiles: carves the
// partial results out of the workspace at *base, runs the pass, then sums the parts into `out`
// (head dimension d).
int run_query_pass(const hstu_attn_params* p, int pass, AttnArgs& a, const BuiltPlan& bp,
                   const SideSpec& s, void* out, int d, char* ws, size_t ws_bytes, size_t* base,
                   hipStream_t stream) {
  a.partial = nullptr;
  (void)s;
  if (bp.split > 1) {
    const size_t at = align_up(*base, 256), bytes = partial_bytes(p, bp.max_items, 32 * bp.waves, d);
    if (at + bytes > ws_bytes) return HSTU_ERR_WORKSPACE_TOO_SMALL;
    a.partial = reinterpret_cast<float*>(ws + at);
    *base = at + bytes;
  }
  int rc = run_pass(p, pass, a, stream);
  if (rc != HSTU_OK || bp.split <= 1) return rc;
  TimedLaunch timed(6, stream);
  return launch_reduce_partials(bp.plan, bp.max_tiles, a.partial, out, p->num_heads, d, 32 * bp.waves,
                                a.accumulate, a.out_f32, stream) == hipSuccess ? HSTU_OK : HSTU_ERR_HIP;
}

// Timestamp bias: argument checks and the per-row records at the start of the workspace.
int check_bias(const hstu_attn_params* p, const hstu_ts_bias* b, bool backward) {
  if (!b) return HSTU_ERR_NULL_PTR;
  if (b->num_buckets < 1 || b->num_buckets > MAX_TS_BUCKETS || b->groups_log2 < 0 || b->groups_log2 > 8)
    return HSTU_ERR_BAD_SHAPE;
  if (!b->timestamps || !b->ts_weights || (backward && !b->d_ts_weights)) return HSTU_ERR_NULL_PTR;
  return HSTU_OK;
}
// The workspace of a call with bias starts with the call's table of sums for the table gradient
// (one double per bucket), then one array of records per layout of rows.
constexpr size_t DW_ACC_BYTES = MAX_TS_BUCKETS * sizeof(double);
size_t ts_record_bytes(const hstu_attn_params* p) {
  return align_up((size_t)(p->total_rows + 64) * sizeof(TsRecord), 256);
}
size_t bias_front_bytes(const hstu_attn_params* p, int arrays) {
  return DW_ACC_BYTES + arrays * ts_record_bytes(p);
}
// Builds the records (and clears the table of sums for a backward call).
int build_ts_records(const hstu_attn_params* p, const hstu_ts_bias* b, const int32_t* off, char* ws,
                     bool backward, hipStream_t stream) {
  TimedLaunch timed(7, stream);
  return launch_ts_records(b->timestamps, off, p->batch, p->total_rows,
                           reinterpret_cast<TsRecord*>(ws + DW_ACC_BYTES),
                           backward ? reinterpret_cast<double*>(ws) : nullptr, b->num_buckets,
                           stream) == hipSuccess
             ? HSTU_OK : HSTU_ERR_HIP;
}
void set_bias(AttnArgs& a, const hstu_ts_bias* b, char* ws, bool backward) {
  a.ts_rec = reinterpret_cast<const TsRecord*>(ws + DW_ACC_BYTES);
  a.ts_rec_own = a.ts_rec;
  a.ts_w = b->ts_weights;
  a.d_ts_acc = backward ? reinterpret_cast<double*>(ws) : nullptr;
  a.nb = b->num_buckets;
  a.fbits = b->groups_log2;
}
// Scales the call's sums into the caller's table gradient.
int finish_dw(const hstu_attn_params* p, const char* ws, float* d_w, int nb, int accumulate,
              hipStream_t stream) {
  TimedLaunch timed(8, stream);
  return launch_dw_finish(reinterpret_cast<const double*>(ws), d_w, nb,
                          (double)p->alpha / (double)p->max_len, accumulate, stream) == hipSuccess
             ? HSTU_OK : HSTU_ERR_HIP;
}

SideSpec full_side(const hstu_attn_params* p, int side, int pass) {
  return SideSpec{side, pass, -1, -1, p->total_rows, p->total_rows, 1, 1};
}

int64_t clamp_rows(int64_t rows, int64_t total) { return rows < total ? rows : total; }

SideSpec cp_side(const hstu_attn_params* p, const hstu_cp_desc* cp, int side, int pass) {
  const int64_t qr = clamp_rows(cp->q_rows, p->total_rows), kr = clamp_rows(cp->kv_rows, p->total_rows);
  if (side == 0) return SideSpec{0, pass, cp->q_rank, cp->kv_rank, qr, kr, 2, cp->kv_rank < 0 ? 1 : 2};
  return SideSpec{1, pass, cp->kv_rank, cp->q_rank, kr, qr, cp->kv_rank < 0 ? 1 : 2, 2};
}

int check_cp(const hstu_attn_params* p, const hstu_cp_desc* cp) {
  if (!cp) return HSTU_ERR_NULL_PTR;
  if (cp->cp_size < 1 || cp->q_rank < 0 || cp->q_rank >= cp->cp_size || cp->kv_rank < -1 ||
      cp->kv_rank >= cp->cp_size || cp->q_rows < 0 || cp->kv_rows < 0 ||
      (int64_t)cp->cp_size * 2 >= (1ll << 31))
    return HSTU_ERR_BAD_CP;
  (void)p;
  return HSTU_OK;
}

}  // namespace

extern "C" {

const char* hstu_attn_status_string(int status) {
  switch (status) {
    case HSTU_OK: return "ok";
    case HSTU_ERR_NULL_PTR: return "a required pointer is NULL";
    case HSTU_ERR_BAD_SHAPE: return "bad shape: batch, num_heads, total_rows, max_len or alpha out of range";
    case HSTU_ERR_UNSUPPORTED: return "unsupported head dimension or dtype";
    case HSTU_ERR_WORKSPACE_TOO_SMALL: return "workspace too small";
    case HSTU_ERR_BAD_CP: return "bad context-parallel descriptor";
    case HSTU_ERR_HIP: return "a HIP call failed";
    case HSTU_ERR_MISALIGNED: return "a data pointer is not 16-byte aligned";
    case HSTU_ERR_STATIC_SCRATCH: return "the problem needs more scratch than the library's static buffer holds";
    default: return "unknown status";
  }
}

int hstu_validate_offsets_host(const int32_t* host_offsets, int32_t batch, int64_t total_rows) {
  if (!host_offsets) return HSTU_ERR_NULL_PTR;
  if (batch < 0 || total_rows < 0) return HSTU_ERR_BAD_SHAPE;
  if (host_offsets[0] != 0) return HSTU_ERR_BAD_SHAPE;
  for (int32_t b = 0; b < batch; ++b)
    if (host_offsets[b + 1] < host_offsets[b]) return HSTU_ERR_BAD_SHAPE;
  if ((int64_t)host_offsets[batch] != total_rows) return HSTU_ERR_BAD_SHAPE;
  return HSTU_OK;
}

int hstu_schedule_tile_rows(const hstu_attn_params* params, int side) {
  const int rc = check_params(params);
  if (rc != HSTU_OK) return rc;
  return tile_rows(params, side == 0 ? PASS_FWD : PASS_DKDV, params->total_rows);
}

size_t hstu_jagged_attn_workspace_bytes(const hstu_attn_params* params, int which) {
  if (check_params(params) != HSTU_OK) return 0;
  const hstu_attn_params* p = params;
  size_t end = 0;
  bool too_large = false;
  // Each pass: its schedule, then the transposed copies of the tensors it streams (bf16 only).
  // d_t: head dimension of the transposed copy, d_p: of the partial results (0: none)
  auto pass_bytes = [&](const SideSpec& s, int d_t, int d_p) {
    // the limits of prepare_plan (with the largest split: the query holds for every share of the rows)
    if (split_items_bound(p, s) * p->num_heads >= (1ll << 31) || stiles_bound(p, s) * p->num_heads >= (1ll << 31) ||
        (d_t && tcopy_bytes(p, s, d_t) && stiles_bound(p, s) * 64 * 2 * 128 >= (1ll << 31)))
      too_large = true;
    end = plan_bytes(p, s, end);
    if (d_t) end = align_up(end, 256) + tcopy_bytes(p, s, d_t);
    if (d_p) end = align_up(end, 256) + partial_bytes_bound(p, s, d_p);
  };
  if (which == HSTU_WS_FWD) {
    pass_bytes(full_side(p, 0, PASS_FWD), p->d_v, p->d_v);
  } else if (which == HSTU_WS_BWD) {
    pass_bytes(full_side(p, 1, PASS_DKDV), 0, 0);
    pass_bytes(full_side(p, 0, PASS_DQ), 0, p->d_qk);
  } else if (which == HSTU_WS_CP) {
    // rank-local sides never hold more rows than the whole batch
    SideSpec s{0, PASS_FWD, 0, 0, p->total_rows, p->total_rows, 2, 2};
    pass_bytes(s, p->d_v, p->d_v);
    s.pass = PASS_DKDV; s.side = 1;
    pass_bytes(s, 0, 0);
    s.pass = PASS_DQ; s.side = 0;
    pass_bytes(s, 0, p->d_qk);
  } else {
    return 0;
  }
  if (too_large) return 0;
  if (which != HSTU_WS_CP && packed_tiles(p)) end = align_up(end, 256) + packed_bytes(p);
  return end + 4096;  // slack for the 256-byte alignment of each piece
}

size_t hstu_jagged_attn_bias_workspace_bytes(const hstu_attn_params* params, int which) {
  if (which != HSTU_WS_FWD && which != HSTU_WS_BWD && which != HSTU_WS_CP) return 0;
  const size_t plain = hstu_jagged_attn_workspace_bytes(params, which);
  if (!plain) return 0;
  // one array of records, or one per side (neither side holds more rows than the whole batch)
  return plain + bias_front_bytes(params, which == HSTU_WS_CP ? 2 : 1);
}

// Forward over the whole batch, with the timestamp bias if `bias` is not null.
static int fwd_impl(const hstu_attn_params* params, const hstu_ts_bias* bias, const void* q,
                    const void* k, const void* v, const int32_t* seq_offsets, void* o,
                    void* workspace, size_t workspace_bytes, void* hip_stream) {
  int rc = check_params(params);
  if (rc != HSTU_OK) return rc;
  if (bias && (rc = check_bias(params, bias, false)) != HSTU_OK) return rc;
  if (params->batch == 0 || params->total_rows == 0) return HSTU_OK;
  if (!q || !k || !v || !o || !seq_offsets || !workspace) return HSTU_ERR_NULL_PTR;
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(o) || !aligned16(workspace))
    return HSTU_ERR_MISALIGNED;
  if (workspace_bytes < (bias ? hstu_jagged_attn_bias_workspace_bytes(params, HSTU_WS_FWD)
                              : hstu_jagged_attn_workspace_bytes(params, HSTU_WS_FWD)))
    return HSTU_ERR_WORKSPACE_TOO_SMALL;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  const size_t first = bias ? bias_front_bytes(params, 1) : 0;  // the records come first
  // (packed tiles: a block's rows may belong to several sequences, so a record's range covers
  // the next 32 rows of the batch whatever sequences they belong to)
  const bool packed = packed_tiles(params);
  if (bias && (rc = build_ts_records(params, bias, packed ? nullptr : seq_offsets, (char*)workspace, false,
                                     stream)) != HSTU_OK)
    return rc;
  if (packed) {
    PackedPlans pp;
    rc = build_packed(params, seq_offsets, (char*)workspace, workspace_bytes, first, stream, &pp);
    if (rc != HSTU_OK) return rc;
    AttnArgs a = base_args(params, pp.side[0], 0);
    a.q = q; a.k = k; a.v = v; a.o = o;
    a.row_seq = pp.row_seq;
    if (bias) set_bias(a, bias, (char*)workspace, false);
    return run_pass(params, PASS_FWD, a, stream);
  }
  BuiltPlan bp;
  rc = build_plan(params, 1, full_side(params, 0, PASS_FWD), seq_offsets, (char*)workspace,
                  workspace_bytes, first, stream, &bp);
  if (rc != HSTU_OK) return rc;
  size_t base = bp.end;
  AttnArgs a = base_args(params, bp, 0);
  a.q = q; a.k = k; a.v = v; a.o = o;
  if (bias) set_bias(a, bias, (char*)workspace, false);
  rc = make_tcopy(params, full_side(params, 0, PASS_FWD), bp, v, params->d_v, (char*)workspace,
                  workspace_bytes, &base, stream, &a.vt);
  if (rc != HSTU_OK) return rc;
  return run_query_pass(params, PASS_FWD, a, bp, full_side(params, 0, PASS_FWD), o, params->d_v,
                        (char*)workspace, workspace_bytes, &base, stream);
}

int hstu_jagged_attn_fwd(const hstu_attn_params* params, const void* q, const void* k,
                         const void* v, const int32_t* seq_offsets, void* o, void* workspace,
                         size_t workspace_bytes, void* hip_stream) {
  return fwd_impl(params, nullptr, q, k, v, seq_offsets, o, workspace, workspace_bytes, hip_stream);
}

int hstu_jagged_attn_bias_fwd(const hstu_attn_params* params, const hstu_ts_bias* bias,
                              const void* q, const void* k, const void* v,
                              const int32_t* seq_offsets, void* o, void* workspace,
                              size_t workspace_bytes, void* hip_stream) {
  if (!bias) return HSTU_ERR_NULL_PTR;
  return fwd_impl(params, bias, q, k, v, seq_offsets, o, workspace, workspace_bytes, hip_stream);
}

// ---- forward for callers that cannot allocate -----------------------------------------------
// The same forward with its scratch (schedule, transposed copy of V, partial results) in a static
// device array instead of a caller's workspace.  Host code never uses the array's name as an
// address: the device address is looked up once per device and kept.
constexpr size_t STATIC_SCRATCH_BYTES = (size_t)HSTU_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];
constexpr int STATIC_MAX_DEVICES = 64;
static std::atomic<void*> g_scratch_ptr[STATIC_MAX_DEVICES];
static std::mutex g_scratch_mutex;

// Address of the current device's copy of the array (looked up at the first call on that device).
static int static_scratch(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= STATIC_MAX_DEVICES) return HSTU_ERR_HIP;
  void* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (!p) {
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    p = g_scratch_ptr[dev].load(std::memory_order_relaxed);
    if (!p) {
      if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return HSTU_ERR_HIP;
      g_scratch_ptr[dev].store(p, std::memory_order_release);
    }
  }
  *out = p;
  return HSTU_OK;
}

size_t hstu_static_scratch_bytes(void) { return STATIC_SCRATCH_BYTES; }

int hstu_jagged_attn_fwd_static(const hstu_attn_params* params, const void* q, const void* k,
                                const void* v, const int32_t* seq_offsets, void* o, void* hip_stream) {
  const int rc = check_params(params);
  if (rc != HSTU_OK) return rc;
  if (params->batch == 0 || params->total_rows == 0) return HSTU_OK;
  if (!q || !k || !v || !o || !seq_offsets) return HSTU_ERR_NULL_PTR;
  const size_t need = hstu_jagged_attn_workspace_bytes(params, HSTU_WS_FWD);
  if (need == 0 || need > STATIC_SCRATCH_BYTES) return HSTU_ERR_STATIC_SCRATCH;
  void* ws = nullptr;
  const int rs = static_scratch(&ws);
  if (rs != HSTU_OK) return rs;
  return fwd_impl(params, nullptr, q, k, v, seq_offsets, o, ws, STATIC_SCRATCH_BYTES, hip_stream);
}

// Backward over the whole batch, with the timestamp bias if `bias` is not null.
static int bwd_impl(const hstu_attn_params* params, const hstu_ts_bias* bias, const void* q,
                    const void* k, const void* v, const void* d_o, const int32_t* seq_offsets,
                    void* dq, void* dk, void* dv, void* workspace, size_t workspace_bytes,
                    void* hip_stream) {
  int rc = check_params(params);
  if (rc != HSTU_OK) return rc;
  if (bias && (rc = check_bias(params, bias, true)) != HSTU_OK) return rc;
  if (params->batch == 0 || params->total_rows == 0) return HSTU_OK;
  if (!q || !k || !v || !d_o || !dq || !dk || !dv || !seq_offsets || !workspace)
    return HSTU_ERR_NULL_PTR;
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(d_o) || !aligned16(dq) ||
      !aligned16(dk) || !aligned16(dv) || !aligned16(workspace))
    return HSTU_ERR_MISALIGNED;
  if (workspace_bytes < (bias ? hstu_jagged_attn_bias_workspace_bytes(params, HSTU_WS_BWD)
                              : hstu_jagged_attn_workspace_bytes(params, HSTU_WS_BWD)))
    return HSTU_ERR_WORKSPACE_TOO_SMALL;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  const size_t first = bias ? bias_front_bytes(params, 1) : 0;  // the records come first
  const bool packed = packed_tiles(params);
  if (bias && (rc = build_ts_records(params, bias, packed ? nullptr : seq_offsets, (char*)workspace, true,
                                     stream)) != HSTU_OK)
    return rc;
  if (packed) {
    PackedPlans pp;
    rc = build_packed(params, seq_offsets, (char*)workspace, workspace_bytes, first, stream, &pp);
    if (rc != HSTU_OK) return rc;
    AttnArgs a = base_args(params, pp.side[1], 0);
    a.q = q; a.k = k; a.v = v; a.d_o = d_o; a.dk = dk; a.dv = dv;
    a.row_seq = pp.row_seq;
    if (bias) set_bias(a, bias, (char*)workspace, true);
    rc = run_pass(params, PASS_DKDV, a, stream);
    if (rc != HSTU_OK) return rc;
    AttnArgs b = base_args(params, pp.side[0], 0);
    b.q = q; b.k = k; b.v = v; b.d_o = d_o; b.dq = dq;
    b.row_seq = pp.row_seq;
    if (bias) set_bias(b, bias, (char*)workspace, true);
    rc = run_pass(params, PASS_DQ, b, stream);
    if (rc != HSTU_OK || !bias) return rc;
    return finish_dw(params, (const char*)workspace, bias->d_ts_weights, bias->num_buckets, 0, stream);
  }
  BuiltPlan pk, pq;
  PlanArgs pa[2];
  rc = prepare_plan(params, 1, full_side(params, 1, PASS_DKDV), seq_offsets, (char*)workspace,
                    workspace_bytes, first, &pa[0], &pk);
  if (rc != HSTU_OK) return rc;
  rc = prepare_plan(params, 1, full_side(params, 0, PASS_DQ), seq_offsets, (char*)workspace,
                    workspace_bytes, pk.end, &pa[1], &pq);
  if (rc != HSTU_OK) return rc;
  rc = launch_built(pa, 2, stream);
  if (rc != HSTU_OK) return rc;
  AttnArgs a = base_args(params, pk, 0);
  a.q = q; a.k = k; a.v = v; a.d_o = d_o; a.dk = dk; a.dv = dv;
  if (bias) set_bias(a, bias, (char*)workspace, true);
  rc = run_pass(params, PASS_DKDV, a, stream);
  if (rc != HSTU_OK) return rc;
  AttnArgs b = base_args(params, pq, 0);
  b.q = q; b.k = k; b.v = v; b.d_o = d_o; b.dq = dq;
  if (bias) set_bias(b, bias, (char*)workspace, true);
  size_t base = pq.end;
  rc = run_query_pass(params, PASS_DQ, b, pq, full_side(params, 0, PASS_DQ), dq, params->d_qk,
                      (char*)workspace, workspace_bytes, &base, stream);
  if (rc != HSTU_OK || !bias) return rc;
  return finish_dw(params, (const char*)workspace, bias->d_ts_weights, bias->num_buckets, 0, stream);
}

int hstu_jagged_attn_bwd(const hstu_attn_params* params, const void* q, const void* k,
                         const void* v, const void* d_o, const int32_t* seq_offsets, void* dq,
                         void* dk, void* dv, void* workspace, size_t workspace_bytes,
                         void* hip_stream) {
  return bwd_impl(params, nullptr, q, k, v, d_o, seq_offsets, dq, dk, dv, workspace, workspace_bytes,
                  hip_stream);
}

int hstu_jagged_attn_bias_bwd(const hstu_attn_params* params, const hstu_ts_bias* bias,
                              const void* q, const void* k, const void* v, const void* d_o,
                              const int32_t* seq_offsets, void* dq, void* dk, void* dv,
                              void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (!bias) return HSTU_ERR_NULL_PTR;
  return bwd_impl(params, bias, q, k, v, d_o, seq_offsets, dq, dk, dv, workspace, workspace_bytes,
                  hip_stream);
}

// The partial of one (query rank, key rank) pair.  acc_q: add to o_local / dq_local;
// acc_kv: add to dk_part / dv_part (the two differ in a ring: a rank's own accumulators run
// over the steps, the key-side gradients belong to the part that is visiting).
static int cp_partial_impl(const hstu_attn_params* params, const hstu_cp_desc* cp,
                           const hstu_cp_ts_bias* bias,
                           const void* q_local, const void* k_part, const void* v_part,
                           const void* d_o_local, const int32_t* seq_offsets_global,
                           void* o_local, void* dq_local, void* dk_part, void* dv_part,
                           int acc_q, int acc_kv, void* workspace, size_t workspace_bytes,
                           void* hip_stream) {
  int rc = check_params(params);
  if (rc != HSTU_OK) return rc;
  rc = check_cp(params, cp);
  if (rc != HSTU_OK) return rc;
  if (params->batch == 0 || params->total_rows == 0) return HSTU_OK;
  const bool backward = d_o_local != nullptr;
  if (!q_local || !k_part || !v_part || !seq_offsets_global || !workspace) return HSTU_ERR_NULL_PTR;
  if (!backward && !o_local) return HSTU_ERR_NULL_PTR;
  if (backward && (!dq_local || !dk_part || !dv_part)) return HSTU_ERR_NULL_PTR;
  const void* ptrs[] = {q_local, k_part, v_part, d_o_local, o_local, dq_local, dk_part, dv_part, workspace};
  for (const void* ptr : ptrs)
    if (ptr && !aligned16(ptr)) return HSTU_ERR_MISALIGNED;
  if (bias) {
    if (bias->num_buckets < 1 || bias->num_buckets > MAX_TS_BUCKETS || bias->groups_log2 < 0 ||
        bias->groups_log2 > 8)
      return HSTU_ERR_BAD_SHAPE;
    if (!bias->q_timestamps || !bias->kv_timestamps || !bias->ts_weights ||
        (backward && !bias->d_ts_weights))
      return HSTU_ERR_NULL_PTR;
  }
  if (workspace_bytes < (bias ? hstu_jagged_attn_bias_workspace_bytes(params, HSTU_WS_CP)
                              : hstu_jagged_attn_workspace_bytes(params, HSTU_WS_CP)))
    return HSTU_ERR_WORKSPACE_TOO_SMALL;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  char* ws = (char*)workspace;
  // the (up to) three schedules are built by one launch
  const bool do_f = o_local && cp->q_rows > 0, do_k = backward && cp->kv_rows > 0,
             do_q = backward && cp->q_rows > 0;
  PlanArgs pa[3];
  BuiltPlan pf, pk, pq;
  int np = 0;
  size_t base = 0, tbase = 0, qbase = 0;
  // with bias: the records of the query side's rows, then of the key side's, come first
  const TsRecord *q_rec = nullptr, *kv_rec = nullptr;
  if (bias) {
    const int64_t qr = clamp_rows(cp->q_rows, params->total_rows), kr = clamp_rows(cp->kv_rows, params->total_rows);
    q_rec = reinterpret_cast<const TsRecord*>(ws + DW_ACC_BYTES);
    kv_rec = reinterpret_cast<const TsRecord*>(ws + DW_ACC_BYTES + ts_record_bytes(params));
    base = bias_front_bytes(params, 2);
    TimedLaunch timed(7, stream);
    // the first launch also clears the call's table of sums
    double* clear = backward ? reinterpret_cast<double*>(ws) : nullptr;
    if (launch_ts_records(bias->q_timestamps, nullptr, 0, qr, const_cast<TsRecord*>(q_rec), clear,
                          bias->num_buckets, stream) != hipSuccess ||
        launch_ts_records(bias->kv_timestamps, cp->kv_rank < 0 ? seq_offsets_global : nullptr,
                          params->batch, kr, const_cast<TsRecord*>(kv_rec), nullptr, bias->num_buckets,
                          stream) != hipSuccess)
      return HSTU_ERR_HIP;
  }
  auto with_bias = [&](AttnArgs& a, bool owners_are_queries) {
    if (!bias) return;
    a.ts_rec = owners_are_queries ? kv_rec : q_rec;
    a.ts_rec_own = owners_are_queries ? q_rec : kv_rec;
    a.ts_w = bias->ts_weights;
    a.d_ts_acc = backward ? reinterpret_cast<double*>(ws) : nullptr;
    a.nb = bias->num_buckets;
    a.fbits = bias->groups_log2;
  };
  const SideSpec sf = cp_side(params, cp, 0, PASS_FWD), sq = cp_side(params, cp, 0, PASS_DQ);
  if (do_f) {
    rc = prepare_plan(params, cp->cp_size, sf, seq_offsets_global, ws, workspace_bytes, base, &pa[np++], &pf);
    if (rc != HSTU_OK) return rc;
    tbase = pf.end;  // the transposed copy of V and the partial results follow the schedule
    base = align_up(pf.end, 256) + tcopy_bytes(params, sf, params->d_v);
    if (pf.split > 1) base = align_up(base, 256) + partial_bytes(params, pf.max_items, 32 * pf.waves, params->d_v);
  }
  if (do_k) {
    rc = prepare_plan(params, cp->cp_size, cp_side(params, cp, 1, PASS_DKDV), seq_offsets_global, ws,
                      workspace_bytes, base, &pa[np++], &pk);
    if (rc != HSTU_OK) return rc;
    base = pk.end;
  }
  if (do_q) {
    rc = prepare_plan(params, cp->cp_size, sq, seq_offsets_global, ws, workspace_bytes, base, &pa[np++], &pq);
    if (rc != HSTU_OK) return rc;
    qbase = pq.end;
  }
  // with bias, a backward call ends by scaling its sums into the caller's table gradient
  auto finish = [&]() -> int {
    if (!bias || !backward) return HSTU_OK;
    return finish_dw(params, ws, bias->d_ts_weights, bias->num_buckets, acc_q, stream);
  };
  if (np == 0) return finish();
  rc = launch_built(pa, np, stream);
  if (rc != HSTU_OK) return rc;
  if (do_f) {
    AttnArgs a = base_args(params, pf, acc_q);
    a.q = q_local; a.k = k_part; a.v = v_part; a.o = o_local;
    with_bias(a, true);
    rc = make_tcopy(params, sf, pf, v_part, params->d_v, ws, workspace_bytes, &tbase, stream, &a.vt);
    if (rc != HSTU_OK) return rc;
    rc = run_query_pass(params, PASS_FWD, a, pf, sf, o_local, params->d_v, ws, workspace_bytes, &tbase, stream);
    if (rc != HSTU_OK) return rc;
  }
  if (do_k) {
    AttnArgs a = base_args(params, pk, acc_kv);
    a.q = q_local; a.k = k_part; a.v = v_part; a.d_o = d_o_local; a.dk = dk_part; a.dv = dv_part;
    with_bias(a, false);
    rc = run_pass(params, PASS_DKDV, a, stream);
    if (rc != HSTU_OK) return rc;
  }
  if (do_q) {
    AttnArgs b = base_args(params, pq, acc_q);
    b.q = q_local; b.k = k_part; b.v = v_part; b.d_o = d_o_local; b.dq = dq_local;
    with_bias(b, true);
    rc = run_query_pass(params, PASS_DQ, b, pq, sq, dq_local, params->d_qk, ws, workspace_bytes, &qbase, stream);
    if (rc != HSTU_OK) return rc;
  }
  return finish();
}

int hstu_jagged_attn_cp_partial(const hstu_attn_params* params, const hstu_cp_desc* cp,
                                const void* q_local, const void* k_part, const void* v_part,
                                const void* d_o_local, const int32_t* seq_offsets_global,
                                void* o_local, void* dq_local, void* dk_part, void* dv_part,
                                void* workspace, size_t workspace_bytes, void* hip_stream) {
  const int acc = (cp && cp->accumulate) ? 1 : 0;
  return cp_partial_impl(params, cp, nullptr, q_local, k_part, v_part, d_o_local, seq_offsets_global,
                         o_local, dq_local, dk_part, dv_part, acc, acc, workspace, workspace_bytes,
                         hip_stream);
}

int hstu_jagged_attn_cp_partial_bias(const hstu_attn_params* params, const hstu_cp_desc* cp,
                                     const hstu_cp_ts_bias* bias, const void* q_local,
                                     const void* k_part, const void* v_part, const void* d_o_local,
                                     const int32_t* seq_offsets_global, void* o_local, void* dq_local,
                                     void* dk_part, void* dv_part, void* workspace,
                                     size_t workspace_bytes, void* hip_stream) {
  if (!bias) return HSTU_ERR_NULL_PTR;
  const int acc = (cp && cp->accumulate) ? 1 : 0;
  return cp_partial_impl(params, cp, bias, q_local, k_part, v_part, d_o_local, seq_offsets_global,
                         o_local, dq_local, dk_part, dv_part, acc, acc, workspace, workspace_bytes,
                         hip_stream);
}

// The ring pass, with the timestamp bias if `bias` is not null.
static int ring_impl(const hstu_attn_params* params, const hstu_cp_ring_desc* ring,
                     const hstu_cp_ring_ts_bias* bias, const void* q_local, const void* d_o_local,
                     const int32_t* seq_offsets_global, void* o_local, void* dq_local, void* workspace,
                     size_t workspace_bytes, void* compute_stream, void* copy_stream) {
  int rc = check_params(params);
  if (rc != HSTU_OK) return rc;
  if (!ring) return HSTU_ERR_NULL_PTR;
  const int cp = ring->cp_size, me = ring->q_rank;
  if (cp < 1 || (int64_t)cp * 2 >= (1ll << 31) || me < 0 || me >= cp || ring->q_rows < 0 ||
      ring->recv_rows < 0)
    return HSTU_ERR_BAD_CP;
  if (ring->reserved != 0) return HSTU_ERR_UNSUPPORTED;
  if (!ring->part_rows || !ring->k_parts || !ring->v_parts) return HSTU_ERR_NULL_PTR;
  const bool backward = d_o_local != nullptr;
  if (backward && (!ring->dk_parts || !ring->dv_parts)) return HSTU_ERR_NULL_PTR;
  if (compute_stream == copy_stream) return HSTU_ERR_UNSUPPORTED;  // the overlap needs two streams
  const size_t eb = params->dtype == HSTU_BF16 ? 2 : 4;
  const size_t krow = (size_t)params->num_heads * params->d_qk * eb;
  const size_t vrow = (size_t)params->num_heads * params->d_v * eb;
  for (int r = 0; r < cp; ++r) {
    if (ring->part_rows[r] < 0) return HSTU_ERR_BAD_CP;
    if (ring->part_rows[r] > 0 && (!ring->k_parts[r] || !ring->v_parts[r])) return HSTU_ERR_NULL_PTR;
    if (backward && ring->part_rows[r] > 0 && (!ring->dk_parts[r] || !ring->dv_parts[r]))
      return HSTU_ERR_NULL_PTR;
    if (r != me && ring->part_rows[r] > ring->recv_rows) return HSTU_ERR_BAD_CP;
    if (bias && ring->part_rows[r] > 0 && (!bias->ts_parts || !bias->ts_parts[r])) return HSTU_ERR_NULL_PTR;
  }
  if (cp > 1 && ring->recv_rows > 0)
    for (int b = 0; b < 2; ++b)
      if (!ring->k_recv[b] || !ring->v_recv[b] || (bias && !bias->ts_recv[b])) return HSTU_ERR_NULL_PTR;
  if (params->batch == 0 || params->total_rows == 0) return HSTU_OK;

  hipStream_t cs = static_cast<hipStream_t>(compute_stream), xs = static_cast<hipStream_t>(copy_stream);
  // landed[b]: the part in receive buffer b has arrived; released[b]: the step that read
  // buffer b has been issued to the end (its kernels are ordered on the compute stream).
  hipEvent_t landed[2] = {nullptr, nullptr}, released[2] = {nullptr, nullptr}, start = nullptr;
  auto cleanup = [&](int code) {
    for (int b = 0; b < 2; ++b) {
      if (landed[b]) (void)hipEventDestroy(landed[b]);
      if (released[b]) (void)hipEventDestroy(released[b]);
    }
    if (start) (void)hipEventDestroy(start);
    return code;
  };
  for (int b = 0; b < 2; ++b) {
    if (hipEventCreateWithFlags(&landed[b], hipEventDisableTiming) != hipSuccess ||
        hipEventCreateWithFlags(&released[b], hipEventDisableTiming) != hipSuccess)
      return cleanup(HSTU_ERR_HIP);
  }
  if (hipEventCreateWithFlags(&start, hipEventDisableTiming) != hipSuccess) return cleanup(HSTU_ERR_HIP);
  // the copy stream must not run ahead of what the caller queued on the compute stream
  if (hipEventRecord(start, cs) != hipSuccess || hipStreamWaitEvent(xs, start, 0) != hipSuccess)
    return cleanup(HSTU_ERR_HIP);

  // Step s works on the part of rank (me - s) mod cp: the rank's own part first, then the
  // parts as they would arrive from the previous rank of the ring.  The transfer of step
  // s + 1's part runs on the copy stream while step s computes.
  auto part_of = [&](int s) { return ((me - s) % cp + cp) % cp; };
  auto fetch = [&](int s) -> int {  // start the transfer for step s (s >= 1) into buffer s & 1
    const int r = part_of(s), b = s & 1;
    if (s >= 3 && hipStreamWaitEvent(xs, released[b], 0) != hipSuccess) return HSTU_ERR_HIP;
    const size_t rows = (size_t)ring->part_rows[r];
    if (rows > 0) {
      if (hipMemcpyAsync(ring->k_recv[b], ring->k_parts[r], rows * krow, hipMemcpyDeviceToDevice, xs) != hipSuccess ||
          hipMemcpyAsync(ring->v_recv[b], ring->v_parts[r], rows * vrow, hipMemcpyDeviceToDevice, xs) != hipSuccess)
        return HSTU_ERR_HIP;
      if (bias && hipMemcpyAsync(bias->ts_recv[b], bias->ts_parts[r], rows * sizeof(int32_t),
                                 hipMemcpyDeviceToDevice, xs) != hipSuccess)
        return HSTU_ERR_HIP;
    }
    return hipEventRecord(landed[b], xs) == hipSuccess ? HSTU_OK : HSTU_ERR_HIP;
  };
  for (int s = 1; s <= 2 && s < cp; ++s) {  // both buffers are free at the start
    rc = fetch(s);
    if (rc != HSTU_OK) return cleanup(rc);
  }
  for (int s = 0; s < cp; ++s) {
    const int r = part_of(s), b = s & 1;
    const void* kp = s == 0 ? ring->k_parts[r] : ring->k_recv[b];
    const void* vp = s == 0 ? ring->v_parts[r] : ring->v_recv[b];
    if (s > 0 && hipStreamWaitEvent(cs, landed[b], 0) != hipSuccess) return cleanup(HSTU_ERR_HIP);
    hstu_cp_desc d = {};
    d.cp_size = cp; d.q_rank = me; d.kv_rank = r; d.accumulate = 0;
    d.q_rows = ring->q_rows; d.kv_rows = ring->part_rows[r];
    if (ring->part_rows[r] > 0 || s == 0) {
      // a rank with no rows in some part still has to clear its own outputs once
      // (pointers of an empty part are never dereferenced; any valid one satisfies the checks)
      void* dkp = backward ? (ring->dk_parts[r] ? ring->dk_parts[r] : dq_local) : nullptr;
      void* dvp = backward ? (ring->dv_parts[r] ? ring->dv_parts[r] : dq_local) : nullptr;
      hstu_cp_ts_bias step_bias = {};
      if (bias) {
        const int32_t* kt = s == 0 ? bias->ts_parts[r] : bias->ts_recv[b];
        step_bias.q_timestamps = bias->q_timestamps;
        step_bias.kv_timestamps = kt ? kt : bias->q_timestamps;  // (an empty part is never read)
        step_bias.ts_weights = bias->ts_weights;
        step_bias.d_ts_weights = bias->d_ts_weights;
        step_bias.num_buckets = bias->num_buckets;
        step_bias.groups_log2 = bias->groups_log2;
      }
      rc = cp_partial_impl(params, &d, bias ? &step_bias : nullptr, q_local, kp ? kp : q_local, vp ? vp : q_local, d_o_local,
                           seq_offsets_global, o_local, dq_local, dkp, dvp, s > 0 ? 1 : 0,
                           ring->accumulate_dkv ? 1 : 0, workspace, workspace_bytes, cs);
      if (rc != HSTU_OK) return cleanup(rc);
    }
    if (s > 0 && hipEventRecord(released[b], cs) != hipSuccess) return cleanup(HSTU_ERR_HIP);
    if (s > 0 && s + 2 < cp) {
      rc = fetch(s + 2);  // into the buffer this step read; the transfer waits for released[b]
      if (rc != HSTU_OK) return cleanup(rc);
    }
  }
  return cleanup(HSTU_OK);
}

int hstu_cp_ring_pass(const hstu_attn_params* params, const hstu_cp_ring_desc* ring,
                      const void* q_local, const void* d_o_local, const int32_t* seq_offsets_global,
                      void* o_local, void* dq_local, void* workspace, size_t workspace_bytes,
                      void* compute_stream, void* copy_stream) {
  return ring_impl(params, ring, nullptr, q_local, d_o_local, seq_offsets_global, o_local, dq_local,
                   workspace, workspace_bytes, compute_stream, copy_stream);
}

int hstu_cp_ring_pass_bias(const hstu_attn_params* params, const hstu_cp_ring_desc* ring,
                           const hstu_cp_ring_ts_bias* bias, const void* q_local,
                           const void* d_o_local, const int32_t* seq_offsets_global, void* o_local,
                           void* dq_local, void* workspace, size_t workspace_bytes,
                           void* compute_stream, void* copy_stream) {
  if (!bias) return HSTU_ERR_NULL_PTR;
  if (!bias->q_timestamps || !bias->ts_weights) return HSTU_ERR_NULL_PTR;
  return ring_impl(params, ring, bias, q_local, d_o_local, seq_offsets_global, o_local, dq_local,
                   workspace, workspace_bytes, compute_stream, copy_stream);
}

int hstu_cp_reorder(int32_t batch, int64_t total_rows, int32_t cp_size, int32_t rank, int32_t scatter,
                    int32_t num_tensors, const void* const* src, void* const* dst,
                    const int64_t* row_bytes, int64_t local_rows, const int32_t* seq_offsets,
                    void* hip_stream) {
  if (batch < 0 || total_rows < 0 || total_rows >= (1ll << 31) || local_rows < 0)
    return HSTU_ERR_BAD_SHAPE;
  if (cp_size < 1 || rank < 0 || rank >= cp_size || (int64_t)cp_size * 2 >= (1ll << 31))
    return HSTU_ERR_BAD_CP;
  if (num_tensors < 1 || num_tensors > 4) return HSTU_ERR_BAD_SHAPE;
  if (!src || !dst || !row_bytes) return HSTU_ERR_NULL_PTR;
  ReorderArgs ra = {};
  for (int t = 0; t < num_tensors; ++t) {
    if (!src[t] || !dst[t]) return HSTU_ERR_NULL_PTR;
    if (row_bytes[t] < 4 || row_bytes[t] % 4 != 0) return HSTU_ERR_BAD_SHAPE;
    if (!aligned16(src[t]) || !aligned16(dst[t])) return HSTU_ERR_MISALIGNED;
    ra.src[t] = (const char*)src[t];
    ra.dst[t] = (char*)dst[t];
    ra.row_bytes[t] = row_bytes[t];
  }
  if (batch == 0 || total_rows == 0 || local_rows == 0) return HSTU_OK;
  if (!seq_offsets) return HSTU_ERR_NULL_PTR;
  const int64_t lr = clamp_rows(local_rows, total_rows);
  // at most two segments per sequence, each with one ragged last tile
  const int64_t max_tiles = max_items_bound(lr, batch, 2, 64);
  if (max_tiles >= (1ll << 31)) return HSTU_ERR_BAD_SHAPE;
  ra.off = seq_offsets;
  ra.count = num_tensors;
  ra.scatter = scatter ? 1 : 0;
  ra.batch = batch; ra.total_rows = (int32_t)total_rows; ra.local_rows = (int32_t)lr;
  ra.cp = cp_size; ra.rank = rank;
  ra.split = 2;  // two workgroups per tile measured a few percent faster than one; more gain nothing
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  TimedLaunch timed(5, stream);
  return launch_reorder(ra, max_tiles, stream) == hipSuccess ? HSTU_OK : HSTU_ERR_HIP;
}

int hstu_debug_mfma_loop(int random_operands, int iterations, float* sink, double* flops_per_launch,
                         void* hip_stream) {
  if (!sink || !flops_per_launch) return HSTU_ERR_NULL_PTR;
  if (iterations < 1 || iterations > (1 << 24)) return HSTU_ERR_BAD_SHAPE;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  TimedLaunch timed(9, stream);
  return launch_mfma_loop(iterations, random_operands ? 1 : 0, sink, flops_per_launch, stream) == hipSuccess
             ? HSTU_OK : HSTU_ERR_HIP;
}

int hstu_debug_dq_atomic_rate(float* dq_f32, int64_t rows, int32_t num_heads, int32_t blocks,
                              int32_t head_per_xcd, double* payload_bytes_per_launch, void* hip_stream) {
  if (!dq_f32 || !payload_bytes_per_launch) return HSTU_ERR_NULL_PTR;
  if (rows < 64 || rows >= (1ll << 31) || num_heads < 1 || blocks < 1 || blocks > (1 << 20))
    return HSTU_ERR_BAD_SHAPE;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  TimedLaunch timed(10, stream);
  return launch_dq_atomic(dq_f32, rows, num_heads, blocks, head_per_xcd ? 1 : 0, payload_bytes_per_launch,
                          stream) == hipSuccess ? HSTU_OK : HSTU_ERR_HIP;
}

int hstu_debug_timing_begin(int max_records) {
  Timing& t = g_timing;
  if (t.on || max_records < 1 || max_records > (1 << 16)) return HSTU_ERR_BAD_SHAPE;
  t.start.assign(max_records, nullptr);
  t.stop.assign(max_records, nullptr);
  t.kind.assign(max_records, -1);
  t.used = 0;
  for (int i = 0; i < max_records; ++i)
    if (hipEventCreate(&t.start[i]) != hipSuccess || hipEventCreate(&t.stop[i]) != hipSuccess)
      return HSTU_ERR_HIP;
  t.on = true;
  return HSTU_OK;
}

int hstu_debug_timing_end(int32_t* kinds, float* milliseconds, int capacity) {
  Timing& t = g_timing;
  if (!t.on) return HSTU_ERR_BAD_SHAPE;
  t.on = false;
  int n = 0, rc = HSTU_OK;
  for (size_t i = 0; i < t.used; ++i) {
    float ms = 0.f;
    if (hipEventSynchronize(t.stop[i]) != hipSuccess ||
        hipEventElapsedTime(&ms, t.start[i], t.stop[i]) != hipSuccess)
      rc = HSTU_ERR_HIP;
    if (n < capacity && kinds && milliseconds) {
      kinds[n] = t.kind[i];
      milliseconds[n] = ms;
      ++n;
    }
  }
  for (size_t i = 0; i < t.start.size(); ++i) {
    if (t.start[i]) (void)hipEventDestroy(t.start[i]);
    if (t.stop[i]) (void)hipEventDestroy(t.stop[i]);
  }
  t.start.clear(); t.stop.clear(); t.kind.clear(); t.used = 0;
  return rc == HSTU_OK ? n : rc;
}

int hstu_debug_dump_schedule(const hstu_attn_params* params, const hstu_cp_desc* cp, int side,
                             const int32_t* seq_offsets, int32_t* items_host, int32_t max_items,
                             void* workspace, size_t workspace_bytes, void* hip_stream) {
  int rc = check_params(params);
  if (rc != HSTU_OK) return rc;
  if (cp) {
    rc = check_cp(params, cp);
    if (rc != HSTU_OK) return rc;
  }
  if (side != 0 && side != 1) return HSTU_ERR_BAD_SHAPE;
  if (params->batch == 0 || params->total_rows == 0) return 0;
  if (!seq_offsets || !items_host || !workspace) return HSTU_ERR_NULL_PTR;
  if (workspace_bytes < hstu_jagged_attn_workspace_bytes(params, cp ? HSTU_WS_CP : HSTU_WS_FWD))
    return HSTU_ERR_WORKSPACE_TOO_SMALL;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  const int pass = side == 0 ? PASS_FWD : PASS_DKDV;
  const SideSpec s = cp ? cp_side(params, cp, side, pass) : full_side(params, side, pass);
  BuiltPlan bp;
  rc = build_plan(params, cp ? cp->cp_size : 1, s, seq_offsets, (char*)workspace, workspace_bytes,
                  0, stream, &bp);
  if (rc != HSTU_OK) return rc;
  int32_t n = 0;
  if (hipMemcpyAsync(&n, bp.plan.header, sizeof(int32_t), hipMemcpyDeviceToHost, stream) != hipSuccess)
    return HSTU_ERR_HIP;
  if (hipStreamSynchronize(stream) != hipSuccess) return HSTU_ERR_HIP;
  if (n > max_items) return HSTU_ERR_WORKSPACE_TOO_SMALL;
  if (n == 0) return 0;
  std::vector<int32_t> order(n);
  std::vector<Item> items(n);
  if (hipMemcpyAsync(order.data(), bp.plan.order, sizeof(int32_t) * n, hipMemcpyDeviceToHost, stream) != hipSuccess ||
      hipMemcpyAsync(items.data(), bp.plan.items, sizeof(Item) * n, hipMemcpyDeviceToHost, stream) != hipSuccess ||
      hipStreamSynchronize(stream) != hipSuccess)
    return HSTU_ERR_HIP;
  for (int32_t i = 0; i < n; ++i) {
    const int32_t idx = order[i];
    if (idx < 0 || idx >= n) return HSTU_ERR_HIP;
    const Item& it = items[idx];
    int32_t* dst = items_host + (size_t)i * 12;
    dst[0] = it.row0; dst[1] = it.nrows; dst[2] = it.pos0; dst[3] = it.nseg;
    dst[4] = it.seg_row0[0]; dst[5] = it.seg_row0[1];
    dst[6] = it.seg_len[0]; dst[7] = it.seg_len[1];
    dst[8] = it.seg_pos0[0]; dst[9] = it.seg_pos0[1];
    dst[10] = it.cost; dst[11] = it.part;
  }
  return n;
}

}  // extern "C"
